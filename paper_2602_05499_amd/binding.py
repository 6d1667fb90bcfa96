"""ctypes declarations mirroring include/sdfp.h one to one (same names, same argument order)."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

SD_F32, SD_BF16 = 0, 1
SD_GREEDY, SD_SAMPLE = 0, 1
SD_LOGITS_DRAFT, SD_LOGITS_VERIFY = 0, 1
SD_OK, SD_EINVAL, SD_ECAPACITY, SD_ESTATE, SD_EHIP, SD_ENOMEM, SD_ETIMEOUT = 0, -1, -2, -3, -4, -5, -6
SD_MAX_K = 8
SD_STATIC_WS_BYTES = 64 << 20
SD_STATIC_MAX_LAYERS = 128

EXPORTED_SYMBOLS = (
    "sd_kv_bytes", "sd_workspace_bytes", "sd_init", "sd_init_static", "sd_set_skip_mask", "sd_prefill", "sd_draft", "sd_verify",
    "sd_accept", "sd_rollback", "sd_decode", "sd_set_pending", "sd_set_draft", "sd_read", "sd_dump_logits",
    "sd_dump_draft", "sd_keep_logits", "sd_phase_trace", "sd_phase_trace_read", "sd_set_spin_limit", "sd_set_turn_span", "sd_set_prefill_mode", "sd_tiled_weights_bytes", "sd_set_tiled_weights", "sd_guard_read", "sd_guard_host_buffer", "sd_sync", "sd_last_hip_error", "sd_free", "sd_strerror",
    "sd_fit_workspace_bytes", "sd_fit_scores", "sd_fit_prune_mask", "sd_fit_prune_sublayers",
)


class SdConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "max_seq", "max_k",
                 "dtype", "max_out")]
    _fields_ += [("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float), ("temperature", ctypes.c_float)]


_PP = ctypes.POINTER(ctypes.c_void_p)


class SdWeights(ctypes.Structure):
    _fields_ = [("tok_emb", ctypes.c_void_p), ("final_norm", ctypes.c_void_p), ("lm_head", ctypes.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP), ("ffn_norm", _PP),
                ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP)]


class SdStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("steps", "drafted", "accepted", "examined", "committed")]
    _fields_ += [(n, ctypes.c_int32) for n in ("cache_len", "t_last", "last_n", "last_k")]


class SdError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        self.hip = hip
        msg = f"{where}: {sd_strerror(code)} ({code})"
        if hip:
            msg += f" [hip error {hip}]"
        super().__init__(msg)


def library_path() -> str:
    return os.path.join(_HERE, "libsdfp.so")


def load_library():
    """Load the built HIP library.  Fails loudly when it is missing: there is no other code path."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(path)
    vp, i32, f32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)
    i32p = ctypes.POINTER(ctypes.c_int32)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.sd_kv_bytes.restype = ctypes.c_size_t
    lib.sd_kv_bytes.argtypes = [ctypes.POINTER(SdConfig)]
    lib.sd_workspace_bytes.restype = ctypes.c_size_t
    lib.sd_workspace_bytes.argtypes = [ctypes.POINTER(SdConfig)]
    lib.sd_init.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(SdConfig), ctypes.POINTER(SdWeights), u8p, vp,
                            ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    lib.sd_init_static.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(SdConfig), ctypes.POINTER(SdWeights), u8p, vp,
                                   ctypes.c_size_t, vp]
    lib.sd_set_skip_mask.argtypes = [vp, u8p]
    lib.sd_prefill.argtypes = [vp, i32p, i32, ctypes.c_int, f32p]
    lib.sd_draft.argtypes = [vp, i32, ctypes.c_int, f32p]
    lib.sd_verify.argtypes = [vp]
    lib.sd_accept.argtypes = [vp, ctypes.c_int, f32p]
    lib.sd_rollback.argtypes = [vp]
    lib.sd_decode.argtypes = [vp, ctypes.c_int, f32p]
    lib.sd_set_pending.argtypes = [vp, i32, i32]
    lib.sd_set_draft.argtypes = [vp, i32p, i32]
    lib.sd_read.argtypes = [vp, i32p, i32, i32p, ctypes.POINTER(SdStats)]
    lib.sd_dump_logits.argtypes = [vp, ctypes.c_int, f32p, ctypes.c_size_t]
    lib.sd_dump_draft.argtypes = [vp, i32p, i32]
    lib.sd_keep_logits.argtypes = [vp, ctypes.c_int]
    lib.sd_phase_trace.argtypes = [vp, ctypes.c_int]
    lib.sd_set_spin_limit.argtypes = [vp, ctypes.c_uint32]
    lib.sd_set_turn_span.argtypes = [vp, ctypes.c_int]
    lib.sd_set_prefill_mode.argtypes = [vp, ctypes.c_int]
    lib.sd_tiled_weights_bytes.restype = ctypes.c_size_t
    lib.sd_tiled_weights_bytes.argtypes = [ctypes.POINTER(SdConfig)]
    lib.sd_set_tiled_weights.argtypes = [vp, vp, ctypes.c_size_t]
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.sd_fit_workspace_bytes.argtypes = [ctypes.POINTER(SdConfig), i32]
    lib.sd_fit_workspace_bytes.restype = ctypes.c_size_t
    lib.sd_fit_scores.argtypes = [ctypes.POINTER(SdConfig), ctypes.POINTER(SdWeights), i32p, i32, i32, vp, ctypes.c_size_t, vp,
                                  f64p, f64p, f64p]
    lib.sd_fit_prune_mask.argtypes = [f64p, f64p, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_uint8)]
    lib.sd_fit_prune_sublayers.argtypes = [f64p, f64p, i32, ctypes.c_double, ctypes.c_double, ctypes.POINTER(ctypes.c_uint8)]
    lib.sd_phase_trace_read.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), i32, i32p]
    lib.sd_guard_read.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.sd_guard_host_buffer.argtypes = [vp, ctypes.c_void_p, ctypes.c_size_t]
    lib.sd_sync.argtypes = [vp]
    lib.sd_last_hip_error.argtypes = [vp]
    lib.sd_free.argtypes = [vp]
    lib.sd_free.restype = None
    lib.sd_strerror.argtypes = [ctypes.c_int]
    lib.sd_strerror.restype = ctypes.c_char_p
    for name in EXPORTED_SYMBOLS:
        fn = getattr(lib, name)
        if fn.restype is ctypes.c_int and name not in ("sd_kv_bytes", "sd_workspace_bytes", "sd_tiled_weights_bytes"):
            fn.restype = ctypes.c_int
    _LIB = lib
    return lib


def _f32p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _u8p(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


# ---- one Python function per C entry point; each returns the C return code --------------------------------
def sd_kv_bytes(cfg: SdConfig) -> int:
    return load_library().sd_kv_bytes(ctypes.byref(cfg))


def sd_workspace_bytes(cfg: SdConfig) -> int:
    return load_library().sd_workspace_bytes(ctypes.byref(cfg))


def sd_init(cfg, weights, skip_mask, kv_ptr, kv_bytes, ws_ptr, ws_bytes, stream):
    """Returns (rc, ctx handle).  skip_mask: numpy uint8[L] or None; *_ptr: integer device addresses."""
    ctx = ctypes.c_void_p()
    rc = load_library().sd_init(ctypes.byref(ctx), ctypes.byref(cfg) if cfg is not None else None,
                                ctypes.byref(weights) if weights is not None else None, _u8p(skip_mask), kv_ptr,
                                kv_bytes, ws_ptr, ws_bytes, stream)
    return rc, ctx


def sd_init_static(cfg, weights, skip_mask, kv_ptr, kv_bytes, stream):
    """Returns (rc, ctx handle); the workspace is the library's own static array on the current device."""
    ctx = ctypes.c_void_p()
    rc = load_library().sd_init_static(ctypes.byref(ctx), ctypes.byref(cfg) if cfg is not None else None,
                                       ctypes.byref(weights) if weights is not None else None, _u8p(skip_mask),
                                       kv_ptr, kv_bytes, stream)
    return rc, ctx


def sd_set_skip_mask(ctx, skip_mask):
    return load_library().sd_set_skip_mask(ctx, _u8p(skip_mask))


def sd_prefill(ctx, prompt, mode, u=None):
    return load_library().sd_prefill(ctx, _i32p(prompt), 0 if prompt is None else len(prompt), mode, _f32p(u))


def sd_draft(ctx, K, mode, u=None):
    return load_library().sd_draft(ctx, K, mode, _f32p(u))


def sd_verify(ctx):
    return load_library().sd_verify(ctx)


def sd_accept(ctx, mode, u=None):
    return load_library().sd_accept(ctx, mode, _f32p(u))


def sd_rollback(ctx):
    return load_library().sd_rollback(ctx)


def sd_decode(ctx, mode, u=None):
    return load_library().sd_decode(ctx, mode, _f32p(u))


def sd_set_pending(ctx, cache_len, token):
    return load_library().sd_set_pending(ctx, cache_len, token)


def sd_set_draft(ctx, d):
    return load_library().sd_set_draft(ctx, _i32p(d), 0 if d is None else len(d))


def sd_read(ctx, tokens, n_committed, stats):
    """tokens: numpy int32 buffer or None; n_committed: ctypes.c_int32 or None; stats: SdStats or None."""
    return load_library().sd_read(ctx, _i32p(tokens), 0 if tokens is None else len(tokens),
                                  None if n_committed is None else ctypes.byref(n_committed),
                                  None if stats is None else ctypes.byref(stats))


def sd_dump_logits(ctx, which, out):
    return load_library().sd_dump_logits(ctx, which, _f32p(out), 0 if out is None else out.size)


def sd_dump_draft(ctx, out):
    return load_library().sd_dump_draft(ctx, _i32p(out), 0 if out is None else len(out))


def sd_keep_logits(ctx, on):
    return load_library().sd_keep_logits(ctx, int(on))


def sd_set_spin_limit(ctx, polls):
    return load_library().sd_set_spin_limit(ctx, int(polls))


def sd_set_turn_span(ctx, mode):
    return load_library().sd_set_turn_span(ctx, int(mode))


def sd_fit_workspace_bytes(cfg, T):
    return load_library().sd_fit_workspace_bytes(ctypes.byref(cfg), int(T))


def sd_fit_scores(cfg, weights, tokens, ws_ptr, ws_bytes, stream=None):
    """tokens: int32 array [n_samples][T].  Returns (rc, t_attn, t_ffn, losses)."""
    tokens = np.ascontiguousarray(tokens, np.int32)
    n, T = tokens.shape
    L = cfg.n_layers
    ta, tf, ls = np.zeros(L, np.float64), np.zeros(L, np.float64), np.zeros(n, np.float64)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = load_library().sd_fit_scores(ctypes.byref(cfg), ctypes.byref(weights), tokens.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      n, T, ctypes.c_void_p(ws_ptr), ws_bytes, ctypes.c_void_p(stream or 0),
                                      ta.ctypes.data_as(f64p), tf.ctypes.data_as(f64p), ls.ctypes.data_as(f64p))
    return rc, ta, tf, ls


def sd_fit_prune_mask(t_attn, t_ffn, ratio):
    """Returns (rc, mask) with mask a uint8 array [n_layers] of SD_SKIP_* bits."""
    ta, tf = np.ascontiguousarray(t_attn, np.float64), np.ascontiguousarray(t_ffn, np.float64)
    mask = np.zeros(len(ta), np.uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = load_library().sd_fit_prune_mask(ta.ctypes.data_as(f64p), tf.ctypes.data_as(f64p), len(ta), float(ratio),
                                          mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return rc, mask


def sd_fit_prune_sublayers(t_attn, t_ffn, ratio_attn, ratio_ffn):
    """Returns (rc, mask) with the attention and feed-forward sub-layers ranked and pruned separately."""
    ta, tf = np.ascontiguousarray(t_attn, np.float64), np.ascontiguousarray(t_ffn, np.float64)
    mask = np.zeros(len(ta), np.uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = load_library().sd_fit_prune_sublayers(ta.ctypes.data_as(f64p), tf.ctypes.data_as(f64p), len(ta), float(ratio_attn),
                                               float(ratio_ffn), mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return rc, mask


def sd_set_prefill_mode(ctx, mode):
    return load_library().sd_set_prefill_mode(ctx, int(mode))


def sd_tiled_weights_bytes(cfg: SdConfig) -> int:
    return load_library().sd_tiled_weights_bytes(ctypes.byref(cfg) if cfg is not None else None)


def sd_set_tiled_weights(ctx, buf_ptr, nbytes):
    """buf_ptr: integer device address (None or 0 detaches the copy)."""
    return load_library().sd_set_tiled_weights(ctx, buf_ptr or None, int(nbytes))


def sd_phase_trace(ctx, on):
    return load_library().sd_phase_trace(ctx, int(on))


def sd_guard_host_buffer(ctx, ptr, nbytes):
    return load_library().sd_guard_host_buffer(ctx, ptr, nbytes)


def sd_guard_read(ctx, out):
    return load_library().sd_guard_read(ctx, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)))


def sd_phase_trace_read(ctx, out, n):
    """out: numpy uint64 buffer; n: ctypes.c_int32 receiving the entry count."""
    return load_library().sd_phase_trace_read(ctx, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), len(out),
                                              ctypes.byref(n))


def sd_sync(ctx):
    return load_library().sd_sync(ctx)


def sd_last_hip_error(ctx):
    return load_library().sd_last_hip_error(ctx)


def sd_free(ctx):
    load_library().sd_free(ctx)


def sd_strerror(code: int) -> str:
    return load_library().sd_strerror(code).decode()
