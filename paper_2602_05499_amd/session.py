"""Session: owns the device buffers (through torch) that the library borrows, and forwards calls to the C-ABI.

Marshalling only.  The one piece of host control flow here, `generate`, is the outer loop of Alg. 1 Stage B
(repeat draft / verify / accept / rollback until enough tokens are committed); all arithmetic and all token
decisions happen in the kernels.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

from . import binding as B

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-shared", "-fPIC"]


def build_library(verbose: bool = False, jobs: int = 8, defines=()) -> str:
    """Compile csrc/*.hip for gfx950 (hipcc cross-compiles without a GPU) and link libsdfp.so next to this
    file.  The kernel instantiations are spread over several translation units built in parallel.
    defines: extra -D macros, e.g. ("SDFP_GUARD",) for the range-checked diagnostic build."""
    import concurrent.futures
    import glob
    out = B.library_path()
    src_dir = os.path.join(_HERE, "csrc")
    obj_dir = os.path.join(_HERE, "_build" + ("_" + "_".join(d.split("=")[0] for d in defines) if defines else ""))
    os.makedirs(obj_dir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(src_dir, "*.hip")))
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + ["-D" + d for d in defines]

    def compile_one(src):
        obj = os.path.join(obj_dir, os.path.basename(src)[:-4] + ".o")
        cmd = ["hipcc", *flags, "-c", "-I", os.path.join(_ROOT, "include"), "-I", src_dir, "-o", obj, src]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on " + src + ":\n" + res.stderr[-4000:])
        return obj

    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, srcs))
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr[-4000:])
    if verbose:
        print("built", out, "from", len(srcs), "translation units")
    return out


LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def make_config(shape, max_seq: int, max_k: int, max_out: int, temperature: float = 1.0):
    """The C configuration struct of a model shape."""
    return B.SdConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      shape.vocab, int(max_seq), int(max_k), B.SD_F32 if shape.dtype == "f32" else B.SD_BF16, int(max_out),
                      shape.rms_eps, shape.rope_theta, temperature)


def make_weights(shape, weights):
    """The C weights struct (device pointers) of torch tensors; returns (struct, arrays to keep alive with it)."""
    L = shape.n_layers
    arrs = {f: (ctypes.c_void_p * L)(*[weights.layers[l][f].data_ptr() for l in range(L)]) for f in LAYER_FIELDS}
    w = B.SdWeights(weights.tok_emb.data_ptr(), weights.final_norm.data_ptr(), weights.lm_head.data_ptr(),
                    *[ctypes.cast(arrs[f], ctypes.POINTER(ctypes.c_void_p)) for f in LAYER_FIELDS])
    return w, arrs


def fit_scores(shape, weights, samples, stream=None, cache_transposes=True):
    """FIT layer scores of a model on the GPU (sd_fit_scores): samples is an int array [n_samples][T].  Returns
    (t_attn, t_ffn, losses) as float64 arrays; allocates the scratch workspace with torch for the call, by default with
    the surplus that lets the library keep its transposed and tile-ordered matrices across the samples."""
    import torch
    toks = np.ascontiguousarray(samples, np.int32)
    cfg = make_config(shape, max_seq=max(64, toks.shape[1]), max_k=0, max_out=1)
    w, keep = make_weights(shape, weights)
    need = B.sd_fit_workspace_bytes(cfg, toks.shape[1])
    if need == 0:
        raise B.SdError(B.SD_EINVAL, "sd_fit_workspace_bytes")
    if cache_transposes and toks.shape[0] > 1:   # room for a transposed copy of every layer matrix and the head
        hq, hk = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
        up = lambda n: (2 * n + 255) // 256 * 256
        per_layer = up(hq * shape.d_model) + 2 * up(hk * shape.d_model) + up(shape.d_model * hq) + 3 * up(shape.d_ffn * shape.d_model)
        # ... twice: the transposed matrices of the backward, and the matrices in tile order for the forward
        need += 2 * (shape.n_layers * per_layer + up(shape.vocab * shape.d_model))
    ws = torch.empty(need, dtype=torch.uint8, device=weights.tok_emb.device)
    st = stream if stream is not None else torch.cuda.current_stream(weights.tok_emb.device)
    rc, ta, tf, ls = B.sd_fit_scores(cfg, w, toks, ws.data_ptr(), need, st.cuda_stream)
    del keep
    if rc != B.SD_OK:
        raise B.SdError(rc, "sd_fit_scores")
    return ta, tf, ls


class Session:
    """One decode context on the current torch device.

    weights: object with torch tensors tok_emb, final_norm, lm_head and `layers` (list of dicts keyed by
    LAYER_FIELDS) already resident on the GPU in the storage dtype (norm gains float32).
    """

    def __init__(self, shape, weights, skip_mask=None, max_seq: Optional[int] = None, max_k: Optional[int] = None,
                 max_out: Optional[int] = None, temperature: float = 1.0, stream=None,
                 static_workspace: bool = False, tiled_weights: Optional[bool] = None):
        import torch
        self.torch = torch
        self.shape = shape
        self.weights = weights          # keep the tensors alive
        max_seq = int(max_seq if max_seq is not None else shape.max_seq)
        max_k = int(max_k if max_k is not None else shape.K)
        max_out = int(max_out if max_out is not None else max_seq + B.SD_MAX_K + 1)
        self.cfg = B.SdConfig(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                              shape.d_ffn, shape.vocab, max_seq, max_k,
                              B.SD_F32 if shape.dtype == "f32" else B.SD_BF16, max_out, shape.rms_eps,
                              shape.rope_theta, temperature)
        kvb, wsb = B.sd_kv_bytes(self.cfg), B.sd_workspace_bytes(self.cfg)
        if kvb == 0 or wsb == 0:
            raise B.SdError(B.SD_EINVAL, "sd_kv_bytes/sd_workspace_bytes")
        dev = weights.tok_emb.device
        self.kv = torch.zeros(kvb, dtype=torch.uint8, device=dev)
        # static_workspace: the library's own static array serves as the workspace (sd_init_static)
        self.ws = None if static_workspace else torch.zeros(wsb, dtype=torch.uint8, device=dev)
        L = shape.n_layers
        self._arrs = {f: (ctypes.c_void_p * L)(*[weights.layers[l][f].data_ptr() for l in range(L)])
                      for f in LAYER_FIELDS}
        w = B.SdWeights(weights.tok_emb.data_ptr(), weights.final_norm.data_ptr(), weights.lm_head.data_ptr(),
                        *[ctypes.cast(self._arrs[f], ctypes.POINTER(ctypes.c_void_p)) for f in LAYER_FIELDS])
        self.stream = stream if stream is not None else torch.cuda.current_stream(dev)
        mask = None if skip_mask is None else np.ascontiguousarray(skip_mask, np.uint8)
        if static_workspace:
            rc, self.ctx = B.sd_init_static(self.cfg, w, mask, self.kv.data_ptr(), kvb, self.stream.cuda_stream)
        else:
            rc, self.ctx = B.sd_init(self.cfg, w, mask, self.kv.data_ptr(), kvb, self.ws.data_ptr(), wsb,
                                     self.stream.cuda_stream)
        if rc != B.SD_OK:
            self.ctx = None
        self._check(rc, "sd_init_static" if static_workspace else "sd_init")
        self.max_seq, self.max_k, self.max_out = max_seq, max_k, max_out
        # bfloat16 storage: a second copy of the layer matrices in the tile order of the matrix-matrix prompt path
        # (sd_set_tiled_weights; optional, the prompt path reads the caller's matrices without it, more slowly)
        # tiled_weights: True = attach it (an allocation failure is raised), False = never, None = attach it if the
        # allocation succeeds (a 70B-shaped model's copy is 128 GB next to 138 GB of weights)
        self.tiled = None
        if tiled_weights is not False and not static_workspace:
            try:
                self.set_tiled_weights(True)
            except torch.OutOfMemoryError:
                if tiled_weights:
                    raise
                self.tiled = None

    def _check(self, rc, where):
        if rc != B.SD_OK:
            raise B.SdError(rc, where, B.sd_last_hip_error(self.ctx) if getattr(self, "ctx", None) else 0)

    def close(self):
        if getattr(self, "ctx", None):
            B.sd_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- one method per entry point ---------------------------------------------------------------------
    @staticmethod
    def _u(u):
        return None if u is None else np.ascontiguousarray(u, np.float32)

    def set_skip_mask(self, mask):
        self._check(B.sd_set_skip_mask(self.ctx, np.ascontiguousarray(mask, np.uint8)), "sd_set_skip_mask")

    def prefill(self, prompt, mode=B.SD_GREEDY, u=None):
        self._check(B.sd_prefill(self.ctx, np.ascontiguousarray(prompt, np.int32), mode, self._u(u)), "sd_prefill")

    def draft(self, K, mode=B.SD_GREEDY, u=None):
        self._check(B.sd_draft(self.ctx, K, mode, self._u(u)), "sd_draft")

    def verify(self):
        self._check(B.sd_verify(self.ctx), "sd_verify")

    def accept(self, mode=B.SD_GREEDY, u=None):
        self._check(B.sd_accept(self.ctx, mode, self._u(u)), "sd_accept")

    def rollback(self):
        self._check(B.sd_rollback(self.ctx), "sd_rollback")

    def decode(self, mode=B.SD_GREEDY, u=None):
        self._check(B.sd_decode(self.ctx, mode, self._u(u)), "sd_decode")

    def set_pending(self, cache_len, token):
        self._check(B.sd_set_pending(self.ctx, int(cache_len), int(token)), "sd_set_pending")

    def set_draft(self, d):
        self._check(B.sd_set_draft(self.ctx, np.ascontiguousarray(d, np.int32)), "sd_set_draft")

    def keep_logits(self, on=True):
        self._check(B.sd_keep_logits(self.ctx, on), "sd_keep_logits")

    def set_spin_limit(self, polls):
        """Bound of every wait inside the forward kernel, in polls (a tiny value forces the time-out path)."""
        self._check(B.sd_set_spin_limit(self.ctx, polls), "sd_set_spin_limit")

    def set_turn_span(self, mode):
        """Which set of decode kernels runs: -1 chosen from the shapes, 0 / 1 ring turns never / always go on into the
        next tile (bit-identical results either way)."""
        self._check(B.sd_set_turn_span(self.ctx, mode), "sd_set_turn_span")

    def set_prefill_mode(self, mode):
        """How sd_prefill runs the prompt: -1 chosen from the prompt, 0 in 16-row chunks through the forward kernel,
        1 as matrix-matrix products (bit-identical results either way)."""
        self._check(B.sd_set_prefill_mode(self.ctx, mode), "sd_set_prefill_mode")

    def set_tiled_weights(self, on):
        """Attach (allocating it with torch) or detach the tiled copy of the layer matrices; bit-identical results
        either way.  No-op for float32 storage."""
        if not on:
            self._check(B.sd_set_tiled_weights(self.ctx, None, 0), "sd_set_tiled_weights")
            self.sync()
            self.tiled = None
            return
        need = B.sd_tiled_weights_bytes(self.cfg)
        if need == 0 or self.tiled is not None:
            return
        self.tiled = self.torch.empty(need, dtype=self.torch.uint8, device=self.kv.device)
        self._check(B.sd_set_tiled_weights(self.ctx, self.tiled.data_ptr(), need), "sd_set_tiled_weights")

    def phase_trace(self, on=True):
        self._check(B.sd_phase_trace(self.ctx, on), "sd_phase_trace")

    def read_phase_trace(self):
        """[(tag, microseconds since the first entry)] of the most recent forward's workgroup 0."""
        buf = np.zeros(1024, np.uint64)
        n = ctypes.c_int32(0)
        self._check(B.sd_phase_trace_read(self.ctx, buf, n), "sd_phase_trace_read")
        ent = buf[:n.value]
        if len(ent) == 0:
            return []
        t = (ent & np.uint64((1 << 56) - 1)).astype(np.int64)
        return [(int(e >> np.uint64(56)), (int(tt) - int(t[0])) / 100.0) for e, tt in zip(ent, t)]

    def guard_read(self):
        """Record of a -DSDFP_GUARD build: (violations, [(site, address, bytes, workgroup, thread)])."""
        buf = np.zeros(32, np.uint64)
        self._check(B.sd_guard_read(self.ctx, buf), "sd_guard_read")
        n = int(buf[0])
        recs = [(int(buf[1 + 3 * i]), hex(int(buf[2 + 3 * i])), int(buf[3 + 3 * i]) & 0xFFFFFFFF,
                 (int(buf[3 + 3 * i]) >> 32) & 0xFFFF, int(buf[3 + 3 * i]) >> 48) for i in range(min(n, 10))]
        return n, recs

    def sync(self):
        self._check(B.sd_sync(self.ctx), "sd_sync")

    def read(self, cap: Optional[int] = None):
        """Returns (tokens int32[n], stats dict).  Waits for the stream."""
        cap = self.max_out if cap is None else cap
        buf = np.zeros(cap, np.int32)
        n = ctypes.c_int32(0)
        st = B.SdStats()
        self._check(B.sd_read(self.ctx, buf, n, st), "sd_read")
        stats = {k: getattr(st, k) for k, _ in B.SdStats._fields_}
        return buf[:min(n.value, cap)].copy(), stats

    def committed(self) -> int:
        n = ctypes.c_int32(0)
        self._check(B.sd_read(self.ctx, None, n, None), "sd_read")
        return n.value

    def dump_logits(self, which, rows):
        out = np.zeros((rows, self.shape.vocab), np.float32)
        if rows:
            self._check(B.sd_dump_logits(self.ctx, which, out), "sd_dump_logits")
        return out

    def dump_draft(self, K):
        out = np.zeros(max(K, 1), np.int32)
        self._check(B.sd_dump_draft(self.ctx, out), "sd_dump_draft")
        return out[:K]

    # ---- outer loops ------------------------------------------------------------------------------------
    def step(self, K, mode=B.SD_GREEDY, u=None):
        """draft -> verify -> accept -> rollback.  Sampling: u holds 2K+1 uniforms (K draft, K accept, 1 resample)."""
        if mode == B.SD_SAMPLE:
            u = np.ascontiguousarray(u, np.float32)
            self.draft(K, mode, u[:K])
            self.verify()
            self.accept(mode, u[K:2 * K + 1])
        else:
            self.draft(K, mode)
            self.verify()
            self.accept(mode)
        self.rollback()

    def generate(self, prompt, G, K, mode=B.SD_GREEDY, uniforms=None, poll_every: int = 1):
        """Exactly G tokens after the prompt (first one from the prefill); the last step is truncated.
        K = 0 is vanilla autoregressive decoding.  The committed count is read back every `poll_every` steps."""
        cur = 0
        if mode == B.SD_SAMPLE:
            self.prefill(prompt, mode, uniforms[0:1]); cur = 1
        else:
            self.prefill(prompt, mode)
        per = 2 * K + 1
        n = 1
        while n < G:
            for _ in range(poll_every):
                if mode == B.SD_SAMPLE:
                    self.step(K, mode, uniforms[cur:cur + per]); cur += per
                else:
                    self.step(K, mode)
                n += 1          # every step commits at least one token
                if n >= G:
                    break
            n = self.committed()
        toks, stats = self.read()
        return toks[:G], stats
