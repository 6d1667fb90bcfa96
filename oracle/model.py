"""ctypes binding of the oracle's C forward pass (sdfp_oracle.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsdfp_oracle.so")
_lib = None

LAYER_ORDER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "max_seq", "dtype")]
    _fields_ += [("rms_eps", ctypes.c_double), ("rope_theta", ctypes.c_double)]


def build_oracle(force: bool = False) -> str:
    """Compile sdfp_oracle.c with gcc (plain C, OpenMP over output rows / heads)."""
    src = os.path.join(_HERE, "sdfp_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-mfma", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build_oracle()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.orc_create.restype = ctypes.c_void_p
        lib.orc_create.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(ctypes.c_void_p)]
        lib.orc_destroy.argtypes = [ctypes.c_void_p]
        lib.orc_forward.restype = ctypes.c_int
        lib.orc_forward.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                    ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        lib.orc_kcache.restype = ctypes.c_void_p
        lib.orc_kcache.argtypes = [ctypes.c_void_p]
        lib.orc_vcache.restype = ctypes.c_void_p
        lib.orc_vcache.argtypes = [ctypes.c_void_p]
        lib.orc_round_storage.restype = ctypes.c_float
        lib.orc_round_storage.argtypes = [ctypes.c_double, ctypes.c_int]
        lib.orc_rmsnorm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_void_p]
        lib.orc_matmul.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                   ctypes.c_int, ctypes.c_void_p]
        lib.orc_rope.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        lib.orc_attend.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_size_t, ctypes.c_void_p]
        lib.orc_silu.restype = ctypes.c_double
        lib.orc_silu.argtypes = [ctypes.c_double]
        _lib = lib
    return _lib


def round_storage(v: float, dtype: str) -> float:
    return float(_load().orc_round_storage(float(v), 0 if dtype == "f32" else 1))


# thin wrappers over the exported primitives, for the pin tests
def rmsnorm(h, g, eps):
    h = np.ascontiguousarray(h, np.float64); g = np.ascontiguousarray(g, np.float32)
    out = np.empty_like(h)
    _load().orc_rmsnorm(h.ctypes.data, g.ctypes.data, h.size, eps, out.ctypes.data)
    return out


def matmul(W, dtype, X):
    """W: [N,Kd] storage-type array (float32, or uint16 bf16 bits); X: [M,Kd] float64 -> [M,N] float64."""
    X = np.ascontiguousarray(X, np.float64)
    W = np.ascontiguousarray(W)
    N, Kd = W.shape
    Y = np.empty((X.shape[0], N), np.float64)
    _load().orc_matmul(W.ctypes.data, 0 if dtype == "f32" else 1, N, Kd, X.ctypes.data, X.shape[0], Y.ctypes.data)
    return Y


def rope(v, pos, theta):
    v = np.array(v, np.float64)
    _load().orc_rope(v.ctypes.data, v.size, pos, theta)
    return v


def attend(q, kc, vc):
    """q [hd] float64; kc, vc [n_pos, hd] float32 -> [hd] float64."""
    q = np.ascontiguousarray(q, np.float64)
    kc = np.ascontiguousarray(kc, np.float32); vc = np.ascontiguousarray(vc, np.float32)
    out = np.empty(q.size, np.float64)
    _load().orc_attend(q.ctypes.data, kc.ctypes.data, vc.ctypes.data, kc.shape[0], q.size, q.size, out.ctypes.data)
    return out


def silu(z: float) -> float:
    return float(_load().orc_silu(float(z)))


class OracleModel:
    """A decoder-only transformer on the host with its own KV cache.

    `weights` is any object with attributes tok_emb, final_norm, lm_head (numpy arrays) and `layers`, a list
    of dicts keyed by LAYER_ORDER; matrices are float32 ("f32") or uint16 bf16 bit patterns ("bf16"), norm
    gains float32.  The arrays are borrowed: they must outlive this object.
    """

    def __init__(self, shape, weights, max_seq: Optional[int] = None):
        lib = _load()
        self.shape = shape
        self.max_seq = int(max_seq if max_seq is not None else shape.max_seq)
        self._keep = weights
        cfg = _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                      shape.vocab, self.max_seq, 0 if shape.dtype == "f32" else 1, shape.rms_eps, shape.rope_theta)
        want = np.float32 if shape.dtype == "f32" else np.uint16
        ptrs = []

        def add(a, dt):
            assert a.dtype == dt and a.flags["C_CONTIGUOUS"], (a.dtype, dt)
            ptrs.append(a.ctypes.data)

        add(weights.tok_emb, want); add(weights.final_norm, np.float32); add(weights.lm_head, want)
        for lw in weights.layers:
            for name in LAYER_ORDER:
                add(lw[name], np.float32 if name.endswith("norm") else want)
        table = (ctypes.c_void_p * len(ptrs))(*ptrs)
        self._h = lib.orc_create(ctypes.byref(cfg), table)
        if not self._h:
            raise ValueError("orc_create rejected the configuration")
        self._lib = lib

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.orc_destroy(self._h)
            self._h = None

    def forward(self, tokens, pos0: int, skip=None, logits_from: int = 0, want_hidden: bool = False):
        """Rows tokens[m] at positions pos0+m (causal); returns float64 logits [M-logits_from, V]."""
        tok = np.ascontiguousarray(tokens, np.int32)
        M = tok.size
        V = self.shape.vocab
        logits = np.empty((M - logits_from, V), np.float64)
        hidden = np.empty((M, self.shape.d_model), np.float64) if want_hidden else None
        sk = None if skip is None else np.ascontiguousarray(skip, np.uint8)
        assert sk is None or sk.size == self.shape.n_layers
        rc = self._lib.orc_forward(self._h, tok.ctypes.data, M, int(pos0), None if sk is None else sk.ctypes.data,
                                   int(logits_from), logits.ctypes.data,
                                   None if hidden is None else hidden.ctypes.data)
        if rc != 0:
            raise ValueError(f"orc_forward failed rc={rc} (M={M}, pos0={pos0}, max_seq={self.max_seq})")
        return (logits, hidden) if want_hidden else logits

    def kv_arrays(self):
        """Views [L, max_seq, H_kv*hd] float32 of the K and V caches (values as stored)."""
        s = self.shape
        n = s.n_layers * self.max_seq * s.n_kv_heads * s.head_dim
        shp = (s.n_layers, self.max_seq, s.n_kv_heads * s.head_dim)
        k = np.ctypeslib.as_array(ctypes.cast(self._lib.orc_kcache(self._h), ctypes.POINTER(ctypes.c_float)), (n,))
        v = np.ctypeslib.as_array(ctypes.cast(self._lib.orc_vcache(self._h), ctypes.POINTER(ctypes.c_float)), (n,))
        return k.reshape(shp), v.reshape(shp)
