"""Counter-based synthetic inputs: every value is a pure function of (seed, tensor id, flat index).

Definition (this numpy code is the definition; `gen_cpu.c` and `gen_fill.hip` are faster
re-implementations of the same integer recipe and are tested bit-for-bit against it):

    z      = mix64(seed + GOLDEN * (tensor_id * 2**40 + idx))          (mod 2**64, splitmix64 finaliser)
    s      = (sum of the 8 bytes of z) - 1020                            (Irwin-Hall(8), mean 0)
    w      = float32(s) * float32(std / sqrt(43690))                     (std of the byte sum = sqrt(43690))
    weight = w rounded to the storage dtype (bf16: round-to-nearest-even)

The byte sum of 8 independent uniform bytes has variance 8*(256**2-1)/12 = 43690, so `w` has mean 0 and
standard deviation `std`: a stand-in for "N(0, std)" whose every step is exact in integer or single
float arithmetic, hence reproducible on any device.  Nothing here depends on the decode method.
"""
from __future__ import annotations

import ctypes
import dataclasses
import math
import os
from typing import Dict, List, Optional

import numpy as np

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
BYTE_SUM_VAR = 43690.0  # 8 * (256**2 - 1) / 12

SEED_WEIGHTS = 1234
SEED_MASK = 42
SEED_PROMPT = 5678
SEED_UNIFORMS = 91011

# tensor slots inside a layer / among the globals
LAYER_SLOTS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")
GLOBAL_SLOTS = ("tok_emb", "final_norm", "lm_head")


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str           # "f32" | "bf16": storage type of weight matrices and of the KV cache
    n_skip: int          # number of whole layers the draft skips
    K: int               # speculation depth
    mode: str            # "greedy" | "sample"
    n_prompt: int
    n_gen: int
    skip_layers: Optional[tuple] = None   # explicit skip set (tiny config); else seeded choice
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    init_std: float = 0.02
    gain_std: float = 0.0   # spread of the RMSNorm gains around 1 (0: all ones, as in the benchmark workloads)

    @property
    def max_seq(self) -> int:
        return self.n_prompt + self.n_gen + self.K + 1

    def with_(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, ModelShape] = {
    "tiny": ModelShape("tiny", 4, 256, 4, 4, 64, 688, 1024, "f32", 2, 4, "greedy", 32, 64,
                       skip_layers=(1, 2)),
    "7b": ModelShape("7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16", 16, 4, "greedy", 512, 256),
    "13b": ModelShape("13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16", 16, 6, "sample", 1024, 256),
    "l3-8b": ModelShape("l3-8b", 32, 4096, 32, 8, 128, 14336, 128256, "bf16", 12, 4, "greedy", 4096, 512),
    "70b": ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 32000, "bf16", 40, 5, "greedy", 1024, 128),
}


def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output finaliser on uint64 arrays (wrapping arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _hash(seed: int, stream: int, idx: np.ndarray) -> np.ndarray:
    idx = np.asarray(idx, dtype=np.uint64)
    with np.errstate(over="ignore"):
        ctr = (np.uint64(stream) << np.uint64(40)) + idx
        return mix64(np.uint64(seed) + GOLDEN * ctr)


def tensor_id(shape: ModelShape, layer: Optional[int], slot: str) -> int:
    if layer is None:
        return shape.n_layers * 16 + GLOBAL_SLOTS.index(slot)
    return layer * 16 + LAYER_SLOTS.index(slot)


def tensor_shapes(s: ModelShape) -> Dict[str, tuple]:
    """Row-major [out_features, in_features] for matrices; [d] for norm gains."""
    hq = s.n_heads * s.head_dim
    hk = s.n_kv_heads * s.head_dim
    return {
        "attn_norm": (s.d_model,), "wq": (hq, s.d_model), "wk": (hk, s.d_model), "wv": (hk, s.d_model),
        "wo": (s.d_model, hq), "ffn_norm": (s.d_model,), "w_gate": (s.d_ffn, s.d_model),
        "w_up": (s.d_ffn, s.d_model), "w_down": (s.d_model, s.d_ffn),
        "tok_emb": (s.vocab, s.d_model), "final_norm": (s.d_model,), "lm_head": (s.vocab, s.d_model),
    }


def scale_f32(std: float) -> np.float32:
    return np.float32(std / math.sqrt(BYTE_SUM_VAR))


def gen_tensor_f32(seed: int, tid: int, n: int, std: float, start: int = 0) -> np.ndarray:
    """n float32 values of tensor `tid` starting at flat index `start` (numpy definition)."""
    z = _hash(seed, tid, np.arange(start, start + n, dtype=np.uint64))
    s = z.view(np.uint8).reshape(-1, 8).sum(axis=1, dtype=np.int32) - 1020
    return s.astype(np.float32) * scale_f32(std)


def gen_gain(seed: int, tid: int, n: int, gain_std: float) -> np.ndarray:
    """RMSNorm gain vector of tensor `tid`: float32(1 + w) with w from the weight recipe at standard deviation
    gain_std (|w| <= 4.9 gain_std), so every norm of every layer has its own values; all ones for gain_std = 0."""
    if gain_std == 0.0:
        return np.ones(n, dtype=np.float32)
    return (np.float32(1.0) + gen_tensor_f32(seed, tid, n, gain_std)).astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16). Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- optional fast CPU fill (same recipe in C, OpenMP) -------------------------------------------------
_HERE = os.path.dirname(os.path.abspath(__file__))
_cpu_lib = None


def _load_cpu_lib():
    global _cpu_lib
    if _cpu_lib is None:
        path = os.path.join(_HERE, "libsynth_cpu.so")
        if os.path.exists(path):
            lib = ctypes.CDLL(path)
            lib.synth_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_float]
            lib.synth_fill_host.restype = None
            _cpu_lib = lib
        else:
            _cpu_lib = False
    return _cpu_lib


def gen_tensor(seed: int, tid: int, n: int, std: float, dtype: str, force_numpy: bool = False) -> np.ndarray:
    """Flat tensor in storage dtype: float32 array for "f32", uint16 bit patterns for "bf16"."""
    lib = None if force_numpy else _load_cpu_lib()
    if lib:
        out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
        lib.synth_fill_host(out.ctypes.data, 0 if dtype == "f32" else 1, seed, tid, 0, n,
                            ctypes.c_float(float(scale_f32(std))))
        return out
    chunks = []
    step = 1 << 22
    for st in range(0, n, step):
        w = gen_tensor_f32(seed, tid, min(step, n - st), std, start=st)
        chunks.append(w if dtype == "f32" else f32_to_bf16_bits(w))
    return np.concatenate(chunks) if chunks else np.empty(0, np.float32 if dtype == "f32" else np.uint16)


def gen_prompt(seed: int, n: int, vocab: int) -> np.ndarray:
    """n token ids, i.i.d. uniform on [0, vocab)."""
    z = _hash(seed, 0xFFFF01, np.arange(n, dtype=np.uint64))
    return (((z >> np.uint64(32)) * np.uint64(vocab)) >> np.uint64(32)).astype(np.int32)


def gen_uniforms(seed: int, n: int) -> np.ndarray:
    """n float32 uniforms on [0, 1): top 24 bits of the hash times 2**-24."""
    z = _hash(seed, 0xFFFF02, np.arange(n, dtype=np.uint64))
    return ((z >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def gen_skip_mask(shape: ModelShape, seed: int = SEED_MASK) -> np.ndarray:
    """uint8[L]: 3 = skip the whole layer (bit0 attention sub-layer, bit1 FFN sub-layer), 0 = keep."""
    L = shape.n_layers
    mask = np.zeros(L, dtype=np.uint8)
    if shape.skip_layers is not None:
        for l in shape.skip_layers:
            mask[l] = 3
        return mask
    perm = list(range(L))
    z = _hash(seed, 0xFFFF03, np.arange(L, dtype=np.uint64))
    for i in range(L - 1, 0, -1):          # Fisher-Yates driven by the hash stream
        j = int(z[i] % np.uint64(i + 1))
        perm[i], perm[j] = perm[j], perm[i]
    for l in perm[:shape.n_skip]:
        mask[l] = 3
    return mask


def gen_sublayer_mask(shape: ModelShape, frac_attn: float, frac_ffn: float, seed: int = SEED_MASK) -> np.ndarray:
    """uint8[L] with the two sub-layer bits drawn separately: round(frac_attn * L) attention sub-layers (bit0) and
    round(frac_ffn * L) FFN sub-layers (bit1) are skipped, each set by its own seeded Fisher-Yates shuffle (the
    setting of Sec. IV-A: a share of the attention and of the FFN sub-layers pruned independently)."""
    L = shape.n_layers
    mask = np.zeros(L, dtype=np.uint8)
    for bit, frac, stream in ((1, frac_attn, 0xFFFF04), (2, frac_ffn, 0xFFFF05)):
        perm = list(range(L))
        z = _hash(seed, stream, np.arange(L, dtype=np.uint64))
        for i in range(L - 1, 0, -1):
            j = int(z[i] % np.uint64(i + 1))
            perm[i], perm[j] = perm[j], perm[i]
        for l in perm[:int(round(frac * L))]:
            mask[l] |= bit
    return mask


@dataclasses.dataclass
class HostWeights:
    """Host copies of every tensor: matrices in storage dtype (float32 / uint16 bf16 bits), norm gains float32."""
    shape: ModelShape
    tok_emb: np.ndarray
    final_norm: np.ndarray
    lm_head: np.ndarray
    layers: List[Dict[str, np.ndarray]]

    def nbytes(self) -> int:
        n = self.tok_emb.nbytes + self.final_norm.nbytes + self.lm_head.nbytes
        return n + sum(a.nbytes for l in self.layers for a in l.values())


def gen_host_weights(shape: ModelShape, seed: int = SEED_WEIGHTS, damp_skipped: float = 1.0,
                     skip_mask: Optional[np.ndarray] = None) -> HostWeights:
    """All tensors of `shape` on the host. `damp_skipped` (gamma) scales W_o of masked attention sub-layers and W_down of masked FFN sub-layers:
    1.0 reproduces the verbatim config; smaller values make the draft agree with the target more often."""
    shp = tensor_shapes(shape)

    def mat(layer, slot, scale=1.0):
        dims = shp[slot]
        n = int(np.prod(dims))
        if slot.endswith("norm"):
            return gen_gain(seed, tensor_id(shape, layer, slot), n, shape.gain_std)
        a = gen_tensor(seed, tensor_id(shape, layer, slot), n, shape.init_std * scale, shape.dtype)
        return a.reshape(dims)

    layers = []
    for l in range(shape.n_layers):
        bits = int(skip_mask[l]) if skip_mask is not None else 0
        damp = {"wo": damp_skipped if bits & 1 else 1.0, "w_down": damp_skipped if bits & 2 else 1.0}
        layers.append({slot: mat(l, slot, damp.get(slot, 1.0)) for slot in LAYER_SLOTS})
    return HostWeights(shape, mat(None, "tok_emb"), mat(None, "final_norm"), mat(None, "lm_head"), layers)
