"""Synthetic weights created directly in GPU memory (same recipe as gen.py, via gen_fill.hip) and their host
copies for the CPU oracle.  Test / benchmark plumbing: holds no arithmetic of the decode method."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from . import gen

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


def build_synth(force: bool = False):
    """Compile the host (gcc) and device (hipcc, gfx950) fill libraries next to their sources."""
    cpu = os.path.join(_HERE, "libsynth_cpu.so")
    hip = os.path.join(_HERE, "libsynth_hip.so")
    if force or not os.path.exists(cpu):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", cpu, os.path.join(_HERE, "gen_cpu.c")])
    if force or not os.path.exists(hip):
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-shared", "-fPIC", "-o", hip, os.path.join(_HERE, "gen_fill.hip")],
                              stderr=subprocess.DEVNULL)
    return cpu, hip


def _load():
    global _lib
    if _lib is None:
        path = os.path.join(_HERE, "libsynth_hip.so")
        if not os.path.exists(path):
            build_synth()
        lib = ctypes.CDLL(path)
        lib.synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                          ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p]
        lib.synth_fill_device.restype = ctypes.c_int
        _lib = lib
    return _lib


class DeviceWeights:
    """Torch tensors on the GPU: matrices in float32 / bfloat16, norm gains float32 (1 + shape.gain_std * recipe value; all ones when gain_std is 0)."""

    def __init__(self, shape, seed=gen.SEED_WEIGHTS, damp_skipped=1.0, skip_mask=None, device="cuda:0"):
        import torch
        self.shape = shape
        lib = _load()
        tdt = torch.float32 if shape.dtype == "f32" else torch.bfloat16
        code = 0 if shape.dtype == "f32" else 1
        shp = gen.tensor_shapes(shape)
        stream = torch.cuda.current_stream(torch.device(device)).cuda_stream

        def mat(layer, slot, scale=1.0):
            dims = shp[slot]
            if slot.endswith("norm"):   # a short vector: made by the host recipe and copied
                return torch.from_numpy(gen.gen_gain(seed, gen.tensor_id(shape, layer, slot), dims[0],
                                                     shape.gain_std)).to(device)
            t = torch.empty(dims, dtype=tdt, device=device)
            rc = lib.synth_fill_device(t.data_ptr(), code, seed, gen.tensor_id(shape, layer, slot), t.numel(),
                                       ctypes.c_float(float(gen.scale_f32(shape.init_std * scale))), stream)
            if rc != 0:
                raise RuntimeError(f"synth_fill_device failed: hip error {rc}")
            return t

        self.layers = []
        for l in range(shape.n_layers):
            bits = int(skip_mask[l]) if skip_mask is not None else 0
            damp = {"wo": damp_skipped if bits & 1 else 1.0, "w_down": damp_skipped if bits & 2 else 1.0}
            self.layers.append({slot: mat(l, slot, damp.get(slot, 1.0)) for slot in gen.LAYER_SLOTS})
        self.tok_emb = mat(None, "tok_emb")
        self.final_norm = mat(None, "final_norm")
        self.lm_head = mat(None, "lm_head")
        torch.cuda.synchronize()

    @staticmethod
    def _np(t):
        import torch
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    def to_host(self) -> gen.HostWeights:
        """Host copies (bf16 as uint16 bit patterns) for the CPU oracle."""
        return gen.HostWeights(self.shape, self._np(self.tok_emb), self._np(self.final_norm), self._np(self.lm_head),
                               [{k: np.ascontiguousarray(self._np(v)) for k, v in l.items()} for l in self.layers])

    def nbytes(self) -> int:
        n = sum(t.numel() * t.element_size() for t in (self.tok_emb, self.final_norm, self.lm_head))
        return n + sum(t.numel() * t.element_size() for l in self.layers for t in l.values())
