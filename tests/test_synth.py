"""The synthetic-input generators: the C fill equals the numpy definition bit for bit, the bf16 rounding is
round-to-nearest-even (checked against torch's own conversion), and the streams have the stated laws."""
import numpy as np
import torch

import synth


def test_c_fill_matches_numpy_definition():
    for dtype in ("f32", "bf16"):
        for tid, n in ((0, 1), (17, 1000), (515, 70001)):
            a = synth.gen_tensor(1234, tid, n, 0.02, dtype)
            b = synth.gen_tensor(1234, tid, n, 0.02, dtype, force_numpy=True)
            assert a.dtype == b.dtype and np.array_equal(a, b)


def test_distribution_moments():
    w = synth.gen_tensor_f32(1234, 3, 400000, 0.02)
    assert abs(w.mean()) < 2e-4
    assert abs(w.std() - 0.02) < 2e-4
    assert np.abs(w).max() <= 0.02 * 1020 / np.sqrt(synth.gen.BYTE_SUM_VAR) * 1.0001
    # different tensors and different seeds decorrelate
    w2 = synth.gen_tensor_f32(1234, 4, 400000, 0.02)
    assert abs(np.corrcoef(w, w2)[0, 1]) < 0.01


def test_bf16_rounding_is_rne_like_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 0.02,
                        np.array([1.0, 1.00390625, 1.005859375, -1.00390625, 3.0e-39, 0.0], np.float32)])
    mine = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, ref)
    assert np.array_equal(synth.bf16_bits_to_f32(mine), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_prompt_uniforms_mask():
    p = synth.gen_prompt(5678, 5000, 1024)
    assert p.dtype == np.int32 and p.min() >= 0 and p.max() < 1024 and len(np.unique(p)) > 900
    u = synth.gen_uniforms(91011, 100000)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5e-3 and abs(u.var() - 1 / 12) < 2e-3
    for name, s in synth.CONFIGS.items():
        m = synth.gen_skip_mask(s)
        assert m.dtype == np.uint8 and m.shape == (s.n_layers,)
        assert int((m == 3).sum()) == s.n_skip and set(np.unique(m)) <= {0, 3}
    assert list(np.nonzero(synth.gen_skip_mask(synth.CONFIGS["tiny"]))[0]) == [1, 2]


def test_config_table_matches_declared_workloads():
    c = synth.CONFIGS
    assert (c["7b"].n_layers, c["7b"].d_model, c["7b"].d_ffn, c["7b"].vocab, c["7b"].K) == (32, 4096, 11008, 32000, 4)
    assert (c["13b"].n_layers, c["13b"].d_model, c["13b"].d_ffn, c["13b"].K, c["13b"].mode) == (40, 5120, 13824, 6, "sample")
    assert (c["l3-8b"].n_kv_heads, c["l3-8b"].vocab, c["l3-8b"].n_prompt) == (8, 128256, 4096)
    assert (c["70b"].n_layers, c["70b"].n_heads, c["70b"].n_kv_heads, c["70b"].d_ffn) == (80, 64, 8, 28672)
    for s in c.values():
        assert s.n_heads * s.head_dim == s.d_model


def test_sublayer_mask_counts_and_determinism():
    s = synth.CONFIGS["13b"]
    m = synth.gen_sublayer_mask(s, 0.5, 0.35)
    assert m.dtype == np.uint8 and m.shape == (s.n_layers,) and int(m.max()) <= 3
    assert int(((m & 1) != 0).sum()) == 20 and int(((m & 2) != 0).sum()) == 14
    assert np.array_equal(m, synth.gen_sublayer_mask(s, 0.5, 0.35))
    assert not np.array_equal(m, synth.gen_sublayer_mask(s, 0.5, 0.35, seed=7))
    assert not synth.gen_sublayer_mask(s, 0.0, 0.0).any()
