"""FIT layer scores (Eq. 11; Alg. 1 Stage A) on the GPU against the oracle: the squared gradient norms of every layer's
attention and feed-forward sub-layer over a small seeded calibration set, the samples' losses, and the prune set that
follows from them.  The GPU works in float32 with bfloat16 weights taken exactly, the oracle in float64 on the same
stored values: scores agree to a relative 1e-3 (asserted; what is measured is printed), losses to 1e-5."""
import ctypes

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

RTOL_SCORE = 1e-3
ATOL_LOSS = 1e-5


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2602_05499_amd as P
    P.load_library()
    return P


def _gpu_scores(P, s, dw, samples):
    import torch
    from paper_2602_05499_amd import binding as B
    from paper_2602_05499_amd.session import make_config, make_weights
    cfg = make_config(s, max_seq=64, max_k=0, max_out=1)
    wts, keep = make_weights(s, dw)
    toks = np.asarray(samples, np.int32)
    need = B.sd_fit_workspace_bytes(cfg, toks.shape[1])
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    rc, ta, tf, ls = B.sd_fit_scores(cfg, wts, toks, ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
    assert rc == B.SD_OK, rc
    del keep
    return ta, tf, ls


def _compare(P, s, T, n_samples, seed=31):
    import torch
    from synth.device import DeviceWeights
    from oracle.fit import fit_scores, prune_set
    dw = DeviceWeights(s)
    samples = [synth.gen_prompt(seed + i, T, s.vocab) for i in range(n_samples)]
    ta, tf, ls = _gpu_scores(P, s, dw, samples)
    ra, rf, rl = fit_scores(s, dw.to_host(), samples)
    ea, ef = np.abs(ta - ra) / ra, np.abs(tf - rf) / rf
    print(f"{s.name} T={T} N={n_samples}: scores attn {ra.min():.3e}..{ra.max():.3e} ffn {rf.min():.3e}..{rf.max():.3e}; "
          f"worst relative error attn {ea.max():.2e} ffn {ef.max():.2e}; losses {rl.round(4).tolist()} "
          f"worst |dloss| {np.abs(ls - rl).max():.2e}", flush=True)
    assert np.isfinite(ta).all() and np.isfinite(tf).all()
    assert ea.max() <= RTOL_SCORE and ef.max() <= RTOL_SCORE
    assert np.abs(ls - rl).max() <= ATOL_LOSS * max(1.0, np.abs(rl).max())
    # the ranking: identical wherever the oracle's scores are further apart than the tolerance
    from paper_2602_05499_amd import binding as B
    for ratio in (0.25, 0.5):
        rc, mask = B.sd_fit_prune_mask(ta, tf, ratio)
        assert rc == B.SD_OK
        want = prune_set(ra + rf, ratio)
        got = sorted(int(l) for l in np.nonzero(mask)[0])
        if got != want:
            tot = np.sort(ra + rf)
            gaps = np.diff(tot) / tot[1:]
            assert gaps.min() < 2 * RTOL_SCORE, (got, want)
        assert all(mask[l] == 3 for l in got) and len(got) == int(np.floor(ratio * s.n_layers + 1e-12))
    del dw
    torch.cuda.empty_cache()
    return ta, tf


def test_fit_scores_small_shapes_against_oracle(gpu, small_shapes):
    """Grouped KV heads (8 query heads on 2 KV heads of 16), four layers, seeded norm gains; a sequence length that is
    no multiple of anything (37: ragged 64-row tile, ragged Gram blocks) and one of exactly 64; two samples."""
    s = small_shapes["gqa_bf16"].with_(name="fit_gqa", vocab=96, init_std=0.15)
    _compare(gpu, s, 37, 2)
    _compare(gpu, s, 64, 1)


def test_fit_scores_long_sequence(gpu, small_shapes):
    """A 600-token sequence: more rows than one 512-row stretch of anything (ten 64-row GEMM tiles, 10 x 10 Gram blocks,
    attention rows of up to 600 probabilities)."""
    s = small_shapes["gqa_bf16"].with_(name="fit_gqa_long", vocab=96, init_std=0.15)
    _compare(gpu, s, 600, 1)


def test_fit_scores_head_dim_64_and_several_panels_of_keys(gpu):
    """head_dim 64, d 256, a 130-token sequence (three 64-row tiles, attention rows longer than a wave)."""
    s = synth.CONFIGS["tiny"].with_(name="fit_hd64", dtype="bf16", d_ffn=704, vocab=512, gain_std=0.1, init_std=0.05)
    _compare(gpu, s, 130, 1)


@pytest.mark.timeout(900)
def test_fit_scores_at_7b_width(gpu):
    """The benchmark's matrices (two layers: d 4096, 32 heads of 128, F 11008, V 32000), 48 tokens."""
    s = synth.CONFIGS["7b"].with_(name="fit_7b_2layers", n_layers=2, n_skip=1, gain_std=0.1)
    _compare(gpu, s, 48, 1)


@pytest.mark.timeout(900)
def test_fit_scores_on_the_benchmark_model(gpu):
    """All 32 layers of the 7B shape, a 512-token sequence (the configuration `bench.py --fit` times).  The oracle cannot
    form 32 layers of float64 weight gradients in test time, so what holds at any size is checked: scores finite and
    positive, the loss near ln(V) for random-init weights, two runs equal to 1e-5 relative (float32 atomic sums), and the
    mean over two samples equal to the mean of the single-sample runs."""
    import torch
    from paper_2602_05499_amd.session import fit_scores
    from synth.device import DeviceWeights
    s = synth.CONFIGS["7b"]
    dw = DeviceWeights(s)
    a, b = synth.gen_prompt(71, 512, s.vocab), synth.gen_prompt(72, 512, s.vocab)
    ta1, tf1, l1 = fit_scores(s, dw, [a])
    ta1b, tf1b, _ = fit_scores(s, dw, [a])
    ta2, tf2, l2 = fit_scores(s, dw, [b])
    tab, tfb, lab = fit_scores(s, dw, [a, b])
    for t in (ta1, tf1, ta2, tf2):
        assert np.isfinite(t).all() and (t > 0).all()
    assert np.abs(ta1 - ta1b).max() <= 1e-5 * ta1.max() and np.abs(tf1 - tf1b).max() <= 1e-5 * tf1.max()
    assert np.allclose(tab, (ta1 + ta2) / 2, rtol=1e-5) and np.allclose(tfb, (tf1 + tf2) / 2, rtol=1e-5)
    assert np.allclose(lab, [l1[0], l2[0]], rtol=1e-6)
    assert abs(l1[0] - np.log(s.vocab)) < 2.0
    del dw
    torch.cuda.empty_cache()


def test_stage_a_then_stage_b(gpu, small_shapes):
    """Alg. 1 end to end on the GPU: FIT scores of a small model, the prune mask at ratio 1/2, and speculative decoding
    with the draft that mask defines -- lossless, i.e. equal to plain greedy decoding of the target."""
    import torch
    from paper_2602_05499_amd import binding as B
    from paper_2602_05499_amd.session import fit_scores
    from synth.device import DeviceWeights
    P = gpu
    s = small_shapes["gqa_bf16"].with_(name="fit_sd", vocab=96, init_std=0.15)
    dw = DeviceWeights(s)
    ta, tf, _ = fit_scores(s, dw, [synth.gen_prompt(5 + i, 40, s.vocab) for i in range(3)])
    rc, mask = B.sd_fit_prune_mask(ta, tf, 0.5)
    assert rc == B.SD_OK and int((mask == 3).sum()) == s.n_layers // 2
    ses = P.Session(s, dw, mask, max_seq=96, max_k=4)
    prompt = synth.gen_prompt(9, 12, s.vocab)
    out, stats = ses.generate(prompt, 30, 4)
    plain, _ = ses.generate(prompt, 30, 0)
    assert np.array_equal(out, plain) and stats["drafted"] > 0
    ses.close()
    del dw
    torch.cuda.empty_cache()


def test_fit_argument_errors(gpu, small_shapes):
    import torch
    from paper_2602_05499_amd import binding as B
    from paper_2602_05499_amd.session import make_config
    s = small_shapes["gqa_bf16"]                 # vocabulary 80: no multiple of 32
    assert B.sd_fit_workspace_bytes(make_config(s, max_seq=64, max_k=0, max_out=1), 16) == 0
    s32 = small_shapes["mha_f32"]                # float32 storage
    assert B.sd_fit_workspace_bytes(make_config(s32, max_seq=64, max_k=0, max_out=1), 16) == 0
    ok = s.with_(vocab=96)
    cfg = make_config(ok, max_seq=64, max_k=0, max_out=1)
    assert B.sd_fit_workspace_bytes(cfg, 1) == 0 and B.sd_fit_workspace_bytes(cfg, 2049) == 0
    assert B.sd_fit_workspace_bytes(cfg, 16) > 0
