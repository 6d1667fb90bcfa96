"""The prompt's two paths on the GPU: the weight-streaming forward kernel 16 rows at a time, and the matrix-matrix
path (panels of rows through a GEMM per projection).  Both must write the same cache and produce the same last-row
logits, bit for bit, as each other and as one-row decoding of the same tokens; the oracle comparisons of long prompts in
the other GPU test files go through the matrix-matrix path by default."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2602_05499_amd as P
    P.load_library()
    return P


def _prefill(P, ses, prompt, mode, n_decode=3):
    import torch
    ses.set_prefill_mode(mode)
    ses.keep_logits(True)
    ses.prefill(prompt)
    z = ses.dump_logits(P.SD_LOGITS_VERIFY, 1)[0].copy()
    _, st = ses.read()
    kv = ses.kv.clone()
    zs = []
    for _ in range(n_decode):
        ses.decode()
        zs.append(ses.dump_logits(P.SD_LOGITS_VERIFY, 1)[0].copy())
    toks, _ = ses.read()
    return z, st["t_last"], kv, zs, toks


def _cache_rows(ses, s, kv, n):
    """The first n positions of every layer's key and value planes, as raw 16-bit words."""
    import torch
    shp = (s.n_layers, 2, s.n_kv_heads, ses.max_seq, s.head_dim)
    return kv.view(torch.int16)[:int(np.prod(shp))].view(shp)[:, :, :, :n]


def _both_paths(P, s, lengths, damp=1.0):
    import torch
    from synth.device import DeviceWeights
    mask = synth.gen_skip_mask(s)
    dw = DeviceWeights(s, damp_skipped=damp, skip_mask=mask)
    ses = P.Session(s, dw, mask, max_seq=max(lengths) + 16, max_k=4)
    for n in lengths:
        prompt = synth.gen_prompt(100 + n, n, s.vocab)
        a = _prefill(P, ses, prompt, 0)
        b = _prefill(P, ses, prompt, 1)          # weights read from the tiled copy (the Session's default)
        assert ses.tiled is not None
        ses.set_tiled_weights(False)
        c = _prefill(P, ses, prompt, 1)          # weights read from the caller's row-major matrices
        ses.set_tiled_weights(True)
        assert np.array_equal(b[0], c[0]) and b[1] == c[1] and torch.equal(b[2], c[2]), (s.name, n, "tiled copy or not")
        # ... and the decode steps that follow (their O / down projections read the copy where the widths allow)
        assert all(np.array_equal(x, y) for x, y in zip(b[3], c[3])) and np.array_equal(b[4], c[4]), (s.name, n, "decode, tiled copy or not")
        assert np.isfinite(a[0]).all()
        assert np.array_equal(a[0], b[0]), (s.name, n, "last-row logits", float(np.abs(a[0] - b[0]).max()))
        assert a[1] == b[1]
        assert torch.equal(_cache_rows(ses, s, a[2], n), _cache_rows(ses, s, b[2], n)), (s.name, n, "cache rows")
        for za, zb in zip(a[3], b[3]):
            assert np.array_equal(za, zb), (s.name, n, "decode after the prompt")
        assert np.array_equal(a[4], b[4])
    ses.close()
    del ses, dw
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["gqa_bf16", "hd32", "hd64"])
def test_matrix_prompt_path_equals_chunk_path_small_shapes(gpu, small_shapes, name):
    """Prompt lengths around the 16-row chunk, the 64-row tile and the 128-position attention split, head_dim 16, 32 and
    64, grouped and plain heads, seeded norm gains: cache rows, last-row logits and the following decode steps equal."""
    if name == "gqa_bf16":
        s = small_shapes["gqa_bf16"].with_(init_std=0.3)
    elif name == "hd32":
        s = small_shapes["gqa_bf16"].with_(name="hd32_bf16", n_heads=2, n_kv_heads=1, head_dim=32, init_std=0.3)
    else:
        s = synth.CONFIGS["tiny"].with_(name="tiny_bf16", dtype="bf16", d_ffn=704, gain_std=0.1, init_std=0.05)
    _both_paths(gpu, s, [1, 17, 63, 64, 65, 130, 200])


@pytest.mark.timeout(600)
def test_matrix_prompt_path_equals_chunk_path_at_7b_width(gpu):
    """The benchmark's matrices (two layers, head_dim 128): a 650-token prompt (two panels, the last 64-row tile and the
    last 16-row chunk ragged) and a 100-token one."""
    s = synth.CONFIGS["7b"].with_(name="7b-2layers", n_layers=2, n_skip=1, gain_std=0.1)
    _both_paths(gpu, s, [650, 100])


@pytest.mark.timeout(600)
def test_matrix_prompt_path_at_llama3_width(gpu):
    """Grouped queries at head_dim 128 (four query heads per KV head, 64 query vectors per chunk and KV head)."""
    s = synth.CONFIGS["l3-8b"].with_(name="l3-8b-2layers", n_layers=2, n_skip=1, gain_std=0.1)
    _both_paths(gpu, s, [300])


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,n", [("13b", 200), ("70b", 130)])
def test_matrix_prompt_path_at_other_baseline_widths(gpu, name, n):
    """d 5120 / F 13824 / 40 heads (a weight row of 5 blocks, tile counts that are no multiple of a workgroup's) and
    d 8192 / F 28672 / 64 query heads on 8 KV heads, two layers each."""
    s = synth.CONFIGS[name].with_(name=name + "-2layers", n_layers=2, n_skip=1, gain_std=0.1)
    _both_paths(gpu, s, [n])


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,lengths", [("7b", [5, 8, 16, 17, 31, 32, 33, 47, 48, 49, 64, 66, 129, 257, 320]),
                                           ("13b", [5, 19, 40, 70]),
                                           ("l3-8b", [6, 18, 50, 96]),
                                           ("70b", [7, 30, 64])])
def test_short_prompts_at_baseline_widths(gpu, name, lengths):
    """Short panels at the full widths, two layers: the GEMM instances that multiply one, two or all four column tiles
    of a panel, QKV's shares dealt to workgroups and summed by the finishing kernel, and every tiles-per-wave choice of
    the launch cost model (panels of 1 to 5 column tiles' worth of rows)."""
    s = synth.CONFIGS[name].with_(name=name + "-2layers", n_layers=2, n_skip=1, gain_std=0.1)
    _both_paths(gpu, s, lengths)


@pytest.mark.timeout(900)
def test_matrix_prompt_path_on_the_benchmark_workload(gpu):
    """The configuration bench.py times (7B shape, all 32 layers, 512-token prompt, 512-row panel): both prompt paths
    give the same cache, logits and following decode steps."""
    _both_paths(gpu, synth.CONFIGS["7b"], [synth.CONFIGS["7b"].n_prompt])


def test_matrix_prompt_rows_equal_one_row_decoding_of_the_same_tokens(gpu, small_shapes):
    """Row i of a prompt is what the one-row decode kernel computes for token i after the prefix: a prompt of n tokens on
    the matrix-matrix path against a prompt of m < n tokens followed by n - m teacher-forced one-row decode steps."""
    import torch
    from synth.device import DeviceWeights
    P = gpu
    for s, n, m in ((small_shapes["gqa_bf16"].with_(init_std=0.3), 150, 120),
                    (synth.CONFIGS["7b"].with_(name="7b-2layers", n_layers=2, n_skip=1, gain_std=0.1), 140, 131)):
        mask = synth.gen_skip_mask(s)
        dw = DeviceWeights(s, skip_mask=mask)
        ses = P.Session(s, dw, mask, max_seq=n + 16, max_k=4)
        prompt = synth.gen_prompt(77, n, s.vocab)
        ses.set_prefill_mode(1)
        ses.keep_logits(True)
        ses.prefill(prompt)
        z_ref = ses.dump_logits(P.SD_LOGITS_VERIFY, 1)[0].copy()
        ses.sync()
        kv_ref = _cache_rows(ses, s, ses.kv.clone(), n)
        ses.prefill(prompt[:m])
        for i in range(m, n):
            ses.set_pending(i, int(prompt[i]))
            ses.decode()
        z = ses.dump_logits(P.SD_LOGITS_VERIFY, 1)[0].copy()
        ses.sync()
        assert torch.equal(kv_ref, _cache_rows(ses, s, ses.kv, n)), (s.name, "cache rows")
        assert np.array_equal(z_ref, z), (s.name, "logits of the last row")
        ses.close()
        del ses, dw
        torch.cuda.empty_cache()


def test_matrix_prompt_path_panel_boundaries(gpu, small_shapes):
    """Prompts around the 512-row panel and over several panels (small shape, so the chunk path stays quick)."""
    s = small_shapes["gqa_bf16"].with_(init_std=0.3)
    _both_paths(gpu, s, [511, 512, 513, 1100])


def test_tiled_weights_argument_errors(gpu, small_shapes):
    from synth.device import DeviceWeights
    P = gpu
    s = small_shapes["gqa_bf16"]
    mask = synth.gen_skip_mask(s)
    ses = P.Session(s, DeviceWeights(s, skip_mask=mask), mask, max_seq=64, tiled_weights=False)
    need = P.binding.sd_tiled_weights_bytes(ses.cfg)
    per_layer = 2 * (s.d_model * (s.n_heads + 2 * s.n_kv_heads) * s.head_dim + s.d_model * s.n_heads * s.head_dim
                     + 3 * s.d_ffn * s.d_model)
    assert need >= s.n_layers * per_layer and need < s.n_layers * (per_layer + 4 * 256)
    buf = ses.torch.empty(need + 256, dtype=ses.torch.uint8, device=ses.kv.device)
    B = P.binding
    assert B.sd_set_tiled_weights(ses.ctx, buf.data_ptr(), need - 1) == P.SD_ENOMEM
    assert B.sd_set_tiled_weights(ses.ctx, buf.data_ptr() + 16, need) == P.SD_EINVAL      # not 256-byte aligned
    assert B.sd_set_tiled_weights(None, buf.data_ptr(), need) == P.SD_EINVAL
    assert B.sd_set_tiled_weights(ses.ctx, buf.data_ptr(), need) == P.SD_OK
    assert B.sd_set_tiled_weights(ses.ctx, None, 0) == P.SD_OK                             # detach
    ses.sync()
    ses.close()


def test_matrix_prompt_path_is_refused_for_float32_storage(gpu, small_shapes):
    from synth.device import DeviceWeights
    P = gpu
    s = small_shapes["mha_f32"]
    mask = synth.gen_skip_mask(s)
    ses = P.Session(s, DeviceWeights(s, skip_mask=mask), mask, max_seq=64)
    with pytest.raises(P.SdError) as e:
        ses.set_prefill_mode(1)
    assert e.value.code == P.SD_EINVAL
    ses.set_prefill_mode(-1)
    assert ses.tiled is None and P.binding.sd_tiled_weights_bytes(ses.cfg) == 0      # no tiled copy for float32 storage
    assert P.binding.sd_set_tiled_weights(ses.ctx, ses.kv.data_ptr(), 1 << 20) == P.SD_EINVAL
    out, _ = ses.generate(synth.gen_prompt(3, 50, s.vocab), 6, 2)     # 50 rows: still the chunk path
    assert len(out) == 6
    ses.close()
