"""sd_init_static: a context whose workspace is the library's own static device array (for callers that cannot
allocate) against sd_init with a caller-allocated workspace -- same inputs, results bit for bit, through the C-ABI.
Two static contexts in a row, the second for a smaller model: the array still holds the first one's contents."""
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


def _run(P, shape, dw, mask, K, G, n_prompt, static, mode, uniforms):
    """Prefill, speculative steps (logits of the last verify forward kept), then a few plain decode steps."""
    ses = P.Session(shape, dw, mask, max_seq=n_prompt + G + K + 8, max_k=K, static_workspace=static)
    assert (ses.ws is None) == static
    prompt = synth.gen_prompt(synth.SEED_PROMPT, n_prompt, shape.vocab)
    ses.keep_logits(True)
    toks, stats = ses.generate(prompt, G, K, mode, uniforms)
    zq = ses.dump_logits(P.SD_LOGITS_DRAFT, K).copy()
    zp = ses.dump_logits(P.SD_LOGITS_VERIFY, K + 1).copy()
    d = ses.dump_draft(K).copy()
    for i in range(3):
        ses.decode(mode, None if uniforms is None else uniforms[-1 - i:len(uniforms) - i])
    z1 = ses.dump_logits(P.SD_LOGITS_VERIFY, 1).copy()
    toks2, stats2 = ses.read()
    kv = ses.kv.clone()
    ses.close()
    return toks, stats, zq, zp, d, z1, toks2, stats2, kv


def _same(a, b):
    import torch
    for x, y in zip(a, b):
        if isinstance(x, dict):
            assert x == y
        elif isinstance(x, torch.Tensor):
            assert torch.equal(x, y)
        else:
            assert np.array_equal(x, y)


def test_static_workspace_context_equals_caller_workspace_context(gpu, small_shapes):
    import torch
    from synth.device import DeviceWeights
    P = gpu
    big = synth.CONFIGS["7b"].with_(name="7b-2layers", n_layers=2, n_skip=1)      # the benchmark's widths, bf16
    small = small_shapes["gqa_bf16"].with_(init_std=0.3)
    tiny = small_shapes["v16"]
    # (shape, K, G, prompt, mode): the second and third calls are for smaller models than the one before
    for shape, K, G, n_prompt, mode in ((big, 4, 11, 140, P.SD_GREEDY), (small, 3, 14, 9, P.SD_GREEDY),
                                        (tiny, 3, 12, 5, P.SD_SAMPLE)):
        mask = synth.gen_skip_mask(shape)
        dw = DeviceWeights(shape, damp_skipped=0.3, skip_mask=mask)
        uni = synth.gen_uniforms(synth.SEED_UNIFORMS, 1 + (2 * K + 1) * G + 4) if mode == P.SD_SAMPLE else None
        ref = _run(P, shape, dw, mask, K, G, n_prompt, False, mode, uni)
        got = _run(P, shape, dw, mask, K, G, n_prompt, True, mode, uni)
        _same(ref, got)
        assert len(got[0]) == G and np.isfinite(got[3]).all()
        del dw
        torch.cuda.empty_cache()


def test_static_workspace_limits_and_single_use(gpu, small_shapes):
    from synth.device import DeviceWeights
    P = gpu
    s = small_shapes["mha_f32"]
    mask = synth.gen_skip_mask(s)
    dw = DeviceWeights(s, skip_mask=mask)
    a = P.Session(s, dw, mask, max_seq=64, static_workspace=True)
    with pytest.raises(P.SdError) as e:                   # the device's array is taken
        P.Session(s, dw, mask, max_seq=64, static_workspace=True)
    assert e.value.code == P.SD_ESTATE
    a.close()
    b = P.Session(s, dw, mask, max_seq=64, static_workspace=True)     # free again
    out, _ = b.generate(synth.gen_prompt(3, 9, s.vocab), 8, 2)
    assert len(out) == 8
    b.close()
    # a configuration whose workspace exceeds the array: refused with SD_ENOMEM before anything is touched
    with pytest.raises(P.SdError) as e:
        P.Session(s, dw, mask, max_seq=1 << 20, static_workspace=True)
    assert e.value.code == P.SD_ENOMEM
