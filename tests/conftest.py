import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def small_shapes():
    """Small model shapes that keep the CPU suite fast but still exercise MHA, GQA, f32 and bf16.  All but the tiny
    benchmark configuration have seeded RMSNorm gains that differ per layer, per norm and per column (1 +- up to 0.5), so
    that a gain vector that is dropped, swapped or shifted changes the result."""
    import synth
    base = synth.CONFIGS["tiny"]
    return {
        "tiny": base,
        "mha_f32": base.with_(name="mha_f32", n_layers=3, d_model=64, n_heads=4, n_kv_heads=4, head_dim=16,
                              d_ffn=176, vocab=96, init_std=0.08, gain_std=0.1, n_skip=1, skip_layers=(1,), n_prompt=9, n_gen=24),
        "gqa_bf16": base.with_(name="gqa_bf16", n_layers=4, d_model=64, n_heads=8, n_kv_heads=2, head_dim=16,
                               d_ffn=160, vocab=80, dtype="bf16", init_std=0.1, gain_std=0.1, n_skip=2, skip_layers=(0, 2),
                               n_prompt=7, n_gen=20),
        "v16": base.with_(name="v16", n_layers=2, d_model=32, n_heads=2, n_kv_heads=2, head_dim=16, d_ffn=64,
                          vocab=16, init_std=0.25, gain_std=0.1, n_skip=1, skip_layers=(1,), K=3, mode="sample", n_prompt=5,
                          n_gen=8),
    }
