"""The C-ABI boundary without a GPU: the library loads, exports exactly what include/sdfp.h declares, the Python
binding carries the same names, the host-only size functions follow the documented layout, and the product path
has no way around the HIP library (no oracle import, a loud failure when the library is missing).
No call here touches a device."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sdfp.h")


def declared_functions():
    """Names of the functions include/sdfp.h declares (comments stripped first)."""
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    names = re.findall(r"\b(sd_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    from paper_2602_05499_amd import binding as B
    if not os.path.exists(B.library_path()):      # a fresh checkout: the built library is not under version control
        from paper_2602_05499_amd.session import build_library
        build_library()
    return B.load_library()


def _config(B, **over):
    base = dict(n_layers=4, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=704, vocab=1024, max_seq=128,
                max_k=4, dtype=B.SD_BF16, max_out=256, rms_eps=1e-5, rope_theta=10000.0, temperature=1.0)
    base.update(over)
    order = [n for n, _ in B.SdConfig._fields_]
    return B.SdConfig(*[base[n] for n in order])


def test_header_declares_the_entry_points_of_the_step():
    names = declared_functions()
    for must in ("sd_kv_bytes", "sd_workspace_bytes", "sd_init", "sd_set_skip_mask", "sd_prefill", "sd_draft",
                 "sd_verify", "sd_accept", "sd_rollback", "sd_decode", "sd_read", "sd_free"):
        assert must in names, must


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        fn = getattr(lib, name)          # dlsym; raises AttributeError when the symbol is missing
        assert ctypes.cast(fn, ctypes.c_void_p).value, name


def test_library_exports_nothing_undeclared(lib):
    from paper_2602_05499_amd import binding as B
    out = subprocess.run(["nm", "-D", "--defined-only", B.library_path()], capture_output=True, text=True, check=True)
    exported = {line.split()[-1] for line in out.stdout.splitlines() if " T " in line}
    api = {s for s in exported if s.startswith("sd_")}
    assert api == set(declared_functions())


def test_binding_has_the_same_names(lib):
    import paper_2602_05499_amd as P
    from paper_2602_05499_amd import binding as B
    assert sorted(P.EXPORTED_SYMBOLS) == declared_functions()     # the list that build() checks after linking
    for name in declared_functions():
        assert callable(getattr(B, name, None)), f"binding lacks {name}"
        assert getattr(lib, name).argtypes is not None, f"{name}: argument types not declared"


def test_size_functions_follow_the_documented_layout(lib):
    from paper_2602_05499_amd import binding as B
    for dtype, esize in ((B.SD_BF16, 2), (B.SD_F32, 4)):
        cfg = _config(B, dtype=dtype, d_ffn=704 if dtype == B.SD_BF16 else 688)
        kv = B.sd_kv_bytes(cfg)
        exact = cfg.n_layers * 2 * cfg.n_kv_heads * cfg.max_seq * cfg.head_dim * esize   # [layer][k|v][kv head][pos][dim]
        assert exact <= kv < exact + 4096
        assert B.sd_workspace_bytes(cfg) > 0
    # a longer cache costs exactly its rows; the workspace grows with it (attention partials per split)
    a, b = _config(B), _config(B, max_seq=256)
    assert B.sd_kv_bytes(b) - B.sd_kv_bytes(a) == a.n_layers * 2 * a.n_kv_heads * 128 * a.head_dim * 2
    assert B.sd_workspace_bytes(b) >= B.sd_workspace_bytes(a)
    # the optional tiled copy is as large as the layer matrices (each projection rounded up to 256 bytes); none for float32
    c = _config(B, dtype=B.SD_BF16, d_ffn=704)
    hq, hk = c.n_heads * c.head_dim, c.n_kv_heads * c.head_dim
    mats = 2 * ((hq + 2 * hk) * c.d_model + c.d_model * hq + 3 * c.d_ffn * c.d_model)
    assert c.n_layers * mats <= B.sd_tiled_weights_bytes(c) < c.n_layers * (mats + 4 * 256)
    assert B.sd_tiled_weights_bytes(_config(B, dtype=B.SD_F32, d_ffn=688)) == 0
    assert B.sd_tiled_weights_bytes(_config(B, head_dim=48)) == 0


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(head_dim=256), dict(n_heads=3, n_kv_heads=2), dict(max_k=9),
                                 dict(d_model=250), dict(dtype=7), dict(max_seq=3), dict(temperature=0.0),
                                 dict(n_layers=0), dict(vocab=0)])
def test_invalid_configurations_are_refused_on_the_host(lib, bad):
    from paper_2602_05499_amd import binding as B
    cfg = _config(B, **bad)
    assert B.sd_kv_bytes(cfg) == 0 and B.sd_workspace_bytes(cfg) == 0


def test_error_strings(lib):
    from paper_2602_05499_amd import binding as B
    seen = set()
    for code in (B.SD_OK, B.SD_EINVAL, B.SD_ECAPACITY, B.SD_ESTATE, B.SD_EHIP, B.SD_ENOMEM, B.SD_ETIMEOUT):
        s = B.sd_strerror(code)
        assert s and s not in seen
        seen.add(s)


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2602_05499_amd import binding as B
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "library_path", lambda: os.path.join(ROOT, "no_such_dir", "libsdfp.so"))
    with pytest.raises(ImportError):
        B.load_library()


def test_product_code_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_05499_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "oracle/" not in text, f


# ---- argument, state and capacity errors are found on the host, before anything is enqueued ------------------------
# sd_init performs no GPU work and keeps the pointers it is given without reading them, so a context over made-up
# (aligned, non-null) device addresses can be created here; every call below must return before it would touch them.
def _fake_context(B, **over):
    cfg = _config(B, **over)
    L = cfg.n_layers
    fake = 0x7F0000000000
    arrs = [(ctypes.c_void_p * L)(*[fake + 4096 * (i + 1) for i in range(L)]) for _ in range(9)]
    w = B.SdWeights(fake, fake + 256, fake + 512, *[ctypes.cast(a, ctypes.POINTER(ctypes.c_void_p)) for a in arrs])
    return cfg, w, arrs, fake


def test_init_refuses_bad_arguments_on_the_host(lib):
    from paper_2602_05499_amd import binding as B
    cfg, w, arrs, fake = _fake_context(B)
    kvb, wsb = B.sd_kv_bytes(cfg), B.sd_workspace_bytes(cfg)
    rc, ctx = B.sd_init(cfg, w, None, fake, kvb, fake, wsb, None)
    assert rc == B.SD_OK and ctx.value
    B.sd_free(ctx)
    assert B.sd_init(None, w, None, fake, kvb, fake, wsb, None)[0] == B.SD_EINVAL
    assert B.sd_init(cfg, None, None, fake, kvb, fake, wsb, None)[0] == B.SD_EINVAL
    assert B.sd_init(cfg, w, None, None, kvb, fake, wsb, None)[0] == B.SD_EINVAL
    assert B.sd_init(cfg, w, None, fake, kvb, None, wsb, None)[0] == B.SD_EINVAL
    assert B.sd_init(cfg, w, None, fake + 8, kvb, fake, wsb, None)[0] == B.SD_EINVAL      # misaligned KV buffer
    assert B.sd_init(cfg, w, None, fake, kvb, fake + 8, wsb, None)[0] == B.SD_EINVAL      # misaligned workspace
    assert B.sd_init(cfg, w, None, fake, kvb - 1, fake, wsb, None)[0] == B.SD_ENOMEM
    assert B.sd_init(cfg, w, None, fake, kvb, fake, wsb - 1, None)[0] == B.SD_ENOMEM
    bad = _config(B, head_dim=48)
    assert B.sd_init(bad, w, None, fake, kvb, fake, wsb, None)[0] == B.SD_EINVAL
    arrs[3][1] = None                                                                      # one layer's wv missing
    assert B.sd_init(cfg, w, None, fake, kvb, fake, wsb, None)[0] == B.SD_EINVAL
    assert lib.sd_init(None, ctypes.byref(cfg), ctypes.byref(w), None, fake, kvb, fake, wsb, None) == B.SD_EINVAL


def test_null_context_is_refused_by_every_call(lib):
    from paper_2602_05499_amd import binding as B
    import numpy as np
    null = ctypes.c_void_p(None)
    one = np.zeros(4, np.int32)
    u = np.zeros(4, np.float32)
    assert B.sd_prefill(null, one, B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_draft(null, 1, B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_verify(null) == B.SD_EINVAL
    assert B.sd_accept(null, B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_rollback(null) == B.SD_EINVAL
    assert B.sd_decode(null, B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_set_pending(null, 1, 0) == B.SD_EINVAL
    assert B.sd_set_draft(null, one) == B.SD_EINVAL
    assert B.sd_set_skip_mask(null, np.zeros(4, np.uint8)) == B.SD_EINVAL
    assert B.sd_read(null, one, None, None) == B.SD_EINVAL
    assert B.sd_dump_logits(null, B.SD_LOGITS_VERIFY, u) == B.SD_EINVAL
    assert B.sd_dump_draft(null, one) == B.SD_EINVAL
    assert B.sd_keep_logits(null, 1) == B.SD_EINVAL
    assert B.sd_set_spin_limit(null, 5) == B.SD_EINVAL
    assert B.sd_set_turn_span(null, 0) == B.SD_EINVAL
    assert B.sd_set_prefill_mode(null, 0) == B.SD_EINVAL
    assert B.sd_set_tiled_weights(null, None, 0) == B.SD_EINVAL
    assert B.sd_sync(null) == B.SD_EINVAL
    assert B.sd_last_hip_error(null) == 0
    B.sd_free(null)                                                                        # a no-op


def test_call_order_and_ranges_are_checked_on_the_host(lib):
    """On a context that has not seen a prompt every step call is out of order, and argument errors win over that:
    all of it is decided before any GPU work (there is no GPU here and the context's pointers are made up)."""
    from paper_2602_05499_amd import binding as B
    import numpy as np
    cfg, w, arrs, fake = _fake_context(B, max_k=4, max_seq=32)
    rc, ctx = B.sd_init(cfg, w, np.array([0, 3, 1, 2], np.uint8), fake, B.sd_kv_bytes(cfg), fake,
                        B.sd_workspace_bytes(cfg), None)
    assert rc == B.SD_OK
    u = np.full(8, 0.5, np.float32)
    # ranges first
    assert B.sd_draft(ctx, 5, B.SD_GREEDY) == B.SD_EINVAL            # K > max_k
    assert B.sd_draft(ctx, -1, B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_draft(ctx, 2, 7) == B.SD_EINVAL                      # unknown mode
    assert B.sd_accept(ctx, 7) == B.SD_EINVAL
    assert B.sd_set_draft(ctx, np.zeros(5, np.int32)) == B.SD_EINVAL
    assert B.sd_set_pending(ctx, 4, cfg.vocab) == B.SD_EINVAL        # token out of the vocabulary
    assert B.sd_set_spin_limit(ctx, 0) == B.SD_EINVAL
    assert B.sd_set_turn_span(ctx, 2) == B.SD_EINVAL
    # then the call order: nothing but sd_prefill may follow sd_init
    assert B.sd_draft(ctx, 2, B.SD_GREEDY) == B.SD_ESTATE
    assert B.sd_verify(ctx) == B.SD_ESTATE
    assert B.sd_accept(ctx, B.SD_GREEDY) == B.SD_ESTATE
    assert B.sd_rollback(ctx) == B.SD_ESTATE
    assert B.sd_decode(ctx, B.SD_GREEDY) == B.SD_ESTATE
    assert B.sd_set_pending(ctx, 4, 1) == B.SD_ESTATE
    assert B.sd_set_draft(ctx, np.zeros(2, np.int32)) == B.SD_ESTATE
    assert B.sd_read(ctx, None, None, None) == B.SD_ESTATE
    assert B.sd_dump_logits(ctx, B.SD_LOGITS_VERIFY, np.zeros(cfg.vocab, np.float32)) == B.SD_ESTATE
    assert B.sd_dump_draft(ctx, np.zeros(8, np.int32)) == B.SD_ESTATE
    # the prompt's own checks
    assert B.sd_prefill(ctx, np.zeros(0, np.int32), B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_prefill(ctx, np.array([1, cfg.vocab], np.int32), B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_prefill(ctx, np.array([1, -2], np.int32), B.SD_GREEDY) == B.SD_EINVAL
    assert B.sd_prefill(ctx, np.zeros(4, np.int32), B.SD_SAMPLE, None) == B.SD_EINVAL      # sampling without a uniform
    assert B.sd_prefill(ctx, np.zeros(4, np.int32), B.SD_SAMPLE, np.array([1.0], np.float32)) == B.SD_EINVAL
    assert B.sd_prefill(ctx, np.zeros(28, np.int32), B.SD_GREEDY) == B.SD_ECAPACITY        # 28 + 4 + 1 > 32
    # settings that need no device
    assert B.sd_keep_logits(ctx, 1) == B.SD_OK and B.sd_set_spin_limit(ctx, 1000) == B.SD_OK
    assert B.sd_set_turn_span(ctx, 1) == B.SD_OK and B.sd_phase_trace(ctx, 0) == B.SD_OK
    assert B.sd_set_skip_mask(ctx, np.zeros(4, np.uint8)) == B.SD_OK
    assert B.sd_last_hip_error(ctx) == 0
    B.sd_free(ctx)


def test_bench_host_helpers():
    """bench.py's host-side arithmetic: flops of a prompt forward, algorithmic bytes, mean context of the timed steps."""
    import importlib.util
    import synth
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    s = synth.CONFIGS["7b"]
    # one token: every projection once, one attended position, the head
    hq = s.n_heads * s.head_dim
    one = 2 * (s.n_layers * (4 * hq * s.d_model + 3 * s.d_ffn * s.d_model + 2 * hq) + s.vocab * s.d_model)
    assert bench.prompt_flops(s, 1) == one
    # n tokens: projections n times, attention n (n + 1) / 2 positions, the head still once
    n = 512
    assert bench.prompt_flops(s, n) - bench.prompt_flops(s, n - 1) == 2 * s.n_layers * (
        4 * hq * s.d_model + 3 * s.d_ffn * s.d_model + 2 * hq * n)
    # a window of 51 steps at one token per step, timed steps 0..50 after a warm-up of a whole number of windows
    assert bench.mean_context(512, 51, 102, 51, 1.0) == 512 + 25.0
    assert bench.mean_context(512, 51, 0, 1, 4.0) == 512
    # weights of a layer dominate the algorithmic bytes; the KV term grows linearly with the context
    b0 = bench.algorithmic_bytes(s, s.n_layers, s.n_layers, 1, 512)
    b1 = bench.algorithmic_bytes(s, s.n_layers, s.n_layers, 1, 513)
    assert b1 - b0 == s.n_layers * 2 * s.n_kv_heads * s.head_dim * 2
    assert 13.4e9 < b0 < 13.6e9


def test_fit_prune_mask_is_the_ranking_rule_of_stage_a():
    """Host-only entry point: the floor(r L) layers of smallest score, equal scores by index, as whole-layer skip bits;
    compared with the oracle's rule on seeded scores with ties."""
    import numpy as np
    from oracle.fit import prune_set
    from paper_2602_05499_amd import binding as B
    rng = np.random.default_rng(3)
    for L in (1, 4, 7, 32):
        for ratio in (0.0, 0.25, 0.5, 0.74, 1.0):
            ta = rng.integers(0, 4, L).astype(np.float64)          # many equal scores
            tf = rng.integers(0, 3, L).astype(np.float64)
            rc, mask = B.sd_fit_prune_mask(ta, tf, ratio)
            assert rc == B.SD_OK
            assert sorted(int(l) for l in np.nonzero(mask)[0]) == prune_set(ta + tf, ratio)
            assert set(mask.tolist()) <= {0, 3}
    rc, _ = B.sd_fit_prune_mask(np.ones(3), np.ones(3), 1.5)
    assert rc == B.SD_EINVAL
    # sub-layers ranked separately (Sec. IV-A): the paper's 13B ratios on 40 layers
    ta, tf = rng.random(40), rng.random(40)
    rc, mask = B.sd_fit_prune_sublayers(ta, tf, 0.5, 0.35)
    assert rc == B.SD_OK
    assert sorted(np.nonzero(mask & 1)[0].tolist()) == prune_set(ta, 0.5) and int((mask & 1).sum()) == 20
    assert sorted(np.nonzero(mask & 2)[0].tolist()) == prune_set(tf, 0.35) and int(((mask & 2) >> 1).sum()) == 14
    rc, _ = B.sd_fit_prune_sublayers(ta, tf, -0.1, 0.5)
    assert rc == B.SD_EINVAL
