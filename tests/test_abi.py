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
