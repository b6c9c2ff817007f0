"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
include/dsa.h declares, validates arguments before touching the device, and computes the
host-only helpers."""
import ctypes
import re
from pathlib import Path

import pytest

import dsa_inputs as di

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def b():
    from paper_2110_11299_amd import binding, build
    if not build.LIB.exists():
        build.build_hip()
    return binding


def declared_functions():
    text = (ROOT / "include" / "dsa.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dsa_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(b):
    names = declared_functions()
    assert "dsa_attention_fwd" in names and "dsa_predict_mask" in names and len(names) >= 9
    lib = b.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in dsa.h but not exported"
    assert sorted(b.EXPORTS) == names


def test_struct_layout_matches_header(b):
    assert ctypes.sizeof(b.DsaShape) == 36
    assert [f[0] for f in b.DsaShape._fields_] == ["B", "H", "L", "d", "k", "keep", "vec", "dtype", "scale"]


def test_keep_from_ratio(b):
    for cfg in di.CONFIGS.values():
        assert b.keep_from_ratio(cfg.L, cfg.ratio) == cfg.keep
    assert b.keep_from_ratio(2000, 0.1) == 200
    assert b.keep_from_ratio(100, 0.0) == 1 and b.keep_from_ratio(100, 5.0) == 100
    assert b.keep_from_ratio(10, 0.25) == 3
    assert b.keep_from_ratio(0, 0.5) == 0
    assert b.keep_from_ratio(100, float("nan")) == 1


def good(b, **kw):
    base = dict(B=2, H=2, L=256, d=64, k=32, keep=26, vec=1, dtype=b.DSA_F32, scale=0.125)
    base.update(kw)
    return b.make_shape(**base)


def test_workspace_bytes(b):
    sh = good(b)
    n = b.workspace_bytes(sh)
    assert n >= 2 * 2 * 256 * 26 * 4 and n % 256 == 0
    assert b.workspace_bytes(good(b, vec=3)) == 0
    assert b.workspace_bytes(good(b, keep=0)) == 0


P = 4096  # a fake, aligned, never dereferenced device address


def test_argument_errors_come_back_as_status_codes(b):
    lib = b.lib()
    ref = ctypes.byref
    big = 1 << 30
    OK_NULL, SHAPE, UNSUP, ALIGN, WS = 1, 2, 3, 4, 5
    assert lib.dsa_predict_mask(None, P, P, P, P, big, None) == OK_NULL
    assert lib.dsa_predict_mask(ref(good(b)), None, P, P, P, big, None) == OK_NULL
    assert lib.dsa_predict_mask(ref(good(b)), P, P, None, P, big, None) == OK_NULL
    for bad, want in [(dict(B=0), SHAPE), (dict(L=0), SHAPE), (dict(keep=0), SHAPE), (dict(keep=257), SHAPE),
                      (dict(vec=8, L=252), SHAPE), (dict(vec=2), UNSUP), (dict(k=8), UNSUP), (dict(k=40), UNSUP),
                      (dict(k=256), UNSUP), (dict(L=1 << 20, keep=5), UNSUP)]:
        assert lib.dsa_predict_mask(ref(good(b, **bad)), P, P, P, P, big, None) == want, bad
    assert lib.dsa_predict_mask(ref(good(b)), P + 4, P, P, P, big, None) == ALIGN
    assert lib.dsa_predict_mask(ref(good(b)), P, P, P + 8, P, big, None) == ALIGN

    assert lib.dsa_sddmm(ref(good(b)), P, P, P, None, None) == OK_NULL
    assert lib.dsa_sddmm(ref(good(b, d=96)), P, P, P, P, None) == UNSUP
    assert lib.dsa_sddmm(ref(good(b, dtype=7)), P, P, P, P, None) == UNSUP
    assert lib.dsa_sddmm(ref(good(b, scale=float("inf"))), P, P, P, P, None) == SHAPE
    assert lib.dsa_sddmm(ref(good(b)), P, P + 2, P, P, None) == ALIGN
    assert lib.dsa_sparse_softmax(ref(good(b)), None, P, None) == OK_NULL
    assert lib.dsa_sparse_softmax(ref(good(b, keep=0)), P, P, None) == SHAPE
    assert lib.dsa_spmm(ref(good(b)), P, P, None, P, None) == OK_NULL
    assert lib.dsa_spmm(ref(good(b, d=32)), P, P, P, P, None) == UNSUP
    assert lib.dsa_masked_attention(ref(good(b)), P, P, P, P, None, None) == OK_NULL
    assert lib.dsa_masked_attention(ref(good(b, vec=2)), P, P, P, P, P, None) == UNSUP

    sh = good(b)
    need = b.workspace_bytes(sh)
    assert lib.dsa_attention_fwd(ref(sh), P, P, P, P, P, None, None, P, need, None) == OK_NULL
    # without idx_out the mask lives in the workspace: too small a workspace is refused
    assert lib.dsa_attention_fwd(ref(sh), P, P, P, P, P, P, None, None, 0, None) == WS
    assert lib.dsa_attention_fwd(ref(sh), P, P, P, P, P, P, None, P, 1024, None) == WS
    assert lib.dsa_attention_fwd(ref(good(b, d=100)), P, P, P, P, P, P, P, P, need, None) == UNSUP
    assert lib.dsa_approx_rowmax(ref(sh), P, None, P, None) == OK_NULL
    assert lib.dsa_approx_rowmax(ref(good(b, k=20)), P, P, P, None) == UNSUP


def test_status_strings(b):
    seen = {b.status_string(i) for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert b.status_string(99) == "unknown status"
    assert re.fullmatch(r"\d+\.\d+", b.version())


def test_binding_refuses_cpu_tensors(b):
    import torch
    sh = good(b)
    t = torch.zeros((2, 2, 256, 32), dtype=torch.int8)
    with pytest.raises(ValueError):
        b.dsa_predict_mask(sh, t, t)


def test_noalloc_rejects_masks_beyond_its_array_on_the_host(b):
    """The size check of dsa_attention_fwd_noalloc comes before any device work."""
    lib = b.lib()
    assert b.noalloc_max_mask_bytes() == 16 << 20
    big = b.make_shape(2, 8, 4096, 64, 32, 205, 1, b.DSA_BF16, 0.125)      # 53.7 MB of mask
    fake = ctypes.c_void_p(0x1000)
    st = lib.dsa_attention_fwd_noalloc(ctypes.byref(big), fake, fake, fake, fake, fake, fake, None)
    assert st == 5 and "workspace" in b.status_string(st)
    assert lib.dsa_attention_fwd_noalloc(ctypes.byref(big), None, fake, fake, fake, fake, fake, None) == 1


def test_attention_rejects_lengths_whose_offsets_would_wrap(b):
    """The attention kernels index a head with 32-bit element offsets: L above 2^22 is refused."""
    lib = b.lib()
    fake = ctypes.c_void_p(0x1000)
    sh = good(b, B=1, H=1, L=(1 << 22) + 8, d=128, keep=8, vec=8)
    assert lib.dsa_sddmm(ctypes.byref(sh), fake, fake, fake, fake, None) == 3
    assert lib.dsa_spmm(ctypes.byref(sh), fake, fake, fake, fake, None) == 3
    assert lib.dsa_masked_attention(ctypes.byref(sh), fake, fake, fake, fake, fake, None) == 3
