"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Mask and index lists bit-exact; float outputs within max-abs 1e-4 (fp32
inputs) / 2e-2 (bf16 inputs)."""
import numpy as np
import pytest

import dsa_inputs as di

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def dsa():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X: run them with -m gpu on the GPU box")
    import paper_2110_11299_amd as pkg
    pkg.binding.lib()          # raises if the HIP library was not built: no fallback
    return pkg


def to_dev(x: di.DsaInputs):
    import torch
    out = {}
    for name in ("Q", "K", "V"):
        a = x.storage(name)
        if x.cfg.dtype == "bf16":
            out[name] = torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        else:
            out[name] = torch.from_numpy(a).cuda()
    out["Qt"] = torch.from_numpy(x.Qt).cuda()
    out["Kt"] = torch.from_numpy(x.Kt).cuda()
    return out


def shape_of(pkg, cfg, keep=None):
    return pkg.make_shape(cfg.B, cfg.H, cfg.L, cfg.d, cfg.k, cfg.keep if keep is None else keep, cfg.vec,
                          pkg.DSA_F32 if cfg.dtype == "f32" else pkg.DSA_BF16, float(cfg.scale))


def check_path(pkg, oracle, x, *, staged=True, label=""):
    """Runs every entry point on x and compares with the oracle.  Returns max-abs errors."""
    import torch
    cfg = x.cfg
    sh = shape_of(pkg, cfg)
    dev = to_dev(x)
    tol = TOL[cfg.dtype]
    print(f"[{label or cfg.name}] B={cfg.B} H={cfg.H} L={cfg.L} d={cfg.d} k={cfg.k} vec={cfg.vec} "
          f"keep={cfg.keep} {cfg.dtype}", flush=True)

    want_idx = oracle.predict_mask(x.Qt, x.Kt, cfg.keep, cfg.vec)
    want_O, want_S, want_P = oracle.masked_attention(x.Q, x.K, x.V, want_idx, cfg.scale, cfg.vec,
                                                     return_sp=True)

    # (a)+(b)
    idx = pkg.dsa_predict_mask(sh, dev["Qt"], dev["Kt"])
    torch.cuda.synchronize()
    got_idx = idx.cpu().numpy().reshape(-1, cfg.keep)
    mism = int((got_idx != want_idx).any(axis=1).sum())
    assert mism == 0, f"{mism} of {want_idx.shape[0]} units differ in the mask"

    errs = {}
    if staged:
        S = pkg.dsa_sddmm(sh, dev["Q"], dev["K"], idx)
        P = pkg.dsa_sparse_softmax(sh, S)
        O = pkg.dsa_spmm(sh, P, idx, dev["V"])
        torch.cuda.synchronize()
        errs["S"] = float(np.abs(S.cpu().numpy().reshape(want_S.shape) - want_S).max())
        errs["P"] = float(np.abs(P.cpu().numpy().reshape(want_P.shape) - want_P).max())
        errs["O_staged"] = float(np.abs(O.cpu().numpy().reshape(want_O.shape) - want_O).max())
        rows = P.sum(dim=-1)
        assert float((rows - 1).abs().max()) < 1e-5 and float(P.min()) >= 0
        # in-place softmax gives the same bits
        P2 = pkg.dsa_sparse_softmax(sh, S, S)
        assert torch.equal(P2, P)
    O = pkg.dsa_masked_attention(sh, dev["Q"], dev["K"], dev["V"], idx)
    torch.cuda.synchronize()
    errs["O_masked"] = float(np.abs(O.cpu().numpy().reshape(want_O.shape) - want_O).max())

    O2, idx2 = pkg.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"])
    O3, none = pkg.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"], want_idx=False)
    torch.cuda.synchronize()
    assert none is None
    assert torch.equal(idx2, idx), "fused entry point returned a different mask"
    assert torch.equal(O2, O) and torch.equal(O3, O), "fused entry point is not reproducible"
    errs["O_fwd"] = float(np.abs(O2.cpu().numpy().reshape(want_O.shape) - want_O).max())
    print(f"    max-abs errors: {errs}", flush=True)
    for name, e in errs.items():
        assert e <= tol, f"{name}: max-abs error {e} > {tol}"
    return errs


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4f", "C4v", "C5"])
def test_config_parity(dsa, oracle, workload, name):
    check_path(dsa, oracle, workload(name), staged=True)


EDGE = [
    # ragged lengths (not a multiple of the wavefront or of any tile), odd head counts
    dict(B=1, H=3, L=100, d=64, dtype="f32", k=16, vec=1, keep=7),
    dict(B=3, H=1, L=104, d=64, dtype="bf16", k=32, vec=8, keep=13),
    dict(B=1, H=2, L=1000, d=128, dtype="f32", k=48, vec=1, keep=100),
    dict(B=1, H=2, L=1096, d=128, dtype="bf16", k=128, vec=8, keep=55),
    dict(B=2, H=2, L=777, d=64, dtype="bf16", k=64, vec=1, keep=39),
    # degenerate keeps
    dict(B=1, H=2, L=96, d=64, dtype="f32", k=16, vec=1, keep=1),
    dict(B=1, H=2, L=96, d=64, dtype="f32", k=16, vec=8, keep=96),
    dict(B=1, H=1, L=8, d=64, dtype="bf16", k=16, vec=8, keep=8),
    dict(B=1, H=1, L=1, d=64, dtype="f32", k=16, vec=1, keep=1),
    dict(B=1, H=1, L=520, d=64, dtype="f32", k=32, vec=1, keep=519),
    dict(B=1, H=1, L=2304, d=64, dtype="bf16", k=32, vec=1, keep=1200, n_global=5),
    # several key chunks per workgroup, fine-grained and vector-wise; long contraction (8 * 80)
    dict(B=1, H=2, L=6000, d=64, dtype="bf16", k=32, vec=1, keep=60, n_global=7),
    dict(B=1, H=1, L=20000, d=64, dtype="bf16", k=16, vec=8, keep=100, n_global=9),
    dict(B=1, H=1, L=12288, d=128, dtype="bf16", k=64, vec=8, keep=600),
    dict(B=2, H=1, L=328, d=64, dtype="f32", k=80, vec=8, keep=33),
    dict(B=1, H=1, L=3000, d=64, dtype="f32", k=112, vec=1, keep=300),
    # 1x4 column vectors (section 5.1, table 3): groups of four query rows share a list
    dict(B=2, H=2, L=2048, d=64, dtype="bf16", k=32, vec=4, keep=102, n_global=8),
    dict(B=1, H=3, L=100, d=64, dtype="f32", k=16, vec=4, keep=9),
    dict(B=1, H=1, L=6000, d=128, dtype="bf16", k=64, vec=4, keep=75),
    dict(B=1, H=2, L=1000, d=64, dtype="f32", k=48, vec=4, keep=1),
]


@pytest.mark.parametrize("spec", EDGE, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items()))
def test_edge_shapes(dsa, oracle, spec):
    cfg = di.custom_config(rank=4, seed=31 + spec["L"], **spec)
    check_path(dsa, oracle, di.make_inputs(cfg), staged=True, label="edge")


@pytest.mark.parametrize("vec", [1, 4, 8])
@pytest.mark.parametrize("lo,hi", [(0, 0), (-1, 1), (-3, 3), (-127, 127)])
def test_mask_with_heavy_ties(dsa, oracle, vec, lo, hi):
    """Narrow int8 ranges make most scores collide, so the lowest-index rule decides
    almost every list; all-zero projections make it decide everything."""
    import torch
    B, H, L, k = 2, 3, 1536, 32
    Qt, Kt = di.random_int8_case(5 + hi, B, H, L, k, lo=lo, hi=hi)
    for keep in (1, 77, 500):
        sh = dsa.make_shape(B, H, L, 64, k, keep, vec, dsa.DSA_F32, 0.125)
        print(f"[ties] range=({lo},{hi}) vec={vec} keep={keep}", flush=True)
        idx = dsa.dsa_predict_mask(sh, torch.from_numpy(Qt).cuda(), torch.from_numpy(Kt).cuda())
        want = oracle.predict_mask(Qt, Kt, keep, vec)
        assert np.array_equal(idx.cpu().numpy().reshape(want.shape), want)


@pytest.mark.parametrize("L,keep,vec", [(512, 51, 1), (256, 33, 1), (640, 45, 1), (2048, 103, 8), (1024, 61, 4)])
def test_mask_with_zero_query_rows(dsa, oracle, L, keep, vec):
    """Units whose projected query is all zero among ordinary ones: every score of such a unit is the same,
    so any score read too early, or any word of its bitmap touched by a neighbour, shows in its list (the
    first `keep` keys).  keep is chosen so that the image of the index rows is the larger part of a
    wavefront's LDS and has an odd length; several launches, because such faults come and go."""
    import torch
    B, H, k = (8, 8, 32) if vec == 8 else (2, 6, 32)       # vec = 8: enough units for the streaming kernel
    Qt, Kt = di.random_int8_case(900 + L, B, H, L, k)
    Qt = Qt.copy()
    for first in (0, 2, 15, 16 * 5 + 7):
        Qt[:, :, first * vec::48 * vec] = 0
        for r in range(1, vec):
            Qt[:, :, first * vec + r::48 * vec] = 0
    sh = dsa.make_shape(B, H, L, 64, k, keep, vec, dsa.DSA_F32, 0.125)
    want = oracle.predict_mask(Qt, Kt, keep, vec)
    q, kk = torch.from_numpy(Qt).cuda(), torch.from_numpy(Kt).cuda()
    for launch in range(4):
        print(f"[zero rows] L={L} keep={keep} vec={vec} launch {launch}", flush=True)
        idx = dsa.dsa_predict_mask(sh, q, kk)
        torch.cuda.synchronize()
        bad = int((idx.cpu().numpy().reshape(want.shape) != want).any(axis=1).sum())
        assert bad == 0, f"{bad} of {want.shape[0]} units differ in launch {launch}"


@pytest.mark.parametrize("L", [4096, 2500])
def test_mask_with_score_plateaus(dsa, oracle, L):
    """Scores that take three values only, on plateaus of several hundred keys: the kept set is
    decided inside a plateau (all ties), at its edge, or needs more candidates than the fast
    selection holds -- the strict-threshold pass, the ties-only answer and the recomputing path."""
    import torch
    B, H, k = 1, 2, 32
    rng = np.random.Generator(np.random.Philox(77 + L))
    Kt = np.zeros((B, H, L, k), np.int8)
    level = rng.permutation(L)
    Kt[:, :, level[:600], 0] = 2           # 600 keys score 2 * q0, 600 keys score q0, the rest 0
    Kt[:, :, level[600:1200], 0] = 1
    Qt = np.zeros((B, H, L, k), np.int8)
    Qt[..., 0] = rng.integers(-3, 4, size=(B, H, L))     # negative q0 reverses the order, 0 ties everything
    for vec in (1, 8):
        for keep in (1, 300, 600, 601, 700, 1200, 1300, L):
            sh = dsa.make_shape(B, H, L if vec == 1 else L - L % 8, 64, k, keep, vec, dsa.DSA_F32, 0.125)
            Lv = sh.L
            q, kk = np.ascontiguousarray(Qt[:, :, :Lv]), np.ascontiguousarray(Kt[:, :, :Lv])
            if keep > Lv:
                continue
            print(f"[plateaus] L={Lv} vec={vec} keep={keep}", flush=True)
            idx = dsa.dsa_predict_mask(sh, torch.from_numpy(q).cuda(), torch.from_numpy(kk).cuda())
            want = oracle.predict_mask(q, kk, keep, vec)
            assert np.array_equal(idx.cpu().numpy().reshape(want.shape), want)


@pytest.mark.parametrize("k,vec,keep", [(16, 1, 100), (32, 8, 1638)])
def test_predictor_at_maximum_length(dsa, oracle, k, vec, keep):
    """L = 32768, the longest sequence the predictor takes: sampled units against the oracle one by
    one, every list ascending and in range."""
    import torch
    L = 32768
    Qt, Kt = di.random_int8_case(L + vec, 1, 1, L, k)
    sh = dsa.make_shape(1, 1, L, 64, k, keep, vec, dsa.DSA_F32, 0.125)
    print(f"[max L] k={k} vec={vec} keep={keep}", flush=True)
    idx = dsa.dsa_predict_mask(sh, torch.from_numpy(Qt).cuda(), torch.from_numpy(Kt).cuda())
    full = idx.cpu().numpy().reshape(-1, keep)
    assert (np.diff(full, axis=1) > 0).all() and full.min() >= 0 and full.max() < L
    units = np.arange(0, L // vec, 97)
    assert np.array_equal(full[units], oracle.predict_mask(Qt, Kt, keep, vec, units=units))


def test_attention_at_maximum_keep(dsa, oracle):
    """keep = 4096, the longest list the attention kernels take (here every key of L = 4096: the
    result is dense attention), fp32 and bf16, sampled rows against the oracle."""
    import torch
    for dtype in ("f32", "bf16"):
        cfg = di.custom_config(B=1, H=1, L=4096, d=64, dtype=dtype, rank=8, k=16, keep=4096, seed=4096)
        x = di.make_inputs(cfg)
        sh = shape_of(dsa, cfg)
        dev = to_dev(x)
        print(f"[max keep] {dtype}", flush=True)
        idx = np.tile(np.arange(4096, dtype=np.int32), (4096, 1))
        O = dsa.dsa_masked_attention(sh, dev["Q"], dev["K"], dev["V"], torch.from_numpy(idx).cuda().view(1, 1, 4096, 4096))
        rows = np.arange(0, 4096, 61)
        want = oracle.masked_attention(x.Q, x.K, x.V, idx, cfg.scale, 1, rows=rows)
        assert float(np.abs(O.cpu().numpy().reshape(4096, 64)[rows] - want).max()) <= TOL[dtype]
    sh = dsa.make_shape(1, 1, 8192, 64, 16, 4097, 1, dsa.DSA_F32, 0.125)       # one more is refused
    z = torch.zeros((1, 1, 8192, 64), device="cuda")
    with pytest.raises(dsa.DsaError) as e:
        dsa.dsa_masked_attention(sh, z, z, z, torch.zeros((1, 1, 8192, 4097), dtype=torch.int32, device="cuda"))
    assert e.value.status == 3


def test_reproducible_and_stream_ordered(dsa, oracle, workload):
    """Same inputs, same bits; and the path runs on whatever stream the caller makes current."""
    import torch
    x = workload("C3")
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    O1, idx1 = dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        O2, idx2 = dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"])
    side.synchronize()
    assert torch.equal(idx1, idx2) and torch.equal(O1, O2)
    x = workload("C2")
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    a = dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"])
    b = dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"])
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_invalid_indices_cannot_leave_the_tensors(dsa):
    """The attention entry points clamp whatever idx holds into [0, L): garbage in, no fault."""
    import torch
    B, H, L, d, keep = 1, 2, 128, 64, 9
    sh = dsa.make_shape(B, H, L, d, 16, keep, 1, dsa.DSA_F32, 0.125)
    Q = torch.randn((B, H, L, d), device="cuda")
    idx = torch.full((B, H, L, keep), 2_000_000_000, dtype=torch.int32, device="cuda")
    idx[..., ::2] = -5
    O = dsa.dsa_masked_attention(sh, Q, Q, Q, idx)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all())


def test_outputs_stay_inside_their_buffers(dsa, oracle, workload):
    """Guard words around idx and O must survive."""
    import torch
    x = workload("C1")
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    pad = 64
    n_idx, n_o = cfg.units * cfg.keep, cfg.N * cfg.L * cfg.d
    idx_buf = torch.full((n_idx + 2 * pad,), -7, dtype=torch.int32, device="cuda")
    o_buf = torch.full((n_o + 2 * pad,), 123.0, dtype=torch.float32, device="cuda")
    idx = idx_buf[pad:pad + n_idx].view(cfg.B, cfg.H, cfg.L // cfg.vec, cfg.keep)
    O = o_buf[pad:pad + n_o].view(cfg.B, cfg.H, cfg.L, cfg.d)
    dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], dev["Qt"], dev["Kt"], O=O, idx_out=idx)
    torch.cuda.synchronize()
    assert bool((idx_buf[:pad] == -7).all()) and bool((idx_buf[pad + n_idx:] == -7).all())
    assert bool((o_buf[:pad] == 123.0).all()) and bool((o_buf[pad + n_o:] == 123.0).all())
    assert bool((idx >= 0).all()) and bool((idx < cfg.L).all())


@pytest.mark.parametrize("name", ["C1", "C2", "C4f", "C5"])
def test_rowmax_of_approximate_scores(dsa, oracle, workload, name):
    """The int8 matrix-core contraction alone: row maxima of S~ are exact integers."""
    import torch
    x = workload(name)
    cfg = x.cfg
    sh = shape_of(dsa, cfg)
    print(f"[rowmax] {name}", flush=True)
    got = dsa.dsa_approx_rowmax(sh, torch.from_numpy(x.Qt).cuda(), torch.from_numpy(x.Kt).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy().reshape(-1)
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, cfg.N * cfg.L - 1], rng.integers(0, cfg.N * cfg.L, 512)]))
    want = oracle.approx_scores(x.Qt, x.Kt, vec=1, units=rows).max(axis=1)
    assert np.array_equal(got[rows], want)


def test_rowmax_ragged(dsa, oracle):
    import torch
    for (L, k) in [(1, 16), (33, 16), (100, 48), (257, 128)]:
        Qt, Kt = di.random_int8_case(L, 1, 3, L, k)
        sh = dsa.make_shape(1, 3, L, 64, k, 1, 1, dsa.DSA_F32, 1.0)
        got = dsa.dsa_approx_rowmax(sh, torch.from_numpy(Qt).cuda(), torch.from_numpy(Kt).cuda())
        want = oracle.approx_scores(Qt, Kt).max(axis=1)
        assert np.array_equal(got.cpu().numpy().reshape(-1), want), (L, k)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4f", "C5"])
def test_projection_and_quantiser(dsa, oracle, workload, name):
    """The step in front of the path: int8 codes bit-exact against the oracle's fp32 recipe,
    then the whole forward from the GPU-made codes against the oracle run on the oracle-made codes."""
    import torch
    x = workload(name)
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    R32 = x.R.astype(np.float32)
    Rd = torch.from_numpy(R32).cuda()
    print(f"[project] {name}", flush=True)
    made = {}
    for which in ("Q", "K"):
        codes, amax = dsa.dsa_project_quantize(sh, dev[which], Rd)
        torch.cuda.synchronize()
        want, want_amax = oracle.project_quantize(getattr(x, which), R32)
        assert float(amax.item()) == float(want_amax)
        assert np.array_equal(codes.cpu().numpy(), want.reshape(codes.shape)), which
        made[which] = (codes, want)
    O, idx = dsa.dsa_attention_fwd(sh, dev["Q"], dev["K"], dev["V"], made["Q"][0], made["K"][0])
    torch.cuda.synchronize()
    want_O, want_idx = oracle.attention_fwd(x.Q, x.K, x.V, made["Q"][1], made["K"][1], cfg.keep, cfg.scale, cfg.vec)
    assert np.array_equal(idx.cpu().numpy().reshape(want_idx.shape), want_idx)
    assert float(np.abs(O.cpu().numpy().reshape(want_O.shape) - want_O).max()) <= TOL[cfg.dtype]


def test_projection_ragged_and_zero(dsa, oracle):
    import torch
    for (L, d, k, dtype) in [(1, 64, 16, "f32"), (77, 128, 48, "bf16"), (300, 64, 128, "f32"), (520, 128, 128, "bf16")]:
        cfg = di.custom_config(B=1, H=3, L=L, d=d, dtype=dtype, rank=3, k=k, keep=1, seed=L)
        x = di.make_inputs(cfg)
        sh = shape_of(dsa, cfg)
        R32 = x.R.astype(np.float32)
        codes, amax = dsa.dsa_project_quantize(sh, to_dev(x)["K"], torch.from_numpy(R32).cuda())
        want, want_amax = oracle.project_quantize(x.K, R32)
        assert np.array_equal(codes.cpu().numpy(), want.reshape(codes.shape)) and float(amax.item()) == float(want_amax)
    sh = dsa.make_shape(1, 1, 32, 64, 16, 1, 1, dsa.DSA_F32, 1.0)
    codes, amax = dsa.dsa_project_quantize(sh, torch.zeros((1, 1, 32, 64), device="cuda"),
                                           torch.ones((64, 16), device="cuda"))
    assert float(amax.item()) == 0.0 and not bool(codes.any())


@pytest.mark.parametrize("name,bits", [("C1", 8), ("C2", 8), ("C4f", 8), ("C4f", 4), ("C5", 8), ("C5", 2)])
def test_ternary_projection(dsa, oracle, workload, name, bits):
    """Equation 5's sparse random projection (signs -1, 0, 1 with probabilities 1/6, 2/3, 1/6): codes bit-exact
    against the oracle's additions and subtractions, and equal to the dense projection with the same signs."""
    import torch
    x = workload(name)
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    rng = np.random.Generator(np.random.Philox(900 + cfg.seed))
    P3 = rng.choice(np.array([-1, 0, 1], dtype=np.int8), size=(cfg.d, cfg.k), p=[1 / 6, 2 / 3, 1 / 6])
    Pd = torch.from_numpy(P3).cuda()
    print(f"[ternary] {name} bits={bits}", flush=True)
    for which in ("Q", "K"):
        packed, amax = dsa.dsa_project_quantize_ternary(sh, bits, dev[which], Pd)
        dense, amax2 = dsa.dsa_project_quantize_bits(sh, bits, dev[which], Pd.float())
        torch.cuda.synchronize()
        want, want_amax = oracle.project_quantize_ternary(getattr(x, which), P3, bits)
        assert float(amax.item()) == float(want_amax) == float(amax2.item())
        assert np.array_equal(packed.cpu().numpy().reshape(-1), oracle.pack_codes(want, bits).reshape(-1)), which
        assert torch.equal(packed, dense)


@pytest.mark.parametrize("bits", [4, 2])
@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4f", "C5"])
def test_low_precision_prediction(dsa, oracle, workload, name, bits):
    """Prediction at INT4 / INT2: packed codes made on the GPU are the oracle's codes in the oracle's
    packing bit for bit, and the mask found from them is the oracle's mask of those integer codes
    (few levels: ties at the threshold in most rows)."""
    import torch
    x = workload(name)
    cfg, dev = x.cfg, to_dev(x)
    sh = shape_of(dsa, cfg)
    R32 = x.R.astype(np.float32)
    Rd = torch.from_numpy(R32).cuda()
    print(f"[low precision] {name} bits={bits}", flush=True)
    packed, codes = {}, {}
    for which in ("Q", "K"):
        got, amax = dsa.dsa_project_quantize_bits(sh, bits, dev[which], Rd)
        torch.cuda.synchronize()
        want, want_amax = oracle.project_quantize(getattr(x, which), R32, bits=bits)
        assert float(amax.item()) == float(want_amax)
        want_packed = oracle.pack_codes(want, bits)
        assert np.array_equal(got.cpu().numpy(), want_packed.reshape(got.shape)), which
        packed[which], codes[which] = got, want
    idx = dsa.dsa_predict_mask_bits(sh, bits, packed["Q"], packed["K"])
    torch.cuda.synchronize()
    want_idx = oracle.predict_mask(codes["Q"], codes["K"], cfg.keep, cfg.vec)
    assert np.array_equal(idx.cpu().numpy().reshape(want_idx.shape), want_idx)
    # the whole path from the packed codes, with and without the mask handed back
    O, idx2 = dsa.dsa_attention_fwd_bits(sh, bits, dev["Q"], dev["K"], dev["V"], packed["Q"], packed["K"])
    O2, none = dsa.dsa_attention_fwd_bits(sh, bits, dev["Q"], dev["K"], dev["V"], packed["Q"], packed["K"], want_idx=False)
    torch.cuda.synchronize()
    assert none is None and np.array_equal(idx2.cpu().numpy().reshape(want_idx.shape), want_idx)
    want_O = oracle.masked_attention(x.Q, x.K, x.V, want_idx, cfg.scale, cfg.vec)
    assert float(np.abs(O.cpu().numpy().reshape(want_O.shape) - want_O).max()) <= TOL[cfg.dtype]
    assert torch.equal(O, O2)
    # bits = 8 through the same entry points is the int8 path
    if bits == 4 and name == "C1":
        p8, _ = dsa.dsa_project_quantize_bits(sh, 8, dev["K"], Rd)
        assert np.array_equal(p8.cpu().numpy().view(np.int8), oracle.project_quantize(x.K, R32)[0].reshape(p8.shape))
        i8 = dsa.dsa_predict_mask_bits(sh, 8, dev["Qt"].view(torch.uint8), dev["Kt"].view(torch.uint8))
        assert np.array_equal(i8.cpu().numpy().reshape(-1, cfg.keep), oracle.predict_mask(x.Qt, x.Kt, cfg.keep, cfg.vec))


@pytest.mark.parametrize("bits", [4, 2])
def test_low_precision_ragged(dsa, oracle, bits):
    """Packed codes on shapes with a ragged tail, the smallest and the largest k, both granularities."""
    import torch
    for (L, k, vec, keep) in [(8, 16, 8, 1), (77, 16, 1, 5), (1000, 128, 8, 40), (4104, 48, 8, 200), (6000, 32, 1, 300)]:
        cfg = di.custom_config(B=1, H=2, L=L, d=64, dtype="f32", rank=4, k=k, keep=keep, vec=vec, seed=L + bits)
        x = di.make_inputs(cfg)
        sh = shape_of(dsa, cfg)
        R32 = x.R.astype(np.float32)
        print(f"[low precision ragged] L={L} k={k} vec={vec} keep={keep} bits={bits}", flush=True)
        q, _ = oracle.project_quantize(x.Q, R32, bits=bits)
        kk, _ = oracle.project_quantize(x.K, R32, bits=bits)
        qp = torch.from_numpy(oracle.pack_codes(q, bits)).cuda()
        kp = torch.from_numpy(oracle.pack_codes(kk, bits)).cuda()
        idx = dsa.dsa_predict_mask_bits(sh, bits, qp, kp)
        want = oracle.predict_mask(q, kk, keep, vec)
        assert np.array_equal(idx.cpu().numpy().reshape(want.shape), want)
        got, _ = dsa.dsa_project_quantize_bits(sh, bits, to_dev(x)["K"], torch.from_numpy(R32).cuda())
        assert np.array_equal(got.cpu().numpy(), oracle.pack_codes(kk, bits).reshape(got.shape))


def test_low_precision_errors(dsa):
    import torch
    sh = dsa.make_shape(1, 1, 64, 64, 16, 8, 1, dsa.DSA_F32, 0.125)
    q = torch.zeros((1, 1, 64, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(dsa.DsaError) as e:                                 # bits = 3 is not a storage format
        dsa.binding._check(dsa.binding.lib().dsa_predict_mask_bits(
            __import__("ctypes").byref(sh), 3, q.data_ptr(), q.data_ptr(), q.data_ptr(), q.data_ptr(), 1 << 20, None), "bits")
    assert e.value.status == 3
    with pytest.raises(dsa.DsaError) as e:                                 # workspace too small for the widened codes
        dsa.dsa_predict_mask_bits(sh, 4, q, q, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 5


def test_errors_launch_nothing(dsa):
    import torch
    sh = dsa.make_shape(1, 1, 64, 64, 16, 65, 1, dsa.DSA_F32, 0.125)      # keep > L
    Qt = torch.zeros((1, 1, 64, 16), dtype=torch.int8, device="cuda")
    with pytest.raises(dsa.DsaError) as e:
        dsa.dsa_predict_mask(sh, Qt, Qt)
    assert e.value.status == 2
    sh = dsa.make_shape(1, 1, 64, 64, 16, 8, 2, dsa.DSA_F32, 0.125)       # vec = 2
    with pytest.raises(dsa.DsaError) as e:
        dsa.dsa_predict_mask(sh, Qt, Qt)
    assert e.value.status == 3
