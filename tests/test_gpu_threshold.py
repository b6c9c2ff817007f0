"""GPU parity of the threshold-mask variant (CSR): dsa_predict_mask_threshold and dsa_masked_attention_csr,
called through the C ABI, against the CPU oracle.  row_ptr and col bit-exact (the scores are exact integers);
O within max-abs 1e-4 (fp32 inputs) / 2e-2 (bf16 inputs)."""
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
    pkg.binding.lib()
    return pkg


def dev_qkv(x):
    import torch
    out = []
    for name in ("Q", "K", "V"):
        a = x.storage(name)
        out.append(torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) if x.cfg.dtype == "bf16"
                   else torch.from_numpy(a).cuda())
    return out


def run_case(pkg, oracle, x, theta, label, capacity=None, check_attention=True):
    import torch
    cfg = x.cfg
    sh = pkg.make_shape(cfg.B, cfg.H, cfg.L, cfg.d, cfg.k, 1, cfg.vec, pkg.DSA_F32 if cfg.dtype == "f32" else pkg.DSA_BF16,
                        float(cfg.scale))
    want_ptr, want_col = oracle.predict_mask_threshold(x.Qt, x.Kt, theta, cfg.vec)
    nnz = int(want_ptr[-1])
    cap = nnz if capacity is None else capacity
    print(f"[{label}] B={cfg.B} H={cfg.H} L={cfg.L} k={cfg.k} vec={cfg.vec} theta={theta}: nnz={nnz} "
          f"(mean {nnz / (want_ptr.size - 1):.1f}, max {int(np.diff(want_ptr).max())} per row), capacity {cap}", flush=True)
    Qt, Kt = torch.from_numpy(x.Qt).cuda(), torch.from_numpy(x.Kt).cuda()
    guard = 64
    col = torch.full((cap + guard,), -7, dtype=torch.int32, device="cuda")
    row_ptr, _ = pkg.dsa_predict_mask_threshold(sh, Qt, Kt, theta, cap, col=col)
    torch.cuda.synchronize()
    got_ptr = row_ptr.cpu().numpy().astype(np.int64)
    assert np.array_equal(got_ptr, want_ptr), "row_ptr differs from the oracle"
    got_col = col.cpu().numpy()
    assert (got_col[cap:] == -7).all(), "wrote past the capacity of col"
    m = min(cap, nnz)
    assert np.array_equal(got_col[:m], want_col[:m]), "col differs from the oracle"
    if not check_attention or cap < nnz:
        return
    Q, K, V = dev_qkv(x)
    O = pkg.dsa_masked_attention_csr(sh, Q, K, V, row_ptr, col)
    torch.cuda.synchronize()
    rows = None if cfg.N * cfg.L <= 70000 else np.arange(0, cfg.N * cfg.L, 13)
    want_O = oracle.masked_attention_csr(x.Q, x.K, x.V, want_ptr, want_col, cfg.scale, cfg.vec, rows=rows)
    got_O = O.cpu().numpy().reshape(-1, cfg.d)
    err = float(np.abs((got_O if rows is None else got_O[rows]) - want_O).max())
    print(f"    max|O - oracle| = {err:.3e}", flush=True)
    assert err <= TOL[cfg.dtype]


def theta_for(oracle, x, fraction):
    """A threshold that about `fraction` of the scores reach (from a sample of units)."""
    n_units = x.cfg.N * (x.cfg.L // x.cfg.vec)
    units = np.arange(0, n_units, max(1, n_units // 256))
    sc = oracle.approx_scores(x.Qt, x.Kt, x.cfg.vec, units=units)
    return int(np.quantile(sc, 1.0 - fraction))


@pytest.mark.parametrize("name,fraction", [("C1", 0.10), ("C2", 0.10), ("C4f", 0.05), ("C3", 0.05), ("C4v", 0.05)])
def test_threshold_configs(dsa, oracle, workload, name, fraction):
    x = workload(name)
    run_case(dsa, oracle, x, theta_for(oracle, x, fraction), name)


RAGGED = [
    dict(B=1, H=3, L=100, d=64, dtype="f32", k=16),
    dict(B=2, H=2, L=777, d=64, dtype="bf16", k=64),
    dict(B=1, H=2, L=1000, d=128, dtype="f32", k=32),
    dict(B=1, H=1, L=1, d=64, dtype="f32", k=16),
    dict(B=1, H=1, L=5000, d=128, dtype="bf16", k=32, n_global=6),
]


RAGGED_GROUPS = [
    dict(B=1, H=3, L=100, d=64, dtype="f32", k=16, vec=4),
    dict(B=2, H=2, L=776, d=64, dtype="bf16", k=64, vec=8),
    dict(B=1, H=2, L=1000, d=128, dtype="f32", k=32, vec=8),
    dict(B=1, H=1, L=4, d=64, dtype="f32", k=16, vec=4),
    dict(B=1, H=2, L=2052, d=64, dtype="bf16", k=32, vec=4, n_global=6),
]


@pytest.mark.parametrize("spec", RAGGED_GROUPS, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items()))
def test_threshold_ragged_vector_wise(dsa, oracle, spec):
    """Groups of 4 or 8 rows as units (the group score is the sum over the rows): ragged key tails, unit
    counts that do not fill the last wavefront, a single unit."""
    cfg = di.custom_config(rank=4, seed=161 + spec["L"], keep=1, **spec)
    x = di.make_inputs(cfg)
    for fraction in (0.02, 0.3):
        run_case(dsa, oracle, x, theta_for(oracle, x, fraction), "ragged groups")
    sc = oracle.approx_scores(x.Qt, x.Kt, cfg.vec)
    run_case(dsa, oracle, x, int(sc.max()) + 1, "no key reaches theta: best key per group")


@pytest.mark.parametrize("spec", RAGGED, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items()))
def test_threshold_ragged_shapes(dsa, oracle, spec):
    cfg = di.custom_config(rank=4, seed=61 + spec["L"], vec=1, keep=1, **spec)
    x = di.make_inputs(cfg)
    for fraction in (0.02, 0.3):
        run_case(dsa, oracle, x, theta_for(oracle, x, fraction), "ragged")


def test_threshold_extremes_and_capacity(dsa, oracle, workload):
    x = workload("C1")
    sc = oracle.approx_scores(x.Qt, x.Kt, 1)
    run_case(dsa, oracle, x, int(sc.max()) + 1, "no key reaches theta: best key per row")
    run_case(dsa, oracle, x, int(sc.min()), "every key reaches theta: dense")
    # rows of more than one chunk of the CSR attention kernel (1024 keys)
    cfg = di.custom_config(B=1, H=2, L=2600, d=64, dtype="bf16", rank=4, k=32, vec=1, keep=1, seed=77)
    y = di.make_inputs(cfg)
    run_case(dsa, oracle, y, theta_for(oracle, y, 0.7), "long rows")
    # col too small: row_ptr still complete, nothing written beyond the capacity
    theta = theta_for(oracle, x, 0.1)
    run_case(dsa, oracle, x, theta, "capacity 1000", capacity=1000)
    # heavy ties: few score levels, theta on a level
    Qt, Kt = di.random_int8_case(91, 1, 2, 640, 32, lo=-1, hi=1)
    z = di.DsaInputs(di.custom_config(B=1, H=2, L=640, d=64, dtype="f32", rank=4, k=32, vec=1, keep=1, seed=3),
                     None, None, None, Qt.reshape(1, 2, 640, 32), Kt.reshape(1, 2, 640, 32), None, None, None)
    for theta in (-2, 0, 1, 3):
        run_case(dsa, oracle, z, theta, "ties", check_attention=False)


def test_threshold_errors_launch_nothing(dsa):
    import ctypes
    b = dsa.binding
    lib = b.lib()
    fake = ctypes.c_void_p(0x1000)
    sh = b.make_shape(1, 2, 256, 64, 32, 1, 2, b.DSA_F32, 0.125)
    assert lib.dsa_predict_mask_threshold(ctypes.byref(sh), fake, fake, 0, fake, fake, 10, fake, 1 << 30, None) == 3
    assert b.threshold_workspace_bytes(sh) == 0
    sh = b.make_shape(1, 2, 256, 64, 32, 1, 1, b.DSA_F32, 0.125)
    assert b.threshold_workspace_bytes(sh) > 0
    assert lib.dsa_predict_mask_threshold(ctypes.byref(sh), fake, fake, 0, fake, fake, 10, fake, 16, None) == 5
    assert lib.dsa_predict_mask_threshold(ctypes.byref(sh), fake, fake, 0, None, fake, 10, fake, 1 << 30, None) == 1
    assert lib.dsa_predict_mask_threshold(ctypes.byref(sh), fake, fake, 0, fake, fake, -1, fake, 1 << 30, None) == 2
    big = b.make_shape(1, 64, 8192, 64, 32, 1, 1, b.DSA_F32, 0.125)       # 64 * 8192 * 8192 > 2^31 - 1
    assert lib.dsa_predict_mask_threshold(ctypes.byref(big), fake, fake, 0, fake, fake, 10, fake, 1 << 40, None) == 3
    assert lib.dsa_masked_attention_csr(ctypes.byref(sh), fake, fake, fake, None, fake, fake, None) == 1
