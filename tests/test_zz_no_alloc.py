"""dsa_attention_fwd_noalloc (the entry point for callers that cannot allocate: the mask lives in the
library's fixed device array) against dsa_attention_fwd on the same inputs, through the C ABI: two
calls in a row, the second with a smaller input, so that what the first call left in the shared
array cannot leak into the second."""
import ctypes

import numpy as np
import pytest

import dsa_inputs as di

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def test_noalloc_matches_workspace_entry_point_twice(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X: run them with -m gpu on the GPU box")
    import paper_2110_11299_amd as pkg
    b = pkg.binding
    lib = b.lib()
    assert b.noalloc_max_mask_bytes() == 16 << 20

    cases = [
        di.custom_config("noalloc-big", B=2, H=3, L=2048, d=64, dtype="bf16", rank=16, k=32, vec=8, keep=102,
                         seed=4201, n_global=8),
        di.custom_config("noalloc-small", B=1, H=2, L=1000, d=64, dtype="f32", rank=8, k=32, vec=1, keep=50,
                         seed=4202),
    ]
    for cfg in cases:
        x = di.make_inputs(cfg)
        print(f"[{cfg.name}] B={cfg.B} H={cfg.H} L={cfg.L} d={cfg.d} k={cfg.k} vec={cfg.vec} keep={cfg.keep} "
              f"{cfg.dtype}", flush=True)
        dt = pkg.DSA_F32 if cfg.dtype == "f32" else pkg.DSA_BF16
        sh = pkg.make_shape(cfg.B, cfg.H, cfg.L, cfg.d, cfg.k, cfg.keep, cfg.vec, dt, float(cfg.scale))

        def dev(name):
            a = x.storage(name)
            if cfg.dtype == "bf16":
                return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(a).cuda()

        Q, K, V = dev("Q"), dev("K"), dev("V")
        Qt, Kt = torch.from_numpy(x.Qt).cuda(), torch.from_numpy(x.Kt).cuda()
        want, _ = pkg.dsa_attention_fwd(sh, Q, K, V, Qt, Kt, want_idx=False)
        got = torch.full_like(want, float("nan"))
        torch.cuda.synchronize()
        # the raw C ABI: plain device pointers, the current stream
        st = lib.dsa_attention_fwd_noalloc(ctypes.byref(sh), Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                                           Qt.data_ptr(), Kt.data_ptr(), got.data_ptr(),
                                           torch.cuda.current_stream().cuda_stream)
        assert st == b.DSA_OK, b.status_string(st)
        torch.cuda.synchronize()
        err = float((got - want).abs().max())
        assert err <= TOL[cfg.dtype], f"{cfg.name}: max-abs difference {err}"
        assert torch.equal(got, want), "same kernels on the same mask must give the same bits"
        ref_O, _ = oracle.attention_fwd(x.Q, x.K, x.V, x.Qt, x.Kt, cfg.keep, cfg.scale, cfg.vec)
        err_o = float(np.abs(got.cpu().numpy().reshape(ref_O.shape) - ref_O).max())
        assert err_o <= TOL[cfg.dtype], f"{cfg.name}: max-abs error against the oracle {err_o}"
        print(f"    equal to dsa_attention_fwd bit for bit; max|O - oracle| = {err_o:.3e}", flush=True)

    # a mask larger than the array is refused on the host, before any device work
    big = pkg.make_shape(2, 8, 4096, 64, 32, 205, 1, pkg.DSA_BF16, 0.125)
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    p = dummy.data_ptr()
    assert lib.dsa_attention_fwd_noalloc(ctypes.byref(big), p, p, p, p, p, p, None) == 5   # DSA_ERR_WORKSPACE
