"""The seeded input generator: determinism, shapes, storage formats."""
import numpy as np
import torch

import dsa_inputs as di


def test_deterministic_and_shaped():
    cfg = di.CONFIGS["C1"]
    a, b = di.make_inputs(cfg), di.make_inputs(cfg)
    for name in ("Q", "K", "V", "Qt", "Kt"):
        assert np.array_equal(getattr(a, name), getattr(b, name))
    assert a.Q.shape == (1, 2, 256, 64) and a.Q.dtype == np.float32
    assert a.Qt.shape == (1, 2, 256, 16) and a.Qt.dtype == np.int8
    assert np.abs(a.Qt).max() == 127 and np.abs(a.Kt).max() == 127     # symmetric, full range
    assert a.storage("Q") is a.Q


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]                   # ties to even both ways
    bits = di.round_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())
    assert np.array_equal(di.bf16_bits_to_f32(bits), want.float().numpy())


def test_bf16_config_values_are_representable():
    cfg = di.custom_config(B=1, H=2, L=64, d=64, dtype="bf16", rank=4, k=16, keep=6, n_global=3)
    x = di.make_inputs(cfg)
    for name in ("Q", "K", "V"):
        bits = x.storage(name)
        assert bits.dtype == np.uint16
        assert np.array_equal(di.bf16_bits_to_f32(bits), getattr(x, name))
    assert x.global_pos.shape == (2, 3)
    # the scaled key rows stand out
    norms = np.linalg.norm(x.K[0, 0], axis=1)
    assert norms[x.global_pos[0]].min() > 2 * np.median(norms)


def test_quantizer():
    assert di.quantize_int8(np.zeros((3, 2))).tolist() == [[0, 0]] * 3
    q = di.quantize_int8(np.array([-2.0, 1.0, 0.5, 2.0 * 0.5 / 127, 2.0 * 1.5 / 127, 2.0 * 2.5 / 127]))
    assert q.tolist() == [-127, 64, 32, 0, 2, 2]                           # rint: halves to even


def test_c4_variants_share_tensors():
    f, v = di.CONFIGS["C4f"], di.CONFIGS["C4v"]
    assert (f.seed, f.L, f.keep) == (v.seed, v.L, v.keep) and (f.vec, v.vec) == (1, 8)
