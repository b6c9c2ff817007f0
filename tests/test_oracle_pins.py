"""Pins for the CPU oracle: each check compares it with something that is not itself --
a closed form, the paper's other formulation of the same quantity, a library routine,
or brute force on tiny inputs.  No GPU needed.

Paper passages: equations 1-3 (dense attention), equation 4 (masked attention with the
additive constant c = 1e4), section 3.1 (approximate scores and top-k mask), section 4.2
(the same kept count in every row), section 5.1 (column-vector sparsity).
"""

import numpy as np
import pytest
import torch

import dsa_inputs as di


def paper_values():
    """tests/golden/paper_values.txt: `name = value  # citation` lines -> dict of floats."""
    from pathlib import Path
    out = {}
    for line in (Path(__file__).parent / "golden" / "paper_values.txt").read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            name, value = (t.strip() for t in line.split("="))
            out[name] = float(value)
    return out


PAPER = paper_values()


def tiny(seed, N=2, L=24, d=8, k=8, lo=-127, hi=127):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((N, L, d)).astype(np.float32)
    K = rng.standard_normal((N, L, d)).astype(np.float32)
    V = rng.standard_normal((N, L, d)).astype(np.float32)
    Qt = rng.integers(lo, hi + 1, (N, L, k)).astype(np.int8)
    Kt = rng.integers(lo, hi + 1, (N, L, k)).astype(np.int8)
    return Q, K, V, Qt, Kt


def python_topk(scores_row, keep):
    """Pure-Python statement of the selection rule: repeatedly take the best remaining key,
    best = highest score, lowest index among equals; report ascending."""
    remaining = list(range(len(scores_row)))
    chosen = []
    for _ in range(keep):
        best = remaining[0]
        for j in remaining[1:]:
            if scores_row[j] > scores_row[best]:
                best = j
        chosen.append(best)
        remaining.remove(best)
    return sorted(chosen)


# ---------------------------------------------------------------- keep from ratio
def test_keep_from_ratio_matches_counts_the_workloads_print(oracle):
    for cfg in di.CONFIGS.values():
        assert oracle.keep_from_ratio(cfg.L, cfg.ratio) == cfg.keep, cfg.name
    # the paper's worked example (section 4.3): DSA-90 on a row of length 2000 keeps 200 positions
    assert oracle.keep_from_ratio(int(PAPER["example_length"]), 1.0 - PAPER["example_sparsity"]) \
        == int(PAPER["example_kept_per_row"])
    c4 = di.CONFIGS["C4f"]          # the long-sequence workload takes the paper's profiling shape (section 5.1)
    assert (c4.H, c4.L, c4.d) == (int(PAPER["profiling_heads"]), int(PAPER["profiling_length"]),
                                  int(PAPER["profiling_head_dim"]))
    assert oracle.keep_from_ratio(100, 0.0) == 1           # clamped below
    assert oracle.keep_from_ratio(100, 2.0) == 100         # clamped above
    assert oracle.keep_from_ratio(10, 0.25) == 3           # 2.5 rounds up


# ---------------------------------------------------------------- step 1-2: integer scores
@pytest.mark.parametrize("k", [1, 16, 32, 64])
def test_scores_equal_int64_matmul(oracle, k):
    _, _, _, Qt, Kt = tiny(k, N=3, L=40, k=k)
    got = oracle.approx_scores(Qt, Kt).reshape(3, 40, 40)
    want = np.einsum("nic,njc->nij", Qt.astype(np.int64), Kt.astype(np.int64))
    assert np.array_equal(got, want)
    assert np.abs(got).max() <= k * 127 * 127


def test_scores_operand_order(oracle):
    # Q~ K~^T, not K~ Q~^T: a non-symmetric case with a known answer.
    Qt = np.zeros((1, 3, 2), np.int8); Kt = np.zeros((1, 3, 2), np.int8)
    Qt[0, 0] = [1, 0]; Qt[0, 1] = [0, 2]; Qt[0, 2] = [3, 3]
    Kt[0, 0] = [5, 0]; Kt[0, 1] = [0, 7]; Kt[0, 2] = [-1, 1]
    got = oracle.approx_scores(Qt, Kt)
    assert got.tolist() == [[5, 0, -1], [0, 14, 2], [15, 21, 0]]


@pytest.mark.parametrize("vec", [2, 8])
def test_group_scores_are_linear_in_the_query(oracle, vec):
    _, _, _, Qt, Kt = tiny(5, N=2, L=32, k=16)
    got = oracle.approx_scores(Qt, Kt, vec=vec).reshape(2, 32 // vec, 32)
    qsum = Qt.astype(np.int64).reshape(2, 32 // vec, vec, 16).sum(axis=2)
    want = np.einsum("ngc,njc->ngj", qsum, Kt.astype(np.int64))
    assert np.array_equal(got, want)
    # groups are aligned blocks of consecutive rows: group g = rows [vec*g, vec*g+vec)
    rows = oracle.approx_scores(Qt, Kt, vec=1).reshape(2, 32, 32)
    assert np.array_equal(got[1, 2], rows[1, 2 * vec:3 * vec].sum(axis=0))


def test_unit_subset_matches_full(oracle):
    _, _, _, Qt, Kt = tiny(6, N=3, L=16, k=8)
    full = oracle.approx_scores(Qt, Kt, vec=8)
    units = np.array([5, 0, 3], dtype=np.int64)
    assert np.array_equal(oracle.approx_scores(Qt, Kt, vec=8, units=units), full[units])
    fullidx = oracle.predict_mask(Qt, Kt, 5, vec=8)
    assert np.array_equal(oracle.predict_mask(Qt, Kt, 5, vec=8, units=units), fullidx[units])


# ---------------------------------------------------------------- step 3: top-k and ties
@pytest.mark.parametrize("lo,hi", [(-127, 127), (-2, 2), (0, 1)])
def test_topk_brute_force_all_keep(oracle, lo, hi):
    L = 20
    _, _, _, Qt, Kt = tiny(11 + hi, N=2, L=L, k=4, lo=lo, hi=hi)
    scores = np.einsum("nic,njc->nij", Qt.astype(np.int64), Kt.astype(np.int64)).reshape(2 * L, L)
    for keep in range(1, L + 1):
        got = oracle.predict_mask(Qt, Kt, keep)
        assert got.shape == (2 * L, keep)
        for u in range(2 * L):
            assert got[u].tolist() == python_topk(scores[u].tolist(), keep), (keep, u)


def test_topk_equals_stable_argsort(oracle):
    _, _, _, Qt, Kt = tiny(3, N=2, L=96, k=8, lo=-3, hi=3)
    for vec in (1, 8):
        scores = oracle.approx_scores(Qt, Kt, vec=vec)
        for keep in (1, 7, 48, 96):
            got = oracle.predict_mask(Qt, Kt, keep, vec=vec)
            order = np.argsort(-scores, axis=1, kind="stable")[:, :keep]   # stable: ties by index
            assert np.array_equal(got, np.sort(order, axis=1))


def test_tie_rule_lowest_index(oracle):
    L, k = 16, 4
    Qt = np.zeros((1, L, k), np.int8)
    Kt = np.random.default_rng(0).integers(-100, 100, (1, L, k)).astype(np.int8)
    for keep in (1, 5, 16):
        got = oracle.predict_mask(Qt, Kt, keep)               # every score is 0
        assert np.array_equal(got, np.tile(np.arange(keep, dtype=np.int32), (L, 1)))
    # duplicated key rows: the later copy is selected only if the earlier one is
    Qt = np.random.default_rng(1).integers(-100, 100, (1, L, k)).astype(np.int8)
    Kt[0, 9] = Kt[0, 2]
    for keep in range(1, L):
        for row in oracle.predict_mask(Qt, Kt, keep):
            assert (9 not in row) or (2 in row)


def test_every_unit_keeps_exactly_keep_distinct_ascending(oracle, workload):
    x = workload("C1")
    idx = oracle.predict_mask(x.Qt, x.Kt, x.cfg.keep)
    assert idx.shape == (x.cfg.units, x.cfg.keep)
    assert (np.diff(idx, axis=1) > 0).all() and idx.min() >= 0 and idx.max() < x.cfg.L


def test_signed_scores_not_magnitudes(oracle):
    # a large negative approximate score must lose against a small positive one
    Qt = np.array([[[1]]], np.int8).repeat(3, axis=1)
    Kt = np.array([[[-100], [1], [0]]], np.int8)
    assert oracle.predict_mask(Qt, Kt, 1).tolist() == [[1], [1], [1]]
    assert oracle.predict_mask(Qt, Kt, 2).tolist() == [[1, 2]] * 3


# ---------------------------------------------------------------- steps 4-6
def dense_attention_f64(Q, K, V, scale):
    S = np.einsum("nic,njc->nij", Q.astype(np.float64), K.astype(np.float64)) * float(scale)
    E = np.exp(S - S.max(axis=-1, keepdims=True))
    return (E / E.sum(axis=-1, keepdims=True)) @ V.astype(np.float64)


def test_keep_all_is_dense_attention(oracle):
    Q, K, V, Qt, Kt = tiny(21, N=3, L=33, d=16)
    scale = np.float32(0.25)
    O, idx = oracle.attention_fwd(Q, K, V, Qt, Kt, keep=33, scale=scale)
    assert np.array_equal(idx, np.tile(np.arange(33, dtype=np.int32), (99, 1)))
    want = dense_attention_f64(Q, K, V, scale).reshape(99, 16)
    assert np.abs(O - want).max() < 1e-12
    sdpa = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q).double(), torch.from_numpy(K).double(), torch.from_numpy(V).double(),
        scale=float(scale)).numpy().reshape(99, 16)
    assert np.abs(O - sdpa).max() < 1e-10


@pytest.mark.parametrize("vec", [1, 8])
def test_sparse_result_equals_additive_mask_form(oracle, vec):
    # equation 4: softmax(S - c (1 - M)) V with c = 1e4 and M scattered from idx
    Q, K, V, Qt, Kt = tiny(22, N=2, L=32, d=8)
    scale, keep = np.float32(8 ** -0.5), 5
    O, idx = oracle.attention_fwd(Q, K, V, Qt, Kt, keep=keep, scale=scale, vec=vec)
    M = np.zeros((2, 32, 32))
    for n in range(2):
        for i in range(32):
            M[n, i, idx[n * (32 // vec) + i // vec]] = 1.0
    S = np.einsum("nic,njc->nij", Q.astype(np.float64), K.astype(np.float64)) * float(scale)
    Sm = S - PAPER["mask_constant"] * (1.0 - M)
    E = np.exp(Sm - Sm.max(axis=-1, keepdims=True))
    A = E / E.sum(axis=-1, keepdims=True)
    assert (A[M == 0] == 0).all()                       # masked weights vanish exactly
    want = (A @ V.astype(np.float64)).reshape(64, 8)
    assert np.abs(O - want).max() < 1e-12


def test_staged_outputs_and_row_sums(oracle, workload):
    x = workload("C1")
    cfg = x.cfg
    idx = oracle.predict_mask(x.Qt, x.Kt, cfg.keep)
    O, S, P = oracle.masked_attention(x.Q, x.K, x.V, idx, cfg.scale, return_sp=True)
    assert (P >= 0).all() and np.abs(P.sum(axis=1) - 1.0).max() < 1e-12
    # each stage alone gives the same numbers as the chain
    assert np.array_equal(oracle.sddmm(x.Q, x.K, idx, cfg.scale), S)
    assert np.array_equal(oracle.sparse_softmax(S), P)
    assert np.array_equal(oracle.spmm(P, idx, x.V), O)
    # S against an independent gather + einsum
    Kg = x.K.reshape(cfg.N, cfg.L, cfg.d)[np.arange(cfg.N).repeat(cfg.L)[:, None], idx].astype(np.float64)
    want = np.einsum("rc,rtc->rt", x.Q.reshape(-1, cfg.d).astype(np.float64), Kg) * float(cfg.scale)
    assert np.abs(S - want).max() < 1e-12
    # softmax against scipy's
    from scipy.special import softmax
    assert np.abs(P - softmax(S, axis=1)).max() < 1e-14


def test_keep_one_copies_a_value_row(oracle):
    Q, K, V, Qt, Kt = tiny(23, N=2, L=24, d=8)
    O, idx = oracle.attention_fwd(Q, K, V, Qt, Kt, keep=1, scale=np.float32(1.0))
    scores = oracle.approx_scores(Qt, Kt)
    assert np.array_equal(idx[:, 0], scores.argmax(axis=1))    # argmax returns the first maximum
    for n in range(2):
        for i in range(24):
            assert np.array_equal(O[n * 24 + i], V[n, idx[n * 24 + i, 0]].astype(np.float64))


def test_identical_value_rows_pass_through(oracle):
    Q, K, V, Qt, Kt = tiny(24, N=1, L=16, d=4)
    V[:] = np.array([1.5, -2.0, 0.25, 3.0], np.float32)
    O, _ = oracle.attention_fwd(Q, K, V, Qt, Kt, keep=6, scale=np.float32(0.5))
    assert np.abs(O - V[0, 0].astype(np.float64)).max() < 1e-14


def test_identity_values_recover_weights(oracle):
    L = 12
    Q, K, _, Qt, Kt = tiny(25, N=1, L=L, d=L)
    V = np.eye(L, dtype=np.float32)[None]
    keep = 4
    idx = oracle.predict_mask(Qt, Kt, keep)
    O, S, P = oracle.masked_attention(Q, K, V, idx, np.float32(0.3), return_sp=True)
    want = np.zeros((L, L))
    for i in range(L):
        want[i, idx[i]] = P[i]
    assert np.array_equal(O, want)


def test_zero_queries_give_mean_of_first_keep_values(oracle):
    # closed form: Q = 0 and Q~ = 0 -> all scores tie -> keys 0..keep-1, uniform weights
    _, K, V, _, Kt = tiny(26, N=2, L=10, d=4)
    Q = np.zeros((2, 10, 4), np.float32)
    Qt = np.zeros((2, 10, 8), np.int8)
    O, idx = oracle.attention_fwd(Q, K, V, Qt, Kt, keep=3, scale=np.float32(1.0))
    want = V[:, :3].astype(np.float64).mean(axis=1)
    assert np.abs(O.reshape(2, 10, 4) - want[:, None, :]).max() < 1e-15


def test_two_key_closed_form(oracle):
    # one query, two kept keys: weights are the logistic function of the score difference
    Q = np.array([[[2.0, 0.0]] * 3], np.float32)
    K = np.array([[[1.0, 0.0], [0.0, 5.0], [-1.0, 0.0]]], np.float32)
    V = np.array([[[1.0, 10.0], [7.0, 7.0], [3.0, -10.0]]], np.float32)
    idx = np.array([[0, 2]] * 3, np.int32)
    scale = np.float32(0.5)
    O, S, P = oracle.masked_attention(Q, K, V, idx, scale, return_sp=True)
    assert S[0].tolist() == [1.0, -1.0]
    w = 1.0 / (1.0 + np.exp(-2.0))
    assert abs(P[0, 0] - w) < 1e-15 and abs(P[0, 1] - (1 - w)) < 1e-15
    assert np.abs(O[0] - (w * V[0, 0] + (1 - w) * V[0, 2])).max() < 1e-14


def test_vector_wise_rows_share_one_list(oracle):
    Q, K, V, Qt, Kt = tiny(27, N=2, L=32, d=8)
    idx = oracle.predict_mask(Qt, Kt, 6, vec=8)
    assert idx.shape == (2 * 4, 6)
    O8 = oracle.masked_attention(Q, K, V, idx, np.float32(0.4), vec=8)
    # same thing with the list repeated for each of the 8 rows and fine-grained execution
    O1 = oracle.masked_attention(Q, K, V, np.repeat(idx, 8, axis=0), np.float32(0.4), vec=1)
    assert np.array_equal(O8, O1)
    assert np.array_equal(oracle.predict_mask(Qt, Kt, 6, vec=1),
                          oracle.predict_mask(Qt, Kt, 6))     # vec=1 is the fine-grained rule


def test_permutation_equivariance(oracle):
    Q, K, V, Qt, Kt = tiny(28, N=1, L=24, d=8)
    keep, scale = 5, np.float32(0.35)
    O, idx = oracle.attention_fwd(Q, K, V, Qt, Kt, keep, scale)
    rng = np.random.default_rng(0)
    # permuting query rows permutes output rows
    pq = rng.permutation(24)
    O2, _ = oracle.attention_fwd(Q[:, pq], K, V, Qt[:, pq], Kt, keep, scale)
    assert np.array_equal(O2, O[pq])
    # permuting keys and values together leaves rows without a tie at the cut unchanged
    pk = rng.permutation(24)
    O3, idx3 = oracle.attention_fwd(Q, K[:, pk], V[:, pk], Qt, Kt[:, pk], keep, scale)
    scores = oracle.approx_scores(Qt, Kt)
    checked = 0
    for i in range(24):
        srt = np.sort(scores[i])[::-1]
        if srt[keep - 1] == srt[keep]:
            continue
        checked += 1
        assert set(pk[idx3[i]].tolist()) == set(idx[i].tolist())
        assert np.abs(O3[i] - O[i]).max() < 1e-13
    assert checked >= 12


def test_mask_recall_beats_random_on_the_workload(oracle, workload):
    # statistic from section 4.3 (overlap of the predicted set with the true top-k of S):
    # not a gate on a value, only that the untrained projection is far better than chance
    x = workload("C1")
    cfg = x.cfg
    idx = oracle.predict_mask(x.Qt, x.Kt, cfg.keep)
    S = np.einsum("nic,njc->nij", x.Q.reshape(cfg.N, cfg.L, cfg.d).astype(np.float64),
                  x.K.reshape(cfg.N, cfg.L, cfg.d).astype(np.float64)).reshape(-1, cfg.L)
    true = np.argsort(-S, axis=1, kind="stable")[:, :cfg.keep]
    recall = np.mean([len(set(a) & set(b)) / cfg.keep for a, b in zip(idx.tolist(), true.tolist())])
    assert recall > 3 * cfg.keep / cfg.L


def test_bad_arguments_raise(oracle):
    _, _, _, Qt, Kt = tiny(1, N=1, L=8, k=4)
    with pytest.raises(ValueError):
        oracle.predict_mask(Qt, Kt, 0)
    with pytest.raises(ValueError):
        oracle.predict_mask(Qt, Kt, 9)
    with pytest.raises(ValueError):
        oracle.predict_mask(Qt, Kt, 2, vec=3)


# ---------------------------------------------------------------- step 0: projection + int8 quantiser
def test_projection_quantiser_closed_forms(oracle):
    # amax = 127 makes the scale exactly 1: the codes are the projected values themselves
    X = np.array([[1.0, 2.0, 0.0], [0.5, 0.0, 0.0], [1.5, 0.0, 0.0], [2.5, 0.0, 0.0], [-2.5, 0.0, 0.0],
                  [0.0, 0.0, 127.0], [0.0, 0.0, -127.0]], np.float32)
    R = np.array([[1.0, -1.0], [10.0, 0.25], [1.0, 0.0]], np.float32)
    codes, amax = oracle.project_quantize(X, R)
    assert amax == np.float32(127.0)
    assert codes.tolist() == [[21, 0], [0, 0], [2, -2], [2, -2], [-2, 2], [127, 0], [-127, 0]]   # halves to even
    z, a0 = oracle.project_quantize(np.zeros((5, 3), np.float32), R)
    assert a0 == 0 and not z.any()
    # operand order: X [rows, d] times R [d, k], not its transpose
    X2 = np.array([[1.0, 0.0], [0.0, 1.0]], np.float32)
    R2 = np.array([[127.0, 1.0], [2.0, 3.0]], np.float32)
    assert oracle.project_quantize(X2, R2)[0].tolist() == [[127, 1], [2, 3]]


def test_projection_quantiser_against_float64(oracle, workload):
    # the fp32 recipe may move a code by one step where float64 lands next to a rounding boundary
    x = workload("C1")
    for T, want in ((x.Q, x.Qt), (x.K, x.Kt)):
        codes, amax = oracle.project_quantize(T, x.R.astype(np.float32))
        y64 = T.astype(np.float64) @ x.R.astype(np.float32).astype(np.float64)
        assert abs(float(amax) - np.abs(y64).max()) <= 1e-5 * np.abs(y64).max()
        ref = di.quantize_int8(y64)
        diff = np.abs(codes.astype(np.int32) - ref.astype(np.int32))
        assert diff.max() <= 1 and (diff != 0).mean() < 2e-3
        # and the workload's own codes (float64 R) are the same up to the same kind of step
        d2 = np.abs(codes.astype(np.int32) - want.astype(np.int32))
        assert d2.max() <= 1 and (d2 != 0).mean() < 2e-2


# ---------------------------------------------------------------- lower prediction precision (section 3.3, table 2)
def test_low_precision_quantiser_closed_forms(oracle):
    # INT4: amax = 7 makes the scale exactly 1, the codes are the projected values, halves go to even
    X = np.array([[7.0], [-7.0], [0.5], [1.5], [2.5], [-3.5], [6.4], [6.6]], np.float32)
    R = np.array([[1.0]], np.float32)
    codes, amax = oracle.project_quantize(X, R, bits=4)
    assert amax == np.float32(7.0)
    assert codes[:, 0].tolist() == [7, -7, 0, 2, 2, -4, 6, 7]
    # INT2: three levels; with amax = 1 the boundaries sit at +-0.5 (halves to even: to 0)
    X2 = np.array([[1.0], [-1.0], [0.5], [-0.5], [0.51], [-0.51], [0.0]], np.float32)
    codes2, amax2 = oracle.project_quantize(X2, R, bits=2)
    assert amax2 == np.float32(1.0)
    assert codes2[:, 0].tolist() == [1, -1, 0, 0, 1, -1, 0]
    # the same tensor at 8 bits uses the full int8 range
    assert oracle.project_quantize(X, R, bits=8)[0][:, 0].tolist() == [127, -127, 9, 27, 45, -64, 116, 120]


@pytest.mark.parametrize("bits", [4, 2])
def test_low_precision_codes_against_float64(oracle, workload, bits):
    x = workload("C1")
    qmax = 2 ** (bits - 1) - 1
    R32 = x.R.astype(np.float32)
    codes, amax = oracle.project_quantize(x.K, R32, bits=bits)
    assert codes.min() >= -qmax and codes.max() <= qmax and np.abs(codes).max() == qmax
    y64 = x.K.astype(np.float64) @ R32.astype(np.float64)
    ref = np.clip(np.rint(y64 * (qmax / np.abs(y64).max())), -qmax, qmax)
    diff = np.abs(codes.astype(np.int32) - ref.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 1e-3


def test_code_packing_layout(oracle):
    # hand-worked bytes: low field first, two's complement fields
    assert oracle.pack_codes(np.array([[7, -7, 0, 1, -1, 3, -4, 5]], np.int8), 4).tolist() == [[0x97, 0x10, 0x3F, 0x5C]]
    assert oracle.pack_codes(np.array([[1, -1, 0, 1, 0, 0, -1, -1]], np.int8), 2).tolist() == [[0b01001101, 0b11110000]]
    assert oracle.pack_codes(np.array([[-5, 100]], np.int8), 8).tolist() == [[251, 100]]
    # every byte value unpacks to what plain integer arithmetic on its fields gives
    allb = np.arange(256, dtype=np.uint8).reshape(1, 256)
    for bits in (4, 2):
        per, half = 8 // bits, 1 << (bits - 1)
        got = oracle.unpack_codes(allb, bits).reshape(256, per)
        for b in range(256):
            fields = [(b >> (bits * f)) % (1 << bits) for f in range(per)]
            assert got[b].tolist() == [v - (1 << bits) if v >= half else v for v in fields]
    # round trip over the whole code range, and a code outside it is refused
    rng = np.random.default_rng(5)
    for bits in (4, 2, 8):
        qmax = 2 ** (bits - 1) - 1
        c = rng.integers(-qmax, qmax + 1, size=(3, 5, 32)).astype(np.int8)
        p = oracle.pack_codes(c, bits)
        assert p.shape == (3, 5, 32 * bits // 8)
        assert np.array_equal(oracle.unpack_codes(p, bits), c)
    with pytest.raises(ValueError):
        oracle.pack_codes(np.array([[8, 0]], np.int8), 4)


def test_low_precision_mask_is_the_mask_of_the_codes(oracle, workload):
    # the predictor sees the integer codes whatever their storage: packing and unpacking changes nothing,
    # and with so few levels ties are everywhere, so the lower index must win often
    x = workload("C1")
    cfg = x.cfg
    R32 = x.R.astype(np.float32)
    q4, _ = oracle.project_quantize(x.Q, R32, bits=4)
    k4, _ = oracle.project_quantize(x.K, R32, bits=4)
    idx = oracle.predict_mask(q4, k4, cfg.keep, cfg.vec)
    back = oracle.predict_mask(oracle.unpack_codes(oracle.pack_codes(q4, 4), 4),
                               oracle.unpack_codes(oracle.pack_codes(k4, 4), 4), cfg.keep, cfg.vec)
    assert np.array_equal(idx, back)
    S = oracle.approx_scores(q4, k4, cfg.vec)
    order = np.argsort(-S, axis=1, kind="stable")[:, :cfg.keep]
    assert np.array_equal(np.sort(order, axis=1), idx)
    kth = np.take_along_axis(S, order[:, -1:], axis=1)
    assert ((S == kth).sum(1) > 1).mean() > 0.5      # most rows have a tie at the threshold


def test_column_locality_counts_on_a_hand_example():
    """Figure 11's accounting on a case small enough to count by hand (section 5.2, table 4)."""
    from oracle import column_locality as cl
    # 4 elements, 3 kept keys each; key 7 is wanted by all, key 2 by two
    tile = np.array([[1, 2, 7], [2, 5, 7], [0, 7, 9], [3, 4, 7]])
    assert cl.fetches_in_order(tile) == 4 + 4 + 2          # steps: {1,2,0,3}, {2,5,7,4}, {7,9}
    assert cl.fetches_union(tile) == 8                     # 0 1 2 3 4 5 7 9
    g = cl.fetches_greedy(tile)
    assert cl.fetches_union(tile) <= g <= 12               # feasible, never worse than row-by-row
    assert g == 8                                          # 7 once for all four; 2 once for two; 0 3 | 1 5 9 4 alone
    same = np.tile(np.arange(5), (8, 1))                   # identical lists: one fetch per step
    assert cl.fetches_in_order(same) == 5 and cl.fetches_greedy(same) == 5 and cl.fetches_union(same) == 5
    f = cl.reduction_factors(same, 1, 8)
    assert f["in_order"] == 8.0 and f["reordered_greedy"] == 8.0 and f["reordered_floor"] == 8.0


# ---------------------------------------------------------------- threshold masks (CSR)
def python_threshold(scores, theta):
    """Pure-Python statement of the threshold rule for one unit: every key at or above theta, ascending;
    if there is none, the single best key (highest score, lowest index among equals)."""
    kept = [j for j in range(len(scores)) if scores[j] >= theta]
    if not kept:
        best = 0
        for j in range(1, len(scores)):
            if scores[j] > scores[best]:
                best = j
        kept = [best]
    return kept


@pytest.mark.parametrize("vec,lo,hi", [(1, -127, 127), (1, -2, 2), (4, -5, 5), (8, -127, 127)])
def test_threshold_mask_brute_force(oracle, vec, lo, hi):
    # section 3.1: masks "using thresholds"; every theta from below every score to above every score
    _, _, _, Qt, Kt = tiny(40 + vec, N=2, L=24, k=8, lo=lo, hi=hi)
    sc = oracle.approx_scores(Qt, Kt, vec)
    thetas = sorted(set(np.quantile(sc, [0, 0.2, 0.5, 0.9, 0.99, 1.0]).astype(np.int64).tolist()
                        + [int(sc.min()) - 1, int(sc.max()) + 1, 0]))
    for theta in thetas:
        row_ptr, col = oracle.predict_mask_threshold(Qt, Kt, theta, vec)
        assert row_ptr[0] == 0 and row_ptr.shape == (sc.shape[0] + 1,) and row_ptr[-1] == col.size
        for u in range(sc.shape[0]):
            assert col[row_ptr[u]:row_ptr[u + 1]].tolist() == python_threshold(sc[u].tolist(), theta), (theta, u)


def test_threshold_empty_units_keep_their_best_key_lowest_index(oracle):
    _, _, _, Qt, Kt = tiny(44, N=1, L=16, k=8, lo=-3, hi=3)
    Kt[0, 5] = Kt[0, 2]                                  # equal scores for keys 2 and 5 in every unit
    sc = oracle.approx_scores(Qt, Kt, 1)
    row_ptr, col = oracle.predict_mask_threshold(Qt, Kt, int(sc.max()) + 1, 1)
    assert (np.diff(row_ptr) == 1).all()
    assert col.tolist() == [int(np.argmax(s)) for s in sc]          # argmax: first maximum
    Qz = np.zeros_like(Qt)                               # all scores 0: key 0 for every unit
    _, col0 = oracle.predict_mask_threshold(Qz, Kt, 1, 1)
    assert (col0 == 0).all()


def test_threshold_at_the_kth_score_is_the_topk_mask(oracle):
    # with no tie at the cut, "score >= k-th largest score" is the top-k mask of section 3.1
    _, _, _, Qt, Kt = tiny(45, N=1, L=32, k=8)
    sc = oracle.approx_scores(Qt, Kt, 1)
    keep = 6
    for u in range(sc.shape[0]):
        srt = np.sort(sc[u])[::-1]
        if srt[keep - 1] == srt[keep]:
            continue
        row_ptr, col = oracle.predict_mask_threshold(Qt, Kt, int(srt[keep - 1]), 1)
        want = oracle.predict_mask(Qt, Kt, keep, 1)[u]
        assert col[row_ptr[u]:row_ptr[u + 1]].tolist() == want.tolist()


@pytest.mark.parametrize("vec", [1, 8])
def test_csr_attention_equals_additive_mask_form(oracle, vec):
    # equation 4 with the mask scattered from the CSR lists, c = 1e4; counts differ from row to row
    Q, K, V, Qt, Kt = tiny(46, N=2, L=32, d=8)
    scale = np.float32(8 ** -0.5)
    sc = oracle.approx_scores(Qt, Kt, vec)
    theta = int(np.quantile(sc, 0.85))
    row_ptr, col = oracle.predict_mask_threshold(Qt, Kt, theta, vec)
    counts = np.diff(row_ptr)
    assert counts.min() >= 1 and counts.max() > counts.min()
    O = oracle.masked_attention_csr(Q, K, V, row_ptr, col, scale, vec)
    G = 32 // vec
    M = np.zeros((2, 32, 32))
    for n in range(2):
        for i in range(32):
            u = n * G + i // vec
            M[n, i, col[row_ptr[u]:row_ptr[u + 1]]] = 1.0
    S = np.einsum("nic,njc->nij", Q.astype(np.float64), K.astype(np.float64)) * float(scale)
    Sm = S - PAPER["mask_constant"] * (1.0 - M)
    E = np.exp(Sm - Sm.max(axis=-1, keepdims=True))
    A = E / E.sum(axis=-1, keepdims=True)
    want = (A @ V.astype(np.float64)).reshape(64, 8)
    assert np.abs(O - want).max() < 1e-12
    # a subset of rows gives the same rows
    rows = np.array([3, 17, 40, 63])
    assert np.array_equal(oracle.masked_attention_csr(Q, K, V, row_ptr, col, scale, vec, rows=rows), O[rows])


def test_csr_attention_with_equal_counts_is_the_ell_result(oracle):
    Q, K, V, Qt, Kt = tiny(47, N=2, L=24, d=8)
    scale, keep = np.float32(0.3), 5
    idx = oracle.predict_mask(Qt, Kt, keep, 1)
    row_ptr = np.arange(idx.shape[0] + 1, dtype=np.int64) * keep
    O_csr = oracle.masked_attention_csr(Q, K, V, row_ptr, idx.reshape(-1), scale, 1)
    assert np.abs(O_csr - oracle.masked_attention(Q, K, V, idx, scale, 1)).max() < 1e-15
    # one key: the value row itself
    one = oracle.masked_attention_csr(Q, K, V, np.arange(49, dtype=np.int64), idx[:, 0].copy(), scale, 1)
    assert np.array_equal(one, V.reshape(48, 8)[np.arange(48) // 24 * 24 + idx[:, 0]].astype(np.float64))


# ---------------------------------------------------------------- ternary projection (equation 5)
def test_ternary_projection_closed_forms_and_dense_equivalent(oracle):
    rng = np.random.default_rng(50)
    d, k, rows = 12, 8, 40
    X = rng.standard_normal((rows, d)).astype(np.float32)
    # the usual sparse random projection: -1, 0, 1 with probabilities 1/6, 2/3, 1/6
    P3 = rng.choice(np.array([-1, 0, 1], dtype=np.int8), size=(d, k), p=[1 / 6, 2 / 3, 1 / 6])
    codes, amax = oracle.project_quantize_ternary(X, P3)
    # sums and differences, written out in float64 (exact for these few terms up to fp32 rounding of each sum)
    Y = np.zeros((rows, k), dtype=np.float32)
    for c in range(d):
        for j in range(k):
            if P3[c, j] > 0:
                Y[:, j] = Y[:, j] + X[:, c]
            elif P3[c, j] < 0:
                Y[:, j] = Y[:, j] - X[:, c]
    assert amax == np.float32(np.abs(Y).max())
    want = np.clip(np.rint(Y * (np.float32(127) / np.float32(amax))), -127, 127).astype(np.int8)
    assert np.array_equal(codes, want)
    # the same codes as the dense projection with the signs as its matrix, at every precision
    for bits in (8, 4, 2):
        a, am = oracle.project_quantize_ternary(X, P3, bits)
        b, bm = oracle.project_quantize(X, P3.astype(np.float32), bits)
        assert np.array_equal(a, b) and am == bm
    # a column with a single +1 copies an input column; a single -1 negates it; an empty column gives zeros
    P1 = np.zeros((d, 3), dtype=np.int8)
    P1[4, 0], P1[7, 1] = 1, -1
    Xi = rng.integers(-127, 128, (rows, d)).astype(np.float32)
    Xi[0, 4] = 127.0
    c1, a1 = oracle.project_quantize_ternary(Xi, P1)
    assert a1 == 127.0 and np.array_equal(c1[:, 0], Xi[:, 4].astype(np.int8))
    assert np.array_equal(c1[:, 1], np.clip(-Xi[:, 7], -127, 127).astype(np.int8)) and (c1[:, 2] == 0).all()
    with pytest.raises(ValueError):
        oracle.project_quantize_ternary(X, np.full((d, k), 2, dtype=np.int8))
