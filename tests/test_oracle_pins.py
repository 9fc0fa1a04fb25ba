"""Pins for the float64 oracle: closed forms, invariants, library special cases
and brute force.  Nothing here touches the HIP library.

Each pin is chosen so that a plausible slip in the oracle (a dropped term, a
wrong sign or index, a transposed operand, sample instead of population std,
floor instead of ceil, ...) fails at least one test.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import compactor_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "leverage_closed_forms.txt")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- golden file
def _parse_matrix(txt):
    return np.array([[float(Fraction(x)) for x in row.split()] for row in txt.split(";")])


def _load_cases():
    cases, cur = [], None
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, rest = line.partition(" ")
            if key == "case":
                cur = {"name": rest, "ridge_rel": 0.0, "Phi": None}
                cases.append(cur)
            elif key == "K":
                cur["K"] = _parse_matrix(rest)
            elif key == "Phi":
                cur["Phi"] = _parse_matrix(rest)
            elif key == "ridge_rel":
                cur["ridge_rel"] = float(rest)
            elif key == "expect":
                cur["expect"] = np.array([float(Fraction(x)) for x in rest.split()])
            elif key == "cite":
                cur["cite"] = rest
    return cases


@pytest.mark.parametrize("case", _load_cases(), ids=lambda c: c["name"])
def test_closed_form_cases(case):
    K, Phi, rr, want = case["K"], case["Phi"], case["ridge_rel"], case["expect"]
    full_rank = np.linalg.matrix_rank(K) == K.shape[1]
    if Phi is None:
        if rr == 0.0:
            np.testing.assert_allclose(O.leverage_svd(K), want, atol=1e-12)
            np.testing.assert_allclose(O.leverage_hat_diagonal(K), want, atol=1e-12)
        if full_rank or rr > 0:
            np.testing.assert_allclose(O.leverage_ridge_exact(K, rr), want, atol=1e-12)
    else:
        np.testing.assert_allclose(O.approx_leverage_alg1(K, Phi), want, atol=1e-12)
        np.testing.assert_allclose(O.approx_leverage_ridge(K, Phi, rr), want, atol=1e-12)
        np.testing.assert_allclose(O.approx_leverage_qr(K, Phi), want, atol=1e-12)
        np.testing.assert_allclose(O.approx_leverage_eig(K, Phi, eps=1e-300), want, atol=1e-12)


# ---------------------------------------------------------------- bf16 widening
def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4000, 0x3F00, 0x41A0, 0x3DCD, 0x8000], dtype=np.uint16)
    want = np.array([0.0, 1.0, -1.0, 2.0, 0.5, 20.0, 0.10009765625, -0.0])
    got = O.bf16_bits_to_f64(bits)
    assert np.array_equal(got, want)
    assert np.signbit(got[-1])


# ---------------------------------------------------------------- P1, P2
@pytest.mark.parametrize("n,d", [(40, 7), (300, 16), (129, 128)])
def test_exact_scores_in_unit_interval_and_sum_to_rank(n, d):
    K = _rng(n + d).standard_normal((n, d))
    for o in (O.leverage_svd(K), O.leverage_ridge_exact(K), O.leverage_hat_diagonal(K)):
        assert o.min() >= -1e-12 and o.max() <= 1 + 1e-12
        assert abs(o.sum() - d) < 1e-8          # Definition 1: sum = rank(K)


def test_sum_is_rank_for_rank_deficient_K():
    r = _rng(0)
    K = r.standard_normal((200, 5)) @ r.standard_normal((5, 12))   # rank 5
    assert abs(O.leverage_svd(K).sum() - 5) < 1e-8
    assert abs(O.leverage_hat_diagonal(K).sum() - 5) < 1e-6


@pytest.mark.parametrize("ridge_rel", [1e-4, 0.3, 2.0])
def test_ridge_sum_closed_form(ridge_rel):
    # sum_i k_i^T (G + rho I)^-1 k_i = trace(G (G + rho I)^-1) = sum_j mu_j / (mu_j + rho)
    r = _rng(3)
    K = r.standard_normal((150, 9)) * r.uniform(0.1, 5.0, 9)
    mu = np.linalg.eigvalsh(K.T @ K)
    rho = ridge_rel * mu.sum() / 9
    o = O.leverage_ridge_exact(K, ridge_rel)
    assert abs(o.sum() - np.sum(mu / (mu + rho))) < 1e-9
    assert o.min() >= 0 and o.max() <= 1
    # a ridge can only lower every score
    assert np.all(o <= O.leverage_ridge_exact(K, 0.0) + 1e-12)

    Phi = r.standard_normal((9, 4))
    Kh = K @ Phi
    mu = np.linalg.eigvalsh(Kh.T @ Kh)
    rho = ridge_rel * mu.sum() / 4
    assert abs(O.approx_leverage_ridge(K, Phi, ridge_rel).sum() - np.sum(mu / (mu + rho))) < 1e-9


# ---------------------------------------------------------------- P3
def test_exact_scores_invariant_under_right_multiplication():
    r = _rng(4)
    K = r.standard_normal((120, 10))
    A = r.standard_normal((10, 10)) + 3 * np.eye(10)
    base = O.leverage_ridge_exact(K)
    np.testing.assert_allclose(O.leverage_ridge_exact(K @ A), base, atol=1e-9)
    # the 4 outlier channels x20 of the synthetic keys must not move exact scores
    s = np.ones(10); s[[1, 4, 6, 9]] = 20.0
    np.testing.assert_allclose(O.leverage_ridge_exact(K * s), base, atol=1e-9)
    np.testing.assert_allclose(O.leverage_svd(K * s), base, atol=1e-9)


# ---------------------------------------------------------------- P4
def test_orthonormal_special_cases():
    r = _rng(5)
    Q, _ = np.linalg.qr(r.standard_normal((60, 8)))
    want = np.sum(Q * Q, axis=1)
    for f in (O.leverage_svd, O.leverage_ridge_exact, O.leverage_hat_diagonal):
        np.testing.assert_allclose(f(Q), want, atol=1e-10)
    # square invertible K: every row has leverage 1
    Ksq = r.standard_normal((8, 8)) + 4 * np.eye(8)
    np.testing.assert_allclose(O.leverage_ridge_exact(Ksq), np.ones(8), atol=1e-9)
    # rank one
    u, v = r.standard_normal(30), r.standard_normal(6)
    np.testing.assert_allclose(O.leverage_svd(np.outer(u, v)), u * u / (u @ u), atol=1e-10)


# ---------------------------------------------------------------- P5
@pytest.mark.parametrize("seed", [0, 1])
def test_three_independent_routes_agree(seed):
    r = _rng(10 + seed)
    K = r.standard_normal((257, 24)) * r.uniform(0.05, 20.0, 24)
    hat = O.leverage_hat_diagonal(K)
    U, _, _ = np.linalg.svd(K, full_matrices=False)
    Q, _ = np.linalg.qr(K)
    np.testing.assert_allclose(O.leverage_ridge_exact(K), hat, rtol=1e-7, atol=1e-10)
    np.testing.assert_allclose(O.leverage_svd(K), np.sum(U * U, axis=1), atol=1e-10)
    np.testing.assert_allclose(O.leverage_ridge_exact(K), np.sum(Q * Q, axis=1), rtol=1e-7, atol=1e-10)


# ---------------------------------------------------------------- Algorithm 1
def _sketch_case(seed, n=400, d=32, ks=12):
    r = _rng(seed)
    K = r.standard_normal((n, d)) * r.uniform(0.1, 10.0, d)
    Phi = r.standard_normal((d, ks)) / math.sqrt(ks)
    return r, K, Phi


def test_alg1_equals_leverage_of_sketched_matrix():
    # Theorem 2 defines the approximate score as the leverage score of K Phi.
    _, K, Phi = _sketch_case(20)
    want = O.leverage_svd(K @ Phi)
    np.testing.assert_allclose(O.approx_leverage_alg1(K, Phi), want, rtol=1e-8, atol=1e-12)
    np.testing.assert_allclose(O.approx_leverage_ridge(K, Phi, 0.0), want, rtol=1e-8, atol=1e-12)
    np.testing.assert_allclose(O.approx_leverage_qr(K, Phi), want, rtol=1e-8, atol=1e-12)
    np.testing.assert_allclose(O.approx_leverage_eig(K, Phi, eps=1e-300), want, rtol=1e-8, atol=1e-12)
    assert abs(want.sum() - Phi.shape[1]) < 1e-8             # rank(K Phi) = k_s


def test_sketched_scores_depend_only_on_range_of_K_Phi():       # P6
    r, K, Phi = _sketch_case(21)
    base = O.approx_leverage_ridge(K, Phi)
    B = r.standard_normal((12, 12)) + 3 * np.eye(12)
    np.testing.assert_allclose(O.approx_leverage_ridge(K, Phi @ B), base, rtol=1e-8, atol=1e-12)
    np.testing.assert_allclose(O.approx_leverage_alg1(K, 7.5 * Phi), base, rtol=1e-8, atol=1e-12)
    # k_s = d and invertible Phi: the sketch is a change of basis, scores are exact
    Phi_sq = r.standard_normal((32, 32)) + 5 * np.eye(32)
    np.testing.assert_allclose(O.approx_leverage_ridge(K, Phi_sq), O.leverage_ridge_exact(K),
                               rtol=1e-7, atol=1e-12)
    np.testing.assert_allclose(O.approx_leverage_alg1(K, Phi_sq), O.leverage_svd(K),
                               rtol=1e-7, atol=1e-12)


def test_sketched_score_never_exceeds_exact_score():             # P7
    # range(K Phi) is a subspace of range(K): projecting onto less can only shrink.
    _, K, Phi = _sketch_case(22)
    assert np.all(O.approx_leverage_ridge(K, Phi) <= O.leverage_ridge_exact(K) + 1e-10)


def test_alg1_pseudo_inverse_when_sketched_gram_is_singular():
    r = _rng(23)
    K = r.standard_normal((50, 3)) @ r.standard_normal((3, 16))      # rank 3 < k_s
    Phi = r.standard_normal((16, 6))
    o = O.approx_leverage_alg1(K, Phi)
    assert abs(o.sum() - 3) < 1e-6 and o.max() <= 1 + 1e-9
    np.testing.assert_allclose(o, O.leverage_svd(K @ Phi), atol=1e-7)


def test_eig_clamp_only_lowers_scores():
    _, K, Phi = _sketch_case(24)
    assert np.all(O.approx_leverage_eig(K, Phi, eps=1e-6) <= O.approx_leverage_alg1(K, Phi) + 1e-12)


# ---------------------------------------------------------------- P8
def test_duplicates_and_row_permutation():
    r = _rng(30)
    K = r.standard_normal((90, 6))
    K[[7, 20, 55]] = K[3]                                   # 4 identical rows
    o = O.leverage_ridge_exact(K)
    assert o[3] == o[7] == o[20] == o[55]
    assert o[3] <= 0.25 + 1e-12                             # m copies: each at most 1/m
    p = r.permutation(90)
    np.testing.assert_allclose(O.leverage_ridge_exact(K[p]), o[p], atol=1e-10)
    Phi = r.standard_normal((6, 3))
    os_ = O.approx_leverage_ridge(K, Phi)
    assert os_[3] == os_[7] == os_[20] == os_[55]
    np.testing.assert_allclose(O.approx_leverage_ridge(K[p], Phi), os_[p], atol=1e-10)


# ---------------------------------------------------------------- P9 select / compact
def _brute_topk(s, k):
    """Repeatedly take the best remaining score: a number beats a NaN, a larger number beats a
    smaller one (float32 comparison, -0.0 = +0.0), the lowest index wins among equals."""
    s = [float(np.float32(x)) for x in s]

    def better(i, j):                     # is token i strictly better than token j?
        if s[i] != s[i] or s[j] != s[j]:
            return s[i] == s[i] and s[j] != s[j]
        return s[i] > s[j]
    left = list(range(len(s)))
    out = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if better(i, best):
                best = i
        out.append(best)
        left.remove(best)
    return sorted(out)


def test_select_ranks_nan_below_minus_infinity():
    """Sec. 3.3 says nothing about scores that are not numbers (they arise only from non-finite
    keys).  Reading: every number, -inf included, outranks a NaN; NaNs among themselves go by
    lower index.  Hand-written expectations for one head holding both."""
    inf, nan = math.inf, math.nan
    s = np.array([nan, -inf, 0.5, nan, -inf, inf, -1.0])
    assert O.select_topk(s, 1).tolist() == [5]
    assert O.select_topk(s, 3).tolist() == [2, 5, 6]
    assert O.select_topk(s, 4).tolist() == [1, 2, 5, 6]          # first -inf before any NaN
    assert O.select_topk(s, 5).tolist() == [1, 2, 4, 5, 6]       # second -inf, still no NaN
    assert O.select_topk(s, 6).tolist() == [0, 1, 2, 4, 5, 6]    # NaNs last, lower index first
    for k in range(1, 8):
        assert O.select_topk(s, k).tolist() == _brute_topk(s, k)
    # the same rule across the heads of a layer
    S = np.array([[nan, -inf, 1.0], [-inf, nan, 2.0]])
    got = O.select_topk_layer(S, 4)
    assert [g.tolist() for g in got] == [[1, 2], [0, 2]]
    got = O.select_topk_layer(S, 5)
    assert [g.tolist() for g in got] == [[0, 1, 2], [0, 2]]


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_brute_force(seed):
    r = _rng(40 + seed)
    n = int(r.integers(1, 60))
    s = r.integers(-3, 4, n).astype(np.float64) / 4.0       # many exact ties, both signs, zeros
    if seed == 3:
        s[r.integers(0, n)] = np.nan
    if seed == 5:                                           # NaN and -inf in one head
        s[r.integers(0, n, 3)] = np.nan
        s[r.integers(0, n, 3)] = -np.inf
    if seed == 4:
        s = np.where(s == 0, -0.0, s)                       # -0.0 ties with +0.0
    for k in {1, max(1, n // 3), n}:
        got = O.select_topk(s, k)
        assert got.dtype == np.int32
        assert got.tolist() == _brute_topk(s, k)


def test_select_properties_and_compact():
    r = _rng(50)
    n, k = 1000, 317
    s = r.standard_normal(n)
    kept = O.select_topk(s, k)
    assert len(kept) == k and np.all(np.diff(kept) > 0)
    mask = np.zeros(n, bool); mask[kept] = True
    assert s[mask].min() >= s[~mask].max()
    Kb = r.integers(0, 65536, (n, 8)).astype(np.uint16)
    Vb = r.integers(0, 65536, (n, 8)).astype(np.uint16)
    Kp, Vp = O.compact_rows(Kb, Vb, kept)
    assert np.array_equal(Kp, Kb[kept]) and np.array_equal(Vp, Vb[kept])
    # r = 1 keeps everything in order
    assert np.array_equal(O.select_topk(s, n), np.arange(n))


@pytest.mark.parametrize("n,r,want", [
    (4096, 0.5, 2048), (32768, 0.3, 9831), (131072, 0.2, 26215), (100000, 0.32, 32000),
    (10, 1.0, 10), (10, 1e-6, 1), (7, 0.5, 4), (1, 0.2, 1), (0, 0.5, 0), (1000, 0.001, 1),
    (3, 1 / 3, 1),
])
def test_keep_count(n, r, want):
    assert O.keep_count(n, r) == want


# ---------------------------------------------------------------- P10 blend
def test_blend():
    r = _rng(60)
    a, o = np.exp(r.standard_normal(500)), r.uniform(0, 1, 500)
    za, zo = O.zscore(a), O.zscore(o)
    for z in (za, zo):
        assert abs(z.mean()) < 1e-12 and abs(np.mean(z * z) - 1) < 1e-12   # population std
    s = O.blend_scores(a, o, 0.3)
    np.testing.assert_allclose(s, za + 0.3 * zo, atol=1e-12)
    # hand value: a=(1,3), o=(4,0): z(a)=(-1,1), z(o)=(1,-1) -> s=(-1+lam, 1-lam)
    np.testing.assert_allclose(O.blend_scores(np.array([1.0, 3.0]), np.array([4.0, 0.0]), 0.3),
                               [-0.7, 0.7], atol=1e-15)
    # lam = 0 ranks by a only; constant a ranks by o only; a = None is s = o
    assert np.array_equal(np.argsort(-O.blend_scores(a, o, 0.0)), np.argsort(-a))
    assert np.array_equal(np.argsort(-O.blend_scores(np.full(500, 2.0), o, 0.3)), np.argsort(-o))
    assert np.array_equal(O.blend_scores(None, o), o)


# ---------------------------------------------------------------- P11 calibration
@pytest.mark.parametrize("b", [0.5, 3.0, 10.0])
@pytest.mark.parametrize("tau", [0.5, 0.9, 0.95])
def test_calibration_curve_and_inverse(b, tau):
    alpha, beta, nll = 0.7, 0.2, (b - 0.2) / 0.7
    f = lambda r: float(O.calibration_curve(r, nll, alpha, beta))
    assert abs(f(0.0)) < 1e-15 and abs(f(1.0) - 1.0) < 1e-15
    rs = np.linspace(0, 1, 101)
    assert np.all(np.diff(O.calibration_curve(rs, nll, alpha, beta)) > 0)
    rstar = O.calibrated_ratio(nll, alpha, beta, tau)
    assert 0 < rstar <= 1 and abs(f(rstar) - tau) < 1e-12
    assert f(rstar - 1e-6) < tau                              # smallest such r


def test_calibration_hand_value():
    # b = ln 2, tau = 1/2: f(r) = (2^r/2 - 1/2)/(1/2) = 2^r - 1 >= 1/2  <=>  r >= log2(3/2)
    assert abs(O.calibrated_ratio(1.0, math.log(2.0), 0.0, 0.5) - math.log2(1.5)) < 1e-14
    assert O.calibrated_ratio(1.0, 1.0, 0.0, 1.0) == 1.0


# ---------------------------------------------------------------- end to end on one head
def test_compress_head_end_to_end_small():
    r = _rng(70)
    n, d, ks = 300, 16, 6
    K = r.standard_normal((n, d)); K[:, [2, 9]] *= 20
    Kb = r.integers(0, 65536, (n, d)).astype(np.uint16)
    Vb = r.integers(0, 65536, (n, d)).astype(np.uint16)
    Phi = r.standard_normal((d, ks)) / math.sqrt(ks)
    s, kept, Kp, Vp = O.compress_head(K, Kb, Vb, 0.25, Phi)
    assert len(kept) == 75
    np.testing.assert_allclose(s, O.leverage_svd(K @ Phi), rtol=1e-8)
    assert np.array_equal(Kp, Kb[kept]) and np.array_equal(Vp, Vb[kept])
    s2, kept2, _, _ = O.compress_head(K, Kb, Vb, 0.25, None)
    np.testing.assert_allclose(s2, O.leverage_hat_diagonal(K), rtol=1e-7)
    assert kept2.tolist() == _brute_topk(s2, 75)


# ---------------------------------------------------------------- attention scores (Sec. 3.2)
def _brute_attention(Q, K, chunk, scale):
    n = K.shape[0]
    a = [0.0] * n
    for i in range(n):                       # query i attends inside its own block only
        lo = (i // chunk) * chunk
        hi = min(n, lo + chunk)
        logits = [scale * float(np.dot(Q[i], K[j])) for j in range(lo, hi)]
        m = max(logits)
        w = [math.exp(x - m) for x in logits]
        z = sum(w)
        for t, j in enumerate(range(lo, hi)):
            a[j] += w[t] / z
    return np.array(a)


def test_attention_scores_raw_against_brute_force_and_invariants():
    r = _rng(80)
    n, d, C = 37, 8, 16                       # ragged last block of 5
    Q, K = r.standard_normal((n, d)) * 2, r.standard_normal((n, d)) * 2
    a = O.attention_scores_raw(Q, K, C, scale=0.5)
    np.testing.assert_allclose(a, _brute_attention(Q, K, C, 0.5), atol=1e-12)
    # every query distributes one unit of attention inside its block
    assert abs(a[:16].sum() - 16) < 1e-10 and abs(a[16:32].sum() - 16) < 1e-10 and abs(a[32:].sum() - 5) < 1e-10
    # blocks are independent: changing block 2's keys leaves block 1's scores alone
    K2 = K.copy(); K2[16:32] += 3.0
    assert np.array_equal(O.attention_scores_raw(Q, K2, C, 0.5)[:16], a[:16])
    # the order of the queries inside a block does not matter (column sums)
    p = np.arange(n); p[:16] = r.permutation(16)
    np.testing.assert_allclose(O.attention_scores_raw(Q[p], K, C, 0.5), a, atol=1e-12)
    # one block covering everything is plain non-causal attention: 1^T softmax(Q K^T)
    S = Q @ K.T * 0.5
    P = np.exp(S - S.max(axis=1, keepdims=True)); P /= P.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(O.attention_scores_raw(Q, K, 64, 0.5), P.sum(axis=0), atol=1e-12)
    # default scale is 1/sqrt(d)
    np.testing.assert_allclose(O.attention_scores_raw(Q, K, C), O.attention_scores_raw(Q, K, C, 1 / math.sqrt(d)), atol=0)


def test_attention_scores_closed_forms():
    # zero queries: uniform attention, every key of a full block gets rows/cols = 1
    K = _rng(81).standard_normal((8, 4))
    np.testing.assert_allclose(O.attention_scores_raw(np.zeros((8, 4)), K, 4), np.ones(8), atol=1e-15)
    # two tokens, logits [[0, ln 3], [0, 0]]: rows (1/4, 3/4) and (1/2, 1/2) -> sums (3/4, 5/4)
    Q = np.array([[1.0], [0.0]]); Kk = np.array([[0.0], [math.log(3.0)]])
    np.testing.assert_allclose(O.attention_scores_raw(Q, Kk, 2, scale=1.0), [0.75, 1.25], atol=1e-15)
    # a dominant key takes everything in its block
    Qb = np.ones((4, 1)); Kb = np.array([[0.0], [100.0], [0.0], [0.0]])
    np.testing.assert_allclose(O.attention_scores_raw(Qb, Kb, 4, scale=1.0), [0, 4, 0, 0], atol=1e-12)


def test_mean_pool_and_group_average():
    np.testing.assert_allclose(O.mean_pool(np.ones(6), 3), [2 / 3, 1, 1, 1, 1, 2 / 3], atol=1e-15)
    np.testing.assert_allclose(O.mean_pool(np.array([0, 0, 7.0, 0, 0, 0]), 7), [1, 1, 1, 1, 1, 1], atol=1e-15)
    x = _rng(82).standard_normal(20)
    assert np.array_equal(O.mean_pool(x, 1), x)
    assert abs(O.mean_pool(x, 5)[10] - x[8:13].mean()) < 1e-15
    # linear: pooling commutes with the average over a group's query heads
    r = _rng(83)
    K = r.standard_normal((40, 6)); Qs = [r.standard_normal((40, 6)) for _ in range(3)]
    a = O.attention_scores(Qs, K, chunk=16, pool=5)
    want = O.mean_pool(np.mean([O.attention_scores_raw(Q, K, 16) for Q in Qs], axis=0), 5)
    np.testing.assert_allclose(a, want, atol=1e-15)
    # a single query head and no pooling is the raw vector
    np.testing.assert_allclose(O.attention_scores([Qs[0]], K, 16, pool=1), O.attention_scores_raw(Qs[0], K, 16), atol=0)


# ---------------------------------------------------------------- head-adaptive selection (Sec. 3.3)
def _brute_layer(S, k_total):
    """Pure-Python reference: sort (score descending, head, token) tuples."""
    H, n = S.shape
    items = []
    for h in range(H):
        for i in range(n):
            v = float(np.float32(S[h, i]))
            nan = v != v
            items.append((nan, -(0.0 if nan else v), h, i))
    items.sort()
    out = [[] for _ in range(H)]
    for _, _, h, i in items[:k_total]:
        out[h].append(i)
    return [sorted(x) for x in out]


def test_select_topk_layer_brute_force_and_ties():
    rng = np.random.default_rng(11)
    for H, n, k in [(1, 7, 3), (3, 5, 1), (4, 9, 20), (2, 6, 12), (5, 8, 17)]:
        # few distinct values: many ties inside and across heads
        S = rng.integers(0, 4, size=(H, n)).astype(np.float64) / 3.0
        S[rng.random((H, n)) < 0.1] = np.nan
        S[rng.random((H, n)) < 0.05] = -np.inf
        got = O.select_topk_layer(S, k)
        want = _brute_layer(S, k)
        assert [g.tolist() for g in got] == want
        assert sum(len(g) for g in got) == k


def test_select_topk_layer_properties():
    rng = np.random.default_rng(12)
    H, n, k_total = 6, 200, 333
    S = rng.standard_normal((H, n)) * rng.uniform(0.2, 3.0, size=(H, 1))
    got = O.select_topk_layer(S, k_total)
    cnt = [len(g) for g in got]
    assert sum(cnt) == k_total
    S32 = S.astype(np.float32)
    kept = np.zeros((H, n), dtype=bool)
    for h in range(H):
        assert np.all(np.diff(got[h]) > 0)
        kept[h, got[h]] = True
        # restricted to one head, the shared budget is that head's own top-cnt[h]
        assert np.array_equal(got[h], O.select_topk(S[h], cnt[h])) or cnt[h] == 0
    # one threshold for the whole layer: nothing evicted beats anything kept
    assert S32[kept].min() >= S32[~kept].max()
    # one head alone is the per-head rule
    assert np.array_equal(O.select_topk_layer(S[:1], 50)[0], O.select_topk(S[0], 50))
    # a head whose scores all exceed every other head's takes its whole length first
    S2 = S.copy()
    S2[2] += 100.0
    got2 = O.select_topk_layer(S2, n + 10)
    assert len(got2[2]) == n and sum(len(g) for g in got2) == n + 10
    # equal scores everywhere: the budget fills heads in order, tokens in order
    got3 = O.select_topk_layer(np.ones((3, 4)), 6)
    assert [g.tolist() for g in got3] == [[0, 1, 2, 3], [0, 1], []]
    # permuting the heads permutes the answer when there are no ties
    perm = rng.permutation(H)
    gotp = O.select_topk_layer(S[perm], k_total)
    for j, h in enumerate(perm):
        assert np.array_equal(gotp[j], got[h])


# ---------------------------------------------------------------- paged compaction target
def test_paged_compaction_matches_dense_and_in_place_matches_snapshot():
    rng = np.random.default_rng(21)
    n, d, ps = 53, 4, 8
    rows = rng.integers(0, 1 << 16, size=(n, d)).astype(np.uint16)
    kept = np.sort(rng.choice(n, size=19, replace=False)).astype(np.int32)
    npages = 12
    table = rng.permutation(npages)[: (n + ps - 1) // ps].astype(np.int32)   # scattered pages
    pool0 = rng.integers(0, 1 << 16, size=(npages, ps, d)).astype(np.uint16)
    # out of place: reading the pages back in logical order gives the dense packed rows
    pool = pool0.copy()
    O.compact_rows_paged(pool, rows, kept, table)
    dense, _ = O.compact_rows(rows, rows, kept)
    logical = pool[table].reshape(-1, d)
    assert np.array_equal(logical[: len(kept)], dense)
    # nothing else in the pool changed
    touched = np.zeros((npages, ps), dtype=bool)
    for j in range(len(kept)):
        touched[table[j // ps], j % ps] = True
    assert np.array_equal(pool[~touched], pool0[~touched])
    # in place: same result as gathering from a snapshot of the pages
    pool = pool0.copy()
    for t in range(n):
        pool[table[t // ps], t % ps] = rows[t]
    snap = pool.copy()
    O.compact_pages_in_place(pool, kept, table)
    assert np.array_equal(pool[table].reshape(-1, d)[: len(kept)], dense)
    assert np.array_equal(pool[~touched], snap[~touched])
    # keeping everything moves nothing; keeping the tail moves it to the front
    pool = snap.copy()
    O.compact_pages_in_place(pool, np.arange(n, dtype=np.int32), table)
    assert np.array_equal(pool, snap)
    pool = snap.copy()
    O.compact_pages_in_place(pool, np.arange(n - 10, n, dtype=np.int32), table)
    assert np.array_equal(pool[table].reshape(-1, d)[:10], rows[n - 10:])


# ---------------------------------------------------------------- SRHT right-sketch (App. D)
def test_srht_sketch_structure_and_scores():
    rng = np.random.default_rng(41)
    d, ks = 128, 48
    H = O.hadamard(d)
    assert np.array_equal(H, H.T) and np.array_equal(H @ H, d * np.eye(d))
    # entry (i, j) is the parity of the common bits of i and j
    i, j = np.meshgrid(np.arange(d), np.arange(d), indexing="ij")
    par = np.zeros((d, d), dtype=np.int64)
    for b in range(7):
        par ^= ((i >> b) & (j >> b) & 1)
    assert np.array_equal(H, 1.0 - 2.0 * par)
    signs = rng.integers(0, 2, d)
    cols = rng.choice(d, ks, replace=False)
    Phi = O.srht_phi(d, ks, signs, cols)
    assert Phi.shape == (d, ks) and np.allclose(np.abs(Phi), math.sqrt(d / ks))
    # orthogonal columns of squared norm d^2/k: K Phi keeps squared row norms in expectation
    np.testing.assert_allclose(Phi.T @ Phi, (d * d / ks) * np.eye(ks), atol=1e-9)
    assert np.array_equal(np.sign(Phi[:, 0]), np.where(signs != 0, -1.0, 1.0) * H[cols[0]])
    # with all d columns the sketch is invertible: sketched scores are the exact ones
    K = rng.standard_normal((300, d))
    full = O.srht_phi(d, d, signs, rng.permutation(d))
    np.testing.assert_allclose(O.approx_leverage_alg1(K, full), O.leverage_svd(K), atol=1e-9)
    # and a k_s-column SRHT is an admissible sketch: scores in [0, 1], sum k_s, below the exact ones
    o = O.approx_leverage_alg1(K, Phi)
    assert o.min() >= -1e-12 and abs(o.sum() - ks) < 1e-8 and np.all(o <= O.leverage_svd(K) + 1e-9)
