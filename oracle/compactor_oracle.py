"""Float64 CPU oracle for the Compactor hot path (score -> select -> compact).

TEST INFRASTRUCTURE ONLY.  This module is the independent checker for the HIP
library: it may be imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py, and by nothing on the product path.  It shares no
code with the HIP kernels or their Python binding and imports neither.

Everything is plain NumPy in float64, written so that each function can be
checked against the paper by eye.  No blocking, fusion or reordering beyond the
formula or the algorithm's own steps.

Notation (the paper overloads two symbols, so this file renames them):
  K        N x d key matrix of one head (rows = tokens)
  Phi      d x k_s Gaussian right-sketch, entries N(0, 1/k_s)     (Algorithm 1)
  k_s      sketch dimension (the paper's "target dimension k", 48 by default)
  k_keep   number of retained tokens, ceil(r * N)                 (Sec. 3 overview)
  lam      blend weight lambda of Eq. (scoring), 0.3 by default
  ridge_rel  relative ridge: rho = ridge_rel * trace(M) / order(M) added to the
           Gram matrix M that is factored (0 reproduces the paper exactly
           whenever M is nonsingular)

Parity status: every function below is pinned by tests/test_oracle_pins.py
against closed forms, invariants, library special cases or brute force, except
the *quality* of the k_s = 48 approximation relative to exact leverage scores,
which the paper itself says falls outside its theorem's bound: that quality is
"parity unpinned" (only the definition of the approximate score is pinned).
"""

from __future__ import annotations

import math

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "leverage_svd",
    "leverage_hat_diagonal",
    "leverage_ridge_exact",
    "approx_leverage_alg1",
    "approx_leverage_ridge",
    "approx_leverage_qr",
    "approx_leverage_eig",
    "hadamard",
    "srht_phi",
    "attention_scores_raw",
    "mean_pool",
    "attention_scores",
    "zscore",
    "blend_scores",
    "keep_count",
    "select_topk",
    "select_topk_layer",
    "compact_rows",
    "compact_rows_paged",
    "compact_pages_in_place",
    "compress_head",
    "calibration_curve",
    "calibrated_ratio",
]


# --------------------------------------------------------------------------
# input widening
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen raw bfloat16 bit patterns (uint16) exactly to float64.

    A bfloat16 is the upper half of an IEEE float32, so shifting the pattern
    into the high 16 bits of a uint32 and reinterpreting is exact.
    """
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    u = b.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# exact leverage scores  (Definition 1; Eq. "fast_svd")
# --------------------------------------------------------------------------
def leverage_svd(K: np.ndarray, rcond: float = 1e-12) -> np.ndarray:
    """Definition 1 as written: l_i = ||U_i||^2 with K = U Sigma V^T.

    Only the left singular vectors of the nonzero singular values belong to U
    (economy SVD truncated at rcond * sigma_max), which is what makes the
    scores sum to rank(K).
    """
    K = np.asarray(K, dtype=np.float64)
    U, sig, _ = np.linalg.svd(K, full_matrices=False)
    if sig.size == 0 or sig[0] == 0.0:
        return np.zeros(K.shape[0])
    keep = sig > rcond * sig[0]
    return np.sum(U[:, keep] ** 2, axis=1)


def leverage_hat_diagonal(K: np.ndarray) -> np.ndarray:
    """Brute force for small N: the diagonal of the hat matrix K (K^T K)^+ K^T.

    U U^T is the orthogonal projector onto range(K), and so is
    K (K^T K)^+ K^T, hence diag(U U^T) equals this diagonal (the outlier-score
    equation of Sec. 3.1, read as diag(U U^T): the printed U^T U is the
    identity and cannot be meant).
    """
    K = np.asarray(K, dtype=np.float64)
    H = K @ np.linalg.pinv(K.T @ K, rcond=1e-12, hermitian=True) @ K.T
    return np.diag(H).copy()


def leverage_ridge_exact(K: np.ndarray, ridge_rel: float = 0.0) -> np.ndarray:
    """o_i = k_i^T (K^T K + rho I)^{-1} k_i,  rho = ridge_rel * trace(K^T K) / d.

    With rho = 0 and K of full column rank this is Definition 1 through the
    Gram identity of Eq. "fast_svd": U = K V Sigma^{-1}, so
    ||U_i||^2 = k_i^T V Sigma^{-2} V^T k_i = k_i^T (K^T K)^{-1} k_i.
    """
    K = np.asarray(K, dtype=np.float64)
    d = K.shape[1]
    G = K.T @ K
    rho = float(ridge_rel) * np.trace(G) / d
    X = np.linalg.solve(G + rho * np.eye(d), K.T)  # d x N, column i = M^{-1} k_i
    return np.einsum("ij,ji->i", K, X)


# --------------------------------------------------------------------------
# approximate leverage scores  (Algorithm 1; Appendix C variants)
# --------------------------------------------------------------------------
def approx_leverage_alg1(K: np.ndarray, Phi: np.ndarray, rcond: float = 1e-12) -> np.ndarray:
    """Algorithm 1, step by step.

      K_hat = K Phi
      G     = K_hat^T K_hat
      svd(G) = V~ Sigma^2 V~^T              (SVD of a k_s x k_s matrix)
      U~    = K_hat V~ Sigma~^{-1}
      o     = diag(U~ U~^T)                 (row norms squared of U~)

    Sigma~^{-1} is undefined for zero singular values; those directions are
    dropped (pseudo-inverse, relative threshold rcond on Sigma^2), the reading
    that keeps U~ orthonormal.
    """
    K = np.asarray(K, dtype=np.float64)
    Phi = np.asarray(Phi, dtype=np.float64)
    K_hat = K @ Phi
    G = K_hat.T @ K_hat
    _, sig2, Vt = np.linalg.svd(G)
    if sig2.size == 0 or sig2[0] == 0.0:
        return np.zeros(K.shape[0])
    keep = sig2 > rcond * sig2[0]
    V = Vt.T[:, keep]
    U = (K_hat @ V) / np.sqrt(sig2[keep])
    return np.sum(U * U, axis=1)


def approx_leverage_ridge(K: np.ndarray, Phi: np.ndarray, ridge_rel: float = 0.0) -> np.ndarray:
    """Ridge form of Algorithm 1 (the form the HIP library evaluates):

      o_i = k^_i^T (K_hat^T K_hat + rho I)^{-1} k^_i,
      k^_i = Phi^T k_i,   rho = ridge_rel * trace(K_hat^T K_hat) / k_s.

    At rho = 0 with K_hat of full column rank, U~ = K_hat V~ Sigma~^{-1} gives
    ||U~_i||^2 = k^_i^T V~ Sigma^{-2} V~^T k^_i = k^_i^T G^{-1} k^_i, i.e. the
    same numbers as approx_leverage_alg1.
    """
    K = np.asarray(K, dtype=np.float64)
    Phi = np.asarray(Phi, dtype=np.float64)
    ks = Phi.shape[1]
    K_hat = K @ Phi
    G = K_hat.T @ K_hat
    rho = float(ridge_rel) * np.trace(G) / ks
    X = np.linalg.solve(G + rho * np.eye(ks), K_hat.T)
    return np.einsum("ij,ji->i", K_hat, X)


def approx_leverage_qr(K: np.ndarray, Phi: np.ndarray) -> np.ndarray:
    """Appendix C, QR route: K_hat = Q R (reduced), l~_i = ||Q_i||^2."""
    K_hat = np.asarray(K, dtype=np.float64) @ np.asarray(Phi, dtype=np.float64)
    Q, _ = np.linalg.qr(K_hat, mode="reduced")
    return np.sum(Q * Q, axis=1)


def approx_leverage_eig(K: np.ndarray, Phi: np.ndarray, eps: float = 1e-6) -> np.ndarray:
    """Appendix C, Gram eigendecomposition route with the eigenvalue clamp:

      G = V Lambda V^T,  lambda_j <- max(lambda_j, eps),
      U~ = K_hat V Lambda^{-1/2},  l~_i = ||U~_i||^2.
    """
    K_hat = np.asarray(K, dtype=np.float64) @ np.asarray(Phi, dtype=np.float64)
    G = K_hat.T @ K_hat
    lam, V = np.linalg.eigh(G)
    lam = np.maximum(lam, eps)
    U = (K_hat @ V) / np.sqrt(lam)
    return np.sum(U * U, axis=1)


def hadamard(d: int) -> np.ndarray:
    """Walsh-Hadamard matrix of order d (a power of two), entries +-1, by Sylvester's
    doubling H_2m = [[H_m, H_m], [H_m, -H_m]]."""
    assert d >= 1 and d & (d - 1) == 0
    H = np.ones((1, 1))
    while H.shape[0] < d:
        H = np.block([[H, H], [H, -H]])
    return H


def srht_phi(d: int, k_s: int, signs: np.ndarray, cols: np.ndarray) -> np.ndarray:
    """Subsampled randomized Hadamard right-sketch (App. D): sqrt(d/k) R H D with D the
    diagonal of Rademacher signs, H the +-1 Walsh-Hadamard matrix and R the choice of k_s
    of its d rows, transposed into the d x k_s matrix that multiplies keys from the right:
    Phi[i, j] = sqrt(d/k_s) * D_i * H[cols[j], i].

    signs: d entries, nonzero = -1.  cols: k_s distinct indices in [0, d).
    """
    D = np.where(np.asarray(signs) != 0, -1.0, 1.0)
    H = hadamard(d)
    return math.sqrt(d / k_s) * (H[np.asarray(cols)] * D[None, :]).T


# --------------------------------------------------------------------------
# attention-based scores  (Sec. 3.2, "Attention-Based Scoring")
# --------------------------------------------------------------------------
def attention_scores_raw(Q: np.ndarray, K: np.ndarray, chunk: int = 256,
                         scale: float | None = None) -> np.ndarray:
    """a = concat_i 1^T softmax(Q[i] K[i]^T): non-causal attention inside blocks of `chunk`
    consecutive positions, summed over the block's queries (column sums), for one query head.

    Q[i], K[i] are rows (i-1)C+1 .. iC; the last block is shorter when C does not divide N.
    The softmax normalises each query's row over the keys of its own block.  The paper's
    formula shows no logit scale; `scale` (default 1/sqrt(d), the model's own attention scale)
    multiplies Q K^T before the softmax.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n, d = K.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    a = np.zeros(n)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        S = (Q[lo:hi] @ K[lo:hi].T) * scale
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)
        a[lo:hi] = P.sum(axis=0)
    return a


def mean_pool(a: np.ndarray, width: int) -> np.ndarray:
    """Mean pooling along the sequence as SnapKV applies it: window `width` (odd), stride 1,
    zero padding of width//2 on both sides, every window divided by `width`."""
    a = np.asarray(a, dtype=np.float64)
    if width <= 1:
        return a.copy()
    h = width // 2
    padded = np.concatenate([np.zeros(h), a, np.zeros(h)])
    out = np.zeros_like(a)
    for u in range(width):
        out += padded[u:u + a.shape[0]]
    return out / width


def attention_scores(Q_heads, K: np.ndarray, chunk: int = 256, pool: int = 7,
                     scale: float | None = None) -> np.ndarray:
    """Attention score vector a of one kv-head: the raw block-wise column sums averaged over
    the query heads that share the kv-head (grouped-query attention), then mean-pooled.

    The paper leaves the reduction over a group's query heads and the pooling width open;
    mean over the group and an odd width (default 7), zero padding at both ends of the
    sequence and division by the full width are this build's readings.
    """
    raw = np.mean([attention_scores_raw(Q, K, chunk, scale) for Q in Q_heads], axis=0)
    return mean_pool(raw, pool)


# --------------------------------------------------------------------------
# blending  (Eq. "scoring")
# --------------------------------------------------------------------------
def zscore(v: np.ndarray) -> np.ndarray:
    """(v - mean(v)) / std(v) with the population standard deviation.

    A constant vector has std 0; its standardised form is taken to be all
    zeros (it then contributes nothing to the ranking).
    """
    v = np.asarray(v, dtype=np.float64)
    mu = v.mean()
    sd = math.sqrt(float(np.mean((v - mu) ** 2)))
    if sd == 0.0:
        return np.zeros_like(v)
    return (v - mu) / sd


def blend_scores(a: np.ndarray | None, o: np.ndarray, lam: float = 0.3) -> np.ndarray:
    """s = z(a) + lam * z(o)  (Eq. "scoring"); without attention scores s = o,
    the paper's "Compactor(o)" / "only o" variant."""
    if a is None:
        return np.asarray(o, dtype=np.float64).copy()
    return zscore(a) + float(lam) * zscore(o)


# --------------------------------------------------------------------------
# selection and compaction  (Sec. 3 overview; Sec. 3.3 "KV selection")
# --------------------------------------------------------------------------
def keep_count(n: int, ratio: float) -> int:
    """k_keep = ceil(r * N), clamped to [1, N].

    r is the float32 the C interface carries, widened to double.  A float32
    ratio is only known to a relative 2^-24, so a product that is an integer
    on paper (r = 0.001, N = 1000) can come out a hair above it; the product
    is therefore shrunk by the factor (1 - 2^-23) before the ceiling.
    """
    if n <= 0:
        return 0
    r = float(np.float32(ratio))
    k = int(math.ceil((r * n) * (1.0 - 2.0 ** -23)))
    return max(1, min(n, k))


def select_topk(s: np.ndarray, k_keep: int) -> np.ndarray:
    """Indices of the k_keep largest scores, ascending.

    Order: higher score first; equal scores by lower index first (the paper
    leaves ties open; this rule is deterministic and position-stable).
    Scores are compared as float32 values, the precision the library stores;
    -0.0 equals +0.0 and a NaN ranks below every number, -inf included.
    """
    s32 = np.asarray(s, dtype=np.float32)
    isnan = np.isnan(s32)
    val = np.where(isnan, 0.0, s32.astype(np.float64))
    n = val.shape[0]
    # lexsort: last key is the primary one
    order = np.lexsort((np.arange(n), -val, isnan))
    kept = np.sort(order[:k_keep])
    return kept.astype(np.int32)


def select_topk_layer(S: np.ndarray, k_total: int):
    """Head-adaptive selection (Sec. 3.3, "across all heads"): the k_total largest of
    the H*n scores of one layer's heads, wherever they fall.

    S is [H, n].  The pool is one layer (scoring stays per head; only the budget
    is shared, so a head with many high scores keeps more than ceil(r n) tokens and
    another fewer, possibly none).  Same order as select_topk: higher score first,
    equal scores by lower (head, token) position first, float32 comparison, NaN
    last.  Returns a list of H ascending int32 index arrays (ragged).
    """
    S32 = np.asarray(S, dtype=np.float32)
    H, n = S32.shape
    flat = S32.reshape(-1)
    isnan = np.isnan(flat)
    val = np.where(isnan, 0.0, flat.astype(np.float64))
    order = np.lexsort((np.arange(H * n), -val, isnan))
    taken = np.zeros(H * n, dtype=bool)
    taken[order[:k_total]] = True
    taken = taken.reshape(H, n)
    return [np.flatnonzero(taken[h]).astype(np.int32) for h in range(H)]


def compact_rows(K_cache: np.ndarray, V: np.ndarray, kept: np.ndarray):
    """Packed cache: the retained rows, in ascending token order (bit copies)."""
    return K_cache[kept].copy(), V[kept].copy()


def compact_rows_paged(pages: np.ndarray, rows: np.ndarray, kept: np.ndarray,
                       block_table: np.ndarray) -> None:
    """Retained rows of one head written into a paged cache (Sec. 3 overview: the
    compressed cache is the retained key/value pairs; here it lives in fixed-size
    pages named by a block table, as serving engines store it).

    pages [num_pages, page_size, d] is this head's view of the page pool and is
    modified in place: retained token j goes to page block_table[j // page_size],
    slot j % page_size.  Everything else in the pool is left as it was.
    """
    ps = pages.shape[1]
    for j, t in enumerate(kept):
        pages[block_table[j // ps], j % ps] = rows[t]


def compact_pages_in_place(pages: np.ndarray, kept: np.ndarray, block_table: np.ndarray) -> None:
    """The same when the head's n tokens already live in these pages (token t at page
    block_table[t // page_size], slot t % page_size): rows move towards the front one
    after the other, in ascending order, so that a row is read before its slot is
    reused (kept[j] >= j).  Afterwards the first ceil(len(kept) / page_size) logical
    pages hold the compressed head and the rest can be released.
    """
    ps = pages.shape[1]
    for j, t in enumerate(kept):
        pages[block_table[j // ps], j % ps] = pages[block_table[t // ps], t % ps]


def compress_head(
    K_score: np.ndarray,
    K_cache_bits: np.ndarray,
    V_bits: np.ndarray,
    ratio: float,
    Phi: np.ndarray | None,
    ridge_rel: float = 0.0,
    attn: np.ndarray | None = None,
    lam: float = 0.3,
):
    """One head end to end: scores -> top-ceil(rN) -> packed rows.

    Phi = None selects exact (ridge) leverage scores.
    Returns (scores float64, kept int32 ascending, K_packed, V_packed).
    """
    if Phi is None:
        o = leverage_ridge_exact(K_score, ridge_rel)
    else:
        o = approx_leverage_ridge(K_score, Phi, ridge_rel)
    s = blend_scores(attn, o, lam)
    kept = select_topk(s, keep_count(K_score.shape[0], ratio))
    Kp, Vp = compact_rows(K_cache_bits, V_bits, kept)
    return s, kept, Kp, Vp


# --------------------------------------------------------------------------
# context-calibrated retention  (Sec. 3.4)
# --------------------------------------------------------------------------
def calibration_curve(r, nll: float, alpha: float, beta: float):
    """f_{alpha,beta}(r, c) = (exp(r b - b) - exp(-b)) / (1 - exp(-b)),
    b = alpha * NLL(c) + beta.  f(0) = 0, f(1) = 1."""
    b = alpha * nll + beta
    r = np.asarray(r, dtype=np.float64)
    if b == 0.0:
        return r.copy()  # limit b -> 0
    return (np.exp(r * b - b) - math.exp(-b)) / (1.0 - math.exp(-b))


def calibrated_ratio(nll: float, alpha: float, beta: float, tau: float) -> float:
    """Smallest r in (0, 1] with f(r) >= tau.

    f is increasing in r, so the retention that just meets the quality budget
    is f^{-1}(tau) = 1 + ln(tau (1 - e^{-b}) + e^{-b}) / b   (the printed
    "arg max" cannot be meant: the maximiser of an increasing f is r = 1).
    """
    b = alpha * nll + beta
    if b == 0.0:
        r = tau
    else:
        r = 1.0 + math.log(tau * (1.0 - math.exp(-b)) + math.exp(-b)) / b
    return min(1.0, max(np.nextafter(0.0, 1.0), r))
