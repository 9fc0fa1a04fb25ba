"""Helpers for the GPU parity tests: run a workload through the C-ABI binding and
compare head by head with the float64 oracle."""
from __future__ import annotations

import numpy as np
import torch

from oracle import compactor_oracle as O
from paper_2507_08143_amd import workloads as W

# spec tolerance for scores: 1e-3 relative (fp32 accumulation); scores live in
# [0, 1] with mean k_s / n, so a tiny absolute floor covers scores at rounding level.
RTOL, ATOL = 1e-3, 1e-6


def binding():
    from paper_2507_08143_amd import compactor as C   # fails loudly if the library is missing
    return C


def make_call(C, w: W.Workload, device, group_bytes=0, phi=None):
    if phi is None and w.sketch_dim > 0:
        phi = W.make_phi(ks=w.sketch_dim, device=device)
    params = C.Params(w.layers, w.kv_heads, sketch_dim=w.sketch_dim, phi=phi,
                      ridge_rel=w.ridge_rel, lambda_blend=W.LAMBDA_BLEND, group_bytes=group_bytes)
    reqs = [C.Request(k_score=r.k, v_cache=r.v, ratio=r.ratio, attn=r.attn) for r in w.requests]
    return params, reqs


def oracle_head(w: W.Workload, b: int, l: int, h: int, phi_np):
    """Oracle on one head -> (scores f64, kept int32, K_packed bits, V_packed bits)."""
    r = w.requests[b]
    kb = W.bf16_bits(r.k[l, h])
    vb = W.bf16_bits(r.v[l, h])
    K = O.bf16_bits_to_f64(kb)
    attn = None if r.attn is None else r.attn[l, h].double().cpu().numpy()
    return O.compress_head(K, kb, vb, r.ratio, phi_np if w.sketch_dim > 0 else None,
                           w.ridge_rel, attn, W.LAMBDA_BLEND)


def check_scores(got: np.ndarray, want: np.ndarray, what=""):
    err = np.abs(got.astype(np.float64) - want)
    bound = RTOL * np.abs(want) + ATOL
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (
        "%s: score %d is %.9g, oracle %.9g (rel err %.3g)" %
        (what, worst, got[worst], want[worst], err[worst] / max(abs(want[worst]), 1e-30)))
    return float(np.max(err / np.maximum(np.abs(want), 1e-12)))


def blend_bound(o: np.ndarray, lam: float) -> np.ndarray:
    """How far the blended score s = z(a) + lam z(o) may move when every o_i moves by at most
    eps_i = RTOL o_i + ATOL (a is the same on both sides).  With mu, sd the mean and population
    standard deviation of o: the mean moves by at most mean(eps) <= RTOL mu + ATOL; sd is the
    root-mean-square of o - mu, so it moves by at most the root-mean-square of the perturbation,
    <= RTOL sqrt(sd^2 + mu^2) + ATOL; hence
      |dz_i| <= (eps_i + mean eps) / sd + |z_i| dsd / sd
             <= RTOL [ (o_i + mu) / sd + |z_i| sqrt(1 + (mu/sd)^2) ] + ATOL (2 + |z_i|) / sd,
    to first order.  1e-5 is added for the fp32 rounding of s itself (|s| stays below ~50)."""
    mu, sd = float(o.mean()), float(o.std())
    z = (o - mu) / sd
    return lam * (RTOL * ((o + mu) / sd + np.abs(z) * np.sqrt(1.0 + (mu / sd) ** 2)) +
                  ATOL * (2.0 + np.abs(z)) / sd) + 1e-5


def check_kept(got_kept: np.ndarray, want_kept: np.ndarray, want_scores: np.ndarray, what="",
               tol_scale=1.0, bound=None):
    """Kept sets must agree except for swaps among tokens whose oracle score lies within the
    score tolerance of the oracle's threshold score: |s_i - thr| <= tol_i + tol_thr, where tol is
    RTOL |s| + ATOL for leverage scores, or `bound` (per token) when given.  Returns the number of
    swapped tokens."""
    assert got_kept.dtype == np.int32 and len(got_kept) == len(want_kept), what
    assert np.all(np.diff(got_kept) > 0), what + ": kept indices not strictly ascending"
    if np.array_equal(got_kept, want_kept):
        return 0
    diff = np.setxor1d(got_kept, want_kept)
    ithr = want_kept[np.argmin(want_scores[want_kept])]
    thr = want_scores[ithr]
    gap = np.abs(want_scores[diff] - thr)
    if bound is None:
        allow = 2.0 * tol_scale * (RTOL * abs(thr) + ATOL)
    else:
        allow = tol_scale * (bound[diff] + bound[ithr])
    assert np.all(gap <= allow), (
        "%s: %d kept tokens differ, largest oracle score gap to the threshold %.3g > %.3g" %
        (what, len(diff), gap.max(), float(np.max(allow))))
    return len(diff)


def check_selection_valid(scores: np.ndarray, kept: np.ndarray, k: int, what=""):
    """Property check on the library's own scores: right count, ascending, and no evicted token
    outranks a kept one (ties by lower index)."""
    assert len(kept) == k and np.all(np.diff(kept) > 0), what
    mask = np.zeros(len(scores), bool)
    mask[kept] = True
    if k == len(scores):
        return
    s = scores.astype(np.float32) + np.float32(0)
    kept_min = s[mask].min()
    ev_max = s[~mask].max()
    assert kept_min >= ev_max, what
    if kept_min == ev_max:   # ties at the threshold: every kept tie precedes every evicted tie
        assert np.flatnonzero(mask & (s == kept_min)).max() < np.flatnonzero(~mask & (s == ev_max)).min(), what


def run_and_check(C, w: W.Workload, device, heads=None, group_bytes=0, kept_tol_scale=1.0, tune=None):
    """Fused compress on the whole workload; oracle on `heads` (list of (b,l,h)) or all.
    tune: launch-shape overrides (fields of Params such as gram_wgs) that must not change results
    beyond the tolerance."""
    params, reqs = make_call(C, w, device, group_bytes)
    for name, value in (tune or {}).items():
        setattr(params, name, value)
    out = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    so, ko, kk = C.compactor_layout(params, reqs)
    LH = w.layers * w.kv_heads
    scores = out["scores"].cpu().numpy()
    kept = out["kept_idx"].cpu().numpy()
    cnt = out["kept_cnt"].cpu().numpy()
    status = out["status"].cpu().numpy()
    phi_np = params.phi.double().cpu().numpy() if params.phi is not None else None
    if heads is None:
        heads = [(b, l, h) for b in range(len(reqs)) for l in range(w.layers) for h in range(w.kv_heads)]
    stats = {"max_rel": 0.0, "swaps": 0, "heads": len(heads)}
    for (b, l, h) in heads:
        n, k = w.requests[b].n, kk[b]
        g = l * w.kv_heads + h
        what = "%s req %d layer %d head %d (n=%d, k=%d)" % (w.name, b, l, h, n, k)
        assert status[b * LH + g] == 0, what + ": status %d" % status[b * LH + g]
        assert cnt[b * LH + g] == k == O.keep_count(n, w.requests[b].ratio), what
        s_gpu = scores[so[b] + g * n: so[b] + (g + 1) * n]
        i_gpu = kept[ko[b] + g * k: ko[b] + (g + 1) * k]
        s_ref, i_ref, kp_ref, vp_ref = oracle_head(w, b, l, h, phi_np)
        bound = None
        if w.requests[b].attn is None:
            stats["max_rel"] = max(stats["max_rel"], check_scores(s_gpu, s_ref, what))
        else:      # blended scores are z-scores: the error of o, carried through the blend
            K = O.bf16_bits_to_f64(W.bf16_bits(w.requests[b].k[l, h]))
            o = (O.approx_leverage_ridge(K, phi_np, w.ridge_rel) if w.sketch_dim > 0
                 else O.leverage_ridge_exact(K, w.ridge_rel))
            bound = blend_bound(o, W.LAMBDA_BLEND)
            err = np.abs(s_gpu.astype(np.float64) - s_ref)
            assert np.all(err <= bound), "%s: blended score off by %.3g (bound %.3g)" % (
                what, float(err.max()), float(bound[np.argmax(err - bound)]))
            stats["max_blend_err_over_bound"] = max(stats.get("max_blend_err_over_bound", 0.0),
                                                    float(np.max(err / bound)))
        stats["swaps"] += check_kept(i_gpu, i_ref, s_ref, what, kept_tol_scale, bound)
        check_selection_valid(s_gpu, i_gpu, k, what)
        rows = slice(ko[b] + g * k, ko[b] + (g + 1) * k)
        kp = out["k_packed"][rows].view(torch.int16).cpu().numpy().view(np.uint16)
        vp = out["v_packed"][rows].view(torch.int16).cpu().numpy().view(np.uint16)
        kb = W.bf16_bits(w.requests[b].k[l, h])
        vb = W.bf16_bits(w.requests[b].v[l, h])
        assert np.array_equal(kp, kb[i_gpu]) and np.array_equal(vp, vb[i_gpu]), what + ": packed rows"
        if np.array_equal(i_gpu, i_ref):
            assert np.array_equal(kp, kp_ref) and np.array_equal(vp, vp_ref), what
    return stats, out
