"""GPU parity: the HIP library (through its C-ABI binding) against the float64 oracle,
element by element, on seeded inputs that span several tiles and ragged tails."""
import math

import numpy as np
import pytest
import torch

from oracle import compactor_oracle as O
from paper_2507_08143_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def C():
    return U.binding()


def _say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ select (integer work: exact)
def _check_layer_selection(C, scores_b, kept, cnt, ko_b, k, b, L, H, n, what):
    """kept/cnt of request b against the oracle's head-adaptive selection of the same scores."""
    for l in range(L):
        want = O.select_topk_layer(scores_b[l * H * n:(l + 1) * H * n].reshape(H, n), H * k)
        pos = ko_b + l * H * k
        for h in range(H):
            c = int(cnt[(b * L + l) * H + h])
            assert c == len(want[h]), "%s: layer %d head %d keeps %d, oracle %d" % (what, l, h, c, len(want[h]))
            assert np.array_equal(kept[pos:pos + c], want[h]), "%s: layer %d head %d" % (what, l, h)
            pos += c


def _select_case(C, ns, ratios, L, H, maker, seed, scope=0):
    rng = np.random.default_rng(seed)
    params = C.Params(L, H, sketch_dim=48, select_scope=scope)
    reqs, host_scores = [], []
    for n, r in zip(ns, ratios):
        k = torch.empty(L, H, n, 128, dtype=torch.bfloat16, device=DEV)   # never read by select
        reqs.append(C.Request(k_score=k, v_cache=k, ratio=r))
        host_scores.append(maker(rng, L * H * n).astype(np.float32))
    flat = torch.from_numpy(np.concatenate(host_scores)).to(DEV)
    kept, cnt = C.compactor_select(params, reqs, flat)
    torch.cuda.synchronize()
    so, ko, kk = C.compactor_layout(params, reqs)
    kept, cnt = kept.cpu().numpy(), cnt.cpu().numpy()
    for b, n in enumerate(ns):
        assert kk[b] == O.keep_count(n, ratios[b])
        if scope == C.SCOPE_LAYER:
            _check_layer_selection(C, host_scores[b], kept, cnt, ko[b], kk[b], b, L, H, n,
                                   "layer select: req %d n=%d k=%d" % (b, n, kk[b]))
            continue
        for g in range(L * H):
            want = O.select_topk(host_scores[b][g * n:(g + 1) * n], kk[b])
            got = kept[ko[b] + g * kk[b]: ko[b] + (g + 1) * kk[b]]
            assert cnt[b * L * H + g] == kk[b]
            assert np.array_equal(got, want), "select mismatch: req %d head %d n=%d k=%d" % (b, g, n, kk[b])


def test_select_random_scores(C):
    _say("select: gaussian scores, ragged batch")
    _select_case(C, [1, 5, 63, 1023, 1024, 4097, 70001], [1.0, 0.5, 0.3, 0.2, 0.999, 0.6, 0.25],
                 2, 3, lambda r, m: r.standard_normal(m), 1)


def test_select_heavy_ties_signs_and_specials(C):
    _say("select: ties, zeros of both signs, NaN, infinities")

    def maker(r, m):
        s = r.integers(-4, 5, m).astype(np.float32) / 8.0
        s[r.integers(0, m, max(1, m // 50))] = np.nan
        s[r.integers(0, m, max(1, m // 60))] = -np.inf
        s[r.integers(0, m, max(1, m // 70))] = np.inf
        z = np.flatnonzero(s == 0)
        s[z[::2]] = -0.0
        return s
    _select_case(C, [7, 300, 4096, 9000, 33000], [0.5, 0.9, 0.1, 0.45, 0.32], 1, 2, maker, 2)


def test_select_all_equal_and_leverage_like(C):
    _say("select: all-equal scores; tiny positive leverage-like scores")
    _select_case(C, [5000, 131072], [0.37, 0.2], 1, 1, lambda r, m: np.full(m, 0.25), 3)
    _select_case(C, [100000], [0.32], 1, 2, lambda r, m: r.chisquare(48, m) / m, 4)


def test_select_across_the_heads_of_a_layer(C):
    _say("select, layer scope: gaussian scores with per-head spread, ragged batch")

    def spread(r, m):          # heads differ in scale, so their shares of the budget differ
        return r.standard_normal(m) * np.repeat(r.uniform(0.2, 3.0, 64), (m + 63) // 64)[:m]
    _select_case(C, [1, 5, 63, 1023, 1024, 4097, 70001], [1.0, 0.5, 0.3, 0.2, 0.999, 0.6, 0.25],
                 2, 3, spread, 5, scope=C.SCOPE_LAYER)
    _say("select, layer scope: ties, zeros of both signs, NaN, infinities; all equal")

    def maker(r, m):
        s = r.integers(-4, 5, m).astype(np.float32) / 8.0
        s[r.integers(0, m, max(1, m // 50))] = np.nan
        s[r.integers(0, m, max(1, m // 60))] = -np.inf
        s[r.integers(0, m, max(1, m // 70))] = np.inf
        z = np.flatnonzero(s == 0)
        s[z[::2]] = -0.0
        return s
    _select_case(C, [7, 300, 4096, 9000, 33000], [0.5, 0.9, 0.1, 0.45, 0.32], 2, 4, maker, 6,
                 scope=C.SCOPE_LAYER)
    _select_case(C, [5000, 40000], [0.37, 0.2], 1, 3, lambda r, m: np.full(m, 0.25), 7,
                 scope=C.SCOPE_LAYER)


def test_layer_scope_compress_end_to_end(C):
    _say("compress, layer scope: config 2 shape (L=2, H=4, n=3000) and a ragged batch")
    for w in (W.config2(DEV, L=2, H=4, n=3000), W.config4(DEV, L=1, H=3, n_req=3, n_lo=500, n_hi=2500)):
        params, reqs = U.make_call(C, w, DEV)
        params.select_scope = C.SCOPE_LAYER
        out = C.compactor_compress(params, reqs, want_scores=True)
        torch.cuda.synchronize()
        so, ko, kk = C.compactor_layout(params, reqs)
        L, H = w.layers, w.kv_heads
        scores = out["scores"].cpu().numpy()
        kept = out["kept_idx"].cpu().numpy()
        cnt = out["kept_cnt"].cpu().numpy()
        phi_np = params.phi.double().cpu().numpy()
        swaps = 0
        for b, r in enumerate(w.requests):
            n, k = r.n, kk[b]
            sb = scores[so[b]:so[b] + L * H * n]
            # exact: the library's selection is the oracle's selection of the library's scores
            _check_layer_selection(C, sb, kept, cnt, ko[b], k, b, L, H, n, "%s req %d" % (w.name, b))
            for l in range(L):
                ref = np.stack([U.oracle_head(w, b, l, h, phi_np)[0] for h in range(H)])
                for h in range(H):
                    U.check_scores(sb[(l * H + h) * n:(l * H + h + 1) * n], ref[h], "%s req %d l %d h %d" % (w.name, b, l, h))
                # against the oracle's own scores: differences only next to the layer's threshold
                want = O.select_topk_layer(ref, H * k)
                thr = min(ref[h][want[h]].min() for h in range(H) if len(want[h]))
                pos = ko[b] + l * H * k
                for h in range(H):
                    c = int(cnt[(b * L + l) * H + h])
                    got = kept[pos:pos + c]
                    diff = np.setxor1d(got, want[h])
                    swaps += len(diff)
                    assert np.all(np.abs(ref[h][diff] - thr) <= 2 * (U.RTOL * abs(thr) + U.ATOL))
                    rows = slice(pos, pos + c)
                    kp = out["k_packed"][rows].view(torch.int16).cpu().numpy().view(np.uint16)
                    vp = out["v_packed"][rows].view(torch.int16).cpu().numpy().view(np.uint16)
                    assert np.array_equal(kp, W.bf16_bits(r.k[l, h])[got])
                    assert np.array_equal(vp, W.bf16_bits(r.v[l, h])[got])
                    pos += c
        _say("  %s: tokens that differ from the oracle's selection (near-threshold): %d" % (w.name, swaps))
        # the three separate calls give the same bits as the fused call
        sc, st = C.compactor_score(params, reqs)
        ki, kc = C.compactor_select(params, reqs, sc)
        kp, vp = C.compactor_compact(params, reqs, ki, kc)
        torch.cuda.synchronize()
        assert torch.equal(ki, out["kept_idx"]) and torch.equal(kc, out["kept_cnt"])
        assert torch.equal(kp.view(torch.int16), out["k_packed"].view(torch.int16))
        assert torch.equal(vp.view(torch.int16), out["v_packed"].view(torch.int16))


# ------------------------------------------------------------------ compact (byte work: exact)
def test_compact_matches_oracle_with_strided_input(C):
    _say("compact: strided K/V views, oracle indices")
    L, H, n = 2, 3, 3000
    g = torch.Generator(device=DEV); g.manual_seed(5)
    big_k = torch.randn(L, H, n, 256, generator=g, device=DEV).to(torch.bfloat16)
    big_v = torch.randn(L, H, n, 256, generator=g, device=DEV).to(torch.bfloat16)
    k, v = big_k[..., :128], big_v[..., :128]        # row stride 256 elements
    params = C.Params(L, H)
    reqs = [C.Request(k_score=k, v_cache=v, ratio=0.4)]
    _, ko, kk = C.compactor_layout(params, reqs)
    rng = np.random.default_rng(6)
    idx = np.concatenate([np.sort(rng.choice(n, kk[0], replace=False)) for _ in range(L * H)]).astype(np.int32)
    cnt = torch.full((L * H,), kk[0], dtype=torch.int32, device=DEV)
    kp, vp = C.compactor_compact(params, reqs, torch.from_numpy(idx).to(DEV), cnt)
    torch.cuda.synchronize()
    for l in range(L):
        for h in range(H):
            gi = l * H + h
            sel = idx[gi * kk[0]:(gi + 1) * kk[0]]
            want_k, want_v = O.compact_rows(W.bf16_bits(k[l, h]), W.bf16_bits(v[l, h]), sel)
            rows = slice(gi * kk[0], (gi + 1) * kk[0])
            assert np.array_equal(W.bf16_bits(kp[rows]), want_k)
            assert np.array_equal(W.bf16_bits(vp[rows]), want_v)


# ------------------------------------------------------------------ scoring + fused path
def test_config1_full_sketched_and_exact(C):
    _say("config 1: single head n=4096, sketched then exact")
    w = W.config1(device=DEV)
    st, out = U.run_and_check(C, w, DEV)
    _say("  sketched: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    assert abs(float(out["scores"].double().sum()) - 48) < 1e-2       # sum = rank(K Phi)
    w.sketch_dim = 0
    st, out = U.run_and_check(C, w, DEV)
    _say("  exact:    max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    assert abs(float(out["scores"].double().sum()) - 128) < 2e-2      # sum = rank(K)


@pytest.mark.parametrize("n", [1, 17, 129, 777, 5000])
def test_ragged_token_counts(C, n):
    _say("gaussian+outlier keys, 2x2 heads, n=%d" % n)
    w = W.config1(device=DEV, L=2, H=2, n=n, ratio=0.37)
    params, reqs = U.make_call(C, w, DEV)
    if n < 48:      # K Phi cannot have rank 48: the head must be flagged, outputs still valid
        out = C.compactor_compress(params, reqs, want_scores=True)
        torch.cuda.synchronize()
        assert np.all(out["status"].cpu().numpy() & C.STATUS_PIVOT)
        s = out["scores"].cpu().numpy()
        assert np.all(np.isfinite(s))
        k = C.compactor_keep_count(n, 0.37)
        for g in range(4):
            U.check_selection_valid(s[g * n:(g + 1) * n], out["kept_idx"].cpu().numpy()[g * k:(g + 1) * k], k)
    else:
        st, _ = U.run_and_check(C, w, DEV)
        _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


@pytest.mark.parametrize("gram_wgs", [1, 2, 5, 12])
def test_gram_partitions_that_cross_heads(C, gram_wgs):
    """The Gram kernel deals 64-row tiles out evenly, across head boundaries.  One workgroup for
    six heads of 11 tiles crosses five boundaries (one partial parked in LDS, four written mid-run);
    5 workgroups of 14 tiles cross one or two; 12 cross none or one.  All must match the oracle."""
    _say("Gram partition with %d workgroup(s) over 6 heads of 700 tokens" % gram_wgs)
    w = W.config2(DEV, L=2, H=3, n=700)
    st, _ = U.run_and_check(C, w, DEV, tune={"gram_wgs": gram_wgs})
    _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


@pytest.mark.parametrize("score_tokens", [128, 1024, 8192, 32768])
def test_score_runs_of_several_bursts(C, score_tokens):
    """A score workgroup takes `score_tokens` tokens and writes its scores in bursts of 4096 (2048
    in exact mode): one partial burst, exactly one, two and a half, and a whole head of 11 bursts
    must all match the oracle; with attention scores the workgroup sums of the blend follow the
    same partition."""
    _say("score workgroups of %d tokens on heads of 10300 tokens, sketched, exact and blended" % score_tokens)
    w = W.config2(DEV, L=1, H=3, n=10300)
    st, _ = U.run_and_check(C, w, DEV, tune={"score_tokens": score_tokens})
    _say("  sketched: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    w.requests[0].attn = W.synthetic_attention_scores(1, 3, 10300, device=DEV, seed=score_tokens)
    st, _ = U.run_and_check(C, w, DEV, tune={"score_tokens": score_tokens})
    _say("  blended: score error at most %.3g of its bound, swaps %d" % (st["max_blend_err_over_bound"], st["swaps"]))
    w = W.config5(DEV, L=1, H=2, n=10300, exact=True)
    st, _ = U.run_and_check(C, w, DEV, tune={"score_tokens": score_tokens})
    _say("  exact ridge 1e-4: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_config2_small(C):
    _say("config 2 shape, 2 layers x 8 heads, n=6000")
    st, _ = U.run_and_check(C, W.config2(device=DEV, L=2, H=8, n=6000), DEV)
    _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_config3_small(C):
    _say("config 3 shape, 2 layers x 4 heads, n=9001")
    st, _ = U.run_and_check(C, W.config3(device=DEV, L=2, H=4, n=9001), DEV)
    _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_config4_small_ragged_batch(C):
    _say("config 4 shape: 6 requests, n in [300, 5000], 2x8 heads")
    w = W.config4(device=DEV, L=2, H=8, n_req=6, n_lo=300, n_hi=5000)
    st, _ = U.run_and_check(C, w, DEV)
    _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_config5_small_sketched_and_exact_ridge(C):
    _say("config 5 shape (rank 96 + duplicates), 1 layer x 8 heads, n=7000")
    w = W.config5(device=DEV, L=1, H=8, n=7000)
    st, out = U.run_and_check(C, w, DEV)
    _say("  sketched: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    # bit-identical rows must get bit-identical scores
    bits = W.bf16_bits(w.requests[0].k[0, 0])
    _, inv, cnt = np.unique(bits, axis=0, return_inverse=True, return_counts=True)
    s0 = out["scores"][:7000].cpu().numpy()
    for gidx in np.flatnonzero(cnt > 1)[:20]:
        assert len(set(s0[inv == gidx].tolist())) == 1
    w = W.config5(device=DEV, L=1, H=8, n=7000, exact=True)
    st, _ = U.run_and_check(C, w, DEV)
    _say("  exact ridge 1e-4: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_blend_with_attention_scores(C):
    _say("blend: s = z(a) + 0.3 z(o)")
    w = W.config2(device=DEV, L=1, H=4, n=4100)
    w.requests[0].attn = W.synthetic_attention_scores(1, 4, 4100, device=DEV)
    params, reqs = U.make_call(C, w, DEV)
    scores, status = C.compactor_score(params, reqs)
    torch.cuda.synchronize()
    assert not status.any()
    phi = params.phi.double().cpu().numpy()
    s = scores.cpu().numpy()
    for h in range(4):
        K = O.bf16_bits_to_f64(W.bf16_bits(w.requests[0].k[0, h]))
        a = w.requests[0].attn[0, h].double().cpu().numpy()
        o = O.approx_leverage_ridge(K, phi)
        want = O.blend_scores(a, o, W.LAMBDA_BLEND)
        assert np.all(np.abs(s[h * 4100:(h + 1) * 4100] - want) <= U.blend_bound(o, W.LAMBDA_BLEND))
    # and the fused path selects on the blended score: kept sets may differ from the oracle's only
    # between tokens whose blended scores are within the propagated score tolerance of the threshold
    st, _ = U.run_and_check(C, w, DEV)
    _say("  fused: blended score error at most %.3g of its bound, swaps %d" % (st["max_blend_err_over_bound"], st["swaps"]))


def test_blend_with_selection_by_several_workgroups(C):
    """Eq. "scoring" followed by the pooled selection paths: the blend rewrites the scores, so the
    score kernel's first histogram cannot be used and the selection tallies its own."""
    _say("blend + heads longer than one selection workgroup (n = 40000, 65537)")
    for n in (40000, 65537):
        w = W.config2(device=DEV, L=1, H=2, n=n)
        w.requests[0].attn = W.synthetic_attention_scores(1, 2, n, device=DEV, seed=n)
        st, out = U.run_and_check(C, w, DEV)
        _say("  n=%d: blended score error at most %.3g of its bound, swaps %d" % (n, st["max_blend_err_over_bound"], st["swaps"]))
        # exact on the library's own scores, ties included
        s = out["scores"].cpu().numpy()
        k = C.compactor_keep_count(n, w.requests[0].ratio)
        kept = out["kept_idx"].cpu().numpy()
        for h in range(2):
            assert np.array_equal(kept[h * k:(h + 1) * k], O.select_topk(s[h * n:(h + 1) * n], k))
    _say("blend + head-adaptive selection across the heads of a layer, ragged batch")
    w = W.config4(DEV, L=2, H=3, n_req=3, n_lo=500, n_hi=40000)
    for b, r in enumerate(w.requests):
        r.attn = W.synthetic_attention_scores(2, 3, r.n, device=DEV, seed=50 + b)
    params, reqs = U.make_call(C, w, DEV)
    params.select_scope = C.SCOPE_LAYER
    out = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    assert int(out["status"].max()) == 0
    so, ko, kk = C.compactor_layout(params, reqs)
    scores, kept, cnt = out["scores"].cpu().numpy(), out["kept_idx"].cpu().numpy(), out["kept_cnt"].cpu().numpy()
    phi_np = params.phi.double().cpu().numpy()
    for b, r in enumerate(w.requests):
        sb = scores[so[b]:so[b + 1]]
        _check_layer_selection(C, sb, kept, cnt, ko[b], kk[b], b, 2, 3, r.n, "blend, layer scope, req %d" % b)
        for g in range(6):          # the blended scores themselves, against the oracle
            l, h = divmod(g, 3)
            K = O.bf16_bits_to_f64(W.bf16_bits(r.k[l, h]))
            o = O.approx_leverage_ridge(K, phi_np)
            want = O.blend_scores(r.attn[l, h].double().cpu().numpy(), o, W.LAMBDA_BLEND)
            assert np.all(np.abs(sb[g * r.n:(g + 1) * r.n] - want) <= U.blend_bound(o, W.LAMBDA_BLEND))


def _same_up_to_rounding(C, w, params, reqs, ref, other, what):
    """A different launch partition changes the fp32 summation order of the Gram matrix, so
    scores may move in their last bits: they must agree to 1e-5 relative, and the selections
    may differ only between tokens whose scores are that close to the threshold."""
    so, ko, kk = C.compactor_layout(params, reqs)
    a, b = ref["scores"].double(), other["scores"].double()
    assert torch.all((a - b).abs() <= 1e-5 * a.abs() + 1e-9), what
    LH = w.layers * w.kv_heads
    sa, ia, ib = ref["scores"].cpu().numpy(), ref["kept_idx"].cpu().numpy(), other["kept_idx"].cpu().numpy()
    kp, vp = other["k_packed"].view(torch.int16).cpu().numpy(), other["v_packed"].view(torch.int16).cpu().numpy()
    for bq, r in enumerate(w.requests):
        for g in range(LH):
            n, k = r.n, kk[bq]
            s = sa[so[bq] + g * n: so[bq] + (g + 1) * n].astype(np.float64)
            rows = slice(ko[bq] + g * k, ko[bq] + (g + 1) * k)
            U.check_kept(ib[rows], ia[rows], s, what, tol_scale=0.01)
            l, h = divmod(g, w.kv_heads)
            assert np.array_equal(kp[rows].view(np.uint16), W.bf16_bits(r.k[l, h])[ib[rows]]), what
            assert np.array_equal(vp[rows].view(np.uint16), W.bf16_bits(r.v[l, h])[ib[rows]]), what


def test_separate_calls_equal_fused_call(C):
    _say("score + select + compact == compress, bit for bit; regrouping only moves last bits")
    w = W.config4(device=DEV, L=2, H=3, n_req=4, n_lo=500, n_hi=3000)
    params, reqs = U.make_call(C, w, DEV)
    fused = C.compactor_compress(params, reqs, want_scores=True)
    scores, status = C.compactor_score(params, reqs)
    kept, cnt = C.compactor_select(params, reqs, scores)
    kp, vp = C.compactor_compact(params, reqs, kept, cnt)
    nosc = C.compactor_compress(params, reqs, want_scores=False)
    torch.cuda.synchronize()
    assert torch.equal(fused["kept_idx"], nosc["kept_idx"])
    assert torch.equal(fused["k_packed"].view(torch.int16), nosc["k_packed"].view(torch.int16))
    assert torch.equal(fused["v_packed"].view(torch.int16), nosc["v_packed"].view(torch.int16))
    assert torch.equal(fused["scores"].view(torch.int32), scores.view(torch.int32))
    assert torch.equal(fused["kept_idx"], kept) and torch.equal(fused["kept_cnt"], cnt)
    assert torch.equal(fused["k_packed"].view(torch.int16), kp.view(torch.int16))
    assert torch.equal(fused["v_packed"].view(torch.int16), vp.view(torch.int16))
    # run-to-run determinism
    again = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(fused["scores"].view(torch.int32), again["scores"].view(torch.int32))
    assert torch.equal(fused["kept_idx"], again["kept_idx"])
    # head groups (one launch sequence per group)
    params_g, _ = U.make_call(C, w, DEV, group_bytes=2 * 1024 * 1024)
    grouped = C.compactor_compress(params_g, reqs, want_scores=True)
    grouped_nosc = C.compactor_compress(params_g, reqs, want_scores=False)
    torch.cuda.synchronize()
    _same_up_to_rounding(C, w, params, reqs, fused, grouped, "grouped")
    assert torch.equal(grouped["kept_idx"], grouped_nosc["kept_idx"])
    assert torch.equal(grouped["k_packed"].view(torch.int16), grouped_nosc["k_packed"].view(torch.int16))


def test_degenerate_inputs_are_flagged_not_fatal(C):
    _say("all-zero keys and a NaN key: status flags, finite-or-flagged outputs, valid selection")
    L, H, n = 1, 2, 600
    w = W.config1(device=DEV, L=L, H=H, n=n, ratio=0.5)
    w.requests[0].k[0, 0].zero_()                                  # head 0: K = 0
    w.requests[0].k[0, 1, 17, 5] = float("nan")                    # head 1: one NaN
    params, reqs = U.make_call(C, w, DEV)
    out = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    status = out["status"].cpu().numpy()
    assert status[0] & C.STATUS_PIVOT
    assert status[1] != 0
    s = out["scores"].cpu().numpy()
    assert np.all(s[:n] == 0)
    kept = out["kept_idx"].cpu().numpy()
    assert np.array_equal(kept[:300], np.arange(300))              # all tie: lowest indices win
    assert np.all(np.diff(kept[300:]) > 0)


def test_error_codes_reach_python(C):
    w = W.config1(device=DEV, L=1, H=1, n=64)
    params, reqs = U.make_call(C, w, DEV)
    with pytest.raises(C.CompactorError) as e:
        C.compactor_compress(params, reqs, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.code == C.EWORKSPACE


def test_a_pending_hip_error_of_the_caller_is_not_reported(C):
    """The elapsed time of two events that were never recorded is an error that stays pending on
    the thread; the next library call must neither fail because of it nor compute anything else."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    e0, e1, ms = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_float()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    w = W.config1(device=DEV, L=1, H=2, n=640)
    params, reqs = U.make_call(C, w, DEV)
    want = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) != 0      # leaves the error pending
    got = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    for k in ("scores", "kept_idx", "k_packed", "v_packed"):
        assert torch.equal(want[k], got[k])
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


# ------------------------------------------------------------------ full sizes (sampled heads)
def _sample_heads(w, per_request=4, seed=11):
    """Random heads of every request, plus the first head of the first request and the last head
    of the last one (lowest and highest addresses of the batch)."""
    rng = np.random.default_rng(seed)
    LH = w.layers * w.kv_heads
    heads = []
    for b in range(len(w.requests)):
        picks = rng.choice(LH, size=min(per_request, LH), replace=False)
        heads += [(b, int(g) // w.kv_heads, int(g) % w.kv_heads) for g in picks]
    for extra in ((0, 0, 0), (len(w.requests) - 1, w.layers - 1, w.kv_heads - 1)):
        if extra not in heads:
            heads.append(extra)
    return heads


def _release(*objs):
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def _structure_checks(C, w, out):
    """Properties that hold at any size, on every head (no oracle): status clear, scores in
    [0, 1] summing to k_s per head, selections valid on the library's own scores."""
    params, reqs = U.make_call(C, w, DEV)
    so, ko, kk = C.compactor_layout(params, reqs)
    assert int(out["status"].max()) == 0
    LH = w.layers * w.kv_heads
    for b, r in enumerate(w.requests):
        s = out["scores"][so[b]:so[b + 1]].view(LH, r.n)
        assert float(s.min()) >= 0.0 and float(s.max()) <= 1.0 + 1e-5
        if w.ridge_rel == 0.0 and w.sketch_dim > 0:
            assert torch.all((s.double().sum(dim=1) - w.sketch_dim).abs() < 2e-2)
        idx = out["kept_idx"][ko[b]:ko[b + 1]].view(LH, kk[b]).long()
        assert torch.all(idx[:, 1:] > idx[:, :-1])
        kept_min = torch.gather(s, 1, idx).min(dim=1).values
        mask = torch.ones_like(s, dtype=torch.bool).scatter_(1, idx, False)
        ev_max = torch.where(mask, s, torch.full_like(s, -1.0)).max(dim=1).values
        assert torch.all(kept_min >= ev_max)
        # packed rows are bit copies of the selected rows
        src_k = r.k.reshape(LH, r.n, 128).view(torch.int16)
        got_k = out["k_packed"][ko[b]:ko[b + 1]].view(LH, kk[b], 128).view(torch.int16)
        assert torch.equal(got_k, torch.gather(src_k, 1, idx.unsqueeze(-1).expand(-1, -1, 128)))
        src_v = r.v.reshape(LH, r.n, 128).view(torch.int16)
        got_v = out["v_packed"][ko[b]:ko[b + 1]].view(LH, kk[b], 128).view(torch.int16)
        assert torch.equal(got_v, torch.gather(src_v, 1, idx.unsqueeze(-1).expand(-1, -1, 128)))


def test_config2_full_size_as_benchmarked(C):
    _say("config 2 at full size (32 x 8 heads, n = 32768), the launch configuration bench.py times")
    w = W.config2(device=DEV)
    st, out = U.run_and_check(C, w, DEV, heads=_sample_heads(w, 6))
    _say("  FULL-SIZE config2 sketched: %d sampled heads, max rel err %.3g, swaps %d" % (st["heads"], st["max_rel"], st["swaps"]))
    _structure_checks(C, w, out)
    del w, out
    _release()


def test_config2_full_size_layer_scope(C):
    _say("config 2 at full size, head-adaptive selection across the 8 heads of each layer")
    w = W.config2(device=DEV)
    params, reqs = U.make_call(C, w, DEV)
    params.select_scope = C.SCOPE_LAYER
    out = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    so, ko, kk = C.compactor_layout(params, reqs)
    L, H, n, k = w.layers, w.kv_heads, w.requests[0].n, kk[0]
    assert int(out["status"].max()) == 0
    cnt = out["kept_cnt"].view(L, H)
    assert torch.all(cnt.sum(dim=1) == H * k) and int(cnt.min()) >= 0
    s = out["scores"].view(L, H * n)
    idx = out["kept_idx"].view(L, H * k).long()
    # flat position (head * n + token) of every retained token, from the ragged per-head counts
    off = torch.cumsum(cnt, dim=1) - cnt
    j = torch.arange(H * k, device=DEV).unsqueeze(0).expand(L, -1)
    head = (j.unsqueeze(-1) >= off.unsqueeze(1)).sum(dim=-1) - 1
    flat = head * n + idx
    assert torch.all(flat[:, 1:] > flat[:, :-1])            # heads in order, tokens ascending
    kept_min = torch.gather(s, 1, flat).min(dim=1).values
    mask = torch.ones_like(s, dtype=torch.bool).scatter_(1, flat, False)
    ev_max = torch.where(mask, s, torch.full_like(s, -1.0)).max(dim=1).values
    assert torch.all(kept_min >= ev_max)                    # one threshold per layer
    src_k = w.requests[0].k.reshape(L, H * n, 128).view(torch.int16)
    src_v = w.requests[0].v.reshape(L, H * n, 128).view(torch.int16)
    sel = flat.unsqueeze(-1).expand(-1, -1, 128)
    assert torch.equal(out["k_packed"].view(L, H * k, 128).view(torch.int16), torch.gather(src_k, 1, sel))
    assert torch.equal(out["v_packed"].view(L, H * k, 128).view(torch.int16), torch.gather(src_v, 1, sel))
    # two layers against the oracle's selection of the same scores: exact, ties included
    sc, ki, kc = out["scores"].cpu().numpy(), out["kept_idx"].cpu().numpy(), out["kept_cnt"].cpu().numpy()
    for l in (3, 29):
        want = O.select_topk_layer(sc[l * H * n:(l + 1) * H * n].reshape(H, n), H * k)
        pos = l * H * k
        for h in range(H):
            c = int(kc[l * H + h])
            assert c == len(want[h]) and np.array_equal(ki[pos:pos + c], want[h]), (l, h)
            pos += c
    _say("  per-head counts of layer 3: %s (uniform would be %d)" % (kc[3 * H:4 * H].tolist(), k))


def test_config3_full_size(C):
    _say("config 3 at full size (28 x 4 heads, n = 131072): 7.5 GB of keys and values")
    w = W.config3(device=DEV)
    st, out = U.run_and_check(C, w, DEV, heads=_sample_heads(w, 3))
    _say("  FULL-SIZE config3 sketched: %d sampled heads, max rel err %.3g, swaps %d" % (st["heads"], st["max_rel"], st["swaps"]))
    _structure_checks(C, w, out)
    del w, out
    _release()


def test_config5_full_size_sketched_and_exact(C):
    _say("config 5 at full size (64 x 8 heads, n = 100000): 26 GB of keys and values, row offsets past 2^31 elements")
    w = W.config5(device=DEV)
    assert w.requests[0].k.numel() > 2 ** 32
    st, out = U.run_and_check(C, w, DEV, heads=_sample_heads(w, 3))
    _say("  FULL-SIZE config5 sketched: %d sampled heads, max rel err %.3g, swaps %d" % (st["heads"], st["max_rel"], st["swaps"]))
    _structure_checks(C, w, out)
    del out
    _release()
    w.sketch_dim, w.ridge_rel = 0, 1e-4
    st, out = U.run_and_check(C, w, DEV, heads=_sample_heads(w, 2))
    _say("  FULL-SIZE config5 exact ridge 1e-4: %d sampled heads, max rel err %.3g, swaps %d" % (st["heads"], st["max_rel"], st["swaps"]))
    _structure_checks(C, w, out)
    del w, out
    _release()


def test_config4_full_size_ragged_batch(C):
    _say("config 4 at full size: 16 requests, n in [8192, 65536], 32 x 8 heads each, one fused call")
    w = W.config4(device=DEV)
    _say("  tokens %d, head-rows %d (%.1f GB of keys and values)" % (w.tokens, w.head_rows, w.head_rows * 512 / 1e9))
    st, out = U.run_and_check(C, w, DEV, heads=_sample_heads(w, 1))
    _say("  FULL-SIZE config4 sketched: %d sampled heads, max rel err %.3g, swaps %d" % (st["heads"], st["max_rel"], st["swaps"]))
    _structure_checks(C, w, out)
    del w, out
    _release()


# ------------------------------------------------------------------ attention scores (Sec. 3.2)
def _attention_case(C, L, H, G, n, keys, pool=7, seed=0):
    w = keys(device=DEV, L=L, H=H, n=n)
    k = w.requests[0].k
    q = W.synthetic_queries(L, H * G, n, device=DEV, seed=seed)
    ap = C.AttnParams(L, H, H * G, pool=pool)
    a = C.compactor_attention_scores(ap, [C.AttnRequest(q, k)])
    torch.cuda.synchronize()
    a = a.view(L, H, n).cpu().numpy()
    worst = 0.0
    for l in range(L):
        for h in range(H):
            K = O.bf16_bits_to_f64(W.bf16_bits(k[l, h]))
            Qs = [O.bf16_bits_to_f64(W.bf16_bits(q[l, h * G + j])) for j in range(G)]
            want = O.attention_scores(Qs, K, chunk=256, pool=pool)
            err = np.abs(a[l, h] - want)
            bound = 1e-3 * np.abs(want) + 1e-6
            assert np.all(err <= bound), "attention scores layer %d head %d: worst rel err %.3g" % (
                l, h, float(np.max(err / np.maximum(want, 1e-12))))
            worst = max(worst, float(np.max(err / np.maximum(want, 1e-12))))
    return worst, w, q, a


@pytest.mark.parametrize("n", [1, 100, 256, 700, 3000])
def test_attention_scores_match_oracle(C, n):
    _say("attention scores: 2 layers x 2 kv heads x 4 query heads, n=%d" % n)
    worst, _, _, a = _attention_case(C, 2, 2, 4, n, W.config1)
    _say("  max rel err %.3g" % worst)
    if n == 256:     # one full block, no pooling: every query hands out one unit of attention
        w2, _, _, raw = _attention_case(C, 1, 1, 2, 256, W.config1, pool=1)
        assert abs(raw.sum() - 256) < 1e-2


@pytest.mark.parametrize("G,n", [(1, 300), (2, 513), (8, 600)])
def test_attention_scores_group_sizes_strided_views_and_batches(C, G, n):
    _say("attention scores: %d query heads per kv head, strided q and k views, two requests (n=%d and 77)" % (G, n))
    L, H, pool = 1, 2, 7
    ap = C.AttnParams(L, H, H * G, pool=pool)
    reqs, want = [], []
    for b, nb in enumerate((n, 77)):
        # rows of 160 and 136 elements of which the first 128 are the head: token stride != d
        qbuf = torch.zeros(L, H * G, nb, 160, dtype=torch.bfloat16, device=DEV)
        kbuf = torch.zeros(L, H, nb, 136, dtype=torch.bfloat16, device=DEV)
        qbuf[..., :128] = W.synthetic_queries(L, H * G, nb, device=DEV, seed=3, request=b)
        kbuf[..., :128] = W.config1(device=DEV, L=L, H=H, n=nb).requests[0].k
        q, k = qbuf[..., :128], kbuf[..., :128]
        assert q.stride(2) == 160 and k.stride(2) == 136
        reqs.append(C.AttnRequest(q, k))
        for l in range(L):
            for h in range(H):
                K = O.bf16_bits_to_f64(W.bf16_bits(k[l, h]))
                Qs = [O.bf16_bits_to_f64(W.bf16_bits(q[l, h * G + j])) for j in range(G)]
                want.append(O.attention_scores(Qs, K, chunk=256, pool=pool))
    a = C.compactor_attention_scores(ap, reqs)
    torch.cuda.synchronize()
    a = a.cpu().numpy()
    want = np.concatenate(want)
    assert a.shape == want.shape
    err = np.abs(a - want)
    assert np.all(err <= 1e-3 * np.abs(want) + 1e-6), float(np.max(err / np.maximum(want, 1e-12)))
    _say("  max rel err %.3g" % float(np.max(err / np.maximum(want, 1e-12))))


def test_attention_scores_with_every_cu_busy(C):
    _say("attention scores: 2 layers x 8 kv heads x 4 query heads, n=16384 (1024 workgroups, two per CU)")
    worst, _, _, _ = _attention_case(C, 2, 8, 4, 16384, W.config2)
    _say("  max rel err %.3g" % worst)


def test_attention_scores_low_rank_keys_and_blend_end_to_end(C):
    _say("attention scores on config-2 keys, then the full blend: compress with a from the GPU")
    L, H, G, n = 1, 4, 4, 4100
    worst, w, q, a = _attention_case(C, L, H, G, n, W.config2)
    _say("  attention max rel err %.3g" % worst)
    w.requests[0].attn = torch.from_numpy(a).to(DEV).contiguous()
    st, _ = U.run_and_check(C, w, DEV)
    _say("  fused compress with blended scores: swaps %d" % st["swaps"])


def test_attention_error_codes(C):
    k = torch.zeros(1, 1, 64, 128, dtype=torch.bfloat16, device=DEV)
    q = torch.zeros(1, 3, 64, 128, dtype=torch.bfloat16, device=DEV)
    k2 = torch.zeros(1, 2, 64, 128, dtype=torch.bfloat16, device=DEV)
    for bad, kk in ((C.AttnParams(1, 2, 3), k2), (C.AttnParams(1, 1, 3, pool=4), k)):
        with pytest.raises(C.CompactorError) as e:       # 3 query heads over 2 kv heads; even window
            C.compactor_attention_scores(bad, [C.AttnRequest(q, kk)])
        assert e.value.code == C.EINVAL
    with pytest.raises(ValueError):                      # tensors that contradict the parameters
        C.compactor_attention_scores(C.AttnParams(1, 2, 4), [C.AttnRequest(q, k)])
    with pytest.raises(C.CompactorError) as e:
        C.compactor_attention_scores(C.AttnParams(1, 1, 3, chunk=128), [C.AttnRequest(q, k)])
    assert e.value.code == C.EUNSUPPORTED


# ------------------------------------------------------------------ paged compaction target
def _paged_case(C, w, scope, page_size, in_place, seed):
    """Selection by the library, then compaction into pages (or inside them) against the oracle
    replaying the same kept lists: byte work, compared over the whole pool."""
    rng = np.random.default_rng(seed)
    params, reqs = U.make_call(C, w, DEV)
    params.select_scope = scope
    out = C.compactor_compress(params, reqs, want_scores=False)
    torch.cuda.synchronize()
    so, ko, kk = C.compactor_layout(params, reqs)
    L, H = w.layers, w.kv_heads
    need = [(r.n + page_size - 1) // page_size for r in w.requests]     # enough for either mode
    num_pages = sum(need) + 5
    perm = rng.permutation(num_pages).astype(np.int32)                  # scattered, disjoint
    tables_np, at = [], 0
    for m in need:
        tables_np.append(perm[at:at + m].copy())
        at += m
    tables = [torch.from_numpy(t).to(DEV) for t in tables_np]
    # storage order [page, slot, layer, head, d], seen as [page, layer, slot, head, d]
    shape = (num_pages, page_size, L, H, 128)
    kpool = torch.randint(-30000, 30000, shape, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    vpool = torch.randint(-30000, 30000, shape, dtype=torch.int16, device=DEV).view(torch.bfloat16)
    kview, vview = kpool.permute(0, 2, 1, 3, 4), vpool.permute(0, 2, 1, 3, 4)
    if in_place:      # the cache already lives in the pages: token t at logical slot t
        for b, r in enumerate(w.requests):
            t = torch.arange(r.n, device=DEV)
            pg, sl = tables[b].long()[t // page_size], t % page_size
            kview[pg, :, sl] = r.k.permute(2, 0, 1, 3)
            vview[pg, :, sl] = r.v.permute(2, 0, 1, 3)
    k_ref = kview.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()
    v_ref = vview.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()
    C.compactor_compact_paged(params, reqs, out["kept_idx"], out["kept_cnt"], kview, vview, tables,
                              in_place=in_place)
    torch.cuda.synchronize()
    kept, cnt = out["kept_idx"].cpu().numpy(), out["kept_cnt"].cpu().numpy()
    for b, r in enumerate(w.requests):
        k = kk[b]
        for l in range(L):
            pos = ko[b] + l * H * k
            for h in range(H):
                c = int(cnt[(b * L + l) * H + h])
                assert scope == C.SCOPE_LAYER or c == k
                mine = kept[pos:pos + c]
                pos += c
                for ref, src in ((k_ref, r.k), (v_ref, r.v)):
                    if in_place:
                        O.compact_pages_in_place(ref[:, l, :, h, :], mine, tables_np[b])
                    else:
                        O.compact_rows_paged(ref[:, l, :, h, :], W.bf16_bits(src[l, h]), mine, tables_np[b])
    got_k = kview.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    got_v = vview.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got_k, k_ref), "paged K differs (scope %d, in_place %s)" % (scope, in_place)
    assert np.array_equal(got_v, v_ref), "paged V differs (scope %d, in_place %s)" % (scope, in_place)


@pytest.mark.parametrize("in_place", [False, True])
def test_compact_into_pages(C, in_place):
    _say("paged target, in_place=%s: head scope and layer scope, ragged batch, page sizes 16 and 7" % in_place)
    _paged_case(C, W.config2(DEV, L=2, H=3, n=1000), C.SCOPE_HEAD, 16, in_place, 31)
    _paged_case(C, W.config4(DEV, L=2, H=2, n_req=3, n_lo=100, n_hi=700), C.SCOPE_HEAD, 7, in_place, 32)
    _paged_case(C, W.config2(DEV, L=1, H=4, n=777), C.SCOPE_LAYER, 16, in_place, 33)
    _paged_case(C, W.config1(DEV, L=1, H=1, n=5000, ratio=1.0), C.SCOPE_HEAD, 256, in_place, 34)


def test_compact_into_pages_error_codes(C):
    w = W.config2(DEV, L=1, H=2, n=300)
    params, reqs = U.make_call(C, w, DEV)
    out = C.compactor_compress(params, reqs)
    pool = torch.zeros(8, 1, 16, 2, 128, dtype=torch.bfloat16, device=DEV)
    short = [torch.arange(2, dtype=torch.int32, device=DEV)]      # 90 rows need 6 pages of 16
    with pytest.raises(C.CompactorError) as e:
        C.compactor_compact_paged(params, reqs, out["kept_idx"], out["kept_cnt"], pool, pool.clone(), short)
    assert e.value.code == C.EINVAL
    # a table naming a page outside the pool is skipped, not followed
    bad = [torch.tensor([0, 1, 99, 3, 4, 5], dtype=torch.int32, device=DEV)]
    vp = pool.clone()
    C.compactor_compact_paged(params, reqs, out["kept_idx"], out["kept_cnt"], pool, vp, bad)
    torch.cuda.synchronize()
    assert float(pool[2].abs().sum()) == 0.0 and float(pool[0].abs().sum()) > 0.0


# ------------------------------------------------------------------ sketch variants (App. C, D)
def test_srht_sketch_and_other_sketch_dims(C):
    rng = np.random.default_rng(51)
    w = W.config2(DEV, L=1, H=2, n=2000)
    for ks in (16, 32, 48, 64):
        _say("SRHT right-sketch, k_s = %d" % ks)
        signs = rng.integers(0, 2, 128)
        cols = rng.choice(128, ks, replace=False)
        phi = C.compactor_srht_phi(ks, signs, cols, DEV)
        torch.cuda.synchronize()
        want = O.srht_phi(128, ks, signs, cols)
        got = phi.cpu().numpy().astype(np.float64)
        assert np.array_equal(np.sign(got), np.sign(want))              # every sign exact
        np.testing.assert_allclose(np.abs(got), math.sqrt(128 / ks), rtol=2e-7)
        w.sketch_dim = ks
        params, reqs = U.make_call(C, w, DEV, phi=phi)
        out = C.compactor_compress(params, reqs, want_scores=True)
        torch.cuda.synchronize()
        assert int(out["status"].max()) == 0
        sc = out["scores"].cpu().numpy()
        n = w.requests[0].n
        for h in range(2):
            K = O.bf16_bits_to_f64(W.bf16_bits(w.requests[0].k[0, h]))
            ref = O.approx_leverage_ridge(K, want)      # the oracle's own Phi: scale is immaterial
            U.check_scores(sc[h * n:(h + 1) * n], ref, "SRHT k_s=%d head %d" % (ks, h))
    with pytest.raises(C.CompactorError):
        C.compactor_srht_phi(48, np.zeros(128), np.zeros(48, dtype=int), DEV)      # repeated rows
    for ks in (16, 32, 64):
        _say("Gaussian right-sketch, k_s = %d" % ks)
        w2 = W.config3(DEV, L=1, H=2, n=1500)
        w2.sketch_dim = ks
        st, _ = U.run_and_check(C, w2, DEV)
        _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))


def test_scores_agree_with_the_qr_and_eigen_routes(C):
    _say("library scores against the oracle's QR and eigendecomposition routes (App. C)")
    w = W.config1(DEV, n=3000)
    params, reqs = U.make_call(C, w, DEV)
    sc, st = C.compactor_score(params, reqs)
    torch.cuda.synchronize()
    K = O.bf16_bits_to_f64(W.bf16_bits(w.requests[0].k[0, 0]))
    Phi = params.phi.double().cpu().numpy()
    got = sc.cpu().numpy()
    U.check_scores(got, O.approx_leverage_qr(K, Phi), "QR route")
    U.check_scores(got, O.approx_leverage_eig(K, Phi, eps=1e-6), "eigen route, clamp 1e-6")
    U.check_scores(got, O.approx_leverage_alg1(K, Phi), "Algorithm 1 (SVD of the sketched Gram matrix)")


# ------------------------------------------------------------------ graph capture
def test_compress_replays_from_a_hip_graph(C):
    """The fused call only launches kernels on the caller's stream (its scratch is cleared by
    kernels), so it can be captured once and replayed: every replay must give what the eager
    call gives on the inputs of that moment."""
    _say("compress captured in a HIP graph, replayed on changing inputs")
    w = W.config2(DEV, L=2, H=4, n=5000)
    params, reqs = U.make_call(C, w, DEV)
    so, ko, kk = C.compactor_layout(params, reqs)
    nh = w.layers * w.kv_heads
    ws = torch.empty(max(256, C.compactor_workspace_size(params, reqs)), dtype=torch.uint8, device=DEV)

    def buffers():
        return dict(kept_idx=torch.empty(ko[-1], dtype=torch.int32, device=DEV),
                    kept_cnt=torch.empty(nh, dtype=torch.int32, device=DEV),
                    k_packed=torch.empty(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                    v_packed=torch.empty(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                    status=torch.empty(nh, dtype=torch.int32, device=DEV),
                    scores=torch.empty(so[-1], dtype=torch.float32, device=DEV))
    gb, eb = buffers(), buffers()
    C.compactor_compress(params, reqs, want_scores=True, workspace=ws, **gb)     # warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        C.compactor_compress(params, reqs, want_scores=True, workspace=ws, **gb)
    for rep in range(3):
        # new keys and values in the same tensors, some eager work and a sync between replays
        fresh = W.config2(DEV, seed=100 + rep, L=2, H=4, n=5000).requests[0]
        w.requests[0].k.copy_(fresh.k)
        w.requests[0].v.copy_(fresh.v)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        C.compactor_compress(params, reqs, want_scores=True, workspace=ws, **eb)
        torch.cuda.synchronize()
        for name in ("scores", "kept_idx", "kept_cnt", "status"):
            assert torch.equal(gb[name], eb[name]), "replay %d: %s differs from the eager call" % (rep, name)
        assert torch.equal(gb["k_packed"].view(torch.int16), eb["k_packed"].view(torch.int16))
        assert torch.equal(gb["v_packed"].view(torch.int16), eb["v_packed"].view(torch.int16))


def test_pooled_and_blended_compress_replays_from_a_hip_graph_on_a_side_stream(C):
    """The same for the kernels of the pooled selection and of the blend (heads longer than one
    selection workgroup's reach, attention scores given), captured on a stream that is not the
    current one: they clear their scratch themselves too."""
    _say("pooled selection + blend captured in a HIP graph on a side stream")
    w = W.config2(DEV, L=1, H=3, n=40000)
    w.requests[0].attn = W.synthetic_attention_scores(1, 3, 40000, device=DEV, seed=9)
    params, reqs = U.make_call(C, w, DEV)
    so, ko, kk = C.compactor_layout(params, reqs)
    ws = torch.empty(max(256, C.compactor_workspace_size(params, reqs)), dtype=torch.uint8, device=DEV)

    def buffers():
        return dict(kept_idx=torch.empty(ko[-1], dtype=torch.int32, device=DEV),
                    kept_cnt=torch.empty(3, dtype=torch.int32, device=DEV),
                    k_packed=torch.empty(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                    v_packed=torch.empty(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                    status=torch.empty(3, dtype=torch.int32, device=DEV),
                    scores=torch.empty(so[-1], dtype=torch.float32, device=DEV))
    gb, eb = buffers(), buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        C.compactor_compress(params, reqs, want_scores=True, workspace=ws, stream=side, **gb)   # warm-up, eager
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        C.compactor_compress(params, reqs, want_scores=True, workspace=ws, stream=side, **gb)
    for rep in range(3):
        fresh = W.config2(DEV, seed=200 + rep, L=1, H=3, n=40000).requests[0]
        w.requests[0].k.copy_(fresh.k)
        w.requests[0].v.copy_(fresh.v)
        w.requests[0].attn.copy_(W.synthetic_attention_scores(1, 3, 40000, device=DEV, seed=300 + rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        C.compactor_compress(params, reqs, want_scores=True, workspace=ws, **eb)
        torch.cuda.synchronize()
        for name in ("scores", "kept_idx", "kept_cnt", "status"):
            assert torch.equal(gb[name], eb[name]), "replay %d: %s differs from the eager call" % (rep, name)
        assert torch.equal(gb["k_packed"].view(torch.int16), eb["k_packed"].view(torch.int16))
        assert torch.equal(gb["v_packed"].view(torch.int16), eb["v_packed"].view(torch.int16))
    # and the eager result is the oracle's
    st, _ = U.run_and_check(C, w, DEV)
    _say("  blended score error at most %.3g of its bound, swaps %d" % (st["max_blend_err_over_bound"], st["swaps"]))


def test_pooled_select_edges_and_regrouping(C):
    _say("pooled selection: k = 1, k = n, n just past one workgroup's reach; layer scope in small head groups")
    mk = lambda r, m: r.standard_normal(m)
    _select_case(C, [32769, 40000, 65537], [1.0 / 32769, 1.0, 0.5], 1, 2, mk, 8)
    _select_case(C, [32769, 40000], [1.0 / 32769, 1.0], 1, 2, mk, 9, scope=C.SCOPE_LAYER)
    _select_case(C, [3, 2], [1.0 / 3, 1.0], 2, 2, mk, 10, scope=C.SCOPE_LAYER)
    # fused call cut into groups of one layer each: every group's selection is still the
    # oracle's selection of that run's scores
    w = W.config2(DEV, L=3, H=4, n=2000)
    params, reqs = U.make_call(C, w, DEV, group_bytes=4 * 2000 * 256)
    params.select_scope = C.SCOPE_LAYER
    out = C.compactor_compress(params, reqs, want_scores=True)
    torch.cuda.synchronize()
    so, ko, kk = C.compactor_layout(params, reqs)
    _check_layer_selection(C, out["scores"].cpu().numpy(), out["kept_idx"].cpu().numpy(),
                           out["kept_cnt"].cpu().numpy(), ko[0], kk[0], 0, 3, 4, 2000,
                           "grouped layer scope")
    assert int(out["status"].max()) == 0


def test_sketched_scores_with_a_ridge(C):
    _say("sketched mode with ridge_rel > 0: scores against the oracle and the closed-form sum")
    for ks, ridge in ((48, 1e-3), (64, 0.05), (16, 1e-6)):
        w = W.config5(DEV, L=1, H=2, n=2500)
        w.sketch_dim, w.ridge_rel = ks, ridge
        st, out = U.run_and_check(C, w, DEV)
        # sum of ridge leverage scores = sum_j mu_j / (mu_j + rho), mu = eigenvalues of the factored Gram
        phi = W.make_phi(ks=ks).double().numpy()
        n = w.requests[0].n
        for h in range(2):
            K = O.bf16_bits_to_f64(W.bf16_bits(w.requests[0].k[0, h]))
            mu = np.linalg.eigvalsh((K @ phi).T @ (K @ phi))
            rho = float(np.float32(ridge)) * mu.sum() / ks
            want = float(np.sum(mu / (mu + rho)))
            got = float(out["scores"][h * n:(h + 1) * n].double().sum())
            assert abs(got - want) <= 1e-3 * want, (ks, ridge, h, got, want)
        _say("  k_s=%d ridge=%g: max rel err %.3g, swaps %d" % (ks, ridge, st["max_rel"], st["swaps"]))


def test_fused_path_on_strided_views(C):
    """K and V as views into larger buffers: token stride 384 elements, layer and head strides
    swapped (the cache stored [H, L, n, 3d])."""
    _say("fused compress on strided K/V views (stride_t = 384, [H, L] storage order)")
    L, H, n = 2, 3, 1500
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    base = W.config2(DEV, L=L, H=H, n=n)
    big_k = torch.randn(H, L, n, 384, generator=g, device=DEV).to(torch.bfloat16)
    big_v = torch.randn(H, L, n, 384, generator=g, device=DEV).to(torch.bfloat16)
    big_k[..., 128:256] = base.requests[0].k.permute(1, 0, 2, 3)
    big_v[..., 256:384] = base.requests[0].v.permute(1, 0, 2, 3)
    k = big_k[..., 128:256].permute(1, 0, 2, 3)        # [L, H, n, 128] view, nothing contiguous
    v = big_v[..., 256:384].permute(1, 0, 2, 3)
    assert k.stride() == (n * 384, L * n * 384, 384, 1)
    w = W.Workload("strided_views", L, H, [W.Request(k, v, 0.37)])
    st, out = U.run_and_check(C, w, DEV)
    _say("  max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    # the same bits as the contiguous tensors give
    w2 = W.Workload("contiguous", L, H, [W.Request(k.contiguous(), v.contiguous(), 0.37)])
    p2, r2 = U.make_call(C, w2, DEV)
    ref = C.compactor_compress(p2, r2, want_scores=True)
    torch.cuda.synchronize()
    for name in ("scores", "kept_idx"):
        assert torch.equal(out[name], ref[name]), name
    assert torch.equal(out["k_packed"].view(torch.int16), ref["k_packed"].view(torch.int16))
    assert torch.equal(out["v_packed"].view(torch.int16), ref["v_packed"].view(torch.int16))
