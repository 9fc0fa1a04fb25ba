"""Seeded input generators: shapes, structure and determinism (CPU, small sizes),
and the oracle's invariants on those inputs."""
import numpy as np
import torch

from oracle import compactor_oracle as O
from paper_2507_08143_amd import workloads as W


def _head(req, l=0, h=0):
    return O.bf16_bits_to_f64(W.bf16_bits(req.k[l, h]))


def test_config1_shape_outliers_and_determinism():
    w = W.config1(n=512)
    w2 = W.config1(n=512)
    k = w.requests[0].k
    assert k.shape == (1, 1, 512, 128) and k.dtype == torch.bfloat16
    assert torch.equal(k, w2.requests[0].k)
    sd = _head(w.requests[0]).std(axis=0)
    assert np.sum(sd > 10) == 4                      # four channels x20
    assert O.keep_count(512, w.requests[0].ratio) == 256


def test_config2_low_rank_structure():
    w = W.config2(L=1, H=2, n=1024)
    K = _head(w.requests[0], 0, 1)
    sv = np.linalg.svd(K / np.where(K.std(axis=0) > 10, 20.0, 1.0), compute_uv=False)
    assert sv[31] / sv[40] > 5                        # rank-32 signal over 0.1 noise
    phi = W.make_phi().double().numpy()
    o = O.approx_leverage_ridge(K, phi)
    assert abs(o.sum() - 48) < 1e-6 and o.min() >= 0 and o.max() <= 1


def test_config3_heavy_tails():
    w = W.config3(L=1, H=1, n=2048)
    K = _head(w.requests[0])
    kurt = np.mean(K ** 4) / np.mean(K ** 2) ** 2
    assert kurt > 3.5                                 # heavier than Gaussian after rotation


def test_config4_ragged():
    w = W.config4(L=1, H=1, n_req=5, n_lo=100, n_hi=400)
    ns = [r.n for r in w.requests]
    assert len(set(ns)) > 1 and all(100 <= n <= 400 for n in ns)
    assert all(0.2 <= r.ratio <= 0.6 for r in w.requests)
    assert w.tokens == sum(ns)


def test_config5_duplicates_and_rank():
    w = W.config5(L=1, H=1, n=2000)
    bits = W.bf16_bits(w.requests[0].k[0, 0])
    uniq = np.unique(bits, axis=0).shape[0]
    assert 2000 - uniq >= 90                          # ~5 % rows are bit copies
    K = O.bf16_bits_to_f64(bits)
    sv = np.linalg.svd(K, compute_uv=False)
    assert sv[95] / sv[96] > 20                       # rank 96 up to bf16 rounding
    o = O.approx_leverage_ridge(K, W.make_phi().double().numpy())
    # bit-identical rows get bit-identical scores
    _, inv, cnt = np.unique(bits, axis=0, return_inverse=True, return_counts=True)
    g = np.flatnonzero(cnt > 1)[0]
    rows = np.flatnonzero(inv == g)
    assert len(set(o[rows].tolist())) == 1


def test_phi_is_fixed():
    p = W.make_phi()
    assert p.shape == (128, 48) and p.dtype == torch.float32
    assert torch.equal(p, W.make_phi())
    assert abs(float(p.var()) - 1 / 48) < 2e-3
