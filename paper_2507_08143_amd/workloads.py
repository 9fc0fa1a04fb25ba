"""Seeded synthetic KV-cache workloads shaped like the paper's models.

This module only *draws inputs*: it holds none of the method's arithmetic and
is the one module that both the HIP-path tests and the CPU oracle tests use, so
that both sides see the same bit patterns.  The paper evaluates on real
Llama-3.1 / Qwen-2.5 KV caches (Sec. 4); neither weights nor datasets exist
here, so these tensors stand in for them: same shapes and dtype (bf16,
head_dim 128), and the structure real keys are known for (a few massive
outlier channels, low effective rank, heavy tails, duplicated rows).

All values are drawn in fp32 on the requested device from a seeded
torch.Generator and rounded to bf16 (round-to-nearest-even).  The CPU and GPU
generators produce different streams for the same seed; a test draws once and
hands the same bits to both implementations.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch

HEAD_DIM = 128
SKETCH_DIM = 48          # k_s, Sec. 4 "sketching dimension k = 48"
LAMBDA_BLEND = 0.3       # Sec. 4
PHI_SEED = 12345


@dataclass
class Request:
    """One context: keys/values of every (layer, kv-head) and its retention."""
    k: torch.Tensor                  # bf16 [L, H, n, d]
    v: torch.Tensor                  # bf16 [L, H, n, d]
    ratio: float
    attn: Optional[torch.Tensor] = None   # fp32 [L, H, n] or None

    @property
    def n(self) -> int:
        return self.k.shape[2]


@dataclass
class Workload:
    name: str
    layers: int
    kv_heads: int
    requests: List[Request] = field(default_factory=list)
    sketch_dim: int = SKETCH_DIM     # 0 = exact leverage scores
    ridge_rel: float = 0.0

    @property
    def tokens(self) -> int:
        return sum(r.n for r in self.requests)

    @property
    def head_rows(self) -> int:
        return self.tokens * self.layers * self.kv_heads


def _gen(device, seed: int, config: int, request: int = 0) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + 1009 * config + request)
    return g


def make_phi(d: int = HEAD_DIM, ks: int = SKETCH_DIM, seed: int = PHI_SEED,
             device="cpu") -> torch.Tensor:
    """Gaussian right-sketch, entries N(0, 1/k_s) (variance 1/k_s), fp32 [d, k_s].
    Drawn on the CPU so that it is the same on every device."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    phi = torch.randn(d, ks, generator=g, dtype=torch.float32) / math.sqrt(ks)
    return phi.to(device)


def _outlier_scale(H: int, d: int, g: torch.Generator, device, n_out: int = 4,
                   factor: float = 20.0) -> torch.Tensor:
    """[H, 1, d] multipliers: n_out channels per head (without replacement) x factor."""
    scale = torch.ones(H, 1, d, device=device, dtype=torch.float32)
    for h in range(H):
        ch = torch.randperm(d, generator=g, device=device)[:n_out]
        scale[h, 0, ch] = factor
    return scale


def _values(L, H, n, d, g, device) -> torch.Tensor:
    v = torch.empty(L, H, n, d, device=device, dtype=torch.bfloat16)
    for l in range(L):
        v[l] = torch.randn(H, n, d, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    return v


def gaussian_outlier_keys(L, H, n, d, g, device) -> torch.Tensor:
    """i.i.d. N(0,1) keys with 4 outlier channels per head scaled x20."""
    k = torch.empty(L, H, n, d, device=device, dtype=torch.bfloat16)
    for l in range(L):
        x = torch.randn(H, n, d, generator=g, device=device, dtype=torch.float32)
        x *= _outlier_scale(H, d, g, device)
        k[l] = x.to(torch.bfloat16)
    return k


def lowrank_outlier_keys(L, H, n, d, g, device, rank=32, noise=0.1) -> torch.Tensor:
    """rank-`rank` Gaussian signal of unit per-entry variance + N(0, noise^2)
    noise (noise is a standard deviation) + 4 outlier channels x20 per head."""
    k = torch.empty(L, H, n, d, device=device, dtype=torch.bfloat16)
    for l in range(L):
        a = torch.randn(H, n, rank, generator=g, device=device, dtype=torch.float32)
        b = torch.randn(H, d, rank, generator=g, device=device, dtype=torch.float32)
        x = torch.bmm(a, b.transpose(1, 2)) / math.sqrt(rank)
        x += noise * torch.randn(H, n, d, generator=g, device=device, dtype=torch.float32)
        x *= _outlier_scale(H, d, g, device)
        k[l] = x.to(torch.bfloat16)
    return k


def student_t_rotated_keys(L, H, n, d, g, device, nu=3) -> torch.Tensor:
    """Heavy-tailed keys: Student-t(nu) entries (normal / sqrt(chi2_nu / nu)),
    right-multiplied by a per-head Haar-random rotation."""
    k = torch.empty(L, H, n, d, device=device, dtype=torch.bfloat16)
    for l in range(L):
        z = torch.randn(H, n, d, generator=g, device=device, dtype=torch.float32)
        chi2 = torch.zeros(H, n, d, device=device, dtype=torch.float32)
        for _ in range(nu):
            chi2 += torch.randn(H, n, d, generator=g, device=device, dtype=torch.float32) ** 2
        t = z / torch.sqrt(chi2 / nu)
        m = torch.randn(H, d, d, generator=g, device=device, dtype=torch.float32)
        q, r = torch.linalg.qr(m.cpu())          # Haar measure after the sign fix
        q = (q * torch.sign(torch.diagonal(r, dim1=1, dim2=2)).unsqueeze(1)).to(device)
        k[l] = torch.bmm(t, q).to(torch.bfloat16)
    return k


def rank_deficient_duplicate_keys(L, H, n, d, g, device, rank=96, dup_frac=0.05) -> torch.Tensor:
    """Rank-`rank` keys (before bf16 rounding) with dup_frac of the rows
    overwritten by the exact bits of another, non-overwritten row."""
    k = torch.empty(L, H, n, d, device=device, dtype=torch.bfloat16)
    n_dup = int(round(dup_frac * n))
    for l in range(L):
        a = torch.randn(H, n, rank, generator=g, device=device, dtype=torch.float32)
        b = torch.randn(H, rank, d, generator=g, device=device, dtype=torch.float32)
        x = (torch.bmm(a, b) / math.sqrt(rank)).to(torch.bfloat16)
        for h in range(H):
            perm = torch.randperm(n, generator=g, device=device)
            dst = perm[:n_dup]
            pool = perm[n_dup:]
            src = pool[torch.randint(0, pool.numel(), (n_dup,), generator=g, device=device)]
            x[h, dst] = x[h, src]
        k[l] = x
    return k


# --------------------------------------------------------------------------
# the five configurations (full sizes by default; tests pass smaller shapes)
# --------------------------------------------------------------------------
def config1(device="cpu", seed=0, L=1, H=1, n=4096, ratio=0.5) -> Workload:
    """Single head, Gaussian keys + 4 outlier channels x20, keep 50 %."""
    g = _gen(device, seed, 1)
    k = gaussian_outlier_keys(L, H, n, HEAD_DIM, g, device)
    v = _values(L, H, n, HEAD_DIM, g, device)
    return Workload("config1_single_head", L, H, [Request(k, v, ratio)])


def config2(device="cpu", seed=0, L=32, H=8, n=32768, ratio=0.3) -> Workload:
    """Llama-3.1-8B shape: low-rank(32) signal + 0.1 noise + outliers, keep 30 %."""
    g = _gen(device, seed, 2)
    k = lowrank_outlier_keys(L, H, n, HEAD_DIM, g, device)
    v = _values(L, H, n, HEAD_DIM, g, device)
    return Workload("config2_llama31_8b_n32768", L, H, [Request(k, v, ratio)])


def config3(device="cpu", seed=0, L=28, H=4, n=131072, ratio=0.2) -> Workload:
    """Qwen-2.5-7B shape: Student-t(3) keys with per-head rotation, keep 20 %."""
    g = _gen(device, seed, 3)
    k = student_t_rotated_keys(L, H, n, HEAD_DIM, g, device)
    v = _values(L, H, n, HEAD_DIM, g, device)
    return Workload("config3_qwen25_7b_n131072", L, H, [Request(k, v, ratio)])


def config4(device="cpu", seed=0, L=32, H=8, n_req=16, n_lo=8192, n_hi=65536,
            r_lo=0.2, r_hi=0.6) -> Workload:
    """Ragged batch: n_req requests, n ~ U{n_lo..n_hi}, per-request retention
    r ~ U[r_lo, r_hi] (stands for a context-calibrated ratio, Sec. 3.4)."""
    g0 = torch.Generator(device="cpu")
    g0.manual_seed(seed * 1000003 + 1009 * 4)
    ns = torch.randint(n_lo, n_hi + 1, (n_req,), generator=g0).tolist()
    rs = (r_lo + (r_hi - r_lo) * torch.rand(n_req, generator=g0)).tolist()
    reqs = []
    for b in range(n_req):
        g = _gen(device, seed, 4, b + 1)
        k = gaussian_outlier_keys(L, H, ns[b], HEAD_DIM, g, device)
        v = _values(L, H, ns[b], HEAD_DIM, g, device)
        reqs.append(Request(k, v, float(rs[b])))
    return Workload("config4_ragged_batch", L, H, reqs)


def config5(device="cpu", seed=0, L=64, H=8, n=100000, ratio=0.32,
            exact=False) -> Workload:
    """Qwen-2.5-32B shape: rank-96 keys with 5 % exact-duplicate rows, keep 32 %.
    exact=True asks for exact ridge leverage scores (ridge_rel 1e-4)."""
    g = _gen(device, seed, 5)
    k = rank_deficient_duplicate_keys(L, H, n, HEAD_DIM, g, device)
    v = _values(L, H, n, HEAD_DIM, g, device)
    w = Workload("config5_qwen25_32b_n100000", L, H, [Request(k, v, ratio)])
    if exact:
        w.sketch_dim, w.ridge_rel = 0, 1e-4
    return w


def synthetic_attention_scores(L, H, n, device="cpu", seed=0) -> torch.Tensor:
    """Stand-in for the attention score vector a (fp32 [L,H,n], positive,
    skewed): exp of a Gaussian.  Only used to exercise the blend."""
    g = _gen(device, seed, 7)
    return torch.exp(torch.randn(L, H, n, generator=g, device=device, dtype=torch.float32))


def synthetic_queries(L, Hq, n, d=HEAD_DIM, device="cpu", seed=0, request=0) -> torch.Tensor:
    """Stand-in for the model's queries, bf16 [L, Hq, n, d]: N(0,1) entries with a per-head
    gain in [0.5, 1.5], so that heads differ in how peaked their attention is."""
    g = _gen(device, seed, 8, request)
    q = torch.empty(L, Hq, n, d, device=device, dtype=torch.bfloat16)
    for l in range(L):
        gain = 0.5 + torch.rand(Hq, 1, 1, generator=g, device=device, dtype=torch.float32)
        q[l] = (gain * torch.randn(Hq, n, d, generator=g, device=device, dtype=torch.float32)).to(torch.bfloat16)
    return q


def bf16_bits(t: torch.Tensor):
    """Raw bit patterns (numpy uint16) of a bf16 tensor, for the oracle."""
    return t.contiguous().view(torch.int16).cpu().numpy().view("uint16")
