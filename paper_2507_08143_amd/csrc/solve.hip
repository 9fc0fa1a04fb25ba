// Small per-head factorisation (paper Algorithm 1 line 4, in the Cholesky form; Appendix C
// notes that routes other than the SVD give the same scores).
//
//   sketched:  S = Phi^T G Phi + rho I  (k_s x k_s),   exact:  S = G + rho I  (d x d)
//   S = L L^T,   W^T = L^{-1} Phi^T  (k_s x d)   [exact: W^T = L^{-1}]
//
// so that the score of a token is o_i = || W^T k_i ||^2 = k^_i^T S^{-1} k^_i, which equals
// diag(U~ U~^T) of Algorithm 1 lines 5-6 when rho = 0.  All arithmetic here is fp64; W^T leaves
// as a sum of bf16 planes for the MFMA score pass.
#include "common.h"

namespace cmp {

typedef double f64x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ Where locate_head(const SegTable &T, int lhead) {
  Where w{0, 0, lhead, 0};
  for (int i = 0; i < T.nseg; ++i) {
    const int hh = lhead - T.s[i].lhead0;
    if (hh < T.s[i].head_count || i == T.nseg - 1) {
      w.seg = i;
      w.head = T.s[i].head_begin + hh;
      return w;
    }
  }
  return w;
}

__device__ __forceinline__ uint16_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);   // inf / nan: truncate
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// A pivot below this fraction of its own (ridged) diagonal entry is below what the fp32-
// accumulated Gram matrix resolves: the direction is dropped and the head flagged.
constexpr double PIVOT_REL = 1.4901161193847656e-08;   // 2^-26

// ---- sketched mode, one kernel: partial Gram blocks -> S -> L -> L^{-1} -> W^T ------------------
// One workgroup (4 waves) per head; every O(n^3)-ish piece runs on the fp64 matrix cores
// (16x16x4 MFMA: A[i][k] in lane (i = l & 15, k = l >> 4), B[k][j] in lane (j = l & 15,
// k = l >> 4), register v of lane l of the result is D[4v + (l >> 4)][l & 15]):
//   1. S = Phi^T G Phi, G summed in fp64 from the head's partial blocks; a wave takes 32 rows of G
//      through T = G Phi to its share of S in registers, then the four shares are added
//   2. blocked right-looking Cholesky of S + rho I with 16-wide panels: wave 0 factors the
//      diagonal block in registers (the only serial part, 16 pivots) and inverts it, the panel
//      below is L_qp = A_qp X_pp^T and the trailing blocks get A_qr -= L_qp L_rp^T
//   3. X = L^{-1} block by block (X_qp = -X_qq sum_r L_qr X_rp), one wave per block column
//   4. W^T = X Phi^T, split into bf16 planes
// A pivot below PIVOT_REL of its own ridged diagonal entry is dropped: 1/L_kk := 0, which zeroes
// column k of L, row and column k of X and row k of W^T, and flags the head.
__device__ __forceinline__ void wave_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ double readlane_f64(double x, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
  return __hiloint2double(hi, lo);
}

// Rows 32 WV + 16t .. + 15 of G = sum of a head's partial Gram matrices, in the arrangement of
// an fp64 MFMA A operand: g[q] of lane (l16, lq) is G[32 WV + 16t + l16][4q + lq].  G is
// symmetric and only its upper blocks are stored, so an element left of the diagonal block is
// read as its mirror image; in the diagonal block and right of it the 16 lanes of a row tile
// read consecutive 16-byte pieces.  Sums are fp64, in split order, two splits in flight.
struct PartialRows {
  const float *src;     // the head's first partial
  int nsplit, l16, lq;
  int wv;               // the wave (uniform): rows 32 wv .. 32 wv + 31
};
__device__ __forceinline__ void fetch_partial_rows(const PartialRows &P, int sp, int t, float (&v)[32]) {
  // float offsets inside a partial: the lane's part (one address register per arrangement) and
  // a part that is the same for all lanes
  const unsigned lane_up = 4 * P.l16 + P.lq;   // stored block (kb, wv): row 4(q&7) + lq, column 16t + l16
  const unsigned lane_lo = (64 * (P.l16 >> 3) + 32 * ((P.l16 >> 2) & 1)) * 4 + (P.l16 & 3) + 4 * P.lq;
                                               // stored block (wv, kb): row 16t + l16, column 4(q&7) + lq
  const float *ps = P.src + (long long)sp * GRAM_PARTIAL_FLOATS;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    if (kb <= P.wv) {                          // uniform
      const float *pb = ps + (upper_block(kb, P.wv) * 1024 + 64 * t);
#pragma unroll
      for (int u = 0; u < 8; ++u) v[8 * kb + u] = (pb + (64 * (u >> 1) + 32 * (u & 1)) * 4)[lane_up];
    } else {
      const float *pb = ps + (upper_block(P.wv, kb) * 1024 + 512 * t);
#pragma unroll
      for (int u = 0; u < 8; ++u) v[8 * kb + u] = (pb + 16 * u)[lane_lo];
    }
  }
}
// v0, v1 hold splits 0 and 1 on entry (fetched by the caller, so that they can be in flight behind
// other work)
__device__ __forceinline__ void sum_partial_rows(const PartialRows &P, int t, float (&v0)[32],
                                                 float (&v1)[32], double (&g)[32]) {
  for (int sp = 0; sp < P.nsplit; sp += 2) {
#pragma unroll
    for (int q = 0; q < 32; ++q) g[q] += (double)v0[q];
    if (sp + 2 < P.nsplit) fetch_partial_rows(P, sp + 2, t, v0);
    if (sp + 1 < P.nsplit) {
#pragma unroll
      for (int q = 0; q < 32; ++q) g[q] += (double)v1[q];
      if (sp + 3 < P.nsplit) fetch_partial_rows(P, sp + 3, t, v1);
    }
  }
}
__device__ __forceinline__ void fetch_first_splits(const PartialRows &P, int t, float (&v0)[32],
                                                   float (&v1)[32]) {
  if (P.nsplit > 0) fetch_partial_rows(P, 0, t, v0);
  if (P.nsplit > 1) fetch_partial_rows(P, 1, t, v1);
}

// Cholesky factor of a 16 x 16 diagonal block held one row per lane (lanes 0..15 of one wave):
// lrow[k] = L[lane][k]; 1 / L[k][k] goes to rs[k] (LDS); returns false if a pivot was dropped.
// The 16 pivots are one dependent chain.  What the next pivot needs of this one (column k + 1)
// comes by a lane read; the rest of the column goes through LDS (col, 64 doubles) and is applied
// one pivot later, behind that pivot's reciprocal square root, so no LDS round trip sits on the
// chain.  Every element still receives its updates in pivot order.
__device__ __forceinline__ bool chol16(double (&row)[16], double d0_mine, bool rowlane, int lane,
                                       double *rs, double *col, double (&lrow)[16]) {
  bool all_ok = true;
  double cv[16], lk_prev = 0.0;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const double piv = readlane_f64(row[k], k);
    const double d0k = readlane_f64(d0_mine, k);
    const bool ok = piv > PIVOT_REL * d0k && piv < 1.0e300;      // false for NaN too
    const double r = ok ? rsqrt(piv) : 0.0;
    all_ok &= ok;
    if (lane == k) rs[k] = r;
    const double lk = (rowlane && lane >= k) ? row[k] * r : 0.0;   // L[lane][k]
    lrow[k] = lk;
    if (k > 0) {
#pragma unroll
      for (int j = k + 1; j < 16; ++j) row[j] -= lk_prev * cv[j];  // pivot k - 1, cv[j] = L[j][k-1]
    }
    if (k < 15) row[k + 1] -= lk * readlane_f64(lk, k + 1);        // pivot k, the column needed next
    wave_fence();
    col[lane] = lk;
    wave_fence();
#pragma unroll
    for (int j = k + 2; j < 16; ++j) cv[j] = col[j];               // L[j][k], for the next round
    lk_prev = lk;
  }
  return all_ok;
}

template <int M>
__global__ __launch_bounds__(256, M > 48 ? 1 : 2) void sketch_solve_kernel(
    const SegTable T, int tiles_per_wg, const float *__restrict__ partials,
    const float *__restrict__ phi, float ridge_rel, uint16_t *__restrict__ wt,
    int32_t *__restrict__ status, int *__restrict__ zero, long long zero_ints) {
  constexpr int P = M / 16, CT = M / 16;
  // LDS pitch in doubles.  Two workgroups fit a CU, so that the serial parts of one overlap the
  // matrix work of the other.
  constexpr int SP = M + 1;
  __shared__ double region[2 * M * SP];
  __shared__ __attribute__((aligned(16))) float PH[D * M];
  double *Ss = region;                 // S, then L in its lower blocks
  double *Xs = region + M * SP;        // L^{-1} (lower blocks)
  __shared__ double d0_s[M], rs_s[M], col_s[64];
  __shared__ int flag_s;

  const int lhead = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  // Phi on its way to LDS: the loads leave first and are stored once the loads of the partial
  // sums and the clearing stores have been issued behind them
  constexpr int PHN = (D * M / 4 + 255) / 256;
  float4 ph_reg[PHN];
#pragma unroll
  for (int i = 0; i < PHN; ++i) {
    const int idx = tid + 256 * i;
    ph_reg[i] = idx < D * M / 4 ? reinterpret_cast<const float4 *>(phi)[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (tid == 0) flag_s = 0;

  // ---- 1. S = Phi^T G Phi ----
  // Wave w owns rows 32w .. 32w+31 of G.  As the A operand of T = G Phi lane (l16, lq) holds
  // G[32w + 16t + l16][4q + lq] for t < 2, q < 32; it fetches these 64 numbers of every partial
  // straight from the stored blocks (G is symmetric, so whichever of (row, col) and (col, row)
  // lies in an upper block is read) and sums them in fp64 in split order.  T's accumulators
  // are in turn B operands of S_w = Phi_w^T T_w (the rows of this wave), so G and T never pass
  // through LDS and nothing waits on a barrier until the four S_w are added.
  int nsplit;
  const long long pb = partial_base(T, lhead, tiles_per_wg, nsplit);
  constexpr int CT2 = CT * CT;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const PartialRows PR{partials + pb * GRAM_PARTIAL_FLOATS, nsplit, l16, lq, wv};
  float v0[32], v1[32];
  fetch_first_splits(PR, 0, v0, v1);
  zero_slice(zero, zero_ints);   // histograms that the score and selection kernels add into
#pragma unroll
  for (int i = 0; i < PHN; ++i) {
    const int idx = tid + 256 * i;
    if (idx < D * M / 4) reinterpret_cast<float4 *>(PH)[idx] = ph_reg[i];
  }
  __syncthreads();                                // Phi is in LDS
  // T_w = G_w Phi, one 16-row tile of G at a time: CT tiles, 32 steps each, independent chains;
  // the first splits of the second tile are in flight during the products of the first
  f64x4 tacc[2][CT];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    double ga[32];
#pragma unroll
    for (int q = 0; q < 32; ++q) ga[q] = 0.0;
    sum_partial_rows(PR, t, v0, v1, ga);
    if (t == 0) fetch_first_splits(PR, 1, v0, v1);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) tacc[t][ct] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q0 = 0; q0 < 32; q0 += 8) {
      float pbv[8][CT];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) pbv[u][ct] = PH[(4 * (q0 + u) + lq) * M + 16 * ct + l16];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          tacc[t][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(ga[q0 + u], (double)pbv[u][ct], tacc[t][ct], 0, 0, 0);
    }
  }
  // S_w = Phi_w^T T_w: register v of T's accumulators is row 4v + lq of the tile, which is the
  // B operand of step v
  f64x4 sacc[CT2];
#pragma unroll
  for (int i = 0; i < CT2; ++i) sacc[i] = f64x4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    float pav[4][CT];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int at = 0; at < CT; ++at) pav[v][at] = PH[(32 * wv + 16 * t + 4 * v + lq) * M + 16 * at + l16];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int at = 0; at < CT; ++at)
#pragma unroll
        for (int bt = 0; bt < CT; ++bt)
          sacc[at * CT + bt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)pav[v][at], tacc[t][bt][v],
                                                                    sacc[at * CT + bt], 0, 0, 0);
  }
  // S = (S_0 + S_2) + (S_1 + S_3), in this order whatever the waves' timing
  auto put = [&](double *dst) {
#pragma unroll
    for (int at = 0; at < CT; ++at)
#pragma unroll
      for (int bt = 0; bt < CT; ++bt)
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[(16 * at + 4 * v + lq) * SP + 16 * bt + l16] = sacc[at * CT + bt][v];
  };
  auto add = [&](const double *src) {
#pragma unroll
    for (int at = 0; at < CT; ++at)
#pragma unroll
      for (int bt = 0; bt < CT; ++bt)
#pragma unroll
        for (int v = 0; v < 4; ++v) sacc[at * CT + bt][v] += src[(16 * at + 4 * v + lq) * SP + 16 * bt + l16];
  };
  if (wave == 2) put(Ss);
  if (wave == 3) put(Xs);
  __syncthreads();
  if (wave == 0) add(Ss);
  if (wave == 1) add(Xs);
  __syncthreads();
  if (wave == 1) put(Xs);
  __syncthreads();
  if (wave == 0) {
    add(Xs);
    put(Ss);
  }
  __syncthreads();

  // ridge: rho = ridge_rel * trace(S) / M (every thread sums in the same order)
  double tr = 0.0;
  for (int a = 0; a < M; ++a) tr += Ss[a * SP + a];
  const double rho = (double)ridge_rel * tr / (double)M;
  __syncthreads();
  if (tid < M) {
    const double v = Ss[tid * SP + tid] + rho;
    Ss[tid * SP + tid] = v;
    d0_s[tid] = v;
  }
  __syncthreads();

  // ---- 2. blocked Cholesky ----
#pragma unroll 1
  for (int p = 0; p < P; ++p) {
    if (wave == 0) {
      const int base = 16 * p;
      const bool rowlane = lane < 16;
      double row[16], lrow[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) row[j] = rowlane ? Ss[(base + lane) * SP + base + j] : 0.0;
      const double d0_mine = rowlane ? d0_s[base + lane] : 0.0;
      if (!chol16(row, d0_mine, rowlane, lane, rs_s + base, col_s, lrow) && lane == 0)
        flag_s = COMPACTOR_STATUS_PIVOT;
      if (rowlane) {
#pragma unroll
        for (int k = 0; k < 16; ++k) Ss[(base + lane) * SP + base + k] = lrow[k];
      }
      wave_fence();
      // X_pp = L_pp^{-1}: lane j solves column j by forward substitution.  Column by column of
      // L: as soon as x[k] is known every later row takes its term, so the dependent chain is 16
      // steps long and not 120 (each row still adds its terms in the order k = 0, 1, ...)
      double x[16], acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = (i == lane) ? 1.0 : 0.0;
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        x[k] = acc[k] * rs_s[base + k];
#pragma unroll
        for (int i = k + 1; i < 16; ++i) acc[i] -= Ss[(base + i) * SP + base + k] * x[k];
      }
      if (rowlane) {
#pragma unroll
        for (int i = 0; i < 16; ++i) Xs[(base + i) * SP + base + lane] = x[i];
      }
    }
    __syncthreads();
    // panel below the diagonal block: L_qp = A_qp X_pp^T
    for (int q = p + 1 + wave; q < P; q += 4) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const double a = Ss[(16 * q + l16) * SP + 16 * p + 4 * ks + lq];
        const double b = Xs[(16 * p + l16) * SP + 16 * p + 4 * ks + lq];
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) Ss[(16 * q + 4 * v + lq) * SP + 16 * p + l16] = acc[v];
    }
    __syncthreads();
    // trailing blocks: A_qr -= L_qp L_rp^T for p < r <= q
    int t = 0;
    for (int q = p + 1; q < P; ++q)
      for (int r = p + 1; r <= q; ++r, ++t) {
        if ((t & 3) != wave) continue;
        f64x4 acc;
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = Ss[(16 * q + 4 * v + lq) * SP + 16 * r + l16];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const double a = -Ss[(16 * q + l16) * SP + 16 * p + 4 * ks + lq];
          const double b = Ss[(16 * r + l16) * SP + 16 * p + 4 * ks + lq];
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) Ss[(16 * q + 4 * v + lq) * SP + 16 * r + l16] = acc[v];
      }
    __syncthreads();
  }

  // ---- 3. the blocks of X = L^{-1} below the diagonal, block column `wave` ----
  if (wave < P - 1) {
    const int p = wave;
    for (int q = p + 1; q < P; ++q) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
      for (int r = p; r < q; ++r) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const double a = Ss[(16 * q + l16) * SP + 16 * r + 4 * ks + lq];      // L_qr[i][k]
          const double b = Xs[(16 * r + 4 * ks + lq) * SP + 16 * p + l16];      // X_rp[k][j]
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
      }
      // X_qp = -X_qq acc: the result layout of acc is the B-operand layout of the next product
      f64x4 out = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const double a = -Xs[(16 * q + l16) * SP + 16 * q + 4 * ks + lq];
        out = __builtin_amdgcn_mfma_f64_16x16x4f64(a, acc[ks], out, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) Xs[(16 * q + 4 * v + lq) * SP + 16 * p + l16] = out[v];
      wave_fence();            // the next block row of this column reads what was just written
    }
  }
  __syncthreads();

  // ---- 4. W^T = X Phi^T (M x 128), lower block triangle of X only ----
  uint16_t *wh = wt + (size_t)lhead * (W_TERMS * M * D);
  auto emit = [&](int mt, int ct, const f64x4 &acc) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int m = 16 * mt + 4 * v + lq, c = 16 * ct + l16;
      float x = (float)acc[v];
#pragma unroll
      for (int tt = 0; tt < W_TERMS; ++tt) {
        const uint16_t b = bf16_rne(x);
        wh[(tt * M + m) * D + c] = b;
        x -= bf16_to_f32(b);
      }
    }
  };
  // a wave takes the column tiles ct = wave and wave + 4 of every row block: two chains
#pragma unroll
  for (int mt = 0; mt < P; ++mt) {
    f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
    const int ct0 = wave, ct1 = wave + 4;
#pragma unroll
    for (int ks = 0; ks < 4 * (mt + 1); ++ks) {
      const double a = Xs[(16 * mt + l16) * SP + 4 * ks + lq];
      const double b0 = (double)PH[(16 * ct0 + l16) * M + 4 * ks + lq];
      const double b1 = (double)PH[(16 * ct1 + l16) * M + 4 * ks + lq];
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b1, acc1, 0, 0, 0);
    }
    emit(mt, ct0, acc0);
    emit(mt, ct1, acc1);
  }
  if (tid == 0) {
    const Where w = locate_head(T, lhead);
    status[T.s[w.seg].ghead0 + w.head] = flag_s;
  }
}

// ---- exact mode, one kernel: partial Gram blocks -> G + rho I -> L -> L^{-1} = W^T -------------
// The same blocked factorisation as above on the full 128 x 128 Gram matrix (8 panels of 16).
// One matrix of 128 x 129 doubles is all LDS has room for, so L lives in its lower block
// triangle and the blocks of X = L^{-1} below the diagonal are written, transposed, into the
// upper block triangle, which the factorisation never reads (element X[j][c], block of j below
// block of c, is at S[c][j]); the eight diagonal blocks of X have an array of their own.
__global__ __launch_bounds__(256) void exact_solve_kernel(
    const SegTable T, int tiles_per_wg, const float *__restrict__ partials, float ridge_rel,
    uint16_t *__restrict__ wt, int32_t *__restrict__ status, int *__restrict__ zero,
    long long zero_ints) {
  constexpr int M = D, P = M / 16, SP = M + 1;
  __shared__ double Ss[M * SP];
  __shared__ double Xd[P][16][17];
  __shared__ double d0_s[M], rs_s[M], col_s[64];
  __shared__ int flag_s;

  const int lhead = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  if (tid == 0) flag_s = 0;
  zero_slice(zero, zero_ints);   // histograms that the score and selection kernels add into

  // ---- 1. G: the head's 10 upper blocks summed over the splits in fp64 (split order) ----
  int nsplit;
  const long long pb = partial_base(T, lhead, tiles_per_wg, nsplit);
  int row0, col;
  partial_quad(tid, row0, col);   // this thread's float4 of a block: rows row0..+3 of column col
  double gsum[10][4];
#pragma unroll
  for (int b = 0; b < 10; ++b)
#pragma unroll
    for (int c = 0; c < 4; ++c) gsum[b][c] = 0.0;
  {
    const float *src = partials + pb * GRAM_PARTIAL_FLOATS + tid * 4;
    for (int s0 = 0; s0 < nsplit; s0 += 2) {
      float4 v[2][10];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int b = 0; b < 10; ++b) {
          v[u][b] = make_float4(0.f, 0.f, 0.f, 0.f);
          if (s0 + u < nsplit)
            v[u][b] = *reinterpret_cast<const float4 *>(src + (long long)(s0 + u) * GRAM_PARTIAL_FLOATS + b * 1024);
        }
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int b = 0; b < 10; ++b) {
          gsum[b][0] += v[u][b].x; gsum[b][1] += v[u][b].y;
          gsum[b][2] += v[u][b].z; gsum[b][3] += v[u][b].w;
        }
    }
  }
  // into the lower triangle: block (I, J), I < J, holds G[32I + r][32J + c] = G[32J + c][32I + r]
#pragma unroll
  for (int I = 0; I < 4; ++I)
#pragma unroll
    for (int J = I; J < 4; ++J) {
      const int blk = upper_block(I, J);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (I == J) Ss[(32 * I + row0 + c) * SP + 32 * J + col] = gsum[blk][c];
        else        Ss[(32 * J + col) * SP + 32 * I + row0 + c] = gsum[blk][c];
      }
    }
  __syncthreads();

  // ridge: rho = ridge_rel * trace(G) / M (every thread sums in the same order)
  double tr = 0.0;
  for (int a = 0; a < M; ++a) tr += Ss[a * SP + a];
  const double rho = (double)ridge_rel * tr / (double)M;
  __syncthreads();
  if (tid < M) {
    const double v = Ss[tid * SP + tid] + rho;
    Ss[tid * SP + tid] = v;
    d0_s[tid] = v;
  }
  __syncthreads();

  // ---- 2. blocked Cholesky ----
#pragma unroll 1
  for (int p = 0; p < P; ++p) {
    if (wave == 0) {
      const int base = 16 * p;
      const bool rowlane = lane < 16;
      double row[16], lrow[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) row[j] = rowlane ? Ss[(base + lane) * SP + base + j] : 0.0;
      const double d0_mine = rowlane ? d0_s[base + lane] : 0.0;
      if (!chol16(row, d0_mine, rowlane, lane, rs_s + base, col_s, lrow) && lane == 0)
        flag_s = COMPACTOR_STATUS_PIVOT;
      if (rowlane) {
#pragma unroll
        for (int k = 0; k < 16; ++k) Ss[(base + lane) * SP + base + k] = lrow[k];
      }
      wave_fence();
      // X_pp = L_pp^{-1}: lane j solves column j by forward substitution.  Column by column of
      // L: as soon as x[k] is known every later row takes its term, so the dependent chain is 16
      // steps long and not 120 (each row still adds its terms in the order k = 0, 1, ...)
      double x[16], acc[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = (i == lane) ? 1.0 : 0.0;
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        x[k] = acc[k] * rs_s[base + k];
#pragma unroll
        for (int i = k + 1; i < 16; ++i) acc[i] -= Ss[(base + i) * SP + base + k] * x[k];
      }
      if (rowlane) {
#pragma unroll
        for (int i = 0; i < 16; ++i) Xd[p][i][lane] = x[i];
      }
    }
    __syncthreads();
    // panel below the diagonal block: L_qp = A_qp X_pp^T
    for (int q = p + 1 + wave; q < P; q += 4) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const double a = Ss[(16 * q + l16) * SP + 16 * p + 4 * ks + lq];
        const double b = Xd[p][l16][4 * ks + lq];
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) Ss[(16 * q + 4 * v + lq) * SP + 16 * p + l16] = acc[v];
    }
    __syncthreads();
    // trailing blocks: A_qr -= L_qp L_rp^T for p < r <= q
    int t = 0;
    for (int q = p + 1; q < P; ++q)
      for (int r = p + 1; r <= q; ++r, ++t) {
        if ((t & 3) != wave) continue;
        f64x4 acc;
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = Ss[(16 * q + 4 * v + lq) * SP + 16 * r + l16];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const double a = -Ss[(16 * q + l16) * SP + 16 * p + 4 * ks + lq];
          const double b = Ss[(16 * r + l16) * SP + 16 * p + 4 * ks + lq];
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) Ss[(16 * q + 4 * v + lq) * SP + 16 * r + l16] = acc[v];
      }
    __syncthreads();
  }

  // ---- 3. the blocks of X = L^{-1} below the diagonal: X_qp = -X_qq sum_r L_qr X_rp.  A wave
  // takes the block columns p = wave and wave + 4; a column only reads what the same wave wrote.
  for (int p = wave; p < P - 1; p += 4) {
    for (int q = p + 1; q < P; ++q) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
      for (int r = p; r < q; ++r) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const double a = Ss[(16 * q + l16) * SP + 16 * r + 4 * ks + lq];        // L_qr[i][k]
          const double b = r == p ? Xd[p][4 * ks + lq][l16]                        // X_pp[k][j]
                                  : Ss[(16 * p + l16) * SP + 16 * r + 4 * ks + lq];  // X_rp[k][j], transposed
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
      }
      // the result layout of acc is the B-operand layout of the next product
      f64x4 out = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const double a = -Xd[q][l16][4 * ks + lq];
        out = __builtin_amdgcn_mfma_f64_16x16x4f64(a, acc[ks], out, 0, 0, 0);
      }
      // X_qp[i = 4v + lq][j = l16], stored transposed in block (p, q) of the upper triangle
#pragma unroll
      for (int v = 0; v < 4; ++v) Ss[(16 * p + l16) * SP + 16 * q + 4 * v + lq] = out[v];
      wave_fence();            // the next block row of this column reads what was just written
    }
  }
  __syncthreads();

  // ---- 4. W^T = X (lower triangular), split into bf16 planes ----
  uint16_t *wh = wt + (size_t)lhead * (W_TERMS * M * D);
  const int ch = tid & 127;
  for (int j = tid >> 7; j < M; j += 2) {
    const int qb = j >> 4, pb2 = ch >> 4;
    double wv = 0.0;
    if (pb2 == qb) wv = Xd[qb][j & 15][ch & 15];
    else if (pb2 < qb) wv = Ss[ch * SP + j];
    float x = (float)wv;
#pragma unroll
    for (int t = 0; t < W_TERMS; ++t) {
      const uint16_t b = bf16_rne(x);
      wh[(t * M + j) * D + ch] = b;
      x -= bf16_to_f32(b);
    }
  }
  if (tid == 0) {
    const Where w = locate_head(T, lhead);
    status[T.s[w.seg].ghead0 + w.head] = flag_s;
  }
}

template <int M>
static hipError_t launch_sketched(const SegTable &T, int tiles_per_wg, const float *partials,
                                  const float *phi, float ridge_rel, uint16_t *wt,
                                  int32_t *status, int *zero, long long zero_ints,
                                  hipStream_t st) {
  hipLaunchKernelGGL((sketch_solve_kernel<M>), dim3((unsigned)T.nheads), dim3(256), 0, st, T,
                     tiles_per_wg, partials, phi, ridge_rel, wt, status, zero, zero_ints);
  return hipGetLastError();
}

// Sketched mode: partial Gram blocks -> W^T in one kernel (see above).
hipError_t launch_sketch_solve(const SegTable &T, int ks, int tiles_per_wg, const float *partials,
                               const float *phi, float ridge_rel, uint16_t *wt,
                               int32_t *status, int *zero, long long zero_ints, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  switch (ks) {
    case 16: return launch_sketched<16>(T, tiles_per_wg, partials, phi, ridge_rel, wt, status, zero, zero_ints, st);
    case 32: return launch_sketched<32>(T, tiles_per_wg, partials, phi, ridge_rel, wt, status, zero, zero_ints, st);
    case 48: return launch_sketched<48>(T, tiles_per_wg, partials, phi, ridge_rel, wt, status, zero, zero_ints, st);
    case 64: return launch_sketched<64>(T, tiles_per_wg, partials, phi, ridge_rel, wt, status, zero, zero_ints, st);
    default: return hipErrorInvalidValue;
  }
}

// Subsampled randomized Hadamard sketch (paper App. D) as a dense Phi: the sign bits and the
// chosen rows of H travel as kernel arguments.
struct SrhtSpec {
  uint32_t sign_bits[D / 32];
  uint8_t cols[64];
};
__global__ __launch_bounds__(256) void srht_phi_kernel(SrhtSpec spec, int ks, float value,
                                                       float *__restrict__ phi) {
  for (int idx = threadIdx.x + blockIdx.x * 256; idx < D * ks; idx += 256 * gridDim.x) {
    const int i = idx / ks, j = idx - i * ks;
    const unsigned neg = ((spec.sign_bits[i >> 5] >> (i & 31)) & 1u) ^
                         (__popc((unsigned)i & (unsigned)spec.cols[j]) & 1u);
    phi[idx] = neg ? -value : value;
  }
}

hipError_t launch_srht_phi(int ks, const uint8_t *signs, const int32_t *cols, float *phi,
                           hipStream_t st) {
  SrhtSpec spec;
  for (int w = 0; w < D / 32; ++w) spec.sign_bits[w] = 0;
  for (int i = 0; i < D; ++i)
    if (signs[i]) spec.sign_bits[i >> 5] |= 1u << (i & 31);
  for (int j = 0; j < 64; ++j) spec.cols[j] = j < ks ? (uint8_t)cols[j] : 0;
  hipLaunchKernelGGL(srht_phi_kernel, dim3(8), dim3(256), 0, st, spec, ks,
                     sqrtf((float)D / (float)ks), phi);
  return hipGetLastError();
}

// Exact mode: partial Gram blocks -> Cholesky of G + rho I -> W^T = L^{-1}, in one kernel.
hipError_t launch_exact_solve(const SegTable &T, int tiles_per_wg, const float *partials,
                              float ridge_rel, uint16_t *wt, int32_t *status, int *zero,
                              long long zero_ints, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(exact_solve_kernel, dim3((unsigned)T.nheads), dim3(256), 0, st, T, tiles_per_wg,
                     partials, ridge_rel, wt, status, zero, zero_ints);
  return hipGetLastError();
}

}  // namespace cmp
