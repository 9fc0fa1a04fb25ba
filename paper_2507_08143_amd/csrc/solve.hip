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

// ---- exact mode: S = G + rho I (128 x 128), one workgroup per head, everything in LDS -------
__global__ __launch_bounds__(256) void solve_exact_kernel(const SegTable T, float ridge_rel,
                                                          const double *__restrict__ g64,
                                                          uint16_t *__restrict__ wt,
                                                          int32_t *__restrict__ status) {
  constexpr int m = D, SP = D + 1;
  __shared__ double S[m * SP];
  __shared__ double dinv[m];
  __shared__ double d0[m];
  __shared__ int flag;

  const int lhead = blockIdx.x;
  const Where w = locate_head(T, lhead);
  const Seg &sg = T.s[w.seg];
  const double *G = g64 + (size_t)lhead * (D * D);
  const int tid = threadIdx.x;
  if (tid == 0) flag = 0;
  for (int idx = tid; idx < m * m; idx += 256) {
    const int a = idx / m, b = idx - a * m;
    if (b <= a) S[a * SP + b] = G[a * D + b];
  }
  __syncthreads();

  // ridge: rho = ridge_rel * trace(S) / m (every thread sums in the same order)
  double tr = 0.0;
  for (int a = 0; a < m; ++a) tr += S[a * SP + a];
  const double rho = (double)ridge_rel * tr / (double)m;
  __syncthreads();
  if (tid < m) {
    const double v = S[tid * SP + tid] + rho;
    S[tid * SP + tid] = v;
    d0[tid] = v;
  }

  // right-looking Cholesky; L overwrites the strict lower triangle, 1/L_kk goes to dinv
  const int tx = tid & 15, ty = tid >> 4;
  for (int k = 0; k < m; ++k) {
    __syncthreads();
    const double piv = S[k * SP + k];
    const bool ok = piv > PIVOT_REL * d0[k] && piv < 1.0e300;   // false for NaN too
    const double dk = ok ? 1.0 / sqrt(piv) : 0.0;
    if (tid == 0) {
      dinv[k] = dk;
      if (!ok) flag = COMPACTOR_STATUS_PIVOT;
    }
    for (int i = k + 1 + tid; i < m; i += 256) S[i * SP + k] = ok ? S[i * SP + k] * dk : 0.0;
    __syncthreads();
    if (ok) {
      for (int i = k + 1 + ty; i < m; i += 16) {
        const double lik = S[i * SP + k];
        for (int j = k + 1 + tx; j <= i; j += 16) S[i * SP + j] -= lik * S[j * SP + k];
      }
    }
  }
  __syncthreads();

  // X = L^{-1}, column c by thread c; X[j][c] (j > c) is kept in the free upper triangle S[c][j]
  if (tid < m) {
    const int c = tid;
    const double xcc = dinv[c];
    for (int j = c + 1; j < m; ++j) {
      double sum = S[j * SP + c] * xcc;
      for (int q = c + 1; q < j; ++q) sum += S[j * SP + q] * S[c * SP + q];
      S[c * SP + j] = -sum * dinv[j];
    }
  }
  __syncthreads();

  // W^T = X (lower triangular), split into bf16 planes
  uint16_t *wh = wt + (size_t)lhead * (W_TERMS * m * D);
  const int ch = tid & 127;
  for (int j = tid >> 7; j < m; j += 2) {
    const double wv = ch < j ? S[ch * SP + j] : (ch == j ? dinv[j] : 0.0);
    float x = (float)wv;
#pragma unroll
    for (int t = 0; t < W_TERMS; ++t) {
      const uint16_t b = bf16_rne(x);
      wh[(t * m + j) * D + ch] = b;
      x -= bf16_to_f32(b);
    }
  }
  if (tid == 0) status[sg.ghead0 + w.head] = flag;
}

// ---- sketched mode -------------------------------------------------------------------------
// Step 1, sketch_kernel: one workgroup per (head, 32-row block I of G).  It sums the head's
// partial Gram blocks in fp64 (split order, deterministic), forms the rows G_I (32 x 128),
// T_I = G_I Phi (32 x k_s) and the contribution S_I = Phi_I^T T_I (k_s x k_s) to
// S = Phi^T G Phi = sum_I S_I, both on the fp64 matrix cores.  All the O(d^2 k_s) work of the
// factorisation step is here, spread over 4 x heads workgroups.
template <int M>
__global__ __launch_bounds__(256) void sketch_kernel(const SegTable T, int tiles_per_wg,
                                                     const float *__restrict__ partials,
                                                     const float *__restrict__ phi,
                                                     double *__restrict__ s_parts,
                                                     int *__restrict__ zero, long long zero_ints) {
  constexpr int GP = D + 1, TP = M + 1;
  __shared__ double Gs[32 * GP];
  __shared__ double Ts[32 * TP];
  __shared__ __attribute__((aligned(16))) float PH[D * M];

  const int lhead = blockIdx.x >> 2, I = blockIdx.x & 3;
  const int tid = threadIdx.x;
  for (int idx = tid; idx < D * M / 4; idx += 256)
    reinterpret_cast<float4 *>(PH)[idx] = reinterpret_cast<const float4 *>(phi)[idx];
  zero_slice(zero, zero_ints);   // histograms that the score and selection kernels add into

  // rows 32I .. 32I+31 of G from the stored upper blocks (mirror blocks read transposed)
  int nsplit;
  const long long pb = partial_base(T, lhead, tiles_per_wg, nsplit);
  const int e = tid * 4, ii = e >> 5, jj = e & 31;
#pragma unroll
  for (int J = 0; J < 4; ++J) {
    const int blk = J >= I ? upper_block(I, J) : upper_block(J, I);
    const float *src = partials + pb * GRAM_PARTIAL_FLOATS + blk * 1024 + e;
    double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    for (int sidx = 0; sidx < nsplit; ++sidx) {
      const float4 v = *reinterpret_cast<const float4 *>(src + (long long)sidx * GRAM_PARTIAL_FLOATS);
      a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
    }
    if (J >= I) {           // stored as (I,J): element (ii, jj+q) is G[32I+ii][32J+jj+q]
      double *d = &Gs[ii * GP + 32 * J + jj];
      d[0] = a0; d[1] = a1; d[2] = a2; d[3] = a3;
    } else {                // stored as (J,I): element (ii, jj+q) is G[32J+ii][32I+jj+q]
      Gs[(jj + 0) * GP + 32 * J + ii] = a0;
      Gs[(jj + 1) * GP + 32 * J + ii] = a1;
      Gs[(jj + 2) * GP + 32 * J + ii] = a2;
      Gs[(jj + 3) * GP + 32 * J + ii] = a3;
    }
  }
  __syncthreads();

  // fp64 MFMA 16x16x4: A[i][k] sits in lane (i = l & 15, k = l >> 4), B[k][j] in lane
  // (j = l & 15, k = l >> 4); register v of lane l of the result is D[4*v + (l >> 4)][l & 15].
  const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, lq = lane >> 4;
  constexpr int CT = M / 16;
  // T_I = G_I Phi (32 x M): 2 x CT tiles, K = 128
  for (int tile = wave; tile < 2 * CT; tile += 4) {
    const int rt = tile / CT, ct = tile - rt * CT;
    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 8
    for (int ks = 0; ks < D / 4; ++ks) {
      const double a = Gs[(16 * rt + l16) * GP + 4 * ks + lq];
      const double b = (double)PH[(4 * ks + lq) * M + 16 * ct + l16];
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) Ts[(16 * rt + 4 * v + lq) * TP + 16 * ct + l16] = acc[v];
  }
  __syncthreads();

  // S_I = Phi_I^T T_I (M x M): CT x CT tiles, K = 32
  double *out = s_parts + ((size_t)lhead * 4 + I) * (M * M);
  for (int tile = wave; tile < CT * CT; tile += 4) {
    const int at = tile / CT, bt = tile - at * CT;
    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const double a = (double)PH[(32 * I + 4 * ks + lq) * M + 16 * at + l16];
      const double b = Ts[(4 * ks + lq) * TP + 16 * bt + l16];
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) out[(16 * at + 4 * v + lq) * M + 16 * bt + l16] = acc[v];
  }
}

__device__ __forceinline__ double readlane_f64(double x, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
  return __hiloint2double(hi, lo);
}

// Step 2, solve_wave_kernel: Cholesky and forward substitution in the registers of one wave,
// with no barrier.  Lane i holds row i of S; a pivot or a column entry needed by every lane is
// read with v_readlane.  The register file is walked with a sliding window so that the loops
// over the pivot index stay rolled (small code): after step k the window has moved one column
// to the right, register 0 always holds the pivot column.  Column k of L is parked in LDS for
// the substitution.  Two waves per head factor the same S redundantly and each produces 64 of
// the 128 columns of W^T = L^{-1} Phi^T (lane = channel).
//
// PANEL steps with a window of WIN registers: one 16-column panel of the factorisation.
template <int WIN>
__device__ __forceinline__ void chol_panel(double (&row)[64], double d0, int k0, int lane,
                                           double *__restrict__ Ls, int LP, double &rsv, int &flag) {
#pragma unroll 1
  for (int k = k0; k < k0 + 16; ++k) {
    const double piv = readlane_f64(row[0], k);
    const double d0k = readlane_f64(d0, k);
    const bool ok = piv > PIVOT_REL * d0k && piv < 1.0e300;      // false for NaN too
    const double rs = ok ? rsqrt(piv) : 0.0;
    rsv = (lane == k) ? rs : rsv;
    if (!ok) flag = COMPACTOR_STATUS_PIVOT;
    const double lk = ok ? row[0] * rs : 0.0;                    // L[lane][k] (lanes > k)
    Ls[k * LP + lane] = lk;
    // the column just parked is read back at wave-uniform addresses (an LDS broadcast costs a
    // third of a pair of v_readlane here); LDS operations of one wave execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const double *lc = Ls + k * LP + k;                          // lc[j] = L[k + j][k]
#pragma unroll
    for (int j = 1; j < WIN; ++j) row[j - 1] = row[j] - lk * lc[j];
  }
}

template <int WIN>
__device__ __forceinline__ void fwd_panel(double (&v)[64], int j0, const double *__restrict__ Ls,
                                          int LP, double rsv, uint16_t *__restrict__ wh, int M,
                                          int ch) {
#pragma unroll 1
  for (int j = j0; j < j0 + 16; ++j) {
    const double y = v[0] * readlane_f64(rsv, j);
    float x = (float)y;
#pragma unroll
    for (int t = 0; t < W_TERMS; ++t) {
      const uint16_t b = bf16_rne(x);
      wh[(t * M + j) * D + ch] = b;
      x -= bf16_to_f32(b);
    }
    const double *lc = Ls + j * LP + j;          // L[j + i][j], i = 1.. (same address in all lanes)
#pragma unroll
    for (int i = 1; i < WIN; ++i) v[i - 1] = v[i] - lc[i] * y;
  }
}

template <int M>
__global__ __launch_bounds__(64) void solve_wave_kernel(const SegTable T,
                                                        const float *__restrict__ phi,
                                                        float ridge_rel,
                                                        const double *__restrict__ s_parts,
                                                        uint16_t *__restrict__ wt,
                                                        int32_t *__restrict__ status) {
  constexpr int LP = 64 + 16;                    // row pitch of the parked L (doubles); the pad
  __shared__ double Ls[M * LP];                  // absorbs the reads past column M-1 below
  const int lhead = blockIdx.x >> 1, half = blockIdx.x & 1;
  const int lane = threadIdx.x;
  const bool rowlane = lane < M;
  const double *sp = s_parts + (size_t)lhead * 4 * (M * M);

  // S is symmetric: lane i reads S[j][i], contiguous across lanes, as its row entry (i, j)
  double row[64];
#pragma unroll
  for (int j = 0; j < 64; ++j) row[j] = 0.0;
#pragma unroll 1
  for (int part = 0; part < 4; ++part) {       // one contribution at a time: M loads in flight
    double tmp[M];
#pragma unroll
    for (int j = 0; j < M; ++j) tmp[j] = rowlane ? sp[part * M * M + j * M + lane] : 0.0;
#pragma unroll
    for (int j = 0; j < M; ++j) row[j] += tmp[j];
  }
  double diag = 0.0;
#pragma unroll
  for (int j = 0; j < M; ++j) diag = (lane == j) ? row[j] : diag;
  double tr = diag;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) tr += __shfl_xor(tr, d);
  const double rho = (double)ridge_rel * tr / (double)M;
  const double d0 = diag + rho;
#pragma unroll
  for (int j = 0; j < M; ++j) row[j] += (lane == j) ? rho : 0.0;
  for (int idx = lane; idx < M * LP; idx += 64) Ls[idx] = 0.0;

  // right-looking Cholesky in 16-column panels; the window shrinks by 16 per panel
  double rsv = 0.0;                              // lane k: 1 / L[k][k] (0 for a dropped pivot)
  int flag = 0;
  if constexpr (M >= 64) chol_panel<64>(row, d0, M - 64, lane, Ls, LP, rsv, flag);
  if constexpr (M >= 48) chol_panel<48>(row, d0, M - 48, lane, Ls, LP, rsv, flag);
  if constexpr (M >= 32) chol_panel<32>(row, d0, M - 32, lane, Ls, LP, rsv, flag);
  chol_panel<16>(row, d0, M - 16, lane, Ls, LP, rsv, flag);
  // the substitution below reads what other lanes parked in LDS: keep the order
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // forward substitution, column oriented, same sliding window: v -= L[:, j] * y_j
  const int ch = 64 * half + lane;
  double v[64];
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (4 * q < M) f = *reinterpret_cast<const float4 *>(phi + ch * M + 4 * q);
    v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
  }
  uint16_t *wh = wt + (size_t)lhead * (W_TERMS * M * D);
  if constexpr (M >= 64) fwd_panel<64>(v, M - 64, Ls, LP, rsv, wh, M, ch);
  if constexpr (M >= 48) fwd_panel<48>(v, M - 48, Ls, LP, rsv, wh, M, ch);
  if constexpr (M >= 32) fwd_panel<32>(v, M - 32, Ls, LP, rsv, wh, M, ch);
  fwd_panel<16>(v, M - 16, Ls, LP, rsv, wh, M, ch);

  if (half == 0 && lane == 0) {
    const Where w = locate_head(T, lhead);
    status[T.s[w.seg].ghead0 + w.head] = flag;
  }
}

template <int M>
static hipError_t launch_sketched(const SegTable &T, int tiles_per_wg, const float *partials,
                                  const float *phi, float ridge_rel, double *s_parts,
                                  uint16_t *wt, int32_t *status, int *zero, long long zero_ints,
                                  hipStream_t st, hipEvent_t mid) {
  hipLaunchKernelGGL((sketch_kernel<M>), dim3((unsigned)T.nheads * 4), dim3(256), 0, st, T,
                     tiles_per_wg, partials, phi, s_parts, zero, zero_ints);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  if (mid && hipEventRecord(mid, st) != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL((solve_wave_kernel<M>), dim3((unsigned)T.nheads * 2), dim3(64), 0, st, T, phi,
                     ridge_rel, s_parts, wt, status);
  return hipGetLastError();
}

// Sketched mode: partial Gram blocks -> W^T in two kernels (see above).  `mid`, if not null, is
// recorded between them (profiling).
hipError_t launch_sketch_solve(const SegTable &T, int ks, int tiles_per_wg, const float *partials,
                               const float *phi, float ridge_rel, double *s_parts, uint16_t *wt,
                               int32_t *status, int *zero, long long zero_ints, hipStream_t st,
                               hipEvent_t mid) {
  if (T.nheads <= 0) return hipSuccess;
  switch (ks) {
    case 16: return launch_sketched<16>(T, tiles_per_wg, partials, phi, ridge_rel, s_parts, wt, status, zero, zero_ints, st, mid);
    case 32: return launch_sketched<32>(T, tiles_per_wg, partials, phi, ridge_rel, s_parts, wt, status, zero, zero_ints, st, mid);
    case 48: return launch_sketched<48>(T, tiles_per_wg, partials, phi, ridge_rel, s_parts, wt, status, zero, zero_ints, st, mid);
    case 64: return launch_sketched<64>(T, tiles_per_wg, partials, phi, ridge_rel, s_parts, wt, status, zero, zero_ints, st, mid);
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

// Exact mode: full G (fp64, from gram_reduce) -> Cholesky of G + rho I -> W^T = L^{-1}.
hipError_t launch_solve(const SegTable &T, float ridge_rel, const double *g64, uint16_t *wt,
                        int32_t *status, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(solve_exact_kernel, dim3((unsigned)T.nheads), dim3(256), 0, st, T, ridge_rel,
                     g64, wt, status);
  return hipGetLastError();
}

}  // namespace cmp
