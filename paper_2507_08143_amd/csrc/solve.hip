// Small per-head factorisation (paper Algorithm 1 line 4, in the Cholesky form; Appendix C
// notes that routes other than the SVD give the same scores).
//
//   sketched:  S = Phi^T G Phi + rho I  (k_s x k_s),   exact:  S = G + rho I  (d x d)
//   S = L L^T,  X = L^{-1},  W^T = X Phi^T  (k_s x d)   [exact: W^T = X]
//
// so that the score of a token is o_i = || W^T k_i ||^2 = k^_i^T S^{-1} k^_i, which equals
// diag(U~ U~^T) of Algorithm 1 lines 5-6 when rho = 0.  All arithmetic here is fp64; W^T leaves
// as the sum of three bf16 planes (an exact split of its fp32 value) for the MFMA score pass.
//
// One workgroup per head; everything lives in LDS (up to 134 KB of the CU's 160 KB).
#include "common.h"

namespace cmp {

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

template <int M_MAX, bool SKETCHED>
__global__ __launch_bounds__(256) void solve_kernel(const SegTable T, int m,
                                                    const float *__restrict__ phi, float ridge_rel,
                                                    const double *__restrict__ g64,
                                                    uint16_t *__restrict__ wt,
                                                    int32_t *__restrict__ status) {
  constexpr int SP = M_MAX + 1;                        // pitch of S (doubles)
  constexpr int TP = M_MAX + 1;                        // pitch of the T / Phi staging area
  __shared__ double S[M_MAX * SP];
  __shared__ double TA[SKETCHED ? D * TP : 1];
  __shared__ double dinv[M_MAX];
  __shared__ double d0[M_MAX];
  __shared__ int flag;

  const int lhead = blockIdx.x;
  const Where w = locate_head(T, lhead);
  const Seg &sg = T.s[w.seg];
  const double *G = g64 + (size_t)lhead * (D * D);
  const int tid = threadIdx.x;
  if (tid == 0) flag = 0;

  if (SKETCHED) {
    // T = G Phi.  Thread (i, half) owns T[i][half + 2*bb]; G is symmetric so column i is read
    // as row-major G[j][i], contiguous across threads.
    const int i = tid & 127, half = tid >> 7;
    double acc[M_MAX / 2];
#pragma unroll
    for (int bb = 0; bb < M_MAX / 2; ++bb) acc[bb] = 0.0;
    for (int j = 0; j < D; ++j) {
      const double gji = G[j * D + i];
      const float *ph = phi + j * m;
#pragma unroll
      for (int bb = 0; bb < M_MAX / 2; ++bb) {
        const int b = half + 2 * bb;
        if (b < m) acc[bb] += gji * (double)ph[b];
      }
    }
#pragma unroll
    for (int bb = 0; bb < M_MAX / 2; ++bb) {
      const int b = half + 2 * bb;
      if (b < m) TA[i * TP + b] = acc[bb];
    }
    __syncthreads();
    // S = Phi^T T, lower triangle
    for (int idx = tid; idx < m * m; idx += 256) {
      const int a = idx / m, b = idx - a * m;
      if (b > a) continue;
      double sum = 0.0;
      for (int i2 = 0; i2 < D; ++i2) sum += (double)phi[i2 * m + a] * TA[i2 * TP + b];
      S[a * SP + b] = sum;
    }
    __syncthreads();
    // the staging area now holds Phi in fp64 for the last step
    for (int idx = tid; idx < D * m; idx += 256) {
      const int i2 = idx / m, b = idx - i2 * m;
      TA[i2 * TP + b] = (double)phi[idx];
    }
  } else {
    for (int idx = tid; idx < m * m; idx += 256) {
      const int a = idx / m, b = idx - a * m;
      if (b <= a) S[a * SP + b] = G[a * D + b];
    }
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

  // W^T[j][ch] = sum_{q <= j} X[j][q] Phi[ch][q]; exact mode: W^T = X (lower triangular)
  uint16_t *wh = wt + (size_t)lhead * (W_TERMS * m * D);
  const int ch = tid & 127;
  for (int j = tid >> 7; j < m; j += 2) {
    double wv;
    if (SKETCHED) {
      wv = dinv[j] * TA[ch * TP + j];
      for (int q = 0; q < j; ++q) wv += S[q * SP + j] * TA[ch * TP + q];
    } else {
      wv = ch < j ? S[ch * SP + j] : (ch == j ? dinv[j] : 0.0);
    }
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

// ---- sketched mode, compile-time order M (k_s): the fast path ------------------------------
// Phases: T = G Phi (registers, Phi broadcast from LDS) -> S = Phi^T T (3x3 register blocks)
// -> Cholesky with one barrier per step (columns stay unscaled until the end)
// -> forward substitution L y = Phi[ch][:]^T with y in registers, one channel per thread.
template <int M>
__global__ __launch_bounds__(256) void solve_sketched_kernel(const SegTable T,
                                                             const float *__restrict__ phi,
                                                             float ridge_rel,
                                                             const double *__restrict__ g64,
                                                             uint16_t *__restrict__ wt,
                                                             int32_t *__restrict__ status) {
  constexpr int SP = M + 1, TP = M + 1, MB = M / 16, HB = M / 2;
  __shared__ double S[M * SP];
  __shared__ double TA[D * TP];
  __shared__ __attribute__((aligned(16))) float PH[D * M];
  __shared__ double piv_s[M];
  __shared__ double d0[M];
  __shared__ int flag;

  const int lhead = blockIdx.x;
  const Where w = locate_head(T, lhead);
  const Seg &sg = T.s[w.seg];
  const double *G = g64 + (size_t)lhead * (D * D);
  const int tid = threadIdx.x;
  if (tid == 0) flag = 0;
  for (int idx = tid; idx < D * M / 4; idx += 256)
    reinterpret_cast<float4 *>(PH)[idx] = reinterpret_cast<const float4 *>(phi)[idx];
  __syncthreads();

  {  // T = G Phi: thread (i, half) owns T[i][half*HB .. half*HB+HB)
    const int i = tid & 127;
    const int half = __builtin_amdgcn_readfirstlane(tid >> 7);
    double acc[HB];
#pragma unroll
    for (int bb = 0; bb < HB; ++bb) acc[bb] = 0.0;
    for (int j0 = 0; j0 < D; j0 += 8) {
      double g[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) g[u] = G[(j0 + u) * D + i];   // symmetric: column i as row reads
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float4 *pr = reinterpret_cast<const float4 *>(&PH[(j0 + u) * M + half * HB]);
#pragma unroll
        for (int q = 0; q < HB / 4; ++q) {
          const float4 f = pr[q];
          acc[4 * q + 0] += g[u] * (double)f.x;
          acc[4 * q + 1] += g[u] * (double)f.y;
          acc[4 * q + 2] += g[u] * (double)f.z;
          acc[4 * q + 3] += g[u] * (double)f.w;
        }
      }
    }
#pragma unroll
    for (int bb = 0; bb < HB; ++bb) TA[i * TP + half * HB + bb] = acc[bb];
  }
  __syncthreads();

  {  // S = Phi^T T, lower 16x16 block pairs; thread (ta, tb) owns an MB x MB register block
    const int ta = tid >> 4, tb = tid & 15;
    double acc[MB][MB];
#pragma unroll
    for (int x = 0; x < MB; ++x)
#pragma unroll
      for (int y = 0; y < MB; ++y) acc[x][y] = 0.0;
    for (int i = 0; i < D; ++i) {
      double pa[MB], tv[MB];
#pragma unroll
      for (int x = 0; x < MB; ++x) pa[x] = (double)PH[i * M + ta + 16 * x];
#pragma unroll
      for (int y = 0; y < MB; ++y) tv[y] = TA[i * TP + tb + 16 * y];
#pragma unroll
      for (int x = 0; x < MB; ++x)
#pragma unroll
        for (int y = 0; y <= x; ++y) acc[x][y] += pa[x] * tv[y];
    }
#pragma unroll
    for (int x = 0; x < MB; ++x)
#pragma unroll
      for (int y = 0; y <= x; ++y) S[(ta + 16 * x) * SP + tb + 16 * y] = acc[x][y];
  }
  __syncthreads();

  double tr = 0.0;
  for (int a = 0; a < M; ++a) tr += S[a * SP + a];
  const double rho = (double)ridge_rel * tr / (double)M;
  __syncthreads();
  if (tid < M) {
    const double v = S[tid * SP + tid] + rho;
    S[tid * SP + tid] = v;
    d0[tid] = v;
  }

  // Cholesky, one barrier per step: column k keeps the values L[i][k] * L[k][k] until the end
  const int tx = tid & 15, ty = tid >> 4;
  for (int k = 0; k < M; ++k) {
    __syncthreads();
    const double piv = S[k * SP + k];
    const bool ok = piv > PIVOT_REL * d0[k] && piv < 1.0e300;
    if (tid == 0) {
      piv_s[k] = ok ? piv : 0.0;
      if (!ok) flag = COMPACTOR_STATUS_PIVOT;
    }
    if (ok) {
      const double inv = 1.0 / piv;
      for (int i = k + 1 + ty; i < M; i += 16) {
        const double lik = S[i * SP + k] * inv;
        for (int j = k + 1 + tx; j <= i; j += 16) S[i * SP + j] -= lik * S[j * SP + k];
      }
    }
  }
  __syncthreads();
  // scale the columns: L[i][k] = S[i][k] / sqrt(piv_k); dropped columns become exact zeros
  for (int idx = tid; idx < M * M; idx += 256) {
    const int i = idx / M, k = idx - i * M;
    if (k < i) {
      const double pk = piv_s[k];
      S[i * SP + k] = pk > 0.0 ? S[i * SP + k] / sqrt(pk) : 0.0;
    }
  }
  __syncthreads();

  // W^T[:, ch] = L^{-1} Phi[ch, :]^T by forward substitution, one channel per thread
  if (tid < D) {
    const int ch = tid;
    double y[M];
#pragma unroll
    for (int j = 0; j < M; ++j) {
      double v = (double)PH[ch * M + j];
#pragma unroll
      for (int q = 0; q < j; ++q) v -= S[j * SP + q] * y[q];
      const double pj = piv_s[j];
      y[j] = pj > 0.0 ? v / sqrt(pj) : 0.0;
    }
    uint16_t *wh = wt + (size_t)lhead * (W_TERMS * M * D);
#pragma unroll
    for (int j = 0; j < M; ++j) {
      float x = (float)y[j];
#pragma unroll
      for (int t = 0; t < W_TERMS; ++t) {
        const uint16_t b = bf16_rne(x);
        wh[(t * M + j) * D + ch] = b;
        x -= bf16_to_f32(b);
      }
    }
  }
  if (tid == 0) status[sg.ghead0 + w.head] = flag;
}

hipError_t launch_solve(const SegTable &T, int ks, const float *phi, float ridge_rel,
                        const double *g64, uint16_t *wt, int32_t *status, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  const dim3 grid((unsigned)T.nheads), block(256);
  if (ks == 16) {
    hipLaunchKernelGGL((solve_sketched_kernel<16>), grid, block, 0, st, T, phi, ridge_rel, g64, wt, status);
  } else if (ks == 32) {
    hipLaunchKernelGGL((solve_sketched_kernel<32>), grid, block, 0, st, T, phi, ridge_rel, g64, wt, status);
  } else if (ks == 48) {
    hipLaunchKernelGGL((solve_sketched_kernel<48>), grid, block, 0, st, T, phi, ridge_rel, g64, wt, status);
  } else if (ks == 64) {
    hipLaunchKernelGGL((solve_sketched_kernel<64>), grid, block, 0, st, T, phi, ridge_rel, g64, wt, status);
  } else if (ks > 0) {
    hipLaunchKernelGGL((solve_kernel<64, true>), dim3((unsigned)T.nheads), dim3(256), 0, st, T, ks,
                       phi, ridge_rel, g64, wt, status);
  } else {
    hipLaunchKernelGGL((solve_kernel<128, false>), dim3((unsigned)T.nheads), dim3(256), 0, st, T,
                       D, phi, ridge_rel, g64, wt, status);
  }
  return hipGetLastError();
}

}  // namespace cmp
