// Gram contraction G_h = K_h^T K_h of every head's key matrix (paper Eq. "fast_svd": the
// d x d Gram matrix stands in for the N x d SVD; Algorithm 1 lines 2-3 in the order
// Phi^T (K^T K) Phi, so that one pass over K serves sketched and exact scoring alike and
// every bf16 x bf16 product is exact in the fp32 accumulator).
//
// The contraction runs over the token axis, so both MFMA operands are "channel x token"
// slices of the same key tile: a wave builds one 8-token operand per 32-channel block and uses
// it as A and as B.  G is symmetric: only the 10 upper 32x32 blocks are accumulated.
#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PITCH = 136;                 // bf16 per LDS row: 272 B keeps 16-B alignment and
                                           // puts rows 8 apart 32 banks apart
constexpr int TILE_BYTES = GRAM_TILE * PITCH * 2;
constexpr int RED_STRIDE = 65;             // floats per (block, register) line of the reduction
constexpr int RED_BYTES = 10 * 16 * RED_STRIDE * 4;
constexpr int GRAM_LDS = (2 * TILE_BYTES > RED_BYTES) ? 2 * TILE_BYTES : RED_BYTES;

__device__ __forceinline__ int upper_block(int I, int J) { return I * 4 - (I * (I - 1)) / 2 + (J - I); }

__global__ __launch_bounds__(256, 2) void gram_kernel(const SegTable T, int rows_per_wg,
                                                      float *__restrict__ partials) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[GRAM_LDS];

  const Where w = locate_block(T, blockIdx.x, rows_per_wg, false);
  const Seg &s = T.s[w.seg];
  const uint16_t *kp = head_ptr(s.k_score, s, w.head);
  const long long stride_t = s.stride_t;
  const int r0 = w.tile * rows_per_wg;
  const int r1 = min(s.n, r0 + rows_per_wg);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int ld_row = tid >> 4, ld_chunk = tid & 15;   // loader: 16 lanes cover one 256-B row

  f32x16 acc[10];
#pragma unroll
  for (int b = 0; b < 10; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  uint4 stage[4];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = r0 + t * GRAM_TILE + ld_row + 16 * i;
      stage[i] = make_uint4(0, 0, 0, 0);
      if (row < r1)
        stage[i] = *reinterpret_cast<const uint4 *>(kp + (long long)row * stride_t + ld_chunk * 8);
    }
  };

  const int ntiles = (r1 - r0 + GRAM_TILE - 1) / GRAM_TILE;
  if (ntiles > 0) load_tile(0);

  const int c = lane & 31, g = lane >> 5;
  for (int t = 0; t < ntiles; ++t) {
    unsigned char *buf = smem + (t & 1) * TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4 *>(buf + ((ld_row + 16 * i) * PITCH + ld_chunk * 8) * 2) = stage[i];
    __syncthreads();
    if (t + 1 < ntiles) load_tile(t + 1);

    // this wave's 16 tokens: lane (c, g) gathers tokens 8g..8g+7 of channel 32*cb + c
    const uint16_t *lp = reinterpret_cast<const uint16_t *>(buf) + (16 * wave + 8 * g) * PITCH + c;
    bf16x8 op[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
      union { uint32_t u[4]; bf16x8 v; } pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t lo = lp[(2 * e) * PITCH + 32 * cb];
        const uint32_t hi = lp[(2 * e + 1) * PITCH + 32 * cb];
        pk.u[e] = lo | (hi << 16);
      }
      op[cb] = pk.v;
    }
#pragma unroll
    for (int I = 0; I < 4; ++I)
#pragma unroll
      for (int J = I; J < 4; ++J) {
        const int b = upper_block(I, J);
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[I], op[J], acc[b], 0, 0, 0);
      }
  }

  // ---- sum the four waves' accumulators (fp32) through LDS, wave 0 collects -------------
  float *red = reinterpret_cast<float *>(smem);
  __syncthreads();
  for (int src = 1; src < 4; ++src) {
    if (wave == src) {
#pragma unroll
      for (int b = 0; b < 10; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(b * 16 + v) * RED_STRIDE + lane] = acc[b][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int b = 0; b < 10; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] += red[(b * 16 + v) * RED_STRIDE + lane];
    }
    __syncthreads();
  }
  if (wave == 0) {
#pragma unroll
    for (int b = 0; b < 10; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[(b * 16 + v) * RED_STRIDE + lane] = acc[b][v];
  }
  __syncthreads();

  // ---- write the full (mirrored) 128 x 128 partial, row-major, coalesced ---------------
  // 32x32 accumulator layout: element (ii, jj) sits in lane jj + 32*((ii>>2)&1),
  // register (ii>>3)*4 + (ii&3).
  float *out = partials + (size_t)blockIdx.x * (D * D);
  for (int idx = tid; idx < D * D; idx += 256) {
    const int i = idx >> 7, j = idx & 127;
    int I = i >> 5, J = j >> 5, ii = i & 31, jj = j & 31;
    if (I > J) { int t2 = I; I = J; J = t2; t2 = ii; ii = jj; jj = t2; }
    const int b = upper_block(I, J);
    const int ln = jj + 32 * ((ii >> 2) & 1);
    const int v = (ii >> 3) * 4 + (ii & 3);
    out[idx] = red[(b * 16 + v) * RED_STRIDE + ln];
  }
}

// First partial and number of row splits of launch-local head `lhead`.
__device__ __forceinline__ long long partial_base(const SegTable &T, int lhead, int rows_per_wg,
                                                  int &nsplit) {
  long long base = 0;
  for (int i = 0; i < T.nseg; ++i) {
    const int bph = blocks_per_head(T.s[i].n, rows_per_wg);
    const int hh = lhead - T.s[i].lhead0;
    if (hh < T.s[i].head_count || i == T.nseg - 1) {
      nsplit = bph;
      return base + (long long)hh * bph;
    }
    base += (long long)bph * T.s[i].head_count;
  }
  nsplit = 0;
  return 0;
}

// G64 = sum of a head's partials in fp64, in split order (deterministic).
__global__ __launch_bounds__(256) void gram_reduce_kernel(const SegTable T, int rows_per_wg,
                                                          const float *__restrict__ partials,
                                                          double *__restrict__ g64) {
  const int lhead = blockIdx.x >> 4;
  const int part = blockIdx.x & 15;
  int nsplit;
  const long long pb = partial_base(T, lhead, rows_per_wg, nsplit);
  const int e = (part * 256 + threadIdx.x) * 4;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (int sidx = 0; sidx < nsplit; ++sidx) {
    const float4 p = *reinterpret_cast<const float4 *>(partials + (pb + sidx) * (D * D) + e);
    a0 += p.x; a1 += p.y; a2 += p.z; a3 += p.w;
  }
  double *o = g64 + (size_t)lhead * (D * D) + e;
  o[0] = a0; o[1] = a1; o[2] = a2; o[3] = a3;
}

hipError_t launch_gram(const SegTable &T, int rows_per_wg, float *partials, hipStream_t st) {
  const long long nb = total_blocks(T, rows_per_wg, false);
  if (nb <= 0) return hipSuccess;
  hipLaunchKernelGGL(gram_kernel, dim3((unsigned)nb), dim3(256), 0, st, T, rows_per_wg, partials);
  return hipGetLastError();
}

hipError_t launch_gram_reduce(const SegTable &T, int rows_per_wg, const float *partials,
                              double *g64, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)T.nheads * 16), dim3(256), 0, st, T,
                     rows_per_wg, partials, g64);
  return hipGetLastError();
}

}  // namespace cmp
