// Gram contraction G_h = K_h^T K_h of every head's key matrix (paper Eq. "fast_svd": the
// d x d Gram matrix stands in for the N x d SVD; Algorithm 1 lines 2-3 in the order
// Phi^T (K^T K) Phi, so that one pass over K serves sketched and exact scoring alike and
// every bf16 x bf16 product is exact in the fp32 accumulator).
//
// The contraction runs over the token axis, so both MFMA operands are "channel x token"
// slices of the same key tile: a wave builds one operand per 32-channel block (LDS transpose
// reads) and uses it as A and as B.  G is symmetric: only the 10 upper 32x32 blocks are
// accumulated and stored.
#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16x4 __attribute__((address_space(3))) *lds_bf16x4_ptr;

constexpr int PITCH = 144;                 // bf16 per LDS row: 288 B keeps 16-B alignment and
                                           // shifts consecutive rows by 8 banks, so the 4 rows x
                                           // 32 B that a 16-lane transpose read touches do not
                                           // collide
constexpr int TILE_BYTES = GRAM_TILE * PITCH * 2;
constexpr int GBLK = 32 * 32;              // one 32x32 block of G

// LDS transpose read (ds_read_b64_tr_b16): within each group of 16 lanes, lane j receives
// element (j & 3) of the 8-byte words addressed by lanes (j >> 2), 4 + (j >> 2), 8 + (j >> 2),
// 12 + (j >> 2).  With lane i pointing at row (i >> 2), columns 4*(i & 3).. of a row-major
// tile, lane j ends up with column j of rows 0..3: a 4 x 16 transpose.
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char *p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p));
}

// The 10 upper blocks are split over the 4 waves of a workgroup (3, 3, 2, 2): every wave sees
// all tokens of the tile but owns its blocks outright, so no cross-wave reduction is needed and
// a wave carries at most 48 accumulator registers.
//   wave 0: (0,0) (0,1) (0,2)   wave 1: (0,3) (1,1) (1,2)   wave 2: (1,3) (2,2)   wave 3: (2,3) (3,3)
#ifndef GRAM_OCC
#define GRAM_OCC 3          // waves per SIMD the register budget is set for
#endif
#ifndef GRAM_TG_UNROLL
#define GRAM_TG_UNROLL 4    // 16-token steps unrolled together (more = more operands in flight)
#endif
__global__ __launch_bounds__(256, GRAM_OCC) void gram_kernel(const SegTable T, int rows_per_wg,
                                                      float *__restrict__ partials) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * TILE_BYTES];

  const Where w = locate_block(T, blockIdx.x, rows_per_wg, GRAM_TILE, false);
  const Seg &s = T.s[w.seg];
  const uint16_t *kp = head_ptr(s.k_score, s, w.head);
  const long long stride_t = s.stride_t;
  const int r0 = w.tile * w.chunk;
  const int r1 = min(s.n, r0 + w.chunk);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ld_row = tid >> 4, ld_chunk = tid & 15;   // loader: 16 lanes cover one 256-B row

  f32x16 acc[3];
#pragma unroll
  for (int b = 0; b < 3; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  const int ntiles = (r1 - r0 + GRAM_TILE - 1) / GRAM_TILE;
  const uint16_t *lp0 = kp + (long long)(r0 + ld_row) * stride_t + ld_chunk * 8;
  auto load_tile = [&](int t, uint4 (&stage)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int roff = t * GRAM_TILE + 16 * i;
      stage[i] = make_uint4(0, 0, 0, 0);
      if (t < ntiles && r0 + roff + ld_row < r1)
        stage[i] = load_stream16(lp0 + (long long)roff * stride_t);
    }
  };

  // transpose-read addressing of this lane (see lds_read_tr): 16-lane group = (channel half,
  // token group of 8); inside the group the lane points at token (lane>>2)&3, channels 4*(lane&3)
  const int c16 = lane & 15, half = (lane >> 4) & 1, g = lane >> 5;
  const int tr_off = ((8 * g + (c16 >> 2)) * PITCH + 16 * half + 4 * (c16 & 3)) * 2;

#define GRAM_MFMA(b, x, y) acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[x], op[y], acc[b], 0, 0, 0)
  auto compute_tile = [&](const unsigned char *buf) {
#pragma unroll GRAM_TG_UNROLL
    for (int tg = 0; tg < GRAM_TILE / 16; ++tg) {        // 16 tokens per MFMA step
      const unsigned char *p = buf + tr_off + tg * 16 * PITCH * 2;
      bf16x8 op[4];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const bf16x4 lo = lds_read_tr(p + cb * 64);                    // tokens 8g .. 8g+3
        const bf16x4 hi = lds_read_tr(p + cb * 64 + 4 * PITCH * 2);    // tokens 8g+4 .. 8g+7
        op[cb] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#if defined(GRAM_ABLATE) && GRAM_ABLATE >= 1
      {  // experiment: keep the LDS reads alive without MFMA
        union { bf16x8 v; float f[4]; } u0, u1, u2, u3;
        u0.v = op[0]; u1.v = op[1]; u2.v = op[2]; u3.v = op[3];
        acc[0][0] += u0.f[0] + u1.f[1] + u2.f[2] + u3.f[3];
        continue;
      }
#endif
      switch (wave) {
        case 0: GRAM_MFMA(0, 0, 0); GRAM_MFMA(1, 0, 1); GRAM_MFMA(2, 0, 2); break;
        case 1: GRAM_MFMA(0, 0, 3); GRAM_MFMA(1, 1, 1); GRAM_MFMA(2, 1, 2); break;
        case 2: GRAM_MFMA(0, 1, 3); GRAM_MFMA(1, 2, 2); break;
        default: GRAM_MFMA(0, 2, 3); GRAM_MFMA(1, 3, 3); break;
      }
    }
  };
#undef GRAM_MFMA
  auto store_tile = [&](unsigned char *buf, const uint4 (&stage)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4 *>(buf + ((ld_row + 16 * i) * PITCH + ld_chunk * 8) * 2) = stage[i];
  };

  // two tiles of global loads stay in flight while a third is being multiplied
  uint4 stA[4], stB[4];
  load_tile(0, stA);
  load_tile(1, stB);
#if defined(GRAM_ABLATE) && GRAM_ABLATE >= 3
  for (int t = 0; t < ntiles; t += 2) {   // experiment: global loads only
    acc[0][1] += __uint_as_float(stA[0].x ^ stA[1].y ^ stA[2].z ^ stA[3].w);
    load_tile(t + 2, stA);
    acc[0][2] += __uint_as_float(stB[0].x ^ stB[1].y ^ stB[2].z ^ stB[3].w);
    load_tile(t + 3, stB);
  }
  if (false)
#elif defined(GRAM_ABLATE) && GRAM_ABLATE == 2
  for (int t = 0; t < ntiles; t += 2) {   // experiment: loads + LDS writes + barriers
    store_tile(smem, stA);
    __syncthreads();
    load_tile(t + 2, stA);
    if (t + 1 < ntiles) {
      store_tile(smem + TILE_BYTES, stB);
      __syncthreads();
      load_tile(t + 3, stB);
    }
  }
  acc[0][3] += smem[tid];
  if (false)
#endif
  for (int t = 0; t < ntiles; t += 2) {
    store_tile(smem, stA);
    __syncthreads();
    load_tile(t + 2, stA);
    compute_tile(smem);
    if (t + 1 < ntiles) {
      store_tile(smem + TILE_BYTES, stB);
      __syncthreads();
      load_tile(t + 3, stB);
      compute_tile(smem + TILE_BYTES);
    }
  }

  // ---- each wave writes the blocks it owns: partial = 10 upper blocks, each [32][32] --------
  // 32x32 accumulator layout: register v of lane l is element (8*(v>>2) + 4*(l>>5) + (v&3), l&31).
  float *out = partials + (size_t)blockIdx.x * (10 * GBLK);
  const int nblk = wave < 2 ? 3 : 2;
  const int first = wave == 0 ? 0 : (wave == 1 ? 3 : (wave == 2 ? 6 : 8));
  // wave-local block b is upper block number first + b in the order listed above
  const int col = lane & 31, rsub = 4 * (lane >> 5);
#pragma unroll
  for (int b = 0; b < 3; ++b) {
    if (b < nblk) {
      float *ob = out + (first + b) * GBLK;
#pragma unroll
      for (int v = 0; v < 16; ++v) ob[(8 * (v >> 2) + rsub + (v & 3)) * 32 + col] = acc[b][v];
    }
  }
}

// Order in which the waves own the upper blocks, as (I, J) per stored block number.
__device__ __constant__ int kBlockI[10] = {0, 0, 0, 0, 1, 1, 1, 2, 2, 3};
__device__ __constant__ int kBlockJ[10] = {0, 1, 2, 3, 1, 2, 3, 2, 3, 3};

// G64 = sum of a head's partials in fp64, in split order (deterministic), written as the full
// symmetric 128 x 128 matrix: one workgroup per (head, upper block), the mirror image goes
// through an LDS transpose so that both stores are coalesced.
__global__ __launch_bounds__(256) void gram_reduce_kernel(const SegTable T, int rows_per_wg,
                                                          const float *__restrict__ partials,
                                                          double *__restrict__ g64) {
  __shared__ double tile[32][33];
  const int lhead = blockIdx.x / 10;
  const int blk = blockIdx.x - lhead * 10;
  int nsplit;
  const long long pb = partial_base(T, lhead, rows_per_wg, nsplit);
  const int e = threadIdx.x * 4;                 // 4 consecutive elements of the block
  const int ii = e >> 5, jj = e & 31;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (int sidx = 0; sidx < nsplit; ++sidx) {
    const float4 p = *reinterpret_cast<const float4 *>(partials + (pb + sidx) * (10 * GBLK) +
                                                       blk * GBLK + e);
    a0 += p.x; a1 += p.y; a2 += p.z; a3 += p.w;
  }
  const int I = kBlockI[blk], J = kBlockJ[blk];
  double *G = g64 + (size_t)lhead * (D * D);
  double *o = G + (32 * I + ii) * D + 32 * J + jj;
  o[0] = a0; o[1] = a1; o[2] = a2; o[3] = a3;
  if (I != J) {
    tile[ii][jj] = a0; tile[ii][jj + 1] = a1; tile[ii][jj + 2] = a2; tile[ii][jj + 3] = a3;
    __syncthreads();
    double *m = G + (32 * J + ii) * D + 32 * I + jj;      // element (jrow = ii, icol = jj..)
    m[0] = tile[jj][ii]; m[1] = tile[jj + 1][ii]; m[2] = tile[jj + 2][ii]; m[3] = tile[jj + 3][ii];
  }
}

hipError_t launch_gram(const SegTable &T, int rows_per_wg, float *partials, hipStream_t st) {
  const long long nb = total_blocks(T, rows_per_wg, GRAM_TILE, false);
  if (nb <= 0) return hipSuccess;
  hipLaunchKernelGGL(gram_kernel, dim3((unsigned)nb), dim3(256), 0, st, T, rows_per_wg, partials);
  return hipGetLastError();
}

hipError_t launch_gram_reduce(const SegTable &T, int rows_per_wg, const float *partials,
                              double *g64, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)T.nheads * 10), dim3(256), 0, st, T,
                     rows_per_wg, partials, g64);
  return hipGetLastError();
}

}  // namespace cmp
