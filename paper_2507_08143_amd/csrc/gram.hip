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

// Persistent kernel: the launch's tiles are dealt out evenly, workgroup i takes tiles
// [i * tiles_per_wg, (i+1) * tiles_per_wg), crossing head boundaries where they fall.  Each
// (workgroup, head) intersection yields one partial Gram matrix, stored in slot
// workgroup + head (unique, because along the tile sequence workgroup and head only grow).
// All workgroups are resident at once and do the same amount of streaming, so there is no
// tail; the partials leave at the end of a workgroup's run where possible.
//
// The 10 upper blocks are split over the 4 waves of a workgroup (3, 3, 2, 2): every wave sees
// all tokens of the tile but owns its blocks outright, so no cross-wave reduction is needed and
// a wave carries at most 48 accumulator registers.
//   wave 0: (0,0) (0,1) (0,2)   wave 1: (0,3) (1,1) (1,2)   wave 2: (1,3) (2,2)   wave 3: (2,3) (3,3)
constexpr int GRAM_OCC = 2;         // waves per SIMD the register budget is set for
constexpr int GRAM_TG_UNROLL = 4;   // 16-token steps unrolled together (more operands in flight)
// The body is compiled once per wave of the workgroup: which blocks a wave owns is then known
// at compile time, and the accumulators stay in fixed registers (a run-time switch inside the
// loop makes the compiler copy them at every join).
template <int wave>
__device__ __forceinline__ void gram_body(const SegTable &T, int tiles_per_wg, long long total,
                                          float *__restrict__ partials, unsigned char *smem) {
  const long long g0 = (long long)blockIdx.x * tiles_per_wg;
  const int count = (int)min((long long)tiles_per_wg, total - g0);
  if (count <= 0) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int ld_row = tid >> 4, ld_chunk = tid & 15;   // loader: 16 lanes cover one 256-B row

  f32x16 acc[3];
#pragma unroll
  for (int b = 0; b < 3; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  TileCursor L, C;                 // load cursor runs two tiles ahead of the compute cursor
  cursor_seek<GRAM_TILE>(T, g0, L);
  C = L;

  auto load_tile = [&](int t, uint4 (&stage)[4]) {   // t: tile number inside this workgroup
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = L.tile * GRAM_TILE + 16 * i + ld_row;
      stage[i] = make_uint4(0, 0, 0, 0);
      if (t < count && row < L.n)
        stage[i] = load_stream16(L.kp + (long long)row * L.stride_t + ld_chunk * 8);
    }
    cursor_next<GRAM_TILE>(T, L);
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
      if constexpr (wave == 0) { GRAM_MFMA(0, 0, 0); GRAM_MFMA(1, 0, 1); GRAM_MFMA(2, 0, 2); }
      if constexpr (wave == 1) { GRAM_MFMA(0, 0, 3); GRAM_MFMA(1, 1, 1); GRAM_MFMA(2, 1, 2); }
      if constexpr (wave == 2) { GRAM_MFMA(0, 1, 3); GRAM_MFMA(1, 2, 2); }
      if constexpr (wave == 3) { GRAM_MFMA(0, 2, 3); GRAM_MFMA(1, 3, 3); }
    }
  };
#undef GRAM_MFMA
  auto store_tile = [&](unsigned char *buf, const uint4 (&stage)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<uint4 *>(buf + ((ld_row + 16 * i) * PITCH + ld_chunk * 8) * 2) = stage[i];
  };

  // Each wave writes the blocks it owns: a partial is the 10 upper blocks, each [32][32].
  // 32x32 accumulator layout: register v of lane l is element (8*(v>>2) + 4*(l>>5) + (v&3), l&31).
  const int nblk = wave < 2 ? 3 : 2;
  const int first = wave == 0 ? 0 : (wave == 1 ? 3 : (wave == 2 ? 6 : 8));
  // A block is stored in accumulator order: float4 number 64*q + lane of a block holds rows
  // 8q + 4*(lane>>5) .. +3 of column lane & 31, so a flush is 16-byte stores, 1 KB per wave
  // instruction (see partial_quad in common.h for the readers).
  // Writes in the middle of the read stream are costly on this memory system (a few tens of MB of
  // them slow a 2 GB read pass by 7 %), so a partial that is finished before the workgroup's run
  // ends is parked in LDS (each wave its own blocks, no barrier needed) and leaves with the last
  // one; only a workgroup that crosses more than one head boundary writes mid-run, with
  // streaming stores.
  float *park = reinterpret_cast<float *>(smem + 2 * TILE_BYTES);
  int parked_lhead = -1;
  enum { TO_GLOBAL, TO_GLOBAL_STREAM, TO_LDS };
  auto flush = [&](int lhead, int how) {
    float *out = how == TO_LDS ? park
                               : partials + ((size_t)blockIdx.x + lhead) * GRAM_PARTIAL_FLOATS;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      if (b < nblk) {
        float *ob = out + (first + b) * GBLK;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 v = make_float4(acc[b][4 * q], acc[b][4 * q + 1], acc[b][4 * q + 2], acc[b][4 * q + 3]);
          if (how == TO_GLOBAL_STREAM)
            store_stream16(ob + (64 * q + lane) * 4, make_uint4(__float_as_uint(v.x), __float_as_uint(v.y),
                                                                 __float_as_uint(v.z), __float_as_uint(v.w)));
          else
            *reinterpret_cast<float4 *>(ob + (64 * q + lane) * 4) = v;
          acc[b][4 * q] = acc[b][4 * q + 1] = acc[b][4 * q + 2] = acc[b][4 * q + 3] = 0.f;
        }
      }
    }
  };
  bool dirty = false;
  auto finish_tile = [&](bool last_of_run) {       // after a tile has been multiplied
    dirty = true;
    if (C.tile + 1 == C.tph) {
      const int lhead = T.s[C.seg].lhead0 + C.hh;
      if (last_of_run) {
        flush(lhead, TO_GLOBAL);
      } else if (parked_lhead < 0) {
        flush(lhead, TO_LDS);
        parked_lhead = lhead;
      } else {
        flush(lhead, TO_GLOBAL_STREAM);
      }
      dirty = false;
    }
    cursor_next<GRAM_TILE>(T, C);
  };

  // two tiles of global loads stay in flight while a third is being multiplied
  uint4 stA[4], stB[4];
  load_tile(0, stA);
  load_tile(1, stB);
  for (int t = 0; t < count; t += 2) {
    store_tile(smem, stA);
    __syncthreads();
    load_tile(t + 2, stA);
    compute_tile(smem);
    finish_tile(t + 1 == count);
    if (t + 1 < count) {
      store_tile(smem + TILE_BYTES, stB);
      __syncthreads();
      load_tile(t + 3, stB);
      compute_tile(smem + TILE_BYTES);
      finish_tile(t + 2 == count);
    }
  }
  if (dirty) flush(T.s[C.seg].lhead0 + C.hh, TO_GLOBAL);
  if (parked_lhead >= 0) {         // the parked partial: every lane copies what it wrote itself
    float *out = partials + ((size_t)blockIdx.x + parked_lhead) * GRAM_PARTIAL_FLOATS;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
      if (b < nblk) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int o = (first + b) * GBLK + (64 * q + lane) * 4;
          *reinterpret_cast<float4 *>(out + o) = *reinterpret_cast<const float4 *>(park + o);
        }
      }
    }
  }
}

__global__ __launch_bounds__(256, GRAM_OCC) void gram_kernel(const SegTable T, int tiles_per_wg,
                                                             long long total,
                                                             float *__restrict__ partials) {
  // two key tiles and room for one parked partial Gram matrix
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * TILE_BYTES + GRAM_PARTIAL_FLOATS * 4];
  // every wave passes the same workgroup barriers, each in its own copy of the loop
  switch (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) {
    case 0: gram_body<0>(T, tiles_per_wg, total, partials, smem); break;
    case 1: gram_body<1>(T, tiles_per_wg, total, partials, smem); break;
    case 2: gram_body<2>(T, tiles_per_wg, total, partials, smem); break;
    default: gram_body<3>(T, tiles_per_wg, total, partials, smem); break;
  }
}

hipError_t launch_gram(const SegTable &T, int nwg, int tiles_per_wg, float *partials,
                       hipStream_t st) {
  const long long total = total_tiles(T);
  if (total <= 0 || nwg <= 0) return hipSuccess;
  hipLaunchKernelGGL(gram_kernel, dim3((unsigned)nwg), dim3(256), 0, st, T, tiles_per_wg, total,
                     partials);
  return hipGetLastError();
}

}  // namespace cmp
