// Per-row quadratic form (paper Algorithm 1 lines 5-6): o_i = || W^T k_i ||^2, the squared row
// norm of U~ = K_hat V~ Sigma~^{-1} written with the Cholesky factor instead of the SVD.
//
// The contraction runs over the channel axis, which is contiguous in memory, so key rows go
// straight from global memory into MFMA B operands (16 B per lane); W^T (k_s x 128, three
// bf16 planes) is staged once per workgroup in LDS and read as the A operand.  The output
// tile D[sketch row][token] leaves every lane with 4 sketch rows of one token: squares are
// summed in-lane and two cross-lane exchanges finish the row norm.
//
// W^T reaches the MFMA as a sum of bf16 planes (hi + lo = 16 mantissa bits with two planes):
// bf16 x bf16 products are exact in the fp32 accumulator, so the only rounding besides the
// accumulation itself is the 2^-17 relative error of the split.
#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int WPITCH = 136;   // bf16 per LDS row of W^T (272 B)

// A workgroup walks SCORE_TOKENS tokens of one head in steps of 256 (64 per wave, four 16-token
// sub-tiles); the next step's key rows are loaded while the current step is multiplied.
template <int M>
__global__ __launch_bounds__(256, 2) void score_kernel(const SegTable T,
                                                       const uint16_t *__restrict__ wt,
                                                       float *__restrict__ scores,
                                                       int32_t *__restrict__ status) {
  __shared__ __attribute__((aligned(16))) uint16_t wl[W_TERMS * M * WPITCH];
  constexpr int NSUB = 4, STEP = 4 * 16 * NSUB;

  const Where w = locate_block(T, blockIdx.x, SCORE_TOKENS, false);
  const Seg &s = T.s[w.seg];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t16 = lane & 15, g = lane >> 4;
  const int n = s.n;
  const int tok_begin = w.tile * SCORE_TOKENS;
  const int tok_end = min(n, tok_begin + SCORE_TOKENS);
  const int nsteps = (tok_end - tok_begin + STEP - 1) / STEP;
  const long long stride_t = s.stride_t;
  const uint16_t *kp = head_ptr(s.k_score, s, w.head) + 8 * g;

  // key rows -> MFMA B operands: lane (t16, g) takes channels 32*kk + 8*g .. +7 of token t16
  auto load_step = [&](int it, uint4 (&kb)[NSUB][4]) {
    const int base = tok_begin + it * STEP + wave * (16 * NSUB) + t16;
#pragma unroll
    for (int st = 0; st < NSUB; ++st) {
      const int tok = base + 16 * st;
      const uint16_t *rp = kp + (long long)tok * stride_t;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        kb[st][kk] = make_uint4(0, 0, 0, 0);
        if (it < nsteps && tok < tok_end) kb[st][kk] = load_stream16(rp + 32 * kk);
      }
    }
  };

  uint4 kbA[NSUB][4], kbB[NSUB][4];
  load_step(0, kbA);          // in flight while W^T is staged

  const uint16_t *wh = wt + (size_t)w.lhead * (W_TERMS * M * D);
  for (int cidx = tid; cidx < W_TERMS * M * 16; cidx += 256) {
    const int row = cidx >> 4, ch = cidx & 15;
    *reinterpret_cast<uint4 *>(&wl[row * WPITCH + ch * 8]) =
        *reinterpret_cast<const uint4 *>(wh + row * D + ch * 8);
  }
  __syncthreads();

  float *sp = scores + s.score_off + (long long)w.head * n;
  bool bad = false;

  auto compute_step = [&](int it, const uint4 (&kb)[NSUB][4]) {
    float sums[NSUB];
#pragma unroll
    for (int st = 0; st < NSUB; ++st) sums[st] = 0.f;
#pragma unroll 1
    for (int jb = 0; jb < M / 16; ++jb) {   // kept rolled: unrolling hoists every W^T operand
      f32x4 acc[NSUB];
#pragma unroll
      for (int st = 0; st < NSUB; ++st) acc[st] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int t = 0; t < W_TERMS; ++t) {
          const bf16x8 a = *reinterpret_cast<const bf16x8 *>(
              &wl[(t * M + jb * 16 + t16) * WPITCH + 32 * kk + 8 * g]);
#pragma unroll
          for (int st = 0; st < NSUB; ++st) {
            union { uint4 u; bf16x8 v; } b;
            b.u = kb[st][kk];
            acc[st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b.v, acc[st], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int st = 0; st < NSUB; ++st)
        sums[st] += acc[st][0] * acc[st][0] + acc[st][1] * acc[st][1] + acc[st][2] * acc[st][2] +
                    acc[st][3] * acc[st][3];
    }
    // lanes (t16, g = 0..3) hold the four quarter-sums of token t16 of every sub-tile; a
    // two-step exchange leaves lane (t16, g) with the full sum of sub-tile g
    const bool up2 = g & 2, up1 = g & 1;
    float k0 = up2 ? sums[2] : sums[0], k1 = up2 ? sums[3] : sums[1];
    k0 += __shfl_xor(up2 ? sums[0] : sums[2], 32);
    k1 += __shfl_xor(up2 ? sums[1] : sums[3], 32);
    float x = up1 ? k1 : k0;
    x += __shfl_xor(up1 ? k0 : k1, 16);
    const int tok = tok_begin + it * STEP + wave * (16 * NSUB) + lane;   // = ... + 16*g + t16
    if (tok < tok_end) {
      sp[tok] = x;
      bad |= !(fabsf(x) <= 3.0e38f);
    }
  };

  for (int it = 0; it < nsteps; it += 2) {
    load_step(it + 1, kbB);
    compute_step(it, kbA);
    if (it + 1 < nsteps) {
      load_step(it + 2, kbA);
      compute_step(it + 1, kbB);
    }
  }
  if (__any(bad)) {
    if (lane == 0) atomicOr(&status[s.ghead0 + w.head], COMPACTOR_STATUS_NONFINITE);
  }
}

template <int M>
static hipError_t launch_m(const SegTable &T, const uint16_t *wt, float *scores, int32_t *status,
                           hipStream_t st) {
  const long long nb = total_blocks(T, SCORE_TOKENS, false);
  if (nb <= 0) return hipSuccess;
  hipLaunchKernelGGL((score_kernel<M>), dim3((unsigned)nb), dim3(256), 0, st, T, wt, scores,
                     status);
  return hipGetLastError();
}

hipError_t launch_score(const SegTable &T, int ks, const uint16_t *wt, float *scores,
                        int32_t *status, hipStream_t st) {
  switch (ks) {
    case 16: return launch_m<16>(T, wt, scores, status, st);
    case 32: return launch_m<32>(T, wt, scores, status, st);
    case 48: return launch_m<48>(T, wt, scores, status, st);
    case 64: return launch_m<64>(T, wt, scores, status, st);
    case 0:  return launch_m<128>(T, wt, scores, status, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cmp
