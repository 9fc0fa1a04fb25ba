// Per-row quadratic form (paper Algorithm 1 lines 5-6): o_i = || W^T k_i ||^2, the squared row
// norm of U~ = K_hat V~ Sigma~^{-1} written with the Cholesky factor instead of the SVD.
//
// The contraction runs over the channel axis, which is contiguous in memory, so key rows go
// straight from global memory into MFMA B operands (16 B per lane); W^T (k_s x 128, three
// bf16 planes) is staged once per workgroup in LDS and read as the A operand.  The output
// tile D[sketch row][token] leaves every lane with 4 sketch rows of one token: squares are
// summed in-lane and two cross-lane exchanges finish the row norm.
#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int WPITCH = 136;   // bf16 per LDS row of W^T (272 B)

template <int M, int NSUB>
__global__ __launch_bounds__(256, 2) void score_kernel(const SegTable T,
                                                       const uint16_t *__restrict__ wt,
                                                       float *__restrict__ scores,
                                                       int32_t *__restrict__ status) {
  __shared__ __attribute__((aligned(16))) uint16_t wl[W_TERMS * M * WPITCH];
  constexpr int TOK_WG = 4 * 16 * NSUB;

  const Where w = locate_block(T, blockIdx.x, TOK_WG, false);
  const Seg &s = T.s[w.seg];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t16 = lane & 15, g = lane >> 4;
  const int n = s.n;
  const int tok0 = w.tile * TOK_WG + wave * (16 * NSUB);

  // key rows -> B operands (issued first so that they fly while W^T is staged)
  const uint16_t *kp = head_ptr(s.k_score, s, w.head);
  uint4 kb[NSUB][4];
#pragma unroll
  for (int st = 0; st < NSUB; ++st) {
    const int tok = tok0 + 16 * st + t16;
    const uint16_t *rp = kp + (long long)tok * s.stride_t + 8 * g;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      kb[st][kk] = make_uint4(0, 0, 0, 0);
      if (tok < n) kb[st][kk] = *reinterpret_cast<const uint4 *>(rp + 32 * kk);
    }
  }

  // W^T of this head -> LDS
  const uint16_t *wh = wt + (size_t)w.lhead * (W_TERMS * M * D);
  for (int cidx = tid; cidx < W_TERMS * M * 16; cidx += 256) {
    const int row = cidx >> 4, ch = cidx & 15;
    *reinterpret_cast<uint4 *>(&wl[row * WPITCH + ch * 8]) =
        *reinterpret_cast<const uint4 *>(wh + row * D + ch * 8);
  }
  __syncthreads();

  float sums[NSUB];
#pragma unroll
  for (int st = 0; st < NSUB; ++st) sums[st] = 0.f;

#pragma unroll
  for (int jb = 0; jb < M / 16; ++jb) {
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

  // lanes t16, t16+16, t16+32, t16+48 hold the four quarter-sums of token t16
  float *sp = scores + s.score_off + (long long)w.head * n;
  bool bad = false;
#pragma unroll
  for (int st = 0; st < NSUB; ++st) {
    float x = sums[st];
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    const int tok = tok0 + 16 * st + t16;
    if ((st & 3) == g && tok < n) {
      sp[tok] = x;
      bad |= !(fabsf(x) <= 3.0e38f);
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
  hipLaunchKernelGGL((score_kernel<M, SCORE_SUB>), dim3((unsigned)nb), dim3(256), 0, st, T, wt,
                     scores, status);
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
