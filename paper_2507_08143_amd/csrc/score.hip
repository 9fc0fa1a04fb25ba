// Per-row quadratic form (paper Algorithm 1 lines 5-6): o_i = || W^T k_i ||^2, the squared row
// norm of U~ = K_hat V~ Sigma~^{-1} written with the Cholesky factor instead of the SVD.
//
// The contraction runs over the channel axis, which is contiguous in memory, so a key row is an
// MFMA B operand as it stands (16 B per lane); W^T (k_s x 128, as bf16 planes) is staged once
// per workgroup in LDS and read as the A operand.  The output
// tile D[sketch row][token] leaves every lane with 4 sketch rows of one token: squares are
// summed in-lane and two cross-lane exchanges finish the row norm.
//
// W^T reaches the MFMA as a sum of bf16 planes (hi + lo = 16 mantissa bits with two planes):
// bf16 x bf16 products are exact in the fp32 accumulator, so the only rounding besides the
// accumulation itself is the 2^-17 relative error of the split.
#include <type_traits>

#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int WPITCH = 136;   // bf16 per LDS row of W^T and of staged key rows (272 B)

// LDS layout of the W^T planes.  Sketched mode: k_s full rows of 128 channels.  Exact mode
// (M = 128): W^T = L^{-1} is lower triangular, row j is zero beyond channel j, so rows are kept in
// four groups of 32 with 32, 64, 96 and 128 channels (a third less LDS, which is what lets two
// workgroups share a CU, and 20 of 32 channel blocks to multiply).  Each row carries 16 bytes of
// padding: consecutive rows are then 20, 36, 52 or 68 banks apart and the 16 rows an MFMA
// operand read touches fall on distinct banks.
template <int M>
struct WLayout {
  static constexpr int PLANE = M * WPITCH;                       // bf16 per plane
  static constexpr int BURST = SCORE_BURST;                      // scores that wait in LDS
  __device__ static __forceinline__ int row(int r) { return r * WPITCH; }
  __device__ static __forceinline__ int blocks(int /*jb*/) { return 4; }   // 32-channel blocks of a row
  static constexpr int CHUNKS = M * 16;                          // 16-byte pieces per plane
  __device__ static __forceinline__ void piece(int c, int &r, int &ch) { r = c >> 4; ch = c & 15; }
};
template <>
struct WLayout<128> {
  static constexpr int PLANE = 32 * (40 + 72 + 104 + 136);      // 11264 bf16
  static constexpr int BURST = SCORE_EXACT_BURST;
  __device__ static __forceinline__ int row(int r) {
    const int g = r >> 5;
    return 1280 * g + 512 * g * (g - 1) + (r & 31) * (40 + 32 * g);
  }
  __device__ static __forceinline__ int blocks(int jb) { return (jb >> 1) + 1; }
  static constexpr int CHUNKS = 32 * (4 + 8 + 12 + 16);          // 1280
  __device__ static __forceinline__ void piece(int c, int &r, int &ch) {
    if (c < 128)      { r = c >> 2;               ch = c & 3; }
    else if (c < 384) { r = 32 + ((c - 128) >> 3); ch = (c - 128) & 7; }
    else if (c < 768) { r = 64 + (c - 384) / 12;   ch = (c - 384) % 12; }
    else              { r = 96 + ((c - 768) >> 4); ch = (c - 768) & 15; }
  }
};

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A workgroup walks tokens_per_wg tokens of one head in steps of 128 (32 per wave, two 16-token
// sub-tiles).  Key rows arrive with fully coalesced streaming loads (a wave instruction covers
// four whole 256-byte rows), pass through a wave-private LDS buffer, and are read back in the
// MFMA B-operand arrangement; two steps of loads are in flight while a third is multiplied.
// The multiply loop needs no workgroup barrier: a wave only reads what it wrote itself.  The
// scores collect in LDS and leave in bursts of BURST tokens; a run may span several bursts (up to
// SCORE_MAX_RUN tokens), so that what a workgroup pays once (staging W^T, the histogram, filling
// and draining its load pipeline) is spread over more rows; the loads of the steps that follow a
// burst are already in flight while it is written.
template <int M>
__global__ __launch_bounds__(256, 2) void score_kernel(
    const SegTable T, const uint16_t *__restrict__ wt, float *__restrict__ scores,
    int32_t *__restrict__ status, int *__restrict__ hist1, double *__restrict__ ostat) {
  constexpr int NSUB = 2, WTOK = 16 * NSUB, STEP = 4 * WTOK;     // tokens per wave / per WG step
  constexpr int NLD = WTOK * 16 / 64;                            // 16-B loads per lane per step
  typedef WLayout<M> WL;
  __shared__ __attribute__((aligned(16))) uint16_t wl[W_TERMS * WL::PLANE];
  // a wave stages 16 tokens at a time (its 32 tokens of a step in two halves); measured, a third
  // workgroup per CU does not pay, the smaller staging buffer does on the long-context shapes
  __shared__ __attribute__((aligned(16))) uint16_t kl[4][16 * WPITCH];
  // first radix digit of the selection, tallied on the way out: two 16-bit counters per word
  __shared__ __attribute__((aligned(16))) unsigned hl[HIST1_BINS / 2];
  // The scores collect here and leave in bursts: 4-byte stores trickling out between the
  // streaming reads cost 12 % of the kernel's time.
  constexpr int BURST = WL::BURST, BSTEPS = BURST / STEP;
  static_assert((BURST & (BURST - 1)) == 0 && BSTEPS % 2 == 0, "bursts end on even steps");
  __shared__ __attribute__((aligned(16))) float sc_l[BURST];
  __shared__ double red[4][4];

  // Where this workgroup works.  Every wave does this scalar work before its first load can
  // leave, so the per-segment numbers come precomputed in the table (index_score_blocks) and
  // one division remains.
  Where w{0, 0, 0, 0, 0};
  for (int i = 1; i < T.nseg; ++i) w.seg += (int)blockIdx.x >= T.s[i].score_blk0;
  const Seg &s = T.s[w.seg];
  {
    const int local = (int)blockIdx.x - s.score_blk0;
    const int hh = (int)((unsigned)local / (unsigned)s.score_bph);
    w.head = s.head_begin + hh;
    w.lhead = s.lhead0 + hh;
    w.tile = local - hh * s.score_bph;
    w.chunk = s.score_chunk;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int t16 = lane & 15, g = lane >> 4;
  const int n = s.n;
  const int tok_begin = w.tile * w.chunk;
  const int tok_end = min(n, tok_begin + w.chunk);
  const int nsteps = (tok_end - tok_begin + STEP - 1) / STEP;
  const long long stride_t = s.stride_t;
  const uint16_t *kp = head_ptr(s.k_score, s, w.head);
  const int ld_row = lane >> 4, ld_chunk = lane & 15;            // loader: 16 lanes per row

  // this lane's piece of its first row; later rows are wave-uniform offsets away
  const uint16_t *lane_base =
      kp + (long long)(tok_begin + wave * WTOK + ld_row) * stride_t + ld_chunk * 8;
  const long long row4 = 4 * stride_t, step_stride = (long long)STEP * stride_t;
  auto load_step = [&](int it, uint4 (&stg)[NLD]) {
    const int base = tok_begin + it * STEP + wave * WTOK + ld_row;
    const uint16_t *p = lane_base + it * step_stride;
    // wave-uniform: all 32 rows of the wave exist (every step but a head's last)
    if (it < nsteps && tok_begin + it * STEP + (wave + 1) * WTOK <= tok_end) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) stg[i] = load_stream16(p + i * row4);
    } else {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int tok = base + 4 * i;
        stg[i] = make_uint4(0, 0, 0, 0);
        if (it < nsteps && tok < tok_end) stg[i] = load_stream16(p + i * row4);
      }
    }
  };

  uint4 stA[NLD], stB[NLD];
  load_step(0, stA);
  load_step(1, stB);
  // W^T follows the first two steps of keys through the load queue and waits in registers, so
  // that the third step of keys can be requested as soon as the first has arrived and not only
  // once W^T is in LDS: a workgroup starts with three steps in flight
  constexpr int WN = (W_TERMS * WL::CHUNKS + 255) / 256;
  uint4 wreg[WN];
  const uint16_t *wh = wt + (size_t)w.lhead * (W_TERMS * M * D);
#pragma unroll
  for (int i = 0; i < WN; ++i) {
    const int cidx = tid + 256 * i;
    wreg[i] = make_uint4(0, 0, 0, 0);
    if (cidx < W_TERMS * WL::CHUNKS) {
      const int t = cidx / WL::CHUNKS;
      int row, ch;
      WL::piece(cidx - t * WL::CHUNKS, row, ch);
      wreg[i] = *reinterpret_cast<const uint4 *>(wh + (t * M + row) * D + ch * 8);
    }
  }
  for (int i = tid; i < HIST1_BINS / 2; i += 256) hl[i] = 0;

  float *sp = scores + s.score_off + (long long)w.head * n;
  uint16_t *kw = kl[wave];
  bool bad = false;

  // In exact mode W^T is 128 rows and its operand reads from LDS weigh as much as the key
  // stream; there two steps are multiplied together, so that an operand of W^T read once serves
  // four MFMAs (a second set of key operands).
  constexpr bool PAIR = M == 128;
  bf16x8 kb[PAIR ? 2 : 1][NSUB][4];
  auto redistribute = [&](const uint4 (&stg)[NLD], int set = 0) {
    // redistribute through the wave's LDS buffer: rows in, B operands out.  Lanes exchange
    // data here without a workgroup barrier (LDS operations of one wave execute in order), so
    // wave-scope fences keep the compiler from moving the reads and writes across each other.
#pragma unroll
    for (int st = 0; st < NSUB; ++st) {
      wave_lds_fence();
#pragma unroll
      for (int i = 0; i < NLD / NSUB; ++i)
        *reinterpret_cast<uint4 *>(&kw[(ld_row + 4 * i) * WPITCH + ld_chunk * 8]) = stg[st * (NLD / NSUB) + i];
      wave_lds_fence();
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        kb[PAIR ? set : 0][st][kk] = *reinterpret_cast<const bf16x8 *>(&kw[t16 * WPITCH + 32 * kk + 8 * g]);
    }
  };
  // steps it .. it + NS - 1 (NS = 1, or 2 with both operand sets filled)
  auto multiply_steps = [&](auto ns, int it) {
    constexpr int NS = decltype(ns)::value;
    float sums[NS][NSUB];
#pragma unroll
    for (int p = 0; p < NS; ++p)
#pragma unroll
      for (int st = 0; st < NSUB; ++st) sums[p][st] = 0.f;
#pragma unroll 1
    for (int jb = 0; jb < M / 16; ++jb) {   // kept rolled: unrolling hoists every W^T operand
      f32x4 acc[NS][NSUB];
#pragma unroll
      for (int p = 0; p < NS; ++p)
#pragma unroll
        for (int st = 0; st < NSUB; ++st) acc[p][st] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int wrow = WL::row(jb * 16 + t16), nblk = WL::blocks(jb);    // nblk is wave-uniform
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kk < nblk) {
#pragma unroll
          for (int t = 0; t < W_TERMS; ++t) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&wl[t * WL::PLANE + wrow + 32 * kk + 8 * g]);
#pragma unroll
            for (int p = 0; p < NS; ++p)
#pragma unroll
              for (int st = 0; st < NSUB; ++st)
                acc[p][st] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, kb[p][st][kk], acc[p][st], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int p = 0; p < NS; ++p)
#pragma unroll
        for (int st = 0; st < NSUB; ++st)
          sums[p][st] += acc[p][st][0] * acc[p][st][0] + acc[p][st][1] * acc[p][st][1] +
                         acc[p][st][2] * acc[p][st][2] + acc[p][st][3] * acc[p][st][3];
    }
#pragma unroll
    for (int p = 0; p < NS; ++p) {
      // lanes (t16, g = 0..3) hold the four quarter-sums of token t16 of both sub-tiles; after
      // the exchange lanes with g < 2 hold the full sum of sub-tile g
      float x0 = sums[p][0] + __shfl_xor(sums[p][0], 32);
      float x1 = sums[p][1] + __shfl_xor(sums[p][1], 32);
      const bool up = g & 1;
      float x = up ? x1 : x0;
      x += __shfl_xor(up ? x0 : x1, 16);
      const int tok = tok_begin + (it + p) * STEP + wave * WTOK + (lane & 31);   // 16*(g&1) + t16
      if (g < 2 && tok < tok_end) {
        sc_l[(tok - tok_begin) & (BURST - 1)] = x;
        bad |= !(fabsf(x) <= 3.0e38f);
        const uint32_t bin = score_key(x) >> 20;
        atomicAdd(&hl[bin >> 1], 1u << (16 * (bin & 1)));
      }
    }
  };
  auto multiply = [&](int it) { multiply_steps(std::integral_constant<int, 1>{}, it); };

  // For the blend (a head whose request brings attention scores a): this thread's share of the
  // sums and sums of squares of the scores and of a over the workgroup's tokens.  a is shifted by
  // the head's first element so that a nearly constant vector does not cancel.
  const bool want_stat = ostat != nullptr && s.attn != nullptr;
  const float *ap = want_stat ? s.attn + (long long)w.head * n : nullptr;
  const double a_shift = want_stat ? (double)ap[0] : 0.0;
  double s1 = 0.0, s2 = 0.0, a1 = 0.0, a2 = 0.0;
  // The scores of tokens [b0, b0 + cnt) of the run leave as 16-byte streaming stores (they disturb
  // the other workgroups' reads least: 1 to 4 % of the kernel's time against plain stores); a
  // burst that does not start on a 16-byte boundary (odd n) gets up to 3 single stores in front.
  constexpr int APT = BURST / 256;          // a-values per thread and burst
  auto fetch_a = [&](int b0, int cnt, float (&av)[APT]) {
    const float *ab = ap + tok_begin + b0;
#pragma unroll
    for (int j = 0; j < APT; ++j) {
      const int i = tid + 256 * j;
      av[j] = (want_stat && i < cnt) ? ab[i] : 0.f;
    }
  };
  auto burst = [&](int b0, int cnt, const float (&av)[APT]) {
    float *dst = sp + tok_begin + b0;
    const int mis = (int)((reinterpret_cast<uintptr_t>(dst) >> 2) & 3u);
    const int lead = min(cnt, mis ? 4 - mis : 0);
    if (tid < lead) dst[tid] = sc_l[tid];
    if (lead == 0) {
      for (int i = 4 * tid; i + 3 < cnt; i += 4 * 256)
        store_stream16(dst + i, *reinterpret_cast<const uint4 *>(&sc_l[i]));
    } else {
      for (int i = lead + 4 * tid; i + 3 < cnt; i += 4 * 256)
        store_stream16(dst + i, make_uint4(__float_as_uint(sc_l[i]), __float_as_uint(sc_l[i + 1]),
                                           __float_as_uint(sc_l[i + 2]), __float_as_uint(sc_l[i + 3])));
    }
    for (int i = lead + ((cnt - lead) & ~3) + tid; i < cnt; i += 256) dst[i] = sc_l[i];
    if (want_stat) {
#pragma unroll
      for (int j = 0; j < APT; ++j) {
        const int i = tid + 256 * j;
        if (i < cnt) {
          const double x = (double)sc_l[i], y = (double)av[j] - a_shift;
          s1 += x;
          s2 += x * x;
          a1 += y;
          a2 += y * y;
        }
      }
    }
  };

  redistribute(stA);            // waits for the first step of keys only
  load_step(2, stA);
#pragma unroll
  for (int i = 0; i < WN; ++i) {
    const int cidx = tid + 256 * i;
    if (cidx < W_TERMS * WL::CHUNKS) {
      const int t = cidx / WL::CHUNKS;
      int row, ch;
      WL::piece(cidx - t * WL::CHUNKS, row, ch);
      *reinterpret_cast<uint4 *>(&wl[t * WL::PLANE + WL::row(row) + ch * 8]) = wreg[i];
    }
  }
  __syncthreads();

  // on entry of an iteration the operands of step `it` are in registers (kb) and the loads of
  // steps it + 1 (stB) and it + 2 (stA) are in flight
  for (int it = 0; it < nsteps; it += 2) {
    if (PAIR && it + 1 < nsteps) {
      redistribute(stB, 1);
      load_step(it + 3, stB);
      multiply_steps(std::integral_constant<int, PAIR ? 2 : 1>{}, it);
    } else {
      multiply(it);
      if (it + 1 < nsteps) {
        redistribute(stB);
        load_step(it + 3, stB);
        multiply(it + 1);
      }
    }
    const bool last = it + 2 >= nsteps;
    if (last || (it + 2) % BSTEPS == 0) {          // uniform: a burst is complete
      const int b0 = (it / BSTEPS) * BURST, cnt = min(BURST, tok_end - tok_begin - b0);
      float av[APT];
      fetch_a(b0, cnt, av);        // on their way while the waves meet
      __syncthreads();
      burst(b0, cnt, av);
      if (!last) __syncthreads();                   // before the next burst's scores overwrite these
    }
    if (!last) {
      redistribute(stA);
      load_step(it + 4, stA);
    }
  }
  if (__any(bad)) {
    if (lane == 0) atomicOr(&status[s.ghead0 + w.head], COMPACTOR_STATUS_NONFINITE);
  }
  if (want_stat) {
    // fixed order: lanes stride every burst, then a butterfly per wave, then the 4 waves
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      s1 += __shfl_xor(s1, d);
      s2 += __shfl_xor(s2, d);
      a1 += __shfl_xor(a1, d);
      a2 += __shfl_xor(a2, d);
    }
    if (lane == 0) { red[wave][0] = s1; red[wave][1] = s2; red[wave][2] = a1; red[wave][3] = a2; }
    __syncthreads();
    if (tid < 4)
      ostat[4 * (size_t)blockIdx.x + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  }
  // a head that will be blended gets its histogram from the blend, over the final scores
  if (hist1 != nullptr && s.attn == nullptr) {   // integer adds: order independent
    int *h1 = hist1 + (size_t)(w.lhead / pool_heads(T, s)) * HIST1_BINS;
    // 16 consecutive bins per thread, fetched with two LDS reads; few of them are occupied
    static_assert(HIST1_BINS == 16 * 256, "16 bins per thread");
    const uint4 ha = *reinterpret_cast<const uint4 *>(&hl[8 * tid]);
    const uint4 hb = *reinterpret_cast<const uint4 *>(&hl[8 * tid + 4]);
    const unsigned wd[8] = {ha.x, ha.y, ha.z, ha.w, hb.x, hb.y, hb.z, hb.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int lo = (int)(wd[j] & 0xffffu), hi = (int)(wd[j] >> 16);
      if (lo) atomicAdd(&h1[16 * tid + 2 * j], lo);
      if (hi) atomicAdd(&h1[16 * tid + 2 * j + 1], hi);
    }
  }
}

template <int M>
static hipError_t launch_m(const SegTable &T, int tokens_per_wg, const uint16_t *wt,
                           float *scores, int32_t *status, int *hist1, double *ostat,
                           hipStream_t st) {
  SegTable Ti = T;
  const long long nb = index_score_blocks(Ti, tokens_per_wg);
  if (nb <= 0) return hipSuccess;
  if (nb > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL((score_kernel<M>), dim3((unsigned)nb), dim3(256), 0, st, Ti, wt, scores, status,
                     hist1, ostat);
  return hipGetLastError();
}

hipError_t launch_score(const SegTable &T, int ks, int tokens_per_wg, const uint16_t *wt,
                        float *scores, int32_t *status, int *hist1, double *ostat, hipStream_t st) {
  switch (ks) {
    case 16: return launch_m<16>(T, tokens_per_wg, wt, scores, status, hist1, ostat, st);
    case 32: return launch_m<32>(T, tokens_per_wg, wt, scores, status, hist1, ostat, st);
    case 48: return launch_m<48>(T, tokens_per_wg, wt, scores, status, hist1, ostat, st);
    case 64: return launch_m<64>(T, tokens_per_wg, wt, scores, status, hist1, ostat, st);
    case 0:  return launch_m<128>(T, tokens_per_wg, wt, scores, status, hist1, ostat, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cmp
