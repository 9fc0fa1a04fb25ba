// Per-head top-k selection (paper Sec. 3.3: retain the top ceil(r N) tokens by score, within a
// single head) and the score blend of Eq. "scoring".
//
// Selection is an exact radix select on an order-preserving 32-bit key of the fp32 score
// (12 + 12 + 8 bits, LDS histograms), followed by an ordered emit: tokens above the threshold
// key, plus the lowest-indexed tokens equal to it until k_keep is reached, written in
// ascending token order.  Ties therefore go to the lower index, deterministically.
// One workgroup of 1024 threads per head; heads of up to 32768 tokens read their scores once
// and keep the keys in LDS (128 KB) for the later passes.
#include "common.h"

namespace cmp {

// Exclusive prefix sum of one int per thread over the 1024-thread workgroup; *total gets the
// workgroup sum.  wsum is 16 ints of LDS.
__device__ __forceinline__ int block_exclusive_scan(int v, int *wsum, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  __syncthreads();                       // wsum may still be read from a previous call
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < SELECT_THREADS / 64; ++i) {
    const int x = wsum[i];
    if (i < wave) base += x;
    tot += x;
  }
  *total = tot;
  return base + inc - v;
}

constexpr int LDS_KEYS = 32768;    // heads up to this many tokens keep their keys in LDS

// Finds, in a histogram of `nb` digits, the digit where the descending cumulative count reaches
// `need`; returns the digit and leaves in *need the count still wanted inside that digit.
__device__ __forceinline__ int find_digit(const int *hist, int nb, int *need, int *wsum, int *found) {
  const int tid = threadIdx.x;
  // thread t owns the 4 digits nb-1-4t .. nb-4-4t (descending), so that an ascending scan over
  // threads is a descending scan over digits
  int c[4], sum = 0;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int dgt = nb - 1 - (4 * tid + q);
    c[q] = dgt >= 0 ? hist[dgt] : 0;
    sum += c[q];
  }
  int total;
  int before = block_exclusive_scan(sum, wsum, &total);   // keys in higher digits
  const int want = *need;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (before < want && want <= before + c[q]) {          // exactly one (thread, q) matches
      found[0] = nb - 1 - (4 * tid + q);
      found[1] = want - before;
    }
    before += c[q];
  }
  __syncthreads();
  *need = found[1];
  return found[0];
}

// One radix pass: histogram `bits` bits at `shift` of the keys whose higher bits equal `prefix`
// (hi_shift = 32 means no prefix), then find_digit.  Keys come from LDS (FROM_LDS) or are
// recomputed from the scores in global memory; with STORE the keys are also parked in LDS.
template <bool FROM_LDS, bool STORE>
__device__ int radix_pass(const float *__restrict__ sp, uint32_t *keys, int n, int shift, int bits,
                          int hi_shift, uint32_t prefix, int *need, int *hist, int *wsum,
                          int *found) {
  const int nb = 1 << bits;
  const int tid = threadIdx.x;
  for (int i = tid; i < 4096; i += SELECT_THREADS) hist[i] = 0;
  __syncthreads();
  auto tally = [&](uint32_t k) {
    if (hi_shift >= 32 || (k >> hi_shift) == prefix) atomicAdd(&hist[(k >> shift) & (nb - 1)], 1);
  };
  // 16-byte accesses where the head's scores (or the LDS keys) allow it, scalars for the rest
  const bool vec = FROM_LDS || (reinterpret_cast<uintptr_t>(sp) & 15u) == 0;
  const int nv = vec ? n >> 2 : 0;
#pragma unroll 4
  for (int i = tid; i < nv; i += SELECT_THREADS) {
    uint4 k4;
    if (FROM_LDS) {
      k4 = reinterpret_cast<const uint4 *>(keys)[i];
    } else {
      const float4 f = reinterpret_cast<const float4 *>(sp)[i];
      k4 = make_uint4(score_key(f.x), score_key(f.y), score_key(f.z), score_key(f.w));
      if (STORE) reinterpret_cast<uint4 *>(keys)[i] = k4;
    }
    tally(k4.x); tally(k4.y); tally(k4.z); tally(k4.w);
  }
#pragma unroll 4
  for (int i = 4 * nv + tid; i < n; i += SELECT_THREADS) {
    const uint32_t k = FROM_LDS ? keys[i] : score_key(sp[i]);
    if (STORE) keys[i] = k;
    tally(k);
  }
  __syncthreads();
  return find_digit(hist, nb, need, wsum, found);
}

// Ordered emit: tokens above the threshold key, plus the first need_eq tokens equal to it, in
// ascending token order; 4 consecutive tokens per thread per round.
template <bool FROM_LDS>
__device__ void emit_kept(const float *__restrict__ sp, const uint32_t *keys, int n, int k,
                          uint32_t thr, int need_eq, int32_t *__restrict__ out, int *wsum) {
  const int tid = threadIdx.x;
  int carry_gt = 0, carry_eq = 0;
  for (int base = 0; base < n; base += 4 * SELECT_THREADS) {
    const int i0 = base + 4 * tid;
    uint32_t key[4];
    int gt = 0, eq = 0;
    if (FROM_LDS && i0 + 3 < n) {
      const uint4 kv = *reinterpret_cast<const uint4 *>(keys + i0);
      key[0] = kv.x; key[1] = kv.y; key[2] = kv.z; key[3] = kv.w;
    } else if (!FROM_LDS && i0 + 3 < n && (reinterpret_cast<uintptr_t>(sp) & 15u) == 0) {
      const float4 f = *reinterpret_cast<const float4 *>(sp + i0);
      key[0] = score_key(f.x); key[1] = score_key(f.y); key[2] = score_key(f.z); key[3] = score_key(f.w);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        key[q] = i0 + q < n ? (FROM_LDS ? keys[i0 + q] : score_key(sp[i0 + q])) : 0u;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (i0 + q < n) {
        gt += key[q] > thr;
        eq += key[q] == thr;
      }
    }
    int total;
    const int packed = block_exclusive_scan(gt | (eq << 16), wsum, &total);
    int pg = carry_gt + (packed & 0xffff), pe = carry_eq + (packed >> 16);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (i0 + q < n) {
        const bool is_gt = key[q] > thr, is_eq = key[q] == thr;
        const int pos = pg + min(pe, need_eq);
        if ((is_gt || (is_eq && pe < need_eq)) && pos < k) out[pos] = i0 + q;
        pg += is_gt;
        pe += is_eq;
      }
    }
    carry_gt += total & 0xffff;
    carry_eq += total >> 16;
  }
}

// Second radix pass for heads too long for LDS: histogram of key bits 19..8 among the keys whose
// top digit is d1, and at the same time those keys are compacted into LDS (wave ballot +
// one LDS atomic per wave) so that the last pass need not read global memory again.
__device__ int radix_pass2_collect(const float *__restrict__ sp, uint32_t *keys, int n, uint32_t d1,
                                   int *need, int *hist, int *wsum, int *found, int *ncand_s,
                                   int *ncand) {
  const int tid = threadIdx.x, lane = tid & 63;
  for (int i = tid; i < 4096; i += SELECT_THREADS) hist[i] = 0;
  if (tid == 0) *ncand_s = 0;
  __syncthreads();
  auto take = [&](uint32_t k, bool valid) {
    const bool c = valid && (k >> 20) == d1;
    const unsigned long long m = __ballot(c);
    if (m) {
      int base = 0;
      if (lane == __ffsll((long long)m) - 1) base = atomicAdd(ncand_s, __popcll(m));
      base = __shfl(base, __ffsll((long long)m) - 1);
      if (c) {
        atomicAdd(&hist[(k >> 8) & 0xfff], 1);
        const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
        if (pos < LDS_KEYS) keys[pos] = k;
      }
    }
  };
  const bool vec = (reinterpret_cast<uintptr_t>(sp) & 15u) == 0;
  const int nv = vec ? n >> 2 : 0;
  for (int i0 = 0; i0 < nv; i0 += SELECT_THREADS) {       // uniform trip count: ballots inside
    const int i = i0 + tid;
    float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < nv) f = reinterpret_cast<const float4 *>(sp)[i];
    take(score_key(f.x), i < nv); take(score_key(f.y), i < nv);
    take(score_key(f.z), i < nv); take(score_key(f.w), i < nv);
  }
  for (int i0 = 4 * nv; i0 < n; i0 += SELECT_THREADS) {
    const int i = i0 + tid;
    take(i < n ? score_key(sp[i]) : 0u, i < n);
  }
  __syncthreads();
  *ncand = *ncand_s;
  return find_digit(hist, 4096, need, wsum, found);
}

__global__ __launch_bounds__(SELECT_THREADS) void select_kernel(const SegTable T,
                                                                const float *__restrict__ scores,
                                                                const int *__restrict__ hist1,
                                                                int32_t *__restrict__ kept_idx,
                                                                int32_t *__restrict__ kept_cnt) {
  __shared__ __attribute__((aligned(16))) uint32_t keys[LDS_KEYS];
  __shared__ int hist[4096];
  __shared__ int wsum[SELECT_THREADS / 64];
  __shared__ int found[2];
  __shared__ int ncand_s;

  const Where w = locate_block(T, blockIdx.x, 0, 1, false);
  const Seg &s = T.s[w.seg];
  const int n = s.n, k = s.k_keep;
  const float *sp = scores + s.score_off + (long long)w.head * n;
  int32_t *out = kept_idx + (s.kept_off + (long long)w.head * k);
  const int tid = threadIdx.x;
  if (tid == 0) kept_cnt[s.ghead0 + w.head] = k;
  const bool small = n <= LDS_KEYS;      // one read of the scores; everything else out of LDS

  // threshold key = the k-th largest, by three radix passes (12 + 12 + 8 bits)
  int need = k;
  uint32_t d1, d2, d3;
  if (hist1 != nullptr) {                // first digit already tallied by the score kernel
    const int *h1 = hist1 + (size_t)w.lhead * HIST1_BINS;
    for (int i = tid; i < HIST1_BINS; i += SELECT_THREADS) hist[i] = h1[i];
    __syncthreads();
    d1 = find_digit(hist, HIST1_BINS, &need, wsum, found);
  } else if (small) {
    d1 = radix_pass<false, true>(sp, keys, n, 20, 12, 32, 0u, &need, hist, wsum, found);
  } else {
    d1 = radix_pass<false, false>(sp, keys, n, 20, 12, 32, 0u, &need, hist, wsum, found);
  }
  if (small) {
    if (hist1 != nullptr)
      d2 = radix_pass<false, true>(sp, keys, n, 8, 12, 20, d1, &need, hist, wsum, found);
    else
      d2 = radix_pass<true, false>(sp, keys, n, 8, 12, 20, d1, &need, hist, wsum, found);
    d3 = radix_pass<true, false>(sp, keys, n, 0, 8, 8, (d1 << 12) | d2, &need, hist, wsum, found);
    emit_kept<true>(sp, keys, n, k, (d1 << 20) | (d2 << 8) | d3, need, out, wsum);
  } else {
    int ncand;
    d2 = radix_pass2_collect(sp, keys, n, d1, &need, hist, wsum, found, &ncand_s, &ncand);
    if (ncand <= LDS_KEYS)               // the candidates (top digit d1) sit in LDS
      d3 = radix_pass<true, false>(sp, keys, ncand, 0, 8, 8, (d1 << 12) | d2, &need, hist, wsum, found);
    else
      d3 = radix_pass<false, false>(sp, keys, n, 0, 8, 8, (d1 << 12) | d2, &need, hist, wsum, found);
    emit_kept<false>(sp, keys, n, k, (d1 << 20) | (d2 << 8) | d3, need, out, wsum);
  }
}

// ---- blend: s = z(a) + lambda z(o), population standard deviation, fp64 statistics --------
__device__ __forceinline__ double block_sum(double v, double *wd) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  __syncthreads();
  if (lane == 0) wd[wave] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int i = 0; i < SELECT_THREADS / 64; ++i) t += wd[i];
  return t;
}

__global__ __launch_bounds__(SELECT_THREADS) void blend_kernel(const SegTable T, float lambda,
                                                               float *__restrict__ scores) {
  __shared__ double wd[SELECT_THREADS / 64];
  const Where w = locate_block(T, blockIdx.x, 0, 1, false);
  const Seg &s = T.s[w.seg];
  if (s.attn == nullptr) return;
  const int n = s.n, tid = threadIdx.x;
  float *o = scores + s.score_off + (long long)w.head * n;
  const float *a = s.attn + (long long)w.head * n;

  double so = 0.0, sa = 0.0;
  for (int i = tid; i < n; i += SELECT_THREADS) { so += o[i]; sa += a[i]; }
  const double mo = block_sum(so, wd) / n, ma = block_sum(sa, wd) / n;
  double vo = 0.0, va = 0.0;
  for (int i = tid; i < n; i += SELECT_THREADS) {
    const double x = o[i] - mo, y = a[i] - ma;
    vo += x * x;
    va += y * y;
  }
  const double sdo = sqrt(block_sum(vo, wd) / n), sda = sqrt(block_sum(va, wd) / n);
  // a constant vector (std 0) contributes nothing
  const double io = sdo > 0.0 ? (double)lambda / sdo : 0.0;
  const double ia = sda > 0.0 ? 1.0 / sda : 0.0;
  for (int i = tid; i < n; i += SELECT_THREADS)
    o[i] = (float)((a[i] - ma) * ia + (o[i] - mo) * io);
}

hipError_t launch_select(const SegTable &T, const float *scores, const int *hist1,
                         int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3((unsigned)T.nheads), dim3(SELECT_THREADS), 0, st, T,
                     scores, hist1, kept_idx, kept_cnt);
  return hipGetLastError();
}

hipError_t launch_blend(const SegTable &T, float lambda, float *scores, hipStream_t st) {
  bool any = false;
  for (int i = 0; i < T.nseg; ++i) any |= T.s[i].attn != nullptr;
  if (!any || T.nheads <= 0) return hipSuccess;
  hipLaunchKernelGGL(blend_kernel, dim3((unsigned)T.nheads), dim3(SELECT_THREADS), 0, st, T,
                     lambda, scores);
  return hipGetLastError();
}

}  // namespace cmp
