// Per-head top-k selection (paper Sec. 3.3: retain the top ceil(r N) tokens by score, within a
// single head) and the score blend of Eq. "scoring".
//
// Selection is an exact radix select on an order-preserving 32-bit key of the fp32 score
// (12 + 12 + 8 bits, LDS histograms), followed by an ordered emit: tokens above the threshold
// key, plus the lowest-indexed tokens equal to it until k_keep is reached, written in
// ascending token order.  Ties therefore go to the lower index, deterministically.
// Heads of up to 32768 tokens get one workgroup of 1024 threads each, which reads the scores
// once and keeps the keys in LDS (128 KB) for the later passes; longer heads, and selection
// across the heads of a layer, are shared by several workgroups (second half of this file).
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
  // 16-byte accesses: the LDS keys are aligned by token; scores in global memory are read from
  // the first 16-byte boundary on, the `lead` tokens in front of it (and the tail) one by one
  const int lead = FROM_LDS ? 0 : min(n, (int)((4u - ((reinterpret_cast<uintptr_t>(sp) >> 2) & 3u)) & 3u));
  const int nv = (n - lead) >> 2;
  if (tid < lead) {
    const uint32_t k = score_key(sp[tid]);
    if (STORE) keys[tid] = k;
    tally(k);
  }
#pragma unroll 4
  for (int i = tid; i < nv; i += SELECT_THREADS) {
    uint4 k4;
    if (FROM_LDS) {
      k4 = reinterpret_cast<const uint4 *>(keys)[i];
    } else {
      const float4 f = reinterpret_cast<const float4 *>(sp + lead)[i];
      k4 = make_uint4(score_key(f.x), score_key(f.y), score_key(f.z), score_key(f.w));
      if (STORE) {
        if (lead == 0) {
          reinterpret_cast<uint4 *>(keys)[i] = k4;
        } else {
          uint32_t *kd = keys + lead + 4 * i;
          kd[0] = k4.x; kd[1] = k4.y; kd[2] = k4.z; kd[3] = k4.w;
        }
      }
    }
    tally(k4.x); tally(k4.y); tally(k4.z); tally(k4.w);
  }
  for (int i = lead + 4 * nv + tid; i < n; i += SELECT_THREADS) {
    const uint32_t k = FROM_LDS ? keys[i] : score_key(sp[i]);
    if (STORE) keys[i] = k;
    tally(k);
  }
  __syncthreads();
  return find_digit(hist, nb, need, wsum, found);
}

// Ordered emit for keys resident in LDS (n <= LDS_KEYS).  Token order is (round, wave, lane,
// element) with 4096 tokens per round, so a token's output position is the sum of the counts of
// the rounds before it, of the waves before it in its round, of the lanes before it in its wave
// and of the elements before it in its lane: a wave scan per round plus one scan of the table of
// (round, wave) counts.  Counts are packed as (above | equal << 16), at most 32768 each.
// Every thread holds its keys in registers by then, so the key array is free to collect the
// retained token indices in order; they leave as one coalesced run.
__device__ void emit_kept_lds(uint32_t *keys, int n, int k, uint32_t thr, int need_eq,
                              int32_t *__restrict__ out, unsigned *table) {
  constexpr int NW = SELECT_THREADS / 64, R = LDS_KEYS / (4 * SELECT_THREADS);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t key[R][4];
  unsigned before[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i0 = 4 * (r * SELECT_THREADS + tid);
    if (4 * r * SELECT_THREADS >= n) {             // uniform: a round past the end of the head
      before[r] = 0;
      if (lane == 63) table[r * NW + wave] = 0;
      continue;
    }
    if (i0 + 3 < n) {
      const uint4 kv = *reinterpret_cast<const uint4 *>(keys + i0);
      key[r][0] = kv.x; key[r][1] = kv.y; key[r][2] = kv.z; key[r][3] = kv.w;
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) key[r][q] = i0 + q < n ? keys[i0 + q] : 0u;
    }
    unsigned mine = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool v = i0 + q < n;
      mine += (v && key[r][q] > thr) ? 1u : 0u;
      mine += (v && key[r][q] == thr) ? 0x10000u : 0u;
    }
    unsigned inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    before[r] = inc - mine;
    if (lane == 63) table[r * NW + wave] = inc;
  }
  __syncthreads();                   // all keys are in registers; the table is complete
  if (wave == 0) {                   // exclusive scan of the R * NW entries, 2 per lane
    constexpr int PER = (R * NW + 63) / 64;
    unsigned v[PER], sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = lane * PER + i;
      v[i] = idx < R * NW ? table[idx] : 0u;
      sum += v[i];
    }
    unsigned inc = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    unsigned run = inc - sum;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = lane * PER + i;
      if (idx < R * NW) table[idx] = run;
      run += v[i];
    }
  }
  __syncthreads();
  int32_t *stage = reinterpret_cast<int32_t *>(keys);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i0 = 4 * (r * SELECT_THREADS + tid);
    if (4 * r * SELECT_THREADS >= n) break;          // uniform
    const unsigned p = table[r * NW + wave] + before[r];
    int pg = (int)(p & 0xffffu), pe = (int)(p >> 16);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (i0 + q < n) {
        const bool is_gt = key[r][q] > thr, is_eq = key[r][q] == thr;
        const int pos = pg + min(pe, need_eq);
        if ((is_gt || (is_eq && pe < need_eq)) && pos < k) stage[pos] = i0 + q;
        pg += is_gt;
        pe += is_eq;
      }
    }
  }
  __syncthreads();
  for (int j = tid; j < k; j += SELECT_THREADS) out[j] = stage[j];
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

  const Where w = locate_block(T, blockIdx.x, 0, 1, false);
  const Seg &s = T.s[w.seg];
  const int n = s.n, k = s.k_keep;
  const float *sp = scores + s.score_off + (long long)w.head * n;
  int32_t *out = kept_idx + (s.kept_off + (long long)w.head * k);
  const int tid = threadIdx.x;
  if (tid == 0) kept_cnt[s.ghead0 + w.head] = k;
  // threshold key = the k-th largest, by three radix passes (12 + 12 + 8 bits); the scores are
  // read once and their keys stay in LDS for the later passes (n <= LDS_KEYS, checked on the host)
  int need = k;
  uint32_t d1, d2, d3;
  if (hist1 != nullptr) {                // first digit already tallied by the score kernel
    const int *h1 = hist1 + (size_t)w.lhead * HIST1_BINS;
    for (int i = tid; i < HIST1_BINS; i += SELECT_THREADS) hist[i] = h1[i];
    __syncthreads();
    d1 = find_digit(hist, HIST1_BINS, &need, wsum, found);
    d2 = radix_pass<false, true>(sp, keys, n, 8, 12, 20, d1, &need, hist, wsum, found);
  } else {
    d1 = radix_pass<false, true>(sp, keys, n, 20, 12, 32, 0u, &need, hist, wsum, found);
    d2 = radix_pass<true, false>(sp, keys, n, 8, 12, 20, d1, &need, hist, wsum, found);
  }
  d3 = radix_pass<true, false>(sp, keys, n, 0, 8, 8, (d1 << 12) | d2, &need, hist, wsum, found);
  emit_kept_lds(keys, n, k, (d1 << 20) | (d2 << 8) | d3, need, out, reinterpret_cast<unsigned *>(hist));
}

// ---- selection by several workgroups per pool ------------------------------------------------
// Used when a head is too long for one workgroup's LDS, and for head-adaptive selection, where
// the pool is the H kv heads of a layer that share one budget of H * k_keep tokens (paper Sec. 3.3:
// the top scores "across all heads"; scoring stays per head).  The same radix select and ordered
// emit as above, cut into chunks of a head (one workgroup each) that meet in per-pool
// histograms in global memory:
//   hist1  top 12 key bits (made by the score kernel, or by msel_hist1_kernel)
//   hist2  next 12 bits among the keys in the threshold's first digit
//   hist3  last 8 bits among the keys that share the threshold's top 24 bits; every chunk also
//          records its own share (and its count of keys above those 24 bits), from which one
//          workgroup per pool derives every chunk's output position and its allowance of
//          threshold ties, in (head, token) order
// The chunk kernels are held to 64 registers so that two 1024-thread workgroups share a CU.
// Four launches: hist2, hist3, scan, emit.  Each finds one digit of the threshold (every
// workgroup of a pool for itself, from a few KB in L2) and passes it on in the pool's state.
constexpr int SEL_CHUNK = 32768;         // tokens per workgroup (chunks never cross heads)
constexpr int SEL_ROUNDS = SEL_CHUNK / (4 * SELECT_THREADS);   // 4-token groups per thread
constexpr int SEL_REC = 260;             // ints per chunk record: [0] keys above the 24-bit
                                         // prefix, [4 + b] keys equal to it with low byte b
constexpr int SEL_STATE = 8;             // ints of state per pool:
enum { ST_D1 = 0, ST_NEED1, ST_D2, ST_NEED2, ST_THR, ST_TIES };
static_assert(SEL_ROUNDS >= 1 && SEL_ROUNDS <= 8, "one validity bit per token in 32 bits");

struct SelWhere {
  Where w;
  int pool;        // launch-local pool index
  int tok_begin, tok_end;
};
__device__ __forceinline__ SelWhere sel_locate(const SegTable &T, int blk) {
  SelWhere q;
  q.w = locate_block(T, blk, SEL_CHUNK, 4, false);
  const Seg &s = T.s[q.w.seg];
  q.pool = q.w.lhead / pool_heads(T, s);
  q.tok_begin = q.w.tile * q.w.chunk;
  q.tok_end = min(s.n, q.tok_begin + q.w.chunk);
  return q;
}

// The keys of a chunk, 4 consecutive tokens per thread and round (token of key[r][e]:
// tok_begin + 4 * (r * SELECT_THREADS + tid) + e); bit 4r+e of the result says that the token
// exists.  Every load is issued before any key is used.
__device__ __forceinline__ unsigned load_chunk_keys(const float *__restrict__ sp, const SelWhere &q,
                                                    uint32_t (&key)[SEL_ROUNDS][4]) {
  // one 16-byte load per 4 tokens also where a head's scores start off a 16-byte boundary (odd
  // n): global memory takes vector loads at any 4-byte address
  typedef float f32x4_any __attribute__((ext_vector_type(4), aligned(4)));
  float f[SEL_ROUNDS][4];
  unsigned valid = 0;
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r) {
    const int i0 = q.tok_begin + 4 * (r * SELECT_THREADS + (int)threadIdx.x);
    if (i0 + 3 < q.tok_end) {
      const f32x4_any v = *reinterpret_cast<const f32x4_any *>(sp + i0);
      f[r][0] = v.x; f[r][1] = v.y; f[r][2] = v.z; f[r][3] = v.w;
      valid |= 0xfu << (4 * r);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[r][e] = 0.f;
        if (i0 + e < q.tok_end) {
          f[r][e] = sp[i0 + e];
          valid |= 1u << (4 * r + e);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e) key[r][e] = score_key(f[r][e]);
  return valid;
}

// find_digit on a histogram in global memory (16-byte aligned, nb a multiple of 4).
__device__ __forceinline__ int find_digit_global(const int *__restrict__ g, int nb, int *need,
                                                 int *wsum, int *found) {
  const int t4 = 4 * threadIdx.x;
  int c[4] = {0, 0, 0, 0}, sum = 0;
  if (t4 < nb) {       // digits nb-1-t4 .. nb-4-t4, descending
    const int4 v = *reinterpret_cast<const int4 *>(g + nb - 4 - t4);
    c[0] = v.w; c[1] = v.z; c[2] = v.y; c[3] = v.x;
    sum = c[0] + c[1] + c[2] + c[3];
  }
  int total;
  int before = block_exclusive_scan(sum, wsum, &total);
  const int want = *need;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (before < want && want <= before + c[q]) {
      found[0] = nb - 1 - (t4 + q);
      found[1] = want - before;
    }
    before += c[q];
  }
  __syncthreads();
  *need = found[1];
  return found[0];
}

__device__ __forceinline__ void flush_hist(const int *hist, int nb, int *__restrict__ g) {
  for (int i = threadIdx.x; i < nb; i += SELECT_THREADS) {
    const int c = hist[i];
    if (c) atomicAdd(&g[i], c);
  }
}

// First digit, for scores that did not come with a histogram (hist1 zero on entry).
__global__ __launch_bounds__(SELECT_THREADS, 8) void msel_hist1_kernel(const SegTable T,
                                                                    const float *__restrict__ scores,
                                                                    int *__restrict__ hist1) {
  __shared__ int hist[4096];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.w.seg];
  const float *sp = scores + s.score_off + (long long)q.w.head * s.n;
  uint32_t key[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_keys(sp, q, key);
  for (int i = threadIdx.x; i < 4096; i += SELECT_THREADS) hist[i] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (valid >> (4 * r + e) & 1) atomicAdd(&hist[key[r][e] >> 20], 1);
  __syncthreads();
  flush_hist(hist, 4096, hist1 + (size_t)q.pool * 4096);
}

// Second digit (hist2 zero on entry).  The first chunk of a head also presets the head's count.
__global__ __launch_bounds__(SELECT_THREADS, 8) void msel_hist2_kernel(const SegTable T,
                                                                    const float *__restrict__ scores,
                                                                    const int *__restrict__ hist1,
                                                                    int *__restrict__ hist2,
                                                                    int *__restrict__ state,
                                                                    int32_t *__restrict__ kept_cnt) {
  __shared__ int hist[4096];
  __shared__ int wsum[SELECT_THREADS / 64];
  __shared__ int found[2];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.w.seg];
  const float *sp = scores + s.score_off + (long long)q.w.head * s.n;
  uint32_t key[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_keys(sp, q, key);
  for (int i = threadIdx.x; i < 4096; i += SELECT_THREADS) hist[i] = 0;
  const int ph = pool_heads(T, s);
  if (q.w.tile == 0 && threadIdx.x == 0)
    kept_cnt[s.ghead0 + q.w.head] = T.layer_scope ? 0 : s.k_keep;   // layer scope: summed later
  int need = ph * s.k_keep;
  const uint32_t d1 = find_digit_global(hist1 + (size_t)q.pool * 4096, 4096, &need, wsum, found);
  if (q.w.tile == 0 && q.w.lhead % ph == 0 && threadIdx.x == 0) {   // the pool's first chunk
    state[q.pool * SEL_STATE + ST_D1] = (int)d1;
    state[q.pool * SEL_STATE + ST_NEED1] = need;
  }
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid >> (4 * r + e) & 1) && (key[r][e] >> 20) == d1)
        atomicAdd(&hist[(key[r][e] >> 8) & 0xfff], 1);
  __syncthreads();
  flush_hist(hist, 4096, hist2 + (size_t)q.pool * 4096);
}

// Third digit (hist3 zero on entry) and the chunk records.
__global__ __launch_bounds__(SELECT_THREADS, 8) void msel_hist3_kernel(const SegTable T,
                                                                    const float *__restrict__ scores,
                                                                    const int *__restrict__ hist2,
                                                                    int *__restrict__ hist3,
                                                                    int *__restrict__ state,
                                                                    int *__restrict__ rec) {
  __shared__ int hist[256];
  __shared__ int wsum[SELECT_THREADS / 64];
  __shared__ int found[2];
  __shared__ int above_s;
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.w.seg];
  const float *sp = scores + s.score_off + (long long)q.w.head * s.n;
  uint32_t key[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_keys(sp, q, key);
  for (int i = threadIdx.x; i < 256; i += SELECT_THREADS) hist[i] = 0;
  if (threadIdx.x == 0) above_s = 0;
  const uint32_t d1 = (uint32_t)state[q.pool * SEL_STATE + ST_D1];
  int need = state[q.pool * SEL_STATE + ST_NEED1];
  const uint32_t d2 = find_digit_global(hist2 + (size_t)q.pool * 4096, 4096, &need, wsum, found);
  if (q.w.tile == 0 && q.w.lhead % pool_heads(T, s) == 0 && threadIdx.x == 0) {
    state[q.pool * SEL_STATE + ST_D2] = (int)d2;
    state[q.pool * SEL_STATE + ST_NEED2] = need;
  }
  const uint32_t prefix = (d1 << 12) | d2;
  int above = 0;
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (!(valid >> (4 * r + e) & 1)) continue;
      const uint32_t top = key[r][e] >> 8;
      above += top > prefix;
      if (top == prefix) atomicAdd(&hist[key[r][e] & 0xff], 1);
    }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) above += __shfl_xor(above, d);
  if ((threadIdx.x & 63) == 0 && above) atomicAdd(&above_s, above);
  __syncthreads();
  int *r = rec + (size_t)blockIdx.x * SEL_REC;
  if (threadIdx.x == 0) r[0] = above_s;
  for (int i = threadIdx.x; i < 256; i += SELECT_THREADS) r[4 + i] = hist[i];
  flush_hist(hist, 256, hist3 + (size_t)q.pool * 256);
}

// One workgroup per pool: the threshold key, and for every chunk of the pool (in head, token
// order) the position of its first retained token in the pool's output and how many
// threshold ties it may keep.
__global__ __launch_bounds__(SELECT_THREADS) void msel_scan_kernel(const SegTable T,
                                                                   const int *__restrict__ hist3,
                                                                   const int *__restrict__ rec,
                                                                   int *__restrict__ coff,
                                                                   int *__restrict__ state,
                                                                   int32_t *__restrict__ kept_cnt) {
  __shared__ int wsum[SELECT_THREADS / 64];
  __shared__ int found[2];
  __shared__ int gt_s[SELECT_THREADS], eq_s[SELECT_THREADS];
  // locate the pool: segment, first head, first chunk
  const int pool = blockIdx.x;
  int seg = 0, chunk0 = 0, head0 = 0;
  {
    int pbase = 0, cbase = 0;
    for (int i = 0; i < T.nseg; ++i) {
      const int ph = pool_heads(T, T.s[i]);
      const int np = T.s[i].head_count / ph;
      const int bph = blocks_per_head(T.s[i].n, SEL_CHUNK, 4);
      if (pool < pbase + np || i == T.nseg - 1) {
        seg = i;
        head0 = T.s[i].head_begin + (pool - pbase) * ph;
        chunk0 = cbase + (pool - pbase) * ph * bph;
        break;
      }
      pbase += np;
      cbase += bph * T.s[i].head_count;
    }
  }
  const Seg &s = T.s[seg];
  const int ph = pool_heads(T, s);
  const int bph = blocks_per_head(s.n, SEL_CHUNK, 4);
  const int nchunks = ph * bph;

  const uint32_t d1 = (uint32_t)state[pool * SEL_STATE + ST_D1];
  const uint32_t d2 = (uint32_t)state[pool * SEL_STATE + ST_D2];
  int need = state[pool * SEL_STATE + ST_NEED2];
  const int d3 = find_digit_global(hist3 + (size_t)pool * 256, 256, &need, wsum, found);
  const int tie_keep = need;             // keys equal to the threshold that are retained
  if (threadIdx.x == 0) {
    state[pool * SEL_STATE + ST_THR] = (int)((d1 << 20) | (d2 << 8) | (uint32_t)d3);
    state[pool * SEL_STATE + ST_TIES] = tie_keep;
  }

  int carry_kept = 0, carry_eq = 0;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int base = 0; base < nchunks; base += SELECT_THREADS) {
    // a wave per chunk record: keys above the threshold and equal to it
    __syncthreads();
    for (int c = base + wave; c < min(nchunks, base + SELECT_THREADS); c += SELECT_THREADS / 64) {
      const int *r = rec + (size_t)(chunk0 + c) * SEL_REC;
      const int4 v = *reinterpret_cast<const int4 *>(r + 4 + 4 * lane);
      const int b0 = 4 * lane;
      int g = (b0 > d3 ? v.x : 0) + (b0 + 1 > d3 ? v.y : 0) + (b0 + 2 > d3 ? v.z : 0) +
              (b0 + 3 > d3 ? v.w : 0);
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) g += __shfl_xor(g, d);
      if (lane == 0) {
        gt_s[c - base] = g + r[0];
        eq_s[c - base] = r[4 + d3];
      }
    }
    __syncthreads();
    const int c = base + threadIdx.x;
    const int gt = c < nchunks ? gt_s[threadIdx.x] : 0, eq = c < nchunks ? eq_s[threadIdx.x] : 0;
    int tot_eq, tot_kept;
    const int eq_before = carry_eq + block_exclusive_scan(eq, wsum, &tot_eq);
    const int allow = max(0, min(eq, tie_keep - eq_before));
    const int kept = gt + allow;
    const int pos = carry_kept + block_exclusive_scan(kept, wsum, &tot_kept);
    if (c < nchunks) {
      coff[2 * (chunk0 + c)] = pos;
      coff[2 * (chunk0 + c) + 1] = allow;
      if (T.layer_scope && kept) atomicAdd(&kept_cnt[s.ghead0 + head0 + c / bph], kept);
    }
    carry_eq += tot_eq;
    carry_kept += tot_kept;
  }
}

// Ordered emit of one chunk.  Token order inside a chunk is (round, wave, lane, element), so a
// token's output position is the sum of four prefixes: rounds before it, waves before it in its
// round, lanes before it in its wave, elements before it in its lane.  The lane prefix is a
// wave scan, the other two come from one table of (round, wave) counts scanned once: two
// workgroup barriers in all.  Counts are packed as (above | equal << 16), at most 32768 each.
__global__ __launch_bounds__(SELECT_THREADS, 8) void msel_emit_kernel(const SegTable T,
                                                                   const float *__restrict__ scores,
                                                                   const int *__restrict__ coff,
                                                                   const int *__restrict__ state,
                                                                   int32_t *__restrict__ kept_idx) {
  constexpr int NW = SELECT_THREADS / 64;
  constexpr int EMIT_STAGE = 16384;
  __shared__ unsigned table[SEL_ROUNDS * NW];
  __shared__ unsigned total_s;
  __shared__ int stage[EMIT_STAGE];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.w.seg];
  const float *sp = scores + s.score_off + (long long)q.w.head * s.n;
  uint32_t key[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_keys(sp, q, key);
  const int ph = pool_heads(T, s);
  const int limit = ph * s.k_keep;                       // rows of the pool's output
  int32_t *out = kept_idx + (s.kept_off + (long long)(q.w.head / ph) * limit);
  const uint32_t thr = (uint32_t)state[q.pool * SEL_STATE + ST_THR];
  const int pos0 = coff[2 * blockIdx.x], allow = coff[2 * blockIdx.x + 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  unsigned before[SEL_ROUNDS];      // packed counts of the lanes before this one, per round
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r) {
    unsigned mine = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool v = valid >> (4 * r + e) & 1;
      mine += (v && key[r][e] > thr) ? 1u : 0u;
      mine += (v && key[r][e] == thr) ? 0x10000u : 0u;
    }
    unsigned inc = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    before[r] = inc - mine;
    if (lane == 63) table[r * NW + wave] = inc;
  }
  __syncthreads();
  if (wave == 0) {                   // exclusive scan of the SEL_ROUNDS * NW entries
    constexpr int PER = (SEL_ROUNDS * NW + 63) / 64;
    unsigned v[PER], sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = lane * PER + i;
      v[i] = idx < SEL_ROUNDS * NW ? table[idx] : 0u;
      sum += v[i];
    }
    unsigned inc = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned o = __shfl_up(inc, d);
      if (lane >= d) inc += o;
    }
    unsigned run = inc - sum;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int idx = lane * PER + i;
      if (idx < SEL_ROUNDS * NW) table[idx] = run;
      run += v[i];
    }
    if (lane == 63) total_s = run;
  }
  __syncthreads();
  // the chunk's retained tokens are consecutive in the output: they are gathered in LDS and
  // written out as one run (what does not fit the stage goes straight to memory)
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r) {
    if (q.tok_begin + 4 * r * SELECT_THREADS >= q.tok_end) break;      // uniform
    const unsigned p = table[r * NW + wave] + before[r];
    int pg = (int)(p & 0xffffu), pe = (int)(p >> 16);
    const int i0 = q.tok_begin + 4 * (r * SELECT_THREADS + (int)threadIdx.x);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (valid >> (4 * r + e) & 1) {
        const bool is_gt = key[r][e] > thr, is_eq = key[r][e] == thr;
        if (is_gt || (is_eq && pe < allow)) {
          const int lp = pg + min(pe, allow);
          if (lp < EMIT_STAGE) stage[lp] = i0 + e;
          else if (pos0 + lp < limit) out[pos0 + lp] = i0 + e;
        }
        pg += is_gt;
        pe += is_eq;
      }
    }
  }
  __syncthreads();
  const int total = (int)(total_s & 0xffffu) + min((int)(total_s >> 16), allow);
  const int staged = min(min(total, EMIT_STAGE), limit - pos0);
  for (int j = threadIdx.x; j < staged; j += SELECT_THREADS) out[pos0 + j] = stage[j];
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

__global__ __launch_bounds__(256) void fill_zero_kernel(int *__restrict__ z, long long count) {
  zero_slice(z, count);
}

bool select_needs_pools(const SegTable &T) {
  if (T.layer_scope) return true;
  for (int i = 0; i < T.nseg; ++i)
    if (T.s[i].n > LDS_KEYS) return true;
  return false;
}

SelectScratch select_scratch(const SegTable &T) {
  SelectScratch z;
  long long pools = 0;
  for (int i = 0; i < T.nseg; ++i) pools += T.s[i].head_count / pool_heads(T, T.s[i]);
  z.pools = (int)pools;
  z.chunks = total_blocks(T, SEL_CHUNK, 4, false);
  z.hist2_ints = pools * 4096;
  z.hist3_ints = pools * 256;
  z.rec_ints = z.chunks * SEL_REC;
  z.coff_ints = z.chunks * 2;
  z.thr_ints = pools * SEL_STATE;
  return z;
}

hipError_t launch_select_pools(const SegTable &T, const float *scores, int *hist1, bool hist1_ready,
                               int *sel, bool zeroed, int32_t *kept_idx, int32_t *kept_cnt,
                               hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  const SelectScratch z = select_scratch(T);
  if (z.chunks > 0x7fffffffll) return hipErrorInvalidValue;
  int *hist2 = sel, *hist3 = hist2 + z.hist2_ints, *rec = hist3 + z.hist3_ints;
  int *coff = rec + z.rec_ints;
  int *state = coff + z.coff_ints;
  const unsigned nb = (unsigned)z.chunks;
  if (!zeroed) {       // hist1 .. hist3 are contiguous
    const long long cnt = (hist3 + z.hist3_ints) - hist1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, st, hist1, cnt);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  if (!hist1_ready) {
    hipLaunchKernelGGL(msel_hist1_kernel, dim3(nb), dim3(SELECT_THREADS), 0, st, T, scores, hist1);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  hipLaunchKernelGGL(msel_hist2_kernel, dim3(nb), dim3(SELECT_THREADS), 0, st, T, scores, hist1,
                     hist2, state, kept_cnt);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL(msel_hist3_kernel, dim3(nb), dim3(SELECT_THREADS), 0, st, T, scores, hist2,
                     hist3, state, rec);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL(msel_scan_kernel, dim3((unsigned)z.pools), dim3(SELECT_THREADS), 0, st, T,
                     hist3, rec, coff, state, kept_cnt);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL(msel_emit_kernel, dim3(nb), dim3(SELECT_THREADS), 0, st, T, scores, coff,
                     state, kept_idx);
  return hipGetLastError();
}

hipError_t launch_select(const SegTable &T, const float *scores, const int *hist1,
                         int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  if (select_needs_pools(T)) return hipErrorInvalidValue;     // longer heads: launch_select_pools
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
