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

// Exclusive prefix sum of one int per thread over a workgroup of NT threads; *total gets the
// workgroup sum.  wsum is NT / 64 ints of LDS.
template <int NT = SELECT_THREADS>
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
  for (int i = 0; i < NT / 64; ++i) {
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
template <int NT = SELECT_THREADS>
__device__ __forceinline__ int find_digit(const int *hist, int nb, int *need, int *wsum, int *found) {
  constexpr int PER = 4096 / NT;     // digits per thread (nb <= 4096)
  const int tid = threadIdx.x;
  // thread t owns the PER digits nb-1-PER*t .. (descending), so that an ascending scan over
  // threads is a descending scan over digits
  int c[PER], sum = 0;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int dgt = nb - 1 - (PER * tid + q);
    c[q] = dgt >= 0 ? hist[dgt] : 0;
    sum += c[q];
  }
  int total;
  int before = block_exclusive_scan<NT>(sum, wsum, &total);   // keys in higher digits
  const int want = *need;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    if (before < want && want <= before + c[q]) {          // exactly one (thread, q) matches
      found[0] = nb - 1 - (PER * tid + q);
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
#pragma unroll 8        // a head of 32768 tokens: all of a thread's loads in flight at once
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
    // keys equal to the threshold are rare (one, unless scores tie): a wave whose 256 tokens of
    // this round hold none only has to place the keys above it
    bool any_eq = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) any_eq |= i0 + q < n && key[r][q] == thr;
    if (!__any(any_eq)) {
      const int base = pg + min(pe, need_eq);
#pragma unroll
      for (int q = 0, at = base; q < 4; ++q) {
        const bool is_gt = i0 + q < n && key[r][q] > thr;
        if (is_gt && at < k) stage[at] = i0 + q;
        at += is_gt;
      }
      continue;
    }
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
// emit as above, with the scores read twice in all.  A pool (head or layer) is cut into chunks of
// up to 8192 tokens of one head, one workgroup each; three launches:
//   cand   the first digit d1 of the threshold key comes from the pool's histogram of the top 12
//          key bits (made by the score kernel, the blend, or msel_hist1_kernel).  Keys above d1
//          are retained for sure and only counted; the keys inside d1 (the candidates: a few
//          percent of the pool unless the scores are heavily tied) leave their low 20 bits in a
//          per-chunk list
//   thr    one workgroup per pool finds the remaining 12 + 8 bits of the threshold among the
//          candidates and derives, chunk by chunk in (head, token) order, every chunk's output
//          position and its allowance of threshold ties
//   emit   ordered emit of every chunk
// Everything is integer work on exact counts, so the result does not depend on the order in which
// candidates are listed.  A chunk workgroup's chain (locate, load, classify, write) is latency
// bound, so the chunk kernels are small workgroups of 256 threads held to 64 registers: eight of
// them share a CU and overlap each other's waits (1024-thread workgroups on 32768-token chunks
// moved 2.4 TB/s).
constexpr int CHUNK_THREADS = 256;
constexpr int SEL_ROUNDS = SEL_CHUNK / (4 * CHUNK_THREADS);    // 4-token groups per thread
constexpr int SEL_STATE = 8;             // ints of state per pool:
enum { ST_D1 = 0, ST_NEED1, ST_THR, ST_TIES };
static_assert(SEL_ROUNDS >= 1 && SEL_ROUNDS <= 8, "one validity bit per token in 32 bits");

struct SelWhere {
  int seg;
  int head;        // l*H + h inside the request
  int lhead;       // launch-local head index
  int tile;        // chunk inside the head
  int pool;        // launch-local pool index
  int tok_begin, tok_end;
};
// Every wave of every chunk workgroup runs this, and it is scalar work that the waves of a CU
// queue up for: the per-segment numbers come precomputed in the table (index_chunks), so that
// one division remains.
__device__ __forceinline__ SelWhere sel_locate(const SegTable &T, int blk) {
  SelWhere q;
  int seg = 0;
  for (int i = 1; i < T.nseg; ++i) seg += blk >= T.s[i].sel_blk0;
  const Seg &s = T.s[seg];
  const int local = blk - s.sel_blk0;
  const int hh = (int)((unsigned)local / (unsigned)s.sel_bph);
  q.seg = seg;
  q.head = s.head_begin + hh;
  q.lhead = s.lhead0 + hh;
  q.tile = local - hh * s.sel_bph;
  q.pool = T.layer_scope ? s.pool0 + hh / s.H : s.pool0 + hh;
  q.tok_begin = q.tile * s.sel_chunk;
  q.tok_end = min(s.n, q.tok_begin + s.sel_chunk);
  return q;
}

// Position of a chunk's first token in the launch's token sequence (segments, heads and tokens in
// order): where its candidate list starts.
__device__ __forceinline__ long long chunk_token_base(const SegTable &T, const SelWhere &q) {
  const Seg &s = T.s[q.seg];
  return s.tok0 + (long long)(q.head - s.head_begin) * s.n + q.tok_begin;
}

// The scores of a chunk, 4 consecutive tokens per thread and round (token of f[r][e]:
// tok_begin + 4 * (r * CHUNK_THREADS + tid) + e); bit 4r+e of the result says that the token
// exists.  The loads are only issued here: whoever calls this first and converts to keys later
// has the latency of everything in between for free.
template <int R>
__device__ __forceinline__ unsigned load_scores_part(const float *__restrict__ sp, const SelWhere &q,
                                                     int r0, float (&f)[R][4]) {
  // one 16-byte load per 4 tokens also where a head's scores start off a 16-byte boundary (odd
  // n): global memory takes vector loads at any 4-byte address
  typedef float f32x4_any __attribute__((ext_vector_type(4), aligned(4)));
  unsigned valid = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i0 = q.tok_begin + 4 * ((r0 + r) * CHUNK_THREADS + (int)threadIdx.x);
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
  return valid;
}
__device__ __forceinline__ unsigned load_chunk_scores(const float *__restrict__ sp, const SelWhere &q,
                                                      float (&f)[SEL_ROUNDS][4]) {
  return load_scores_part<SEL_ROUNDS>(sp, q, 0, f);
}
__device__ __forceinline__ void scores_to_keys(const float (&f)[SEL_ROUNDS][4],
                                               uint32_t (&key)[SEL_ROUNDS][4]) {
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e) key[r][e] = score_key(f[r][e]);
}

// find_digit on the 4096-digit histogram of a pool in global memory (16-byte aligned), by a
// workgroup of CHUNK_THREADS.
__device__ __forceinline__ int find_digit_global(const int *__restrict__ g, int *need, int *wsum,
                                                 int *found) {
  constexpr int NB = 4096, PER = NB / CHUNK_THREADS;
  const int t0 = PER * threadIdx.x;      // digits NB-1-t0 .. NB-PER-t0, descending
  int c[PER], sum = 0;
#pragma unroll
  for (int u = 0; u < PER / 4; ++u) {
    const int4 v = *reinterpret_cast<const int4 *>(g + NB - 4 - t0 - 4 * u);
    c[4 * u] = v.w; c[4 * u + 1] = v.z; c[4 * u + 2] = v.y; c[4 * u + 3] = v.x;
    sum += v.x + v.y + v.z + v.w;
  }
  int total;
  int before = block_exclusive_scan<CHUNK_THREADS>(sum, wsum, &total);
  const int want = *need;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    if (before < want && want <= before + c[q]) {
      found[0] = NB - 1 - (t0 + q);
      found[1] = want - before;
    }
    before += c[q];
  }
  __syncthreads();
  *need = found[1];
  return found[0];
}

template <int NT>
__device__ __forceinline__ void flush_hist(const int *hist, int nb, int *__restrict__ g) {
  for (int i = threadIdx.x; i < nb; i += NT) {
    const int c = hist[i];
    if (c) atomicAdd(&g[i], c);
  }
}

// First digit, for scores that did not come with a histogram (hist1 zero on entry).
__global__ __launch_bounds__(CHUNK_THREADS, 8) void msel_hist1_kernel(const SegTable T,
                                                                    const float *__restrict__ scores,
                                                                    int *__restrict__ hist1) {
  __shared__ int hist[4096];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.seg];
  const float *sp = scores + s.score_off + (long long)q.head * s.n;
  float f[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_scores(sp, q, f);
  for (int i = threadIdx.x; i < 4096; i += CHUNK_THREADS) hist[i] = 0;
  __syncthreads();
  uint32_t key[SEL_ROUNDS][4];
  scores_to_keys(f, key);
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (valid >> (4 * r + e) & 1) atomicAdd(&hist[key[r][e] >> 20], 1);
  __syncthreads();
  flush_hist<CHUNK_THREADS>(hist, 4096, hist1 + (size_t)q.pool * 4096);
}

// Candidates of a chunk: counts the keys above the threshold's first digit and lists the low 20
// bits of the keys inside it (cand, at the chunk's position in the launch's token sequence, so a
// list can never outgrow its room).  rec[chunk] = (keys above, candidates listed).
__global__ __launch_bounds__(CHUNK_THREADS, 6) void msel_cand_kernel(const SegTable T,
                                                                  const float *__restrict__ scores,
                                                                  const int *__restrict__ hist1,
                                                                  uint32_t *__restrict__ cand,
                                                                  int *__restrict__ rec,
                                                                  int *__restrict__ state) {
  __shared__ int wsum[CHUNK_THREADS / 64];
  __shared__ int found[2];
  __shared__ int above_s, ncand_s;
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.seg];
  const float *sp = scores + s.score_off + (long long)q.head * s.n;
  float f[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_scores(sp, q, f);    // in flight while the digit is found
  if (threadIdx.x == 0) { above_s = 0; ncand_s = 0; }
  const int ph = pool_heads(T, s);
  int need = ph * s.k_keep;
  const uint32_t d1 = find_digit_global(hist1 + (size_t)q.pool * 4096, &need, wsum, found);
  if (q.tile == 0 && q.lhead % ph == 0 && threadIdx.x == 0) {   // the pool's first chunk
    state[q.pool * SEL_STATE + ST_D1] = (int)d1;
    state[q.pool * SEL_STATE + ST_NEED1] = need;
  }
  uint32_t *list = cand + chunk_token_base(T, q);
  uint32_t key[SEL_ROUNDS][4];
  scores_to_keys(f, key);
  const int lane = threadIdx.x & 63;
  // A thread's candidates go to consecutive slots: count, scan inside the wave, one LDS add per
  // wave for the wave's share of the list (the order in which waves claim theirs does not matter).
  int above = 0, mine = 0;
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool v = valid >> (4 * r + e) & 1;
      const uint32_t top = key[r][e] >> 20;
      above += (v && top > d1) ? 1 : 0;
      mine += (v && top == d1) ? 1 : 0;
    }
  int inc = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(inc, d);
    if (lane >= d) inc += o;
  }
  int base = 0;
  if (lane == 63 && inc) base = atomicAdd(&ncand_s, inc);
  int off = __shfl(base, 63) + inc - mine;
#pragma unroll
  for (int r = 0; r < SEL_ROUNDS; ++r)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if ((valid >> (4 * r + e) & 1) && (key[r][e] >> 20) == d1) list[off++] = key[r][e] & 0xfffffu;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) above += __shfl_xor(above, d);
  if (lane == 0 && above) atomicAdd(&above_s, above);
  __syncthreads();
  if (threadIdx.x == 0) {
    rec[2 * blockIdx.x] = above_s;
    rec[2 * blockIdx.x + 1] = ncand_s;
  }
}

// Visits the `cnt` values of a candidate list, f(value) for each: a wave's lanes take 4
// consecutive values each with one 16-byte load (at any 4-byte address), two loads in flight.
template <class F>
__device__ __forceinline__ void for_each_cand(const uint32_t *__restrict__ l, int cnt, int lane, F &&f) {
  typedef uint32_t u32x4_any __attribute__((ext_vector_type(4), aligned(4)));
  for (int i = 4 * lane; i < cnt; i += 512) {
    uint32_t v[2][4];
    int have[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = i + 256 * h;
      have[h] = min(4, cnt - j);
      if (have[h] == 4) {
        const u32x4_any t = *reinterpret_cast<const u32x4_any *>(l + j);
        v[h][0] = t.x; v[h][1] = t.y; v[h][2] = t.z; v[h][3] = t.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[h][e] = e < have[h] ? l[j + e] : 0u;
      }
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (e < have[h]) f(v[h][e]);
  }
}

// One workgroup per pool: the threshold key from the pool's candidates, then for every chunk of
// the pool (in head, token order) the position of its first retained token in the pool's
// output and how many threshold ties it may keep; the per-head counts.
// Two passes over the candidates: (1) histogram of their bits 19..8 -> second digit d2;
// (2) per chunk the count above d2, a histogram of the low 8 bits of those inside d2, and those
// few themselves as (chunk, low byte) in a short LDS list, from which, once the last digit is
// known, every chunk's counts above and at the threshold follow.  If the list overflows (heavily
// tied scores) or the pool has more than THR_BLOCK chunks, a third pass counts instead.
// The chunks' records are fetched into LDS in blocks of THR_BLOCK (a load per chunk in turn
// would string their latencies together); inside a block a wave takes every fourth chunk.
constexpr int THR_THREADS = 256, THR_BLOCK = 512, THR_SHORT = 2048;
__global__ __launch_bounds__(THR_THREADS) void msel_thr_kernel(const SegTable T,
                                                               const uint32_t *__restrict__ cand,
                                                               const int *__restrict__ rec,
                                                               int *__restrict__ coff,
                                                               int *__restrict__ state,
                                                               int32_t *__restrict__ kept_cnt) {
  constexpr int NW = THR_THREADS / 64;
  __shared__ int hist[4096];
  __shared__ int wsum[NW];
  __shared__ int found[2];
  __shared__ int above_c[THR_BLOCK], cnt_c[THR_BLOCK], gt_c[THR_BLOCK], eq_c[THR_BLOCK];
  __shared__ uint32_t short_l[THR_SHORT];
  __shared__ int nshort;
  // locate the pool: segment, first head, first chunk, first token
  const int pool = blockIdx.x;
  int seg = 0;
  for (int i = 1; i < T.nseg; ++i) seg += pool >= T.s[i].pool0;
  const Seg &s = T.s[seg];
  const int ph = pool_heads(T, s);
  const int bph = s.sel_bph, csize = s.sel_chunk;
  const int head0 = s.head_begin + (pool - s.pool0) * ph;
  const int chunk0 = s.sel_blk0 + (pool - s.pool0) * ph * bph;
  const long long tok0 = s.tok0 + (long long)(pool - s.pool0) * ph * s.n;
  const int nchunks = ph * bph;
  const bool single = nchunks <= THR_BLOCK;      // all records fit LDS at once
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // candidate list of chunk c of the pool
  auto list_of = [&](int c) { return cand + tok0 + (long long)(c / bph) * s.n + (long long)(c % bph) * csize; };
  // records of the chunks [cb, cb + THR_BLOCK) into LDS
  auto fetch = [&](int cb) {
    __syncthreads();
    for (int u = tid; u < THR_BLOCK && cb + u < nchunks; u += THR_THREADS) {
      const int2 r = *reinterpret_cast<const int2 *>(rec + 2 * (chunk0 + cb + u));
      above_c[u] = r.x;
      cnt_c[u] = r.y;
    }
    __syncthreads();
  };

  const uint32_t d1 = (uint32_t)state[pool * SEL_STATE + ST_D1];
  int need = state[pool * SEL_STATE + ST_NEED1];

  // pass 1: bits 19..8 of every candidate
  for (int i = tid; i < 4096; i += THR_THREADS) hist[i] = 0;
  if (tid == 0) nshort = 0;
  for (int cb = 0; cb < nchunks; cb += THR_BLOCK) {
    fetch(cb);
    for (int u = wave; u < THR_BLOCK && cb + u < nchunks; u += NW)
      for_each_cand(list_of(cb + u), cnt_c[u], lane,
                    [&](uint32_t v) { atomicAdd(&hist[(v >> 8) & 0xfffu], 1); });
  }
  __syncthreads();
  const uint32_t d2 = (uint32_t)find_digit<THR_THREADS>(hist, 4096, &need, wsum, found);
  // pass 2: bits 7..0 of the candidates that share the second digit; per chunk those above it
  for (int i = tid; i < 256; i += THR_THREADS) hist[i] = 0;
  for (int cb = 0; cb < nchunks; cb += THR_BLOCK) {
    if (!single) fetch(cb); else __syncthreads();
    for (int u = wave; u < THR_BLOCK && cb + u < nchunks; u += NW) {
      int gt = 0;
      for_each_cand(list_of(cb + u), cnt_c[u], lane, [&](uint32_t v) {
        const uint32_t top = v >> 8;
        gt += top > d2;
        if (top == d2) {
          atomicAdd(&hist[v & 0xffu], 1);
          if (single) {
            const int at = atomicAdd(&nshort, 1);
            if (at < THR_SHORT) short_l[at] = ((uint32_t)u << 8) | (v & 0xffu);
          }
        }
      });
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) gt += __shfl_xor(gt, d);
      if (lane == 0) { gt_c[u] = gt; eq_c[u] = 0; }
    }
  }
  __syncthreads();
  const uint32_t d3 = (uint32_t)find_digit<THR_THREADS>(hist, 256, &need, wsum, found);
  const int tie_keep = need;             // keys equal to the threshold that are retained
  const uint32_t thr20 = (d2 << 8) | d3;
  if (tid == 0) {
    state[pool * SEL_STATE + ST_THR] = (int)((d1 << 20) | thr20);
    state[pool * SEL_STATE + ST_TIES] = tie_keep;
  }
  const bool from_short = single && nshort <= THR_SHORT;
  if (from_short) {                      // the chunks' counts at the last digit, from the short list
    for (int i = tid; i < nshort; i += THR_THREADS) {
      const uint32_t e = short_l[i];
      const uint32_t low = e & 0xffu;
      if (low > d3) atomicAdd(&gt_c[e >> 8], 1);
      else if (low == d3) atomicAdd(&eq_c[e >> 8], 1);
    }
  }

  // every chunk's output position and tie allowance: thread 0 runs the prefix over the chunks in
  // order, a block at a time
  int pos = 0, eq_before = 0, head_kept = 0;
  for (int cb = 0; cb < nchunks; cb += THR_BLOCK) {
    if (!from_short) {                   // pass 3: count against the full threshold
      if (!single) fetch(cb); else __syncthreads();
      for (int u = wave; u < THR_BLOCK && cb + u < nchunks; u += NW) {
        int gt = 0, eq = 0;
        for_each_cand(list_of(cb + u), cnt_c[u], lane, [&](uint32_t v) {
          gt += v > thr20;
          eq += v == thr20;
        });
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
          gt += __shfl_xor(gt, d);
          eq += __shfl_xor(eq, d);
        }
        if (lane == 0) { gt_c[u] = gt; eq_c[u] = eq; }
      }
    }
    __syncthreads();
    if (tid == 0) {
      for (int u = 0; u < THR_BLOCK && cb + u < nchunks; ++u) {
        const int cc = cb + u;
        const int allow = max(0, min(eq_c[u], tie_keep - eq_before));
        const int kept = above_c[u] + gt_c[u] + allow;
        *reinterpret_cast<int2 *>(coff + 2 * (chunk0 + cc)) = make_int2(pos, allow);
        pos += kept;
        eq_before += eq_c[u];
        head_kept += kept;
        if ((cc + 1) % bph == 0) {       // last chunk of a head
          kept_cnt[s.ghead0 + head0 + cc / bph] = T.layer_scope ? head_kept : s.k_keep;
          head_kept = 0;
        }
      }
    }
  }
}

// Ordered emit of one chunk.  Token order inside a chunk is (round, wave, lane, element), so a
// token's output position is the sum of four prefixes: rounds before it, waves before it in its
// round, lanes before it in its wave, elements before it in its lane.  The lane prefix is a
// wave scan, the other two come from one table of (round, wave) counts scanned once: two
// workgroup barriers in all.  Counts are packed as (above | equal << 16), at most 8192 each.
__global__ __launch_bounds__(CHUNK_THREADS, 6) void msel_emit_kernel(const SegTable T,
                                                                   const float *__restrict__ scores,
                                                                   const int *__restrict__ coff,
                                                                   const int *__restrict__ state,
                                                                   int32_t *__restrict__ kept_idx) {
  constexpr int NW = CHUNK_THREADS / 64;
  constexpr int EMIT_STAGE = 4096;
  __shared__ unsigned table[SEL_ROUNDS * NW];
  __shared__ unsigned total_s;
  __shared__ int stage[EMIT_STAGE];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.seg];
  const float *sp = scores + s.score_off + (long long)q.head * s.n;
  float f[SEL_ROUNDS][4];
  const unsigned valid = load_chunk_scores(sp, q, f);    // in flight with the three loads below
  const int ph = pool_heads(T, s);
  const int limit = ph * s.k_keep;                       // rows of the pool's output
  int32_t *out = kept_idx + (s.kept_off + (long long)(q.head / ph) * limit);
  const uint32_t thr = (uint32_t)state[q.pool * SEL_STATE + ST_THR];
  const int2 pa = *reinterpret_cast<const int2 *>(coff + 2 * blockIdx.x);
  const int pos0 = pa.x, allow = pa.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t key[SEL_ROUNDS][4];
  scores_to_keys(f, key);

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
    if (q.tok_begin + 4 * r * CHUNK_THREADS >= q.tok_end) break;       // uniform
    const unsigned p = table[r * NW + wave] + before[r];
    int pg = (int)(p & 0xffffu), pe = (int)(p >> 16);
    const int i0 = q.tok_begin + 4 * (r * CHUNK_THREADS + (int)threadIdx.x);
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
  for (int j = threadIdx.x; j < staged; j += CHUNK_THREADS) out[pos0 + j] = stage[j];
}

// ---- blend: s = z(a) + lambda z(o) (paper Eq. "scoring"), population standard deviation ------
// The sums that the two standardisations need are gathered on the way, in the score kernel's
// epilogue: per score workgroup the fp64 (sum, sum of squares) of its scores o and of the
// attention scores a of the same tokens, a shifted by the head's first element so that a nearly
// constant vector does not cancel (ostat, four doubles per workgroup).  blend_apply_kernel adds a
// head's pairs up in index order (every chunk of the head gets the same mean and deviation, bit
// for bit), rewrites the scores in place and tallies the first selection histogram.
// Mean and reciprocal deviation of a head's scores o and attention scores a from `count`
// quadruples (sum and sum of squares of o, then of a less `shift`), added in index order.
struct Moments { double mo, io, ma, ia; };
__device__ __forceinline__ Moments moments(const double *__restrict__ quads, int count, int n,
                                           double shift, double (*wd)[4]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  double v[4] = {0.0, 0.0, 0.0, 0.0};
  for (int i = threadIdx.x; i < count; i += CHUNK_THREADS) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] += quads[4 * i + c];
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] += __shfl_xor(v[c], d);
  }
  if (lane == 0) {
#pragma unroll
    for (int c = 0; c < 4; ++c) wd[wave][c] = v[c];
  }
  __syncthreads();
  double t[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < CHUNK_THREADS / 64; ++i) {
#pragma unroll
    for (int c = 0; c < 4; ++c) t[c] += wd[i][c];
  }
  Moments m;
  // a constant vector (deviation 0) contributes nothing
  const double mo = t[0] / n, ma = t[2] / n;
  double vo = t[1] / n - mo * mo, va = t[3] / n - ma * ma;
  m.mo = mo;
  m.io = vo > 0.0 ? 1.0 / sqrt(vo) : 0.0;
  m.ma = shift + ma;
  m.ia = va > 0.0 ? 1.0 / sqrt(va) : 0.0;
  return m;
}

// Where a segment's pairs start in ostat (its first score workgroup) and how many a head has.
struct OstatIndex {
  long long first[MAX_SEG];
  int per_head[MAX_SEG];
};
__global__ __launch_bounds__(CHUNK_THREADS) void blend_apply_kernel(
    const SegTable T, const OstatIndex X, float lambda, float *__restrict__ scores,
    const double *__restrict__ ostat, int *__restrict__ hist1) {
  __shared__ double wd[CHUNK_THREADS / 64][4];
  __shared__ int hist[HIST1_BINS];
  const SelWhere q = sel_locate(T, blockIdx.x);
  const Seg &s = T.s[q.seg];
  if (s.attn == nullptr) return;
  const int n = s.n, tid = threadIdx.x;
  float *o = scores + s.score_off + (long long)q.head * n;
  const float *a = s.attn + (long long)q.head * n;
  // where the head's sums start: its first score workgroup
  const int obph = X.per_head[q.seg];
  const long long ob = X.first[q.seg] + (long long)(q.head - s.head_begin) * obph;
  if (hist1 != nullptr)
    for (int i = tid; i < HIST1_BINS; i += CHUNK_THREADS) hist[i] = 0;
  const Moments M = moments(ostat + 4 * ob, obph, n, (double)a[0], wd);     // has a barrier
  const double mo = M.mo, ma = M.ma, ia = M.ia, io = M.io * (double)lambda;
  typedef float f32x4_any __attribute__((ext_vector_type(4), aligned(4)));
  // the chunk in parts of PART rounds: the fp64 arithmetic of a whole chunk at once would take
  // so many registers that only three workgroups fit a CU
  constexpr int PART = 4;
#pragma unroll 1
  for (int r0 = 0; r0 < SEL_ROUNDS; r0 += PART) {
    if (q.tok_begin + 4 * r0 * CHUNK_THREADS >= q.tok_end) break;       // uniform
    float fa[PART][4], fo[PART][4];
    const unsigned valid = load_scores_part<PART>(a, q, r0, fa);
    load_scores_part<PART>(o, q, r0, fo);
#pragma unroll
    for (int r = 0; r < PART; ++r) {
      const unsigned m = (valid >> (4 * r)) & 0xfu;
      if (m == 0) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = (float)(((double)fa[r][e] - ma) * ia + ((double)fo[r][e] - mo) * io);
        if (hist1 != nullptr && (m >> e & 1)) atomicAdd(&hist[score_key(v[e]) >> 20], 1);
      }
      const int i0 = q.tok_begin + 4 * ((r0 + r) * CHUNK_THREADS + tid);
      if (m == 0xfu) {
        f32x4_any t;
        t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        *reinterpret_cast<f32x4_any *>(o + i0) = t;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (m >> e & 1) o[i0 + e] = v[e];
      }
    }
  }
  if (hist1 != nullptr) {
    __syncthreads();
    flush_hist<CHUNK_THREADS>(hist, HIST1_BINS, hist1 + (size_t)q.pool * HIST1_BINS);
  }
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
  long long pools = 0, rows = 0;
  for (int i = 0; i < T.nseg; ++i) {
    pools += T.s[i].head_count / pool_heads(T, T.s[i]);
    rows += (long long)T.s[i].n * T.s[i].head_count;
  }
  z.pools = (int)pools;
  z.chunks = total_blocks(T, SEL_CHUNK, 4, false);
  z.cand_ints = rows;
  z.rec_ints = z.chunks * 2;
  z.coff_ints = z.chunks * 2;
  z.state_ints = pools * SEL_STATE;
  return z;
}

long long select_chunks(const SegTable &T) { return total_blocks(T, SEL_CHUNK, 4, false); }

hipError_t launch_select_pools(const SegTable &T, const float *scores, int *hist1, bool hist1_ready,
                               int *sel, int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  const SelectScratch z = select_scratch(T);
  if (z.chunks > 0x7fffffffll) return hipErrorInvalidValue;
  uint32_t *cand = reinterpret_cast<uint32_t *>(sel);
  int *rec = sel + z.cand_ints, *coff = rec + z.rec_ints, *state = coff + z.coff_ints;
  const unsigned nb = (unsigned)z.chunks;
  if (!hist1_ready) {
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, st, hist1,
                       (long long)z.pools * HIST1_BINS);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    hipLaunchKernelGGL(msel_hist1_kernel, dim3(nb), dim3(CHUNK_THREADS), 0, st, T, scores, hist1);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  hipLaunchKernelGGL(msel_cand_kernel, dim3(nb), dim3(CHUNK_THREADS), 0, st, T, scores, hist1, cand,
                     rec, state);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL(msel_thr_kernel, dim3((unsigned)z.pools), dim3(THR_THREADS), 0, st, T, cand,
                     rec, coff, state, kept_cnt);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  hipLaunchKernelGGL(msel_emit_kernel, dim3(nb), dim3(CHUNK_THREADS), 0, st, T, scores, coff,
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

bool blend_wanted(const SegTable &T) {
  for (int i = 0; i < T.nseg; ++i)
    if (T.s[i].attn != nullptr) return true;
  return false;
}

hipError_t launch_blend(const SegTable &T, float lambda, int score_tokens, float *scores,
                        const double *ostat, int *hist1, hipStream_t st) {
  if (!blend_wanted(T) || T.nheads <= 0) return hipSuccess;
  const long long nb = select_chunks(T);
  if (nb > 0x7fffffffll) return hipErrorInvalidValue;
  OstatIndex X;
  long long ob = 0;
  for (int i = 0; i < MAX_SEG; ++i) {
    X.first[i] = ob;
    X.per_head[i] = i < T.nseg ? blocks_per_head(T.s[i].n, score_tokens, SCORE_STEP) : 0;
    if (i < T.nseg) ob += (long long)X.per_head[i] * T.s[i].head_count;
  }
  hipLaunchKernelGGL(blend_apply_kernel, dim3((unsigned)nb), dim3(CHUNK_THREADS), 0, st, T, X, lambda,
                     scores, ostat, hist1);
  return hipGetLastError();
}

}  // namespace cmp
