// Internal declarations shared by the HIP translation units of libcompactor.
// Nothing here is part of the public boundary (see include/compactor.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "compactor.h"

namespace cmp {

constexpr int D = 128;            // head_dim, the only supported value
constexpr int MAX_SEG = 24;       // segments (request x head range) per launch
constexpr int KS_MAX = 128;       // largest factored order (exact mode)
constexpr int W_TERMS = 2;        // W^T is carried as a sum of this many bf16 planes:
                                  // 2 planes keep 16 mantissa bits (measured score error
                                  // <= 5e-5 relative against a 1e-3 bound), 3 planes all 24

// Launch-time tile sizes.
constexpr int GRAM_PARTIAL_FLOATS = 10 * 32 * 32;   // upper blocks of one partial Gram matrix
constexpr int GRAM_TILE = 64;         // rows staged in LDS per step of the Gram kernel
constexpr int SCORE_STEP = 128;       // tokens a score workgroup multiplies per step
constexpr int SCORE_BURST = 4096;     // scores a score workgroup collects in LDS before writing them
constexpr int SCORE_EXACT_BURST = 2048;   // the same in exact mode, where W^T takes more of the LDS
constexpr int SCORE_MAX_RUN = 32768;  // most tokens a score workgroup takes (its histogram counts in
                                      // 16 bits)
constexpr int SELECT_THREADS = 1024;
constexpr int SEL_CHUNK = 8192;       // tokens per workgroup of the chunked selection and blend
                                      // kernels (chunks never cross heads)
constexpr int GATHER_THREADS = 128;   // a gather workgroup: 8 groups of 16 lanes, one row each
constexpr int GATHER_ROWS = 16;       // kept rows per gather workgroup (2 per 16-lane group)

// One contiguous head range of one request, as seen by one launch.
struct Seg {
  const uint16_t *k_score;
  const uint16_t *k_cache;
  const uint16_t *v_cache;
  const float *attn;
  long long stride_l, stride_h, stride_t;  // elements
  long long score_off;   // float offset of this request's head (0,0) in the scores buffer
  long long kept_off;    // row offset of this request in kept_idx / packed buffers
  int n;                 // tokens
  int k_keep;            // retained tokens per head
  int head_begin;        // first head (l*H+h) of the request covered by this segment
  int head_count;        // heads covered
  int ghead0;            // global index of the request's head 0 (status / kept_cnt)
  int lhead0;            // launch-local index of this segment's first head (workspace arrays)
  int H;                 // kv heads per layer
  int req;               // index of the request in the call
  // Chunk enumeration of the selection and blend kernels, filled by index_chunks(): a workgroup
  // finds its place from these instead of redoing the divisions for every segment before it.
  int sel_blk0;          // number of the segment's first chunk in the launch
  int sel_bph;           // chunks per head
  int sel_chunk;         // tokens per chunk (the last chunk of a head may be shorter)
  int pool0;             // launch-local index of the segment's first selection pool
  long long tok0;        // position of the segment's first token in the launch's token sequence
  // The same for the score kernel's workgroups, filled by index_score_blocks() for the run
  // length of the launch.
  int score_blk0;        // number of the segment's first score workgroup in the launch
  int score_bph;         // score workgroups per head
  int score_chunk;       // tokens per score workgroup
};

struct SegTable {
  Seg s[MAX_SEG];
  int nseg;
  int nheads;            // launch-local heads in total
  int layer_scope;       // selection pool: 0 = one head, 1 = the kv heads of one layer (every
                         // segment then covers whole layers)
};

// Heads per selection pool of a segment.
__host__ __device__ __forceinline__ int pool_heads(const SegTable &T, const Seg &s) {
  return T.layer_scope ? s.H : 1;
}

// Where a workgroup works: segment, head inside the request, tile inside the head.
struct Where {
  int seg;
  int head;      // l*H + h inside the request
  int lhead;     // launch-local head index
  int tile;      // block index inside the head
  int chunk;     // units per block of this head: the block covers [tile*chunk, (tile+1)*chunk)
};

// Work of a head (n tokens, or k_keep kept rows) is cut into equal chunks: the caller names a
// target chunk size `per_block`; the head gets ceil(units / per_block) blocks and every block
// takes chunk_of(units, per_block, step) units (a multiple of `step`), so that the blocks of a
// head are as even as the step allows.  per_block <= 0 means one block per head.
__host__ __device__ __forceinline__ int chunk_of(int units, int per_block, int step) {
  if (per_block <= 0) return units > 0 ? units : 1;
  // 32-bit unsigned arithmetic (units < 2^31 - 64, per_block and step small): every workgroup
  // of a launch evaluates this once per segment
  const unsigned u = units > 0 ? (unsigned)units : 0u, pb = (unsigned)per_block, st = (unsigned)step;
  const unsigned splits = (u + pb - 1) / pb;
  const unsigned even = (u + splits - 1) / (splits > 0 ? splits : 1u);
  const unsigned c = (even + st - 1) / st * st;
  return (int)(c > 0 ? c : st);
}
__host__ __device__ __forceinline__ int blocks_per_head(int units, int per_block, int step) {
  if (per_block <= 0) return 1;
  const unsigned c = (unsigned)chunk_of(units, per_block, step);
  const unsigned u = units > 0 ? (unsigned)units : 0u;
  return (int)((u + c - 1) / c);
}

__device__ __forceinline__ Where locate_block(const SegTable &T, int blk, int per_block, int step,
                                              bool by_keep) {
  Where w{0, 0, 0, 0, 0};
  int base = 0;
  for (int i = 0; i < T.nseg; ++i) {
    const int units = by_keep ? T.s[i].k_keep : T.s[i].n;
    const int bph = blocks_per_head(units, per_block, step);
    const int nb = bph * T.s[i].head_count;
    if (blk < base + nb || i == T.nseg - 1) {
      const int local = blk - base;
      const int hh = local / bph;
      w.seg = i;
      w.chunk = chunk_of(units, per_block, step);
      w.head = T.s[i].head_begin + hh;
      w.lhead = T.s[i].lhead0 + hh;
      w.tile = local - hh * bph;
      return w;
    }
    base += nb;
  }
  return w;
}

// Order-preserving 32-bit key of an fp32 score: larger score <=> larger key.  NaN ranks below
// everything (key 0); -0.0 is folded onto +0.0 first.
__device__ __forceinline__ uint32_t score_key(float s) {
  s += 0.0f;
  if (s != s) return 0u;
  const uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
constexpr int HIST1_BINS = 4096;      // first radix digit of the selection: the top 12 key bits

// Streaming (non-temporal) 16-byte accesses for data that is touched once per pass: they do
// not allocate in the caches and sustain a higher HBM rate than ordinary loads (measured:
// about 7.1 TB/s against 6.2 TB/s for a plain slab read on MI355X).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void *p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void *p, const uint4 &v) {
  u32x4 t;
  t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4 *>(p));
}

// Clears z[0, count), the work split evenly over the workgroups of the launch (scratch that a
// later kernel of the same stream adds into).
__device__ __forceinline__ void zero_slice(int *__restrict__ z, long long count) {
  if (z == nullptr) return;
  const long long per = (count + gridDim.x - 1) / gridDim.x;
  const long long b = per * blockIdx.x, e = b + per < count ? b + per : count;
  for (long long i = b + threadIdx.x; i < e; i += blockDim.x) z[i] = 0;
}

__device__ __forceinline__ const uint16_t *head_ptr(const uint16_t *base, const Seg &s, int head) {
  const int l = head / s.H, h = head - l * s.H;
  return base + (long long)l * s.stride_l + (long long)h * s.stride_h;
}

// Inside a stored 32x32 block of a partial Gram matrix the elements are in MFMA accumulator
// order: float4 number f (0..255) holds rows row0 .. row0+3 of one column.
__host__ __device__ __forceinline__ void partial_quad(int f, int &row0, int &col) {
  row0 = 8 * (f >> 6) + 4 * ((f >> 5) & 1);
  col = f & 31;
}

// Stored order of the 10 upper 32x32 blocks of a partial Gram matrix.
__host__ __device__ __forceinline__ int upper_block(int I, int J) {
  return I * 4 - (I * (I - 1)) / 2 + (J - I);
}

// ---- persistent streaming kernels: tile cursors ----------------------------------------------
// The key rows of a launch form one sequence of TILE-row tiles, head after head (a head of n
// rows has ceil(n / TILE) tiles, the last one ragged).  A persistent kernel deals the sequence
// out evenly; a cursor tracks where in it a workgroup is.
struct TileCursor {
  int seg, hh, tile, tph, n;        // segment, head inside the segment, tile inside the head,
  long long stride_t;               // tiles per head, rows of the head
  const uint16_t *kp;               // first row of the head
};

template <int TILE>
__host__ __device__ __forceinline__ int tiles_in(int n) { return (n + TILE - 1) / TILE; }

template <int TILE>
inline long long total_tiles_of(const SegTable &T) {
  long long t = 0;
  for (int i = 0; i < T.nseg; ++i) t += (long long)tiles_in<TILE>(T.s[i].n) * T.s[i].head_count;
  return t;
}

template <int TILE>
__device__ __forceinline__ void cursor_head(const SegTable &T, TileCursor &c) {
  const Seg &s = T.s[c.seg];
  c.n = s.n;
  c.tph = tiles_in<TILE>(s.n);
  c.stride_t = s.stride_t;
  c.kp = head_ptr(s.k_score, s, s.head_begin + c.hh);
}

template <int TILE>
__device__ __forceinline__ void cursor_seek(const SegTable &T, long long g, TileCursor &c) {
  long long base = 0;
  c.seg = 0; c.hh = 0; c.tile = 0;
  for (int i = 0; i < T.nseg; ++i) {
    const int tph = tiles_in<TILE>(T.s[i].n);
    const long long cnt = (long long)tph * T.s[i].head_count;
    if (g < base + cnt || i == T.nseg - 1) {
      const long long local = g - base;
      c.seg = i;
      c.hh = (int)(local / tph);
      c.tile = (int)(local - (long long)c.hh * tph);
      break;
    }
    base += cnt;
  }
  cursor_head<TILE>(T, c);
}

// Moves to the next tile.  Past the last tile of the launch the cursor wraps inside the last
// segment; such positions are never loaded (the callers mask by tile count).
template <int TILE>
__device__ __forceinline__ void cursor_next(const SegTable &T, TileCursor &c) {
  if (++c.tile == c.tph) {
    c.tile = 0;
    if (++c.hh == T.s[c.seg].head_count) {
      c.hh = 0;
      if (c.seg + 1 < T.nseg) ++c.seg;
    }
    cursor_head<TILE>(T, c);
  }
}

// The Gram kernel numbers the launch's 64-row tiles head after head and deals them out evenly,
// tiles_per_wg to a workgroup; the partial of (workgroup i, head h) lives in slot i + h.
__host__ __device__ __forceinline__ int tiles_of(int n) { return (n + GRAM_TILE - 1) / GRAM_TILE; }

inline long long total_tiles(const SegTable &T) {
  long long t = 0;
  for (int i = 0; i < T.nseg; ++i) t += (long long)tiles_of(T.s[i].n) * T.s[i].head_count;
  return t;
}

// First partial slot of launch-local head `lhead` and the number of consecutive slots (one per
// workgroup that touched the head).
__device__ __forceinline__ long long partial_base(const SegTable &T, int lhead, int tiles_per_wg,
                                                  int &nsplit) {
  long long base = 0;
  for (int i = 0; i < T.nseg; ++i) {
    const int tph = tiles_of(T.s[i].n);
    const int hh = lhead - T.s[i].lhead0;
    if (hh < T.s[i].head_count || i == T.nseg - 1) {
      const long long t0 = base + (long long)hh * tph;        // first tile of the head
      const long long first = t0 / tiles_per_wg, last = (t0 + tph - 1) / tiles_per_wg;
      nsplit = (int)(last - first + 1);
      return first + lhead;
    }
    base += (long long)tph * T.s[i].head_count;
  }
  nsplit = 0;
  return 0;
}

// ---- host-side launchers (one per translation unit) -------------------------------------
// All of them enqueue on `st` and return the hipGetLastError() of their launches.

// Partial Gram matrices: the 10 upper 32x32 blocks (fp32) per (workgroup, head) intersection,
// nwg + nheads slots.
hipError_t launch_gram(const SegTable &T, int nwg, int tiles_per_wg, float *partials,
                       hipStream_t st);

// Exact mode: partial Gram blocks -> G + rho I -> Cholesky -> W^T = L^{-1} (as W_TERMS bf16
// planes, [term][128][128] per head) and the status word, in one kernel.
// zero[0, zero_ints) is cleared on the way (selection histograms), if not null.
hipError_t launch_exact_solve(const SegTable &T, int tiles_per_wg, const float *partials,
                              float ridge_rel, uint16_t *wt, int32_t *status, int *zero,
                              long long zero_ints, hipStream_t st);

// Sketched mode: partial Gram blocks -> S = Phi^T G Phi + rho I -> W^T ([term][k_s][128] per
// head) and status, in one kernel.
hipError_t launch_sketch_solve(const SegTable &T, int ks, int tiles_per_wg, const float *partials,
                               const float *phi, float ridge_rel, uint16_t *wt,
                               int32_t *status, int *zero, long long zero_ints, hipStream_t st);

// phi[128][ks] = sqrt(128/ks) * D H[cols]^T (signs, cols: host arrays, copied into the launch)
hipError_t launch_srht_phi(int ks, const uint8_t *signs, const int32_t *cols, float *phi,
                           hipStream_t st);

// scores[i] = || W^T k_i ||^2
// Also tallies the scores of heads that will not be blended into hist1[selection pool][HIST1_BINS]
// (top 12 key bits; the pool is the head, or the layer when T.layer_scope), which must be zero on
// entry; hist1 may be null.  ostat, if not null, receives four doubles per workgroup of the launch
// (for the blend): sum and sum of squares of its scores, and of the attention scores a of the same
// tokens (less the head's first element), for heads whose request has attn.
hipError_t launch_score(const SegTable &T, int ks, int tokens_per_wg, const uint16_t *wt,
                        float *scores, int32_t *status, int *hist1, double *ostat, hipStream_t st);

// s = z(a) + lambda z(o) in place over the scores of heads whose request has attn; their first
// selection histogram goes to hist1 (may be null).  score_tokens: the tokens_per_wg the score
// launch ran with (it decides which entries of ostat belong to a head).
bool blend_wanted(const SegTable &T);
long long select_chunks(const SegTable &T);
hipError_t launch_blend(const SegTable &T, float lambda, int score_tokens, float *scores,
                        const double *ostat, int *hist1, hipStream_t st);

// hist1: per-head histogram of the top 12 key bits made by the score kernel, or null.
hipError_t launch_select(const SegTable &T, const float *scores, const int *hist1,
                         int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st);

// Selection by several workgroups per pool (long heads, or layer scope).  hist1: pools x 4096
// ints; hist1_ready: it holds the histogram of the scores' top 12 key bits already (otherwise it
// is cleared and tallied here).  sel: scratch of select_scratch(T).ints() ints (candidate lists,
// one slot per token of the launch; per-chunk records and offsets; per-pool state), none of which
// needs clearing.
struct SelectScratch {
  int pools;
  long long chunks, cand_ints, rec_ints, coff_ints, state_ints;
  long long ints() const { return cand_ints + rec_ints + coff_ints + state_ints; }
};
SelectScratch select_scratch(const SegTable &T);
bool select_needs_pools(const SegTable &T);
hipError_t launch_select_pools(const SegTable &T, const float *scores, int *hist1, bool hist1_ready,
                               int *sel, int32_t *kept_idx, int32_t *kept_cnt, hipStream_t st);

// kept_cnt is read in layer scope only (ragged heads inside a layer's region).
hipError_t launch_gather(const SegTable &T, const int32_t *kept_idx, const int32_t *kept_cnt,
                         uint16_t *k_packed, uint16_t *v_packed, hipStream_t st);

// A paged destination (or source and destination) for the retained rows: a pool of fixed-size
// pages addressed through one block table per request.
struct PageTab {
  const int32_t *pages;   // physical page of each logical page of the segment's request
  int len, pad_;
};
struct PagePool {
  uint16_t *k, *v;
  long long page_stride, layer_stride, head_stride, slot_stride;   // elements
  int page_size, num_pages;
  PageTab t[MAX_SEG];     // by segment of the launch
};
// in_place: the rows are read from the pages themselves (token t at logical slot t).
hipError_t launch_gather_paged(const SegTable &T, const PagePool &P, const int32_t *kept_idx,
                               const int32_t *kept_cnt, bool in_place, hipStream_t st);

// Fills the chunk enumeration fields of every segment (host, after the table is otherwise
// complete).
inline void index_chunks(SegTable &T) {
  int blk = 0, pool = 0;
  long long tok = 0;
  for (int i = 0; i < T.nseg; ++i) {
    Seg &s = T.s[i];
    s.sel_blk0 = blk;
    s.sel_bph = blocks_per_head(s.n, SEL_CHUNK, 4);
    s.sel_chunk = chunk_of(s.n, SEL_CHUNK, 4);
    s.pool0 = pool;
    s.tok0 = tok;
    blk += s.sel_bph * s.head_count;
    pool += s.head_count / pool_heads(T, s);
    tok += (long long)s.n * s.head_count;
  }
}

// Fills the score kernel's enumeration fields for workgroups of about tokens_per_wg tokens;
// returns the number of workgroups.
inline long long index_score_blocks(SegTable &T, int tokens_per_wg) {
  long long blk = 0;
  for (int i = 0; i < T.nseg; ++i) {
    Seg &s = T.s[i];
    s.score_blk0 = (int)blk;
    s.score_bph = blocks_per_head(s.n, tokens_per_wg, SCORE_STEP);
    s.score_chunk = chunk_of(s.n, tokens_per_wg, SCORE_STEP);
    blk += (long long)s.score_bph * s.head_count;
  }
  return blk;
}

// Total workgroups of a launch whose blocks-per-head rule is (per_block, by_keep).
inline long long total_blocks(const SegTable &T, int per_block, int step, bool by_keep) {
  long long nb = 0;
  for (int i = 0; i < T.nseg; ++i)
    nb += (long long)blocks_per_head(by_keep ? T.s[i].k_keep : T.s[i].n, per_block, step) *
          T.s[i].head_count;
  return nb;
}

}  // namespace cmp
