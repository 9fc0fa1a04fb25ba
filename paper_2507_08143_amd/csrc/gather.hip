// Gather-compaction: the retained K/V rows of every head, in ascending token order, copied
// into a dense packed cache (paper Sec. 3: the compressed cache consists of the retained
// key/value pairs).  Pure copy, bit exact: 16 lanes move one 256-byte row with 16-byte
// accesses, four rows per wave instruction, K and V in the same pass.
//
// Small workgroups with few rows per lane do best on this read + write stream (measured on the
// benchmark's shape with random retained sets: 128 threads x 2 rows per 16-lane group 6.1 TB/s,
// 256 x 4 5.7 TB/s, 256 x 8 2.8 TB/s): a workgroup is 2 waves and moves GATHER_ROWS = 16 rows.
#include "common.h"

namespace cmp {

constexpr int GATHER_GROUPS = GATHER_THREADS / 16;        // 16-lane groups, one row each per pass
constexpr int GATHER_PASSES = GATHER_ROWS / GATHER_GROUPS;
static_assert(GATHER_ROWS % GATHER_GROUPS == 0, "whole passes");

// Workgroup -> (segment, head, tile of GATHER_ROWS retained rows).  The gather launches many small
// workgroups, so this avoids the 64-bit divisions of the general block locator.
__device__ __forceinline__ Where locate_rows(const SegTable &T, unsigned blk) {
  Where w{0, 0, 0, 0, GATHER_ROWS};
  unsigned base = 0;
  for (int i = 0; i < T.nseg; ++i) {
    const unsigned bph = ((unsigned)T.s[i].k_keep + GATHER_ROWS - 1) / GATHER_ROWS;
    const unsigned nb = bph * (unsigned)T.s[i].head_count;
    if (blk < base + nb || i == T.nseg - 1) {
      const unsigned local = blk - base, hh = local / bph;
      w.seg = i;
      w.head = T.s[i].head_begin + (int)hh;
      w.lhead = T.s[i].lhead0 + (int)hh;
      w.tile = (int)(local - hh * bph);
      return w;
    }
    base += nb;
  }
  return w;
}

__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(const SegTable T,
                                                     const int32_t *__restrict__ kept_idx,
                                                     uint16_t *__restrict__ k_packed,
                                                     uint16_t *__restrict__ v_packed) {
  const Where w = locate_rows(T, blockIdx.x);
  const Seg &s = T.s[w.seg];
  const int k = s.k_keep;
  const long long row0 = s.kept_off + (long long)w.head * k;      // first packed row of the head
  const int32_t *idx = kept_idx + row0;
  const uint16_t *ksrc = head_ptr(s.k_cache ? s.k_cache : s.k_score, s, w.head);
  const uint16_t *vsrc = head_ptr(s.v_cache, s, w.head);
  const int chunk = threadIdx.x & 15, sub = threadIdx.x >> 4;     // GATHER_GROUPS rows per pass

  uint4 kv[GATHER_PASSES], vv[GATHER_PASSES];
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    const int j = w.tile * GATHER_ROWS + p * GATHER_GROUPS + sub;
    kv[p] = make_uint4(0, 0, 0, 0);
    vv[p] = make_uint4(0, 0, 0, 0);
    if (j < k) {
      const int tok = idx[j];
      if (tok >= 0 && tok < s.n) {
        const long long off = (long long)tok * s.stride_t + chunk * 8;
        kv[p] = load_stream16(ksrc + off);
        vv[p] = load_stream16(vsrc + off);
      }
    }
  }
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    const int j = w.tile * GATHER_ROWS + p * GATHER_GROUPS + sub;
    if (j < k) {
      const long long off = (row0 + j) * D + chunk * 8;
      store_stream16(k_packed + off, kv[p]);
      store_stream16(v_packed + off, vv[p]);
    }
  }
}

// Layer scope: the retained rows of a layer's heads are packed one head after the other, head h
// holding kept_cnt[h] rows (ragged; the counts of a layer add up to H * k_keep).  A workgroup
// takes GATHER_ROWS rows of a layer's region and looks every row's head up in the counts.
__global__ __launch_bounds__(GATHER_THREADS) void gather_layer_kernel(const SegTable T,
                                                           const int32_t *__restrict__ kept_idx,
                                                           const int32_t *__restrict__ kept_cnt,
                                                           uint16_t *__restrict__ k_packed,
                                                           uint16_t *__restrict__ v_packed) {
  int seg = 0, layer = 0, tile = 0;
  {
    int base = 0;
    for (int i = 0; i < T.nseg; ++i) {
      const int bpl = (T.s[i].H * T.s[i].k_keep + GATHER_ROWS - 1) / GATHER_ROWS;
      const int nb = bpl * (T.s[i].head_count / T.s[i].H);
      if ((int)blockIdx.x < base + nb || i == T.nseg - 1) {
        const int local = blockIdx.x - base;
        seg = i;
        layer = local / bpl;
        tile = local - layer * bpl;
        break;
      }
      base += nb;
    }
  }
  const Seg &s = T.s[seg];
  const int head0 = s.head_begin + layer * s.H;                   // first head of the layer
  const int rows = s.H * s.k_keep;
  const long long row0 = s.kept_off + (long long)head0 * s.k_keep;
  const int32_t *idx = kept_idx + row0;
  const int32_t *cnt = kept_cnt + s.ghead0 + head0;
  const int chunk = threadIdx.x & 15, sub = threadIdx.x >> 4;

  uint4 kv[GATHER_PASSES], vv[GATHER_PASSES];
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    const int j = tile * GATHER_ROWS + p * GATHER_GROUPS + sub;
    kv[p] = make_uint4(0, 0, 0, 0);
    vv[p] = make_uint4(0, 0, 0, 0);
    if (j < rows) {
      int h = -1, run = 0;
      for (int hh = 0; hh < s.H; ++hh) {
        const int c = cnt[hh];
        if (j < run + c) { h = hh; break; }
        run += c;
      }
      const int tok = idx[j];
      if (h >= 0 && tok >= 0 && tok < s.n) {
        const long long off = (long long)tok * s.stride_t + chunk * 8;
        kv[p] = load_stream16(head_ptr(s.k_cache ? s.k_cache : s.k_score, s, head0 + h) + off);
        vv[p] = load_stream16(head_ptr(s.v_cache, s, head0 + h) + off);
      }
    }
  }
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    const int j = tile * GATHER_ROWS + p * GATHER_GROUPS + sub;
    if (j < rows) {
      const long long off = (row0 + j) * D + chunk * 8;
      store_stream16(k_packed + off, kv[p]);
      store_stream16(v_packed + off, vv[p]);
    }
  }
}

// ---- paged cache as the target (and, in place, the source) ----------------------------------
// Element offset of (logical slot j, layer l, head h) of a segment's request in the page pool,
// or -1 when the block table does not cover it or names a page outside the pool.
__device__ __forceinline__ long long page_slot(const PagePool &P, int seg, int l, int h, int j) {
  const int lp = j / P.page_size, slot = j - lp * P.page_size;
  if (lp >= P.t[seg].len) return -1;
  const int pg = P.t[seg].pages[lp];
  if (pg < 0 || pg >= P.num_pages) return -1;
  return (long long)pg * P.page_stride + (long long)l * P.layer_stride +
         (long long)h * P.head_stride + (long long)slot * P.slot_stride;
}

// Retained rows from the dense source tensors into pages: retained token j of a head goes to
// logical slot j of that head.  Workgroups are dealt as in the dense gathers.
__global__ __launch_bounds__(GATHER_THREADS) void gather_paged_kernel(const SegTable T, const PagePool P,
                                                           const int32_t *__restrict__ kept_idx,
                                                           const int32_t *__restrict__ kept_cnt) {
  int seg = 0, head0 = 0, tile = 0, rows = 0;       // head0: the head, or the layer's first head
  if (T.layer_scope) {
    int base = 0;
    for (int i = 0; i < T.nseg; ++i) {
      const int bpl = (T.s[i].H * T.s[i].k_keep + GATHER_ROWS - 1) / GATHER_ROWS;
      const int nb = bpl * (T.s[i].head_count / T.s[i].H);
      if ((int)blockIdx.x < base + nb || i == T.nseg - 1) {
        const int local = blockIdx.x - base, layer = local / bpl;
        seg = i;
        head0 = T.s[i].head_begin + layer * T.s[i].H;
        tile = local - layer * bpl;
        rows = T.s[i].H * T.s[i].k_keep;
        break;
      }
      base += nb;
    }
  } else {
    const Where w = locate_rows(T, blockIdx.x);
    seg = w.seg; head0 = w.head; tile = w.tile; rows = T.s[w.seg].k_keep;
  }
  const Seg &s = T.s[seg];
  const int32_t *idx = kept_idx + (s.kept_off + (long long)head0 * s.k_keep);
  const int32_t *cnt = kept_cnt + s.ghead0 + head0;
  const int chunk = threadIdx.x & 15, sub = threadIdx.x >> 4;
  const int layer = head0 / s.H;

  uint4 kv[GATHER_PASSES], vv[GATHER_PASSES];
  long long dst[GATHER_PASSES];
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    const int j = tile * GATHER_ROWS + p * GATHER_GROUPS + sub;
    dst[p] = -1;
    kv[p] = make_uint4(0, 0, 0, 0);
    vv[p] = make_uint4(0, 0, 0, 0);
    if (j < rows) {
      int head = head0, jh = j;                      // head of the row and its rank in that head
      if (T.layer_scope) {
        head = -1;
        int run = 0;
        for (int hh = 0; hh < s.H; ++hh) {
          const int c = cnt[hh];
          if (j < run + c) { head = head0 + hh; jh = j - run; break; }
          run += c;
        }
      }
      const int tok = idx[j];
      if (head >= 0 && tok >= 0 && tok < s.n) {
        const long long off = (long long)tok * s.stride_t + chunk * 8;
        kv[p] = load_stream16(head_ptr(s.k_cache ? s.k_cache : s.k_score, s, head) + off);
        vv[p] = load_stream16(head_ptr(s.v_cache, s, head) + off);
        dst[p] = page_slot(P, seg, layer, head - layer * s.H, jh);
      }
    }
  }
#pragma unroll
  for (int p = 0; p < GATHER_PASSES; ++p) {
    if (dst[p] >= 0) {
      store_stream16(P.k + dst[p] + chunk * 8, kv[p]);
      store_stream16(P.v + dst[p] + chunk * 8, vv[p]);
    }
  }
}

// In place: a head's tokens already live in the pages (token t at logical slot t) and its
// retained rows move to the front.  One workgroup per head walks the retained list in ascending
// runs of 256 rows: all rows of a run are read, the workgroup meets, the run is written.  A run's
// sources lie at or behind its own destinations and strictly behind those of earlier runs
// (kept[j] >= j, ascending), so nothing is overwritten before it has been read; for the same
// reason the next run's rows can be fetched while this run is being written (its sources lie
// behind every slot written so far), which keeps loads in flight across the barrier.
constexpr int INPLACE_THREADS = 1024, INPLACE_RUN = 256;
struct InplaceRun {
  uint4 kv[INPLACE_RUN / 64], vv[INPLACE_RUN / 64];
  long long dst[INPLACE_RUN / 64];
};
__global__ __launch_bounds__(INPLACE_THREADS) void compact_inplace_kernel(
    const SegTable T, const PagePool P, const int32_t *__restrict__ kept_idx,
    const int32_t *__restrict__ kept_cnt) {
  const Where w = locate_block(T, blockIdx.x, 0, 1, false);      // one block per head
  const Seg &s = T.s[w.seg];
  const int layer = w.head / s.H, h = w.head - layer * s.H;
  int rows = s.k_keep;
  long long first = s.kept_off + (long long)w.head * s.k_keep;
  if (T.layer_scope) {                  // ragged: this head's rows follow those of heads 0..h-1
    const int32_t *cnt = kept_cnt + s.ghead0 + layer * s.H;
    first = s.kept_off + (long long)layer * s.H * s.k_keep;
    for (int hh = 0; hh < h; ++hh) first += cnt[hh];
    rows = cnt[h];
  }
  const int32_t *idx = kept_idx + first;
  const int chunk = threadIdx.x & 15, sub = threadIdx.x >> 4;    // 64 rows per pass
  auto fetch = [&](int base, InplaceRun &r) {
#pragma unroll
    for (int p = 0; p < INPLACE_RUN / 64; ++p) {
      const int j = base + p * 64 + sub;
      r.dst[p] = -1;
      r.kv[p] = make_uint4(0, 0, 0, 0);
      r.vv[p] = make_uint4(0, 0, 0, 0);
      if (j < rows) {
        const int tok = idx[j];
        const long long src = (tok >= j && tok < s.n) ? page_slot(P, w.seg, layer, h, tok) : -1;
        if (src >= 0) {
          r.kv[p] = load_stream16(P.k + src + chunk * 8);
          r.vv[p] = load_stream16(P.v + src + chunk * 8);
          r.dst[p] = tok == j ? -1 : page_slot(P, w.seg, layer, h, j);   // already in place
        }
      }
    }
  };
  auto write = [&](const InplaceRun &r) {
#pragma unroll
    for (int p = 0; p < INPLACE_RUN / 64; ++p) {
      if (r.dst[p] >= 0) {
        store_stream16(P.k + r.dst[p] + chunk * 8, r.kv[p]);
        store_stream16(P.v + r.dst[p] + chunk * 8, r.vv[p]);
      }
    }
  };
  InplaceRun a, b;
  fetch(0, a);
  for (int base = 0; base < rows; base += 2 * INPLACE_RUN) {
    __syncthreads();      // every row of run `a` has been read (the barrier waits for the loads)
    fetch(base + INPLACE_RUN, b);
    write(a);
    if (base + INPLACE_RUN >= rows) break;         // uniform
    __syncthreads();
    fetch(base + 2 * INPLACE_RUN, a);
    write(b);
  }
}

hipError_t launch_gather_paged(const SegTable &T, const PagePool &P, const int32_t *kept_idx,
                               const int32_t *kept_cnt, bool in_place, hipStream_t st) {
  if (T.nheads <= 0) return hipSuccess;
  if (in_place) {
    hipLaunchKernelGGL(compact_inplace_kernel, dim3((unsigned)T.nheads), dim3(INPLACE_THREADS), 0,
                       st, T, P, kept_idx, kept_cnt);
    return hipGetLastError();
  }
  long long nb = 0;
  if (T.layer_scope) {
    for (int i = 0; i < T.nseg; ++i)
      nb += (long long)((T.s[i].H * (long long)T.s[i].k_keep + GATHER_ROWS - 1) / GATHER_ROWS) *
            (T.s[i].head_count / T.s[i].H);
  } else {
    nb = total_blocks(T, GATHER_ROWS, GATHER_ROWS, true);
  }
  if (nb <= 0) return hipSuccess;
  if (nb > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_paged_kernel, dim3((unsigned)nb), dim3(GATHER_THREADS), 0, st, T, P, kept_idx,
                     kept_cnt);
  return hipGetLastError();
}

hipError_t launch_gather(const SegTable &T, const int32_t *kept_idx, const int32_t *kept_cnt,
                         uint16_t *k_packed, uint16_t *v_packed, hipStream_t st) {
  if (T.layer_scope) {
    long long nb = 0;
    for (int i = 0; i < T.nseg; ++i)
      nb += (long long)((T.s[i].H * (long long)T.s[i].k_keep + GATHER_ROWS - 1) / GATHER_ROWS) *
            (T.s[i].head_count / T.s[i].H);
    if (nb <= 0) return hipSuccess;
    if (nb > 0x7fffffffll) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gather_layer_kernel, dim3((unsigned)nb), dim3(GATHER_THREADS), 0, st, T, kept_idx,
                       kept_cnt, k_packed, v_packed);
    return hipGetLastError();
  }
  const long long nb = total_blocks(T, GATHER_ROWS, GATHER_ROWS, true);
  if (nb <= 0) return hipSuccess;
  if (nb > 0x7fffffffll) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gather_kernel, dim3((unsigned)nb), dim3(GATHER_THREADS), 0, st, T, kept_idx, k_packed,
                     v_packed);
  return hipGetLastError();
}

}  // namespace cmp
