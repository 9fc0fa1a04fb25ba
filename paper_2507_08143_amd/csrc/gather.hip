// Gather-compaction: the retained K/V rows of every head, in ascending token order, copied
// into a dense packed cache (paper Sec. 3: the compressed cache consists of the retained
// key/value pairs).  Pure copy, bit exact: 16 lanes move one 256-byte row with 16-byte
// accesses, four rows per wave instruction, K and V in the same pass.
#include "common.h"

namespace cmp {

__global__ __launch_bounds__(256) void gather_kernel(const SegTable T,
                                                     const int32_t *__restrict__ kept_idx,
                                                     uint16_t *__restrict__ k_packed,
                                                     uint16_t *__restrict__ v_packed) {
#ifdef GATHER_REVERSE
  const Where w = locate_block(T, gridDim.x - 1 - blockIdx.x, GATHER_ROWS, GATHER_ROWS, true);
#else
  const Where w = locate_block(T, blockIdx.x, GATHER_ROWS, GATHER_ROWS, true);
#endif
  const Seg &s = T.s[w.seg];
  const int k = s.k_keep;
  const long long row0 = s.kept_off + (long long)w.head * k;      // first packed row of the head
  const int32_t *idx = kept_idx + row0;
  const uint16_t *ksrc = head_ptr(s.k_cache ? s.k_cache : s.k_score, s, w.head);
  const uint16_t *vsrc = head_ptr(s.v_cache, s, w.head);
  const int chunk = threadIdx.x & 15, sub = threadIdx.x >> 4;     // 16 rows per pass

  uint4 kv[GATHER_ROWS / 16], vv[GATHER_ROWS / 16];
#pragma unroll
  for (int p = 0; p < GATHER_ROWS / 16; ++p) {
    const int j = w.tile * GATHER_ROWS + p * 16 + sub;
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
  for (int p = 0; p < GATHER_ROWS / 16; ++p) {
    const int j = w.tile * GATHER_ROWS + p * 16 + sub;
    if (j < k) {
      const long long off = (row0 + j) * D + chunk * 8;
#ifdef GATHER_PLAIN_STORES
      *reinterpret_cast<uint4 *>(k_packed + off) = kv[p];
      *reinterpret_cast<uint4 *>(v_packed + off) = vv[p];
#else
      store_stream16(k_packed + off, kv[p]);
      store_stream16(v_packed + off, vv[p]);
#endif
    }
  }
}

// Layer scope: the retained rows of a layer's heads are packed one head after the other, head h
// holding kept_cnt[h] rows (ragged; the counts of a layer add up to H * k_keep).  A workgroup
// takes 64 rows of a layer's region and looks every row's head up in the counts.
__global__ __launch_bounds__(256) void gather_layer_kernel(const SegTable T,
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

  uint4 kv[GATHER_ROWS / 16], vv[GATHER_ROWS / 16];
#pragma unroll
  for (int p = 0; p < GATHER_ROWS / 16; ++p) {
    const int j = tile * GATHER_ROWS + p * 16 + sub;
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
  for (int p = 0; p < GATHER_ROWS / 16; ++p) {
    const int j = tile * GATHER_ROWS + p * 16 + sub;
    if (j < rows) {
      const long long off = (row0 + j) * D + chunk * 8;
      store_stream16(k_packed + off, kv[p]);
      store_stream16(v_packed + off, vv[p]);
    }
  }
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
    hipLaunchKernelGGL(gather_layer_kernel, dim3((unsigned)nb), dim3(256), 0, st, T, kept_idx,
                       kept_cnt, k_packed, v_packed);
    return hipGetLastError();
  }
  const long long nb = total_blocks(T, GATHER_ROWS, GATHER_ROWS, true);
  if (nb <= 0) return hipSuccess;
  hipLaunchKernelGGL(gather_kernel, dim3((unsigned)nb), dim3(256), 0, st, T, kept_idx, k_packed,
                     v_packed);
  return hipGetLastError();
}

}  // namespace cmp
