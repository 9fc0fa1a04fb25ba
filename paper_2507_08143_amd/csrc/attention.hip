// Attention-based scores (paper Sec. 3.2, "Attention-Based Scoring"):
//     a = concat_i 1^T softmax(Q[i] K[i]^T)
// non-causal attention inside blocks of C = 256 consecutive positions, summed over the block's
// queries, averaged over the query heads that share a kv-head, then mean-pooled along the
// sequence.  The result is the `attn` input of the scoring entry points (Eq. "scoring").
//
// One workgroup per (kv-head, block).  The transposed product S^T = K Q^T is formed so that the
// softmax statistics of a query are per-lane quantities: wave w keeps its 64 keys as MFMA A
// operands in registers for the whole block; the query rows (64 at a time, every query head of
// the group in turn) pass through LDS as B operands.  Both operands are plain 16-byte pieces of
// rows (the contraction runs over channels), so nothing is transposed.  The four waves each
// see a quarter of a query's keys; they exchange (max, sum) once per step through LDS and
// merge them as in an online softmax.  The column sums accumulate in 32 registers per lane and
// are reduced across lanes once per block.
#include <math.h>
#include <string.h>

#include "common.h"

namespace cmp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int ATT_C = 256;          // block (chunk) size C of the paper
constexpr int ATT_QB = 64;          // queries per step
constexpr int ATT_QBUF = 4;         // staged query tiles in flight (three steps ahead)
constexpr int ATT_MAX_SEG = 16;

struct AttnSeg {
  const uint16_t *q, *k;
  long long q_stride_l, q_stride_h, q_stride_t;
  long long k_stride_l, k_stride_h, k_stride_t;
  long long out_off;      // float offset of the request's head (0,0) in the output
  int n;
  int head_begin, head_count;   // kv heads (l*H+h) of the request covered by this launch
  int H, G;               // kv heads per layer, query heads per kv head
};
struct AttnTable {
  AttnSeg s[ATT_MAX_SEG];
  int nseg;
  float scale;
  int pool;
};

// Exchange between the two halves of a wave with the row-swap instruction of gfx950: after
// swapping the upper half of one copy with the lower half of the other, the two results of a
// lane are its own value and that of the lane 32 away, so a max or a sum of the pair finishes
// the reduction in every lane, without LDS traffic.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ float halves_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// the largest of three finite-or-infinite numbers in one instruction
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// A staged query tile is 64 rows of 256 B without padding; the 16-byte pieces of row r are
// stored at position (piece ^ (r & 15)), so that the 16 lanes that read the same piece of 16
// consecutive rows touch every bank once.
struct AttnLds {
  uint16_t ql[ATT_QBUF][ATT_QB * D];   // staged query rows, filled by loads that write LDS directly
  float st_m[2][4][ATT_QB];          // per wave: scaled maximum of every query of the step
  float st_l[2][4][ATT_QB];          //           and the sum of its exponentials
};

// One (kv-head, block) of the column sums.  RAGGED is the last block of a head whose length is
// not a multiple of the block: only there keys and queries past the end have to be masked.
//
// The products are 32x32x16 MFMAs: D[key][query] leaves lane l with 16 keys of query l & 31
// (keys 8*(v>>2) + 4*(l>>5) + (v&3), v = 0..15), so a query's 64 keys of this wave are the 32
// registers of two key tiles in lanes l and l ^ 32.
template <bool RAGGED>
__device__ __forceinline__ void attn_block(const AttnSeg &s, float scale, int head, int c0,
                                           AttnLds &L, float *__restrict__ raw) {
  const int n = s.n;
  const int layer = head / s.H, kvh = head - layer * s.H;
  const uint16_t *kp = s.k + (long long)layer * s.k_stride_l + (long long)kvh * s.k_stride_h;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, lh = lane >> 5;

  // this wave's 64 keys as A operands: tile kt, lane (key l32, channels 16*kk + 8*lh ..)
  bf16x8 ka[2][8];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    const int key = c0 + 64 * wave + 32 * kt + l32;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      union { uint4 u; bf16x8 v; } t;
      t.u = make_uint4(0, 0, 0, 0);
      if (!RAGGED || key < n)
        t.u = *reinterpret_cast<const uint4 *>(kp + (long long)key * s.k_stride_t + 16 * kk + 8 * lh);
      ka[kt][kk] = t.v;
    }
  }
  // key of register v of key tile kt in this lane
  auto key_of = [&](int kt, int v) { return c0 + 64 * wave + 32 * kt + 8 * (v >> 2) + 4 * lh + (v & 3); };

  float pacc[2][16];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int v = 0; v < 16; ++v) pacc[kt][v] = 0.f;

  // Query rows go from memory into LDS without passing through registers, so that the tiles of
  // three later steps can be in flight at no cost in registers (one step of arithmetic is
  // shorter than the latency of a load while the memory system is busy).  One such load of a
  // wave moves four rows: lane l brings a 16-byte piece of row l >> 4 to LDS position
  // base + 16 l, which is position l & 15 of that row; it fetches the piece that belongs there.
  const int nsteps = s.G * (ATT_C / ATT_QB);          // (query head of the group, 64-query block)
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const int ld_row = 4 * wv + (lane >> 4);            // row within a group of 16
  const int ld_piece = (lane & 15) ^ (ld_row & 15);
  const uint16_t *q_head0 = s.q + (long long)layer * s.q_stride_l + (long long)(kvh * s.G) * s.q_stride_h;
  // this lane's piece of row c0 + ld_row of the group's first query head; a step adds an offset
  // that is the same for all lanes
  const uint16_t *q_lane = q_head0 + (long long)(c0 + ld_row) * s.q_stride_t + ld_piece * 8;
  auto issue_q = [&](int step) {
    const int qh = step / (ATT_C / ATT_QB), r0 = (step % (ATT_C / ATT_QB)) * ATT_QB;
    uint16_t *dst = &L.ql[step % ATT_QBUF][4 * wv * D];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint16_t *src;
      if (RAGGED) {      // past the end: any valid row, masked below
        const int row = min(c0 + r0 + 16 * i + ld_row, n - 1);
        src = q_head0 + (long long)qh * s.q_stride_h + (long long)row * s.q_stride_t + ld_piece * 8;
      } else {
        src = q_lane + ((long long)qh * s.q_stride_h + (long long)(r0 + 16 * i) * s.q_stride_t);
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                       (__attribute__((address_space(3))) void *)(dst + 16 * i * D),
                                       16, 0, 0);
    }
  };
  int q_piece[8];    // where piece 2*kk + lh of this lane's query row (l32 of a tile) is stored
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) q_piece[kk] = l32 * D + 8 * ((2 * kk + lh) ^ (l32 & 15));

  // S^T tiles of one 32-query tile: acc[qt][kt] = keys (tile kt) x queries, contraction over
  // channels; the two key tiles alternate so that consecutive MFMAs are independent
  f32x16 acc[2][2];
  auto product = [&](int buf, int qt) {
    bf16x8 qb[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qb[kk] = *reinterpret_cast<const bf16x8 *>(&L.ql[buf][32 * qt * D + q_piece[kk]]);
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[qt][kt][v] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        acc[qt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kt][kk], qb[kk], acc[qt][kt], 0, 0, 0);
  };

  // The compiler does not count loads that write LDS when it places its waits, and a
  // __syncthreads() would wait for all of them; the waits and barriers of the query pipeline
  // are therefore written out.  Loads complete in order and every step issues four per wave, so
  // "at most 8 outstanding" means: everything up to the next step's tile has arrived.
  issue_q(0);
  issue_q(1);
  issue_q(2);
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  product(0, 0);

  const float c2 = scale * 1.4426950408889634f;       // logits in units of log 2
  for (int step = 0; step < nsteps; ++step) {
    const int buf = step % ATT_QBUF, sb = step & 1;
    // the tile of three steps ahead replaces the one of the previous step, which every wave
    // has finished reading before the barrier that ended that step
    if (step + 3 < nsteps) issue_q(step + 3);

    // Local softmax statistics of every query over this wave's 64 keys, in the base-2 domain:
    // e = 2^(c*s - m) with c = scale * log2(e), so an element costs half a max3, one fma, one
    // exp and one add.  The product of the second query tile is issued ahead of the arithmetic
    // of the first.
    float m_mine = 0.f, l_mine = 0.f;    // statistics of query `lane` of the step (tile lh)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      if (qt == 0) product(buf, 1);
      if (RAGGED) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (key_of(kt, v) >= n) acc[qt][kt][v] = -INFINITY;
      }
      // two independent chains each for the maximum and for the sum (one per key tile)
      float mk[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        mk[kt] = max3(acc[qt][kt][0], acc[qt][kt][1], acc[qt][kt][2]);
#pragma unroll
        for (int v = 3; v < 15; v += 2) mk[kt] = max3(mk[kt], acc[qt][kt][v], acc[qt][kt][v + 1]);
      }
      const float m = halves_max(max3(mk[0], mk[1], fmaxf(acc[qt][0][15], acc[qt][1][15])));
      float mc = m * c2;
      const float mx = mc;
      if (RAGGED && m == -INFINITY) mc = 0.f;           // a wave whose keys are all past the end
      float lk[2] = {0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 16; ++v)
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
          const float e = __builtin_amdgcn_exp2f(fmaf(acc[qt][kt][v], c2, -mc));
          acc[qt][kt][v] = e;
          lk[kt] += e;
        }
      float l = lk[0] + lk[1];
      l = halves_sum(l);
      if (lh == qt) {
        m_mine = mx;
        l_mine = l;
      }
    }
    L.st_m[sb][wave][lane] = m_mine;
    L.st_l[sb][wave][lane] = l_mine;

    // statistics of this step and the next step's queries are in LDS after this barrier
    if (step + 3 < nsteps)
      asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // merge the four waves' statistics, one query per lane, then hand both tiles their factor
    float mw[4], m = L.st_m[sb][0][lane];
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) {
      mw[w2] = L.st_m[sb][w2][lane];
      m = fmaxf(m, mw[w2]);
    }
    float l = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < 4; ++w2) l = fmaf(L.st_l[sb][w2][lane], __builtin_amdgcn_exp2f(mw[w2] - m), l);
    float f = __builtin_amdgcn_exp2f(m_mine - m) * __builtin_amdgcn_rcpf(l);
    if (RAGGED) {
      const int q0 = c0 + (step % (ATT_C / ATT_QB)) * ATT_QB;
      if (q0 + lane >= n) f = 0.f;
    }
    const u32x2 fr = __builtin_amdgcn_permlane32_swap(__float_as_uint(f), __float_as_uint(f), false, false);
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      const float fq = __uint_as_float(fr[qt]);        // factor of query 32*qt + l32
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) pacc[kt][v] = fmaf(acc[qt][kt][v], fq, pacc[kt][v]);
      // First tile of the next step, in the same basic block as the accumulation so that the two
      // interleave; after the last step it multiplies an old tile and the result is dropped.
      if (qt == 0) product((step + 1) % ATT_QBUF, 0);
    }
  }

  // column sums: add over the 32 query lanes of each half, average over the query heads.  After
  // the reduction every lane of a half holds the sum of key 8*(v>>2) + 4*lh + (v&3) of its tile;
  // lane l32 keeps the one whose key number is l32, so that a tile's 32 sums leave as one
  // 128-byte store instead of 32 single ones (small stores between streaming reads are costly).
  const float inv_g = 1.f / (float)s.G;
  float *out = raw + s.out_off + (long long)head * n;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    float mine = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float x = pacc[kt][v];
      x += __shfl_xor(x, 1);
      x += __shfl_xor(x, 2);
      x += __shfl_xor(x, 4);
      x += __shfl_xor(x, 8);
      x += __shfl_xor(x, 16);
      if (l32 == 8 * (v >> 2) + 4 * lh + (v & 3)) mine = x;
    }
    const int key = c0 + 64 * wave + 32 * kt + l32;
    if (lh == ((l32 >> 2) & 1) && key < n) out[key] = mine * inv_g;
  }
}

__global__ __launch_bounds__(256, 2) void attn_colsum_kernel(const AttnTable T,
                                                             float *__restrict__ raw) {
  __shared__ __attribute__((aligned(16))) AttnLds L;

  // locate (segment, kv head, block)
  int seg = 0, head = 0, blk = 0;
  {
    int base = 0;
    for (int i = 0; i < T.nseg; ++i) {
      const int bph = (T.s[i].n + ATT_C - 1) / ATT_C;
      const int nb = bph * T.s[i].head_count;
      if ((int)blockIdx.x < base + nb || i == T.nseg - 1) {
        const int local = blockIdx.x - base;
        seg = i;
        head = T.s[i].head_begin + local / bph;
        blk = local % bph;
        break;
      }
      base += nb;
    }
  }
  const AttnSeg &s = T.s[seg];
  const int c0 = blk * ATT_C;
  if (c0 + ATT_C > s.n)
    attn_block<true>(s, T.scale, head, c0, L, raw);
  else
    attn_block<false>(s, T.scale, head, c0, L, raw);
}

// Mean pooling along the sequence: window `pool` (odd), zero padding, divided by `pool`.
// A workgroup stages its 1024 positions and the halo once in LDS.
__global__ __launch_bounds__(256) void attn_pool_kernel(const AttnTable T,
                                                        const float *__restrict__ raw,
                                                        float *__restrict__ attn) {
  constexpr int SPAN = 1024, HALO = 32;           // pool <= 63: at most 31 positions each side
  __shared__ float tile[SPAN + 2 * HALO];
  int seg = 0, head = 0, blk = 0;
  {
    int base = 0;
    for (int i = 0; i < T.nseg; ++i) {
      const int bph = (T.s[i].n + SPAN - 1) / SPAN;
      const int nb = bph * T.s[i].head_count;
      if ((int)blockIdx.x < base + nb || i == T.nseg - 1) {
        const int local = blockIdx.x - base;
        seg = i;
        head = T.s[i].head_begin + local / bph;
        blk = local % bph;
        break;
      }
      base += nb;
    }
  }
  const AttnSeg &s = T.s[seg];
  const int n = s.n, h = T.pool / 2;
  const float *src = raw + s.out_off + (long long)head * n;
  float *dst = attn + s.out_off + (long long)head * n;
  const int t0 = blk * SPAN;
  for (int i = threadIdx.x; i < SPAN + 2 * HALO; i += 256) {
    const int j = t0 - HALO + i;
    tile[i] = (j >= 0 && j < n) ? src[j] : 0.f;   // zero padding at both ends of the sequence
  }
  __syncthreads();
  const float inv = 1.f / (float)T.pool;
  for (int i = threadIdx.x; i < SPAN && t0 + i < n; i += 256) {
    float acc = 0.f;
    for (int u = -h; u <= h; ++u) acc += tile[HALO + i + u];
    dst[t0 + i] = acc * inv;
  }
}

}  // namespace cmp

using namespace cmp;

extern "C" {
#pragma GCC visibility push(default)

int compactor_attention_workspace_size(const compactor_attn_params_t *p,
                                       const compactor_attn_request_t *reqs, int32_t nreq,
                                       size_t *bytes) {
  if (!p || !reqs || !bytes || nreq < 1) return COMPACTOR_EINVAL;
  if (p->layers < 1 || p->kv_heads < 1) return COMPACTOR_EINVAL;
  size_t tot = 0;
  for (int b = 0; b < nreq; ++b) {
    if (reqs[b].n < 1) return COMPACTOR_EINVAL;
    tot += (size_t)p->layers * p->kv_heads * reqs[b].n;
  }
  *bytes = (tot * sizeof(float) + 255) / 256 * 256;
  return COMPACTOR_OK;
}

int compactor_attention_scores(const compactor_attn_params_t *p,
                               const compactor_attn_request_t *reqs, int32_t nreq, float *attn,
                               void *workspace, size_t workspace_bytes, void *stream) {
  if (!p || !reqs || nreq < 1 || !attn) return COMPACTOR_EINVAL;
  if (p->layers < 1 || p->kv_heads < 1 || p->q_heads < p->kv_heads || p->q_heads % p->kv_heads)
    return COMPACTOR_EINVAL;
  if (p->head_dim != D || p->chunk != ATT_C) return COMPACTOR_EUNSUPPORTED;
  if (p->pool < 1 || p->pool > 63 || !(p->pool & 1)) return COMPACTOR_EINVAL;
  if (!(p->scale >= 0.f) || !isfinite(p->scale)) return COMPACTOR_EINVAL;
  for (int b = 0; b < nreq; ++b) {
    const compactor_attn_request_t &r = reqs[b];
    if (r.n < 1 || !r.q || !r.k) return COMPACTOR_EINVAL;
    if (r.q_stride_t < D || r.k_stride_t < D) return COMPACTOR_EINVAL;
    if ((r.q_stride_t | r.q_stride_h | r.q_stride_l | r.k_stride_t | r.k_stride_h | r.k_stride_l) & 7)
      return COMPACTOR_EALIGN;
    if ((reinterpret_cast<uintptr_t>(r.q) | reinterpret_cast<uintptr_t>(r.k)) & 15u) return COMPACTOR_EALIGN;
  }
  size_t need;
  int rc = compactor_attention_workspace_size(p, reqs, nreq, &need);
  if (rc) return rc;
  if (!workspace || workspace_bytes < need) return COMPACTOR_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return COMPACTOR_EALIGN;

  hipStream_t st = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();   // a leftover of earlier, unrelated HIP calls is not this call's error
  float *raw = static_cast<float *>(workspace);
  const int LH = p->layers * p->kv_heads;
  long long off = 0;
  for (int b0 = 0; b0 < nreq; b0 += ATT_MAX_SEG) {
    AttnTable T;
    memset(&T, 0, sizeof(T));
    T.scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)D);
    T.pool = p->pool;
    long long nb_col = 0, nb_pool = 0;
    for (int b = b0; b < nreq && b < b0 + ATT_MAX_SEG; ++b) {
      const compactor_attn_request_t &r = reqs[b];
      AttnSeg &s = T.s[T.nseg++];
      s.q = static_cast<const uint16_t *>(r.q);
      s.k = static_cast<const uint16_t *>(r.k);
      s.q_stride_l = r.q_stride_l; s.q_stride_h = r.q_stride_h; s.q_stride_t = r.q_stride_t;
      s.k_stride_l = r.k_stride_l; s.k_stride_h = r.k_stride_h; s.k_stride_t = r.k_stride_t;
      s.out_off = off;
      s.n = r.n;
      s.head_begin = 0; s.head_count = LH;
      s.H = p->kv_heads; s.G = p->q_heads / p->kv_heads;
      off += (long long)LH * r.n;
      nb_col += (long long)LH * ((r.n + ATT_C - 1) / ATT_C);
      nb_pool += (long long)LH * ((r.n + 1023) / 1024);
    }
    if (nb_col > 0x7fffffffll) return COMPACTOR_EINVAL;
    hipLaunchKernelGGL(attn_colsum_kernel, dim3((unsigned)nb_col), dim3(256), 0, st, T, raw);
    if (hipGetLastError() != hipSuccess) return COMPACTOR_EHIP;
    hipLaunchKernelGGL(attn_pool_kernel, dim3((unsigned)nb_pool), dim3(256), 0, st, T, raw, attn);
    if (hipGetLastError() != hipSuccess) return COMPACTOR_EHIP;
  }
  return COMPACTOR_OK;
}

#pragma GCC visibility pop
}  // extern "C"
