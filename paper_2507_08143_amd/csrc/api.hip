// C boundary of libcompactor: argument checks, output layout, workspace carving and the
// stream-ordered launch sequence.  Declarations and their contracts: include/compactor.h.
#include <math.h>
#include <string.h>

#include <mutex>

#include "common.h"

using namespace cmp;

namespace {

constexpr long long DEFAULT_GROUP_BYTES = 1ll << 40;   // one group unless the caller asks
constexpr size_t WS_ALIGN = 256;

inline size_t align_up(size_t x) { return (x + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

enum Need { NEED_SCORE = 1, NEED_PACK = 2 };

int check_params(const compactor_params_t *p, bool scoring) {
  if (!p) return COMPACTOR_EINVAL;
  if (p->layers < 1 || p->kv_heads < 1) return COMPACTOR_EINVAL;
  if ((long long)p->layers * p->kv_heads > (1 << 20)) return COMPACTOR_EINVAL;
  if (p->head_dim != D) return COMPACTOR_EUNSUPPORTED;
  const int ks = p->sketch_dim;
  if (!(ks == 0 || ks == 16 || ks == 32 || ks == 48 || ks == 64)) return COMPACTOR_EUNSUPPORTED;
  if (scoring) {
    if (ks > 0 && !p->phi) return COMPACTOR_EINVAL;
    if (ks > 0 && !aligned16(p->phi)) return COMPACTOR_EALIGN;
    if (!(p->ridge_rel >= 0.f) || !isfinite(p->ridge_rel)) return COMPACTOR_EINVAL;
    if (!isfinite(p->lambda_blend)) return COMPACTOR_EINVAL;
  }
  if (p->group_bytes < 0 || p->gram_wgs < 0 || p->score_tokens < 0)
    return COMPACTOR_EINVAL;
  if (p->select_scope != COMPACTOR_SCOPE_HEAD && p->select_scope != COMPACTOR_SCOPE_LAYER)
    return COMPACTOR_EINVAL;
  return COMPACTOR_OK;
}

// Layer scope pools H heads: their tokens and their budget are counted in 32-bit integers.
int check_scope(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq) {
  if (p->select_scope != COMPACTOR_SCOPE_LAYER) return COMPACTOR_OK;
  for (int b = 0; b < nreq; ++b)
    if ((long long)reqs[b].n * p->kv_heads > 0x7fffffffll - 64) return COMPACTOR_EINVAL;
  return COMPACTOR_OK;
}

int check_requests(const compactor_request_t *reqs, int32_t nreq, int need) {
  if (!reqs || nreq < 1 || nreq > (1 << 20)) return COMPACTOR_EINVAL;
  for (int b = 0; b < nreq; ++b) {
    const compactor_request_t &r = reqs[b];
    if (r.n < 1 || r.n > 0x7fffffff - 64) return COMPACTOR_EINVAL;
    if (!(r.ratio > 0.f && r.ratio <= 1.f)) return COMPACTOR_EINVAL;
    if (need) {
      if ((need & NEED_SCORE) && !r.k_score) return COMPACTOR_EINVAL;
      if ((need & NEED_PACK) && (!r.v_cache || (!r.k_cache && !r.k_score))) return COMPACTOR_EINVAL;
      if (r.stride_t < D || r.stride_l < 0 || r.stride_h < 0) return COMPACTOR_EINVAL;
      if ((r.stride_t & 7) || (r.stride_l & 7) || (r.stride_h & 7)) return COMPACTOR_EALIGN;
      if (!aligned16(r.k_score) || !aligned16(r.k_cache) || !aligned16(r.v_cache) ||
          (reinterpret_cast<uintptr_t>(r.attn) & 3u))
        return COMPACTOR_EALIGN;
    }
  }
  return COMPACTOR_OK;
}

int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
    n = 256;
  return n;
}

// Gram: a persistent launch of 2 workgroups per compute unit (or as many as there are tiles),
// each taking an equal run of 64-row tiles.
struct GramPlan { int nwg, tiles_per_wg; };
GramPlan gram_plan(const compactor_params_t *p, const SegTable &T, int cus) {
  const long long total = total_tiles(T);
  long long want = p->gram_wgs > 0 ? p->gram_wgs : 2ll * cus;
  if (want > total) want = total;
  if (want < 1) want = 1;
  GramPlan g;
  g.tiles_per_wg = (int)((total + want - 1) / want);
  // not below 8 tiles (512 rows) a workgroup: every partial costs a 40 KB round trip
  if (g.tiles_per_wg < 8 && p->gram_wgs <= 0) g.tiles_per_wg = 8;
  g.nwg = (int)((total + g.tiles_per_wg - 1) / g.tiles_per_wg);
  return g;
}

// Score: workgroups of equal token runs inside a head, 2 per compute unit at a time.  A launch
// of W workgroups takes ceil(W / slots) rounds; the run length is chosen to keep the last
// round full and the per-workgroup fixed cost (staging W^T, about 32 KB) small.
int score_tokens_for(const compactor_params_t *p, const SegTable &T, int cus) {
  if (p->score_tokens > 0) {
    const int t = (p->score_tokens + SCORE_STEP - 1) / SCORE_STEP * SCORE_STEP;
    return t > SCORE_MAX_RUN ? SCORE_MAX_RUN : t;
  }
  // Sketched mode: one burst per workgroup (measured on MI355X: runs of two bursts are 2 to 9 %
  // slower, the barriers around a burst in mid-run cost more than the longer run saves, and many
  // short workgroups balance the CUs better).  Exact mode stages four times as much W^T per
  // workgroup and gains 4 % from runs of 16384 tokens.
  const int cap = p->sketch_dim == 0 ? 16384 : SCORE_BURST;
  const int slots = 2 * cus;
  int best = cap;
  double best_score = -1.0;
  for (int c = cap; c >= 1024; c -= SCORE_STEP) {
    const double w = (double)total_blocks(T, c, SCORE_STEP, false);
    const double rounds = ceil(w / slots);
    const double score = w / (rounds * slots) * (c * 256.0) / (c * 256.0 + 32768.0);
    if (score > best_score + 1e-9) { best_score = score; best = c; }
  }
  return best;
}

struct GroupBytes {
  size_t partials, wt, hist1, sel, bstat, scores;   // in this order in the workspace
  size_t total() const { return partials + wt + hist1 + sel + bstat + scores; }
  size_t off_wt() const { return partials; }
  size_t off_hist1() const { return off_wt() + wt; }
  size_t off_sel() const { return off_hist1() + hist1; }
  size_t off_bstat() const { return off_sel() + sel; }
  size_t off_scores() const { return off_bstat() + bstat; }
};

GroupBytes group_bytes_needed(const compactor_params_t *p, const SegTable &T, bool need_scores) {
  const int ks = p->sketch_dim;
  long long rows = 0;
  for (int i = 0; i < T.nseg; ++i) rows += (long long)T.s[i].n * T.s[i].head_count;
  const int m = ks > 0 ? ks : D;
  GroupBytes g;
  g.partials = align_up(((size_t)gram_plan(p, T, compute_units()).nwg + T.nheads) *
                        GRAM_PARTIAL_FLOATS * sizeof(float));
  g.wt = align_up((size_t)T.nheads * W_TERMS * m * D * sizeof(uint16_t));
  g.hist1 = align_up((size_t)T.nheads * HIST1_BINS * sizeof(int));
  g.sel = select_needs_pools(T) ? align_up((size_t)select_scratch(T).ints() * sizeof(int)) : 0;
  // the blend's sums: four doubles per score workgroup
  g.bstat = 0;
  if (blend_wanted(T))
    g.bstat = align_up((size_t)total_blocks(T, score_tokens_for(p, T, compute_units()), SCORE_STEP, false) *
                       4 * sizeof(double));
  g.scores = need_scores ? align_up((size_t)rows * sizeof(float)) : 0;
  return g;
}

// Walks the batch in head order and cuts it into launch groups of about group_rows key rows
// (at most MAX_SEG request pieces each).  fn(T, group_score_rows) is called per group; with
// local_scores the segments' score offsets address a group-local buffer.
template <class F>
int for_each_group(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                   long long group_rows, bool local_scores, F &&fn) {
  const int LH = p->layers * p->kv_heads;
  if ((long long)nreq * LH > 0x7fffffffll) return COMPACTOR_EINVAL;   // heads are numbered in int
  long long score_off = 0, kept_off = 0;
  int b = 0, h = 0;
  while (b < nreq) {
    SegTable T;
    memset(&T, 0, sizeof(T));
    T.layer_scope = p->select_scope == COMPACTOR_SCOPE_LAYER;
    const int unit = T.layer_scope ? p->kv_heads : 1;     // heads are taken in whole pools
    long long rows = 0, local_off = 0;
    while (b < nreq && T.nseg < MAX_SEG && rows < group_rows) {
      const compactor_request_t &r = reqs[b];
      const int kk = compactor_keep_count(r.n, r.ratio);
      long long can = (group_rows - rows + r.n - 1) / r.n;
      can = (can + unit - 1) / unit * unit;
      if (can < unit) can = unit;
      const int take = (int)(can < (long long)(LH - h) ? can : (long long)(LH - h));
      Seg &s = T.s[T.nseg++];
      s.k_score = static_cast<const uint16_t *>(r.k_score);
      s.k_cache = static_cast<const uint16_t *>(r.k_cache);
      s.v_cache = static_cast<const uint16_t *>(r.v_cache);
      s.attn = r.attn;
      s.stride_l = r.stride_l; s.stride_h = r.stride_h; s.stride_t = r.stride_t;
      s.score_off = local_scores ? local_off - (long long)h * r.n : score_off;
      s.kept_off = kept_off;
      s.n = r.n; s.k_keep = kk;
      s.head_begin = h; s.head_count = take;
      s.ghead0 = b * LH; s.lhead0 = T.nheads; s.H = p->kv_heads; s.req = b;
      T.nheads += take;
      rows += (long long)take * r.n;
      local_off += (long long)take * r.n;
      h += take;
      if (h == LH) {
        score_off += (long long)LH * r.n;
        kept_off += (long long)LH * kk;
        h = 0;
        ++b;
      }
    }
    index_chunks(T);
    const int rc = fn(T, rows);
    if (rc != COMPACTOR_OK) return rc;
  }
  return COMPACTOR_OK;
}

// Key rows per head group: an explicit group_bytes wins, otherwise the whole call is one group.
long long group_rows_of(const compactor_params_t *p) {
  if (p->group_bytes > 0) {
    const long long r = p->group_bytes / (D * 2);
    return r < 1 ? 1 : r;
  }
  return DEFAULT_GROUP_BYTES / (D * 2);
}

// Bytes of workspace a call needs: what its largest head group needs (groups run one after the
// other on the stream and reuse the workspace).
int workspace_need(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                   bool local_scores, size_t *bytes) {
  size_t need = 0;
  const int rc = for_each_group(p, reqs, nreq, group_rows_of(p), local_scores,
                                [&](const SegTable &T, long long) {
                                  const size_t t = group_bytes_needed(p, T, local_scores).total();
                                  if (t > need) need = t;
                                  return COMPACTOR_OK;
                                });
  *bytes = need;
  return rc;
}

// The launchers report hipGetLastError(), which also returns an error that an earlier, unrelated
// HIP call left pending on this thread.  Every enqueueing entry point discards such a leftover
// first, so that COMPACTOR_EHIP always speaks of the library's own calls.
inline void drop_pending_error() { (void)hipGetLastError(); }

#define HIP_TRY(expr)                                \
  do {                                               \
    if ((expr) != hipSuccess) return COMPACTOR_EHIP; \
  } while (0)

// Optional profiling events (compactor_params_t.stage_events): mark(i) records event i.
struct Marks {
  void **ev;
  hipStream_t st;
  int mark(int i) const {
    if (ev && ev[i] && hipEventRecord(static_cast<hipEvent_t>(ev[i]), st) != hipSuccess)
      return COMPACTOR_EHIP;
    return COMPACTOR_OK;
  }
};
#define MARK(m, i)                       \
  do {                                   \
    const int rc_ = (m).mark(i);         \
    if (rc_ != COMPACTOR_OK) return rc_; \
  } while (0)

// score (+ blend) of one group.  With want_hist1 the per-pool histogram of the top 12 key bits
// of the final scores is left at gb.off_hist1() of the workspace (for the selection).
int enqueue_score(const compactor_params_t *p, const SegTable &T, long long rows, float *scores,
                  int32_t *status, unsigned char *ws, hipStream_t st, bool want_hist1) {
  const GroupBytes gb = group_bytes_needed(p, T, false);
  float *partials = reinterpret_cast<float *>(ws);
  uint16_t *wt = reinterpret_cast<uint16_t *>(ws + gb.off_wt());
  int *hist1 = want_hist1 ? reinterpret_cast<int *>(ws + gb.off_hist1()) : nullptr;
  double *ostat = gb.bstat ? reinterpret_cast<double *>(ws + gb.off_bstat()) : nullptr;
  // the histogram is cleared on the way, by the factorisation kernel
  int *zero = hist1;
  const long long zero_ints = hist1 ? (long long)T.nheads * HIST1_BINS : 0;
  const int cus = compute_units();
  const GramPlan gp = gram_plan(p, T, cus);
  const int rpw = gp.tiles_per_wg;
  const Marks m{p->stage_events, st};
  MARK(m, 0);
  HIP_TRY(launch_gram(T, gp.nwg, gp.tiles_per_wg, partials, st));
  MARK(m, COMPACTOR_STAGE_GRAM + 1);
  MARK(m, COMPACTOR_STAGE_REDUCE + 1);       // the fp64 sum of the partials is part of the next kernel
  if (p->sketch_dim > 0) {
    HIP_TRY(launch_sketch_solve(T, p->sketch_dim, rpw, partials, p->phi, p->ridge_rel, wt, status,
                                zero, zero_ints, st));
  } else {
    HIP_TRY(launch_exact_solve(T, rpw, partials, p->ridge_rel, wt, status, zero, zero_ints, st));
  }
  MARK(m, COMPACTOR_STAGE_SOLVE + 1);
  const int score_tokens = score_tokens_for(p, T, cus);
  HIP_TRY(launch_score(T, p->sketch_dim, score_tokens, wt, scores, status, hist1, ostat, st));
  MARK(m, COMPACTOR_STAGE_SCORE + 1);
  if (ostat != nullptr) {
    HIP_TRY(launch_blend(T, p->lambda_blend, score_tokens, scores, ostat, hist1, st));
  }
  MARK(m, COMPACTOR_STAGE_BLEND + 1);
  return COMPACTOR_OK;
}

// Scratch of compactor_compress_static: part of the device image, one copy per GPU.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device address it yields
// (per device) is what kernels, and everything else that touches the memory, are given.
constexpr size_t STATIC_SCRATCH_BYTES = COMPACTOR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each GPU, once looked up

// Address of the current device's copy of `scratch` (looked up once per device).
int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return COMPACTOR_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
      return COMPACTOR_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return COMPACTOR_OK;
}

// Argument checks of the fused call (everything but the workspace).
int check_compress(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                   const int32_t *kept_idx, const int32_t *kept_cnt, const void *k_packed,
                   const void *v_packed, const int32_t *status) {
  int rc = check_params(p, true);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, NEED_SCORE | NEED_PACK);
  if (rc) return rc;
  rc = check_scope(p, reqs, nreq);
  if (rc) return rc;
  if (!kept_idx || !kept_cnt || !k_packed || !v_packed || !status) return COMPACTOR_EINVAL;
  if (!aligned16(k_packed) || !aligned16(v_packed)) return COMPACTOR_EALIGN;
  return COMPACTOR_OK;
}

// score -> select -> gather of every head group on `st`, scratch in [workspace, +workspace_bytes).
int enqueue_compress(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                     float *scores, int32_t *kept_idx, int32_t *kept_cnt, void *k_packed,
                     void *v_packed, int32_t *status, void *workspace, size_t workspace_bytes,
                     hipStream_t st) {
  const bool local_scores = scores == nullptr;
  size_t need;
  const int rc = workspace_need(p, reqs, nreq, local_scores, &need);
  if (rc) return rc;
  if (!workspace || workspace_bytes < need) return COMPACTOR_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)) return COMPACTOR_EALIGN;
  drop_pending_error();
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  return for_each_group(p, reqs, nreq, group_rows_of(p), local_scores,
                        [&](const SegTable &T, long long rows) {
    float *sc = scores;
    const GroupBytes gb = group_bytes_needed(p, T, true);
    if (local_scores) sc = reinterpret_cast<float *>(ws + gb.off_scores());
    const int rc2 = enqueue_score(p, T, rows, sc, status, ws, st, true);
    if (rc2) return rc2;
    const Marks m{p->stage_events, st};
    int *hist1 = reinterpret_cast<int *>(ws + gb.off_hist1());
    if (select_needs_pools(T)) {
      int *sel = reinterpret_cast<int *>(ws + gb.off_sel());
      HIP_TRY(launch_select_pools(T, sc, hist1, true, sel, kept_idx, kept_cnt, st));
    } else {
      HIP_TRY(launch_select(T, sc, hist1, kept_idx, kept_cnt, st));
    }
    MARK(m, COMPACTOR_STAGE_SELECT + 1);
    HIP_TRY(launch_gather(T, kept_idx, kept_cnt, static_cast<uint16_t *>(k_packed),
                          static_cast<uint16_t *>(v_packed), st));
    MARK(m, COMPACTOR_STAGE_GATHER + 1);
    return (int)COMPACTOR_OK;
  });
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

void compactor_default_params(compactor_params_t *p, int32_t layers, int32_t kv_heads) {
  if (!p) return;
  memset(p, 0, sizeof(*p));
  p->layers = layers;
  p->kv_heads = kv_heads;
  p->head_dim = D;
  p->sketch_dim = 48;
  p->phi = nullptr;
  p->ridge_rel = 0.f;
  p->lambda_blend = 0.3f;
  p->group_bytes = 0;
  p->gram_wgs = 0;
  p->score_tokens = 0;
  p->select_scope = COMPACTOR_SCOPE_HEAD;
  p->stage_events = nullptr;
}

int32_t compactor_keep_count(int32_t n, float ratio) {
  if (n <= 0) return 0;
  const double x = ((double)ratio * (double)n) * (1.0 - 0x1p-23);
  double k = ceil(x);
  if (!(k >= 1.0)) k = 1.0;
  if (k > (double)n) k = (double)n;
  return (int32_t)k;
}

int compactor_layout(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                     int64_t *score_off, int64_t *kept_off, int32_t *k_keep) {
  int rc = check_params(p, false);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, 0);
  if (rc) return rc;
  const long long LH = (long long)p->layers * p->kv_heads;
  long long so = 0, ko = 0;
  for (int b = 0; b < nreq; ++b) {
    const int kk = compactor_keep_count(reqs[b].n, reqs[b].ratio);
    if (score_off) score_off[b] = so;
    if (kept_off) kept_off[b] = ko;
    if (k_keep) k_keep[b] = kk;
    so += LH * reqs[b].n;
    ko += LH * kk;
  }
  if (score_off) score_off[nreq] = so;
  if (kept_off) kept_off[nreq] = ko;
  return COMPACTOR_OK;
}

int compactor_srht_phi(int32_t sketch_dim, const uint8_t *signs, const int32_t *cols, float *phi,
                       void *stream) {
  if (!(sketch_dim == 16 || sketch_dim == 32 || sketch_dim == 48 || sketch_dim == 64))
    return COMPACTOR_EUNSUPPORTED;
  if (!signs || !cols || !phi) return COMPACTOR_EINVAL;
  if (!aligned16(phi)) return COMPACTOR_EALIGN;
  bool seen[D] = {false};
  for (int j = 0; j < sketch_dim; ++j) {
    if (cols[j] < 0 || cols[j] >= D || seen[cols[j]]) return COMPACTOR_EINVAL;
    seen[cols[j]] = true;
  }
  drop_pending_error();
  HIP_TRY(launch_srht_phi(sketch_dim, signs, cols, phi, static_cast<hipStream_t>(stream)));
  return COMPACTOR_OK;
}

int compactor_workspace_size(const compactor_params_t *p, const compactor_request_t *reqs,
                             int32_t nreq, size_t *bytes) {
  if (!bytes) return COMPACTOR_EINVAL;
  int rc = check_params(p, false);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, 0);
  if (rc) return rc;
  // sized for the fused call that keeps its scores in the workspace, the largest user
  return workspace_need(p, reqs, nreq, true, bytes);
}

int compactor_score(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                    float *scores, int32_t *status, void *workspace, size_t workspace_bytes,
                    void *stream) {
  int rc = check_params(p, true);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, NEED_SCORE);
  if (rc) return rc;
  if (!scores || !status) return COMPACTOR_EINVAL;
  size_t need;
  rc = workspace_need(p, reqs, nreq, false, &need);
  if (rc) return rc;
  if (!workspace || workspace_bytes < need) return COMPACTOR_EWORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)) return COMPACTOR_EALIGN;
  drop_pending_error();
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  return for_each_group(p, reqs, nreq, group_rows_of(p), false,
                        [&](const SegTable &T, long long rows) {
                          return enqueue_score(p, T, rows, scores, status, ws, st, false);
                        });
}

int compactor_select(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                     const float *scores, int32_t *kept_idx, int32_t *kept_cnt,
                     void *workspace, size_t workspace_bytes, void *stream) {
  int rc = check_params(p, false);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, 0);
  if (rc) return rc;
  rc = check_scope(p, reqs, nreq);
  if (rc) return rc;
  if (!scores || !kept_idx || !kept_cnt) return COMPACTOR_EINVAL;
  // only a pooled selection (long heads, layer scope) uses the workspace: its histograms
  const long long grows = group_rows_of(p);
  size_t need = 0;
  rc = for_each_group(p, reqs, nreq, grows, false, [&](const SegTable &T, long long) {
    if (select_needs_pools(T)) {
      const GroupBytes gb = group_bytes_needed(p, T, false);
      if (gb.hist1 + gb.sel > need) need = gb.hist1 + gb.sel;
    }
    return COMPACTOR_OK;
  });
  if (rc) return rc;
  if (need > 0) {
    if (!workspace || workspace_bytes < need) return COMPACTOR_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & (WS_ALIGN - 1)) return COMPACTOR_EALIGN;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  drop_pending_error();
  return for_each_group(p, reqs, nreq, grows, false, [&](const SegTable &T, long long) {
    if (select_needs_pools(T)) {
      const GroupBytes gb = group_bytes_needed(p, T, false);
      int *hist1 = static_cast<int *>(workspace);
      int *sel = reinterpret_cast<int *>(static_cast<unsigned char *>(workspace) + gb.hist1);
      HIP_TRY(launch_select_pools(T, scores, hist1, false, sel, kept_idx, kept_cnt, st));
    } else {
      HIP_TRY(launch_select(T, scores, nullptr, kept_idx, kept_cnt, st));
    }
    return COMPACTOR_OK;
  });
}

int compactor_compact(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                      const int32_t *kept_idx, const int32_t *kept_cnt, void *k_packed,
                      void *v_packed, void *stream) {
  int rc = check_params(p, false);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, NEED_PACK);
  if (rc) return rc;
  rc = check_scope(p, reqs, nreq);
  if (rc) return rc;
  if (!kept_idx || !kept_cnt || !k_packed || !v_packed) return COMPACTOR_EINVAL;
  if (!aligned16(k_packed) || !aligned16(v_packed)) return COMPACTOR_EALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  drop_pending_error();
  return for_each_group(p, reqs, nreq, 1ll << 60, false, [&](const SegTable &T, long long) {
    HIP_TRY(launch_gather(T, kept_idx, kept_cnt, static_cast<uint16_t *>(k_packed),
                          static_cast<uint16_t *>(v_packed), st));
    return COMPACTOR_OK;
  });
}

int compactor_compact_paged(const compactor_params_t *p, const compactor_request_t *reqs,
                            int32_t nreq, const int32_t *kept_idx, const int32_t *kept_cnt,
                            const compactor_page_pool_t *pool, const compactor_page_table_t *tables,
                            int32_t in_place, void *stream) {
  int rc = check_params(p, false);
  if (rc) return rc;
  rc = check_requests(reqs, nreq, in_place ? 0 : NEED_PACK);
  if (rc) return rc;
  rc = check_scope(p, reqs, nreq);
  if (rc) return rc;
  if (!kept_idx || !kept_cnt || !pool || !tables) return COMPACTOR_EINVAL;
  if (!pool->k_pages || !pool->v_pages || pool->page_size < 1 || pool->num_pages < 1)
    return COMPACTOR_EINVAL;
  if (pool->page_stride < 0 || pool->layer_stride < 0 || pool->head_stride < 0 ||
      pool->slot_stride < D)
    return COMPACTOR_EINVAL;
  if (!aligned16(pool->k_pages) || !aligned16(pool->v_pages) ||
      ((pool->page_stride | pool->layer_stride | pool->head_stride | pool->slot_stride) & 7))
    return COMPACTOR_EALIGN;
  for (int b = 0; b < nreq; ++b) {
    // logical pages a head can need: all its tokens when they are read from the pages, else
    // what it can retain (in layer scope one head may take the whole layer's budget)
    const long long kk = compactor_keep_count(reqs[b].n, reqs[b].ratio);
    long long rows = p->select_scope == COMPACTOR_SCOPE_LAYER ? kk * p->kv_heads : kk;
    if (rows > reqs[b].n || in_place) rows = reqs[b].n;
    if (!tables[b].pages || tables[b].len < (rows + pool->page_size - 1) / pool->page_size)
      return COMPACTOR_EINVAL;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  drop_pending_error();
  return for_each_group(p, reqs, nreq, 1ll << 60, false, [&](const SegTable &T, long long) {
    PagePool P;
    memset(&P, 0, sizeof(P));
    P.k = static_cast<uint16_t *>(pool->k_pages);
    P.v = static_cast<uint16_t *>(pool->v_pages);
    P.page_stride = pool->page_stride; P.layer_stride = pool->layer_stride;
    P.head_stride = pool->head_stride; P.slot_stride = pool->slot_stride;
    P.page_size = pool->page_size; P.num_pages = pool->num_pages;
    for (int i = 0; i < T.nseg; ++i) {
      P.t[i].pages = tables[T.s[i].req].pages;
      P.t[i].len = tables[T.s[i].req].len;
    }
    HIP_TRY(launch_gather_paged(T, P, kept_idx, kept_cnt, in_place != 0, st));
    return COMPACTOR_OK;
  });
}

int compactor_compress(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                       float *scores, int32_t *kept_idx, int32_t *kept_cnt, void *k_packed,
                       void *v_packed, int32_t *status, void *workspace, size_t workspace_bytes,
                       void *stream) {
  const int rc = check_compress(p, reqs, nreq, kept_idx, kept_cnt, k_packed, v_packed, status);
  if (rc) return rc;
  return enqueue_compress(p, reqs, nreq, scores, kept_idx, kept_cnt, k_packed, v_packed, status,
                          workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int compactor_compress_static(const compactor_params_t *p, const compactor_request_t *reqs,
                              int32_t nreq, float *scores, int32_t *kept_idx, int32_t *kept_cnt,
                              void *k_packed, void *v_packed, int32_t *status, void *stream) {
  int rc = check_compress(p, reqs, nreq, kept_idx, kept_cnt, k_packed, v_packed, status);
  if (rc) return rc;
  size_t need;
  rc = workspace_need(p, reqs, nreq, scores == nullptr, &need);
  if (rc) return rc;
  if (need > STATIC_SCRATCH_BYTES) return COMPACTOR_EWORKSPACE;
  drop_pending_error();
  void *ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc) return rc;
  return enqueue_compress(p, reqs, nreq, scores, kept_idx, kept_cnt, k_packed, v_packed, status,
                          ptr, STATIC_SCRATCH_BYTES, static_cast<hipStream_t>(stream));
}

double compactor_calibrated_ratio(double nll, double alpha, double beta, double tau) {
  const double b = alpha * nll + beta;
  double r = (b == 0.0) ? tau : 1.0 + log(tau * (1.0 - exp(-b)) + exp(-b)) / b;
  if (!(r > 0.0)) r = 4.9406564584124654e-324;
  if (r > 1.0) r = 1.0;
  return r;
}

const char *compactor_error_string(int code) {
  switch (code) {
    case COMPACTOR_OK: return "ok";
    case COMPACTOR_EINVAL: return "invalid argument";
    case COMPACTOR_EUNSUPPORTED: return "unsupported shape (head_dim must be 128; sketch_dim 0, 16, 32, 48 or 64)";
    case COMPACTOR_EWORKSPACE: return "workspace missing or too small (or the batch needs more than the static scratch)";
    case COMPACTOR_EALIGN: return "pointer or stride not 16-byte aligned";
    case COMPACTOR_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char *compactor_version(void) { return "0.1"; }

#pragma GCC visibility pop
}  // extern "C"
