/*
 * compactor.h -- C boundary of the MI355X (gfx950) Compactor hot path.
 *
 * Compactor is a query-agnostic KV-cache eviction method: every cached token of
 * every (layer, kv-head) gets an importance score, the top ceil(r*N) tokens per
 * head are retained, and their key/value rows form the compressed cache
 * (paper Sec. 3, "Preliminaries & Overview").  This library runs that path on
 * one GPU:
 *
 *   score    outlier scores o = approximate statistical leverage scores of the
 *            head's key matrix (Sec. 3.1 Definition 1 and Eq. "fast_svd";
 *            Sec. 3.2 Algorithm 1), optionally blended with caller-supplied
 *            attention scores a as s = z(a) + lambda*z(o) (Sec. 3.3 Eq. "scoring")
 *   select   per-head top-ceil(r*N) of s (Sec. 3.3, "KV selection")
 *   compact  gather of the retained K/V rows into a packed cache
 *   compress the three fused on one stream
 * and, beyond that path: the attention-based scores a themselves (Sec. 3.2), head-adaptive
 * selection across the heads of a layer (Sec. 3.3), a paged destination for the compaction,
 * and the Hadamard right-sketch of App. D.
 *
 * General conventions
 *   - Every pointer marked "device" is GPU memory owned by the caller; every
 *     pointer marked "host" is ordinary host memory owned by the caller.  The
 *     library never allocates, frees or synchronises: all work is enqueued on
 *     the stream that is passed in (a hipStream_t cast to void*, NULL = the
 *     default stream), and outputs are valid once that stream has drained.
 *   - Keys and values are bfloat16 (raw 16-bit patterns), head_dim contiguous.
 *   - Heads are numbered request-major: head g = (sum of L*H of earlier
 *     requests) + layer*H + kv_head.  All per-head outputs use this order and
 *     the element offsets reported by compactor_layout().
 *   - Return value: COMPACTOR_OK or a negative COMPACTOR_E* code.  Errors are
 *     detected on the host before anything is enqueued; a failing call leaves
 *     the outputs untouched.  Numerical trouble inside a head never aborts: it
 *     is reported in that head's status word (see COMPACTOR_STATUS_*).
 *   - Thread safety: concurrent calls are safe when they use distinct workspaces
 *     and output buffers; the library keeps no state between calls (but see
 *     compactor_compress_static, whose scratch is shared per GPU).
 */
#ifndef COMPACTOR_H
#define COMPACTOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COMPACTOR_OK                   0
#define COMPACTOR_EINVAL             (-1)  /* null pointer, n <= 0, ratio outside (0,1], ... */
#define COMPACTOR_EUNSUPPORTED       (-2)  /* head_dim != 128, sketch_dim not in {0,16,32,48,64} */
#define COMPACTOR_EWORKSPACE         (-3)  /* workspace pointer null or too small; or the batch needs
                                              more scratch than compactor_compress_static has */
#define COMPACTOR_EALIGN             (-4)  /* a pointer or a row stride is not 16-byte aligned */
#define COMPACTOR_EHIP               (-5)  /* a HIP runtime call of the library failed (launch error);
                                              an error that earlier HIP calls of the caller left
                                              pending on the thread is discarded, not reported */

/* per-head status bits written by the scoring step */
#define COMPACTOR_STATUS_OK            0
#define COMPACTOR_STATUS_PIVOT         1   /* the factored Gram matrix was numerically singular:
                                              the offending direction was dropped */
#define COMPACTOR_STATUS_NONFINITE     2   /* a non-finite score was produced (non-finite input) */

/* One request = one context whose cache is compressed (Sec. 3: K, V in R^{N x d}
 * per head; retention r in (0,1]). */
typedef struct compactor_request {
  const void  *k_score;   /* device, bf16 [L,H,n,d]: keys that are scored.  The paper scores the
                             keys before positional encoding (Sec. 3.1/3.2). */
  const void  *k_cache;   /* device, bf16 [L,H,n,d]: keys that are packed (the cached, position-
                             encoded keys); NULL = pack k_score. Same strides as k_score. */
  const void  *v_cache;   /* device, bf16 [L,H,n,d]: values that are packed. Same strides. */
  const float *attn;      /* device, fp32 [L,H,n] contiguous attention scores a, or NULL.
                             NULL gives s = o, the paper's "only o" variant. */
  int64_t stride_l;       /* element strides of the three bf16 tensors; d has stride 1 */
  int64_t stride_h;
  int64_t stride_t;       /* >= head_dim and a multiple of 8 elements (16 bytes) */
  int32_t n;              /* tokens N in this context, 1 <= n < 2^31 - 64 */
  float   ratio;          /* retention r in (0,1], requested or context-calibrated (Sec. 3.4) */
} compactor_request_t;

typedef struct compactor_params {
  int32_t layers;         /* L >= 1 */
  int32_t kv_heads;       /* H >= 1 */
  int32_t head_dim;       /* d; 128 is the only supported value */
  int32_t sketch_dim;     /* k_s of Algorithm 1: 16, 32, 48 (paper default) or 64;
                             0 = exact leverage scores (no sketch, Definition 1) */
  const float *phi;       /* device, fp32 [d, k_s] row-major right-sketch Phi, entries
                             N(0, 1/k_s) (Algorithm 1 line 1); drawn by the caller so that the
                             library holds no random state.  Ignored when sketch_dim = 0. */
  float   ridge_rel;      /* >= 0.  rho = ridge_rel * trace(M)/order(M) is added to the diagonal
                             of the Gram matrix M that is factored (M = Phi^T K^T K Phi, or
                             K^T K in exact mode).  0 is Algorithm 1 as printed. */
  float   lambda_blend;   /* lambda of Eq. "scoring" (paper default 0.3); used only where
                             attn != NULL */
  int64_t group_bytes;    /* heads are processed in groups whose keys total about this many bytes,
                             one launch sequence per group: bounds the workspace (sized for the
                             largest group).  0 = one group.  Not a speed knob: on MI355X a second
                             pass that finds a group's keys in the last-level cache is no faster
                             than one that streams them from HBM. */
  int32_t gram_wgs;       /* tuning: workgroups of the persistent Gram kernel and target tokens */
  int32_t score_tokens;   /* per workgroup of the score kernel (at most 32768; larger values are
                             clamped); 0 = chosen by the library */
  int32_t select_scope;   /* COMPACTOR_SCOPE_HEAD (default): every head keeps its own top k_keep.
                             COMPACTOR_SCOPE_LAYER: head-adaptive selection (Sec. 3.3, retain the
                             top scores "across all heads"; the paper's experiments, Sec. 4): the
                             H kv heads of a layer share one budget of H*k_keep tokens, taken from
                             the H*n scores of the layer wherever they fall; equal scores go to
                             the lower (head, token) position.  Needs H*n < 2^31 - 64.  Heads
                             then keep different numbers of tokens: see compactor_select. */
  void  **stage_events;   /* profiling aid, normally NULL.  host array of COMPACTOR_NUM_STAGES+1
                             hipEvent_t created by the caller: event[0] is recorded on the stream
                             before the first kernel of a group and event[i+1] after stage i's
                             kernel (COMPACTOR_STAGE_*), so hipEventElapsedTime(event[i],
                             event[i+1]) is stage i's duration.  With several groups the events
                             hold the last group's times.  Stages a call does not run leave
                             their events unrecorded. */
} compactor_params_t;

#define COMPACTOR_SCOPE_HEAD    0
#define COMPACTOR_SCOPE_LAYER   1

/* stage indices for compactor_params_t.stage_events */
#define COMPACTOR_STAGE_GRAM     0   /* partial Gram matrices K^T K (MFMA) */
#define COMPACTOR_STAGE_REDUCE   1   /* fp64 sum of the partials */
#define COMPACTOR_STAGE_SOLVE    2   /* sketch, Cholesky, W */
#define COMPACTOR_STAGE_SCORE    3   /* o_i = ||W^T k_i||^2 (MFMA) */
#define COMPACTOR_STAGE_BLEND    4   /* Eq. "scoring" (only with attn) */
#define COMPACTOR_STAGE_SELECT   5   /* per-head top-k */
#define COMPACTOR_STAGE_GATHER   6   /* packed K/V rows */
#define COMPACTOR_NUM_STAGES     7

/* Fills *p with the paper's defaults (Sec. 4: k = 48, lambda = 0.3), d = 128,
 * ridge_rel = 0, phi = NULL.  host. */
void compactor_default_params(compactor_params_t *p, int32_t layers, int32_t kv_heads);

/* k_keep = clamp(ceil(r*N), 1, N) (Sec. 3: "top-k with k = ceil(r N)").  r is widened to
 * double and the product shrunk by (1 - 2^-23) before the ceiling, so that a float32 ratio whose
 * product with N is an integer on paper (r = 0.001f, N = 1000) does not round up to the next
 * integer.  The price: a product that lies less than r*N*2^-23 above an integer is taken for
 * that integer, so for an arbitrary float ratio k_keep is ceil(r*N) - 1 in about 2 of 1000
 * (r, N) pairs and ceil(r*N) otherwise.  Returns 0 for n <= 0. host. */
int32_t compactor_keep_count(int32_t n, float ratio);

/* Element offsets of each request inside the flat output buffers. host.
 *   score_off[b]  offset (floats)  of request b in scores:   prefix sum of L*H*n_b
 *   kept_off[b]   offset (rows)    of request b in kept_idx / k_packed / v_packed:
 *                 prefix sum of L*H*k_keep_b; within a request, head (l,h) starts at
 *                 kept_off[b] + (l*H+h)*k_keep_b
 *   k_keep[b]     retained tokens per head of request b
 * score_off and kept_off have nreq+1 entries (the last is the total); k_keep has nreq.
 * Any of the three may be NULL. */
int compactor_layout(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                     int64_t *score_off, int64_t *kept_off, int32_t *k_keep);

/* Fills phi with the subsampled randomized Hadamard right-sketch of App. D,
 * Phi = (sqrt(d/k_s) R H D)^T: phi[i*k_s + j] = sqrt(d/k_s) * (signs[i] ? -1 : +1) * H[cols[j]][i],
 * H the +-1 Walsh-Hadamard matrix of order d = 128 (H[a][b] = (-1)^popcount(a & b)).  An
 * alternative to a Gaussian phi for compactor_params_t.phi; the random choices are the caller's.
 *   signs  host, uint8 [128]: the Rademacher diagonal D (nonzero = -1)
 *   cols   host, int32 [k_s]: the k_s rows of H that R selects, distinct, in [0, 128)
 *   phi    device, fp32 [128, k_s], written on `stream`
 * k_s in {16, 32, 48, 64}.  The host arrays are consumed before the call returns. */
int compactor_srht_phi(int32_t sketch_dim, const uint8_t *signs, const int32_t *cols, float *phi,
                       void *stream);

/* Bytes of device workspace that score / select / compress need for this batch. host.
 * The workspace must be 256-byte aligned; its contents are scratch (no state is kept
 * between calls).  The size depends on the number of compute units of the current HIP device
 * (it sets the number of partial Gram matrices): ask with the device current that will run the
 * call.  Where no device can be queried the size for 256 compute units (MI355X) is returned. */
int compactor_workspace_size(const compactor_params_t *p, const compactor_request_t *reqs,
                             int32_t nreq, size_t *bytes);

/* Scores every token of every head.
 *   scores  device, fp32 [sum_b L*H*n_b] at compactor_layout's score_off: s (= o when a request
 *           has attn == NULL, else Eq. "scoring")
 *   status  device, int32 [nreq*L*H]: COMPACTOR_STATUS_* bits per head
 * Sec. 3.1-3.3; Algorithm 1 evaluated as o_i = ||L^{-1} Phi^T k_i||^2 with
 * L L^T = Phi^T K^T K Phi + rho I, equal to diag(U~ U~^T) of Algorithm 1 when rho = 0. */
int compactor_score(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                    float *scores, int32_t *status, void *workspace, size_t workspace_bytes,
                    void *stream);

/* Per-head top-k_keep of the given scores (Sec. 3.3 step 2, selection "within a single head").
 *   scores    device, fp32, layout as written by compactor_score
 *   kept_idx  device, int32 [sum_b L*H*k_keep_b] at kept_off: token indices of the retained
 *             tokens of each head, ascending
 *   kept_cnt  device, int32 [nreq*L*H]: number of indices written per head (= k_keep_b)
 * Order: higher score first, equal scores by lower token index; NaN ranks below every number
 * and -0.0 equals +0.0.  The reqs' tensors are not read, only n and ratio.
 * Layer scope (params.select_scope): the region of layer l of request b, kept_off[b] + l*H*k_keep_b
 * .. + H*k_keep_b, holds the retained tokens of head 0 (ascending), then head 1, and so on,
 * kept_cnt[b][l][h] of them for head h (any number from 0 to n; they add up to H*k_keep_b).
 * compactor_compact packs rows in the same ragged order.
 * workspace: needed (size: compactor_workspace_size) in layer scope or when a head has more than
 * 32768 tokens; may be NULL otherwise. */
int compactor_select(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                     const float *scores, int32_t *kept_idx, int32_t *kept_cnt,
                     void *workspace, size_t workspace_bytes, void *stream);

/* Gathers the retained rows: k_packed[row j of head g] = k_cache[kept_idx[j]], same for v.
 *   k_packed, v_packed  device, bf16 [sum_b L*H*k_keep_b, d] dense rows at kept_off
 * Bit copies.  An index outside [0, n) is a caller error; such a row is written as zeros. */
int compactor_compact(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                      const int32_t *kept_idx, const int32_t *kept_cnt,
                      void *k_packed, void *v_packed, void *stream);

/* ---- paged cache as the compaction target ------------------------------------------------- */
/* Serving engines keep the cache in fixed-size pages named by a block table per context; the
 * compressed cache (Sec. 3: the retained key/value pairs) can be written there directly, or an
 * existing paged cache can be compacted in place so that its tail pages can be released. */
typedef struct compactor_page_pool {
  void *k_pages;          /* device, bf16.  Element (page p, layer l, kv head h, slot s, channel c) */
  void *v_pages;          /* is at p*page_stride + l*layer_stride + h*head_stride + s*slot_stride + c */
  int64_t page_stride, layer_stride, head_stride, slot_stride;   /* elements, multiples of 8;
                             slot_stride >= head_dim.  E.g. a [pages, page_size, H, d] pool per
                             layer has slot_stride = H*d, head_stride = d. */
  int32_t page_size;      /* slots (tokens) per page, >= 1 */
  int32_t num_pages;      /* pages in the pool; a table entry outside [0, num_pages) is skipped */
} compactor_page_pool_t;

typedef struct compactor_page_table {
  const int32_t *pages;   /* device, int32 [len]: physical page of logical page i of this context.
                             The pages of one context must be distinct. */
  int32_t len;
} compactor_page_table_t;

/* compactor_compact with a paged destination: retained token j of head (l,h) of request b goes to
 * logical slot j of that head, i.e. page tables[b].pages[j / page_size], slot j % page_size
 * (in layer scope j counts inside the head: 0 .. kept_cnt-1).  Slots that receive no row keep
 * their contents.  tables: host array of nreq entries.
 * in_place = 0: rows are read from the requests' k_cache / v_cache tensors as in compactor_compact.
 * in_place = 1: rows are read from the pool itself, token t of a head at logical slot t (the
 *   requests' tensors are not used and may be NULL); afterwards the first ceil(count / page_size)
 *   logical pages hold the head and the others can be released.  kept_idx must be ascending
 *   per head (as compactor_select writes it); an entry below its own rank is skipped.
 * tables[b].len must cover ceil(rows / page_size) logical pages, rows = n_b when in place, else
 * k_keep_b (layer scope: min(n_b, H*k_keep_b), since one head may take the whole budget).
 * For callers whose cache is paged; no part of the paper. */
int compactor_compact_paged(const compactor_params_t *p, const compactor_request_t *reqs,
                            int32_t nreq, const int32_t *kept_idx, const int32_t *kept_cnt,
                            const compactor_page_pool_t *pool, const compactor_page_table_t *tables,
                            int32_t in_place, void *stream);

/* score -> select -> compact on one stream, with no host synchronisation in between.
 * scores may be NULL (they then live in the workspace only). */
int compactor_compress(const compactor_params_t *p, const compactor_request_t *reqs, int32_t nreq,
                       float *scores, int32_t *kept_idx, int32_t *kept_cnt,
                       void *k_packed, void *v_packed, int32_t *status,
                       void *workspace, size_t workspace_bytes, void *stream);

/* compactor_compress without a workspace argument, for callers that cannot allocate device memory
 * or obtain a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The scratch that compactor_compress takes as `workspace` lives in a buffer of
 * COMPACTOR_STATIC_SCRATCH_BYTES that is part of the library's device image: every GPU the
 * library runs on holds its own copy from the first use until the process ends.  The call
 * allocates and frees nothing (no hipMalloc, no hipFree, no allocating library routine); inputs
 * and outputs are the caller's, as in compactor_compress, and the results are the same bits.
 * A batch whose scratch (compactor_workspace_size; pass scores != NULL to keep the scores out of
 * it) exceeds COMPACTOR_STATIC_SCRATCH_BYTES is refused with COMPACTOR_EWORKSPACE before anything
 * is enqueued; params.group_bytes bounds the scratch of a large batch.  All calls on one GPU share
 * that GPU's buffer: calls that overlap in time on one GPU (two streams, two threads) race on it
 * and must be serialised by the caller.  The buffer keeps the last call's contents; whatever has
 * to start at zero is cleared by the call's own kernels.  The first call on a device looks the
 * buffer's address up (no stream work): make it outside a graph capture. */
#define COMPACTOR_STATIC_SCRATCH_BYTES (64u << 20)
int compactor_compress_static(const compactor_params_t *p, const compactor_request_t *reqs,
                              int32_t nreq, float *scores, int32_t *kept_idx, int32_t *kept_cnt,
                              void *k_packed, void *v_packed, int32_t *status, void *stream);

/* ---- attention-based scores (Sec. 3.2, "Attention-Based Scoring") ------------------------- */

/* One context: the queries and keys its attention scores are computed from. */
typedef struct compactor_attn_request {
  const void *q;          /* device, bf16 [L, Hq, n, d]: queries (as the model's attention sees
                             them, i.e. position-encoded), d contiguous */
  const void *k;          /* device, bf16 [L, H, n, d]: keys (likewise) */
  int64_t q_stride_l, q_stride_h, q_stride_t;   /* element strides, multiples of 8 */
  int64_t k_stride_l, k_stride_h, k_stride_t;
  int32_t n;              /* tokens */
} compactor_attn_request_t;

typedef struct compactor_attn_params {
  int32_t layers;         /* L */
  int32_t kv_heads;       /* H */
  int32_t q_heads;        /* Hq, a multiple of H: query heads h*G .. h*G+G-1 share kv head h */
  int32_t head_dim;       /* 128 */
  int32_t chunk;          /* block size C of Sec. 3.2; 256 (the paper's value) is supported */
  int32_t pool;           /* mean-pooling window along the sequence: odd, 1..63; 1 = none */
  float   scale;          /* logit scale; 0 = 1/sqrt(head_dim) */
} compactor_attn_params_t;

/* Bytes of device workspace compactor_attention_scores needs (the unpooled sums). host. */
int compactor_attention_workspace_size(const compactor_attn_params_t *p,
                                       const compactor_attn_request_t *reqs, int32_t nreq,
                                       size_t *bytes);

/* a = concat_i 1^T softmax(scale * Q[i] K[i]^T) over blocks i of `chunk` consecutive positions
 * (non-causal inside a block; the last block may be shorter), averaged over the query heads of
 * each kv head, then mean-pooled with window `pool` (stride 1, zero padding, divided by pool,
 * as SnapKV pools its scores).
 *   attn  device, fp32 [sum_b L*H*n_b], request b at the prefix sum of L*H*n_b (the layout of
 *         the scores buffer): pass attn + offset_b as compactor_request_t.attn.
 * The group average and the pooling width are this library's readings of passages the paper
 * leaves open. */
int compactor_attention_scores(const compactor_attn_params_t *p,
                               const compactor_attn_request_t *reqs, int32_t nreq, float *attn,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Context-calibrated retention (Sec. 3.4): the smallest r in (0,1] with
 * f(r) = (exp(r b - b) - exp(-b)) / (1 - exp(-b)) >= tau, b = alpha*nll + beta, i.e.
 * r* = 1 + ln(tau (1 - e^-b) + e^-b) / b (r* = tau in the limit b -> 0). host. */
double compactor_calibrated_ratio(double nll, double alpha, double beta, double tau);

/* Human-readable text for a return code. host; the string is static. */
const char *compactor_error_string(int code);

/* Library version, "major.minor". host; static string. */
const char *compactor_version(void);

#ifdef __cplusplus
}
#endif
#endif /* COMPACTOR_H */
