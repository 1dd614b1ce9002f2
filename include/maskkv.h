/*
 * maskkv.h - C ABI of the MaskKV eviction hot path for AMD MI355X (gfx950).
 *
 * The library implements, for one transformer layer at a time, the data-parallel steps
 * of MaskKV (arXiv 2510.09309, Section 3.3 "The MaskKV Framework"):
 *
 *   maskkv_score    Stage 1 "Mask-Voting": A = softmax_row(Q_mask K_full^T / sqrt(d_k)),
 *                   I_j = sum_i A_ij for the prompt tokens j.
 *   maskkv_select   S_keep = argtopk(I, k_{l,h}) per (layer, head) with ragged budgets
 *                   (last equation of Stage 2), after an optional smoothing window.
 *   maskkv_compact  eviction: the cache keeps only the selected prompt K/V rows
 *                   (appendix "Prompt-state Exclusion": only prompt K/V are cached).
 *   maskkv_attend   bidirectional attention of the response span over
 *                   [kept prompt KV ; response KV] (layer forward equation, Section 3.1;
 *                   appendix proof: AttnOut_m = sum_j alpha_mj V_j).
 *   maskkv_attend_full   the same attention over the un-evicted sequence (the cost the
 *                   eviction removes; used for the speed-up figure).
 *   maskkv_head_budgets  Stage 2, head level: prompt preference P_h and
 *                   k_{l,h} = floor(alpha k_l + (1-alpha) N_h k_l P_h / sum_j P_j).
 *   maskkv_layer_importance, maskkv_layer_budgets   Stage 2, layer level: I^(l) = 1 - mean
 *                   cosine similarity of the attention sub-layer's input and output states, and
 *                   the boundary-aware split of the total budget over the layers.
 *   maskkv_value_shift   Section 3.1 (feature-cache background): response tokens whose value
 *                   vector turned by more than a threshold between two denoising steps.
 *
 * Conventions
 *  - Every pointer marked DEVICE must be device memory reachable from the current HIP
 *    device; pointers marked HOST are ordinary host memory read during the call only.
 *  - The library never allocates, frees or synchronises.  All work is enqueued on the
 *    given stream (a hipStream_t passed as void*; NULL is the default stream).  The
 *    caller owns every buffer, including the workspace, and must keep it alive until the
 *    stream has drained.  Inputs are never modified; outputs are fully overwritten in
 *    their valid region.
 *  - Every function returns a maskkv_status.  On any status other than MASKKV_OK nothing
 *    has been enqueued.  maskkv_last_error() gives a per-thread detail string.
 *  - Sequences: batch item b has P_b prompt tokens followed by n_resp response-span
 *    tokens (N_b = P_b + n_resp keys).  Key/value heads are independent.
 *  - Grouped-query attention (the Dream-7B model of Section 4.1): desc->H counts KEY/VALUE
 *    heads and desc->q_per_kv = g > 1 says that query heads h*g .. h*g+g-1 read KV head h.
 *    Views of queries and outputs (Q_mask, Q_resp, O) then have H*g heads, lse has
 *    B*H*g*n_resp entries, and everything per head (scores, prompt_mass, budgets, cu_budget,
 *    the cache, K and V views) stays per KV head.  The paper does not say how votes map to a
 *    shared KV head; here every mask query of every query head in the group votes
 *    (scores = sum over the group of the per-head column sums).  g <= 64.
 */
#ifndef MASKKV_H
#define MASKKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MASKKV_VERSION 1
#define MASKKV_MAX_BATCH 64 /* per call; split larger batches */

typedef enum maskkv_status {
  MASKKV_OK = 0,
  MASKKV_EINVAL = 1,     /* null pointer, negative size, bad window, bad stride, ... */
  MASKKV_ESHAPE = 2,     /* unsupported head_dim (64 and 128 are supported) or batch too large */
  MASKKV_EDTYPE = 3,     /* dtype is neither MASKKV_F32 nor MASKKV_BF16 */
  MASKKV_EWORKSPACE = 4, /* workspace missing or smaller than maskkv_*_workspace_bytes */
  MASKKV_EHIP = 5,       /* a HIP launch failed; detail string carries hipGetErrorString */
  MASKKV_ECAPACITY = 6   /* (host-checkable) output capacity too small */
} maskkv_status;

typedef enum maskkv_dtype { MASKKV_F32 = 0, MASKKV_BF16 = 1 } maskkv_dtype;

typedef enum maskkv_pool_mode { MASKKV_POOL_MEAN = 0, MASKKV_POOL_MAX = 1 } maskkv_pool_mode;

/*
 * A 4-D view [B, H, T, d] of Q, K, V or O in DEVICE memory.  Element (b, h, t, e) lives at
 *   ptr + ((b*stride_b + h*stride_h + (seq_start[b] + t)*stride_t + e) * sizeof(element)),
 * strides in elements, the head_dim axis contiguous.  Rows must be 16-byte aligned
 * (ptr and all strides multiples of 16 bytes) and stride_t may not exceed 16 MiB in bytes
 * (MASKKV_EINVAL otherwise).  [B,H,T,d], [B,T,H,d] and packed
 * variable-length [T_total,H,d] (stride_b = 0 with seq_start) are all expressible.
 */
typedef struct maskkv_tensor {
  void* ptr;             /* DEVICE */
  int64_t stride_b;
  int64_t stride_h;
  int64_t stride_t;
  const int32_t* seq_start; /* HOST [B] token offset of each sequence on the T axis, or NULL for 0 */
} maskkv_tensor;

/* Problem description shared by all calls. */
typedef struct maskkv_desc {
  int32_t B;        /* sequences in the batch, 1..MASKKV_MAX_BATCH */
  int32_t H;        /* attention heads */
  int32_t d;        /* head_dim: 64 or 128 */
  int32_t dtype;    /* maskkv_dtype of Q, K, V, the cache and O */
  int32_t n_resp;   /* response-span length n_m: response keys per sequence; queries in attend */
  int32_t n_query;  /* mask queries per query head that vote in maskkv_score (normally n_resp; a sub-span,
                       e.g. only the late response positions of the position-aware voting study, is
                       expressed by pointing Q_mask at its first row) */
  int32_t P_max;    /* longest prompt in the batch */
  int32_t q_per_kv; /* grouped-query attention: query heads per key/value head; 0 or 1 = one each (MHA) */
  const int32_t* prompt_len; /* HOST [B] prompt lengths P_b in 0..P_max, or NULL: every P_b = P_max */
} maskkv_desc;

/* Library version (MASKKV_VERSION of the build). */
int maskkv_version(void);
/* Static string for a status code. */
const char* maskkv_strerror(int status);
/* Detail of the calling thread's most recent failure ("" if none). */
const char* maskkv_last_error(void);

/*
 * Workspace (DEVICE bytes) needed by maskkv_score for this description.  The workspace
 * holds per-key-segment softmax row statistics between the two passes and, with more than
 * 256 voting rows per head, the column sums of every group of 256 rows; contents are
 * scratch.  The size depends on prompt_len: query it with the description the call will
 * use.  256-byte alignment is required.
 */
int maskkv_score_workspace_bytes(const maskkv_desc* desc, size_t* bytes);

/*
 * Stage 1, Mask-Voting.  For every (b, h):
 *   A = softmax over all N_b keys of (Q_mask[b,h] K_full[b,h]^T * scale)   (no mask)
 *   scores[(b*H + h)*score_stride + j] = sum_{i < n_query} A[i, j],  j in [0, P_b)
 *                          (summed over the g query heads of the group too when q_per_kv = g > 1)
 *   prompt_mass[b*H + h] = sum_{j < P_b} scores[..j]   (the mask-to-prompt attention sum
 *                          S_{m->p} of the prompt-preference metric), if not NULL.
 * Q_mask: view [B, H*g, n_query, d].  K_full: view [B, H, N_b, d], prompt rows then
 * response rows.  scale <= 0 selects 1/sqrt(d).  scores: DEVICE float, score_stride >=
 * P_max; entries j >= P_b are left untouched.  Accumulation is fp32 throughout.
 */
int maskkv_score(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                 float scale, float* scores, int64_t score_stride, float* prompt_mass,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Mask-Voting when the softmax normaliser of every voting row is already known.  At the initial inference step
 * (the step whose mask queries vote, Stage 1) the model's own attention over the un-evicted sequence forms the
 * same logits over the same keys, and a flash-style attention call returns each row's log-sum-exp: given those,
 * the scores need one sweep over the keys instead of two.
 *   row_lse[(b*H + h)*g*n_query + r] = log sum_j exp(q_r . k_j * scale)   (natural log, all N_b keys)
 * for voting row r of key/value head h (rows numbered as the rows of Q_mask: query head first, then query) - the
 * layout in which maskkv_attend_full writes `lse` when it is called with the same queries (n_query = n_resp) and
 * the same scale.  scores and prompt_mass as for maskkv_score; they equal its results up to the rounding of the
 * normalisers.  workspace: maskkv_score_workspace_bytes (only the part for more than 256 voting rows is used).
 */
int maskkv_score_given_lse(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                           float scale, const float* row_lse, float* scores, int64_t score_stride,
                           float* prompt_mass, void* workspace, size_t workspace_bytes, void* stream);

/*
 * maskkv_score for callers that cannot allocate device memory or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and same result as maskkv_score, but the
 * scratch between the passes lives in an array of MASKKV_STATIC_SCRATCH_BYTES that is part of the library image
 * (every GPU the library runs on holds its own copy until the process ends).  The call allocates and frees
 * nothing.  Descriptions whose maskkv_score_workspace_bytes exceed MASKKV_STATIC_SCRATCH_BYTES are rejected with
 * MASKKV_EWORKSPACE (nothing enqueued).  All calls on one GPU share that GPU's array: two calls that overlap in
 * time on one GPU (different streams, or different host threads) race; calls on one stream are ordered.  Every
 * scratch word a call reads is written by the same call first, so nothing needs clearing between calls.  The
 * first call on a device resolves the array's device address (hipGetSymbolAddress); make that call outside graph
 * capture.
 */
#define MASKKV_STATIC_SCRATCH_BYTES (16u << 20)
int maskkv_score_static(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full,
                        float scale, float* scores, int64_t score_stride, float* prompt_mass, void* stream);

/* Workspace (DEVICE bytes) needed by maskkv_select: the candidates that the first
 * stage (one workgroup per 4096 prompt positions) hands to the per-head final stage, and their counts; 0 for
 * prompts of at most 4096 tokens.  256-byte alignment. */
int maskkv_select_workspace_bytes(const maskkv_desc* desc, size_t* bytes);

/*
 * Smoothing + per-head top-k.  For every (b, h), with k = min(max(budgets[b*H+h], 0), P_b):
 *   pooled_j = mean (MASKKV_POOL_MEAN) or max (MASKKV_POOL_MAX) of scores over the window
 *              [max(0, j-r), min(P_b-1, j+r)], r = (pool_window-1)/2; the mean is evaluated
 *              in fp32 by adding the in-range terms from the lowest index upwards and
 *              dividing by their count.  pool_window must be odd, 1 (= no pooling) .. 63.
 *   keep     = the k positions with the largest pooled score, ties to the lower position,
 *              written in ascending order to idx[cu_budget[b*H+h] .. cu_budget[b*H+h+1]).
 *   cu_budget = exclusive prefix sum of the clamped budgets, B*H+1 entries.
 * budgets: DEVICE int32 [B*H] (device-resident so that maskkv_head_budgets can feed it
 * without a host round trip).  budgets_host: HOST int32 [B*H] copy of the same values, or
 * NULL.  With the copy the call checks them before anything is enqueued: a negative budget
 * is MASKKV_EINVAL, clamped budgets that sum to more than capacity are MASKKV_ECAPACITY.
 * Without it (budgets that only exist on the device) negative budgets count as 0, and if
 * the clamped budgets sum to more than capacity the rows beyond capacity are not written
 * while cu_budget still holds the unclipped prefix sums: size capacity as the sum of the
 * budgets, or B*H*k_l for budgets from maskkv_head_budgets (their sum never exceeds it).
 * idx: DEVICE int32 [capacity]; cu_budget: DEVICE int32 [B*H+1].  P_max may not exceed
 * 4 Mi tokens and B*H*P_max must fit 31 bits (MASKKV_ESHAPE).
 */
int maskkv_select(const maskkv_desc* desc, const float* scores, int64_t score_stride,
                  int pool_window, int pool_mode, const int32_t* budgets, const int32_t* budgets_host,
                  int32_t* idx, int32_t* cu_budget, int64_t capacity,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Eviction as a gather.  Row r of the packed caches, r in [cu_budget[bh], cu_budget[bh+1]),
 * receives prompt row idx[r] of head bh:  Kc[r, :] = K[b, h, idx[r], :], same for V.
 * Kc, Vc: DEVICE [capacity, d] in desc->dtype, rows contiguous.  Rows >= min(capacity,
 * cu_budget[B*H]) are left untouched.  K, V: views whose first P_b rows are the prompt.
 */
int maskkv_compact(const maskkv_desc* desc, const maskkv_tensor* K, const maskkv_tensor* V,
                   const int32_t* idx, const int32_t* cu_budget, int64_t capacity,
                   void* Kc, void* Vc, void* stream);

/* Workspace (DEVICE bytes) for maskkv_attend (full = 0: the order in which the heads are processed, longest key
 * axis first; 0 for small launches) or maskkv_attend_full (full = 1: key-split partial results).  256-byte
 * alignment. */
int maskkv_attend_workspace_bytes(const maskkv_desc* desc, int full, size_t* bytes);

/*
 * Attention over the evicted cache.  For every (b, h), query head hq of h's group (hq = h when
 * q_per_kv <= 1) and response query i < n_resp:
 *   O[b,hq,i,:] = sum_j softmax_j(Q_resp[b,hq,i,:] . k_j * scale) v_j
 * with j over the cache rows [cu_budget[bh], cu_budget[bh+1]) of Kc/Vc (DEVICE [capacity, d];
 * row numbers are clipped to capacity) followed by the n_resp rows of K_resp/V_resp (views
 * [B, H, n_resp, d]).  No mask.  lse (DEVICE float
 * [B*H*g*n_resp], optional) receives the natural-log softmax normaliser of every row.
 * Inputs in desc->dtype, fp32 accumulation; probabilities are rounded to desc->dtype only
 * as the operand of the P.V product.  Q_resp, O: views [B, H*g, n_resp, d]; O is written in desc->dtype.
 */
int maskkv_attend(const maskkv_desc* desc, const maskkv_tensor* Q_resp,
                  const void* Kc, const void* Vc, const int32_t* cu_budget, int64_t capacity,
                  const maskkv_tensor* K_resp, const maskkv_tensor* V_resp, float scale,
                  const maskkv_tensor* O, float* lse,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The same attention over all N_b = P_b + n_resp rows of K_full/V_full (nothing evicted). */
int maskkv_attend_full(const maskkv_desc* desc, const maskkv_tensor* Q_resp,
                       const maskkv_tensor* K_full, const maskkv_tensor* V_full, float scale,
                       const maskkv_tensor* O, float* lse,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 2, head level, on the device.  For every b:
 *   P_h = prompt_mass[b*H+h] / (g*n_query)  (mask-to-prompt share of the voting rows' attention)
 *   budgets[b*H+h] = floor(alpha*k_l + (1-alpha) * H * k_l * P_h / sum_h' P_h')
 * prompt_mass: DEVICE float [B*H] as written by maskkv_score; budgets: DEVICE int32 [B*H].
 * k_l is the layer's per-head average budget; 0 <= alpha <= 1.  A sequence whose masses are all zero (empty
 * prompt) gets budgets[..] = k_l for every head.
 */
int maskkv_head_budgets(const maskkv_desc* desc, const float* prompt_mass, int32_t k_l, float alpha,
                        int32_t* budgets, void* stream);

/* Workspace (DEVICE bytes) needed by maskkv_layer_importance.  256-byte alignment. */
int maskkv_layer_importance_workspace_bytes(size_t* bytes);

/*
 * Stage 2, layer level, the layer importance metric:
 *   importance[0] = 1 - (1/n) sum_i cos_sim(h_in[i, :], h_out[i, :])
 * over the n_tokens rows of a layer's attention sub-layer input and output hidden states.
 * h_in, h_out: DEVICE [n_tokens, hidden] in `dtype` (a maskkv_dtype), rows row_stride elements apart
 * (row_stride >= hidden), pointers and row stride multiples of 16 bytes, hidden a multiple of 8
 * elements.  importance: DEVICE float [1].  fp32 accumulation.  n_tokens >= 1.
 */
int maskkv_layer_importance(const void* h_in, const void* h_out, int64_t n_tokens, int32_t hidden, int32_t dtype,
                            int64_t row_stride, float* importance, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * Stage 2, layer level, the boundary-aware budget allocation (host arithmetic, no device work):
 *   k_base = floor(beta * k_p / L),  k_imp = k_p - L * k_base;
 *   k_imp is split between the boundary layers and the other (middle) layers in proportion to the sums
 *   of their importances; every layer receives k_base plus the floor of an equal share of its group's part.
 * importance: HOST float [n_layers]; boundary: HOST int32 [n_boundary] layer numbers, or NULL for
 * {first, last}; k_l: HOST int64 [n_layers] output.  k_p >= 0, 0 <= beta <= 1, importances >= 0 with a
 * positive sum.  The budget lost to the floors is left unallocated (sum k_l <= k_p).
 */
int maskkv_layer_budgets(const float* importance, int32_t n_layers, int64_t k_p, float beta,
                         const int32_t* boundary, int32_t n_boundary, int64_t* k_l);

/*
 * Response-token refresh criterion of the feature-cache background (Section 3.1, the set S_shift):
 *   cos[i]  = cos_sim(V_now[i, :], V_prev[i, :])  for the n_tokens response tokens of a layer
 *   refresh = ascending positions i with cos[i] < delta (strict), count[0] of them.
 * V_now, V_prev: DEVICE [n_tokens, width] in `dtype` (a maskkv_dtype; width = heads * head_dim), rows
 * row_stride elements apart, pointers and row stride multiples of 16 bytes, width a multiple of 8.
 * cos: DEVICE float [n_tokens]; refresh: DEVICE int32 [n_tokens] (entries >= count[0] untouched); count:
 * DEVICE int32 [1].  fp32 accumulation; the comparison is made on the fp32 cosine.  A row of zeros has no
 * cosine (NaN) and is not listed.  No workspace.
 */
int maskkv_value_shift(const void* V_now, const void* V_prev, int64_t n_tokens, int32_t width, int32_t dtype,
                       int64_t row_stride, float delta, float* cos, int32_t* refresh, int32_t* count, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MASKKV_H */
