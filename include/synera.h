/*
 * synera.h - C ABI of the cloud-side batched verification of offloaded draft
 * chunks (Synera, arXiv 2511.07423) for AMD MI355X (gfx950).
 *
 * What the calls compute follows the paper's statement of the problem:
 *   - a verification request = cached tokens + uncached device-accepted tokens
 *     + pending-verify draft tokens (Section 3.4, Fig. "cloud_serving");
 *   - its forward pass is a "partial prefill": like a prefill, but against an
 *     existing KV-cached prefix (Section 3.4, Takeaway-3);
 *   - the batch is flattened across requests before it enters the transformer
 *     and is executed with the list of per-request uncached counts
 *     (Section 4.5, Algorithm 1: execute_partialprefill(B_verify, L_uncached));
 *   - verification then uses the LLM's k+1 distributions q(x|prefix) ..
 *     q(x|prefix, d_0..d_{k-1}) for k drafts (Section 4.5) and returns what the
 *     device merges on: the rejection position and the correction (Section 4.4);
 *   - the confidence score of a token is its top-1 softmax probability
 *     (Section 3.2); entropy (nats) is reported beside it.
 *
 * General rules
 *   - Pointers named h_* are HOST memory, d_* are DEVICE memory (gfx950 HBM).
 *     The caller owns every buffer it passes; the library owns only the opaque
 *     context and the scratch inside it.  Nothing passed in is freed or kept
 *     beyond the call, except the weight pointers recorded by synera_create,
 *     which must stay valid and unchanged until synera_destroy.
 *   - Every call returns 0 (SYNERA_OK) or a negative synera_status.  Metadata
 *     (lengths, block tables) is validated on the host BEFORE anything is
 *     launched; a failed call has launched nothing and written nothing.
 *   - Work is enqueued on the caller's HIP stream (`stream`, a hipStream_t cast
 *     to void*, NULL = the default stream) and the call returns without
 *     waiting.  Outputs are valid once the stream has reached that point.
 *     Calls on one context must be issued from one host thread at a time and
 *     onto one stream (the scratch is shared).
 *   - There is no CPU fallback: without a usable gfx950 device the calls that
 *     launch work fail with SYNERA_EHIP.
 *
 * KV cache layout (part of the ABI; page indexing is exact)
 *   page size P = 16 positions.  Position t of request i lives in page
 *   block_table[i][t / 16], slot t % 16.  Pages may sit anywhere in the pool.
 *     k_pool : bf16 [n_layers][n_pages][n_kv_heads][16 slots][head_dim]
 *     v_pool : bf16 [n_layers][n_pages][n_kv_heads][head_dim][16 slots]
 *   (V is stored dim-major inside a page so that the P*V matrix-core operand of
 *   the attention kernel is a plain contiguous load.)
 *   The library never allocates pages and never changes a request's length:
 *   after a verify the caller commits L_i += u_i + accept_len_i; K/V written
 *   beyond that are dead and get overwritten by the next chunk.
 *
 * Weights: bf16, row-major [out_features][in_features]; norm gains bf16 [d].
 * Matrix weights must be below 256 in magnitude (they are widened to fp16 with
 * their exponent raised by 8 on the way into the matrix cores).
 *
 * Measurement and test hooks (stage timing, the bare projection GEMM, measured
 * ceilings, planner dumps) are declared in synera_debug.h.
 */
#ifndef SYNERA_H
#define SYNERA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SYNERA_PAGE_SIZE 16
#define SYNERA_MAX_CHUNK 32 /* u_i + k_i per request and call (Section 4.5: chunks of 32) */

typedef enum synera_status {
  SYNERA_OK = 0,
  SYNERA_EINVAL = -1, /* null pointer, non-positive size, k_i < 1, u_i < 0, bad dtype        */
  SYNERA_ERANGE = -2, /* negative length, page id outside the pool, page used twice          */
  SYNERA_ENOSPC = -3, /* block table / batch / token / row capacity too small                */
  SYNERA_EUNSUP = -4, /* shape the kernels do not cover (see synera_create), chunk > 32      */
  SYNERA_EHIP = -5,   /* HIP runtime error or no gfx950 device                               */
  SYNERA_ENOMEM = -6  /* scratch allocation failed                                           */
} synera_status;

typedef struct synera_model_desc {
  int32_t n_layers;
  int32_t d_model;    /* multiple of 128                                         */
  int32_t n_q_heads;  /* multiple of n_kv_heads; group size G = q/kv <= 16;       */
  int32_t n_kv_heads; /* n_q_heads*head_dim and n_kv_heads*head_dim multiples of 128 */
  int32_t head_dim;   /* 64 or 128                                               */
  int32_t d_ffn;      /* multiple of 64                                          */
  int32_t vocab;      /* multiple of 128                                         */
  float rope_base;    /* rotary base (10000)                              */
  float rms_eps;
} synera_model_desc;

typedef struct synera_layer_weights { /* all DEVICE pointers, bf16 */
  const void* attn_norm; /* [d]                 */
  const void* wq;        /* [Hq*h][d]           */
  const void* wk;        /* [Hkv*h][d]          */
  const void* wv;        /* [Hkv*h][d]          */
  const void* wo;        /* [d][Hq*h]           */
  const void* mlp_norm;  /* [d]                 */
  const void* w_gate;    /* [f][d]              */
  const void* w_up;      /* [f][d]              */
  const void* w_down;    /* [d][f]              */
} synera_layer_weights;

typedef struct synera_weights {
  const void* embed;                  /* device bf16 [V][d]                          */
  const synera_layer_weights* layers; /* HOST array [n_layers] of device pointers    */
  const void* final_norm;             /* device bf16 [d]                             */
  const void* lm_head;                /* device bf16 [V][d]                          */
} synera_weights;

typedef struct synera_ctx synera_ctx;

/* Library version (major*10000 + minor*100 + patch). */
int32_t synera_version(void);

/* Static string for a status code. */
const char* synera_strerror(int32_t status);

/*
 * Create a context for one model on the current HIP device.  Copies `desc` and
 * the pointer table `w` (not the weights) and allocates device scratch sized
 * for at most max_batch requests, max_tokens flattened chunk tokens
 * (sum of u_i + k_i) and max_pages block-table columns per request.
 * Errors: EINVAL (null / non-positive), EUNSUP (shape rules in synera_model_desc),
 * EHIP, ENOMEM.  On error *out is NULL.
 */
int32_t synera_create(synera_ctx** out, const synera_model_desc* desc, const synera_weights* w,
                      int32_t max_batch, int32_t max_tokens, int32_t max_pages);

/* Free the scratch.  Waits for the device to finish first.  NULL is allowed. */
int32_t synera_destroy(synera_ctx* ctx);

/*
 * Host-only validation of a batch description (no device access; callable
 * without a GPU).  synera_verify and synera_kv_append apply exactly this check
 * before launching.  n_second may be NULL (then treated as zeros); for
 * synera_kv_append pass h_n_new as n_first and NULL.
 *   EINVAL: null pointer, B < 1, n_first[i] < 1 or n_second[i] < 0
 *   ERANGE: ctx_len[i] < 0; a page id needed by request i outside [0, n_pages);
 *           the same page needed twice (within or across requests)
 *   ENOSPC: B > max_batch; sum of chunk lengths > max_tokens;
 *           ceil((ctx_len[i] + chunk_i) / 16) > max_pages
 *   EUNSUP: chunk_i > chunk_limit (pass 0 for no limit)
 * Block-table entries beyond the pages a request needs are ignored.
 */
int32_t synera_validate_batch(int32_t B, const int32_t* h_ctx_len, const int32_t* h_n_first,
                              const int32_t* h_n_second, const int32_t* h_block_table,
                              int32_t max_pages, int32_t n_pages_in_pool, int32_t max_batch,
                              int64_t max_tokens, int32_t chunk_limit);

/*
 * One flattened ragged verification (Section 4.5): for each request i the chunk
 * [u_i uncached accepted tokens | k_i drafts] is forwarded at positions
 * L_i .. L_i+u_i+k_i-1 against the cached prefix 0..L_i-1; chunk row j attends
 * to keys 0..L_i+j.  K/V of every chunk token are appended to the pools.
 *
 *   h_ctx_len     host [B]  L_i >= 0
 *   h_n_uncached  host [B]  u_i >= 0
 *   h_n_draft     host [B]  k_i >= 1,  u_i + k_i <= 32
 *   d_tokens      dev  [T]  T = sum(u_i + k_i); request-major, uncached then drafts
 *   d_anchor      dev  [B]  the LLM's greedy token after the cached context; read
 *                           only for requests with u_i == 0 (otherwise the row of
 *                           the last uncached token supplies q(x|prefix))
 *   h_block_table host [B][max_pages]
 *   d_k_pool, d_v_pool   dev, layout above, n_pages_in_pool pages per layer, 16-byte aligned
 * Outputs (device).  R = sum k_i rows, request-major, one per draft position:
 *   d_logits    f32 [R][vocab]   may be NULL
 *   d_argmax    i32 [R]          greedy token AFTER draft j (lowest id on ties)
 *   d_top1_prob f32 [R]          may be NULL
 *   d_entropy   f32 [R]  nats    may be NULL
 *   d_accept_len  i32 [B]  n_i in 0..k_i: longest prefix with d_j == a_j, where
 *                          a_0 is the anchor (or the last uncached row's argmax)
 *                          and a_j the argmax of draft j-1's row
 *   d_correction  i32 [B]  a_{n_i} (for n_i == k_i the token after the last draft)
 * Errors: as synera_validate_batch (limits from synera_create), EINVAL for null
 * required pointers and for pools that are not 16-byte aligned, EHIP.
 */
int32_t synera_verify(synera_ctx* ctx, int32_t B, const int32_t* h_ctx_len,
                      const int32_t* h_n_uncached, const int32_t* h_n_draft,
                      const int32_t* d_tokens, const int32_t* d_anchor,
                      const int32_t* h_block_table, int32_t max_pages, int32_t n_pages_in_pool,
                      void* d_k_pool, void* d_v_pool, float* d_logits, int32_t* d_argmax,
                      float* d_top1_prob, float* d_entropy, int32_t* d_accept_len,
                      int32_t* d_correction, void* stream);

/*
 * Standalone confidence statistics over a logits matrix (Section 3.2): per row
 * the argmax (lowest id on ties), its softmax probability, and the entropy in
 * nats.  d_logits: device, dtype 0 = f32, 1 = bf16, `rows` rows of `vocab`
 * entries, consecutive rows row_stride_elems apart (>= vocab; the row start must
 * be 16-byte aligned, i.e. stride a multiple of 4 (f32) / 8 (bf16) elements).
 * Outputs device [rows]; d_top1_prob / d_entropy may be NULL.  rows == 0 is a
 * no-op.  Errors: EINVAL, EHIP.
 */
int32_t synera_confidence(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab,
                          int64_t row_stride_elems, int32_t* d_top1_id, float* d_top1_prob,
                          float* d_entropy, void* stream);

/*
 * The same vocabulary pass, keeping the k most probable tokens of each row: the compressed form of a
 * distribution that is transmitted instead of the full vector (Section 4.2, "Compression before
 * transmission": top-1 / top-k of the sampling method in use; a list that cuts 32000 entries by over 99.5 %
 * has up to 160), and the margin score, top-1 minus top-2 probability, that drives the layer-wise early exit
 * (Section 4.3).  1 <= k <= SYNERA_MAX_TOPK.  d_logits / dtype / rows / vocab / row_stride_elems as
 * synera_confidence; entries may be -inf (probability 0), not NaN.
 * Outputs, device: d_topk_id i32 [rows][k] and d_topk_prob f32 [rows][k], most probable first,
 * equal logits by the lower token id first; d_margin f32 [rows] (NULL to skip), d_entropy f32
 * [rows] in nats (NULL to skip).  A row with fewer than k comparable entries (NaN) reports id 0,
 * probability 0 for the missing ones.  Errors: EINVAL; EUNSUP for k > SYNERA_MAX_TOPK or k > vocab; EHIP.
 */
#define SYNERA_MAX_TOPK 256
int32_t synera_confidence_topk(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab,
                               int64_t row_stride_elems, int32_t k, int32_t* d_topk_id,
                               float* d_topk_prob, float* d_margin, float* d_entropy, void* stream);

/*
 * Top-p (nucleus) cut over the FULL vocabulary (Section 4.2 names top-p beside top-1 and top-k as the sampling
 * methods whose lists are transmitted; Section 4.5 verifies under it): per row the smallest number of tokens,
 * most probable first (equal logits by the lower id), whose softmax probabilities sum to at least top_p.
 * d_count i32 [rows]; d_mass f32 [rows] (NULL to skip) = the probability those tokens hold; d_cut_logit f32
 * [rows] (NULL to skip) = the smallest logit kept: the nucleus is every token above it plus the first
 * count - #{above} holders of it in id order, i.e. the first d_count entries of synera_confidence_topk's order.
 * Logits finite or -inf.  Masses are summed in 40-bit fixed point (order-independent: the count is reproducible);
 * a running sum that passes within ~1e-6 of top_p may fall either way against an exact evaluation.
 * Errors: EINVAL (top_p outside (0, 1], null pointers, alignment as synera_confidence), EHIP.
 */
int32_t synera_nucleus(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab, int64_t row_stride_elems,
                       float top_p, int32_t* d_count, float* d_mass, float* d_cut_logit, void* stream);

/*
 * Top-p (nucleus) cut INSIDE compressed distributions ("Compression before transmission", Section 4.2:
 * top-1 / top-k / top-p of the sampling method in use).  d_topk_prob: device f32 [rows][k], each row most
 * probable first (synera_confidence_topk's output).  d_count[r] = the smallest n whose float32 running
 * sum p_0 + ... + p_{n-1}, taken in that order, reaches top_p; all k if the window never does.
 * d_mass[r] (NULL to skip) = that sum.  Errors: EINVAL (top_p outside (0, 1], k < 1, null pointers), EHIP.
 */
int32_t synera_topp_count(const float* d_topk_prob, int64_t rows, int32_t k, float top_p, int32_t* d_count,
                          float* d_mass, void* stream);

/*
 * Dispatch probability of token chunks from their confidence (Section 4.2, first equation):
 * chunk b owns rows d_cu_rows[b] .. d_cu_rows[b+1]-1 of d_top1_prob (device, i32 [B+1] prefix
 * sums and f32 per-row top-1 probabilities, e.g. synera_verify's or synera_confidence's
 * output); c_b = their mean (0 for an empty chunk), P_conf(c) = 1 for c <= c_th, else
 * 1 / (1 + exp(k_slope * ((c - c_th) / (1 - c_th) - 1/2))); the paper uses k_slope = 10 and
 * c_th in [0.7, 1).  Outputs device f32 [B].  Errors: EINVAL (c_th outside [0, 1), null
 * pointers), EHIP.
 */
int32_t synera_chunk_dispatch(const float* d_top1_prob, const int32_t* d_cu_rows, int32_t B, float c_th,
                              float k_slope, float* d_mean_conf, float* d_p_conf, void* stream);

/*
 * Stochastic verification of the batch that the LAST synera_verify on this context forwarded: speculative
 * sampling against the LLM distributions that call computed (Section 4.5 verifies with q(x | prefix), ...,
 * q(x | prefix, x_1..x_k) under top-k / top-p sampling and Section 4.2 transmits the SLM distributions p in
 * compressed form; the acceptance rule itself is the published speculative-sampling rule the paper cites).
 * Per request: draft j is accepted with probability min(1, q_j(x_j) / p_j(x_j)); at the first rejection the
 * emitted token is drawn from norm(max(0, q_j - p_j)); after k_i acceptances from the distribution that
 * follows the last draft.  q = softmax of the LM-head rows (temperature 1); p_j = the transmitted top-k list
 * of draft row j, renormalised to sum 1 (0 outside the list; a draft absent from its list is rejected).
 *   d_tokens    dev [T]            as given to synera_verify
 *   d_p_id / d_p_prob  dev [R][k_list], 1 <= k_list <= SYNERA_MAX_TOPK (EUNSUP above): the lists, row order = draft rows
 *   d_u_accept  dev f32 [R]        uniform numbers in [0, 1), one per draft row
 *   d_u_sample  dev f32 [B]        one per request, for the emitted token (smallest id whose inclusive
 *                                   cumulative weight, in id order, exceeds u * total)
 *   d_accept_len dev i32 [B], d_token dev i32 [B]
 * Every request of that verify must have had u_i >= 1 (the row of its last uncached token supplies the
 * first distribution): EUNSUP otherwise.  Errors: EINVAL (null pointers, k_list < 1, no verify to read), EHIP.
 */
int32_t synera_stochastic_accept(synera_ctx* ctx, const int32_t* d_tokens, int32_t k_list, const int32_t* d_p_id,
                                 const float* d_p_prob, const float* d_u_accept, const float* d_u_sample,
                                 int32_t* d_accept_len, int32_t* d_token, void* stream);

/*
 * Importance scores of the batch that the LAST synera_verify on this context forwarded (Section 3.2:
 * the column-wise sum of the attention matrix softmax(Q K^T / sqrt(d_k)); the paper names neither layer
 * nor head handling: these are the last decoder layer's, averaged over the query heads).  For request i
 * with cached length L_i and chunk length c_i = u_i + k_i the call writes L_i + c_i scores, one per key
 * position, request after request: score_j = (1/Hq) sum_heads sum_{rows r: L_i + r >= j} p(r, j), so
 * the scores of a request sum to c_i.  It reads the rotated queries and the per-row softmax statistics
 * that verify left in the context, and the last layer's K pages (d_k_pool / n_pages_in_pool as given
 * to that verify, whose block tables are reused).  n_scores must equal sum_i (L_i + c_i).
 * Optional outputs, device f32 [B]: d_mean_importance = mean score of the request's k_i draft
 * positions; d_p_imp = the probability of offloading by importance (Section 4.2, second equation):
 * 0 for i <= i_th/2, 1 for i > i_th, else 1 / (1 + exp(theta ((i - i_th/2) / (i_th/2) - 1/2))); the paper
 * uses theta = -10.  Errors: EINVAL (null pointers, no verify since the last kv_append / verify error,
 * a pool or n_scores other than that verify's, i_th <= 0 with d_p_imp), EHIP.
 */
int32_t synera_importance(synera_ctx* ctx, int32_t n_pages_in_pool, const void* d_k_pool, int64_t n_scores,
                          float* d_importance, float i_th, float theta, float* d_mean_importance,
                          float* d_p_imp, void* stream);

/*
 * Scatter K/V rows of one layer into the paged pools: request i appends n_new_i
 * rows at positions L_i .. L_i+n_new_i-1 (what the partial prefill does for
 * every forwarded token, Section 3.4; exported so a prefill engine or a test
 * can fill the cache).  d_k, d_v: device bf16 [sum n_new][n_kv_heads][head_dim],
 * request-major, already rotated.  No chunk limit applies here.
 * Errors: as synera_validate_batch, EINVAL (layer outside the model), EHIP.
 */
int32_t synera_kv_append(synera_ctx* ctx, int32_t layer, int32_t B, const int32_t* h_ctx_len,
                         const int32_t* h_n_new, const void* d_k, const void* d_v,
                         const int32_t* h_block_table, int32_t max_pages,
                         int32_t n_pages_in_pool, void* d_k_pool, void* d_v_pool, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SYNERA_H */
