/*
 * Verification-aware scheduler (Section 4.5, Algorithm 1) as a host module in front of
 * synera_verify: it keeps the request pool, decides what the next engine call forwards, owns the KV
 * page table of every request, and hands back the host arrays synera_verify takes.
 *
 * One pass of the algorithm's outer loop is an *iteration*.  If prefill requests are waiting, the
 * iteration executes them and nothing else (prefill priority, never mixed with verifications);
 * otherwise it gathers every waiting verification request with its number of uncached tokens and
 * executes them as one partial prefill; requests marked finished leave the active batch at the end of
 * an iteration that executed no prefill.  Execution is a sequence of *engine calls* on fixed chunks
 * of at most SYNERA_MAX_CHUNK (32) tokens per request ("chunked partial prefill"): the requests of an
 * iteration advance together, a verification's drafts ride in its last chunk, and in a chunk without
 * drafts the last token is presented as the one LM-head row the engine call needs (n_draft = 1,
 * final_verify = 0; its result matters only after the last prompt token, whose greedy token is the
 * request's first anchor).
 *
 * What the algorithm leaves open is fixed as follows.  Requests are admitted in arrival order while
 * they fit: at most max_batch requests per iteration, at most max_tokens chunk tokens per engine call,
 * and KV pages (16 tokens each) for the request's whole new length, taken from the pool when the
 * request joins an iteration; the first request that does not fit stays at the head of its queue and
 * ends the gathering.  A request that could never fit is refused at submission (ENOSPC).  After a
 * verification with accept length a the request's cached length is L + u + a.
 *
 * All pointers are host memory.  Not thread-safe: one caller drives submit / next / commit.
 * Status codes are those of synera.h.
 */
#ifndef SYNERA_SCHED_H
#define SYNERA_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct synera_sched synera_sched;

enum { SYNERA_SCHED_IDLE = 0, SYNERA_SCHED_PREFILL = 1, SYNERA_SCHED_VERIFY = 2 };

typedef struct synera_sched_stats {
  int64_t iterations_prefill; /* iterations that executed prefills */
  int64_t iterations_verify;  /* iterations that executed a verification batch */
  int64_t iterations_idle;    /* iterations that found nothing to execute */
  int64_t engine_calls;       /* synera_sched_next calls that returned a batch */
  int64_t tokens_forwarded;   /* sum of u + k over all engine calls */
  int64_t host_ns;            /* wall time spent inside synera_sched_next and synera_sched_commit */
  int32_t active_requests;    /* size of the active batch B */
  int32_t waiting_prefill;    /* queue lengths */
  int32_t waiting_verify;
  int32_t free_pages;
} synera_sched_stats;

/*
 * n_pages_in_pool: pages the scheduler may hand out (ids 0 .. n-1); max_pages: block-table columns
 * per request (a request can never hold more); max_batch, max_tokens: limits of the synera_ctx the
 * engine calls go to.  Errors: EINVAL (null / non-positive), ENOMEM.
 */
int32_t synera_sched_create(synera_sched** out, int32_t n_pages_in_pool, int32_t max_pages,
                            int32_t max_batch, int32_t max_tokens);
int32_t synera_sched_destroy(synera_sched* s);

/*
 * A new request with n_prompt >= 1 prompt tokens.  Errors: EINVAL (id in use, n_prompt < 1),
 * ENOSPC (the prompt needs more pages than max_pages or the pool holds).
 */
int32_t synera_sched_submit_prefill(synera_sched* s, int64_t request_id, int32_t n_prompt);

/*
 * A verification request for an active request (prefilled, not finished, none pending):
 * n_uncached >= 0 tokens the device accepted locally since the last verification, then
 * 1 <= n_draft <= 32 drafts.  Errors: EINVAL, ENOSPC (L + u + k can never fit).
 */
int32_t synera_sched_submit_verify(synera_sched* s, int64_t request_id, int32_t n_uncached,
                                   int32_t n_draft);

/* Marks an active request with no pending work as completed; it leaves the active batch, and its
 * pages return to the pool, at the end of the next iteration that executes no prefill. */
int32_t synera_sched_finish(synera_sched* s, int64_t request_id);

/*
 * The next engine call: continues the iteration in progress, or starts a new one.  Outputs
 * (arrays sized for max_batch entries; the block table [max_batch][max_pages], row i holding request
 * i's pages in order, unused entries -1):
 *   *kind  SYNERA_SCHED_PREFILL / _VERIFY, or _IDLE with *B = 0 when nothing can run
 *   h_request_id, h_ctx_len (L), h_n_uncached (u), h_n_draft (k): one entry per request of the call;
 *     h_ctx_len / h_n_uncached / h_n_draft / h_block_table go to synera_verify unchanged
 *   h_token_begin: index of the chunk's first token within the tokens of the request's submission
 *   h_final_verify: 1 where the chunk carries the request's drafts (its accept length is wanted)
 * Every call that returns a batch must be followed by synera_sched_commit before the next one
 * (EINVAL otherwise).
 */
int32_t synera_sched_next(synera_sched* s, int32_t* kind, int32_t* B, int64_t* h_request_id,
                          int32_t* h_ctx_len, int32_t* h_n_uncached, int32_t* h_n_draft,
                          int32_t* h_token_begin, int32_t* h_final_verify, int32_t* h_block_table);

/*
 * Result of the engine call handed out last: h_accept_len[i] in 0 .. k_i is read for the entries with
 * final_verify = 1 (others ignored; the pointer may be NULL if there are none).  Advances the
 * requests; when the iteration's requests are all done it closes the iteration (joins them to the
 * active batch, removes completed requests).  Errors: EINVAL (no call outstanding, accept length
 * out of range: then nothing is changed).
 */
int32_t synera_sched_commit(synera_sched* s, const int32_t* h_accept_len);

/* Cached length L of a request, or -1 if the id is unknown. */
int64_t synera_sched_cached_len(const synera_sched* s, int64_t request_id);

int32_t synera_sched_get_stats(const synera_sched* s, synera_sched_stats* out);

#ifdef __cplusplus
}
#endif
#endif
