/*
 * synera_debug.h - measurement and test hooks of the verification library (see synera.h for the product
 * ABI).  Nothing here is needed to serve requests: these calls time the stages of a verify, expose the
 * projection GEMM and the planners on their own, and measure what the GPU gives a bare copy or MFMA loop.
 * Same rules as synera.h: h_* host, d_* device, int32 status, work is enqueued on `stream`.
 */
#ifndef SYNERA_DEBUG_H
#define SYNERA_DEBUG_H

#include "synera.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SYNERA_MAX_GEMM_SLICES 8 /* K slices a projection may be stored in (synera_debug_gemm_slices) */

/*
 * Stage timing, for the roofline measurement of the kernels inside a verify
 * (the paper gives no breakdown of where the forward pass spends its time;
 * Section 6.7 only separates scheduling from compute).  After
 * synera_profile_begin(ctx, stage) every launch of that stage in later
 * synera_verify calls is bracketed by a HIP event pair on the call's stream.
 * synera_profile_end waits for those events, returns how many launches were
 * bracketed and the sum of their durations in milliseconds, and switches the
 * timing off.  Errors: EINVAL (null, unknown stage), EHIP.
 */
typedef enum synera_stage {
  SYNERA_STAGE_NONE = 0,
  SYNERA_STAGE_QKV = 1,        /* Wq|Wk|Wv projection                       */
  SYNERA_STAGE_ATTENTION = 2,  /* paged chunk attention incl. the split merge */
  SYNERA_STAGE_O = 3,          /* output projection + residual              */
  SYNERA_STAGE_GATE_UP = 4,    /* gate/up projection + SiLU*mul             */
  SYNERA_STAGE_DOWN = 5,       /* down projection + residual                */
  SYNERA_STAGE_LM_HEAD = 6,
  SYNERA_STAGE_CONFIDENCE = 7, /* fused softmax/argmax/entropy              */
  SYNERA_STAGE_NORM = 8,       /* RMSNorm launches inside the layers        */
  SYNERA_STAGE_ROPE_APPEND = 9
} synera_stage;
int32_t synera_profile_begin(synera_ctx* ctx, int32_t stage);
int32_t synera_profile_end(synera_ctx* ctx, int32_t* n_launches, float* total_ms);

/*
 * C = (A_hi + A_lo) * W^T on the matrix cores, the contraction every projection of the decoder uses
 * (Section 3.4's partial prefill is a stack of these; exported for tests and the GEMM roofline sweep).
 * d_a, d_a_lo: fp16 [M][K] row-major, the (hi, lo) pair of the activations (hi = fp16(v), lo = fp16(v - hi):
 * 22 mantissa bits of v); d_w bf16 [N][K] row-major; d_c f32 [M][N].  d_a_lo may be NULL: the high part alone is
 * multiplied (11 mantissa bits, half the matrix-core work: the form the LM head runs in).
 * K must be a multiple of 64 and N of 128 (else EUNSUP).  Errors: EINVAL, EUNSUP, EHIP.
 */
int32_t synera_gemm_pair(const void* d_a, const void* d_a_lo, const void* d_w, float* d_c,
                         int32_t M, int32_t N, int32_t K, void* stream);

/*
 * The same contraction for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments and result as
 * synera_gemm_pair; the K slices that synera_debug_gemm_slices stores to the caller's buffer go to a static
 * device array of SYNERA_MAX_GEMM_SLICES x SYNERA_STATIC_GEMM_MAX_OUT floats (16 MiB on every GPU the library
 * runs on, held until the process ends) and are summed in order into d_c; the call allocates and frees
 * nothing.  M x N beyond SYNERA_STATIC_GEMM_MAX_OUT: ENOSPC.  All calls on one GPU share that GPU's array:
 * calls that overlap on one GPU (other streams, other threads) race.  Errors: EINVAL, EUNSUP, ENOSPC, EHIP.
 */
#define SYNERA_STATIC_GEMM_MAX_OUT 524288
int32_t synera_gemm_pair_static(const void* d_a, const void* d_a_lo, const void* d_w, float* d_c,
                                int32_t M, int32_t N, int32_t K, void* stream);

/*
 * Measured ceilings: what this GPU gives the kernels above, taken in the same process as their timings.
 * The caller times the launches (HIP events on `stream`).
 *
 * synera_measure_hbm_copy: one plain device copy d_dst[0 .. bytes) = d_src[0 .. bytes) by a kernel of
 * 16-byte accesses; HBM moves 2 x bytes.  bytes a positive multiple of 16, both pointers 16-byte aligned device
 * memory that does not overlap (else EINVAL).
 *
 * synera_measure_hbm_read: a read-only stream over d_src[0 .. bytes) by SYNERA_MEASURE_READ_BLOCKS blocks of
 * 256 lanes; with seg = ceil(bytes / 16 / blocks), lane t of block b reads the 16-byte pieces b * seg + t + 256 j
 * (j = 0, 1, ... while below (b + 1) * seg and the end), and stores the xor of all their 32-bit words to
 * d_out[b * 256 + t] (device, SYNERA_MEASURE_READ_BLOCKS x 256 words).  HBM moves `bytes`.  Same conditions on
 * bytes and d_src.
 *
 * synera_measure_mfma_bf16: `blocks` blocks of four wavefronts, each issuing iters x 16
 * v_mfma_f32_32x32x16_bf16 on register-resident operands (no memory traffic inside the loop);
 * random_operands != 0 fills the operand registers with random signs and mantissas (the rate real data gets:
 * the clock drops under the switching activity), 0 with constants.  d_out (device, blocks x 256 floats)
 * receives one accumulator sum per lane -- with constant operands exactly 2 x iters.  *h_flops (host, may be
 * NULL) receives the FLOPs of the launch.  1 <= blocks <= 4096, 1 <= iters <= 200000, else EINVAL.
 *
 * synera_measure_mfma_f16: the same on the instruction the projection kernel issues: iters x 32
 * v_mfma_f32_16x16x32_f16 per wavefront on 8 independent accumulators; with constant operands every lane's sum is
 * exactly 8 x iters.  Same arguments and errors.
 */
#define SYNERA_MEASURE_READ_BLOCKS 4096
int32_t synera_measure_hbm_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream);
int32_t synera_measure_hbm_read(uint32_t* d_out, const void* d_src, int64_t bytes, void* stream);
int32_t synera_measure_mfma_bf16(float* d_out, int32_t blocks, int32_t iters, int32_t random_operands,
                                 int64_t* h_flops, void* stream);
int32_t synera_measure_mfma_f16(float* d_out, int32_t blocks, int32_t iters, int32_t random_operands,
                                int64_t* h_flops, void* stream);

/*
 * Tuning hook for the GEMM sweep: force the tile for every later contraction whose shape it fits
 * (-1 restores the automatic choice).  tile = rows / 16 (1 .. 17) for 256-column tiles, 100 + rows / 16
 * (rows / 16 = 1 .. 12) for 128-column tiles; + 200 for the form with two MFMA K steps per stage (256 columns:
 * rows / 16 = 1 .. 5, 128 columns: 1 .. 9).  Process-wide.
 */
int32_t synera_debug_set_gemm_tile(int32_t tile);

/*
 * Test hook, host only (no GPU call, no context): the work plan of the chunk attention of Section 3.2 for one
 * batch, as synera_verify lays it out for `attn_blocks` (2 .. 8192) persistent blocks.  Inputs as for
 * synera_verify (host).
 * Outputs (host, int32): h_shares[attn_blocks][4] = (first position, positions, row blocks 4 | 2, 0) per block;
 * h_prog[prog_cap][4] = the positions (tag, a, b, c): tag & 7 = 0 padding / 1 a 32-key tile (tag >> 4 = KV
 * head, a / b = its two pages, c = first key) / 2 query rows of a stream (tag >> 4 = unit, a = first chunk
 * token, b = rows, c = first of the 32 rows carried | KV head << 8), tag & 8 = the share of the stream ends with
 * this iteration; h_units[unit_cap][8] = (first chunk token, rows, last key the first token sees, end of the
 * share's keys, partial slot or -1, KV head, 0, 0); h_cuts[cut_cap][8] = (first partial slot, slots, first chunk
 * token, rows, KV head, 0, 0, 0) per stream split over blocks; h_counts[4] = shares, positions, units, cuts.
 * Errors: EINVAL, EUNSUP, ENOSPC (an output capacity is too small), ENOMEM.
 */
int32_t synera_debug_attention_plan(const synera_model_desc* desc, int32_t attn_blocks, int32_t B,
                                    const int32_t* h_ctx_len, const int32_t* h_n_uncached, const int32_t* h_n_draft,
                                    const int32_t* h_block_table, int32_t max_pages, int32_t* h_shares,
                                    int32_t* h_prog, int64_t prog_cap, int32_t* h_units, int64_t unit_cap,
                                    int32_t* h_cuts, int64_t cut_cap, int32_t* h_counts);

/*
 * Tuning hook: the constants of the attention share planner of one context, for sweeps.  attn_blocks:
 * persistent blocks (0 keeps the current number; at most twice the default of two per compute unit);
 * stream_cost: what a stream costs a block beyond its tiles, in iterations (default 1); cut_slack: a stream
 * overshooting its block's share by less is not cut (default 1.5); t_iter_ratio: relative iteration time of
 * the class of row groups of up to 32 rows against the class above (default 1.84).  Errors: EINVAL.
 */
int32_t synera_debug_set_attention_plan(synera_ctx* ctx, int32_t attn_blocks, float stream_cost, float cut_slack,
                                        float t_iter_ratio);

/*
 * Test hook, host only (no GPU call): the tile (rows x columns) and the number of K slices the planner
 * gives a projection of M rows -- the form every projection of Section 3.4's partial prefill takes.
 * epilogue as in synera_debug_gemm_epilogue; stored_slices != 0 plans the decoder layers' mode (K may be
 * split into slices stored for the consumer kernel), 0 the stand-alone mode (K is never split).  Outputs are
 * host pointers.  Errors: EINVAL, EUNSUP (N % 128, 256 for SwiGLU, K % 64).
 */
int32_t synera_debug_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t stored_slices,
                               int32_t* h_tile_rows, int32_t* h_tile_cols, int32_t* h_k_slices);

/*
 * The same question for the K extent of one LDS stage of that plan: 32 (one MFMA K step per barrier) or 64 (two,
 * the form the short tiles take).  *h_stage_k is a host pointer.  Same errors.
 */
int32_t synera_debug_gemm_plan_bk(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t stored_slices,
                                  int32_t* h_stage_k);

/*
 * Test hook: one launch of the projection GEMM with the epilogue the decoder layers use
 * (Section 3.4's partial prefill runs these three forms per layer).  Activations are the
 * fp16 pair d_a + d_a_lo ([M][K] each).  epilogue 0: d_c f32 [M][N] = A W0^T; 1: d_c += A W0^T
 * (the residual add of the O and down projections); 2: SwiGLU, d_w0 = gate and d_w1 = up
 * (bf16 [N/2][K] each), d_c / d_c_lo = fp16 pair [M][N/2] of 8 x silu(A gate^T) * (A up^T) (the scale the
 * down projection expects of its input).  N % 128 == 0 (256 for epilogue 2), K % 64 == 0, else EUNSUP.
 * All pointers device.
 */
int32_t synera_debug_gemm_epilogue(const void* d_a, const void* d_a_lo, const void* d_w0, const void* d_w1,
                                   void* d_c, void* d_c_lo, int32_t M, int32_t N, int32_t K, int32_t epilogue,
                                   void* stream);

/*
 * Test hook: synera_debug_gemm_epilogue with the activation pair in the form the decoder layers hand it over in
 * where a stage of the kernel holds one 32-wide K block: one fp16 array d_a_pairs [M][K / 32][64], the 32 high
 * parts of a K block followed by its 32 low parts (a copy then moves whole 128-byte lines).  Epilogues 0 and 1 as
 * above; epilogue 2 writes its output pair in the same form into d_c (fp16 [M][N / 64][64]).  Any tile forced
 * with synera_debug_set_gemm_tile that has 64-wide stages (variant >= 200) is ignored: the planner chooses.
 * All pointers device.
 */
int32_t synera_debug_gemm_paired(const void* d_a_pairs, const void* d_w0, const void* d_w1, void* d_c, int32_t M,
                                 int32_t N, int32_t K, int32_t epilogue, void* stream);

/*
 * Test hook: the store-form projection GEMM (epilogue 0 above) in the mode the decoder layers run it in:
 * when the tile planner splits K, slice s of the product is stored to d_parts[s][M][N] (f32) for the
 * consumer kernel to add, in a fixed order and without atomics.  d_parts must hold SYNERA_MAX_GEMM_SLICES
 * x M x N floats; *h_n_parts (host) receives the number of slices written (1 when K was not split: the
 * whole product is then in slice 0).  N % 128 == 0, K % 64 == 0, else EUNSUP.
 */
int32_t synera_debug_gemm_slices(const void* d_a, const void* d_a_lo, const void* d_w, float* d_parts,
                                 int32_t M, int32_t N, int32_t K, int32_t* h_n_parts, void* stream);

/*
 * Test hook: copy one of the context's intermediate buffers, as the LAST layer of the last
 * verify left it, to caller device memory.  which: 0 residual x (f32 [T][d]; when the last
 * down projection ran K-split, its slices have been added only to the rows the LM head reads), 1/2 rotated q
 * hi/lo (bf16 [T][Hq*h]), 3/4 attention output hi/lo (fp16 [T][Hq*h], scaled by 64), 5/6 SiLU*mul output
 * hi/lo (fp16 [T][f], scaled by 8).  Where the projection that reads such a pair takes it as one array
 * (synera_debug_gemm_paired's form: its plan has 32-wide stages and no low part is switched off), buffers 3 + 4
 * (5 + 6), which lie back to back, hold that array instead: [T][n / 32][hi 32 | lo 32], read from `which` 3 (5)
 * on.  Errors: EINVAL, ENOSPC (bytes beyond the buffer), EHIP.
 */
int32_t synera_debug_read_scratch(synera_ctx* ctx, int32_t which, void* d_dst, int64_t bytes, void* stream);

/*
 * Ablation hook: the inputs of the projections and of the attention products travel as (hi, lo) pairs; a bit
 * set in `sites` makes later synera_verify calls on this context write the low part of that site as zeros
 * (numerically: the second matrix-core term of that product dropped).  1 normed rows -> QKV, 2 normed rows ->
 * gate/up, 4 SiLU*mul output -> down, 8 attention output -> O, 16 final normed rows -> LM head, 32 rotated q,
 * 64 attention probabilities.  The LM head runs on the high part alone by default (its bit, 16, changes
 * nothing); 128 gives it the pair.  0 restores the defaults.  Errors: EINVAL.
 */
#define SYNERA_LO_QKV_IN 1
#define SYNERA_LO_GATE_UP_IN 2
#define SYNERA_LO_DOWN_IN 4
#define SYNERA_LO_O_IN 8
#define SYNERA_LO_LM_HEAD_IN 16
#define SYNERA_LO_Q 32
#define SYNERA_LO_P 64
#define SYNERA_LO_KEEP_LM_HEAD 128
int32_t synera_debug_set_lo_off(synera_ctx* ctx, int32_t sites);

#ifdef __cplusplus
}
#endif
#endif /* SYNERA_DEBUG_H */
