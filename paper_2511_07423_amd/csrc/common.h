// Shared declarations of the HIP sources: vector types for the gfx950 matrix
// cores, launch helpers, and the host-side launchers each .hip file exports to
// the orchestration code in synera.cpp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bf16 bits in memory
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define SY_PAGE 16

// fp32 -> bf16, round-to-nearest-even, two at a time with gfx950's v_cvt_pk_bf16_f32.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint32_t f2bf(float f) { return pack_bf2(f, 0.f) & 0xFFFFu; }
__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }

// The inputs of the projection GEMMs travel between kernels as an fp16 pair (hi, lo): hi = fp16(s v),
// lo = fp16(s v - hi), 22 mantissa bits of the fp32 value v.  s is a power of two fixed per producer (below) that
// lifts typical activations to 2^3 .. 2^6, so that the lo part of all but tiny elements stays in fp16's normal
// range whether or not the matrix cores flush subnormal inputs; the consuming GEMM divides it out again.
// Scaled values beyond +-65504 (activations of magnitude 1000 / 8000) overflow to infinity and surface as
// non-finite logits: nothing is clamped, so a NaN in the input stays a NaN too.
#define SY_Y_SCALE 64.0f      // RMSNorm output (|y| <= sqrt(d) |gain|)
#define SY_O_SCALE 64.0f      // attention output (a convex combination of V rows)
#define SY_ACT_SCALE 8.0f     // SiLU(gate) * up
#define SY_W_SHIFT 8          // exponent added to the bf16 weights on their way to fp16 (weights below 256)
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
__device__ __forceinline__ void split_f16x2(float a, float b, uint32_t& hi, uint32_t& lo) {   // a, b: scaled values
  const f32x2_t v = {a, b};
  const f16x2_t h = __builtin_convertvector(v, f16x2_t);
  const f32x2_t r = v - __builtin_convertvector(h, f32x2_t);
  hi = __builtin_bit_cast(uint32_t, h);
  lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, f16x2_t));
}

// ---------------------------------------------------------------- elementwise.hip
struct BatchMeta {        // device pointers into one uploaded metadata blob (all int32)
  const int32_t* ctx_len;      // [B]
  const int32_t* cu_tok;       // [B+1] prefix sums of chunk lengths (u_i + k_i)
  const int32_t* block_table;  // [B][max_pages]
  const int32_t* tok_req;      // [T] request of each flattened chunk token
  const int32_t* sel_rows;     // [R'] chunk-token index feeding LM-head row r
  const int32_t* cu_draft;     // [B+1] prefix sums of k_i (output row offsets)
  const int32_t* first_row;    // [B] LM-head row of the last uncached token, or -1
  const int32_t* n_unc;        // [B]
  int32_t max_pages;
};

hipError_t launch_embed(const bf16_t* embed, const int32_t* tokens, float* x, int T, int d, int vocab,
                        hipStream_t s);
// parts / n_parts: pending K-split slices [n_parts][T][d] of the projection that feeds the residual; the
// kernel adds them to x first (and writes x back), so the GEMM needs no atomics.  n_parts = 0: none.
// y_hi / y_lo: the normalised rows as an fp16 pair scaled by SY_Y_SCALE (lo_off: the low part is written as zeros);
// paired: the pair goes to y_hi as one array [rows][d / 32][hi 32 | lo 32] (y_lo unused).
hipError_t launch_rmsnorm(float* x, const float* parts, int n_parts, size_t part_stride, const bf16_t* gain,
                          const int32_t* rows, uint16_t* y_hi, uint16_t* y_lo, int n_rows, int d, float eps,
                          bool lo_off, bool paired, hipStream_t s);
hipError_t launch_rope_table(const BatchMeta& m, float2* cs, int T, int head_dim, float base, hipStream_t s);
// n_parts > 0: qkv points at K-split slices [n_parts][T][(Hq+2Hkv) hd] whose sum is the projection.
hipError_t launch_rope_append(const float* qkv, int n_parts, size_t part_stride, const float2* cs, const BatchMeta& m,
                              bf16_t* q_hi, bf16_t* q_lo, bf16_t* k_layer, bf16_t* v_layer, int T, int Hq, int Hkv,
                              int hd, bool lo_off, hipStream_t s);
hipError_t launch_kv_append(const bf16_t* k, const bf16_t* v, const BatchMeta& m, int B, bf16_t* k_layer,
                            bf16_t* v_layer, int T, int Hkv, int hd, hipStream_t s);
hipError_t launch_accept(const int32_t* tokens, const int32_t* anchor, const int32_t* lm_argmax, const BatchMeta& m,
                         int B, int R, int32_t* out_argmax, int32_t* accept_len, int32_t* correction,
                         hipStream_t s);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s);

// ---------------------------------------------------------------- confidence.hip
hipError_t launch_confidence(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride,
                             int32_t* ids, float* p1, float* H, hipStream_t s);

hipError_t launch_confidence_topk(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride, int k,
                                  int32_t* ids, float* probs, float* margin, float* H, hipStream_t s);
hipError_t launch_nucleus(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride, float top_p,
                          int32_t* count, float* mass, float* cut_logit, hipStream_t s);
hipError_t launch_topp_count(const float* probs, int64_t rows, int k, float top_p, int32_t* n, float* mass,
                             hipStream_t s);
hipError_t launch_stochastic_accept(const float* logits, int vocab, const int32_t* lm_ids, const float* lm_p,
                                    const int32_t* tokens, const BatchMeta& m, int B, int k_list, const int32_t* p_id,
                                    const float* p_prob, const float* u_accept, const float* u_sample,
                                    int32_t* accept_len, int32_t* out_token, hipStream_t s);
hipError_t launch_chunk_dispatch(const float* p1, const int32_t* cu_rows, int B, float c_th, float k_slope,
                                 float* mean_conf, float* p_conf, hipStream_t s);

// ---------------------------------------------------------------- attention.hip
// The attention work of one call is a flat program of tile positions, cut into one share per persistent block.
enum { ATTN_POS_PAD = 0, ATTN_POS_KV = 1, ATTN_POS_Q = 2 };
#define ATTN_POS_KIND_MASK 7
#define ATTN_POS_LAST_BIT 8     // on the first position of an iteration: the stream's share ends with this iteration
struct AttnPos {       // 16 bytes, read with one scalar load
  int32_t tag;         // kind | LAST bit | payload << 4 (KV: KV head; Q: unit index)
  int32_t a;           // KV: page of keys 0..15 of the tile;  Q: flattened index of the group's first chunk token
  int32_t b;           // KV: page of keys 16..31 (or `a` again past the end);  Q: rows of the group (tokens x G)
  int32_t c;           // KV: first key of the tile;  Q: first of the 32 rows this position carries | KV head << 8
};
struct AttnUnit {      // one stream's share inside one block; 32 bytes, read with one scalar load
  int32_t tok0;        // flattened index of the group's first chunk token
  int32_t nrows;       // tokens x G (<= 64)
  int32_t lim0;        // last key the group's first token may see: L_i + j0 (row r: lim0 + r / G)
  int32_t key_end;     // exclusive end of this share's keys (the stream's end, or a multiple of 32)
  int32_t part;        // partial-result slot, or -1: the stream is whole here and writes o
  int32_t kh;          // KV head
  int32_t pad[2];
};
struct AttnShare {     // what one persistent block executes
  int32_t pos_begin, n_pos;   // its slice of the program (n_pos a multiple of 4 / rbn)
  int32_t rbn;                // 4: groups of more than 32 rows, 2: up to 32 rows
  int32_t pad;
};
struct AttnCut {       // a stream whose keys were split over several blocks
  int32_t part0, nsplit;      // its partial slots
  int32_t tok0, nrows, kh;
  int32_t pad[3];
};
struct AttnLaunch {
  const bf16_t* q;           // [T][Hq][hd], high part of the (hi, lo) bf16 pair
  const bf16_t* q_lo;        // low part
  const bf16_t* k_layer;     // pool of this layer
  const bf16_t* v_layer;
  const AttnPos* prog;       // device
  const AttnUnit* units;
  const AttnShare* shares;
  const AttnCut* cuts;
  int32_t n_shares, n_cuts;
  float* part_o;             // [slots][64][hd]
  float* part_ml;            // [slots][64][2]
  uint16_t* o;               // [T][Hq][hd], high part of the output's fp16 pair (scaled by SY_O_SCALE)
  uint16_t* o_lo;            // low part
  bool o_paired;             // write the pair to o as one array [T][Hq hd / 32][hi 32 | lo 32] instead (o_lo unused)
  int32_t lo_off;            // ablation: bit 0 drops the low part of the probabilities, bit 1 writes o_lo as zeros
  float2* row_ml;            // optional [T][Hq]: per query row the softmax reference m (exponent-2 domain) and
                             // the sum l of 2^(s - m) over its keys, i.e. p(key) = 2^(s scale log2e - m) / l
  int32_t T, Hq, Hkv, hd;
};
hipError_t launch_attention(const AttnLaunch& a, hipStream_t s);

// Importance scores (column sums of the attention matrix, mean over query heads) of one layer, from the
// rotated queries, the K pool and the per-row softmax statistics the attention kernel left.
struct ImportanceLaunch {
  const bf16_t* q;           // [T][Hq][hd] (hi, lo)
  const bf16_t* q_lo;
  float* qf;                 // scratch [T][Hq][hd]: the queries recombined to fp32
  const bf16_t* k_layer;
  const float2* row_ml;      // [T][Hq]
  const int32_t* ctx_len;    // device [B]
  const int32_t* cu_tok;     // device [B+1]
  const int32_t* block_table;// device [B][max_pages]
  const int32_t* cu_keys;    // device [B+1]: prefix sums of L_i + chunk_i (output offsets)
  const int32_t* items;      // device [n_items][2]: request, first key of the block's 256 keys
  int32_t n_items, max_pages, T, Hq, Hkv, hd, total_keys;
  float* importance;         // [cu_keys[B]]
  float* parts;              // scratch: the Hkv shares of a pass's items, [Hkv][items][256]
  size_t parts_cap;          // floats
};
hipError_t launch_importance(const ImportanceLaunch& a, hipStream_t s);
// mean score of each request's draft positions and P_imp of it (Section 4.2, second equation)
hipError_t launch_importance_dispatch(const float* importance, const int32_t* cu_keys, const int32_t* ctx_len,
                                      const int32_t* n_unc, const int32_t* cu_draft, int B, float i_th, float theta,
                                      float* mean_imp, float* p_imp, hipStream_t s);

// ---------------------------------------------------------------- gemm.hip
enum GemmEpilogue { GEMM_STORE_F32 = 0, GEMM_ADD_F32 = 1, GEMM_SWIGLU = 2 };
struct GemmArgs {
  const uint16_t* a;     // [M][K], high part of the activation's fp16 pair -- or, with a_paired, the whole pair as
                         // [M][K / 32][hi 32 | lo 32] (a_lo unused)
  const uint16_t* a_lo;  // [M][K], low part; nullptr without a_paired (STORE only): the high part alone is multiplied
  const bf16_t* w[3];    // up to three row segments of the bf16 weight (each [rows][K])
  int32_t w_rows[3];     // rows per segment (multiples of the N tile); unused = 0
  void* c;               // f32 [M][N] (STORE/ADD) or the high part of an fp16 pair [M][N/2] (SWIGLU: w[0] = gate, w[1] = up)
  void* c_lo;            // SWIGLU only: low part of the output pair
  int32_t M, N, K;       // N = total output columns of the contraction (gate + up for SWIGLU)
  int32_t epilogue;
  int32_t split_k;       // >= 1; > 1 only with STORE or ADD and c_parts: slice z is stored plainly to
                         // c_parts + z*M*N and c is left alone; the consumer kernel (RMSNorm, RoPE) adds the slices
  float* c_parts;        // [split_k][M][N] fp32, or nullptr (then the planner never splits K)
  float out_scale;       // accumulators x this = the product: 2^-SY_W_SHIFT / (the activation pair's scale)
  float c_scale;         // SWIGLU only: scale of the output pair (SY_ACT_SCALE)
  bool a_paired;         // the activations are one paired array (see a); only with tiles of one K step per stage
  bool c_paired;         // SWIGLU only: write the output pair as one paired array [M][N/2 / 32][hi 32 | lo 32] to c
};
// Element offset of column `col` inside a row of a paired array (row pitch: 2 x columns); the low part is 32 on.
__host__ __device__ __forceinline__ size_t pair_col(int col) { return (size_t)(col >> 5) * 64 + (col & 31); }
#define SY_MAX_K_SLICES 8
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);
int gemm_pick_split(const GemmArgs& g);                             // K slices launch_gemm should be given (1 without c_parts)
void gemm_plan(const GemmArgs& g, int* bm, int* bn, int* split);    // tile and K slices launch_gemm would use (host only)
void gemm_force_variant(int v);   // tuning hook: -1 automatic, else tile rows / 16 + (128-column tile ? 100 : 0) + (BK = 64 ? 200 : 0)
int gemm_plan_bk(const GemmArgs& g);                               // K extent of a stage the plan uses (32 or 64)
// the instantiations live in three translation units (compile time)
hipError_t launch_proj_nf4_low(int mt, const GemmArgs& g, hipStream_t s);    // 256 columns, 16 .. 144 rows
hipError_t launch_proj_nf4_high(int mt, const GemmArgs& g, hipStream_t s);   // 256 columns, 160 .. 272 rows
hipError_t launch_proj_nf2(int mt, const GemmArgs& g, hipStream_t s);        // 128 columns, 16 .. 192 rows
hipError_t launch_proj_k64(int mt, int nf, const GemmArgs& g, hipStream_t s);   // BK = 64: 128 columns x 16 .. 144 rows, 256 x 16 .. 80
