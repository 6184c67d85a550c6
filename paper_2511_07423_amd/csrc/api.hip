// Host side of the C ABI declared in include/synera.h: validation of the batch
// description, the context with its device scratch, the per-call plan (flattening
// of the ragged batch, attention work items) and the launch sequence of one verify.
// No arithmetic of the method happens on the host.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/synera.h"
#include "../../include/synera_debug.h"
#include "common.h"

#define SY_VERSION 100
#define N_STAGE 4              // metadata staging slots (calls may run this far ahead of the GPU)

#define HIP_TRY(expr)                       \
  do {                                      \
    if ((expr) != hipSuccess) {             \
      (void)hipGetLastError();              \
      return SYNERA_EHIP;                   \
    }                                       \
  } while (0)

extern "C" int32_t synera_version(void) { return SY_VERSION; }

extern "C" const char* synera_strerror(int32_t st) {
  switch (st) {
    case SYNERA_OK: return "ok";
    case SYNERA_EINVAL: return "invalid argument";
    case SYNERA_ERANGE: return "length or page id out of range, or page used twice";
    case SYNERA_ENOSPC: return "capacity (batch, tokens, block table) too small";
    case SYNERA_EUNSUP: return "unsupported shape or chunk length";
    case SYNERA_EHIP: return "HIP runtime error or no usable device";
    case SYNERA_ENOMEM: return "out of device memory";
    default: return "unknown status";
  }
}

// ------------------------------------------------------------------------------------ validation
extern "C" int32_t synera_validate_batch(int32_t B, const int32_t* h_ctx_len, const int32_t* h_n_first,
                                         const int32_t* h_n_second, const int32_t* h_block_table,
                                         int32_t max_pages, int32_t n_pages_in_pool, int32_t max_batch,
                                         int64_t max_tokens, int32_t chunk_limit) {
  if (!h_ctx_len || !h_n_first || !h_block_table) return SYNERA_EINVAL;
  if (B < 1 || max_pages < 1 || n_pages_in_pool < 1) return SYNERA_EINVAL;
  if (B > max_batch) return SYNERA_ENOSPC;
  int64_t total = 0;
  for (int i = 0; i < B; ++i) {
    const int32_t second = h_n_second ? h_n_second[i] : 0;
    if (h_n_first[i] < 1 || second < 0) return SYNERA_EINVAL;
    if (h_ctx_len[i] < 0) return SYNERA_ERANGE;
    const int64_t chunk = (int64_t)h_n_first[i] + second;
    if (chunk_limit > 0 && chunk > chunk_limit) return SYNERA_EUNSUP;
    total += chunk;
    const int64_t need = ((int64_t)h_ctx_len[i] + chunk + SYNERA_PAGE_SIZE - 1) / SYNERA_PAGE_SIZE;
    if (need > max_pages) return SYNERA_ENOSPC;
  }
  if (total > max_tokens) return SYNERA_ENOSPC;
  std::vector<uint8_t> used((size_t)n_pages_in_pool, 0);
  for (int i = 0; i < B; ++i) {
    const int64_t chunk = (int64_t)h_n_first[i] + (h_n_second ? h_n_second[i] : 0);
    const int64_t need = ((int64_t)h_ctx_len[i] + chunk + SYNERA_PAGE_SIZE - 1) / SYNERA_PAGE_SIZE;
    for (int64_t p = 0; p < need; ++p) {
      const int32_t id = h_block_table[(size_t)i * max_pages + p];
      if (id < 0 || id >= n_pages_in_pool) return SYNERA_ERANGE;
      if (used[id]) return SYNERA_ERANGE;
      used[id] = 1;
    }
  }
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ context
struct synera_ctx {
  synera_model_desc desc;
  std::vector<synera_layer_weights> layers;
  const void* embed;
  const void* final_norm;
  const void* lm_head;
  int32_t max_batch, max_tokens, max_pages, max_rows, rows_per_group_tokens;
  int32_t attn_blocks, attn_blocks_cap;   // persistent attention blocks in use / the most the scratch is sized for
  size_t pos_cap, unit_cap, part_cap;   // capacities of the attention program, its stream shares, the partial slots
  int device;
  // attention share planner (set once in synera_create)
  double attn_stream_cost, attn_cut_slack, attn_t_iter[2];
  int32_t lo_off;              // test hook: SYNERA_LO_* sites whose low activation part is written as zeros
  // device scratch (one allocation)
  char* arena;
  float* x;
  uint16_t* y;      // GEMM inputs travel as scaled fp16 (hi, lo) pairs: *_lo is the low part
  uint16_t* y_lo;
  float* qkv;
  bf16_t* q;        // rotated queries: a bf16 pair (they meet the bf16 cache in the attention kernel)
  bf16_t* q_lo;
  uint16_t* o;
  uint16_t* o_lo;
  uint16_t* act;
  uint16_t* act_lo;
  uint16_t* ysel;
  uint16_t* ysel_lo;
  float* logits;
  int32_t* lm_ids;
  float* lm_p;
  float* lm_h;
  float2* cs;
  float* part_o;
  float* part_ml;
  float2* row_ml;              // [max_tokens][Hq] softmax statistics of the last layer's attention rows
  // batch of the last synera_verify, for synera_importance: device pointers into that call's metadata slot
  struct {
    const int32_t *ctx_len, *cu_tok, *block_table, *cu_keys, *items, *n_unc, *cu_draft;
    BatchMeta meta;
    int32_t B, T, R, n_items, max_pages, total_keys, n_pages_in_pool, slot;
    const void* k_pool;
    bool valid;
    bool all_rows_kept;          // every request had an uncached token: c->logits / lm_ids / lm_p hold all LM-head rows
  } last;
  float* gparts;               // K-split slices of one projection: [SY_MAX_K_SLICES][max_tokens][max(d, q+2kv)]
  size_t gpart_elems;          // elements of one slice slot
  // metadata staging ring
  size_t meta_cap;             // bytes per slot
  int32_t* h_meta[N_STAGE];    // pinned host
  int32_t* d_meta[N_STAGE];
  hipEvent_t done[N_STAGE];
  bool pending[N_STAGE];
  uint64_t calls;
  // optional per-stage timing: every launch of `prof_stage` is bracketed by an event pair
  int32_t prof_stage;
  std::vector<hipEvent_t> prof_events;   // start/stop pairs, created on demand and reused
  size_t prof_used;
};

struct StageTimer {                      // brackets one stage launch when profiling of it is on
  synera_ctx* c;
  hipStream_t s;
  bool on;
  StageTimer(synera_ctx* c_, int32_t stage, hipStream_t s_) : c(c_), s(s_), on(c_->prof_stage == stage) {
    if (on) mark();
  }
  ~StageTimer() {
    if (on) mark();
  }
  void mark() {
    if (c->prof_used == c->prof_events.size()) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) { on = false; (void)hipGetLastError(); return; }
      c->prof_events.push_back(e);
    }
    (void)hipEventRecord(c->prof_events[c->prof_used++], s);
  }
};

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Capacities of the per-call metadata (c->desc, max_batch / max_tokens / max_pages / max_rows and attn_blocks_cap
// are set).  Worst case: every request at the full block table.  A stream (row group x KV head) has at most
// max_pages / 2 + 1 key tiles; every share of a stream adds two query positions and at most one padding
// position; cutting adds at most one share per block.
static void size_plan(synera_ctx* c) {
  const synera_model_desc& m = c->desc;
  const int G = m.n_q_heads / m.n_kv_heads;
  c->rows_per_group_tokens = std::max(1, 64 / G);
  const int rg_max = (SYNERA_MAX_CHUNK + c->rows_per_group_tokens - 1) / c->rows_per_group_tokens;
  const size_t streams = (size_t)c->max_batch * rg_max * m.n_kv_heads;
  const size_t tiles = (size_t)c->max_pages / 2 + 2;
  c->unit_cap = streams + (size_t)c->attn_blocks_cap;
  c->pos_cap = streams * tiles + c->unit_cap * 4 + 2 * (size_t)c->attn_blocks_cap;
  c->part_cap = 2 * (size_t)c->attn_blocks_cap;
  const size_t meta_ints = (size_t)c->max_batch * 5 + 2 + (size_t)c->max_tokens + (size_t)c->max_rows +
                           (size_t)c->max_batch * c->max_pages + c->pos_cap * 4 + c->unit_cap * 8 +
                           (size_t)c->attn_blocks_cap * 4 + c->part_cap * 8 + 128 + ((size_t)c->max_batch + 1) +
                           2 * (size_t)c->max_batch * ((size_t)c->max_pages / 16 + 2);
  c->meta_cap = align_up(meta_ints * 4, 256);
}

// Constants of the attention share planner (build_plan).
static void attention_plan_defaults(synera_ctx* c) {
  // What a stream costs a block beyond its tiles and query positions (its last iteration merges the key phases
  // or writes partials, and stores the rows), in iterations: part of the balance between blocks.  One iteration,
  // from a sweep on the 8B ragged batch of 64 (512 streams of 4 to 128 tiles on 512 blocks: 94 us per layer
  // without the term, 89 - 90 us with 1, 91 us with 2; the uniform batches do not care).
  c->attn_stream_cost = 1.0;
  // A stream that overshoots its block's share by less than this is not cut (iterations; swept: 0 .. 1.5 best,
  // 3 +1.5 %, 8 +9 %).
  c->attn_cut_slack = 1.5;
  // Relative time per iteration of the two classes (four row blocks, one tile: 1; two row blocks x two key
  // phases, two tiles: 1.85), which decides how many of the persistent blocks each class gets.  From a sweep of
  // the ratio on that batch, where the classes hold about half of the tiles each: 1.8 - 2.0 gives the shortest
  // launch (94 us against 98 us at 1.4, the ratio of the two classes timed alone).
  c->attn_t_iter[0] = 1.85;
  c->attn_t_iter[1] = 3.4;
}

extern "C" int32_t synera_create(synera_ctx** out, const synera_model_desc* desc, const synera_weights* w,
                                 int32_t max_batch, int32_t max_tokens, int32_t max_pages) {
  if (!out) return SYNERA_EINVAL;
  *out = nullptr;
  if (!desc || !w || !w->layers || !w->embed || !w->final_norm || !w->lm_head) return SYNERA_EINVAL;
  if (max_batch < 1 || max_tokens < 1 || max_pages < 1) return SYNERA_EINVAL;
  const synera_model_desc& m = *desc;
  if (m.n_layers < 1 || m.d_model < 1 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.d_ffn < 1 || m.vocab < 1)
    return SYNERA_EINVAL;
  if (!(m.rope_base > 1.0f) || !(m.rms_eps >= 0.0f)) return SYNERA_EINVAL;
  if (m.head_dim != 64 && m.head_dim != 128) return SYNERA_EUNSUP;
  if (m.n_q_heads % m.n_kv_heads != 0 || m.n_q_heads / m.n_kv_heads > 16) return SYNERA_EUNSUP;
  const int64_t qd = (int64_t)m.n_q_heads * m.head_dim, kd = (int64_t)m.n_kv_heads * m.head_dim;
  // GEMM tiles are 128 output columns by 64 of K; Wq | Wk | Wv are segments of one launch.
  if (m.d_model % 128 || m.d_ffn % 64 || m.vocab % 128 || qd % 128 || kd % 128) return SYNERA_EUNSUP;
  for (int l = 0; l < m.n_layers; ++l) {
    const synera_layer_weights& lw = w->layers[l];
    if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.mlp_norm || !lw.w_gate || !lw.w_up ||
        !lw.w_down)
      return SYNERA_EINVAL;
  }
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));

  synera_ctx* c = new (std::nothrow) synera_ctx();
  if (!c) return SYNERA_ENOMEM;
  c->desc = m;
  c->layers.assign(w->layers, w->layers + m.n_layers);
  c->embed = w->embed;
  c->final_norm = w->final_norm;
  c->lm_head = w->lm_head;
  c->max_batch = max_batch;
  c->max_tokens = max_tokens;
  c->max_pages = max_pages;
  c->max_rows = max_tokens + max_batch;
  c->device = dev;
  // Attention runs as persistent blocks, two per compute unit (80 KB of LDS each at head_dim 128).
  {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
      (void)hipGetLastError();
      delete c;
      return SYNERA_EHIP;
    }
    c->attn_blocks = 2 * std::max(1, prop.multiProcessorCount);
    c->attn_blocks_cap = 2 * c->attn_blocks;
  }
  attention_plan_defaults(c);
  c->lo_off = 0;
  size_plan(c);

  const size_t T = (size_t)max_tokens, R = (size_t)c->max_rows;
  const size_t qkv_dim = (size_t)(qd + 2 * kd);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
  // Each (hi, lo) pair is taken back to back: where a projection reads its pair as one array (gemm_takes_pairs),
  // that array starts at the high part's place and spans both.
  const size_t o_x = take(T * m.d_model * 4), o_y = take(T * m.d_model * 2), o_yl = take(T * m.d_model * 2);
  const size_t o_qkv = take(T * qkv_dim * 4);
  const size_t o_q = take(T * qd * 2), o_ql = take(T * qd * 2), o_o = take(T * qd * 2), o_ol = take(T * qd * 2);
  const size_t o_act = take(T * (size_t)m.d_ffn * 2), o_actl = take(T * (size_t)m.d_ffn * 2);
  const size_t o_ysel = take(R * m.d_model * 2), o_ysell = take(R * m.d_model * 2);
  const size_t o_logits = take(R * (size_t)m.vocab * 4);
  const size_t o_ids = take(R * 4), o_p = take(R * 4), o_h = take(R * 4);
  const size_t o_cs = take(T * (m.head_dim / 2) * 8);
  const size_t o_po = take(c->part_cap * 64 * m.head_dim * 4);
  const size_t o_pml = take(c->part_cap * 64 * 2 * 4);
  const size_t o_rml = take(T * (size_t)m.n_q_heads * 8);
  c->gpart_elems = T * std::max<size_t>(qkv_dim, (size_t)m.d_model);
  const size_t o_gp = take(SY_MAX_K_SLICES * c->gpart_elems * 4);
  if (hipMalloc(reinterpret_cast<void**>(&c->arena), off) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return SYNERA_ENOMEM;
  }
  c->x = reinterpret_cast<float*>(c->arena + o_x);
  c->y = reinterpret_cast<uint16_t*>(c->arena + o_y);
  c->y_lo = reinterpret_cast<uint16_t*>(c->arena + o_yl);
  c->q_lo = reinterpret_cast<bf16_t*>(c->arena + o_ql);
  c->o_lo = reinterpret_cast<uint16_t*>(c->arena + o_ol);
  c->act_lo = reinterpret_cast<uint16_t*>(c->arena + o_actl);
  c->ysel_lo = reinterpret_cast<uint16_t*>(c->arena + o_ysell);
  c->qkv = reinterpret_cast<float*>(c->arena + o_qkv);
  c->q = reinterpret_cast<bf16_t*>(c->arena + o_q);
  c->o = reinterpret_cast<uint16_t*>(c->arena + o_o);
  c->act = reinterpret_cast<uint16_t*>(c->arena + o_act);
  c->ysel = reinterpret_cast<uint16_t*>(c->arena + o_ysel);
  c->logits = reinterpret_cast<float*>(c->arena + o_logits);
  c->lm_ids = reinterpret_cast<int32_t*>(c->arena + o_ids);
  c->lm_p = reinterpret_cast<float*>(c->arena + o_p);
  c->lm_h = reinterpret_cast<float*>(c->arena + o_h);
  c->cs = reinterpret_cast<float2*>(c->arena + o_cs);
  c->part_o = reinterpret_cast<float*>(c->arena + o_po);
  c->part_ml = reinterpret_cast<float*>(c->arena + o_pml);
  c->row_ml = reinterpret_cast<float2*>(c->arena + o_rml);
  c->last.valid = false;
  c->gparts = reinterpret_cast<float*>(c->arena + o_gp);

  for (int s = 0; s < N_STAGE; ++s) {
    c->h_meta[s] = nullptr;
    c->d_meta[s] = nullptr;
    c->done[s] = nullptr;
    c->pending[s] = false;
  }
  bool ok = true;
  for (int s = 0; s < N_STAGE && ok; ++s) {
    ok = hipHostMalloc(reinterpret_cast<void**>(&c->h_meta[s]), c->meta_cap, hipHostMallocDefault) == hipSuccess &&
         hipMalloc(reinterpret_cast<void**>(&c->d_meta[s]), c->meta_cap) == hipSuccess &&
         hipEventCreateWithFlags(&c->done[s], hipEventDisableTiming) == hipSuccess;
  }
  if (!ok) {
    (void)hipGetLastError();
    synera_destroy(c);
    return SYNERA_ENOMEM;
  }
  c->calls = 0;
  c->prof_stage = SYNERA_STAGE_NONE;
  c->prof_used = 0;
  *out = c;
  return SYNERA_OK;
}

extern "C" int32_t synera_destroy(synera_ctx* c) {
  if (!c) return SYNERA_OK;
  (void)hipDeviceSynchronize();
  for (int s = 0; s < N_STAGE; ++s) {
    if (c->done[s]) (void)hipEventDestroy(c->done[s]);
    if (c->h_meta[s]) (void)hipHostFree(c->h_meta[s]);
    if (c->d_meta[s]) (void)hipFree(c->d_meta[s]);
  }
  for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
  if (c->arena) (void)hipFree(c->arena);
  delete c;
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ per-call plan
struct Plan {
  BatchMeta meta;
  const AttnPos* d_prog;
  const AttnUnit* d_units;
  const AttnShare* d_shares;
  const AttnCut* d_cuts;
  int32_t n_shares, n_cuts;
  int32_t T, R, R_all;      // chunk tokens, draft rows, LM-head rows (drafts + last-uncached rows)
  const int32_t *d_cu_keys, *d_imp_items;   // importance-score blocks: prefix sums of L_i + chunk_i; (request, first key)
  int32_t n_imp_items, total_keys;
  int slot;
};

// Lays the metadata out in the staging slot, uploads it, and returns device pointers.
// n_second == nullptr means "append only": no LM rows, no attention items.
static int32_t build_plan(synera_ctx* c, int32_t B, const int32_t* ctx_len, const int32_t* n_unc,
                          const int32_t* n_draft, const int32_t* block_table, int32_t max_pages, bool with_attention,
                          hipStream_t stream, Plan& p, bool host_only = false, bool* uploaded = nullptr) {
  c->last.valid = false;       // the metadata slots rotate: what synera_importance reads belongs to the newest verify only
  const int slot = (int)(c->calls % N_STAGE);
  if (!host_only && c->pending[slot]) {
    HIP_TRY(hipEventSynchronize(c->done[slot]));
    c->pending[slot] = false;
  }
  int32_t* h = c->h_meta[slot];
  int32_t* d = c->d_meta[slot];
  size_t at = 0;
  auto region = [&](size_t n) { size_t r = at; at += n; return r; };
  const size_t o_ctx = region(B), o_cu = region(B + 1), o_cud = region(B + 1), o_first = region(B), o_unc = region(B);
  int32_t T = 0, R = 0;
  for (int i = 0; i < B; ++i) {
    const int u = n_unc ? n_unc[i] : 0;
    h[o_ctx + i] = ctx_len[i];
    h[o_cu + i] = T;
    h[o_cud + i] = R;
    h[o_unc + i] = u;
    T += u + n_draft[i];
    R += n_draft[i];
  }
  h[o_cu + B] = T;
  h[o_cud + B] = R;
  const size_t o_bt = region((size_t)B * max_pages);
  std::memcpy(h + o_bt, block_table, (size_t)B * max_pages * sizeof(int32_t));
  size_t o_req = 0, o_sel = 0;
  int32_t R_all = R;
  p.n_shares = p.n_cuts = 0;
  p.d_prog = nullptr;
  p.d_units = nullptr;
  p.d_shares = nullptr;
  p.d_cuts = nullptr;
  if (with_attention) {
    o_req = region(T);
    o_sel = region((size_t)R + B);
    for (int i = 0; i < B; ++i) {
      const int u = n_unc[i], base = h[o_cu + i];
      for (int j = 0; j < u + n_draft[i]; ++j) h[o_req + base + j] = i;
      for (int j = 0; j < n_draft[i]; ++j) h[o_sel + h[o_cud + i] + j] = base + u + j;
    }
    for (int i = 0; i < B; ++i) {           // rows of the last uncached tokens follow the draft rows
      if (n_unc[i] > 0) {
        h[o_first + i] = R_all;
        h[o_sel + R_all] = h[o_cu + i] + n_unc[i] - 1;
        ++R_all;
      } else {
        h[o_first + i] = -1;
      }
    }
    // ---- blocks of the optional importance-score pass: 256 consecutive keys of one request each
    {
      const size_t o_cuk = region((size_t)B + 1);
      int32_t keys = 0, n_items = 0;
      for (int i = 0; i < B; ++i) {
        h[o_cuk + i] = keys;
        keys += ctx_len[i] + n_unc[i] + n_draft[i];
      }
      h[o_cuk + B] = keys;
      const size_t o_items = region(2 * (size_t)B * ((size_t)max_pages / 16 + 2));
      for (int i = 0; i < B; ++i)
        for (int k0 = 0; k0 < ctx_len[i] + n_unc[i] + n_draft[i]; k0 += 256) {
          h[o_items + 2 * n_items] = i;
          h[o_items + 2 * n_items + 1] = k0;
          ++n_items;
        }
      p.d_cu_keys = d + o_cuk;
      p.d_imp_items = d + o_items;
      p.n_imp_items = n_items;
      p.total_keys = keys;
    }
    // ---- attention program.  A stream = (row group of up to `tg` chunk tokens x G heads <= 64 rows, KV head)
    // with the keys 0 .. L + j_last it sees, in 32-key tiles.  Streams of a class (more than 32 rows /
    // up to 32 rows) are laid end to end and cut into shares of equal modelled time, one per block.
    const int G = c->desc.n_q_heads / c->desc.n_kv_heads, Hkv = c->desc.n_kv_heads;
    const int tg = c->rows_per_group_tokens;
    const double stream_cost = c->attn_stream_cost, cut_slack = c->attn_cut_slack;
    struct Stream { int req, tok0, j0, ntok, keys; };
    std::vector<Stream> cls[2];                      // [0]: rbn 4, [1]: rbn 2
    double iters[2] = {0.0, 0.0};                    // iterations of each class (every stream once per KV head)
    for (int i = 0; i < B; ++i) {
      const int qn = n_unc[i] + n_draft[i];
      for (int j0 = 0; j0 < qn; j0 += tg) {
        const int ntok = std::min(tg, qn - j0);
        const Stream st{i, h[o_cu + i] + j0, j0, ntok, ctx_len[i] + j0 + ntok};
        const int k = ntok * G > 32 ? 0 : 1;
        const int tiles = (st.keys + 31) / 32;
        cls[k].push_back(st);
        iters[k] += Hkv * ((k == 0 ? 2 + tiles : 1 + (tiles + 1) / 2) + stream_cost);
      }
    }
    const double t_iter[2] = {c->attn_t_iter[0], c->attn_t_iter[1]};
    const double time_all = iters[0] * t_iter[0] + iters[1] * t_iter[1];
    int nb[2] = {0, 0};
    for (int k = 0; k < 2; ++k)
      if (!cls[k].empty()) {
        nb[k] = (int)std::lround(c->attn_blocks * iters[k] * t_iter[k] / time_all);
        nb[k] = std::max(1, std::min(nb[k], (int)(iters[k] / 8) + 1));   // at least ~8 iterations per block
      }
    if (nb[0] + nb[1] > c->attn_blocks) (nb[0] > nb[1] ? nb[0] : nb[1]) -= nb[0] + nb[1] - c->attn_blocks;

    at = (at + 7) & ~(size_t)7;                      // 32-byte alignment for the structs
    // the program goes last: only its used part is uploaded
    const size_t o_units = region(c->unit_cap * 8), o_shares = region((size_t)c->attn_blocks_cap * 4);
    const size_t o_cuts = region(c->part_cap * 8), o_prog = region(c->pos_cap * 4);
    AttnPos* prog = reinterpret_cast<AttnPos*>(h + o_prog);
    AttnUnit* units = reinterpret_cast<AttnUnit*>(h + o_units);
    AttnShare* shares = reinterpret_cast<AttnShare*>(h + o_shares);
    AttnCut* cuts = reinterpret_cast<AttnCut*>(h + o_cuts);
    size_t n_pos = 0, n_units = 0, n_shares = 0, n_cuts = 0, n_part = 0;
    for (int k = 0; k < 2; ++k) {
      if (cls[k].empty()) continue;
      const int rbn = k == 0 ? 4 : 2, KP = 4 / rbn, q_iters = k == 0 ? 2 : 1;
      // Every share aims at an equal part of what is left (a cut adds the second share's query positions
      // to the total, so the aim is renewed at each share rather than fixed up front).
      double rest = iters[k];
      int blocks_left = nb[k];
      const double q_cost = q_iters + stream_cost;       // modelled cost of starting (and ending) a share
      double target = rest / blocks_left + q_cost;
      double load = 0.0;
      size_t share_begin = n_pos;
      auto close_share = [&]() {
        if (n_pos > share_begin) {
          shares[n_shares++] = AttnShare{(int32_t)share_begin, (int32_t)(n_pos - share_begin), rbn, 0};
          --blocks_left;
          if (blocks_left > 0) target = std::max(rest, 0.0) / blocks_left + q_cost;
        }
        share_begin = n_pos;
        load = 0.0;
      };
      for (const Stream& st : cls[k]) {
        const int tiles = (st.keys + 31) / 32, pages = (st.keys + SYNERA_PAGE_SIZE - 1) / SYNERA_PAGE_SIZE;
        const int32_t* bt = block_table + (size_t)st.req * max_pages;
        for (int kh = 0; kh < Hkv; ++kh) {
          int t_done = 0, cut = -1;                  // cut: index into cuts[] once the stream is split
          while (t_done < tiles) {
            const int t_left = tiles - t_done;
            const double room = target - load;
            const double need_all = q_cost + (t_left + KP - 1) / KP;
            int take = t_left;
            if (blocks_left > 1 && need_all > room + cut_slack) {    // does not fit: cut here, or start in the next block
              const int fit = (int)(room - q_cost) * KP;
              if (fit < 4 * KP) {
                if (load > 0.0) {
                  close_share();
                  continue;
                }
                take = std::min(t_left, std::max(KP, (int)(target - q_cost) * KP));
              } else {
                take = std::min(t_left, fit);
              }
            }
            const bool whole = take == tiles;
            if (!whole && cut < 0) {
              if (n_cuts >= c->part_cap) return SYNERA_ENOSPC;
              cut = (int)n_cuts++;
              cuts[cut] = AttnCut{(int32_t)n_part, 0, st.tok0, st.ntok * G, kh, {0, 0, 0}};
            }
            if (n_units >= c->unit_cap || n_pos + (size_t)take + 4 > c->pos_cap || n_part >= c->part_cap)
              return SYNERA_ENOSPC;                  // cannot happen: the capacities are worst cases
            const int t_end = t_done + take;
            AttnUnit& u = units[n_units];
            u = AttnUnit{st.tok0, st.ntok * G, ctx_len[st.req] + st.j0, std::min(st.keys, 32 * t_end),
                         whole ? -1 : (int32_t)n_part, kh, {0, 0}};
            if (!whole) {
              ++n_part;
              ++cuts[cut].nsplit;
            }
            // query positions (32 rows each; the two-phase class pads its pair), then the key tiles
            prog[n_pos++] = AttnPos{ATTN_POS_Q | (int32_t)(n_units << 4), st.tok0, st.ntok * G, 0 | (kh << 8)};
            if (k == 0) prog[n_pos++] = AttnPos{ATTN_POS_Q | (int32_t)(n_units << 4), st.tok0, st.ntok * G, 32 | (kh << 8)};
            else prog[n_pos++] = AttnPos{ATTN_POS_PAD, 0, 0, 0};
            ++n_units;
            const size_t first_kv = n_pos;
            for (int t = t_done; t < t_end; ++t) {
              const int pa = bt[2 * t], pb = 2 * t + 1 < pages ? bt[2 * t + 1] : pa;
              prog[n_pos++] = AttnPos{ATTN_POS_KV | (kh << 4), pa, pb, 32 * t};
            }
            if ((n_pos - first_kv) % KP) prog[n_pos++] = AttnPos{ATTN_POS_PAD, 0, 0, 0};
            prog[n_pos - KP].tag |= ATTN_POS_LAST_BIT;       // first position of the share's last iteration
            load += q_cost + (take + KP - 1) / KP;
            rest -= (t_done == 0 ? q_cost : 0.0) + (take + KP - 1) / KP;
            t_done = t_end;
            if (blocks_left > 1 && load >= target - 0.5) close_share();
          }
        }
      }
      close_share();
    }
    p.n_shares = (int32_t)n_shares;
    p.n_cuts = (int32_t)n_cuts;
    p.d_prog = reinterpret_cast<const AttnPos*>(d + o_prog);
    p.d_units = reinterpret_cast<const AttnUnit*>(d + o_units);
    p.d_shares = reinterpret_cast<const AttnShare*>(d + o_shares);
    p.d_cuts = reinterpret_cast<const AttnCut*>(d + o_cuts);
    at = o_prog + n_pos * 4;
  }
  if (at * 4 > c->meta_cap) return SYNERA_ENOSPC;
  p.slot = slot;
  if (!host_only) {
    HIP_TRY(hipMemcpyAsync(d, h, at * 4, hipMemcpyHostToDevice, stream));
    if (uploaded) *uploaded = true;
  }
  p.meta.ctx_len = d + o_ctx;
  p.meta.cu_tok = d + o_cu;
  p.meta.cu_draft = d + o_cud;
  p.meta.first_row = d + o_first;
  p.meta.n_unc = d + o_unc;
  p.meta.block_table = d + o_bt;
  p.meta.tok_req = d + o_req;
  p.meta.sel_rows = d + o_sel;
  p.meta.max_pages = max_pages;
  p.T = T;
  p.R = R;
  p.R_all = R_all;
  p.slot = slot;
  return SYNERA_OK;
}

static int32_t finish_call(synera_ctx* c, const Plan& p, hipStream_t stream) {
  HIP_TRY(hipEventRecord(c->done[p.slot], stream));
  c->pending[p.slot] = true;
  c->calls++;
  return SYNERA_OK;
}

// The planner's view of a projection of M rows (host only: the pointers are only asked whether they are there).
static int32_t plan_args(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t stored_slices, GemmArgs* g) {
  if (M < 1 || N < 1 || K < 1 || epilogue < 0 || epilogue > 2) return SYNERA_EINVAL;
  if (N % (epilogue == GEMM_SWIGLU ? 256 : 128) != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  *g = GemmArgs{};
  g->a_lo = reinterpret_cast<const uint16_t*>(uintptr_t(64));
  g->w_rows[0] = epilogue == GEMM_SWIGLU ? N / 2 : N;
  g->w_rows[1] = epilogue == GEMM_SWIGLU ? N / 2 : 0;
  g->M = M;
  g->N = N;
  g->K = K;
  g->epilogue = epilogue;
  g->split_k = 1;
  g->c_parts = stored_slices && epilogue != GEMM_SWIGLU ? reinterpret_cast<float*>(uintptr_t(64)) : nullptr;
  return SYNERA_OK;
}

// Whether a two-term projection of M rows takes its activations as one paired array ([M][K / 32][hi | lo]: whole
// 128-byte lines per copy): where its plan has one MFMA K step per stage.  The producer kernel is told the same.
static bool gemm_takes_pairs(int M, int N, int K, int epi, bool stored) {
  GemmArgs g;
  return plan_args(M, N, K, epi, stored, &g) == SYNERA_OK && gemm_plan_bk(g) == 32;
}

// One projection.  a / a_lo: the fp16 pair of a_scale x activation; a_paired: both in the one array a
// ([M][K / 32][hi 32 | lo 32]); c_paired (SwiGLU): the output pair in that form in cbuf.  parts / n_parts: if given, the planner may
// split K; the slices are then stored to `parts` ([n][M][N], *n_parts = n) for the consumer kernel to add, and
// cbuf is left alone; otherwise *n_parts = 0 and cbuf holds the result.
static int32_t run_gemm(const uint16_t* a, const uint16_t* a_lo, float a_scale, const void* w0, int r0, const void* w1,
                        int r1, const void* w2, int r2, void* cbuf, void* cbuf_lo, int M, int N, int K, int epi,
                        hipStream_t s, float* parts = nullptr, int* n_parts = nullptr, bool a_paired = false,
                        bool c_paired = false) {
  GemmArgs g;
  g.a = a;
  g.a_lo = a_paired ? nullptr : a_lo;
  g.a_paired = a_paired;
  g.c_paired = c_paired;
  g.c_lo = cbuf_lo;
  g.w[0] = static_cast<const bf16_t*>(w0);
  g.w[1] = static_cast<const bf16_t*>(w1);
  g.w[2] = static_cast<const bf16_t*>(w2);
  g.w_rows[0] = r0;
  g.w_rows[1] = r1;
  g.w_rows[2] = r2;
  g.c = cbuf;
  g.M = M;
  g.N = N;
  g.K = K;
  g.epilogue = epi;
  g.split_k = 1;
  g.c_parts = (parts && n_parts && epi != GEMM_SWIGLU) ? parts : nullptr;
  g.out_scale = 1.0f / ((float)(1 << SY_W_SHIFT) * a_scale);
  g.c_scale = SY_ACT_SCALE;
  g.split_k = gemm_pick_split(g);
  if (n_parts) *n_parts = g.split_k > 1 ? g.split_k : 0;
  HIP_TRY(launch_gemm(g, s));
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ verify
// Sites whose activations travel as (hi, lo) pairs; a bit set in synera_ctx::lo_off makes the producer write the
// low part as zeros (synera_debug_set_lo_off: the ablation that shows which sites need the second term).
enum { LO_QKV_IN = SYNERA_LO_QKV_IN, LO_GATE_UP_IN = SYNERA_LO_GATE_UP_IN, LO_DOWN_IN = SYNERA_LO_DOWN_IN,
       LO_O_IN = SYNERA_LO_O_IN, LO_LM_HEAD_IN = SYNERA_LO_LM_HEAD_IN, LO_Q = SYNERA_LO_Q, LO_P = SYNERA_LO_P };

// Every launch of one verify, after the plan's metadata upload has been queued.
static int32_t verify_launches(synera_ctx* c, const Plan& p, int32_t B, const int32_t* d_tokens, const int32_t* d_anchor,
                               int32_t n_pages_in_pool, void* d_k_pool, void* d_v_pool, float* d_logits,
                               int32_t* d_argmax, float* d_top1_prob, float* d_entropy, int32_t* d_accept_len,
                               int32_t* d_correction, hipStream_t s) {
  const synera_model_desc& m = c->desc;
  int32_t st;
  const int T = p.T, d = m.d_model, Hq = m.n_q_heads, Hkv = m.n_kv_heads, hd = m.head_dim;
  const int qd = Hq * hd, kd = Hkv * hd;
  const int lo_off = c->lo_off;
  const size_t layer_elems = (size_t)n_pages_in_pool * Hkv * SY_PAGE * hd;
  HIP_TRY(launch_embed(static_cast<const bf16_t*>(c->embed), d_tokens, c->x, T, d, m.vocab, s));
  HIP_TRY(launch_rope_table(p.meta, c->cs, T, hd, m.rope_base, s));

  AttnLaunch al;
  al.q = c->q;
  al.q_lo = c->q_lo;
  al.o_lo = c->o_lo;
  al.prog = p.d_prog;
  al.units = p.d_units;
  al.shares = p.d_shares;
  al.cuts = p.d_cuts;
  al.n_shares = p.n_shares;
  al.n_cuts = p.n_cuts;
  al.part_o = c->part_o;
  al.part_ml = c->part_ml;
  al.o = c->o;
  al.lo_off = ((lo_off & LO_P) ? 1 : 0) | ((lo_off & LO_O_IN) ? 2 : 0);
  al.T = T;
  al.Hq = Hq;
  al.Hkv = Hkv;
  al.hd = hd;

  // Which projections read their activation pair as one paired array (the producer writes it that way then).  The
  // ablation of low parts works on separate arrays: any of its bits keeps them.
  const bool pair_qkv = !lo_off && gemm_takes_pairs(T, qd + 2 * kd, d, GEMM_STORE_F32, true);
  const bool pair_o = !lo_off && gemm_takes_pairs(T, d, qd, GEMM_ADD_F32, true);
  const bool pair_gu = !lo_off && gemm_takes_pairs(T, 2 * m.d_ffn, d, GEMM_SWIGLU, true);
  const bool pair_down = !lo_off && gemm_takes_pairs(T, d, m.d_ffn, GEMM_ADD_F32, true);
  al.o_paired = pair_o;

  // K-split projections leave their slices in c->gparts; the kernel that reads the result next adds them
  // (RMSNorm for the two residual projections, RoPE for QKV).  pend = slices waiting to be added to x.
  int pend = 0;
  const size_t x_stride = (size_t)T * d, qkv_stride = (size_t)T * (qd + 2 * kd);
  for (int l = 0; l < m.n_layers; ++l) {
    const synera_layer_weights& w = c->layers[l];
    bf16_t* k_layer = static_cast<bf16_t*>(d_k_pool) + (size_t)l * layer_elems;
    bf16_t* v_layer = static_cast<bf16_t*>(d_v_pool) + (size_t)l * layer_elems;
    {
      StageTimer t(c, SYNERA_STAGE_NORM, s);
      HIP_TRY(launch_rmsnorm(c->x, c->gparts, pend, x_stride, static_cast<const bf16_t*>(w.attn_norm), nullptr, c->y,
                             c->y_lo, T, d, m.rms_eps, (lo_off & LO_QKV_IN) != 0, pair_qkv, s));
      pend = 0;
    }
    int qkv_parts = 0;
    {
      StageTimer t(c, SYNERA_STAGE_QKV, s);
      if ((st = run_gemm(c->y, c->y_lo, SY_Y_SCALE, w.wq, qd, w.wk, kd, w.wv, kd, c->qkv, nullptr, T, qd + 2 * kd, d,
                         GEMM_STORE_F32, s, c->gparts, &qkv_parts, pair_qkv)))
        return st;
    }
    {
      StageTimer t(c, SYNERA_STAGE_ROPE_APPEND, s);
      HIP_TRY(launch_rope_append(qkv_parts ? c->gparts : c->qkv, qkv_parts, qkv_stride, c->cs, p.meta, c->q, c->q_lo,
                                 k_layer, v_layer, T, Hq, Hkv, hd, (lo_off & LO_Q) != 0, s));
    }
    al.k_layer = k_layer;
    al.v_layer = v_layer;
    al.row_ml = l == m.n_layers - 1 ? c->row_ml : nullptr;   // kept for synera_importance
    {
      StageTimer t(c, SYNERA_STAGE_ATTENTION, s);
      HIP_TRY(launch_attention(al, s));
    }
    {
      StageTimer t(c, SYNERA_STAGE_O, s);
      if ((st = run_gemm(c->o, c->o_lo, SY_O_SCALE, w.wo, d, nullptr, 0, nullptr, 0, c->x, nullptr, T, d, qd,
                         GEMM_ADD_F32, s, c->gparts, &pend, pair_o)))
        return st;
    }
    {
      StageTimer t(c, SYNERA_STAGE_NORM, s);
      HIP_TRY(launch_rmsnorm(c->x, c->gparts, pend, x_stride, static_cast<const bf16_t*>(w.mlp_norm), nullptr, c->y,
                             c->y_lo, T, d, m.rms_eps, (lo_off & LO_GATE_UP_IN) != 0, pair_gu, s));
      pend = 0;
    }
    {
      StageTimer t(c, SYNERA_STAGE_GATE_UP, s);
      if ((st = run_gemm(c->y, c->y_lo, SY_Y_SCALE, w.w_gate, 0, w.w_up, 0, nullptr, 0, c->act,
                         c->act_lo, T, 2 * m.d_ffn, d, GEMM_SWIGLU, s, nullptr, nullptr, pair_gu, pair_down)))
        return st;
    }
    if (lo_off & LO_DOWN_IN) HIP_TRY(launch_fill_zero(reinterpret_cast<float*>(c->act_lo), (size_t)T * m.d_ffn / 2, s));
    {
      StageTimer t(c, SYNERA_STAGE_DOWN, s);
      if ((st = run_gemm(c->act, c->act_lo, SY_ACT_SCALE, w.w_down, d, nullptr, 0, nullptr, 0, c->x, nullptr, T, d,
                         m.d_ffn, GEMM_ADD_F32, s, c->gparts, &pend, pair_down)))
        return st;
    }
  }

  // LM head over the draft rows (plus the last uncached row of requests that have one).
  const bool extra = p.R_all > p.R;
  // (the last down projection's slices are added here, for the selected rows only)
  HIP_TRY(launch_rmsnorm(c->x, c->gparts, pend, x_stride, static_cast<const bf16_t*>(c->final_norm), p.meta.sel_rows,
                         c->ysel, c->ysel_lo, p.R_all, d, m.rms_eps, (lo_off & LO_LM_HEAD_IN) != 0, false, s));
  float* logits = (d_logits && !extra) ? d_logits : c->logits;
  {
    StageTimer t(c, SYNERA_STAGE_LM_HEAD, s);
    // The LM head takes the high part alone: its input's rounding (11 bits) reaches the logits once, at the 1e-3
    // level, instead of being carried through the layers (measured: dropping this low part leaves max |dlogit| of
    // the 8B ragged batch at its 9e-3; dropping any other site's costs 2e-3 .. 9e-2).
    const uint16_t* ysel_lo = (c->lo_off & SYNERA_LO_KEEP_LM_HEAD) ? c->ysel_lo : nullptr;
    if ((st = run_gemm(c->ysel, ysel_lo, SY_Y_SCALE, c->lm_head, m.vocab, nullptr, 0, nullptr, 0, logits, nullptr,
                       p.R_all, m.vocab, d, GEMM_STORE_F32, s)))
      return st;
  }
  float* p_out = (d_top1_prob && !extra) ? d_top1_prob : c->lm_p;
  float* h_out = (d_entropy && !extra) ? d_entropy : c->lm_h;
  {
    StageTimer t(c, SYNERA_STAGE_CONFIDENCE, s);
    HIP_TRY(launch_confidence(logits, 0, p.R_all, m.vocab, m.vocab, c->lm_ids, p_out, h_out, s));
  }
  if (extra) {
    if (d_logits)
      HIP_TRY(hipMemcpyAsync(d_logits, c->logits, (size_t)p.R * m.vocab * 4, hipMemcpyDeviceToDevice, s));
    if (d_top1_prob) HIP_TRY(hipMemcpyAsync(d_top1_prob, c->lm_p, (size_t)p.R * 4, hipMemcpyDeviceToDevice, s));
    if (d_entropy) HIP_TRY(hipMemcpyAsync(d_entropy, c->lm_h, (size_t)p.R * 4, hipMemcpyDeviceToDevice, s));
  }
  HIP_TRY(launch_accept(d_tokens, d_anchor, c->lm_ids, p.meta, B, p.R, d_argmax, d_accept_len, d_correction, s));
  return SYNERA_OK;
}

extern "C" int32_t synera_verify(synera_ctx* c, int32_t B, const int32_t* h_ctx_len, const int32_t* h_n_uncached,
                                 const int32_t* h_n_draft, const int32_t* d_tokens, const int32_t* d_anchor,
                                 const int32_t* h_block_table, int32_t max_pages, int32_t n_pages_in_pool,
                                 void* d_k_pool, void* d_v_pool, float* d_logits, int32_t* d_argmax,
                                 float* d_top1_prob, float* d_entropy, int32_t* d_accept_len,
                                 int32_t* d_correction, void* stream_) {
  if (!c || !h_n_uncached || !d_tokens || !d_anchor || !d_k_pool || !d_v_pool || !d_argmax || !d_accept_len ||
      !d_correction)
    return SYNERA_EINVAL;
  // the attention kernel copies 16 bytes per lane out of the pools
  if (((reinterpret_cast<uintptr_t>(d_k_pool) | reinterpret_cast<uintptr_t>(d_v_pool)) & 15) != 0) return SYNERA_EINVAL;
  if (max_pages > c->max_pages) return SYNERA_ENOSPC;
  int32_t st = synera_validate_batch(B, h_ctx_len, h_n_draft, h_n_uncached, h_block_table, max_pages,
                                     n_pages_in_pool, c->max_batch, c->max_tokens, SYNERA_MAX_CHUNK);
  if (st != SYNERA_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream_);
  Plan p;
  bool uploaded = false;
  st = build_plan(c, B, h_ctx_len, h_n_uncached, h_n_draft, h_block_table, max_pages, true, s, p, false, &uploaded);
  if (st == SYNERA_OK)
    st = verify_launches(c, p, B, d_tokens, d_anchor, n_pages_in_pool, d_k_pool, d_v_pool, d_logits, d_argmax,
                         d_top1_prob, d_entropy, d_accept_len, d_correction, s);
  if (uploaded) {
    // Whatever was queued reads the metadata slot: mark it busy and move on to the next one even when a launch
    // failed half way, so that the next call cannot overwrite a slot the stream has not finished with.
    const int32_t fin = finish_call(c, p, s);
    if (st == SYNERA_OK) st = fin;
  }
  if (st != SYNERA_OK) return st;
  c->last.ctx_len = p.meta.ctx_len;
  c->last.cu_tok = p.meta.cu_tok;
  c->last.block_table = p.meta.block_table;
  c->last.n_unc = p.meta.n_unc;
  c->last.cu_draft = p.meta.cu_draft;
  c->last.cu_keys = p.d_cu_keys;
  c->last.items = p.d_imp_items;
  c->last.B = B;
  c->last.T = p.T;
  c->last.n_pages_in_pool = n_pages_in_pool;
  c->last.k_pool = d_k_pool;
  c->last.R = p.R;
  c->last.meta = p.meta;
  c->last.all_rows_kept = p.R_all == p.R + B;
  c->last.n_items = p.n_imp_items;
  c->last.max_pages = max_pages;
  c->last.total_keys = p.total_keys;
  c->last.slot = p.slot;
  c->last.valid = true;
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ stochastic verification
extern "C" int32_t synera_stochastic_accept(synera_ctx* c, const int32_t* d_tokens, int32_t k_list,
                                            const int32_t* d_p_id, const float* d_p_prob, const float* d_u_accept,
                                            const float* d_u_sample, int32_t* d_accept_len, int32_t* d_token,
                                            void* stream_) {
  if (!c || !d_tokens || !d_p_id || !d_p_prob || !d_u_accept || !d_u_sample || !d_accept_len || !d_token)
    return SYNERA_EINVAL;
  if (k_list < 1) return SYNERA_EINVAL;
  if (k_list > SYNERA_MAX_TOPK) return SYNERA_EUNSUP;
  if (!c->last.valid) return SYNERA_EINVAL;                  // no verification to take the distributions from
  if (!c->last.all_rows_kept) return SYNERA_EUNSUP;          // a request without an uncached token has no q(x | prefix)
  HIP_TRY(launch_stochastic_accept(c->logits, c->desc.vocab, c->lm_ids, c->lm_p, d_tokens, c->last.meta, c->last.B,
                                   k_list, d_p_id, d_p_prob, d_u_accept, d_u_sample, d_accept_len, d_token,
                                   static_cast<hipStream_t>(stream_)));
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ importance scores
extern "C" int32_t synera_importance(synera_ctx* c, int32_t n_pages_in_pool, const void* d_k_pool,
                                     int64_t n_scores, float* d_importance, float i_th, float theta,
                                     float* d_mean_importance, float* d_p_imp, void* stream_) {
  if (!c || !d_k_pool || !d_importance || n_pages_in_pool < 1) return SYNERA_EINVAL;
  if (!c->last.valid) return SYNERA_EINVAL;                  // no verification to take the scores from
  if (n_scores != c->last.total_keys) return SYNERA_EINVAL;
  // the block tables kept from that verify index this pool and no other
  if (d_k_pool != c->last.k_pool || n_pages_in_pool != c->last.n_pages_in_pool) return SYNERA_EINVAL;
  if (d_p_imp && !(i_th > 0.0f)) return SYNERA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream_);
  const synera_model_desc& m = c->desc;
  const size_t layer_elems = (size_t)n_pages_in_pool * m.n_kv_heads * SY_PAGE * m.head_dim;
  ImportanceLaunch a;
  a.q = c->q;
  a.q_lo = c->q_lo;
  a.qf = c->qkv;                 // the QKV projection's fp32 buffer is free between verifies
  a.T = c->last.T;
  a.total_keys = c->last.total_keys;
  a.k_layer = static_cast<const bf16_t*>(d_k_pool) + (size_t)(m.n_layers - 1) * layer_elems;
  a.row_ml = c->row_ml;
  a.ctx_len = c->last.ctx_len;
  a.cu_tok = c->last.cu_tok;
  a.block_table = c->last.block_table;
  a.cu_keys = c->last.cu_keys;
  a.items = c->last.items;
  a.n_items = c->last.n_items;
  a.max_pages = c->last.max_pages;
  a.Hq = m.n_q_heads;
  a.Hkv = m.n_kv_heads;
  a.hd = m.head_dim;
  a.importance = d_importance;
  a.parts = c->gparts;           // the projections' K-slice buffer is free between verifies, like qkv
  a.parts_cap = c->gpart_elems * SY_MAX_K_SLICES;
  HIP_TRY(launch_importance(a, s));
  HIP_TRY(launch_importance_dispatch(d_importance, c->last.cu_keys, c->last.ctx_len, c->last.n_unc, c->last.cu_draft,
                                     c->last.B, i_th, theta, d_mean_importance, d_p_imp, s));
  // these kernels read that verify's metadata slot: it stays busy until they are through
  HIP_TRY(hipEventRecord(c->done[c->last.slot], s));
  c->pending[c->last.slot] = true;
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ stage timing
extern "C" int32_t synera_profile_begin(synera_ctx* c, int32_t stage) {
  if (!c || stage < SYNERA_STAGE_NONE || stage > SYNERA_STAGE_ROPE_APPEND) return SYNERA_EINVAL;
  c->prof_stage = stage;
  c->prof_used = 0;
  return SYNERA_OK;
}

extern "C" int32_t synera_profile_end(synera_ctx* c, int32_t* n_launches, float* total_ms) {
  if (!c || !n_launches || !total_ms) return SYNERA_EINVAL;
  *n_launches = 0;
  *total_ms = 0.f;
  c->prof_stage = SYNERA_STAGE_NONE;
  const size_t pairs = c->prof_used / 2;
  c->prof_used = 0;
  for (size_t i = 0; i < pairs; ++i) {
    HIP_TRY(hipEventSynchronize(c->prof_events[2 * i + 1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->prof_events[2 * i], c->prof_events[2 * i + 1]));
    *total_ms += ms;
  }
  *n_launches = (int32_t)pairs;
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ confidence
extern "C" int32_t synera_confidence(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab,
                                     int64_t row_stride_elems, int32_t* d_top1_id, float* d_top1_prob,
                                     float* d_entropy, void* stream) {
  if (rows < 0 || vocab < 1 || (dtype != 0 && dtype != 1)) return SYNERA_EINVAL;
  if (rows == 0) return SYNERA_OK;
  if (!d_logits || !d_top1_id || row_stride_elems < vocab) return SYNERA_EINVAL;
  if (rows > 0x7FFFFFFF || vocab > 0x7FFFFFFF) return SYNERA_EINVAL;
  const int64_t align = dtype == 1 ? 8 : 4;
  if (row_stride_elems % align != 0 || (reinterpret_cast<uintptr_t>(d_logits) & 15) != 0) return SYNERA_EINVAL;
  HIP_TRY(launch_confidence(d_logits, dtype, rows, vocab, row_stride_elems, d_top1_id, d_top1_prob, d_entropy,
                            static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

extern "C" int32_t synera_confidence_topk(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab,
                                          int64_t row_stride_elems, int32_t k, int32_t* d_topk_id,
                                          float* d_topk_prob, float* d_margin, float* d_entropy, void* stream) {
  if (rows < 0 || vocab < 1 || (dtype != 0 && dtype != 1) || k < 1) return SYNERA_EINVAL;
  if (k > SYNERA_MAX_TOPK || k > vocab) return SYNERA_EUNSUP;
  if (rows == 0) return SYNERA_OK;
  if (!d_logits || !d_topk_id || !d_topk_prob || row_stride_elems < vocab) return SYNERA_EINVAL;
  if (rows > 0x7FFFFFFF / SYNERA_MAX_TOPK || vocab > 0x7FFFFFFF) return SYNERA_EINVAL;
  const int64_t align = dtype == 1 ? 8 : 4;
  if (row_stride_elems % align != 0 || (reinterpret_cast<uintptr_t>(d_logits) & 15) != 0) return SYNERA_EINVAL;
  HIP_TRY(launch_confidence_topk(d_logits, dtype, rows, vocab, row_stride_elems, k, d_topk_id, d_topk_prob, d_margin,
                                 d_entropy, static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

extern "C" int32_t synera_nucleus(const void* d_logits, int32_t dtype, int64_t rows, int64_t vocab,
                                  int64_t row_stride_elems, float top_p, int32_t* d_count, float* d_mass,
                                  float* d_cut_logit, void* stream) {
  if (rows < 0 || vocab < 1 || (dtype != 0 && dtype != 1) || !(top_p > 0.0f && top_p <= 1.0f)) return SYNERA_EINVAL;
  if (rows == 0) return SYNERA_OK;
  if (!d_logits || !d_count || row_stride_elems < vocab) return SYNERA_EINVAL;
  if (rows > 0x7FFFFFFF || vocab > 0x7FFFFFFF) return SYNERA_EINVAL;
  const int64_t align = dtype == 1 ? 8 : 4;
  if (row_stride_elems % align != 0 || (reinterpret_cast<uintptr_t>(d_logits) & 15) != 0) return SYNERA_EINVAL;
  HIP_TRY(launch_nucleus(d_logits, dtype, rows, vocab, row_stride_elems, top_p, d_count, d_mass, d_cut_logit,
                         static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

extern "C" int32_t synera_topp_count(const float* d_topk_prob, int64_t rows, int32_t k, float top_p, int32_t* d_count,
                                     float* d_mass, void* stream) {
  if (rows < 0 || k < 1 || !(top_p > 0.0f && top_p <= 1.0f)) return SYNERA_EINVAL;
  if (rows == 0) return SYNERA_OK;
  if (!d_topk_prob || !d_count) return SYNERA_EINVAL;
  HIP_TRY(launch_topp_count(d_topk_prob, rows, k, top_p, d_count, d_mass, static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

extern "C" int32_t synera_chunk_dispatch(const float* d_top1_prob, const int32_t* d_cu_rows, int32_t B, float c_th,
                                         float k_slope, float* d_mean_conf, float* d_p_conf, void* stream) {
  if (B < 0 || !(c_th >= 0.0f && c_th < 1.0f)) return SYNERA_EINVAL;
  if (B == 0) return SYNERA_OK;
  if (!d_top1_prob || !d_cu_rows || !d_mean_conf || !d_p_conf) return SYNERA_EINVAL;
  HIP_TRY(launch_chunk_dispatch(d_top1_prob, d_cu_rows, B, c_th, k_slope, d_mean_conf, d_p_conf,
                                static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

// ------------------------------------------------------------------------------------ kv append
extern "C" int32_t synera_kv_append(synera_ctx* c, int32_t layer, int32_t B, const int32_t* h_ctx_len,
                                    const int32_t* h_n_new, const void* d_k, const void* d_v,
                                    const int32_t* h_block_table, int32_t max_pages, int32_t n_pages_in_pool,
                                    void* d_k_pool, void* d_v_pool, void* stream_) {
  if (!c || !d_k || !d_v || !d_k_pool || !d_v_pool) return SYNERA_EINVAL;
  if (layer < 0 || layer >= c->desc.n_layers) return SYNERA_EINVAL;
  if (max_pages > c->max_pages) return SYNERA_ENOSPC;
  int32_t st = synera_validate_batch(B, h_ctx_len, h_n_new, nullptr, h_block_table, max_pages, n_pages_in_pool,
                                     c->max_batch, INT64_MAX, 0);
  if (st != SYNERA_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream_);
  Plan p;
  st = build_plan(c, B, h_ctx_len, nullptr, h_n_new, h_block_table, max_pages, false, s, p);
  if (st != SYNERA_OK) return st;
  const int Hkv = c->desc.n_kv_heads, hd = c->desc.head_dim;
  const size_t layer_elems = (size_t)n_pages_in_pool * Hkv * SY_PAGE * hd;
  const hipError_t e = launch_kv_append(static_cast<const bf16_t*>(d_k), static_cast<const bf16_t*>(d_v), p.meta, B,
                                        static_cast<bf16_t*>(d_k_pool) + (size_t)layer * layer_elems,
                                        static_cast<bf16_t*>(d_v_pool) + (size_t)layer * layer_elems, p.T, Hkv, hd, s);
  if (e != hipSuccess) (void)hipGetLastError();
  const int32_t fin = finish_call(c, p, s);      // the upload is queued either way: the slot is busy
  return e != hipSuccess ? SYNERA_EHIP : fin;
}

// ------------------------------------------------------------------------------------ plain GEMM
extern "C" int32_t synera_debug_read_scratch(synera_ctx* c, int32_t which, void* d_dst, int64_t bytes, void* stream) {
  if (!c || !d_dst || bytes < 0) return SYNERA_EINVAL;
  const synera_model_desc& m = c->desc;
  const int64_t T = c->max_tokens, qd = (int64_t)m.n_q_heads * m.head_dim;
  const void* src = nullptr;
  int64_t cap = 0;
  switch (which) {
    case 0: src = c->x; cap = T * m.d_model * 4; break;
    case 1: src = c->q; cap = T * qd * 2; break;
    case 2: src = c->q_lo; cap = T * qd * 2; break;
    case 3: src = c->o; cap = T * qd * 2; break;
    case 4: src = c->o_lo; cap = T * qd * 2; break;
    case 5: src = c->act; cap = T * (int64_t)m.d_ffn * 2; break;
    case 6: src = c->act_lo; cap = T * (int64_t)m.d_ffn * 2; break;
    default: return SYNERA_EINVAL;
  }
  if (bytes > cap && !((which == 3 || which == 5) && bytes <= 2 * cap)) return SYNERA_ENOSPC;
  HIP_TRY(hipMemcpyAsync(d_dst, src, (size_t)bytes, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)));
  return SYNERA_OK;
}

extern "C" int32_t synera_debug_set_gemm_tile(int32_t variant) {
  gemm_force_variant(variant);
  return SYNERA_OK;
}

extern "C" int32_t synera_debug_attention_plan(const synera_model_desc* desc, int32_t attn_blocks, int32_t B,
                                               const int32_t* h_ctx_len, const int32_t* h_n_uncached,
                                               const int32_t* h_n_draft, const int32_t* h_block_table,
                                               int32_t max_pages, int32_t* h_shares, int32_t* h_prog, int64_t prog_cap,
                                               int32_t* h_units, int64_t unit_cap, int32_t* h_cuts, int64_t cut_cap,
                                               int32_t* h_counts) {
  if (!desc || !h_ctx_len || !h_n_uncached || !h_n_draft || !h_block_table || !h_shares || !h_prog || !h_units ||
      !h_cuts || !h_counts || attn_blocks < 2 || attn_blocks > 8192 || B < 1 || max_pages < 1)
    return SYNERA_EINVAL;
  const synera_model_desc& m = *desc;
  if (m.n_q_heads < 1 || m.n_kv_heads < 1 || m.n_q_heads % m.n_kv_heads != 0 || m.n_q_heads / m.n_kv_heads > 16)
    return SYNERA_EUNSUP;
  int64_t T = 0;
  for (int i = 0; i < B; ++i) {
    if (h_ctx_len[i] < 0 || h_n_uncached[i] < 0 || h_n_draft[i] < 1 || h_n_uncached[i] + h_n_draft[i] > SYNERA_MAX_CHUNK ||
        (int64_t)h_ctx_len[i] + h_n_uncached[i] + h_n_draft[i] > (int64_t)max_pages * SYNERA_PAGE_SIZE)
      return SYNERA_EINVAL;
    T += h_n_uncached[i] + h_n_draft[i];
  }
  synera_ctx* c = new (std::nothrow) synera_ctx();   // host-only: no arena, no events, one malloc'ed staging slot
  if (!c) return SYNERA_ENOMEM;
  c->desc = m;
  c->max_batch = B;
  c->max_tokens = (int32_t)T;
  c->max_pages = max_pages;
  c->max_rows = (int32_t)T + B;
  c->attn_blocks = c->attn_blocks_cap = attn_blocks;
  attention_plan_defaults(c);
  c->arena = nullptr;
  c->calls = 0;
  for (int s = 0; s < N_STAGE; ++s) {
    c->h_meta[s] = c->d_meta[s] = nullptr;
    c->done[s] = nullptr;
    c->pending[s] = false;
  }
  size_plan(c);
  std::vector<int32_t> blob(c->meta_cap / 4);
  c->h_meta[0] = c->d_meta[0] = blob.data();        // "device" addresses of the plan point into the same blob
  Plan p;
  int32_t st = build_plan(c, B, h_ctx_len, h_n_uncached, h_n_draft, h_block_table, max_pages, true, nullptr, p, true);
  if (st == SYNERA_OK) {
    int64_t n_pos = 0, n_units = 0;
    for (int i = 0; i < p.n_shares; ++i) n_pos = std::max<int64_t>(n_pos, p.d_shares[i].pos_begin + p.d_shares[i].n_pos);
    for (int64_t i = 0; i < n_pos; ++i)
      if ((p.d_prog[i].tag & ATTN_POS_KIND_MASK) == ATTN_POS_Q) n_units = std::max<int64_t>(n_units, (p.d_prog[i].tag >> 4) + 1);
    if (n_pos > prog_cap || n_units > unit_cap || p.n_cuts > cut_cap) {
      st = SYNERA_ENOSPC;
    } else {
      std::memcpy(h_shares, p.d_shares, (size_t)p.n_shares * sizeof(AttnShare));
      std::memcpy(h_prog, p.d_prog, (size_t)n_pos * sizeof(AttnPos));
      std::memcpy(h_units, p.d_units, (size_t)n_units * sizeof(AttnUnit));
      std::memcpy(h_cuts, p.d_cuts, (size_t)p.n_cuts * sizeof(AttnCut));
      h_counts[0] = p.n_shares;
      h_counts[1] = (int32_t)n_pos;
      h_counts[2] = (int32_t)n_units;
      h_counts[3] = p.n_cuts;
    }
  }
  delete c;
  return st;
}

extern "C" int32_t synera_debug_gemm_plan(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t stored_slices,
                                          int32_t* h_tile_rows, int32_t* h_tile_cols, int32_t* h_k_slices) {
  if (!h_tile_rows || !h_tile_cols || !h_k_slices) return SYNERA_EINVAL;
  GemmArgs g;
  const int32_t st = plan_args(M, N, K, epilogue, stored_slices, &g);
  if (st != SYNERA_OK) return st;
  int bm = 0, bn = 0, split = 1;
  gemm_plan(g, &bm, &bn, &split);
  *h_tile_rows = bm;
  *h_tile_cols = bn;
  *h_k_slices = split;
  return SYNERA_OK;
}

extern "C" int32_t synera_debug_gemm_plan_bk(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t stored_slices,
                                             int32_t* h_stage_k) {
  if (!h_stage_k) return SYNERA_EINVAL;
  GemmArgs g;
  const int32_t st = plan_args(M, N, K, epilogue, stored_slices, &g);
  if (st != SYNERA_OK) return st;
  *h_stage_k = gemm_plan_bk(g);
  return SYNERA_OK;
}

extern "C" int32_t synera_debug_gemm_epilogue(const void* d_a, const void* d_a_lo, const void* d_w0, const void* d_w1,
                                              void* d_c, void* d_c_lo, int32_t M, int32_t N, int32_t K,
                                              int32_t epilogue, void* stream) {
  if (!d_a || !d_a_lo || !d_w0 || !d_c || M < 1 || N < 1 || K < 1 || epilogue < 0 || epilogue > 2) return SYNERA_EINVAL;
  if (epilogue == GEMM_SWIGLU && (!d_w1 || !d_c_lo)) return SYNERA_EINVAL;
  if (N % (epilogue == GEMM_SWIGLU ? 256 : 128) != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  const bool glu = epilogue == GEMM_SWIGLU;
  return run_gemm(static_cast<const uint16_t*>(d_a), static_cast<const uint16_t*>(d_a_lo), 1.0f, d_w0, glu ? N / 2 : N,
                  glu ? d_w1 : nullptr, glu ? N / 2 : 0, nullptr, 0, d_c, d_c_lo, M, N, K, epilogue,
                  static_cast<hipStream_t>(stream));
}

extern "C" int32_t synera_debug_gemm_paired(const void* d_a_pairs, const void* d_w0, const void* d_w1, void* d_c,
                                            int32_t M, int32_t N, int32_t K, int32_t epilogue, void* stream) {
  if (!d_a_pairs || !d_w0 || !d_c || M < 1 || N < 1 || K < 1 || epilogue < 0 || epilogue > 2) return SYNERA_EINVAL;
  if (epilogue == GEMM_SWIGLU && !d_w1) return SYNERA_EINVAL;
  if (N % (epilogue == GEMM_SWIGLU ? 256 : 128) != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  const bool glu = epilogue == GEMM_SWIGLU;
  return run_gemm(static_cast<const uint16_t*>(d_a_pairs), nullptr, 1.0f, d_w0, glu ? N / 2 : N, glu ? d_w1 : nullptr,
                  glu ? N / 2 : 0, nullptr, 0, d_c, nullptr, M, N, K, epilogue, static_cast<hipStream_t>(stream),
                  nullptr, nullptr, true, glu);
}

static_assert(SYNERA_MAX_GEMM_SLICES == SY_MAX_K_SLICES, "header and planner disagree on the slice limit");
extern "C" int32_t synera_debug_gemm_slices(const void* d_a, const void* d_a_lo, const void* d_w, float* d_parts,
                                            int32_t M, int32_t N, int32_t K, int32_t* h_n_parts, void* stream) {
  if (!d_a || !d_a_lo || !d_w || !d_parts || !h_n_parts || M < 1 || N < 1 || K < 1) return SYNERA_EINVAL;
  if (N % 128 != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  int n_parts = 0;
  const int32_t st = run_gemm(static_cast<const uint16_t*>(d_a), static_cast<const uint16_t*>(d_a_lo), 1.0f, d_w, N,
                              nullptr, 0, nullptr, 0, d_parts, nullptr, M, N, K, GEMM_STORE_F32,
                              static_cast<hipStream_t>(stream), d_parts, &n_parts);
  *h_n_parts = n_parts > 0 ? n_parts : 1;
  return st;
}

extern "C" int32_t synera_gemm_pair(const void* d_a, const void* d_a_lo, const void* d_w, float* d_c, int32_t M,
                                    int32_t N, int32_t K, void* stream) {
  if (!d_a || !d_w || !d_c || M < 1 || N < 1 || K < 1) return SYNERA_EINVAL;
  if (N % 128 != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  return run_gemm(static_cast<const uint16_t*>(d_a), static_cast<const uint16_t*>(d_a_lo), 1.0f, d_w, N, nullptr, 0,
                  nullptr, 0, d_c, nullptr, M, N, K, GEMM_STORE_F32, static_cast<hipStream_t>(stream));
}

extern "C" int32_t synera_debug_set_lo_off(synera_ctx* c, int32_t sites) {
  if (!c || sites < 0 || sites > 255) return SYNERA_EINVAL;
  c->lo_off = sites;
  return SYNERA_OK;
}

extern "C" int32_t synera_debug_set_attention_plan(synera_ctx* c, int32_t attn_blocks, float stream_cost,
                                                   float cut_slack, float t_iter_ratio) {
  if (!c) return SYNERA_EINVAL;
  if (attn_blocks != 0 && (attn_blocks < 2 || attn_blocks > c->attn_blocks_cap)) return SYNERA_EINVAL;
  if (!(stream_cost >= 0.0f && stream_cost <= 16.0f) || !(cut_slack >= 0.0f && cut_slack <= 64.0f) ||
      !(t_iter_ratio >= 0.25f && t_iter_ratio <= 8.0f))
    return SYNERA_EINVAL;
  if (attn_blocks) c->attn_blocks = attn_blocks;
  c->attn_stream_cost = stream_cost;
  c->attn_cut_slack = cut_slack;
  c->attn_t_iter[1] = c->attn_t_iter[0] * t_iter_ratio;
  return SYNERA_OK;
}
