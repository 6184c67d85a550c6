// Tile planner and launcher of the projection GEMM (kernel: gemm_tile.h).  Host code only.
//
// A tile is 16 MT rows (MT = 1..17) by 256 columns, or by 128 columns (MT = 1..12) for outputs whose width is
// not a multiple of 256 and for small batches; the short ones (128 columns x <= 144 rows, 256 x <= 80) come with
// two MFMA K steps per stage as well.  Why 128 columns: at M = 128 a 256-column tiling gives the 8B gate/up projection
// only 112 blocks and every block pulls its weight stream at the ~24 GB/s one compute unit sustains from HBM;
// 224 blocks of 128 columns stream on twice the compute units.  K may be split into stored slices.
#include "common.h"

static int g_forced = -1;   // tuning hook: forced tile (see gemm_force_variant), -1 = automatic
void gemm_force_variant(int v) { g_forced = v; }

static bool tile_fits(const GemmArgs& g, int mt, int nf, int ksub) {
  if (mt < 1 || (nf == 4 ? mt > 17 : mt > 12)) return false;
  if (g.a_paired && ksub != 1) return false;                       // the paired activation array: one K step per stage
  if (ksub == 2 && (nf == 4 ? mt > 5 : mt > 9)) return false;      // three stages of 128-byte rows must fit the LDS
  if (g.K % (32 * ksub) != 0) return false;
  const int bn = 64 * nf;
  if (g.N % bn != 0) return false;
  if (g.epilogue != GEMM_SWIGLU)
    for (int i = 0; i < 3; ++i)
      if (g.w_rows[i] % bn != 0) return false;
  return true;
}

// Modelled time of one stage (32 ksub of K) of one block, us.  Fit of MI355X timings of the 8B gate/up projection at
// M = 532 on 256-column tiles of 128, 144 and 272 rows: 0.17 us plus 0.086 us per 16-row block and MFMA K step; a
// 128-column tile pays the activation-fragment reads of a 256-column one for half the MFMAs: 0.6x, not 0.5x.  A
// short tile is bound by its weight stream instead: BN rows x 64 bytes per K step at the ~24 GB/s one compute
// unit pulls from HBM.
static double step_us(int mt, int nf, bool lo, int ksub) {
  const double mfma = 0.17 + ksub * 0.086 * mt * (nf == 4 ? 1.0 : 0.6) * (lo ? 1.0 : 0.55);   // hi alone: half the MFMAs
  const double stream = ksub * 64 * nf * 64 / 24e3;
  return mfma > stream ? mfma : stream;
}
static int max_split(const GemmArgs& g, int mt, int nf) {
  if (g.epilogue == GEMM_SWIGLU || !g.c_parts) return 1;
  const long tiles = (long)((g.M + 16 * mt - 1) / (16 * mt)) * (g.N / (64 * nf));
  long split = 256 / tiles;
  const long most = g.K / 32 / 8;               // at least 8 K steps per slice
  split = split < most ? split : most;
  if (split > SY_MAX_K_SLICES) split = SY_MAX_K_SLICES;
  return split < 1 ? 1 : (int)split;
}
// Blocks are equal-sized and one runs per compute unit, so a launch takes ceil(blocks / 256) rounds of
// stages per block x step_us, plus per stored K slice and 2.2 M outputs ~2.4 us to store it and read it back
// (QKV and down projection at M = 532 on 272-row tiles with 5 and 8 slices: 18 - 19 us beyond their K steps).
static double plan_cost(const GemmArgs& g, int mt, int nf, int ksub, int split) {
  const long tiles = (long)((g.M + 16 * mt - 1) / (16 * mt)) * (g.N / (64 * nf));
  const long rounds = (tiles * split + 255) / 256;
  const double steps = (double)(g.K / (32 * ksub)) / split;
  const double merge = split > 1 ? 2.4 * split * ((double)g.M * g.N / 2.2e6) : 0.0;
  return rounds * steps * step_us(mt, nf, g.a_lo != nullptr || g.a_paired, ksub) + merge;
}

static void pick(const GemmArgs& g, int* mt_out, int* nf_out, int* ksub_out, int* split_out) {
  if (g_forced >= 0) {
    // forced tile: rows / 16 + 100 for 128 columns + 200 for two K steps per stage
    const int mt = g_forced % 100, nf = (g_forced / 100) % 2 ? 2 : 4, ksub = g_forced >= 200 ? 2 : 1;
    if (tile_fits(g, mt, nf, ksub)) {
      *mt_out = mt;
      *nf_out = nf;
      *ksub_out = ksub;
      *split_out = max_split(g, mt, nf);         // forced tile: as many slices as fit
      return;
    }
  }
  // Tiles below 128 rows only where M itself is smaller: the model's fixed cost per K step was fitted on tall tiles.
  const int need = (g.M + 15) / 16, mt_min = need < 8 ? need : 8;
  int best_mt = -1, best_nf = 4, best_ksub = 1, best_split = 1;
  double best_cost = 0.0;
  for (int nf = 4; nf >= 2; nf -= 2)
    for (int mt = mt_min; mt <= 17; ++mt)
      for (int ksub = 2; ksub >= 1; --ksub) {    // two K steps per stage wherever the tile allows them
        if (!tile_fits(g, mt, nf, ksub)) continue;
        const int most = max_split(g, mt, nf);
        for (int split = 1; split <= most; ++split) {    // fewer slices than fit can win: less to merge
          const double c = plan_cost(g, mt, nf, ksub, split);
          if (best_mt < 0 || c < best_cost) {
            best_mt = mt;
            best_nf = nf;
            best_ksub = ksub;
            best_cost = c;
            best_split = split;
          }
        }
      }
  *mt_out = best_mt;
  *nf_out = best_nf;
  *ksub_out = best_ksub;
  *split_out = best_split;
}

void gemm_plan(const GemmArgs& g, int* bm, int* bn, int* split) {
  int mt = -1, nf = 4, ksub = 1;
  pick(g, &mt, &nf, &ksub, split);
  *bm = 16 * mt;
  *bn = 64 * nf;
}

int gemm_plan_bk(const GemmArgs& g) {
  int mt = -1, nf = 4, ksub = 1, split = 1;
  pick(g, &mt, &nf, &ksub, &split);
  return 32 * ksub;
}

int gemm_pick_split(const GemmArgs& g) {
  int mt, nf, ksub, split;
  pick(g, &mt, &nf, &ksub, &split);
  return mt < 0 ? 1 : split;
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0) return hipSuccess;
  if (!g.a || !g.w[0] || !g.c || g.N < 128 || g.K < 64 || g.K % 64 != 0 || g.split_k < 1)
    return hipErrorInvalidValue;
  int mt, nf, ksub, split;
  pick(g, &mt, &nf, &ksub, &split);
  if (mt < 0 || g.split_k > g.K / 32 || g.split_k > SY_MAX_K_SLICES) return hipErrorInvalidValue;
  if (g.split_k > 1 && (!g.c_parts || g.epilogue == GEMM_SWIGLU)) return hipErrorInvalidValue;
  if (!g.a_lo && !g.a_paired && g.epilogue != GEMM_STORE_F32) return hipErrorInvalidValue;
  if (g.a_paired && ksub != 1) return hipErrorInvalidValue;
  if (g.c_paired && g.epilogue != GEMM_SWIGLU) return hipErrorInvalidValue;
  if (g.epilogue == GEMM_SWIGLU) {
    if ((!g.c_lo && !g.c_paired) || !g.w[1]) return hipErrorInvalidValue;
  } else {
    long rows = 0;
    for (int i = 0; i < 3; ++i) {
      rows += g.w_rows[i];
      if (g.w_rows[i] % 16 != 0) return hipErrorInvalidValue;   // a copy's 16 tile rows come from one array
    }
    if (rows != g.N) return hipErrorInvalidValue;
  }
  if (ksub == 2) return launch_proj_k64(mt, nf, g, s);
  if (nf == 2) return launch_proj_nf2(mt, g, s);
  return mt <= 9 ? launch_proj_nf4_low(mt, g, s) : launch_proj_nf4_high(mt, g, s);
}
