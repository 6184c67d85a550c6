// The projection GEMM of the decoder: C[M][N] = A[M][K] * W[N][K]^T on the matrix cores with fp32 accumulation
// (v_mfma_f32_16x16x32_f16).  Both operands are K-major, so an MFMA operand fragment (8 consecutive k of one
// row) is one 16-byte read.
//
// Operand formats.  Activations arrive as an fp16 pair (hi, lo), hi = fp16(v), lo = fp16(v - hi): 22 mantissa
// bits of the fp32 value, and the kernel accumulates A_hi * W and A_lo * W into the same accumulators.  Weights
// are bf16 in memory (8 mantissa bits: exact in fp16) and are turned into fp16 in registers, four vector
// instructions per packed pair, with their exponents raised by SY_W_SHIFT so that small weights stay in fp16's
// normal range (2^-14 2^-SY_W_SHIFT .. 65504 2^-SY_W_SHIFT); the epilogue multiplies the accumulators by
// GemmArgs::out_scale, which takes that factor and the producer's activation scale out again (powers of two:
// exact).  The lo term reuses the weight fragments already in registers, so it costs MFMA issue slots but no
// extra weight traffic from HBM, L2 or LDS.  A contraction whose result tolerates 11-bit activations (the LM head:
// its rounding reaches the logits once, not through 32 layers) is launched without a low part (a_lo = nullptr)
// and skips those copies and MFMAs.  (The same pair in bf16 carries 16 bits; its rounding noise, amplified
// layer by layer through bf16 KV-cache roundings that fall the other way, put the logits of an 80-layer decoder
// of width 8192 at 5e-2 from the exact result.)
//
// Tile: BM = 16 MT rows x BN = 64 NF columns, four wavefronts (one per SIMD), each owning all BM rows of 16 NF
// columns.  A stage holds BK = 32 KSUB of K: one MFMA K step (lane l holds row l % 16 and the 8 k values of chunk
// l / 16 for both operands), or two for the short tiles (KSUB = 2: tile rows of 128 bytes, so every copy moves
// whole cache lines, half the requests for the same bytes, and the K loop has half the barriers; small batches
// are bound by exactly these).  The weight fragment is the MFMA's first operand, so a lane ends up with 4 consecutive output
// columns of one row and the epilogue stores 16 bytes per lane.  Per K step a wavefront reads its NF weight
// fragments once and streams the 2 MT activation fragments (hi, lo) through them; each activation fragment feeds
// NF independent accumulators, which is what this 4-pass MFMA needs to issue back to back.  Accumulators 0..255
// live in AGPRs, the rest in VGPRs.
//
// Data movement: the rows [A_hi | A_lo | W] of K step s+2 stream straight from global memory into LDS
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions) while step s is multiplied; three
// LDS stages.  A copy instruction of one wavefront fills 1 KB = 16 (or 8) tile rows; the XOR swizzle that keeps the
// fragment reads bank-conflict free is applied on the global side (lane i fetches the chunk that belongs at LDS
// position i).  Per K step each wavefront waits for its own copies of the step (s_waitcnt vmcnt) and one
// s_barrier makes every wavefront's copies visible and certifies that the stage about to be overwritten is no
// longer read.  The copies of step s+2 are spread between the MFMAs of step s: issued in a burst they queue on
// the compute unit's one address unit and delay every wavefront's first MFMA.
//
// The MFMAs and the weight conversion are inline assembly.  MFMAs: with the accumulator tied to the destination
// (left to the compiler, accumulators migrate between registers from one K step to the next, and spill once
// they need more than the 256 AGPRs).  Conversion: so that it sits exactly between the MFMAs whose shadow hides
// it.  A wavefront copies the weight rows of its own columns itself, so it can read the weights of step s+1 as
// soon as its own copies have landed, before the barrier: it does so during the last four row blocks of step
// s and converts them, two instructions after each MFMA; step s+1 then starts with its weight fragments in registers.
// The price of inline MFMAs: the compiler does not know the accumulators are matrix-core results and may copy
// or spill one right behind the MFMA, which the hardware does not interlock.  Every basic block of the K loop
// therefore ends with explicit wait states, the epilogue pins its accumulator reads behind a final wait, and the
// build reads the generated assembly and fails on any access that comes too early (mfma_hazards.py).
//
// K may be split over blockIdx.z in units of BK; slice z is stored plainly to c_parts[z] and the kernel that
// reads the result next adds the slices in order (no atomics, fixed summation order).
#pragma once
#include "common.h"

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// Asynchronous 16-byte-per-lane copy global -> LDS; m0 carries the wavefront-uniform LDS address, lane i lands
// at that address + 16 i.  (Through the compiler builtin every later LDS read is preceded by a wait for ALL
// copies in flight, which would serialise the pipeline.)
// The global address is a wavefront-uniform base (a scalar register pair, advanced along K with scalar adds) plus a
// 32-bit byte offset per lane that never changes: no vector arithmetic per copy, half the address registers.
__device__ __forceinline__ void glds16_at(const void* base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}
// Element offset of 16-byte chunk `chunk` of tile row `row` (rows of CPR = 4 or 8 chunks: 64 or 128 bytes).  A
// fragment read (lane = row l % 16, chunk 4 ks + l / 16) is served 16 lanes per cycle over the 64 banks, lanes
// l and l + 16 together: the chunk position varies with the row's bits 1..2 (XORed into chunk bits 0..1 of a
// 64-byte row, bits 1..2 of a 128-byte row, whose bit 0 of the row already selects the half of the bank cycle),
// which spreads the rows of a fragment over all banks.
template <int CPR>
__device__ __forceinline__ int swz16(int row, int chunk) {
  return (row * CPR + (chunk ^ (((row >> 1) & 3) << (CPR == 8 ? 1 : 0)))) * 8;
}

template <int MT, int NF, int EPI, bool LO = true, int KSUB = 1, bool PAIRED = false>
__global__ __launch_bounds__(256) void proj_kernel(GemmArgs g) {
  // PAIRED: the activations come as one array [M][K / 32][hi 32 | lo 32] (GemmArgs::a, a_lo unused): the 64 bytes of
  // a row's high part and the 64 of its low part for one K step are one 128-byte line, so an activation copy moves
  // 8 whole lines instead of 16 half lines (the tall tiles run into the rate at which L2 takes requests).  In LDS an
  // activation row is then those 128 bytes (chunks 0..3 high, 4..7 low); the weight rows keep their 64.
  static_assert(!PAIRED || (LO && KSUB == 1), "paired activations: two terms, one MFMA K step per stage");
  // KSUB MFMA K steps per stage and barrier (BK = 32 KSUB).  KSUB = 2, for the short tiles whose three stages still
  // fit: half the barriers and full 128-byte rows per copy (half the requests to L2 for the same bytes).
  constexpr int BM = 16 * MT, BN = 64 * NF, BK = 32 * KSUB;
  constexpr int CPR = BK / 8, RPI = 64 / CPR;    // 16-byte chunks per tile row; tile rows per copy instruction
  static_assert(KSUB == 1 || KSUB == 2, "one or two MFMA K steps per stage");
  static_assert(NF == 2 || NF == 4, "SwiGLU pairs the fragments (gate, up): NF must be even");
  static_assert(MT >= 1 && MT <= 17, "accumulators: 4 NF MT registers per lane, stages: 3 (2 BM + BN) x 64 B of LDS");
  constexpr int TERMS = LO ? 2 : 1;              // activation terms: (hi, lo), or hi alone (LO = false: the low part is
                                                 // neither copied nor multiplied; 11 mantissa bits, half the MFMAs)
  constexpr int A_INS = TERMS * BM / RPI;        // copy instructions (RPI tile rows = 1 KB each) for [A_hi | A_lo]
  constexpr int A_IPW = (A_INS + 3) / 4;         // per wavefront; a surplus one repeats the last group
  constexpr int W_IPW = BN / RPI / 4;
  constexpr int IPW = A_IPW + W_IPW;
  constexpr int R = TERMS * BM + BN;
  static_assert(3 * R * BK * 2 <= 163840, "three stages of (TERMS BM + BN) rows must fit the 160 KB of LDS");
  // The K loop walks MV = MT KSUB "row blocks": row block i at K sub-step ks, ks fastest.
  constexpr int MV = MT * KSUB;
  constexpr int CVT_RB = (LO ? 4 : 8) * KSUB;    // row blocks whose MFMAs give the 16 NF KSUB conversion instructions cover
  constexpr int C_END = MV > CVT_RB ? MV - CVT_RB : 1;   // the copies of step s+2 go out during row blocks 0 .. C_END-1
  constexpr int CPB = (IPW + C_END - 1) / C_END; // copies per row block
  constexpr int SLOTS = TERMS * NF;              // MFMAs per row block
  constexpr int NW = KSUB * NF;                  // weight fragments of a stage per wavefront
  __shared__ __attribute__((aligned(16))) uint16_t st0[R * BK];
  __shared__ __attribute__((aligned(16))) uint16_t st1[R * BK];
  __shared__ __attribute__((aligned(16))) uint16_t st2[R * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so block b
  // runs on XCD b % 8.  Within an XCD consecutive blocks walk the M tiles of one N tile: the blocks that share
  // a weight tile run together on one L2 and the weights leave HBM once.
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / BN;
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int n_tile = (within / m_tiles) * 8 + xcd;
  if (n_tile >= n_tiles) return;
  const int m0 = (within % m_tiles) * BM, n0 = n_tile * BN;
  const int K = g.K, M = g.M;
  const int total_steps = K / BK;
  const int step_begin = (int)((long)blockIdx.z * total_steps / g.split_k);
  const int n_steps = (int)((long)(blockIdx.z + 1) * total_steps / g.split_k) - step_begin;
  if (n_steps <= 0) return;

  const uint16_t* src[IPW];                      // wavefront-uniform part of the copy's global address
  uint32_t off[IPW];                             // this lane's byte offset from it (constant along K)
  uint32_t dst[IPW];                             // byte offset of the copy's 16 rows inside a stage
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    int grp;                                     // group of RPI rows of the stage
    if (j < A_IPW) {
      grp = wave + 4 * j;
      grp = grp < A_INS ? grp : A_INS - 1;       // same bytes to the same place: harmless
    } else {
      grp = A_INS + wave * W_IPW + (j - A_IPW);
    }
    const int r = grp * RPI + lane / CPR;
    const int ch = (lane % CPR) ^ (((r >> 1) & 3) << (CPR == 8 ? 1 : 0));
    dst[j] = grp * 1024;
    if (PAIRED && grp < A_INS) {                 // 8 activation rows of 128 bytes
      const int r8 = grp * 8 + lane / 8;
      int am = m0 + r8;
      am = am < M ? am : M - 1;                  // rows past M are copied (clamped) and never stored
      src[j] = g.a + (size_t)m0 * 2 * K + (size_t)step_begin * 64;
      off[j] = (uint32_t)(am - m0) * (uint32_t)(4 * K) + (((lane % 8) ^ (((r8 >> 1) & 3) << 1)) * 16);
      continue;
    }
    if (grp * RPI < TERMS * BM) {                // a group lies in one array: BM is a multiple of RPI
      const int first = grp * RPI;
      int am = m0 + (r < BM ? r : r - BM);
      am = am < M ? am : M - 1;                  // rows past M are copied (clamped) and never stored
      src[j] = (first < BM ? g.a : g.a_lo) + (size_t)m0 * K + (size_t)step_begin * BK;
      off[j] = (uint32_t)(am - m0) * (uint32_t)(2 * K) + ch * 16;
    } else {
      const int col = grp * RPI - TERMS * BM;    // the group's first column: all its rows are in one weight array
      int wrow;
      const bf16_t* wbase;
      if (EPI == GEMM_SWIGLU) {                  // 16-column groups alternate gate, up
        wrow = (n0 >> 1) + ((col >> 5) << 4) + (col & 15);
        wbase = ((col >> 4) & 1) ? g.w[1] : g.w[0];
      } else {
        wrow = n0 + col;
        wbase = g.w[0];
        if (wrow >= g.w_rows[0]) {
          wrow -= g.w_rows[0];
          wbase = g.w[1];
          if (wrow >= g.w_rows[1]) {
            wrow -= g.w_rows[1];
            wbase = g.w[2];
          }
        }
      }
      src[j] = wbase + (size_t)wrow * K + (size_t)step_begin * BK;
      off[j] = (uint32_t)(lane / CPR) * (uint32_t)(2 * K) + ch * 16;
    }
  }

  f32x4 acc[MT][NF];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NF; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int l16 = lane & 15, kc = lane >> 4;
  const int a_pair[2] = {swz16<8>(l16, kc), swz16<8>(l16, 4 + kc)};   // PAIRED: high and low fragment of a 128-byte row
  int a_off[KSUB], w_off[KSUB];                                   // per K sub-step; + i * 16 rows (+ BM rows: lo), + j * 16 rows
#pragma unroll
  for (int ks = 0; ks < KSUB; ++ks) {
    a_off[ks] = swz16<CPR>(l16, 4 * ks + kc);
    w_off[ks] = TERMS * BM * BK + swz16<CPR>(wave * 16 * NF + l16, 4 * ks + kc);
  }
  // bf16 pair -> fp16 pair: exponent raised on both halves at once, each half widened to fp32 (a shift, a mask),
  // and the two packed again (exact: 8 mantissa bits into 11).  A zero becomes 2^(SY_W_SHIFT - 127) in fp32 and
  // goes back to zero in the packing.
  const uint32_t exp_add = ((uint32_t)SY_W_SHIFT << 7) * 0x00010001u, hi_mask = 0xFFFF0000u;
#define SY_COPY(J_, NXT, STEP) glds16_at(src[J_] + (size_t)(STEP) * (PAIRED && (J_) < A_IPW ? 64 : BK), off[J_], NXT + dst[J_]);
#define SY_ISSUE(NXT, STEP) _Pragma("unroll") for (int j = 0; j < IPW; ++j) SY_COPY(j, NXT, STEP)
#define SY_MFMA(ACC, FW, FA, I_)                                                                  \
  {                                                                                               \
    if (((I_) + 1) * NF * 4 <= 256) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(ACC) : "v"(FW), "v"(FA)); \
    else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(ACC) : "v"(FW), "v"(FA));   \
  }
#define SY_CVT1(FW, Q_)                                                                           \
  {                                                                                               \
    uint32_t x_ = (FW)[Q_], ta_, tb_;                                                             \
    asm volatile("v_add_u32 %0, %3, %0\n\tv_lshlrev_b32 %1, 16, %0\n\tv_and_b32 %2, %4, %0\n\t"   \
                 "v_cvt_pkrtz_f16_f32 %0, %1, %2"                                                 \
                 : "+v"(x_), "=&v"(ta_), "=&v"(tb_) : "s"(exp_add), "s"(hi_mask));                \
    (FW)[Q_] = x_;                                                                                \
  }
// The same conversion for the next step's fragments fwn, cut into single instructions so that two of them fit
// behind each MFMA without holding up the next one: operation P of 16 NF = fragment P / 16, stage (P % 16) / 4
// (raise the exponents; low half to fp32; high half to fp32, in place; pack), register P % 4.  Consecutive
// operations touch different registers: no instruction waits for the one before it.
#define SY_CVT_OP(P_)                                                                             \
  if ((P_) < 16 * NW) {                                                                           \
    uint32_t x_ = fwn[(P_) / 16][(P_) % 4];                                                       \
    if (((P_) % 16) / 4 == 0) asm volatile("v_add_u32 %0, %1, %0" : "+v"(x_) : "s"(exp_add));     \
    else if (((P_) % 16) / 4 == 1) asm volatile("v_lshlrev_b32 %0, 16, %1" : "=v"(tq[(P_) % 4]) : "v"(x_)); \
    else if (((P_) % 16) / 4 == 2) asm volatile("v_and_b32 %0, %1, %0" : "+v"(x_) : "s"(hi_mask)); \
    else asm volatile("v_cvt_pkrtz_f16_f32 %0, %1, %0" : "+v"(x_) : "v"(tq[(P_) % 4]));           \
    fwn[(P_) / 16][(P_) % 4] = x_;                                                                \
  }
// A wavefront copies exactly the weight rows of its own columns, so it may read them as soon as its own copies
// have landed, ahead of the barrier that publishes the other wavefronts' activation rows.
#define SY_NEXT_W(NEXTSTAGE)                                                                      \
  {                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(IPW) : "memory");                                    \
    _Pragma("unroll") for (int j = 0; j < NW; ++j)                                                \
        fwn[j] = *reinterpret_cast<const u32x4*>(NEXTSTAGE + w_off[j / NF] + (j % NF) * 16 * BK); \
  }
// One K step on the stage CUR with this step's weight fragments fw already converted in registers.  The copies
// of step s+2 go out during the first row blocks; during the last four the weights of step s+1 (NEXTSTAGE) are
// read and converted, two instructions after each MFMA, in the shadow of the matrix core.
#define SY_AT(V_) (PAIRED ? a_pair[0] + (V_) * 16 * 64 : a_off[(V_) % KSUB] + ((V_) / KSUB) * 16 * BK)
#define SY_AT_LO(V_) (PAIRED ? a_pair[1] + (V_) * 16 * 64 : a_off[(V_) % KSUB] + ((V_) / KSUB) * 16 * BK + BM * BK)
#define SY_MULT(STAGE, NXT, NSTEP, NEXTSTAGE)                                                     \
  {                                                                                               \
    u32x4 fa[MV + 2], fl[MV + 2], fwn[NW];                                                        \
    uint32_t tq[4];                                                                               \
    _Pragma("unroll") for (int v = 0; v < 2 && v < MV; ++v) {                                     \
      fa[v] = *reinterpret_cast<const u32x4*>(STAGE + SY_AT(v));                                  \
      if (LO) fl[v] = *reinterpret_cast<const u32x4*>(STAGE + SY_AT_LO(v));                       \
    }                                                                                             \
    __builtin_amdgcn_sched_barrier(0);                                                            \
    _Pragma("unroll") for (int v = 0; v < MV; ++v) {                                              \
      if (v == C_END) SY_NEXT_W(NEXTSTAGE)                                                        \
      _Pragma("unroll") for (int t = 0; t < SLOTS; ++t) {                                         \
        if (t < NF) SY_MFMA(acc[v / KSUB][t], fw[(v % KSUB) * NF + t], fa[v], v / KSUB)           \
        else SY_MFMA(acc[v / KSUB][t - NF], fw[(v % KSUB) * NF + t - NF], fl[v], v / KSUB)        \
        if (v >= C_END) {                                                                         \
          SY_CVT_OP(((v - C_END) * SLOTS + t) * 2)                                                \
          SY_CVT_OP(((v - C_END) * SLOTS + t) * 2 + 1)                                            \
        }                                                                                         \
        if (t == 0 && v + 2 < MV) fa[v + 2] = *reinterpret_cast<const u32x4*>(STAGE + SY_AT(v + 2)); \
        if (LO && t == NF && v + 2 < MV)                                                          \
          fl[v + 2] = *reinterpret_cast<const u32x4*>(STAGE + SY_AT_LO(v + 2));                   \
        _Pragma("unroll") for (int c = 0; c < CPB; ++c)                                           \
            if ((c + 1) % SLOTS == t && v < C_END && v * CPB + c < IPW) SY_COPY(v * CPB + c, NXT, NSTEP) \
        __builtin_amdgcn_sched_barrier(0);                                                        \
      }                                                                                           \
    }                                                                                             \
    if (C_END >= MV) SY_NEXT_W(NEXTSTAGE)                                                         \
    _Pragma("unroll") for (int p = (MV > C_END ? (MV - C_END) * 2 * SLOTS : 0); p < 16 * NW; ++p) SY_CVT_OP(p) \
    _Pragma("unroll") for (int j = 0; j < NW; ++j) fw[j] = fwn[j];                                \
  }
// CUR holds step s; NXT (the stage read in step s-1) receives step s+2.  Past the end the last step is copied
// again (never used): exactly one younger copy group is then always in flight, so the wait count is a constant
// and no branch surrounds the copies.
#define SY_STEP(CUR, NXT, S_, SETTLE, NEXTSTAGE)                                                  \
  {                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(IPW) : "memory");                         \
    asm volatile("s_barrier" ::: "memory");                                                       \
    const int nxt_ = (S_) + 2 < n_steps ? (S_) + 2 : n_steps - 1;                                 \
    SY_MULT(CUR, NXT, nxt_, NEXTSTAGE)                                                            \
    if (SETTLE) asm volatile("s_nop 15" ::: "memory");                                            \
  }

  const uint32_t l0 = lds_addr_of(st0), l1 = lds_addr_of(st1), l2 = lds_addr_of(st2);
  SY_ISSUE(l0, 0)
  {
    const int one_ = n_steps > 1 ? 1 : 0;
    SY_ISSUE(l1, one_)
  }
  // the first step's weights: own copies of stage 0 have landed once at most the IPW younger ones are in flight
  u32x4 fw[NW];
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(IPW) : "memory");
#pragma unroll
  for (int j = 0; j < NW; ++j) fw[j] = *reinterpret_cast<const u32x4*>(st0 + w_off[j / NF] + (j % NF) * 16 * BK);
#pragma unroll
  for (int j = 0; j < NW; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) SY_CVT1(fw[j], q)
  int s = 0;
  // SETTLE: the last step of every basic block ends with wait states that let its final MFMAs finish.  The
  // compiler does not know that the accumulators are MFMA results and is free to copy one to another register
  // where control flow joins -- at the loop's back edge and exits -- where it would read a result the matrix
  // core has not written yet.
  for (; s + 3 <= n_steps; s += 3) {
    SY_STEP(st0, l2, s, false, st1)
    SY_STEP(st1, l0, s + 1, false, st2)
    SY_STEP(st2, l1, s + 2, true, st0)
  }
  if (s < n_steps) {
    SY_STEP(st0, l2, s, true, st1)
    if (s + 1 < n_steps) SY_STEP(st1, l0, s + 1, true, st2)
  }
#undef SY_COPY
#undef SY_ISSUE
#undef SY_MFMA
#undef SY_CVT1
#undef SY_CVT_OP
#undef SY_NEXT_W
#undef SY_MULT
#undef SY_AT
#undef SY_AT_LO
#undef SY_STEP
  // The surplus copies of the last steps are still in flight: let them land before the block's LDS is released;
  // MFMA results settle before they are read.  The empty statements "rewrite" each accumulator: every later read
  // of one depends on them, and they stay behind the wait, so the compiler cannot hoist an accumulator read over it.
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      if ((i + 1) * NF * 4 <= 256) asm volatile("" : "+a"(acc[i][j]));
      else asm volatile("" : "+v"(acc[i][j]));
    }

  const int nq = kc * 4;                         // this lane's 4 consecutive columns inside a 16-column fragment
  const float os = g.out_scale;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + l16;
    if (m >= M) continue;
    if (EPI == GEMM_SWIGLU) {
#pragma unroll
      for (int j = 0; j < NF; j += 2) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float gate = acc[i][j][r] * os, up = acc[i][j + 1][r] * os;
          v[r] = gate / (1.0f + __expf(-gate)) * up * g.c_scale;
        }
        uint32_t h0, l0_, h1, l1_;
        split_f16x2(v[0], v[1], h0, l0_);
        split_f16x2(v[2], v[3], h1, l1_);
        const int col = (n0 >> 1) + (wave * (NF / 2) + (j >> 1)) * 16 + nq;
        if (g.c_paired) {
          uint16_t* at = reinterpret_cast<uint16_t*>(g.c) + (size_t)m * g.N + pair_col(col);
          *reinterpret_cast<uint2*>(at) = make_uint2(h0, h1);
          *reinterpret_cast<uint2*>(at + 32) = make_uint2(l0_, l1_);
        } else {
          const size_t at = (size_t)m * (g.N >> 1) + col;
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.c) + at) = make_uint2(h0, h1);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(g.c_lo) + at) = make_uint2(l0_, l1_);
        }
      }
    } else {
      float* c = (g.split_k > 1 ? g.c_parts + (size_t)blockIdx.z * M * g.N : reinterpret_cast<float*>(g.c)) +
                 (size_t)m * g.N + n0 + wave * 16 * NF + nq;
#pragma unroll
      for (int j = 0; j < NF; ++j) {
        float4 o = make_float4(acc[i][j][0] * os, acc[i][j][1] * os, acc[i][j][2] * os, acc[i][j][3] * os);
        if (EPI == GEMM_ADD_F32 && g.split_k == 1) {
          const float4 old = *reinterpret_cast<float4*>(c + j * 16);
          o.x += old.x;
          o.y += old.y;
          o.z += old.z;
          o.w += old.w;
        }
        *reinterpret_cast<float4*>(c + j * 16) = o;
      }
    }
  }
}

template <int MT, int NF, int KSUB = 1>
static hipError_t launch_proj(const GemmArgs& g, hipStream_t s) {
  constexpr int BM = 16 * MT;
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / (64 * NF);
  const dim3 grid(8 * ((n_tiles + 7) / 8) * m_tiles, 1, g.split_k);
  if (g.K % (32 * KSUB) != 0) return hipErrorInvalidValue;
  if (!g.a_lo && !g.a_paired) {                  // single-term activations: the plain store form only
    if (g.epilogue != GEMM_STORE_F32) return hipErrorInvalidValue;
    proj_kernel<MT, NF, GEMM_STORE_F32, false, KSUB><<<grid, 256, 0, s>>>(g);
    return hipGetLastError();
  }
  if (g.a_paired) {                              // one array [M][K / 32][hi | lo]: the forms with one K step per stage
    if constexpr (KSUB == 1) {
      switch (g.epilogue) {
        case GEMM_STORE_F32: proj_kernel<MT, NF, GEMM_STORE_F32, true, 1, true><<<grid, 256, 0, s>>>(g); break;
        case GEMM_ADD_F32: proj_kernel<MT, NF, GEMM_ADD_F32, true, 1, true><<<grid, 256, 0, s>>>(g); break;
        case GEMM_SWIGLU: proj_kernel<MT, NF, GEMM_SWIGLU, true, 1, true><<<grid, 256, 0, s>>>(g); break;
        default: return hipErrorInvalidValue;
      }
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  switch (g.epilogue) {
    case GEMM_STORE_F32: proj_kernel<MT, NF, GEMM_STORE_F32, true, KSUB><<<grid, 256, 0, s>>>(g); break;
    case GEMM_ADD_F32: proj_kernel<MT, NF, GEMM_ADD_F32, true, KSUB><<<grid, 256, 0, s>>>(g); break;
    case GEMM_SWIGLU: proj_kernel<MT, NF, GEMM_SWIGLU, true, KSUB><<<grid, 256, 0, s>>>(g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
