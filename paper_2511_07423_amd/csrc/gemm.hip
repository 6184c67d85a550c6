// bf16 matrix-core GEMM for the decoder's projections: C[M][N] = A[M][K] * W[N][K]^T
// with fp32 accumulation (v_mfma_f32_32x32x16_bf16).  Both operands are K-major, so
// an MFMA operand fragment (8 consecutive k of one row) is one 16-byte read.
//
// Activations arrive as a bf16 pair (hi, lo) with hi + lo equal to the fp32 value to
// about 16 mantissa bits; the kernel accumulates A_hi*W and A_lo*W into the same
// accumulators.  (bf16 weights are exact; a single bf16 activation term leaves the
// logits of a 32-layer decoder an order of magnitude outside the parity tolerance.)
// The lo term reuses the weight fragments already in registers, so it costs MFMA
// issue slots but no extra weight traffic from HBM, L2 or LDS.
//
// Launch: a 1-D grid whose block index is mapped to (M tile, N tile) so that the blocks sharing a
// weight tile land on the same XCD (see the kernel).
//
// Tiling: a block of WGM x WGN wavefronts owns a BM x BN output tile; each wavefront
// a (BM/WGM) x (BN/WGN) sub-tile made of 32x32 MFMA blocks.  K advances in steps of BK
// through double-buffered LDS tiles whose 16-byte chunks are XOR-swizzled by row, so
// fragment reads are bank-conflict free.  Global loads of step i+1 are issued before
// the MFMAs of step i and parked in registers.
//
// The weight may be given as up to three row segments (Wq | Wk | Wv share one
// launch).  Epilogues: store fp32; add into fp32 (residual stream); SwiGLU, where the
// tile's even 32-column blocks come from W_gate and the odd ones from W_up at the same
// rows, so one lane holds gate and up of the same output and writes
// silu(gate) * up as a bf16 (hi, lo) pair.  split_k > 1 spreads K over blockIdx.z and
// adds the partial sums with hardware fp32 atomics (the order of those adds is not fixed).
#include "common.h"

// LDS tiles hold K-major rows of CPR 16-byte chunks; chunk c of row r sits at position c ^ swz_mask(r).
// A 16-byte fragment read (lane = row l % 32, chunk from l / 32) is served 16 lanes per cycle over the 64
// banks, lanes l and l + 16 in the same cycle: the mask therefore varies with the row's low bits (rows
// 128 bytes or less apart would share banks) AND with bit 4 of the row (rows r and r + 16 would collide
// otherwise -- measured: every second LDS cycle of the fragment reads was a bank conflict without it).
// Which k a lane feeds to an MFMA is free as long as both operands agree: in sub-step ks of a BK-wide
// tile the lower 32 lanes take chunk ks and the upper 32 lanes chunk BK/16 + ks, which keeps the two
// halves of the wavefront on different banks under that mask as well.
template <int CPR>
__device__ __forceinline__ int swz_mask(int row) {
  return ((row / (8 / CPR)) % CPR) ^ ((row >> 4) & 1);
}
template <int CPR>
__device__ __forceinline__ int swz(int row, int chunk) {
  // element offset of 16-byte chunk `chunk` of `row` in a tile with CPR chunks per row
  return (row * CPR + (chunk ^ swz_mask<CPR>(row))) * 8;
}

template <int BM, int BN, int BK, int WGM, int WGN, bool SPLIT, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmArgs g) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NJ = WN / 32;
  constexpr int CPR = BK / 8;
  constexpr int A_CH = BM * CPR / NT, B_CH = BN * CPR / NT;
  constexpr int NA = SPLIT ? 2 : 1;
  constexpr int A_ELEMS = BM * BK, B_ELEMS = BN * BK;
  constexpr int STAGE = NA * A_ELEMS + B_ELEMS;
  static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile / thread mismatch");
  static_assert(EPI != GEMM_SWIGLU_BF16 || NJ % 2 == 0, "SwiGLU needs gate/up column-block pairs per wavefront");
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so
  // block b runs on XCD b % 8.  Within an XCD consecutive blocks walk the M tiles of one N tile: the
  // blocks that share a weight tile run together on one L2 and the weights leave HBM once.
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / BN;
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int n_tile = (within / m_tiles) * 8 + xcd;
  if (n_tile >= n_tiles) return;
  const int m0 = (within % m_tiles) * BM, n0 = n_tile * BN;
  const int K = g.K, M = g.M;
  const int k_per = K / g.split_k;                 // multiple of BK (checked by the launcher)
  const int k_begin = blockIdx.z * k_per;
  const int n_steps = k_per / BK;

  const bf16_t* a_src[A_CH];
  int a_off[A_CH];
  size_t lo_delta = 0;
  if (SPLIT) lo_delta = (size_t)(g.a_lo - g.a);
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int id = tid + i * NT, row = id / CPR, ch = id % CPR;
    int am = m0 + row;
    am = am < M ? am : M - 1;                      // rows past M are loaded (clamped) and never stored
    a_src[i] = g.a + (size_t)am * K + k_begin + ch * 8;
    a_off[i] = swz<CPR>(row, ch);
  }
  const bf16_t* b_src[B_CH];
  int b_off[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int id = tid + i * NT, row = id / CPR, ch = id % CPR;
    int wrow;                                      // weight row feeding tile column `row`
    const bf16_t* wbase;
    if (EPI == GEMM_SWIGLU_BF16) {
      wrow = (n0 >> 1) + ((row >> 6) << 5) + (row & 31);
      wbase = ((row >> 5) & 1) ? g.w[1] : g.w[0];
    } else {
      wrow = n0 + row;
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
    b_src[i] = wbase + (size_t)wrow * K + k_begin + ch * 8;
    b_off[i] = swz<CPR>(row, ch);
  }

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Staging registers for the next K step.  The loop body is branch-free (the last step is peeled):
  // with the fetch under a condition the compiler kept these arrays in scratch memory.
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  u32x4 ra[A_CH], rl[A_CH], rb[B_CH];
#define SY_FETCH(STEP)                                                                              \
  _Pragma("unroll") for (int i = 0; i < A_CH; ++i) {                                                \
    ra[i] = *reinterpret_cast<const u32x4*>(a_src[i] + (size_t)(STEP) * BK);                        \
    if (SPLIT) rl[i] = *reinterpret_cast<const u32x4*>(a_src[i] + lo_delta + (size_t)(STEP) * BK);  \
  }                                                                                                 \
  _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                                  \
      rb[i] = *reinterpret_cast<const u32x4*>(b_src[i] + (size_t)(STEP) * BK);
#define SY_PARK(BUF)                                                                                \
  {                                                                                                 \
    bf16_t* s_ = smem + (BUF) * STAGE;                                                              \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i) {                                              \
      *reinterpret_cast<u32x4*>(s_ + a_off[i]) = ra[i];                                             \
      if (SPLIT) *reinterpret_cast<u32x4*>(s_ + A_ELEMS + a_off[i]) = rl[i];                        \
    }                                                                                               \
    _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                                \
        *reinterpret_cast<u32x4*>(s_ + NA * A_ELEMS + b_off[i]) = rb[i];                            \
  }
  const int l32 = lane & 31, kb = lane >> 5;
#define SY_COMPUTE(BUF)                                                                             \
  {                                                                                                 \
    const bf16_t* sA = smem + (BUF) * STAGE;                                                        \
    const bf16_t* sB = sA + NA * A_ELEMS;                                                           \
    _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                        \
      bf16x8 fb[NJ];                                                                                \
      _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                                \
          fb[j] = *reinterpret_cast<const bf16x8*>(sB + swz<CPR>(wn * WN + j * 32 + l32, kb * (BK / 16) + ks)); \
      _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                              \
        const int ar = wm * WM + i * 32 + l32;                                                      \
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(sA + swz<CPR>(ar, kb * (BK / 16) + ks));         \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                              \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[j], acc[i][j], 0, 0, 0);     \
        if (SPLIT) {                                                                                \
          const bf16x8 fl = *reinterpret_cast<const bf16x8*>(sA + A_ELEMS + swz<CPR>(ar, kb * (BK / 16) + ks)); \
          _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                            \
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl, fb[j], acc[i][j], 0, 0, 0);   \
        }                                                                                           \
      }                                                                                             \
    }                                                                                               \
  }

  // Instruction order inside one K step: the fragment reads of k-slice ks+1 are interleaved one by one
  // with the MFMAs of k-slice ks, so a wavefront covers its own LDS latency.
#define SY_SCHED()                                                                                  \
  {                                                                                                 \
    constexpr int RPK = NJ + MI * NA, MPK = MI * NJ * NA, KSN = BK / 16;                            \
    constexpr int REST = MPK > RPK ? MPK - RPK : 0;                                                 \
    __builtin_amdgcn_sched_group_barrier(0x100, RPK, 0);                                            \
    _Pragma("unroll") for (int ks = 0; ks + 1 < KSN; ++ks) {                                        \
      _Pragma("unroll") for (int i = 0; i < RPK; ++i) {                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                          \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
      }                                                                                             \
      __builtin_amdgcn_sched_group_barrier(0x008, REST, 0);                                         \
    }                                                                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, MPK, 0);                                            \
  }

  SY_FETCH(0)
  SY_PARK(0)
  __syncthreads();
  for (int step = 0; step + 1 < n_steps; ++step) {
    const int buf = step & 1;
    SY_FETCH(step + 1)
    __builtin_amdgcn_sched_barrier(0);   // keep the global loads ahead of the MFMAs: the scheduler otherwise
    SY_COMPUTE(buf)                      // sinks them to just before the LDS stores and exposes their latency
    SY_SCHED()
    __builtin_amdgcn_sched_barrier(0);
    SY_PARK(buf ^ 1)
    __syncthreads();
  }
  SY_COMPUTE((n_steps - 1) & 1)
#undef SY_FETCH
#undef SY_PARK
#undef SY_COMPUTE
#undef SY_SCHED

  // Epilogue.  A 32x32 accumulator block leaves lane (l32, kb) with column l32 and rows
  // 8*(r/4) + 4*kb + r%4, r = 0..15.
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
      if (m >= M) continue;
      if (EPI == GEMM_SWIGLU_BF16) {
#pragma unroll
        for (int j = 0; j < NJ; j += 2) {
          const float gate = acc[i][j][r], up = acc[i][j + 1][r];
          const float v = gate / (1.0f + __expf(-gate)) * up;
          const size_t at = (size_t)m * (g.N >> 1) + (n0 >> 1) + ((wn * WN + j * 32) >> 1) + l32;
          const uint32_t hi = f2bf(v);
          reinterpret_cast<bf16_t*>(g.c)[at] = (bf16_t)hi;
          reinterpret_cast<bf16_t*>(g.c_lo)[at] = (bf16_t)f2bf(v - bf2f(hi));
        }
      } else {
        float* c = reinterpret_cast<float*>(g.c) + (size_t)m * g.N + n0 + wn * WN + l32;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const float v = acc[i][j][r];
          if (g.split_k > 1) {
            unsafeAtomicAdd(c + j * 32, v);
          } else if (EPI == GEMM_ADD_F32) {
            c[j * 32] += v;
          } else {
            c[j * 32] = v;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Variant with asynchronous global->LDS copies (global_load_lds_dwordx4): the tile rows
// [A_hi | A_lo | W] of K step s+2 stream straight into LDS while step s is multiplied, with no
// staging registers and no LDS store instructions.  Three LDS stages, BK = 32.  A copy instruction
// of one wavefront fills 1 KB = 16 tile rows; the XOR swizzle is applied on the global side (lane i
// fetches the chunk that belongs at LDS position i).  Synchronisation per K step: each wavefront
// waits for its own copies of the step (s_waitcnt vmcnt), one s_barrier makes every wavefront's
// copies visible and certifies that the stage about to be overwritten is no longer read.
// The three stages are separate arrays so the compiler can tell copies in flight from fragment
// reads apart (with one array it waits for ALL copies before every LDS read).
// The copy is issued from inline assembly: through the compiler builtin every later LDS read is
// preceded by a wait for ALL copies in flight once more than a few distinct copy instructions
// exist, which would serialise the pipeline.  m0 carries the wavefront-uniform LDS address; lane i
// lands at that address + 16 i.
__device__ __forceinline__ void glds16(const void* gptr, const void* lds_ptr) {
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds_ptr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
#define SY_GLDS16(gptr, lptr) glds16((gptr), (lptr))
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ void glds16_at(const void* gptr, uint32_t lds_addr) {   // lds_addr: wavefront-uniform
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}

template <int BM, int BN, int BK, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_dma_kernel(GemmArgs g) {
  constexpr int CPR = BK / 8, NW = WGM * WGN;
  constexpr int RPI = 64 / CPR;             // tile rows filled by one copy instruction (1 KB)
  constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NJ = WN / 32;
  constexpr int R = 2 * BM + BN;            // tile rows per stage: A_hi, A_lo, W
  constexpr int IPS = R / RPI, IPW = IPS / NW;
  static_assert(R % RPI == 0 && IPS % NW == 0, "rows per stage must split evenly over the wavefronts");
  static_assert(EPI != GEMM_SWIGLU_BF16 || NJ % 2 == 0, "SwiGLU needs gate/up column-block pairs per wavefront");
  __shared__ __attribute__((aligned(16))) bf16_t st0[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st1[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st2[R * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / BN;
  const int xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
  const int n_tile = (within / m_tiles) * 8 + xcd;
  if (n_tile >= n_tiles) return;
  const int m0 = (within % m_tiles) * BM, n0 = n_tile * BN;
  const int K = g.K, M = g.M;
  const int k_per = K / g.split_k;
  const int k_begin = blockIdx.z * k_per;
  const int n_steps = k_per / BK;

  // Source of this lane for each of the wavefront's copy instructions.
  const bf16_t* src[IPW];
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    const int r = (wave * IPW + j) * RPI + lane / CPR;
    const int ch = (lane % CPR) ^ swz_mask<CPR>(r);
    const bf16_t* base;
    if (r < 2 * BM) {
      int am = m0 + (r < BM ? r : r - BM);
      am = am < M ? am : M - 1;                    // rows past M are copied (clamped) and never stored
      base = (r < BM ? g.a : g.a_lo) + (size_t)am * K;
    } else {
      const int col = r - 2 * BM;
      int wrow;
      const bf16_t* wbase;
      if (EPI == GEMM_SWIGLU_BF16) {
        wrow = (n0 >> 1) + ((col >> 6) << 5) + (col & 31);
        wbase = ((col >> 5) & 1) ? g.w[1] : g.w[0];
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
      base = wbase + (size_t)wrow * K;
    }
    src[j] = base + k_begin + ch * 8;
  }

  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int l32 = lane & 31, kb = lane >> 5;
#define SY_ISSUE(STAGE, STEP)                                                                     \
  _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                                 \
      SY_GLDS16(src[j] + (size_t)(STEP) * BK, STAGE + (wave * IPW + j) * RPI * BK);
#define SY_MULT(STAGE)                                                                            \
  {                                                                                               \
    _Pragma("unroll") for (int ks = 0; ks < BK / 16; ++ks) {                                      \
      bf16x8 fb[NJ];                                                                              \
      _Pragma("unroll") for (int j = 0; j < NJ; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(    \
          STAGE + 2 * BM * BK + swz<CPR>(wn * WN + j * 32 + l32, kb * (BK / 16) + ks));                   \
      _Pragma("unroll") for (int i = 0; i < MI; ++i) {                                            \
        const int ar = wm * WM + i * 32 + l32;                                                    \
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(STAGE + swz<CPR>(ar, kb * (BK / 16) + ks));    \
        const bf16x8 fl = *reinterpret_cast<const bf16x8*>(STAGE + BM * BK + swz<CPR>(ar, kb * (BK / 16) + ks)); \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                            \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[j], acc[i][j], 0, 0, 0);   \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                            \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl, fb[j], acc[i][j], 0, 0, 0);   \
      }                                                                                           \
    }                                                                                             \
  }
  // One K step: CUR holds step s; NXT (the stage read in step s-1) receives step s+2.  Past the end
  // the last step is copied again (never read): exactly one younger copy group is then always in
  // flight, so the wait count is a constant and no branch surrounds the copies (under a branch the
  // compiler loses track of which stage a copy targets and waits for all of them before every read).
#define SY_STEP(CUR, NXT, S_)                                                                     \
  {                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(IPW) : "memory");                         \
    asm volatile("s_barrier" ::: "memory");                                                       \
    const int nxt_ = (S_) + 2 < n_steps ? (S_) + 2 : n_steps - 1;                                 \
    SY_ISSUE(NXT, nxt_)                                                                           \
    SY_MULT(CUR)                                                                                  \
  }

  SY_ISSUE(st0, 0)
  {
    const int one_ = n_steps > 1 ? 1 : 0;
    SY_ISSUE(st1, one_)
  }
  int s = 0;
  for (; s + 3 <= n_steps; s += 3) {
    SY_STEP(st0, st2, s)
    SY_STEP(st1, st0, s + 1)
    SY_STEP(st2, st1, s + 2)
  }
  if (s < n_steps) {
    SY_STEP(st0, st2, s)
    if (s + 1 < n_steps) SY_STEP(st1, st0, s + 1)
  }
#undef SY_ISSUE
#undef SY_MULT
#undef SY_STEP
  // the surplus copies of the last steps are still in flight: let them land before the block's LDS is released
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
      if (m >= M) continue;
      if (EPI == GEMM_SWIGLU_BF16) {
#pragma unroll
        for (int j = 0; j < NJ; j += 2) {
          const float gate = acc[i][j][r], up = acc[i][j + 1][r];
          const float v = gate / (1.0f + __expf(-gate)) * up;
          const size_t at = (size_t)m * (g.N >> 1) + (n0 >> 1) + ((wn * WN + j * 32) >> 1) + l32;
          const uint32_t hi = f2bf(v);
          reinterpret_cast<bf16_t*>(g.c)[at] = (bf16_t)hi;
          reinterpret_cast<bf16_t*>(g.c_lo)[at] = (bf16_t)f2bf(v - bf2f(hi));
        }
      } else {
        float* c = reinterpret_cast<float*>(g.c) + (size_t)m * g.N + n0 + wn * WN + l32;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const float v = acc[i][j][r];
          if (g.split_k > 1) {
            unsafeAtomicAdd(c + j * 32, v);
          } else if (EPI == GEMM_ADD_F32) {
            c[j * 32] += v;
          } else {
            c[j * 32] = v;
          }
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WGM, int WGN>
static hipError_t launch_dma(const GemmArgs& g, hipStream_t s) {
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / BN;
  const dim3 grid(8 * ((n_tiles + 7) / 8) * m_tiles, 1, g.split_k);
  const dim3 block(64 * WGM * WGN);
  switch (g.epilogue) {
    case GEMM_STORE_F32: gemm_dma_kernel<BM, BN, BK, WGM, WGN, GEMM_STORE_F32><<<grid, block, 0, s>>>(g); break;
    case GEMM_ADD_F32: gemm_dma_kernel<BM, BN, BK, WGM, WGN, GEMM_ADD_F32><<<grid, block, 0, s>>>(g); break;
    case GEMM_SWIGLU_BF16: gemm_dma_kernel<BM, BN, BK, WGM, WGN, GEMM_SWIGLU_BF16><<<grid, block, 0, s>>>(g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Tall-tile variant for verification batches (a few hundred rows): the block tile spans BM = 32 MB
// rows -- half of M, or all of it -- by 256 columns, so a weight tile is pulled from L2 at most
// twice and the operand bytes moved L2 -> LDS per multiply drop by about 2.5x against the 64-row
// tile (that traffic, not the matrix cores, bounds the smaller tiles).  Four wavefronts, one per
// SIMD, each own all BM rows of 64 columns: 2 MB accumulator fragments of v_mfma_f32_32x32x16_bf16
// (a single wavefront keeps the matrix core busy with this 8-pass instruction; with the 4-pass 16x16x32
// one it reaches about half the rate).  Per K step of 32 a wavefront reads its 4 weight fragments once
// and streams the 4 MB activation fragments (hi, lo) through them.  LDS: three stages of
// (2 BM + 256) rows x 64 B, filled by the same asynchronous copies as above; one block per CU.
// K may be split unevenly over blockIdx.z (in units of BK) so that tiles x splits fills the chip.
//
// The MFMAs are issued from inline assembly with the accumulator tied to the destination: left to the
// compiler, accumulators migrate between registers from one K step to the next (dozens of copies per
// step, and spills once they need more than the 256 AGPRs).  Row blocks 0..7 accumulate in AGPRs, a
// ninth in VGPRs.  The copies of K step s+2 are spread over the row blocks of step s: issued together
// right after the barrier, the four wavefronts queue ~50 copy instructions on the CU's one address
// unit and none of them reaches its first MFMA for several hundred cycles.
template <int MB, int EPI>
__global__ __launch_bounds__(256) void gemm_tall_kernel(GemmArgs g) {
  constexpr int BM = 32 * MB, BN = 256, BK = 32, CPR = 4;
  constexpr int A_INS = 4 * MB;                  // copy instructions (16 tile rows each) for [A_hi | A_lo]
  constexpr int A_IPW = MB;                      // per wavefront
  constexpr int W_IPW = BN / 16 / 4;
  constexpr int IPW = A_IPW + W_IPW;
  constexpr int R = 2 * BM + BN;
  static_assert(MB >= 1 && MB <= 9, "accumulators: 32 MB registers per lane, stages: 3 (2 BM + 256) x 64 B of LDS");
  __shared__ __attribute__((aligned(16))) bf16_t st0[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st1[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st2[R * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

  const bf16_t* src[IPW];
  uint32_t dst[IPW];                             // byte offset of the copy's 16 rows inside a stage
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    const int grp = j < A_IPW ? wave + 4 * j : A_INS + wave * W_IPW + (j - A_IPW);   // 16-row group of the stage
    const int r = grp * 16 + lane / CPR;
    const int ch = (lane % CPR) ^ swz_mask<CPR>(r);
    const bf16_t* base;
    if (r < 2 * BM) {
      int am = m0 + (r < BM ? r : r - BM);
      am = am < M ? am : M - 1;                  // rows past M are copied (clamped) and never stored
      base = (r < BM ? g.a : g.a_lo) + (size_t)am * K;
    } else {
      const int col = r - 2 * BM;
      int wrow;
      const bf16_t* wbase;
      if (EPI == GEMM_SWIGLU_BF16) {             // 32-column blocks alternate gate, up
        wrow = (n0 >> 1) + ((col >> 6) << 5) + (col & 31);
        wbase = ((col >> 5) & 1) ? g.w[1] : g.w[0];
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
      base = wbase + (size_t)wrow * K;
    }
    src[j] = base + (size_t)step_begin * BK + ch * 8;
    dst[j] = grp * 16 * BK * 2;
  }

  f32x16 acc[MB][2];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int l32 = lane & 31, kb = lane >> 5;
  // fragment offsets of sub-step 0; sub-step 1 is the next chunk (its XOR partner, see swz)
  const int a_off0 = swz<CPR>(l32, kb * 2), a_off1 = swz<CPR>(l32, kb * 2 + 1);             // + i * 32 rows; + BM rows: lo
  const int w_off0 = 2 * BM * BK + swz<CPR>(wave * 64 + l32, kb * 2);                        // + j * 32 rows
  const int w_off1 = 2 * BM * BK + swz<CPR>(wave * 64 + l32, kb * 2 + 1);
#define SY_COPY(J_, NXT, STEP) glds16_at(src[J_] + (size_t)(STEP) * BK, NXT + dst[J_]);
#define SY_ISSUE(NXT, STEP) _Pragma("unroll") for (int j = 0; j < IPW; ++j) SY_COPY(j, NXT, STEP)
#define SY_MFMA(ACC, FA, FW, I_)                                                                  \
  {                                                                                               \
    if ((I_) < 8) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(FA), "v"(FW)); \
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(FA), "v"(FW));  \
  }
#define SY_LOAD_A(I_, STAGE)                                                                      \
  if ((I_) < MB) {                                                                                \
    fa[((I_) >> 1) & 1][(I_) & 1][0] = *reinterpret_cast<const bf16x8*>(STAGE + a_off0 + (I_) * 32 * BK);        \
    fa[((I_) >> 1) & 1][(I_) & 1][1] = *reinterpret_cast<const bf16x8*>(STAGE + a_off1 + (I_) * 32 * BK);        \
    fa[((I_) >> 1) & 1][(I_) & 1][2] = *reinterpret_cast<const bf16x8*>(STAGE + a_off0 + (BM + (I_) * 32) * BK); \
    fa[((I_) >> 1) & 1][(I_) & 1][3] = *reinterpret_cast<const bf16x8*>(STAGE + a_off1 + (BM + (I_) * 32) * BK); \
  }
// Row blocks go through the matrix core in pairs: (block, column half) gives four independent
// accumulators per fragment term, so an accumulator is needed again only four MFMAs later (an MFMA that
// accumulates onto the result of the one issued just before the previous one still waits for it).
#define SY_MULT(STAGE, NXT, NSTEP)                                                                \
  {                                                                                               \
    constexpr int NP = (MB + 1) / 2;                                                              \
    bf16x8 fw[2][2], fa[2][2][4];                /* fw[j][ks]; fa[buffer][block of the pair][hi ks0, hi ks1, lo ks0, lo ks1] */ \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                               \
      fw[j][0] = *reinterpret_cast<const bf16x8*>(STAGE + w_off0 + j * 32 * BK);                  \
      fw[j][1] = *reinterpret_cast<const bf16x8*>(STAGE + w_off1 + j * 32 * BK);                  \
    }                                                                                             \
    SY_LOAD_A(0, STAGE)                                                                           \
    SY_LOAD_A(1, STAGE)                                                                           \
    _Pragma("unroll") for (int p = 0; p < NP; ++p) {                                              \
      SY_LOAD_A(2 * p + 2, STAGE)                                                                 \
      SY_LOAD_A(2 * p + 3, STAGE)                                                                 \
      _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                             \
          if (j * NP / IPW == p) SY_COPY(j, NXT, NSTEP)                                           \
      _Pragma("unroll") for (int t = 0; t < 4; ++t)                                               \
          _Pragma("unroll") for (int b = 0; b < 2; ++b)                                           \
              _Pragma("unroll") for (int j = 0; j < 2; ++j)                                       \
                  if (2 * p + b < MB) SY_MFMA(acc[2 * p + b][j], fa[p & 1][b][t], fw[j][t & 1], 2 * p + b) \
    }                                                                                             \
  }
#define SY_STEP(CUR, NXT, S_, SETTLE)                                                             \
  {                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(IPW) : "memory");                         \
    asm volatile("s_barrier" ::: "memory");                                                       \
    const int nxt_ = (S_) + 2 < n_steps ? (S_) + 2 : n_steps - 1;                                 \
    SY_MULT(CUR, NXT, nxt_)                                                                       \
    if (SETTLE) asm volatile("s_nop 15" ::: "memory");                                            \
  }

  const uint32_t l0 = lds_addr_of(st0), l1 = lds_addr_of(st1), l2 = lds_addr_of(st2);
  SY_ISSUE(l0, 0)
  {
    const int one_ = n_steps > 1 ? 1 : 0;
    SY_ISSUE(l1, one_)
  }
  int s = 0;
  // SETTLE: the last step of every basic block ends with wait states that let its final MFMAs finish.  The
  // compiler does not know that the accumulators are MFMA results (see below) and is free to copy one to
  // another register where control flow joins -- at the loop's back edge and exits -- where it would read
  // a result the matrix core has not written yet.
  for (; s + 3 <= n_steps; s += 3) {
    SY_STEP(st0, l2, s, false)
    SY_STEP(st1, l0, s + 1, false)
    SY_STEP(st2, l1, s + 2, true)
  }
  if (s < n_steps) {
    SY_STEP(st0, l2, s, true)
    if (s + 1 < n_steps) SY_STEP(st1, l0, s + 1, true)
  }
#undef SY_COPY
#undef SY_ISSUE
#undef SY_MFMA
#undef SY_LOAD_A
#undef SY_MULT
#undef SY_STEP
  // The surplus copies of the last steps are still in flight: let them land before the block's LDS is
  // released.  The MFMAs above are inline assembly: the compiler does not know that the accumulators were
  // just written by them, so the wait the hardware needs before other instructions read an MFMA result is
  // spelled out here.
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  // (empty statements that "rewrite" each accumulator: every later read of one depends on them, and they
  // stay behind the wait above, so the compiler cannot hoist an accumulator read over it)
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (i < 8) asm volatile("" : "+a"(acc[i][j]));
      else asm volatile("" : "+v"(acc[i][j]));
    }

#pragma unroll
  for (int i = 0; i < MB; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
      if (m >= M) continue;
      if (EPI == GEMM_SWIGLU_BF16) {
        const float gate = acc[i][0][r], up = acc[i][1][r];
        const float v = gate / (1.0f + __expf(-gate)) * up;
        const size_t at = (size_t)m * (g.N >> 1) + (n0 >> 1) + wave * 32 + l32;
        const uint32_t hi = f2bf(v);
        reinterpret_cast<bf16_t*>(g.c)[at] = (bf16_t)hi;
        reinterpret_cast<bf16_t*>(g.c_lo)[at] = (bf16_t)f2bf(v - bf2f(hi));
      } else {
        const bool defer = g.deferred && g.split_k > 1;
        float* c = (defer ? g.c_parts + (size_t)blockIdx.z * M * g.N : reinterpret_cast<float*>(g.c)) +
                   (size_t)m * g.N + n0 + wave * 64 + l32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const float v = acc[i][j][r];
          if (defer) {
            c[j * 32] = v;
          } else if (g.split_k > 1) {
            unsafeAtomicAdd(c + j * 32, v);
          } else if (EPI == GEMM_ADD_F32) {
            c[j * 32] += v;
          } else {
            c[j * 32] = v;
          }
        }
      }
    }
  }
}

template <int MT>
static hipError_t launch_tall(const GemmArgs& g, hipStream_t s) {
  constexpr int BM = 32 * MT;
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / 256;
  const dim3 grid(8 * ((n_tiles + 7) / 8) * m_tiles, 1, g.split_k);
  switch (g.epilogue) {
    case GEMM_STORE_F32: gemm_tall_kernel<MT, GEMM_STORE_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_ADD_F32: gemm_tall_kernel<MT, GEMM_ADD_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_SWIGLU_BF16: gemm_tall_kernel<MT, GEMM_SWIGLU_BF16><<<grid, 256, 0, s>>>(g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// The same tall tile built from v_mfma_f32_16x16x32_bf16: BM = 16 MT rows, so the tile height moves in
// steps of 16 rows and two tiles can hug an M that two 32-row-granular tiles overshoot (M = 532: 2 x 272
// against 2 x 288).  BK = 32 is exactly one MFMA K step: lane l holds row l % 16 and the 8 k values of
// chunk l / 16 for both operands.  The weight fragment is the MFMA's first operand, so a lane ends up with
// 4 consecutive output columns of one row and the epilogue stores 16 bytes per lane.  Per K step a
// wavefront reads its 4 weight fragments once and streams the 2 MT activation fragments (hi, lo) through
// them; each activation fragment feeds 4 independent accumulators, which is what this 4-pass MFMA needs
// to issue back to back.  Row blocks 0..15 accumulate in AGPRs, a seventeenth in VGPRs.  Within a 16-row
// fragment the chunk position only has to vary with the row's bits 1..2 (see swz_mask: bit 4 is constant
// inside one fragment), so the stage layout uses that plain mask.  K slices are only ever stored for
// the consumer to add (GemmArgs::deferred): there is no atomic path, whose per-element operands would
// need every accumulator in a VGPR at once.
// (Tried on top of this: the four wavefronts as 2 x 2 -- each owning half the rows of half the columns --
// with 224-column tiles, which halves the activation-fragment reads from LDS and gives the 8B gate/up
// projection 256 tiles instead of 224.  Correct, and exactly as fast: the launch is limited by how much MFMA
// work the chip sustains on real data, not by LDS traffic or idle compute units.  Likewise a software-
// pipelined K loop that issues each step's last 16 MFMAs behind the next step's barrier, over the LDS round
// trip of its first fragment reads: correct, same speed.  The shader clock reads 2.08 GHz instead of
// 2.4 GHz while this kernel runs on random operands; on all-zero operands it stays at 2.4 GHz and the same
// launch takes 157 us instead of 199.)
__device__ __forceinline__ int swz16(int row, int chunk) { return (row * 4 + (chunk ^ ((row >> 1) & 3))) * 8; }

template <int MT, int NF, int EPI>
__global__ __launch_bounds__(256) void gemm_tall16_kernel(GemmArgs g) {
  constexpr int BM = 16 * MT, BN = 64 * NF, BK = 32;   // NF column fragments of 16 per wavefront
  static_assert(NF == 2 || NF == 4, "SwiGLU pairs the fragments (gate, up): NF must be even");
  constexpr int A_INS = 2 * MT;                  // copy instructions (16 tile rows each) for [A_hi | A_lo]
  constexpr int A_IPW = (A_INS + 3) / 4;         // per wavefront; a surplus one repeats the last group
  constexpr int W_IPW = BN / 16 / 4;
  constexpr int IPW = A_IPW + W_IPW;
  constexpr int R = 2 * BM + BN;
  static_assert(MT >= 1 && MT <= 17, "accumulators: 16 MT registers per lane, stages: 3 (2 BM + 256) x 64 B of LDS");
  __shared__ __attribute__((aligned(16))) bf16_t st0[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st1[R * BK];
  __shared__ __attribute__((aligned(16))) bf16_t st2[R * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

  const bf16_t* src[IPW];
  uint32_t dst[IPW];                             // byte offset of the copy's 16 rows inside a stage
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    int grp;                                     // 16-row group of the stage
    if (j < A_IPW) {
      grp = wave + 4 * j;
      grp = grp < A_INS ? grp : A_INS - 1;       // same bytes to the same place: harmless
    } else {
      grp = A_INS + wave * W_IPW + (j - A_IPW);
    }
    const int r = grp * 16 + lane / 4;
    const int ch = (lane % 4) ^ ((r >> 1) & 3);
    const bf16_t* base;
    if (r < 2 * BM) {
      int am = m0 + (r < BM ? r : r - BM);
      am = am < M ? am : M - 1;                  // rows past M are copied (clamped) and never stored
      base = (r < BM ? g.a : g.a_lo) + (size_t)am * K;
    } else {
      const int col = r - 2 * BM;
      int wrow;
      const bf16_t* wbase;
      if (EPI == GEMM_SWIGLU_BF16) {             // 16-column groups alternate gate, up
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
      base = wbase + (size_t)wrow * K;
    }
    src[j] = base + (size_t)step_begin * BK + ch * 8;
    dst[j] = grp * 16 * BK * 2;
  }

  f32x4 acc[MT][NF];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NF; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int l16 = lane & 15, kc = lane >> 4;
  const int a_off = swz16(l16, kc);                               // + i * 16 rows; + BM rows: lo
  const int w_off = 2 * BM * BK + swz16(wave * 16 * NF + l16, kc);   // + j * 16 rows
#define SY_COPY(J_, NXT, STEP) glds16_at(src[J_] + (size_t)(STEP) * BK, NXT + dst[J_]);
#define SY_ISSUE(NXT, STEP) _Pragma("unroll") for (int j = 0; j < IPW; ++j) SY_COPY(j, NXT, STEP)
#define SY_MFMA(ACC, FW, FA, I_)                                                                  \
  {                                                                                               \
    if ((I_) * NF < 64) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(FW), "v"(FA)); \
    else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(ACC) : "v"(FW), "v"(FA)); \
  }
// The copies of K step s+2 are spread over the row blocks of step s, one per block (see gemm_tall_kernel).
#define SY_MULT(STAGE, NXT, NSTEP)                                                                \
  {                                                                                               \
    bf16x8 fw[NF];                                                                                \
    _Pragma("unroll") for (int j = 0; j < NF; ++j)                                                \
        fw[j] = *reinterpret_cast<const bf16x8*>(STAGE + w_off + j * 16 * BK);                    \
    bf16x8 fa[MT + 2], fl[MT + 2];                                                                \
    _Pragma("unroll") for (int i = 0; i < 2 && i < MT; ++i) {                                     \
      fa[i] = *reinterpret_cast<const bf16x8*>(STAGE + a_off + i * 16 * BK);                      \
      fl[i] = *reinterpret_cast<const bf16x8*>(STAGE + a_off + (BM + i * 16) * BK);               \
    }                                                                                             \
    _Pragma("unroll") for (int i = 0; i < MT; ++i) {                                              \
      if (i + 2 < MT) {                                                                           \
        fa[i + 2] = *reinterpret_cast<const bf16x8*>(STAGE + a_off + (i + 2) * 16 * BK);          \
        fl[i + 2] = *reinterpret_cast<const bf16x8*>(STAGE + a_off + (BM + (i + 2) * 16) * BK);   \
      }                                                                                           \
      if (i < IPW) SY_COPY(i, NXT, NSTEP)                                                         \
      _Pragma("unroll") for (int j = 0; j < NF; ++j) SY_MFMA(acc[i][j], fw[j], fa[i], i)          \
      _Pragma("unroll") for (int j = 0; j < NF; ++j) SY_MFMA(acc[i][j], fw[j], fl[i], i)          \
    }                                                                                             \
    _Pragma("unroll") for (int j = MT; j < IPW; ++j) SY_COPY(j, NXT, NSTEP)                       \
  }
#define SY_STEP(CUR, NXT, S_, SETTLE)                                                             \
  {                                                                                               \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(IPW) : "memory");                         \
    asm volatile("s_barrier" ::: "memory");                                                       \
    const int nxt_ = (S_) + 2 < n_steps ? (S_) + 2 : n_steps - 1;                                 \
    SY_MULT(CUR, NXT, nxt_)                                                                       \
    if (SETTLE) asm volatile("s_nop 15" ::: "memory");                                            \
  }

  const uint32_t l0 = lds_addr_of(st0), l1 = lds_addr_of(st1), l2 = lds_addr_of(st2);
  SY_ISSUE(l0, 0)
  {
    const int one_ = n_steps > 1 ? 1 : 0;
    SY_ISSUE(l1, one_)
  }
  int s = 0;
  // SETTLE: the last step of every basic block ends with wait states that let its final MFMAs finish.  The
  // compiler does not know that the accumulators are MFMA results (see below) and is free to copy one to
  // another register where control flow joins -- at the loop's back edge and exits -- where it would read
  // a result the matrix core has not written yet.
  for (; s + 3 <= n_steps; s += 3) {
    SY_STEP(st0, l2, s, false)
    SY_STEP(st1, l0, s + 1, false)
    SY_STEP(st2, l1, s + 2, true)
  }
  if (s < n_steps) {
    SY_STEP(st0, l2, s, true)
    if (s + 1 < n_steps) SY_STEP(st1, l0, s + 1, true)
  }
#undef SY_COPY
#undef SY_ISSUE
#undef SY_MFMA
#undef SY_MULT
#undef SY_STEP
  // surplus copies land before the LDS is released; MFMA results settle before they are read (see above)
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NF; ++j) {
      if (i * NF < 64) asm volatile("" : "+a"(acc[i][j]));
      else asm volatile("" : "+v"(acc[i][j]));
    }

  const int nq = kc * 4;                         // this lane's 4 consecutive columns inside a 16-column fragment
  const bool defer = g.deferred && g.split_k > 1;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int m = m0 + i * 16 + l16;
    if (m >= M) continue;
    if (EPI == GEMM_SWIGLU_BF16) {
#pragma unroll
      for (int j = 0; j < NF; j += 2) {
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float gate = acc[i][j][r], up = acc[i][j + 1][r];
          const float v = gate / (1.0f + __expf(-gate)) * up;
          hi[r] = f2bf(v);
          lo[r] = f2bf(v - bf2f(hi[r]));
        }
        const size_t at = (size_t)m * (g.N >> 1) + (n0 >> 1) + (wave * (NF / 2) + (j >> 1)) * 16 + nq;
        *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.c) + at) = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
        *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(g.c_lo) + at) = make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
      }
    } else {
      float* c = (defer ? g.c_parts + (size_t)blockIdx.z * M * g.N : reinterpret_cast<float*>(g.c)) +
                 (size_t)m * g.N + n0 + wave * 16 * NF + nq;
#pragma unroll
      for (int j = 0; j < NF; ++j) {
        if (EPI == GEMM_ADD_F32 && !defer) {
          float4 o = *reinterpret_cast<float4*>(c + j * 16);
          o.x += acc[i][j][0];
          o.y += acc[i][j][1];
          o.z += acc[i][j][2];
          o.w += acc[i][j][3];
          *reinterpret_cast<float4*>(c + j * 16) = o;
        } else {
          *reinterpret_cast<float4*>(c + j * 16) = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
        }
      }
    }
  }
}

template <int MT, int NF = 4>
static hipError_t launch_tall16(const GemmArgs& g, hipStream_t s) {
  constexpr int BM = 16 * MT;
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / (64 * NF);
  const dim3 grid(8 * ((n_tiles + 7) / 8) * m_tiles, 1, g.split_k);
  switch (g.epilogue) {
    case GEMM_STORE_F32: gemm_tall16_kernel<MT, NF, GEMM_STORE_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_ADD_F32: gemm_tall16_kernel<MT, NF, GEMM_ADD_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_SWIGLU_BF16: gemm_tall16_kernel<MT, NF, GEMM_SWIGLU_BF16><<<grid, 256, 0, s>>>(g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// Tile configurations.  N tile 256 halves the weight re-reads from L2 per MFMA; the 128-wide
// one serves outputs whose N is not a multiple of 256 and small problems.
template <int BM, int BN, int BK, int WGM, int WGN, bool SPLIT>
static hipError_t launch_cfg(const GemmArgs& g, hipStream_t s) {
  constexpr int NA = SPLIT ? 2 : 1;
  const size_t lds = (size_t)2 * (NA * BM * BK + BN * BK) * sizeof(bf16_t);
  const int m_tiles = (g.M + BM - 1) / BM, n_tiles = g.N / BN;
  const dim3 grid(8 * ((n_tiles + 7) / 8) * m_tiles, 1, g.split_k);
  const dim3 block(64 * WGM * WGN);
#define SY_LAUNCH(EPI)                                                                                      \
  do {                                                                                                      \
    static bool attr_done = false;                                                                          \
    if (!attr_done) {                                                                                       \
      hipError_t e = hipFuncSetAttribute(                                                                   \
          reinterpret_cast<const void*>(&gemm_kernel<BM, BN, BK, WGM, WGN, SPLIT, EPI>),                    \
          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                                            \
      if (e != hipSuccess) return e;                                                                        \
      attr_done = true;                                                                                     \
    }                                                                                                       \
    gemm_kernel<BM, BN, BK, WGM, WGN, SPLIT, EPI><<<grid, block, lds, s>>>(g);                              \
  } while (0)
  switch (g.epilogue) {
    case GEMM_STORE_F32: SY_LAUNCH(GEMM_STORE_F32); break;
    case GEMM_ADD_F32: SY_LAUNCH(GEMM_ADD_F32); break;
    case GEMM_SWIGLU_BF16: SY_LAUNCH(GEMM_SWIGLU_BF16); break;
    default: return hipErrorInvalidValue;
  }
#undef SY_LAUNCH
  return hipGetLastError();
}

static int g_gemm_variant = -1;   // tuning hook: force a tile configuration (-1 = automatic)
void gemm_force_variant(int v) { g_gemm_variant = v; }

struct Variant { int bm, bn; };
static const Variant kVariants[] = {{128, 128}, {128, 256}, {256, 128}, {256, 256}, {64, 256}, {192, 256}, {256, 256},
                                   {128, 256}, {64, 128}, {128, 128}, {64, 256},
                                   {128, 128}, {128, 256}, {128, 256}, {64, 256},    // 11..: async-copy kernels
                                   {64, 256}, {128, 128}, {64, 128},
                                   {128, 256}, {160, 256}, {192, 256}, {224, 256}, {256, 256}, {288, 256},   // 18..: tall tiles, 32-row blocks
                                   {144, 256}, {176, 256}, {208, 256}, {240, 256}, {272, 256},   // 24..: tall tiles, 16-row blocks
                                   {128, 256}, {160, 256}, {192, 256}, {224, 256}, {256, 256},
                                   {128, 128}, {144, 128}, {160, 128}, {176, 128}, {192, 128}};   // 34..: the same, 128 columns
static const int kFirstTall = 18, kFirstTall16 = 24;
static const int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

static bool variant_fits(const GemmArgs& g, int v) {
  const int bn = kVariants[v].bn;
  if (g.N % bn != 0) return false;
  if (g.epilogue != GEMM_SWIGLU_BF16)
    for (int i = 0; i < 3; ++i)
      if (g.w_rows[i] % bn != 0) return false;
  return true;
}

// Tall-tile plan: the tile (variants kFirstTall.., BM rows) and the K split with the least modelled time.
// Blocks are equal-sized and one runs per compute unit, so a launch takes ceil(blocks / 256) rounds of
//   K steps per block x t_step(BM) us              (fits of MI355X timings at M = 200..1030: 0.12 us plus
//                                                    0.19 us per 32-row block, or 0.0825 us per 16-row block:
//                                                    at equal height the 16-row form is ~13 % faster, the
//                                                    32-row form is the only one that reaches 288 rows;
//                                                    128-column tiles scale the MFMA part by 0.6)
// plus, with K split, the merge of the partial tiles (atomic adds, or stores that the consumer kernel sums).
static double tall_step_us(int v) {
  const int bm = kVariants[v].bm, bn = kVariants[v].bn;
  if (v < kFirstTall16) return 0.12 + 0.19 * (bm / 32);
  // a 128-column tile pays the activation-fragment reads of a 256-column one for half the MFMAs: 0.6x, not 0.5x
  // (M = 532: QKV 64.7 us on 128 x 128 tiles against 58.9 us on 128 x 256 with two K slices)
  const double mfma = 0.12 + 0.0825 * (bm / 16) * (bn == 256 ? 1.0 : 0.6);
  // a short tile is bound by its weight stream instead: BN rows x 64 bytes per K step at the ~24 GB/s one compute
  // unit pulls from HBM (which is why small batches want 128-column tiles: twice the blocks, all CUs streaming)
  const double stream = bn * 64 / 24e3;
  return mfma > stream ? mfma : stream;
}
static int tall_split(const GemmArgs& g, int v) {
  if (g.epilogue == GEMM_SWIGLU_BF16) return 1;
  if (v >= kFirstTall16 && !g.deferred) return 1;   // these tiles split K only into stored slices
  const int bm = kVariants[v].bm;
  const long tiles = (long)((g.M + bm - 1) / bm) * (g.N / kVariants[v].bn);
  long split = 256 / tiles;
  const long most = g.K / 32 / 8;               // at least 8 K steps per slice
  split = split < most ? split : most;
  if (g.deferred && split > SY_MAX_DEFERRED_SPLIT) split = SY_MAX_DEFERRED_SPLIT;
  return split < 1 ? 1 : (int)split;
}
static double tall_cost(const GemmArgs& g, int v, int split) {
  const int bm = kVariants[v].bm;
  const long tiles = (long)((g.M + bm - 1) / bm) * (g.N / kVariants[v].bn);
  const long rounds = (tiles * split + 255) / 256;
  const double steps = (double)(g.K / 32) / split;
  // per K slice and 2.2 M outputs: ~8.5 us of atomic adds, or ~3 us to store the slice and read it back
  const double merge = split > 1 ? (g.deferred ? 3.0 : 8.5) * split * ((double)g.M * g.N / 2.2e6) : 0.0;
  return rounds * steps * tall_step_us(v) + merge;
}
static int pick_tall(const GemmArgs& g, int* split_out) {
  int best = -1, best_split = 1;
  double best_cost = 0.0;
  for (int v = kFirstTall; v < kNumVariants; ++v) {
    if (!variant_fits(g, v)) continue;
    const int tile_split = tall_split(g, v);
    for (int split = 1; split <= tile_split; ++split) {    // fewer slices than fit can win: less to merge
      const double c = tall_cost(g, v, split);
      if (best < 0 || c < best_cost) {
        best = v;
        best_cost = c;
        best_split = split;
      }
    }
  }
  if (split_out) *split_out = best_split;
  return best;
}

static int pick_variant(const GemmArgs& g) {
  if (g_gemm_variant >= 0 && g_gemm_variant < kNumVariants && variant_fits(g, g_gemm_variant) &&
      (g_gemm_variant < 11 || g.a_lo))
    return g_gemm_variant;
  // From the tile sweeps on MI355X.  With (hi, lo) activations: tall tiles from about a hundred rows up
  // (verification batches), the 64-row asynchronous-copy kernel below that (decode steps), 128x128 where N
  // is not a multiple of 256.
  if (g.a_lo) {
    if (g.M > 96) {
      const int v = pick_tall(g, nullptr);
      if (v >= 0) return v;
    }
    if (variant_fits(g, 14)) return 14;
    return 11;
  }
  if (g.M >= 768 && variant_fits(g, 7)) return 7;
  if (g.M > 128) return 9;
  return 8;
}

bool gemm_uses_tall_tiles(const GemmArgs& g) { return pick_variant(g) >= kFirstTall; }

void gemm_plan(const GemmArgs& g, int* bm, int* bn, int* split) {   // host only: what launch_gemm would run
  const int v = pick_variant(g);
  *bm = kVariants[v].bm;
  *bn = kVariants[v].bn;
  *split = gemm_pick_split(g);
}

int gemm_pick_split(const GemmArgs& g) {
  if (g.epilogue == GEMM_SWIGLU_BF16) return 1;
  const int vi = pick_variant(g);
  if (vi >= kFirstTall) {
    int split = 1;
    if (g_gemm_variant >= 0) return tall_split(g, vi);   // forced tile: as many slices as fit
    pick_tall(g, &split);
    return split;
  }
  const Variant v = kVariants[vi];
  const long tiles = (long)((g.M + v.bm - 1) / v.bm) * (g.N / v.bn);
  // Enough blocks to cover the 256 compute units about twice; K slices stay >= 512.
  int split = 1;
  while (tiles * split < 512 && g.K % (split * 2 * 64) == 0 && g.K / (split * 2) >= 512) split *= 2;
  return split;
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0) return hipSuccess;
  const int v = pick_variant(g);
  if (!variant_fits(g, v) || g.K % 64 != 0 || g.split_k < 1) return hipErrorInvalidValue;
  if (v >= kFirstTall ? g.split_k > g.K / 32 : g.K % (g.split_k * 64) != 0) return hipErrorInvalidValue;
  if (v >= 11 && !g.a_lo) return hipErrorInvalidValue;
  if (v >= kFirstTall16 && g.split_k > 1 && !g.deferred) return hipErrorInvalidValue;
  if (g.deferred && g.split_k > 1 &&
      (v < kFirstTall || !g.c_parts || g.split_k > SY_MAX_DEFERRED_SPLIT || g.epilogue == GEMM_SWIGLU_BF16))
    return hipErrorInvalidValue;
  if (g.epilogue == GEMM_SWIGLU_BF16) {
    if (g.split_k != 1 || !g.c_lo) return hipErrorInvalidValue;
  } else {
    long rows = 0;
    for (int i = 0; i < 3; ++i) rows += g.w_rows[i];
    if (rows != g.N) return hipErrorInvalidValue;
  }
  const bool split = g.a_lo != nullptr;
#define SY_VARIANT(BM_, BN_, BK_, WGM_, WGN_) \
  return split ? launch_cfg<BM_, BN_, BK_, WGM_, WGN_, true>(g, s) : launch_cfg<BM_, BN_, BK_, WGM_, WGN_, false>(g, s)
  switch (v) {
    case 0: SY_VARIANT(128, 128, 64, 2, 2);
    case 1: SY_VARIANT(128, 256, 32, 2, 2);
    case 2: SY_VARIANT(256, 128, 32, 2, 2);
    case 3: SY_VARIANT(256, 256, 32, 2, 4);
    case 4: SY_VARIANT(64, 256, 32, 1, 4);
    case 5: SY_VARIANT(192, 256, 32, 2, 2);
    case 6: SY_VARIANT(256, 256, 32, 2, 2);
    case 7: SY_VARIANT(128, 256, 32, 2, 4);
    case 8: SY_VARIANT(64, 128, 32, 1, 2);
    case 9: SY_VARIANT(128, 128, 32, 2, 2);
    case 10: SY_VARIANT(64, 256, 64, 1, 4);
    case 11: return launch_dma<128, 128, 32, 2, 2>(g, s);
    case 12: return launch_dma<128, 256, 32, 2, 2>(g, s);
    case 13: return launch_dma<128, 256, 32, 2, 4>(g, s);
    case 14: return launch_dma<64, 256, 32, 1, 4>(g, s);
    case 15: return launch_dma<64, 256, 64, 1, 4>(g, s);
    case 16: return launch_dma<128, 128, 64, 2, 2>(g, s);
    case 17: return launch_dma<64, 128, 64, 2, 2>(g, s);
    case 18: return launch_tall<4>(g, s);
    case 19: return launch_tall<5>(g, s);
    case 20: return launch_tall<6>(g, s);
    case 21: return launch_tall<7>(g, s);
    case 22: return launch_tall<8>(g, s);
    case 23: return launch_tall<9>(g, s);
    case 24: return launch_tall16<9>(g, s);
    case 25: return launch_tall16<11>(g, s);
    case 26: return launch_tall16<13>(g, s);
    case 27: return launch_tall16<15>(g, s);
    case 28: return launch_tall16<17>(g, s);
    case 29: return launch_tall16<8>(g, s);
    case 30: return launch_tall16<10>(g, s);
    case 31: return launch_tall16<12>(g, s);
    case 32: return launch_tall16<14>(g, s);
    case 33: return launch_tall16<16>(g, s);
    case 34: return launch_tall16<8, 2>(g, s);
    case 35: return launch_tall16<9, 2>(g, s);
    case 36: return launch_tall16<10, 2>(g, s);
    case 37: return launch_tall16<11, 2>(g, s);
    case 38: return launch_tall16<12, 2>(g, s);
    default: return hipErrorInvalidValue;
  }
#undef SY_VARIANT
}
