// bf16 matrix-core GEMM for the decoder's projections: C[M][N] = A[M][K] * W[N][K]^T
// with fp32 accumulation (v_mfma_f32_32x32x16_bf16).  Both operands are K-major, so
// an MFMA operand fragment (8 consecutive k of one row) is one 16-byte read.
//
// Tiling: a 256-thread block (4 wavefronts, 2x2) owns a BM x BN = 128 x 128 output
// tile; each wavefront a 64 x 64 sub-tile (2x2 MFMA blocks, 64 fp32 accumulators per
// lane).  K advances in steps of 64 through double-buffered LDS tiles whose 16-byte
// chunks are XOR-swizzled by row so fragment reads are bank-conflict free.  Global
// loads of step i+1 are issued before the MFMAs of step i.
//
// The weight may be given as up to three row segments (Wq | Wk | Wv share one
// launch).  Epilogues: store fp32; add into fp32 (residual stream); SwiGLU, where the
// tile's even 32-column blocks come from W_gate and the odd ones from W_up at the same
// rows, so one lane holds gate and up of the same output and writes
// silu(gate) * up as bf16.  split_k > 1 spreads K over blockIdx.z and adds the
// partial sums with hardware fp32 atomics (the order of those adds is not fixed).
#include "common.h"

#define BM 128
#define BN 128
#define BK 64

__device__ __forceinline__ int swz(int row, int chunk) { return row * BK + ((chunk ^ (row & 7)) << 3); }

template <int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][BM * BK];
  __shared__ __attribute__((aligned(16))) bf16_t sB[2][BN * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int K = g.K, M = g.M;
  const int k_per = K / g.split_k;                 // multiple of BK (checked by the launcher)
  const int k_begin = blockIdx.z * k_per;
  const int n_steps = k_per / BK;

  // Each thread moves four 16-byte chunks of A and four of B per K step.
  const bf16_t* a_src[4];
  const bf16_t* b_src[4];
  int lds_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int id = tid + i * 256, row = id >> 3, ch = id & 7;
    int am = m0 + row;
    am = am < M ? am : M - 1;                      // rows past M are loaded (clamped) and never stored
    a_src[i] = g.a + (size_t)am * K + k_begin + ch * 8;
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
    lds_off[i] = swz(row, ch);
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *reinterpret_cast<const uint4*>(a_src[i]);
    rb[i] = *reinterpret_cast<const uint4*>(b_src[i]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *reinterpret_cast<uint4*>(&sA[0][lds_off[i]]) = ra[i];
    *reinterpret_cast<uint4*>(&sB[0][lds_off[i]]) = rb[i];
  }
  __syncthreads();

  const int l32 = lane & 31, kb = lane >> 5;
  for (int step = 0; step < n_steps; ++step) {
    const int buf = step & 1;
    if (step + 1 < n_steps) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const uint4*>(a_src[i] + (size_t)(step + 1) * BK);
        rb[i] = *reinterpret_cast<const uint4*>(b_src[i] + (size_t)(step + 1) * BK);
      }
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ar = wm * 64 + i * 32 + l32;
        fa[i] = *reinterpret_cast<const bf16x8*>(&sA[buf][swz(ar, ks * 2 + kb)]);
        const int br = wn * 64 + i * 32 + l32;
        fb[i] = *reinterpret_cast<const bf16x8*>(&sB[buf][swz(br, ks * 2 + kb)]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (step + 1 < n_steps) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<uint4*>(&sA[buf ^ 1][lds_off[i]]) = ra[i];
        *reinterpret_cast<uint4*>(&sB[buf ^ 1][lds_off[i]]) = rb[i];
      }
    }
    __syncthreads();
  }

  // Epilogue.  A 32x32 accumulator block leaves lane (l32, kb) with column l32 and rows
  // 8*(r/4) + 4*kb + r%4, r = 0..15.
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * kb + (r & 3);
      if (m >= M) continue;
      if (EPI == GEMM_SWIGLU_BF16) {
        const float gate = acc[i][0][r], up = acc[i][1][r];
        const float v = gate / (1.0f + __expf(-gate)) * up;
        bf16_t* c = reinterpret_cast<bf16_t*>(g.c);
        c[(size_t)m * (g.N >> 1) + (n0 >> 1) + wn * 32 + l32] = (bf16_t)f2bf(v);
      } else {
        float* c = reinterpret_cast<float*>(g.c) + (size_t)m * g.N + n0 + wn * 64 + l32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
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

int gemm_pick_split(int M, int N, int K) {
  // Enough blocks to cover the 256 compute units about twice; K slices stay >= 512.
  const long tiles = (long)((M + BM - 1) / BM) * (N / BN);
  int split = 1;
  while (tiles * split < 512 && K % (split * 2 * BK) == 0 && K / (split * 2) >= 512) split *= 2;
  return split;
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0) return hipSuccess;
  if (g.N % BN != 0 || g.K % BK != 0 || g.split_k < 1 || g.K % (g.split_k * BK) != 0) return hipErrorInvalidValue;
  if (g.epilogue == GEMM_SWIGLU_BF16) {
    if (g.split_k != 1) return hipErrorInvalidValue;
  } else {
    long rows = 0;
    for (int i = 0; i < 3; ++i) {
      if (g.w_rows[i] % BN != 0) return hipErrorInvalidValue;
      rows += g.w_rows[i];
    }
    if (rows != g.N) return hipErrorInvalidValue;
  }
  const dim3 grid(g.N / BN, (g.M + BM - 1) / BM, g.split_k);
  switch (g.epilogue) {
    case GEMM_STORE_F32: gemm_kernel<GEMM_STORE_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_ADD_F32: gemm_kernel<GEMM_ADD_F32><<<grid, 256, 0, s>>>(g); break;
    case GEMM_SWIGLU_BF16: gemm_kernel<GEMM_SWIGLU_BF16><<<grid, 256, 0, s>>>(g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
