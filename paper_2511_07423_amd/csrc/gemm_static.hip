// synera_gemm_pair_static: the projection GEMM for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  It is synera_debug_gemm_slices with
// the workspace taken from a static device array instead of a caller buffer, followed by the in-order sum of the
// K slices: the same kernels, the same slices, no hipMalloc / hipFree and no allocating library call.
//
// The array is one per GPU the library runs on (each device holds its own copy at its own address, until the
// process ends).  Host code never passes the array's name to a kernel: the device address is looked up once per
// device with hipGetSymbolAddress, with that device current, and kept.  Every call on a GPU shares that GPU's
// array: calls that overlap on one GPU (two streams, two threads) race on it.  Nothing in it has to start at
// zero: every slice entry a call reads was written by that call's own GEMM launch before.
#include "../../include/synera_debug.h"
#include "common.h"

#define SY_STATIC_FLOATS ((size_t)SYNERA_MAX_GEMM_SLICES * SYNERA_STATIC_GEMM_MAX_OUT)
static __device__ __align__(256) float scratch[SY_STATIC_FLOATS];

#define SY_MAX_DEVICES 64
static float* g_scratch_ptr[SY_MAX_DEVICES];   // device address of `scratch` per device, nullptr until looked up

// out[i] = parts[0][i] + parts[1][i] + ... in that order (what the decoder's consumer kernels do with the slices)
__global__ void sum_slices_kernel(const float* __restrict__ parts, int n_parts, size_t stride, float* __restrict__ out,
                                  size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += step) {
    float4 v = reinterpret_cast<const float4*>(parts)[i];
    for (int s = 1; s < n_parts; ++s) {
      const float4 p = reinterpret_cast<const float4*>(parts + (size_t)s * stride)[i];
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    reinterpret_cast<float4*>(out)[i] = v;
  }
}

extern "C" int32_t synera_gemm_pair_static(const void* d_a, const void* d_a_lo, const void* d_w, float* d_c, int32_t M,
                                           int32_t N, int32_t K, void* stream_) {
  if (!d_a || !d_a_lo || !d_w || !d_c || M < 1 || N < 1 || K < 1) return SYNERA_EINVAL;
  if (N % 128 != 0 || K % 64 != 0) return SYNERA_EUNSUP;
  if ((int64_t)M * N > SYNERA_STATIC_GEMM_MAX_OUT) return SYNERA_ENOSPC;   // beyond what the static workspace holds
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SY_MAX_DEVICES) {
    (void)hipGetLastError();
    return SYNERA_EHIP;
  }
  if (!g_scratch_ptr[dev]) {                    // first call on this device (current): its copy of the array
    float* p = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return SYNERA_EHIP;
    }
    g_scratch_ptr[dev] = p;
  }
  float* parts = g_scratch_ptr[dev];
  hipStream_t s = static_cast<hipStream_t>(stream_);
  GemmArgs g{};
  g.a = static_cast<const uint16_t*>(d_a);
  g.a_lo = static_cast<const uint16_t*>(d_a_lo);
  g.w[0] = static_cast<const bf16_t*>(d_w);
  g.w_rows[0] = N;
  g.c = parts;                                  // not written when K is split; slice 0 otherwise
  g.M = M;
  g.N = N;
  g.K = K;
  g.epilogue = GEMM_STORE_F32;
  g.split_k = 1;
  g.c_parts = parts;
  g.out_scale = 1.0f / (float)(1 << SY_W_SHIFT);
  g.c_scale = 1.0f;
  g.split_k = gemm_pick_split(g);               // <= SYNERA_MAX_GEMM_SLICES
  if (launch_gemm(g, s) != hipSuccess) {
    (void)hipGetLastError();
    return SYNERA_EHIP;
  }
  const size_t n = (size_t)M * N;               // a multiple of 4 (N % 128 == 0)
  int blocks = (int)((n / 4 + 255) / 256);
  blocks = blocks > 2048 ? 2048 : blocks;
  sum_slices_kernel<<<blocks, 256, 0, s>>>(parts, g.split_k, n, d_c, n / 4);
  if (hipGetLastError() != hipSuccess) return SYNERA_EHIP;
  return SYNERA_OK;
}
