// What the chip gives, measured beside the kernels it bounds: a plain device copy and a read-only stream for
// the HBM rate, and a register-resident MFMA loop for the matrix-core rate.  Neither is part of the verification path; the
// measurement tools launch them in the same process as the kernels they compare with, because the
// sustained matrix-core rate depends on the operands (the clock drops under the switching activity of
// random mantissas) and differs from box to box.
#include "../../include/synera_debug.h"
#include "common.h"

// Both streams split the `n16` 16-byte pieces into one contiguous segment of `seg` pieces per block; lane t
// of block b takes pieces b * seg + t + 256 j and keeps four loads in flight.
__global__ __launch_bounds__(256) void ceiling_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16,
                                                           size_t seg) {
  const size_t begin = (size_t)blockIdx.x * seg;
  const size_t end = begin + seg < n16 ? begin + seg : n16;
  size_t i = begin + threadIdx.x;
  for (; i + 768 < end; i += 1024) {
    const uint4 v0 = src[i], v1 = src[i + 256], v2 = src[i + 512], v3 = src[i + 768];
    dst[i] = v0;
    dst[i + 256] = v1;
    dst[i + 512] = v2;
    dst[i + 768] = v3;
  }
  for (; i < end; i += 256) dst[i] = src[i];
}

// Read-only: every lane folds the pieces it reads into one word and stores it (so no load can be dropped):
// out[b * 256 + t] = xor of all 32-bit words of the lane's pieces.
__global__ __launch_bounds__(256) void ceiling_read_kernel(uint32_t* __restrict__ out, const uint4* __restrict__ src, size_t n16,
                                                           size_t seg) {
  const size_t begin = (size_t)blockIdx.x * seg;
  const size_t end = begin + seg < n16 ? begin + seg : n16;
  size_t i = begin + threadIdx.x;
  uint4 acc = {0u, 0u, 0u, 0u};
  for (; i + 768 < end; i += 1024) {
    const uint4 v0 = src[i], v1 = src[i + 256], v2 = src[i + 512], v3 = src[i + 768];
    acc.x ^= v0.x ^ v1.x ^ v2.x ^ v3.x;
    acc.y ^= v0.y ^ v1.y ^ v2.y ^ v3.y;
    acc.z ^= v0.z ^ v1.z ^ v2.z ^ v3.z;
    acc.w ^= v0.w ^ v1.w ^ v2.w ^ v3.w;
  }
  for (; i < end; i += 256) {
    const uint4 v = src[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

__device__ __forceinline__ uint32_t ceiling_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}
// Two bf16 values with random signs and mantissas and exponents within a few steps of 2^-1 .. 2^0
// (finite, so the accumulators stay finite over any loop length the entry point admits).
__device__ __forceinline__ uint32_t ceiling_random_bf2(uint32_t seed) {
  const uint32_t h = ceiling_hash(seed);
  return (0x3f003f00u + (h & 0x007f007fu)) ^ (h & 0x80008000u);
}

// Four wavefronts per block, each issuing `iters` x 16 v_mfma_f32_32x32x16_bf16 on operands that never
// leave registers: 8 A fragments, 4 B fragments, 4 independent accumulators (an accumulator is reused
// every fourth MFMA, past the instruction's 8 passes).  RANDOM = false: every operand element 1.0 / 2^-7.
template <bool RANDOM>
__global__ __launch_bounds__(256) void ceiling_mfma_kernel(float* __restrict__ out, int iters) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  bf16x8 a[8], b[4];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    u32x4 v;
    for (int i = 0; i < 4; ++i) v[i] = RANDOM ? ceiling_random_bf2(threadIdx.x * 131 + q * 17 + i + blockIdx.x * 7919) : 0x3f803f80u;
    a[q] = __builtin_bit_cast(bf16x8, v);
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    u32x4 v;
    for (int i = 0; i < 4; ++i) v[i] = RANDOM ? ceiling_random_bf2(threadIdx.x * 257 + q * 29 + i + 99991) : 0x3c003c00u;
    b[q] = __builtin_bit_cast(bf16x8, v);
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 16; ++n) acc[n % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[n & 7], b[n & 3], acc[n % 4], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s += acc[i][0];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// The same loop on the instruction the projection kernel issues, v_mfma_f32_16x16x32_f16 (4 passes): 8 A fragments,
// 4 B fragments, 8 independent accumulators (one is reused every eighth MFMA).  Inline assembly with the
// accumulator tied to its register, as in the projection kernel: through the builtin the compiler moves the
// accumulators between registers in every iteration and the loop measures those moves.  The build checks the
// generated assembly for accumulator accesses that come too early (mfma_hazards.py).
// RANDOM: fp16 values with random signs and mantissas in [0.5, 1); else 1.0 against 2^-7.
template <bool RANDOM>
__global__ __launch_bounds__(256) void ceiling_mfma_f16_kernel(float* __restrict__ out, int iters) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  u32x4 a[8], b[4];
#pragma unroll
  for (int q = 0; q < 8; ++q)
    for (int i = 0; i < 4; ++i) {
      const uint32_t h = ceiling_hash(threadIdx.x * 131 + q * 17 + i + blockIdx.x * 7919);
      a[q][i] = RANDOM ? ((0x38003800u + (h & 0x03ff03ffu)) ^ (h & 0x80008000u)) : 0x3c003c00u;
    }
#pragma unroll
  for (int q = 0; q < 4; ++q)
    for (int i = 0; i < 4; ++i) {
      const uint32_t h = ceiling_hash(threadIdx.x * 257 + q * 29 + i + 99991);
      b[q][i] = RANDOM ? ((0x38003800u + (h & 0x03ff03ffu)) ^ (h & 0x80008000u)) : 0x20002000u;
    }
  f32x4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 32; ++n)
      asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[n % 8]) : "v"(a[n & 7]), "v"(b[(n >> 3) & 3]));
    asm volatile("s_nop 7" ::: "memory");          // the back edge: the last MFMAs settle before anything may move
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
  for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(acc[i]));
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

extern "C" int32_t synera_measure_hbm_copy(void* d_dst, const void* d_src, int64_t bytes, void* stream) {
  if (!d_dst || !d_src || bytes < 16 || bytes % 16 != 0) return SYNERA_EINVAL;
  if (((uintptr_t)d_dst | (uintptr_t)d_src) % 16 != 0) return SYNERA_EINVAL;
  const size_t n16 = (size_t)bytes / 16;
  const size_t seg = (n16 + SYNERA_MEASURE_READ_BLOCKS - 1) / SYNERA_MEASURE_READ_BLOCKS;
  ceiling_copy_kernel<<<SYNERA_MEASURE_READ_BLOCKS, 256, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<uint4*>(d_dst), static_cast<const uint4*>(d_src), n16, seg);
  return hipGetLastError() == hipSuccess ? SYNERA_OK : SYNERA_EHIP;
}

extern "C" int32_t synera_measure_hbm_read(uint32_t* d_out, const void* d_src, int64_t bytes, void* stream) {
  if (!d_out || !d_src || bytes < 16 || bytes % 16 != 0 || (uintptr_t)d_src % 16 != 0) return SYNERA_EINVAL;
  const size_t n16 = (size_t)bytes / 16;
  const size_t seg = (n16 + SYNERA_MEASURE_READ_BLOCKS - 1) / SYNERA_MEASURE_READ_BLOCKS;
  ceiling_read_kernel<<<SYNERA_MEASURE_READ_BLOCKS, 256, 0, static_cast<hipStream_t>(stream)>>>(
      d_out, static_cast<const uint4*>(d_src), n16, seg);
  return hipGetLastError() == hipSuccess ? SYNERA_OK : SYNERA_EHIP;
}

extern "C" int32_t synera_measure_mfma_bf16(float* d_out, int32_t blocks, int32_t iters, int32_t random_operands,
                                            int64_t* h_flops, void* stream) {
  if (!d_out || blocks < 1 || blocks > 4096 || iters < 1 || iters > 200000) return SYNERA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (random_operands) ceiling_mfma_kernel<true><<<blocks, 256, 0, s>>>(d_out, iters);
  else ceiling_mfma_kernel<false><<<blocks, 256, 0, s>>>(d_out, iters);
  if (h_flops) *h_flops = (int64_t)blocks * 4 * iters * 16 * (2LL * 32 * 32 * 16);
  return hipGetLastError() == hipSuccess ? SYNERA_OK : SYNERA_EHIP;
}

extern "C" int32_t synera_measure_mfma_f16(float* d_out, int32_t blocks, int32_t iters, int32_t random_operands,
                                           int64_t* h_flops, void* stream) {
  if (!d_out || blocks < 1 || blocks > 4096 || iters < 1 || iters > 200000) return SYNERA_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (random_operands) ceiling_mfma_f16_kernel<true><<<blocks, 256, 0, s>>>(d_out, iters);
  else ceiling_mfma_f16_kernel<false><<<blocks, 256, 0, s>>>(d_out, iters);
  if (h_flops) *h_flops = (int64_t)blocks * 4 * iters * 32 * (2LL * 16 * 16 * 32);
  return hipGetLastError() == hipSuccess ? SYNERA_OK : SYNERA_EHIP;
}
