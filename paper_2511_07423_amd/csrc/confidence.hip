// Fused vocabulary-wide reduction: per logits row the argmax (lowest id on ties),
// its softmax probability (the confidence score, Section 3.2 of the paper) and the
// entropy in nats, in ONE pass over the row.
//
// Each thread keeps an online state (m, Z, S, id) over the elements it has seen:
//   m = running max, Z = sum e^(x-m), S = sum e^(x-m) (x-m), id = lowest index with x == m.
// A larger max rescales (Z, S) once per 16-byte chunk at most.  States combine
// associatively, first inside a wavefront by lane shuffles, then across the four
// wavefronts of the block through LDS.  At the end p_top1 = 1/Z and
// H = ln Z - S/Z.  HBM-bound: rows*vocab*sizeof(elem) bytes are read exactly once.
#include "common.h"

#define LOG2E 1.4426950408889634f
#define LN2 0.6931471805599453f

struct ConfState {
  float m, Z, S;
  int id;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Fold state b into a.
__device__ __forceinline__ void conf_merge(ConfState& a, const ConfState& b) {
  const float M = fmaxf(a.m, b.m);
  const float da = a.m - M, db = b.m - M;               // <= 0, finite (m starts at -1e30)
  const float ea = fast_exp2(da * LOG2E), eb = fast_exp2(db * LOG2E);
  const float S = ea * (a.S + a.Z * da) + eb * (b.S + b.Z * db);
  const float Z = ea * a.Z + eb * b.Z;
  int id = a.id;
  if (b.m > a.m || (b.m == a.m && b.id < a.id)) id = b.id;
  a.m = M; a.Z = Z; a.S = S; a.id = id;
}

template <int N>
__device__ __forceinline__ void conf_chunk(ConfState& st, const float (&v)[N], int base) {
  float cmax = v[0];
#pragma unroll
  for (int i = 1; i < N; ++i) cmax = fmaxf(cmax, v[i]);
  if (cmax > st.m) {                                       // rare after the first few chunks
    const float dm = st.m - cmax;
    const float sc = fast_exp2(dm * LOG2E);
    st.S = sc * (st.S + st.Z * dm);
    st.Z *= sc;
    st.m = cmax;
    int at = N - 1;
#pragma unroll
    for (int i = N - 2; i >= 0; --i) at = (v[i] == cmax) ? i : at;
    st.id = base + at;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float t = v[i] - st.m;
    const float e = fast_exp2(t * LOG2E);
    st.Z += e;
    st.S = fmaf(e, t, st.S);
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void confidence_kernel(const void* __restrict__ logits, int64_t vocab,
                                                         int64_t stride, int32_t* __restrict__ ids,
                                                         float* __restrict__ p1, float* __restrict__ H) {
  constexpr int VEC = BF16 ? 8 : 4;                        // elements per 16-byte load
  const int64_t row = blockIdx.x;
  const char* base = reinterpret_cast<const char*>(logits) + row * stride * (BF16 ? 2 : 4);
  const uint4* src = reinterpret_cast<const uint4*>(base);
  const int n_vec = (int)(vocab / VEC);
  // id starts at 0: a row without any finite entry (all NaN) then reports token 0, never an id
  // outside the vocabulary.
  ConfState st = {-1e30f, 0.f, 0.f, 0};

  auto consume = [&](const uint4& raw, int c) {
    float v[VEC];
    if constexpr (BF16) {
      v[0] = bf2f(raw.x & 0xFFFF); v[1] = bf2f(raw.x >> 16);
      v[2] = bf2f(raw.y & 0xFFFF); v[3] = bf2f(raw.y >> 16);
      v[4] = bf2f(raw.z & 0xFFFF); v[5] = bf2f(raw.z >> 16);
      v[6] = bf2f(raw.w & 0xFFFF); v[7] = bf2f(raw.w >> 16);
    } else {
      v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
      v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
    }
    conf_chunk<VEC>(st, v, c * VEC);
  };

  int c = threadIdx.x;
  for (; c + 3 * 256 < n_vec; c += 4 * 256) {              // four 16-byte loads in flight per thread
    const uint4 r0 = src[c], r1 = src[c + 256], r2 = src[c + 512], r3 = src[c + 768];
    consume(r0, c); consume(r1, c + 256); consume(r2, c + 512); consume(r3, c + 768);
  }
  for (; c < n_vec; c += 256) consume(src[c], c);
  // ragged tail (vocab not a multiple of the vector width): one element per thread
  for (int64_t e = (int64_t)n_vec * VEC + threadIdx.x; e < vocab; e += 256) {
    float v[1];
    v[0] = BF16 ? bf2f(reinterpret_cast<const bf16_t*>(base)[e]) : reinterpret_cast<const float*>(base)[e];
    conf_chunk<1>(st, v, (int)e);
  }

  for (int o = 1; o < 64; o <<= 1) {
    ConfState other;
    other.m = __shfl_xor(st.m, o);
    other.Z = __shfl_xor(st.Z, o);
    other.S = __shfl_xor(st.S, o);
    other.id = __shfl_xor(st.id, o);
    conf_merge(st, other);
  }
  __shared__ ConfState red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = st;
  __syncthreads();
  if (threadIdx.x == 0) {
    ConfState a = red[0];
    conf_merge(a, red[1]);
    conf_merge(a, red[2]);
    conf_merge(a, red[3]);
    ids[row] = a.id;
    if (p1) p1[row] = 1.0f / a.Z;
    if (H) H[row] = logf(a.Z) - a.S / a.Z;
  }
}

hipError_t launch_confidence(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride,
                             int32_t* ids, float* p1, float* H, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == 1)
    confidence_kernel<true><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, ids, p1, H);
  else
    confidence_kernel<false><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, ids, p1, H);
  return hipGetLastError();
}
