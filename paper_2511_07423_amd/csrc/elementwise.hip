// Small HBM-streaming kernels of the verify path: embedding gather, RMSNorm,
// rotary embedding fused with the paged KV append, the standalone KV append, the
// greedy accept-prefix scan, and a zero fill.  All are O(T*d) bytes and far from
// any roofline that matters; they are written for coalesced 16-byte accesses.
#include "common.h"

// ------------------------------------------------------------------ embedding
// x[t][:] = float(E[token[t]][:]).  One block per token.  Token ids live on the device and cannot
// be validated by the host: an id outside [0, vocab) is clamped into the table instead of being
// followed out of bounds.
__global__ __launch_bounds__(256) void embed_kernel(const bf16_t* __restrict__ embed,
                                                    const int32_t* __restrict__ tokens,
                                                    float* __restrict__ x, int d, int vocab) {
  const int t = blockIdx.x;
  int tok = tokens[t];
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const bf16_t* src = embed + (size_t)tok * d;
  float* dst = x + (size_t)t * d;
  for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
    uint4 v = *reinterpret_cast<const uint4*>(src + c);
    float4 lo = {bf2f(v.x & 0xFFFF), bf2f(v.x >> 16), bf2f(v.y & 0xFFFF), bf2f(v.y >> 16)};
    float4 hi = {bf2f(v.z & 0xFFFF), bf2f(v.z >> 16), bf2f(v.w & 0xFFFF), bf2f(v.w >> 16)};
    *reinterpret_cast<float4*>(dst + c) = lo;
    *reinterpret_cast<float4*>(dst + c + 4) = hi;
  }
}

hipError_t launch_embed(const bf16_t* embed, const int32_t* tokens, float* x, int T, int d, int vocab,
                        hipStream_t s) {
  if (T <= 0) return hipSuccess;
  embed_kernel<<<T, 256, 0, s>>>(embed, tokens, x, d, vocab);
  return hipGetLastError();
}

// ------------------------------------------------------------------ RMSNorm
// y = x * rsqrt(mean(x^2) + eps) * g, fp32 in, fp16 (hi, lo) pair of SY_Y_SCALE y out (lo_off: lo = 0).  One block
// per output row; `rows` (optional) selects which input row feeds output row r.
// With n_parts > 0 the row first takes the pending K-split slices of the projection before it,
// x += sum_s parts[s], and the sum is written back to x (each thread re-reads only what it wrote).
__global__ __launch_bounds__(256) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ parts,
                                                      int n_parts, size_t part_stride,
                                                      const bf16_t* __restrict__ gain,
                                                      const int32_t* __restrict__ rows,
                                                      uint16_t* __restrict__ y, uint16_t* __restrict__ y_lo, int d,
                                                      float eps, bool lo_off, bool paired) {
  const int r = blockIdx.x;
  const size_t row_at = (size_t)(rows ? rows[r] : r) * d;
  float* src = x + row_at;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < d; c += 256 * 4) {
    float4 v = *reinterpret_cast<const float4*>(src + c);
    if (n_parts > 0) {
      for (int s = 0; s < n_parts; ++s) {
        const float4 pv = *reinterpret_cast<const float4*>(parts + (size_t)s * part_stride + row_at + c);
        v.x += pv.x; v.y += pv.y; v.z += pv.z; v.w += pv.w;
      }
      *reinterpret_cast<float4*>(src + c) = v;
    }
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps) * SY_Y_SCALE;
  // the pair as two arrays [rows][d], or (paired) as one array [rows][d / 32][hi 32 | lo 32]
  uint16_t* dst = y + (size_t)r * d * (paired ? 2 : 1);
  uint16_t* dst_lo = paired ? dst + 32 : y_lo + (size_t)r * d;
  for (int c = threadIdx.x * 4; c < d; c += 256 * 4) {
    float4 v = *reinterpret_cast<const float4*>(src + c);
    uint2 g = *reinterpret_cast<const uint2*>(gain + c);
    const float o0 = v.x * inv * bf2f(g.x & 0xFFFF), o1 = v.y * inv * bf2f(g.x >> 16);
    const float o2 = v.z * inv * bf2f(g.y & 0xFFFF), o3 = v.w * inv * bf2f(g.y >> 16);
    uint2 hi, lo;
    split_f16x2(o0, o1, hi.x, lo.x);
    split_f16x2(o2, o3, hi.y, lo.y);
    const size_t at = paired ? pair_col(c) : (size_t)c;
    *reinterpret_cast<uint2*>(dst + at) = hi;
    *reinterpret_cast<uint2*>(dst_lo + at) = lo_off ? make_uint2(0u, 0u) : lo;
  }
}

// The same for rows of at most 1024 IT values: the row stays in registers between the two passes (no re-read
// of x), and all loads of a pass are issued before anything is stored, so they are in flight together; the
// pending K slices are taken four at a time for the same reason (a slice per round trip is what a small batch,
// whose projections split K eight ways, otherwise spends its time on).
template <int IT>
__global__ __launch_bounds__(256) void rmsnorm_row_in_registers_kernel(
    float* __restrict__ x, const float* __restrict__ parts, int n_parts, size_t part_stride,
    const bf16_t* __restrict__ gain, const int32_t* __restrict__ rows, uint16_t* __restrict__ y,
    uint16_t* __restrict__ y_lo, int d, float eps, bool lo_off, bool paired) {
  const int r = blockIdx.x;
  const size_t row_at = (size_t)(rows ? rows[r] : r) * d;
  float* src = x + row_at;
  float4 v[IT];
#pragma unroll
  for (int k = 0; k < IT; ++k) {
    const int c = threadIdx.x * 4 + k * 1024;
    v[k] = c < d ? *reinterpret_cast<const float4*>(src + c) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int s = 0; s < n_parts; s += 4) {
    float4 pv[4][IT];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool on = s + u < n_parts;
      const float* ps = parts + (size_t)(on ? s + u : s) * part_stride + row_at;
#pragma unroll
      for (int k = 0; k < IT; ++k) {
        const int c = threadIdx.x * 4 + k * 1024;
        pv[u][k] = on && c < d ? *reinterpret_cast<const float4*>(ps + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)               // slices are added in their order, as before
#pragma unroll
      for (int k = 0; k < IT; ++k) {
        v[k].x += pv[u][k].x; v[k].y += pv[u][k].y; v[k].z += pv[u][k].z; v[k].w += pv[u][k].w;
      }
  }
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < IT; ++k) {
    const int c = threadIdx.x * 4 + k * 1024;
    if (n_parts > 0 && c < d) *reinterpret_cast<float4*>(src + c) = v[k];
    ss += v[k].x * v[k].x + v[k].y * v[k].y + v[k].z * v[k].z + v[k].w * v[k].w;
  }
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps) * SY_Y_SCALE;
  // the pair as two arrays [rows][d], or (paired) as one array [rows][d / 32][hi 32 | lo 32]
  uint16_t* dst = y + (size_t)r * d * (paired ? 2 : 1);
  uint16_t* dst_lo = paired ? dst + 32 : y_lo + (size_t)r * d;
#pragma unroll
  for (int k = 0; k < IT; ++k) {
    const int c = threadIdx.x * 4 + k * 1024;
    if (c >= d) continue;
    const uint2 g = *reinterpret_cast<const uint2*>(gain + c);
    const float o0 = v[k].x * inv * bf2f(g.x & 0xFFFF), o1 = v[k].y * inv * bf2f(g.x >> 16);
    const float o2 = v[k].z * inv * bf2f(g.y & 0xFFFF), o3 = v[k].w * inv * bf2f(g.y >> 16);
    uint2 hi, lo;
    split_f16x2(o0, o1, hi.x, lo.x);
    split_f16x2(o2, o3, hi.y, lo.y);
    const size_t at = paired ? pair_col(c) : (size_t)c;
    *reinterpret_cast<uint2*>(dst + at) = hi;
    *reinterpret_cast<uint2*>(dst_lo + at) = lo_off ? make_uint2(0u, 0u) : lo;
  }
}

hipError_t launch_rmsnorm(float* x, const float* parts, int n_parts, size_t part_stride, const bf16_t* gain,
                          const int32_t* rows, uint16_t* y_hi, uint16_t* y_lo, int n_rows, int d, float eps,
                          bool lo_off, bool paired, hipStream_t s) {
  if (n_rows <= 0) return hipSuccess;
  if (d <= 4096)
    rmsnorm_row_in_registers_kernel<4><<<n_rows, 256, 0, s>>>(x, parts, n_parts, part_stride, gain, rows, y_hi, y_lo, d, eps, lo_off, paired);
  else if (d <= 8192)
    rmsnorm_row_in_registers_kernel<8><<<n_rows, 256, 0, s>>>(x, parts, n_parts, part_stride, gain, rows, y_hi, y_lo, d, eps, lo_off, paired);
  else
    rmsnorm_kernel<<<n_rows, 256, 0, s>>>(x, parts, n_parts, part_stride, gain, rows, y_hi, y_lo, d, eps, lo_off, paired);
  return hipGetLastError();
}

// ------------------------------------------------------------------ rotary table
// cs[t][i] = (cos, sin)(pos_t * base^(-2i/hd)), angle formed in double.
__global__ void rope_table_kernel(BatchMeta m, float2* __restrict__ cs, int T, int half, float base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * half) return;
  const int t = idx / half, i = idx % half;
  const int r = m.tok_req[t];
  const int pos = m.ctx_len[r] + (t - m.cu_tok[r]);
  const double ang = (double)pos * pow((double)base, -(double)i / (double)half);
  double sn, cn;
  sincos(ang, &sn, &cn);
  cs[idx] = make_float2((float)cn, (float)sn);
}

hipError_t launch_rope_table(const BatchMeta& m, float2* cs, int T, int head_dim, float base, hipStream_t s) {
  const int n = T * (head_dim / 2);
  if (n <= 0) return hipSuccess;
  rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(m, cs, T, head_dim / 2, base);
  return hipGetLastError();
}

// ------------------------------------------------------------------ rotary + append
// One block per chunk token.  Input row: fp32 [q heads | k heads | v heads] x hd.
// q and k are rotated on adjacent pairs; q goes to a bf16 (hi, lo) pair [T][Hq][hd]; k and v go to
// the token's page (position t lives in page block_table[t/16], slot t%16):
// K page [kv_head][slot][dim], V page [kv_head][dim][slot].
__global__ __launch_bounds__(256) void rope_append_kernel(const float* __restrict__ qkv, int n_parts,
                                                          size_t part_stride,
                                                          const float2* __restrict__ cs, BatchMeta m,
                                                          bf16_t* __restrict__ q, bf16_t* __restrict__ q_lo,
                                                          bf16_t* __restrict__ k_layer, bf16_t* __restrict__ v_layer,
                                                          int Hq, int Hkv, int hd, bool lo_off) {
  const int t = blockIdx.x;
  const int r = m.tok_req[t];
  const int pos = m.ctx_len[r] + (t - m.cu_tok[r]);
  const int page = m.block_table[(size_t)r * m.max_pages + pos / SY_PAGE];
  const int slot = pos % SY_PAGE;
  const int half = hd / 2;
  const int n_pairs = (Hq + 2 * Hkv) * half;
  const float* row = qkv + (size_t)t * (Hq + 2 * Hkv) * hd;
  // the token's pairs are spread over gridDim.y blocks: few iterations per thread, all loads in flight at once
  for (int p = blockIdx.y * 256 + threadIdx.x; p < n_pairs; p += 256 * gridDim.y) {
    const int head = p / half, i = p % half;
    float2 v = *reinterpret_cast<const float2*>(row + (size_t)head * hd + 2 * i);
#pragma unroll 4
    for (int s = 1; s < n_parts; ++s) {         // the projection arrives as K-split slices: add them
      const float2 pv = *reinterpret_cast<const float2*>(row + (size_t)s * part_stride + (size_t)head * hd + 2 * i);
      v.x += pv.x;
      v.y += pv.y;
    }
    if (head < Hq + Hkv) {
      const float2 c = cs[(size_t)t * half + i];
      const float r0 = v.x * c.x - v.y * c.y;
      const float r1 = v.x * c.y + v.y * c.x;
      if (head < Hq) {
        const uint32_t hi = pack_bf2(r0, r1);
        const size_t at = ((size_t)t * Hq + head) * hd + 2 * i;
        *reinterpret_cast<uint32_t*>(q + at) = hi;
        *reinterpret_cast<uint32_t*>(q_lo + at) = lo_off ? 0u : pack_bf2(r0 - bf2f(hi & 0xFFFF), r1 - bf2f(hi >> 16));
      } else {
        const int kh = head - Hq;
        bf16_t* dst = k_layer + (((size_t)page * Hkv + kh) * SY_PAGE + slot) * hd + 2 * i;
        *reinterpret_cast<uint32_t*>(dst) = pack_bf2(r0, r1);
      }
    } else {
      const int kh = head - Hq - Hkv;
      bf16_t* dst = v_layer + (((size_t)page * Hkv + kh) * hd + 2 * i) * SY_PAGE + slot;
      dst[0] = (bf16_t)f2bf(v.x);
      dst[SY_PAGE] = (bf16_t)f2bf(v.y);
    }
  }
}

hipError_t launch_rope_append(const float* qkv, int n_parts, size_t part_stride, const float2* cs, const BatchMeta& m,
                              bf16_t* q_hi, bf16_t* q_lo, bf16_t* k_layer, bf16_t* v_layer, int T, int Hq, int Hkv,
                              int hd, bool lo_off, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  rope_append_kernel<<<dim3(T, 4), 256, 0, s>>>(qkv, n_parts, part_stride, cs, m, q_hi, q_lo, k_layer, v_layer, Hq, Hkv, hd, lo_off);
  return hipGetLastError();
}

// ------------------------------------------------------------------ standalone append
// Rows are bf16 already; a pure scatter.  The owning request of row t is found by
// binary search in the prefix sums, so any number of rows per request is allowed.
__global__ __launch_bounds__(128) void kv_append_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                        BatchMeta m, int B, bf16_t* __restrict__ k_layer,
                                                        bf16_t* __restrict__ v_layer, int Hkv, int hd) {
  const int t = blockIdx.x;
  int lo = 0, hi = B;                       // find r with cu_tok[r] <= t < cu_tok[r+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (m.cu_tok[mid] <= t) lo = mid; else hi = mid;
  }
  const int r = lo;
  const int pos = m.ctx_len[r] + (t - m.cu_tok[r]);
  const int page = m.block_table[(size_t)r * m.max_pages + pos / SY_PAGE];
  const int slot = pos % SY_PAGE;
  const int n = Hkv * hd;
  const bf16_t* ks = k + (size_t)t * n;
  const bf16_t* vs = v + (size_t)t * n;
  for (int e = threadIdx.x * 2; e < n; e += 128 * 2) {
    const int kh = e / hd, dim = e % hd;
    *reinterpret_cast<uint32_t*>(k_layer + (((size_t)page * Hkv + kh) * SY_PAGE + slot) * hd + dim) =
        *reinterpret_cast<const uint32_t*>(ks + e);
    const uint32_t vv = *reinterpret_cast<const uint32_t*>(vs + e);
    bf16_t* dst = v_layer + (((size_t)page * Hkv + kh) * hd + dim) * SY_PAGE + slot;
    dst[0] = (bf16_t)(vv & 0xFFFF);
    dst[SY_PAGE] = (bf16_t)(vv >> 16);
  }
}

hipError_t launch_kv_append(const bf16_t* k, const bf16_t* v, const BatchMeta& m, int B, bf16_t* k_layer,
                            bf16_t* v_layer, int T, int Hkv, int hd, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  kv_append_kernel<<<T, 128, 0, s>>>(k, v, m, B, k_layer, v_layer, Hkv, hd);
  return hipGetLastError();
}

// ------------------------------------------------------------------ accept-prefix scan
// Thread i < B: a_0 = anchor (or the argmax of the last uncached token's row),
// a_j = argmax of draft j-1's row; n = longest prefix with d_j == a_j; correction
// = a_n.  Threads also copy the per-draft argmax rows to the caller's buffer.
__global__ void accept_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ anchor,
                              const int32_t* __restrict__ lm_argmax, BatchMeta m, int B, int R,
                              int32_t* __restrict__ out_argmax, int32_t* __restrict__ accept_len,
                              int32_t* __restrict__ correction) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < R) out_argmax[i] = lm_argmax[i];
  if (i >= B) return;
  const int u = m.n_unc[i];
  const int r0 = m.cu_draft[i], k = m.cu_draft[i + 1] - r0;
  const int32_t* d = tokens + m.cu_tok[i] + u;
  int32_t a = (u > 0) ? lm_argmax[m.first_row[i]] : anchor[i];
  int n = 0;
  while (n < k && d[n] == a) {
    a = lm_argmax[r0 + n];
    ++n;
  }
  accept_len[i] = n;
  correction[i] = a;
}

hipError_t launch_accept(const int32_t* tokens, const int32_t* anchor, const int32_t* lm_argmax, const BatchMeta& m,
                         int B, int R, int32_t* out_argmax, int32_t* accept_len, int32_t* correction,
                         hipStream_t s) {
  const int n = B > R ? B : R;
  if (n <= 0) return hipSuccess;
  accept_kernel<<<(n + 255) / 256, 256, 0, s>>>(tokens, anchor, lm_argmax, m, B, R, out_argmax, accept_len,
                                               correction);
  return hipGetLastError();
}

__global__ void fill_zero_kernel(float4* __restrict__ p, size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t n4 = n / 4;   // callers pass multiples of 4
  int blocks = (int)((n4 + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  fill_zero_kernel<<<blocks, 256, 0, s>>>(reinterpret_cast<float4*>(p), n4);
  return hipGetLastError();
}
