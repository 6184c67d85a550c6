// Importance scores (Section 3.2): column-wise sums of the attention matrix softmax(Q K^T / sqrt(h)).
//
// For request i with chunk rows r = 0 .. c_i - 1 at positions L_i + r, key j in 0 .. L_i + c_i - 1:
//   I_j = (1 / Hq) sum over query heads hq, sum over rows r with L_i + r >= j of p_hq(r, j),
//   p_hq(r, j) = 2^(s scale log2e - m) / l,   s = q_hq(r) . k_kh(j),   (m, l) = the row's softmax
// statistics, which the attention kernel of the same layer has already formed and left in row_ml.  So
// one pass over the keys suffices: no second softmax reduction.
//
// A block owns 256 consecutive keys of one request, one per thread.  Per KV head the thread pulls its
// key's row (head_dim bf16, 256 contiguous bytes of the page) into registers as fp32.  The query rows are
// the same for every thread of the block, so they come in through the scalar unit: a small kernel first
// recombines the (hi, lo) pairs to fp32 once per call, and the main kernel reads those rows through the
// constant address space (s_load into SGPRs) and feeds them to the FMAs as scalar operands -- no LDS, no
// barrier, no per-lane address arithmetic.  Rows are walked uniformly; a key inside the chunk simply does
// not add the rows that cannot see it.  A block covers one KV head (the grid's second dimension: with the
// heads in one block the launch had only about one wavefront per SIMD and ran five times longer); the
// Hkv shares of a key are stored side by side in scratch and a second small kernel adds them in head order (no
// atomics: the scores are bit-reproducible).  Each K byte of the layer is read once.  Vector-ALU bound:
// 2 Hq c h FLOP per key, about 5 GFLOP on the headline batch.
#include "common.h"

#define SY_CONST_AS __attribute__((address_space(4)))

__global__ __launch_bounds__(256) void importance_q_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ q_lo,
                                                           float* __restrict__ qf, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  const uint2 h = reinterpret_cast<const uint2*>(q)[i], l = reinterpret_cast<const uint2*>(q_lo)[i];
  float4 v;
  v.x = bf2f(h.x & 0xFFFF) + bf2f(l.x & 0xFFFF);
  v.y = bf2f(h.x >> 16) + bf2f(l.x >> 16);
  v.z = bf2f(h.y & 0xFFFF) + bf2f(l.y & 0xFFFF);
  v.w = bf2f(h.y >> 16) + bf2f(l.y >> 16);
  reinterpret_cast<float4*>(qf)[i] = v;
}

template <int HD>
__global__ __launch_bounds__(256) void importance_kernel(ImportanceLaunch a, int item0, int n_batch, float scale_log2) {
  const SY_CONST_AS int32_t* items = reinterpret_cast<const SY_CONST_AS int32_t*>((uintptr_t)a.items) + 2 * item0;
  const int req = items[2 * blockIdx.x], key0 = items[2 * blockIdx.x + 1];
  const int L = a.ctx_len[req], tok0 = a.cu_tok[req], c = a.cu_tok[req + 1] - tok0;
  const int Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
  const int n_keys = L + c;
  const int key = key0 + (int)threadIdx.x;
  const bool live = key < n_keys;
  const int r_first = live ? max(0, key - L) : c;                      // rows that see this key: r >= key - L
  const int page = live ? a.block_table[(size_t)req * a.max_pages + key / SY_PAGE] : 0;
  const SY_CONST_AS float* qf = reinterpret_cast<const SY_CONST_AS float*>((uintptr_t)a.qf);
  const SY_CONST_AS float* row_ml = reinterpret_cast<const SY_CONST_AS float*>((uintptr_t)a.row_ml);   // (m, l) pairs
  float total = 0.f;
  {
    const int kh = blockIdx.y;                                         // one KV head (G query heads) per block
    float k[HD];
    if (live) {
      const bf16_t* src = a.k_layer + (((size_t)page * Hkv + kh) * SY_PAGE + key % SY_PAGE) * HD;
#pragma unroll
      for (int d = 0; d < HD; d += 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(src + d);
        k[d + 0] = bf2f(v.x & 0xFFFF); k[d + 1] = bf2f(v.x >> 16);
        k[d + 2] = bf2f(v.y & 0xFFFF); k[d + 3] = bf2f(v.y >> 16);
        k[d + 4] = bf2f(v.z & 0xFFFF); k[d + 5] = bf2f(v.z >> 16);
        k[d + 6] = bf2f(v.w & 0xFFFF); k[d + 7] = bf2f(v.w >> 16);
      }
    } else {
#pragma unroll
      for (int d = 0; d < HD; ++d) k[d] = 0.f;
    }
    for (int g = 0; g < G; ++g) {
      const int hq = kh * G + g;
      for (int r = 0; r < c; ++r) {                                    // block-uniform: scalar loads
        const SY_CONST_AS float* qr = qf + ((size_t)(tok0 + r) * Hq + hq) * HD;
        const float ml_m = row_ml[2 * ((size_t)(tok0 + r) * Hq + hq)], ml_l = row_ml[2 * ((size_t)(tok0 + r) * Hq + hq) + 1];
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
        for (int d = 0; d < HD; d += 4) {
          s0 = fmaf(qr[d + 0], k[d + 0], s0);
          s1 = fmaf(qr[d + 1], k[d + 1], s1);
          s2 = fmaf(qr[d + 2], k[d + 2], s2);
          s3 = fmaf(qr[d + 3], k[d + 3], s3);
        }
        const float p = __builtin_amdgcn_exp2f(((s0 + s1) + (s2 + s3)) * scale_log2 - ml_m) / ml_l;
        total += r >= r_first ? p : 0.f;
      }
    }
  }
  // this KV head's share of the block's 256 keys; importance_sum_kernel adds the Hkv shares in head order
  a.parts[((size_t)blockIdx.y * n_batch + blockIdx.x) * 256 + threadIdx.x] = live ? total / (float)Hq : 0.f;
}

// Block = one item (256 keys of a request): score = sum of the Hkv shares, in head order.
__global__ __launch_bounds__(256) void importance_sum_kernel(ImportanceLaunch a, int item0, int n_batch) {
  const int req = a.items[2 * (item0 + blockIdx.x)], key0 = a.items[2 * (item0 + blockIdx.x) + 1];
  const int n_keys = a.ctx_len[req] + a.cu_tok[req + 1] - a.cu_tok[req];
  const int key = key0 + (int)threadIdx.x;
  if (key >= n_keys) return;
  float sum = 0.f;
  for (int kh = 0; kh < a.Hkv; ++kh) sum += a.parts[((size_t)kh * n_batch + blockIdx.x) * 256 + threadIdx.x];
  a.importance[a.cu_keys[req] + key] = sum;
}

hipError_t launch_importance(const ImportanceLaunch& a, hipStream_t s) {
  if (a.n_items <= 0) return hipSuccess;
  if (!a.parts || a.parts_cap < (size_t)a.Hkv * 256) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)a.hd);
  const size_t n4 = (size_t)a.T * a.Hq * a.hd / 4;
  importance_q_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, s>>>(a.q, a.q_lo, a.qf, n4);
  // as many items per pass as the scratch holds shares for (one pass on every workload measured)
  const size_t fit = a.parts_cap / ((size_t)a.Hkv * 256);
  const int per_pass = (int)(fit < (size_t)a.n_items ? fit : (size_t)a.n_items);
  for (int item0 = 0; item0 < a.n_items; item0 += per_pass) {
    const int n_batch = a.n_items - item0 < per_pass ? a.n_items - item0 : per_pass;
    const dim3 grid(n_batch, a.Hkv);
    if (a.hd == 128) importance_kernel<128><<<grid, 256, 0, s>>>(a, item0, n_batch, scale_log2);
    else if (a.hd == 64) importance_kernel<64><<<grid, 256, 0, s>>>(a, item0, n_batch, scale_log2);
    else return hipErrorInvalidValue;
    importance_sum_kernel<<<n_batch, 256, 0, s>>>(a, item0, n_batch);
  }
  return hipGetLastError();
}

// Thread i: mean score of request i's draft positions, and the probability of offloading by importance:
//   0 for i <= i_th / 2, 1 for i > i_th, else 1 / (1 + exp(theta ((i - i_th/2) / (i_th/2) - 1/2))).
__global__ void importance_dispatch_kernel(const float* __restrict__ importance, const int32_t* __restrict__ cu_keys,
                                           const int32_t* __restrict__ ctx_len, const int32_t* __restrict__ n_unc,
                                           const int32_t* __restrict__ cu_draft, int B, float i_th, float theta,
                                           float* __restrict__ mean_imp, float* __restrict__ p_imp) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B) return;
  const int k = cu_draft[i + 1] - cu_draft[i];
  const float* at = importance + cu_keys[i] + ctx_len[i] + n_unc[i];
  float sum = 0.f;
  for (int j = 0; j < k; ++j) sum += at[j];
  const float m = k > 0 ? sum / (float)k : 0.f;
  if (mean_imp) mean_imp[i] = m;
  if (p_imp) {
    const float half = 0.5f * i_th;
    float p;
    if (m <= half) p = 0.f;
    else if (m > i_th) p = 1.f;
    else p = 1.0f / (1.0f + expf(theta * ((m - half) / half - 0.5f)));
    p_imp[i] = p;
  }
}

hipError_t launch_importance_dispatch(const float* importance, const int32_t* cu_keys, const int32_t* ctx_len,
                                      const int32_t* n_unc, const int32_t* cu_draft, int B, float i_th, float theta,
                                      float* mean_imp, float* p_imp, hipStream_t s) {
  if (B <= 0 || (!mean_imp && !p_imp)) return hipSuccess;
  importance_dispatch_kernel<<<(B + 127) / 128, 128, 0, s>>>(importance, cu_keys, ctx_len, n_unc, cu_draft, B, i_th,
                                                             theta, mean_imp, p_imp);
  return hipGetLastError();
}
