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
// Entries of -inf (tokens masked out by a top-k / top-p filter, Section 4.5) carry probability 0 and add
// nothing to the entropy; a row needs at least one finite entry.
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
    // bounded below: a masked logit (-inf) has weight e = 0 and must add 0 to S, not 0 * -inf
    const float t = fmaxf(v[i] - st.m, -1e30f);
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

// ---------------------------------------------------------------------------------------------
// The same pass, keeping the k <= 8 most probable tokens of the row as well: the compressed form of a
// distribution that is transmitted instead of the full vector (Section 4.2, "Compression before
// transmission"), and the margin score p_top1 - p_top2 of the layer-wise early exit (Section 4.3).
// Each WAVEFRONT keeps the 8 best (logit, id) it has seen, sorted (equal logits: lower id first), the
// same in all its lanes.  An element is looked at more closely only if it is not below the list's last
// entry: a ballot finds such lanes, their values are broadcast one by one and inserted.  Over a row a
// wavefront meets about 8 ln(n / 8) such elements, so the common path costs one compare and one ballot
// per element.  (Per-thread lists cost ten times more: with 64 lanes in lockstep nearly every 16-byte
// chunk has some lane that must insert.)  After the row the four lists are merged by one thread.
#define TOPK_MAX 8

struct TopEntry {
  float v;
  int id;
};
__device__ __forceinline__ bool top_before(float va, int ia, float vb, int ib) { return va > vb || (va == vb && ia < ib); }

template <bool BF16>
__global__ __launch_bounds__(256) void confidence_topk_kernel(const void* __restrict__ logits, int64_t vocab,
                                                              int64_t stride, int k, int32_t* __restrict__ ids,
                                                              float* __restrict__ probs, float* __restrict__ margin,
                                                              float* __restrict__ H) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int64_t row = blockIdx.x;
  const char* base = reinterpret_cast<const char*>(logits) + row * stride * (BF16 ? 2 : 4);
  const uint4* src = reinterpret_cast<const uint4*>(base);
  const int n_vec = (int)(vocab / VEC);
  ConfState st = {-1e30f, 0.f, 0.f, 0};
  float tv[TOPK_MAX];                                // wavefront-uniform
  int ti[TOPK_MAX];
#pragma unroll
  for (int i = 0; i < TOPK_MAX; ++i) {
    tv[i] = -INFINITY;
    ti[i] = 0x7FFFFFFF;
  }
  // v, id: this lane's element; lanes whose element is not below the list's last entry get a closer look
  auto offer = [&](float v, int id) {
    unsigned long long mask = __builtin_amdgcn_ballot_w64(v >= tv[TOPK_MAX - 1]);
    while (mask) {                                   // wavefront-uniform loop
      const int l = __builtin_ctzll(mask);
      mask &= mask - 1;
      const float cv = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), l));
      const int ci = __builtin_amdgcn_readlane(id, l);
      if (!top_before(cv, ci, tv[TOPK_MAX - 1], ti[TOPK_MAX - 1])) continue;
      tv[TOPK_MAX - 1] = cv;
      ti[TOPK_MAX - 1] = ci;
#pragma unroll
      for (int i = TOPK_MAX - 1; i > 0; --i) {
        if (top_before(tv[i], ti[i], tv[i - 1], ti[i - 1])) {
          const float fv = tv[i]; tv[i] = tv[i - 1]; tv[i - 1] = fv;
          const int fi = ti[i]; ti[i] = ti[i - 1]; ti[i - 1] = fi;
        }
      }
    }
  };
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
    float cmax = v[0];
#pragma unroll
    for (int i = 1; i < VEC; ++i) cmax = fmaxf(cmax, v[i]);
    if (__builtin_amdgcn_ballot_w64(cmax >= tv[TOPK_MAX - 1]) != 0) {   // some lane of the wavefront has a candidate
#pragma unroll
      for (int i = 0; i < VEC; ++i) offer(v[i], c * VEC + i);
    }
    conf_chunk<VEC>(st, v, c * VEC);
  };
  // One 16-byte chunk per lane and round, all lanes of a wavefront in the same round: the lanes that hold
  // data must meet in the same ballot (an unrolled loop whose last trip only some lanes take would split
  // them).  In the last round the lanes past the end of the row just sit out; lane 0 of a wavefront is
  // active whenever any of its lanes is, and its list is the one used.
  for (int c = threadIdx.x; c < n_vec; c += 256) consume(src[c], c);
  {
    const int64_t tail0 = (int64_t)n_vec * VEC;
    const int n_tail = (int)(vocab - tail0);         // < VEC
    if (n_tail > 0) {                                // block-uniform
      const int e = threadIdx.x;
      float v[1] = {-INFINITY};
      if (e < n_tail)
        v[0] = BF16 ? bf2f(reinterpret_cast<const bf16_t*>(base)[tail0 + e]) : reinterpret_cast<const float*>(base)[tail0 + e];
      offer(e < n_tail ? v[0] : -INFINITY, e < n_tail ? (int)(tail0 + e) : 0x7FFFFFFF);
      if (e < n_tail) conf_chunk<1>(st, v, (int)(tail0 + e));
    }
  }

  // row statistics (m, Z, S)
  for (int o = 1; o < 64; o <<= 1) {
    ConfState other;
    other.m = __shfl_xor(st.m, o);
    other.Z = __shfl_xor(st.Z, o);
    other.S = __shfl_xor(st.S, o);
    other.id = __shfl_xor(st.id, o);
    conf_merge(st, other);
  }
  __shared__ ConfState red[4];
  __shared__ TopEntry cand[4][TOPK_MAX];
  if ((threadIdx.x & 63) == 0) {
    red[threadIdx.x >> 6] = st;
#pragma unroll
    for (int i = 0; i < TOPK_MAX; ++i) cand[threadIdx.x >> 6][i] = TopEntry{tv[i], ti[i]};
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ConfState a = red[0];
    conf_merge(a, red[1]);
    conf_merge(a, red[2]);
    conf_merge(a, red[3]);
    if (H) H[row] = logf(a.Z) - a.S / a.Z;
    // merge the four sorted lists: k rounds of "best head"
    int head[4] = {0, 0, 0, 0};
    float p_first = 0.f, p_second = 0.f;
    const int rounds = k > 2 ? k : 2;                // the margin needs the two best whatever k is
    for (int r = 0; r < rounds; ++r) {
      int best = -1;
      for (int w = 0; w < 4; ++w) {
        if (head[w] >= TOPK_MAX) continue;
        const TopEntry e = cand[w][head[w]];
        if (best < 0 || top_before(e.v, e.id, cand[best][head[best]].v, cand[best][head[best]].id)) best = w;
      }
      const TopEntry wn = best >= 0 ? cand[best][head[best]] : TopEntry{-INFINITY, 0x7FFFFFFF};
      if (best >= 0) ++head[best];
      const bool have = wn.id != 0x7FFFFFFF;         // false only for a row with fewer than r+1 comparable entries
      const float pr = have ? fast_exp2((wn.v - a.m) * LOG2E) / a.Z : 0.f;
      if (r < k) {
        ids[row * k + r] = have ? wn.id : 0;
        probs[row * k + r] = pr;
      }
      if (r == 0) p_first = pr;
      if (r == 1) p_second = pr;
    }
    if (margin) margin[row] = p_first - p_second;
  }
}

hipError_t launch_confidence_topk(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride, int k,
                                  int32_t* ids, float* probs, float* margin, float* H, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == 1)
    confidence_topk_kernel<true><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H);
  else
    confidence_topk_kernel<false><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H);
  return hipGetLastError();
}

// Mean confidence of each chunk (rows cu_rows[b] .. cu_rows[b+1]) and its dispatch probability, the scaled
// sigmoid of Section 4.2: 1 for c <= c_th, else 1 / (1 + exp(k (c - c_th) / (1 - c_th) - k / 2)).
__global__ void chunk_dispatch_kernel(const float* __restrict__ p1, const int32_t* __restrict__ cu_rows, int B,
                                      float c_th, float k_slope, float* __restrict__ mean_conf,
                                      float* __restrict__ p_conf) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int r0 = cu_rows[b], r1 = cu_rows[b + 1];
  float sum = 0.f;
  for (int r = r0; r < r1; ++r) sum += p1[r];
  const float c = r1 > r0 ? sum / (float)(r1 - r0) : 0.f;
  mean_conf[b] = c;
  float pc = 1.0f;
  if (c > c_th) {
    const float norm = (c - c_th) / (1.0f - c_th) - 0.5f;
    pc = 1.0f / (1.0f + expf(k_slope * norm));
  }
  p_conf[b] = pc;
}

hipError_t launch_chunk_dispatch(const float* p1, const int32_t* cu_rows, int B, float c_th, float k_slope,
                                 float* mean_conf, float* p_conf, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  chunk_dispatch_kernel<<<(B + 127) / 128, 128, 0, s>>>(p1, cu_rows, B, c_th, k_slope, mean_conf, p_conf);
  return hipGetLastError();
}

// Top-p (nucleus) cut of compressed distributions: row r holds k probabilities, most probable first (the
// output of confidence_topk_kernel); n[r] = the smallest count whose float32 running sum, in list order,
// reaches top_p (all k if it never does), mass[r] = that sum.
__global__ void topp_count_kernel(const float* __restrict__ probs, int64_t rows, int k, float top_p,
                                  int32_t* __restrict__ n, float* __restrict__ mass) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  float acc = 0.f;
  int kept = 0;
  for (int i = 0; i < k; ++i) {
    acc += probs[r * k + i];
    kept = i + 1;
    if (acc >= top_p) break;
  }
  n[r] = kept;
  if (mass) mass[r] = acc;
}

hipError_t launch_topp_count(const float* probs, int64_t rows, int k, float top_p, int32_t* n, float* mass,
                             hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  topp_count_kernel<<<(unsigned)((rows + 127) / 128), 128, 0, s>>>(probs, rows, k, top_p, n, mass);
  return hipGetLastError();
}

// ------------------------------------------------------------------ stochastic verification
// Speculative sampling of one request per block (the rule the paper cites for its "draft & verify" under
// top-k / top-p sampling): draft j is accepted with probability min(1, q_j(x_j) / p_j(x_j)); at the first
// rejection a token is drawn from norm(max(0, q_j - p_j)), after k acceptances from q_{k+1}.  q_j is the softmax
// of an LM-head row that the verify call left behind (row of the last uncached token for j = 0, of draft
// j-1 after that; its maximum and normaliser come from the confidence pass: q_v = exp(l_v - l_max) p_top1);
// p_j is the device's transmitted top-k list renormalised to 1.  The uniforms are inputs.
// Thread 0 walks the drafts; the draw is block-wide: every thread sums a contiguous slice of the vocabulary
// (fp64 accumulators), the slices are scanned, and the thread whose slice holds the target walks it.
__global__ __launch_bounds__(256) void stochastic_accept_kernel(
    const float* __restrict__ logits, int vocab, const int32_t* __restrict__ lm_ids, const float* __restrict__ lm_p,
    const int32_t* __restrict__ tokens, BatchMeta m, int k_list, const int32_t* __restrict__ p_id,
    const float* __restrict__ p_prob, const float* __restrict__ u_accept, const float* __restrict__ u_sample,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ out_token) {
  __shared__ int sh_n, sh_slice, sh_token;
  __shared__ double sh_sum[256];
  __shared__ double sh_before;
  const int i = blockIdx.x, tid = threadIdx.x;
  const int r0 = m.cu_draft[i], k = m.cu_draft[i + 1] - r0;
  const int32_t* d = tokens + m.cu_tok[i] + m.n_unc[i];
  if (tid == 0) {
    int n = 0;
    for (; n < k; ++n) {
      const int row = n == 0 ? m.first_row[i] : r0 + n - 1;
      const float* l = logits + (size_t)row * vocab;
      int x = d[n];
      x = x < 0 ? 0 : (x >= vocab ? vocab - 1 : x);
      const float q_x = __expf(l[x] - l[lm_ids[row]]) * lm_p[row];
      float sum = 0.f, p_x = 0.f;
      for (int e = 0; e < k_list; ++e) {
        const float pe = p_prob[(size_t)(r0 + n) * k_list + e];
        sum += pe;
        if (p_id[(size_t)(r0 + n) * k_list + e] == x) p_x += pe;
      }
      const float ratio = p_x > 0.f ? fminf(1.0f, q_x * sum / p_x) : 0.f;
      if (!(u_accept[r0 + n] < ratio)) break;
    }
    sh_n = n;
    sh_token = -1;
  }
  __syncthreads();
  const int n = sh_n;
  const int row = (n == 0) ? m.first_row[i] : r0 + n - 1;      // n == k: the row after the last draft
  const float* l = logits + (size_t)row * vocab;
  const float l_max = l[lm_ids[row]], p_top = lm_p[row];
  // the list to subtract (none after a full accept)
  int ids[8];
  float pr[8];
  float list_sum = 0.f;
  const int n_list = n < k ? k_list : 0;
  for (int e = 0; e < 8; ++e) {
    ids[e] = -1;
    pr[e] = 0.f;
    if (e < n_list) {
      ids[e] = p_id[(size_t)(r0 + n) * k_list + e];
      pr[e] = p_prob[(size_t)(r0 + n) * k_list + e];
      list_sum += pr[e];
    }
  }
  const float list_inv = list_sum > 0.f ? 1.0f / list_sum : 0.f;   // an all-zero list subtracts nothing
  auto weight = [&](int v) {
    float w = __expf(l[v] - l_max) * p_top;
    for (int e = 0; e < 8; ++e)
      if (ids[e] == v) w -= pr[e] * list_inv;
    return w > 0.f ? w : 0.f;
  };
  const int seg = (vocab + 255) / 256;
  const int v0 = tid * seg, v1 = min(vocab, v0 + seg);
  double mine = 0.0;
  for (int v = v0; v < v1; ++v) mine += (double)weight(v);
  sh_sum[tid] = mine;
  __syncthreads();
  if (tid == 0) {
    double total = 0.0;
    for (int t = 0; t < 256; ++t) total += sh_sum[t];
    const double target = (double)u_sample[i] * total;
    double c = 0.0;
    int slice = 255;
    for (int t = 0; t < 256; ++t) {
      if (c + sh_sum[t] > target) {
        slice = t;
        break;
      }
      c += sh_sum[t];
    }
    if (slice == 255 && !(c + sh_sum[255] > target)) {          // rounding put the target at the very end
      c = 0.0;
      for (int t = 0; t < 255; ++t) c += sh_sum[t];
    }
    sh_slice = slice;
    sh_before = c;
  }
  __syncthreads();
  if (tid == sh_slice) {
    double total = 0.0;
    for (int t = 0; t < 256; ++t) total += sh_sum[t];
    const double target = (double)u_sample[i] * total;
    double c = sh_before;
    int token = -1, last_positive = -1;
    for (int v = v0; v < v1; ++v) {
      const float w = weight(v);
      if (w > 0.f) last_positive = v;
      c += (double)w;
      if (c > target && w > 0.f) {
        token = v;
        break;
      }
    }
    sh_token = token >= 0 ? token : last_positive;
  }
  __syncthreads();
  if (tid == 0) {
    accept_len[i] = n;
    out_token[i] = sh_token >= 0 ? sh_token : lm_ids[row];      // degenerate residual (p == q): the row's mode
  }
}

hipError_t launch_stochastic_accept(const float* logits, int vocab, const int32_t* lm_ids, const float* lm_p,
                                    const int32_t* tokens, const BatchMeta& m, int B, int k_list, const int32_t* p_id,
                                    const float* p_prob, const float* u_accept, const float* u_sample,
                                    int32_t* accept_len, int32_t* out_token, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  stochastic_accept_kernel<<<B, 256, 0, s>>>(logits, vocab, lm_ids, lm_p, tokens, m, k_list, p_id, p_prob, u_accept,
                                             u_sample, accept_len, out_token);
  return hipGetLastError();
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
