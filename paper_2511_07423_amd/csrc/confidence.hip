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

// ---------------------------------------------------------------------------------------------
// The same for 8 < k <= 256, the size of a transmitted list ("Compression before transmission" cuts 32000
// entries by over 99.5 %: up to 160).  Two levels.  Level 1: each wavefront keeps its k best (logit, id) sorted
// across its LANES -- entry p lives in register p / 64 of lane p % 64 -- so an insertion is a handful of
// wavefront-wide instructions whatever k is: a ballot counts the entries that come before the candidate, every
// lane at or behind that position takes its left neighbour's entry (the entry of lane 63 crosses into lane 0 of
// the next register), and the lane at the position takes the candidate.  Candidates are found as above (a
// ballot against the list's k-th entry).  Level 2: the four sorted lists meet in LDS and every entry computes its
// final rank as its position in its own list plus, by binary search, the number of entries of the other three
// lists that come before it; ranks below k are the result, already in order.
#define TOPK_WIDE_MAX 256

template <bool BF16, int R>
__global__ __launch_bounds__(256) void confidence_topk_wide_kernel(const void* __restrict__ logits, int64_t vocab,
                                                                   int64_t stride, int k, int32_t* __restrict__ ids,
                                                                   float* __restrict__ probs, float* __restrict__ margin,
                                                                   float* __restrict__ H) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int64_t row = blockIdx.x;
  const char* base = reinterpret_cast<const char*>(logits) + row * stride * (BF16 ? 2 : 4);
  const uint4* src = reinterpret_cast<const uint4*>(base);
  const int n_vec = (int)(vocab / VEC);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  ConfState st = {-1e30f, 0.f, 0.f, 0};
  float ev[R];                                       // entry p = r * 64 + lane of the wavefront's sorted list
  int ei[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    ev[r] = -INFINITY;
    ei[r] = 0x7FFFFFFF;
  }
  float thr_v = -INFINITY;                           // the list's k-th entry (wavefront-uniform)
  int thr_i = 0x7FFFFFFF;
  const int kr = (k - 1) >> 6, kl = (k - 1) & 63;    // where entry k - 1 lives

  auto insert = [&](float cv, int ci) {              // wavefront-uniform candidate that comes before the k-th entry
    int pos = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
      pos += __builtin_popcountll(__builtin_amdgcn_ballot_w64(top_before(ev[r], ei[r], cv, ci)));
#pragma unroll
    for (int r = R - 1; r >= 0; --r) {
      float upv = __shfl_up(ev[r], 1);
      int upi = __shfl_up(ei[r], 1);
      if (r > 0) {
        const float cross_v = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(ev[r - 1]), 63));
        const int cross_i = __builtin_amdgcn_readlane(ei[r - 1], 63);
        if (lane == 0) {
          upv = cross_v;
          upi = cross_i;
        }
      }
      const int p = r * 64 + lane;
      ev[r] = p < pos ? ev[r] : (p == pos ? cv : upv);
      ei[r] = p < pos ? ei[r] : (p == pos ? ci : upi);
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (r == kr) {
        thr_v = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(ev[r]), kl));
        thr_i = __builtin_amdgcn_readlane(ei[r], kl);
      }
  };
  auto offer = [&](float v, int id) {
    unsigned long long mask = __builtin_amdgcn_ballot_w64(top_before(v, id, thr_v, thr_i));
    while (mask) {                                   // wavefront-uniform loop
      const int l = __builtin_ctzll(mask);
      mask &= mask - 1;
      const float cv = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), l));
      const int ci = __builtin_amdgcn_readlane(id, l);
      if (top_before(cv, ci, thr_v, thr_i)) insert(cv, ci);   // the k-th entry may have moved up meanwhile
    }
  };
  // The list lives across the lanes, so EVERY lane of the wavefront walks through every insertion: the loop
  // below has no divergent arm; a lane past the end of the row carries -inf entries that are never candidates.
  auto consume = [&](const uint4& raw, int c, bool valid) {
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
    float cmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < VEC; ++i) cmax = fmaxf(cmax, valid ? v[i] : -INFINITY);
    if (__builtin_amdgcn_ballot_w64(cmax >= thr_v) != 0) {   // wavefront-uniform
#pragma unroll
      for (int i = 0; i < VEC; ++i) offer(valid ? v[i] : -INFINITY, valid ? c * VEC + i : 0x7FFFFFFF);
    }
    if (valid) conf_chunk<VEC>(st, v, c * VEC);        // per-lane state: may diverge
  };
  const int rounds = (n_vec + 255) / 256;
  for (int it = 0; it < rounds; ++it) {
    const int c = it * 256 + threadIdx.x;
    const bool valid = c < n_vec;
    const uint4 raw = valid ? src[c] : make_uint4(0u, 0u, 0u, 0u);
    consume(raw, c, valid);
  }
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

  for (int o = 1; o < 64; o <<= 1) {
    ConfState other;
    other.m = __shfl_xor(st.m, o);
    other.Z = __shfl_xor(st.Z, o);
    other.S = __shfl_xor(st.S, o);
    other.id = __shfl_xor(st.id, o);
    conf_merge(st, other);
  }
  __shared__ ConfState red[4];
  __shared__ float cv_[4][TOPK_WIDE_MAX];
  __shared__ int ci_[4][TOPK_WIDE_MAX];
  __shared__ int n_valid[4];
  __shared__ float sh_m, sh_z;
  if (lane == 0) red[wave] = st;
  int mine = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    cv_[wave][r * 64 + lane] = ev[r];
    ci_[wave][r * 64 + lane] = ei[r];
    mine += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ei[r] != 0x7FFFFFFF && r * 64 + lane < k));
  }
  if (lane == 0) n_valid[wave] = mine;
  // defaults for a row with fewer than k comparable entries
  for (int e = threadIdx.x; e < k; e += 256) {
    ids[row * k + e] = 0;
    probs[row * k + e] = 0.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    ConfState a = red[0];
    conf_merge(a, red[1]);
    conf_merge(a, red[2]);
    conf_merge(a, red[3]);
    if (H) H[row] = logf(a.Z) - a.S / a.Z;
    sh_m = a.m;
    sh_z = a.Z;
  }
  __syncthreads();
  const float m = sh_m, Z = sh_z;
  __shared__ float p_top[2];
  if (threadIdx.x < 2) p_top[threadIdx.x] = 0.f;
  __syncthreads();
  for (int w = 0; w < 4; ++w) {
    const int e = threadIdx.x;                       // entry e of list w
    if (e >= n_valid[w]) continue;
    const float v = cv_[w][e];
    const int id = ci_[w][e];
    int rank = e;
    for (int o = 0; o < 4; ++o) {
      if (o == w) continue;
      int lo = 0, hi = n_valid[o];                   // first entry of list o that does not come before (v, id)
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (top_before(cv_[o][mid], ci_[o][mid], v, id)) lo = mid + 1; else hi = mid;
      }
      rank += lo;
    }
    if (rank < k) {
      const float pr = fast_exp2((v - m) * LOG2E) / Z;
      ids[row * k + rank] = id;
      probs[row * k + rank] = pr;
      if (rank < 2) p_top[rank] = pr;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && margin) margin[row] = p_top[0] - p_top[1];
}

hipError_t launch_confidence_topk(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride, int k,
                                  int32_t* ids, float* probs, float* margin, float* H, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const unsigned grid = (unsigned)rows;
  if (k <= TOPK_MAX) {
    if (dtype == 1)
      confidence_topk_kernel<true><<<grid, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H);
    else
      confidence_topk_kernel<false><<<grid, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H);
    return hipGetLastError();
  }
  if (k > TOPK_WIDE_MAX) return hipErrorInvalidValue;
#define SY_WIDE(R_)                                                                                              \
  if (dtype == 1)                                                                                                \
    confidence_topk_wide_kernel<true, R_><<<grid, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H); \
  else                                                                                                           \
    confidence_topk_wide_kernel<false, R_><<<grid, 256, 0, s>>>(logits, vocab, stride, k, ids, probs, margin, H);
  if (k <= 64) { SY_WIDE(1) } else if (k <= 128) { SY_WIDE(2) } else if (k <= 192) { SY_WIDE(3) } else { SY_WIDE(4) }
#undef SY_WIDE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Full-vocabulary top-p (nucleus): per row the smallest number of tokens, most probable first (equal logits by
// the lower id), whose probabilities sum to top_p, their mass, and the smallest logit kept.  One block per row.
// After the statistics pass (m, Z) the cut is found by a radix search over the 32-bit order-preserving key of the
// logits, 8 bits per pass from the top: every pass re-reads the row (from L2), adds each element whose key
// matches the prefix found so far to one of 256 bins -- its count and its probability mass -- and the bin in which
// the running mass, taken from the largest keys down, reaches top_p extends the prefix.  Masses are summed as
// 40-bit fixed point with integer atomics, so the sums do not depend on the order in which the threads arrive and
// the integer result is reproducible.  After four passes the prefix is one logit value; of its holders (ties) only
// as many as needed are counted.
__device__ __forceinline__ uint32_t order_key(float v) {
  const uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

template <bool BF16>
__global__ __launch_bounds__(256) void nucleus_kernel(const void* __restrict__ logits, int64_t vocab, int64_t stride,
                                                      float top_p, int32_t* __restrict__ count, float* __restrict__ mass,
                                                      float* __restrict__ cut_logit) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int64_t row = blockIdx.x;
  const char* base = reinterpret_cast<const char*>(logits) + row * stride * (BF16 ? 2 : 4);
  const uint4* src = reinterpret_cast<const uint4*>(base);
  const int n_vec = (int)(vocab / VEC);
  auto load = [&](int c, float (&v)[VEC]) {
    const uint4 raw = src[c];
    if constexpr (BF16) {
      v[0] = bf2f(raw.x & 0xFFFF); v[1] = bf2f(raw.x >> 16);
      v[2] = bf2f(raw.y & 0xFFFF); v[3] = bf2f(raw.y >> 16);
      v[4] = bf2f(raw.z & 0xFFFF); v[5] = bf2f(raw.z >> 16);
      v[6] = bf2f(raw.w & 0xFFFF); v[7] = bf2f(raw.w >> 16);
    } else {
      v[0] = __uint_as_float(raw.x); v[1] = __uint_as_float(raw.y);
      v[2] = __uint_as_float(raw.z); v[3] = __uint_as_float(raw.w);
    }
  };
  auto tail_value = [&](int64_t e) {
    return BF16 ? bf2f(reinterpret_cast<const bf16_t*>(base)[e]) : reinterpret_cast<const float*>(base)[e];
  };
  // ---- statistics
  ConfState st = {-1e30f, 0.f, 0.f, 0};
  for (int c = threadIdx.x; c < n_vec; c += 256) {
    float v[VEC];
    load(c, v);
    conf_chunk<VEC>(st, v, c * VEC);
  }
  for (int64_t e = (int64_t)n_vec * VEC + threadIdx.x; e < vocab; e += 256) {
    float v[1] = {tail_value(e)};
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
  __shared__ unsigned long long bin_mass[256];
  __shared__ unsigned int bin_count[256];
  __shared__ uint32_t sh_prefix;
  __shared__ unsigned long long sh_mass_above;
  __shared__ unsigned int sh_count_above;
  __shared__ float sh_m, sh_inv_z;
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = st;
  __syncthreads();
  if (threadIdx.x == 0) {
    ConfState a = red[0];
    conf_merge(a, red[1]);
    conf_merge(a, red[2]);
    conf_merge(a, red[3]);
    sh_m = a.m;
    sh_inv_z = 1.0f / a.Z;
    sh_prefix = 0;
    sh_mass_above = 0;
    sh_count_above = 0;
  }
  __syncthreads();
  const float m = sh_m, inv_z = sh_inv_z;
  const double FIX = 1099511627776.0;                // 2^40
  auto fixed_mass = [&](float v) {
    const float p = fast_exp2(fmaxf(v - m, -1e30f) * LOG2E) * inv_z;
    return (unsigned long long)((double)p * FIX + 0.5);
  };
  // the target in the same fixed point, against the mass the row really sums to in it is not needed: p sums to
  // 1 within rounding, and top_p = 1 is met by the last element at the latest (the search then ends at the
  // smallest key present)
  const unsigned long long target = (unsigned long long)((double)top_p * FIX);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    bin_mass[threadIdx.x] = 0;
    bin_count[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t pmask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    auto add = [&](float v) {
      const uint32_t key = order_key(v);
      if ((key & pmask) != prefix) return;
      const int b = (key >> shift) & 255;
      atomicAdd(&bin_mass[b], fixed_mass(v));
      atomicAdd(&bin_count[b], 1u);
    };
    for (int c = threadIdx.x; c < n_vec; c += 256) {
      float v[VEC];
      load(c, v);
#pragma unroll
      for (int i = 0; i < VEC; ++i) add(v[i]);
    }
    for (int64_t e = (int64_t)n_vec * VEC + threadIdx.x; e < vocab; e += 256) add(tail_value(e));
    __syncthreads();
    if (threadIdx.x == 0) {
      unsigned long long acc = sh_mass_above;
      unsigned int cnt = sh_count_above;
      int b = -1, last = -1;
      unsigned long long acc_last = acc;             // the sums as they stood before bin `last` was added
      unsigned int cnt_last = cnt;
      for (int t = 255; t >= 0; --t) {
        if (bin_count[t] == 0) continue;
        if (acc + bin_mass[t] >= target) {
          b = t;
          break;
        }
        if (bin_mass[t] > 0 || last < 0) {           // the smallest keys that still carry probability
          last = t;
          acc_last = acc;
          cnt_last = cnt;
        }
        acc += bin_mass[t];
        cnt += bin_count[t];
      }
      if (b < 0) {                                   // rounding left the whole row below the target (top_p ~ 1): the cut
        b = last < 0 ? 0 : last;                     // is the smallest key that carries probability (masked tokens,
        acc = acc_last;                              // -inf, are never part of a nucleus)
        cnt = cnt_last;
      }
      sh_mass_above = acc;
      sh_count_above = cnt;
      sh_prefix = prefix | ((uint32_t)b << shift);
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    // the prefix is now one key: bin_count / bin_mass of its last-pass bin are its holders
    const uint32_t key = sh_prefix;
    const int b = key & 255;
    const unsigned int holders = bin_count[b];
    const unsigned long long each = holders ? bin_mass[b] / holders : 0;
    unsigned long long acc = sh_mass_above;
    unsigned int need = holders;
    if (each > 0 && acc < target) {
      const unsigned long long want = (target - acc + each - 1) / each;
      need = want < holders ? (unsigned int)want : holders;
    } else if (acc >= target) {
      need = 0;                                      // cannot happen: the bin was chosen because acc < target
    }
    if (need == 0) need = 1;
    count[row] = (int32_t)(sh_count_above + need);
    if (mass) mass[row] = (float)((double)(acc + each * need) / FIX);
    if (cut_logit) cut_logit[row] = key_value(key);
  }
}

hipError_t launch_nucleus(const void* logits, int dtype, int64_t rows, int64_t vocab, int64_t stride, float top_p,
                          int32_t* count, float* mass, float* cut_logit, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dtype == 1)
    nucleus_kernel<true><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, top_p, count, mass, cut_logit);
  else
    nucleus_kernel<false><<<(unsigned)rows, 256, 0, s>>>(logits, vocab, stride, top_p, count, mass, cut_logit);
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
  __shared__ int l_id[TOPK_WIDE_MAX];                // the list to subtract at the rejected position
  __shared__ float l_p[TOPK_WIDE_MAX];               // its probabilities, renormalised to 1
  __shared__ float l_sum;
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
  const int n_list = n < k ? k_list : 0;                       // nothing to subtract after a full accept
  if (tid == 0) {
    float sum = 0.f;
    for (int e = 0; e < n_list; ++e) sum += p_prob[(size_t)(r0 + n) * k_list + e];   // in list order, as above
    l_sum = sum;
  }
  __syncthreads();
  const float list_inv = l_sum > 0.f ? 1.0f / l_sum : 0.f;     // an all-zero list subtracts nothing
  for (int e = tid; e < n_list; e += 256) {
    l_id[e] = p_id[(size_t)(r0 + n) * k_list + e];
    l_p[e] = p_prob[(size_t)(r0 + n) * k_list + e] * list_inv;
  }
  __syncthreads();
  auto q_of = [&](int v) { return __expf(l[v] - l_max) * p_top; };
  auto weight = [&](int v) {                                   // max(0, q - p) at token v
    float w = q_of(v);
    for (int e = 0; e < n_list; ++e)
      if (l_id[e] == v) w -= l_p[e];
    return w > 0.f ? w : 0.f;
  };
  // Slice sums of max(0, q - p): every thread sums q over its slice of the vocabulary; the (few) tokens of the
  // list are then corrected one by one, in list order, by the thread that owns the slice they fall in.
  const int seg = (vocab + 255) / 256;
  const int v0 = tid * seg, v1 = min(vocab, v0 + seg);
  double mine = 0.0;
  for (int v = v0; v < v1; ++v) mine += (double)q_of(v);
  for (int e = 0; e < n_list; ++e) {
    const int v = l_id[e];
    if (v < v0 || v >= v1) continue;
    bool first = true;                                         // a token listed twice is corrected once, by its total
    for (int f = 0; f < e; ++f) first = first && l_id[f] != v;
    if (first) mine += (double)weight(v) - (double)q_of(v);
  }
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
