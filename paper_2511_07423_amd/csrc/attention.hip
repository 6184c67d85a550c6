// Paged ragged chunk attention for the partial prefill of draft chunks:
//   o = softmax(q K^T / sqrt(h)) V          (attention definition, Section 3.2)
// where chunk row j of request i sees keys 0..L_i+j: the whole cached prefix and,
// causally, the chunk itself (a prefill "with an existing KV-cached prefix",
// Section 3.4).  Grouped-query attention: q head hq reads KV head hq / G.
//
// Design (gfx950, 64-wide wavefronts, no LDS in the main loop):
//   * A work item is (request, group of <= 64 query rows = chunk tokens x G heads
//     of one KV head, key range).  One 256-thread block per (item, KV head); its
//     four wavefronts take 32-key tiles (two pages) round-robin, each running its
//     own online softmax, and merge through LDS once at the end.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16:
//     the A operand is a K page read straight from HBM (lane = (slot, 16-byte dim
//     chunk), so a page is fetched as whole 64-byte segments exactly once), the B
//     operand is Q held in registers for the whole item.  The result leaves each
//     lane with 4 keys x 1 query row, so softmax statistics are per-lane plus two
//     cross-lane exchanges, and the probabilities are already laid out as the B
//     operand of O^T = V^T P^T.  V pages are stored dim-major ([dim][slot]), which
//     makes the A operand of that product two plain 8-byte loads per lane.
//   * q and the probabilities enter the matrix cores as bf16 (hi, lo) pairs (two MFMAs per
//     product, K/V fragments reused), and o leaves as a pair: single bf16 terms here cost the
//     logits of a deep decoder an order of magnitude in accuracy.  The Q pairs of the row
//     group sit in LDS in fragment order (each lane re-reads its own 16 bytes per tile).
//   * Every K/V byte of the key range is read once per KV head and shared by the
//     G x k_i query rows.  Ranges are split across blocks for occupancy; partial
//     (m, l, O) results are merged by attn_combine_kernel.
#include "common.h"

#define NEG_BIG (-1e30f)

template <int HD>
struct KVTile {
  bf16x8 k[2][HD / 32];   // [page][k-step]: 8 dims of one key slot
  uint2 v[HD / 16][2];    // [dim block][page]: 4 key slots of one dim
};

template <int HD>
__device__ __forceinline__ void load_tile(KVTile<HD>& t, const bf16_t* __restrict__ k_layer,
                                          const bf16_t* __restrict__ v_layer, int pa, int pb, int Hkv, int kh,
                                          int n16, int g) {
  const bf16_t* ka = k_layer + ((size_t)pa * Hkv + kh) * (SY_PAGE * HD) + n16 * HD + 8 * g;
  const bf16_t* kb = k_layer + ((size_t)pb * Hkv + kh) * (SY_PAGE * HD) + n16 * HD + 8 * g;
#pragma unroll
  for (int s = 0; s < HD / 32; ++s) {
    t.k[0][s] = *reinterpret_cast<const bf16x8*>(ka + 32 * s);
    t.k[1][s] = *reinterpret_cast<const bf16x8*>(kb + 32 * s);
  }
  const bf16_t* va = v_layer + ((size_t)pa * Hkv + kh) * (SY_PAGE * HD) + n16 * SY_PAGE + 4 * g;
  const bf16_t* vb = v_layer + ((size_t)pb * Hkv + kh) * (SY_PAGE * HD) + n16 * SY_PAGE + 4 * g;
#pragma unroll
  for (int db = 0; db < HD / 16; ++db) {
    t.v[db][0] = *reinterpret_cast<const uint2*>(va + db * 16 * SY_PAGE);
    t.v[db][1] = *reinterpret_cast<const uint2*>(vb + db * 16 * SY_PAGE);
  }
}

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// Four consecutive outputs as a bf16 (hi, lo) pair: 8 bytes to each array.
__device__ __forceinline__ void store_pair(bf16_t* hi, bf16_t* lo, float a, float b, float c, float d) {
  uint2 h, l;
  h.x = pack_bf2(a, b);
  h.y = pack_bf2(c, d);
  l.x = pack_bf2(a - bf2f(h.x & 0xFFFF), b - bf2f(h.x >> 16));
  l.y = pack_bf2(c - bf2f(h.y & 0xFFFF), d - bf2f(h.y >> 16));
  *reinterpret_cast<uint2*>(hi) = h;
  *reinterpret_cast<uint2*>(lo) = l;
}

template <int HD, int RB>
__global__ __launch_bounds__(256) void attn_kernel(AttnLaunch a, int item_base, float scale_log2) {
  constexpr int KS = HD / 32;
  constexpr int DB = HD / 16;
  constexpr int ROWS = RB * 16;
  constexpr int OSTRIDE = HD + 4;                 // padded LDS row (floats)
  extern __shared__ float lds[];
  float* s_o = lds;                               // [4][ROWS][OSTRIDE]
  float* s_m = lds + 4 * ROWS * OSTRIDE;          // [4][ROWS]
  float* s_l = s_m + 4 * ROWS;                    // [4][ROWS]
  float* s_ms = s_l + 4 * ROWS;                   // [ROWS] merged max
  float* s_ls = s_ms + ROWS;                      // [ROWS] merged sum

  const AttnItem it = a.items[item_base + blockIdx.x];
  const int kh = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = lane & 15, g = lane >> 4;
  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int nrows = it.ntok * G;
  const int32_t* bt = a.block_table + (size_t)it.req * a.max_pages;

  // Q fragments (B operand: lane = (row n16, dim chunk g)) as (hi, lo) pairs, parked in LDS in
  // fragment order: fragment f = (rb * KS + s) * 2 + part, 64 lanes x 16 bytes each.  Rows past the
  // group are zero.  The region is reused by the merge at the end.
  bf16x8* s_q = reinterpret_cast<bf16x8*>(lds);
  int lim[RB];                                    // last key this lane's row may see
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = rb * 16 + n16;
    lim[rb] = row < nrows ? it.ctx_len + it.j0 + row / G : 0x7FFFFFFF;
  }
  for (int f = wave; f < RB * KS * 2; f += 4) {
    const int part = f & 1, s = (f >> 1) % KS, rb = (f >> 1) / KS;
    const int row = rb * 16 + n16;
    bf16x8 v = bf16x8{};
    if (row < nrows) {
      const bf16_t* qp = (part ? a.q_lo : a.q) + ((size_t)(it.tok0 + row / G) * Hq + kh * G + row % G) * HD;
      v = *reinterpret_cast<const bf16x8*>(qp + 32 * s + 8 * g);
    }
    s_q[f * 64 + lane] = v;
  }
  __syncthreads();

  float m_run[RB], l_run[RB];
  f32x4 acc[RB][DB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = NEG_BIG;
    l_run[rb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[rb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int key_end = it.key_end;
  const int free_end = min(key_end, it.ctx_len + it.j0 + 1);   // keys below this need no mask at all
  int kb = it.key_begin + 32 * wave;

  auto pages_of = [&](int kbase, int& pa, int& pb) {
    pa = bt[kbase >> 4];
    pb = (kbase + 16 < key_end) ? bt[(kbase >> 4) + 1] : pa;
  };

  KVTile<HD> cur;
  int pa = 0, pb = 0;
  if (kb < key_end) {
    pages_of(kb, pa, pb);
    load_tile<HD>(cur, a.k_layer, a.v_layer, pa, pb, Hkv, kh, n16, g);
  }
  while (kb < key_end) {
    const int kb_next = kb + 128;
    KVTile<HD> nxt;
    if (kb_next < key_end) {                       // issue the next tile's loads before computing
      int na, nb;
      pages_of(kb_next, na, nb);
      load_tile<HD>(nxt, a.k_layer, a.v_layer, na, nb, Hkv, kh, n16, g);
    }

    if (kb + 32 > key_end) {                       // tail tile: blank V slots past the range (may be junk)
#pragma unroll
      for (int pg = 0; pg < 2; ++pg) {
        const int t0 = kb + 16 * pg + 4 * g;
        const uint32_t m0 = (t0 + 0 < key_end ? 0x0000FFFFu : 0u) | (t0 + 1 < key_end ? 0xFFFF0000u : 0u);
        const uint32_t m1 = (t0 + 2 < key_end ? 0x0000FFFFu : 0u) | (t0 + 3 < key_end ? 0xFFFF0000u : 0u);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          cur.v[db][pg].x &= m0;
          cur.v[db][pg].y &= m1;
        }
      }
    }
    const bool need_mask = kb + 32 > free_end;

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bf16x8 qh = s_q[((rb * KS + s) * 2 + 0) * 64 + lane];
        const bf16x8 ql = s_q[((rb * KS + s) * 2 + 1) * 64 + lane];
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[0][s], qh, s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[1][s], qh, s1, 0, 0, 0);
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[0][s], ql, s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[1][s], ql, s1, 0, 0, 0);
      }
      float sv[8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        sv[r] = s0[r] * scale_log2;
        sv[4 + r] = s1[r] * scale_log2;
      }
      bool vis[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) vis[r] = true;
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int tau = kb + 16 * (r >> 2) + 4 * g + (r & 3);
          vis[r] = (tau < key_end) && (tau <= lim[rb]);
          sv[r] = vis[r] ? sv[r] : NEG_BIG;
        }
      }
      float mx = sv[0];
#pragma unroll
      for (int r = 1; r < 8; ++r) mx = fmaxf(mx, sv[r]);
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[rb], mx);
      const float alpha = ex2(m_run[rb] - m_new);
      m_run[rb] = m_new;
      float p[8], psum = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        p[r] = vis[r] ? ex2(sv[r] - m_new) : 0.f;
        psum += p[r];
      }
      l_run[rb] = l_run[rb] * alpha + psum;
      uint4 pk, pl;
      pk.x = pack_bf2(p[0], p[1]);
      pk.y = pack_bf2(p[2], p[3]);
      pk.z = pack_bf2(p[4], p[5]);
      pk.w = pack_bf2(p[6], p[7]);
      pl.x = pack_bf2(p[0] - bf2f(pk.x & 0xFFFF), p[1] - bf2f(pk.x >> 16));
      pl.y = pack_bf2(p[2] - bf2f(pk.y & 0xFFFF), p[3] - bf2f(pk.y >> 16));
      pl.z = pack_bf2(p[4] - bf2f(pk.z & 0xFFFF), p[5] - bf2f(pk.z >> 16));
      pl.w = pack_bf2(p[6] - bf2f(pk.w & 0xFFFF), p[7] - bf2f(pk.w >> 16));
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pk);
      const bf16x8 pfl = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        uint4 vv;
        vv.x = cur.v[db][0].x; vv.y = cur.v[db][0].y;
        vv.z = cur.v[db][1].x; vv.w = cur.v[db][1].y;
        const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
        f32x4 o = acc[rb][db];
        o[0] *= alpha; o[1] *= alpha; o[2] *= alpha; o[3] *= alpha;
        o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, o, 0, 0, 0);
        acc[rb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pfl, o, 0, 0, 0);
      }
    }
    cur = nxt;
    kb = kb_next;
  }

  // ---- merge the four wavefronts' (m, l, O) through LDS (which held Q until now)
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    float l = l_run[rb];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (g == 0) {
      s_m[wave * ROWS + rb * 16 + n16] = m_run[rb];
      s_l[wave * ROWS + rb * 16 + n16] = l;
    }
  }
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = rb * 16 + n16;
    const float m0 = s_m[row], m1 = s_m[ROWS + row], m2 = s_m[2 * ROWS + row], m3 = s_m[3 * ROWS + row];
    const float ms = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
    const float f = ex2(m_run[rb] - ms);
    if (wave == 0 && g == 0) {
      s_ms[row] = ms;
      s_ls[row] = s_l[row] * ex2(m0 - ms) + s_l[ROWS + row] * ex2(m1 - ms) + s_l[2 * ROWS + row] * ex2(m2 - ms) +
                  s_l[3 * ROWS + row] * ex2(m3 - ms);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      f32x4 o = acc[rb][db];
      float4 w = {o[0] * f, o[1] * f, o[2] * f, o[3] * f};
      *reinterpret_cast<float4*>(s_o + ((size_t)wave * ROWS + row) * OSTRIDE + db * 16 + 4 * g) = w;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < nrows * (HD / 4); e += 256) {
    const int row = e / (HD / 4), d4 = (e % (HD / 4)) * 4;
    float4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float4 v = *reinterpret_cast<const float4*>(s_o + ((size_t)w * ROWS + row) * OSTRIDE + d4);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    if (it.part < 0) {
      const float inv = 1.0f / s_ls[row];
      const size_t at = ((size_t)(it.tok0 + row / G) * Hq + kh * G + row % G) * HD + d4;
      store_pair(a.o + at, a.o_lo + at, sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
    } else {
      *reinterpret_cast<float4*>(a.part_o + (((size_t)it.part * Hkv + kh) * 64 + row) * HD + d4) = sum;
    }
  }
  if (it.part >= 0 && threadIdx.x < nrows) {
    float2 ml = {s_ms[threadIdx.x], s_ls[threadIdx.x]};
    *reinterpret_cast<float2*>(a.part_ml + (((size_t)it.part * Hkv + kh) * 64 + threadIdx.x) * 2) = ml;
  }
}

// Merge the key-range partials of one chunk token: o = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnLaunch a) {
  const int t = blockIdx.x;
  const AttnCombine c = a.comb[t];
  if (c.part0 < 0) return;
  const int HD = a.hd, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
  for (int e = threadIdx.x; e < Hq * (HD / 4); e += 256) {
    const int hq = e / (HD / 4), d4 = (e % (HD / 4)) * 4;
    const int kh = hq / G, row = c.row0 + hq % G;
    float M = NEG_BIG;
    for (int s = 0; s < c.nsplit; ++s)
      M = fmaxf(M, a.part_ml[(((size_t)(c.part0 + s) * Hkv + kh) * 64 + row) * 2]);
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int s = 0; s < c.nsplit; ++s) {
      const size_t base = ((size_t)(c.part0 + s) * Hkv + kh) * 64 + row;
      const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + base * 2);
      const float w = ex2(ml.x - M);
      const float4 v = *reinterpret_cast<const float4*>(a.part_o + base * HD + d4);
      sum.x += w * v.x; sum.y += w * v.y; sum.z += w * v.z; sum.w += w * v.w;
      l += w * ml.y;
    }
    const float inv = 1.0f / l;
    const size_t at = ((size_t)t * Hq + hq) * HD + d4;
    store_pair(a.o + at, a.o_lo + at, sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
  }
}

template <int HD, int RB>
static hipError_t launch_class(const AttnLaunch& a, int cls, float scale_log2, hipStream_t s) {
  const int n = a.class_begin[cls + 1] - a.class_begin[cls];
  if (n <= 0) return hipSuccess;
  constexpr int ROWS = RB * 16;
  const size_t lds_merge = (size_t)(4 * ROWS * (HD + 4) + 8 * ROWS + 2 * ROWS) * sizeof(float);
  const size_t lds_q = (size_t)RB * (HD / 32) * 2 * 64 * 16;
  const size_t lds = lds_merge > lds_q ? lds_merge : lds_q;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<HD, RB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  attn_kernel<HD, RB><<<dim3(n, a.Hkv), 256, lds, s>>>(a, a.class_begin[cls], scale_log2);
  return hipGetLastError();
}

template <int HD>
static hipError_t launch_hd(const AttnLaunch& a, hipStream_t s) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  hipError_t e;
  if ((e = launch_class<HD, 1>(a, 0, scale_log2, s)) != hipSuccess) return e;
  if ((e = launch_class<HD, 2>(a, 1, scale_log2, s)) != hipSuccess) return e;
  if ((e = launch_class<HD, 4>(a, 2, scale_log2, s)) != hipSuccess) return e;
  if (a.any_split) {
    attn_combine_kernel<<<a.T, 256, 0, s>>>(a);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_attention(const AttnLaunch& a, hipStream_t s) {
  if (a.T <= 0) return hipSuccess;
  if (a.hd == 128) return launch_hd<128>(a, s);
  if (a.hd == 64) return launch_hd<64>(a, s);
  return hipErrorInvalidValue;
}
