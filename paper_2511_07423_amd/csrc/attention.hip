// Paged ragged chunk attention for the partial prefill of draft chunks:
//   o = softmax(q K^T / sqrt(h)) V          (attention definition, Section 3.2)
// where chunk row j of request i sees keys 0..L_i+j: the whole cached prefix and,
// causally, the chunk itself (a prefill "with an existing KV-cached prefix",
// Section 3.4).  Grouped-query attention: q head hq reads KV head hq / G.
//
// Design (gfx950, 64-wide wavefronts):
//   * A work item is (request, group of <= 64 query rows = chunk tokens x G heads of one KV head,
//     key range).  One 256-thread block per (item, KV head).
//   * K/V pages are staged in LDS by asynchronous global->LDS copies (global_load_lds_dwordx4): a
//     page tile is 4 KB (2 KB at head_dim 64) contiguous in HBM, so every copy instruction moves one
//     fully coalesced kilobyte, needs no registers, and a ring of 4 key tiles per block (two blocks,
//     64-96 KB per compute unit) stays in flight behind the ones being multiplied.  Each K/V byte of the key range leaves
//     HBM once per KV head and is shared by all G x k_i query rows.
//   * The four wavefronts split the row group into 16-row blocks (RBN = 2 or 4 of them) and, with
//     two blocks, the keys of a super-tile into two phases of 32 keys (two pages); a wavefront
//     owns one (row block, phase).  Phases merge through LDS at the
//     end; key ranges of one row group merge in attn_combine_kernel.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: the A operand is
//     a K page fragment (lane = (slot, 16-byte dim chunk); chunks are XOR-swizzled by slot on the
//     way into LDS so the reads are bank-conflict free), the B operand is Q in registers.  The
//     result leaves each lane with 4 keys x 1 query row: softmax statistics are per-lane plus two
//     cross-lane exchanges, and the probabilities are already the B operand of O^T = V^T P^T.
//     V pages are stored dim-major ([dim][slot]), which makes the A operand of that product plain
//     8-byte LDS reads.
//   * q and the probabilities enter the matrix cores as bf16 (hi, lo) pairs (two MFMAs per
//     product, K/V fragments reused), and o leaves as a pair: single bf16 terms here cost the
//     logits of a deep decoder an order of magnitude in accuracy.
#include "common.h"

#define NEG_BIG (-1e30f)

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// Reductions over the four lanes l, l^16, l^32, l^48 that hold one query row, with gfx950's lane-swap
// instructions (plain vector ALU work, no trip through the LDS crossbar).
__device__ __forceinline__ float row_max4(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
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

// Asynchronous 16-byte-per-lane copy global -> LDS; lane i lands at lds_addr + 16 i (m0 carries the
// wavefront-uniform LDS address).  Issued from inline assembly so that the waits are exactly the
// ones written below.
__device__ __forceinline__ void copy_to_lds(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}

// XOR mask of a K slot's 16-byte chunks in LDS.  A fragment read (lane = slot l % 16, chunk 4 s + l / 16)
// is served 16 lanes per cycle over 64 banks, lanes l and l + 16 together: slots that share banks (all of
// them at head_dim 128, every second one at 64) must differ in the chunk bits that l / 16 leaves alone.
template <int HD>
__device__ __forceinline__ int kswz(int slot) {
  return HD == 128 ? (((slot & 3) << 2) | (((slot >> 2) & 1) << 1)) : ((((slot >> 1) & 1) << 2) | (((slot >> 2) & 1) << 1));
}

// Wait until at most `tiles` x IPP of this wavefront's copies are in flight and its LDS reads are done
// (the wait count is an immediate, so the few possible values are spelled out; `tiles` is wavefront-uniform).
template <int IPP, int MAX_TILES>
__device__ __forceinline__ void wait_copies(int tiles) {
  static_assert(MAX_TILES <= 3, "add cases");
  if (tiles >= 3 && MAX_TILES >= 3) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(3 * IPP) : "memory");
  } else if (tiles == 2 && MAX_TILES >= 2) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * IPP) : "memory");
  } else if (tiles == 1 && MAX_TILES >= 1) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(1 * IPP) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  }
}

template <int HD, int RBN>
__device__ __forceinline__ void attn_body(const AttnLaunch& a, const AttnItem& it, float scale_log2) {
  constexpr int KP = 4 / RBN;                       // key phases: 32-key tiles consumed per iteration
  constexpr int NT = 5;                             // LDS ring: tile t lives in slot t % NT; NT - KP tiles stay
                                                    // in flight behind the KP being multiplied (80 KB at
                                                    // head_dim 128, so two blocks share a compute unit)
  constexpr int KS = HD / 32, DB = HD / 16;
  constexpr int PAGE_B = SY_PAGE * HD * 2;          // bytes of one K or V page tile
  constexpr int TILE_B = 4 * PAGE_B;                // K page a, K page b, V page a, V page b
  constexpr int IPP = PAGE_B / 1024;                // copy instructions per page = per wavefront and tile
  constexpr int CPS = HD / 8;                       // 16-byte chunks per K slot
  constexpr int OSTRIDE = HD + 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int kh = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n16 = lane & 15, g = lane >> 4;
  const int rb = wave % RBN, kp = wave / RBN;
  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int nrows = it.ntok * G;
  const int32_t* bt = a.block_table + (size_t)__builtin_amdgcn_readfirstlane(it.req) * a.max_pages;
  const int key_end = it.key_end;
  const int last_page = (key_end - 1) >> 4;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds;

  // ---- copies: of every tile this wavefront copies page tile `wave` (K page a, K page b, V page a, V page b),
  //      IPP instructions of one kilobyte; the lane's element offset inside the page is fixed
  //      (K chunks are swizzled by slot, V is copied straight)
  int c_off[IPP];
#pragma unroll
  for (int j = 0; j < IPP; ++j) {
    if (wave < 2) {
      const int slot = j * (1024 / (HD * 2)) + lane / CPS;
      c_off[j] = slot * HD + (((lane % CPS) ^ kswz<HD>(slot)) << 3);
    } else {
      c_off[j] = j * 512 + lane * 8;
    }
  }
  const size_t page_elems = (size_t)Hkv * SY_PAGE * HD;
  const bf16_t* my_pool = (wave < 2 ? a.k_layer : a.v_layer) + (size_t)kh * SY_PAGE * HD;

  const int n_keys = key_end - it.key_begin;
  const int n_tiles = (n_keys + 31) / 32;
  const int n_iter = (n_tiles + KP - 1) / KP;
  // A key range spans at most 64 pages (the host cuts ranges at <= 1024 keys): lane l keeps the id of
  // the range's page l, and a copy reads its page id with v_readlane.
  const int first_page = it.key_begin >> 4;
  const int n_pages_rng = last_page - first_page + 1;
  const int my_page = bt[first_page + (lane < n_pages_rng ? lane : n_pages_rng - 1)];
  // Copies of tile t into slot t % NT; nothing past the range's last tile.
  auto issue_tile = [&](int t) {
    if (t >= n_tiles) return;                         // wavefront-uniform
    int pi = 2 * t + (wave & 1);                      // page index relative to the range's first page
    pi = pi < n_pages_rng - 1 ? pi : n_pages_rng - 1; // the last tile may have one page only
    const bf16_t* src = my_pool + (size_t)__builtin_amdgcn_readlane(my_page, pi) * page_elems;
    const uint32_t dst = lds_base + (uint32_t)(t % NT) * TILE_B + wave * PAGE_B;
#pragma unroll
    for (int j = 0; j < IPP; ++j) copy_to_lds(src + c_off[j], dst + j * 1024);
  };
#pragma unroll
  for (int t = 0; t < NT - KP; ++t) issue_tile(t);

  // ---- Q fragments of this wavefront's row block (B operand: lane = (row n16, dim chunk g))
  const int row = rb * 16 + n16;
  bf16x8 qh[KS], ql[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    qh[s] = bf16x8{};
    ql[s] = bf16x8{};
  }
  if (row < nrows) {
    const size_t qat = ((size_t)(it.tok0 + row / G) * Hq + kh * G + row % G) * HD + 8 * g;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      qh[s] = *reinterpret_cast<const bf16x8*>(a.q + qat + 32 * s);
      ql[s] = *reinterpret_cast<const bf16x8*>(a.q_lo + qat + 32 * s);
    }
  }
  // Make the compiler finish the Q loads HERE.  It cannot see the asynchronous copies issued from inline
  // assembly, so with the Q loads still "pending" at the loop head it guards every first use of a Q register
  // inside the loop with s_waitcnt vmcnt(k), k counted from the Q loads: in reality those waits drain the
  // K/V copies just issued, once per iteration, and the ring never runs ahead.
#pragma unroll
  for (int s = 0; s < KS; ++s) asm volatile("" ::"v"(qh[s]), "v"(ql[s]));
  const int lim = row < nrows ? it.ctx_len + it.j0 + row / G : 0x7FFFFFFF;   // last key this row may see
  const int free_end = min(key_end, it.ctx_len + it.j0 + 1);                 // keys below need no mask

  float m_run = NEG_BIG;
  f32x4 acc_l = {0.f, 0.f, 0.f, 0.f};
  bf16x8 ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
  f32x4 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int iter = 0; iter < n_iter; ++iter) {
    // Own copies of this iteration's KP tiles have landed (the NT - 2 KP younger tiles may still be in
    // flight), own LDS reads of the previous ones are done; the barrier extends both facts to the block.
    // Tiles issued so far: min(n_tiles, iter KP + NT - KP); the ones after this iteration's may stay in flight.
    {
      const int issued = min(n_tiles, iter * KP + NT - KP);
      const int younger = max(0, issued - (iter + 1) * KP);
      wait_copies<IPP, NT - 2 * KP>(younger);
    }
    asm volatile("s_barrier" ::: "memory");
#pragma unroll
    for (int q = 0; q < KP; ++q) issue_tile(iter * KP + NT - KP + q);   // into the slots read last iteration
    const int tile_no = iter * KP + kp;
    const int kb = it.key_begin + tile_no * 32;
    if (kb >= key_end) continue;                      // wavefront-uniform
    const unsigned char* tile = lds + (size_t)(tile_no % NT) * TILE_B;

    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int ch = ((4 * s + g) ^ kswz<HD>(n16)) << 4;
      const bf16x8 ka = *reinterpret_cast<const bf16x8*>(tile + n16 * (HD * 2) + ch);
      const bf16x8 kbf = *reinterpret_cast<const bf16x8*>(tile + PAGE_B + n16 * (HD * 2) + ch);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qh[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kbf, qh[s], s1, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, ql[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kbf, ql[s], s1, 0, 0, 0);
    }
    // Softmax in the exponent-2 domain on the raw scores: p = 2^(s c - m c), c = log2(e) / sqrt(h) > 0,
    // m the running row maximum of the raw scores.
    float sv[8];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      sv[r] = s0[r];
      sv[4 + r] = s1[r];
    }
    const bool masked = kb + 32 > free_end;           // wavefront-uniform: only the last tiles of a range
    bool vis[8];
    if (masked) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int tau = kb + 16 * (r >> 2) + 4 * g + (r & 3);
        vis[r] = (tau < key_end) && (tau <= lim);
        sv[r] = vis[r] ? sv[r] : NEG_BIG;
      }
    }
    float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    mx = row_max4(mx);
    const float m_new = fmaxf(m_run, mx);
    const float alpha = ex2((m_run - m_new) * scale_log2);
    const float mc = m_new * scale_log2;
    m_run = m_new;
    float p[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) p[r] = ex2(fmaf(sv[r], scale_log2, -mc));
    if (masked) {
#pragma unroll
      for (int r = 0; r < 8; ++r) p[r] = vis[r] ? p[r] : 0.f;
    }
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
    // Rescale the accumulators only when some row's running max moved (rare after the first tiles).
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        acc[db][0] *= alpha; acc[db][1] *= alpha; acc[db][2] *= alpha; acc[db][3] *= alpha;
      }
      acc_l[0] *= alpha; acc_l[1] *= alpha; acc_l[2] *= alpha; acc_l[3] *= alpha;
    }
    // Row sums ride on the matrix core: an all-ones "V row" accumulates sum_k p[k] of the lane's query
    // row, the (hi, lo) pair makes it exact to fp32, and no cross-lane reduction is needed.
    acc_l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf, acc_l, 0, 0, 0);
    acc_l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pfl, acc_l, 0, 0, 0);
    if (kb + 32 > key_end) {
      // Last tile of the range: V slots past it may hold junk (0 * NaN), blank them.
      uint32_t vm[4];
#pragma unroll
      for (int pg = 0; pg < 2; ++pg) {
        const int t0 = kb + 16 * pg + 4 * g;
        vm[2 * pg] = (t0 + 0 < key_end ? 0x0000FFFFu : 0u) | (t0 + 1 < key_end ? 0xFFFF0000u : 0u);
        vm[2 * pg + 1] = (t0 + 2 < key_end ? 0x0000FFFFu : 0u) | (t0 + 3 < key_end ? 0xFFFF0000u : 0u);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const uint2 va = *reinterpret_cast<const uint2*>(tile + 2 * PAGE_B + (db * 16 + n16) * 32 + 8 * g);
        const uint2 vb = *reinterpret_cast<const uint2*>(tile + 3 * PAGE_B + (db * 16 + n16) * 32 + 8 * g);
        uint4 vv;
        vv.x = va.x & vm[0];
        vv.y = va.y & vm[1];
        vv.z = vb.x & vm[2];
        vv.w = vb.y & vm[3];
        const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pfl, acc[db], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const uint2 va = *reinterpret_cast<const uint2*>(tile + 2 * PAGE_B + (db * 16 + n16) * 32 + 8 * g);
        const uint2 vb = *reinterpret_cast<const uint2*>(tile + 3 * PAGE_B + (db * 16 + n16) * 32 + 8 * g);
        uint4 vv;
        vv.x = va.x;
        vv.y = va.y;
        vv.z = vb.x;
        vv.w = vb.y;
        const bf16x8 vf = __builtin_bit_cast(bf16x8, vv);
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pfl, acc[db], 0, 0, 0);
      }
    }
  }

  // ---- finish: every copy has landed and every wavefront is past its last read before LDS is reused
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  asm volatile("s_barrier" ::: "memory");
  const float l_run = acc_l[0];
  const float m_fin = m_run * scale_log2;             // running maximum in the exponent-2 domain, as the merges use it

  if (KP == 1) {                                      // the wavefront owns its rows outright
    if (row < nrows) {
      const float inv = 1.0f / l_run;
      if (it.part < 0) {
        const size_t at = ((size_t)(it.tok0 + row / G) * Hq + kh * G + row % G) * HD + 4 * g;
#pragma unroll
        for (int db = 0; db < DB; ++db)
          store_pair(a.o + at + db * 16, a.o_lo + at + db * 16, acc[db][0] * inv, acc[db][1] * inv,
                     acc[db][2] * inv, acc[db][3] * inv);
      } else {
        const size_t base = ((size_t)it.part * Hkv + kh) * 64 + row;
#pragma unroll
        for (int db = 0; db < DB; ++db)
          *reinterpret_cast<float4*>(a.part_o + base * HD + db * 16 + 4 * g) =
              make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
        if (g == 0) *reinterpret_cast<float2*>(a.part_ml + base * 2) = make_float2(m_fin, l_run);
      }
    }
    return;
  }

  // ---- merge the key phases of each row block through LDS
  float* s_o = reinterpret_cast<float*>(lds);         // [4 wavefronts][16][OSTRIDE]
  float* s_m = s_o + 4 * 16 * OSTRIDE;                // [4][16]
  float* s_l = s_m + 64;                              // [4][16]
  if (g == 0) {
    s_m[wave * 16 + n16] = m_fin;
    s_l[wave * 16 + n16] = l_run;
  }
  __syncthreads();
  {
    float ms = NEG_BIG;
#pragma unroll
    for (int q = 0; q < KP; ++q) ms = fmaxf(ms, s_m[(q * RBN + rb) * 16 + n16]);
    const float f = ex2(m_fin - ms);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      *reinterpret_cast<float4*>(s_o + ((size_t)wave * 16 + n16) * OSTRIDE + db * 16 + 4 * g) =
          make_float4(acc[db][0] * f, acc[db][1] * f, acc[db][2] * f, acc[db][3] * f);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < nrows * (HD / 4); e += 256) {
    const int orow = e / (HD / 4), d4 = (e % (HD / 4)) * 4;
    const int orb = orow >> 4, r16 = orow & 15;
    float ms = NEG_BIG;
#pragma unroll
    for (int q = 0; q < KP; ++q) ms = fmaxf(ms, s_m[(q * RBN + orb) * 16 + r16]);
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
#pragma unroll
    for (int q = 0; q < KP; ++q) {
      const int w = q * RBN + orb;
      const float4 v = *reinterpret_cast<const float4*>(s_o + ((size_t)w * 16 + r16) * OSTRIDE + d4);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
      l += s_l[w * 16 + r16] * ex2(s_m[w * 16 + r16] - ms);
    }
    if (it.part < 0) {
      const float inv = 1.0f / l;
      const size_t at = ((size_t)(it.tok0 + orow / G) * Hq + kh * G + orow % G) * HD + d4;
      store_pair(a.o + at, a.o_lo + at, sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
    } else {
      const size_t base = ((size_t)it.part * Hkv + kh) * 64 + orow;
      *reinterpret_cast<float4*>(a.part_o + base * HD + d4) = sum;
      if (d4 == 0) *reinterpret_cast<float2*>(a.part_ml + base * 2) = make_float2(ms, l);
    }
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

// One launch covers every work item; the block picks the code path for its row-group size.
template <int HD>
__global__ __launch_bounds__(256) void attn_kernel(AttnLaunch a, float scale_log2) {
  const AttnItem it = a.items[blockIdx.x];
  const int rows = it.ntok * (a.Hq / a.Hkv);
  if (rows <= 32)                       // up to two 16-row blocks x two key phases
    attn_body<HD, 2>(a, it, scale_log2);
  else                                  // four 16-row blocks, every wavefront sees every key
    attn_body<HD, 4>(a, it, scale_log2);
}

template <int HD>
static hipError_t launch_hd(const AttnLaunch& a, hipStream_t s) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  const int n = a.class_begin[3];
  if (n > 0) {
    const size_t lds_ring = (size_t)5 * 4 * SY_PAGE * HD * 2;              // 5 tiles of 32 keys
    const size_t lds_merge = (size_t)(4 * 16 * (HD + 4) + 128) * sizeof(float);
    const size_t lds = lds_ring > lds_merge ? lds_ring : lds_merge;
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<HD>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    attn_kernel<HD><<<dim3(n, a.Hkv), 256, lds, s>>>(a, scale_log2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
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
