// Paged ragged chunk attention for the partial prefill of draft chunks:
//   o = softmax(q K^T / sqrt(h)) V          (attention definition, Section 3.2)
// where chunk row j of request i sees keys 0..L_i+j: the whole cached prefix and,
// causally, the chunk itself (a prefill "with an existing KV-cached prefix",
// Section 3.4).  Grouped-query attention: q head hq reads KV head hq / G.
//
// Design (gfx950, 64-wide wavefronts):
//   * A stream is (request, group of <= 64 query rows = chunk tokens x G heads of one KV head) with all
//     the keys those rows see.  The host lays the streams of a call end to end, cuts the line into equal
//     shares of modelled cost, one per persistent block (two blocks per compute unit), and writes each
//     block's share out as a flat program of 32-key tile positions.  A stream that ends up in several
//     blocks leaves partial results that attn_combine_kernel merges; most streams are whole.
//   * Every position flows through one LDS ring of five 16 KB slots (8 KB at head_dim 64), filled by
//     asynchronous global->LDS copies (global_load_lds_dwordx4; a K/V page tile is 4 KB contiguous in
//     HBM, every copy instruction moves one coalesced kilobyte and needs no registers).  The ring runs
//     3-4 positions ahead of the arithmetic and straight across stream boundaries: a new stream's
//     query rows travel through the ring too, as positions of their own, so nothing in the block ever
//     waits for a load that was not issued several tiles earlier.  Each K/V byte leaves HBM once per
//     KV head and is shared by all G x k_i query rows.
//   * The four wavefronts split the row group into 16-row blocks (RBN = 4), or for groups of <= 32 rows
//     into 2 row blocks x 2 key phases (RBN = 2: two tile positions per iteration, merged through LDS
//     when the stream's share ends).
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: the A operand is
//     a K page fragment (lane = (slot, 16-byte dim chunk); chunks are XOR-swizzled by slot on the
//     way into LDS so the reads are bank-conflict free), the B operand is Q in registers.  The
//     result leaves each lane with 4 keys x 1 query row: softmax statistics are per-lane plus two
//     cross-lane exchanges, and the probabilities are already the B operand of O^T = V^T P^T.
//     V pages are stored dim-major ([dim][slot]), which makes the A operand of that product plain
//     8-byte LDS reads.  Row sums ride on the matrix core (an all-ones A operand).
//   * q and the probabilities enter the matrix cores as bf16 (hi, lo) pairs (two MFMAs per
//     product, K/V fragments reused; the cache is bf16, so these products stay bf16), and o leaves as
//     the fp16 pair the output projection consumes: single bf16 terms here cost the logits of a deep
//     decoder an order of magnitude in accuracy.
//   * The compiler cannot see the asynchronous copies (inline assembly), and any vector-memory load it
//     emits itself inside the loop would be guarded by a wait that drains them.  The loop's own small
//     reads -- program entries, stream descriptors -- therefore go through the constant address space
//     (scalar loads, which wait on a different counter), one iteration ahead of their use.
#include "common.h"

#define NEG_BIG (-1e30f)

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
#define SY_CONST_AS __attribute__((address_space(4)))

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum over the four lanes l, l^16, l^32, l^48 that hold one query row, with gfx950's lane-swap
// instructions (plain vector ALU work, no trip through the LDS crossbar).
__device__ __forceinline__ float row_max4(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// Four consecutive outputs as the fp16 (hi, lo) pair of SY_O_SCALE x value: 8 bytes to each array.
__device__ __forceinline__ void store_pair(uint16_t* hi, uint16_t* lo, float a, float b, float c, float d, bool lo_off) {
  uint2 h, l;
  split_f16x2(a * SY_O_SCALE, b * SY_O_SCALE, h.x, l.x);
  split_f16x2(c * SY_O_SCALE, d * SY_O_SCALE, h.y, l.y);
  *reinterpret_cast<uint2*>(hi) = h;
  *reinterpret_cast<uint2*>(lo) = lo_off ? make_uint2(0u, 0u) : l;
}

// Four consecutive outputs of token row `tok`, columns col .. col + 3 of its Hq x hd values: to the two arrays of
// the pair, or (o_paired) to the one array [T][Hq hd / 32][hi 32 | lo 32] the output projection then reads.
__device__ __forceinline__ void store_o(const AttnLaunch& a, size_t tok, int col, float v0, float v1, float v2, float v3) {
  const size_t width = (size_t)a.Hq * a.hd;
  if (a.o_paired) {
    uint16_t* at = a.o + tok * 2 * width + pair_col(col);
    store_pair(at, at + 32, v0, v1, v2, v3, (a.lo_off & 2) != 0);
  } else {
    store_pair(a.o + tok * width + col, a.o_lo + tok * width + col, v0, v1, v2, v3, (a.lo_off & 2) != 0);
  }
}

// Asynchronous 16-byte-per-lane copy global -> LDS; lane i lands at lds_addr + 16 i (m0 carries the
// wavefront-uniform LDS address).
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
// (the wait count is an immediate, so the few possible values are spelled out; `tiles` is
// wavefront-uniform).
template <int IPP>
__device__ __forceinline__ void wait_copies(int tiles) {
  if (tiles >= 3) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(3 * IPP) : "memory");
  } else if (tiles == 2) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * IPP) : "memory");
  } else if (tiles == 1) {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(1 * IPP) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  }
}

template <int HD, int RBN>
__device__ __forceinline__ void attn_body(const AttnLaunch& a, const int pos_begin, const int n_pos, float scale_log2) {
  constexpr int KP = 4 / RBN;                       // tile positions consumed per iteration
  constexpr int NT = 5;                             // ring slots: position p lives in slot p % NT; NT - KP
                                                    // positions stay in flight behind the KP being consumed
  constexpr int KS = HD / 32, DB = HD / 16;
  constexpr int PAGE_B = SY_PAGE * HD * 2;          // bytes of one K or V page tile
  constexpr int TILE_B = 4 * PAGE_B;                // K page a, K page b, V page a, V page b -- or, for a
                                                    // query position: [hi | lo] x 32 rows x HD
  constexpr int IPP = PAGE_B / 1024;                // copy instructions per wavefront and position
  constexpr int CPS = HD / 8;                       // 16-byte chunks per K slot / query row
  constexpr int RPC = 64 / CPS;                     // query rows per copy instruction
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n16 = lane & 15, g = lane >> 4;
  const int rb = wave % RBN, kp = wave / RBN;
  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds;
  const SY_CONST_AS i32x4* prog = reinterpret_cast<const SY_CONST_AS i32x4*>((uintptr_t)(a.prog + pos_begin));
  const SY_CONST_AS i32x8* units = reinterpret_cast<const SY_CONST_AS i32x8*>((uintptr_t)a.units);
  const int n_iter = n_pos / KP;                    // the host pads every share to a multiple of KP

  // ---- copies: of a K/V position this wavefront copies page tile `wave` (K page a, K page b, V page a,
  //      V page b), of a query position 16 rows of the hi (wave 0, 1) or lo (wave 2, 3) part; IPP
  //      instructions of one kilobyte each.  K chunks are swizzled by slot, Q chunks by row, V halves by row.
  int c_off[IPP];
#pragma unroll
  for (int j = 0; j < IPP; ++j) {
    if (wave < 2) {
      const int slot = j * (1024 / (HD * 2)) + lane / CPS;
      c_off[j] = slot * HD + (((lane % CPS) ^ kswz<HD>(slot)) << 3);
    } else {
      // V rows ([dim][16 slots], 32 bytes) keep their place; the two 16-byte halves of every second group of
      // 8 rows are swapped, so that rows d and d + 8, which share banks, are read from different ones
      const int pos = j * 64 + lane, vrow = pos >> 1;
      c_off[j] = (vrow * 2 + ((pos & 1) ^ ((vrow >> 3) & 1))) * 8;
    }
  }
  const size_t page_elems = (size_t)Hkv * SY_PAGE * HD;
  const bf16_t* my_pool = wave < 2 ? a.k_layer : a.v_layer;
  const bf16_t* my_q = wave < 2 ? a.q : a.q_lo;

  auto issue = [&](int p, const i32x4 e) {          // e = prog[p]
    const int kind = e[0] & ATTN_POS_KIND_MASK;
    const uint32_t dst = lds_base + (uint32_t)(p % NT) * TILE_B + wave * PAGE_B;
    if (kind == ATTN_POS_KV) {                        // e[0] >> 4 = KV head, e[1] / e[2] = pages of the tile
      const int kh = e[0] >> 4;
      const bf16_t* src = my_pool + (size_t)((wave & 1) ? e[2] : e[1]) * page_elems + (size_t)kh * SY_PAGE * HD;
#pragma unroll
      for (int j = 0; j < IPP; ++j) copy_to_lds(src + c_off[j], dst + j * 1024);
    } else if (kind == ATTN_POS_Q) {
      // 32 rows from row0 of the stream's group: e[1] = first chunk token, e[2] = rows of the group,
      // e[3] = row0 | KV head << 8
      const int nrows = e[2], row0 = (e[3] & 255) + 16 * (wave & 1), kh = e[3] >> 8;
#pragma unroll
      for (int j = 0; j < IPP; ++j) {
        int row = row0 + j * RPC + lane / CPS;
        row = row < nrows ? row : nrows - 1;          // rows past the group: copies of its last row, never stored
        const int chunk = (lane % CPS) ^ kswz<HD>((j * RPC + lane / CPS) & 15);   // swizzled like the K slots
        const bf16_t* src = my_q + ((size_t)(e[1] + row / G) * Hq + kh * G + row % G) * HD + chunk * 8;
        copy_to_lds(src, dst + j * 1024);
      }
    }
    // padding position: nothing to copy.  The wait counts assume IPP copies per position, so a padding
    // position only makes a wait stricter than needed, never laxer.
  };

  // ---- prologue: fill the ring
#pragma unroll
  for (int p = 0; p < NT - KP; ++p)
    if (p < n_pos) issue(p, prog[p]);

  // ---- per-stream state
  bf16x8 qh[KS], ql[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    qh[s] = bf16x8{};
    ql[s] = bf16x8{};
  }
  float m_run = NEG_BIG;
  f32x4 acc_l = {0.f, 0.f, 0.f, 0.f};
  bf16x8 ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
  f32x4 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  // descriptor of the stream being consumed (scalar registers)
  int u_tok0 = 0, u_nrows = 0, u_lim0 = 0, u_key_end = 0, u_part = -1, u_kh = 0;
  int u_fresh = 0;                                    // this wavefront has not yet seen a tile of the stream

  // program entries of the coming iteration: the KP positions to consume and the KP positions to issue
  i32x4 ce[KP], ie[KP];
#pragma unroll
  for (int q = 0; q < KP; ++q) {
    ce[q] = prog[q];
    const int ip = NT - KP + q;
    ie[q] = prog[ip < n_pos ? ip : n_pos - 1];
  }

  for (int iter = 0; iter < n_iter; ++iter) {
    const int p0 = iter * KP;                         // first position of this iteration
    // Own copies of this iteration's positions have landed (the younger positions may stay in flight), own
    // LDS reads of the previous ones are done; the barrier extends both facts to the block.
    wait_copies<IPP>(max(0, min(n_pos, p0 + NT - KP) - (p0 + KP)));
    asm volatile("s_barrier" ::: "memory");
    i32x4 cur[KP];
#pragma unroll
    for (int q = 0; q < KP; ++q) {
      cur[q] = ce[q];
      const int ip = p0 + NT - KP + q;                // lands in a slot consumed last iteration
      if (ip < n_pos) issue(ip, ie[q]);
    }
    if (iter + 1 < n_iter) {                          // entries for the next iteration
#pragma unroll
      for (int q = 0; q < KP; ++q) {
        ce[q] = prog[p0 + KP + q];
        const int ip = p0 + NT + q;
        ie[q] = prog[ip < n_pos ? ip : n_pos - 1];
      }
    }

    if ((cur[0][0] & ATTN_POS_KIND_MASK) == ATTN_POS_Q) {
      // ---- a stream begins: 32 of its query rows sit in this position's slot; fetch this wavefront's
      //      fragments (B operand: lane = (row n16, dim chunk g)); at the first of them also the stream's
      //      descriptor, and reset the state
      const int row0 = cur[0][3] & 255;
      if (RBN == 2 || (rb >> 1) == (row0 >> 5)) {
        const unsigned char* slot = lds + (size_t)(p0 % NT) * TILE_B;
        const int r32 = (rb * 16 + n16) & 31;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const int ch = ((4 * s + g) ^ kswz<HD>(n16)) << 4;
          qh[s] = *reinterpret_cast<const bf16x8*>(slot + r32 * (HD * 2) + ch);
          ql[s] = *reinterpret_cast<const bf16x8*>(slot + 32 * (HD * 2) + r32 * (HD * 2) + ch);
        }
      }
      if (row0 == 0) {
        const i32x8 u = units[cur[0][0] >> 4];
        u_tok0 = u[0];
        u_nrows = u[1];
        u_lim0 = u[2];
        u_key_end = u[3];
        u_part = u[4];
        u_kh = u[5];
        // The accumulators are cleared at the stream's first tile, not here: cleared in this branch they
        // became loop-carried values with two definitions, and the compiler copied all 36 registers in and
        // out in every iteration of the tile loop.
        u_fresh = 1;
        m_run = NEG_BIG;
      }
      continue;
    }

    const i32x4 me = cur[kp < KP ? kp : KP - 1];      // this wavefront's position
    const int row = rb * 16 + n16;
    if ((me[0] & ATTN_POS_KIND_MASK) == ATTN_POS_KV) {
      const int kb = me[3];
      const int key_end = u_key_end;
      const int lim = row < u_nrows ? u_lim0 + row / G : 0x7FFFFFFF;   // last key this row may see
      const int free_end = min(key_end, u_lim0 + 1);                   // keys below need no mask
      const unsigned char* tile = lds + (size_t)((p0 + kp) % NT) * TILE_B;

      // All fragment reads of the tile go out first: the K fragments feed the score MFMAs as they arrive,
      // the V fragments land while the softmax runs (issued where they are needed, every group of MFMAs
      // would wait out an LDS round trip of its own).
      bf16x8 kf[KS][2];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int ch = ((4 * s + g) ^ kswz<HD>(n16)) << 4;
        kf[s][0] = *reinterpret_cast<const bf16x8*>(tile + n16 * (HD * 2) + ch);
        kf[s][1] = *reinterpret_cast<const bf16x8*>(tile + PAGE_B + n16 * (HD * 2) + ch);
      }
      uint4 vf[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int piece = 16 * ((g >> 1) ^ (n16 >> 3)) + 8 * (g & 1);      // see the copy: halves swapped in rows 8..15
        const uint2 va = *reinterpret_cast<const uint2*>(tile + 2 * PAGE_B + (db * 16 + n16) * 32 + piece);
        const uint2 vb = *reinterpret_cast<const uint2*>(tile + 3 * PAGE_B + (db * 16 + n16) * 32 + piece);
        vf[db] = make_uint4(va.x, va.y, vb.x, vb.y);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][0], qh[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][1], qh[s], s1, 0, 0, 0);
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][0], ql[s], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[s][1], ql[s], s1, 0, 0, 0);
      }
      // Softmax in the exponent-2 domain on the raw scores: p = 2^(s c - m c), c = log2(e) / sqrt(h) > 0,
      // m the running row maximum of the raw scores.
      float sv[8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        sv[r] = s0[r];
        sv[4 + r] = s1[r];
      }
      const bool masked = kb + 32 > free_end;           // wavefront-uniform: only the last tiles of a stream
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
      // The reference m only has to keep 2^(s c - m c) in range, it need not be the exact running maximum:
      // it moves when a score exceeds it by more than 2^8 in the exponent.  Moving it means rescaling 36
      // accumulator registers, and an exact running maximum moves in most tiles of a short context.
      const float m_new = (mx - m_run) * scale_log2 > 8.0f ? mx : m_run;
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
      if (a.lo_off & 1) pl = make_uint4(0u, 0u, 0u, 0u);   // ablation of the probabilities' low part (block-uniform)
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pk);
      const bf16x8 pfl = __builtin_bit_cast(bf16x8, pl);
      // Rescale the accumulators only when some row's reference moved (the first tile, then hardly ever).
      if (u_fresh) {
        // first tile of the stream for this wavefront: what the previous stream left goes, by assignment (a
        // product with alpha = 0 would keep an inf or NaN of a request with bad data alive in the next one)
        u_fresh = 0;
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc_l = f32x4{0.f, 0.f, 0.f, 0.f};
      } else if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
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
      // O^T += V^T P^T.  The two arms repeat the MFMAs so that the blanked fragments of the rare arm are not
      // merged with the plain ones in registers (that merge cost 24 copies per tile on the common arm).
      if (kb + 32 > key_end) {
        // Last tile of the stream: V slots past it may hold junk (0 * NaN), blank them.
        uint32_t vm[4];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
          const int t0 = kb + 16 * pg + 4 * g;
          vm[2 * pg] = (t0 + 0 < key_end ? 0x0000FFFFu : 0u) | (t0 + 1 < key_end ? 0xFFFF0000u : 0u);
          vm[2 * pg + 1] = (t0 + 2 < key_end ? 0x0000FFFFu : 0u) | (t0 + 3 < key_end ? 0xFFFF0000u : 0u);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const uint4 vb = make_uint4(vf[db].x & vm[0], vf[db].y & vm[1], vf[db].z & vm[2], vf[db].w & vm[3]);
          const bf16x8 v8 = __builtin_bit_cast(bf16x8, vb);
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, pf, acc[db], 0, 0, 0);
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, pfl, acc[db], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 v8 = __builtin_bit_cast(bf16x8, vf[db]);
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, pf, acc[db], 0, 0, 0);
          acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v8, pfl, acc[db], 0, 0, 0);
        }
      }
    }

    if (!(cur[0][0] & ATTN_POS_LAST_BIT)) continue;     // block-uniform: set on the iteration's first position

    // ---- the stream's share in this block ends here: write its result
    const bool idle = u_fresh != 0;                     // this wavefront saw no tile of the stream: leftovers
    float l_run = idle ? 0.f : acc_l[0];
    float m_fin = m_run * scale_log2;                   // running maximum in the exponent-2 domain
    if (KP == 2) {
      // Merge the two key phases through the two slots just consumed: nothing is copied into them before
      // the next iteration's barrier.  Phase 1 parks (acc, m, l), phase 0 folds them in.
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      asm volatile("s_barrier" ::: "memory");           // every wavefront is done reading both slots
      float* park = reinterpret_cast<float*>(lds + (size_t)((p0 + rb) % NT) * TILE_B);   // [DB * 4 + 2][64 lanes]
      if (kp == 1) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 4; ++r) park[(db * 4 + r) * 64 + lane] = idle ? 0.f : acc[db][r];
        park[(DB * 4) * 64 + lane] = m_fin;
        park[(DB * 4 + 1) * 64 + lane] = l_run;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      asm volatile("s_barrier" ::: "memory");
      if (kp == 0) {
        const float m1 = park[(DB * 4) * 64 + lane], l1 = park[(DB * 4 + 1) * 64 + lane];
        const float ms = fmaxf(m_fin, m1);
        const float f0 = ex2(m_fin - ms), f1 = ex2(m1 - ms);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[db][r] = acc[db][r] * f0 + park[(db * 4 + r) * 64 + lane] * f1;
        l_run = l_run * f0 + l1 * f1;
        m_fin = ms;
      }
    }
    if (kp == 0 && row < u_nrows) {
      if (u_part < 0) {
        const float inv = 1.0f / l_run;
        const size_t tok = (size_t)(u_tok0 + row / G);
        const int col = (u_kh * G + row % G) * HD + 4 * g;
#pragma unroll
        for (int db = 0; db < DB; ++db)
          store_o(a, tok, col + db * 16, acc[db][0] * inv, acc[db][1] * inv, acc[db][2] * inv, acc[db][3] * inv);
        if (a.row_ml && g == 0)
          a.row_ml[(size_t)(u_tok0 + row / G) * Hq + u_kh * G + row % G] = make_float2(m_fin, l_run);
      } else {
        const size_t base = (size_t)u_part * 64 + row;
#pragma unroll
        for (int db = 0; db < DB; ++db)
          *reinterpret_cast<float4*>(a.part_o + base * HD + db * 16 + 4 * g) =
              make_float4(acc[db][0], acc[db][1], acc[db][2], acc[db][3]);
        if (g == 0) *reinterpret_cast<float2*>(a.part_ml + base * 2) = make_float2(m_fin, l_run);
      }
    }
  }
  // every copy has landed before the block's LDS is released
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
}

// Merge the partial results of a stream that was cut across blocks:
//   o = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// (Merging inside attn_kernel -- the block that publishes a stream's last partial does it, found with an
// arrival counter -- was tried: correct, but the device-scope release and acquire it needs write back and
// invalidate the whole L2 of the block's XCD, once per block, and the kernel took twice as long.)
// Grid: (cuts, 8); a thread merges at most one 16-byte piece of one row, so all its loads are in flight
// together (the kernel is latency, not bandwidth).
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnLaunch a) {
  const AttnCut c = a.cuts[blockIdx.x];
  const int HD = a.hd, Hq = a.Hq, Hkv = a.Hkv, G = Hq / Hkv;
  for (int e = blockIdx.y * 256 + threadIdx.x; e < c.nrows * (HD / 4); e += 256 * gridDim.y) {
    const int row = e / (HD / 4), d4 = (e % (HD / 4)) * 4;
    float M = NEG_BIG;
    for (int s = 0; s < c.nsplit; ++s) M = fmaxf(M, a.part_ml[((size_t)(c.part0 + s) * 64 + row) * 2]);
    float4 sum = {0.f, 0.f, 0.f, 0.f};
    float l = 0.f;
    for (int s = 0; s < c.nsplit; ++s) {
      const size_t base = (size_t)(c.part0 + s) * 64 + row;
      const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + base * 2);
      const float w = ex2(ml.x - M);
      const float4 v = *reinterpret_cast<const float4*>(a.part_o + base * HD + d4);
      sum.x += w * v.x; sum.y += w * v.y; sum.z += w * v.z; sum.w += w * v.w;
      l += w * ml.y;
    }
    const float inv = 1.0f / l;
    store_o(a, (size_t)(c.tok0 + row / G), (c.kh * G + row % G) * HD + d4, sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
    if (a.row_ml && d4 == 0) a.row_ml[(size_t)(c.tok0 + row / G) * Hq + c.kh * G + row % G] = make_float2(M, l);
  }
}

// One persistent block per share of the program; the share's row-group class picks the code path.
template <int HD>
__global__ __launch_bounds__(256) void attn_kernel(AttnLaunch a, float scale_log2) {
  const AttnShare sh = a.shares[blockIdx.x];
  if (sh.n_pos <= 0) return;
  if (sh.rbn == 2)                      // two 16-row blocks x two key phases
    attn_body<HD, 2>(a, sh.pos_begin, sh.n_pos, scale_log2);
  else                                  // four 16-row blocks, every wavefront sees every key
    attn_body<HD, 4>(a, sh.pos_begin, sh.n_pos, scale_log2);
}

template <int HD>
static hipError_t launch_hd(const AttnLaunch& a, hipStream_t s) {
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  if (a.n_shares > 0) {
    const size_t lds = (size_t)5 * 4 * SY_PAGE * HD * 2;              // the ring's five slots
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<HD>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    attn_kernel<HD><<<a.n_shares, 256, lds, s>>>(a, scale_log2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (a.n_cuts > 0) {
    attn_combine_kernel<<<dim3(a.n_cuts, 8), 256, 0, s>>>(a);
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
