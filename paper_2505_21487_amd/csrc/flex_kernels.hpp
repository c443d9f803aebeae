// Second MFMA decode-attention kernel, for the head shapes the tuned kernel has
// no variant for: small tied states (GTA with d_h 64 / 96 and a RoPE key of
// d_h / 2), latent heads of 128 dims, and grouped-query attention with keys
// and values in separate caches (the baseline GTA is compared with, paper
// Section 3.3.1).  Same operation as everywhere in this library:
//     score = scale * (q_nope . key[:DN] + q_rope . rope_key),  out = softmax(score) . value[:DV]
// with key = the first DN dims of the value row (GLA / GTA) or a row of a key
// cache of its own (SEPK).
//
// These shapes have few query rows per group and little arithmetic per cache
// byte, so the design is the simplest one that streams well: ONE WAVE per piece
// of work, no cooperation between waves, hence no barriers.  The key tiles of
// all sequences form one flat list, cut into equal chunks; a wave takes one
// chunk for one (group block, block of 16 query rows) and walks through the
// sequences its chunk touches, so ragged batches balance by construction.  It
// moves its tiles of 32 tokens global -> LDS with direct-to-LDS loads of whole
// cache rows through its own ring of stages (the fetch runs ahead across the
// boundaries between sequences) and works in the transposed form on 16x16x16
// bf16 MFMAs:
//     S^T = K . Q^T       A operand: key rows from LDS (8 bytes per lane), B: query fragments in registers
//     O^T += V^T . P^T    A: value tile read with transposing LDS reads, B: the score accumulators, which
//                         already have the B-operand layout (key 4 * (lane / 16) + i of query row lane % 16)
// Softmax statistics of a row live in the four lanes {r, r + 16, r + 32, r + 48}.
// Weights are taken relative to a lazily moved reference, rounded to bf16 and
// normalised by the sum of the rounded weights (a ones-valued MFMA); a tile in
// which one weight holds more than a quarter of its row's running sum gets a
// second pass with the rounding residuals, so no row, however few keys carry
// it, is limited by the weight rounding.  16-byte chunks of a cache row are
// rotated by the row index inside LDS (slot = (chunk + row) mod chunks per row)
// so that reads of one column over 16 rows spread over the banks; each lane of
// a load fetches the chunk whose rotated home is its slot.
//
// A sequence that one chunk holds entirely is written directly.  Otherwise each
// chunk leaves its piece (16 rows x d_v fp32, normalised, + log-sum-exp) in one
// of its two slots, the waves holding a sequence's first and last piece note
// their chunk numbers, and flex_combine_kernel merges the pieces.
#pragma once

#include "common.hpp"
#include "tuned_device.hpp"

namespace gla {

typedef __attribute__((ext_vector_type(4))) short flex_s16x4_t;

__device__ __forceinline__ void flex_lds_read_b64(u32x2_t& dst, unsigned addr) {
  asm volatile("ds_read_b64 %0, %1" : "=v"(dst) : "v"(addr));
}
__device__ __forceinline__ void flex_lds_read_tr(u32x2_t& dst, unsigned addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(dst) : "v"(addr));
}
__device__ __forceinline__ void flex_lds_zero_b128(unsigned addr) {
  const u32x4_t z = {0, 0, 0, 0};
  asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(z) : "memory");
}
__device__ __forceinline__ void flex_tie(u32x2_t& x) { asm volatile("" : "+v"(x)); }
__device__ __forceinline__ float flex_max3(float a, float b, float c) {
  float r;  // (as an instruction of its own: fmaxf() first canonicalises every operand that comes out of an MFMA)
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
// MFMAs as asm with every operand in an architectural VGPR.  (Left to the compiler, the accumulators go
// to accumulation registers and are copied out and back around every piece of vector arithmetic on
// them, the scores of every tile included.)  The compiler does not see the matrix pipe's latency behind
// an asm statement: a result is read by other instructions only after flex_mfma_settle() on it.
// Back-to-back MFMAs that accumulate into the same registers need no gap.
__device__ __forceinline__ void flex_mfma0(f32x4_t& acc, const u32x2_t& a, const u32x2_t& b) {
  asm volatile("v_mfma_f32_16x16x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void flex_mfma(f32x4_t& acc, const u32x2_t& a, const u32x2_t& b) {
  asm volatile("v_mfma_f32_16x16x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// The same when an operand may have been written by the vector instruction just before (an MFMA reads
// a VGPR two wait states after a vector instruction wrote it, and the compiler, which keeps that gap
// for its own MFMAs, is free to place such an instruction directly in front of an asm statement).
__device__ __forceinline__ void flex_mfma_fresh(f32x4_t& acc, const u32x2_t& a, const u32x2_t& b) {
  asm volatile("s_nop 1\n\tv_mfma_f32_16x16x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// 4-pass MFMA result -> read or overwrite by a vector instruction: 7 wait states; 8 given
__device__ __forceinline__ void flex_mfma_settle(f32x4_t& a, f32x4_t& b) { asm volatile("s_nop 7" : "+v"(a), "+v"(b)); }
template <int N>
__device__ __forceinline__ void flex_mfma_settle(f32x4_t (&o)[N], f32x4_t& one) {
  asm volatile("s_nop 7" : "+v"(one));
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(o[i]));
}
template <int N>
__device__ __forceinline__ void flex_lds_wait_all(u32x2_t (&x)[N]) {
  // every LDS read issued so far has returned; tied to the registers so that no use moves ahead of it
#pragma unroll
  for (int i = 0; i < N; ++i) flex_tie(x[i]);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < N; ++i) flex_tie(x[i]);
}

// GPW: groups per wave.  With at most eight query rows per group two groups share the 16 rows of a wave
// (rows 0 .. 7 the first group, 8 .. 15 the second): each group's queries are zero in the other's rows,
// so the score MFMAs of both groups and of the shared RoPE key add up in ONE accumulator, the softmax
// arithmetic runs once on 16 full rows instead of twice on half-empty ones, and the RoPE-key tile is
// fetched and read once for both.  The value products keep one accumulator set per group (each holds
// all 16 rows against its group's values; only the group's own rows are stored).
template <int DN, int DR, int DV, bool SEPK, int GPW = 1>
struct FlexTraits {
  static constexpr int kVB = DV * 2, kKB = DN * 2, kRB = DR * 2;  // row bytes of the value / key / RoPE tiles
  static constexpr int kStage = 32 * (GPW * kVB + (SEPK ? kKB : 0) + kRB);
  // Ring stages per wave.  Small tiles: three stages in 20 KB, so that two workgroups (two waves per SIMD)
  // share a compute unit and one wave's LDS and MFMA latencies hide behind the other's work; larger
  // tiles: as many stages as 40 KB hold, at most six (one workgroup per compute unit).
  static constexpr int kNST = 3 * kStage <= 20 * 1024 ? 3 : (40 * 1024 / kStage) < 6 ? (40 * 1024 / kStage) : 6;
  static constexpr int loads(int rb) { return rb / 32; }  // load instructions (64 lanes x 16 bytes) for 32 rows of rb bytes
  static constexpr int kLPT = GPW * loads(kVB) + (SEPK ? loads(kKB) : 0) + loads(kRB);
  static_assert(GPW == 1 || (GPW == 2 && !SEPK), "two groups per wave: tied / latent states only");
  static_assert(kNST >= 2, "at least two stages");
  static_assert(kLPT * (kNST - 1) <= 63, "vmcnt range");
  static_assert(DN % 16 == 0 && DR % 16 == 0 && DV % 16 == 0 && (SEPK || DN <= DV), "dims");
  static_assert(kVB % 32 == 0 && kKB % 32 == 0 && kRB % 32 == 0, "a tile is a whole number of load instructions");
};

// LANE: pages of fewer than 32 tokens.  The rows of a tile then lie in up to 32 pages, so every lane forms
// the address of the row it fetches in each load from that row's page id, taken with a cross-lane read
// from the page ids the wave holds: an aligned window of 256 table entries in four registers, one entry
// per lane each (a tile's pages lie in one aligned block of 32 entries, hence in one of the registers).
// With larger pages a tile lies inside one page and has one base address.
template <int DN, int DR, int DV, bool SEPK, int GPW = 1, bool LANE = false>
__global__ __launch_bounds__(256) void flex_main_kernel(DevParams p) {
  using FT = FlexTraits<DN, DR, DV, SEPK, GPW>;
  constexpr int NST = FT::kNST, STAGE = FT::kStage, LPT = FT::kLPT;
  constexpr int VB = FT::kVB, KB = FT::kKB, RB = FT::kRB;
  constexpr int OFF_K = GPW * 32 * VB, OFF_R = OFF_K + (SEPK ? 32 * KB : 0);  // tile offsets inside a stage
  constexpr int NKN = DN / 16, NKR = DR / 16;                                  // contraction steps of the scores
  constexpr int NDB = DV / 16;                                                 // 16-dim output blocks
  constexpr int NLV = FT::loads(VB), NLK = SEPK ? FT::loads(KB) : 0, NLR = FT::loads(RB);
  constexpr int NKF = GPW * NKN + NKR;  // key operands per 16-key block
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * NST * STAGE];
  static_assert(sizeof(smem) <= 160 * 1024, "LDS capacity");

  const int lane = threadIdx.x & 63;
  const int wave = uniform((int)threadIdx.x >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const unsigned ring_addr =
      (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + (unsigned)(wave * (NST * STAGE));

  // ---- this wave's share of the work.  A "strand" is one (group block, block of 16 query rows); every
  //      strand walks the same flat list of key tiles (all tiles of sequence 0, of sequence 1, ...), cut
  //      into num_chunks equal chunks, one wave per (chunk, strand): ragged batches balance by
  //      construction.  Strands are numbered fastest, group blocks first, so the waves of a workgroup
  //      fetch the SAME shared RoPE-key rows at about the same time (one trip to HBM for all of them).
  const int rows_group = p.g_q * p.T;
  const unsigned HB = (unsigned)p.h_c / GPW;             // group blocks
  const unsigned NSTR = HB * (unsigned)p.flex_rb;        // strands
  const unsigned unit = blockIdx.x * 4u + (unsigned)wave;  // (the host keeps the number of waves below 2^31)
  if (unit >= NSTR * (unsigned)p.num_chunks) return;
  const int chunk = (int)(unit / NSTR);
  const int strand = (int)(unit - (unsigned)chunk * NSTR);
  const int rb = (int)((unsigned)strand / HB);
  const int g0 = (strand - rb * (int)HB) * GPW;  // first group of this wave
  const int L_first = lane < p.B ? p.seq_lens[lane] : 0;
  const int incl0 = wave_incl_scan(tiles_of<32>(L_first));
  const int total = total_tiles<32>(p, 1, lane, incl0);
  const int C = p.chunk_tiles > 0 ? p.chunk_tiles : max(1, (int)(((unsigned)total + (unsigned)p.num_chunks - 1) / (unsigned)p.num_chunks));
  const int pos0 = chunk * C;  // (the host keeps num_chunks * max tiles per chunk below 2^31)
  if (pos0 >= total) return;
  int left = min(C, total - pos0);  // tiles of this chunk not yet worked on
  // a cache larger than the chip's last-level cache is fetched with the streaming hint (read once per call, it
  // would only push the page table, the queries and the partial results out of the caches)
  const bool stream_hint = (int64_t)total * 32 * (p.h_c * (VB + (SEPK ? KB : 0)) + RB) > p.stream_min_bytes;

  // ---- the query row of this lane within its group (rows past the end repeat the last one, never stored)
  const int jg = GPW == 2 ? r16 >> 3 : 0;                  // which of the wave's groups the row belongs to
  const int R = GPW == 2 ? (r16 & 7) : rb * 16 + r16;      // row within the group
  const bool row_valid = R < rows_group;
  const int Rc = row_valid ? R : rows_group - 1;
  const int t = Rc / p.g_q;
  const int h = (g0 + jg) * p.g_q + (Rc - t * p.g_q);

  // ---- tile loads.  A tile of 32 rows of LPR 16-byte chunks is 32 * LPR consecutive LDS slots, 64 per
  //      load instruction (LPR is even: every instruction is full).  Slot n belongs to row n / LPR and holds
  //      the chunk that rotation by the row index sends there; the byte offset of that chunk from the tile's
  //      first row is all a lane needs per load, and it is the same for every tile.
  unsigned goff_v[NLV], goff_k[NLK > 0 ? NLK : 1], goff_r[NLR > 0 ? NLR : 1];
  auto lane_offsets = [&](auto rbc, auto& goff) {
    constexpr int RBY = decltype(rbc)::value;
    constexpr int LPR = RBY / 16;
    static_assert(LPR % 2 == 0, "whole load instructions");
#pragma unroll
    for (int j = 0; j < LPR / 2; ++j) {
      const int n = j * 64 + lane, row = n / LPR, slot = n % LPR;
      int chunk_i = slot - row % LPR;
      chunk_i += chunk_i < 0 ? LPR : 0;
      goff[j] = (unsigned)(row * RBY + chunk_i * 16);
    }
  };
  lane_offsets(std::integral_constant<int, VB>{}, goff_v);
  if constexpr (SEPK) lane_offsets(std::integral_constant<int, KB>{}, goff_k);
  if constexpr (DR > 0) lane_offsets(std::integral_constant<int, RB>{}, goff_r);
  // LANE: the same offsets split into the row of the tile and the byte offset inside that row
  int row_v[NLV] = {}, row_k[NLK > 0 ? NLK : 1] = {}, row_r[NLR > 0 ? NLR : 1] = {};
  if constexpr (LANE) {
#pragma unroll
    for (int i = 0; i < NLV; ++i) row_v[i] = (int)(goff_v[i] / VB), goff_v[i] -= (unsigned)row_v[i] * VB;
    if constexpr (SEPK) {
#pragma unroll
      for (int i = 0; i < NLK; ++i) row_k[i] = (int)(goff_k[i] / KB), goff_k[i] -= (unsigned)row_k[i] * KB;
    }
    if constexpr (DR > 0) {
#pragma unroll
      for (int i = 0; i < NLR; ++i) row_r[i] = (int)(goff_r[i] / RB), goff_r[i] -= (unsigned)row_r[i] * RB;
    }
  }
  const unsigned char* const state_b = (const unsigned char*)(p.state + g0 * p.st_s[1]);
  const unsigned char* const key_b = SEPK ? (const unsigned char*)(p.kstate + g0 * p.k_s[1]) : nullptr;
  const unsigned char* const rope_b = (const unsigned char*)p.rope;

  // ---- two cursors over the chunk: `cur`, the tile being worked on, and `pre`, NST - 1 tiles ahead,
  //      the tile being fetched (it crosses into the next sequence without the ring running dry)
  TileCursor cur = locate_tile<32>(p, 1, pos0, lane, L_first, incl0);
  TileCursor pre = cur;
  int pre_left = left;
  const int lgP = p.lg_page;             // page size is a power of two (of at least 32 tokens unless LANE)
  const int tpp_lg = lgP - 5;            // log2(tiles per page)
  // 64 page ids of sequence pt_b, one per lane: from page pt_base on (LANE: the register of the window below
  // that serves the tile being fetched; pt_base is then the window's index)
  int pt_b = -1, pt_base = 0, pt_vec = 0;
  const unsigned char *src_v = state_b, *src_k = key_b, *src_r = rope_b;
  int ln_tok0 = 0, ln_last = 0;          // LANE: first token of the tile being fetched, last page its sequence holds
  int pt_w0 = 0, pt_w1 = 0, pt_w2 = 0, pt_w3 = 0;  // LANE: entries [256 * pt_base, +256) of the page-table row of sequence pt_b
  // fetch the tile at `pre` into a stage and step `pre`; past the end of the chunk: the last tile again
  // (keeps the count of loads in flight the same in every iteration)
  auto issue_next = [&](int stage) {
    if constexpr (LANE) {
      if (pre_left > 0) {
        // Rows past the end of the sequence take its last page (valid memory, masked later; at or after the
        // tile's first page, so inside the same block of entries), never an unused table entry.
        ln_tok0 = pre.j << 5;
        ln_last = (pre.L - 1) >> lgP;
        const int pg0 = ln_tok0 >> lgP;
        if (pre.b != pt_b || (pg0 >> 8) != pt_base) {  // (every eighth tile at one token per page; the wave waits for it)
          pt_b = pre.b;
          pt_base = pg0 >> 8;
          const int32_t* row = p.page_table + (int64_t)pre.b * p.max_pages;
          const int e0 = pt_base * 256 + lane;
          load_i32x4_sync(pt_w0, pt_w1, pt_w2, pt_w3, row + min(e0, ln_last), row + min(e0 + 64, ln_last),
                          row + min(e0 + 128, ln_last), row + min(e0 + 192, ln_last));
        }
        const int reg = (pg0 >> 6) & 3;  // (uniform)
        pt_vec = reg == 0 ? pt_w0 : reg == 1 ? pt_w1 : reg == 2 ? pt_w2 : pt_w3;
        if (--pre_left > 0) advance<32>(p, 1, pre);
      }
    } else if (pre_left > 0) {
      const int pg = pre.j >> tpp_lg;
      if (pre.b != pt_b || pg < pt_base || pg >= pt_base + 64) {
        pt_b = pre.b;
        pt_base = pg;
        pt_vec = load_i32_sync(p.page_table + (int64_t)pre.b * p.max_pages + min(pg + lane, p.max_pages - 1));
      }
      const int64_t page = __builtin_amdgcn_readlane(pt_vec, pg - pt_base);
      const int tok = (pre.j << 5) & ((1 << lgP) - 1);  // first token of the tile inside its page
      src_v = state_b + (page * p.st_s[0] + (int64_t)tok * DV) * 2;
      if constexpr (SEPK) src_k = key_b + (page * p.k_s[0] + (int64_t)tok * DN) * 2;
      if constexpr (DR > 0) src_r = rope_b + (page * p.rp_s[0] + (int64_t)tok * DR) * 2;
      if (--pre_left > 0) advance<32>(p, 1, pre);
    }
    unsigned char* dst = smem + wave * (NST * STAGE) + stage * STAGE;
    // LANE: element offset of tile row `row` in a pool with pages of `page_stride` elements and rows of `dims`
    auto row_at = [&](int row, int64_t page_stride, int dims) -> int64_t {
      const int t = ln_tok0 + row;
      const int e = min(t >> lgP, ln_last);
      const int64_t id = __builtin_amdgcn_ds_bpermute((e & 63) << 2, pt_vec);
      return id * page_stride + (int64_t)(t & ((1 << lgP) - 1)) * dims;
    };
    auto loads = [&](auto hint) {
      constexpr int aux = decltype(hint)::value;
#pragma unroll
      for (int i = 0; i < NLV; ++i) {
        const unsigned char* src = src_v;
        if constexpr (LANE) src = state_b + row_at(row_v[i], p.st_s[0], DV) * 2;
#pragma unroll
        for (int j = 0; j < GPW; ++j)
          __builtin_amdgcn_global_load_lds((global_cvoid_t*)(src + j * p.st_s[1] * 2 + goff_v[i]),
                                           (lds_void_t*)(dst + j * 32 * VB + i * 1024), 16, 0, aux);
      }
      if constexpr (SEPK) {
#pragma unroll
        for (int j = 0; j < NLK; ++j) {
          const unsigned char* src = src_k;
          if constexpr (LANE) src = key_b + row_at(row_k[j], p.k_s[0], DN) * 2;
          __builtin_amdgcn_global_load_lds((global_cvoid_t*)(src + goff_k[j]), (lds_void_t*)(dst + OFF_K + j * 1024), 16, 0, aux);
        }
      }
      if constexpr (DR > 0) {
#pragma unroll
        for (int j = 0; j < NLR; ++j) {  // (shared by the strands: left cacheable)
          const unsigned char* src = src_r;
          if constexpr (LANE) src = rope_b + row_at(row_r[j], p.rp_s[0], DR) * 2;
          __builtin_amdgcn_global_load_lds((global_cvoid_t*)(src + goff_r[j]), (lds_void_t*)(dst + OFF_R + j * 1024), 16, 0, 0);
        }
      }
    };
    if (stream_hint) loads(std::integral_constant<int, 2>{});
    else loads(std::integral_constant<int, 0>{});
  };

  // ---- LDS offsets of this lane's operand reads inside a stage (the same for every tile)
  //      scores: key row 16 * kb + r16, chunk 2 * ks + q / 2, half q % 2; operand order per key block:
  //      the non-RoPE steps of group 0, of group 1, then the RoPE steps
  //      values (transposing read): block q of 16 lanes reads keys 4q .. 4q + 3: lane 4r' + c' takes key r', dims 4c' .. 4c' + 3
  unsigned koff[2][NKF], voff[2][GPW * NDB];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const int row = 16 * kb + r16;
#pragma unroll
    for (int j = 0; j < GPW; ++j)
#pragma unroll
      for (int ks = 0; ks < NKN; ++ks) {
        constexpr int LPRK = (SEPK ? KB : VB) / 16;
        const int slot = (2 * ks + (q >> 1) + row) % LPRK;
        koff[kb][j * NKN + ks] = (unsigned)((SEPK ? OFF_K : j * 32 * VB) + row * (SEPK ? KB : VB) + slot * 16 + (q & 1) * 8);
      }
#pragma unroll
    for (int ks = 0; ks < NKR; ++ks) {
      constexpr int LPRR = RB > 0 ? RB / 16 : 1;
      const int slot = (2 * ks + (q >> 1) + row) % LPRR;
      koff[kb][GPW * NKN + ks] = (unsigned)(OFF_R + row * RB + slot * 16 + (q & 1) * 8);
    }
    constexpr int LPRV = VB / 16;
    const int tr_r = r16 >> 2, tr_c = r16 & 3;
    const int vrow = 16 * kb + 4 * q + tr_r;
#pragma unroll
    for (int j = 0; j < GPW; ++j)
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const int slot = (2 * db + (tr_c >> 1) + vrow) % LPRV;
        voff[kb][j * NDB + db] = (unsigned)(j * 32 * VB + vrow * VB + slot * 16 + (tr_c & 1) * 8);
      }
  }

  constexpr float kRebase = 8.f;
  constexpr float kLogHeavyShare = -2.f;  // a weight above a quarter of its row's running sum gets its rounding residual added
  const float sc2 = p.scale * 1.4426950408889634f;
  u32x2_t ones = {0x3f803f80u, 0x3f803f80u};  // four bf16 ones
  flex_tie(ones);  // (opaque from here on: a constant would be re-created by a vector move right in front of the MFMA that reads it)
  f32x4_t o[GPW * NDB], o_one;  // o_one: row sum of the weights as the MFMAs saw them (bf16-rounded)

  // value MFMAs of one pass over the tile: every group's accumulators against that group's values
  auto value_mfmas = [&](u32x2_t (&vf)[2 * GPW * NDB], const u32x2_t (&pb)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      flex_mfma_fresh(o[0], vf[kb * GPW * NDB], pb[kb]);
#pragma unroll
      for (int d = 1; d < GPW * NDB; ++d) flex_mfma(o[d], vf[kb * GPW * NDB + d], pb[kb]);
      flex_mfma_fresh(o_one, ones, pb[kb]);
    }
  };
  auto own = [&](int db) -> f32x4_t {  // the accumulators of this lane's own group
    if constexpr (GPW == 2) return jg ? o[NDB + db] : o[db];
    else return o[db];
  };

#pragma unroll
  for (int st = 0; st < NST - 1; ++st) issue_next(st);
  int st_cur = 0, st_load = NST - 1;
  bool first_segment = true;

  // ---- one segment per sequence that the chunk touches
  while (left > 0) {
    const int b = cur.b, L = cur.L, j0 = cur.j;
    const int seg = min(cur.tiles_b - j0, left);
    if (seg <= 0) break;  // (cannot happen while the lengths stay what they were when the chunk was located)
    const int n_vis = p.causal ? L - p.T + 1 + t : L;
    const int n_vis_min = uniform(n_vis);  // lane 0 holds the block's first row, which sees the fewest keys
    const int64_t row_idx = ((int64_t)b * p.T + t) * p.h_q + h;

    // query fragments: B operand of the score MFMAs, dims 16 * ks + 4 * q .. + 3 of row r16; the
    // non-RoPE part once per group of the wave, zero in the rows of the other group
    u32x2_t qn[GPW][NKN], qr[NKR > 0 ? NKR : 1];
    {
      const uint16_t* src = p.q_nope + b * p.qn_s[0] + t * p.qn_s[1] + h * p.qn_s[2] + 4 * q;
#pragma unroll
      for (int ks = 0; ks < NKN; ++ks) {
        const u32x2_t v = *reinterpret_cast<const u32x2_t*>(src + 16 * ks);
#pragma unroll
        for (int j = 0; j < GPW; ++j) qn[j][ks] = (GPW == 1 || jg == j) ? v : u32x2_t{0u, 0u};
      }
      if constexpr (NKR > 0) {
        const uint16_t* srcr = p.q_rope + b * p.qr_s[0] + t * p.qr_s[1] + h * p.qr_s[2] + 4 * q;
#pragma unroll
        for (int ks = 0; ks < NKR; ++ks) qr[ks] = *reinterpret_cast<const u32x2_t*>(srcr + 16 * ks);
      }
      // (pinned here: nothing that produces these operands may move down to the MFMAs that read them)
#pragma unroll
      for (int j = 0; j < GPW; ++j)
#pragma unroll
        for (int ks = 0; ks < NKN; ++ks) flex_tie(qn[j][ks]);
#pragma unroll
      for (int ks = 0; ks < NKR; ++ks) flex_tie(qr[ks]);
    }

    // per-row state.  Weights are taken relative to a reference m_ref (log2 domain, the same in the four
    // lanes of a row) that is moved up only when a score exceeds it by more than kRebase: most tiles
    // need no cross-lane traffic and no rescaling.  m_ref starts finite so that a masked score
    // (-inf) gives weight exp2(-inf) = 0 and never inf - inf.
    o_one = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int db = 0; db < GPW * NDB; ++db) o[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_ref = -1e30f, l_run = 0.f;  // l_run: this lane's share of the exact fp32 row sum
    float heavy_thr = -INFINITY;        // refreshed lazily; the running sum only grows, so a stale value errs on the safe side

    for (int i = 0; i < seg; ++i) {
      issue_next(st_load);
      st_load = st_load == NST - 1 ? 0 : st_load + 1;
      wait_vmcnt<LPT * (NST - 1)>();  // all but the NST - 1 newest tiles have landed: this tile is in LDS
      const int tile = j0 + i;
      const unsigned st_addr = ring_addr + (unsigned)(st_cur * STAGE);
      st_cur = st_cur == NST - 1 ? 0 : st_cur + 1;
      // value rows at or past the end of the sequence may hold anything: zero them (weight 0 x NaN must not leak)
      if ((tile << 5) + 32 > L) {
        const int valid = L - (tile << 5);
#pragma unroll
        for (int j = 0; j < GPW; ++j)
          for (int off = valid * VB + lane * 16; off < 32 * VB; off += 64 * 16) flex_lds_zero_b128(st_addr + j * 32 * VB + off);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      }

      // ---- scores of the two 16-key blocks: S^T[key 4q + i][row r16]
      u32x2_t kf[2 * NKF];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ks = 0; ks < NKF; ++ks) flex_lds_read_b64(kf[kb * NKF + ks], st_addr + koff[kb][ks]);
      flex_lds_wait_all(kf);
      f32x4_t sc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) flex_mfma0(sc[kb], kf[kb * NKF], qn[0][0]);
      static_for<1, NKF>([&](auto ksc) {
        constexpr int ks = decltype(ksc)::value;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          if constexpr (ks < GPW * NKN)
            flex_mfma(sc[kb], kf[kb * NKF + ks], qn[ks / NKN][ks % NKN]);
          else
            flex_mfma(sc[kb], kf[kb * NKF + ks], qr[ks - GPW * NKN]);
        }
      });
      flex_mfma_settle(sc[0], sc[1]);
      // ---- mask by select (last tiles only), then this lane's largest score
      if ((tile << 5) + 32 > n_vis_min) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            sc[kb][e] = (tile << 5) + 16 * kb + 4 * q + e < n_vis ? sc[kb][e] : -INFINITY;
      }
      const float mx = flex_max3(flex_max3(flex_max3(sc[0][0], sc[0][1], sc[0][2]), sc[0][3], sc[1][0]),
                                 flex_max3(sc[1][1], sc[1][2], sc[1][3]), -INFINITY);
      float lg = __builtin_fmaf(mx, sc2, -m_ref);  // log2 of this lane's largest weight
      if (__ballot(lg > kRebase) != 0) {
        flex_mfma_settle(o, o_one);  // (the value MFMAs of the tile before may still be on their way)
        float mrow = mx * sc2;
        mrow = fmaxf(mrow, __shfl_xor(mrow, 16, 64));
        mrow = fmaxf(mrow, __shfl_xor(mrow, 32, 64));
        const float m_new = fmaxf(m_ref, mrow);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_run *= alpha;
        o_one *= alpha;
#pragma unroll
        for (int db = 0; db < GPW * NDB; ++db) o[db] *= alpha;
        heavy_thr = -INFINITY;
        lg = __builtin_fmaf(mx, sc2, -m_ref);
      }
      // ---- value operands on their way while the weights are computed
      u32x2_t vf[2 * GPW * NDB];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int d = 0; d < GPW * NDB; ++d) flex_lds_read_tr(vf[kb * GPW * NDB + d], st_addr + voff[kb][d]);
      asm volatile("" : "+v"(sc[0]), "+v"(sc[1]));  // (keeps the reads above ahead of the arithmetic below)
      float pw[8], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pw[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e >> 2][e & 3], sc2, -m_ref));
        psum += pw[e];
      }
      l_run += psum;
      u32x2_t p_hi[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e2 = 0; e2 < 2; ++e2) p_hi[kb][e2] = cvt_pk_bf16(pw[4 * kb + 2 * e2], pw[4 * kb + 2 * e2 + 1]);
      flex_lds_wait_all(vf);
      // ---- O^T += V^T . P^T, and the row sums of the rounded weights through a ones-valued operand
      value_mfmas(vf, p_hi);
      // ---- rows that put much of their weight on one key of this tile: add the rounding residuals
      //      p - bf16(p) (as bf16) in a second pass, so those weights carry 16 significant bits
      if (__builtin_expect(__ballot(lg > heavy_thr) != 0, 0)) {
        float l_row = l_run + __shfl_xor(l_run, 16, 64);
        l_row += __shfl_xor(l_row, 32, 64);
        heavy_thr = __builtin_amdgcn_logf(l_row) + kLogHeavyShare;
        if (__ballot(lg > heavy_thr) != 0) {
          u32x2_t p_lo[2];
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e2 = 0; e2 < 2; ++e2) {
              const float a0 = pw[4 * kb + 2 * e2], a1 = pw[4 * kb + 2 * e2 + 1];
              const uint32_t hi = p_hi[kb][e2];
              p_lo[kb][e2] = cvt_pk_bf16(a0 - __builtin_bit_cast(float, hi << 16), a1 - __builtin_bit_cast(float, hi & 0xffff0000u));
            }
          value_mfmas(vf, p_lo);
        }
      }
    }
    flex_mfma_settle(o, o_one);

    // ---- result of this segment: O^T[dim 16 * db + 4q + i][row r16]
    float l_tot = l_run + __shfl_xor(l_run, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    const float inv = o_one[0] > 0.f ? 1.f / o_one[0] : 0.f;
    const float lse = l_tot > 0.f ? (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
    const bool whole = j0 == 0 && seg == cur.tiles_b;
    if (whole) {
      if (row_valid) {
        if (q == 0) p.lse[row_idx] = lse;
        const int64_t ob = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
          const int dim = 16 * db + 4 * q;
          const f32x4_t v = own(db) * inv;
          if (p.out_fp32) {
            *(f32x4_t*)((float*)p.out + ob + dim) = v;
          } else {
            u32x2_t pk;
            pk[0] = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
            pk[1] = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
            *(u32x2_t*)((uint16_t*)p.out + ob + dim) = pk;
          }
        }
      }
    } else {
      // a piece of a sequence that other chunks share: slot 0 of this (chunk, strand) for the segment the
      // chunk begins with, slot 1 for a later one (only the chunk's last segment can be such a piece)
      const int64_t slot = ((int64_t)unit * 2 + (first_segment ? 0 : 1)) * 16 + r16;
      if (row_valid) {
        if (q == 0) p.ws_lse[slot] = lse;
        float* dst = p.ws_out + slot * DV;
#pragma unroll
        for (int db = 0; db < NDB; ++db) *(f32x4_t*)(dst + 16 * db + 4 * q) = own(db) * inv;
      }
    }
    // which chunks hold the pieces of (sequence, strand): the first one with its slot, and the last one
    if (lane == 0) {
      int32_t* rng = p.flex_rng + ((int64_t)b * NSTR + strand) * 2;
      if (j0 == 0) rng[0] = chunk * 2 + (first_segment ? 0 : 1);
      if (j0 + seg == cur.tiles_b) rng[1] = chunk;
    }
    left -= seg;
    first_segment = false;
    if (left > 0) {
      cur.j = j0 + seg - 1;
      advance<32>(p, 1, cur);
    }
  }
  wait_vmcnt<0>();  // (tiles fetched again past the end of the chunk: let them land before the wave leaves)
}

// Merge of the pieces of the rows whose sequence was cut between chunks: one wave per output row.
// Rows of sequences that one chunk held entirely were written by the main kernel; empty sequences
// are filled here (out = 0, lse = -inf).
template <int GPW>
__global__ __launch_bounds__(64) void flex_combine_kernel(DevParams p) {
  const int row = blockIdx.x;
  const int lane = threadIdx.x;
  const int h = row % p.h_q;
  const int t = (row / p.h_q) % p.T;
  const int b = row / (p.h_q * p.T);
  const int64_t base = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
  const int L = p.seq_lens[b];
  if (L <= 0) {
    if (lane == 0) p.lse[row] = -INFINITY;
    for (int d = lane; d < p.d_v; d += 64) {
      if (p.out_fp32) ((float*)p.out)[base + d] = 0.f;
      else ((uint16_t*)p.out)[base + d] = 0;
    }
    return;
  }
  const int g = h / p.g_q;
  const int lr = t * p.g_q + (h - g * p.g_q);  // row within the group
  const int HB = p.h_c / GPW, NSTR = HB * p.flex_rb;
  const int strand = GPW == 2 ? g / 2 : (lr / 16) * HB + g;
  const int r16 = GPW == 2 ? (g % 2) * 8 + lr : lr % 16;
  const int32_t* rng = p.flex_rng + ((int64_t)b * NSTR + strand) * 2;
  const int c_first = rng[0] >> 1, slot_first = rng[0] & 1, c_last = rng[1];
  if (c_first == c_last) return;  // one chunk held the whole sequence: written by the main kernel
  auto slot_of = [&](int c) -> int64_t {
    return (((int64_t)c * NSTR + strand) * 2 + (c == c_first ? slot_first : 0)) * 16 + r16;
  };
  float m = -INFINITY;
  for (int c = c_first + lane; c <= c_last; c += 64) m = fmaxf(m, p.ws_lse[slot_of(c)]);
  for (int sh = 32; sh > 0; sh >>= 1) m = fmaxf(m, __shfl_xor(m, sh, 64));
  float z = 0.f;
  if (m != -INFINITY)
    for (int c = c_first + lane; c <= c_last; c += 64) z += expf(p.ws_lse[slot_of(c)] - m);
  for (int sh = 32; sh > 0; sh >>= 1) z += __shfl_xor(z, sh, 64);
  const float lse = (m == -INFINITY) ? -INFINITY : m + logf(z);
  if (lane == 0) p.lse[row] = lse;
  // four dims per lane; the lanes left over take every pgs-th piece each, summed at the end
  const int nd4 = p.d_v / 4, pgs = 64 / nd4;
  const int pg = lane / nd4, d4 = lane - pg * nd4;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  if (m != -INFINITY && pg < pgs) {
    for (int c = c_first + pg; c <= c_last; c += pgs) {
      const int64_t sl = slot_of(c);
      const float ls = p.ws_lse[sl];
      if (ls != -INFINITY) acc += *(const f32x4_t*)(p.ws_out + sl * p.d_v + 4 * d4) * expf(ls - lse);
    }
  }
  for (int g = 1; g < pgs; ++g) {
    const int src = d4 + g * nd4;  // (the same for every lane of a piece group; lanes of group 0 keep the sum)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float v = __shfl(acc[e], src & 63, 64);
      if (pg == 0) acc[e] += v;
    }
  }
  if (pg == 0) {
    if (p.out_fp32) {
      *(f32x4_t*)((float*)p.out + base + 4 * d4) = acc;
    } else {
      u32x2_t pk;
      pk[0] = (uint32_t)f32_to_bf16_bits(acc[0]) | ((uint32_t)f32_to_bf16_bits(acc[1]) << 16);
      pk[1] = (uint32_t)f32_to_bf16_bits(acc[2]) | ((uint32_t)f32_to_bf16_bits(acc[3]) << 16);
      *(u32x2_t*)((uint16_t*)p.out + base + 4 * d4) = pk;
    }
  }
}

}  // namespace gla
