// Tuned decode-attention path for gfx950: split-KV main kernel on bf16 MFMA
// with LDS-staged page tiles, plus the merge kernel for its partial results.
//
// Work decomposition.  A "unit" is (sequence b, group g, row block mb): the
// g_q * T query rows of one group (ordered t-major) cut into blocks of
// ROWS = 32 * NWAVES rows.  A unit owns ceil(L_b / TOK) key tiles of TOK = 64
// tokens (one page).  All tiles of all units, in unit order, form one flat list
// that is cut into equal chunks, one workgroup per chunk, so ragged batches
// balance by construction and at most two units per chunk are left incomplete.
// A unit that lies inside one chunk is written straight to the output; one that
// spans chunks leaves one partial (normalised fp32 output + log-sum-exp) per
// chunk in the workspace, merged afterwards by tuned_combine_kernel.
//
// Inside a workgroup every wave owns 32 query rows and works in the transposed
// form: S^T = K . Q^T with the key tile as the MFMA A operand (from LDS) and
// the query fragments as B operand (registers, loaded once per unit), then
// O^T += V^T . P^T where P^T comes straight from the S^T accumulators (the
// accumulator layout of a 32x32 MFMA already is a valid B-operand layout for a
// suitable order of the contraction index) and V^T is read from the SAME LDS
// tile with transposing LDS reads.  Row max / row sum therefore live in one
// lane plus its partner lane (lane ^ 32): no cross-wave softmax traffic.
//
// The operation itself is the absorbed-form attention of the paper (Sections
// 2.1, 3.3.1, 3.3.2): score = scale * (q_nope . state[:DN] + q_rope . rope_key),
// softmax over the visible keys, output = weights . state[:DV].
#pragma once

#include "../../include/gla_decode.h"
#include <type_traits>

#include "common.hpp"

namespace gla {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((address_space(3))) void lds_void_t;

constexpr int kTok = 64;  // tokens per key tile == page size of the tuned path

// ---- small device helpers -------------------------------------------------

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroup barrier that waits for this wave's LDS traffic only: outstanding
// global->LDS tile loads of later pipeline stages stay in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(v, off, 64);
    if (lane >= off) v += o;
  }
  return v;
}

__device__ __forceinline__ int tiles_of(int L) { return L > 0 ? (L + kTok - 1) / kTok : 0; }

// Position of a chunk's first tile in the flat tile list.
struct TileCursor {
  int b;        // sequence
  int ub;       // unit within the sequence: g * MB + mb
  int j;        // tile within the unit
  int tiles_b;  // tiles per unit of this sequence
  int L;        // its length
};

// Total number of tiles of the batch (every wave computes the same value).
__device__ __forceinline__ int total_tiles(const DevParams& p, int UPB, int lane) {
  int acc = 0;
  for (int base = 0; base < p.B; base += 64) {
    const int idx = base + lane;
    acc += idx < p.B ? tiles_of(p.seq_lens[idx]) * UPB : 0;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
  return uniform(acc);
}

// Locate flat tile index `pos` (< total): which sequence / unit / tile.
__device__ __forceinline__ TileCursor locate_tile(const DevParams& p, int UPB, int pos, int lane) {
  TileCursor c = {0, 0, 0, 0, 0};
  int before = 0;
  for (int base = 0; base < p.B; base += 64) {
    const int idx = base + lane;
    const int L = idx < p.B ? p.seq_lens[idx] : 0;
    const int tl = tiles_of(L);
    const int w = tl * UPB;
    const int incl = wave_incl_scan(w, lane) + before;
    const int excl = incl - w;
    const unsigned long long hit = __ballot(w > 0 && excl <= pos && pos < incl);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      const int ex = __shfl(excl, src, 64);
      c.tiles_b = uniform(__shfl(tl, src, 64));
      c.L = uniform(__shfl(L, src, 64));
      c.b = uniform(base + src);
      const int rem = uniform(pos - ex);
      c.ub = rem / c.tiles_b;
      c.j = rem - c.ub * c.tiles_b;
      return c;
    }
    before = uniform(__shfl(incl, 63, 64));
  }
  return c;
}

// Flat index of the first tile of sequence b (sum over earlier sequences).
__device__ __forceinline__ int tiles_before(const DevParams& p, int UPB, int b, int lane) {
  int acc = 0;
  for (int base = 0; base < b; base += 64) {
    const int idx = base + lane;
    acc += idx < b ? tiles_of(p.seq_lens[idx]) * UPB : 0;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
  return uniform(acc);
}

__device__ __forceinline__ void advance(const DevParams& p, int UPB, TileCursor& c) {
  if (++c.j < c.tiles_b) return;
  c.j = 0;
  if (++c.ub < UPB) return;
  c.ub = 0;
  do {
    ++c.b;
    c.L = c.b < p.B ? p.seq_lens[c.b] : 0;
    c.tiles_b = tiles_of(c.L);
  } while (c.b < p.B && c.tiles_b == 0);
}

// 16-byte-chunk swizzles of the LDS tiles.  State rows are DV*2 bytes; within
// every aligned run of 16 chunks the chunk index is XORed with a 4-bit key of
// the token so that (a) 16 consecutive tokens reading the same logical chunk
// (score MFMA operand reads) and (b) 4 consecutive tokens reading the same 64
// bytes (transposing value reads) both spread over all LDS banks.
__device__ __forceinline__ int swz16(int t) { return ((t & 3) << 2) | ((t >> 2) & 3); }
// RoPE rows are 128 bytes (8 chunks): two tokens share a 256-byte bank row.
__device__ __forceinline__ int swz8(int t) { return (t >> 1) & 7; }

template <int DV, int DN, int DR, int NWAVES, int STAGES>
struct TunedTraits {
  static constexpr int kRows = 32 * NWAVES;
  static constexpr int kStateBytes = kTok * DV * 2;
  static constexpr int kRopeBytes = kTok * DR * 2;
  static constexpr int kStageBytes = kStateBytes + kRopeBytes;
  static constexpr int kSmemBytes = STAGES * kStageBytes;
  static constexpr int kStateLoads = kStateBytes / 1024;  // wave-wide 16 B/lane loads
  static constexpr int kRopeLoads = kRopeBytes / 1024;
  static constexpr int kLoadsPerWave = (kStateLoads + kRopeLoads) / NWAVES;
  static constexpr int kThreads = 64 * NWAVES;
  static constexpr size_t kSlotFloats = (size_t)kRows * DV + kRows;  // partial out + lse
  static_assert(kStateLoads % NWAVES == 0 && kRopeLoads % NWAVES == 0, "tile loads must split evenly over waves");
  static_assert(kLoadsPerWave * (STAGES - 2 > 0 ? STAGES - 2 : 0) <= 63, "vmcnt range");
  static_assert(DR == 64, "RoPE key tile layout assumes 64 dims");
};

template <int DV, int DN, int DR, int NWAVES, int STAGES>
__global__ __launch_bounds__(64 * NWAVES) void tuned_main_kernel(DevParams p) {
  using TT = TunedTraits<DV, DN, DR, NWAVES, STAGES>;
  // One LDS array per pipeline stage, always addressed with a compile-time
  // stage index: the compiler can then tell that a tile load into one stage
  // does not alias operand reads from another and keeps the loads in flight.
  __shared__ __attribute__((aligned(1024))) unsigned char smem0[TT::kStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char smem1[STAGES > 1 ? TT::kStageBytes : 16];
  __shared__ __attribute__((aligned(1024))) unsigned char smem2[STAGES > 2 ? TT::kStageBytes : 16];
  __shared__ __attribute__((aligned(1024))) unsigned char smem3[STAGES > 3 ? TT::kStageBytes : 16];
  auto stage_ptr = [&](auto sc) -> unsigned char* {
    constexpr int S = decltype(sc)::value;
    if constexpr (S == 0) return smem0;
    else if constexpr (S == 1) return smem1;
    else if constexpr (S == 2) return smem2;
    else return smem3;
  };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int col = lane & 31;  // query row inside the wave's 32-row slab == MFMA column
  const int hi = lane >> 5;   // which half of the contraction slots this lane feeds

  const int rows_group = p.g_q * p.T;
  const int MB = (rows_group + TT::kRows - 1) / TT::kRows;
  const int UPB = p.h_c * MB;

  // ---- plan: this workgroup's chunk [c0, c1) of the flat tile list
  const int n_total = total_tiles(p, UPB, lane);
  const int chunk = p.chunk_tiles > 0 ? p.chunk_tiles
                                      : (n_total + (int)gridDim.x - 1) / (int)gridDim.x;
  if (chunk <= 0) return;
  const int c0 = (int)blockIdx.x * chunk;
  if (c0 >= n_total) return;
  const int c1 = min(n_total, c0 + chunk);
  const int n_tiles = c1 - c0;

  TileCursor cur = locate_tile(p, UPB, c0, lane);  // compute position
  TileCursor pre = cur;                             // prefetch position

  // ---- lane-constant pieces of the tile-load addressing (global -> LDS, 16 B per lane)
  // A wave-wide load fills 1 KiB of LDS linearly; the lane picks the global
  // chunk whose swizzled home is its LDS slot.
  auto issue_tile_loads = [&](const TileCursor& c, auto sc) {
    const int g = c.ub / MB;
    const int64_t page = p.page_table[(int64_t)c.b * p.max_pages + c.j];
    const unsigned char* sbase =
        (const unsigned char*)(p.state + page * p.st_s[0] + (int64_t)g * p.st_s[1]);
    const unsigned char* rbase = (const unsigned char*)(p.rope + page * p.rp_s[0]);
    unsigned char* stage_base = stage_ptr(sc);
#pragma unroll
    for (int ii = 0; ii < TT::kStateLoads / NWAVES; ++ii) {
      const int inst = ii * NWAVES + wave;  // 1 KiB slice index within the state tile
      const int off = inst * 1024 + lane * 16;
      const int t = off / (DV * 2);
      const int pc = (off % (DV * 2)) >> 4;
      const int lc = (pc & ~15) | ((pc & 15) ^ swz16(t));
      const unsigned goff = (unsigned)(t * (DV * 2) + (lc << 4));
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(sbase + goff),
                                       (lds_void_t*)(stage_base + inst * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int ii = 0; ii < TT::kRopeLoads / NWAVES; ++ii) {
      const int rinst = ii * NWAVES + wave;
      const int off = rinst * 1024 + lane * 16;
      const int t = off >> 7;
      const int pc = (off >> 4) & 7;
      const int lc = pc ^ swz8(t);
      const unsigned goff = (unsigned)(t * 128 + (lc << 4));
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(rbase + goff),
                                       (lds_void_t*)(stage_base + TT::kStateBytes + rinst * 1024), 16, 0, 0);
    }
  };

  // ---- prologue: fill STAGES-1 stages
  int issued = 0;
  auto prologue_stage = [&](auto sc) {
    if (issued < n_tiles) {
      issue_tile_loads(pre, sc);
      advance(p, UPB, pre);
      ++issued;
    }
  };
  if constexpr (STAGES > 1) prologue_stage(std::integral_constant<int, 0>{});
  if constexpr (STAGES > 2) prologue_stage(std::integral_constant<int, 1>{});
  if constexpr (STAGES > 3) prologue_stage(std::integral_constant<int, 2>{});

  // ---- lane-constant LDS read addresses
  // score operand (K rows, 16 B): token = 32*tb + col, logical chunk = 2*ks + hi
  const int sw_col = swz16(col);
  int k_addr[8];  // index: (2*ks) & 15 >> 1
#pragma unroll
  for (int e = 0; e < 8; ++e) k_addr[e] = col * (DV * 2) + ((((2 * e) | hi) ^ sw_col) << 4);
  int r_addr[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) r_addr[e] = TT::kStateBytes + col * 128 + ((((2 * e) | hi) ^ swz8(col)) << 4);
  // value operand (transposing 8 B reads): 16-lane block bk = lane / 16 covers
  // 4 tokens x 16 dims; lane 4r+q of the block addresses token r, dims 4q..4q+3.
  const int i16 = lane & 15;
  const int tr_r = i16 >> 2, tr_q = i16 & 3;
  const int dh = (lane >> 4) & 1;
  int v_addr[4][2];  // [db & 3][a]
#pragma unroll
  for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const int key = (tr_r << 2) | (2 * a + hi);           // swz16 of token 8a + 4hi + r
      const int lc = (4 * d4 + 2 * dh + (tr_q >> 1)) ^ key;  // chunk within the 16-chunk run
      v_addr[d4][a] = (4 * hi + tr_r) * (DV * 2) + (lc << 4) + (tr_q & 1) * 8;
    }

  const float sc2 = p.scale * 1.4426950408889634f;  // scores in base-2 units

  // ---- per-unit state
  bf16x8_t qn[DN / 16];
  bf16x8_t qr[DR / 16];
  f32x16_t o[DV / 32];
  float m_ref = -INFINITY, l_run = 0.f;
  int n_vis = 0, n_vis_min = 0;
  bool row_valid = false;
  int row_b = 0, row_t = 0, row_h = 0;
  bool unit_start = true;

  auto tile_step = [&](auto sc, int k) {
    constexpr int S = decltype(sc)::value;
    unsigned char* sb = stage_ptr(sc);

    if (unit_start) {
      // query fragments of this wave's 32 rows: B operand, lane holds 8 dims of row `col`
      const int g = cur.ub / MB;
      const int mb = cur.ub - g * MB;
      const int R = mb * TT::kRows + wave * 32 + col;
      row_valid = R < rows_group;
      row_t = row_valid ? R / p.g_q : 0;
      row_h = g * p.g_q + (row_valid ? R - row_t * p.g_q : 0);
      row_b = cur.b;
      const uint16_t* qn_ptr = p.q_nope + row_b * p.qn_s[0] + row_t * p.qn_s[1] + row_h * p.qn_s[2] + 8 * hi;
      const uint16_t* qr_ptr = p.q_rope + row_b * p.qr_s[0] + row_t * p.qr_s[1] + row_h * p.qr_s[2] + 8 * hi;
      const u32x4_t zero4 = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < DN / 16; ++ks) {
        u32x4_t v = row_valid ? *(const u32x4_t*)(qn_ptr + 16 * ks) : zero4;
        qn[ks] = __builtin_bit_cast(bf16x8_t, v);
      }
#pragma unroll
      for (int ks = 0; ks < DR / 16; ++ks) {
        u32x4_t v = row_valid ? *(const u32x4_t*)(qr_ptr + 16 * ks) : zero4;
        qr[ks] = __builtin_bit_cast(bf16x8_t, v);
      }
#pragma unroll
      for (int db = 0; db < DV / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
      m_ref = -INFINITY;
      l_run = 0.f;
      // visible keys of this lane's row; padding rows are left unmasked (never stored)
      n_vis = row_valid ? (p.causal ? cur.L - p.T + 1 + row_t : cur.L) : 0x7fffffff;
      int mn = n_vis;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) mn = min(mn, __shfl_xor(mn, off, 64));
      n_vis_min = uniform(mn);
      unit_start = false;
    }

    // ---- wait for tile k, make it visible to all waves, free stage (k-1) % STAGES
    if (k + (STAGES - 2) < n_tiles) wait_vmcnt<TT::kLoadsPerWave*(STAGES - 2 > 0 ? STAGES - 2 : 0)>();
    else wait_vmcnt<0>();
    lds_barrier();

    const int tile_tok0 = cur.j * kTok;
    if (tile_tok0 + kTok > cur.L) {
      // last tile of the sequence: slots at or beyond L may hold anything (NaN
      // included); zero those value rows so that 0-weight x garbage cannot leak.
      const int valid = cur.L - tile_tok0;
      for (int off = valid * (DV * 2) + tid * 16; off < TT::kStateBytes; off += TT::kThreads * 16)
        *(u32x4_t*)(sb + off) = u32x4_t{0, 0, 0, 0};
      lds_barrier();
    }

    // ---- prefetch tile k + STAGES - 1 into the stage just released
    if (issued < n_tiles) {
      issue_tile_loads(pre, std::integral_constant<int, (S + STAGES - 1) % STAGES>{});
      advance(p, UPB, pre);
      ++issued;
    }

    // ---- S^T = K . Q^T  (two 32-token blocks)
    f32x16_t s[2];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[tb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < DN / 16; ++ks) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        const int addr = k_addr[ks & 7] + tb * 32 * (DV * 2) + ((2 * ks) & ~15) * 16;
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(sb + addr));
        s[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qn[ks], s[tb], 0, 0, 0);
      }
    }
#pragma unroll
    for (int ks = 0; ks < DR / 16; ++ks) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        const int addr = r_addr[ks] + tb * 32 * 128;
        const bf16x8_t a = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(sb + addr));
        s[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qr[ks], s[tb], 0, 0, 0);
      }
    }

    // ---- online softmax in base 2; lane holds 32 scores of row `col`:
    // token(tb, i) = 32*tb + 8*(i/4) + 4*hi + i%4
    const bool need_mask = tile_tok0 + kTok > n_vis_min;
    float mx = -INFINITY;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float x = s[tb][i] * sc2;
        if (need_mask) {
          const int tok = tile_tok0 + 32 * tb + 8 * (i >> 2) + 4 * hi + (i & 3);
          x = tok < n_vis ? x : -INFINITY;
        }
        s[tb][i] = x;
        mx = fmaxf(mx, x);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // lazy reference update: keep the old reference while the row max stays
    // within 2^8 of it (probabilities then stay <= 256, exact enough in fp32/bf16)
    const bool bump = mx > m_ref + 8.0f;
    if (__ballot(bump)) {
      const float m_new = bump ? mx : m_ref;
      const float alpha = bump ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.0f;  // m_ref = -inf -> 0
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DV / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
      m_ref = m_new;
    }
    const float m_use = m_ref == -INFINITY ? 0.f : m_ref;
    float lsum = 0.f;
    bf16x8_t pf[4];  // B operands of the four 16-token contraction steps
#pragma unroll
    for (int tb = 0; tb < 2; ++tb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pv = __builtin_amdgcn_exp2f(s[tb][i] - m_use);
        lsum += pv;
        pf[tb * 2 + (i >> 3)][i & 7] = (__bf16)pv;
      }
    l_run += lsum;

    // ---- O^T += V^T . P^T ; contraction slot (hi, j) of step (tb, s2) is token
    // 32*tb + 16*s2 + 8*(j/4) + 4*hi + j%4, matching the accumulator layout above
#pragma unroll
    for (int st = 0; st < 4; ++st) {
#pragma unroll
      for (int db = 0; db < DV / 32; ++db) {
        const int base = st * 16 * (DV * 2) + (db >> 2) * 256;
        const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4_t*)(sb + v_addr[db & 3][0] + base));
        const bf16x4_t hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (__attribute__((address_space(3))) bf16x4_t*)(sb + v_addr[db & 3][1] + base + 8 * (DV * 2)));
        const bf16x8_t a = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[st], o[db], 0, 0, 0);
      }
    }

    // ---- end of unit (or of chunk): write the result
    const bool unit_done = cur.j + 1 == cur.tiles_b;
    if (unit_done || k + 1 == n_tiles) {
      // the unit is complete here iff this chunk also held its first tile
      const bool complete = unit_done && (k >= cur.j);
      const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      const float lse = l_tot > 0.f ? (m_ref + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
      if (complete) {
        if (row_valid) {
          const int64_t ob = row_b * p.out_s[0] + row_t * p.out_s[1] + row_h * p.out_s[2];
          if (hi == 0) p.lse[((int64_t)row_b * p.T + row_t) * p.h_q + row_h] = lse;
#pragma unroll
          for (int db = 0; db < DV / 32; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const int dim = 32 * db + 8 * q4 + 4 * hi;
              f32x4_t v = {o[db][4 * q4] * inv, o[db][4 * q4 + 1] * inv, o[db][4 * q4 + 2] * inv,
                           o[db][4 * q4 + 3] * inv};
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
        // partial: slot 0 if the unit began before this chunk, slot 1 otherwise
        const int which = (k < cur.j) ? 0 : 1;  // k < j: first tile of the unit is in an earlier chunk
        float* slot = p.ws_out + ((size_t)blockIdx.x * 2 + which) * TT::kSlotFloats;
        const int lr = wave * 32 + col;
        if (hi == 0) slot[(size_t)TT::kRows * DV + lr] = lse;
#pragma unroll
        for (int db = 0; db < DV / 32; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int dim = 32 * db + 8 * q4 + 4 * hi;
            f32x4_t v = {o[db][4 * q4] * inv, o[db][4 * q4 + 1] * inv, o[db][4 * q4 + 2] * inv,
                         o[db][4 * q4 + 3] * inv};
            *(f32x4_t*)(slot + (size_t)lr * DV + dim) = v;
          }
      }
      unit_start = true;
    }
    advance(p, UPB, cur);
  };

  for (int k = 0; k < n_tiles; k += STAGES) {
    tile_step(std::integral_constant<int, 0>{}, k);
    if constexpr (STAGES > 1) if (k + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, k + 1);
    if constexpr (STAGES > 2) if (k + 2 < n_tiles) tile_step(std::integral_constant<int, 2>{}, k + 2);
    if constexpr (STAGES > 3) if (k + 3 < n_tiles) tile_step(std::integral_constant<int, 3>{}, k + 3);
  }
}

// Merge of the partial results of units that span several chunks, and zero fill
// of units without any key:  lse = ln sum_s exp(lse_s),
// out = sum_s exp(lse_s - lse) out_s.  One workgroup per unit.
template <int DV, int NWAVES>
__global__ __launch_bounds__(256) void tuned_combine_kernel(DevParams p) {
  constexpr int kRows = 32 * NWAVES;
  constexpr size_t kSlotFloats = (size_t)kRows * DV + kRows;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rows_group = p.g_q * p.T;
  const int MB = (rows_group + kRows - 1) / kRows;
  const int UPB = p.h_c * MB;
  const int unit = blockIdx.x;
  const int b = unit / UPB;
  const int ub = unit - b * UPB;
  const int g = ub / MB, mb = ub - g * MB;
  const int L = p.seq_lens[b];
  const int tl = tiles_of(L);

  int k_first = 0, k_last = -1, s_u = 0;
  if (tl > 0) {
    const int n_total = total_tiles(p, UPB, lane);
    const int chunk = p.chunk_tiles > 0 ? p.chunk_tiles : (n_total + p.num_chunks - 1) / p.num_chunks;
    s_u = tiles_before(p, UPB, b, lane) + ub * tl;
    k_first = s_u / chunk;
    k_last = (s_u + tl - 1) / chunk;
    if (k_first == k_last) return;  // written directly by the main kernel
    // partial slot of chunk k: 0 if the unit began before the chunk, else 1
    // (only chunk k_first can hold the unit's first tile)
    for (int r = wave; r < kRows; r += 4) {
      const int R = mb * kRows + r;
      if (R >= rows_group) break;
      const int t = R / p.g_q;
      const int h = g * p.g_q + (R - t * p.g_q);
      float m = -INFINITY;
      for (int k = k_first; k <= k_last; ++k) {
        const int which = (k == k_first && s_u >= k * chunk) ? 1 : 0;
        m = fmaxf(m, p.ws_out[((size_t)k * 2 + which) * kSlotFloats + (size_t)kRows * DV + r]);
      }
      float z = 0.f;
      if (m != -INFINITY)
        for (int k = k_first; k <= k_last; ++k) {
          const int which = (k == k_first && s_u >= k * chunk) ? 1 : 0;
          z += expf(p.ws_out[((size_t)k * 2 + which) * kSlotFloats + (size_t)kRows * DV + r] - m);
        }
      const float lse = m == -INFINITY ? -INFINITY : m + logf(z);
      if (lane == 0) p.lse[((int64_t)b * p.T + t) * p.h_q + h] = lse;
      float acc[DV / 64];
#pragma unroll
      for (int i = 0; i < DV / 64; ++i) acc[i] = 0.f;
      if (m != -INFINITY)
        for (int k = k_first; k <= k_last; ++k) {
          const int which = (k == k_first && s_u >= k * chunk) ? 1 : 0;
          const float* slot = p.ws_out + ((size_t)k * 2 + which) * kSlotFloats;
          const float ls = slot[(size_t)kRows * DV + r];
          if (ls == -INFINITY) continue;
          const float w = expf(ls - lse);
#pragma unroll
          for (int i = 0; i < DV / 64; ++i) acc[i] += w * slot[(size_t)r * DV + lane + 64 * i];
        }
      const int64_t ob = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
#pragma unroll
      for (int i = 0; i < DV / 64; ++i) {
        if (p.out_fp32) ((float*)p.out)[ob + lane + 64 * i] = acc[i];
        else ((uint16_t*)p.out)[ob + lane + 64 * i] = f32_to_bf16_bits(acc[i]);
      }
    }
  } else {
    // no cached token: zeros and -inf
    for (int r = wave; r < kRows; r += 4) {
      const int R = mb * kRows + r;
      if (R >= rows_group) break;
      const int t = R / p.g_q;
      const int h = g * p.g_q + (R - t * p.g_q);
      if (lane == 0) p.lse[((int64_t)b * p.T + t) * p.h_q + h] = -INFINITY;
      const int64_t ob = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
      for (int d = lane; d < DV; d += 64) {
        if (p.out_fp32) ((float*)p.out)[ob + d] = 0.f;
        else ((uint16_t*)p.out)[ob + d] = 0;
      }
    }
  }
}

// ---- host side ---------------------------------------------------------------

struct TunedPlan {
  int variant;     // index into the instantiation table below, -1: none
  int nwaves;      // waves per workgroup
  int rows;        // 32 * nwaves
  int mb;          // row blocks per (sequence, group)
  int num_chunks;  // main-kernel grid
  int chunk_tiles; // fixed tiles per chunk, 0: derived on the device
  size_t slot_floats;
};

inline int device_cu_count() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;  // MI355X
  }
  return cus;
}

inline bool aligned16(const void* ptr) { return ((uintptr_t)ptr & 15u) == 0; }

inline bool tuned_plan(const gla_decode_params* p, int is_gta, TunedPlan* plan) {
  if (p->page_size != kTok || p->d_rope != 64) return false;
  int variant = -1;
  if (!is_gta && p->d_v == 256) variant = 0;
  else if (is_gta && p->d_v == 128) variant = 2;
  if (variant < 0) return false;
  // layout the kernels assume: token rows contiguous, everything 16-byte aligned
  if (p->state_stride[2] != p->d_v || p->rope_stride[1] != p->d_rope) return false;
  if (p->state_stride[0] % 8 || p->state_stride[1] % 8 || p->rope_stride[0] % 8) return false;
  for (int i = 0; i < 3; ++i)
    if (p->q_nope_stride[i] % 8 || p->q_rope_stride[i] % 8 || p->out_stride[i] % 4) return false;
  if (p->q_nope && !(aligned16(p->q_nope) && aligned16(p->q_rope) && aligned16(p->state_cache) &&
                     aligned16(p->rope_cache) && aligned16(p->out)))
    return false;
  const int rows_group = (p->num_q_heads / p->num_groups) * p->q_len;
  const int nwaves = rows_group <= 32 ? 1 : (rows_group <= 64 ? 2 : 4);
  plan->variant = variant;
  plan->nwaves = nwaves;
  plan->rows = 32 * nwaves;
  plan->mb = (rows_group + plan->rows - 1) / plan->rows;
  const int64_t max_tiles = p->max_pages_per_seq;
  const int64_t bound = (int64_t)p->batch * p->num_groups * plan->mb * max_tiles;
  if (bound > 0x3fffffff) return false;
  if (p->num_splits > 0) {
    plan->chunk_tiles = (int)((max_tiles + p->num_splits - 1) / p->num_splits);
    plan->num_chunks = (int)std::max<int64_t>(1, (bound + plan->chunk_tiles - 1) / plan->chunk_tiles);
  } else {
    plan->chunk_tiles = 0;
    const int per_cu = nwaves == 4 ? 1 : (nwaves == 2 ? 2 : 3);
    plan->num_chunks = (int)std::max<int64_t>(1, std::min<int64_t>(bound, (int64_t)device_cu_count() * per_cu));
  }
  plan->slot_floats = (size_t)plan->rows * p->d_v + plan->rows;
  return true;
}

inline bool tuned_supported(const gla_decode_params* p, int is_gta) {
  TunedPlan plan;
  return tuned_plan(p, is_gta, &plan);
}

inline size_t tuned_workspace(const gla_decode_params* p, int is_gta) {
  TunedPlan plan;
  if (!tuned_plan(p, is_gta, &plan)) return 0;
  return (size_t)plan.num_chunks * 2 * plan.slot_floats * sizeof(float);
}

template <int DV, int DN, int NWAVES, int STAGES>
inline int launch_tuned_variant(const TunedPlan& plan, DevParams& d, int units, hipStream_t st,
                                hipEvent_t* ev) {
  if (ev) (void)hipEventRecord(ev[0], st);
  hipLaunchKernelGGL((tuned_main_kernel<DV, DN, 64, NWAVES, STAGES>), dim3(plan.num_chunks),
                     dim3(64 * NWAVES), 0, st, d);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[1], st);
  hipLaunchKernelGGL((tuned_combine_kernel<DV, NWAVES>), dim3(units), dim3(256), 0, st, d);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[2], st);
  return GLA_OK;
}

inline int tuned_launch(const gla_decode_params* p, int is_gta, DevParams& d, hipStream_t st,
                        hipEvent_t* ev) {
  TunedPlan plan;
  if (!tuned_plan(p, is_gta, &plan)) return GLA_ERR_UNSUPPORTED_SHAPE;
  d.ws_out = (float*)p->workspace;
  d.num_chunks = plan.num_chunks;
  d.chunk_tiles = plan.chunk_tiles;
  const int units = p->batch * p->num_groups * plan.mb;
  if (plan.variant == 0) {
    if (plan.nwaves == 1) return launch_tuned_variant<256, 256, 1, 2>(plan, d, units, st, ev);
    if (plan.nwaves == 2) return launch_tuned_variant<256, 256, 2, 2>(plan, d, units, st, ev);
    return launch_tuned_variant<256, 256, 4, 3>(plan, d, units, st, ev);
  }
  if (plan.variant == 2) {
    if (plan.nwaves == 1) return launch_tuned_variant<128, 64, 1, 2>(plan, d, units, st, ev);
    if (plan.nwaves == 2) return launch_tuned_variant<128, 64, 2, 2>(plan, d, units, st, ev);
    return launch_tuned_variant<128, 64, 4, 3>(plan, d, units, st, ev);
  }
  return GLA_ERR_UNSUPPORTED_SHAPE;
}

}  // namespace gla
