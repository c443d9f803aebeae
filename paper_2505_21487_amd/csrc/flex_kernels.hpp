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
// byte, so the design is the simplest one that streams well: ONE WAVE per
// (sequence, group, block of 16 query rows, key range), no cooperation between
// waves, hence no barriers.  A wave moves its tiles of 32 tokens global -> LDS
// with direct-to-LDS loads of whole cache rows through its own ring of stages
// and works in the transposed form on 16x16x16 bf16 MFMAs:
//     S^T = K . Q^T       A operand: key rows from LDS (8 bytes per lane), B: query fragments in registers
//     O^T += V^T . P^T    A: value tile read with transposing LDS reads, B: the score accumulators, which
//                         already have the B-operand layout (key 4 * (lane / 16) + i of query row lane % 16)
// Softmax statistics of a row live in the four lanes {r, r + 16, r + 32, r + 48}.
// Weights enter the value product as bf16 pairs hi + lo (two MFMAs): they carry
// 16 significant bits, so no row, however few keys carry it, is limited by the
// weight rounding.  16-byte chunks of a cache row are rotated by the row index
// inside LDS (slot = (chunk + row) mod chunks per row) so that reads of one
// column over 16 rows spread over the banks; each lane of a load fetches the
// chunk whose rotated home is its slot.
//
// Partial results of the key ranges use the layout of the generic kernel
// ([range][row][d_v] fp32 + log-sum-exp) and are merged by generic_combine_kernel.
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
template <int N>
__device__ __forceinline__ void flex_lds_wait_all(u32x2_t (&x)[N]) {
  // every LDS read issued so far has returned; tied to the registers so that no use moves ahead of it
#pragma unroll
  for (int i = 0; i < N; ++i) flex_tie(x[i]);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int i = 0; i < N; ++i) flex_tie(x[i]);
}

template <int DN, int DR, int DV, bool SEPK>
struct FlexTraits {
  static constexpr int kVB = DV * 2, kKB = DN * 2, kRB = DR * 2;  // row bytes of the value / key / RoPE tiles
  static constexpr int kStage = 32 * (kVB + (SEPK ? kKB : 0) + kRB);
  static constexpr int kNST = (40 * 1024 / kStage) < 6 ? (40 * 1024 / kStage) : 6;  // ring stages per wave (40 KB each)
  static constexpr int loads(int rb) {  // load instructions for 32 rows of rb bytes
    return rb == 0 ? 0 : (32 + 64 / (rb / 16) - 1) / (64 / (rb / 16));
  }
  static constexpr int kLPT = loads(kVB) + (SEPK ? loads(kKB) : 0) + loads(kRB);
  static_assert(kNST >= 2, "at least two stages");
  static_assert(kLPT * (kNST - 1) <= 63, "vmcnt range");
  static_assert(DN % 16 == 0 && DR % 16 == 0 && DV % 16 == 0 && (SEPK || DN <= DV), "dims");
};

template <int DN, int DR, int DV, bool SEPK>
__global__ __launch_bounds__(256) void flex_main_kernel(DevParams p) {
  using FT = FlexTraits<DN, DR, DV, SEPK>;
  constexpr int NST = FT::kNST, STAGE = FT::kStage, LPT = FT::kLPT;
  constexpr int VB = FT::kVB, KB = FT::kKB, RB = FT::kRB;
  constexpr int OFF_K = 32 * VB, OFF_R = OFF_K + (SEPK ? 32 * KB : 0);  // tile offsets inside a stage
  constexpr int NKN = DN / 16, NKR = DR / 16, NKS = NKN + NKR;         // contraction steps of the scores
  constexpr int NDB = DV / 16;                                          // 16-dim output blocks
  __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * NST * STAGE];
  static_assert(sizeof(smem) <= 160 * 1024, "LDS capacity");

  const int lane = threadIdx.x & 63;
  const int wave = uniform((int)threadIdx.x >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  unsigned char* const ring = smem + wave * (NST * STAGE);
  const unsigned ring_addr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)ring;

  // ---- this wave's unit: key ranges fastest, so the waves of a workgroup read disjoint keys
  const int rows_group = p.g_q * p.T;
  const int RBK = p.flex_rb;  // blocks of 16 rows per group
  const int64_t unit = (int64_t)blockIdx.x * 4 + wave;
  if (unit >= (int64_t)p.B * p.h_c * RBK * p.splits) return;
  const int s = (int)(unit % p.splits);
  const int rb = (int)((unit / p.splits) % RBK);
  const int g = (int)((unit / ((int64_t)p.splits * RBK)) % p.h_c);
  const int b = (int)(unit / ((int64_t)p.splits * RBK * p.h_c));
  const int L = p.seq_lens[b];
  const int tiles_b = L > 0 ? (L + 31) >> 5 : 0;
  const int t0 = min(s * p.pages_per_split, tiles_b);  // (for this kernel: tiles per range)
  const int t1 = min(t0 + p.pages_per_split, tiles_b);
  const int n_t = t1 - t0;

  // ---- the query row of this lane (rows past the end of the group repeat the last one, never stored)
  const int R = rb * 16 + r16;
  const bool row_valid = R < rows_group;
  const int Rc = row_valid ? R : rows_group - 1;
  const int t = Rc / p.g_q;
  const int h = g * p.g_q + (Rc - t * p.g_q);
  const int n_vis = row_valid ? (p.causal ? L - p.T + 1 + t : L) : 0;
  const int64_t row_idx = ((int64_t)b * p.T + t) * p.h_q + h;

  // ---- query fragments: B operand of the score MFMAs, dims 16 * ks + 4 * q .. + 3 of row r16
  u32x2_t qf[NKS];
  {
    const uint16_t* qn = p.q_nope + b * p.qn_s[0] + t * p.qn_s[1] + h * p.qn_s[2] + 4 * q;
#pragma unroll
    for (int ks = 0; ks < NKN; ++ks) qf[ks] = *reinterpret_cast<const u32x2_t*>(qn + 16 * ks);
    if constexpr (NKR > 0) {
      const uint16_t* qr = p.q_rope + b * p.qr_s[0] + t * p.qr_s[1] + h * p.qr_s[2] + 4 * q;
#pragma unroll
      for (int ks = 0; ks < NKR; ++ks) qf[NKN + ks] = *reinterpret_cast<const u32x2_t*>(qr + 16 * ks);
    }
  }

  // ---- page ids of this wave's key range: 64 at a time, one per lane
  const int lgP = p.lg_page;             // page size is a power of two of at least 32 tokens
  const int tpp_lg = lgP - 5;            // log2(tiles per page)
  int pt_base = -1, pt_vec = 0;
  auto page_of_tile = [&](int tile) -> int {
    const int pg = tile >> tpp_lg;
    if (pt_base < 0 || pg < pt_base || pg >= pt_base + 64) {
      pt_base = pg;
      pt_vec = load_i32_sync(p.page_table + (int64_t)b * p.max_pages + min(pg + lane, p.max_pages - 1));
    }
    return __builtin_amdgcn_readlane(pt_vec, pg - pt_base);
  };

  // ---- tile loads.  A load instruction moves 64 / LPR whole rows (LPR = 16-byte chunks per row); lane l
  //      writes slot l % LPR of row l / LPR and fetches the chunk whose rotated home that slot is.
  auto issue_rows = [&](auto rbc, const unsigned char* src_tile, int64_t row_stride_bytes, unsigned char* dst) {
    constexpr int RBY = decltype(rbc)::value;
    constexpr int LPR = RBY / 16, RPI = 64 / LPR, NI = (32 + RPI - 1) / RPI;
    const int lrow = lane / LPR, slot = lane % LPR;
    static_for<0, NI>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const int row = j * RPI + lrow;
      if (lane < RPI * LPR && row < 32) {
        int chunk = slot - (row % LPR);
        chunk += chunk < 0 ? LPR : 0;
        __builtin_amdgcn_global_load_lds((global_cvoid_t*)(src_tile + row * row_stride_bytes + chunk * 16),
                                         (lds_void_t*)(dst + j * RPI * RBY), 16, 0, 0);
      }
    });
  };
  auto issue_tile = [&](int tile, int stage) {
    const int64_t page = page_of_tile(tile);
    const int tok = (tile << 5) & ((1 << lgP) - 1);  // first token of the tile inside its page
    unsigned char* dst = ring + stage * STAGE;
    const unsigned char* v = (const unsigned char*)(p.state + page * p.st_s[0] + g * p.st_s[1] + (int64_t)tok * p.st_s[2]);
    issue_rows(std::integral_constant<int, VB>{}, v, p.st_s[2] * 2, dst);
    if constexpr (SEPK) {
      const unsigned char* k = (const unsigned char*)(p.kstate + page * p.k_s[0] + g * p.k_s[1] + (int64_t)tok * p.k_s[2]);
      issue_rows(std::integral_constant<int, KB>{}, k, p.k_s[2] * 2, dst + OFF_K);
    }
    if constexpr (DR > 0) {
      const unsigned char* rp = (const unsigned char*)(p.rope + page * p.rp_s[0] + (int64_t)tok * p.rp_s[1]);
      issue_rows(std::integral_constant<int, RB>{}, rp, p.rp_s[1] * 2, dst + OFF_R);
    }
  };

  // ---- per-row state
  f32x4_t o[NDB];
#pragma unroll
  for (int db = 0; db < NDB; ++db) o[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane's share of the row sum
  const float sc2 = p.scale * 1.4426950408889634f;

  if (n_t > 0) {
#pragma unroll
    for (int st = 0; st < NST - 1; ++st) issue_tile(t0 + min(st, n_t - 1), st);  // (tiles past the end: the last one again)
  }
  for (int i = 0; i < n_t; ++i) {
    issue_tile(t0 + min(i + NST - 1, n_t - 1), (i + NST - 1) % NST);
    wait_vmcnt<LPT * (NST - 1)>();  // all but the NST - 1 newest tiles have landed: tile i is in LDS
    const int tile = t0 + i;
    const unsigned st_addr = ring_addr + (unsigned)((i % NST) * STAGE);
    // value rows at or past the end of the sequence may hold anything: zero them (weight 0 x NaN must not leak)
    if ((tile << 5) + 32 > L) {
      const int valid = L - (tile << 5);
      for (int off = valid * VB + lane * 16; off < 32 * VB; off += 64 * 16) flex_lds_zero_b128(st_addr + off);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }

    // ---- scores of the two 16-key blocks: S^T[key 4q + i][row r16]
    f32x4_t sc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int row = 16 * kb + r16;  // key row this lane reads
      u32x2_t kf[NKS];
      static_for<0, NKS>([&](auto ksc) {
        constexpr int ks = decltype(ksc)::value;
        if constexpr (ks < NKN) {
          constexpr int LPRK = (SEPK ? KB : VB) / 16;
          const int slot = (2 * ks + (q >> 1) + row) % LPRK;  // chunk 2 * ks + q / 2, rotated by the row
          flex_lds_read_b64(kf[ks], st_addr + (SEPK ? OFF_K : 0) + row * (SEPK ? KB : VB) + slot * 16 + (q & 1) * 8);
        } else {
          constexpr int LPRR = RB / 16;
          const int slot = (2 * (ks - NKN) + (q >> 1) + row) % LPRR;
          flex_lds_read_b64(kf[ks], st_addr + OFF_R + row * RB + slot * 16 + (q & 1) * 8);
        }
      });
      flex_lds_wait_all(kf);
      f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
      static_for<0, NKS>([&](auto ksc) {
        constexpr int ks = decltype(ksc)::value;
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(flex_s16x4_t, kf[ks]),
                                                         __builtin_bit_cast(flex_s16x4_t, qf[ks]), acc, 0, 0, 0);
      });
      sc[kb] = acc;
    }
    // ---- mask by select, row max over the row's four lanes, online softmax
    float x[8];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int key = (tile << 5) + 16 * kb + 4 * q + e;
        const float v = key < n_vis ? sc[kb][e] * sc2 : -INFINITY;
        x[4 * kb + e] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);  // (m_run = -inf: 0)
    float pw[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pw[e] = m_new == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(x[e] - m_new);
      psum += pw[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < NDB; ++db) o[db] *= alpha;
    // weights as bf16 pairs hi + lo
    u32x2_t p_hi[2], p_lo[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e2 = 0; e2 < 2; ++e2) {
        const float a0 = pw[4 * kb + 2 * e2], a1 = pw[4 * kb + 2 * e2 + 1];
        const uint32_t hi = cvt_pk_bf16(a0, a1);
        const float h0 = __builtin_bit_cast(float, hi << 16), h1 = __builtin_bit_cast(float, hi & 0xffff0000u);
        p_hi[kb][e2] = hi;
        p_lo[kb][e2] = cvt_pk_bf16(a0 - h0, a1 - h1);
      }
    // ---- O^T += V^T . P^T: block q of 16 lanes reads keys 4q .. 4q + 3 (lane 4r' + c': key r', dims 4c' .. 4c' + 3)
    constexpr int LPRV = VB / 16;
    const int tr_r = r16 >> 2, tr_c = r16 & 3;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int row = 16 * kb + 4 * q + tr_r;
      u32x2_t vf[NDB];
      static_for<0, NDB>([&](auto dbc) {
        constexpr int db = decltype(dbc)::value;
        const int slot = (2 * db + (tr_c >> 1) + row) % LPRV;
        flex_lds_read_tr(vf[db], st_addr + row * VB + slot * 16 + (tr_c & 1) * 8);
      });
      flex_lds_wait_all(vf);
      static_for<0, NDB>([&](auto dbc) {
        constexpr int db = decltype(dbc)::value;
        const flex_s16x4_t a = __builtin_bit_cast(flex_s16x4_t, vf[db]);
        o[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(flex_s16x4_t, p_hi[kb]), o[db], 0, 0, 0);
        o[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, __builtin_bit_cast(flex_s16x4_t, p_lo[kb]), o[db], 0, 0, 0);
      });
    }
  }
  wait_vmcnt<0>();  // (tiles fetched again past the end of the range: let them land before the wave leaves)

  // ---- result of this key range: O^T[dim 16 * db + 4q + i][row r16]
  float l_tot = l_run + __shfl_xor(l_run, 16, 64);
  l_tot += __shfl_xor(l_tot, 32, 64);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  if (!row_valid) return;
  if (p.splits == 1) {
    if (q == 0) p.lse[row_idx] = lse;
    const int64_t ob = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const int dim = 16 * db + 4 * q;
      const f32x4_t v = o[db] * inv;
      if (p.out_fp32) {
        *(f32x4_t*)((float*)p.out + ob + dim) = v;
      } else {
        u32x2_t pk;
        pk[0] = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
        pk[1] = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
        *(u32x2_t*)((uint16_t*)p.out + ob + dim) = pk;
      }
    }
  } else {
    const int64_t rows = (int64_t)p.B * p.T * p.h_q;
    if (q == 0) p.ws_lse[(int64_t)s * rows + row_idx] = lse;
    float* dst = p.ws_out + ((int64_t)s * rows + row_idx) * DV;
#pragma unroll
    for (int db = 0; db < NDB; ++db) *(f32x4_t*)(dst + 16 * db + 4 * q) = o[db] * inv;
  }
}

}  // namespace gla
