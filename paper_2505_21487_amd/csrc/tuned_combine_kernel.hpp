// Merge kernel of the tuned decode-attention path: combines the partial
// results the main kernel leaves for units that span several chunks.
#pragma once

#include "tuned_device.hpp"

namespace gla {

// Merge of the partial results of units that span several chunks, and zero fill
// of units without any key:  lse = ln sum_s exp(lse_s),
// out = sum_s exp(lse_s - lse) out_s.  The main kernel leaves, per unit, the
// range of chunks that hold it, and stores partial outputs in the register
// order of its waves (one contiguous 1 KiB block per wave, 32-dim block and
// quarter), so a task here is one (32-row slab, 32-dim block) of a unit and
// every access of a partial is a full 1 KiB line run.  The KW waves of a
// workgroup share one task: wave j merges chunks first + j, first + j + KW, ...
// around its own reference, and the KW results are merged once more through
// LDS (long single sequences are cut into hundreds of chunks).  With QS = 4
// (very few units, each spread over very many chunks: few tasks) a task is cut
// once more into the four quarters of its 32-dim block, one workgroup each,
// so that four times as many compute units pull the partials.
// Grid (units, NG * WPG * DV / 32 * QS), KW waves per workgroup.
template <int DV, int NG, int WPG, int KS, int TOK, int KW, int QS, int U>
__global__ __launch_bounds__(64 * KW) void tuned_combine_kernel(DevParams p) {
  constexpr int NWAVES = NG * WPG * KS;
  constexpr int NDB = DV / KS / 32;  // 32-dim blocks per wave of the main kernel
  constexpr int kRows = 32 * NG * WPG;
  constexpr size_t kSlotFloats = (size_t)kRows * DV + 32 * NWAVES;
  static_assert(KW == 1 || KW == 4 || KW == 16, "waves per task");
  static_assert(QS == 1 || (QS == 4 && KW > 1), "workgroups per task");
  constexpr int NQ4 = 4 / QS;  // quarters of the block per workgroup
  __shared__ float red_m[KW][64], red_z[KW][64];
  __shared__ f32x4_t red_a[KW][NQ4][64];
  const int tid = threadIdx.x, lane = tid & 63, kw = tid >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const int wv = blockIdx.y / QS;
  const int q_base = QS == 1 ? 0 : (int)blockIdx.y % QS;  // first quarter this workgroup handles
  const int w = wv / NDB, db = wv - w * NDB;  // wave of the main kernel and one of its 32-dim blocks
  const int wpos = w % (WPG * KS), kx = wpos % KS;
  const int rows_group = p.g_q * p.T;
  const int MB = p.mb;
  const int UPB = p.upb * MB;
  const int unit = blockIdx.x;  // (sequence, group block, row block)
  const int b = (int)fast_div((unsigned)unit, p.fd_upb_mb);
  const int ub = unit - b * UPB;
  const int gb = (int)fast_div((unsigned)ub, p.fd_mb), mb = ub - gb * MB;
  const int L = p.seq_lens[b];
  const int2 span = ((const int2*)p.ws_lse)[unit];  // garbage for units without tiles: not used then
  const bool empty = tiles_of<TOK>(L) == 0;
  if (!empty && span.x == span.y) return;  // written directly by the main kernel (whole workgroup leaves)
  const int g = gb * NG + w / (WPG * KS);
  const int R = (mb * WPG + wpos / KS) * 32 + col;
  const bool valid = R < rows_group;
  const int Rc = valid ? R : 0;
  const int t = (int)fast_div((unsigned)Rc, p.fd_gq);
  const int h = g * p.g_q + (Rc - t * p.g_q);
  const int r = w * 32 + col;  // this lane's entry among the slot's log-sum-exps
  // Chunk span.x holds the unit's first tile (partial slot 1); every later
  // chunk sees a unit that began before it (slot 0).
  const int k_first = empty ? 0 : span.x, k_last = empty ? -1 : span.y;
  auto slot_of = [&](int k) { return (((size_t)k * MB + mb) * 2 + (k == k_first)) * kSlotFloats; };
  const float* const lse0 = p.ws_out + (size_t)kRows * DV + r;
  const float* const frag0 = p.ws_out + (size_t)((w * NDB + db) * 4) * 256 + lane * 4;

  // This wave's share, in one pass: a running (reference, sum of weights,
  // weighted sum), the reference being the running maximum; the sums are
  // rescaled when it moves.  Full groups of U chunks are requested together
  // (their loads do not depend on one another: a long chunk list is bound by
  // memory latency, not bandwidth; U is small where lists are short, since the
  // registers it takes cost resident waves), the rest one at a time.
  float m = -INFINITY;
  float z = 0.f;
  f32x4_t acc[NQ4];
#pragma unroll
  for (int q4 = 0; q4 < NQ4; ++q4) acc[q4] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  auto rebase = [&](float m_new) {  // m_new > -inf
    const float keep = m == -INFINITY ? 0.f : expf(m - m_new);
    z *= keep;
#pragma unroll
    for (int q4 = 0; q4 < NQ4; ++q4) acc[q4] *= keep;
    m = m_new;
  };
  auto fold = [&](float ls, const f32x4_t (&v)[NQ4]) {  // m is at least ls
    // a slot marked "no key" may hold anything: its values are dropped, not multiplied by zero
    const bool live = ls != -INFINITY;
    const float wgt = live ? expf(ls - m) : 0.f;
    z += wgt;
#pragma unroll
    for (int q4 = 0; q4 < NQ4; ++q4) acc[q4] += wgt * (live ? v[q4] : f32x4_t{0.f, 0.f, 0.f, 0.f});
  };
  int k = k_first + kw;
  for (; k + (U - 1) * KW <= k_last; k += U * KW) {
    float ls[U];
    f32x4_t v[U][NQ4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t so = slot_of(k + u * KW);
      ls[u] = lse0[so];
#pragma unroll
      for (int q4 = 0; q4 < NQ4; ++q4) v[u][q4] = *(const f32x4_t*)(frag0 + so + (q_base + q4) * 256);
    }
    float m_new = m;
#pragma unroll
    for (int u = 0; u < U; ++u) m_new = fmaxf(m_new, ls[u]);
    if (m_new == -INFINITY) continue;
    if (m_new != m) rebase(m_new);
#pragma unroll
    for (int u = 0; u < U; ++u) fold(ls[u], v[u]);
  }
  for (; k <= k_last; k += KW) {
    const size_t so = slot_of(k);
    const float ls = lse0[so];
    f32x4_t v[NQ4];
#pragma unroll
    for (int q4 = 0; q4 < NQ4; ++q4) v[q4] = *(const f32x4_t*)(frag0 + so + (q_base + q4) * 256);
    if (ls > m) rebase(ls);
    if (m != -INFINITY) fold(ls, v);
  }
  // merge of the KW shares; wave q4 < 4 then finishes quarter q4 of the block
  float lse;
  f32x4_t res;
  int q_mine;
  if constexpr (KW == 1) {
    lse = m == -INFINITY ? -INFINITY : m + logf(z);
    const float inv = z > 0.f ? 1.0f / z : 0.f;
#pragma unroll
    for (int q4 = 0; q4 < NQ4; ++q4) acc[q4] *= inv;
    q_mine = -1;  // all four quarters, below
    res = acc[0];
  } else {
    red_m[kw][lane] = m;
    red_z[kw][lane] = z;
#pragma unroll
    for (int q4 = 0; q4 < NQ4; ++q4) red_a[kw][q4][lane] = acc[q4];
    __syncthreads();
    if (kw >= NQ4) return;
    q_mine = q_base + kw;
    float mm = -INFINITY;
#pragma unroll
    for (int j = 0; j < KW; ++j) mm = fmaxf(mm, red_m[j][lane]);
    float zz = 0.f;
    res = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (mm != -INFINITY) {
#pragma unroll
      for (int j = 0; j < KW; ++j) {
        const float mj = red_m[j][lane];
        const float e = mj == -INFINITY ? 0.f : expf(mj - mm);
        zz += e * red_z[j][lane];
        res += e * red_a[j][kw][lane];
      }
    }
    lse = mm == -INFINITY ? -INFINITY : mm + logf(zz);
    res *= zz > 0.f ? 1.0f / zz : 0.f;
  }
  if (!valid) return;
  if (db == 0 && hi == 0 && kx == 0 && q_mine <= 0) p.lse[((int64_t)b * p.T + t) * p.h_q + h] = lse;
  const int64_t ob = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    if (q_mine >= 0 && q4 != q_mine) continue;
    const f32x4_t v = q_mine >= 0 ? res : acc[q4 < NQ4 ? q4 : 0];
    const int dim = kx * (DV / KS) + 32 * db + 8 * q4 + 4 * hi;
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

}  // namespace gla
