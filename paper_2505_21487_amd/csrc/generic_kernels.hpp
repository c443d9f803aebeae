// Shape-agnostic decode-attention kernels: one wave64 per (sequence, query row,
// head, key split), scalar fp32 FMAs, online softmax one key at a time.  Slow
// (every head re-reads its group's cache) but valid for any dims, page size and
// strides; it serves shapes without a tuned kernel and cross-checks the tuned
// one.  Same operation as the tuned path: score = scale * (q_nope . state[:d_n]
// + q_rope . rope_key), softmax over visible keys, output = weights . state
// (paper Sections 2.1, 3.3.1, 3.3.2).
#pragma once

#include "common.hpp"

namespace gla {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// NV = ceil(d_v / 64): state elements owned by one lane.
template <int NV>
__global__ __launch_bounds__(64) void generic_main_kernel(DevParams p) {
  const int row = blockIdx.x;
  const int s = blockIdx.y;
  const int lane = threadIdx.x;
  const int h = row % p.h_q;
  const int t = (row / p.h_q) % p.T;
  const int b = row / (p.h_q * p.T);
  const int g = h / p.g_q;

  const int64_t L = p.seq_lens[b];
  const int64_t n_vis = p.causal ? L - p.T + 1 + t : L;
  const int64_t span = (int64_t)p.pages_per_split * p.P;
  const int64_t j0 = (int64_t)s * span;
  const int64_t j1 = (j0 + span < n_vis) ? j0 + span : n_vis;

  float qn[NV], qr[2], o[NV];
  const uint16_t* qn_ptr = p.q_nope + b * p.qn_s[0] + t * p.qn_s[1] + h * p.qn_s[2];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int d = lane + 64 * i;
    qn[i] = (d < p.d_n) ? bf16_bits_to_f32(qn_ptr[d]) : 0.f;
    o[i] = 0.f;
  }
  if (p.d_r > 0) {
    const uint16_t* qr_ptr = p.q_rope + b * p.qr_s[0] + t * p.qr_s[1] + h * p.qr_s[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int d = lane + 64 * i;
      qr[i] = (d < p.d_r) ? bf16_bits_to_f32(qr_ptr[d]) : 0.f;
    }
  } else {
    qr[0] = qr[1] = 0.f;
  }

  float m = -INFINITY, l = 0.f;
  int64_t page = 0;
  for (int64_t j = j0; j < j1; ++j) {
    const int off = (int)(j % p.P);
    if (off == 0 || j == j0) page = p.page_table[(int64_t)b * p.max_pages + j / p.P];
    const uint16_t* c = p.state + page * p.st_s[0] + g * p.st_s[1] + off * p.st_s[2];
    const uint16_t* kk = p.kstate ? p.kstate + page * p.k_s[0] + g * p.k_s[1] + off * p.k_s[2] : nullptr;
    float cv[NV];
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int d = lane + 64 * i;
      cv[i] = (d < p.d_v) ? bf16_bits_to_f32(c[d]) : 0.f;
      // key: the first d_n dims of the state row, or a row of the separate key cache (qn is zero beyond d_n)
      acc += qn[i] * (kk ? ((d < p.d_n) ? bf16_bits_to_f32(kk[d]) : 0.f) : cv[i]);
    }
    if (p.d_r > 0) {
      const uint16_t* k = p.rope + page * p.rp_s[0] + off * p.rp_s[1];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int d = lane + 64 * i;
        if (d < p.d_r) acc += qr[i] * bf16_bits_to_f32(k[d]);
      }
    }
    const float sj = p.scale * wave_sum(acc);
    const float m_new = fmaxf(m, sj);
    const float alpha = expf(m - m_new);  // m = -inf on the first key -> 0
    const float pj = expf(sj - m_new);
    l = l * alpha + pj;
#pragma unroll
    for (int i = 0; i < NV; ++i) o[i] = o[i] * alpha + pj * cv[i];
    m = m_new;
  }

  const bool empty = j1 <= j0;
  const float inv = empty ? 0.f : 1.f / l;
  const float lse = empty ? -INFINITY : m + logf(l);
  if (p.splits == 1) {
    if (lane == 0) p.lse[row] = lse;
    const int64_t base = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int d = lane + 64 * i;
      if (d < p.d_v) {
        if (p.out_fp32) ((float*)p.out)[base + d] = o[i] * inv;
        else ((uint16_t*)p.out)[base + d] = f32_to_bf16_bits(o[i] * inv);
      }
    }
  } else {
    const int64_t rows = (int64_t)p.B * p.T * p.h_q;
    if (lane == 0) p.ws_lse[(int64_t)s * rows + row] = lse;
    float* dst = p.ws_out + ((int64_t)s * rows + row) * p.d_v;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int d = lane + 64 * i;
      if (d < p.d_v) dst[d] = o[i] * inv;
    }
  }
}

// Merge of the per-split partial results: lse = ln sum_s exp(lse_s),
// out = sum_s exp(lse_s - lse) * out_s.  One wave per output row.
__global__ __launch_bounds__(64) void generic_combine_kernel(DevParams p) {
  const int row = blockIdx.x;
  const int lane = threadIdx.x;
  const int h = row % p.h_q;
  const int t = (row / p.h_q) % p.T;
  const int b = row / (p.h_q * p.T);
  const int64_t rows = (int64_t)p.B * p.T * p.h_q;
  float m = -INFINITY;
  for (int s = 0; s < p.splits; ++s) m = fmaxf(m, p.ws_lse[(int64_t)s * rows + row]);
  float z = 0.f;
  if (m != -INFINITY)
    for (int s = 0; s < p.splits; ++s) z += expf(p.ws_lse[(int64_t)s * rows + row] - m);
  const float lse = (m == -INFINITY) ? -INFINITY : m + logf(z);
  if (lane == 0) p.lse[row] = lse;
  const int64_t base = b * p.out_s[0] + t * p.out_s[1] + h * p.out_s[2];
  for (int d = lane; d < p.d_v; d += 64) {
    float acc = 0.f;
    if (m != -INFINITY) {
      for (int s = 0; s < p.splits; ++s) {
        const float ls = p.ws_lse[(int64_t)s * rows + row];
        if (ls != -INFINITY) acc += expf(ls - lse) * p.ws_out[((int64_t)s * rows + row) * p.d_v + d];
      }
    }
    if (p.out_fp32) ((float*)p.out)[base + d] = acc;
    else ((uint16_t*)p.out)[base + d] = f32_to_bf16_bits(acc);
  }
}

}  // namespace gla
