// Shared device-side declarations of the decode-attention library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gla {

// Kernel-argument block: a flattened copy of the caller's parameter struct.
struct DevParams {
  const uint16_t* q_nope;
  const uint16_t* q_rope;
  const uint16_t* state;
  const uint16_t* rope;
  const int32_t* page_table;
  const int32_t* seq_lens;
  void* out;
  float* lse;
  float* ws_out;   // partial outputs (fp32, normalised by their own row sum)
  float* ws_lse;   // partial log-sum-exp
  int64_t qn_s[3];
  int64_t qr_s[3];
  int64_t st_s[3];
  int64_t rp_s[2];
  int64_t out_s[3];
  int32_t B, T, h_q, h_c, g_q;
  int32_t d_v, d_n, d_r;
  int32_t P, max_pages;
  int32_t causal, out_fp32;
  float scale;
  // generic kernel: uniform split of every sequence's page range
  int32_t splits, pages_per_split;
  // tuned kernel: flat partition of all key tiles of the batch into chunks
  int32_t num_chunks;       // chunks of the tile list (the main kernel runs one workgroup per chunk and row block)
  int32_t chunk_tiles;      // > 0: fixed tiles per chunk; 0: ceil(total / num_chunks)
};

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t v) {
  return __builtin_bit_cast(float, ((uint32_t)v) << 16);
}

// Round-to-nearest-even fp32 -> bf16 (NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace gla
