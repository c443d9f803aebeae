// Shared device-side declarations of the decode-attention library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gla {

// Division of a 32-bit unsigned number by a divisor fixed on the host, as one
// multiply-high and two shifts:  n / d == (t + ((n - t) >> s1)) >> s2  with
// t = mulhi(n, m), exact for every n < 2^32 (round-up method: m = floor(2^32 *
// (2^l - d) / d) + 1 with l = ceil(log2 d), s1 = min(l, 1), s2 = l - s1).
struct FastDiv {
  uint32_t m, s1, s2;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f = {0u, 0u, 0u};
  if (d <= 1) return f;  // t = 0, q = n
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
  f.s1 = 1;
  f.s2 = l - 1;
  return f;
}
__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f) {
  const uint32_t t = __umulhi(n, f.m);
  return (t + ((n - t) >> f.s1)) >> f.s2;
}

// Cache bytes of a batch from which the MFMA kernels fetch the cache with the streaming hint: the 256 MB
// of the chip's last-level cache (a smaller cache can still be there at the next decode step).
constexpr int64_t kLastLevelCacheBytes = 256ll << 20;

// Kernel-argument block: a flattened copy of the caller's parameter struct.
struct DevParams {
  const uint16_t* q_nope;
  const uint16_t* q_rope;
  const uint16_t* state;
  const uint16_t* rope;
  const uint16_t* kstate;  // keys in a cache of their own (grouped-query baseline); null: key = first d_n dims of the state row
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
  int64_t k_s[3];          // strides of kstate (page, head, token)
  int64_t out_s[3];
  int32_t B, T, h_q, h_c, g_q;
  int32_t d_v, d_n, d_r;
  int32_t P, max_pages;
  int32_t causal, out_fp32;
  float scale;
  // generic kernel: uniform split of every sequence's page range
  int32_t splits, pages_per_split;
  int64_t stream_min_bytes; // second MFMA kernel: a batch with more cache bytes than this is fetched with the streaming hint
  int32_t flex_rb;          // flex kernel: blocks of 16 query rows per group
  int32_t* flex_rng;        // flex kernel: per (sequence, strand) the first chunk holding a piece of it (x 2 + its slot) and the last
  // tuned kernel: flat partition of all key tiles of the batch into chunks
  int32_t num_chunks;       // chunks of the tile list (the main kernel runs one workgroup per chunk and row block)
  int32_t chunk_tiles;      // > 0: fixed tiles per chunk; 0: ceil(total / num_chunks)
  // tuned kernel: constants of the plan, worked out once on the host
  int32_t mb;               // row blocks per group (workgroups per chunk)
  int32_t upb;              // units (group blocks) per sequence
  int32_t lg_page;          // log2(page size)
  int32_t xcd_map;          // 1: grid is a multiple of 8 * mb, chunks are laid out per XCD
  int32_t tiles_full;       // tiles of a sequence that fills its page-table row
  int32_t chunk_guess;      // chunk length if every sequence did
  FastDiv fd_mb, fd_chunks, fd_gq, fd_tiles_full, fd_units_full, fd_upb_mb;
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
