// Host side of the tuned decode-attention path: shape check and plan, workspace
// size, and the launches of the main and merge kernels.
#pragma once

#include <algorithm>

#include "../../include/gla_decode.h"
#include "tuned_combine_kernel.hpp"
#include "tuned_main_kernel.hpp"

namespace gla {

// ---- host side ---------------------------------------------------------------

struct TunedPlan {
  int dv, dn;      // state dims (value / score)
  int ng, wpg, ks; // groups per workgroup, row slabs per group, waves per row slab
  int tok, stages; // tile tokens and pipeline depth of the chosen instantiation
  int rows;        // 32 * ng * wpg
  int mb;          // row blocks per (sequence, group)
  int units;       // batch * (h_c / ng) * mb
  int num_chunks;  // chunks of the tile list; the main-kernel grid is num_chunks * mb
  int chunk_tiles; // fixed tiles per chunk, 0: derived on the device
  size_t slot_floats;
  bool stream;     // fetch the cache with the streaming hint
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

constexpr int kMinChunkTiles = 4;

inline bool tuned_plan(const gla_decode_params* p, int is_gta, TunedPlan* plan) {
  const int ps = p->page_size;
  if (ps < 1 || ps > 64 || (ps & (ps - 1))) return false;  // 64, 32, ..., 1 tokens
  if (p->d_rope != 64 && p->d_rope != 48 && p->d_rope != 32) return false;  // (fewer than 64: padded inside the kernel)
  const bool lane = ps < 16;  // addresses per row and lane
  if (!(p->softmax_scale > 0.f)) return false;  // row maxima are taken on the raw dot products
  if (!((!is_gta && (p->d_v == 256 || p->d_v == 512)) || (is_gta && p->d_v == 128))) return false;
  // layout the kernels assume: token rows contiguous, everything 16-byte aligned
  if (p->state_stride[2] != p->d_v || p->rope_stride[1] != p->d_rope) return false;
  if (p->state_stride[0] % 8 || p->state_stride[1] % 8 || p->rope_stride[0] % 8) return false;
  if (p->state_stride[0] < 0 || p->state_stride[1] < 0 || p->rope_stride[0] < 0 ||
      p->state_stride[0] >= (1ll << 30) || p->state_stride[1] >= (1ll << 30) || p->rope_stride[0] >= (1ll << 30))
    return false;  // page / group strides are handled as 32-bit byte counts
  if (p->num_pages >= (1ll << 31)) return false;
  for (int i = 0; i < 3; ++i)
    if (p->q_nope_stride[i] % 8 || p->q_rope_stride[i] % 8 || p->out_stride[i] % 4) return false;
  if (p->q_nope && !(aligned16(p->q_nope) && aligned16(p->q_rope) && aligned16(p->state_cache) &&
                     aligned16(p->rope_cache) && aligned16(p->out)))
    return false;
  const int rows_group = (p->num_q_heads / p->num_groups) * p->q_len;
  // waves per group from the rows of a group, then as many groups per workgroup
  // as four waves allow (they share one RoPE-key tile)
  // A latent of 512 dims needs two waves per row slab: 32 rows x 512 fp32
  // output accumulators alone would fill a wave's accumulation registers.
  const int ks = p->d_v > 256 ? 2 : 1;
  const int wpg = rows_group <= 32 ? 1 : ((rows_group <= 64 || ks == 2) ? 2 : 4);
  int ng = 4 / (wpg * ks);
  while (ng > 1 && (p->num_groups % ng || 4 * (ng * 32 * p->d_v * 2 + 32 * 128) > 160 * 1024)) ng >>= 1;
  plan->dv = p->d_v;
  plan->dn = p->d_nope;
  plan->ng = ng;
  plan->wpg = wpg;
  plan->ks = ks;
  plan->rows = 32 * ng * wpg;
  plan->mb = (rows_group + 32 * wpg - 1) / (32 * wpg);
  plan->units = p->batch * (p->num_groups / ng) * plan->mb;
  // (small pages: page-id windows in LDS where tiles and mailboxes leave room for them, else in registers)
  const bool lds_windows = lane && tuned_windows_fit(p->d_v, ng, wpg, ks);
  const int tok = kTok, stages = tuned_stages(p->d_v, ng, wpg, ks, lds_windows);
  // co-resident workgroups per CU: one wave per SIMD, 160 KiB of LDS
  const int smem = stages * (ng * tok * p->d_v * 2 + tok * 128) + (ks > 1 ? ng * wpg * ks * 4096 : 0) +
                   (lds_windows ? ng * wpg * ks * 2 * kPageWindow * 4 : 0);
  if (smem > 160 * 1024) return false;
  const int per_cu = std::max(1, std::min((160 * 1024) / smem, 4 / (ng * wpg * ks)));
  plan->tok = tok;
  plan->stages = stages;
  // the tile list holds each (sequence, group block) once; every chunk of it is
  // worked on by mb workgroups (one per row block), so the grid is num_chunks * mb
  const int64_t max_tiles = ((int64_t)p->max_pages_per_seq * p->page_size + tok - 1) / tok;
  const int64_t bound = (int64_t)(plan->units / plan->mb) * max_tiles;
  if (bound * plan->mb > 0x3fffffff) return false;
  if (p->num_splits > 0) {
    plan->chunk_tiles = (int)((max_tiles + p->num_splits - 1) / p->num_splits);
    plan->num_chunks = (int)std::max<int64_t>(1, (bound + plan->chunk_tiles - 1) / plan->chunk_tiles);
  } else {
    plan->chunk_tiles = 0;
    // one chunk per resident workgroup, but no chunk shorter than kMinChunkTiles
    // (by the upper bound on the list length): a partial costs as much memory
    // traffic as three or four tiles, and every extra chunk is one more to merge
    const int64_t resident = std::max<int64_t>(1, (int64_t)device_cu_count() * per_cu / plan->mb);
    const int64_t by_length = std::max<int64_t>(1, bound / kMinChunkTiles);
    plan->num_chunks = (int)std::max<int64_t>(1, std::min<int64_t>(by_length, resident));
  }
  plan->slot_floats = (size_t)plan->rows * p->d_v + (size_t)32 * ng * wpg * ks;
  // upper bound of the batch's cache bytes (the lengths are known on the device only) against the chip's
  // last-level cache
  plan->stream = bound * tok * 2 * ((int64_t)ng * p->d_v + p->d_rope) > kLastLevelCacheBytes;
  return true;
}

inline bool tuned_supported(const gla_decode_params* p, int is_gta) {
  TunedPlan plan;
  return tuned_plan(p, is_gta, &plan);
}

// Workspace: two partial slots per chunk, then per unit the chunk range holding it.
inline size_t tuned_slots_bytes(const TunedPlan& plan) {
  return (((size_t)plan.num_chunks * plan.mb * 2 * plan.slot_floats * sizeof(float)) + 255) & ~(size_t)255;
}

inline size_t tuned_workspace(const gla_decode_params* p, int is_gta) {
  TunedPlan plan;
  if (!tuned_plan(p, is_gta, &plan)) return 0;
  return tuned_slots_bytes(plan) + (size_t)plan.units * 2 * sizeof(int32_t);
}

template <int DV, int DN, int NG, int WPG, int KS, int TOK, bool STREAM>
inline int launch_tuned_main(const DevParams& d, dim3 mgrid, dim3 mblock, hipStream_t st) {
  constexpr int STAGES = tuned_stages(DV, NG, WPG, KS), STAGES_LANE = tuned_stages(DV, NG, WPG, KS, true);
  constexpr bool kLaneFits = tuned_windows_fit(DV, NG, WPG, KS);
  if (d.lg_page == 6) {
    hipLaunchKernelGGL((tuned_main_kernel<DV, DN, 64, NG, WPG, KS, TOK, STAGES, 0, STREAM>), mgrid, mblock, 0, st, d);
  } else if (d.lg_page >= 4) {
    hipLaunchKernelGGL((tuned_main_kernel<DV, DN, 64, NG, WPG, KS, TOK, STAGES, 1, STREAM>), mgrid, mblock, 0, st, d);
  } else {
    if constexpr (kLaneFits)
      hipLaunchKernelGGL((tuned_main_kernel<DV, DN, 64, NG, WPG, KS, TOK, STAGES_LANE, 2, STREAM>), mgrid, mblock, 0, st, d);
    else  // (no LDS left for the page-id windows: kept in registers)
      hipLaunchKernelGGL((tuned_main_kernel<DV, DN, 64, NG, WPG, KS, TOK, STAGES, 3, STREAM>), mgrid, mblock, 0, st, d);
  }
  return GLA_OK;
}

template <int DV, int DN, int NG, int WPG, int KS, int TOK>
inline int launch_tuned_variant(const TunedPlan& plan, DevParams& d, hipStream_t st, hipEvent_t* ev) {
  if (ev) (void)hipEventRecord(ev[0], st);
  const dim3 mgrid(plan.num_chunks * plan.mb), mblock(64 * NG * WPG * KS);
  // (plan.stream: the cache of this batch can be larger than the last-level cache: fetch it with the streaming hint)
  const int lrc = plan.stream ? launch_tuned_main<DV, DN, NG, WPG, KS, TOK, true>(d, mgrid, mblock, st)
                              : launch_tuned_main<DV, DN, NG, WPG, KS, TOK, false>(d, mgrid, mblock, st);
  if (lrc != GLA_OK) return lrc;
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[1], st);
  // waves per merge task from the expected number of chunks per unit
  const int64_t span_est = (plan.num_chunks + std::max(1, plan.units / plan.mb) - 1) / std::max(1, plan.units / plan.mb) + 1;
  const dim3 cgrid(plan.units, NG * WPG * (DV / 32));
  if (span_est <= 2)
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 1, 1, 2>), cgrid, dim3(64), 0, st, d);
  else if (span_est <= 6)  // (one wave with four chunks in flight: a fourth of the waves to launch, no merge through LDS)
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 1, 1, 4>), cgrid, dim3(64), 0, st, d);
  else if (span_est <= 12)
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 4, 1, 2>), cgrid, dim3(256), 0, st, d);
  else if (span_est <= 64)  // (a wave folds eight chunks per round trip: four waves do for fairly long lists)
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 4, 1, 8>), cgrid, dim3(256), 0, st, d);
  else if ((int64_t)cgrid.x * cgrid.y * 4 > 4 * device_cu_count())
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 16, 1, 4>), cgrid, dim3(1024), 0, st, d);
  else  // few tasks: each cut into quarters (see the kernel)
    hipLaunchKernelGGL((tuned_combine_kernel<DV, NG, WPG, KS, TOK, 16, 4, 4>), dim3(cgrid.x, cgrid.y * 4), dim3(1024), 0, st, d);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[2], st);
  return GLA_OK;
}

template <int DV, int DN>
inline int launch_tuned_shape(const TunedPlan& plan, DevParams& d, hipStream_t st, hipEvent_t* ev) {
  if constexpr (DV > 256) {
    switch (plan.ng * 100 + plan.wpg * 10 + plan.ks) {
      case 112: return launch_tuned_variant<DV, DN, 1, 1, 2, kTok>(plan, d, st, ev);
      case 122: return launch_tuned_variant<DV, DN, 1, 2, 2, kTok>(plan, d, st, ev);
      default: return GLA_ERR_UNSUPPORTED_SHAPE;
    }
  } else {
    switch (plan.ng * 100 + plan.wpg * 10 + plan.ks) {
      case 111: return launch_tuned_variant<DV, DN, 1, 1, 1, kTok>(plan, d, st, ev);
      case 121: return launch_tuned_variant<DV, DN, 1, 2, 1, kTok>(plan, d, st, ev);
      case 141: return launch_tuned_variant<DV, DN, 1, 4, 1, kTok>(plan, d, st, ev);
      case 211: return launch_tuned_variant<DV, DN, 2, 1, 1, kTok>(plan, d, st, ev);
      case 221: return launch_tuned_variant<DV, DN, 2, 2, 1, kTok>(plan, d, st, ev);
      case 411:
        if constexpr (DV <= 128) return launch_tuned_variant<DV, DN, 4, 1, 1, kTok>(plan, d, st, ev);
        else return GLA_ERR_UNSUPPORTED_SHAPE;
      default: return GLA_ERR_UNSUPPORTED_SHAPE;
    }
  }
}

inline int tuned_launch(const gla_decode_params* p, int is_gta, DevParams& d, hipStream_t st,
                        hipEvent_t* ev) {
  TunedPlan plan;
  if (!tuned_plan(p, is_gta, &plan)) return GLA_ERR_UNSUPPORTED_SHAPE;
  d.ws_out = (float*)p->workspace;
  d.ws_lse = (float*)((char*)p->workspace + tuned_slots_bytes(plan));  // per-unit chunk ranges (int32 pairs)
  d.num_chunks = plan.num_chunks;
  d.chunk_tiles = plan.chunk_tiles;
  {
    const int g_q = p->num_q_heads / p->num_groups;
    int lg = 0;
    while ((1 << lg) < p->page_size) ++lg;
    d.mb = plan.mb;
    d.upb = p->num_groups / plan.ng;
    d.lg_page = lg;
    d.xcd_map = (plan.num_chunks * plan.mb) % (8 * plan.mb) == 0 ? 1 : 0;
    d.tiles_full = (int)(((int64_t)p->max_pages_per_seq * p->page_size + plan.tok - 1) / plan.tok);
    const int64_t total_full = (int64_t)p->batch * d.upb * d.tiles_full;
    d.chunk_guess = plan.chunk_tiles > 0 ? plan.chunk_tiles
                                         : (int)((total_full + plan.num_chunks - 1) / plan.num_chunks);
    d.fd_mb = make_fastdiv((uint32_t)plan.mb);
    d.fd_chunks = make_fastdiv((uint32_t)plan.num_chunks);
    d.fd_gq = make_fastdiv((uint32_t)g_q);
    d.fd_tiles_full = make_fastdiv((uint32_t)d.tiles_full);
    d.fd_units_full = make_fastdiv((uint32_t)(d.upb * d.tiles_full));
    d.fd_upb_mb = make_fastdiv((uint32_t)(d.upb * plan.mb));
  }
  if (plan.dv == 256 && plan.dn == 256) return launch_tuned_shape<256, 256>(plan, d, st, ev);
  if (plan.dv == 128 && plan.dn == 64) return launch_tuned_shape<128, 64>(plan, d, st, ev);
  if (plan.dv == 512 && plan.dn == 512) return launch_tuned_shape<512, 512>(plan, d, st, ev);
  return GLA_ERR_UNSUPPORTED_SHAPE;
}

}  // namespace gla
