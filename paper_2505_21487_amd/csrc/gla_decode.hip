// Host side of the decode-attention library: argument checks, kernel choice,
// workspace sizing and launches.  The exported functions and their contracts
// are declared in include/gla_decode.h.
#include "../../include/gla_decode.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>

#include "common.hpp"
#include "flex_kernels.hpp"
#include "generic_kernels.hpp"
#include "proj_kernels.hpp"
#include "tuned_kernels.hpp"

namespace gla {
namespace {

constexpr int kVersion = 104;  // 1.04: gqa_decode; second MFMA kernel for small head shapes

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// `is_gta` arguments: 0 = GLA / MLA shape, 1 = GTA, kModeGqa = grouped-query baseline with its own key cache.
constexpr int kModeGqa = 2;
// The key cache of a gqa_decode call in flight (host-side hand-over from the entry point to the launch code).
struct KeyCache {
  const void* ptr;
  int64_t stride[3];
};

int check_shape(const gla_decode_params* p, int is_gta) {
  if (!p) return GLA_ERR_INVALID_ARG;
  if (p->batch < 0 || p->q_len < 1 || p->q_len > 4) return GLA_ERR_INVALID_ARG;
  if (p->num_q_heads < 1 || p->num_groups < 1 || p->num_q_heads % p->num_groups != 0)
    return GLA_ERR_INVALID_ARG;
  if (p->d_v < 1 || p->d_nope < 1 || p->d_rope < 0) return GLA_ERR_INVALID_ARG;
  if (is_gta == kModeGqa) {
    if (p->d_rope != 0) return GLA_ERR_INVALID_ARG;  // (rotated dims are part of the cached key)
  } else if (is_gta) {
    if (p->d_v % 2 != 0 || p->d_nope != p->d_v / 2) return GLA_ERR_INVALID_ARG;
  } else {
    if (p->d_nope != p->d_v) return GLA_ERR_INVALID_ARG;
  }
  if (p->page_size < 1 || p->max_pages_per_seq < 1 || p->num_pages < 0) return GLA_ERR_INVALID_ARG;
  if (p->num_splits < 0) return GLA_ERR_INVALID_ARG;
  if (p->out_dtype != GLA_OUT_BF16 && p->out_dtype != GLA_OUT_FP32) return GLA_ERR_INVALID_ARG;
  if (p->impl != GLA_IMPL_AUTO && p->impl != GLA_IMPL_GENERIC && p->impl != GLA_IMPL_TUNED)
    return GLA_ERR_INVALID_ARG;
  if ((int64_t)p->batch * p->q_len * p->num_q_heads > (int64_t)0x7fffffff) return GLA_ERR_INVALID_ARG;
  return GLA_OK;
}

bool generic_supported(const gla_decode_params* p) { return p->d_v <= 1024 && p->d_nope <= 1024 && p->d_rope <= 128; }

// ---- flex kernel (flex_kernels.hpp): which instantiation, how the key tiles are cut into chunks
struct FlexPlan {
  int id;           // index into the instantiation list below, -1: none
  int gpw;          // groups per wave (2: two groups of at most eight rows share a wave's 16 rows)
  int rb;           // blocks of 16 rows per group
  int strands;      // (group block, row block) pairs: each walks the whole tile list
  int chunks;       // chunks of the tile list (one wave per chunk and strand)
  int chunk_tiles;  // > 0: fixed tiles per chunk; 0: ceil(total / chunks), worked out on the device
  bool lane;        // pages of fewer than 32 tokens: the kernel variant that forms one address per row and lane
};

int flex_variant(const gla_decode_params* p, int mode) {
  if (mode == kModeGqa) {
    if (p->d_nope == 128 && p->d_v == 128) return 0;
    if (p->d_nope == 64 && p->d_v == 64) return 1;
    return -1;
  }
  if (mode == 1) {  // GTA: tied state d_h, key = its first half + a RoPE key of d_h / 2
    if (p->d_v == 64 && p->d_rope == 32) return 2;
    if (p->d_v == 96 && p->d_rope == 48) return 3;
    return -1;
  }
  if (p->d_v == 128 && p->d_rope == 32) return 4;  // latent heads of 2 x 64 dims
  return -1;
}

bool flex_plan(const gla_decode_params* p, int mode, const KeyCache* kc, FlexPlan* plan) {
  plan->id = flex_variant(p, mode);
  if (plan->id < 0) return false;
  const int ps = p->page_size;
  if (ps < 1 || (ps & (ps - 1))) return false;
  plan->lane = ps < 32;  // (else a tile of 32 tokens lies inside one page)
  if (!(p->softmax_scale > 0.f)) return false;
  // layout the kernel assumes: contiguous rows, 16-byte aligned rows and bases
  if (p->state_stride[2] != p->d_v || p->state_stride[0] % 8 || p->state_stride[1] % 8) return false;
  if (p->d_rope > 0 && (p->rope_stride[1] != p->d_rope || p->rope_stride[0] % 8)) return false;
  for (int i = 0; i < 3; ++i)
    if (p->q_nope_stride[i] % 4 || (p->d_rope > 0 && p->q_rope_stride[i] % 4) || p->out_stride[i] % 4) return false;
  if (p->q_nope && (((uintptr_t)p->q_nope | (uintptr_t)p->q_rope) & 7u)) return false;
  if (p->q_nope && (((uintptr_t)p->state_cache | (uintptr_t)p->rope_cache | (uintptr_t)p->out) & 15u)) return false;
  if (mode == kModeGqa && kc && kc->ptr) {
    if (kc->stride[2] != p->d_nope || kc->stride[0] % 8 || kc->stride[1] % 8 || ((uintptr_t)kc->ptr & 15u)) return false;
  }
  const int rows_group = (p->num_q_heads / p->num_groups) * p->q_len;
  plan->rb = (rows_group + 15) / 16;
  plan->gpw = (plan->id == 2 && rows_group <= 8 && p->num_groups % 2 == 0) ? 2 : 1;
  plan->strands = (p->num_groups / plan->gpw) * plan->rb;
  // the tile list holds every sequence once; its length is known on the device only, here its upper bound
  const int64_t max_tiles = std::max<int64_t>(1, ((int64_t)p->max_pages_per_seq * ps + 31) / 32);
  const int64_t bound = (int64_t)p->batch * max_tiles;
  int64_t chunks;
  if (p->num_splits > 0) {
    plan->chunk_tiles = (int)((max_tiles + p->num_splits - 1) / p->num_splits);
    chunks = (bound + plan->chunk_tiles - 1) / plan->chunk_tiles;
  } else {
    // one wave per SIMD (what is resident at once), chunks of at least eight tiles (by the upper bound):
    // a wave's start (lengths, page ids, queries, first tiles) costs several tiles' worth of time
    plan->chunk_tiles = 0;
    chunks = std::min<int64_t>((4 * (int64_t)device_cu_count() + plan->strands - 1) / plan->strands, bound / 8);
  }
  chunks = std::max<int64_t>(1, chunks);
  if (chunks * plan->strands > (int64_t)0x3fffffff || bound + chunks > (int64_t)0x7fffffff) return false;
  plan->chunks = (int)chunks;
  return true;
}

// Workspace: two partial slots of 16 rows per wave, then per (sequence, strand) the chunks holding its pieces.
size_t flex_slots(const FlexPlan& plan) { return (size_t)plan.chunks * plan.strands * 2 * 16; }
size_t flex_workspace(const gla_decode_params* p, const FlexPlan& plan) {
  return align_up(flex_slots(plan) * p->d_v * sizeof(float), 256) + align_up(flex_slots(plan) * sizeof(float), 256) +
         align_up((size_t)p->batch * plan.strands * 2 * sizeof(int32_t), 256);
}

int generic_splits(const gla_decode_params* p) {
  const int64_t rows = std::max<int64_t>(1, (int64_t)p->batch * p->q_len * p->num_q_heads);
  int64_t s = p->num_splits > 0 ? p->num_splits : (4096 + rows - 1) / rows;
  s = std::min<int64_t>(s, p->max_pages_per_seq);
  s = std::min<int64_t>(s, 65535);
  return (int)std::max<int64_t>(s, 1);
}

// Internal choice: GLA_IMPL_TUNED (the tuned kernel), kImplFlex (the second MFMA kernel, reported to
// callers as GLA_IMPL_TUNED: "an MFMA kernel"), GLA_IMPL_GENERIC, or an error.
constexpr int kImplFlex = 3;
int select_kernel(const gla_decode_params* p, int is_gta, const KeyCache* kc) {
  int rc = check_shape(p, is_gta);
  if (rc != GLA_OK) return rc;
  const bool tuned_ok = is_gta != kModeGqa && tuned_supported(p, is_gta);
  FlexPlan fp;
  const bool flex_ok = !tuned_ok && flex_plan(p, is_gta, kc, &fp);
  if (p->impl != GLA_IMPL_GENERIC) {
    if (tuned_ok) return GLA_IMPL_TUNED;
    if (flex_ok) return kImplFlex;
    if (p->impl == GLA_IMPL_TUNED) return GLA_ERR_UNSUPPORTED_SHAPE;
  }
  return generic_supported(p) ? GLA_IMPL_GENERIC : GLA_ERR_UNSUPPORTED_SHAPE;
}
int select_impl(const gla_decode_params* p, int is_gta) {
  const int k = select_kernel(p, is_gta, nullptr);
  return k == kImplFlex ? GLA_IMPL_TUNED : k;
}

size_t generic_workspace(const gla_decode_params* p) {
  const int s = generic_splits(p);
  if (s == 1) return 0;
  const size_t rows = (size_t)p->batch * p->q_len * p->num_q_heads;
  return align_up((size_t)s * rows * p->d_v * sizeof(float), 256) +
         align_up((size_t)s * rows * sizeof(float), 256);
}

int check_pointers(const gla_decode_params* p) {
  if (p->batch == 0) return GLA_OK;
  if (!p->q_nope || !p->state_cache || !p->page_table || !p->seq_lens || !p->out || !p->lse)
    return GLA_ERR_INVALID_ARG;
  if (p->d_rope > 0 && (!p->q_rope || !p->rope_cache)) return GLA_ERR_INVALID_ARG;
  return GLA_OK;
}

template <int DN, int DR, int DV, bool SEPK, int GPW>
void launch_flex_main(bool lane, dim3 grid, dim3 block, hipStream_t st, const DevParams& d) {
  if (lane) hipLaunchKernelGGL((flex_main_kernel<DN, DR, DV, SEPK, GPW, true>), grid, block, 0, st, d);
  else hipLaunchKernelGGL((flex_main_kernel<DN, DR, DV, SEPK, GPW, false>), grid, block, 0, st, d);
}

int launch_flex(const gla_decode_params* p, const FlexPlan& plan, DevParams& d, hipStream_t st, hipEvent_t* ev) {
  d.num_chunks = plan.chunks;
  d.chunk_tiles = plan.chunk_tiles;
  d.flex_rb = plan.rb;
  int lg = 0;
  while ((1 << lg) < p->page_size) ++lg;
  d.lg_page = lg;
  const size_t rows = (size_t)p->batch * p->q_len * p->num_q_heads;
  {
    char* w = (char*)p->workspace;
    d.ws_out = (float*)w;
    w += align_up(flex_slots(plan) * p->d_v * sizeof(float), 256);
    d.ws_lse = (float*)w;
    w += align_up(flex_slots(plan) * sizeof(float), 256);
    d.flex_rng = (int32_t*)w;
  }
  const int64_t waves = (int64_t)plan.chunks * plan.strands;
  const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
  if (ev) (void)hipEventRecord(ev[0], st);
  switch (plan.id) {
    case 0: launch_flex_main<128, 0, 128, true, 1>(plan.lane, grid, block, st, d); break;
    case 1: launch_flex_main<64, 0, 64, true, 1>(plan.lane, grid, block, st, d); break;
    case 2:
      if (plan.gpw == 2) launch_flex_main<32, 32, 64, false, 2>(plan.lane, grid, block, st, d);
      else launch_flex_main<32, 32, 64, false, 1>(plan.lane, grid, block, st, d);
      break;
    case 3: launch_flex_main<48, 48, 96, false, 1>(plan.lane, grid, block, st, d); break;
    case 4: launch_flex_main<128, 32, 128, false, 1>(plan.lane, grid, block, st, d); break;
    default: return GLA_ERR_UNSUPPORTED_SHAPE;
  }
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[1], st);
  // (always: it also fills the rows of empty sequences, which no chunk holds)
  if (plan.gpw == 2)
    hipLaunchKernelGGL(flex_combine_kernel<2>, dim3((unsigned)rows), dim3(64), 0, st, d);
  else
    hipLaunchKernelGGL(flex_combine_kernel<1>, dim3((unsigned)rows), dim3(64), 0, st, d);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[2], st);
  return GLA_OK;
}

void fill_dev(const gla_decode_params* p, DevParams* d) {
  std::memset(d, 0, sizeof(*d));
  d->q_nope = (const uint16_t*)p->q_nope;
  d->q_rope = (const uint16_t*)p->q_rope;
  d->state = (const uint16_t*)p->state_cache;
  d->rope = (const uint16_t*)p->rope_cache;
  d->page_table = p->page_table;
  d->seq_lens = p->seq_lens;
  d->out = p->out;
  d->lse = p->lse;
  for (int i = 0; i < 3; ++i) {
    d->qn_s[i] = p->q_nope_stride[i];
    d->qr_s[i] = p->q_rope_stride[i];
    d->st_s[i] = p->state_stride[i];
    d->out_s[i] = p->out_stride[i];
  }
  d->rp_s[0] = p->rope_stride[0];
  d->rp_s[1] = p->rope_stride[1];
  d->B = p->batch;
  d->T = p->q_len;
  d->h_q = p->num_q_heads;
  d->h_c = p->num_groups;
  d->g_q = p->num_q_heads / p->num_groups;
  d->d_v = p->d_v;
  d->d_n = p->d_nope;
  d->d_r = p->d_rope;
  d->P = p->page_size;
  d->max_pages = p->max_pages_per_seq;
  d->causal = p->causal ? 1 : 0;
  d->out_fp32 = p->out_dtype == GLA_OUT_FP32;
  d->scale = p->softmax_scale;
  d->stream_min_bytes = kLastLevelCacheBytes;
}

int launch_generic(const gla_decode_params* p, DevParams& d, hipStream_t st, hipEvent_t* ev) {
  const int s = generic_splits(p);
  d.splits = s;
  d.pages_per_split = (p->max_pages_per_seq + s - 1) / s;
  const size_t rows = (size_t)p->batch * p->q_len * p->num_q_heads;
  if (s > 1) {
    d.ws_out = (float*)p->workspace;
    d.ws_lse = (float*)((char*)p->workspace + align_up((size_t)s * rows * p->d_v * sizeof(float), 256));
  }
  dim3 grid((unsigned)rows, (unsigned)s), block(64);
  const int nv = (std::max(p->d_v, p->d_nope) + 63) / 64;
  if (ev) (void)hipEventRecord(ev[0], st);
  if (nv <= 2) hipLaunchKernelGGL(generic_main_kernel<2>, grid, block, 0, st, d);
  else if (nv <= 4) hipLaunchKernelGGL(generic_main_kernel<4>, grid, block, 0, st, d);
  else if (nv <= 8) hipLaunchKernelGGL(generic_main_kernel<8>, grid, block, 0, st, d);
  else hipLaunchKernelGGL(generic_main_kernel<16>, grid, block, 0, st, d);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (ev) (void)hipEventRecord(ev[1], st);
  if (s > 1) {
    hipLaunchKernelGGL(generic_combine_kernel, dim3((unsigned)rows), block, 0, st, d);
    if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  }
  if (ev) (void)hipEventRecord(ev[2], st);
  return GLA_OK;
}

size_t workspace_need(const gla_decode_params* p, int is_gta, int kernel, const KeyCache* kc) {
  if (kernel == GLA_IMPL_TUNED) return tuned_workspace(p, is_gta);
  if (kernel == kImplFlex) {
    FlexPlan fp;
    return flex_plan(p, is_gta, kc, &fp) ? flex_workspace(p, fp) : 0;
  }
  return generic_workspace(p);
}

int run(const gla_decode_params* p, int is_gta, hipEvent_t* ev, const KeyCache* kc = nullptr) {
  const int impl = select_kernel(p, is_gta, kc);
  if (impl < 0) return impl;
  int rc = check_pointers(p);
  if (rc != GLA_OK) return rc;
  if (is_gta == kModeGqa && p->batch > 0 && (!kc || !kc->ptr)) return GLA_ERR_INVALID_ARG;
  if (p->batch == 0) return GLA_OK;
  const size_t need = workspace_need(p, is_gta, impl, kc);
  if (need > 0 && (!p->workspace || p->workspace_bytes < need)) return GLA_ERR_WORKSPACE_TOO_SMALL;
  if (need > 0 && ((uintptr_t)p->workspace & 255u)) return GLA_ERR_INVALID_ARG;
  DevParams d;
  fill_dev(p, &d);
  if (is_gta == kModeGqa) {
    d.kstate = (const uint16_t*)kc->ptr;
    for (int i = 0; i < 3; ++i) d.k_s[i] = kc->stride[i];
  }
  hipStream_t st = (hipStream_t)p->stream;
  if (impl == GLA_IMPL_TUNED) return tuned_launch(p, is_gta, d, st, ev);
  if (impl == kImplFlex) {
    FlexPlan fp;
    if (!flex_plan(p, is_gta, kc, &fp)) return GLA_ERR_UNSUPPORTED_SHAPE;
    return launch_flex(p, fp, d, st, ev);
  }
  return launch_generic(p, d, st, ev);
}

// ---- fixed scratch buffer of the allocation-free entry point -------------------
// One array per GPU the library runs on, in that GPU's memory for the lifetime
// of the process.  In host code the array's name is only a handle: the device
// address is asked for once per device (with that device current) and every
// later use goes through the address kept here.
constexpr size_t kScratchBytes = (size_t)GLA_DECODE_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static void* scratch_addr[kMaxDevices];  // device address of `scratch` per device, null until asked for
static std::mutex scratch_mutex;

int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GLA_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_addr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return GLA_ERR_LAUNCH;
    }
    scratch_addr[dev] = ptr;
  }
  *out = scratch_addr[dev];
  return GLA_OK;
}

int run_noalloc(const gla_decode_params* p, int is_gta) {
  const int impl = select_impl(p, is_gta);
  if (impl < 0) return impl;
  const size_t need = workspace_need(p, is_gta, select_kernel(p, is_gta, nullptr), nullptr);
  if (need > kScratchBytes) return GLA_ERR_WORKSPACE_TOO_SMALL;  // beyond the fixed buffer: use gla_decode / gta_decode
  gla_decode_params q = *p;
  void* ptr = nullptr;
  if (p->batch > 0) {
    const int rc = scratch_of_current_device(&ptr);
    if (rc != GLA_OK) return rc;
  }
  q.workspace = ptr;
  q.workspace_bytes = kScratchBytes;
  // (nothing in the buffer has to start at zero: every word a call reads back
  // was written by that call's own kernels first)
  return run(&q, is_gta, nullptr);
}

// ---- projections around the attention ------------------------------------------
struct ProjPlan {
  int mt;          // 32-row blocks of query rows per workgroup (1 or 2)
  int nt;          // 32-row blocks of output features per wave (1 or 2)
  int ksplit;      // ranges the input features of a group are cut into
  int k_per_split;
  bool direct;     // no partials: the kernel writes the result itself
  size_t part_bytes;
};

int proj_plan(const gla_proj_params* p, int sum_groups, ProjPlan* plan) {
  if (!p || p->rows < 0 || p->groups < 1 || p->n < 1 || p->k < 1) return GLA_ERR_INVALID_ARG;
  if (p->c_dtype != GLA_OUT_BF16 && p->c_dtype != GLA_OUT_FP32) return GLA_ERR_INVALID_ARG;
  if ((int64_t)p->rows * p->groups * p->n > (int64_t)0x7fffffff) return GLA_ERR_INVALID_ARG;
  // what the kernel assumes: whole steps of 64 input features, whole waves of 32 output features, 16-byte loads
  if (p->k % 64 || p->n % 32) return GLA_ERR_UNSUPPORTED_SHAPE;
  if (p->a_row_stride % 8 || p->a_group_stride % 8 || p->c_row_stride % 4 || p->c_group_stride % 4)
    return GLA_ERR_UNSUPPORTED_SHAPE;
  plan->mt = p->rows <= 32 ? 1 : 2;
  const int cus = device_cu_count();
  const int64_t row_tiles = (p->rows + 32 * plan->mt - 1) / (32 * plan->mt);
  // Long sums (the output projection): 64 output features per wave, i.e. 256 per workgroup, and as many
  // ranges per group as give one workgroup per compute unit in a single round (its ring of three 40 KB
  // stages fills the LDS).  Against 32 features per wave that halves the re-reads of the query rows (every
  // workgroup fetches its range of them: rows x k x 2 bytes per 128 or 256 output features) and needs
  // fewer partial results (output projection of the benchmark shape: 240 workgroups, 93 -> 74 us).
  // Taken when such a grid covers at least three quarters of the compute units; ranges of at least 512
  // features, of ceil(steps / ranges) steps of 64 each, the last one shorter.
  int ks = 1;
  plan->nt = 1;
  plan->k_per_split = p->k;
  {
    const int64_t base = (int64_t)((p->n + 255) / 256) * row_tiles * p->groups;
    const int64_t want = std::min<int64_t>(std::max(1, p->k / 512), cus / std::max<int64_t>(1, base));
    if (want >= 1 && base * want * 4 >= (int64_t)cus * 3) {
      const int steps = p->k / 64, per = (int)((steps + want - 1) / want);
      plan->nt = 2;
      ks = (steps + per - 1) / per;  // (no empty range)
      plan->k_per_split = per * 64;
    }
  }
  if (plan->nt == 1) {
    const int64_t tiles = (int64_t)((p->n + 127) / 128) * row_tiles;
    // Ranges per group: the grid runs in rounds of as many workgroups as there are compute units.  Among
    // the cuts into ranges of at least 512 features pick the one with the least estimated time: rounds x
    // (steps per range + a fixed cost per workgroup of about four steps: start-up latency, partial store).
    double best = 1e30;
    for (int c = 1; c <= 64 && p->k / c >= 512 && (p->k / c) % 64 == 0; c *= 2) {
      const int64_t wgs = tiles * p->groups * c;
      const double t = (double)((wgs + cus - 1) / cus) * (p->k / c / 64 + 4);
      if (t < best * 0.999) { best = t; ks = c; }
    }
    plan->k_per_split = p->k / ks;
  }
  plan->ksplit = ks;
  plan->direct = ks == 1 && (!sum_groups || p->groups == 1);
  plan->part_bytes = plan->direct ? 0 : (size_t)p->groups * ks * p->rows * p->n * sizeof(float);
  return GLA_OK;
}

int run_proj(const gla_proj_params* p, int sum_groups) {
  ProjPlan plan;
  const int rc = proj_plan(p, sum_groups, &plan);
  if (rc != GLA_OK) return rc;
  if (p->rows == 0) return GLA_OK;
  if (!p->a || !p->w || !p->c) return GLA_ERR_INVALID_ARG;
  if (((uintptr_t)p->a | (uintptr_t)p->w | (uintptr_t)p->c) & 15u) return GLA_ERR_UNSUPPORTED_SHAPE;
  if (plan.part_bytes > 0 && (!p->workspace || p->workspace_bytes < plan.part_bytes)) return GLA_ERR_WORKSPACE_TOO_SMALL;
  if (plan.part_bytes > 0 && ((uintptr_t)p->workspace & 255u)) return GLA_ERR_INVALID_ARG;
  ProjParams d;
  d.a = (const uint16_t*)p->a;
  d.w = (const uint16_t*)p->w;
  d.c = p->c;
  d.part = (float*)p->workspace;
  d.a_row = p->a_row_stride;
  d.a_group = p->a_group_stride;
  d.c_row = p->c_row_stride;
  d.c_group = p->c_group_stride;
  d.M = p->rows;
  d.G = p->groups;
  d.N = p->n;
  d.K = p->k;
  d.ksplit = plan.ksplit;
  d.k_per_split = plan.k_per_split;
  d.sum_groups = sum_groups ? 1 : 0;
  d.c_fp32 = p->c_dtype == GLA_OUT_FP32;
  d.direct = plan.direct ? 1 : 0;
  hipStream_t st = (hipStream_t)p->stream;
  const int wg_n = 128 * plan.nt;
  const dim3 grid((unsigned)((p->n + wg_n - 1) / wg_n), (unsigned)((p->rows + 32 * plan.mt - 1) / (32 * plan.mt)),
                  (unsigned)(p->groups * plan.ksplit));
  if (grid.y > 65535u || grid.z > 65535u) return GLA_ERR_UNSUPPORTED_SHAPE;
  if (plan.nt == 2) {
    if (plan.mt == 1) hipLaunchKernelGGL((proj_kernel<1, 2>), grid, dim3(256), 0, st, d);
    else hipLaunchKernelGGL((proj_kernel<2, 2>), grid, dim3(256), 0, st, d);
  } else {
    if (plan.mt == 1) hipLaunchKernelGGL((proj_kernel<1, 1>), grid, dim3(256), 0, st, d);
    else hipLaunchKernelGGL((proj_kernel<2, 1>), grid, dim3(256), 0, st, d);
  }
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (!plan.direct) {
    const int64_t outs = (int64_t)p->rows * (sum_groups ? 1 : p->groups) * (p->n / 4);
    hipLaunchKernelGGL(proj_reduce_kernel, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, st, d);
    if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  }
  return GLA_OK;
}

__global__ void zero_int_kernel(int* x) { *x = 0; }

// Device contents the decode kernels trust: one thread per (sequence, table
// entry).  Counts lengths outside [0, max_pages * page_size] and held table
// entries outside [0, num_pages) into *bad (a vector-memory atomic).
__global__ void check_contents_kernel(const int32_t* seq_lens, const int32_t* page_table, int B, int max_pages,
                                      int page_size, int64_t num_pages, int* bad) {
  // (the batch is folded into grid.x: grid.y would cap it at 65535 sequences)
  const int bpr = (max_pages + (int)blockDim.x - 1) / (int)blockDim.x;  // blocks per table row
  const int b = (int)(blockIdx.x / (unsigned)bpr);
  const int j = (int)(blockIdx.x % (unsigned)bpr) * (int)blockDim.x + (int)threadIdx.x;
  if (b >= B) return;
  const int L = seq_lens[b];
  const int64_t cap = (int64_t)max_pages * page_size;
  if (L < 0 || L > cap) {
    if (j == 0) atomicAdd(bad, 1);
    return;
  }
  const int held = (L + page_size - 1) / page_size;
  if (j < held) {
    const int32_t pg = page_table[(int64_t)b * max_pages + j];
    if (pg < 0 || (int64_t)pg >= num_pages) atomicAdd(bad, 1);
  }
}

int check_contents(const gla_decode_params* p, int is_gta, int* n_bad) {
  const int impl = select_impl(p, is_gta);
  if (impl < 0) return impl;
  int rc = check_pointers(p);
  if (rc != GLA_OK) return rc;
  if (!n_bad || p->num_pages <= 0) return GLA_ERR_INVALID_ARG;
  *n_bad = 0;
  if (p->batch == 0) return GLA_OK;
  if (!p->workspace || p->workspace_bytes < 256) return GLA_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)p->stream;
  int* counter = (int*)p->workspace;
  hipLaunchKernelGGL(zero_int_kernel, dim3(1), dim3(1), 0, st, counter);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  const int threads = 256;
  const int64_t blocks = (int64_t)((p->max_pages_per_seq + threads - 1) / threads) * p->batch;
  if (blocks > 0x7fffffff) return GLA_ERR_INVALID_ARG;
  const dim3 grid((unsigned)blocks);
  hipLaunchKernelGGL(check_contents_kernel, grid, dim3(threads), 0, st, p->seq_lens, p->page_table, p->batch,
                     p->max_pages_per_seq, p->page_size, p->num_pages, counter);
  if (hipGetLastError() != hipSuccess) return GLA_ERR_LAUNCH;
  if (hipMemcpyAsync(n_bad, counter, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return GLA_ERR_LAUNCH;
  return GLA_OK;
}

}  // namespace
}  // namespace gla

extern "C" {

int gla_decode_check_contents(const gla_decode_params* p, int is_gta, int* n_bad) {
  return gla::check_contents(p, is_gta, n_bad);
}

int gla_decode(const gla_decode_params* p) { return gla::run(p, 0, nullptr); }

int gta_decode(const gla_decode_params* p) { return gla::run(p, 1, nullptr); }

int gla_decode_noalloc(const gla_decode_params* p, int is_gta) { return gla::run_noalloc(p, is_gta); }

size_t gla_decode_workspace_size(const gla_decode_params* p, int is_gta) {
  const int impl = gla::select_kernel(p, is_gta, nullptr);
  if (impl < 0) return 0;
  // A little more than nothing, so callers can always pass a real buffer.
  return std::max<size_t>(gla::workspace_need(p, is_gta, impl, nullptr), 256);
}

int gqa_decode(const gla_decode_params* p, const void* key_cache, const int64_t* key_stride) {
  if (!key_stride) return GLA_ERR_INVALID_ARG;
  const gla::KeyCache kc = {key_cache, {key_stride[0], key_stride[1], key_stride[2]}};
  return gla::run(p, gla::kModeGqa, nullptr, &kc);
}

int gla_absorb_query(const gla_proj_params* p) { return gla::run_proj(p, 0); }

int gla_output_proj(const gla_proj_params* p) { return gla::run_proj(p, 1); }

size_t gla_proj_workspace_size(const gla_proj_params* p, int sum_groups) {
  gla::ProjPlan plan;
  if (gla::proj_plan(p, sum_groups, &plan) != GLA_OK) return 0;
  return std::max<size_t>(plan.part_bytes, 256);
}

int gla_decode_select_impl(const gla_decode_params* p, int is_gta) {
  return gla::select_impl(p, is_gta);
}

int gla_decode_profile(const gla_decode_params* p, int is_gta, int iters, float* main_us,
                       float* combine_us) {
  if (!p || !main_us || !combine_us || iters < 1 || iters > 256) return GLA_ERR_INVALID_ARG;
  hipEvent_t ev[3 * 256];
  int made = 0;
  int rc = GLA_OK;
  for (; made < 3 * iters; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) { rc = GLA_ERR_LAUNCH; break; }
  for (int i = 0; rc == GLA_OK && i < iters; ++i) rc = gla::run(p, is_gta, &ev[3 * i]);
  if (hipStreamSynchronize((hipStream_t)p->stream) != hipSuccess && rc == GLA_OK) rc = GLA_ERR_LAUNCH;
  if (rc == GLA_OK && p->batch > 0) {
    double a = 0, b = 0;
    for (int i = 0; i < iters; ++i) {
      float t0 = 0, t1 = 0;
      if (hipEventElapsedTime(&t0, ev[3 * i], ev[3 * i + 1]) != hipSuccess ||
          hipEventElapsedTime(&t1, ev[3 * i + 1], ev[3 * i + 2]) != hipSuccess) {
        rc = GLA_ERR_LAUNCH;
        break;
      }
      a += t0;
      b += t1;
    }
    *main_us = (float)(a * 1000.0 / iters);
    *combine_us = (float)(b * 1000.0 / iters);
  } else {
    *main_us = *combine_us = 0.f;
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

const char* gla_status_string(int status) {
  switch (status) {
    case GLA_OK: return "ok";
    case GLA_ERR_INVALID_ARG: return "invalid argument";
    case GLA_ERR_UNSUPPORTED_SHAPE: return "no kernel for this shape with the requested implementation";
    case GLA_ERR_WORKSPACE_TOO_SMALL: return "workspace missing or too small (allocation-free entry point: the problem needs more than its fixed buffer)";
    case GLA_ERR_LAUNCH: return "HIP launch or event call failed";
    default: return "unknown status";
  }
}

int gla_decode_version(void) { return gla::kVersion; }

}  // extern "C"
