// Split-KV main kernel of the tuned decode-attention path (see the overview in
// tuned_kernels.hpp): LDS tile layout and the kernel itself.
#pragma once

#include "tuned_device.hpp"

namespace gla {

// 16-byte-chunk swizzles of the LDS tiles.  State rows are DV*2 bytes; within
// every aligned run of 16 chunks the chunk index is XORed with a 4-bit key of
// the token so that (a) 16 consecutive tokens reading the same logical chunk
// (score MFMA operand reads) and (b) 4 consecutive tokens reading the same 64
// bytes (transposing value reads) both spread over all LDS banks.  The key is
// a bit permutation, hence XOR-linear in the token index.
__host__ __device__ constexpr int swz16(int t) { return ((t & 3) << 2) | ((t >> 2) & 3); }
// RoPE rows are 128 bytes (8 chunks): two tokens share a 256-byte bank row.
__host__ __device__ constexpr int swz8(int t) { return (t >> 1) & 7; }

template <int DV, int DN, int DR, int NG, int WPG, int KS, int TOK, int STAGES>
struct TunedTraits {
  static constexpr int NWAVES = NG * WPG * KS;
  static constexpr int kRows = 32 * NG * WPG;  // query rows of a unit, all groups together
  static constexpr int kRowBytes = DV * 2;
  static constexpr int kStateBytes = TOK * kRowBytes;
  static constexpr int kRopeBytes = TOK * DR * 2;
  // LDS layout: for each of the NG groups its STAGES state tiles, then the
  // STAGES RoPE tiles, so that stepping to the next stage is one add for every
  // operand address and each wave's group is a constant folded into its bases.
  static constexpr int kGroupBytes = STAGES * kStateBytes;
  static constexpr int kRopeBase = NG * kGroupBytes;
  static constexpr int kTileBytes = STAGES * (NG * kStateBytes + kRopeBytes);
  // KS > 1: one 4 KiB mailbox per wave for the partial scores the KS waves of a row slab exchange
  static constexpr int kXchgBase = kTileBytes;
  static constexpr int kSmemBytes = kTileBytes + (KS > 1 ? NWAVES * 4096 : 0);
  static constexpr int kStateLoads = kStateBytes / 1024;  // wave-wide 16 B/lane loads per group tile
  static constexpr int kRopeLoads = kRopeBytes / 1024;
  static constexpr int kLoadsPerWave = kStateLoads / (WPG * KS) + kRopeLoads / NWAVES;
  static constexpr int kThreads = 64 * NWAVES;
  static constexpr size_t kSlotFloats = (size_t)kRows * DV + 32 * NWAVES;  // partial out + one lse per wave row
  static_assert(TOK == 32, "tiles of 32 tokens: two, one or half of them per page");
  static_assert(STAGES >= 3 && STAGES % 2 == 0, "PV stage + score stage + loading stages; even for the score register swap");
  static_assert(KS == 1 || (KS == 2 && DN == DV), "row slabs are split over 1 or 2 waves; the split is by state dims");
  static_assert(kStateLoads % (WPG * KS) == 0 && kRopeLoads % NWAVES == 0, "tile loads must split evenly over waves");
  static_assert(((kStateLoads / (WPG * KS)) & (kStateLoads / (WPG * KS) - 1)) == 0, "per-wave state blocks: power of two (swizzle keys combine by XOR)");
  static_assert(KS == 1 || ((DN / KS * 2) % 256 == 0 && (DV / KS * 2) % 256 == 0), "a wave's share of a state row starts on a swizzle-run boundary");
  static_assert(kLoadsPerWave * (STAGES - 2) <= 63, "vmcnt range");
  static_assert(DR == 64, "RoPE key tile layout assumes 64 dims");
  static_assert(kRowBytes >= 256 && (kRowBytes & (kRowBytes - 1)) == 0 && kRowBytes <= 1024, "state row bytes");
  static_assert(kSmemBytes <= 160 * 1024, "LDS capacity");
};

// PM, the page mode, selects the address code of the tile loads:
//   0: pages of 64 tokens (a tile is half a page: one base address per tile),
//   1: pages of 32 or 16 tokens (one base address per run of up to 16 rows),
//   2: pages of 8, 4, 2 or 1 tokens (one address per row and lane, from page ids
//      that each wave keeps in windows of the page table in LDS),
//   3: the same with the windows in registers, one entry per lane and register,
//      for the shape whose tiles and mailboxes leave no LDS for them (a few
//      per cent slower where both fit).
constexpr int kPageWindow = 256;  // page-table entries per window (PM == 2)

// Tile tokens and pipeline depth of the instantiation for a shape: the deepest
// even ring (at most 8 stages) that fits the LDS and whose loads in flight per
// wave stay countable by the 6-bit vmcnt.
constexpr int kTok = 32;
constexpr int tuned_stages(int dv, int ng, int wpg, int ks, bool lane = false) {
  const int stage_bytes = ng * kTok * dv * 2 + kTok * 128;
  // besides the tiles: score mailboxes (ks > 1), page-id windows (pages of 8 tokens or fewer)
  const int mailboxes = (ks > 1 ? ng * wpg * ks * 4096 : 0) + (lane ? ng * wpg * ks * 2 * kPageWindow * 4 : 0);
  const int loads_per_wave = (kTok * dv * 2 / 1024) / (wpg * ks) + (kTok * 128 / 1024) / (ng * wpg * ks);
  int st = 8;
  while (st > 4 && (st * stage_bytes + mailboxes > 160 * 1024 || loads_per_wave * (st - 2) > 63)) st -= 2;
  return st;
}

// Do the LDS page-id windows of page mode 2 fit beside the tile ring and the mailboxes?  (Else: page mode 3.)
constexpr bool tuned_windows_fit(int dv, int ng, int wpg, int ks) {
  return tuned_stages(dv, ng, wpg, ks, true) * (ng * kTok * dv * 2 + kTok * 128) + (ks > 1 ? ng * wpg * ks * 4096 : 0) +
             ng * wpg * ks * 2 * kPageWindow * 4 <= 160 * 1024;
}

template <int DV, int DN, int DR, int NG, int WPG, int KS, int TOK, int STAGES, int PM, bool STREAM>
__global__ __launch_bounds__(64 * NG * WPG * KS) void tuned_main_kernel(DevParams p) {
  using TT = TunedTraits<DV, DN, DR, NG, WPG, KS, TOK, STAGES>;
  constexpr int NWAVES = NG * WPG * KS;
  constexpr bool kLane = PM >= 2;
  constexpr bool kRegWin = PM == 3;
  constexpr int kWinBase = TT::kSmemBytes;                                     // two windows per wave
  constexpr int kSmemAll = TT::kSmemBytes + (PM == 2 ? NWAVES * 2 * kPageWindow * 4 : 0);
  static_assert(kSmemAll <= 160 * 1024, "LDS capacity");
  constexpr int ROWB = TT::kRowBytes;
  constexpr int STB = TT::kStateBytes;   // state tile bytes
  constexpr int RTB = TT::kRopeBytes;    // RoPE tile bytes
  constexpr int NTB = TOK / 32;          // 32-token blocks per tile
  // With KS = 2 the two waves of a row slab each take half of the state dims
  // (for the scores and for the output) and half of the RoPE dims, and add up
  // their partial scores through LDS; everything below is per wave.
  constexpr int DVW = DV / KS, DNW = DN / KS, DRW = DR / KS;
  constexpr int NKN = DNW / 16;          // contraction steps over the state dims
  constexpr int NKR = DRW / 16;          // ... over the RoPE dims
  constexpr int NDB = DVW / 32;          // 32-dim output blocks
  constexpr int NE = 16 * NTB;           // scores per lane per tile
  constexpr int NS = (NKN + NKR) * NTB;  // score MFMAs per tile
  constexpr int NP = (TOK / 16) * NDB;   // value MFMAs per tile
  constexpr int NB = NP + TOK / 16;      // ... plus the row-sum MFMAs
  constexpr int LPW = TT::kLoadsPerWave;
  constexpr int SLW = TT::kStateLoads / (WPG * KS);  // 1 KiB state blocks per wave and tile
  constexpr int RLW = TT::kRopeLoads / NWAVES;   // 1 KiB RoPE blocks per wave and tile
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kSmemAll];
  const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int gl = wave / (WPG * KS);    // this wave's group within the unit's group block
  const int wpos = wave % (WPG * KS);  // position among the waves of that group
  const int wg = wpos / KS;            // this wave's 32-row slab within the group's row block
  const int kx = wpos % KS;            // which share of the state / RoPE dims this wave works on
  const int col = lane & 31;  // query row inside the wave's 32-row slab == MFMA column
  const int hi = lane >> 5;   // which half of the contraction slots this lane feeds

  const int rows_group = p.g_q * p.T;
  const int MB = p.mb;    // row blocks per group
  const int UPB = p.upb;  // units (group blocks) per sequence

  // A chunk of the list is worked on by MB workgroups, one per row block of its
  // groups (MB > 1 when a group has more query rows than a workgroup holds).
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): the
  // MB workgroups of a chunk are placed on ONE XCD, where they run side by side
  // so that the tiles the first one fetches are L2 hits for the others, and
  // every XCD gets a contiguous run of chunks (same page-table rows, same
  // queries).  Grids that do not divide evenly fall back to a plain order.
  const int n_chunks = p.num_chunks;  // the host launches n_chunks * MB workgroups
  int chunk_id, mb_wg;
  if (p.xcd_map) {
    const int xcd = (int)blockIdx.x & 7, n = (int)blockIdx.x >> 3;
    const int q = (int)fast_div((unsigned)n, p.fd_mb);
    mb_wg = n - q * MB;
    chunk_id = xcd * (n_chunks >> 3) + q;
  } else {
    chunk_id = (int)fast_div(blockIdx.x, p.fd_mb);
    mb_wg = (int)blockIdx.x - chunk_id * MB;
  }

  // ---- a guess, made before anything is known about the lengths: if every
  // sequence filled its page-table row, this chunk would start at page pg of
  // sequence b_g.  That stretch of the page table is requested right away, next
  // to the lengths, and used if the plan below lands inside it (always, for a
  // batch of equal full-length sequences): one dependent memory round trip less
  // before the first tile can be requested.
  int pt_b = -1, pt_base = 0;
  int pt_vec = 0;
  int L_first;  // lengths of the first 64 sequences (0 beyond the batch), reused by the plan
  {
    // (all products below stay under 2^30: the host refuses larger plans)
    const unsigned total_g = (unsigned)p.B * (unsigned)UPB * (unsigned)p.tiles_full;
    const unsigned c0_g = min((unsigned)chunk_id * (unsigned)p.chunk_guess, total_g - 1);  // (chunks past the end: any valid row)
    const int b_g = (int)fast_div(c0_g, p.fd_units_full);
    const unsigned j_g = c0_g - fast_div(c0_g, p.fd_tiles_full) * (unsigned)p.tiles_full;
    const int pg = (int)((j_g * TOK) >> (PM == 0 ? 6 : p.lg_page));
    const int32_t* ptr_pt = p.page_table + (int64_t)b_g * p.max_pages + min(pg + lane, p.max_pages - 1);
    const int32_t* ptr_len = p.seq_lens + (lane < p.B ? lane : 0);
    // both requests in flight together, both complete when the statement ends
    asm volatile("global_load_dword %0, %2, off\n\tglobal_load_dword %1, %3, off\n\ts_waitcnt vmcnt(0)"
                 : "=&v"(pt_vec), "=&v"(L_first)
                 : "v"(ptr_pt), "v"(ptr_len)
                 : "memory");
    if (lane >= p.B) L_first = 0;
    pt_b = b_g;
    pt_base = pg;
  }

  // ---- plan: this workgroup's chunk [c0, c1) of the flat tile list
  const int incl0 = wave_incl_scan(tiles_of<TOK>(L_first) * UPB);
  const int n_total = total_tiles<TOK>(p, UPB, lane, incl0);
  if (n_total <= 0) return;
  // Chunk i covers tiles [i * chunk, (i + 1) * chunk): a fixed length if the
  // caller chose a split count, else an equal share of the list.
  const int chunk = p.chunk_tiles > 0 ? p.chunk_tiles : (int)fast_div((unsigned)(n_total + n_chunks - 1), p.fd_chunks);
  auto chunk_start = [&](int i) -> int { return (int)min((int64_t)n_total, (int64_t)i * chunk); };
  const int c0 = chunk_start(chunk_id);
  const int c1 = chunk_start(chunk_id + 1);
  if (c0 >= c1) return;  // only chunks past the end of the list are empty: no unit spans them
  const int n_tiles = c1 - c0;

  TileCursor cur = locate_tile<TOK>(p, UPB, c0, lane, L_first, incl0);  // compute position
  TileCursor pre = cur;                                  // prefetch position

  // ---- tile loads, global -> LDS, 16 B per lane, 1 KiB per wave instruction.
  // The LDS side is linear in the lane index, so each lane fetches the global
  // chunk whose swizzled home is its LDS slot.  Wave w moves the contiguous
  // 1 KiB blocks [wg*SLW, (wg+1)*SLW) of its own group's state tile and blocks
  // [w*RLW, (w+1)*RLW) of the RoPE tile; block i of a wave sits at  i*1024 + (lane_part ^ key(i) << 4)
  // past the wave's start, i.e. one XOR per load, and four loads share one
  // pair of base addresses through the instruction's immediate offset (which
  // the hardware adds to the global and to the LDS address alike).  Page ids
  // are fetched 64 at a time, one per lane, and broadcast from the owning lane.
  constexpr int RPL = 1024 / ROWB;  // state rows per wave load
  constexpr int CPR = ROWB / 16;    // 16 B chunks per state row
  const int s_rl = lane / CPR, s_pc = lane % CPR;
  const unsigned s_lane_w =
      (unsigned)(s_rl * ROWB + ((s_pc & ~15) << 4) + (((s_pc & 15) ^ swz16(s_rl) ^ swz16(wpos * SLW * RPL)) << 4));
  const int r_rl = lane >> 3, r_pc = lane & 7;
  // RoPE keys of fewer than 64 dims (32 or 48): the LDS tile keeps its 128-byte
  // rows and all four contraction steps; the query's RoPE fragments beyond the
  // real dims are zero and the lanes whose LDS slot would hold a chunk the cache
  // rows do not have fetch one of the row's real chunks a second time (finite
  // data of a valid token times a zero query dim).  rrb: bytes of a RoPE row in
  // the cache, cpg: its 16-byte chunks; r_voff[x]: this lane's byte offset inside
  // a block of 8 cache rows for the two chunk keys a wave's loads alternate between.
  const unsigned rrb = (unsigned)p.d_r * 2u, cpg = (unsigned)p.d_r >> 3;
  unsigned r_voff[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const unsigned ch = (unsigned)(r_pc ^ (r_rl >> 1) ^ (((wave * RLW) & 1) << 2)) ^ ((unsigned)x << 2);
    r_voff[x] = (unsigned)r_rl * rrb + ((ch >= cpg ? ch - cpg : ch) << 4);  // (cpg >= 4)
  }
  const uint32_t st_page_bytes = (uint32_t)p.st_s[0] * 2u, st_group_bytes = (uint32_t)p.st_s[1] * 2u;
  const uint32_t rp_page_bytes = (uint32_t)p.rp_s[0] * 2u;
  const unsigned char* const state_w = (const unsigned char*)p.state + gl * (uint64_t)st_group_bytes;
  const unsigned char* const rope_w = (const unsigned char*)p.rope;
  // Page sizes 64, 32 and 16 tokens (PM 0 and 1): a tile of 32 tokens is half a page, a page
  // or two pages.  The loads of a wave come in groups of up to four 1 KiB blocks
  // (at most 16 token rows) and single 1 KiB RoPE blocks (8 token rows); such a
  // run never straddles a page, so each has one base address, computed by the
  // wave that issues it from the page id of its own rows.
  const int lgP = PM == 0 ? 6 : p.lg_page;
  constexpr int NSGW = (SLW + 3) / 4;                 // load groups of the state tile per wave
  constexpr int GROWS = (SLW < 4 ? SLW : 4) * RPL;    // token rows per load group
  static_assert(GROWS <= 16 && (16 % GROWS) == 0, "a load group stays inside a 16-token page");
  unsigned char* const lds_state_w = smem + gl * TT::kGroupBytes + wpos * (SLW * 1024);
  unsigned char* const lds_rope_w = smem + TT::kRopeBase + wave * (RLW * 1024);

  uint64_t pre_goff = (uint64_t)pre.ub * NG * st_group_bytes;  // byte offset of the cursor's group block in a page
  const unsigned char* pre_sp = nullptr;  // state / RoPE page of the prefetch cursor
  const unsigned char* pre_rp = nullptr;
  bool pre_page_valid = false;
  // addresses of the tile being issued (this wave's share)
  const unsigned char* dma_s[NSGW] = {};
  const unsigned char* dma_r[RLW] = {};
  unsigned char* dma_ls = nullptr;
  unsigned char* dma_lr = nullptr;
  int issued = 0;  // tiles whose loads have been issued
  // PM == 2, pages of 8 tokens or fewer: every token row of a load may lie in
  // its own page, so each lane forms the address of the row it fetches, from
  // the page id of that row.  The ids come from LDS: every wave keeps two
  // windows of kPageWindow consecutive page-table entries of the sequence it is
  // fetching, the one in use and the one after it, requested (direct to LDS)
  // when the first is entered, so a window has long arrived when the prefetch
  // cursor reaches it.  Only the first window of a sequence, and windows
  // entered within a few tiles of their request, are waited for.
  //   With the windows in registers (PM == 3) a window is kWinRegs registers,
  // lane l of register r holding entry 64 r + l, and spans at least STAGES
  // tiles at one token per page.  A tile's pages lie in one aligned block of 32
  // entries, hence in one register: that register is chosen when the tiles enter
  // a new block of 64 entries, and every load takes its row's id from it with a
  // cross-lane read.  (Named scalars, read through pinned copies: an array, or a
  // choice between the variables themselves, would be placed in scratch memory.
  // The loads into them are predicated inside one assembly statement with the
  // registers as read-write operands, and the registers have no other writer: a
  // register whose load is in flight must never be copied.)
  constexpr int kWinRegs = STAGES <= 4 ? 2 : 4;
  constexpr int kWinEntries = kRegWin ? 64 * kWinRegs : kPageWindow;
  unsigned char* const win_w = smem + kWinBase + wave * (2 * kPageWindow * 4);
  int win_a0 = 0, win_a1 = 0, win_a2 = 0, win_a3 = 0, win_b0 = 0, win_b1 = 0, win_b2 = 0, win_b3 = 0;
  int ids = 0, ids_key = -1;  // the register's worth of entries the tiles being prepared lie in: [64 * ids_key, +64)
  int win_b = -1, win_id0 = -1, win_id1 = -1, win_at0 = 0, win_at1 = 0, win_sel = 0;
  int pg_s[SLW] = {}, pg_r[RLW] = {};  // page id of this lane's row, per load of the prepared tile
  uint64_t dma_goff = 0;               // group-block offset the prepared tile's addresses use
  unsigned dma_pmask = 0;
  auto win_fetch = [&](int slot, int b_seq, int id, int last_page) {
    // entries [id * kPageWindow, +kPageWindow) of row b_seq, those past the last held page replaced by it
    const int32_t* row = p.page_table + (int64_t)b_seq * p.max_pages;
#pragma unroll
    for (int i = 0; i < kPageWindow / 64; ++i) {
      const int e = min(id * kPageWindow + i * 64 + lane, last_page);
      __builtin_amdgcn_global_load_lds((global_cvoid_t*)(row + e), (lds_void_t*)(win_w + slot * (kPageWindow * 4) + i * 256), 4, 0, 0);
    }
  };

  // Prepare the loads of the next tile into `stage`.  Once every tile of the
  // chunk has been issued the previous tile's addresses are kept: the loads
  // then re-read lines that are still in L2 into a stage nobody reads, which
  // keeps the steady-state loop free of branches around the load instructions.
  // The preparation is scalar work (a few dozen instructions).  It is cut in
  // three pieces so that the tile loop can place them between value MFMAs
  // instead of running them in one stretch with the matrix pipe idle.
  bool prep_active = false, prep_need_page = false;
  unsigned prep_page_idx = 0, prep_tip = 0;
  auto dma_prepare_0 = [&](int stage) {  // where to, and are page ids needed
    dma_ls = lds_state_w + stage * STB;
    dma_lr = lds_rope_w + stage * RTB;
    prep_active = issued < n_tiles;
    const unsigned tok0 = (unsigned)pre.j * TOK;
    prep_page_idx = tok0 >> lgP;                    // first page of the tile
    prep_tip = (tok0 & ((1u << lgP) - 1)) / TOK;  // tile within the page (pages of 64)
    prep_need_page = prep_active && (lgP < 6 || prep_tip == 0 || !pre_page_valid);
    const int last_idx = (int)((tok0 + TOK - 1) >> lgP);
    if constexpr (kRegWin) {
      // fetch0 / fetch1: request window id0 / id1 into the first / second set of registers
      int fetch0 = 0, fetch1 = 0, id0 = 0, id1 = 0, last_page = 0;
      bool wait_before = false, wait_after = false;
      if (prep_active) {
        last_page = (pre.L - 1) >> lgP;
        const int want = (int)prep_page_idx / kWinEntries, nxt = want + 1;
        const bool has_nxt = nxt * kWinEntries <= last_page;
        if (pre.b != win_b || (want != win_id0 && want != win_id1)) {
          // first window of a sequence: it and the one after it, waited for
          win_b = pre.b;
          win_sel = 0;
          ids_key = -1;
          win_id0 = want;
          win_id1 = has_nxt ? nxt : -1;
          win_at0 = win_at1 = issued - STAGES;
          fetch0 = 1, id0 = want;
          fetch1 = has_nxt ? 1 : 0, id1 = nxt;
          wait_after = true;
        } else {
          win_sel = want == win_id1 ? 1 : 0;
          // requested too recently for the rolling waits of the tile loop to have covered it
          wait_before = issued - (win_sel ? win_at1 : win_at0) < STAGES;
          if (has_nxt && (win_sel ? win_id0 : win_id1) != nxt) {
            if (win_sel) { win_id0 = nxt; win_at0 = issued; fetch0 = 1; id0 = nxt; }
            else { win_id1 = nxt; win_at1 = issued; fetch1 = 1; id1 = nxt; }
          }
        }
      }
      if (wait_before) wait_vmcnt<0>();
      if (uniform(fetch0 | fetch1)) {  // (once per window: every fourth tile at most)
        // entries [id * kWinEntries, +kWinEntries) of the sequence's row, those past its last page replaced by that page
        const int32_t* const row = p.page_table + (int64_t)pre.b * p.max_pages;
        const int ea = id0 * kWinEntries + lane, eb = id1 * kWinEntries + lane;
        load_window<kWinRegs>(uniform(fetch0), row, min(ea, last_page) * 4, min(ea + 64, last_page) * 4,
                              min(ea + 128, last_page) * 4, min(ea + 192, last_page) * 4, win_a0, win_a1, win_a2, win_a3);
        load_window<kWinRegs>(uniform(fetch1), row, min(eb, last_page) * 4, min(eb + 64, last_page) * 4,
                              min(eb + 128, last_page) * 4, min(eb + 192, last_page) * 4, win_b0, win_b1, win_b2, win_b3);
      }
      if (wait_after) wait_vmcnt<0>();
    } else if constexpr (kLane) {
      if (prep_active) {
        const int last_page = (pre.L - 1) >> lgP;
        const int want = (int)prep_page_idx / kPageWindow;
        if (pre.b != win_b || (want != win_id0 && want != win_id1)) {
          win_b = pre.b;
          win_id0 = want;
          win_id1 = -1;
          win_sel = 0;
          win_fetch(0, pre.b, want, last_page);
          wait_vmcnt<0>();
          win_at0 = issued - STAGES;
        } else {
          win_sel = want == win_id1 ? 1 : 0;
          // requested too recently for the rolling waits of the tile loop to have covered it
          if (issued - (win_sel ? win_at1 : win_at0) < STAGES) wait_vmcnt<0>();
        }
        const int nxt = want + 1;
        if (nxt * kPageWindow <= last_page && (win_sel ? win_id0 : win_id1) != nxt) {
          if (win_sel) { win_id0 = nxt; win_at0 = issued; } else { win_id1 = nxt; win_at1 = issued; }
          win_fetch(win_sel ^ 1, pre.b, nxt, last_page);
        }
      }
    } else if (prep_need_page && (pre.b != pt_b || (int)prep_page_idx < pt_base || last_idx >= pt_base + 64)) {
      pt_b = pre.b;
      pt_base = (int)prep_page_idx;
      const int idx = min((int)prep_page_idx + lane, p.max_pages - 1);
      pt_vec = load_i32_sync(p.page_table + (int64_t)pre.b * p.max_pages + idx);
    }
  };
  auto dma_prepare_1 = [&]() {  // pages of 64: page id -> page base addresses (kept for the page's second tile)
    if (prep_need_page && lgP == 6) {
      const uint32_t page = (uint32_t)__builtin_amdgcn_readlane(pt_vec, (int)prep_page_idx - pt_base);
      pre_sp = state_w + ((uint64_t)page * st_page_bytes + pre_goff);
      pre_rp = rope_w + (uint64_t)page * rp_page_bytes;
      pre_page_valid = true;
    }
  };
  auto dma_prepare_2 = [&]() {  // base address of every load group; advance the prefetch cursor
    if (!prep_active) return;
    if constexpr (kRegWin) {
      const unsigned tok0 = (unsigned)pre.j * TOK;
      const int last_page = (pre.L - 1) >> lgP;
      // (rows past the end of the sequence take its last page: at or after the tile's first page, same register)
      if ((int)(prep_page_idx >> 6) != ids_key) {  // (every second tile at most)
        ids_key = (int)(prep_page_idx >> 6);
        const int reg = (int)((prep_page_idx & (kWinEntries - 1)) >> 6);
        // (copies through pins: the reads stay behind the waits of the first piece; the copy of a register
        // whose load is still in flight is not the one chosen)
        int a0 = win_a0, a1 = win_a1, b0 = win_b0, b1 = win_b1;
        asm volatile("" : "+v"(a0), "+v"(a1), "+v"(b0), "+v"(b1));
        int ia = reg == 1 ? a1 : a0, ib = reg == 1 ? b1 : b0;
        if constexpr (kWinRegs > 2) {
          int a2 = win_a2, a3 = win_a3, b2 = win_b2, b3 = win_b3;
          asm volatile("" : "+v"(a2), "+v"(a3), "+v"(b2), "+v"(b3));
          ia = reg == 2 ? a2 : (reg == 3 ? a3 : ia);
          ib = reg == 2 ? b2 : (reg == 3 ? b3 : ib);
        }
        ids = win_sel ? ib : ia;
      }
#pragma unroll
      for (int i = 0; i < SLW; ++i) {
        const unsigned rho = (unsigned)((wpos * SLW + i) * RPL + s_rl);
        const int e = min((int)((tok0 + rho) >> lgP), last_page);
        pg_s[i] = __builtin_amdgcn_ds_bpermute((e & 63) << 2, ids);
      }
#pragma unroll
      for (int ir = 0; ir < RLW; ++ir) {
        const unsigned rho = (unsigned)((wave * RLW + ir) * 8 + r_rl);
        const int e = min((int)((tok0 + rho) >> lgP), last_page);
        pg_r[ir] = __builtin_amdgcn_ds_bpermute((e & 63) << 2, ids);
      }
      dma_goff = pre_goff;
      dma_pmask = (1u << lgP) - 1;
    } else if constexpr (kLane) {
      const unsigned tok0 = (unsigned)pre.j * TOK;
      const int last_page = (pre.L - 1) >> lgP;
      const unsigned char* const win = win_w + win_sel * (kPageWindow * 4);
#pragma unroll
      for (int i = 0; i < SLW; ++i) {
        const unsigned rho = (unsigned)((wpos * SLW + i) * RPL + s_rl);
        const int e = min((int)((tok0 + rho) >> lgP), last_page);
        pg_s[i] = *reinterpret_cast<const int*>(win + (e & (kPageWindow - 1)) * 4);
      }
#pragma unroll
      for (int ir = 0; ir < RLW; ++ir) {
        const unsigned rho = (unsigned)((wave * RLW + ir) * 8 + r_rl);
        const int e = min((int)((tok0 + rho) >> lgP), last_page);
        pg_r[ir] = *reinterpret_cast<const int*>(win + (e & (kPageWindow - 1)) * 4);
      }
      dma_goff = pre_goff;
      dma_pmask = (1u << lgP) - 1;
    } else if (lgP == 6) {
#pragma unroll
      for (int gi = 0; gi < NSGW; ++gi) dma_s[gi] = pre_sp + prep_tip * STB + (wpos * SLW + 4 * gi) * 1024;
#pragma unroll
      for (int ir = 0; ir < RLW; ++ir) dma_r[ir] = pre_rp + (prep_tip * TOK + (wave * RLW + ir) * 8) * rrb;
    } else {
      // Smaller pages: one page lookup per load group.  Rows past the end of the
      // sequence may lie in a page the table does not hold: they are fetched from
      // the sequence's last page instead (any finite-or-not data will do, those
      // rows are masked and zeroed), never through an unused table entry.
      const unsigned tok0 = (unsigned)pre.j * TOK, pmask = (1u << lgP) - 1;
      const int last_page = (pre.L - 1) >> lgP;
#pragma unroll
      for (int gi = 0; gi < NSGW; ++gi) {
        const unsigned tok = tok0 + (unsigned)(wpos * SLW + 4 * gi) * RPL;
        const int pi = min((int)(tok >> lgP), last_page);
        const uint32_t page = (uint32_t)__builtin_amdgcn_readlane(pt_vec, pi - pt_base);
        dma_s[gi] = state_w + ((uint64_t)page * st_page_bytes + pre_goff + (uint64_t)(tok & pmask) * ROWB);
      }
#pragma unroll
      for (int ir = 0; ir < RLW; ++ir) {
        const unsigned tok = tok0 + (unsigned)(wave * RLW + ir) * 8;
        const int pi = min((int)(tok >> lgP), last_page);
        const uint32_t page = (uint32_t)__builtin_amdgcn_readlane(pt_vec, pi - pt_base);
        dma_r[ir] = rope_w + ((uint64_t)page * rp_page_bytes + (uint64_t)(tok & pmask) * rrb);
      }
    }
    ++issued;
    if (++pre.j == pre.tiles_b) {
      pre.j = 0;
      pre_page_valid = false;
      if (++pre.ub == UPB) {
        pre.ub = 0;
        do {
          ++pre.b;
          pre.L = pre.b < p.B ? uniform(load_i32_sync(p.seq_lens + pre.b)) : 0;
          pre.tiles_b = tiles_of<TOK>(pre.L);
        } while (pre.b < p.B && pre.tiles_b == 0);
      }
      pre_goff = (uint64_t)pre.ub * NG * st_group_bytes;
    }
  };
  auto dma_prepare = [&](int stage) {
    dma_prepare_0(stage);
    dma_prepare_1();
    dma_prepare_2();
  };
  // One direct-to-LDS load of 16 bytes per lane.  STREAM: with the streaming hint.  The host picks that
  // variant for a batch whose cache can be larger than the chip's last-level cache: its lines, read once
  // per call, then do not push the page table, the queries and the partial results out of L2 and the
  // last-level cache (measured on the benchmark shapes: 5-6 % per call); a smaller cache is left
  // cacheable, since the next decode step reads it again.  (A compile-time choice: a branch on every
  // load cost the issue-bound variants 1-3 %.)
  // (the RoPE-key tile, a ninth of the bytes and the part that group blocks of a sequence share, stays cacheable)
  auto rope_dma = [&](auto immc, const unsigned char* src, unsigned char* dst) {
    constexpr int imm = decltype(immc)::value;
    __builtin_amdgcn_global_load_lds((global_cvoid_t*)src, (lds_void_t*)dst, 16, imm, 0);
  };
  auto tile_dma = [&](auto immc, const unsigned char* src, unsigned char* dst) {
    constexpr int imm = decltype(immc)::value;
    if constexpr (STREAM)
      __builtin_amdgcn_global_load_lds((global_cvoid_t*)src, (lds_void_t*)dst, 16, imm, 2);
    else
      __builtin_amdgcn_global_load_lds((global_cvoid_t*)src, (lds_void_t*)dst, 16, imm, 0);
  };
  // i-th of this wave's LPW loads of the prepared tile
  auto dma_load = [&](auto ic) {
    constexpr int i = decltype(ic)::value;
    if constexpr (kLane) {
      // address of this lane's row: page base + row within the page + the chunk
      // of the row whose swizzled home is this lane's LDS slot
      if constexpr (i < SLW) {
        const unsigned voff = s_lane_w ^ ((unsigned)swz16(i * RPL) << 4);
        const unsigned rho = (unsigned)((wpos * SLW + i) * RPL + s_rl);
        const unsigned off = (rho & dma_pmask) * ROWB + (voff & (ROWB - 1));
        const unsigned char* src = state_w + ((uint64_t)(uint32_t)pg_s[i] * st_page_bytes + dma_goff + off);
        tile_dma(std::integral_constant<int, 0>{}, src, dma_ls + i * 1024);
      } else {
        constexpr int ir = i - SLW;
        const unsigned rho = (unsigned)((wave * RLW + ir) * 8 + r_rl);
        const unsigned off = (rho & dma_pmask) * rrb + (r_voff[ir & 1] - (unsigned)r_rl * rrb);
        const unsigned char* src = rope_w + ((uint64_t)(uint32_t)pg_r[ir] * rp_page_bytes + off);
        rope_dma(std::integral_constant<int, 0>{}, src, dma_lr + ir * 1024);
      }
    } else if constexpr (i < SLW) {
      const unsigned voff = s_lane_w ^ ((unsigned)swz16(i * RPL) << 4);
      tile_dma(std::integral_constant<int, (i % 4) * 1024>{}, dma_s[i / 4] + voff, dma_ls + (i / 4) * 4096);
    } else {
      constexpr int ir = i - SLW;
      rope_dma(std::integral_constant<int, 0>{}, dma_r[ir] + r_voff[ir & 1], dma_lr + ir * 1024);
    }
  };

  // ---- query fragments of the unit at `cur`: this wave's 32 rows, B operand of
  //      the score MFMAs, lane holds 8 dims of row `col` per contraction step.
  //      Requested at the start of every segment, after the first tiles.
  u32x4_t qn[NKN];  // raw bf16 bits (accumulation VGPRs)
  u32x4_t qr[NKR];
  bool row_valid = false;
  int row_b = 0, row_t = 0, row_h = 0;
  auto q_issue = [&]() {
    const int gb = cur.ub;
    const int mb = mb_wg;
    const int g = gb * NG + gl;
    const int R = (mb * WPG + wg) * 32 + col;
    row_valid = R < rows_group;
    const int Rc = row_valid ? R : rows_group - 1;
    row_t = (int)fast_div((unsigned)Rc, p.fd_gq);
    row_h = g * p.g_q + (Rc - row_t * p.g_q);
    row_b = cur.b;
    const uint16_t* qn_ptr = p.q_nope + row_b * p.qn_s[0] + row_t * p.qn_s[1] + row_h * p.qn_s[2] + kx * DNW + 8 * hi;
    const uint16_t* qr_ptr = p.q_rope + row_b * p.qr_s[0] + row_t * p.qr_s[1] + row_h * p.qr_s[2] + kx * DRW + 8 * hi;
    // padding rows re-read the last valid row: their columns are computed and never stored
#pragma unroll
    for (int ks = 0; ks < NKN; ++ks) load_b128_async(qn[ks], qn_ptr + 16 * ks);
#pragma unroll
    for (int ks = 0; ks < NKR; ++ks)  // (dims the RoPE key does not have: the row's first dims again, zeroed after the wait)
      load_b128_async(qr[ks], kx * DRW + 16 * ks < p.d_r ? qr_ptr + 16 * ks : qr_ptr - kx * DRW);
  };

  // ---- prologue: fill STAGES-1 stages
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s) {
    if (issued < n_tiles) {
      dma_prepare(s);
      static_for<0, LPW>(dma_load);
    }
  }

  // ---- lane-constant LDS read addresses (stage 0; other stages are immediates)
  // score operand (K rows, 16 B): token = 32*tb + col, logical chunk = 2*ks + hi
  const int sw_col = swz16(col);
  unsigned k_off[8], ka[8];  // index: ks & 7; ka: working copy pointing at a stage
#pragma unroll
  for (int e = 0; e < 8; ++e)
    k_off[e] = lds_base + (unsigned)(gl * TT::kGroupBytes + col * ROWB + kx * (DNW * 2) + ((((2 * e) | hi) ^ sw_col) << 4));
  unsigned r_off[NKR], ra[NKR];
#pragma unroll
  for (int e = 0; e < NKR; ++e)
    r_off[e] = lds_base + (unsigned)(TT::kRopeBase + col * 128 + (((kx * (DRW / 8) + ((2 * e) | hi)) ^ swz8(col)) << 4));
  // value operand (transposing 8 B reads): 16-lane block bk = lane / 16 covers
  // 4 tokens x 16 dims; lane 4r+q of the block addresses token r, dims 4q..4q+3.
  const int i16 = lane & 15;
  const int tr_r = i16 >> 2, tr_q = i16 & 3;
  const int dh = (lane >> 4) & 1;
  unsigned v_off[4][2], va[4][2];  // [db & 3][a]
#pragma unroll
  for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const int key = (tr_r << 2) | (2 * a + hi);           // swz16 of token 8a + 4hi + r
      const int lc = (4 * d4 + 2 * dh + (tr_q >> 1)) ^ key;  // chunk within the 16-chunk run
      v_off[d4][a] = lds_base + (unsigned)(gl * TT::kGroupBytes + (4 * hi + tr_r) * ROWB + kx * (DVW * 2) + (lc << 4) + (tr_q & 1) * 8);
    }

  float sc2 = p.scale * 1.4426950408889634f;  // scores in base-2 units (scale > 0)
  pin_arch(sc2);
  u32x4_t ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // bf16 1.0 x 8
  pin_arch(ones_bits);  // a live register, never re-materialised right in front of an MFMA

  // ---- per-unit state
  f32x16_t o[NDB];
  f32x16_t o_one;   // every row: sum of the bf16-rounded weights (V block of ones)
  float m_ref = -INFINITY, l_run = 0.f;
  float heavy_thr = -INFINITY;  // see the heavy-weight test in tile_iter
  // log2 of the share of a row's running sum from which a weight counts as heavy.
  // 1/4: keys passed over end below a quarter of their row's sum each, which
  // bounds what their rounding can leave at 2^-8 times the weighted mean
  // distance of at least five values from the output (about 1e-3 for values of
  // unit variance; rows of four to eight random keys with every weight rounded
  // stay below 4.7e-3 in a CPU model of this arithmetic, and there the largest
  // weights, which this test catches, carry most of that).  At the start of a
  // segment, while the running sums are small, some row of a workgroup passes
  // the test on the first two or three tiles without holding a key that
  // matters in the end: that is the cost, about 0.6 % of a long chunk (with a
  // share of 1/8 it is 1.5 %).
  constexpr float kLogHeavyShare = -2.0f;
  int n_vis = 0, n_vis_min = 0;

  // ---- building blocks of the tile pipeline ---------------------------------------
  // The blocks take a stage parameter SG: SG >= 0 folds a compile-time stage into
  // the immediate offsets; SG < 0 (what the loop uses) means the stage has been
  // added to the address registers ka / ra / va by the caller.

  // zero the value rows at or beyond the sequence end in a freshly landed tile:
  // those slots may hold anything (NaN included) and 0-weight x garbage must not leak
  auto zero_tail = [&](int stage, int tile_j, int L) {
    const int tok0 = tile_j * TOK;
    if (tok0 + TOK > L) {
      const int valid = L - tok0;
#pragma unroll
      for (int g2 = 0; g2 < NG; ++g2) {
        unsigned char* sb = smem + g2 * TT::kGroupBytes + stage * STB;
        for (int off = valid * ROWB + tid * 16; off < STB; off += TT::kThreads * 16)
          *(u32x4_t*)(sb + off) = u32x4_t{0, 0, 0, 0};
      }
    }
  };

  // score operand ring: RS slots, all RS reads in flight, waited for in groups of 4
  constexpr int RS = 8;
  u32x4_t kfrag[RS];
  auto s_issue = [&](auto sgc, auto ic) {
    constexpr int SG = decltype(sgc)::value;
    constexpr int i = decltype(ic)::value;
    constexpr int ks = i / NTB, tb = i % NTB;
    constexpr int so = SG < 0 ? 0 : SG * STB, ro = SG < 0 ? 0 : SG * RTB;
    u32x4_t& f = kfrag[i % RS];
    if constexpr (ks < NKN) lds_read_b128<so + tb * 32 * ROWB + ((2 * ks) & ~15) * 16>(f, ka[ks & 7]);
    else lds_read_b128<ro + tb * 32 * 128>(f, ra[ks - NKN]);
  };
  auto s_wait = [&](auto ic) {  // before step i (i % 4 == 0): fragments i .. i+3 have arrived
    constexpr int i = decltype(ic)::value;
    constexpr int issued_r = (i + RS < NS ? i + RS : NS);
    constexpr int need = (i + 4 < NS ? i + 4 : NS);
    u32x4_t &f0 = kfrag[i % RS], &f1 = kfrag[(i + 1) % RS], &f2 = kfrag[(i + 2) % RS], &f3 = kfrag[(i + 3) % RS];
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f0), "+v"(f1), "+v"(f2), "+v"(f3) : "n"(issued_r - need));
  };
  auto s_mfma = [&](auto sgc, auto ic, f32x16_t (&acc)[NTB]) {
    constexpr int i = decltype(ic)::value;
    constexpr int ks = i / NTB, tb = i % NTB;
    if constexpr (ks == 0) mfma_first_v(acc[tb], kfrag[i % RS], qn[0]);
    else if constexpr (ks < NKN) mfma_acc_v(acc[tb], kfrag[i % RS], qn[ks]);
    else mfma_acc_v(acc[tb], kfrag[i % RS], qr[ks - NKN]);
    if constexpr (i + RS < NS) s_issue(sgc, std::integral_constant<int, i + RS>{});
  };

  // value operand ring: VRS fragments of two transposing reads each, waited for in pairs
  constexpr int VRS = 6;
  u32x2_t vlo[VRS], vhi[VRS];
  auto v_issue = [&](auto sgc, auto ic) {
    constexpr int SG = decltype(sgc)::value;
    constexpr int i = decltype(ic)::value;
    constexpr int st = i / NDB, db = i % NDB;
    constexpr int base = (SG < 0 ? 0 : SG * STB) + st * 16 * ROWB + (db >> 2) * 256;
    u32x2_t &l = vlo[i % VRS], &h = vhi[i % VRS];
    lds_read_tr16_b64<base>(l, va[db & 3][0]);
    lds_read_tr16_b64<base + 8 * ROWB>(h, va[db & 3][1]);
  };
  auto v_wait = [&](auto ic) {  // before step i (i even): fragments i, i+1 have arrived
    constexpr int i = decltype(ic)::value;
    constexpr int issued_f = (i + VRS < NP ? i + VRS : NP);
    constexpr int need = (i + 2 < NP ? i + 2 : NP);
    u32x2_t &l0 = vlo[i % VRS], &h0 = vhi[i % VRS], &l1 = vlo[(i + 1) % VRS], &h1 = vhi[(i + 1) % VRS];
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(l0), "+v"(h0), "+v"(l1), "+v"(h1) : "n"(2 * (issued_f - need)));
  };
  uint32_t pkw[TOK / 16][4];  // bf16 weight pairs: B operands of the 16-token contraction steps
  auto v_mfma = [&](auto sgc, auto ic) {
    constexpr int i = decltype(ic)::value;
    if constexpr (i < NP) {
      constexpr int st = i / NDB, db = i % NDB;
      const u32x4_t a4 = {vlo[i % VRS][0], vlo[i % VRS][1], vhi[i % VRS][0], vhi[i % VRS][1]};
      const u32x4_t b4 = {pkw[st][0], pkw[st][1], pkw[st][2], pkw[st][3]};
      mfma_acc_a(o[db], a4, b4);
      if constexpr (i + VRS < NP) v_issue(sgc, std::integral_constant<int, i + VRS>{});
    } else {
      const u32x4_t b4 = {pkw[i - NP][0], pkw[i - NP][1], pkw[i - NP][2], pkw[i - NP][3]};
      mfma_acc_a(o_one, ones_bits, b4);
    }
  };

  // softmax of one tile: three-deep software pipeline over its NE scores
  float neg_m = 0.f, lsum = 0.f;
  float sx[NE + 1], sp[NE + 1];
  auto sm_slot = [&](auto qc, f32x16_t (&sc)[NTB]) {
    constexpr int q = decltype(qc)::value;
    constexpr int e = q - 2;  // element whose weight is summed (and maybe packed) in this slot
    constexpr bool pack = e >= 1 && (e & 1) == 1;
    constexpr int pi = e >= 0 ? (e / 16) * 2 + ((e % 16) >> 3) : 0, pj = e >= 0 ? (e & 7) >> 1 : 0;
    if constexpr (q == 0) {
      sm_ops_f(sx[0], sc[0][0], sc2, neg_m);
    } else if constexpr (q == 1) {
      sm_ops_fe(sx[1], sc[1 / 16][1 % 16], sc2, neg_m, sp[0], sx[0]);
    } else if constexpr (q < NE) {
      if constexpr (pack) sm_ops_feac(sx[q], sc[q / 16][q % 16], sc2, neg_m, sp[q - 1], sx[q - 1], lsum, sp[e], pkw[pi][pj], sp[e - 1]);
      else sm_ops_fea(sx[q], sc[q / 16][q % 16], sc2, neg_m, sp[q - 1], sx[q - 1], lsum, sp[e]);
    } else if constexpr (q == NE) {
      if constexpr (pack) sm_ops_eac(sp[q - 1], sx[q - 1], lsum, sp[e], pkw[pi][pj], sp[e - 1]);
      else sm_ops_ea(sp[q - 1], sx[q - 1], lsum, sp[e]);
    } else {
      if constexpr (pack) sm_ops_ac(lsum, sp[e], pkw[pi][pj], sp[e - 1]);
      else sm_ops_a(lsum, sp[e]);
    }
  };
  constexpr int NQ = NE + 2;                            // pipeline slots
  constexpr int S0 = NS >= 16 ? 4 : (NS >= 8 ? 2 : 1);  // score steps that overlap the row-max search
  // Without a score exchange between waves (KS == 1) the masking and the row max
  // of a tile are computed one phase early, under the value MFMAs of the tile
  // before it, where the vector ALU is otherwise idle.
  constexpr bool kEarlyMax = KS == 1;
  constexpr int SA = kEarlyMax ? 0 : S0;                // first score step that carries softmax slots
  constexpr int IW = ((NS - 1) / 4) * 4;                // step of the last wait for score operands
  constexpr int VPRE = VRS < NP ? VRS : NP;             // value operands requested ahead of [B]
  constexpr int MXS = 4;                                // [B] steps over which the row-max chain is spread
  // With a deep tile ring (and no score exchange) the per-tile workgroup barrier
  // sits in the middle of [B] instead of at the top of the iteration: there it
  // waits for the tile after next, so the first score operands of the next
  // iteration can be requested under the last value MFMAs and their LDS latency
  // no longer opens the iteration; the loads of the iteration follow the barrier
  // (they overwrite the stage of the tile before this one, which every wave has
  // left by then).  One tile less is in flight at the wait, hence the deep ring.
  constexpr bool kEarlyBar = KS == 1 && STAGES >= 8;
  constexpr int JB = NB / 2 - 1;                        // [B] step that carries the barrier
  constexpr int RSN = RS < NS ? RS : NS;                // score operands requested ahead
  static_assert(!kEarlyBar || (JB >= 3 && NB - 3 > JB && NP - 2 < NB - 3), "step layout of [B] with the barrier inside");
  static_assert(2 + MXS <= NB, "row-max steps fit into [B]");
  float mx_carry = -INFINITY;                           // kEarlyMax: lane-local max of the next tile's scores
  auto mask_tile = [&](f32x16_t (&sc)[NTB], int tile_j) {
    const int tile_tok0 = tile_j * TOK;
    if (tile_tok0 + TOK > n_vis_min) {
      const int lim = n_vis - tile_tok0 - 4 * hi;  // element (tb, i) is visible iff its constant < lim
#pragma unroll
      for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          sc[tb][i] = (32 * tb + 8 * (i >> 2) + (i & 3)) < lim ? sc[tb][i] : -INFINITY;
    }
  };

  // KS = 2: the two waves of a row slab hold partial scores (each over its share
  // of the contraction dims).  Each posts its 16 values per lane in its own
  // mailbox; after the next workgroup barrier it adds its partner's to its own
  // (both get bit-identical sums: a + b == b + a), and a second barrier lets
  // the mailboxes be overwritten.
  const unsigned xchg_mine = lds_base + (unsigned)(TT::kXchgBase + wave * 4096 + lane * 16);
  const unsigned xchg_peer = lds_base + (unsigned)(TT::kXchgBase + (wave ^ 1) * 4096 + lane * 16);
  auto xchg_post = [&](f32x16_t (&sc)[NTB]) {
    if constexpr (KS > 1) {
      static_assert(NTB == 1, "mailbox holds one 32-token block");
      // MFMA results are read by the LDS stores below.  The wait is tied to the
      // accumulator so that no copy of it can be scheduled ahead of the wait.
      asm volatile("s_nop 15" : "+v"(sc[0]));
      static_for<0, 4>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        // (vector elements go through scalars: a bit cast applied directly to an
        // element of a vector reads the vector's first element)
        const float f0 = sc[0][4 * i], f1 = sc[0][4 * i + 1], f2 = sc[0][4 * i + 2], f3 = sc[0][4 * i + 3];
        const u32x4_t v = {__builtin_bit_cast(uint32_t, f0), __builtin_bit_cast(uint32_t, f1),
                           __builtin_bit_cast(uint32_t, f2), __builtin_bit_cast(uint32_t, f3)};
        lds_write_b128<i * 1024>(xchg_mine, v);
      });
    }
  };
  u32x4_t xin[4];
  auto xchg_fetch = [&]() {  // issue the reads of the partner's mailbox
    if constexpr (KS > 1) static_for<0, 4>([&](auto ic) { lds_read_b128<decltype(ic)::value * 1024>(xin[decltype(ic)::value], xchg_peer); });
  };
  auto xchg_add = [&](f32x16_t (&sc)[NTB]) {  // call with exactly the RS score-operand reads issued after xchg_fetch
    if constexpr (KS > 1) {
      asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(xin[0]), "+v"(xin[1]), "+v"(xin[2]), "+v"(xin[3]) : "n"(RS < NS ? RS : NS));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const uint32_t u = xin[i >> 2][i & 3];
        sc[0][i] += __builtin_bit_cast(float, u);
      }
      asm volatile("s_barrier" ::: "memory");
    }
  };
  // Second value pass of a tile with heavy weights (rare: the first tiles of a
  // segment, rows with a few dominant keys).  The weights are formed again from
  // the scores exactly as the softmax slots formed them, p = 2^(s * sc2 - m),
  // split as p = hi + lo with hi = bf16(p) (what the first pass used), and lo,
  // exact in fp32 and itself rounded to bf16, goes through the same value and
  // row-sum MFMAs: the tile's weights then carry 16 significant bits.  Runs
  // right behind [B] of the same tile: its stage is still intact (no wave can
  // pass the next barrier, after which the stage is reloaded, before this wave
  // has), the address registers still point at it and the operand rings are free.
  auto residual_pass = [&](f32x16_t (&sc)[NTB]) {
    static_for<0, NE / 2>([&](auto jc) {
      constexpr int e = 2 * decltype(jc)::value;
      constexpr int pi = (e / 16) * 2 + ((e % 16) >> 3), pj = (e & 7) >> 1;
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[e / 16][e % 16], sc2, neg_m));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[(e + 1) / 16][(e + 1) % 16], sc2, neg_m));
      const uint32_t hi_pk = cvt_pk_bf16(p0, p1);
      const float h0 = __builtin_bit_cast(float, hi_pk << 16), h1 = __builtin_bit_cast(float, hi_pk & 0xffff0000u);
      const float l0 = p0 - h0, l1 = p1 - h1;  // (0 - 0 for masked elements; padding rows may hold anything)
      pkw[pi][pj] = cvt_pk_bf16(l0, l1);
    });
    constexpr std::integral_constant<int, -1> psgc{};
    static_for<0, VPRE>([&](auto jc) { v_issue(psgc, jc); });
    wait_states<2>();  // the residuals were packed by the vector ALU just above
    static_for<0, NB>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      if constexpr (i < NP && i % 2 == 0) v_wait(ic);
      v_mfma(psgc, ic);
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // One tile: [A] softmax of tile k (scores in s_rd) under the score MFMAs of
  // tile k+1 (into s_wr), then [B] value MFMAs of tile k under the loads of tile
  // k + STAGES - 1.  k: chunk-local tile index, tile_j: index in the unit, PSG /
  // SSG: stage of tile k / of tile k+1 (or -1, see above), pv_stage: stage of tile k.
  auto tile_iter = [&](f32x16_t (&s_rd)[NTB], f32x16_t (&s_wr)[NTB], int k, int tile_j, bool has_next, bool has_next2,
                       int seg_L) {
    constexpr std::integral_constant<int, -1> psgc{}, ssgc{};  // stages live in the address registers
    const int pv_stage = k % STAGES;
    // ---- tile k+1 landed?  (also: every wave is done with tile k-1, so its stage is free)
    if constexpr (!kEarlyBar) {
      if (has_next) {
        if (issued - 2 - k >= STAGES - 3) wait_vmcnt<LPW * (STAGES - 3)>();
        else wait_vmcnt<0>();
      }
      lds_barrier();
    }
    if constexpr (!kEarlyBar) {
      if (has_next) zero_tail((pv_stage + 1) % STAGES, tile_j + 1, seg_L);
    }

    // ---- [A] first score steps of tile k+1 (without a next tile they read
    //          whatever is in that stage and the result is dropped), under the
    //          masking and row-max search of tile k
    xchg_fetch();
    if constexpr (!kEarlyBar) static_for<0, RSN>([&](auto ic) { s_issue(ssgc, ic); });  // (else: requested in the previous [B])
    xchg_add(s_rd);
    float mx;
    if constexpr (kEarlyMax) {
      // masking and row max of tile k were done while the previous tile's value
      // MFMAs ran (or in the segment prologue): only the cross-half step is left
      mx = half_swap_max(mx_carry) * sc2;
    } else {
      mask_tile(s_rd, tile_j);
      mx = -INFINITY;
      pin_arch(mx);
      static_for<0, S0>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        if constexpr (i % 4 == 0) s_wait(ic);
        constexpr int e0 = (i * NE) / S0, e1 = ((i + 1) * NE) / S0;
        static_for<e0 / 2, e1 / 2>([&](auto jc) {
          constexpr int e = 2 * decltype(jc)::value;
          asm_max3(mx, s_rd[e / 16][e % 16], s_rd[(e + 1) / 16][(e + 1) % 16]);
        });
        s_mfma(ssgc, ic, s_wr);
        __builtin_amdgcn_sched_barrier(0);
      });
      mx = half_swap_max(mx) * sc2;
    }
    // lazy reference update: keep the old reference while the row max stays
    // within 2^8 of it (weights then stay <= 256, exact enough in fp32 / bf16)
    const bool bump = mx > m_ref + 8.0f;
    if (__ballot(bump)) {
      wait_states<16>();  // output accumulators are about to be read by the vector ALU
      const float m_new = bump ? mx : m_ref;
      const float alpha = bump ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.0f;  // m_ref = -inf -> 0
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db) {  // one 16-register block at a time through the vector ALU
        f32x16_t t = o[db];
        pin_arch(t);
#pragma unroll
        for (int i = 0; i < 16; ++i) t[i] *= alpha;
        o[db] = t;
        pin_acc(o[db]);
      }
      {
        f32x16_t t = o_one;
        pin_arch(t);
#pragma unroll
        for (int i = 0; i < 16; ++i) t[i] *= alpha;
        o_one = t;
        pin_acc(o_one);
      }
      m_ref = m_new;
    }
    neg_m = m_ref == -INFINITY ? 0.f : -m_ref;
    lsum = 0.f;
    pin_arch(neg_m);
    pin_arch(lsum);
    // ---- [A] (remaining) score steps of tile k+1 under the exponentials of tile k.
    //          Once the last score operands have been waited for, the first value
    //          operands of [B] are requested so that they arrive under these MFMAs.
    static_for<SA, NS>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      if constexpr (i % 4 == 0) s_wait(ic);
      constexpr int q0 = ((i - SA) * NQ) / (NS - SA), q1 = ((i - SA + 1) * NQ) / (NS - SA);
      static_for<q0, q1>([&](auto qc) { sm_slot(qc, s_rd); });
      s_mfma(ssgc, ic, s_wr);
      if constexpr (i >= IW)
        static_for<((i - IW) * VPRE) / (NS - IW), ((i - IW + 1) * VPRE) / (NS - IW)>([&](auto jc) { v_issue(psgc, jc); });
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run += lsum;
    xchg_post(s_wr);

    // ---- [B] O^T += V^T . P^T for tile k under the loads of the tile that reuses
    //          the stage of tile k-1.  Contraction slot (hi, j) of step st is token
    //          16*st + 8*(j/4) + 4*hi + j%4, matching the score accumulator layout.
    //          The address registers move on to the next stages in the gaps.
    const bool s_wrap = (pv_stage + 2) % STAGES == 0, v_wrap = (pv_stage + 1) % STAGES == 0;
    const int k_step = s_wrap ? -(STAGES - 1) * STB : STB, r_step = s_wrap ? -(STAGES - 1) * RTB : RTB;
    const int v_step = v_wrap ? -(STAGES - 1) * STB : STB;
    wait_states<2>();  // the last weights were packed by the vector ALU just above
    static_for<0, NB>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      if constexpr (i < NP && i % 2 == 0) v_wait(ic);
      v_mfma(psgc, ic);
      if constexpr (kEarlyMax) {  // masking and lane-local row max of tile k+1 (its scores are complete)
        if constexpr (i == 1) {
          if (has_next) mask_tile(s_wr, tile_j + 1);
          mx_carry = -INFINITY;
          pin_arch(mx_carry);
        } else if constexpr (i >= 2 && i < 2 + MXS) {
          static_for<((i - 2) * (NE / 2)) / MXS, ((i - 1) * (NE / 2)) / MXS>([&](auto jc) {
            constexpr int e = 2 * decltype(jc)::value;
            asm_max3(mx_carry, s_wr[e / 16][e % 16], s_wr[(e + 1) / 16][(e + 1) % 16]);
          });
        }
      }
      // preparation of the next loads in the first steps, the loads themselves after it
      if constexpr (i == 0) dma_prepare_0((pv_stage + STAGES - 1) % STAGES);
      else if constexpr (i == 1) dma_prepare_1();
      else if constexpr (i == 2) dma_prepare_2();
      if constexpr (!kEarlyBar) {
        if constexpr (i >= 3) static_for<((i - 3) * LPW) / (NB - 3), ((i - 2) * LPW) / (NB - 3)>(dma_load);
        // score addresses: next used in the next tile's [A]
        static_for<(i * (8 + NKR)) / NB, ((i + 1) * (8 + NKR)) / NB>([&](auto ec) {
          constexpr int e = decltype(ec)::value;
          if constexpr (e < 8) ka[e] += k_step;
          else ra[e - 8] += r_step;
        });
      } else {
        if constexpr (i == JB) {
          // tile k+2 landed?  The loads of this iteration have not been issued yet
          // (`issued` already counts its tile if one was prepared above): behind
          // tile k+2 there are then the tiles up to k + STAGES - 2.
          if (has_next2) {
            if (issued - (prep_active ? 1 : 0) - (k + 3) >= STAGES - 4) wait_vmcnt<LPW * (STAGES - 4)>();
            else wait_vmcnt<0>();
          }
          bare_barrier();  // (value operands of this tile stay in flight across it)
          if (has_next2) zero_tail((pv_stage + 2) % STAGES, tile_j + 2, seg_L);
        } else if constexpr (i > JB) {
          static_for<((i - JB - 1) * LPW) / (NB - JB - 1), ((i - JB) * LPW) / (NB - JB - 1)>(dma_load);
        }
        // score addresses: moved on to the stage of tile k+2 before the last three steps ...
        if constexpr (i < NB - 3) {
          static_for<(i * (8 + NKR)) / (NB - 3), ((i + 1) * (8 + NKR)) / (NB - 3)>([&](auto ec) {
            constexpr int e = decltype(ec)::value;
            if constexpr (e < 8) ka[e] += k_step;
            else ra[e - 8] += r_step;
          });
        } else {
          // ... in which the first score operands of the next iteration are requested
          // (no value operand is waited for any more at this point)
          if (has_next)
            static_for<((i - (NB - 3)) * RSN) / 3, ((i - (NB - 3) + 1) * RSN) / 3>([&](auto jc) { s_issue(ssgc, jc); });
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // Weights went into the value product rounded to bf16 (relative error up to
    // 2^-8 each).  Spread over many keys that averages out; a row whose sum is
    // carried by two or three keys keeps up to 2^-8 w_1 w_2 |v_1 - v_2| of it.  So a
    // tile holding a weight above kHeavyShare of its row's running sum gets a
    // second value pass with the rounding residuals (residual_pass).  Later
    // tiles only make the sum larger, so every key this test passes over ends
    // with a normalised weight below that share.  In base-2 logarithms the test
    // reads (row max of the tile) > log2(row sum) + log2(share), all taken
    // absolute (not relative to the lazy reference), and the right-hand side
    // only grows along a segment: heavy_thr holds its value from the last time
    // it was worked out, one compare per tile decides whether it has to be
    // worked out again.  Kept out of the straight-line path.
    if (__builtin_expect(__ballot(mx > heavy_thr) != 0, 0)) {
      const float l_row = half_swap_sum(l_run);  // both halves of the row
      heavy_thr = __builtin_amdgcn_logf(l_row) + kLogHeavyShare - neg_m;  // (-inf while the row has no key)
      if (__ballot(mx > heavy_thr) != 0) residual_pass(s_rd);
    }
    // value addresses: every read of this tile has been issued
#pragma unroll
    for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
      for (int a = 0; a < 2; ++a) va[d4][a] += v_step;
  };
  // the two score register sets: tile t of a segment reads the one tile t-1 wrote
  f32x16_t s_even[NTB], s_odd[NTB];
  int k = 0;  // chunk-local index of the tile at `cur`
  while (k < n_tiles) {
    // ================= segment: the tiles of cur's unit that lie in this chunk
    const int seg_n = min(n_tiles - k, cur.tiles_b - cur.j);
    const int seg_j0 = cur.j;
    const int seg_L = cur.L;
    const int seg_tiles_b = cur.tiles_b;
    const int seg_unit = (cur.b * UPB + cur.ub) * MB + mb_wg;  // index of this (unit, row block)
    // Query fragments of this unit.  The wait follows at once (it also covers the
    // tiles already requested): the registers the loads write must not be
    // touched, not even copied, before the data has arrived, and only a wait
    // right behind the requests guarantees that.
    q_issue();
    wait_vmcnt<0>();
    {
#pragma unroll
      for (int ks = 0; ks < NKN; ++ks) pin_acc(qn[ks]);
#pragma unroll
      for (int ks = 0; ks < NKR; ++ks) {
        pin_acc(qr[ks]);  // (first: a use of the loaded value that cannot move ahead of the wait)
        if (kx * DRW + 16 * ks >= p.d_r) qr[ks] = u32x4_t{0, 0, 0, 0};  // RoPE keys of fewer than 64 dims
        pin_acc(qr[ks]);
      }
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
        pin_acc(o[db]);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) o_one[i] = 0.f;
      pin_acc(o_one);
      m_ref = -INFINITY;
      l_run = 0.f;
      heavy_thr = -INFINITY;
      // visible keys of this lane's row; padding rows are left unmasked (never stored)
      n_vis = row_valid ? (p.causal ? cur.L - p.T + 1 + row_t : cur.L) : 0x7fffffff;
      // the smallest count of the wave: its first row (lane 0) has the earliest query position
      n_vis_min = __builtin_amdgcn_readlane(n_vis, 0);
    }

    // ---- segment prologue: point the address registers at the stages of tile k
    //      (value reads) and, after its scores are done, of tile k+1 (score reads)
    lds_barrier();
    zero_tail(k % STAGES, seg_j0, seg_L);
    if constexpr (kEarlyBar) {  // the tile after it has landed too (everything requested so far has)
      if (seg_n >= 2) zero_tail((k + 1) % STAGES, seg_j0 + 1, seg_L);
      // The zeroing is spread over all threads and the first iteration has no
      // barrier before its value reads of tile k (they are requested at the end
      // of its phase [A]): every wave's zeros must have landed before that.
      if constexpr (NWAVES > 1) lds_barrier();
    }
    {
      const int ss = k % STAGES;
#pragma unroll
      for (int e = 0; e < 8; ++e) ka[e] = k_off[e] + ss * STB;
#pragma unroll
      for (int e = 0; e < NKR; ++e) ra[e] = r_off[e] + ss * RTB;
#pragma unroll
      for (int d4 = 0; d4 < 4; ++d4)
#pragma unroll
        for (int a = 0; a < 2; ++a) va[d4][a] = v_off[d4][a] + ss * STB;
      constexpr std::integral_constant<int, -1> rt{};
      static_for<0, (RS < NS ? RS : NS)>([&](auto ic) { s_issue(rt, ic); });
      static_for<0, NS>([&](auto ic) {
        if constexpr (decltype(ic)::value % 4 == 0) s_wait(ic);
        s_mfma(rt, ic, s_even);
      });
      const bool wrap = (ss + 1) % STAGES == 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) ka[e] += wrap ? -(STAGES - 1) * STB : STB;
#pragma unroll
      for (int e = 0; e < NKR; ++e) ra[e] += wrap ? -(STAGES - 1) * RTB : RTB;
      if constexpr (kEarlyBar) static_for<0, RSN>([&](auto ic) { s_issue(rt, ic); });  // for the first iteration's [A]
    }
    // the scores are read by the vector ALU next; the wait is tied to them so
    // that no read can be scheduled ahead of it
    asm volatile("s_nop 15" : "+v"(s_even[0]));
    if constexpr (kEarlyMax) {
      mask_tile(s_even, seg_j0);
      mx_carry = -INFINITY;
      pin_arch(mx_carry);
      static_for<0, NE / 2>([&](auto jc) {
        constexpr int e = 2 * decltype(jc)::value;
        asm_max3(mx_carry, s_even[e / 16][e % 16], s_even[(e + 1) / 16][(e + 1) % 16]);
      });
    }
    xchg_post(s_even);

    // two tiles per trip so that the two score register sets swap roles without copies
    for (int t = 0; t < seg_n; t += 2) {
      tile_iter(s_even, s_odd, k, seg_j0 + t, t + 1 < seg_n, t + 2 < seg_n, seg_L);
      ++k;
      if (t + 1 < seg_n) {
        tile_iter(s_odd, s_even, k, seg_j0 + t + 1, t + 2 < seg_n, t + 3 < seg_n, seg_L);
        ++k;
      }
    }
    for (int i = 0; i < seg_n; ++i) advance<TOK>(p, UPB, cur);

    // ================= end of segment: write the unit's result or its partial
    wait_states<16>();  // output accumulators: last MFMA -> vector ALU reads
    {
      const bool unit_done = seg_j0 + seg_n == (seg_L + TOK - 1) / TOK;
      const bool complete = unit_done && seg_j0 == 0;
      const float l_tot = half_swap_sum(l_run);
      f32x16_t one_t = o_one;
      pin_arch(one_t);
      const float r_tot = one_t[0];
      const float inv = r_tot > 0.f ? 1.0f / r_tot : 0.f;
      const float lse = l_tot > 0.f ? (m_ref + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
      const int lr = wave * 32 + col;
      const int64_t ob = row_b * p.out_s[0] + row_t * p.out_s[1] + row_h * p.out_s[2];
      // partial: slot 1 if the unit's first tile is in this chunk, slot 0 if it began earlier
      float* slot = p.ws_out + (((size_t)chunk_id * MB + mb_wg) * 2 + (seg_j0 == 0 ? 1 : 0)) * TT::kSlotFloats;
      if (seg_j0 == 0 && tid == 0) {
        // tell the merge kernel which chunks hold this unit: it starts here and
        // ends in the chunk of its last tile
        const int s_u = c0 + (k - seg_n);
        int2 span;
        span.x = chunk_id;
        span.y = (s_u + seg_tiles_b - 1) / chunk;
        ((int2*)p.ws_lse)[seg_unit] = span;
      }
      if (hi == 0) {
        if (!complete) slot[(size_t)TT::kRows * DV + lr] = lse;
        else if (row_valid && kx == 0) p.lse[((int64_t)row_b * p.T + row_t) * p.h_q + row_h] = lse;
      }
#pragma unroll
      for (int db = 0; db < NDB; ++db) {  // one 16-register block at a time
        f32x16_t t16 = o[db];
        pin_arch(t16);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int dim = kx * DVW + 32 * db + 8 * q4 + 4 * hi;
          const f32x4_t v = {t16[4 * q4] * inv, t16[4 * q4 + 1] * inv, t16[4 * q4 + 2] * inv, t16[4 * q4 + 3] * inv};
          if (!complete) {
            // fragment order: one contiguous 1 KiB block per (wave, db, q4), lane-linear
            *(f32x4_t*)(slot + (size_t)((wave * NDB + db) * 4 + q4) * 256 + lane * 4) = v;
          } else if (row_valid) {
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
      }
    }
  }
}

}  // namespace gla
