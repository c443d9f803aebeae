// Device-side building blocks of the tuned decode-attention path: vector
// types, hand-issued LDS / MFMA / wait instructions, register-class pins,
// half-wave exchanges, the wave scan, and the cursor over the flat tile list.
#pragma once

#include <cstdint>
#include <type_traits>

#include <hip/hip_runtime.h>

#include "common.hpp"

namespace gla {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_cvoid_t;

// ---- small device helpers -------------------------------------------------

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

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

// Workgroup barrier alone: LDS reads of this wave that are in flight stay in
// flight (used where the barrier only orders tile loads against other waves).
__device__ __forceinline__ void bare_barrier() {
  asm volatile("s_barrier" ::: "memory");
}

// Hand-issued LDS reads.  The result registers are valid only after a matching
// lds_wait on them; LDS returns data in issue order, so "at most N reads still
// outstanding" identifies which reads have completed.
template <int OFF>
__device__ __forceinline__ void lds_read_b128(u32x4_t& dst, unsigned addr) {
  static_assert(OFF >= 0 && OFF < 65536, "ds offset field");
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// Transposing read: within each block of 16 lanes, lanes 4r..4r+3 address row r
// (4 x b16 each) of a 4 x 16 matrix; lane i receives column i (4 x b16).
template <int OFF>
__device__ __forceinline__ void lds_read_tr16_b64(u32x2_t& dst, unsigned addr) {
  static_assert(OFF >= 0 && OFF < 65536, "ds offset field");
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void lds_write_b128(unsigned addr, const u32x4_t& v) {
  static_assert(OFF >= 0 && OFF < 65536, "ds offset field");
  asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(OFF) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x4_t& x) {
  static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lds_wait2(u32x2_t& x, u32x2_t& y) {
  static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(N));
}

// MFMA 32x32x16 bf16 issued as inline asm so that every operand's register file
// is fixed: score accumulators live in architectural VGPRs (the vector ALU
// reads them), output accumulators and query fragments in accumulation VGPRs.
// The compiler does not see these as matrix instructions, so the wait states
// the hardware needs around them are provided by hand where the surrounding
// code does not already guarantee them:
//   * a vector-ALU write of an MFMA source needs 2 wait states before the MFMA;
//   * an MFMA result needs 12 wait states before anything but a dependent MFMA
//     on the same accumulator reads it (back-to-back accumulation needs none).
__device__ __forceinline__ void mfma_first_v(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b_acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b_acc));
}
__device__ __forceinline__ void mfma_acc_v(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b_acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b_acc));
}
__device__ __forceinline__ void mfma_acc_a(f32x16_t& acc, const u32x4_t& a, const u32x4_t& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
template <int N>
__device__ __forceinline__ void wait_states() {
  static_assert(N >= 1 && N <= 16, "s_nop covers 1..16 wait states");
  asm volatile("s_nop %0" ::"n"(N - 1));
}

// Vector-ALU pieces of the softmax, issued by hand so that they stay exactly
// where they are written between the MFMAs they overlap with.  One statement
// per pipeline slot: x_q = s_q * sc2 - m ; p_{q-1} = 2^{x_{q-1}} ; sum += p_{q-2} ;
// on odd q-2 also pack (p_{q-3}, p_{q-2}) to bf16.  Inside a statement no
// instruction reads the result of the one before it (v_exp_f32 is a
// transcendental: its result must not be consumed by the next instruction).
__device__ __forceinline__ void sm_ops_f(float& x, float s, float sc2, float neg_m) {
  asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(x) : "v"(s), "v"(sc2), "v"(neg_m));
}
__device__ __forceinline__ void sm_ops_fe(float& x, float s, float sc2, float neg_m, float& p1, float x1) {
  asm volatile("v_fma_f32 %0, %2, %3, %4\n\tv_exp_f32 %1, %5"
               : "=&v"(x), "=v"(p1) : "v"(s), "v"(sc2), "v"(neg_m), "v"(x1));
}
__device__ __forceinline__ void sm_ops_fea(float& x, float s, float sc2, float neg_m, float& p1, float x1,
                                           float& sum, float p2) {
  asm volatile("v_fma_f32 %0, %3, %4, %5\n\tv_exp_f32 %1, %6\n\tv_add_f32 %2, %2, %7"
               : "=&v"(x), "=&v"(p1), "+v"(sum) : "v"(s), "v"(sc2), "v"(neg_m), "v"(x1), "v"(p2));
}
__device__ __forceinline__ void sm_ops_feac(float& x, float s, float sc2, float neg_m, float& p1, float x1,
                                            float& sum, float p2, uint32_t& pk, float p3) {
  asm volatile("v_fma_f32 %0, %4, %5, %6\n\tv_exp_f32 %1, %7\n\tv_add_f32 %2, %2, %8\n\tv_cvt_pk_bf16_f32 %3, %9, %8"
               : "=&v"(x), "=&v"(p1), "+v"(sum), "=&v"(pk)
               : "v"(s), "v"(sc2), "v"(neg_m), "v"(x1), "v"(p2), "v"(p3));
}
__device__ __forceinline__ void sm_ops_ea(float& p1, float x1, float& sum, float p2) {
  asm volatile("v_exp_f32 %0, %2\n\tv_add_f32 %1, %1, %3" : "=&v"(p1), "+v"(sum) : "v"(x1), "v"(p2));
}
__device__ __forceinline__ void sm_ops_eac(float& p1, float x1, float& sum, float p2, uint32_t& pk, float p3) {
  asm volatile("v_exp_f32 %0, %3\n\tv_add_f32 %1, %1, %4\n\tv_cvt_pk_bf16_f32 %2, %5, %4"
               : "=&v"(p1), "+v"(sum), "=&v"(pk) : "v"(x1), "v"(p2), "v"(p3));
}
__device__ __forceinline__ void sm_ops_a(float& sum, float p2) {
  asm volatile("s_nop 0\n\tv_add_f32 %0, %0, %1" : "+v"(sum) : "v"(p2));
}
__device__ __forceinline__ void sm_ops_ac(float& sum, float p2, uint32_t& pk, float p3) {
  asm volatile("s_nop 0\n\tv_add_f32 %0, %0, %2\n\tv_cvt_pk_bf16_f32 %1, %3, %2" : "+v"(sum), "=&v"(pk) : "v"(p2), "v"(p3));
}
// Two fp32 values rounded to bf16 (nearest even), `a` in the low half: one
// v_cvt_pk_bf16_f32.  Left to the compiler (not inline asm) so that it sees the
// instruction and provides the wait state a transcendental result needs before
// its first use.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{a, b}, bf16x2_t));
}
__device__ __forceinline__ void asm_max3(float& m, float a, float b) {
  asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(m) : "v"(a), "v"(b));
}
// 16-byte global load straight into an accumulation VGPR tuple (no staging in
// architectural VGPRs); complete after the next wait_vmcnt<0>().
__device__ __forceinline__ void load_b128_async(u32x4_t& dst, const void* ptr) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(dst) : "v"(ptr) : "memory");
}

// Predicated 32-bit global loads into N registers the caller keeps: issued when
// `cond` (uniform) is not zero, complete after a wait_vmcnt that covers them.
// One statement that is executed either way, with the registers as read-write
// operands: each keeps its place whether or not it is loaded.  row: uniform
// base address; o0..o3: byte offsets per lane (non-negative, below 2^31).
template <int N>
__device__ __forceinline__ void load_window(int cond, const int32_t* row, int o0, int o1, int o2, int o3, int& w0,
                                            int& w1, int& w2, int& w3) {
  static_assert(N == 2 || N == 4, "registers per window");
  if constexpr (N == 2)
    asm volatile(
        "s_cmp_eq_u32 %[c], 0\n\t"
        "s_cbranch_scc1 .Lgla_win_skip%=\n\t"
        "global_load_dword %[w0], %[o0], %[row]\n\t"
        "global_load_dword %[w1], %[o1], %[row]\n"
        ".Lgla_win_skip%=:"
        : [w0] "+v"(w0), [w1] "+v"(w1)
        : [c] "s"(cond), [row] "s"(row), [o0] "v"(o0), [o1] "v"(o1)
        : "memory", "scc");
  else
    asm volatile(
        "s_cmp_eq_u32 %[c], 0\n\t"
        "s_cbranch_scc1 .Lgla_win_skip%=\n\t"
        "global_load_dword %[w0], %[o0], %[row]\n\t"
        "global_load_dword %[w1], %[o1], %[row]\n\t"
        "global_load_dword %[w2], %[o2], %[row]\n\t"
        "global_load_dword %[w3], %[o3], %[row]\n"
        ".Lgla_win_skip%=:"
        : [w0] "+v"(w0), [w1] "+v"(w1), [w2] "+v"(w2), [w3] "+v"(w3)
        : [c] "s"(cond), [row] "s"(row), [o0] "v"(o0), [o1] "v"(o1), [o2] "v"(o2), [o3] "v"(o3)
        : "memory", "scc");
}

// A 32-bit global load that is complete when the statement ends.  Used for the
// rare bookkeeping reads inside the tile loop (page ids, next sequence length):
// being opaque to the compiler's memory-counter tracking, it cannot make the
// compiler place a "wait for every outstanding load" in the steady-state path,
// which would drain the tile prefetch ring on every iteration.
__device__ __forceinline__ int load_i32_sync(const int32_t* ptr) {
  int v;
  asm volatile("global_load_dword %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(ptr) : "memory");
  return v;
}

// Four such loads in flight together, complete when the statement ends.
__device__ __forceinline__ void load_i32x4_sync(int& v0, int& v1, int& v2, int& v3, const int32_t* p0, const int32_t* p1,
                                                const int32_t* p2, const int32_t* p3) {
  asm volatile(
      "global_load_dword %0, %4, off\n\tglobal_load_dword %1, %5, off\n\tglobal_load_dword %2, %6, off\n\t"
      "global_load_dword %3, %7, off\n\ts_waitcnt vmcnt(0)"
      : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3)
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
}

// Register-class pins (no instruction is emitted).  MFMA accumulators and the
// query fragments, which are only ever MFMA operands inside the tile loop, are
// kept in the accumulation half of the unified register file; everything the
// vector ALU touches stays in the architectural half.  Without the pins the
// allocator shuttles the output accumulators between the halves every tile.
template <class V>
__device__ __forceinline__ void pin_acc(V& x) { asm volatile("" : "+a"(x)); }
template <class V>
__device__ __forceinline__ void pin_arch(V& x) { asm volatile("" : "+v"(x)); }

// max / sum over the two half-waves (lane and lane ^ 32).  v_permlane32_swap
// exchanges the upper half of its first register with the lower half of its
// second, so afterwards the pair holds (lower, lower) and (upper, upper).
// Issued as inline asm: the compiler's builtin folds the two results of a swap
// of a value with itself into one.  The s_nop covers the wait states this
// instruction needs after a vector-ALU write of its operands.
__device__ __forceinline__ void half_swap(float x, float& a, float& b) {
  a = x;
  b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float half_swap_max(float x) {
  float a, b;
  half_swap(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float half_swap_sum(float x) {
  float a, b;
  half_swap(x, a, b);
  return a + b;
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves
// (no LDS round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes, then
// the last lane of row 0 / 2 is broadcast into row 1 / 3 and lane 31 into the
// upper half.  Lanes that receive nothing add zero.
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

template <int TOK>
__device__ __forceinline__ int tiles_of(int L) {
  return L > 0 ? (L + TOK - 1) / TOK : 0;
}

// Position in the flat tile list.
struct TileCursor {
  int b;        // sequence
  int ub;       // unit within the sequence (group block)
  int j;        // tile within the unit
  int tiles_b;  // tiles per unit of this sequence
  int L;        // its length
};

// Total number of tiles of the batch (every wave computes the same value).
// incl0: inclusive prefix sums of the tile counts of the first 64 sequences.
template <int TOK>
__device__ __forceinline__ int total_tiles(const DevParams& p, int UPB, int lane, int incl0) {
  int total = __builtin_amdgcn_readlane(incl0, 63);
  for (int base = 64; base < p.B; base += 64) {
    const int idx = base + lane;
    const int w = idx < p.B ? tiles_of<TOK>(p.seq_lens[idx]) * UPB : 0;
    total += __builtin_amdgcn_readlane(wave_incl_scan(w), 63);
  }
  return total;
}

// Locate flat tile index `pos` (< total): which sequence / unit / tile.
// L_first / incl0: length and inclusive tile prefix of the first 64 sequences.
template <int TOK>
__device__ __forceinline__ TileCursor locate_tile(const DevParams& p, int UPB, int pos, int lane, int L_first,
                                                  int incl0) {
  TileCursor c = {0, 0, 0, 0, 0};
  int before = 0;
  for (int base = 0; base < p.B; base += 64) {
    const int idx = base + lane;
    const int L = base == 0 ? L_first : (idx < p.B ? p.seq_lens[idx] : 0);
    const int tl = tiles_of<TOK>(L);
    const int w = tl * UPB;
    const int incl = (base == 0 ? incl0 : wave_incl_scan(w)) + before;
    const int excl = incl - w;
    const unsigned long long hit = __ballot(w > 0 && excl <= pos && pos < incl);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      const int ex = __builtin_amdgcn_readlane(excl, src);
      c.tiles_b = __builtin_amdgcn_readlane(tl, src);
      c.L = __builtin_amdgcn_readlane(L, src);
      c.b = base + src;
      const int rem = pos - ex;
      c.ub = (int)((unsigned)rem / (unsigned)c.tiles_b);
      c.j = rem - c.ub * c.tiles_b;
      return c;
    }
    before = __builtin_amdgcn_readlane(incl, 63);
  }
  return c;
}

template <int TOK>
__device__ __forceinline__ void advance(const DevParams& p, int UPB, TileCursor& c) {
  if (++c.j < c.tiles_b) return;
  c.j = 0;
  if (++c.ub < UPB) return;
  c.ub = 0;
  do {
    ++c.b;
    c.L = c.b < p.B ? uniform(load_i32_sync(p.seq_lens + c.b)) : 0;
    c.tiles_b = tiles_of<TOK>(c.L);
  } while (c.b < p.B && c.tiles_b == 0);
}

}  // namespace gla
