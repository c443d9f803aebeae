// The two projections around the decode attention (paper Sections 2.1 and
// 3.3.2), both instances of a skinny grouped GEMM on bf16 MFMA:
//
//     C[m][g][n] = sum_k A[m][g][k] * W[g][n][k]              (absorbed query)
//     C[m][n]    = sum_g sum_k A[m][g][k] * W[g][n][k]        (grouped output projection)
//
// m runs over the few query rows of a decode step (batch x q_len), so the
// work is reading W once: the kernel is bound by HBM, and the weights are the
// operand that streams.  Transposed form C^T = W . A^T: a wave owns 32*NT output
// features (rows of W, the MFMA A operand) and all 32*MT query rows of its
// workgroup (columns, the B operand).
//
// Both operands travel global -> LDS with direct-to-LDS loads of 16 bytes per
// lane, one instruction moving eight rows of 128 bytes (64 input features): whole
// cache lines per instruction, each line touched by exactly one instruction
// (register-direct loads in MFMA operand order touch every line four times and
// run at a quarter of the rate).  The workgroup keeps one ring of NST stages in
// LDS; a stage holds 64 input features of each wave's 32*NT weight rows (fetched
// and read by that wave alone) and of the 32*MT query rows, which all four waves
// read and each fetches a quarter of (fetched once per wave they cost three
// times the weights' bytes in L2 traffic).  One barrier per stage; NST - 1
// stages stay in flight.  The LDS side of such a load is linear in the lane, so
// each lane fetches the 16-byte chunk whose swizzled home is its slot (chunk
// index XOR row mod 8: the operand reads, 32 rows at one chunk index, spread
// over the banks).  Operand reads are 16 bytes per lane: lane (r, h) takes
// chunks 4h .. 4h + 3 of row r for the four MFMA steps of a stage; both
// operands use the same assignment of input features to contraction slots.
//
// The input features of a group can be cut into KSPLIT ranges (and, for the
// output projection, the groups themselves are ranges of one long sum): each
// (group, range) is one grid.z slice that leaves an fp32 partial [m][n] in the
// workspace, summed by proj_reduce_kernel.  Without a cut the result is
// written directly.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"
#include "tuned_device.hpp"

namespace gla {

typedef __attribute__((ext_vector_type(8))) __bf16 proj_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float proj_f32x16_t;
typedef __attribute__((ext_vector_type(4))) float proj_f32x4_t;

struct ProjParams {
  const uint16_t* a;
  const uint16_t* w;
  void* c;
  float* part;             // [z][M][N] fp32 partials (z = g * ksplit + s), used when direct == 0
  int64_t a_row, a_group;  // element strides of A
  int64_t c_row, c_group;  // element strides of C
  int32_t M, G, N, K;
  int32_t ksplit, k_per_split;
  int32_t sum_groups, c_fp32, direct;
};

template <int MT, int NT>
__global__ __launch_bounds__(256) void proj_kernel(ProjParams p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int n0 = blockIdx.x * (128 * NT) + wave * (32 * NT);  // (N is a multiple of 32: a block of 32 output features exists or does not)
  const int m0 = blockIdx.y * (32 * MT);
  const int g = (int)blockIdx.z / p.ksplit, ks = (int)blockIdx.z % p.ksplit;
  const int k_begin = ks * p.k_per_split;
  const int k_end = min(p.K, k_begin + p.k_per_split);

  // One ring of NST stages per workgroup; a stage holds, for 64 input features, the 32 weight rows of each
  // of the four waves (private to the wave) and the 32*MT query rows (shared: each wave fetches a quarter).
  // (NT = 1: three or four stages, 72-80 KB: two workgroups per compute unit, one streaming while the other
  // starts up or stores.  NT = 2: three stages of up to 40 KB, one workgroup per compute unit; the host
  // then launches about one workgroup per compute unit.  Two and four stages measured 5 % and 1 % slower.)
  constexpr int NST = NT > 1 ? 3 : (MT == 1 ? 4 : 3);
  constexpr int kStage = (4 * NT + MT) * 4096;
  constexpr int kAOff = 4 * NT * 4096;  // the query rows follow the weights in a stage
  __shared__ __attribute__((aligned(1024))) unsigned char smem[NST * kStage];
  static_assert(sizeof(smem) <= 160 * 1024, "LDS capacity");
  const unsigned smem_addr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // load side: lane l of an instruction moves row l / 8 of its block of 8 rows; its LDS slot l % 8 is home to
  // chunk (l % 8) ^ (row % 8)
  const int lr = lane >> 3, lc = (lane & 7) ^ (lane >> 3);
  const unsigned char* wsrc[4 * NT];
  const unsigned char* asrc[MT];
#pragma unroll
  for (int j = 0; j < 4 * NT; ++j)  // (waves past the last output feature fetch the last rows again and store nothing)
    wsrc[j] = (const unsigned char*)(p.w + ((int64_t)g * p.N + min(n0 + 8 * j + lr, p.N - 1)) * p.K) + lc * 16;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {  // query rows 32 * mt + 8 * wave .. + 7 (rows past the end repeat the last one)
    const int m = min(m0 + mt * 32 + 8 * wave + lr, p.M - 1);
    asrc[mt] = (const unsigned char*)(p.a + m * p.a_row + g * p.a_group) + lc * 16;
  }
  auto issue = [&](int k, int stage) {  // 4 * NT + MT loads
    unsigned char* dst = smem + stage * kStage;
#pragma unroll
    for (int j = 0; j < 4 * NT; ++j)
      __builtin_amdgcn_global_load_lds((global_cvoid_t*)(wsrc[j] + (int64_t)k * 2), (lds_void_t*)(dst + wave * (NT * 4096) + j * 1024), 16, 0, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      __builtin_amdgcn_global_load_lds((global_cvoid_t*)(asrc[mt] + (int64_t)k * 2), (lds_void_t*)(dst + kAOff + mt * 4096 + wave * 1024), 16, 0, 0);
  };
  // operand side: row r, chunk 4h + s at slot (4h + s) ^ (r % 8)
  unsigned rd[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) rd[s] = smem_addr + (unsigned)(r * 128 + (((4 * h + s) ^ (r & 7)) << 4));
  const unsigned w_off = (unsigned)wave * (unsigned)(NT * 4096);

  proj_f32x16_t acc[NT][MT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nt][mt][i] = 0.f;

  constexpr int LPS = 4 * NT + MT;  // loads per wave and stage
  static_assert(LPS * (NST - 2) <= 63, "vmcnt range");
  const int k_last = k_end - 64;
#pragma unroll
  for (int st = 0; st < NST - 1; ++st) issue(min(k_begin + 64 * st, k_last), st);  // (steps past the end fetch the last one again)
  for (int k = k_begin; k < k_end; k += 64 * NST) {
    static_for<0, NST>([&](auto stc) {
      constexpr int st = decltype(stc)::value;
      if (k + 64 * st < k_end) {  // (uniform over the workgroup)
        // this wave's part of stage st has landed (the NST - 2 stages behind it may be in flight); after the
        // barrier so has everybody's, and everybody is done reading the stage before it, which is loaded next
        wait_vmcnt<LPS * (NST - 2)>();
        bare_barrier();
        issue(min(k + 64 * (st + NST - 1), k_last), (st + NST - 1) % NST);
        u32x4_t wf[NT][4], af[MT][4];
        static_for<0, 4>([&](auto sc) {
          constexpr int s = decltype(sc)::value;
          // (the stage offset goes into the address register: the instruction's offset field has 16 bits)
          static_for<0, NT>([&](auto nc) {
            lds_read_b128<decltype(nc)::value * 4096>(wf[decltype(nc)::value][s], rd[s] + (w_off + (unsigned)(st * kStage)));
          });
          static_for<0, MT>([&](auto mc) {
            lds_read_b128<kAOff + decltype(mc)::value * 4096>(af[decltype(mc)::value][s], rd[s] + (unsigned)(st * kStage));
          });
        });
        static_for<0, 4>([&](auto sc) {
          constexpr int s = decltype(sc)::value;
          constexpr int left = (3 - s) * (NT + MT);  // reads of later steps may still be in flight
          lds_wait<left>(wf[0][s]);
          static_for<0, NT>([&](auto nc) {
            constexpr int nt = decltype(nc)::value;
            asm volatile("" : "+v"(wf[nt][s]));  // (covered by the wait above: LDS returns in order)
            static_for<0, MT>([&](auto mc) {
              constexpr int mt = decltype(mc)::value;
              asm volatile("" : "+v"(af[mt][s]));
              acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(proj_bf16x8_t, wf[nt][s]),
                                                                     __builtin_bit_cast(proj_bf16x8_t, af[mt][s]), acc[nt][mt], 0, 0, 0);
            });
          });
        });
      }
    });
  }

  wait_vmcnt<0>();  // (re-fetched steps past the end of the range: let them land before the wave leaves)
  // accumulator element i of lane (r, h): output feature n0 + 32 * nt + 8 * (i / 4) + 4 * h + i % 4, query row m0 + 32 * mt + r
#pragma unroll
  for (int nm = 0; nm < NT * MT; ++nm) {
    const int nt = nm / MT, mt = nm % MT;
    const int m = m0 + mt * 32 + r;
    if (m >= p.M || n0 + 32 * nt >= p.N) continue;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int n = n0 + 32 * nt + 8 * q4 + 4 * h;
      const proj_f32x4_t v = {acc[nt][mt][4 * q4], acc[nt][mt][4 * q4 + 1], acc[nt][mt][4 * q4 + 2], acc[nt][mt][4 * q4 + 3]};
      if (!p.direct) {
        *reinterpret_cast<proj_f32x4_t*>(p.part + ((int64_t)blockIdx.z * p.M + m) * p.N + n) = v;
      } else {
        const int64_t off = m * p.c_row + (p.sum_groups ? 0 : g * p.c_group) + n;
        if (p.c_fp32) {
          *reinterpret_cast<proj_f32x4_t*>((float*)p.c + off) = v;
        } else {
          uint2 pk;
          pk.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
          pk.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
          *reinterpret_cast<uint2*>((uint16_t*)p.c + off) = pk;
        }
      }
    }
  }
}

// Sum of the partials of one output: over all grid.z slices (output projection)
// or over the ksplit slices of each group (absorbed query).  One thread per four
// consecutive output features, slices added in index order (deterministic).
__global__ __launch_bounds__(256) void proj_reduce_kernel(ProjParams p) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int n4 = p.N / 4;
  const int outs = p.sum_groups ? 1 : p.G;
  if (idx >= (int64_t)p.M * outs * n4) return;
  const int n = (int)(idx % n4) * 4;
  const int g = (int)((idx / n4) % outs);
  const int m = (int)(idx / ((int64_t)n4 * outs));
  const int z0 = p.sum_groups ? 0 : g * p.ksplit, z1 = p.sum_groups ? p.G * p.ksplit : (g + 1) * p.ksplit;
  proj_f32x4_t v = {0.f, 0.f, 0.f, 0.f};
  const float* src = p.part + ((int64_t)z0 * p.M + m) * p.N + n;
  const int64_t step = (int64_t)p.M * p.N;
  int z = z0;
  for (; z + 4 <= z1; z += 4, src += 4 * step) {  // four slices in flight, added in index order
    const proj_f32x4_t a0 = *reinterpret_cast<const proj_f32x4_t*>(src);
    const proj_f32x4_t a1 = *reinterpret_cast<const proj_f32x4_t*>(src + step);
    const proj_f32x4_t a2 = *reinterpret_cast<const proj_f32x4_t*>(src + 2 * step);
    const proj_f32x4_t a3 = *reinterpret_cast<const proj_f32x4_t*>(src + 3 * step);
    v = (((v + a0) + a1) + a2) + a3;
  }
  for (; z < z1; ++z, src += step) v += *reinterpret_cast<const proj_f32x4_t*>(src);
  const int64_t off = m * p.c_row + (p.sum_groups ? 0 : g * p.c_group) + n;
  if (p.c_fp32) {
    *reinterpret_cast<proj_f32x4_t*>((float*)p.c + off) = v;
  } else {
    uint2 pk;
    pk.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
    pk.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
    *reinterpret_cast<uint2*>((uint16_t*)p.c + off) = pk;
  }
}

}  // namespace gla
