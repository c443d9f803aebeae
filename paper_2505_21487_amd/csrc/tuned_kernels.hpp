// Tuned decode-attention path for gfx950: split-KV main kernel on bf16 MFMA
// with LDS-staged page tiles, plus the merge kernel for its partial results.
//
// Work decomposition.  A workgroup has NG * WPG * KS waves: it serves NG groups
// (latent heads / tied KV heads) at once with WPG slabs of 32 query rows per
// group, so that the RoPE-key tile, which all groups share, is fetched once
// for all of them; KS = 2 waves share a slab when the state has 512 dims (each
// takes half of the dims, see the score exchange below).  The g_q * T query
// rows of a group (ordered t-major) are cut into row blocks of 32 * WPG rows,
// the h_c groups into blocks of NG.  A "unit" of the work list is (sequence b,
// group block gb): it owns ceil(L_b / TOK) key tiles of TOK = 32 tokens (half
// a page, a page, two pages ... 32 pages for page sizes 64, 32, 16 ... 1; the
// address code comes in four forms, see the page modes of the main kernel);
// a tile is the NG state tiles of its groups plus one RoPE tile.  All tiles of all units, in
// unit order, form one flat list that is cut into equal chunks, so ragged
// batches balance by construction and at most two units per chunk are left
// incomplete.  A chunk is worked on by one workgroup per row block.  A (unit,
// row block) that lies inside one chunk is written straight to the output; one
// that spans chunks leaves one partial (normalised fp32 output + log-sum-exp)
// per chunk in the workspace, merged by tuned_combine_kernel.
//
// Inside a workgroup every wave owns 32 query rows and works in the transposed
// form: S^T = K . Q^T with the key tile as the MFMA A operand (from LDS) and
// the query fragments as B operand (registers, loaded once per unit), then
// O^T += V^T . P^T where P^T comes straight from the S^T accumulators (the
// accumulator layout of a 32x32 MFMA already is a valid B-operand layout for a
// suitable order of the contraction index) and V^T is read from the SAME LDS
// tile with transposing LDS reads.  Row max / row sum therefore live in one
// lane plus its partner lane (lane ^ 32): no cross-wave softmax traffic.
//
// Tiles travel HBM -> LDS with direct-to-LDS loads through a STAGES-deep ring;
// the only waits on them are explicit vmcnt counts, and all operand reads from
// LDS are issued by hand (inline asm) a few MFMAs ahead of their use.
//
// The operation itself is the absorbed-form attention of the paper (Sections
// 2.1, 3.3.1, 3.3.2): score = scale * (q_nope . state[:DN] + q_rope . rope_key),
// softmax over the visible keys, output = weights . state[:DV].
//
// Files: tuned_device.hpp (device helpers), tuned_main_kernel.hpp, tuned_combine_kernel.hpp,
// tuned_host.hpp (plan and launches).
#pragma once

#include "tuned_device.hpp"
#include "tuned_main_kernel.hpp"
#include "tuned_combine_kernel.hpp"
#include "tuned_host.hpp"
