/*
 * gla_decode.h — C ABI of the MI355X (gfx950) decode-attention library for
 * Grouped Latent Attention (GLA) and Grouped-Tied Attention (GTA).
 *
 * Operation (paper Sections 2.1, 3.3.1, 3.3.2).  For every sequence b, query
 * row t in [0, q_len) and query head h (group g = h / (num_q_heads/num_groups),
 * heads of a group are a contiguous block):
 *
 *     s_j  = softmax_scale * ( q_nope[b,t,h,:d_nope] . state[b,j,g,:d_nope]
 *                            + q_rope[b,t,h,:]       . rope[b,j,:] )
 *     lse  = ln sum_j exp(s_j)                          over the visible keys j
 *     out  = sum_j exp(s_j - lse) * state[b,j,g,:d_v]
 *
 * i.e. attention in the weight-absorbed form: each group's queries score
 * directly against that group's cached state (latent head c_g for GLA, tied KV
 * head for GTA) plus ONE decoupled-RoPE key per token shared by all heads, and
 * the same cached state is the value, so the output stays in the state's space.
 *   gla_decode: d_nope == d_v (GLA; num_groups == 1 is the MLA shape).
 *   gta_decode: d_nope == d_v / 2 (the key reuses only the first half of the
 *               tied state; the RoPE half comes from the shared key).
 * Visible keys: j < L_b - q_len + 1 + t when causal (the q_len queries are the
 * last q_len cached positions, as in linear-chain speculative decoding), else
 * j < L_b, with L_b = seq_lens[b].  A row with no visible key gets out = 0 and
 * lse = -inf.
 *
 * The cache is paged: token j of sequence b lives in physical page
 * page_table[b][j / page_size] at slot j % page_size.  Table entries at or
 * beyond ceil(L_b / page_size) are never used as page ids (they may hold
 * anything, -1 included; a kernel may load them along with their row); slots at or beyond L_b inside a page the table does hold may be
 * fetched but never reach a result, whatever they contain (NaN included).
 * The main MFMA kernel runs for every power-of-two page_size from 64 down to 1
 * (paper Section 4.2 for the small ones), state dims (d_v, d_nope) = (256, 256),
 * (512, 512), (128, 64) and RoPE dims 64, 48 or 32.  A second, simpler MFMA
 * kernel covers GTA states of 64 and 96 dims (RoPE key d_v / 2), latent heads of
 * 128 dims with a RoPE key of 32, and gqa_decode, at any power-of-two
 * page_size.  Everything else takes the generic kernel.  GLA_IMPL_TUNED means
 * "one of the MFMA kernels".
 *
 * Ownership and execution.  Every pointer in the struct is a DEVICE pointer
 * owned by the caller unless stated otherwise; the library allocates no device
 * memory, never synchronises the device and never blocks: it enqueues a few
 * kernels on `stream` and returns.  Intermediate results (partial outputs of
 * the split over the key axis) go to the caller's `workspace`.  All functions
 * are thread-safe for distinct streams and workspaces.
 *
 * Errors.  Functions return GLA_OK (0) or a negative GLA_ERR_* code; nothing
 * is enqueued when an error is returned.  Only host-visible fields can be
 * validated; device contents (page ids, lengths) are trusted.
 */
#ifndef GLA_DECODE_H_
#define GLA_DECODE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  GLA_OK = 0,
  GLA_ERR_INVALID_ARG = -1,        /* null pointer, bad count, h_q % h_c != 0, q_len outside 1..4 ... */
  GLA_ERR_UNSUPPORTED_SHAPE = -2,  /* valid problem, but no kernel for it (see `impl`)               */
  GLA_ERR_WORKSPACE_TOO_SMALL = -3,
  GLA_ERR_LAUNCH = -4              /* the HIP runtime refused a launch                                */
};

enum {
  GLA_IMPL_AUTO = 0,     /* tuned MFMA kernel when the shape has one, else the generic kernel */
  GLA_IMPL_GENERIC = 1,  /* shape-agnostic scalar kernel (any dims, any page size)            */
  GLA_IMPL_TUNED = 2     /* tuned kernel or GLA_ERR_UNSUPPORTED_SHAPE                          */
};

enum { GLA_OUT_BF16 = 0, GLA_OUT_FP32 = 1 };

typedef struct gla_decode_params {
  int32_t batch;              /* B >= 0                                                        */
  int32_t q_len;              /* T in 1..4                                                     */
  int32_t num_q_heads;        /* h_q                                                           */
  int32_t num_groups;         /* h_c (GLA latent heads / GTA tied KV heads); divides h_q       */
  int32_t d_v;                /* state dim used as value (GLA: d_c, GTA: d_h)                  */
  int32_t d_nope;             /* leading state dims used in the score                          */
  int32_t d_rope;             /* shared RoPE key dim (0 allowed on the generic kernel)         */
  int32_t page_size;          /* tokens per page                                               */
  int32_t max_pages_per_seq;  /* row length of page_table                                      */
  int32_t causal;             /* 1: row t sees j <= L_b - q_len + t ; 0: every j < L_b         */
  int64_t num_pages;          /* pool size (used for argument checks only)                     */

  /* Strides are in ELEMENTS; the last dimension is always contiguous. */
  const void* q_nope;         /* bf16 [B, T, h_q, d_nope]                                      */
  int64_t q_nope_stride[3];   /* strides of (b, t, h)                                          */
  const void* q_rope;         /* bf16 [B, T, h_q, d_rope]                                      */
  int64_t q_rope_stride[3];
  const void* state_cache;    /* bf16 [num_pages, h_c, page_size, d_v]                         */
  int64_t state_stride[3];    /* strides of (page, group, token)                               */
  const void* rope_cache;     /* bf16 [num_pages, page_size, d_rope]                           */
  int64_t rope_stride[2];     /* strides of (page, token)                                      */
  const int32_t* page_table;  /* int32 [B, max_pages_per_seq], row-major                       */
  const int32_t* seq_lens;    /* int32 [B]; cached tokens INCLUDING the q_len newest ones      */

  float softmax_scale;        /* multiplies the summed (nope + rope) score                     */
  int32_t out_dtype;          /* GLA_OUT_BF16 or GLA_OUT_FP32                                  */
  void* out;                  /* [B, T, h_q, d_v] of out_dtype                                 */
  int64_t out_stride[3];      /* strides of (b, t, h)                                          */
  float* lse;                 /* fp32 [B, T, h_q] contiguous; natural log                      */

  void* workspace;            /* >= gla_decode_workspace_size() bytes, 256-byte aligned        */
  size_t workspace_bytes;
  int32_t num_splits;         /* 0 = automatic.  n > 0: cut the key axis so that a sequence of
                                 max_pages_per_seq pages falls into about n chunks            */
  int32_t impl;               /* GLA_IMPL_*                                                    */
  void* stream;               /* hipStream_t (0 = the null stream)                             */
} gla_decode_params;

/* GLA / MLA-shape decode (Section 3.3.2).  Requires d_nope == d_v. */
int gla_decode(const gla_decode_params* p);

/* GTA decode (Section 3.3.1).  Requires d_nope == d_v / 2 (d_v even). */
int gta_decode(const gla_decode_params* p);

/* Grouped-query attention decode with keys and values in separate paged caches:
 * the baseline that Grouped-Tied Attention is compared with (Section 3.3.1: the
 * tied state stands in for a GQA group's key and value, about half the cache
 * bytes per token).  Same parameter block with these readings: state_cache is
 * the VALUE cache [num_pages, h_kv, page_size, d_v] (num_groups = h_kv);
 * key_cache is bf16 [num_pages, h_kv, page_size, d_nope] with element strides
 * key_stride (page, head, token), last dim contiguous; q_nope holds the whole
 * query [B, T, h_q, d_nope] (rotary embedding already applied to it and to the
 * cached keys); d_rope must be 0, q_rope and rope_cache are ignored.
 *     s_j = softmax_scale * q . key[j],  out = softmax(s) . value
 * Visible keys, empty rows, paging, workspace and errors as for gla_decode
 * (workspace size: gla_decode_workspace_size(p, 2)).  An MFMA kernel runs for
 * head dims (d_nope, d_v) = (128, 128) and (64, 64) at any power-of-two
 * page_size; other shapes take the generic kernel. */
int gqa_decode(const gla_decode_params* p, const void* key_cache, const int64_t key_stride[3]);

/* For callers that cannot allocate device memory or obtain a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same operation as gla_decode (is_gta == 0) or gta_decode
 * (is_gta != 0), with the partial results of the split over the key axis kept
 * in a buffer of GLA_DECODE_NOALLOC_SCRATCH_BYTES that is part of the library
 * image, one per GPU, held from the library's load to the end of the process.
 * p->workspace and p->workspace_bytes are ignored; inputs and outputs are the
 * caller's as before.  The call allocates and frees nothing.  The buffer covers
 * every automatic plan (num_splits == 0) of the MFMA kernels; a problem that
 * needs more (large explicit num_splits, or the generic kernel on very many
 * rows) returns GLA_ERR_WORKSPACE_TOO_SMALL and enqueues nothing.  All calls on
 * one GPU share that GPU's buffer: calls that may overlap in time (different
 * streams, different threads) race on it and must be serialised by the caller.
 * The GPU the buffer belongs to is the one current at the call. */
#define GLA_DECODE_NOALLOC_SCRATCH_BYTES (72u << 20)
int gla_decode_noalloc(const gla_decode_params* p, int is_gta);

/* Bytes of workspace a call with these parameters needs (host only; pointer
 * fields are ignored).  is_gta: 0 for gla_decode, 1 for gta_decode, 2 for
 * gqa_decode (the helpers below take the same values; they have no passage of
 * the paper to cite: they describe this library's own kernels).  Returns 0 for
 * an invalid parameter set. */
size_t gla_decode_workspace_size(const gla_decode_params* p, int is_gta);

/* ---- the two projections around the attention -----------------------------------
 * Both compute, on bf16 operands with fp32 accumulation,
 *
 *     gla_absorb_query:  C[m][g][n] = sum_k A[m][g][k] * W[g][n][k]
 *     gla_output_proj:   C[m][n]    = sum_g sum_k A[m][g][k] * W[g][n][k]
 *
 * over the `rows` query rows m of a decode step (batch * q_len, flattened).
 *
 * gla_absorb_query (Section 2.1: the key up-projection W^UK absorbed on the query
 * side).  groups = query heads, k = d_h (raw head dim), n = d_c (latent dim):
 * A = raw non-RoPE queries [rows][h_q][d_h], W[g] = W^UK of head g stored
 * [d_c][d_h], C = the absorbed queries [rows][h_q][d_c] that gla_decode takes as
 * q_nope (q . (W^UK^T c) == (W^UK q) . c).  The RoPE part of the query is not
 * touched.
 *
 * gla_output_proj (Section 3.3.2: O~_g = O_g W_g^vo, summed over the groups; the
 * value up-projection W^UV is absorbed in W^vo).  groups = latent heads h_c,
 * k = g_q * d_c (the latent outputs of the group's heads side by side, which is
 * how gla_decode lays out `out`), n = model dim D: A = out [rows][h_c][g_q * d_c],
 * W[g] = W_g^vo stored output-major [D][g_q * d_c], C = [rows][D].  On several
 * devices each rank would run this on its own groups and all-reduce C.
 *
 * Weights are contiguous [groups][n][k] (k fastest).  All pointers are device
 * pointers, 16-byte aligned; strides in elements.  Needs k % 64 == 0,
 * n % 32 == 0, a strides % 8 == 0, c strides % 4 == 0 (else
 * GLA_ERR_UNSUPPORTED_SHAPE).  When the input features are cut into ranges
 * (always for gla_output_proj with more than one group) fp32 partial sums go to
 * `workspace` (gla_proj_workspace_size bytes, 256-byte aligned) and are added
 * in a fixed order by a second kernel: results are reproducible bit for bit.
 * Nothing is allocated, nothing synchronises. */
typedef struct gla_proj_params {
  int32_t rows;             /* M = batch * q_len                                              */
  int32_t groups;           /* G                                                              */
  int32_t n;                /* output features per group                                      */
  int32_t k;                /* input features per group                                       */
  const void* a;            /* bf16 A[m][g][k]                                                */
  int64_t a_row_stride;     /* elements between rows m                                        */
  int64_t a_group_stride;   /* elements between groups g                                      */
  const void* w;            /* bf16 W[g][n][k], contiguous                                    */
  void* c;                  /* c_dtype; absorb: C[m][g][n], output projection: C[m][n]        */
  int64_t c_row_stride;     /* elements between rows m                                        */
  int64_t c_group_stride;   /* elements between groups g (ignored by gla_output_proj)         */
  int32_t c_dtype;          /* GLA_OUT_BF16 or GLA_OUT_FP32                                   */
  void* workspace;
  size_t workspace_bytes;
  void* stream;             /* hipStream_t                                                    */
} gla_proj_params;

int gla_absorb_query(const gla_proj_params* p);
int gla_output_proj(const gla_proj_params* p);
/* Bytes of workspace (host only; pointer fields ignored); sum_groups = 0 for
 * gla_absorb_query, 1 for gla_output_proj.  0 for an invalid parameter set. */
size_t gla_proj_workspace_size(const gla_proj_params* p, int sum_groups);

/* Which implementation a call would run: GLA_IMPL_GENERIC or GLA_IMPL_TUNED,
 * or a negative error code.  Host only; pointer fields are ignored. */
int gla_decode_select_impl(const gla_decode_params* p, int is_gta);

/* Benchmark helper: enqueue `iters` calls (1..256) bracketed by HIP events on
 * p->stream, wait for them, and report the mean duration in microseconds of
 * the main (split-KV attention) kernel and of the combine kernel.  This call
 * DOES synchronise the stream.  Host pointers for the two results. */
int gla_decode_profile(const gla_decode_params* p, int is_gta, int iters, float* main_us,
                       float* combine_us);

/* Debug helper for callers that build page tables themselves: checks the
 * device contents the decode calls trust (they are not checked there, and a
 * bad page id makes a decode call read outside the pools).  Counts, into the
 * host int *n_bad, the sequences whose length is outside
 * [0, max_pages_per_seq * page_size] and the page-table entries a sequence
 * holds (the first ceil(L_b / page_size) of its row) that are outside
 * [0, num_pages).  Needs num_pages > 0 and 256 bytes of workspace (whose first
 * bytes it overwrites); enqueues one small kernel on p->stream and DOES
 * synchronise the stream.  Returns GLA_OK when the check itself ran. */
int gla_decode_check_contents(const gla_decode_params* p, int is_gta, int* n_bad);

/* Static, NUL-terminated description of a status code. */
const char* gla_status_string(int status);

/* ABI version (major * 100 + minor). */
int gla_decode_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GLA_DECODE_H_ */
