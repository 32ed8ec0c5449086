/*
 * sinkrouter.h - C ABI of the MI355X (gfx950) SinkRouter decode-attention library.
 *
 * One decode step of one attention layer: a single query token per sequence attends
 * over a long bf16 grouped-query KV cache.  Before any cache row beyond token 0 is
 * read, each KV group is classified from the cosine between its query heads and the
 * cached key of token 0; Sink Groups are written as zeros and their K/V are never
 * loaded, Active Groups get exact softmax attention computed Split-K over the
 * sequence and merged by log-sum-exp (paper Sections 4.2 and 4.3).
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory on the current device, "host" pointers
 *     are ordinary host memory.  The caller owns every buffer; the library allocates
 *     no device memory and keeps no state between calls (sinkrouter_decode_static alone
 *     works on a device array that belongs to the library, see there).
 *   - bf16 tensors are raw 16-bit patterns, row-major, innermost dimension D, and must
 *     be 16-byte aligned.
 *   - Calls are asynchronous on params->stream and never synchronise (except the
 *     *_profiled variant, which says so).  Buffers must stay alive until the stream
 *     has passed the call.  Inputs are never written; outputs are fully overwritten.
 *   - Every argument check runs on the host before the first HIP call, so error paths
 *     need no GPU.  Return value: SR_OK (0) or a negative sr_status.
 *   - No C++ exception crosses this boundary.  Concurrent calls are safe when they use
 *     distinct workspaces and outputs.
 */
#ifndef SINKROUTER_H
#define SINKROUTER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sr_status {
  SR_OK = 0,
  SR_ERR_NULL = -1,        /* a required pointer is NULL */
  SR_ERR_SHAPE = -2,       /* sizes are non-positive, inconsistent or overflow */
  SR_ERR_UNSUPPORTED = -3, /* head_dim != 128, group size > 16, kv_block != 64, bad struct_size */
  SR_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or smaller than required */
  SR_ERR_ALIGN = -5,       /* a tensor pointer is not 16-byte aligned */
  SR_ERR_HIP = -6,         /* the HIP runtime reported an error (launch, event, ...) */
  SR_ERR_STATIC_LIMIT = -7 /* sinkrouter_decode_static: the shape needs more than the static scratch */
} sr_status;

/*
 * Shape, routing rule and launch resources of one call.  Plain data, host memory.
 *
 * Routing rule (Section 4.2): for KV group g of sequence b with r = n_q_heads / n_kv_heads
 * query heads, s_i = cos(q_{g,i}, K_0) (Eq. 11), S_g = mean_i s_i (Eq. 12), and the group is a
 * Sink Group iff S_g > tau(L_b), strictly (Eq. 13), with the length-dependent threshold
 * tau(x) = a x^3 + b x^2 + c x + d of Appendix A evaluated at x = seq_lens[b] / len_norm.
 * The paper prints neither the coefficients nor the normalisation, so both are inputs; a
 * fixed threshold t is {0,0,0,t} (the paper's operating point is 0.55).  K_0 is row 0 of the
 * group's key cache.  A cosine whose denominator is not a positive number (a zero or NaN norm) is
 * 0; a NaN score (NaN anchor with a finite cached norm) leaves the group active.  A cached norm
 * that is negative or NaN counts as not cached and is recomputed from the anchor.
 */
typedef struct sr_route_params {
  uint32_t struct_size;     /* sizeof(sr_route_params); anything else -> SR_ERR_UNSUPPORTED */
  int32_t batch;            /* B >= 1 */
  int32_t n_q_heads;        /* H_q, a multiple of n_kv_heads; H_q / H_kv <= 16 */
  int32_t n_kv_heads;       /* H_kv >= 1 */
  int32_t head_dim;         /* D; only 128 is built */
  int32_t max_seq_len;      /* L_max >= 1: token stride of both caches */
  int32_t kv_block;         /* B_K, tokens per online-softmax block; only 64 is built */
  int32_t num_splits;       /* Split-K chunks per sequence; 0 = balanced schedule (sinkrouter_plan) */
  int32_t routing_enabled;  /* 0 = every group active (dense Split-K; the paper routes no
                               group in its first two layers, Appendix B) */
  float sm_scale;           /* softmax scale; 0 = 1/sqrt(D) */
  float tau_coef[4];        /* a, b, c, d */
  float len_norm;           /* x = seq_len / len_norm; <= 0 means x = 0 */
  const float* k0_norm;     /* device, optional [B,H_kv]: ||K_0||_2 cached at prefill
                               (Section 4.1, Eq. 7); NULL = recompute from the anchor */
  const void* k0;           /* device, optional bf16 [B,H_kv,D]: the token-0 keys kept apart from
                               the cache (the K_0 tensor of Section 4.3); NULL = row 0 of k_cache */
  void* workspace;          /* device, 256-byte aligned, >= sinkrouter_workspace_bytes() */
  size_t workspace_bytes;
  void* stream;             /* hipStream_t; NULL = the default stream */
} sr_route_params;

/* The launch plan the library derives from the shape (host only, no GPU). */
typedef struct sr_plan {
  int32_t schedule;         /* 1 = balanced, 0 = fixed chunks (see sinkrouter_plan) */
  int32_t chunk_tokens;     /* fixed: tokens per Split-K chunk (multiple of 256); balanced: 0 */
  int32_t num_splits;       /* fixed: ceil(max_seq_len / chunk_tokens); balanced: 0 */
  int32_t group_size;       /* r = H_q / H_kv */
  int32_t partial_grid;     /* workgroups of the Split-K partial kernel */
  int32_t slots_per_head;   /* partial (m, l, o) records reserved per query head */
  size_t workspace_bytes;
} sr_plan;

/*
 * Fills *plan for params (workspace fields of params are ignored).  Split-K of Section 4.3:
 * the tokens of a sequence are cut into chunks, each chunk yields a partial result per head,
 * and the partials are merged.  Two schedules:
 *   params->num_splits > 0  "fixed": [0, L_max) is cut into num_splits equal chunks (rounded up
 *                           to 256 tokens), one workgroup per (chunk, sequence, KV group), as
 *                           the paper states it; workgroups of Sink Groups exit immediately.
 *   params->num_splits == 0 "balanced": the 64-token blocks of the Active Groups only are dealt
 *                           out to one workgroup per compute unit (256), on the device, once
 *                           the skip decisions are known: every Active Group gets workgroups
 *                           in proportion to its blocks (or, with more than 128 Active
 *                           Groups, or where that would leave a quarter of the workgroups
 *                           idle, every workgroup an equal run of the blocks laid end to
 *                           end), so the chunk length adapts to the skip pattern.
 *                           Needs B*H_kv <= 2048; larger batches fall back to fixed chunks.
 * The result does not depend on the schedule beyond fp32 rounding.
 */
int sinkrouter_plan(const sr_route_params* params /*host*/, sr_plan* plan /*host*/);

/* Bytes of device workspace sinkrouter_decode needs for params (0 if params are invalid). */
size_t sinkrouter_workspace_bytes(const sr_route_params* params /*host*/);

/*
 * One routed decode step (Sections 4.2-4.3; Eq. 1 for Active Groups, Eq. 14 for Sink Groups).
 *   q             device bf16 [B,H_q,D]; head h belongs to KV group h / r (the paper's
 *                 [B,H_kv,G,D] layout, same memory)
 *   k_cache       device bf16 [B,H_kv,L_max,D]
 *   v_cache       device bf16 [B,H_kv,L_max,D]
 *   seq_lens      device int32 [B]: valid rows per sequence, current token included;
 *                 values outside [0,L_max] are clamped on the device.  Rows at or beyond
 *                 seq_lens[b] are never read, with one exception: row 0 of every (sequence,
 *                 KV group) key cache is always read by the routing probe (unless params->k0
 *                 supplies the anchors), also for an empty sequence, whose result is then
 *                 discarded; the caches must therefore hold at least one row.
 *   params        host
 *   out           device bf16 [B,H_q,D]: softmax(scale q K^T) V for heads of Active Groups
 *                 (fp32 accumulation, rounded to nearest even), exact zeros for heads of
 *                 Sink Groups and for sequences of length 0
 *   skip_mask_out device uint8 [B,H_kv]: 1 = Sink Group (skipped), 0 = Active Group
 * Enqueued on params->stream: the Split-K partial kernel, which evaluates the routing rule itself
 * (a separate routing-probe kernel precedes it for routed batches of more than 256 query heads
 * or with fixed chunks), then the merge kernel.  Nothing is allocated, no memset is recorded and nothing
 * synchronises, so the call can be captured into a HIP graph.
 */
int sinkrouter_decode(const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* seq_lens, const sr_route_params* params,
                      void* out, uint8_t* skip_mask_out);

/*
 * The routing decision alone (Section 4.2, Eq. 11-13): reads q and row 0 of k_cache only.
 *   group_score_out device fp32 [B,H_kv], optional: S_g
 *   skip_mask_out   device uint8 [B,H_kv]
 * Needs no workspace.
 */
int sinkrouter_probe(const void* q, const void* k_cache, const int32_t* seq_lens,
                     const sr_route_params* params, float* group_score_out,
                     uint8_t* skip_mask_out);

/*
 * sinkrouter_decode with per-kernel timing, for benchmarks.  The call SYNCHRONISES params->stream
 * before returning.  stage_us (host, 4 floats), in microseconds:
 *   [0] the separate routing-probe kernel (0 when the probe is fused into the partial kernel),
 *   [1] the Split-K partial kernel, [2] the merge kernel: each from the begin to the end of the
 *       kernel's own execution, taken from HIP events attached to the launch (the times a
 *       profiler's kernel trace shows);
 *   [3] the whole call, between two events recorded on the stream before the first and after the
 *       last launch, dispatch latencies included.
 */
int sinkrouter_decode_profiled(const void* q, const void* k_cache, const void* v_cache,
                               const int32_t* seq_lens, const sr_route_params* params,
                               void* out, uint8_t* skip_mask_out, float* stage_us);

/*
 * sinkrouter_decode with two per-head diagnostics of the attention it computed (at least one of
 * the two pointers non-NULL):
 *   lse_out    device fp32 [B,H_q]: natural-log sum-exp of the scaled scores
 *   alpha0_out device fp32 [B,H_q]: softmax mass on token 0, the quantity whose exceeding gamma
 *              defines the target regime the routing signal stands in for (Section 4.2, first
 *              paragraph; Appendix C measures the proxy against it)
 * Heads of Sink Groups are not computed: both are NaN there (run with routing_enabled = 0 to get
 * them for every head).  An empty sequence gives lse = -inf, alpha0 = NaN.
 */
int sinkrouter_decode_diag(const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* seq_lens, const sr_route_params* params,
                           void* out, uint8_t* skip_mask_out, float* lse_out, float* alpha0_out);

/*
 * Attention-concentration statistics per head, the quantities of Table 1 (Section 3): with alpha the
 * softmax weights of the scaled scores over the whole cache (Eq. 1),
 *   alpha0_out    device fp32 [B,H_q]: alpha_0, the weight of token 0
 *   max_rest_out  device fp32 [B,H_q]: the largest weight among tokens 1..L-1
 *   mean_rest_out device fp32 [B,H_q]: the mean weight of tokens 1..L-1
 *   out_rest      device bf16 [B,H_q,D]: the head update with token 0 left out and the other
 *                 weights renormalised (what the head would write without its sink token)
 * (the table's Ratio is alpha0 / max_rest).  Every head is measured: routing_enabled, k0 and
 * k0_norm of params are ignored and skip_mask_out [B,H_kv] is written as zeros.  One pass over
 * tokens 1..L-1 with the decode kernels; token 0 is folded in by the merge.  A one-token cache
 * gives alpha0 = 1, max = mean = 0, out_rest = 0; an empty one gives NaN statistics, out_rest = 0.
 * Contiguous caches only.  Same workspace, stream and error conventions as sinkrouter_decode.
 */
int sinkrouter_concentration(const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* seq_lens, const sr_route_params* params,
                             void* out_rest, uint8_t* skip_mask_out,
                             float* alpha0_out, float* max_rest_out, float* mean_rest_out);

/*
 * Paged KV cache (serving layout; the paper's kernel takes contiguous caches, Section 4.3).
 * Pages hold page_tokens tokens, a power of two >= 64, so a 64-token block never straddles a
 * page; the pools are laid out [n_pages, H_kv, page_tokens, D] bf16.
 */
typedef struct sr_paged_layout {
  uint32_t struct_size;     /* sizeof(sr_paged_layout) */
  int32_t page_tokens;      /* tokens per page: 64, 128, 256, ... */
  int32_t pages_per_seq;    /* row stride of block_table; pages_per_seq * page_tokens >= max_seq_len */
  int32_t n_pages;          /* pages in the pools; table entries are clamped to [0, n_pages) on the device */
} sr_paged_layout;

/*
 * sinkrouter_decode over a paged cache: identical result to sinkrouter_decode on the cache that
 * gathering the pages would give.
 *   k_pages, v_pages device bf16 [n_pages,H_kv,page_tokens,D]
 *   block_table      device int32 [B,pages_per_seq]: physical page of each logical page; only
 *                    entries below ceil(seq_lens[b] / page_tokens) are read, and entry 0 of
 *                    every sequence (the anchor's page; for an empty sequence any value will
 *                    do, it is clamped to the pool like every entry)
 * params->max_seq_len bounds the sequence lengths (they are clamped to it); params->k0 and
 * params->k0_norm work as for the contiguous entry point.  Token 0 is the first token of the
 * page block_table[b][0].
 */
int sinkrouter_decode_paged(const void* q, const void* k_pages, const void* v_pages,
                            const int32_t* block_table, const int32_t* seq_lens,
                            const sr_route_params* params, const sr_paged_layout* layout,
                            void* out, uint8_t* skip_mask_out);

/*
 * sinkrouter_decode for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, schedule and result (bit for bit) as sinkrouter_decode, except that
 * params->workspace and params->workspace_bytes are ignored: the partial records live in a device
 * array of SINKROUTER_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU
 * the library runs on holds it until the process ends).  The call allocates and frees nothing; the
 * array's address is looked up on the first call on each device, so make that first call outside
 * stream capture.  A shape whose
 * sinkrouter_plan().workspace_bytes exceeds SINKROUTER_STATIC_SCRATCH_BYTES returns
 * SR_ERR_STATIC_LIMIT (checked on the host, before any HIP call); all five benchmark shapes fit.
 * Nothing in the array has to start at zero (every record is written before it is read), so
 * nothing is cleared.  All calls on one GPU share the array: calls that overlap on one GPU (other
 * streams, other threads) race; calls on one stream are ordered and safe.
 */
#define SINKROUTER_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int sinkrouter_decode_static(const void* q, const void* k_cache, const void* v_cache,
                             const int32_t* seq_lens, const sr_route_params* params,
                             void* out, uint8_t* skip_mask_out);

/*
 * Prefill-side anchor caching (Section 4.1): copies row 0 of every (sequence, KV group) key cache
 * to k0_out (device bf16 [B,H_kv,D], optional) and writes its Euclidean norm to k0_norm_out
 * (device fp32 [B,H_kv], optional); at least one must be given.  The norm is computed exactly as
 * the probe recomputes it, so passing these back through params->k0 / params->k0_norm leaves
 * every routing decision unchanged.  Uses params for the shape and the stream only.
 */
int sinkrouter_extract_anchor(const void* k_cache, const sr_route_params* params,
                              void* k0_out, float* k0_norm_out);

/*
 * Measurement helpers (no part of the method): a streaming read of `bytes` bytes of device
 * memory (128-bit loads, every byte read once, one 4-byte result per workgroup written to
 * sink, which must hold at least 4096 bytes), and a plain device-to-device copy kernel of
 * known traffic used to calibrate hardware byte counters.  bytes must be a multiple of 16
 * and the pointers 16-byte aligned.
 */
int sinkrouter_hbm_read_probe(const void* buf, size_t bytes, void* sink, void* stream);
int sinkrouter_hbm_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/*
 * 0 in the product build.  The measurement variant of the library (built with -DSR_TIMELINE=1, used
 * only by the benchmark's per-phase accounting) appends this many bytes of per-workgroup wall-clock
 * stamps to the workspace, already included in sinkrouter_workspace_bytes().
 */
size_t sinkrouter_timeline_bytes(void);

/* Static, human-readable text for a status code. */
const char* sinkrouter_status_string(int status);

/* ABI version of this header: bumped on any incompatible change. */
int sinkrouter_abi_version(void);
#define SINKROUTER_ABI_VERSION 2

#ifdef __cplusplus
}
#endif
#endif /* SINKROUTER_H */
