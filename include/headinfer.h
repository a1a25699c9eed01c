/*
 * headinfer.h - C ABI of the head-wise offloaded attention library for AMD MI355X (gfx950).
 *
 * The library computes exact causal grouped-query attention ONE KV HEAD AT A TIME, with that head's K/V
 * history streamed between a pinned host-DRAM cache and a small HBM staging ring (HeadInfer, arXiv 2502.12574:
 * Section 3.2 "Head-wise Offload", Section 4, Algorithm 1).  Every pointer below is either "host" or "device"
 * as stated; no framework types cross this boundary.  All functions return an hi_status (0 = success,
 * negative = error), never throw, never abort and never print.
 *
 * Notation (the paper's): L layers, H KV heads per layer, G query heads per KV head (grouped-query sharing),
 * D_h head dimension, S context length, C chunk length, P past length (rows already cached when a call starts).
 * Element type is bf16 (2 bytes); one token of one KV head is 2 * D_h * 2 = 512 bytes of K plus V.
 */
#ifndef HEADINFER_H
#define HEADINFER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t hi_status;
enum {
  HI_OK = 0,
  HI_ERR_ARG = -1,         /* null pointer, negative size, layer/head out of range, misaligned pointer      */
  HI_ERR_UNSUPPORTED = -2, /* head_dim != 128, dtype_bytes != 2, gqa_group not in {1,2,4,8}, batch != 1      */
  HI_ERR_HBM_BUDGET = -3,  /* the staging ring does not fit the HBM KV budget (fewer than 2 slices)          */
  HI_ERR_HOST_MEM = -4,    /* the host cache would exceed hi_problem.host_mem_limit_bytes                    */
  HI_ERR_RANGE = -5,       /* past_len + len > max_context, or chunk_len > chunk                             */
  HI_ERR_NOT_PINNED = -6,  /* the cache pointer is not pinned host memory (offload) / device memory (resident)*/
  HI_ERR_HIP = -7          /* a HIP call failed; hi_last_error() has the text                                */
};

enum { HI_MODE_OFFLOAD = 0, HI_MODE_RESIDENT = 1 };
enum { HI_REGIME_COMPUTE = 0, HI_REGIME_LINK = 1, HI_REGIME_HBM = 2 };
/* debug/measurement switches for hi_ctx_set_flags: skip the attention kernels (transfer-only timing) or
 * skip the H2D/D2H copies (compute-only timing on stale staging contents) - results are meaningless then;
 * time the attention kernels with HIP events; force a prefill kernel variant (by default the library picks by
 * chunk length and group size between DEEP: 8 wavefronts per workgroup alternating matrix and softmax phases,
 * split over the K/V rows when the chunk alone would not fill the chip, and NARROW: 4 wavefronts, for very short
 * chunks); with the DEEP kernel, PAIRED / UNPAIRED force or forbid the balanced partition of the causal triangle
 * (deep and shallow blocks of query positions share their tiles), which the library otherwise picks when it saves
 * the deepest workgroups at least a few tiles. Do not change the variant between the calls of one (chunk, head) unit. */
enum { HI_FLAG_SKIP_KERNELS = 1, HI_FLAG_SKIP_COPIES = 2, HI_FLAG_TIME_KERNELS = 4, HI_FLAG_PREFILL_NARROW = 8,
       HI_FLAG_PREFILL_PAIRED = 16, HI_FLAG_PREFILL_DEEP = 32, HI_FLAG_PREFILL_UNPAIRED = 64,
       HI_FLAG_PREFILL_MFMA32 = 256 /* the DEEP kernel in its 32x32x16 MFMA form (by default it uses 16x16x32) */,
       HI_FLAG_PREFILL_8WAVE = 512, HI_FLAG_PREFILL_WIDE = 1024 /* the 16x16x32 DEEP kernel has two forms: 8 wavefronts of
          32 query rows, and 4 wavefronts of 64 (half the LDS operand reads per MFMA, but slow first and last tiles); by
          default each launch takes the second when it sweeps at least 640 K/V tiles; these flags force one (their
          state images are the same, so a unit's launches may mix them) */,
       HI_FLAG_PREFILL_SINGLE_SLICES = 2048 /* one attention launch per staging slice, also where the library would hand
          two short slices to one launch (measurement) */,
       HI_FLAG_INJECT_FAILURE = 128 /* test hook: the next unit call fails with HI_ERR_HIP right after its checks, as a
                                       failed launch or copy would; no GPU work is skipped or broken by it */ };

/* The paper's statement of the problem (Algorithm 1 "Require": L layers, H heads, sequence length S). */
typedef struct hi_problem {
  int32_t n_layers;            /* L */
  int32_t n_kv_heads;          /* H: KV heads per layer */
  int32_t gqa_group;           /* G: query heads sharing one KV head; 1, 2, 4 or 8 */
  int32_t head_dim;            /* D_h; 128 */
  int64_t max_context;         /* S_max: rows pre-allocated per head in the cache */
  int32_t chunk;               /* C: largest number of rows one hi_prefill_head call may carry */
  int32_t gpu_kv_budget_heads; /* HBM KV budget, in whole-head equivalents of S_max rows (>= 1 + resident_heads) */
  int32_t dtype_bytes;         /* 2 (bf16) */
  int32_t out_fp32;            /* 0: outputs are bf16, 1: outputs are fp32 */
  int32_t n_compute_units;     /* 0 = 256 (MI355X) */
  int32_t resident_heads;      /* Algorithm 1's H_on: the first resident_heads (layer, retrieval KV head) pairs, in
                                  layer-major order, keep their K/V in HBM and never cross the link (offload mode); the
                                  rest of the budget is the staging ring of the offloaded heads.  0 = none */
  int64_t host_mem_limit_bytes;/* 0 = no check */
  double link_GBps;            /* host link peak used by the regime prediction; 0 = 64 (PCIe Gen5 x16) */
  double hbm_GBps;             /* 0 = 8000 */
  double mfma_TFLOPs;          /* 0 = 2500 (dense bf16) */
  int32_t streaming_heads;     /* Appendix E (head-wise sparsity): the LAST streaming_heads KV heads of every layer are
                                  streaming heads, which keep only sink_tokens initial and recent_tokens most recent
                                  tokens, in HBM; the other heads ("retrieval heads") keep everything and are offloaded
                                  or resident as above.  0 = none; at most n_kv_heads - 1 */
  int32_t sink_tokens;         /* n_sink >= 0 */
  int32_t recent_tokens;       /* n_recent >= 1 (the token itself included) when streaming_heads > 0 */
  int32_t link_kv_bits;        /* representation of an offloaded head's rows in the host cache and on the link: 0 or 16 =
                                  bf16 rows (exact attention); 4 = 4-bit codes, 80 bytes per row of 128 channels (see
                                  "4-bit rows on the link" below; offload mode only).  Rows that stay in HBM (the chunk
                                  being processed, resident and streaming heads) are always bf16 */
  const uint8_t* streaming_mask; /* HOST, optional, [n_layers][n_kv_heads]: 1 = streaming head, 0 = retrieval head, for
                                  models whose split differs from layer to layer (Appendix E takes the roles from a
                                  trained model; Table 14 runs at 50 % streaming heads overall).  When given it replaces
                                  the "last streaming_heads heads of every layer" rule (streaming_heads is then ignored);
                                  every layer keeps at least one retrieval head.  Read by hi_offload_plan and copied by
                                  hi_ctx_create; the caller may free it afterwards.  With a mask, the cache holds the
                                  retrieval heads of all layers back to back in (layer, head) order, a layer's
                                  allocation (hi_ctx_set_layer_cache) its own retrieval heads in head order, and the
                                  streaming stores follow (layer, head) order likewise */
  int32_t q_prescaled;         /* 0: the queries handed to the attention calls are the q of Eq. 3 and a weight is
                                  exp(q.k / sqrt(head_dim) - max); 1: they are HI_Q_PRESCALE times that q (folded into
                                  the query projection, as hi_qkv_rope does with q_scale = HI_Q_PRESCALE: one rounding
                                  to bf16 either way) and a weight is 2^(q.k - max) - the same function of the model's
                                  q, one multiplication per score less in the attention kernels */
} hi_problem;

/* log2(e) / sqrt(128): the factor between the q of Eq. 3 and a pre-scaled query (hi_problem.q_prescaled) */
#define HI_Q_PRESCALE 0.12751743082459868f

/* Output of hi_offload_plan.  Sizes in bytes. */
typedef struct hi_plan {
  int32_t heads_per_group;       /* recommended KV heads per call (hi_prefill_group / hi_decode_group): Section 4's
                                    adaptive grouping, by context length as measured on MI355X; callers may use any */
  int32_t n_groups;              /* = ceil(n_kv_heads / heads_per_group) */
  int32_t paper_heads_per_group; /* what the paper's context-length rule would pick (Section 4, adaptive
                                    head-wise offloading: 8 up to 500K, 4 to 1M, 2 to 2M, 1 beyond); informational */
  int32_t n_slices_ring;         /* staging ring: number of slots */
  int64_t slice_tokens;          /* rows per slot (K part then V part, each slice_tokens * D_h * 2 bytes) */
  int32_t n_split_decode;        /* workgroups (KV partitions) of one decode launch */
  int32_t prefill_rows_per_wg;   /* query positions one prefill workgroup covers */
  int64_t host_bytes_per_head;   /* Eq. 11: 2 * S_max * D_h * sizeof */
  int64_t host_bytes_total;      /* Eq. 4:  L * H * host_bytes_per_head (H less the streaming heads) */
  int64_t hbm_staging_bytes;     /* the ring, n_slices_ring * slice_tokens * 2 * D_h * sizeof, followed by the resident
                                    heads' K/V (hbm_resident_bytes at hbm_resident_offset); <= budget * host_bytes_per_head;
                                    then the streaming heads' stores (hbm_stream_bytes more) */
  int64_t hbm_pingpong_paper_bytes; /* the paper's two-whole-heads ping-pong buffer, for comparison (Appendix A.3) */
  int64_t workspace_bytes;       /* fp32 (m, l, O) carry of a prefill unit + split-KV partials of a decode unit */
  int64_t ws_partials_offset;    /* byte offset of the decode partials inside the workspace */
  double alpha;                  /* Eq. 10: budget / (L * H) */
  double flop_prefill_unit;      /* useful (causal) flops of one (chunk, head) unit at P = S_max - C */
  double bytes_link_prefill_unit;/* H2D + D2H bytes of that unit */
  double bytes_link_decode_unit; /* H2D + D2H bytes of one (token, head) unit at P = S_max - 1 */
  double t_comp_prefill_s, t_link_prefill_s, t_hbm_prefill_s; /* Section 5: T ~ max(T_comp, T_mem) */
  double t_comp_decode_s, t_link_decode_s, t_hbm_decode_s;
  int32_t regime_prefill, regime_decode;                      /* HI_REGIME_* with offloading */
  int64_t hbm_resident_offset;   /* inside the staging buffer: [resident head][K|V][S_max][D_h] */
  int64_t hbm_resident_bytes;    /* resident_heads * host_bytes_per_head */
  int64_t hbm_stream_offset;     /* inside the staging buffer: the streaming heads' stores,
                                    [layer][streaming head][K|V][stream_rows][D_h] */
  int64_t hbm_stream_bytes;      /* L * streaming_heads * 2 * stream_rows * D_h * sizeof; outside the whole-head budget */
  int64_t stream_rows;           /* sink_tokens + recent_tokens (0 without streaming heads): sink token j at row j,
                                    token j >= sink_tokens at row sink_tokens + (j - sink_tokens) mod recent_tokens */
  int64_t link_row_bytes;        /* bytes of one K (or V) row in the host cache: D_h * sizeof, or 80 with link_kv_bits = 4;
                                    the cache is [layer][retrieval head][K|V][S_max][link_row_bytes] */
  int64_t hbm_packed_offset;     /* inside the staging buffer, with link_kv_bits = 4: where slices land as they come off
                                    the link, one area per ring slot, before they are expanded into the slot; the ring
                                    is sized so that ring + these areas stay inside the HBM budget */
  int64_t hbm_packed_bytes;      /* n_slices_ring * slice_tokens * 2 * link_row_bytes, or 0 */
  int64_t ws_writeback_offset;   /* inside the workspace, with link_kv_bits = 4: two buffers in which a call's new rows
                                    are encoded before their write-back */
  int64_t ws_writeback_bytes;    /* 2 * 2 * retrieval heads * chunk * link_row_bytes, or 0 */
} hi_plan;

typedef struct hi_stats {
  int64_t bytes_h2d, bytes_d2h;      /* enqueued so far */
  int64_t n_h2d_copies, n_d2h_copies;
  int64_t n_prefill_kernels, n_decode_kernels, n_combine_kernels;
  int64_t peak_staging_bytes;        /* largest number of staging bytes holding live K/V at once */
  double prefill_kernel_ms, decode_kernel_ms; /* HIP-event time of the attention kernels since the last
                                                 hi_reset_stats; only with HI_FLAG_TIME_KERNELS; hi_get_stats
                                                 synchronises to read them */
  double h2d_copy_ms, d2h_copy_ms;   /* the same for the prefetch copies (on stream_h2d) and the write-backs (on
                                        stream_d2h): time the copy engines spent on them */
  double exposed_copy_ms;            /* time stream_compute spent between consecutive attention launches (from the same
                                        events): the wait for the next staging slice - the part of the transfers that
                                        no kernel covered - plus launch latency and the expansion of 4-bit slices; an
                                        upper bound of the exposed transfer time */
} hi_stats;

typedef struct hi_ctx hi_ctx;

/*
 * P0 - planning (Algorithm 1 "Initialization"; Eq. 4-6, 10-11; Section 4 "pre-allocates the CPU's KV cache
 * memory and the GPU's ping-pong memory"; Section 5 performance model).
 * Pure host arithmetic: needs no GPU and makes no HIP call.  `problem` and `plan` are host pointers owned by
 * the caller.  Errors: HI_ERR_ARG, HI_ERR_UNSUPPORTED, HI_ERR_HBM_BUDGET, HI_ERR_HOST_MEM; `plan` is left
 * untouched on error.
 */
hi_status hi_offload_plan(const hi_problem* problem, hi_plan* plan);

/*
 * Context.  The caller owns every large buffer and keeps it alive until hi_ctx_destroy:
 *   kv_cache       HI_MODE_OFFLOAD : pinned HOST memory, plan.host_bytes_total bytes, layout
 *                                    [layer][kv_head][K|V][S_max][D_h] bf16 (each head's K rows contiguous, then
 *                                    its V rows: the head-wise partition of Eq. 7-8; kv_head runs over the
 *                                    n_kv_heads - streaming_heads retrieval heads only);
 *                  HI_MODE_RESIDENT: DEVICE memory of the same size and layout (no copies; HBM-roofline runs).
 *   hbm_staging    DEVICE, plan.hbm_staging_bytes (in resident mode only the streaming heads' stores are used; may
 *                  be null there without streaming heads).  With
 *                  hi_problem.resident_heads > 0 its tail holds those heads' K/V: units of a resident head read
 *                  and append there, move nothing over the link and leave the host cache rows of that head
 *                  untouched; a head group must be all resident or all offloaded.
 *   hbm_workspace  DEVICE, plan.workspace_bytes.
 *   stream_*       hipStream_t handles (as void*), all at default priority.  Kernels run on stream_compute,
 *                  host-to-device prefetches on stream_h2d, write-backs on stream_d2h.
 * With hi_problem.link_kv_bits = 4 the cache layout is [layer][kv_head][K|V][S_max][plan.link_row_bytes] bytes.
 * A context is used by one host thread at a time (its calls mutate the ring's bookkeeping without locks); different
 * contexts are independent.  Errors: HI_ERR_ARG, HI_ERR_NOT_PINNED, HI_ERR_UNSUPPORTED, HI_ERR_HIP.
 * kv_cache may be null when every layer's rows are given by hi_ctx_set_layer_cache before the layer is first used.
 */
hi_status hi_ctx_create(const hi_problem* problem, const hi_plan* plan, int32_t mode, void* kv_cache,
                        void* hbm_staging, void* hbm_workspace, void* stream_compute, void* stream_h2d,
                        void* stream_d2h, hi_ctx** out);
hi_status hi_ctx_destroy(hi_ctx* ctx);
/*
 * One allocation per layer (Eq. 7-8 partition the cache by layer and head; Algorithm 1 only ever touches one
 * (layer, head) at a time, so nothing requires the layers to be contiguous): kv_layer holds the rows of `layer`,
 * [kv_head][K|V][S_max][plan.link_row_bytes], plan.host_bytes_total / n_layers bytes, pinned host memory in
 * HI_MODE_OFFLOAD, device memory in HI_MODE_RESIDENT; it replaces whatever the layer had.  A 1M-token, 32-layer
 * cache is then 32 allocations of 4 GiB instead of one of 128 GiB.  Synchronises the context's streams first.
 * Errors: HI_ERR_ARG, HI_ERR_NOT_PINNED, HI_ERR_HIP.
 */
hi_status hi_ctx_set_layer_cache(hi_ctx* ctx, int32_t layer, void* kv_layer);
hi_status hi_ctx_set_flags(hi_ctx* ctx, int32_t flags);
/* Bounded run-ahead of the caller: hi_prefill_head / hi_decode_head first wait (on the host) until the unit
 * `units` calls earlier has finished on stream_compute; the history of the unit being enqueued is already being
 * prefetched by then, so the link stays busy, and the runtime's queues stay short (with hundreds of cross-stream
 * waits queued ahead the copy engine leaves gaps between transfers).  Default 2; 0 = never wait; at most 15. */
hi_status hi_ctx_set_run_ahead(hi_ctx* ctx, int32_t units);

/*
 * T1 + K1 + T3 - one prefill unit: one chunk, one KV head, its G query heads (Algorithm 1, prefill phase, the
 * body of the head loop; Eq. 9).  Appends, then attends:
 *   - rows [past_len, past_len + chunk_len) of (layer, kv_head) in the cache receive k_new / v_new
 *     (asynchronous write-back on stream_d2h; a device copy in resident mode);
 *   - out[g][i][:] = softmax_j<=past_len+i( q[g][i] . K[j] / sqrt(D_h) ) V[j]  over the head's rows 0..past_len+i,
 *     the past rows streamed from the cache through the staging ring, the chunk's own rows read from k_new/v_new.
 * q_dev   DEVICE bf16 [G][chunk_len][D_h]; k_new_dev, v_new_dev DEVICE bf16 [chunk_len][D_h];
 * out_dev DEVICE [G][chunk_len][D_h], bf16 or fp32 per hi_problem.out_fp32.  All 16-byte aligned.
 * next_* name the unit that will be called next (Algorithm 1 "Async Prefetch next KV cache"): its past rows are
 * prefetched into free ring slots while this unit computes; next_layer = -1 means none.  The hint must be
 * honoured by the next call, or that call simply fetches on demand.
 * Asynchronous: enqueues and returns (after the bounded run-ahead wait described at hi_ctx_set_run_ahead).  Results
 * and the cache append are valid after hi_sync.  The caller's
 * buffers are borrowed until then.  1 <= chunk_len <= chunk; past_len >= 0; no alignment is required of either.
 * Errors (synchronous, nothing enqueued, cache and staging ring untouched): HI_ERR_ARG, HI_ERR_RANGE,
 * HI_ERR_HBM_BUDGET, HI_ERR_UNSUPPORTED - every check comes before the first enqueue.  HI_ERR_HIP means a HIP call
 * failed after work had been enqueued: copies, kernels and the ring's bookkeeping are then half-advanced, so the
 * context is closed - every later unit call returns HI_ERR_HIP - and can only be synchronised and destroyed.
 */
hi_status hi_prefill_head(hi_ctx* ctx, int32_t layer, int32_t kv_head, const void* q_dev, const void* k_new_dev,
                          const void* v_new_dev, int64_t past_len, int32_t chunk_len, void* out_dev,
                          int32_t next_layer, int32_t next_kv_head, int64_t next_past_len);

/*
 * T1 + K2 + K3 + T3 - one decode unit: one new token, one KV head, its G query rows (Algorithm 1, decode phase).
 * Appends the token's K/V row at row past_len, then attends over rows 0..past_len inclusive (the token sees
 * itself).  Split-KV: each partition of the streamed rows yields a partial (max, sum, weighted V); a combine
 * kernel merges the partials of all partitions and slices with the new row.
 * q_dev DEVICE bf16 [G][D_h]; k_new_dev, v_new_dev DEVICE bf16 [D_h]; out_dev DEVICE [G][D_h].
 * Same asynchrony, ownership, hint and error rules as hi_prefill_head.
 */
hi_status hi_decode_head(hi_ctx* ctx, int32_t layer, int32_t kv_head, const void* q_dev, const void* k_new_dev,
                         const void* v_new_dev, int64_t past_len, void* out_dev, int32_t next_layer,
                         int32_t next_kv_head, int64_t next_past_len);

/*
 * Head groups (Section 4, "adaptive head-wise offloading": several heads fused per transfer and per launch at
 * shorter contexts, to amortise the per-head overheads; a group of all heads is layer-wise offload).  The same
 * two operations over n_heads consecutive KV heads kv_head .. kv_head + n_heads - 1 of one layer, in one call:
 * one launch per staging slice covers all heads of the group, and a staging slice holds
 * plan.slice_tokens / n_heads rows (rounded down to a multiple of 64) of each, so the HBM budget is unchanged.
 * q_dev   DEVICE bf16 [n_heads][G][len][D_h]; k_new_dev, v_new_dev DEVICE bf16 [n_heads][len][D_h];
 * out_dev DEVICE [n_heads][G][len][D_h]  (len = chunk_len, or 1 with that axis dropped for decode).
 * The hint names the next group (first head and size).  hi_prefill_head / hi_decode_head are the n_heads = 1
 * case; results are identical whatever the grouping.  Extra errors: HI_ERR_HBM_BUDGET when a slice cannot hold
 * 64 rows of every head of the group.
 */
hi_status hi_prefill_group(hi_ctx* ctx, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                           const void* k_new_dev, const void* v_new_dev, int64_t past_len, int32_t chunk_len,
                           void* out_dev, int32_t next_layer, int32_t next_kv_head, int32_t next_n_heads,
                           int64_t next_past_len);
hi_status hi_decode_group(hi_ctx* ctx, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                          const void* k_new_dev, const void* v_new_dev, int64_t past_len, void* out_dev,
                          int32_t next_layer, int32_t next_kv_head, int32_t next_n_heads, int64_t next_past_len);

/*
 * A decode step over n_heads (<= 64) consecutive HBM-RESIDENT KV heads whose histories differ in length - a batch of
 * sequences of different lengths served as more KV heads (the paper runs batch 1; Section 3.2 notes the head-wise
 * partition extends to the batch dimension): head j has past_lens[j] rows (HOST array, read before the call returns),
 * its token's row is appended at row past_lens[j] and attends over rows 0..past_lens[j].  One split-KV launch over
 * all heads (a head with fewer rows than partitions leaves neutral partials), one combine launch.  Buffers as in
 * hi_decode_group.  HI_ERR_UNSUPPORTED for offloaded or streaming heads (the heads of an offloaded group share
 * staging slices of one length: call those one by one, each at its own past_len).
 */
hi_status hi_decode_group_ragged(hi_ctx* ctx, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                                 const void* k_new_dev, const void* v_new_dev, const int64_t* past_lens, void* out_dev);

/*
 * Streaming heads (Appendix E, "Efficient Management of KV cache": retrieval heads retain all tokens and are
 * offloaded, streaming heads retain only recent tokens and stay on the GPU).  With hi_problem.streaming_heads > 0
 * the same four calls serve the last streaming_heads KV heads of a layer, with these differences:
 *   - row at absolute position p attends over key j iff j <= p and (j < sink_tokens or p - j < recent_tokens)
 *     - a different function from the exact attention of the other heads, by design of the extension;
 *   - the head's K/V is the bounded HBM store described at hi_plan.stream_rows; nothing crosses the link and the
 *     host cache has no rows for it; a prefill call reads the store, then enters the chunk's rows into it; a
 *     decode call writes the token's row over the row that left the window and attends over the store;
 *   - past_len is still the absolute position of the call's first row, and calls of one head must come in
 *     position order without gaps (the store holds only what earlier calls left in it);
 *   - a head group must not mix streaming and retrieval heads (HI_ERR_ARG); a hint naming a streaming unit
 *     prefetches nothing.
 * With hi_problem.streaming_mask the roles are given per (layer, head) instead; everything above holds head by head.
 */

/*
 * The steps either side of the head-wise attention calls (Section 3.1, Eq. 1: the key and value - and the query -
 * of a token are linear projections of its hidden state; Eq. 9: the head outputs are concatenated, then projected
 * by the model's output matrix).  Stateless: no context, only device buffers and a stream.  Weights are bf16 in
 * [out_features][in_features] layout (y = x W^T); accumulation is fp32.
 *
 * hi_qkv_rope: for a chunk X [chunk_len][d_model] of hidden states whose first row is at absolute position
 *   past_len, computes [Q | K | V] = X W_qkv^T with W_qkv [(n_q_heads + 2 n_kv_heads) * 128][d_model] (the rows of
 *   W_Q, then W_K, then W_V), rotates every query and key head by the rotary position embedding of the evaluated
 *   model (dimension i < 64 paired with i + 64, angle position * rope_theta^(-i / 64); rope_theta = 0: no
 *   rotation) and writes head-major q_out [n_q_heads][chunk_len][128], k_out and v_out
 *   [n_kv_heads][chunk_len][128] - exactly the q_dev / k_new_dev / v_new_dev of hi_prefill_group over all heads
 *   (bf16, or fp32 with out_fp32 = 1 for checking).  workspace_dev: DEVICE, hi_proj_workspace_bytes(chunk_len)
 *   bytes (the chunk's cos / sin table, computed in double precision); may be null when rope_theta = 0.
 *   q_scale: factor applied to the query heads after the rotation, in fp32, before the one rounding of the output
 *   (> 0; 1 = none; HI_Q_PRESCALE for a context with hi_problem.q_prescaled = 1).
 * hi_out_proj: Y [chunk_len][d_model] = Concat_h(attn[h]) W_o^T for the head-major attention output
 *   attn [n_q_heads][chunk_len][128] (the out_dev of the attention calls) and W_o [d_model][n_q_heads * 128].
 * d_model must be a multiple of 128; every operand must be smaller than 4 GiB; all pointers 16-byte aligned.
 * Both enqueue on `stream` (a hipStream_t) and return.  Errors: HI_ERR_ARG, HI_ERR_UNSUPPORTED, HI_ERR_HIP.
 * chunk_len = 1 (decode) takes a matrix-vector kernel bound by the HBM read of the weights (workspace not used).
 */
hi_status hi_proj_workspace_bytes(int32_t chunk_len, int64_t* bytes);
hi_status hi_qkv_rope(void* stream, const void* x_dev, const void* w_qkv_dev, int32_t d_model, int32_t n_q_heads,
                      int32_t n_kv_heads, int32_t chunk_len, int64_t past_len, double rope_theta, int32_t out_fp32,
                      void* q_out_dev, void* k_out_dev, void* v_out_dev, void* workspace_dev, float q_scale);
hi_status hi_out_proj(void* stream, const void* attn_dev, const void* w_o_dev, int32_t n_q_heads, int32_t d_model,
                      int32_t chunk_len, int32_t out_fp32, void* y_out_dev);

/*
 * hi_qkv_rope for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and the same results as hi_qkv_rope;
 * the chunk's cos / sin table is written to an 8 MiB array built into the library's device image (one copy per GPU,
 * held until the process ends) instead of workspace_dev.  chunk_len may be at most 16384 (HI_ERR_RANGE beyond, nothing
 * enqueued).  The call allocates nothing and frees nothing.  All calls on one GPU share that GPU's array: calls that
 * may overlap in time on one GPU (different streams, different host threads) race on it and must be ordered by the
 * caller; calls on one stream are ordered by the stream.  Nothing needs clearing between calls: a call rewrites the
 * table for every token it rotates.  Otherwise as hi_qkv_rope (arguments, layouts, errors).
 */
hi_status hi_qkv_rope_static(void* stream, const void* x_dev, const void* w_qkv_dev, int32_t d_model, int32_t n_q_heads,
                             int32_t n_kv_heads, int32_t chunk_len, int64_t past_len, double rope_theta,
                             int32_t out_fp32, void* q_out_dev, void* k_out_dev, void* v_out_dev, float q_scale);

/*
 * 4-bit rows on the link (Appendix B and Section 6.3 describe 4-bit KV quantisation as a representation that shrinks
 * the cache about 4x and is converted back on the GPU; Section 3.3 finds offloaded decode bound by the link).  With
 * hi_problem.link_kv_bits = 4 the rows of an offloaded head are stored in the host cache, and cross the link, as
 * 80-byte rows: 64 bytes of 4-bit codes (channel 2i in the low nibble of byte i, channel 2i + 1 in the high one),
 * then 4 bf16 scales and 4 bf16 zeros, one pair per group of 32 consecutive channels.  Per group, in binary32 with one
 * rounding per operation: zero = min, scale = bf16((max - min) * (1/15)) (taken as 0 below 2^-120: a constant group),
 * code = min(15, rint((x - zero) * (1 / scale))), and the row is read back as x^ = bf16(zero + code * scale).
 * The same four attention calls then compute: rows of the call itself (the chunk, the token) take part as the exact
 * bf16 values the caller passed; rows of earlier calls take part as x^ - an approximation of exact attention by
 * design, identical in prefill and decode.  A call encodes its new rows on the compute stream, writes the encoded
 * rows back, and expands each slice that comes off the link into the staging ring before the attention kernel
 * reads it; link bytes and host bytes shrink by 3.2x, and the ring shrinks so that ring plus landing areas stay
 * inside the HBM budget.  Inputs must be finite with a range (max - min of a group) below 2^127; when a group's
 * minimum is a zero, either sign of zero may be stored for it (the decoded values are equal).  HBM-resident and
 * streaming heads are unaffected.  HI_MODE_RESIDENT rejects it (HI_ERR_UNSUPPORTED): there is no link to save.
 *
 * hi_kv_quantize / hi_kv_dequantize: the two conversions alone, for n_rows rows of 128 channels, DEVICE bf16
 * [n_rows][128] <-> DEVICE bytes [n_rows][80]; 16-byte aligned; enqueue on `stream` and return.
 */
hi_status hi_kv_quantize(void* stream, const void* rows_dev, int64_t n_rows, void* packed_dev);
hi_status hi_kv_dequantize(void* stream, const void* packed_dev, int64_t n_rows, void* rows_dev);

/* T4 - drain the three streams; surfaces deferred HIP errors (HI_ERR_HIP). */
hi_status hi_sync(hi_ctx* ctx);

hi_status hi_get_stats(hi_ctx* ctx, hi_stats* out);
hi_status hi_reset_stats(hi_ctx* ctx);

/* Static strings; never null. hi_last_error is per calling thread. */
const char* hi_status_string(hi_status s);
const char* hi_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HEADINFER_H */
