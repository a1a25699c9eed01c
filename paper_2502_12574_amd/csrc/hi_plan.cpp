// hi_offload_plan: pure host arithmetic (no HIP calls).
// Follows Algorithm 1 "Initialization", Eq. 4-6 and 10-11 (cache size, on-GPU fraction), Section 4
// (pre-allocation; adaptive head-wise offloading thresholds) and the Section 5 performance model.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include "hi_internal.h"

namespace hi {

static thread_local char g_last_error[512] = "";

void set_last_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
  va_end(ap);
}

hi_status validate_problem(const hi_problem* p) {
  if (!p) { set_last_error("problem is null"); return HI_ERR_ARG; }
  if (p->n_layers < 1 || p->n_kv_heads < 1 || p->max_context < 1 || p->chunk < 1 ||
      p->gpu_kv_budget_heads < 1 || p->n_compute_units < 0 || p->host_mem_limit_bytes < 0 ||
      p->link_GBps < 0 || p->hbm_GBps < 0 || p->mfma_TFLOPs < 0 || (p->out_fp32 != 0 && p->out_fp32 != 1) ||
      (p->q_prescaled != 0 && p->q_prescaled != 1)) {
    set_last_error("problem field out of range");
    return HI_ERR_ARG;
  }
  if (p->chunk > p->max_context) { set_last_error("chunk %d exceeds max_context", p->chunk); return HI_ERR_ARG; }
  if (!p->streaming_mask && (p->streaming_heads < 0 || p->streaming_heads >= p->n_kv_heads)) {
    set_last_error("streaming_heads must be in [0, n_kv_heads)");
    return HI_ERR_ARG;
  }
  if (p->streaming_mask) {
    for (int l = 0; l < p->n_layers; ++l) {
      int n = 0;
      for (int h = 0; h < p->n_kv_heads; ++h) {
        const uint8_t m = p->streaming_mask[(int64_t)l * p->n_kv_heads + h];
        if (m > 1) { set_last_error("streaming_mask entries must be 0 or 1"); return HI_ERR_ARG; }
        n += m;
      }
      if (n >= p->n_kv_heads) { set_last_error("layer %d has no retrieval head", l); return HI_ERR_ARG; }
    }
  }
  const int64_t n_streaming = count_streaming(*p);
  if (p->link_kv_bits != 0 && p->link_kv_bits != 16 && p->link_kv_bits != 4) {
    set_last_error("link_kv_bits must be 0, 16 (bf16 rows) or 4");
    return HI_ERR_ARG;
  }
  if (n_streaming > 0 && (p->sink_tokens < 0 || p->recent_tokens < 1 ||
                                 (int64_t)p->sink_tokens + p->recent_tokens > kStreamMaxRows)) {
    set_last_error("streaming heads need sink_tokens >= 0, recent_tokens >= 1 and at most %lld rows in all",
                   (long long)kStreamMaxRows);
    return HI_ERR_ARG;
  }
  if (p->resident_heads < 0 ||
      (int64_t)p->resident_heads > (int64_t)p->n_layers * p->n_kv_heads - n_streaming) {
    set_last_error("resident_heads out of range");
    return HI_ERR_ARG;
  }
  if (p->gpu_kv_budget_heads < p->resident_heads + 1) {
    set_last_error("an HBM budget of %d heads cannot keep %d heads resident and stream the others", p->gpu_kv_budget_heads,
                   p->resident_heads);
    return HI_ERR_HBM_BUDGET;
  }
  if (p->head_dim != kHeadDim) { set_last_error("head_dim %d unsupported (128 only)", p->head_dim); return HI_ERR_UNSUPPORTED; }
  if (p->dtype_bytes != 2) { set_last_error("dtype_bytes %d unsupported (bf16 only)", p->dtype_bytes); return HI_ERR_UNSUPPORTED; }
  const int g = p->gqa_group;
  if (!(g == 1 || g == 2 || g == 4 || g == 8)) { set_last_error("gqa_group %d unsupported", g); return HI_ERR_UNSUPPORTED; }
  return HI_OK;
}

}  // namespace hi

using namespace hi;

extern "C" hi_status hi_offload_plan(const hi_problem* p, hi_plan* out) {
  if (!out) { set_last_error("plan is null"); return HI_ERR_ARG; }
  hi_status st = validate_problem(p);
  if (st != HI_OK) return st;

  hi_plan pl;
  std::memset(&pl, 0, sizeof(pl));
  const int64_t S = p->max_context;
  const int64_t C = p->chunk;
  const int G = p->gqa_group;
  const int64_t row = 2LL * p->head_dim * p->dtype_bytes;  // K row + V row of one head, in HBM
  const bool packed = p->link_kv_bits == 4;
  pl.link_row_bytes = packed ? kLinkRowBytes4 : p->head_dim * p->dtype_bytes;
  const int64_t link_row = 2 * pl.link_row_bytes;          // the same pair in the host cache and on the link

  // Eq. 11 and Eq. 4
  pl.host_bytes_per_head = S * link_row;
  const int64_t n_streaming = count_streaming(*p);
  pl.host_bytes_total = ((int64_t)p->n_layers * p->n_kv_heads - n_streaming) * pl.host_bytes_per_head;
  if (p->host_mem_limit_bytes > 0 && pl.host_bytes_total > p->host_mem_limit_bytes) {
    set_last_error("host cache of %lld bytes exceeds the limit", (long long)pl.host_bytes_total);
    return HI_ERR_HOST_MEM;
  }
  // Eq. 10
  pl.alpha = (double)p->gpu_kv_budget_heads / ((double)p->n_layers * p->n_kv_heads);
  pl.hbm_pingpong_paper_bytes = 2 * S * row;

  // heads_per_group is filled in below, once the ring geometry is known
  {  // Section 4: all heads fused up to 500K, two groups to 1M, four to 2M, eight beyond
    int groups = S <= 500 * 1024 ? 1 : S <= 1024 * 1024 ? 2 : S <= 2048 * 1024 ? 4 : 8;
    int hpg = p->n_kv_heads / groups;
    pl.paper_heads_per_group = hpg < 1 ? 1 : hpg;
  }

  // staging ring: sequence slices inside the HBM budget, so that a slice can land while another is consumed
  // (Algorithm 1's H_on heads take whole-head shares of the budget; the ring gets what is left)
  // (with 4-bit rows on the link every slot also has a landing area for the encoded slice: the budget then pays
  // row + link_row bytes per ring row)
  const int64_t budget_rows = (int64_t)(p->gpu_kv_budget_heads - p->resident_heads) * S;
  const int64_t budget_tokens = packed ? budget_rows * row / (row + link_row) : budget_rows;
  // (four slices: measured against eight, the larger copies and fewer launches win 1-3 % of prefill time and up to
  // 14 % of offloaded decode time at a 128K context, and nothing is lost in overlap; three or two slices are within
  // 1.5 % of four either way at 128K and 1M contexts)
  // (4-bit rows: two slices - a slice is 3.2x fewer link bytes, and the larger copies matter more than the depth of
  // the ring: measured at a 128K context, decode 4.0 -> 3.5 ms per token and prefill 1 % faster; at 1M, 25.0 -> 24.5 ms,
  // and 24.2 ms with slices of up to 524288 rows)
  int64_t slice = (budget_tokens / (packed ? 2 : 4)) / 64 * 64;
  if (slice < 64) slice = 64;
  const int64_t slice_cap = packed ? 524288 : 262144;     // about 128 MiB (bf16) / 80 MiB (4-bit) of link bytes
  if (slice > slice_cap) slice = slice_cap;
  if (budget_tokens / slice > 64) slice = round_up(ceil_div(budget_tokens, 64), 64);
  const int64_t n_slices = budget_tokens / slice;
  if (n_slices < 2) {
    set_last_error("HBM KV budget of %lld rows cannot hold two staging slices", (long long)budget_tokens);
    return HI_ERR_HBM_BUDGET;
  }
  pl.slice_tokens = slice;
  pl.n_slices_ring = (int32_t)n_slices;

  // Section 4, adaptive head grouping, as measured on MI355X with this library (layer_bench --heads-per-call): up to 16K tokens the
  // per-call overheads dominate and as many heads as the slice can hold (64 rows each) go into one call; up to 256K
  // two heads per call still gain a few per cent; beyond, one head per call (the finest granularity) is as fast.
  {
    // a group never mixes the two kinds of head (with a mask: the layer with the fewest retrieval heads decides)
    int n_retrieval = p->n_kv_heads - p->streaming_heads, n_stream_layer = p->streaming_heads;
    if (p->streaming_mask) {
      n_retrieval = p->n_kv_heads;
      n_stream_layer = 0;
      for (int l = 0; l < p->n_layers; ++l) {
        int n = 0;
        for (int h = 0; h < p->n_kv_heads; ++h) n += p->streaming_mask[(int64_t)l * p->n_kv_heads + h];
        if (p->n_kv_heads - n < n_retrieval) n_retrieval = p->n_kv_heads - n;
        if (n > n_stream_layer) n_stream_layer = n;
      }
    }
    int hpg = 1;
    if (S <= 16 * 1024 + p->chunk) {
      while (hpg * 2 <= n_retrieval && (int64_t)hpg * 2 * 64 <= slice) hpg *= 2;
    } else if (S <= 256 * 1024 + p->chunk) {
      if (n_retrieval >= 2 && 2 * 64 <= slice) hpg = 2;
    }
    pl.heads_per_group = hpg;
    pl.n_groups = (int32_t)(ceil_div(n_retrieval, hpg) + ceil_div(n_stream_layer, hpg));
  }
  pl.hbm_resident_offset = n_slices * slice * row;
  pl.hbm_resident_bytes = (int64_t)p->resident_heads * S * row;
  // Appendix E: the streaming heads' bounded stores, small and outside the whole-head budget
  pl.stream_rows = n_streaming > 0 ? (int64_t)p->sink_tokens + p->recent_tokens : 0;
  pl.hbm_stream_offset = pl.hbm_resident_offset + pl.hbm_resident_bytes;
  pl.hbm_stream_bytes = n_streaming * pl.stream_rows * row;
  pl.hbm_packed_offset = pl.hbm_stream_offset + pl.hbm_stream_bytes;
  pl.hbm_packed_bytes = packed ? n_slices * slice * link_row : 0;
  pl.hbm_staging_bytes = pl.hbm_packed_offset + pl.hbm_packed_bytes;

  const int n_cu = p->n_compute_units > 0 ? p->n_compute_units : 256;
  pl.n_split_decode = n_cu;
  pl.prefill_rows_per_wg = prefill_strip(G);

  // any kernel variant: the same bytes per position, times the split-KV factor of the 8-wave kernel
  const int64_t carry_bytes = prefill_carry_bound(G, C, p->n_kv_heads);
  const int64_t partial_bytes = decode_part_head_stride(S, slice, pl.n_split_decode, G) * 4 * p->n_kv_heads;
  pl.ws_partials_offset = round_up(carry_bytes, 256);
  pl.ws_writeback_offset = pl.ws_partials_offset + round_up(partial_bytes, 256);
  pl.ws_writeback_bytes = packed ? 2 * round_up((int64_t)(p->streaming_mask ? p->n_kv_heads : p->n_kv_heads - p->streaming_heads) * C * link_row, 256) : 0;
  pl.workspace_bytes = pl.ws_writeback_offset + pl.ws_writeback_bytes;

  // Section 5: T ~ max(T_comp, T_mem), evaluated for the deepest unit
  const double link = (p->link_GBps > 0 ? p->link_GBps : 64.0) * 1e9;
  const double hbm = (p->hbm_GBps > 0 ? p->hbm_GBps : 8000.0) * 1e9;
  const double mfma = (p->mfma_TFLOPs > 0 ? p->mfma_TFLOPs : 2500.0) * 1e12;
  const double P = (double)(S - C);
  const double d = p->head_dim;
  pl.flop_prefill_unit = 4.0 * d * G * ((double)C * P + 0.5 * (double)C * ((double)C + 1.0));
  pl.bytes_link_prefill_unit = (double)link_row * (P + (double)C);
  pl.bytes_link_decode_unit = (double)link_row * (double)S;
  const double qo_bytes = 2.0 * G * (double)C * d * p->dtype_bytes;
  pl.t_comp_prefill_s = pl.flop_prefill_unit / mfma;
  pl.t_link_prefill_s = pl.bytes_link_prefill_unit / link;
  pl.t_hbm_prefill_s = ((double)row * (P + (double)C) + qo_bytes) / hbm;
  pl.t_comp_decode_s = 4.0 * d * G * (double)S / mfma;
  pl.t_link_decode_s = pl.bytes_link_decode_unit / link;
  pl.t_hbm_decode_s = (double)row * (double)S / hbm;
  auto regime = [](double tc, double tl, double th) {
    if (tc >= tl && tc >= th) return (int32_t)HI_REGIME_COMPUTE;
    return tl >= th ? (int32_t)HI_REGIME_LINK : (int32_t)HI_REGIME_HBM;
  };
  pl.regime_prefill = regime(pl.t_comp_prefill_s, pl.t_link_prefill_s, pl.t_hbm_prefill_s);
  pl.regime_decode = regime(pl.t_comp_decode_s, pl.t_link_decode_s, pl.t_hbm_decode_s);

  *out = pl;
  return HI_OK;
}

extern "C" const char* hi_status_string(hi_status s) {
  switch (s) {
    case HI_OK: return "HI_OK";
    case HI_ERR_ARG: return "HI_ERR_ARG";
    case HI_ERR_UNSUPPORTED: return "HI_ERR_UNSUPPORTED";
    case HI_ERR_HBM_BUDGET: return "HI_ERR_HBM_BUDGET";
    case HI_ERR_HOST_MEM: return "HI_ERR_HOST_MEM";
    case HI_ERR_RANGE: return "HI_ERR_RANGE";
    case HI_ERR_NOT_PINNED: return "HI_ERR_NOT_PINNED";
    case HI_ERR_HIP: return "HI_ERR_HIP";
    default: return "HI_ERR_UNKNOWN";
  }
}

extern "C" const char* hi_last_error(void) { return hi::g_last_error; }
