// Host-side pipeline: T1 prefetch (H2D), T3 write-back (D2H), T4 events, and the per-head entry points.
//
// Section 4 / Algorithm 1: while head h computes, the next head's K/V history is prefetched from the pinned host
// cache and the current head's new rows are written back, on separate streams (full-duplex link).  Here the
// "ping-pong memory" is a ring of sequence slices that together never exceed the HBM KV budget (one head's worth
// by default): the kernel consumes slice n while later slices - of this head, then of the next one - land, and the
// softmax state is carried from slice to slice.  Calls only enqueue work; the one host-side wait is the bounded
// run-ahead (a call waits until the unit two calls earlier has finished), which keeps the runtime's queues short.
#include <hip/hip_runtime.h>
#include <cstring>
#include <new>
#include <vector>
#include "hi_internal.h"

using namespace hi;

#define HI_HIP(call)                                                                   \
  do {                                                                                 \
    hipError_t e_ = (call);                                                            \
    if (e_ != hipSuccess) {                                                            \
      set_last_error("%s failed: %s", #call, hipGetErrorString(e_));                   \
      return HI_ERR_HIP;                                                               \
    }                                                                                  \
  } while (0)

#define HI_TRY(call)                  \
  do {                                \
    hi_status s_ = (call);            \
    if (s_ != HI_OK) return s_;       \
  } while (0)

struct TimedSpan {
  hipEvent_t start, stop;
  int kind;   // 0 prefill kernels, 1 decode kernels, 2 host-to-device copy, 3 device-to-host copy, 4 compute stream
              // waiting for a slice (the part of a transfer that is not hidden)
};

struct hi_ctx {
  hi_problem prob;
  hi_plan plan;
  int mode = HI_MODE_OFFLOAD;
  int flags = 0;
  // Appendix E head roles, per (layer, head): index among the retrieval heads (layer-major order; -1: a streaming
  // head) and among the streaming heads (-1: a retrieval head); the retrieval index of each layer's first one
  std::vector<uint8_t> mask;
  std::vector<int32_t> retr_idx, strm_idx, layer_retr0;
  std::vector<char*> kv_layer;   // per layer: host (offload) or device (resident) cache rows, null: not given yet
  bool failed = false;       // an error after work had been enqueued: the ring's bookkeeping cannot be trusted
  bool enqueuing = false;    // the running call has passed its checks and started to enqueue
  char* staging = nullptr;
  char* ws = nullptr;
  hipStream_t sc = nullptr, sh = nullptr, sd = nullptr;

  int n_slots = 0;
  int64_t slice_tokens = 0;
  std::vector<hipEvent_t> ev_ready, ev_free;   // per ring slot
  hipEvent_t ev_entry = nullptr;               // compute-stream position when a call starts
  std::vector<hipEvent_t> ev_wb;               // per (layer, head): last write-back of that head finished
  std::vector<char> wb_valid;
  hipEvent_t ev_wbq[2] = {nullptr, nullptr};   // 4-bit link rows: the write-back that read encode buffer b has finished
  char wbq_valid[2] = {0, 0};
  int wbq_turn = 0;

  // the ring is a FIFO: slices are consumed in the order they were fetched
  int64_t seq_issued = 0;     // slices whose H2D has been enqueued
  int64_t seq_consumed = 0;   // slices whose consuming kernel has been enqueued (or that were dropped)

  struct Unit {
    bool valid = false;
    int layer = 0, head = 0;  // first head of the group
    int nh = 1;               // heads in the group
    int64_t past = 0;
    int64_t n_slices = 0;
    int64_t issued = 0;       // slices of this unit already fetched
    int64_t first_seq = 0;
  } pend;                     // the unit whose history is (partly) in the ring

  // bounded run-ahead of the calling thread: a call first waits until the unit `run_ahead` calls earlier has
  // finished on the compute stream (its successor's history is already being prefetched by then)
  int run_ahead = 2;
  std::vector<hipEvent_t> ev_unit;             // ring of "unit finished" events
  int64_t n_units = 0;

  hi_stats stats;
  std::vector<TimedSpan> spans;
  std::vector<TimedSpan> span_pool;
};

namespace {

// heads of a layer that keep their whole history (Appendix E: "retrieval heads"); the last streaming_heads heads
// of each layer are streaming heads, which have no rows in the cache
inline bool unit_streaming(const hi_ctx* c, int layer, int head) { return c->strm_idx[layer * c->prob.n_kv_heads + head] >= 0; }
inline int64_t retr_index(const hi_ctx* c, int layer, int head) { return c->retr_idx[layer * c->prob.n_kv_heads + head]; }

// one K (or V) row in the host cache and on the link: bf16, or 4-bit codes with a scale and a zero per 32 channels
inline int64_t link_row(const hi_ctx* c) { return c->plan.link_row_bytes; }
inline bool link_packed(const hi_ctx* c) { return c->prob.link_kv_bits == 4; }

// rows of (layer, head) in the cache: each layer has its own base pointer, [kv_head][K|V][S_max][row bytes] behind it
inline char* cache_plane(const hi_ctx* c, int layer, int head, int which /*0 K, 1 V*/) {
  const int64_t plane = c->prob.max_context * link_row(c);
  return c->kv_layer[layer] + ((retr_index(c, layer, head) - c->layer_retr0[layer]) * 2 + which) * plane;
}

// A ring slot holds one sequence slice of every head of a group: rows_of(nh) rows of K then of V per head, the
// heads head_pitch(nh) bytes apart (Section 4, adaptive head grouping: more heads per transfer and launch, each
// with a shorter slice, inside the same HBM budget).
inline int64_t rows_of(const hi_ctx* c, int nh) {
  const int64_t r = (c->slice_tokens / nh) / 64 * 64;
  return r < 64 ? 64 : r;
}
inline int64_t head_pitch(const hi_ctx* c, int nh) { return rows_of(c, nh) * 2 * kRowBytes; }
// Algorithm 1, "if h in H_on": the unit's K/V live in HBM (the whole cache in resident mode; the first
// resident_heads (layer, head) pairs, kept behind the ring in the staging buffer, in offload mode)
inline bool unit_resident(const hi_ctx* c, int layer, int head) {
  if (unit_streaming(c, layer, head)) return false;
  return c->mode == HI_MODE_RESIDENT || retr_index(c, layer, head) < c->prob.resident_heads;
}
inline char* res_plane(const hi_ctx* c, int layer, int head, int which) {
  if (c->mode == HI_MODE_RESIDENT) return cache_plane(c, layer, head, which);
  const int64_t plane = c->prob.max_context * kRowBytes;
  return c->staging + c->plan.hbm_resident_offset + (retr_index(c, layer, head) * 2 + which) * plane;
}
// 0 offloaded, 1 HBM-resident, 2 streaming: a head group is of one kind
inline int unit_kind(const hi_ctx* c, int layer, int head) {
  return unit_streaming(c, layer, head) ? 2 : unit_resident(c, layer, head) ? 1 : 0;
}
// a streaming head's bounded store (K plane, then V plane, stream_rows rows each)
inline int64_t stream_head_stride(const hi_ctx* c) { return 2 * c->plan.stream_rows * kRowBytes; }
inline char* stream_plane(const hi_ctx* c, int layer, int head, int which) {
  const int64_t t = c->strm_idx[layer * c->prob.n_kv_heads + head];
  return c->staging + c->plan.hbm_stream_offset + t * stream_head_stride(c) + which * c->plan.stream_rows * kRowBytes;
}

inline char* slot_k(const hi_ctx* c, int slot) { return c->staging + (int64_t)slot * c->slice_tokens * 2 * kRowBytes; }
inline char* slot_v(const hi_ctx* c, int slot, int nh) { return slot_k(c, slot) + rows_of(c, nh) * kRowBytes; }
// where a slot's slice lands when it crosses the link as 4-bit rows: the same planes, link_row bytes per row
inline char* packed_slot(const hi_ctx* c, int slot) {
  return c->staging + c->plan.hbm_packed_offset + (int64_t)slot * c->slice_tokens * 2 * link_row(c);
}

inline int64_t slices_of(const hi_ctx* c, int64_t past, int nh) { return ceil_div(past, rows_of(c, nh)); }

inline bool can_issue(const hi_ctx* c) { return c->seq_issued - c->n_slots < c->seq_consumed; }

void note_peak(hi_ctx* c) {
  const int64_t live = (c->seq_issued - c->seq_consumed) * c->slice_tokens * 2 *
                       (kRowBytes + (link_packed(c) ? link_row(c) : 0));
  if (live > c->stats.peak_staging_bytes) c->stats.peak_staging_bytes = live;
}

hi_status span_begin(hi_ctx* c, int kind, TimedSpan* out, hipStream_t stream = nullptr) {
  TimedSpan s;
  if (!c->span_pool.empty()) {
    s = c->span_pool.back();
    c->span_pool.pop_back();
  } else {
    HI_HIP(hipEventCreate(&s.start));
    HI_HIP(hipEventCreate(&s.stop));
  }
  s.kind = kind;
  HI_HIP(hipEventRecord(s.start, stream ? stream : c->sc));
  *out = s;
  return HI_OK;
}

hi_status span_end(hi_ctx* c, TimedSpan& s, hipStream_t stream = nullptr) {
  HI_HIP(hipEventRecord(s.stop, stream ? stream : c->sc));
  c->spans.push_back(s);
  return HI_OK;
}

// enqueue the H2D of the next not-yet-fetched slice of unit u (all heads of its group)
hi_status issue_slice(hi_ctx* c, hi_ctx::Unit& u) {
  const int64_t i = u.issued;
  const int64_t seq = c->seq_issued;
  const int slot = (int)(seq % c->n_slots);
  const int64_t st = rows_of(c, u.nh);
  const int64_t row0 = i * st;
  int64_t rows = u.past - row0;
  if (rows > st) rows = st;
  if (i == 0) {
    u.first_seq = seq;
    for (int j = 0; j < u.nh; ++j) {
      const int idx = u.layer * c->prob.n_kv_heads + u.head + j;
      if (c->wb_valid[idx]) HI_HIP(hipStreamWaitEvent(c->sh, c->ev_wb[idx], 0));   // rows written by an earlier call
    }
  }
  if (seq >= c->n_slots) HI_HIP(hipStreamWaitEvent(c->sh, c->ev_free[slot], 0));  // slot's previous tenant consumed
  if (!(c->flags & HI_FLAG_SKIP_COPIES)) {
    // The K and V planes of consecutive heads are equally spaced in the cache and in the slot: one strided copy of
    // 2 * nh runs per slice (also for a single head: one call instead of two measured 48 -> 54 GB/s with 8 MiB
    // runs and 55 -> 57.6 GB/s with 64 MiB runs).
    const int64_t lr = link_row(c);
    const char* hk = cache_plane(c, u.layer, u.head, 0) + row0 * lr;
    char* dst = link_packed(c) ? packed_slot(c, slot) : slot_k(c, slot);
    const bool timed = (c->flags & HI_FLAG_TIME_KERNELS) != 0;
    TimedSpan sp;
    if (timed) HI_TRY(span_begin(c, 2, &sp, c->sh));
    HI_HIP(hipMemcpy2DAsync(dst, (size_t)(st * lr), hk, (size_t)(c->prob.max_context * lr), (size_t)(rows * lr),
                            (size_t)(2 * u.nh), hipMemcpyHostToDevice, c->sh));
    if (timed) HI_TRY(span_end(c, sp, c->sh));
    c->stats.n_h2d_copies += 1;
    c->stats.bytes_h2d += 2 * rows * lr * u.nh;
  }
  HI_HIP(hipEventRecord(c->ev_ready[slot], c->sh));
  u.issued += 1;
  c->seq_issued += 1;
  note_peak(c);
  return HI_OK;
}

// fetch as far ahead as free slots allow: first the current unit, then the hinted next one
hi_status top_up(hi_ctx* c, hi_ctx::Unit& cur, hi_ctx::Unit& next) {
  while (cur.valid && cur.issued < cur.n_slices && can_issue(c)) HI_TRY(issue_slice(c, cur));
  if (cur.valid && cur.issued < cur.n_slices) return HI_OK;     // keep FIFO order
  while (next.valid && next.issued < next.n_slices && can_issue(c)) HI_TRY(issue_slice(c, next));
  return HI_OK;
}

// 4-bit link rows: expand the slice that has landed for `slot` into the slot's bf16 planes (compute stream, after
// the wait on the slot's arrival)
hi_status expand_slice(hi_ctx* c, int slot, int64_t rows, int nh) {
  if (!link_packed(c)) return HI_OK;
  const int64_t st = rows_of(c, nh);
  return launch_kv_dequant(c->sc, packed_slot(c, slot), st * link_row(c), slot_k(c, slot), st * kRowBytes, rows, 2 * nh);
}

// a slice has been handed to a kernel (or dropped): its slot becomes free when the compute stream gets here
hi_status retire_slice(hi_ctx* c, int slot) {
  HI_HIP(hipEventRecord(c->ev_free[slot], c->sc));
  c->seq_consumed += 1;
  return HI_OK;
}

constexpr float kIdleGapCapMs = 50.f;     // longer pauses are the caller's (between phases), not the pipeline's

hi_status collect_spans(hi_ctx* c) {
  const TimedSpan* prev_kernel = nullptr;
  for (auto& s : c->spans) {
    HI_HIP(hipEventSynchronize(s.stop));
    float ms = 0.f;
    HI_HIP(hipEventElapsedTime(&ms, s.start, s.stop));
    if (s.kind <= 1) {
      // what stream_compute did between two attention launches: launch latency, the wait for the next staging
      // slice, the expansion of 4-bit slices.  Spans of one stream are in issue order.
      if (prev_kernel) {
        float gap = 0.f;
        if (hipEventElapsedTime(&gap, prev_kernel->stop, s.start) == hipSuccess && gap > 0.f && gap < kIdleGapCapMs)
          c->stats.exposed_copy_ms += gap;
      }
      prev_kernel = &s;
    }
    switch (s.kind) {
      case 0: c->stats.prefill_kernel_ms += ms; break;
      case 1: c->stats.decode_kernel_ms += ms; break;
      case 2: c->stats.h2d_copy_ms += ms; break;
      case 3: c->stats.d2h_copy_ms += ms; break;
      default: c->stats.exposed_copy_ms += ms; break;
    }
    c->span_pool.push_back(s);
  }
  c->spans.clear();
  return HI_OK;
}

// the compute stream waits for a slice
hi_status wait_slice(hi_ctx* c, int slot) {
  HI_HIP(hipStreamWaitEvent(c->sc, c->ev_ready[slot], 0));
  return HI_OK;
}

constexpr int kUnitRing = 16;

// Pace the host: with hundreds of cross-stream waits queued far ahead the copy engine sees gaps between
// consecutive transfers (measured: 45 GB/s free-running against 55 GB/s when at most 1-3 units are queued).
hi_status pace_begin(hi_ctx* c) {
  if (c->run_ahead > 0 && c->n_units >= c->run_ahead)
    HI_HIP(hipEventSynchronize(c->ev_unit[(c->n_units - c->run_ahead) % kUnitRing]));
  return HI_OK;
}

hi_status pace_end(hi_ctx* c) {
  HI_HIP(hipEventRecord(c->ev_unit[c->n_units % kUnitRing], c->sc));
  c->n_units += 1;
  return HI_OK;
}

int pf_variant(const hi_ctx* c) {
  return ((c->flags & HI_FLAG_PREFILL_NARROW) ? 1 : (c->flags & HI_FLAG_PREFILL_DEEP) ? 3 : 0) |
         ((c->flags & HI_FLAG_PREFILL_PAIRED) ? 4 : 0) | ((c->flags & HI_FLAG_PREFILL_UNPAIRED) ? 8 : 0) |
         ((c->flags & HI_FLAG_PREFILL_MFMA32) ? 16 : 0) | (c->prob.q_prescaled ? 32 : 0) |
         ((c->flags & HI_FLAG_PREFILL_8WAVE) ? 64 : 0) | ((c->flags & HI_FLAG_PREFILL_WIDE) ? 128 : 0);
}

bool q_pre(const hi_ctx* c) { return c->prob.q_prescaled != 0; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hi_status check_unit_args(const hi_ctx* c, int layer, int head, int nh, const void* q, const void* k, const void* v,
                          int64_t past, int64_t len, const void* out, int next_layer, int next_head, int next_nh,
                          int64_t next_past) {
  if (!c) { set_last_error("ctx is null"); return HI_ERR_ARG; }
  if (c->failed) {
    set_last_error("an earlier call failed after it had enqueued work: the context can only be synchronised and destroyed");
    return HI_ERR_HIP;
  }
  if (!q || !k || !v || !out) { set_last_error("null buffer"); return HI_ERR_ARG; }
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) { set_last_error("buffers must be 16-byte aligned"); return HI_ERR_ARG; }
  if (layer < 0 || layer >= c->prob.n_layers || head < 0 || nh < 1 || head + nh > c->prob.n_kv_heads) { set_last_error("layer/head out of range"); return HI_ERR_ARG; }
  if (next_layer >= 0 && (next_layer >= c->prob.n_layers || next_head < 0 || next_nh < 1 || next_head + next_nh > c->prob.n_kv_heads || next_past < 0)) {
    set_last_error("prefetch hint out of range");
    return HI_ERR_ARG;
  }
  auto one_kind = [&](int l, int h0, int n) {
    for (int j = 1; j < n; ++j)
      if (unit_kind(c, l, h0 + j) != unit_kind(c, l, h0)) return false;
    return true;
  };
  if (!one_kind(layer, head, nh) || (next_layer >= 0 && !one_kind(next_layer, next_head, next_nh))) {
    set_last_error("a head group must be all HBM-resident, all offloaded or all streaming");
    return HI_ERR_ARG;
  }
  const bool ring_now = unit_kind(c, layer, head) == 0;
  const bool ring_next = next_layer >= 0 && unit_kind(c, next_layer, next_head) == 0;
  if (c->mode == HI_MODE_OFFLOAD && ((ring_now && (int64_t)nh * 64 > c->slice_tokens) || (ring_next && (int64_t)next_nh * 64 > c->slice_tokens))) {
    set_last_error("a staging slice of %lld rows cannot hold 64 rows of each head of the group", (long long)c->slice_tokens);
    return HI_ERR_HBM_BUDGET;
  }
  if ((unit_kind(c, layer, head) != 2 && !c->kv_layer[layer]) ||
      (next_layer >= 0 && unit_kind(c, next_layer, next_head) != 2 && !c->kv_layer[next_layer])) {
    set_last_error("no cache was given for this layer (hi_ctx_create / hi_ctx_set_layer_cache)");
    return HI_ERR_ARG;
  }
  if (past < 0 || len < 1) { set_last_error("negative past_len or empty call"); return HI_ERR_ARG; }
  if (len > c->prob.chunk || past + len > c->prob.max_context) { set_last_error("past_len %lld + len %lld exceeds the plan", (long long)past, (long long)len); return HI_ERR_RANGE; }
  if (next_layer >= 0 && next_past > c->prob.max_context) { set_last_error("prefetch hint beyond max_context"); return HI_ERR_RANGE; }
  return HI_OK;
}

// make `pend` describe (layer, head group, past); drop a stale prefetch if the hint was not honoured
hi_status adopt_unit(hi_ctx* c, int layer, int head, int nh, int64_t past) {
  auto& p = c->pend;
  if (p.valid && (p.layer != layer || p.head != head || p.nh != nh || p.past != past)) {
    for (int64_t i = 0; i < p.issued; ++i) HI_TRY(retire_slice(c, (int)((p.first_seq + i) % c->n_slots)));
    p.valid = false;
  }
  if (!p.valid) {
    p = hi_ctx::Unit();
    p.valid = true;
    p.layer = layer; p.head = head; p.nh = nh; p.past = past;
    p.n_slices = slices_of(c, past, nh);
  }
  return HI_OK;
}

// 4-bit link rows: encode the new rows of an offloaded unit on the compute stream into one of two buffers, then write
// the encoded rows back; a buffer is encoded into again only after the write-back that read it has finished
hi_status write_back_packed(hi_ctx* c, int layer, int head, int nh, const void* k_new, const void* v_new, int64_t past,
                            int64_t len) {
  const int b = c->wbq_turn;
  const int64_t lr = link_row(c);
  char* qk = c->ws + c->plan.ws_writeback_offset + b * (c->plan.ws_writeback_bytes / 2);
  char* qv = qk + (int64_t)nh * len * lr;
  if (2 * (int64_t)nh * len * lr > c->plan.ws_writeback_bytes / 2) { set_last_error("write-back buffer too small"); return HI_ERR_RANGE; }
  c->wbq_turn ^= 1;
  if (c->wbq_valid[b]) HI_HIP(hipStreamWaitEvent(c->sc, c->ev_wbq[b], 0));
  HI_TRY(launch_kv_quant(c->sc, k_new, len * kRowBytes, qk, len * lr, len, nh));
  HI_TRY(launch_kv_quant(c->sc, v_new, len * kRowBytes, qv, len * lr, len, nh));
  HI_HIP(hipEventRecord(c->ev_entry, c->sc));
  HI_HIP(hipStreamWaitEvent(c->sd, c->ev_entry, 0));
  const bool timed = (c->flags & HI_FLAG_TIME_KERNELS) != 0;
  TimedSpan sp;
  if (timed) HI_TRY(span_begin(c, 3, &sp, c->sd));
  if (!(c->flags & HI_FLAG_SKIP_COPIES)) {
    // the heads' K planes (and V planes) are two planes apart in the cache: one strided copy each
    const size_t dpitch = (size_t)(2 * c->prob.max_context * lr), w = (size_t)(len * lr);
    HI_HIP(hipMemcpy2DAsync(cache_plane(c, layer, head, 0) + past * lr, dpitch, qk, w, w, (size_t)nh,
                            hipMemcpyDeviceToHost, c->sd));
    HI_HIP(hipMemcpy2DAsync(cache_plane(c, layer, head, 1) + past * lr, dpitch, qv, w, w, (size_t)nh,
                            hipMemcpyDeviceToHost, c->sd));
    c->stats.bytes_d2h += 2 * len * lr * nh;
    c->stats.n_d2h_copies += 2;
  }
  if (timed) HI_TRY(span_end(c, sp, c->sd));
  HI_HIP(hipEventRecord(c->ev_wbq[b], c->sd));
  c->wbq_valid[b] = 1;
  for (int j = 0; j < nh; ++j) {
    const int idx = layer * c->prob.n_kv_heads + head + j;
    HI_HIP(hipEventRecord(c->ev_wb[idx], c->sd));
    c->wb_valid[idx] = 1;
  }
  return HI_OK;
}

// k_new / v_new: [nh][len][128]
hi_status write_back(hi_ctx* c, int layer, int head, int nh, const void* k_new, const void* v_new, int64_t past,
                     int64_t len) {
  const bool resident = unit_resident(c, layer, head);
  if (!resident && link_packed(c)) return write_back_packed(c, layer, head, nh, k_new, v_new, past, len);
  const bool timed = !resident && (c->flags & HI_FLAG_TIME_KERNELS) != 0;
  TimedSpan sp;
  if (!resident) {
    // the new rows were produced by earlier work on the compute stream
    HI_HIP(hipEventRecord(c->ev_entry, c->sc));
    HI_HIP(hipStreamWaitEvent(c->sd, c->ev_entry, 0));
    if (timed) HI_TRY(span_begin(c, 3, &sp, c->sd));
  }
  if (nh > 1) {
    // the heads' K planes (and V planes) are two planes apart in the cache: one strided copy each
    const hipMemcpyKind kind = resident ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost;
    hipStream_t st = resident ? c->sc : c->sd;
    if (resident || !(c->flags & HI_FLAG_SKIP_COPIES)) {
      const size_t dpitch = (size_t)(2 * c->prob.max_context * kRowBytes), w = (size_t)(len * kRowBytes);
      char* dk = resident ? res_plane(c, layer, head, 0) : cache_plane(c, layer, head, 0);
      char* dv = resident ? res_plane(c, layer, head, 1) : cache_plane(c, layer, head, 1);
      HI_HIP(hipMemcpy2DAsync(dk + past * kRowBytes, dpitch, k_new, w, w, (size_t)nh, kind, st));
      HI_HIP(hipMemcpy2DAsync(dv + past * kRowBytes, dpitch, v_new, w, w, (size_t)nh, kind, st));
      if (!resident) {
        c->stats.bytes_d2h += 2 * len * kRowBytes * nh;
        c->stats.n_d2h_copies += 2;
      }
    }
  }
  for (int j = 0; j < (nh > 1 ? 0 : 1); ++j) {
    char* dk = (resident ? res_plane(c, layer, head + j, 0) : cache_plane(c, layer, head + j, 0)) + past * kRowBytes;
    char* dv = (resident ? res_plane(c, layer, head + j, 1) : cache_plane(c, layer, head + j, 1)) + past * kRowBytes;
    const char* sk = (const char*)k_new + j * len * kRowBytes;
    const char* sv = (const char*)v_new + j * len * kRowBytes;
    if (resident) {
      HI_HIP(hipMemcpyAsync(dk, sk, len * kRowBytes, hipMemcpyDeviceToDevice, c->sc));
      HI_HIP(hipMemcpyAsync(dv, sv, len * kRowBytes, hipMemcpyDeviceToDevice, c->sc));
    } else if (!(c->flags & HI_FLAG_SKIP_COPIES)) {
      HI_HIP(hipMemcpyAsync(dk, sk, len * kRowBytes, hipMemcpyDeviceToHost, c->sd));
      HI_HIP(hipMemcpyAsync(dv, sv, len * kRowBytes, hipMemcpyDeviceToHost, c->sd));
      c->stats.bytes_d2h += 2 * len * kRowBytes;
      c->stats.n_d2h_copies += 2;
    }
  }
  if (!resident) {
    if (timed) HI_TRY(span_end(c, sp, c->sd));
    for (int j = 0; j < nh; ++j) {
      const int idx = layer * c->prob.n_kv_heads + head + j;
      HI_HIP(hipEventRecord(c->ev_wb[idx], c->sd));
      c->wb_valid[idx] = 1;
    }
  }
  return HI_OK;
}

// the cache must be pinned host memory (offload) or device memory (resident)
hi_status check_cache_memory(int mode, const void* p) {
  hipPointerAttribute_t attr;
  const hipError_t e = hipPointerGetAttributes(&attr, p);
  if (mode == HI_MODE_OFFLOAD) {
    if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
      (void)hipGetLastError();
      set_last_error("kv_cache is not pinned host memory");
      return HI_ERR_NOT_PINNED;
    }
  } else if (e != hipSuccess || attr.type != hipMemoryTypeDevice) {
    (void)hipGetLastError();
    set_last_error("resident kv_cache is not device memory");
    return HI_ERR_NOT_PINNED;
  }
  return HI_OK;
}

}  // namespace

extern "C" hi_status hi_ctx_create(const hi_problem* problem, const hi_plan* plan, int32_t mode, void* kv_cache,
                                   void* hbm_staging, void* hbm_workspace, void* stream_compute, void* stream_h2d,
                                   void* stream_d2h, hi_ctx** out) {
  if (!out || !plan) { set_last_error("null argument"); return HI_ERR_ARG; }
  HI_TRY(validate_problem(problem));
  if (mode != HI_MODE_OFFLOAD && mode != HI_MODE_RESIDENT) { set_last_error("unknown mode"); return HI_ERR_ARG; }
  if (!hbm_workspace || ((mode == HI_MODE_OFFLOAD || count_streaming(*problem) > 0) && !hbm_staging)) { set_last_error("null buffer"); return HI_ERR_ARG; }
  if (problem->link_kv_bits == 4 && mode != HI_MODE_OFFLOAD) {
    set_last_error("link_kv_bits = 4 describes the host link: offload mode only");
    return HI_ERR_UNSUPPORTED;
  }
  hi_plan ref;
  HI_TRY(hi_offload_plan(problem, &ref));
  if (std::memcmp(&ref, plan, sizeof(ref)) != 0) { set_last_error("plan does not belong to this problem"); return HI_ERR_ARG; }

  if (kv_cache) HI_TRY(check_cache_memory(mode, kv_cache));
  hipError_t e = hipSuccess;

  hi_ctx* c = new (std::nothrow) hi_ctx();
  if (!c) { set_last_error("out of host memory"); return HI_ERR_ARG; }
  c->prob = *problem;
  c->plan = *plan;
  c->mode = mode;
  {  // head roles, and one pointer for the whole cache: the retrieval heads of all layers back to back
    const int L = problem->n_layers, H = problem->n_kv_heads;
    if (problem->streaming_mask) c->mask.assign(problem->streaming_mask, problem->streaming_mask + (size_t)L * H);
    c->prob.streaming_mask = nullptr;          // the caller's table is not kept
    c->retr_idx.assign((size_t)L * H, -1);
    c->strm_idx.assign((size_t)L * H, -1);
    c->layer_retr0.assign(L, 0);
    int32_t nr = 0, ns = 0;
    for (int l = 0; l < L; ++l) {
      c->layer_retr0[l] = nr;
      for (int h = 0; h < H; ++h) {
        if (head_is_streaming(*problem, c->mask.empty() ? nullptr : c->mask.data(), l, h)) c->strm_idx[(size_t)l * H + h] = ns++;
        else c->retr_idx[(size_t)l * H + h] = nr++;
      }
    }
    c->kv_layer.assign(L, nullptr);
    if (kv_cache)
      for (int l = 0; l < L; ++l) c->kv_layer[l] = (char*)kv_cache + c->layer_retr0[l] * plan->host_bytes_per_head;
  }
  c->staging = (char*)hbm_staging;
  c->ws = (char*)hbm_workspace;
  c->sc = (hipStream_t)stream_compute;
  c->sh = (hipStream_t)stream_h2d;
  c->sd = (hipStream_t)stream_d2h;
  c->n_slots = plan->n_slices_ring;
  c->slice_tokens = plan->slice_tokens;
  std::memset(&c->stats, 0, sizeof(c->stats));
  auto fail = [&](hipError_t err, const char* what) {
    set_last_error("%s failed: %s", what, hipGetErrorString(err));
    hi_ctx_destroy(c);
    return (hi_status)HI_ERR_HIP;
  };
  c->ev_unit.assign(kUnitRing, nullptr);
  for (int i = 0; i < kUnitRing; ++i)
    if ((e = hipEventCreateWithFlags(&c->ev_unit[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
  if (mode == HI_MODE_OFFLOAD) {
    c->ev_ready.assign(c->n_slots, nullptr);
    c->ev_free.assign(c->n_slots, nullptr);
    for (int i = 0; i < c->n_slots; ++i) {
      if ((e = hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
      if ((e = hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
    }
    const int n_heads = problem->n_layers * problem->n_kv_heads;
    c->ev_wb.assign(n_heads, nullptr);
    c->wb_valid.assign(n_heads, 0);
    for (int i = 0; i < n_heads; ++i)
      if ((e = hipEventCreateWithFlags(&c->ev_wb[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
    if ((e = hipEventCreateWithFlags(&c->ev_entry, hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
    if (link_packed(c))
      for (int i = 0; i < 2; ++i)
        if ((e = hipEventCreateWithFlags(&c->ev_wbq[i], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
  }
  *out = c;
  return HI_OK;
}

extern "C" hi_status hi_ctx_destroy(hi_ctx* c) {
  if (!c) return HI_OK;
  for (auto ev : c->ev_ready) if (ev) (void)hipEventDestroy(ev);
  for (auto ev : c->ev_free) if (ev) (void)hipEventDestroy(ev);
  for (auto ev : c->ev_wb) if (ev) (void)hipEventDestroy(ev);
  for (auto ev : c->ev_unit) if (ev) (void)hipEventDestroy(ev);
  if (c->ev_entry) (void)hipEventDestroy(c->ev_entry);
  for (auto ev : c->ev_wbq) if (ev) (void)hipEventDestroy(ev);
  for (auto& s : c->spans) { (void)hipEventDestroy(s.start); (void)hipEventDestroy(s.stop); }
  for (auto& s : c->span_pool) { (void)hipEventDestroy(s.start); (void)hipEventDestroy(s.stop); }
  delete c;
  return HI_OK;
}

extern "C" hi_status hi_ctx_set_layer_cache(hi_ctx* c, int32_t layer, void* kv_layer) {
  if (!c || !kv_layer || layer < 0 || layer >= c->prob.n_layers) { set_last_error("layer cache: bad argument"); return HI_ERR_ARG; }
  HI_TRY(check_cache_memory(c->mode, kv_layer));
  // work that reads or writes the layer's previous rows may still be queued
  HI_HIP(hipStreamSynchronize(c->sh));
  HI_HIP(hipStreamSynchronize(c->sc));
  HI_HIP(hipStreamSynchronize(c->sd));
  if (c->pend.valid && c->pend.layer == layer) {      // a prefetch of the old rows is in the ring: drop it
    for (int64_t i = 0; i < c->pend.issued; ++i) HI_TRY(retire_slice(c, (int)((c->pend.first_seq + i) % c->n_slots)));
    c->pend.valid = false;
  }
  c->kv_layer[layer] = (char*)kv_layer;
  return HI_OK;
}

extern "C" hi_status hi_ctx_set_flags(hi_ctx* c, int32_t flags) {
  if (!c || (flags & ~(HI_FLAG_SKIP_KERNELS | HI_FLAG_SKIP_COPIES | HI_FLAG_TIME_KERNELS | HI_FLAG_PREFILL_NARROW |
                      HI_FLAG_PREFILL_PAIRED | HI_FLAG_PREFILL_DEEP | HI_FLAG_PREFILL_UNPAIRED |
                      HI_FLAG_INJECT_FAILURE | HI_FLAG_PREFILL_MFMA32 | HI_FLAG_PREFILL_8WAVE | HI_FLAG_PREFILL_WIDE |
                      HI_FLAG_PREFILL_SINGLE_SLICES))) { set_last_error("bad flags"); return HI_ERR_ARG; }
  if ((flags & HI_FLAG_PREFILL_8WAVE) && (flags & HI_FLAG_PREFILL_WIDE)) {
    set_last_error("HI_FLAG_PREFILL_8WAVE and HI_FLAG_PREFILL_WIDE exclude each other");
    return HI_ERR_ARG;
  }
  c->flags = flags;
  return HI_OK;
}

extern "C" hi_status hi_ctx_set_run_ahead(hi_ctx* c, int32_t units) {
  if (!c || units < 0 || units >= kUnitRing) { set_last_error("run-ahead must be in [0, %d)", kUnitRing); return HI_ERR_ARG; }
  c->run_ahead = units;
  return HI_OK;
}

// The unit a call names as its successor (not valid: no hint, or an HBM-resident unit, which has nothing to fetch)
static hi_ctx::Unit hinted_unit(const hi_ctx* c, int32_t next_layer, int32_t next_kv_head, int32_t next_nh,
                                int64_t next_past_len) {
  hi_ctx::Unit next;
  if (next_layer >= 0 && unit_kind(c, next_layer, next_kv_head) == 0) {
    next.valid = true;
    next.layer = next_layer; next.head = next_kv_head; next.nh = next_nh; next.past = next_past_len;
    next.n_slices = slices_of(c, next_past_len, next_nh);
  }
  return next;
}

// An HBM-resident unit of an offloading context runs: start (or keep) the prefetch of the hinted offloaded unit
static hi_status prefetch_hint(hi_ctx* c, const hi_ctx::Unit& next) {
  if (c->mode != HI_MODE_OFFLOAD || !next.valid) return HI_OK;
  auto& p = c->pend;
  if (p.valid && (p.layer != next.layer || p.head != next.head || p.nh != next.nh || p.past != next.past)) {
    for (int64_t i = 0; i < p.issued; ++i) HI_TRY(retire_slice(c, (int)((p.first_seq + i) % c->n_slots)));
    p.valid = false;
  }
  if (!p.valid) p = next;
  hi_ctx::Unit none;
  return top_up(c, none, p);
}

// A call runs in two parts: checks that can refuse it (nothing enqueued yet, the cache and the ring untouched), then
// the enqueues.  An error in the second part leaves copies, kernels and the ring's bookkeeping half-advanced - the
// next call could hand a kernel a slot whose copy was never issued - so it closes the context: every later call is
// refused until the context is destroyed.
template <class F>
static hi_status guarded(hi_ctx* c, F&& body) {
  c->enqueuing = false;
  hi_status st = pace_begin(c);
  if (st == HI_OK) st = body();
  if (st == HI_OK) {
    c->enqueuing = true;
    st = pace_end(c);
  }
  if (st != HI_OK && c->enqueuing) c->failed = true;
  c->enqueuing = false;
  return st;
}

// One prefill unit: a group of nh KV heads starting at kv_head (nh = 1: the paper's finest granularity).
static hi_status prefill_impl(hi_ctx* c, int32_t layer, int32_t kv_head, int32_t nh, const void* q_dev,
                              const void* k_new_dev, const void* v_new_dev, int64_t past_len, int32_t chunk_len,
                              void* out_dev, int32_t next_layer, int32_t next_kv_head, int32_t next_nh,
                              int64_t next_past_len) {
  const int G = c->prob.gqa_group;
  const bool run = !(c->flags & HI_FLAG_SKIP_KERNELS);
  const bool timed = (c->flags & HI_FLAG_TIME_KERNELS) != 0;
  PrefillSegment diag{k_new_dev, v_new_dev, chunk_len, 1};
  auto launch = [&](const PrefillSegment& seg, const PrefillSegment& own, int first, int last) -> hi_status {
    TimedSpan sp;
    if (timed) HI_TRY(span_begin(c, 0, &sp));
    HI_TRY(launch_prefill(c->sc, q_dev, G, chunk_len, seg, own, first, last, c->ws, out_dev, c->prob.out_fp32,
                          pf_variant(c), nh, c->plan.ws_partials_offset));
    if (timed) HI_TRY(span_end(c, sp));
    c->stats.n_prefill_kernels += 1;
    return HI_OK;
  };

  // Everything that can be refused is refused here, before the first enqueue: the state images of the chosen
  // kernel must fit the carry, the encoded rows the write-back buffer.
  if (!unit_streaming(c, layer, kv_head)) {
    const PrefillLaunch shape = prefill_launch_shape(G, chunk_len, nh, pf_variant(c), 1, 1);
    if (shape.carry_bytes > c->plan.ws_partials_offset) {
      set_last_error("prefill: the workspace holds %lld bytes of attention state, %lld needed",
                     (long long)c->plan.ws_partials_offset, (long long)shape.carry_bytes);
      return HI_ERR_UNSUPPORTED;
    }
    if (!unit_resident(c, layer, kv_head) && link_packed(c) &&
        2 * (int64_t)nh * chunk_len * link_row(c) > c->plan.ws_writeback_bytes / 2) {
      set_last_error("prefill: write-back buffer too small for %d heads x %d rows", nh, chunk_len);
      return HI_ERR_UNSUPPORTED;
    }
  }
  c->enqueuing = true;
  if (c->flags & HI_FLAG_INJECT_FAILURE) {       // test hook: behave as if a launch had failed half-way
    set_last_error("injected failure");
    return HI_ERR_HIP;
  }

  hi_ctx::Unit next = hinted_unit(c, next_layer, next_kv_head, next_nh, next_past_len);
  if (unit_streaming(c, layer, kv_head)) {
    // Appendix E: attention over what the bounded store holds of the past plus the chunk, then the chunk's rows
    // enter the store; nothing crosses the link
    char* sk = stream_plane(c, layer, kv_head, 0);
    char* sv = stream_plane(c, layer, kv_head, 1);
    HI_TRY(prefetch_hint(c, next));
    if (run) {
      TimedSpan sp;
      if (timed) HI_TRY(span_begin(c, 0, &sp));
      HI_TRY(launch_prefill_window(c->sc, q_dev, G, chunk_len, sk, sv, stream_head_stride(c), k_new_dev, v_new_dev,
                                   past_len, c->prob.sink_tokens, c->prob.recent_tokens, out_dev, c->prob.out_fp32, nh,
                                   q_pre(c)));
      if (timed) HI_TRY(span_end(c, sp));
      c->stats.n_prefill_kernels += 1;
    }
    return launch_stream_store_update(c->sc, k_new_dev, v_new_dev, chunk_len, past_len, c->prob.sink_tokens,
                                      c->prob.recent_tokens, sk, sv, stream_head_stride(c), nh);
  }
  if (unit_resident(c, layer, kv_head)) {
    PrefillSegment pastseg{res_plane(c, layer, kv_head, 0), res_plane(c, layer, kv_head, 1), past_len, 0,
                           2 * c->prob.max_context * kRowBytes};
    HI_TRY(prefetch_hint(c, next));
    if (run) HI_TRY(launch(pastseg, diag, 1, 1));
    return write_back(c, layer, kv_head, nh, k_new_dev, v_new_dev, past_len, chunk_len);
  }

  HI_TRY(adopt_unit(c, layer, kv_head, nh, past_len));
  HI_TRY(write_back(c, layer, kv_head, nh, k_new_dev, v_new_dev, past_len, chunk_len));

  hi_ctx::Unit& cur = c->pend;
  const int64_t ns = cur.n_slices;
  const int64_t st = rows_of(c, nh);
  if (ns == 0 && run) HI_TRY(launch(PrefillSegment{nullptr, nullptr, 0, 0}, diag, 1, 1));
  // Short slices go to the kernel two at a time (one launch over two ring slots, the second slot's rows addressed as
  // a jump inside the past segment): a launch costs a round trip of the softmax state through HBM, a ring to fill
  // and a tail to drain, about 30 us, which is 7 % of a launch over one 16 384-row slice of two heads.  Two slots are
  // half the ring, so the copies of the next pair still run under the kernel of this one.
  const PrefillLaunch shape = prefill_launch_shape(G, chunk_len, nh, pf_variant(c), 1, 1);
  const bool pairs = shape.deep && !(pf_variant(c) & 16) && c->n_slots >= 4 && st / 64 < kPrefillWideMinTiles &&
                     !(c->flags & HI_FLAG_PREFILL_SINGLE_SLICES);
  for (int64_t i = 0; i < ns;) {
    HI_TRY(top_up(c, cur, next));          // guarantees slice i has been fetched
    const int slot = (int)((cur.first_seq + i) % c->n_slots);
    const int slot2 = (int)((cur.first_seq + i + 1) % c->n_slots);
    int64_t rows = past_len - i * st;
    if (rows > st) rows = st;
    int64_t rows2 = past_len - (i + 1) * st;
    if (rows2 > st) rows2 = st;
    const int64_t jump = (slot_k(c, slot2) - slot_k(c, slot)) - st * kRowBytes;
    const bool two = pairs && i + 1 < ns && cur.issued >= i + 2 &&
                     (slot_v(c, slot2, nh) - slot_v(c, slot, nh)) - st * kRowBytes == jump;
    HI_TRY(wait_slice(c, slot));
    if (two) HI_TRY(wait_slice(c, slot2));
    if (run) {
      HI_TRY(expand_slice(c, slot, rows, nh));
      if (two) HI_TRY(expand_slice(c, slot2, rows2, nh));
      const bool is_last = (i + (two ? 2 : 1) == ns);
      PrefillSegment seg{slot_k(c, slot), slot_v(c, slot, nh), rows + (two ? rows2 : 0), 0, head_pitch(c, nh)};
      if (two) {
        seg.jump_rows = st;
        seg.jump_bytes = jump;
      }
      HI_TRY(launch(seg, is_last ? diag : PrefillSegment{nullptr, nullptr, 0, 1}, i == 0, is_last));
    }
    HI_TRY(retire_slice(c, slot));
    if (two) HI_TRY(retire_slice(c, slot2));
    i += two ? 2 : 1;
  }
  cur.valid = false;
  hi_ctx::Unit none;
  HI_TRY(top_up(c, none, next));
  c->pend = next;
  return HI_OK;
}

// One decode unit: the token's rows of a group of nh KV heads.
static hi_status decode_impl(hi_ctx* c, int32_t layer, int32_t kv_head, int32_t nh, const void* q_dev,
                             const void* k_new_dev, const void* v_new_dev, int64_t past_len, void* out_dev,
                             int32_t next_layer, int32_t next_kv_head, int32_t next_nh, int64_t next_past_len) {
  const int G = c->prob.gqa_group;
  const bool run = !(c->flags & HI_FLAG_SKIP_KERNELS);
  const bool timed = (c->flags & HI_FLAG_TIME_KERNELS) != 0;
  float* partials = (float*)(c->ws + c->plan.ws_partials_offset);
  const int64_t part_stride = decode_part_head_stride(c->prob.max_context, c->slice_tokens, c->plan.n_split_decode, G);
  const int64_t part_cap = part_stride / (G * kPartialFloats);       // partials one head may write
  const int n_split = c->plan.n_split_decode / nh > 0 ? c->plan.n_split_decode / nh : 1;
  auto splits_for = [&](int64_t rows) {
    const int64_t need = ceil_div(rows, 64);      // one workgroup covers at least 64 rows
    return (int)(need < n_split ? need : n_split);
  };
  auto partial = [&](const void* k, const void* v, int64_t rows, int np, int part0, int64_t kv_stride,
                     int64_t skip_row = -1) -> hi_status {
    if (part0 + np > part_cap) { set_last_error("decode: partial workspace exhausted"); return HI_ERR_UNSUPPORTED; }
    TimedSpan sp;
    if (timed) HI_TRY(span_begin(c, 1, &sp));
    HI_TRY(launch_decode_partial(c->sc, q_dev, G, k, v, rows, np, partials, part0, q_pre(c), nh, kv_stride, part_stride,
                                 skip_row));
    if (timed) HI_TRY(span_end(c, sp));
    c->stats.n_decode_kernels += 1;
    return HI_OK;
  };

  // refusals come before the first enqueue
  if (unit_kind(c, layer, kv_head) == 0 && slices_of(c, past_len, nh) * n_split > part_cap) {
    set_last_error("decode: the partial workspace cannot hold %lld slices x %d partitions",
                   (long long)slices_of(c, past_len, nh), n_split);
    return HI_ERR_UNSUPPORTED;
  }
  if (unit_kind(c, layer, kv_head) != 0 && n_split > part_cap) {
    set_last_error("decode: the partial workspace cannot hold %d partitions", n_split);
    return HI_ERR_UNSUPPORTED;
  }
  if (unit_kind(c, layer, kv_head) == 0 && link_packed(c) && 2 * (int64_t)nh * link_row(c) > c->plan.ws_writeback_bytes / 2) {
    set_last_error("decode: write-back buffer too small for %d heads", nh);
    return HI_ERR_UNSUPPORTED;
  }
  c->enqueuing = true;
  if (c->flags & HI_FLAG_INJECT_FAILURE) {       // test hook: behave as if a launch had failed half-way
    set_last_error("injected failure");
    return HI_ERR_HIP;
  }

  hi_ctx::Unit next = hinted_unit(c, next_layer, next_kv_head, next_nh, next_past_len);
  if (unit_streaming(c, layer, kv_head)) {
    // Appendix E: the store holds the sink tokens and the n_recent tokens before this one; the oldest of those
    // has just left the window: it takes no part, and the token's row replaces it
    const int64_t n_sink = c->prob.sink_tokens, n_recent = c->prob.recent_tokens;
    const int64_t in_ring = past_len > n_sink ? (past_len - n_sink < n_recent ? past_len - n_sink : n_recent) : 0;
    const int64_t n_store = (past_len < n_sink ? past_len : n_sink) + in_ring;
    const int64_t slot = past_len < n_sink ? past_len : n_sink + (past_len - n_sink) % n_recent;
    const int64_t skip = in_ring == n_recent ? slot : -1;
    char* sk = stream_plane(c, layer, kv_head, 0);
    char* sv = stream_plane(c, layer, kv_head, 1);
    HI_TRY(prefetch_hint(c, next));
    if (!run) {
      for (int j = 0; j < nh; ++j) {
        HI_HIP(hipMemcpyAsync(sk + j * stream_head_stride(c) + slot * kRowBytes, (const char*)k_new_dev + j * kRowBytes,
                              kRowBytes, hipMemcpyDeviceToDevice, c->sc));
        HI_HIP(hipMemcpyAsync(sv + j * stream_head_stride(c) + slot * kRowBytes, (const char*)v_new_dev + j * kRowBytes,
                              kRowBytes, hipMemcpyDeviceToDevice, c->sc));
      }
      return HI_OK;
    }
    int n_part = 0;
    if (n_store > 0) {
      n_part = splits_for(n_store);
      HI_TRY(partial(sk, sv, n_store, n_part, 0, stream_head_stride(c), skip));
    }
    HI_TRY(launch_decode_combine(c->sc, q_dev, G, k_new_dev, v_new_dev, partials, n_part, out_dev, c->prob.out_fp32,
                                 sk + slot * kRowBytes, sv + slot * kRowBytes, q_pre(c), nh, part_stride,
                                 stream_head_stride(c)));
    c->stats.n_combine_kernels += 1;
    return HI_OK;
  }
  if (unit_resident(c, layer, kv_head)) {
    const int64_t plane2 = 2 * c->prob.max_context * kRowBytes;
    int n_part = 0;
    HI_TRY(prefetch_hint(c, next));
    if (run) {
      if (past_len > 0) {
        n_part = splits_for(past_len);
        HI_TRY(partial(res_plane(c, layer, kv_head, 0), res_plane(c, layer, kv_head, 1), past_len, n_part, 0, plane2));
      }
      HI_TRY(launch_decode_combine(c->sc, q_dev, G, k_new_dev, v_new_dev, partials, n_part, out_dev, c->prob.out_fp32,
                                   res_plane(c, layer, kv_head, 0) + past_len * kRowBytes,
                                   res_plane(c, layer, kv_head, 1) + past_len * kRowBytes, q_pre(c), nh, part_stride,
                                   plane2));
      c->stats.n_combine_kernels += 1;
      return HI_OK;
    }
    return write_back(c, layer, kv_head, nh, k_new_dev, v_new_dev, past_len, 1);
  }

  HI_TRY(adopt_unit(c, layer, kv_head, nh, past_len));
  HI_TRY(write_back(c, layer, kv_head, nh, k_new_dev, v_new_dev, past_len, 1));
  hi_ctx::Unit& cur = c->pend;
  const int64_t ns = cur.n_slices;
  const int64_t st = rows_of(c, nh);
  int n_part = 0;
  for (int64_t i = 0; i < ns; ++i) {
    HI_TRY(top_up(c, cur, next));
    const int slot = (int)((cur.first_seq + i) % c->n_slots);
    int64_t rows = past_len - i * st;
    if (rows > st) rows = st;
    HI_TRY(wait_slice(c, slot));
    if (run) {
      HI_TRY(expand_slice(c, slot, rows, nh));
      const int np = splits_for(rows);
      HI_TRY(partial(slot_k(c, slot), slot_v(c, slot, nh), rows, np, n_part, head_pitch(c, nh)));
      n_part += np;
    }
    HI_TRY(retire_slice(c, slot));
  }
  if (run) {
    HI_TRY(launch_decode_combine(c->sc, q_dev, G, k_new_dev, v_new_dev, partials, n_part, out_dev, c->prob.out_fp32,
                                 nullptr, nullptr, q_pre(c), nh, part_stride, 0));
    c->stats.n_combine_kernels += 1;
  }
  cur.valid = false;
  hi_ctx::Unit none;
  HI_TRY(top_up(c, none, next));
  c->pend = next;
  return HI_OK;
}

extern "C" hi_status hi_prefill_group(hi_ctx* c, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                                      const void* k_new_dev, const void* v_new_dev, int64_t past_len,
                                      int32_t chunk_len, void* out_dev, int32_t next_layer, int32_t next_kv_head,
                                      int32_t next_n_heads, int64_t next_past_len) {
  HI_TRY(check_unit_args(c, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, chunk_len, out_dev,
                         next_layer, next_kv_head, next_n_heads, next_past_len));
  return guarded(c, [&] {
    return prefill_impl(c, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, chunk_len, out_dev, next_layer,
                        next_kv_head, next_n_heads, next_past_len);
  });
}

extern "C" hi_status hi_decode_group(hi_ctx* c, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                                     const void* k_new_dev, const void* v_new_dev, int64_t past_len, void* out_dev,
                                     int32_t next_layer, int32_t next_kv_head, int32_t next_n_heads,
                                     int64_t next_past_len) {
  HI_TRY(check_unit_args(c, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, 1, out_dev, next_layer,
                         next_kv_head, next_n_heads, next_past_len));
  return guarded(c, [&] {
    return decode_impl(c, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, past_len, out_dev, next_layer,
                       next_kv_head, next_n_heads, next_past_len);
  });
}

// One token of n_heads HBM-resident KV heads whose histories differ in length (a batch of sequences served as more KV
// heads): one split-KV launch over all of them, each head reading its own number of rows, one combine launch.
extern "C" hi_status hi_decode_group_ragged(hi_ctx* c, int32_t layer, int32_t kv_head, int32_t n_heads, const void* q_dev,
                                            const void* k_new_dev, const void* v_new_dev, const int64_t* past_lens,
                                            void* out_dev) {
  if (!past_lens) { set_last_error("past_lens is null"); return HI_ERR_ARG; }
  if (n_heads < 1 || n_heads > kDecodeMaxRagged) { set_last_error("a ragged call takes 1 to %d heads", kDecodeMaxRagged); return HI_ERR_ARG; }
  int64_t longest = 0;
  for (int j = 0; j < n_heads; ++j) {
    if (past_lens[j] < 0) { set_last_error("negative past_len"); return HI_ERR_ARG; }
    if (past_lens[j] > longest) longest = past_lens[j];
  }
  HI_TRY(check_unit_args(c, layer, kv_head, n_heads, q_dev, k_new_dev, v_new_dev, longest, 1, out_dev, -1, 0, 1, 0));
  if (unit_kind(c, layer, kv_head) != 1) {
    set_last_error("heads of different lengths in one call: HBM-resident heads only (offloaded heads share staging slices "
                   "of one length; call them one by one)");
    return HI_ERR_UNSUPPORTED;
  }
  const int G = c->prob.gqa_group;
  const int64_t part_stride = decode_part_head_stride(c->prob.max_context, c->slice_tokens, c->plan.n_split_decode, G);
  const int64_t part_cap = part_stride / (G * kPartialFloats);
  int n_split = c->plan.n_split_decode / n_heads > 0 ? c->plan.n_split_decode / n_heads : 1;
  const int64_t need = ceil_div(longest, 64);
  if (need < n_split) n_split = (int)need;
  if (n_split > part_cap) { set_last_error("decode: the partial workspace cannot hold %d partitions", n_split); return HI_ERR_UNSUPPORTED; }
  return guarded(c, [&]() -> hi_status {
    c->enqueuing = true;
    if (c->flags & HI_FLAG_SKIP_KERNELS) { set_last_error("a ragged call has no copies to time"); return HI_ERR_UNSUPPORTED; }
    DecodeLens lens = {};
    for (int j = 0; j < n_heads; ++j) lens.n[j] = past_lens[j];
    float* partials = (float*)(c->ws + c->plan.ws_partials_offset);
    const int64_t plane2 = 2 * c->prob.max_context * kRowBytes;
    const bool timed = (c->flags & HI_FLAG_TIME_KERNELS) != 0;
    if (longest > 0) {
      TimedSpan sp;
      if (timed) HI_TRY(span_begin(c, 1, &sp));
      HI_TRY(launch_decode_partial(c->sc, q_dev, G, res_plane(c, layer, kv_head, 0), res_plane(c, layer, kv_head, 1), longest,
                                   n_split, partials, 0, q_pre(c), n_heads, plane2, part_stride, -1, &lens));
      if (timed) HI_TRY(span_end(c, sp));
      c->stats.n_decode_kernels += 1;
    }
    HI_TRY(launch_decode_combine(c->sc, q_dev, G, k_new_dev, v_new_dev, partials, longest > 0 ? n_split : 0, out_dev,
                                 c->prob.out_fp32, res_plane(c, layer, kv_head, 0), res_plane(c, layer, kv_head, 1), q_pre(c),
                                 n_heads, part_stride, plane2, &lens));
    c->stats.n_combine_kernels += 1;
    return HI_OK;
  });
}

extern "C" hi_status hi_prefill_head(hi_ctx* c, int32_t layer, int32_t kv_head, const void* q_dev,
                                     const void* k_new_dev, const void* v_new_dev, int64_t past_len,
                                     int32_t chunk_len, void* out_dev, int32_t next_layer, int32_t next_kv_head,
                                     int64_t next_past_len) {
  return hi_prefill_group(c, layer, kv_head, 1, q_dev, k_new_dev, v_new_dev, past_len, chunk_len, out_dev, next_layer,
                          next_kv_head, 1, next_past_len);
}

extern "C" hi_status hi_decode_head(hi_ctx* c, int32_t layer, int32_t kv_head, const void* q_dev,
                                    const void* k_new_dev, const void* v_new_dev, int64_t past_len, void* out_dev,
                                    int32_t next_layer, int32_t next_kv_head, int64_t next_past_len) {
  return hi_decode_group(c, layer, kv_head, 1, q_dev, k_new_dev, v_new_dev, past_len, out_dev, next_layer,
                         next_kv_head, 1, next_past_len);
}

extern "C" hi_status hi_sync(hi_ctx* c) {
  if (!c) { set_last_error("ctx is null"); return HI_ERR_ARG; }
  HI_HIP(hipStreamSynchronize(c->sh));
  HI_HIP(hipStreamSynchronize(c->sc));
  HI_HIP(hipStreamSynchronize(c->sd));
  return HI_OK;
}

extern "C" hi_status hi_get_stats(hi_ctx* c, hi_stats* out) {
  if (!c || !out) { set_last_error("null argument"); return HI_ERR_ARG; }
  HI_TRY(collect_spans(c));
  *out = c->stats;
  return HI_OK;
}

extern "C" hi_status hi_reset_stats(hi_ctx* c) {
  if (!c) { set_last_error("ctx is null"); return HI_ERR_ARG; }
  HI_TRY(collect_spans(c));
  std::memset(&c->stats, 0, sizeof(c->stats));
  return HI_OK;
}
