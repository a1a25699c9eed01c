// Internal declarations shared by the host-side sources of the library (not part of the ABI).
#pragma once
#include <cstdint>
#include <cstddef>
#include "headinfer.h"

namespace hi {

constexpr int kHeadDim = 128;
constexpr int kRowBytes = kHeadDim * 2;          // one K (or V) row of one head, bf16
constexpr int kLinkRowBytes4 = kHeadDim / 2 + 4 * (kHeadDim / 32);   // a row as 4-bit codes + bf16 scale/zero per 32 channels
constexpr int kWgThreads = 256;                  // 4 wavefronts of 64
constexpr int kCarryFloatsPerLane = 68;          // 64 O^T accumulators + running maxima + row-sum shares (one of each
                                                 // in the 32x32x16 kernels, two in the 16x16x32 kernel)
constexpr int kPartialFloats = kHeadDim + 2;     // O[128], m, l of one (partition, query head)

void set_last_error(const char* fmt, ...);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// query positions covered by one prefill workgroup, and the grid's second dimension, for a GQA group size
inline int prefill_strip(int G) { return 32 * (4 / (G < 4 ? G : 4)); }
inline int prefill_grid_y(int G) { return G > 4 ? G / 4 : 1; }

// The 8-wave prefill kernel covers 2 * strip positions per workgroup.  When a chunk gives it fewer workgroups than
// would fill the chip, `split` workgroups share each block of positions and divide the tiles of every launch
// between them (their states are merged after the unit's last launch).  The launcher picks that kernel when
// workgroups * split reaches kPrefillDeepMinWorkgroups, the 4-wave kernel otherwise.
constexpr int kPrefillFillWorkgroups = 192;
constexpr int kPrefillDeepMinWorkgroups = 128;
constexpr int kPrefillMaxSplit = 8;
inline int prefill_split(int G, int64_t chunk_len, int n_heads = 1) {
  const int64_t wgs = ceil_div(chunk_len, 2 * prefill_strip(G)) * prefill_grid_y(G) * n_heads;
  int split = 1;
  while (wgs * split < kPrefillFillWorkgroups && split < kPrefillMaxSplit) split *= 2;
  return split;
}
// What one launch of a prefill unit looks like (host side; the kernels derive the rest from these numbers).
// variant: low two bits 0 = pick the kernel by chunk length, 1 = 4-wave kernel, 3 = 8-wave kernel; + 4: pair deep and
// shallow blocks in every last launch that has two blocks, + 8: never pair (measurement); + 16: the 8-wave kernel in
// its 32x32x16 MFMA form instead of the 16x16x32 one; + 64 / + 128: the 16x16x32 kernel with 8 wavefronts of 32 query rows
// (prefill_kernel_deep16) / with 4 wavefronts of 64 (prefill_kernel_wide) whatever the launch's length (by default the
// second for launches of kPrefillWideMinTiles tiles and more).
constexpr int kPrefillWideMinTiles = 640;
constexpr int kPdLanes = 512;                   // lanes of an 8-wave workgroup
constexpr int kPrefillPairMinTiles = 4;         // pair when it saves the deepest workgroup at least this many tiles
struct PrefillLaunch {
  int deep;            // 8-wave kernel (else the 4-wave one)
  int split;           // workgroups per block of positions
  int paired;          // balanced partition over (deep, shallow) pairs of blocks
  int nbk;             // blocks of positions per head (8-wave kernel)
  int merge;           // a merge launch follows
  int64_t carry_bytes; // state images the launches of this unit address in the carry
};
inline PrefillLaunch prefill_launch_shape(int G, int64_t chunk_len, int n_heads, int variant, int last, int has_own) {
  PrefillLaunch p;
  const int strip = prefill_strip(G), gy = prefill_grid_y(G), base = variant & 3;
  p.split = prefill_split(G, chunk_len, n_heads);
  p.nbk = (int)ceil_div(chunk_len, 2 * strip);
  p.deep = base == 3 || (base == 0 && (int64_t)p.nbk * gy * n_heads * p.split >= kPrefillDeepMinWorkgroups);
  p.paired = p.merge = 0;
  if (p.deep) {
    // tiles the workgroups of the deepest block sweep beyond the average (the causal triangle), which pairing removes
    const int64_t saved = (int64_t)(2 * strip / 64) * (p.nbk - 1) / (2 * p.split);
    p.paired = last && has_own && p.nbk >= 2 && !(variant & 8) && ((variant & 4) || saved >= kPrefillPairMinTiles);
    p.merge = last && (p.split > 1 || p.paired);
    p.carry_bytes = (int64_t)2 * p.nbk * p.split * gy * n_heads * kPdLanes * kCarryFloatsPerLane * 4;
  } else {
    p.split = 1;
    p.carry_bytes = ceil_div(chunk_len, strip) * gy * n_heads * kWgThreads * kCarryFloatsPerLane * 4;
  }
  return p;
}
// the largest carry any launch of chunks up to C rows over groups of up to n_heads heads can address, whatever the
// kernel variant (both kernels' image counts are step functions of the chunk length with steps at multiples of strip)
inline int64_t prefill_carry_bound(int G, int64_t C, int n_heads) {
  const int strip = prefill_strip(G);
  int64_t worst = 0;
  for (int64_t len = strip; ; len += strip) {
    const int64_t l = len < C ? len : C;
    for (int nh = 1; nh <= n_heads; ++nh)
      for (int variant = 0; variant <= 3; ++variant) {
        if (variant == 2) continue;
        const int64_t need = prefill_launch_shape(G, l, nh, variant, 1, 1).carry_bytes;
        if (need > worst) worst = need;
      }
    if (len >= C) break;
  }
  return worst;
}

// floats of decode partials one head can produce (one launch per staging slice, n_split partials each; a head of
// a group has 1/n of the slice and 1/n of the partitions, up to rounding - hence the factor 2): the distance
// between the heads' partials in the workspace
inline int64_t decode_part_head_stride(int64_t max_context, int64_t slice_tokens, int n_split, int G) {
  return 2 * (ceil_div(max_context, slice_tokens) + 1) * n_split * G * kPartialFloats;
}

hi_status validate_problem(const hi_problem* p);

// Appendix E head roles: is (layer, head) a streaming head?  (the mask if given, else the last streaming_heads heads)
inline bool head_is_streaming(const hi_problem& p, const uint8_t* mask, int layer, int head) {
  if (mask) return mask[(int64_t)layer * p.n_kv_heads + head] != 0;
  return head >= p.n_kv_heads - p.streaming_heads;
}
// streaming heads of all layers
inline int64_t count_streaming(const hi_problem& p) {
  if (!p.streaming_mask) return (int64_t)p.n_layers * p.streaming_heads;
  int64_t n = 0;
  for (int64_t i = 0; i < (int64_t)p.n_layers * p.n_kv_heads; ++i) n += p.streaming_mask[i] != 0;
  return n;
}

// ---- kernel launchers (defined in the .hip files) ------------------------------------------------------
struct PrefillSegment {
  const void* k;      // device, [n][128] bf16 (first head of a group)
  const void* v;
  int64_t n;          // rows
  int causal;         // 1: rows are the chunk's own (row j visible to query i iff j <= i)
  int64_t head_stride = 0;   // bytes from one head's K (V) rows to the next head's, for launches over a head group
  // A past segment may consist of two pieces (two staging slots in one launch): rows [0, jump_rows) start at k / v,
  // the rows after them jump_bytes further on than they would in one piece.  jump_rows is a multiple of 64; 0: one
  // piece.  Only the 16x16x32 8-wave and 4-wave kernels take such a segment.
  int64_t jump_rows = 0;
  int64_t jump_bytes = 0;
};

// One launch of the prefill kernel over up to two KV segments.  first: start from an empty softmax state
// instead of loading the carry; last: normalise and write `out` instead of storing the carry.
// variant: as at prefill_launch_shape (+ 32: the queries are pre-scaled, see softmax_scale_log2); every launch of one
// unit must use the same variant (the carry layouts differ).
// carry_bytes: size of the carry buffer (checked against what the launch will use; -1: not checked).
// n_heads > 1: one launch over a group of KV heads; q is [n_heads][G][chunk_len][128], out likewise, the causal
// segment's rows [n_heads][chunk_len][128], the other segment's heads head_stride bytes apart.
hi_status launch_prefill(void* stream, const void* q, int G, int chunk_len, const PrefillSegment& a,
                         const PrefillSegment& b, int first, int last, void* carry, void* out, int out_fp32,
                         int variant, int n_heads = 1, int64_t carry_bytes = -1);

// The factor between a query-key dot product and the base-2 exponent of its softmax weight: log2(e) / sqrt(128) for
// the q of Eq. 3, 1 for queries that already carry that factor (hi_problem.q_prescaled).
inline float softmax_scale_log2(bool q_prescaled) { return q_prescaled ? 1.0f : 1.4426950408889634f / 11.313708498984761f; }

// rows per head of a decode launch whose heads differ in length (passed to the kernels by value)
constexpr int kDecodeMaxRagged = 64;
struct DecodeLens { int64_t n[kDecodeMaxRagged]; };

// Split-KV decode over rows [0, n) of one slice: writes n_split partials starting at partial index part0.
// n_heads > 1: q is [n_heads][G][128], the heads' K (V) rows kv_head_stride bytes apart, their partials
// part_head_stride floats apart.
// skip_row >= 0: that row takes no part (the row of a streaming head's store that the token replaces).
hi_status launch_decode_partial(void* stream, const void* q, int G, const void* k, const void* v, int64_t n,
                                int n_split, void* partials, int part0, bool q_prescaled, int n_heads = 1,
                                int64_t kv_head_stride = 0,
                                int64_t part_head_stride = 0, int64_t skip_row = -1, const DecodeLens* lens = nullptr);
// lens != null: head h has lens->n[h] rows instead of n (n = the largest of them), and launch_decode_combine appends
// head h's row at row lens->n[h] behind k_append / v_append (which then point at row 0 of the first head)
// Merge n_part partials with the token's own row and write out[G][128]; if k_append/v_append are not null the
// token's K/V row is also copied there (device rows of an HBM-resident cache; heads append_head_stride bytes
// apart).  n_heads > 1: q and out are [n_heads][G][128], k_new / v_new [n_heads][128].
hi_status launch_decode_combine(void* stream, const void* q, int G, const void* k_new, const void* v_new,
                                const void* partials, int n_part, void* out, int out_fp32, void* k_append,
                                void* v_append, bool q_prescaled, int n_heads = 1, int64_t part_head_stride = 0,
                                int64_t append_head_stride = 0, const DecodeLens* lens = nullptr);

// Streaming heads (Appendix E): a head that keeps n_sink initial and n_recent recent tokens in an HBM store of
// n_sink + n_recent rows (sink token j at row j; token j >= n_sink at row n_sink + (j - n_sink) mod n_recent).
constexpr int64_t kStreamMaxRows = 1 << 22;
// One chunk of such a head (a group of n_heads, their stores store_head_stride bytes apart): row past_len + i
// sees key j iff j <= past_len + i and (j < n_sink or past_len + i - j < n_recent); the past comes from the
// store, the chunk's own rows from k_new / v_new.  Layouts of q, k_new, v_new, out as in launch_prefill.
hi_status launch_prefill_window(void* stream, const void* q, int G, int chunk_len, const void* store_k,
                                const void* store_v, int64_t store_head_stride, const void* k_new, const void* v_new,
                                int64_t past_len, int n_sink, int n_recent, void* out, int out_fp32, int n_heads,
                                bool q_prescaled);
// The chunk's rows enter the store (run it after the chunk's attention, on the same stream).
hi_status launch_stream_store_update(void* stream, const void* k_new, const void* v_new, int chunk_len,
                                     int64_t past_len, int n_sink, int n_recent, void* store_k, void* store_v,
                                     int64_t store_head_stride, int n_heads);

// 4-bit rows of the host link: `planes` planes of `rows` rows each, plane p at base + p * pitch on either side
// (bf16 rows of 256 bytes <-> encoded rows of kLinkRowBytes4 bytes).
hi_status launch_kv_quant(void* stream, const void* src, int64_t src_pitch, void* dst, int64_t dst_pitch,
                          int64_t rows, int planes);
hi_status launch_kv_dequant(void* stream, const void* src, int64_t src_pitch, void* dst, int64_t dst_pitch,
                            int64_t rows, int planes);

}  // namespace hi
