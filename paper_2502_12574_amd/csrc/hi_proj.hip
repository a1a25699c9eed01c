// The steps either side of head-wise attention, for gfx950: Q/K/V projection (Section 3.1, Eq. 1: K_t = W_K E(x_t),
// V_t = W_V E(x_t), the query likewise) with the rotary position embedding of the evaluated model fused into its
// epilogue and the results written head-major - the layout the attention calls take - and the output projection
// that consumes the concatenated head outputs (Eq. 9).
//
// Both are one bf16 MFMA contraction D[a][b] = sum_k A[a][k] B[b][k] over two row-major operands whose contraction
// index is contiguous (activations [tokens][features] and weights [out_features][in_features] both are):
//   * a workgroup (4 wavefronts, one per SIMD) owns a 256 x 256 tile of D and walks the contraction in steps of 64;
//     each step's 256 x 64 slices of A and of B (32 KiB each) go HBM/L2 -> LDS by direct-to-LDS 128-bit loads into
//     one of two stages; one barrier per step, placed before the step's last 16 MFMAs, which cover the first operand
//     reads of the next step and the issue of the loads of the step after it;
//   * rows are 128 bytes in LDS; 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7), which makes
//     the 32x32x16 MFMA operand reads (16 lanes = 16 consecutive rows, one chunk each) bank-conflict free;
//   * a wavefront owns 128 rows of A x 128 rows of B (4 x 4 accumulator blocks, 256 accumulator registers): 8
//     operand reads per 16 MFMAs, read one sub-step (16 contraction elements) ahead of their use.  In the Q/K/V
//     projection A is the weight and a wavefront's A rows are one whole head, so the two members of every rotary
//     pair (dimension i and i + 64: blocks ia and ia + 2, same register) meet in one lane;
//   * the tiles of one XCD (workgroups are dealt to the 8 XCDs round-robin) form a compact block of the tile grid
//     and advance through the contraction together, so each operand slice is fetched into that XCD's L2 about once.
//   * workgroups are persistent (one per compute unit, looping over their XCD's tiles): the next tile's first loads
//     are issued under the current tile's epilogue; the epilogue's stores are 16 bytes wide after an exchange between
//     the two half-waves.
// Measured (Llama-3-8B shapes, chunk 16384): 1.05 PFLOP/s for the Q/K/V projection (1.27 without the rotation),
// 1.25 PFLOP/s for the output projection; on constant operands, where the clock is not power-managed, 1.36 / 1.63.
#include <mutex>
#include <type_traits>
#include "hi_device.h"
#include "hi_internal.h"

namespace hi {

typedef __attribute__((address_space(3))) bf16x8* lds_bf16x8_p;

constexpr int kPjTile = 256;                              // rows of A, and of B, per workgroup
constexpr int kPjK = 64;                                  // contraction elements per step
constexpr int kPjRowBytes = kPjK * 2;
constexpr int kPjOperandBytes = kPjTile * kPjRowBytes;    // 32 KiB
constexpr int kPjStageBytes = 2 * kPjOperandBytes;        // A slice then B slice
constexpr int kPjLdsBytes = 2 * kPjStageBytes;            // 128 KiB
constexpr int kPjWaves = 4;
constexpr int kPjWgsPerXcd = 32;

enum { kPjQkv = 0, kPjOut = 1 };

struct ProjArgs {
  const char* a; const char* b;       // operand rows (bf16), contraction index contiguous: A the weight, B the activations
  int a_rows, b_rows;                 // valid rows (loads clamp, the epilogue masks)
  uint32_t a_stride, b_stride;        // bytes between rows
  int64_t b_head_stride;              // kPjOut: B[row][k] is at b + (k / 128) * b_head_stride + row * 256 + (k % 128) * 2
  int K;                              // contraction length, a multiple of 128 (an even number of steps)
  int a_tiles, b_tiles, ga;           // tile grid; tiles are ordered in groups of ga A-tiles (see pj_tile_of)
  int out_fp32;
  // kPjQkv: A = W_qkv [(Hq + 2 Hkv) * 128][K], B = X [C][K]
  void* q_out; void* k_out; void* v_out;   // [Hq][C][128], [Hkv][C][128], [Hkv][C][128]
  int n_q_heads, n_kv_heads;
  const float2* rope;                 // [16][C][4] (cos, sin) of pair 4 g + e at the chunk's token t: [g][t][e]; null: no rotation
  float q_scale;                      // kPjQkv: factor on the query heads' outputs (after the rotation, before rounding)
  // kPjOut: A = W_o [D][Hq * 128], B = attention output [Hq][C][128]
  void* y; int64_t y_stride;          // [C][y_stride] elements
};

// tile j of the grid: groups of ga A-tiles; inside a group B-major with the A-tile index fastest, so that any run of
// consecutive j is a compact block
__device__ __forceinline__ void pj_tile_of(const ProjArgs& p, int j, int& ta, int& tb) {
  const int full = p.a_tiles / p.ga;            // groups of exactly ga A-tiles
  const int per_group = p.ga * p.b_tiles;
  const int g = j / per_group;
  if (g < full) {
    const int w = j - g * per_group;
    ta = g * p.ga + w % p.ga;
    tb = w / p.ga;
  } else {
    const int rem = p.a_tiles - full * p.ga;
    const int w = j - full * per_group;
    ta = full * p.ga + w % rem;
    tb = w / rem;
  }
}

// One rotary pair (x, y) -> (x cos - y sin, y cos + x sin), with the roundings spelled out so that every epilogue
// (and the one-token kernel's caller-visible contract: bf16 output = fp32 output rounded) produces the same bits.
__device__ __forceinline__ float pj_rot_lo(float x, float y, float c, float sn) { return __builtin_fmaf(x, c, -(y * sn)); }
__device__ __forceinline__ float pj_rot_hi(float x, float y, float c, float sn) { return __builtin_fmaf(y, c, x * sn); }

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pj_pack2(float x, float y) {
  const bf16x2 v = {(__bf16)x, (__bf16)y};      // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// Write 16 rows (features 16 rp .. 16 rp + 15 of a 32-row block of D) of this lane's token as bf16 to dst + 2 * row.
// o[0..3] are the lane's rows 16 rp + 4 hl + 0..3, o[4..7] its rows 16 rp + 8 + 4 hl + 0..3: the two half-waves
// exchange, so that each lane stores 8 consecutive rows (16 bytes) at once.
__device__ __forceinline__ void pj_store_rows_bf16(char* dst, const float (&o)[8], int rp, int hl, bool ok) {
  uint32_t x0 = pj_pack2(o[0], o[1]), x1 = pj_pack2(o[2], o[3]);
  uint32_t y0 = pj_pack2(o[4], o[5]), y1 = pj_pack2(o[6], o[7]);
  // lanes < 32 end up with rows 16 rp .. +7 (their own x, then the partner's x), lanes >= 32 with rows 16 rp + 8 .. +15
  auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
  auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
  if (ok) *(uint4*)(dst + (16 * rp + 8 * hl) * 2) = make_uint4(s0[0], s1[0], s0[1], s1[1]);
}

// WIDE: bf16 output in whole runs of 128 features with a 16-byte aligned row pitch (decided by the launcher for the
// whole launch, so that each kernel holds one epilogue only and the accumulators never meet a control-flow join)
template <int MODE, bool WIDE>
__global__ __launch_bounds__(256, 1) void proj_gemm_kernel(ProjArgs p) {
  extern __shared__ __attribute__((aligned(1024))) char lds_dyn[];
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_char*)lds_dyn;
  const int lane = lane_id();
  const int wave = wave_id();
  const int l = lane & 31, hl = lane >> 5;
  const int wa = wave & 1, wb = wave >> 1;      // this wavefront: A rows 128 wa .. +127, B rows 128 wb .. +127

  // Persistent workgroups: XCD x (= blockIdx % 8) owns tiles [x * per, (x + 1) * per) of the ordered list, and its
  // workgroups take them round-robin; a workgroup's next tile starts loading while this one's results are written.
  const int total = p.a_tiles * p.b_tiles;
  const int per = (total + 7) >> 3;
  const int xcd = (int)(blockIdx.x & 7), li = (int)(blockIdx.x >> 3), n_li = (int)(gridDim.x >> 3);
  auto tile_index = [&](int s) __attribute__((always_inline)) { return s < per && xcd * per + s < total ? xcd * per + s : -1; };

  // ---- tile traffic: this wavefront's 8 load instructions per operand cover rows 64 w + 8 u + lane / 8
  uint32_t ga_off[8], gb_off[8];
  auto set_offsets = [&](int ta, int tb) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int row = 64 * wave + 8 * u + (lane >> 3);
      const int chunk = (lane & 7) ^ (4 * (u & 1) + (lane >> 4));      // = (lane & 7) ^ ((row >> 1) & 7)
      int ra = ta * kPjTile + row, rb = tb * kPjTile + row;
      ra = ra < p.a_rows ? ra : p.a_rows - 1;
      rb = rb < p.b_rows ? rb : p.b_rows - 1;
      ga_off[u] = (uint32_t)ra * p.a_stride + (chunk << 4);
      gb_off[u] = (uint32_t)rb * p.b_stride + (chunk << 4);
    }
  };
  // one of the 16 load instructions (8 of A, then 8 of B) of step t's slices into `stage`
  auto issue_one = [&](int t, int stage, int u) __attribute__((always_inline)) {
    const int k0 = t * kPjK;
    const uint32_t la = lds_base + stage * kPjStageBytes + wave * 8192;
    if (u < 8) {
      g2lds16_s<0>(p.a + (int64_t)k0 * 2, ga_off[u], la + u * 1024);
    } else {
      const char* bb = MODE == kPjOut ? p.b + (int64_t)(k0 >> 7) * p.b_head_stride + (k0 & 127) * 2 : p.b + (int64_t)k0 * 2;
      g2lds16_s<0>(bb, gb_off[u - 8], la + kPjOperandBytes + (u - 8) * 1024);
    }
  };

  // ---- operand reads: lane l reads row (32 * block + l), chunk (2 kk + hl), of the A and of the B slice.  The
  // addresses are kept whole in registers per (stage, sub-step), the block is an immediate: no vector ALU work in
  // the loop (with one wavefront per SIMD every such instruction between two MFMAs is matrix-pipe time lost)
  uint32_t va[2][4], vb[2][4];
  {
    const int sw = (l >> 1) & 7;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint32_t ko = (uint32_t)(l * kPjRowBytes + (((2 * kk + hl) ^ sw) << 4));
        va[st][kk] = lds_base + st * kPjStageBytes + wa * 128 * kPjRowBytes + ko;
        vb[st][kk] = lds_base + st * kPjStageBytes + kPjOperandBytes + wb * 128 * kPjRowBytes + ko;
      }
  }
  // operand i of a contraction sub-step, in the order the MFMAs below first need them: A0 B0 A1 A2 A3 B1 B2 B3
  auto read_op = [&](int st, int kk, int i) __attribute__((always_inline)) -> bf16x8 {
    const bool is_a = i == 0 || (i >= 2 && i < 5);
    const int blk = i == 0 ? 0 : i == 1 ? 0 : i < 5 ? i - 1 : i - 4;
    return *(lds_bf16x8_p)((lds_char*)(uintptr_t)(is_a ? va[st][kk] : vb[st][kk]) + blk * 4096);
  };

  const int T = p.K / kPjK;
  int cur_j = tile_index(li);
  if (cur_j < 0) return;
  int ta, tb;
  pj_tile_of(p, cur_j, ta, tb);
  set_offsets(ta, tb);
#pragma unroll
  for (int u = 0; u < 16; ++u) issue_one(0, 0, u);
#pragma unroll
  for (int u = 0; u < 16; ++u) issue_one(1, 1, u);

  for (int s = li; cur_j >= 0; s += n_li) {
    f32x16 acc[4][4];
#pragma unroll
    for (int ia = 0; ia < 4; ++ia)
#pragma unroll
      for (int ib = 0; ib < 4; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ia][ib][r] = 0.f;

    // MFMA j of a sub-step multiplies A block j % 4 with B block j / 4
    auto mfma_j = [&](const bf16x8 (&o)[8], int j) __attribute__((always_inline)) {
      const int ia = j & 3, ib = j >> 2;
      acc[ia][ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o[ia == 0 ? 0 : ia + 1], o[ib == 0 ? 1 : ib + 4], acc[ia][ib], 0, 0, 0);
    };

    // The schedule.  One wavefront per SIMD keeps the matrix pipe busy on its own: operand reads run one sub-step (16
    // contraction elements, 16 MFMAs) ahead of their use, across the step boundary too.  The barrier that publishes
    // step t+1's slices sits before the LAST sub-step of step t, whose MFMAs then cover the first operand reads of
    // step t+1 and the issue of step t+2's loads into the stage step t has just finished reading.  One barrier per
    // step; a wavefront waiting at it still has 16 MFMAs in the pipe.
    bf16x8 cur[8], nxt[8];
    wait_vmcnt<16>();          // step 0 has landed (at most step 1's loads and earlier stores are still in flight)
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) cur[i] = read_op(0, 0, i);

    // MORE1: step t + 1 exists (its first operands are read here); MORE2: step t + 2 exists (its loads are issued here)
    auto step = [&](int t, auto stage_tag, auto more1_tag, auto more2_tag) __attribute__((always_inline)) {
      constexpr int STAGE = decltype(stage_tag)::value;
      constexpr int ST = STAGE, SN = 1 - STAGE;             // this stage and the other one
      constexpr bool MORE1 = decltype(more1_tag)::value, MORE2 = decltype(more2_tag)::value;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < 3; ++kk) {
        // sub-step kk from one operand set while sub-step kk + 1 is read into the other
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          if (j < 8) {
            if (kk & 1) cur[j] = read_op(ST, kk + 1, j); else nxt[j] = read_op(ST, kk + 1, j);
          }
          mfma_j((kk & 1) ? nxt : cur, j);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // every read of this stage has been issued; the last sub-step's operands are in nxt
      wait_vmcnt<0>();                                      // this wave's loads of step t + 1 have landed
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave is done reading this stage
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if (j < 8 && MORE1) cur[j] = read_op(SN, 0, j);
        mfma_j(nxt, j);
        if (MORE2) issue_one(t + 2, STAGE, j);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    // T is even (the contraction length is a multiple of 128): pairs of steps, the last pair without look-ahead.
    // Straight-line code around one loop: the 256 accumulators never meet at a control-flow join.
    int t = 0;
    for (; t + 2 < T; t += 2) {
      step(t, S0(), std::true_type(), std::true_type());
      step(t + 1, S1(), std::true_type(), std::true_type());
    }
    step(t, S0(), std::true_type(), std::false_type());

    // ---- where this wavefront's results go.  Register r of block (ia, ib): A-row 128 wa + 32 ia + 8 (r / 4) + 4 hl
    // + r % 4 (an output feature), B-row 128 wb + 32 ib + l (a token): a lane owns one token and, with its partner in
    // the other half-wave, runs of 8 consecutive features.
    const int my_ta = ta, my_tb = tb;
    char* base = nullptr;        // where feature 0 of this wavefront's 128 A-rows goes, for token 0
    int64_t row_bytes = 0;       // bytes from one token's output row to the next
    bool rotate = false;
    float osc = 1.0f;            // factor on this wavefront's outputs (the query heads' q_scale; 1 is exact)
    int n_valid = 128;           // valid A-rows of the wavefront
    const int esz = p.out_fp32 ? 4 : 2;
    if (MODE == kPjQkv) {
      const int head = 2 * my_ta + wa;
      int hh;
      if (head < p.n_q_heads) { base = (char*)p.q_out; hh = head; }
      else if (head < p.n_q_heads + p.n_kv_heads) { base = (char*)p.k_out; hh = head - p.n_q_heads; }
      else { base = (char*)p.v_out; hh = head - p.n_q_heads - p.n_kv_heads; }
      if (head >= p.n_q_heads + 2 * p.n_kv_heads) n_valid = 0;
      rotate = p.rope != nullptr && head < p.n_q_heads + p.n_kv_heads;
      if (head < p.n_q_heads) osc = p.q_scale;
      base += (int64_t)hh * p.b_rows * kHeadDim * esz;
      row_bytes = (int64_t)kHeadDim * esz;
    } else {
      const int n0 = my_ta * kPjTile + wa * 128;
      base = (char*)p.y + (int64_t)n0 * esz;
      row_bytes = p.y_stride * esz;
      n_valid = p.a_rows - n0 < 128 ? (p.a_rows - n0 > 0 ? p.a_rows - n0 : 0) : 128;
    }
    const int m0 = my_tb * kPjTile + wb * 128 + l;                    // this lane's token in token block 0

    // The rotary table, (cos, sin) of 8 pairs of the lane's token per group (token block ib, pair half ip) of the
    // epilogue, is fetched two groups ahead (each buffer is refilled as soon as its group is rotated): a lone
    // wavefront per SIMD has nobody to hide a load's latency behind (fetched where it is used, the 32 load-wait rounds
    // of a tile took a fifth of its time).  The loads are unconditional and their addresses are a wave-uniform base, one lane
    // offset and immediates: the table of C tokens is [16 groups of 4 pairs][C][4] (cos, sin), 32 bytes per (group,
    // token), and holds a token block's worth of slack behind its last row, so that lanes past the end of a ragged
    // chunk still read inside it.  A wavefront that has no table reads the first bytes of the weights instead and,
    // like a V head, keeps its unrotated values.
    const bool have_table = MODE == kPjQkv && p.rope != nullptr;
    const char* tab_base = have_table ? (const char*)p.rope : p.a;
    const uint32_t group_bytes = have_table ? (uint32_t)p.b_rows * 32u : 0u;
    const uint32_t tab_lane = have_table ? (uint32_t)m0 * 32u + (uint32_t)hl * group_bytes : 0u;
    float4 tab0[8], tab1[8];     // the buffers of pair half 0 and 1 (two arrays: every index is a compile-time constant)
    auto tab_load = [&](int ib, int ip, float4 (&dst)[8]) __attribute__((always_inline)) {
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        // pairs i0 .. i0 + 3 with i0 = 32 ip + 8 rq + 4 hl: group i0 / 4 = 8 ip + 2 rq + hl
        const char* src = tab_base + (size_t)(8 * ip + 2 * rq) * group_bytes;       // wave-uniform
        const float4* cs = (const float4*)(src + tab_lane + ib * 1024);
        dst[2 * rq] = cs[0];
        dst[2 * rq + 1] = cs[1];
      }
    };
    step(t + 1, S1(), std::false_type(), std::false_type());

    // nobody reads LDS after the last barrier: the next tile's first two steps start loading under the epilogue
    cur_j = tile_index(s + n_li);
    if (cur_j >= 0) {
      pj_tile_of(p, cur_j, ta, tb);
      set_offsets(ta, tb);
#pragma unroll
      for (int u = 0; u < 16; ++u) issue_one(0, 0, u);
#pragma unroll
      for (int u = 0; u < 16; ++u) issue_one(1, 1, u);
    }

    if (MODE == kPjQkv) { tab_load(0, 0, tab0); tab_load(0, 1, tab1); }
    if (WIDE) {
      // bf16 output of whole heads / whole 128-feature runs: straight-line code, 16-byte stores
      auto group = [&](int ib, int ip, float4 (&tb8)[8], char* row, bool tok_ok) __attribute__((always_inline)) {
        if (MODE == kPjQkv) __builtin_amdgcn_sched_barrier(0);    // one group at a time: nothing of the next is computed early
        float lo[16], hi[16];                     // blocks ip and ip + 2 hold the rotary pairs
#pragma unroll
        for (int r = 0; r < 16; ++r) { lo[r] = acc[ip][ib][r]; hi[r] = acc[ip + 2][ib][r]; }
        if (MODE == kPjQkv) {
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const float4 c01 = tb8[2 * rq], c23 = tb8[2 * rq + 1];                   // (cos, sin) of two pairs each
            const float cv[4] = {c01.x, c01.z, c23.x, c23.z}, sv[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float x = lo[4 * rq + e], y = hi[4 * rq + e];
              const float xr = pj_rot_lo(x, y, cv[e], sv[e]), yr = pj_rot_hi(x, y, cv[e], sv[e]);
              lo[4 * rq + e] = (rotate ? xr : x) * osc;   // selects, not a branch: V heads keep their values bit for bit
              hi[4 * rq + e] = (rotate ? yr : y) * osc;
            }
          }
          if (ib + 1 < 4) tab_load(ib + 1, ip, tb8);      // the buffer this group has just used: two groups ahead
        }
#pragma unroll
        for (int rp = 0; rp < 2; ++rp) {
          const float l8[8] = {lo[8 * rp], lo[8 * rp + 1], lo[8 * rp + 2], lo[8 * rp + 3],
                               lo[8 * rp + 4], lo[8 * rp + 5], lo[8 * rp + 6], lo[8 * rp + 7]};
          const float h8[8] = {hi[8 * rp], hi[8 * rp + 1], hi[8 * rp + 2], hi[8 * rp + 3],
                               hi[8 * rp + 4], hi[8 * rp + 5], hi[8 * rp + 6], hi[8 * rp + 7]};
          pj_store_rows_bf16(row + 32 * ip * 2, l8, rp, hl, tok_ok);
          pj_store_rows_bf16(row + 32 * (ip + 2) * 2, h8, rp, hl, tok_ok);
        }
      };
#pragma unroll
      for (int ib = 0; ib < 4; ++ib) {
        const int m = m0 + ib * 32;
        const bool tok_ok = m < p.b_rows && n_valid > 0;              // n_valid is 128 or, for a head past the last, 0
        char* row = base + (int64_t)m * row_bytes;                    // only stored to when tok_ok
        group(ib, 0, tab0, row, tok_ok);
        group(ib, 1, tab1, row, tok_ok);
      }
    } else {
      // fp32 output, a ragged last run of features or an odd row pitch: element by element
      int hl_slow = hl;            // opaque per tile: keeps this path's offsets from being hoisted out of the tile loop,
      asm volatile("" : "+v"(hl_slow));   // where they would sit in registers (or scratch) for nothing
      auto group = [&](int ib, int ip, float4 (&tb8)[8], char* row, bool tok_ok) __attribute__((always_inline)) {
        if (MODE == kPjQkv && ib > 0) tab_load(ib, ip, tb8);          // token block 0 was fetched above
        if (!tok_ok) return;
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int f = 32 * (ip + 2 * half) + 8 * (r >> 2) + 4 * hl_slow + (r & 3);
            float x = half ? acc[ip + 2][ib][r] : acc[ip][ib][r];
            if (MODE == kPjQkv && rotate) {
              const float4 cq = tb8[2 * (r >> 2) + ((r & 3) >> 1)];
              const float c = (r & 1) ? cq.z : cq.x, sn = (r & 1) ? cq.w : cq.y;
              const float other = half ? acc[ip][ib][r] : acc[ip + 2][ib][r];
              x = half ? pj_rot_hi(other, x, c, sn) : pj_rot_lo(x, other, c, sn);
            }
            if (MODE == kPjQkv) x *= osc;
            if (f >= n_valid) continue;
            if (p.out_fp32) *(float*)(row + f * 4) = x;
            else *(uint16_t*)(row + f * 2) = float_to_bf16_bits(x);
          }
      };
#pragma unroll
      for (int ib = 0; ib < 4; ++ib) {
        const int m = m0 + ib * 32;
        char* row = base + (int64_t)m * row_bytes;
        group(ib, 0, tab0, row, m < p.b_rows);
        group(ib, 1, tab1, row, m < p.b_rows);
      }
    }
    // The next tile's load offsets are formed again here rather than kept across the epilogue: kept, they are spilled
    // and reloaded, and the waits the compiler then puts before their first uses inside the contraction loop count
    // memory operations it cannot see - they would drain the operand loads that are meant to stay in flight.
    if (cur_j >= 0) {
      int ta2 = ta, tb2 = tb;
      asm volatile("" : "+v"(ta2), "+v"(tb2));
      set_offsets(ta2, tb2);
    }
  }
}

// (cos, sin) of position (past + t) times theta^(-i / 64) for i < 64, in double precision: at a million tokens the
// angle of the fastest pair is a million radians, beyond what fp32 can reduce
struct RopeFreqs { double inv[64]; };
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ out, int64_t past, int n, RopeFreqs f) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * 64) return;
  const int t = idx >> 6, i = idx & 63;
  double s, c;
  sincos((double)(past + t) * f.inv[i], &s, &c);
  out[((int64_t)(i >> 2) * n + t) * 4 + (i & 3)] = make_float2((float)c, (float)s);   // [i / 4][token][i % 4]
}

// ---- one token (decode): the same two projections as matrix-vector products, bound by the HBM read of the weights.
// A wavefront takes pairs of weight rows (for Q/K/V: dimension i and i + 64 of a head, the two members of a rotary
// pair), each lane 16 bytes of every 1 KiB of the row against the matching 16 bytes of x, fp32 accumulation, one
// cross-lane reduction per row.
struct GemvArgs {
  const uint16_t* w;      // [rows][K] bf16
  const uint16_t* x;      // [K] bf16
  int rows, K;
  int mode, out_fp32;
  void* q_out; void* k_out; void* v_out; int n_q_heads, n_kv_heads;   // kPjQkv
  int64_t position; double log2_theta;                                // rotation angle position * 2^(-i/64 * log2_theta); < 0: none
  float q_scale;                                                      // kPjQkv: factor on the query heads' outputs
  void* y;                                                            // kPjOut
};

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ uint4 gemv_load_stream(const uint16_t* p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4*)p);
  return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float gemv_dot8(uint4 a, uint4 b) {
  const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s = __builtin_fmaf(__uint_as_float(av[e] << 16), __uint_as_float(bv[e] << 16), s);
    s = __builtin_fmaf(__uint_as_float(av[e] & 0xFFFF0000u), __uint_as_float(bv[e] & 0xFFFF0000u), s);
  }
  return s;
}

constexpr int kGemvChunks = 8;
__global__ __launch_bounds__(256) void proj_gemv_kernel(GemvArgs g) {
  const int lane = lane_id();
  const int wave_global = blockIdx.x * 4 + wave_id();
  const int n_waves = gridDim.x * 4;
  const int n_pairs = g.mode == kPjQkv ? g.rows / 2 : (g.rows + 1) / 2;
  for (int pr = wave_global; pr < n_pairs; pr += n_waves) {
    int ra, rb;
    if (g.mode == kPjQkv) { ra = (pr >> 6) * kHeadDim + (pr & 63); rb = ra + 64; }
    else { ra = 2 * pr; rb = ra + 1 < g.rows ? ra + 1 : ra; }
    const uint16_t* wa = g.w + (int64_t)ra * g.K;
    const uint16_t* wb = g.w + (int64_t)rb * g.K;
    float sa = 0.f, sb = 0.f;
    // 8 x 512 contraction elements per round: both rows of a Llama-3-8B pair (4096 each) are in flight at once,
    // 16 loads of 16 bytes per lane, instead of two dependent rounds of 8
    for (int k0 = lane * 8; k0 < g.K; k0 += kGemvChunks * 512) {
      uint4 a[kGemvChunks], b[kGemvChunks], xv[kGemvChunks];
#pragma unroll
      for (int c = 0; c < kGemvChunks; ++c) {
        const int k = k0 + c * 512;
        const int kc = k < g.K ? k : 0;                  // in bounds; the product is dropped below
        a[c] = gemv_load_stream(wa + kc);                // the weights are read once: non-temporal
        b[c] = gemv_load_stream(wb + kc);
        xv[c] = *(const uint4*)(g.x + kc);
      }
#pragma unroll
      for (int c = 0; c < kGemvChunks; ++c)
        if (k0 + c * 512 < g.K) { sa += gemv_dot8(a[c], xv[c]); sb += gemv_dot8(b[c], xv[c]); }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { sa += __shfl_xor(sa, off); sb += __shfl_xor(sb, off); }
    if (lane != 0) continue;
    if (g.mode == kPjQkv) {
      const int head = pr >> 6, i = pr & 63;
      char* base;
      int hh;
      if (head < g.n_q_heads) { base = (char*)g.q_out; hh = head; }
      else if (head < g.n_q_heads + g.n_kv_heads) { base = (char*)g.k_out; hh = head - g.n_q_heads; }
      else { base = (char*)g.v_out; hh = head - g.n_q_heads - g.n_kv_heads; }
      float lo = sa, hi = sb;
      if (g.log2_theta >= 0 && head < g.n_q_heads + g.n_kv_heads) {
        double sn, cs;
        sincos((double)g.position * exp2(-(double)i / 64.0 * g.log2_theta), &sn, &cs);
        const float c = (float)cs, s = (float)sn;
        lo = sa * c - sb * s;
        hi = sb * c + sa * s;
      }
      if (head < g.n_q_heads) { lo *= g.q_scale; hi *= g.q_scale; }
      const int64_t at = (int64_t)hh * kHeadDim + i;
      if (g.out_fp32) { ((float*)base)[at] = lo; ((float*)base)[at + 64] = hi; }
      else { ((uint16_t*)base)[at] = float_to_bf16_bits(lo); ((uint16_t*)base)[at + 64] = float_to_bf16_bits(hi); }
    } else {
      if (g.out_fp32) { ((float*)g.y)[ra] = sa; if (rb != ra) ((float*)g.y)[rb] = sb; }
      else { ((uint16_t*)g.y)[ra] = float_to_bf16_bits(sa); if (rb != ra) ((uint16_t*)g.y)[rb] = float_to_bf16_bits(sb); }
    }
  }
}

static hi_status gemv_launch(void* stream, const GemvArgs& g) {
  const int n_pairs = (g.rows + 1) / 2;
  int wgs = (n_pairs + 3) / 4;              // at least one pair per wavefront
  if (wgs > 2048) wgs = 2048;
  hipLaunchKernelGGL(proj_gemv_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("projection (one token) launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

static hi_status pj_launch(void* stream, ProjArgs& p, int mode) {
  static std::once_flag attr_once;      // the projections are stateless: any host thread may get here first
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [] {
    const void* kernels[4] = {(const void*)proj_gemm_kernel<kPjQkv, true>, (const void*)proj_gemm_kernel<kPjQkv, false>,
                              (const void*)proj_gemm_kernel<kPjOut, true>, (const void*)proj_gemm_kernel<kPjOut, false>};
    for (int i = 0; i < 4 && attr_err == hipSuccess; ++i)
      attr_err = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, kPjLdsBytes);
  });
  if (attr_err != hipSuccess) { set_last_error("hipFuncSetAttribute: %s", hipGetErrorString(attr_err)); return HI_ERR_HIP; }
  p.a_tiles = (int)ceil_div(p.a_rows, kPjTile);
  p.b_tiles = (int)ceil_div(p.b_rows, kPjTile);
  p.ga = p.a_tiles / 8 > 0 ? p.a_tiles / 8 : 1;
  const int total = p.a_tiles * p.b_tiles;
  const int per = (total + 7) / 8;
  // persistent workgroups: at most 32 per XCD (one per compute unit), each looping over its share of the tiles
  dim3 grid((unsigned)(8 * (per < kPjWgsPerXcd ? per : kPjWgsPerXcd)));
  // 16-byte stores need bf16 output, whole runs of 128 features per wavefront and an aligned row pitch
  const bool wide = !p.out_fp32 && p.a_rows % 128 == 0 && (mode == kPjQkv || (p.y_stride * 2) % 16 == 0);
  const dim3 block(kPjWaves * 64);
  if (mode == kPjQkv && wide) hipLaunchKernelGGL((proj_gemm_kernel<kPjQkv, true>), grid, block, kPjLdsBytes, (hipStream_t)stream, p);
  else if (mode == kPjQkv) hipLaunchKernelGGL((proj_gemm_kernel<kPjQkv, false>), grid, block, kPjLdsBytes, (hipStream_t)stream, p);
  else if (wide) hipLaunchKernelGGL((proj_gemm_kernel<kPjOut, true>), grid, block, kPjLdsBytes, (hipStream_t)stream, p);
  else hipLaunchKernelGGL((proj_gemm_kernel<kPjOut, false>), grid, block, kPjLdsBytes, (hipStream_t)stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("projection launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

static bool pj_aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

#define HI_PJ_TRY(call)               \
  do {                                \
    hi_status s_ = (call);            \
    if (s_ != HI_OK) return s_;       \
  } while (0)

}  // namespace hi

using namespace hi;

extern "C" hi_status hi_proj_workspace_bytes(int32_t chunk, int64_t* bytes) {
  if (chunk < 1 || !bytes) { set_last_error("projection workspace: bad argument"); return HI_ERR_ARG; }
  // the table of the chunk plus a token block's worth of slack (see the epilogue of proj_gemm_kernel)
  *bytes = (int64_t)chunk * 64 * sizeof(float2) + kPjTile * 32;
  return HI_OK;
}

// hi_qkv_rope and its variant without a workspace argument; the rotary table goes to workspace_dev either way
static hi_status qkv_rope_impl(void* stream, const void* x_dev, const void* w_qkv_dev, int32_t d_model,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t chunk_len, int64_t past_len,
                               double rope_theta, int32_t out_fp32, void* q_out_dev, void* k_out_dev,
                               void* v_out_dev, void* workspace_dev, float q_scale) {
  if (!x_dev || !w_qkv_dev || !q_out_dev || !k_out_dev || !v_out_dev || (rope_theta > 0 && chunk_len > 1 && !workspace_dev)) {
    set_last_error("qkv projection: null buffer");
    return HI_ERR_ARG;
  }
  if (!pj_aligned16(x_dev) || !pj_aligned16(w_qkv_dev) || !pj_aligned16(q_out_dev) || !pj_aligned16(k_out_dev) ||
      !pj_aligned16(v_out_dev) || !pj_aligned16(workspace_dev)) {
    set_last_error("qkv projection: buffers must be 16-byte aligned");
    return HI_ERR_ARG;
  }
  if (n_q_heads < 1 || n_kv_heads < 1 || chunk_len < 1 || past_len < 0 || rope_theta < 0 || (out_fp32 != 0 && out_fp32 != 1) ||
      !(q_scale > 0.0f) || !(q_scale < 3.0e38f)) {
    set_last_error("qkv projection: bad shape");
    return HI_ERR_ARG;
  }
  const int64_t n_out = (int64_t)(n_q_heads + 2 * n_kv_heads) * kHeadDim;
  if (d_model < 2 * kPjK || d_model % (2 * kPjK) != 0 || n_out * d_model * 2 >= (1LL << 32) ||
      (int64_t)chunk_len * d_model * 2 >= (1LL << 32)) {
    set_last_error("qkv projection: d_model must be a multiple of %d and each operand smaller than 4 GiB", 2 * kPjK);
    return HI_ERR_UNSUPPORTED;
  }
  if (chunk_len == 1) {
    GemvArgs g = {};
    g.w = (const uint16_t*)w_qkv_dev; g.x = (const uint16_t*)x_dev;
    g.rows = (int)n_out; g.K = d_model;
    g.mode = kPjQkv; g.out_fp32 = out_fp32;
    g.q_out = q_out_dev; g.k_out = k_out_dev; g.v_out = v_out_dev;
    g.n_q_heads = n_q_heads; g.n_kv_heads = n_kv_heads;
    g.position = past_len;
    g.log2_theta = rope_theta > 0 ? log2(rope_theta) : -1.0;
    g.q_scale = q_scale;
    return gemv_launch(stream, g);
  }
  ProjArgs p = {};
  p.a = (const char*)w_qkv_dev; p.b = (const char*)x_dev;
  p.a_rows = (int)n_out; p.b_rows = chunk_len;
  p.a_stride = (uint32_t)d_model * 2; p.b_stride = (uint32_t)d_model * 2;
  p.K = d_model;
  p.out_fp32 = out_fp32;
  p.q_out = q_out_dev; p.k_out = k_out_dev; p.v_out = v_out_dev;
  p.n_q_heads = n_q_heads; p.n_kv_heads = n_kv_heads;
  p.rope = nullptr;
  p.q_scale = q_scale;
  if (rope_theta > 0) {
    RopeFreqs f;
    for (int i = 0; i < 64; ++i) f.inv[i] = pow(rope_theta, -(double)i / 64.0);
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)ceil_div((int64_t)chunk_len * 64, 256)), dim3(256), 0,
                       (hipStream_t)stream, (float2*)workspace_dev, past_len, chunk_len, f);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_last_error("rope table launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
    p.rope = (const float2*)workspace_dev;
  }
  return pj_launch(stream, p, kPjQkv);
}

extern "C" hi_status hi_qkv_rope(void* stream, const void* x_dev, const void* w_qkv_dev, int32_t d_model,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t chunk_len, int64_t past_len,
                                 double rope_theta, int32_t out_fp32, void* q_out_dev, void* k_out_dev,
                                 void* v_out_dev, void* workspace_dev, float q_scale) {
  return qkv_rope_impl(stream, x_dev, w_qkv_dev, d_model, n_q_heads, n_kv_heads, chunk_len, past_len, rope_theta,
                       out_fp32, q_out_dev, k_out_dev, v_out_dev, workspace_dev, q_scale);
}

// ---- the variant for callers that cannot allocate: the chunk's rotary table lives in a file-scope device array.
// Every GPU holds its own copy of the array at its own address; in host code the array's name is only a stand-in,
// so the address is looked up once per device (with that device current) and only that pointer is handed to kernels.
constexpr int kQkvStaticMaxChunk = 16384;
constexpr int kQkvStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[(size_t)kQkvStaticMaxChunk * 64 * sizeof(float2)];   // 8 MiB

static hi_status qkv_static_scratch(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[kQkvStaticMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_last_error("hipGetDevice: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  if (dev < 0 || dev >= kQkvStaticMaxDevices) { set_last_error("device index %d out of range", dev); return HI_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { set_last_error("hipGetSymbolAddress: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
    ptr_of_device[dev] = p;
  }
  *out = ptr_of_device[dev];
  return HI_OK;
}

extern "C" hi_status hi_qkv_rope_static(void* stream, const void* x_dev, const void* w_qkv_dev, int32_t d_model,
                                        int32_t n_q_heads, int32_t n_kv_heads, int32_t chunk_len, int64_t past_len,
                                        double rope_theta, int32_t out_fp32, void* q_out_dev, void* k_out_dev,
                                        void* v_out_dev, float q_scale) {
  if (chunk_len > kQkvStaticMaxChunk) {
    set_last_error("qkv projection without a workspace: chunk_len %d exceeds the built-in table of %d tokens", chunk_len,
                   kQkvStaticMaxChunk);
    return HI_ERR_RANGE;
  }
  void* table = nullptr;
  HI_PJ_TRY(qkv_static_scratch(&table));
  // the table is rewritten for tokens [0, chunk_len) by every call that rotates: nothing to clear
  return qkv_rope_impl(stream, x_dev, w_qkv_dev, d_model, n_q_heads, n_kv_heads, chunk_len, past_len, rope_theta,
                       out_fp32, q_out_dev, k_out_dev, v_out_dev, table, q_scale);
}

extern "C" hi_status hi_out_proj(void* stream, const void* attn_dev, const void* w_o_dev, int32_t n_q_heads,
                                 int32_t d_model, int32_t chunk_len, int32_t out_fp32, void* y_out_dev) {
  if (!attn_dev || !w_o_dev || !y_out_dev) { set_last_error("output projection: null buffer"); return HI_ERR_ARG; }
  if (!pj_aligned16(attn_dev) || !pj_aligned16(w_o_dev) || !pj_aligned16(y_out_dev)) {
    set_last_error("output projection: buffers must be 16-byte aligned");
    return HI_ERR_ARG;
  }
  if (n_q_heads < 1 || d_model < 1 || chunk_len < 1 || (out_fp32 != 0 && out_fp32 != 1)) {
    set_last_error("output projection: bad shape");
    return HI_ERR_ARG;
  }
  const int64_t K = (int64_t)n_q_heads * kHeadDim;
  if ((int64_t)d_model * K * 2 >= (1LL << 32) || (int64_t)chunk_len * kRowBytes >= (1LL << 32)) {
    set_last_error("output projection: each operand must be smaller than 4 GiB");
    return HI_ERR_UNSUPPORTED;
  }
  if (chunk_len == 1) {                      // one token: the head-major output is the concatenation itself
    GemvArgs g = {};
    g.w = (const uint16_t*)w_o_dev; g.x = (const uint16_t*)attn_dev;
    g.rows = d_model; g.K = (int)K;
    g.mode = kPjOut; g.out_fp32 = out_fp32;
    g.log2_theta = -1.0;
    g.y = y_out_dev;
    return gemv_launch(stream, g);
  }
  ProjArgs p = {};
  p.a = (const char*)w_o_dev; p.b = (const char*)attn_dev;
  p.a_rows = d_model; p.b_rows = chunk_len;
  p.a_stride = (uint32_t)K * 2; p.b_stride = kRowBytes;
  p.b_head_stride = (int64_t)chunk_len * kRowBytes;
  p.K = (int)K;
  p.out_fp32 = out_fp32;
  p.y = y_out_dev; p.y_stride = d_model;
  return pj_launch(stream, p, kPjOut);
}
