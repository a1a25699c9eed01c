// K1: chunked-prefill attention of one (chunk, KV head) unit for gfx950.
//
// Algorithm 1, prefill phase: the chunk's G*C query rows attend over the head's past rows [0, P) (streamed into
// HBM staging) and, causally, over the chunk's own rows (Eq. 3 / Eq. 9).  The evaluation is the usual tiled
// online softmax with fp32 running max / sum / output, built for 64-wide wavefronts and the 32x32x16 bf16 MFMA:
//
//   * The transposed product S^T = K Q^T is computed, so a query row lives in ONE lane column (lane % 32):
//     its running max and sum are per-lane scalars, rescaling O is a per-lane multiply, and the fp32 scores a
//     lane holds are already laid out as the B operand of the second product O^T += V^T P^T once rounded to
//     bf16 - no cross-lane shuffles between the two contractions.
//   * The V^T operand comes from LDS transpose reads (ds_read_b64_tr_b16) of the row-major V tile.
//   * K/V tiles of 64 rows go HBM -> LDS by direct-to-LDS 128-bit loads, swizzled for conflict-free operand
//     reads.
//   * The G query heads at the same positions share a workgroup (for G = 4), so all its waves share the causal
//     boundary and sweep the same K/V tiles.
//   * Workgroups of a unit sweep the K/V rows in near lock-step, so each tile is pulled from HBM about once per
//     XCD and served to the other compute units from that XCD's L2.
//
// Two kernels share this arithmetic: prefill_kernel (4 waves, 2 LDS stages, two workgroups per compute unit, one
// barrier per tile: short chunks) and prefill_kernel_deep (8 waves, one workgroup per compute unit, the two waves of
// a SIMD alternating between a matrix phase and a softmax phase: long chunks, the fast one).
//
// The softmax state (m, l, O) can be carried across launches (one launch per staging slice) in a register-image
// workspace, which is how a unit is computed while later slices of its past are still on the host link.
#include <mutex>
#include <type_traits>
#include "hi_device.h"
#include "hi_internal.h"
#include "hi_prefill_part.h"

namespace hi {

constexpr int kPfTileRows = 64;
constexpr int kPfTileBytes = kPfTileRows * kRowBytes;   // 16 KiB of K (or V)
constexpr int kPfStageBytes = 2 * kPfTileBytes;         // K tile then V tile
constexpr int kPfStages = 2;
constexpr int kPfLdsBytes = kPfStages * kPfStageBytes;  // 64 KiB: two workgroups per compute unit

struct PrefillArgs {
  const uint16_t* q;      // [G][C][128]
  const char* ka; const char* va; int64_t na;   // past segment (not causal)
  const char* kb; const char* vb; int64_t nb;   // the chunk's own rows (causal)
  float* carry;           // [n_wg][66][256]
  void* out;              // [G][C][128]
  int G, C, first, last, out_fp32;
  float c;                // log2(e) / sqrt(d)
  int split;              // 8-wave kernel: workgroups per block of positions (they divide the block's tile sequence)
  int gy;                 // grid y per head; blockIdx.y / gy is the head of a group launch
  int64_t a_head_stride;  // bytes between the heads' rows in the past segment
  int paired;             // 8-wave kernel: deep and shallow blocks of the causal triangle share their tiles
  int nbk;                // 8-wave kernel: blocks of positions per head
  int a_jump_tile;        // the past segment's tiles from this one on lie a_jump_bytes further on (0: one piece)
  int64_t a_jump_bytes;
};

// Group launches: point the arguments at this workgroup's head; returns blockIdx.y within the head.
__device__ __forceinline__ int pf_select_head(PrefillArgs& a) {
  const int head = blockIdx.y / a.gy;
  const int64_t rows = (int64_t)head * a.C;
  a.q += rows * a.G * kHeadDim;
  a.out = (char*)a.out + rows * a.G * kHeadDim * (a.out_fp32 ? 4 : 2);
  a.ka += head * a.a_head_stride;
  a.va += head * a.a_head_stride;
  a.kb += rows * kRowBytes;
  a.vb += rows * kRowBytes;
  return blockIdx.y - head * a.gy;
}

__device__ __forceinline__ int swz_k(int row) { return row & 15; }
__device__ __forceinline__ int swz_v(int row) { return ((row & 3) << 2) | (row & 2); }

// combine a value with the one held by lane ^ 32 (the other 32 K/V rows of the same query row)
__device__ __forceinline__ float max_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Per-lane constants of the tile traffic, computed once per kernel.
struct PfLaneConst {
  uint32_t gk[4];    // global byte offset inside a 64-row K tile of this lane's 4 load instructions
  uint32_t gv;       // same for V (instruction i adds i * 1024)
  uint32_t koff[8];  // LDS byte offset of the K operand read for contraction step kk (sub-block 1 adds 8192)
  uint32_t voff[4];  // LDS byte offset of the V^T transpose read for dim block db (+2048 next 4 rows of the
                     // pair, +4096 second 16-row group, +8192 second sub-block)
};

// One tile's K loads (or V loads) by the whole workgroup of NW wavefronts: 16 / NW instructions per wavefront.
// Full tiles need no vector ALU work at all; the last tile of a segment clamps its row indices (rows past the
// end re-read the last row and are masked by the caller).  lds_tile is the LDS byte address of the 16 KiB tile.
template <int NW>
__device__ __forceinline__ void pf_issue_k(const char* kt, int rows, uint32_t lds_tile, int wave, int lane,
                                           const PfLaneConst& lc) {
  constexpr int NI = 16 / NW;
  const uint32_t ldk = lds_tile + wave * (NI * 1024);
  if (rows >= kPfTileRows) {
    g2lds16_s<0>(kt, lc.gk[0], ldk);
    g2lds16_s<0>(kt, lc.gk[1], ldk + 1024);
    if (NI > 2) {
      g2lds16_s<0>(kt, lc.gk[2], ldk + 2048);
      g2lds16_s<0>(kt, lc.gk[3], ldk + 3072);
    }
  } else {
    const int r_in = lane >> 4;
    const int cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = (wave * NI + i) * 4 + r_in;
      const int rc = r < rows ? r : rows - 1;
      g2lds16_s<0>(kt, (uint32_t)(rc * kRowBytes + ((cpos ^ swz_k(r)) << 4)), ldk + i * 1024);
    }
  }
}

template <int NW>
__device__ __forceinline__ void pf_issue_v(const char* vt, int rows, uint32_t lds_tile, int wave, int lane,
                                           const PfLaneConst& lc) {
  constexpr int NI = 16 / NW;
  const uint32_t ldv = lds_tile + wave * (NI * 1024);
  if (rows >= kPfTileRows) {
    g2lds16_s<0>(vt, lc.gv, ldv);
    g2lds16_s<1024>(vt, lc.gv, ldv);     // the immediate advances the global AND the LDS address
    if (NI > 2) {
      g2lds16_s<2048>(vt, lc.gv, ldv);
      g2lds16_s<3072>(vt, lc.gv, ldv);
    }
  } else {
    const int r_in = lane >> 4;
    const int cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = (wave * NI + i) * 4 + r_in;
      const int rc = r < rows ? r : rows - 1;
      g2lds16_s<0>(vt, (uint32_t)(rc * kRowBytes + ((cpos ^ swz_v(r)) << 4)), ldv + i * 1024);
    }
  }
}

// One stage's tile loads (K tile, then V tile).
template <int NW>
__device__ __forceinline__ void pf_issue_tile(const char* kt, const char* vt, int rows, uint32_t lds_stage,
                                              int wave, int lane, const PfLaneConst& lc) {
  pf_issue_k<NW>(kt, rows, lds_stage, wave, lane, lc);
  pf_issue_v<NW>(vt, rows, lds_stage + kPfTileBytes, wave, lane, lc);
}

typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

struct PfState {
  f32x16 o[4];
  float m, l;
};

// Normalise one query row's accumulators and write out[g][i][:]: register r of block db is dim
// 32*db + 8*(r/4) + 4*hl + r%4; l is this half-wave's part of the row sum.
__device__ __forceinline__ void pf_write_row(void* out, int out_fp32, int C, int g, int i, int hl,
                                             const f32x16 (&o)[4], float l) {
  const float inv = 1.0f / sum_halves(l);
  if (i >= C) return;
  const int64_t base = ((int64_t)g * C + i) * kHeadDim;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int dim = 32 * db + 8 * rq + 4 * hl;
      const float x0 = o[db][4 * rq] * inv, x1 = o[db][4 * rq + 1] * inv;
      const float x2 = o[db][4 * rq + 2] * inv, x3 = o[db][4 * rq + 3] * inv;
      if (out_fp32) {
        *(float4*)((float*)out + base + dim) = make_float4(x0, x1, x2, x3);
      } else {
        uint2 pk;
        pk.x = (uint32_t)float_to_bf16_bits(x0) | ((uint32_t)float_to_bf16_bits(x1) << 16);
        pk.y = (uint32_t)float_to_bf16_bits(x2) | ((uint32_t)float_to_bf16_bits(x3) << 16);
        *(uint2*)((uint16_t*)out + base + dim) = pk;
      }
    }
}


// S^T = K Q^T for one 64-row K tile at kt: register r of sub-block sb is tile row 32*sb + 8*(r/4) + 4*hl + r%4
// (query row = lane % 32).  The two sub-blocks' accumulation chains alternate, so consecutive MFMAs never
// depend on each other.
__device__ __forceinline__ void pf_scores(lds_char* kt, const PfLaneConst& lc, const bf16x8 (&qf)[8],
                                          f32x16 (&s)[2]) {
#pragma unroll
  for (int r = 0; r < 16; ++r) { s[0][r] = 0.f; s[1][r] = 0.f; }
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const bf16x8 k0 = *(lds_bf16x8*)(kt + lc.koff[kk]);
    const bf16x8 k1 = *(lds_bf16x8*)(kt + lc.koff[kk] + 8192);
    s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[kk], s[0], 0, 0, 0);
    s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[kk], s[1], 0, 0, 0);
  }
}

// Online softmax of one tile's scores: per lane = per query row; the other half-wave holds the other 32 rows of
// the tile.  Updates (m, l), rescales O when the running maximum moved, and leaves the probabilities rounded to
// bf16 in pb, laid out as the B operands of the second product.
// mask_rel: rows of the tile with index > mask_rel are masked for this lane (>= 63 means no masking).
__device__ __forceinline__ void pf_softmax(f32x16 (&s)[2], PfState& st, float c, bool masked, int mask_rel, int hl,
                                           bf16x8 (&pb)[2][2]) {
  if (masked) {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
        if (row > mask_rel) s[sb][r] = kNegBig;
      }
  }
  float mx = s[0][0];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
  mx = max_halves(mx);
  const float m_new = fmaxf(st.m, mx);
  if (__builtin_amdgcn_ballot_w64(m_new > st.m) != 0) {
    const float alpha = fast_exp2((st.m - m_new) * c);
    st.l *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    st.m = m_new;
  }
  const float mc = st.m * c;
  float lsum = 0.f;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float p = fast_exp2(__builtin_fmaf(s[sb][8 * u + j], c, -mc));
        lsum += p;
        pb[sb][u][j] = (__bf16)p;
      }
  st.l += lsum;
  // the conversions belong to this phase (the values are first used after the caller's barrier)
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int u = 0; u < 2; ++u) asm volatile("" : "+v"(pb[sb][u]));
}

// Softmax phase of a steady-state tile whose scores left the matrix pipe as s - m (relative to the running
// reference m of the row: the score accumulators start from negm = -m instead of zero), so p = 2^(c (s - m)) is
// one multiplication and one exponential.  The reference only moves when it must: the lane's share of the row sum,
// which the phase needs anyway, bounds every p of the lane, and as long as it stays below kPfSumLimit the p are as
// harmless in fp32 and bf16 as p <= 1 - no maximum is taken at all.  On the rare tile where a lane's sum exceeds
// the limit (or overflowed), the row maxima are formed, O, l, this tile's scores and negm are rescaled in place,
// and the p are computed again.  Measured against taking the maximum of every tile first: 1270 -> 1320 TFLOP/s
// on the same device (32 of the phase's ~145 vector instructions gone).
constexpr float kPfSumLimit = 4096.0f;     // 2^12

__device__ __forceinline__ void pf_softmax_fast(f32x16 (&s)[2], PfState& st, float c, f32x16& negm,
                                                bf16x8 (&pb)[2][2]) {
  // p and the lane's share of the row sum first; the sum bounds every p of the lane, so the row maximum is only
  // needed on the rare tile whose sum says the reference has to move
  auto probs = [&]() __attribute__((always_inline)) {
    float lq[4];                            // four short accumulation chains, each started by its first term
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float p = fast_exp2(s[sb][8 * u + j] * c);
          lq[2 * sb + u] = j == 0 ? p : lq[2 * sb + u] + p;
          pb[sb][u][j] = (__bf16)p;
        }
    return (lq[0] + lq[1]) + (lq[2] + lq[3]);
  };
  float lsum = probs();
  if (__builtin_amdgcn_ballot_w64(!(lsum <= kPfSumLimit)) != 0) {     // also true for inf and NaN
    float mx = s[0][0];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
    mx = max_halves(mx);
    const float d = fmaxf(mx, 0.f);       // lanes whose maximum did not move keep their reference
    const float alpha = fast_exp2(-d * c);
    st.l *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sb][r] -= d;
    st.m += d;
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = -st.m;
    lsum = probs();
  }
  st.l += lsum;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int u = 0; u < 2; ++u) asm volatile("" : "+v"(pb[sb][u]));
}

// O^T += V^T P^T for one 64-row V tile at vt: contraction index 8*hl + j of MFMA (sb,u) is tile row
// 32*sb + 16*u + 8*(j/4) + 4*hl + j%4.
__device__ __forceinline__ void pf_pv(lds_char* vt, const PfLaneConst& lc, const bf16x8 (&pb)[2][2], PfState& st) {
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const bf16x4 v0 = lds_read_tr8(vt + lc.voff[db] + sb * 8192 + u * 4096);
        const bf16x4 v1 = lds_read_tr8(vt + lc.voff[db] + sb * 8192 + u * 4096 + 2048);
        const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[sb][u], st.o[db], 0, 0, 0);
      }
    }
}

// ---- helpers of the 8-wave kernel.  Its LDS holds a ring of K tiles at [0, 64 KiB) and a ring of V tiles at
// [64 KiB, 128 KiB); the lane constants koff / voff are absolute LDS byte addresses (voff includes the V ring's
// base), so that with a compile-time ring slot every operand read is "register + immediate" (the immediate of an
// LDS instruction reaches 64 KiB).
constexpr int kPdWaves = 8;
constexpr int kPdStages = 4;
constexpr uint32_t kPdVRing = 65536;
constexpr int kPdLdsBytes = 2 * kPdStages * kPfTileBytes;   // 128 KiB

// Matrix phase of the alternating schedule: O^T += V^T P^T of the previous tile (V tile at ring offset v_off,
// probabilities pb), then S^T = K Q^T of the next (K tile at ring offset k_off), as ONE software-pipelined
// sequence of 32 MFMAs whose LDS operand reads run kPfAhead steps ahead of their use: a wavefront that has the
// matrix pipe to itself must hide the LDS latency on its own.  Operand i < 16 is the V^T fragment of step
// (sb, u, db) = (i / 8, i / 4 % 2, i % 4); operand 16 + j is the K fragment of step (kk, sb) = (j / 2, j % 2).
constexpr int kPfAhead = 4;

// step i of a matrix phase: which sub-block, half, dim block (i < 16) or contraction step (i >= 16) it is
__device__ __forceinline__ constexpr int pd_sb(int i) { return i < 16 ? i >> 3 : (i - 16) & 1; }
__device__ __forceinline__ constexpr int pd_u(int i) { return (i >> 2) & 1; }
__device__ __forceinline__ constexpr int pd_db(int i) { return i & 3; }
__device__ __forceinline__ constexpr int pd_kk(int i) { return (i - 16) >> 1; }

__device__ __forceinline__ bf16x8 pd_operand(int i, uint32_t v_off, uint32_t k_off, const PfLaneConst& lc) {
  if (i < 16) {
    const int sb = pd_sb(i), u = pd_u(i), db = pd_db(i);
    const uint32_t ad = lc.voff[db] + v_off + sb * 8192 + u * 4096;
    const bf16x4 v0 = lds_read_tr8((lds_char*)(uintptr_t)ad);
    const bf16x4 v1 = lds_read_tr8((lds_char*)(uintptr_t)(ad + 2048));
    return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
  }
  const int kk = pd_kk(i), sb = pd_sb(i);
  return *(lds_bf16x8*)(uintptr_t)(lc.koff[kk] + k_off + sb * 8192);
}

// The tile loads a wavefront issues while it runs a matrix phase: its two K and two V instructions (full tiles
// only; k / v are null otherwise) ride in the gaps between the first MFMAs, where their scalar set-up and the
// issue itself cost next to nothing.
struct PfPhaseLoads {
  const char* k;      // K tile base (global), null: nothing to issue
  const char* v;      // V tile base
  uint32_t ldk, ldv;  // LDS byte address of this wave's first destination row group in the K / V tile
};

// the first kPfAhead operands of a matrix phase (they are V^T fragments), read ahead of the phase
__device__ __forceinline__ void pd_preread(uint32_t v_off, const PfLaneConst& lc, bf16x8 (&pre)[kPfAhead]) {
#pragma unroll
  for (int i = 0; i < kPfAhead; ++i) pre[i] = pd_operand(i, v_off, 0, lc);
}

// PREREAD: the caller has already read the first kPfAhead operands into pre (during its softmax phase).
// CINIT: the score accumulators start from cinit (minus the row's running reference) instead of zero.
// EARLY_BARRIER: the workgroup barrier that ends the phase is passed before the last MFMA is issued instead of after
// it (every LDS operand of the phase is in registers by then), so the barrier's latency and the other group's first
// issue hide under that MFMA; the caller then omits its own barrier.
template <bool LOADS_ALWAYS, bool PREREAD, bool CINIT, bool EARLY_BARRIER = false>
__device__ __forceinline__ void pd_matrix_phase(uint32_t v_off, uint32_t k_off, const PfLaneConst& lc,
                                                const bf16x8 (&qf)[8], const bf16x8 (&pb)[2][2], PfState& st,
                                                f32x16 (&s)[2], const PfPhaseLoads& ld,
                                                const bf16x8 (&pre)[kPfAhead], const f32x16& cinit) {
  static_assert(kPfAhead <= 16, "pre-read operands are V fragments");
  bf16x8 op[kPfAhead + 1];
#pragma unroll
  for (int i = 0; i < kPfAhead; ++i) op[i] = PREREAD ? pre[i] : pd_operand(i, v_off, k_off, lc);
  if (!CINIT) {
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[0][r] = 0.f; s[1][r] = 0.f; }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    if (i + kPfAhead < 32) op[(i + kPfAhead) % (kPfAhead + 1)] = pd_operand(i + kPfAhead, v_off, k_off, lc);
    bf16x8 x = op[i % (kPfAhead + 1)];
    if (EARLY_BARRIER && i == 31) {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x) : : "memory");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    }
    if (i < 16) {
      const int sb = pd_sb(i), u = pd_u(i), db = pd_db(i);
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, pb[sb][u], st.o[db], 0, 0, 0);
    } else {
      const int kk = pd_kk(i), sb = pd_sb(i);
      if (CINIT && kk == 0) s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qf[kk], cinit, 0, 0, 0);
      else s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, qf[kk], s[sb], 0, 0, 0);
    }
    if (i == 1 && (LOADS_ALWAYS || ld.k)) g2lds16_s<0>(ld.k, lc.gk[0], ld.ldk);
    if (i == 3 && (LOADS_ALWAYS || ld.k)) g2lds16_s<0>(ld.k, lc.gk[1], ld.ldk + 1024);
    if (i == 5 && (LOADS_ALWAYS || ld.v)) g2lds16_s<0>(ld.v, lc.gv, ld.ldv);
    if (i == 7 && (LOADS_ALWAYS || ld.v)) g2lds16_s<1024>(ld.v, lc.gv, ld.ldv);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Lane constants of a 4-wavefront workgroup whose LDS stage is a K tile followed by a V tile (offsets relative
// to the tile).
__device__ __forceinline__ PfLaneConst pf_lane_const_4w(int wave, int lane) {
  PfLaneConst lc;
  const int hl = lane >> 5, col = lane & 31;
  const int r_in = lane >> 4, cpos = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (wave * 4 + i) * 4 + r_in;
    lc.gk[i] = (uint32_t)(r * kRowBytes + ((cpos ^ swz_k(r)) << 4));
  }
  const int r0 = wave * 16 + r_in;                // swz_v depends on r & 3 only, so +4 rows = +1024 bytes
  lc.gv = (uint32_t)(r0 * kRowBytes + ((cpos ^ swz_v(r0)) << 4));
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) lc.koff[kk] = (uint32_t)(col * kRowBytes + (((2 * kk + hl) ^ swz_k(col)) << 4));
  const int s16 = lane & 15, q16 = col >> 4;
  const int row_lo = 4 * hl + (s16 >> 2);
#pragma unroll
  for (int db = 0; db < 4; ++db) {
    const int chunk = 4 * db + 2 * q16 + ((s16 & 3) >> 1);
    lc.voff[db] = (uint32_t)(row_lo * kRowBytes + ((chunk ^ swz_v(row_lo)) << 4) + ((s16 & 1) << 3));
  }
  return lc;
}

// One 64-row tile out of the LDS stage starting at kt, straight through.
__device__ __forceinline__ void pf_compute_tile(lds_char* kt, const PfLaneConst& lc, const bf16x8 (&qf)[8],
                                                PfState& st, float c, bool masked, int mask_rel, int hl) {
  f32x16 s[2];
  bf16x8 pb[2][2];
  pf_scores(kt, lc, qf, s);
  pf_softmax(s, st, c, masked, mask_rel, hl, pb);
  pf_pv(kt + kPfTileBytes, lc, pb, st);
}

__global__ __launch_bounds__(256, 2) void prefill_kernel(PrefillArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds_raw[kPfLdsBytes];
  lds_char* lds = (lds_char*)lds_raw;
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
  const int lane = lane_id();
  const int wave = wave_id();
  const int hl = lane >> 5;            // which half of the wavefront
  const int col = lane & 31;           // query row within the wave's 32

  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (4 / gl);
  const int bx = gridDim.x - 1 - blockIdx.x;        // deepest causal rows are dispatched first
  const int g = pf_select_head(a) * 4 + (wave % gl);
  const int i0 = bx * strip + 32 * (wave / gl);     // first query position of this wave
  const int i_hi = bx * strip + strip - 1;          // last query position of the workgroup
  int qi = i0 + col;
  const int my_i = qi;
  if (qi > a.C - 1) qi = a.C - 1;

  const PfLaneConst lc = pf_lane_const_4w(wave, lane);

  // Q^T operand: lane holds q[g][qi][16*kk + 8*hl .. +7]
  bf16x8 qf[8];
  {
    const uint16_t* qrow = a.q + ((int64_t)g * a.C + qi) * kHeadDim + 8 * hl;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *(const uint4*)(qrow + 16 * kk));
  }

  PfState st;
  const int64_t wg_linear = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
  float* carry = a.carry + wg_linear * (kCarryFloatsPerLane * kWgThreads) + threadIdx.x;
  if (a.first) {
    st.m = kNegBig;
    st.l = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
  } else {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] = carry[(db * 16 + r) * kWgThreads];
    st.m = carry[64 * kWgThreads];
    st.l = carry[65 * kWgThreads];
  }
  // the compiler's own waits for the loads above belong here, not inside the tile loop
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(qf[kk]));
  asm volatile("" : "+v"(st.m), "+v"(st.l));
#pragma unroll
  for (int db = 0; db < 4; ++db) asm volatile("" : "+v"(st.o[db]));

  // tiles: segment A (all of it), then the part of segment B at or below the workgroup's causal boundary
  const int ta = (int)((a.na + kPfTileRows - 1) / kPfTileRows);
  const int64_t nb_vis = a.nb < (int64_t)i_hi + 1 ? a.nb : (int64_t)i_hi + 1;
  const int tb = (int)((nb_vis + kPfTileRows - 1) / kPfTileRows);
  const int T = ta + tb;

  auto issue = [&](int t) {
    const uint32_t stage = lds_base + (uint32_t)(t & (kPfStages - 1)) * kPfStageBytes;
    if (t < ta) {
      const int64_t row0 = (int64_t)t * kPfTileRows;
      const int64_t left = a.na - row0;
      pf_issue_tile<4>(a.ka + row0 * kRowBytes, a.va + row0 * kRowBytes, left < kPfTileRows ? (int)left : kPfTileRows,
                       stage, wave, lane, lc);
    } else {
      const int64_t row0 = (int64_t)(t - ta) * kPfTileRows;
      const int64_t left = a.nb - row0;
      pf_issue_tile<4>(a.kb + row0 * kRowBytes, a.vb + row0 * kRowBytes, left < kPfTileRows ? (int)left : kPfTileRows,
                       stage, wave, lane, lc);
    }
  };

  if (T > 0) issue(0);

  const float c = a.c;
  // one tile: wait for it, let everybody see it (and be done with the previous one), refill the freed stage,
  // compute.  The loop is unrolled by the two LDS stages so every LDS address is an immediate and the
  // accumulators never meet at a control-flow join inside the loop.
  auto step = [&](int t, auto stage_tag) {
    constexpr int STAGE = decltype(stage_tag)::value;
    wait_vmcnt<0>();
    __syncthreads();
    if (t + 1 < T) issue(t + 1);
    // masks: rows past the end of the segment, and (chunk's own rows) rows after the query's position
    const bool in_b = t >= ta;
    const int64_t j0 = (int64_t)(in_b ? (t - ta) : t) * kPfTileRows;
    const int64_t n_seg = in_b ? a.nb : a.na;
    const bool masked = (j0 + kPfTileRows > n_seg) || (in_b && (j0 + kPfTileRows - 1 > i0));
    int rel = kPfTileRows;
    if (masked) {
      int64_t lim = n_seg - 1;                       // last visible row index
      if (in_b && (int64_t)my_i < lim) lim = my_i;
      const int64_t d = lim - j0;
      rel = d < -1 ? -1 : (d > kPfTileRows ? kPfTileRows : (int)d);
    }
    pf_compute_tile(lds + STAGE * kPfStageBytes, lc, qf, st, c, masked, rel, hl);
  };
  int t = 0;
  for (; t + 1 < T; t += 2) {
    step(t, std::integral_constant<int, 0>());
    step(t + 1, std::integral_constant<int, 1>());
  }
  if (t < T) step(t, std::integral_constant<int, 0>());

  if (!a.last) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) carry[(db * 16 + r) * kWgThreads] = st.o[db][r];
    carry[64 * kWgThreads] = st.m;
    carry[65 * kWgThreads] = st.l;
    return;
  }

  pf_write_row(a.out, a.out_fp32, a.C, g, my_i, hl, st.o, st.l);
}

// ---------------------------------------------------------------------------------------------------------
// The 8-wave kernel: 8 wavefronts per workgroup (two per SIMD, 32 positions each: the G query heads at 64
// positions for G = 4), one workgroup per compute unit, four K and four V tiles in LDS, every K/V byte pulled
// from L2 serves 256 query rows.  The two wavefronts of a SIMD alternate between a matrix phase and a softmax
// phase (see the schedule below); used for chunks long enough to give every compute unit a workgroup.
__global__ __launch_bounds__(512, 2) void prefill_kernel_deep(PrefillArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char lds_dyn[];
  lds_char* lds = (lds_char*)lds_dyn;
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
  const int lane = lane_id();
  const int wave = wave_id();
  const int hl = lane >> 5;
  const int col = lane & 31;

  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (kPdWaves / gl);
  const int g = pf_select_head(a) * 4 + (wave % gl);

  PfLaneConst lc;
  {
    const int r_in = lane >> 4, cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = (wave * 2 + i) * 4 + r_in;
      lc.gk[i] = (uint32_t)(r * kRowBytes + ((cpos ^ swz_k(r)) << 4));
    }
    lc.gk[2] = lc.gk[3] = 0;
    const int r0 = wave * 8 + r_in;
    lc.gv = (uint32_t)(r0 * kRowBytes + ((cpos ^ swz_v(r0)) << 4));
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      lc.koff[kk] = lds_base + (uint32_t)(col * kRowBytes + (((2 * kk + hl) ^ swz_k(col)) << 4));
    const int s16 = lane & 15, q16 = col >> 4;
    const int row_lo = 4 * hl + (s16 >> 2);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const int chunk = 4 * db + 2 * q16 + ((s16 & 3) >> 1);
      lc.voff[db] = lds_base + kPdVRing +
                    (uint32_t)(row_lo * kRowBytes + ((chunk ^ swz_v(row_lo)) << 4) + ((s16 & 1) << 3));
    }
  }


  // How the launch divides its tiles among workgroups is pure arithmetic on the launch's shape: at most two passes
  // per workgroup, each over a range of one block's tile sequence (its past tiles, then the chunk's own tiles up to
  // the block's causal boundary), each with a softmax state of its own.
  PfShape sh;
  sh.nbk = a.nbk; sh.m = strip / kPfTileRows;
  sh.ta = (int)((a.na + kPfTileRows - 1) / kPfTileRows);
  sh.tb_all = (int)((a.nb + kPfTileRows - 1) / kPfTileRows);
  sh.split = a.split; sh.paired = a.paired; sh.carried = !a.first;
  constexpr int kLanes = kPdWaves * 64;
  constexpr int kImageFloats = kCarryFloatsPerLane * kLanes;
  float* const images = a.carry + (int64_t)blockIdx.y * pf_images_per_row(a.nbk, a.split) * kImageFloats + threadIdx.x;
  // the pass that holds past tiles goes first, so that the workgroups of a range walk the past rows in step
  int first_which = 0;
  {
    const PfPass d = pf_pass(sh, blockIdx.x, 0, a.last), sw = pf_pass(sh, blockIdx.x, 1, a.last);
    if (sw.run && sw.a1 > sw.a0 && !(d.run && d.a1 > d.a0)) first_which = 1;
  }
#pragma nounroll
  for (int pi = 0; pi < 2; ++pi) {
    const PfPass ps = pf_pass(sh, blockIdx.x, first_which ^ pi, a.last);
    if (ps.init) {                 // a range without tiles in the first launch of a unit: an empty state
      float* im = images + (int64_t)ps.store * kImageFloats;
#pragma unroll
      for (int i = 0; i < 64; ++i) im[i * kLanes] = 0.f;
      im[64 * kLanes] = kNegBig;
      im[65 * kLanes] = 0.f;
    }
    if (!ps.run) continue;
    __syncthreads();               // the LDS rings are free again (a previous pass may still be reading V tiles)
    const int bx = ps.bx;
    const int i0 = bx * strip + 32 * (wave / gl);
    int qi = i0 + col;
    const int my_i = qi;
    if (qi > a.C - 1) qi = a.C - 1;

    // Q^T operand: lane holds q[g][qi][16*kk + 8*hl .. +7]
    bf16x8 qf[8];
    {
      const uint16_t* qrow = a.q + ((int64_t)g * a.C + qi) * kHeadDim + 8 * hl;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *(const uint4*)(qrow + 16 * kk));
    }

    // this pass's tiles: past rows [64 a0, min(64 a1, na)) of the launch, own tiles [b0, b1) of the chunk
    const char* const ka_p = a.ka + (int64_t)ps.a0 * kPfTileBytes;
    const char* const va_p = a.va + (int64_t)ps.a0 * kPfTileBytes;
    int64_t na_p = (int64_t)ps.a1 * kPfTileRows;
    if (na_p > a.na) na_p = a.na;
    na_p -= (int64_t)ps.a0 * kPfTileRows;
    const int b_t0 = ps.b0;
    const int tb = ps.b1 - ps.b0;

    PfState st;
    if (ps.load < 0) {
      st.m = kNegBig;
      st.l = 0.f;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
    } else {
      const float* im = images + (int64_t)ps.load * kImageFloats;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][r] = im[(db * 16 + r) * kLanes];
      st.m = im[64 * kLanes];
      st.l = im[65 * kLanes];
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(qf[kk]));
    asm volatile("" : "+v"(st.m), "+v"(st.l));
#pragma unroll
    for (int db = 0; db < 4; ++db) asm volatile("" : "+v"(st.o[db]));

    const int ta = (int)((na_p + kPfTileRows - 1) / kPfTileRows);
    const int T = ta + tb;
    const int tb_base = b_t0 - ta;      // tile t >= ta of the sweep is tile t + tb_base of the chunk's own rows

    // K tile t (which = 0) or V tile t (which = 1) of the sweep: this wave's share of its loads
    auto issue = [&](int t, int which) __attribute__((always_inline)) {
      if (t >= T) return;
      const bool in_b = t >= ta;
      const int64_t row0 = (int64_t)(in_b ? t + tb_base : t) * kPfTileRows;
      const int64_t left = (in_b ? a.nb : na_p) - row0;
      const int rows = left < kPfTileRows ? (int)left : kPfTileRows;
      const uint32_t slot = lds_base + (uint32_t)(t & (kPdStages - 1)) * kPfTileBytes;
      if (which == 0) pf_issue_k<kPdWaves>((in_b ? a.kb : ka_p) + row0 * kRowBytes, rows, slot, wave, lane, lc);
      else pf_issue_v<kPdWaves>((in_b ? a.vb : va_p) + row0 * kRowBytes, rows, slot + kPdVRing, wave, lane, lc);
    };
    // Every wave issues, in this order: K0 | K1 V0 | K2 V1 | then, in the matrix phase of tile t, K(t+3) V(t+2)
    // (2 instructions each).  The one wait per tile is at the end of the softmax phase of tile t: everything up to
    // V(t+1) has landed when at most K(t+3) V(t+2) are still in flight.
    auto wait_landed = [&](int t) {
      if (t + 3 < T) wait_vmcnt<4>();
      else wait_vmcnt<0>();
    };
    auto phase_barrier = [&]() {
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
    };

    // The two wavefronts of a SIMD alternate: while one runs its matrix phase (O += V P of the previous tile, then
    // the scores of the next), the other runs its softmax phase on the vector ALU.  Both groups execute the same
    // program with two barriers per tile; group 1 passes one extra barrier first, so it is always one phase behind
    // (and group 0 passes one extra at the end: every wave executes the same number of barriers).
    //   phase index (barriers passed so far):  group 0: matrix(t) = 2t, softmax(t) = 2t + 1;  group 1: one later.
    //   Reads: K(t) in phases 2t, 2t+1; V(t) in phases 2t+1 (operands read ahead during softmax(t)) .. 2t+3.
    //   Writes: K(t+3) replaces K(t-1) (last read in phase 2t-1) and V(t+2) replaces V(t-2) (last read in phase
    //   2t-1): both are issued in matrix(t), phase >= 2t.
    //   Landing: each wave waits at the end of softmax(t-1) for its share of everything up to V(t): that is phase
    //   2t at the latest, and K(t+1) is first read in phase 2t+2, V(t) in phase 2t+1.
    const int group = wave >> 2;       // waves w and w + 4 share a SIMD
    const float c = a.c;
    wait_vmcnt<0>();                   // the waits below count this pass's tile loads only (a previous pass's stores are done)
    issue(0, 0);
    issue(1, 0); issue(0, 1);
    issue(2, 0); issue(1, 1);
    wait_landed(-1);                           // K(0), K(1), V(0)
    phase_barrier();
    if (group == 1) phase_barrier();

    f32x16 sc[2];
    bf16x8 pb[2][2];
    auto softmax_phase = [&](int t) __attribute__((always_inline)) {
      const bool in_b = t >= ta;
      const int64_t j0 = (int64_t)(in_b ? t + tb_base : t) * kPfTileRows;
      const int64_t n_seg = in_b ? a.nb : na_p;
      const bool masked = (j0 + kPfTileRows > n_seg) || (in_b && (j0 + kPfTileRows - 1 > i0));
      int rel = kPfTileRows;
      if (masked) {
        int64_t lim = n_seg - 1;
        if (in_b && (int64_t)my_i < lim) lim = my_i;
        const int64_t d = lim - j0;
        rel = d < -1 ? -1 : (d > kPfTileRows ? kPfTileRows : (int)d);
      }
      pf_softmax(sc, st, c, masked, rel, hl, pb);
    };
    // tile 0: nothing to accumulate yet
    issue(3, 0);
    issue(2, 1);
#pragma unroll
    for (int r = 0; r < 16; ++r) { sc[0][r] = 0.f; sc[1][r] = 0.f; }
#pragma unroll
    for (int i = 16; i < 32; ++i)
      sc[pd_sb(i)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pd_operand(i, 0, 0, lc), qf[pd_kk(i)], sc[pd_sb(i)], 0, 0, 0);
    phase_barrier();
    softmax_phase(0);
    wait_landed(0);
    phase_barrier();
    bf16x8 pre[kPfAhead];
    f32x16 negm;       // minus the row's running reference, the start value of the steady-state score accumulators
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = 0.f;
    // any tile t >= 1
    auto generic_tile = [&](int t) __attribute__((always_inline)) {
      // K(t+3) and V(t+2): full tiles are issued from inside the matrix phase, partial ones (row clamping) here
      PfPhaseLoads ld;
      ld.k = ld.v = nullptr;
      const int tk = t + 3, tv = t + 2;
      const bool kb = tk >= ta, vb = tv >= ta;
      const int64_t krow0 = (int64_t)(kb ? tk + tb_base : tk) * kPfTileRows;
      const int64_t vrow0 = (int64_t)(vb ? tv + tb_base : tv) * kPfTileRows;
      const bool kfull = tk < T && (kb ? a.nb : na_p) - krow0 >= kPfTileRows;
      const bool vfull = tv < T && (vb ? a.nb : na_p) - vrow0 >= kPfTileRows;
      if (kfull) ld.k = (kb ? a.kb : ka_p) + krow0 * kRowBytes; else issue(tk, 0);
      if (vfull) ld.v = (vb ? a.vb : va_p) + vrow0 * kRowBytes; else issue(tv, 1);
      ld.ldk = lds_base + (uint32_t)(tk & (kPdStages - 1)) * kPfTileBytes + wave * 2048;
      ld.ldv = lds_base + kPdVRing + (uint32_t)(tv & (kPdStages - 1)) * kPfTileBytes + wave * 2048;
      pd_matrix_phase<false, false, false>((uint32_t)((t - 1) & (kPdStages - 1)) * kPfTileBytes,
                                           (uint32_t)(t & (kPdStages - 1)) * kPfTileBytes, lc, qf, pb, st, sc, ld, pre,
                                           negm);
      phase_barrier();
      softmax_phase(t);
      wait_landed(t);
      phase_barrier();
    };
    // Steady state: tile t of the past segment with K(t+3), V(t+2) full tiles of the same segment and nothing
    // masked.  The stage t % 4 is a compile-time constant (every LDS address is an immediate) and the scalar work
    // per tile is two pointer increments.
    const char* kp = ka_p;     // K(t+3), V(t+2) of the next fast tile
    const char* vp = va_p;
    const uint32_t ld_wave = lds_base + wave * 2048;
    auto fast_tile = [&](auto stage_tag) __attribute__((always_inline)) {
      constexpr int S = decltype(stage_tag)::value;
      PfPhaseLoads ld;
      ld.k = kp;
      ld.v = vp;
      ld.ldk = ld_wave + ((S + 3) & 3) * kPfTileBytes;
      ld.ldv = ld_wave + kPdVRing + ((S + 2) & 3) * kPfTileBytes;
      __builtin_amdgcn_s_setprio(2);
      pd_matrix_phase<true, true, true, true>(((S + 3) & 3) * kPfTileBytes, S * kPfTileBytes, lc, qf, pb, st, sc, ld,
                                              pre, negm);       // passes the phase's barrier itself
      __builtin_amdgcn_s_setprio(0);
      pd_preread(S * kPfTileBytes, lc, pre);     // V(t), for the next matrix phase
      __builtin_amdgcn_sched_barrier(0);
      pf_softmax_fast(sc, st, c, negm, pb);
      wait_vmcnt<4>();
      phase_barrier();
      kp += kPfTileBytes;
      vp += kPfTileBytes;
    };
    // A run of steady-state tiles [t, t_end) of one segment whose tile 0 is tile `tile0` of the sweep and whose rows
    // start at kbase / vbase: general tiles up to a multiple of four, then the unrolled loop.
    int t = 1;
    auto fast_run = [&](int t_end, const char* kbase, const char* vbase, int tile0) __attribute__((always_inline)) {
      if (t_end - t < 8) return;
      while (t & 3) { generic_tile(t); ++t; }
      kp = kbase + (int64_t)(t + 3 - tile0) * kPfTileBytes;
      vp = vbase + (int64_t)(t + 2 - tile0) * kPfTileBytes;
      pd_preread((uint32_t)((t - 1) & (kPdStages - 1)) * kPfTileBytes, lc, pre);
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[r] = -st.m;
      for (; t + 4 <= t_end; t += 4) {
        fast_tile(std::integral_constant<int, 0>());
        fast_tile(std::integral_constant<int, 1>());
        fast_tile(std::integral_constant<int, 2>());
        fast_tile(std::integral_constant<int, 3>());
      }
    };
    // past segment: tile t qualifies if K(t+3) and V(t+2) are full tiles of the segment too
    fast_run((int)(na_p / kPfTileRows) - 3, ka_p, va_p, 0);
    // the chunk's own rows: tiles that end at or before the first position of the workgroup are not masked for any
    // of its lanes (own tile j = t + tb_base; its rows are 64 j .. 64 j + 63)
    while (t < ta && t < T) { generic_tile(t); ++t; }
    {
      const int64_t unmasked = ((int64_t)bx * strip + 1) / kPfTileRows;          // own tiles 0 .. unmasked - 1
      const int64_t loadable = a.nb / kPfTileRows - 3;                           // K(t+3), V(t+2) full
      const int64_t j_end = unmasked < loadable ? unmasked : loadable;
      const int64_t t_end = j_end - tb_base < T - 3 ? j_end - tb_base : T - 3;
      fast_run((int)t_end, a.kb, a.vb, -tb_base);
    }
    for (; t < T; ++t) generic_tile(t);
    {
      const uint32_t v_off = (uint32_t)((T - 1) & (kPdStages - 1)) * kPfTileBytes;
#pragma unroll
      for (int i = 0; i < 16; ++i)
        st.o[pd_db(i)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pd_operand(i, v_off, 0, lc), pb[pd_sb(i)][pd_u(i)],
                                                                 st.o[pd_db(i)], 0, 0, 0);
    }
    if (group == 0) phase_barrier();

    if (ps.store >= 0) {
      float* im = images + (int64_t)ps.store * kImageFloats;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) im[(db * 16 + r) * kLanes] = st.o[db][r];
      im[64 * kLanes] = st.m;
      im[65 * kLanes] = st.l;
    } else {
      pf_write_row(a.out, a.out_fp32, a.C, g, my_i, hl, st.o, st.l);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// The 8-wave kernel on the 16x16x32 bf16 MFMA.  Same tiles, LDS rings, alternating schedule, barrier protocol, pass
// loop and work partition as prefill_kernel_deep; what differs is the matrix instruction and with it the register
// layouts (and so the layout of a state image, which has a merge kernel of its own).  Measured on this part, a
// register-only loop of v_mfma_f32_16x16x32_bf16 on random operands sustains 2.10 PFLOP/s under the board's power limit
// where v_mfma_f32_32x32x16_bf16 sustains 1.84: less energy per flop, and the kernel runs against that limit.
// PRESCALED: the queries carry the softmax scale (a.c is 1), and the steady-state softmax has no multiplication.
//   * A wavefront still owns 32 query rows of one query head, now as two blocks of 16 (qb = 0, 1): lane = (query
//     l % 16 of each block, g = l / 16).  S^T = K Q^T per 16-key block kb: register r of s[kb][qb] is key row
//     16 kb + 4 g + r.  A K operand read (16 keys x 32 dims) feeds the MFMAs of both query blocks.
//   * O^T += V^T P^T over 32 keys per MFMA: the lane's 4 + 4 scores of key blocks 2 kp and 2 kp + 1 are, rounded to
//     bf16, its B operand (contraction index 8 g + j is key 32 kp + 16 (j / 4) + 4 g + j % 4), and the V^T operand
//     takes the same permutation: two transpose reads of 4 consecutive rows each.  Register r of o[db][qb] is dim
//     16 db + 4 g + r of the lane's query in block qb.
//   * A lane serves two query rows, so it carries two running references and two shares of the row sums.
//   * V tiles take one more swizzle bit than in the other kernels (rows 4 apart are read by neighbouring 16-lane
//     groups of one transpose read and must not share banks).
static_assert(kCarryFloatsPerLane >= 68, "a state image holds 64 O^T accumulators, two running maxima and two row-sum shares per lane");

__device__ __forceinline__ int swz_v16(int row) { return swz_v(row) ^ (((row >> 2) & 1) << 1); }

struct PfLane16 {
  uint32_t gk[2];     // global byte offset inside a 64-row K tile of this lane's 2 load instructions
  uint32_t gv[2];     // same for V
  uint32_t koff[4];   // absolute LDS address of the K operand read of contraction step kk (key block kb adds 4096)
  uint32_t voff[8];   // absolute LDS address of the V^T transpose read of dim block db (+4096: the second 16 rows
                      // of the key pair, +8192: key pair 1)
};

// The 4-register accumulator tiles of the 16x16x32 MFMA are kept as quarters of 16-register vectors: a result that has to
// land in a quarter of the vector its accumulator came from is computed in place, where free-standing 4-register tiles
// were moved from tuple to tuple by most MFMAs (and the register file overflowed).
__device__ __forceinline__ f32x4 q4_get(const f32x16& v, int k) { return (f32x4){v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]}; }
__device__ __forceinline__ void q4_set(f32x16& v, int k, const f32x4& x) {
  v[4 * k] = x[0]; v[4 * k + 1] = x[1]; v[4 * k + 2] = x[2]; v[4 * k + 3] = x[3];
}

struct PfState16 {
  f32x16 o[4];        // tile (db, qb) is quarter (2 db + qb) % 4 of o[(2 db + qb) / 4]
  float m[2], l[2];
};
// element r of accumulator tile (db, qb) of O^T, and of score tile (kb, qb) in f32x16 s[2]
#define PF16_O(st, db, qb, r) (st).o[(2 * (db) + (qb)) >> 2][4 * ((2 * (db) + (qb)) & 3) + (r)]
#define PF16_S(s, kb, qb, r) (s)[(2 * (kb) + (qb)) >> 2][4 * ((2 * (kb) + (qb)) & 3) + (r)]

__device__ __forceinline__ void pf16_issue_k(const char* kt, int rows, uint32_t lds_tile, int wave, int lane,
                                             const PfLane16& lc) {
  const uint32_t ldk = lds_tile + wave * 2048;
  if (rows >= kPfTileRows) {
    g2lds16_s<0>(kt, lc.gk[0], ldk);
    g2lds16_s<0>(kt, lc.gk[1], ldk + 1024);
  } else {
    const int r_in = lane >> 4, cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = (wave * 2 + i) * 4 + r_in;
      const int rc = r < rows ? r : rows - 1;
      g2lds16_s<0>(kt, (uint32_t)(rc * kRowBytes + ((cpos ^ swz_k(r)) << 4)), ldk + i * 1024);
    }
  }
}

__device__ __forceinline__ void pf16_issue_v(const char* vt, int rows, uint32_t lds_tile, int wave, int lane,
                                             const PfLane16& lc) {
  const uint32_t ldv = lds_tile + wave * 2048;
  if (rows >= kPfTileRows) {
    g2lds16_s<0>(vt, lc.gv[0], ldv);
    g2lds16_s<0>(vt, lc.gv[1], ldv + 1024);
  } else {
    const int r_in = lane >> 4, cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = (wave * 2 + i) * 4 + r_in;
      const int rc = r < rows ? r : rows - 1;
      g2lds16_s<0>(vt, (uint32_t)(rc * kRowBytes + ((cpos ^ swz_v16(r)) << 4)), ldv + i * 1024);
    }
  }
}

// operand i of a matrix phase: i < 16 the V^T fragment of (key pair, dim block) = (i / 8, i % 8), i >= 16 the K
// fragment of (contraction step, key block) = ((i - 16) / 4, (i - 16) % 4); each feeds the MFMAs of both query blocks
__device__ __forceinline__ constexpr int pd16_kp(int i) { return i >> 3; }
__device__ __forceinline__ constexpr int pd16_db(int i) { return i & 7; }
__device__ __forceinline__ constexpr int pd16_kk(int i) { return (i - 16) >> 2; }
__device__ __forceinline__ constexpr int pd16_kb(int i) { return (i - 16) & 3; }

__device__ __forceinline__ bf16x8 pd16_operand(int i, uint32_t v_off, uint32_t k_off, const PfLane16& lc) {
  if (i < 16) {
    const uint32_t ad = lc.voff[pd16_db(i)] + v_off + pd16_kp(i) * 8192;
    const bf16x4 v0 = lds_read_tr8((lds_char*)(uintptr_t)ad);
    const bf16x4 v1 = lds_read_tr8((lds_char*)(uintptr_t)(ad + 4096));
    return __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
  }
  return *(lds_bf16x8*)(uintptr_t)(lc.koff[pd16_kk(i)] + k_off + pd16_kb(i) * 4096);
}

__device__ __forceinline__ void pd16_preread(uint32_t v_off, const PfLane16& lc, bf16x8 (&pre)[kPfAhead]) {
#pragma unroll
  for (int i = 0; i < kPfAhead; ++i) pre[i] = pd16_operand(i, v_off, 0, lc);
}

// The matrix phase: O^T += V^T P^T of the previous tile, then S^T = K Q^T of the next - 64 MFMAs, their 32 LDS operands
// read kPfAhead operands ahead.  LOADS: 0 = the phase issues the global loads that ld names (either may be null),
// 1 = both unconditionally.  Other switches as in pd_matrix_phase.
template <int LOADS, bool PREREAD, bool CINIT, bool EARLY_BARRIER = false>
__device__ __forceinline__ void pd16_matrix_phase(uint32_t v_off, uint32_t k_off, const PfLane16& lc,
                                                  const bf16x8 (&qf)[4][2], const bf16x8 (&pb)[2][2], PfState16& st,
                                                  f32x16 (&s)[2], const PfPhaseLoads& ld,
                                                  const bf16x8 (&pre)[kPfAhead], const f32x4 (&cinit)[2]) {
  bf16x8 op[kPfAhead + 1];
#pragma unroll
  for (int i = 0; i < kPfAhead; ++i) op[i] = PREREAD ? pre[i] : pd16_operand(i, v_off, k_off, lc);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    if (i + kPfAhead < 32) op[(i + kPfAhead) % (kPfAhead + 1)] = pd16_operand(i + kPfAhead, v_off, k_off, lc);
    bf16x8 x = op[i % (kPfAhead + 1)];
    if (EARLY_BARRIER && i == 31) {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x) : : "memory");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
    }
    if (i < 16) {
      const int kp = pd16_kp(i), db = pd16_db(i);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int t4 = 2 * db + qb;
        q4_set(st.o[t4 >> 2], t4 & 3,
               __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, pb[kp][qb], q4_get(st.o[t4 >> 2], t4 & 3), 0, 0, 0));
      }
    } else {
      const int kk = pd16_kk(i), kb = pd16_kb(i);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int t4 = 2 * kb + qb;
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        const f32x4 c0 = kk == 0 ? (CINIT ? cinit[qb] : z) : q4_get(s[t4 >> 2], t4 & 3);
        q4_set(s[t4 >> 2], t4 & 3, __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, qf[kk][qb], c0, 0, 0, 0));
      }
    }
    if (i == 1 && (LOADS == 1 || ld.k)) g2lds16_s<0>(ld.k, lc.gk[0], ld.ldk);
    if (i == 3 && (LOADS == 1 || ld.k)) g2lds16_s<0>(ld.k, lc.gk[1], ld.ldk + 1024);
    if (i == 5 && (LOADS == 1 || ld.v)) g2lds16_s<0>(ld.v, lc.gv[0], ld.ldv);
    if (i == 7 && (LOADS == 1 || ld.v)) g2lds16_s<0>(ld.v, lc.gv[1], ld.ldv + 1024);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// maximum over the four 16-lane groups that hold the key rows of one query
__device__ __forceinline__ float max_groups16(float x) {
  x = fmaxf(x, __shfl_xor(x, 16));
  return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float sum_groups16(float x) {
  x += __shfl_xor(x, 16);
  return x + __shfl_xor(x, 32);
}

// Online softmax of one tile (general form: raw scores, running maximum moved when it must, masks).  rel[qb]: key
// rows of the tile with index > rel[qb] are hidden from the lane's query of block qb.
__device__ __forceinline__ void pf16_softmax(f32x16 (&s)[2], PfState16& st, float c, bool masked, const int (&rel)[2],
                                             int g16, bf16x8 (&pb)[2][2]) {
  if (masked) {
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (16 * kb + 4 * g16 + r > rel[qb]) PF16_S(s, kb, qb, r) = kNegBig;
  }
  float m_new[2];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    float mx = PF16_S(s, 0, qb, 0);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) mx = fmaxf(mx, PF16_S(s, kb, qb, r));
    m_new[qb] = fmaxf(st.m[qb], max_groups16(mx));
  }
  if (__builtin_amdgcn_ballot_w64(m_new[0] > st.m[0] || m_new[1] > st.m[1]) != 0) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float alpha = fast_exp2((st.m[qb] - m_new[qb]) * c);
      st.l[qb] *= alpha;
#pragma unroll
      for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) PF16_O(st, db, qb, r) *= alpha;
      st.m[qb] = m_new[qb];
    }
  }
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float mc = st.m[qb] * c;
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float p = fast_exp2(__builtin_fmaf(PF16_S(s, kb, qb, r), c, -mc));
        lsum += p;
        pb[kb >> 1][qb][4 * (kb & 1) + r] = (__bf16)p;
      }
    st.l[qb] += lsum;
  }
#pragma unroll
  for (int kp = 0; kp < 2; ++kp)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) asm volatile("" : "+v"(pb[kp][qb]));
}

// Softmax phase of a steady-state tile: the scores left the matrix pipe relative to the running reference (the
// accumulators started from cinit = -m), p = 2^(c s); the reference only moves when a lane's share of a row sum says
// it must (see pf_softmax_fast).  The scores are scaled in place first, so that the 32 multiplications and the 32
// exponentials are independent instructions (with a shared temporary they formed one dependent chain).
// PRESCALED: the queries carry the softmax scale already (c is 1): the scores are exponents as they leave the matrix pipe.
template <bool PRESCALED>
__device__ __forceinline__ void pf16_softmax_fast(f32x16 (&s)[2], PfState16& st, float c, f32x4 (&cinit)[2],
                                                  bf16x8 (&pb)[2][2]) {
  if (!PRESCALED) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[j][r] *= c;
  }
  float ls[2];
  auto probs = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float lq[2];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float p = fast_exp2(PF16_S(s, kb, qb, r));
          lq[kb & 1] = (kb < 2 && r == 0) ? p : lq[kb & 1] + p;
          pb[kb >> 1][qb][4 * (kb & 1) + r] = (__bf16)p;
        }
      ls[qb] = lq[0] + lq[1];
    }
  };
  probs();
  if (__builtin_amdgcn_ballot_w64(!(ls[0] <= kPfSumLimit) || !(ls[1] <= kPfSumLimit)) != 0) {    // also inf and NaN
    const float inv_c = 1.0f / c;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      float mx = PF16_S(s, 0, qb, 0);
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, PF16_S(s, kb, qb, r));
      // queries whose maximum did not move keep their reference; the step is taken in score units (the reference
      // is kept in them) and applied here as the exponent it becomes
      const float d = fmaxf(max_groups16(mx), 0.f) * inv_c;
      const float dc = d * c;
      const float alpha = fast_exp2(-dc);
      st.l[qb] *= alpha;
#pragma unroll
      for (int db = 0; db < 8; ++db)
#pragma unroll
        for (int r = 0; r < 4; ++r) PF16_O(st, db, qb, r) *= alpha;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) PF16_S(s, kb, qb, r) -= dc;
      st.m[qb] += d;
#pragma unroll
      for (int r = 0; r < 4; ++r) cinit[qb][r] = -st.m[qb];
    }
    probs();
  }
  st.l[0] += ls[0];
  st.l[1] += ls[1];
#pragma unroll
  for (int kp = 0; kp < 2; ++kp)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) asm volatile("" : "+v"(pb[kp][qb]));
}

// Normalise and write the lane's parts of the query row of block QB: dims 16 (db0 + d) + 4 g16 + 0..3 for d < NDB
// (o[d] holds dim block db0 + d); l is the lane's share of the row sum.
template <int NDB>
__device__ __forceinline__ void pf16_write_row(void* out, int out_fp32, int C, int g, int i, int g16, int db0,
                                               const f32x4 (&o)[NDB], float l) {
  const float inv = 1.0f / sum_groups16(l);
  if (i >= C) return;
  const int64_t base = ((int64_t)g * C + i) * kHeadDim;
#pragma unroll
  for (int d = 0; d < NDB; ++d) {
    const f32x4 v = o[d];
    const int dim = 16 * (db0 + d) + 4 * g16;
    const float x0 = v[0] * inv, x1 = v[1] * inv, x2 = v[2] * inv, x3 = v[3] * inv;
    if (out_fp32) {
      *(float4*)((float*)out + base + dim) = make_float4(x0, x1, x2, x3);
    } else {
      uint2 pk;
      pk.x = (uint32_t)float_to_bf16_bits(x0) | ((uint32_t)float_to_bf16_bits(x1) << 16);
      pk.y = (uint32_t)float_to_bf16_bits(x2) | ((uint32_t)float_to_bf16_bits(x3) << 16);
      *(uint2*)((uint16_t*)out + base + dim) = pk;
    }
  }
}

template <bool PRESCALED>
__global__ __launch_bounds__(512, 2) void prefill_kernel_deep16(PrefillArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char lds_dyn[];
  lds_char* lds = (lds_char*)lds_dyn;
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
  const int lane = lane_id();
  const int wave = wave_id();
  const int g16 = lane >> 4;
  const int c16 = lane & 15;

  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (kPdWaves / gl);
  const int g = pf_select_head(a) * 4 + (wave % gl);

  PfLane16 lc;
  {
    const int r_in = lane >> 4, cpos = lane & 15;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = (wave * 2 + i) * 4 + r_in;
      lc.gk[i] = (uint32_t)(r * kRowBytes + ((cpos ^ swz_k(r)) << 4));
      lc.gv[i] = (uint32_t)(r * kRowBytes + ((cpos ^ swz_v16(r)) << 4));
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      lc.koff[kk] = lds_base + (uint32_t)(c16 * kRowBytes + (((4 * kk + g16) ^ swz_k(c16)) << 4));
    const int row = 4 * g16 + (c16 >> 2);             // the row of the 4-row block this lane addresses
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      const int chunk = 2 * db + ((c16 & 3) >> 1);
      lc.voff[db] = lds_base + kPdVRing +
                    (uint32_t)(row * kRowBytes + ((chunk ^ swz_v16(row)) << 4) + ((c16 & 1) << 3));
    }
  }

  PfShape sh;
  sh.nbk = a.nbk; sh.m = strip / kPfTileRows;
  sh.ta = (int)((a.na + kPfTileRows - 1) / kPfTileRows);
  sh.tb_all = (int)((a.nb + kPfTileRows - 1) / kPfTileRows);
  sh.split = a.split; sh.paired = a.paired; sh.carried = !a.first;
  constexpr int kLanes = kPdWaves * 64;
  constexpr int kImageFloats = kCarryFloatsPerLane * kLanes;
  float* const images = a.carry + (int64_t)blockIdx.y * pf_images_per_row(a.nbk, a.split) * kImageFloats + threadIdx.x;
  int first_which = 0;
  {
    const PfPass d = pf_pass(sh, blockIdx.x, 0, a.last), sw = pf_pass(sh, blockIdx.x, 1, a.last);
    if (sw.run && sw.a1 > sw.a0 && !(d.run && d.a1 > d.a0)) first_which = 1;
  }
#pragma nounroll
  for (int pi = 0; pi < 2; ++pi) {
    const PfPass ps = pf_pass(sh, blockIdx.x, first_which ^ pi, a.last);
    if (ps.init) {
      float* im = images + (int64_t)ps.store * kImageFloats;
#pragma unroll
      for (int i = 0; i < 64; ++i) im[i * kLanes] = 0.f;
      im[64 * kLanes] = kNegBig;
      im[65 * kLanes] = kNegBig;
      im[66 * kLanes] = 0.f;
      im[67 * kLanes] = 0.f;
    }
    if (!ps.run) continue;
    __syncthreads();
    const int bx = ps.bx;
    const int i0 = bx * strip + 32 * (wave / gl);
    int my_i[2], qi[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      my_i[qb] = i0 + 16 * qb + c16;
      qi[qb] = my_i[qb] > a.C - 1 ? a.C - 1 : my_i[qb];
    }

    // Q^T operands: lane holds q[g][qi[qb]][32*kk + 8*g16 .. +7]
    bf16x8 qf[4][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const uint16_t* qrow = a.q + ((int64_t)g * a.C + qi[qb]) * kHeadDim + 8 * g16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) qf[kk][qb] = __builtin_bit_cast(bf16x8, *(const uint4*)(qrow + 32 * kk));
    }

    // a past segment in two pieces: the pass's tiles from jr on lie a.a_jump_bytes further on
    int jr = a.a_jump_tile > 0 ? a.a_jump_tile - ps.a0 : 0x7fffffff;
    const int64_t jump0 = jr <= 0 ? a.a_jump_bytes : 0;        // the whole pass is behind the jump
    if (jr <= 0) jr = 0x7fffffff;
    const char* const ka_p = a.ka + (int64_t)ps.a0 * kPfTileBytes + jump0;
    const char* const va_p = a.va + (int64_t)ps.a0 * kPfTileBytes + jump0;
    auto a_jump = [&](int t) { return t >= jr ? a.a_jump_bytes : (int64_t)0; };
    int64_t na_p = (int64_t)ps.a1 * kPfTileRows;
    if (na_p > a.na) na_p = a.na;
    na_p -= (int64_t)ps.a0 * kPfTileRows;
    const int b_t0 = ps.b0;
    const int tb = ps.b1 - ps.b0;

    PfState16 st;
    if (ps.load < 0) {
      st.m[0] = st.m[1] = kNegBig;
      st.l[0] = st.l[1] = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[j][r] = 0.f;
    } else {
      const float* im = images + (int64_t)ps.load * kImageFloats;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[j][r] = im[(16 * j + r) * kLanes];     // = ((2 db + qb) * 4 + r)
      st.m[0] = im[64 * kLanes];
      st.m[1] = im[65 * kLanes];
      st.l[0] = im[66 * kLanes];
      st.l[1] = im[67 * kLanes];
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[kk][0]), "+v"(qf[kk][1]));
    asm volatile("" : "+v"(st.m[0]), "+v"(st.m[1]), "+v"(st.l[0]), "+v"(st.l[1]));
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(st.o[j]));

    const int ta = (int)((na_p + kPfTileRows - 1) / kPfTileRows);
    const int T = ta + tb;
    const int tb_base = b_t0 - ta;

    auto issue = [&](int t, int which) __attribute__((always_inline)) {
      if (t >= T) return;
      const bool in_b = t >= ta;
      const int64_t row0 = (int64_t)(in_b ? t + tb_base : t) * kPfTileRows;
      const int64_t left = (in_b ? a.nb : na_p) - row0;
      const int rows = left < kPfTileRows ? (int)left : kPfTileRows;
      const uint32_t slot = lds_base + (uint32_t)(t & (kPdStages - 1)) * kPfTileBytes;
      if (which == 0) pf16_issue_k((in_b ? a.kb : ka_p + a_jump(t)) + row0 * kRowBytes, rows, slot, wave, lane, lc);
      else pf16_issue_v((in_b ? a.vb : va_p + a_jump(t)) + row0 * kRowBytes, rows, slot + kPdVRing, wave, lane, lc);
    };
    auto wait_landed = [&](int t) {
      if (t + 3 < T) wait_vmcnt<4>();
      else wait_vmcnt<0>();
    };
    auto phase_barrier = [&]() {
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
    };

    // the alternating schedule, barrier protocol and ring discipline of prefill_kernel_deep
    const int group = wave >> 2;
    const float c = a.c;
    wait_vmcnt<0>();
    issue(0, 0);
    issue(1, 0); issue(0, 1);
    issue(2, 0); issue(1, 1);
    wait_landed(-1);
    phase_barrier();
    if (group == 1) phase_barrier();

    f32x16 sc[2];
    bf16x8 pb[2][2];
    auto softmax_phase = [&](int t) __attribute__((always_inline)) {
      const bool in_b = t >= ta;
      const int64_t j0 = (int64_t)(in_b ? t + tb_base : t) * kPfTileRows;
      const int64_t n_seg = in_b ? a.nb : na_p;
      const bool masked = (j0 + kPfTileRows > n_seg) || (in_b && (j0 + kPfTileRows - 1 > i0));
      int rel[2] = {kPfTileRows, kPfTileRows};
      if (masked) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          int64_t lim = n_seg - 1;
          if (in_b && (int64_t)my_i[qb] < lim) lim = my_i[qb];
          const int64_t d = lim - j0;
          rel[qb] = d < -1 ? -1 : (d > kPfTileRows ? kPfTileRows : (int)d);
        }
      }
      pf16_softmax(sc, st, c, masked, rel, g16, pb);
    };
    // tile 0: nothing to accumulate yet
    issue(3, 0);
    issue(2, 1);
#pragma unroll
    for (int i = 16; i < 32; ++i) {
      const bf16x8 x = pd16_operand(i, 0, 0, lc);
      const int kk = pd16_kk(i), kb = pd16_kb(i);
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const int t4 = 2 * kb + qb;
        q4_set(sc[t4 >> 2], t4 & 3,
               __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, qf[kk][qb], kk == 0 ? z : q4_get(sc[t4 >> 2], t4 & 3), 0, 0, 0));
      }
    }
    phase_barrier();
    softmax_phase(0);
    wait_landed(0);
    phase_barrier();
    bf16x8 pre[kPfAhead];
    f32x4 cinit[2];      // minus the running references, the start values of the steady-state score accumulators
    cinit[0] = cinit[1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    auto generic_tile = [&](int t) __attribute__((always_inline)) {
      PfPhaseLoads ld;
      ld.k = ld.v = nullptr;
      const int tk = t + 3, tv = t + 2;
      const bool kb = tk >= ta, vb = tv >= ta;
      const int64_t krow0 = (int64_t)(kb ? tk + tb_base : tk) * kPfTileRows;
      const int64_t vrow0 = (int64_t)(vb ? tv + tb_base : tv) * kPfTileRows;
      const bool kfull = tk < T && (kb ? a.nb : na_p) - krow0 >= kPfTileRows;
      const bool vfull = tv < T && (vb ? a.nb : na_p) - vrow0 >= kPfTileRows;
      if (kfull) ld.k = (kb ? a.kb : ka_p + a_jump(tk)) + krow0 * kRowBytes; else issue(tk, 0);
      if (vfull) ld.v = (vb ? a.vb : va_p + a_jump(tv)) + vrow0 * kRowBytes; else issue(tv, 1);
      ld.ldk = lds_base + (uint32_t)(tk & (kPdStages - 1)) * kPfTileBytes + wave * 2048;
      ld.ldv = lds_base + kPdVRing + (uint32_t)(tv & (kPdStages - 1)) * kPfTileBytes + wave * 2048;
      pd16_matrix_phase<0, false, false>((uint32_t)((t - 1) & (kPdStages - 1)) * kPfTileBytes,
                                             (uint32_t)(t & (kPdStages - 1)) * kPfTileBytes, lc, qf, pb, st, sc, ld, pre,
                                             cinit);
      phase_barrier();
      softmax_phase(t);
      wait_landed(t);
      phase_barrier();
    };
    const char* kp = ka_p;
    const char* vp = va_p;
    const uint32_t ld_wave = lds_base + wave * 2048;
    auto fast_tile = [&](auto stage_tag) __attribute__((always_inline)) {
      constexpr int S = decltype(stage_tag)::value;
      PfPhaseLoads ld;
      ld.k = kp;
      ld.v = vp;
      ld.ldk = ld_wave + ((S + 3) & 3) * kPfTileBytes;
      ld.ldv = ld_wave + kPdVRing + ((S + 2) & 3) * kPfTileBytes;
      __builtin_amdgcn_s_setprio(2);
      pd16_matrix_phase<1, true, true, true>(((S + 3) & 3) * kPfTileBytes, S * kPfTileBytes, lc, qf, pb, st, sc, ld,
                                             pre, cinit);
      __builtin_amdgcn_s_setprio(0);
      pd16_preread(S * kPfTileBytes, lc, pre);
      __builtin_amdgcn_sched_barrier(0);
      pf16_softmax_fast<PRESCALED>(sc, st, c, cinit, pb);
      wait_vmcnt<4>();
      phase_barrier();
      kp += kPfTileBytes;
      vp += kPfTileBytes;
    };
    int t = 1;
    // t_min: the run may not start before this tile (the tiles up to it go through the general routine first)
    auto fast_run = [&](int t_end, const char* kbase, const char* vbase, int tile0, int t_min) __attribute__((always_inline)) {
      if (t_end - (t > t_min ? t : t_min) < 8) return;
      while ((t & 3) || t < t_min) { generic_tile(t); ++t; }
      kp = kbase + (int64_t)(t + 3 - tile0) * kPfTileBytes;
      vp = vbase + (int64_t)(t + 2 - tile0) * kPfTileBytes;
      pd16_preread((uint32_t)((t - 1) & (kPdStages - 1)) * kPfTileBytes, lc, pre);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r = 0; r < 4; ++r) cinit[qb][r] = -st.m[qb];
      for (; t + 4 <= t_end; t += 4) {
        fast_tile(std::integral_constant<int, 0>());
        fast_tile(std::integral_constant<int, 1>());
        fast_tile(std::integral_constant<int, 2>());
        fast_tile(std::integral_constant<int, 3>());
      }
    };
    {
      // steady-state tiles load K(t+3) and V(t+2) through running pointers: a run stays on one side of a jump (one
      // call site for both sides: every copy of the loop the compiler has to fit costs the others registers)
      const int a_end = (int)(na_p / kPfTileRows) - 3;
      const int pieces = jr < ta ? 2 : 1;
#pragma nounroll
      for (int piece = 0; piece < pieces; ++piece) {
        const int64_t off = piece ? a.a_jump_bytes : 0;
        int end = a_end;
        if (piece == 0 && pieces == 2 && jr - 3 < end) end = jr - 3;
        fast_run(end, ka_p + off, va_p + off, 0, piece ? jr - 2 : 0);
      }
    }
    while (t < ta && t < T) { generic_tile(t); ++t; }
    {
      const int64_t unmasked = ((int64_t)bx * strip + 1) / kPfTileRows;
      const int64_t loadable = a.nb / kPfTileRows - 3;
      const int64_t j_end = unmasked < loadable ? unmasked : loadable;
      const int64_t t_end = j_end - tb_base < T - 3 ? j_end - tb_base : T - 3;
      fast_run((int)t_end, a.kb, a.vb, -tb_base, 0);
    }
    for (; t < T; ++t) generic_tile(t);
    {
      const uint32_t v_off = (uint32_t)((T - 1) & (kPdStages - 1)) * kPfTileBytes;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const bf16x8 x = pd16_operand(i, v_off, 0, lc);
        const int kp2 = pd16_kp(i), db = pd16_db(i);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const int t4 = 2 * db + qb;
          q4_set(st.o[t4 >> 2], t4 & 3,
                 __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, pb[kp2][qb], q4_get(st.o[t4 >> 2], t4 & 3), 0, 0, 0));
        }
      }
    }
    if (group == 0) phase_barrier();

    if (ps.store >= 0) {
      float* im = images + (int64_t)ps.store * kImageFloats;
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) im[(16 * j + r) * kLanes] = st.o[j][r];
      im[64 * kLanes] = st.m[0];
      im[65 * kLanes] = st.m[1];
      im[66 * kLanes] = st.l[0];
      im[67 * kLanes] = st.l[1];
    } else {
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        f32x4 rows[8];
#pragma unroll
        for (int db = 0; db < 8; ++db) rows[db] = q4_get(st.o[(2 * db + qb) >> 2], (2 * db + qb) & 3);
        pf16_write_row<8>(a.out, a.out_fp32, a.C, g, my_i[qb], g16, 0, rows, st.l[qb]);
      }
    }
  }
}

// Merge of the states of prefill_kernel_deep16 (its own image layout): grid (blocks, grid rows, 4): quarter z combines
// dim blocks 2 z and 2 z + 1 of both query rows of the lane.
__global__ __launch_bounds__(512) void prefill_merge16_kernel(PrefillArgs a) {
  const int lane = lane_id();
  const int wave = wave_id();
  const int g16 = lane >> 4;
  const int c16 = lane & 15;
  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (kPdWaves / gl);
  const int bx = blockIdx.x;
  const int zq = blockIdx.z;
  const int g = pf_select_head(a) * 4 + (wave % gl);
  const int i0 = bx * strip + 32 * (wave / gl);
  constexpr int kLanes = kPdWaves * 64;
  constexpr int kImageFloats = kCarryFloatsPerLane * kLanes;
  PfShape sh;
  sh.nbk = a.nbk; sh.m = strip / kPfTileRows;
  sh.ta = (int)((a.na + kPfTileRows - 1) / kPfTileRows);
  sh.tb_all = (int)((a.nb + kPfTileRows - 1) / kPfTileRows);
  sh.split = a.split; sh.paired = a.paired; sh.carried = !a.first;
  int n_e, n_x;
  pf_block_images(sh, bx, n_e, n_x);
  if (n_e + n_x == 1 && a.split == 1) return;
  const float* images = a.carry + (int64_t)blockIdx.y * pf_images_per_row(a.nbk, a.split) * kImageFloats + threadIdx.x;
  auto image_of = [&](int i) { return images + (int64_t)(i < n_e ? pf_image_e(sh, bx, i) : pf_image_x(sh, bx, i - n_e)) * kImageFloats; };
  float m[2] = {kNegBig, kNegBig};
  for (int i = 0; i < n_e + n_x; ++i) {
    const float* im = image_of(i);
    m[0] = fmaxf(m[0], im[64 * kLanes]);
    m[1] = fmaxf(m[1], im[65 * kLanes]);
  }
  f32x4 o[2][2];      // [dim block 2 zq + d][qb]
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) o[d][qb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float l[2] = {0.f, 0.f};
  for (int i = 0; i < n_e + n_x; ++i) {
    const float* im = image_of(i);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float w = fast_exp2((im[(64 + qb) * kLanes] - m[qb]) * a.c);
      l[qb] += w * im[(66 + qb) * kLanes];
#pragma unroll
      for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int r = 0; r < 4; ++r) o[d][qb][r] += w * im[(((2 * zq + d) * 2 + qb) * 4 + r) * kLanes];
    }
  }
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const f32x4 rows[2] = {o[0][qb], o[1][qb]};
    pf16_write_row<2>(a.out, a.out_fp32, a.C, g, i0 + 16 * qb + c16, g16, 2 * zq, rows, l[qb]);
  }
}

#include "hi_prefill_wide.inc"

// One dim block (32 of the 128 output dims) of pf_write_row: register r of o is dim 32*db + 8*(r/4) + 4*hl + r%4.
__device__ __forceinline__ void pf_write_row_db(void* out, int out_fp32, int C, int g, int i, int hl, int db,
                                                const f32x16& o, float l) {
  const float inv = 1.0f / sum_halves(l);
  if (i >= C) return;
  const int64_t base = ((int64_t)g * C + i) * kHeadDim;
#pragma unroll
  for (int rq = 0; rq < 4; ++rq) {
    const int dim = 32 * db + 8 * rq + 4 * hl;
    const float x0 = o[4 * rq] * inv, x1 = o[4 * rq + 1] * inv, x2 = o[4 * rq + 2] * inv, x3 = o[4 * rq + 3] * inv;
    if (out_fp32) {
      *(float4*)((float*)out + base + dim) = make_float4(x0, x1, x2, x3);
    } else {
      uint2 pk;
      pk.x = (uint32_t)float_to_bf16_bits(x0) | ((uint32_t)float_to_bf16_bits(x1) << 16);
      pk.y = (uint32_t)float_to_bf16_bits(x2) | ((uint32_t)float_to_bf16_bits(x3) << 16);
      *(uint2*)((uint16_t*)out + base + dim) = pk;
    }
  }
}

// Merge of the states of the 8-wave kernel, run once after a unit's last launch when a block of positions can have
// more than one state (split > 1, or the paired partition): grid (blocks, grid rows, 4 dim blocks), the kernel's
// own lane layout, so every lane combines its own register images - m = max m_i, O = sum O_i 2^(c (m_i - m)),
// l likewise - then normalises and writes its part of out[g][i][:].  A block with a single state was written by
// the pass that computed it.
__global__ __launch_bounds__(512) void prefill_merge_kernel(PrefillArgs a) {
  const int lane = lane_id();
  const int wave = wave_id();
  const int hl = lane >> 5;
  const int col = lane & 31;
  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (kPdWaves / gl);
  const int bx = blockIdx.x;
  const int db = blockIdx.z;
  const int g = pf_select_head(a) * 4 + (wave % gl);
  const int my_i = bx * strip + 32 * (wave / gl) + col;
  constexpr int kLanes = kPdWaves * 64;
  constexpr int kImageFloats = kCarryFloatsPerLane * kLanes;
  PfShape sh;
  sh.nbk = a.nbk; sh.m = strip / kPfTileRows;
  sh.ta = (int)((a.na + kPfTileRows - 1) / kPfTileRows);
  sh.tb_all = (int)((a.nb + kPfTileRows - 1) / kPfTileRows);
  sh.split = a.split; sh.paired = a.paired; sh.carried = !a.first;
  int n_e, n_x;
  pf_block_images(sh, bx, n_e, n_x);
  if (n_e + n_x == 1 && a.split == 1) return;
  const float* images = a.carry + (int64_t)blockIdx.y * pf_images_per_row(a.nbk, a.split) * kImageFloats + threadIdx.x;
  auto image_of = [&](int i) { return images + (int64_t)(i < n_e ? pf_image_e(sh, bx, i) : pf_image_x(sh, bx, i - n_e)) * kImageFloats; };
  float m = kNegBig;
  for (int i = 0; i < n_e + n_x; ++i) m = fmaxf(m, image_of(i)[64 * kLanes]);
  f32x16 o;
#pragma unroll
  for (int r = 0; r < 16; ++r) o[r] = 0.f;
  float l = 0.f;
  for (int i = 0; i < n_e + n_x; ++i) {
    const float* im = image_of(i);
    const float w = fast_exp2((im[64 * kLanes] - m) * a.c);
    l += w * im[65 * kLanes];
#pragma unroll
    for (int r = 0; r < 16; ++r) o[r] += w * im[(db * 16 + r) * kLanes];
  }
  pf_write_row_db(a.out, a.out_fp32, a.C, g, my_i, hl, db, o, l);
}

// ---------------------------------------------------------------------------------------------------------
// Streaming heads (Appendix E, head-wise sparsity: a streaming head keeps only recent tokens - here n_sink initial
// tokens and the n_recent most recent ones - and lives in HBM).  Query row at absolute position p sees key j iff
// j <= p and (j < n_sink or p - j < n_recent).  The head's K/V is a bounded store of n_sink + n_recent rows: sink
// row j at row j, token j >= n_sink in ring slot n_sink + (j - n_sink) mod n_recent.
//
// One launch computes a chunk.  The keys form two sequences: A, what the store holds of the past (its ns sink
// rows, then the m most recent past rows in token order, read through the ring mapping), and B, the chunk's own
// rows.  A workgroup visits only the 64-row tiles some of its rows can see: the sink tiles and the tiles from its
// first row's window start on, in each sequence.
struct PrefillWindowArgs {
  const uint16_t* q;      // [G][C][128]
  const char* ks; const char* vs;   // the store's K and V planes
  const char* kb; const char* vb;   // the chunk's own rows
  void* out;
  int G, C, out_fp32, gy;
  float c;
  int n_sink, n_recent;
  int ns;                 // sink rows of the past: min(P, n_sink)
  int m;                  // recent rows of the past held by the ring: tokens t0 .. P-1, t0 = max(n_sink, P-n_recent+1)
  int ring0;              // ring slot of token t0
  int lo0;                // index in A of the first recent row visible to chunk row 0 (row i: lo0 + i); may be < ns
  int sink_b;             // chunk rows that are sink tokens: clamp(n_sink - P, 0, C)
  int64_t s_head_stride;  // bytes between the heads' stores
};

// pf_softmax for a tile in which lane-dependent sets of rows are hidden: row is visible iff row <= hi and
// (row < sk or row >= lo).  A lane may see nothing of the tile (and nothing so far): hidden entries contribute
// exactly zero whatever the running maximum is.
__device__ __forceinline__ void pf_softmax_window(f32x16 (&s)[2], PfState& st, float c, bool masked, int hi, int sk,
                                                  int lo, int hl, bf16x8 (&pb)[2][2]) {
  if (masked) {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
        const bool vis = row <= hi && (row < sk || row >= lo);
        if (!vis) s[sb][r] = kNegBig;
      }
  }
  float mx = s[0][0];
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
  mx = max_halves(mx);
  const float m_new = fmaxf(st.m, mx);
  if (__builtin_amdgcn_ballot_w64(m_new > st.m) != 0) {
    const float alpha = fast_exp2((st.m - m_new) * c);
    st.l *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    st.m = m_new;
  }
  const float mc = st.m * c;
  float lsum = 0.f;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float p = fast_exp2(__builtin_fmaf(s[sb][8 * u + j], c, -mc));
        if (masked && s[sb][8 * u + j] == kNegBig) p = 0.f;
        lsum += p;
        pb[sb][u][j] = (__bf16)p;
      }
  st.l += lsum;
}

__global__ __launch_bounds__(256, 2) void prefill_window_kernel(PrefillWindowArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds_raw[kPfLdsBytes];
  lds_char* lds = (lds_char*)lds_raw;
  const uint32_t lds_base = (uint32_t)(uintptr_t)lds;
  const int lane = lane_id();
  const int wave = wave_id();
  const int hl = lane >> 5;
  const int col = lane & 31;

  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (4 / gl);
  const int bx = blockIdx.x;
  const int head = blockIdx.y / a.gy;
  {  // group launches: this workgroup's head
    const int64_t rows = (int64_t)head * a.C;
    a.q += rows * a.G * kHeadDim;
    a.out = (char*)a.out + rows * a.G * kHeadDim * (a.out_fp32 ? 4 : 2);
    a.ks += head * a.s_head_stride;
    a.vs += head * a.s_head_stride;
    a.kb += rows * kRowBytes;
    a.vb += rows * kRowBytes;
  }
  const int g = (blockIdx.y - head * a.gy) * 4 + (wave % gl);
  const int i_lo = bx * strip;                      // first and last query position of the workgroup
  const int i_hi = i_lo + strip - 1;
  const int i0 = i_lo + 32 * (wave / gl);           // first query position of this wave
  const int my_i = i0 + col;
  const int qi = my_i > a.C - 1 ? a.C - 1 : my_i;

  const PfLaneConst lc = pf_lane_const_4w(wave, lane);

  bf16x8 qf[8];
  {
    const uint16_t* qrow = a.q + ((int64_t)g * a.C + qi) * kHeadDim + 8 * hl;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, *(const uint4*)(qrow + 16 * kk));
  }
  PfState st;
  st.m = kNegBig;
  st.l = 0.f;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(qf[kk]));

  // tiles this workgroup visits: A [0, a1) and [a2, ta), then B [0, b1) and [b2, tb)
  const int nA = a.ns + a.m;
  const int ta = (nA + kPfTileRows - 1) / kPfTileRows;
  const int nb_vis = a.C < i_hi + 1 ? a.C : i_hi + 1;
  const int tb = (nb_vis + kPfTileRows - 1) / kPfTileRows;
  int a1 = (a.ns + kPfTileRows - 1) / kPfTileRows;
  if (a1 > ta) a1 = ta;
  const int loA = a.lo0 + i_lo;
  int a2 = loA <= 0 ? 0 : loA / kPfTileRows;
  a2 = a2 < a1 ? a1 : (a2 > ta ? ta : a2);
  int b1 = (a.sink_b + kPfTileRows - 1) / kPfTileRows;
  if (b1 > tb) b1 = tb;
  const int loB = i_lo - a.n_recent + 1;
  int b2 = loB <= 0 ? 0 : loB / kPfTileRows;
  b2 = b2 < b1 ? b1 : (b2 > tb ? tb : b2);
  const int nAv = a1 + (ta - a2);
  const int T = nAv + b1 + (tb - b2);            // >= 1: the tile holding the workgroup's first row

  // visit v -> (sequence, tile)
  auto locate = [&](int v, bool& in_b) __attribute__((always_inline)) {
    in_b = v >= nAv;
    if (!in_b) return v < a1 ? v : a2 + (v - a1);
    const int w = v - nAv;
    return w < b1 ? w : b2 + (w - b1);
  };

  auto issue = [&](int v) __attribute__((always_inline)) {
    const uint32_t stage = lds_base + (uint32_t)(v & (kPfStages - 1)) * kPfStageBytes;
    bool in_b;
    const int tile = locate(v, in_b);
    if (in_b) {
      const int row0 = tile * kPfTileRows;
      const int left = a.C - row0;
      pf_issue_tile<4>(a.kb + (int64_t)row0 * kRowBytes, a.vb + (int64_t)row0 * kRowBytes,
                       left < kPfTileRows ? left : kPfTileRows, stage, wave, lane, lc);
    } else {
      // rows of A come through the ring mapping: per-lane addresses
      const int r_in = lane >> 4, cpos = lane & 15;
      const uint32_t ld = stage + wave * 4096;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = (wave * 4 + i) * 4 + r_in;
        int u = tile * kPfTileRows + r;
        if (u > nA - 1) u = nA - 1;
        int phys = u;
        if (u >= a.ns) {
          int w = a.ring0 + (u - a.ns);
          if (w >= a.n_recent) w -= a.n_recent;
          phys = a.n_sink + w;
        }
        g2lds16_s<0>(a.ks, (uint32_t)phys * kRowBytes + ((cpos ^ swz_k(r)) << 4), ld + i * 1024);
        g2lds16_s<0>(a.vs, (uint32_t)phys * kRowBytes + ((cpos ^ swz_v(r)) << 4), ld + kPfTileBytes + i * 1024);
      }
    }
  };

  issue(0);
  const float c = a.c;
  auto step = [&](int v, auto stage_tag) __attribute__((always_inline)) {
    constexpr int STAGE = decltype(stage_tag)::value;
    wait_vmcnt<0>();
    __syncthreads();
    if (v + 1 < T) issue(v + 1);
    bool in_b;
    const int j0 = locate(v, in_b) * kPfTileRows;
    // per lane: row visible iff row <= hi and (row < sk or row >= lo), rows relative to the tile
    int hi, sk, lo;
    bool full;          // wave-uniform: every row of the tile is visible to every query row of this wave
    if (in_b) {
      hi = (my_i < a.C - 1 ? my_i : a.C - 1) - j0;
      sk = a.sink_b - j0;
      lo = my_i - a.n_recent + 1 - j0;
      full = j0 + kPfTileRows - 1 <= (i0 < a.C - 1 ? i0 : a.C - 1) &&
             (j0 + kPfTileRows - 1 < a.sink_b || j0 >= i0 + 31 - a.n_recent + 1);
    } else {
      hi = nA - 1 - j0;
      sk = a.ns - j0;
      lo = a.lo0 + my_i - j0;
      full = j0 + kPfTileRows - 1 <= nA - 1 && (j0 + kPfTileRows - 1 < a.ns || j0 >= a.lo0 + i0 + 31);
    }
    lds_char* kt = lds + STAGE * kPfStageBytes;
    f32x16 s[2];
    bf16x8 pb[2][2];
    pf_scores(kt, lc, qf, s);
    pf_softmax_window(s, st, c, !full, hi, sk, lo, hl, pb);
    pf_pv(kt + kPfTileBytes, lc, pb, st);
  };
  int v = 0;
  for (; v + 1 < T; v += 2) {
    step(v, std::integral_constant<int, 0>());
    step(v + 1, std::integral_constant<int, 1>());
  }
  if (v < T) step(v, std::integral_constant<int, 0>());

  pf_write_row(a.out, a.out_fp32, a.C, g, my_i, hl, st.o, st.l);
}

// The chunk's rows enter a streaming head's store (after the chunk's attention has read it): chunk rows that are
// sink tokens go to their sink rows, the last n_recent rows (that are not sinks) to their ring slots.
// grid (row blocks, heads, 2: K and V); 16 bytes per thread.
__global__ __launch_bounds__(256) void stream_store_update_kernel(const char* __restrict__ k_new,
                                                                  const char* __restrict__ v_new,
                                                                  char* __restrict__ ks, char* __restrict__ vs, int C,
                                                                  int64_t P, int n_sink, int n_recent, int cs, int u0r,
                                                                  int cr, int64_t s_head_stride) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int r = (int)(idx >> 4), part = (int)(idx & 15);
  if (r >= cs + cr) return;
  const int u = r < cs ? r : u0r + (r - cs);                       // chunk row
  const int64_t j = P + u;                                         // its token
  const int64_t dst = r < cs ? j : n_sink + (j - n_sink) % n_recent;
  const char* src = (blockIdx.z ? v_new : k_new) + ((int64_t)blockIdx.y * C + u) * kRowBytes + part * 16;
  char* d = (blockIdx.z ? vs : ks) + blockIdx.y * s_head_stride + dst * kRowBytes + part * 16;
  *(uint4*)d = *(const uint4*)src;
}


hi_status launch_prefill(void* stream, const void* q, int G, int chunk_len, const PrefillSegment& sa,
                         const PrefillSegment& sb, int first, int last, void* carry, void* out, int out_fp32,
                         int variant, int n_heads, int64_t carry_bytes) {
  if (n_heads < 1 || (variant & 3) == 2) { set_last_error("prefill launch: head group or variant"); return HI_ERR_UNSUPPORTED; }
  if (chunk_len < 1 || !(G == 1 || G == 2 || G == 4 || G == 8)) { set_last_error("prefill launch: bad shape"); return HI_ERR_ARG; }
  if (sa.causal || (sb.n > 0 && !sb.causal)) { set_last_error("prefill launch: segment order"); return HI_ERR_ARG; }
  if (sa.n + sb.n <= 0) { set_last_error("prefill launch: no rows"); return HI_ERR_ARG; }
  PrefillArgs a;
  a.q = (const uint16_t*)q;
  a.ka = (const char*)sa.k; a.va = (const char*)sa.v; a.na = sa.n;
  a.kb = (const char*)sb.k; a.vb = (const char*)sb.v; a.nb = sb.n;
  a.carry = (float*)carry;
  a.out = out;
  a.G = G; a.C = chunk_len; a.first = first; a.last = last; a.out_fp32 = out_fp32;
  const bool q_prescaled = (variant & 32) != 0;
  a.c = softmax_scale_log2(q_prescaled);
  const int strip = prefill_strip(G);
  const int gy = prefill_grid_y(G);
  a.gy = gy;
  a.a_jump_tile = (int)(sa.jump_rows / kPfTileRows);
  a.a_jump_bytes = sa.jump_bytes;
  if (sa.jump_rows != 0 && (sa.jump_rows % kPfTileRows != 0 || sa.jump_rows < 0 || sa.jump_rows >= sa.n)) {
    set_last_error("prefill launch: a past segment in two pieces breaks at a multiple of 64 rows inside it");
    return HI_ERR_ARG;
  }
  a.a_head_stride = sa.head_stride;
  const PrefillLaunch pl = prefill_launch_shape(G, chunk_len, n_heads, variant, last, sb.n > 0);
  if (sa.n >= (1LL << 31) || sb.n >= (1LL << 31)) { set_last_error("prefill launch: more than 2^31 rows"); return HI_ERR_RANGE; }
  if (carry_bytes >= 0 && pl.carry_bytes > carry_bytes) {     // the carry must hold every state image of the launch
    set_last_error("prefill launch: carry of %lld bytes needed, %lld provided", (long long)pl.carry_bytes, (long long)carry_bytes);
    return HI_ERR_ARG;
  }
  a.split = pl.split;
  a.paired = pl.paired;
  a.nbk = pl.nbk;
  if (sa.jump_rows != 0 && !(pl.deep && (variant & 16) == 0)) {
    set_last_error("prefill launch: this kernel takes its past segment in one piece");
    return HI_ERR_UNSUPPORTED;
  }
  if (pl.deep) {
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [] {
      attr_err = hipFuncSetAttribute((const void*)prefill_kernel_deep, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     kPdLdsBytes);
      if (attr_err == hipSuccess)
        attr_err = hipFuncSetAttribute((const void*)prefill_kernel_deep16<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kPdLdsBytes);
      if (attr_err == hipSuccess)
        attr_err = hipFuncSetAttribute((const void*)prefill_kernel_deep16<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kPdLdsBytes);
      if (attr_err == hipSuccess)
        attr_err = hipFuncSetAttribute((const void*)prefill_kernel_wide<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kPdLdsBytes);
      if (attr_err == hipSuccess)
        attr_err = hipFuncSetAttribute((const void*)prefill_kernel_wide<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kPdLdsBytes);
    });
    if (attr_err != hipSuccess) { set_last_error("hipFuncSetAttribute: %s", hipGetErrorString(attr_err)); return HI_ERR_HIP; }
    dim3 grid((unsigned)(pl.nbk * pl.split), (unsigned)(gy * n_heads));
    const bool mfma32 = (variant & 16) != 0;        // the 32x32x16 form of the kernel (its state images differ)
    // the 4-wave, 64-rows-per-wavefront form of the 16x16x32 kernel: for launches long enough to pay for its slow
    // straight-line tiles (it gains about 3 % per steady-state tile and loses about 20 tiles' worth at the ends)
    const bool wide = !mfma32 && ((variant & 128) != 0 ||
                                  ((variant & 64) == 0 && (sa.n + sb.n) / kPfTileRows >= kPrefillWideMinTiles));
    if (mfma32) hipLaunchKernelGGL(prefill_kernel_deep, grid, dim3(kPdWaves * 64), kPdLdsBytes, (hipStream_t)stream, a);
    else if (wide && q_prescaled) hipLaunchKernelGGL(prefill_kernel_wide<true>, grid, dim3(kPwWaves * 64), kPdLdsBytes, (hipStream_t)stream, a);
    else if (wide) hipLaunchKernelGGL(prefill_kernel_wide<false>, grid, dim3(kPwWaves * 64), kPdLdsBytes, (hipStream_t)stream, a);
    else if (q_prescaled) hipLaunchKernelGGL(prefill_kernel_deep16<true>, grid, dim3(kPdWaves * 64), kPdLdsBytes, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(prefill_kernel_deep16<false>, grid, dim3(kPdWaves * 64), kPdLdsBytes, (hipStream_t)stream, a);
    if (pl.merge) {
      hipError_t e1 = hipGetLastError();
      if (e1 != hipSuccess) { set_last_error("prefill launch: %s", hipGetErrorString(e1)); return HI_ERR_HIP; }
      if (mfma32) hipLaunchKernelGGL(prefill_merge_kernel, dim3((unsigned)pl.nbk, grid.y, 4), dim3(kPdWaves * 64), 0, (hipStream_t)stream, a);
      else hipLaunchKernelGGL(prefill_merge16_kernel, dim3((unsigned)pl.nbk, grid.y, 4), dim3(kPdWaves * 64), 0, (hipStream_t)stream, a);
    }
  } else {
    dim3 grid((unsigned)ceil_div(chunk_len, strip), (unsigned)(gy * n_heads));
    hipLaunchKernelGGL(prefill_kernel, grid, dim3(kWgThreads), 0, (hipStream_t)stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("prefill launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

hi_status launch_prefill_window(void* stream, const void* q, int G, int chunk_len, const void* store_k,
                                const void* store_v, int64_t store_head_stride, const void* k_new, const void* v_new,
                                int64_t past_len, int n_sink, int n_recent, void* out, int out_fp32, int n_heads,
                                bool q_prescaled) {
  if (n_heads < 1 || chunk_len < 1 || !(G == 1 || G == 2 || G == 4 || G == 8) || past_len < 0 || n_sink < 0 ||
      n_recent < 1 || (int64_t)n_sink + n_recent > kStreamMaxRows) {
    set_last_error("windowed prefill launch: bad shape");
    return HI_ERR_ARG;
  }
  PrefillWindowArgs a;
  a.q = (const uint16_t*)q;
  a.ks = (const char*)store_k; a.vs = (const char*)store_v;
  a.kb = (const char*)k_new; a.vb = (const char*)v_new;
  a.out = out;
  a.G = G; a.C = chunk_len; a.out_fp32 = out_fp32;
  a.gy = prefill_grid_y(G);
  a.c = softmax_scale_log2(q_prescaled);
  a.n_sink = n_sink; a.n_recent = n_recent;
  const int64_t P = past_len;
  const int64_t t0 = P - n_recent + 1 > n_sink ? P - n_recent + 1 : n_sink;
  a.ns = (int)(P < n_sink ? P : n_sink);
  a.m = (int)(P > t0 ? P - t0 : 0);
  a.ring0 = a.m > 0 ? (int)((t0 - n_sink) % n_recent) : 0;
  a.lo0 = (int)(P - n_recent - t0 + 1) + a.ns;       // token P - n_recent + 1 as an index into A
  a.sink_b = (int)(n_sink > P ? (n_sink - P < chunk_len ? n_sink - P : chunk_len) : 0);
  a.s_head_stride = store_head_stride;
  dim3 grid((unsigned)ceil_div(chunk_len, prefill_strip(G)), (unsigned)(a.gy * n_heads));
  hipLaunchKernelGGL(prefill_window_kernel, grid, dim3(kWgThreads), 0, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("windowed prefill launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

hi_status launch_stream_store_update(void* stream, const void* k_new, const void* v_new, int chunk_len,
                                     int64_t past_len, int n_sink, int n_recent, void* store_k, void* store_v,
                                     int64_t store_head_stride, int n_heads) {
  if (n_heads < 1 || chunk_len < 1 || past_len < 0 || n_sink < 0 || n_recent < 1) {
    set_last_error("store update launch: bad shape");
    return HI_ERR_ARG;
  }
  const int cs = (int)(n_sink > past_len ? (n_sink - past_len < chunk_len ? n_sink - past_len : chunk_len) : 0);
  int u0r = chunk_len - n_recent;
  if (u0r < cs) u0r = cs;
  const int cr = chunk_len - u0r;
  if (cs + cr == 0) return HI_OK;
  dim3 grid((unsigned)ceil_div((int64_t)(cs + cr) * 16, 256), (unsigned)n_heads, 2);
  hipLaunchKernelGGL(stream_store_update_kernel, grid, dim3(256), 0, (hipStream_t)stream, (const char*)k_new,
                     (const char*)v_new, (char*)store_k, (char*)store_v, chunk_len, past_len, n_sink, n_recent, cs, u0r,
                     cr, store_head_stride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("store update launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

}  // namespace hi
