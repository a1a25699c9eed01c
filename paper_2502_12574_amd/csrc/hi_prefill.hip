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
//   * K/V tiles of 64 rows go HBM -> LDS by direct-to-LDS 128-bit loads, double buffered, swizzled for
//     conflict-free operand reads; one workgroup barrier per tile.
//   * A workgroup is 4 wavefronts = the G query heads at the same 32 positions (for G = 4), so all waves share
//     the causal boundary and sweep the same K/V tiles: 128 query rows per K/V byte fetched from L2.
//   * Workgroups of a unit sweep the K/V rows in near lock-step, so each tile is pulled from HBM about once per
//     XCD and served to the other compute units from that XCD's L2.
//
// The softmax state (m, l, O) can be carried across launches (one launch per staging slice) in a register-image
// workspace, which is how a unit is computed while later slices of its past are still on the host link.
#include "hi_device.h"
#include "hi_internal.h"

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
};

__device__ __forceinline__ int swz_k(int row) { return row & 15; }
__device__ __forceinline__ int swz_v(int row) { return ((row & 3) << 2) | (row & 2); }

// the whole workgroup loads one 64-row K tile and V tile: 8 instructions per wavefront
__device__ __forceinline__ void pf_issue_tile(const char* __restrict__ k, const char* __restrict__ v, int64_t row0,
                                              int64_t n, lds_char* stage, int wave, int lane) {
  const int r_in = lane >> 4;
  const int cpos = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (wave * 4 + i) * 4 + r_in;
    int64_t row = row0 + r;
    row = row < n ? row : n - 1;
    g2lds16(k + row * kRowBytes + ((cpos ^ swz_k(r)) << 4), stage + (wave * 4 + i) * 1024);
    g2lds16(v + row * kRowBytes + ((cpos ^ swz_v(r)) << 4), stage + kPfTileBytes + (wave * 4 + i) * 1024);
  }
}

// combine a value with the one held by lane ^ 32 (the other 32 K/V rows of the same query row)
__device__ __forceinline__ float max_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_halves(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ __launch_bounds__(256, 2) void prefill_kernel(PrefillArgs a) {
  __shared__ __attribute__((aligned(1024))) char lds_raw[kPfLdsBytes];
  lds_char* lds = (lds_char*)lds_raw;
  const int lane = lane_id();
  const int wave = wave_id();
  const int hl = lane >> 5;            // which half of the wavefront
  const int col = lane & 31;           // query row within the wave's 32

  const int gl = a.G < 4 ? a.G : 4;
  const int strip = 32 * (4 / gl);
  const int bx = gridDim.x - 1 - blockIdx.x;        // deepest causal rows are dispatched first
  const int g = blockIdx.y * 4 + (wave % gl);
  const int i0 = bx * strip + 32 * (wave / gl);     // first query position of this wave
  const int i_hi = bx * strip + strip - 1;          // last query position of the workgroup
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

  f32x16 o[4];
  float m, l;
  const int64_t wg_linear = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
  float* carry = a.carry + wg_linear * (kCarryFloatsPerLane * kWgThreads) + threadIdx.x;
  if (a.first) {
    m = kNegBig;
    l = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  } else {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = carry[(db * 16 + r) * kWgThreads];
    m = carry[64 * kWgThreads];
    l = carry[65 * kWgThreads];
  }
  // the compiler's own waits for the loads above belong here, not inside the tile loop
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(qf[kk]));
  asm volatile("" : "+v"(m), "+v"(l));
#pragma unroll
  for (int db = 0; db < 4; ++db) asm volatile("" : "+v"(o[db]));

  // tiles: segment A (all of it), then the part of segment B at or below the workgroup's causal boundary
  const int64_t ta = (a.na + kPfTileRows - 1) / kPfTileRows;
  int64_t nb_vis = a.nb < (int64_t)i_hi + 1 ? a.nb : (int64_t)i_hi + 1;
  const int64_t tb = (nb_vis + kPfTileRows - 1) / kPfTileRows;
  const int64_t T = ta + tb;

  auto issue = [&](int64_t t) {
    lds_char* stage = lds + (int)(t & (kPfStages - 1)) * kPfStageBytes;
    if (t < ta) pf_issue_tile(a.ka, a.va, t * kPfTileRows, a.na, stage, wave, lane);
    else pf_issue_tile(a.kb, a.vb, (t - ta) * kPfTileRows, a.nb, stage, wave, lane);
  };

  if (T > 0) issue(0);

  const float c = a.c;
  for (int64_t t = 0; t < T; ++t) {
    wait_vmcnt<0>();
    __syncthreads();
    if (t + 1 < T) issue(t + 1);

    lds_char* kt = lds + (int)(t & (kPfStages - 1)) * kPfStageBytes;
    lds_char* vt = kt + kPfTileBytes;

    // S^T tile: 64 K/V rows x 32 query rows; register r of sub-block sb is row 32*sb + 8*(r/4) + 4*hl + r%4
    f32x16 s[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[sb][r] = 0.f;
      const int tok = 32 * sb + col;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        bf16x8 kf = lds_read16(kt + tok * kRowBytes + (((2 * kk + hl) ^ swz_k(tok)) << 4));
        s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s[sb], 0, 0, 0);
      }
    }

    // masks: rows past the end of the segment, and (chunk's own rows) rows after the query's position
    const bool in_b = t >= ta;
    const int64_t j0 = (in_b ? (t - ta) : t) * kPfTileRows;
    const int64_t n_seg = in_b ? a.nb : a.na;
    const bool tail = j0 + kPfTileRows > n_seg;
    const bool diag = in_b && (j0 + kPfTileRows - 1 > i0);
    if (tail || diag) {
      int64_t lim = n_seg - 1;                       // last visible row index
      if (in_b && (int64_t)my_i < lim) lim = my_i;
      const int rel = (int)(lim - j0);               // rows with index > rel are masked
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 32 * sb + 8 * (r >> 2) + 4 * hl + (r & 3);
          if (row > rel) s[sb][r] = kNegBig;
        }
    }

    // online softmax (per lane = per query row; the other half-wave holds the other 32 rows of the tile)
    float mx = s[0][0];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sb][r]);
    mx = max_halves(mx);
    const float m_new = fmaxf(m, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
      const float alpha = fast_exp2((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      m = m_new;
    }
    const float mc = m * c;
    float lsum = 0.f;
    bf16x8 pb[2][2];
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
    l += lsum;

    // O^T += V^T P^T : contraction index 8*hl + j of MFMA (sb,u) is tile row 32*sb + 16*u + 8*(j/4) + 4*hl + j%4
    const int q16 = col >> 4;
    const int s16 = lane & 15;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int row_lo = 32 * sb + 16 * u + 4 * hl + (s16 >> 2);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int chunk = 4 * db + 2 * q16 + ((s16 & 3) >> 1);
          const int sub8 = (s16 & 1) << 3;
          bf16x4 v0 = lds_read_tr8(vt + row_lo * kRowBytes + ((chunk ^ swz_v(row_lo)) << 4) + sub8);
          bf16x4 v1 = lds_read_tr8(vt + (row_lo + 8) * kRowBytes + ((chunk ^ swz_v(row_lo + 8)) << 4) + sub8);
          bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[sb][u], o[db], 0, 0, 0);
        }
      }
  }

  if (!a.last) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) carry[(db * 16 + r) * kWgThreads] = o[db][r];
    carry[64 * kWgThreads] = m;
    carry[65 * kWgThreads] = l;
    return;
  }

  // normalise and write out[g][i][:]; register r of block db is dim 32*db + 8*(r/4) + 4*hl + r%4
  const float l_tot = sum_halves(l);
  const float inv = 1.0f / l_tot;
  if (my_i < a.C) {
    const int64_t base = ((int64_t)g * a.C + my_i) * kHeadDim;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int dim = 32 * db + 8 * rq + 4 * hl;
        const float x0 = o[db][4 * rq] * inv, x1 = o[db][4 * rq + 1] * inv;
        const float x2 = o[db][4 * rq + 2] * inv, x3 = o[db][4 * rq + 3] * inv;
        if (a.out_fp32) {
          *(float4*)((float*)a.out + base + dim) = make_float4(x0, x1, x2, x3);
        } else {
          uint2 pk;
          pk.x = (uint32_t)float_to_bf16_bits(x0) | ((uint32_t)float_to_bf16_bits(x1) << 16);
          pk.y = (uint32_t)float_to_bf16_bits(x2) | ((uint32_t)float_to_bf16_bits(x3) << 16);
          *(uint2*)((uint16_t*)a.out + base + dim) = pk;
        }
      }
  }
}

static const float kScaleLog2e = 1.4426950408889634f / 11.313708498984761f;   // log2(e) / sqrt(128)

hi_status launch_prefill(void* stream, const void* q, int G, int chunk_len, const PrefillSegment& sa,
                         const PrefillSegment& sb, int first, int last, void* carry, void* out, int out_fp32) {
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
  a.c = kScaleLog2e;
  const int strip = prefill_strip(G);
  dim3 grid((unsigned)ceil_div(chunk_len, strip), (unsigned)prefill_grid_y(G));
  hipLaunchKernelGGL(prefill_kernel, grid, dim3(kWgThreads), 0, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("prefill launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

}  // namespace hi
