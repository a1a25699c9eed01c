// K2 (split-KV decode attention) and K3 (log-sum-exp combine) for gfx950.
//
// Algorithm 1, decode phase: one new query row per query head attends over the head's whole K/V history
// (Eq. 3 / Eq. 9).  The work is bandwidth bound (Section 5: decode intensity is O(1) flop per byte), so the
// kernel is organised around the memory pipeline: every wavefront streams its share of the 16-row
// K/V blocks through a private 4-stage LDS ring filled by direct-to-LDS 128-bit loads (24 KiB in flight per
// wavefront, nothing staged in VGPRs, no workgroup barriers in the loop).  The G <= 16 query heads ride along
// as the 16 columns of small MFMA tiles (S^T = K Q^T, O^T += V^T P^T), which keeps the vector ALU nearly idle;
// the matrix unit runs at a few percent of its rate and is not the bound.
#include <mutex>
#include "hi_device.h"
#include "hi_internal.h"

namespace hi {

constexpr int kDecStages = 4;
constexpr int kDecBlockRows = 16;
constexpr int kDecTileBytes = kDecBlockRows * kRowBytes;         // 4 KiB of K (or V)
constexpr int kDecStageBytes = 2 * kDecTileBytes;                // K tile then V tile
constexpr int kDecWaveLds = kDecStages * kDecStageBytes;         // 32 KiB per wavefront
constexpr int kDecLdsBytes = 4 * kDecWaveLds;                    // 128 KiB per workgroup

// issue the 8 loads (4 K + 4 V) of block `blk` into `stage`; rows beyond n-1 re-read row n-1 (masked later)
__device__ __forceinline__ void dec_issue_block(const char* __restrict__ k, const char* __restrict__ v, int64_t blk,
                                                int64_t n, lds_char* stage, int lane) {
  const int r_in = lane >> 4;        // row within the 4-row group of one load instruction
  const int cpos = lane & 15;        // LDS chunk position within the row
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 4 * i + r_in;
    int64_t row = blk * kDecBlockRows + r;
    row = row < n ? row : n - 1;
    const int ck = cpos ^ (r & 15);          // K swizzle
    const int cv = cpos ^ ((r & 7) << 1);    // V swizzle
    g2lds16_stream(k + row * kRowBytes + ck * 16, stage + i * 1024);
    g2lds16_stream(v + row * kRowBytes + cv * 16, stage + kDecTileBytes + i * 1024);
  }
}

// RAGGED: the heads of the launch have their own numbers of rows (sequences of different lengths served as more KV
// heads); a head with fewer 16-row blocks than the grid has wavefronts leaves neutral partials.
template <bool RAGGED>
__global__ __launch_bounds__(256) void decode_partial_kernel(const uint16_t* __restrict__ q, int G,
                                                             const char* __restrict__ k, const char* __restrict__ v,
                                                             int64_t n, float* __restrict__ partials, int part0,
                                                             float c, int64_t kv_head_stride,
                                                             int64_t part_head_stride, int64_t skip_row,
                                                             DecodeLens lens) {
  // group launches: blockIdx.y is the head
  if (RAGGED) n = lens.n[blockIdx.y];
  q += (int64_t)blockIdx.y * G * kHeadDim;
  k += blockIdx.y * kv_head_stride;
  v += blockIdx.y * kv_head_stride;
  partials += blockIdx.y * part_head_stride;
  extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
  lds_char* lds = (lds_char*)lds_raw;
  const int lane = lane_id();
  const int wave = wave_id();
  lds_char* wlds = lds + wave * kDecWaveLds;

  const int head = lane & 15;
  const int g4 = lane >> 4;

  // Q^T as the B operand of S^T = K Q^T: lane holds q[head][32*kk + 8*g4 .. +7]; heads >= G are zero columns
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (head < G) raw = *(const uint4*)(q + head * kHeadDim + 32 * kk + 8 * g4);
    qf[kk] = __builtin_bit_cast(bf16x8, raw);
  }
  // make the compiler wait for these loads here, not inside the loop (a vmcnt(0) there would drain the ring)
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[kk]));

  // 16-row blocks are dealt round-robin to the wavefronts of the grid, so at any moment the whole chip reads one
  // compact window of the K and V streams (friendlier to HBM pages and TLBs than one far-apart range per wave)
  const int64_t n_blocks = (n + kDecBlockRows - 1) / kDecBlockRows;
  const int64_t n_waves = (int64_t)gridDim.x * 4;
  const int64_t wid = (int64_t)blockIdx.x * 4 + wave;
  const int64_t cnt = wid < n_blocks ? (n_blocks - wid + n_waves - 1) / n_waves : 0;   // blocks of this wave
  const int64_t skip_blk = skip_row >= 0 ? skip_row / kDecBlockRows : -1;

  float m = kNegBig, l = 0.f;
  f32x4 o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // prologue: up to three blocks in flight
  for (int s = 0; s < kDecStages - 1; ++s)
    if (s < cnt) dec_issue_block(k, v, wid + s * n_waves, n, wlds + s * kDecStageBytes, lane);

  // lane-constant LDS offsets of the operand reads
  const int k_tok = lane & 15;
  const int v_row = 4 * g4 + ((lane & 15) >> 2);
  const int v_sub = lane & 3;      // which 8-byte quarter of the 32-byte column group

  for (int64_t i = 0; i < cnt; ++i) {
    const int64_t b = wid + i * n_waves;
    const int stage = (int)(i & (kDecStages - 1));
    if (i + (kDecStages - 1) < cnt) {
      dec_issue_block(k, v, b + (kDecStages - 1) * n_waves, n,
                      wlds + (int)((i + kDecStages - 1) & (kDecStages - 1)) * kDecStageBytes, lane);
      wait_vmcnt<24>();   // everything but the 3 newest blocks has landed
    } else {
      wait_vmcnt<0>();
    }
    lds_char* kt = wlds + stage * kDecStageBytes;
    lds_char* vt = kt + kDecTileBytes;

    f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 a = lds_read16(kt + k_tok * kRowBytes + (((4 * kk + g4) ^ k_tok) << 4));
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[kk], s, 0, 0, 0);
    }
    // register r of lane (g4, head) is the score of row 16*b + 4*g4 + r
    // hidden rows: beyond the end, or the one row a streaming head's token is about to replace
    const bool hides = (b + 1) * kDecBlockRows > n || b == skip_blk;
    if (hides) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t row = b * kDecBlockRows + 4 * g4 + r;
        if (row >= n || row == skip_row) s[r] = kNegBig;
      }
    }
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
      const float alpha = fast_exp2((m - m_new) * c);
      l *= alpha;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] *= alpha;
      m = m_new;
    }
    const float mc = m * c;
    float p[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) p[r] = fast_exp2(__builtin_fmaf(s[r], c, -mc));
    if (hides) {   // exactly zero even while nothing visible has been seen (m still at its initial value)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (s[r] == kNegBig) p[r] = 0.f;
    }
    l += (p[0] + p[1]) + (p[2] + p[3]);
    bf16x4 pb;
#pragma unroll
    for (int r = 0; r < 4; ++r) pb[r] = (__bf16)p[r];
    const short4v pbs = __builtin_bit_cast(short4v, pb);
#pragma unroll
    for (int db = 0; db < 8; ++db) {
      // V^T operand: lane receives dim 16*db + (lane & 15) of rows 4*g4 .. 4*g4+3
      const int chunk = (2 * db + (v_sub >> 1)) ^ ((v_row & 7) << 1);
      bf16x4 a = lds_read_tr8(vt + v_row * kRowBytes + (chunk << 4) + ((v_sub & 1) << 3));
      o[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4v, a), pbs, o[db], 0, 0, 0);
    }
    asm volatile("" ::: "memory");
  }

  // per-lane-group partial sums -> per-head sums
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // merge the four wavefronts through LDS (the ring is idle now)
  __syncthreads();
  float* red = (float*)lds_raw;                 // [4 waves][16 heads][130]
  float* mine = red + wave * 16 * kPartialFloats;
#pragma unroll
  for (int db = 0; db < 8; ++db)
#pragma unroll
    for (int r = 0; r < 4; ++r) mine[head * kPartialFloats + 16 * db + 4 * g4 + r] = o[db][r];
  if (g4 == 0) {
    mine[head * kPartialFloats + kHeadDim] = m;
    mine[head * kPartialFloats + kHeadDim + 1] = l;
  }
  __syncthreads();
  float* dst = partials + (int64_t)(part0 + blockIdx.x) * G * kPartialFloats;
  for (int idx = threadIdx.x; idx < G * kHeadDim; idx += blockDim.x) {
    const int h = idx >> 7, dim = idx & 127;
    float mw[4], M = kNegBig;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mw[w] = red[(w * 16 + h) * kPartialFloats + kHeadDim];
      M = fmaxf(M, mw[w]);
    }
    float acc = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = fast_exp2((mw[w] - M) * c);
      acc += wgt * red[(w * 16 + h) * kPartialFloats + dim];
      L += wgt * red[(w * 16 + h) * kPartialFloats + kHeadDim + 1];
    }
    dst[h * kPartialFloats + dim] = acc;
    if (dim == 0) {
      dst[h * kPartialFloats + kHeadDim] = M;
      dst[h * kPartialFloats + kHeadDim + 1] = L;
    }
  }
}

// K3: out[g][:] = (sum_s O_s w_s + p_new v_new) / (sum_s l_s w_s + p_new),  w_s = 2^{(m_s - M) c},
// p_new = 2^{(q_g . k_new - M) c}, M = max(max_s m_s, q_g . k_new).   grid (G, 8): one query head, 16 dims;
// thread = (one of 16 partition lanes, one dim), several independent loads in flight per thread.
constexpr int kCombDims = 16;
constexpr int kCombLanes = 256 / kCombDims;

__global__ __launch_bounds__(256) void decode_combine_kernel(const uint16_t* __restrict__ q, int G,
                                                             const uint16_t* __restrict__ k_new,
                                                             const uint16_t* __restrict__ v_new,
                                                             const float* __restrict__ partials, int n_part,
                                                             void* __restrict__ out, int out_fp32, float c,
                                                             uint16_t* __restrict__ k_append,
                                                             uint16_t* __restrict__ v_append,
                                                             int64_t part_head_stride, int64_t append_head_stride,
                                                             int ragged, DecodeLens lens) {
  // group launches: blockIdx.z is the head
  q += (int64_t)blockIdx.z * G * kHeadDim;
  k_new += blockIdx.z * kHeadDim;
  v_new += blockIdx.z * kHeadDim;
  partials += blockIdx.z * part_head_stride;
  out = (char*)out + (int64_t)blockIdx.z * G * kHeadDim * (out_fp32 ? 4 : 2);
  if (k_append != nullptr) {
    // (ragged: k_append / v_append point at row 0 of the first head; each head appends at its own length)
    const int64_t row_off = ragged ? lens.n[blockIdx.z] * kRowBytes : 0;
    k_append = (uint16_t*)((char*)k_append + blockIdx.z * append_head_stride + row_off);
    v_append = (uint16_t*)((char*)v_append + blockIdx.z * append_head_stride + row_off);
  }
  __shared__ float red[4];
  __shared__ float red_o[kCombLanes][kCombDims + 1];
  __shared__ float bc;
  const int g = blockIdx.x;
  const int tid = threadIdx.x;
  const float* base = partials + (int64_t)g * kPartialFloats;
  const int64_t stride = (int64_t)G * kPartialFloats;

  // HBM-resident cache: the token's K/V row is appended here instead of by two tiny device copies
  if (k_append != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && tid < kHeadDim) {
    k_append[tid] = k_new[tid];
    v_append[tid] = v_new[tid];
  }

  // score of the token's own row (first wavefront), and the maximum over all partitions
  float mx = kNegBig;
  for (int p = tid; p < n_part; p += 256) mx = fmaxf(mx, base[p * stride + kHeadDim]);
  if (tid < 64) {
    float d = bf16_bits_to_float(q[g * kHeadDim + tid]) * bf16_bits_to_float(k_new[tid]) +
              bf16_bits_to_float(q[g * kHeadDim + 64 + tid]) * bf16_bits_to_float(k_new[64 + tid]);
    for (int off = 32; off > 0; off >>= 1) d += __shfl_xor(d, off);
    if (tid == 0) bc = d;
  }
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  const float s_new = bc;
  const float M = fmaxf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])), s_new);

  const int pl = tid / kCombDims;
  const int dim = blockIdx.y * kCombDims + (tid % kCombDims);
  float acc = 0.f, L = 0.f;
#pragma unroll 4
  for (int p = pl; p < n_part; p += kCombLanes) {
    const float* src = base + p * stride;
    const float w = fast_exp2((src[kHeadDim] - M) * c);
    acc = __builtin_fmaf(w, src[dim], acc);
    L = __builtin_fmaf(w, src[kHeadDim + 1], L);
  }
  red_o[pl][tid % kCombDims] = acc;
  if ((tid % kCombDims) == 0) red_o[pl][kCombDims] = L;
  __syncthreads();
  if (tid < kCombDims) {
    float a = 0.f, lsum = 0.f;
#pragma unroll
    for (int i = 0; i < kCombLanes; ++i) { a += red_o[i][tid]; lsum += red_o[i][kCombDims]; }
    const float p_new = fast_exp2((s_new - M) * c);
    a += p_new * bf16_bits_to_float(v_new[dim]);
    lsum += p_new;
    const float r = a / lsum;
    if (out_fp32) ((float*)out)[g * kHeadDim + dim] = r;
    else ((uint16_t*)out)[g * kHeadDim + dim] = float_to_bf16_bits(r);
  }
}


hi_status launch_decode_partial(void* stream, const void* q, int G, const void* k, const void* v, int64_t n,
                                int n_split, void* partials, int part0, bool q_prescaled, int n_heads,
                                int64_t kv_head_stride, int64_t part_head_stride, int64_t skip_row,
                                const DecodeLens* lens) {
  if (n <= 0 || n_split <= 0 || n_heads < 1 || (lens && n_heads > kDecodeMaxRagged)) { set_last_error("decode partial: empty launch"); return HI_ERR_ARG; }
  static std::once_flag attr_once;      // contexts on different host threads may get here together
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [] {
    attr_err = hipFuncSetAttribute((const void*)decode_partial_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   kDecLdsBytes);
    if (attr_err == hipSuccess)
      attr_err = hipFuncSetAttribute((const void*)decode_partial_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     kDecLdsBytes);
  });
  if (attr_err != hipSuccess) { set_last_error("hipFuncSetAttribute: %s", hipGetErrorString(attr_err)); return HI_ERR_HIP; }
  static const DecodeLens no_lens = {};
  if (lens)
    hipLaunchKernelGGL(decode_partial_kernel<true>, dim3(n_split, n_heads), dim3(256), kDecLdsBytes, (hipStream_t)stream,
                       (const uint16_t*)q, G, (const char*)k, (const char*)v, n, (float*)partials, part0, softmax_scale_log2(q_prescaled),
                       kv_head_stride, part_head_stride, skip_row, *lens);
  else
    hipLaunchKernelGGL(decode_partial_kernel<false>, dim3(n_split, n_heads), dim3(256), kDecLdsBytes, (hipStream_t)stream,
                       (const uint16_t*)q, G, (const char*)k, (const char*)v, n, (float*)partials, part0, softmax_scale_log2(q_prescaled),
                       kv_head_stride, part_head_stride, skip_row, no_lens);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("decode_partial launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

hi_status launch_decode_combine(void* stream, const void* q, int G, const void* k_new, const void* v_new,
                                const void* partials, int n_part, void* out, int out_fp32, void* k_append,
                                void* v_append, bool q_prescaled, int n_heads, int64_t part_head_stride,
                                int64_t append_head_stride, const DecodeLens* lens) {
  static const DecodeLens no_lens = {};
  if (lens && n_heads > kDecodeMaxRagged) { set_last_error("decode combine: too many heads of their own length"); return HI_ERR_ARG; }
  hipLaunchKernelGGL(decode_combine_kernel, dim3(G, kHeadDim / kCombDims, n_heads), dim3(256), 0, (hipStream_t)stream,
                     (const uint16_t*)q, G, (const uint16_t*)k_new, (const uint16_t*)v_new, (const float*)partials,
                     n_part, out, out_fp32, softmax_scale_log2(q_prescaled), (uint16_t*)k_append, (uint16_t*)v_append, part_head_stride,
                     append_head_stride, lens ? 1 : 0, lens ? *lens : no_lens);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("decode_combine launch: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

}  // namespace hi
