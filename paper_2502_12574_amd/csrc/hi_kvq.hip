// 4-bit K/V rows for the far side of the host link (Appendix B / Section 6.3 describe the 4-bit representation as a
// stand-alone baseline; here it is what an offloaded head's rows look like in host memory and on the link, which is
// the bound of offloaded decode, Section 3.3).
//
// Format of one row of 128 channels (80 bytes): 64 bytes of codes (channel 2i in the low nibble of byte i), then
// 4 bf16 scales and 4 bf16 zeros, one pair per group of 32 channels.  Arithmetic, one binary32 rounding per step:
//   zero = min of the group, s = (max - min) * (1/15), scale = bf16(s) (0 if below 2^-120),
//   code = min(15, rint((x - zero) * (1 / scale))),  x^ = bf16(zero + code * scale).
// Both kernels move planes of rows: plane p starts p * pitch bytes after the base on either side, so one launch
// covers the K and V slices of every head of a group.  Pure streaming work: HBM-bound, one pass.
#include <hip/hip_runtime.h>
#include "hi_device.h"
#include "hi_internal.h"

namespace hi {

namespace {

constexpr int kRowsPerWg = 64;       // 256 threads: 4 groups of 32 channels per row

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(256) void kv_quant_kernel(const char* __restrict__ src, int64_t src_pitch,
                                                       char* __restrict__ dst, int64_t dst_pitch, int64_t rows) {
  const int g = threadIdx.x & 3;
  const int64_t row = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 2);
  const bool live = row < rows;
  const int64_t r = live ? row : rows - 1;                       // keep every lane in the shuffles below
  const char* s = src + (int64_t)blockIdx.y * src_pitch + r * kRowBytes + g * 64;
  u32x4 w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = *(const u32x4*)(s + 16 * i);
  float x[32];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[8 * i + 2 * j] = __uint_as_float(w[i][j] << 16);
      x[8 * i + 2 * j + 1] = __uint_as_float(w[i][j] & 0xFFFF0000u);
    }
  float mn = x[0], mx = x[0];
#pragma unroll
  for (int i = 1; i < 32; ++i) {
    mn = fminf(mn, x[i]);
    mx = fmaxf(mx, x[i]);
  }
  const float s32 = __fmul_rn(__fsub_rn(mx, mn), __fdiv_rn(1.0f, 15.0f));
  uint32_t sbits = float_to_bf16_bits(s32);
  float scale = bf16_bits_to_float((uint16_t)sbits);
  if (!(scale >= 0x1p-120f)) {
    scale = 0.f;
    sbits = 0;
  }
  const float inv = scale > 0.f ? __fdiv_rn(1.0f, scale) : 0.f;
  u32x4 codes;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    uint32_t word = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float t = __fmul_rn(__fsub_rn(x[8 * i + j], mn), inv);
      const uint32_t c = (uint32_t)fminf(rintf(t), 15.0f);
      word |= c << (4 * j);
    }
    codes[i] = word;
  }
  // the four lanes of a row gather scales and zeros; lane 0 of the quad writes them as one 16-byte piece
  const uint32_t mine = sbits | ((uint32_t)float_to_bf16_bits(mn) << 16);     // zero is a bf16 value: exact
  const int base = (threadIdx.x & 63) & ~3;
  const uint32_t q0 = __shfl(mine, base + 0), q1 = __shfl(mine, base + 1), q2 = __shfl(mine, base + 2),
                 q3 = __shfl(mine, base + 3);
  if (!live) return;
  char* d = dst + (int64_t)blockIdx.y * dst_pitch + row * kLinkRowBytes4;
  *(u32x4*)(d + 16 * g) = codes;
  if (g == 0) {
    u32x4 sz;
    sz[0] = (q0 & 0xFFFFu) | (q1 << 16);
    sz[1] = (q2 & 0xFFFFu) | (q3 << 16);
    sz[2] = (q0 >> 16) | (q1 & 0xFFFF0000u);
    sz[3] = (q2 >> 16) | (q3 & 0xFFFF0000u);
    *(u32x4*)(d + 64) = sz;
  }
}

// A thread expands 8 channels (4 bytes of codes -> 16 bytes of bf16): the 16 threads of a row write its 256 bytes
// side by side, so every store instruction of a wave covers 1 KB of consecutive addresses; a workgroup takes
// kRowsPerWg rows in 4 passes of 16 rows, all loads issued before the first conversion.
__global__ __launch_bounds__(256) void kv_dequant_kernel(const char* __restrict__ src, int64_t src_pitch,
                                                         char* __restrict__ dst, int64_t dst_pitch, int64_t rows) {
  const int c = threadIdx.x & 15;
  const int g = c >> 2;
  const int64_t row0 = (int64_t)blockIdx.x * kRowsPerWg + (threadIdx.x >> 4);
  const char* sp = src + (int64_t)blockIdx.y * src_pitch;
  char* dp = dst + (int64_t)blockIdx.y * dst_pitch;
  uint32_t codes[4];
  uint16_t sb[4], zb[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int64_t row = row0 + 16 * it;
    if (row < rows) {
      const char* s = sp + row * kLinkRowBytes4;
      codes[it] = *(const uint32_t*)(s + 4 * c);
      sb[it] = *(const uint16_t*)(s + 64 + 2 * g);
      zb[it] = *(const uint16_t*)(s + 72 + 2 * g);
    }
  }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int64_t row = row0 + 16 * it;
    if (row < rows) {
      const float scale = bf16_bits_to_float(sb[it]), zero = bf16_bits_to_float(zb[it]);
      u32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float lo = __fmaf_rn((float)((codes[it] >> (8 * j)) & 15u), scale, zero);
        const float hi = __fmaf_rn((float)((codes[it] >> (8 * j + 4)) & 15u), scale, zero);
        o[j] = (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
      }
      *(u32x4*)(dp + row * kRowBytes + 16 * c) = o;
    }
  }
}

}  // namespace

hi_status launch_kv_quant(void* stream, const void* src, int64_t src_pitch, void* dst, int64_t dst_pitch,
                          int64_t rows, int planes) {
  if (rows < 0 || planes < 1 || planes > 65535) { set_last_error("kv quantise: bad shape"); return HI_ERR_ARG; }
  if (rows == 0) return HI_OK;
  if (ceil_div(rows, kRowsPerWg) > 0x7FFFFFFF) { set_last_error("kv quantise: too many rows"); return HI_ERR_RANGE; }
  hipLaunchKernelGGL(kv_quant_kernel, dim3((unsigned)ceil_div(rows, kRowsPerWg), planes), dim3(256), 0,
                     (hipStream_t)stream, (const char*)src, src_pitch, (char*)dst, dst_pitch, rows);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("kv quantise launch failed: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

hi_status launch_kv_dequant(void* stream, const void* src, int64_t src_pitch, void* dst, int64_t dst_pitch,
                            int64_t rows, int planes) {
  if (rows < 0 || planes < 1 || planes > 65535) { set_last_error("kv dequantise: bad shape"); return HI_ERR_ARG; }
  if (rows == 0) return HI_OK;
  if (ceil_div(rows, kRowsPerWg) > 0x7FFFFFFF) { set_last_error("kv dequantise: too many rows"); return HI_ERR_RANGE; }
  hipLaunchKernelGGL(kv_dequant_kernel, dim3((unsigned)ceil_div(rows, kRowsPerWg), planes), dim3(256), 0,
                     (hipStream_t)stream, (const char*)src, src_pitch, (char*)dst, dst_pitch, rows);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error("kv dequantise launch failed: %s", hipGetErrorString(e)); return HI_ERR_HIP; }
  return HI_OK;
}

}  // namespace hi

using namespace hi;

static bool kvq_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" hi_status hi_kv_quantize(void* stream, const void* rows_dev, int64_t n_rows, void* packed_dev) {
  if (!rows_dev || !packed_dev || n_rows < 0) { set_last_error("hi_kv_quantize: null buffer or negative size"); return HI_ERR_ARG; }
  if (!kvq_aligned16(rows_dev) || !kvq_aligned16(packed_dev)) { set_last_error("buffers must be 16-byte aligned"); return HI_ERR_ARG; }
  return launch_kv_quant(stream, rows_dev, 0, packed_dev, 0, n_rows, 1);
}

extern "C" hi_status hi_kv_dequantize(void* stream, const void* packed_dev, int64_t n_rows, void* rows_dev) {
  if (!rows_dev || !packed_dev || n_rows < 0) { set_last_error("hi_kv_dequantize: null buffer or negative size"); return HI_ERR_ARG; }
  if (!kvq_aligned16(rows_dev) || !kvq_aligned16(packed_dev)) { set_last_error("buffers must be 16-byte aligned"); return HI_ERR_ARG; }
  return launch_kv_dequant(stream, packed_dev, 0, rows_dev, 0, n_rows, 1);
}
