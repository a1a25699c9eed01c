// Device-side building blocks shared by the prefill and decode kernels (gfx950 only).
//
// K/V tiles travel HBM -> LDS with direct-to-LDS 128-bit loads (no VGPR staging).  The hardware writes lane i's
// 16 bytes at (uniform LDS base) + 16*i, so the LDS image is "lane order"; bank conflicts of the later MFMA
// operand reads are avoided by choosing WHICH global 16-byte chunk each lane fetches: LDS chunk position p of
// row r holds global chunk p ^ swz(r).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace hi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(1))) const char glb_char;

constexpr float kNegBig = -1.0e30f;   // finite stand-in for -inf: exp2 of (kNegBig - m) * c underflows to 0

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

// 16 bytes per lane, global -> LDS at lds_uniform + 16 * lane (M0 carries the wave-uniform LDS byte address).
// Issued as opaque assembly on purpose: the compiler then keeps no record of an asynchronous LDS write, so it
// never guards later LDS reads with a full vmcnt(0) drain; the kernels place their own `s_waitcnt vmcnt(N)`
// before touching a tile, which is what lets several tiles stay in flight.  M0 is written without being declared
// (the compiler rejects it as a clobber); nothing else in these kernels uses M0: no dynamic register indexing,
// no compiler-issued LDS-DMA.
__device__ __forceinline__ void g2lds16_stream(const char* gsrc, lds_char* lds_uniform) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_uniform);
  // non-temporal: the decode kernel reads every K/V byte exactly once; keeping the stream from displacing the L2's
  // contents measured 5.9 -> 6.6 TB/s over a million rows
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt"
               :
               : "s"(m0v), "v"(gsrc)
               : "memory");
}

// Same, addressed as (64-bit scalar base) + (32-bit per-lane byte offset) + immediate: no vector ALU work per load.
// The instruction's immediate offset is added to the global address and to the LDS address alike.
template <int IMM>
__device__ __forceinline__ void g2lds16_s(const char* sbase, uint32_t voff, uint32_t lds_uniform_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
               :
               : "s"(lds_uniform_addr), "v"(voff), "s"(sbase), "n"(IMM)
               : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ bf16x8 lds_read16(lds_char* p) {
  return *(__attribute__((address_space(3))) bf16x8*)p;
}

// LDS transpose read: within each group of 16 lanes, lane s supplies the address of 4 consecutive bf16 (one
// row of a 4-row x 16-column block: row s/4, columns 4*(s%4)..+3); lane L receives column L of the 4 rows.
__device__ __forceinline__ bf16x4 lds_read_tr8(lds_char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4*)p);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

}  // namespace hi
