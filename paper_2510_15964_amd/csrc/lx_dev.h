// Device-side helpers shared by the HIP kernels of this library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lx_launch.h"   // kBf16 / kF16

namespace lx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// The 16-bit kernels are templates over the element type of their operands: DT = kBf16
// (bfloat16) or kF16 (IEEE half).  Storage is uint16_t either way; products accumulate in fp32.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// two floats -> packed pair of 16-bit elements, round to nearest even
template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  if constexpr (DT == kF16)
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  else
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// 16-bit element (in the low half of the argument) -> float
template <int DT>
__device__ __forceinline__ float to_f32(uint32_t bits16) {
  if constexpr (DT == kF16)
    return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
  else
    return __builtin_bit_cast(float, bits16 << 16);
}

// 32x32x16 MFMA on 16-bit operands.  Operand a: lane l holds row (l % 32), k = 8*(l/32)..+7.
// Operand b: lane l holds column (l % 32), same k.  Accumulator register v of
// lane l is C[8*(v/4) + 4*(l/32) + v%4][l % 32].
template <int DT>
__device__ __forceinline__ f32x16 mfma32(uint4 a, uint4 b, f32x16 c) {
  if constexpr (DT == kF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Asynchronous 16-byte-per-lane copy global -> LDS (global_load_lds_dwordx4): lane l of the
// wave lands at lds_wave_base + 16*l; completion is counted by vmcnt.  Issued as assembly so
// that the waits are entirely under the kernel's control: for DMA it knows about, the compiler
// conservatively drains vmcnt before LDS reads and barriers, which defeats multi-stage
// pipelining.  Callers pair it with explicit s_waitcnt vmcnt(N) + barrier before reading.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_wave_base) {
  const uint32_t l = __builtin_amdgcn_readfirstlane(lds_wave_base);   // must be a scalar register
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(gptr)
               : "memory", "m0");
}
// Same with 4 bytes per lane (lane l lands at lds_wave_base + 4*l).
__device__ __forceinline__ void dma4(const void* gptr, uint32_t lds_wave_base) {
  const uint32_t l = __builtin_amdgcn_readfirstlane(lds_wave_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(l), "v"(gptr)
               : "memory", "m0");
}
// s_waitcnt vmcnt(N) alone (expcnt / lgkmcnt left open); N < 64.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Byte address of an LDS object as a wave-uniform scalar (operand of dma16).
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p);
}
// LDS-only barrier: waits for this wave's LDS traffic, not for DMA still in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#define LX_AS1 __attribute__((address_space(1)))
#define LX_AS3 __attribute__((address_space(3)))

// LDS reads by byte address.  lds_read8_tr is the transposing read (ds_read_b64_tr_b16): within
// 16 lanes, lane j receives element j of the four 16-element rows whose 8-byte quarters are
// addressed by lanes 0-3, 4-7, 8-11 and 12-15.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 lds_read16(uint32_t addr) {
  return __builtin_bit_cast(uint4, *reinterpret_cast<const LX_AS3 u32x4*>((uintptr_t)addr));
}
__device__ __forceinline__ uint2 lds_read8_tr(uint32_t addr) {
  return __builtin_bit_cast(
      uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LX_AS3 short4v*>((uintptr_t)addr)));
}

}  // namespace lx
