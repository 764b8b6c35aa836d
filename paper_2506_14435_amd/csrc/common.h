// Shared device helpers for the gfx950 MoTE kernels: vector types, bf16 conversion,
// wavefront reductions.  Everything here assumes 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mote {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));  // 16-byte register quad (plain vector: stays in VGPRs)
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr float kEps = 1e-5f;  // clamp of alpha and beta (zero matrix / zero token)

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// Two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// SiLU(g) = g / (1 + exp(-g)) on the hardware exp2 / reciprocal units (about 2 ulp).
__device__ __forceinline__ float silu_fast(float g) {
  const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
  return g * __builtin_amdgcn_rcpf(1.0f + e);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Q_a element (Eq.8, Eq.10): clip(round_half_even(x * s), -128, 127), one fp32 multiply.
__device__ __forceinline__ int quant_i8(float x, float s) {
  float r = rintf(x * s);
  r = fminf(fmaxf(r, -128.0f), 127.0f);
  return static_cast<int>(r);
}

// One 32-bit word of the packed ternary format = 16 codes t+1, code i at bit 8*(i%4) + 2*(i/4):
// (w >> 2j) & 0x03030303 are the four int8 operand registers of one v_mfma_i32_32x32x32_i8.
__device__ __forceinline__ v4i unpack_codes(uint32_t w) {
  v4i b;
  b.x = static_cast<int>(w & 0x03030303u);
  b.y = static_cast<int>((w >> 2) & 0x03030303u);
  b.z = static_cast<int>((w >> 4) & 0x03030303u);
  b.w = static_cast<int>((w >> 6) & 0x03030303u);
  return b;
}

// Load of a wavefront-uniform value through the constant address space: a scalar load
// (s_load, counted by lgkmcnt) instead of a vector-memory operation.  Only for memory that no
// kernel writes while this one runs.
template <typename T>
__device__ __forceinline__ T load_uniform(const T* p) {
  return *(const __attribute__((address_space(4))) T*)(p);
}

}  // namespace mote
