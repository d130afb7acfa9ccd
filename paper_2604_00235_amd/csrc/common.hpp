// Shared device-side helpers for the MAC-Attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mac {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kHeadDim = 128;      // d; a K or V row is 256 bytes = 16 chunks of 16 bytes
constexpr int kTileTokens = 32;    // tokens per MFMA tile of the attention kernel (two 16-token sub-tiles)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// v_perm_b32: result bytes 0..3 are picked from the 8 bytes {hi_src(4..7), lo_src(0..3)} by the selector.
__device__ __forceinline__ uint32_t perm(uint32_t hi_src, uint32_t lo_src, uint32_t sel) {
    return __builtin_amdgcn_perm(hi_src, lo_src, sel);
}
// (lo16(first), lo16(second)) and (hi16(first), hi16(second)) packed into one dword, first in the low half
__device__ __forceinline__ uint32_t pack_lo16(uint32_t first, uint32_t second) { return perm(second, first, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi16(uint32_t first, uint32_t second) { return perm(second, first, 0x07060302u); }

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

}  // namespace mac
