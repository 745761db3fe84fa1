// Device-side helpers shared by the HiRE kernels: bf16 decoding, order-preserving
// integer keys, wave64 and workgroup reductions/scans.  gfx950 only (wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hire {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Number of set bits of `mask` below this lane.
__device__ __forceinline__ int mask_prefix(uint64_t mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---- bf16 ----------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xFFFF0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Nearest bf16 of a double, round-half-even, straight from the binary64 bits
// (no intermediate binary32, which would round twice).  Finite inputs whose
// result is a normal bf16; smaller magnitudes flush through the generic path.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double v) {
  uint64_t u = (uint64_t)__double_as_longlong(v);
  uint32_t sign = (uint32_t)(u >> 48) & 0x8000u;
  int e = (int)((u >> 52) & 0x7FF);
  uint64_t man = u & 0x000FFFFFFFFFFFFFull;
  if (e == 0) return (uint16_t)sign;                       // zero / binary64 subnormal
  int e32 = e - 1023 + 127;
  if (e32 >= 255) return (uint16_t)(sign | 0x7F80u);       // overflow -> inf
  if (e32 <= 0) {
    // result is a bf16 subnormal (spacing 2^-133) or zero: round the scaled value
    double q = rint(fabs(v) * 0x1p133);                    // exact scaling, half-even
    return (uint16_t)(sign | (uint32_t)q);                 // q <= 128 -> carries into the exponent field
  }
  // keep 7 mantissa bits out of 52
  uint64_t keep = man >> 45;
  uint64_t rest = man & ((1ull << 45) - 1);
  uint64_t half = 1ull << 44;
  uint32_t r = ((uint32_t)e32 << 7) | (uint32_t)keep;
  if (rest > half || (rest == half && (keep & 1))) r += 1; // may carry into the exponent: still correct
  return (uint16_t)(sign | r);
}

// ---- order-preserving unsigned keys ----------------------------------------
// a < b (as numbers, with -0 == +0 canonicalised to +0)  <=>  key(a) < key(b).
__device__ __forceinline__ uint32_t order_key(float v) {
  if (v == 0.0f) v = 0.0f;
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ uint64_t order_key(double v) {
  if (v == 0.0) v = 0.0;
  uint64_t u = (uint64_t)__double_as_longlong(v);
  return (u & 0x8000000000000000ull) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __uint_as_float(u);
}
__device__ __forceinline__ double key_value(uint64_t k) {
  uint64_t u = (k & 0x8000000000000000ull) ? (k & 0x7FFFFFFFFFFFFFFFull) : ~k;
  return __longlong_as_double((long long)u);
}

// ---- wave64 reductions -----------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T w = __shfl_xor(v, o);
    v = w > v ? w : v;
  }
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_min(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T w = __shfl_xor(v, o);
    v = w < v ? w : v;
  }
  return v;
}
// Inclusive prefix sum over the lanes of a wave.
__device__ __forceinline__ int wave_scan_incl(int v) {
  int l = lane_id();
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    int w = __shfl_up(v, o);
    if (l >= o) v += w;
  }
  return v;
}

__device__ __forceinline__ int ilog2_u64(uint64_t v) { return 63 - __clzll((long long)v); }

}  // namespace hire
