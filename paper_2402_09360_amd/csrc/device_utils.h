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

// ---- streaming loads --------------------------------------------------------
// 16-byte load marked non-temporal: for weight rows that are read once per step in whole cache lines per
// instruction (a wave reading 1 KB of a row), so that they do not displace the small, re-read working set (keys,
// histograms, tokens) from the caches.  Measured on the 263 MB vocabulary scorer: 5.8 -> 6.4 TB/s.  Not for the
// matrix-core kernels, whose loads take 64 bytes of a row at a time.
__device__ __forceinline__ uint4 load_streaming(const uint4* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
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

// ---- wave64 reductions on the DPP data path ---------------------------------
// Cross-lane moves inside the vector ALU (row shifts within 16 lanes, then the row_bcast steps across rows)
// instead of LDS permutes: a 64-lane reduction is six dependent VALU operations.  After the sequence lane 63
// holds the reduction of all lanes and lane l the inclusive prefix over lanes 0..l.
template <int CTRL, int ROW_MASK, typename T>
__device__ __forceinline__ T dpp_move(T identity, T v) {
  static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit values");
  if constexpr (sizeof(T) == 4) {
    int o, x;
    __builtin_memcpy(&o, &identity, 4);
    __builtin_memcpy(&x, &v, 4);
    const int r = __builtin_amdgcn_update_dpp(o, x, CTRL, ROW_MASK, 0xF, false);
    T out;
    __builtin_memcpy(&out, &r, 4);
    return out;
  } else {
    int o[2], x[2], r[2];
    __builtin_memcpy(o, &identity, 8);
    __builtin_memcpy(x, &v, 8);
    r[0] = __builtin_amdgcn_update_dpp(o[0], x[0], CTRL, ROW_MASK, 0xF, false);
    r[1] = __builtin_amdgcn_update_dpp(o[1], x[1], CTRL, ROW_MASK, 0xF, false);
    T out;
    __builtin_memcpy(&out, r, 8);
    return out;
  }
}

template <typename T, typename Op>
__device__ __forceinline__ T wave_prefix(T v, T identity, Op op) {
  v = op(v, dpp_move<0x111, 0xF>(identity, v));  // row_shr:1
  v = op(v, dpp_move<0x112, 0xF>(identity, v));  // row_shr:2
  v = op(v, dpp_move<0x114, 0xF>(identity, v));  // row_shr:4
  v = op(v, dpp_move<0x118, 0xF>(identity, v));  // row_shr:8
  v = op(v, dpp_move<0x142, 0xA>(identity, v));  // row_bcast:15 into rows 1 and 3
  v = op(v, dpp_move<0x143, 0xC>(identity, v));  // row_bcast:31 into rows 2 and 3
  return v;
}

template <typename T>
__device__ __forceinline__ T read_lane63(T v) {
  if constexpr (sizeof(T) == 4) {
    int x;
    __builtin_memcpy(&x, &v, 4);
    x = __builtin_amdgcn_readlane(x, 63);
    T out;
    __builtin_memcpy(&out, &x, 4);
    return out;
  } else {
    int x[2];
    __builtin_memcpy(x, &v, 8);
    x[0] = __builtin_amdgcn_readlane(x[0], 63);
    x[1] = __builtin_amdgcn_readlane(x[1], 63);
    T out;
    __builtin_memcpy(&out, x, 8);
    return out;
  }
}

// Value of lane `src` (wave-uniform index), to all lanes.
template <typename T>
__device__ __forceinline__ T read_lane(T v, int src) {
  if constexpr (sizeof(T) == 4) {
    int x;
    __builtin_memcpy(&x, &v, 4);
    x = __builtin_amdgcn_readlane(x, src);
    T out;
    __builtin_memcpy(&out, &x, 4);
    return out;
  } else {
    int x[2];
    __builtin_memcpy(x, &v, 8);
    x[0] = __builtin_amdgcn_readlane(x[0], src);
    x[1] = __builtin_amdgcn_readlane(x[1], src);
    T out;
    __builtin_memcpy(&out, x, 8);
    return out;
  }
}

// Sum / max / min over the 64 lanes, returned to every lane (wave-uniform).
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
  return read_lane63(wave_prefix(v, (T)0, [](T a, T b) { return a + b; }));
}
// identity: the type's lowest value for max, highest for min; the callers here reduce unsigned keys and
// non-negative floats, for which 0 is the lowest value
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
  return read_lane63(wave_prefix(v, (T)0, [](T a, T b) { return b > a ? b : a; }));
}
template <typename T>
__device__ __forceinline__ T wave_min(T v) {
  return read_lane63(wave_prefix(v, (T)~(T)0, [](T a, T b) { return b < a ? b : a; }));
}
// Inclusive prefix sum over the lanes of a wave.
__device__ __forceinline__ int wave_scan_incl(int v) {
  return wave_prefix(v, 0, [](int a, int b) { return a + b; });
}

__device__ __forceinline__ int ilog2_u64(uint64_t v) { return 63 - __clzll((long long)v); }

}  // namespace hire
