// Workgroup-cooperative exact selection: the k-th largest key of a set that a
// workgroup of NT threads holds in registers or streams from memory.
//
// Method (range narrowing): keep a closed key interval [lo, hi] known to
// contain the k-th largest key together with `need` = its rank inside the
// interval.  Each round bins the interval into 2048 bins in LDS, walks the
// bins from the top to the one holding the rank, and tightens [lo, hi] to the
// keys of that bin.  The first round bins linearly in *value* space (a bell
// shaped distribution then spreads over all bins and LDS atomics rarely
// collide); later rounds bin the integer key space, which removes at least 11
// bits of range per round and therefore terminates.  Once at most 64 keys are
// left they are ranked directly.  Bin 0 is never counted with atomics (ReLU
// zeros would all collide there); its population follows from the total.
#pragma once

#include "device_utils.h"

// Phase stamps for a profiling build (-DHIRE_TIMESTAMPS): thread 0 of workgroup (0, 0) stores the 100 MHz wall
// clock at numbered points of the selecting kernels; each translation unit keeps its own table and exports a
// reader.  Compiled out of the product build.
#ifdef HIRE_TIMESTAMPS
static __device__ unsigned long long hire_ts[128];  // [i]: 100 MHz wall clock; [64 + i]: shader clock cycles
#define HIRE_TS(i)                                                 \
  do {                                                             \
    if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0) {  \
      hire_ts[i] = wall_clock64();                                 \
      hire_ts[64 + (i)] = clock64();                               \
    }                                                              \
  } while (0)
#else
#define HIRE_TS(i) ((void)0)
#endif

namespace hire {

constexpr int kSelThreads = 1024;  // workgroup size of the general selection kernels
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelBins = 2048;
constexpr int kSelSmall = 64;

template <int NT>
struct SelSharedT {
  static constexpr int NW = NT / kWave;
  uint32_t hist[kSelBins];
  unsigned long long red_a[NW];
  unsigned long long red_b[NW];
  int wave_tot[NW];
  int bc_bin, bc_above, bc_cnt;
  unsigned long long bc_key;
  int list_n;
  unsigned long long list_key[kSelSmall];
};
using SelShared = SelSharedT<kSelThreads>;

// min and max over the workgroup; every thread gets both.
template <typename K, int NT>
__device__ __forceinline__ void wg_minmax(K& vmin, K& vmax, SelSharedT<NT>& sh) {
  constexpr int NW = NT / kWave;
  K a = wave_min(vmin), b = wave_max(vmax);
  __syncthreads();  // previous readers of red_a/red_b are done
  if (lane_id() == 0) {
    sh.red_a[wave_id()] = (unsigned long long)a;
    sh.red_b[wave_id()] = (unsigned long long)b;
  }
  __syncthreads();
  a = (K)sh.red_a[0];
  b = (K)sh.red_b[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    K x = (K)sh.red_a[w], y = (K)sh.red_b[w];
    a = x < a ? x : a;
    b = y > b ? y : b;
  }
  vmin = a;
  vmax = b;
}

// Inclusive prefix sum over the NT threads in thread order; *total (optional) receives the sum of all.
// Wave totals go through LDS once; every wave then scans them itself in registers.
// FRESH: no thread can still be reading wave_tot from an earlier use, so the leading barrier is left out.
template <int NT, bool FRESH = false>
__device__ __forceinline__ int wg_scan_incl(int v, SelSharedT<NT>& sh, int* total = nullptr) {
  constexpr int NW = NT / kWave;
  const int incl = wave_scan_incl(v);
  if (!FRESH) __syncthreads();  // previous readers of wave_tot are done
  if (lane_id() == kWave - 1) sh.wave_tot[wave_id()] = incl;
  __syncthreads();
  const int t = lane_id() < NW ? sh.wave_tot[lane_id()] : 0;
  const int p = wave_scan_incl(t);
  const int w = __builtin_amdgcn_readfirstlane(wave_id());
  const int base = w > 0 ? __builtin_amdgcn_readlane(p, w - 1) : 0;
  if (total) *total = __builtin_amdgcn_readlane(p, NW - 1);
  return incl + base;
}

// Largest of one value per thread, to all threads.
template <int NT>
__device__ __forceinline__ uint32_t wg_max_u32(uint32_t m, SelSharedT<NT>& sh) {
  constexpr int NW = NT / kWave;
  m = wave_max(m);
  __syncthreads();
  if (lane_id() == 0) sh.wave_tot[wave_id()] = (int)m;
  __syncthreads();
  return wave_max(lane_id() < NW ? (uint32_t)sh.wave_tot[lane_id()] : 0u);
}

template <typename K>
struct KeyTraits;
template <>
struct KeyTraits<uint32_t> {
  using V = float;
};
template <>
struct KeyTraits<uint64_t> {
  using V = double;
};

// for_each(f): calls f(key) for every key this thread owns.  n keys in total
// over the workgroup, 1 <= k <= n.  Returns the k-th largest key to all threads.
// Keys are order keys (device_utils.h), so key_value() recovers the number.
template <typename K, int NT, typename ForEach>
__device__ K wg_kth_largest(ForEach&& for_each, int n, int k, SelSharedT<NT>& sh) {
  using V = typename KeyTraits<K>::V;
  constexpr int kBinsPerThread = kSelBins / NT;
  static_assert(kBinsPerThread >= 2 && kSelBins % NT == 0, "each thread walks a whole number of bins");
  K lo = ~(K)0, hi = 0;
  for_each([&](K key) {
    lo = key < lo ? key : lo;
    hi = key > hi ? key : hi;
  });
  HIRE_TS(1);
  wg_minmax(lo, hi, sh);
  HIRE_TS(2);
  int need = k, nact = n;
  bool value_round = true;
  const int tid = (int)threadIdx.x;
  while (true) {
    if (lo == hi) return lo;
    if (nact <= kSelSmall) break;
    // ---- histogram of the active interval ----
    for (int b = tid; b < kSelBins; b += NT) sh.hist[b] = 0;
    __syncthreads();
    const V vlo = key_value(lo);
    const V vscale = (V)(kSelBins - 1) / (key_value(hi) - vlo);
    const int shift = max(0, ilog2_u64((uint64_t)(hi - lo)) + 1 - 11);
    auto bin_of = [&](K key) -> int {
      if (value_round) {
        int b = (int)((key_value(key) - vlo) * vscale);
        return min(max(b, 0), kSelBins - 1);
      }
      return (int)((key - lo) >> shift);
    };
    for_each([&](K key) {
      if (key >= lo && key <= hi) {
        int b = bin_of(key);
        if (b) atomicAdd(&sh.hist[b], 1u);
      }
    });
    __syncthreads();
    HIRE_TS(3);
    // ---- walk the bins from the top: thread t owns the kBinsPerThread bins ending at bin 2047 - t*kBinsPerThread ----
    const int b_top = kSelBins - 1 - kBinsPerThread * tid;
    int c[kBinsPerThread], s = 0;
#pragma unroll
    for (int q = 0; q < kBinsPerThread; ++q) {
      c[q] = (int)sh.hist[b_top - q];
      s += c[q];
    }
    int total;
    const int incl = wg_scan_incl(s, sh, &total);
    int run = incl - s;
    if (run < need && need <= incl) {
#pragma unroll
      for (int q = 0; q < kBinsPerThread; ++q) {
        if (run < need && need <= run + c[q]) {
          sh.bc_bin = b_top - q;
          sh.bc_above = run;
          sh.bc_cnt = c[q];
        }
        run += c[q];
      }
    }
    if (tid == 0 && total < need) {  // the rank falls into the uncounted bin 0
      sh.bc_bin = 0;
      sh.bc_above = total;
      sh.bc_cnt = nact - total;
    }
    __syncthreads();
    const int beta = sh.bc_bin;
    need -= sh.bc_above;
    nact = sh.bc_cnt;
    HIRE_TS(4);
    // ---- tighten [lo, hi] to the keys of bin beta ----
    K nlo = ~(K)0, nhi = 0;
    for_each([&](K key) {
      if (key >= lo && key <= hi && bin_of(key) == beta) {
        nlo = key < nlo ? key : nlo;
        nhi = key > nhi ? key : nhi;
      }
    });
    wg_minmax(nlo, nhi, sh);
    lo = nlo;
    hi = nhi;
    value_round = false;
    HIRE_TS(5);
  }
  // ---- at most 64 keys left in [lo, hi]: rank them directly ----
  __syncthreads();
  if (tid == 0) sh.list_n = 0;
  __syncthreads();
  for_each([&](K key) {
    if (key >= lo && key <= hi) {
      int p = atomicAdd(&sh.list_n, 1);
      if (p < kSelSmall) sh.list_key[p] = (unsigned long long)key;
    }
  });
  __syncthreads();
  const int m = min(sh.list_n, kSelSmall);
  if (tid < m) {
    const K mine = (K)sh.list_key[tid];
    int cg = 0, cge = 0;
    for (int u = 0; u < m; ++u) {
      const K other = (K)sh.list_key[u];
      cg += other > mine;
      cge += other >= mine;
    }
    if (cg < need && need <= cge) sh.bc_key = (unsigned long long)mine;  // equal keys write the same value
  }
  __syncthreads();
  HIRE_TS(6);
  return (K)sh.bc_key;
}

// Consumer-side compaction of a bitmap: the workgroup finds the indices of the set bits with ranks
// [r0, r0 + R) in ascending order and learns the total number of set bits, without a pass of its own kernel.
// Wave w owns a contiguous block of words and reads it 64 words at a time (one coalesced load per step, kept
// in registers); the waves' totals give every wave the rank of its first bit, and only a wave whose ranks meet
// the wanted ones walks its steps again, from registers, with a wave prefix sum per step.  out_sh[r - r0]
// receives the index of rank r; entries at and past the total are left alone.  words <= NT / 64 * 64 * STEPS;
// callers with short bitmaps take the variant with few steps, whose unrolled loops are correspondingly short.
constexpr int kLocateSteps = 32;       // 64-word steps per wave
constexpr int kLocateStepsShort = 4;

template <int NT, int STEPS = kLocateSteps>
__device__ __forceinline__ int union_locate(const uint32_t* __restrict__ bitmap, int words, SelSharedT<NT>& sh,
                                            int r0, int R, int32_t* out_sh) {
  constexpr int NW = NT / kWave;
  const int lane = lane_id(), w = wave_id();
  const int per_wave = ((words + NW - 1) / NW + kWave - 1) / kWave * kWave;
  const int w0 = w * per_wave, w1 = min(words, w0 + per_wave);
  const int steps = max(0, (w1 - w0 + kWave - 1) / kWave);  // <= STEPS
  uint32_t keep[STEPS];
  int cnt = 0;
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    keep[st] = 0u;
    // uniform over the wave, clamped, and nothing done to the value yet: the loads of the block go out together
    if (st < steps) keep[st] = bitmap[min(w0 + st * kWave + lane, words - 1)];
  }
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    keep[st] = w0 + st * kWave + lane < w1 ? keep[st] : 0u;
    cnt += __popc(keep[st]);
  }
  const int mine = wave_sum(cnt);
  __syncthreads();  // previous readers of wave_tot are done
  if (lane == 0) sh.wave_tot[w] = mine;
  __syncthreads();
  int base = 0, total = 0;
#pragma unroll
  for (int u = 0; u < NW; ++u) {
    const int t = sh.wave_tot[u];
    base += u < w ? t : 0;
    total += t;
  }
  if (base < r0 + R && base + mine > r0) {  // this wave's bits meet the wanted ranks (uniform over the wave)
    int run = base;
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st < steps && run < r0 + R) {
        uint32_t m = keep[st];
        const int c = __popc(m);
        const int incl = wave_scan_incl(c);
        const int tot = __builtin_amdgcn_readlane(incl, kWave - 1);
        if (run + tot > r0) {
          int rank = run + incl - c;  // rank of this lane's first bit
          const int q = w0 + st * kWave + lane;
          while (m) {
            const int bit = __ffs((int)m) - 1;
            if (rank >= r0 && rank < r0 + R) out_sh[rank - r0] = q * 32 + bit;
            ++rank;
            m &= m - 1;
          }
        }
        run += tot;
      }
    }
  }
  __syncthreads();
  return total;
}

}  // namespace hire
