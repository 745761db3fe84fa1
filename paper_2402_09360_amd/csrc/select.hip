// Exact top-k selection kernels (TopInd_k / Top_k of arXiv 2402.09360 Sec. 3.1,
// used on both lines of Algorithm 1) and the bitmap compaction that forms the
// batch union of Sec. 3.4.1.
//
// One 1024-thread workgroup per score row.  Wave w owns the contiguous index
// range [w*M, (w+1)*M), M a multiple of 64, and walks it 64 at a time, so a
// wave ballot is a 64-bit slice of the selection mask in index order: ordered
// output positions come from popcounts, no sorting, and ties at the threshold
// go to the lowest indices by construction.
#include "fast_select.h"
#include "hist.h"
#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kItemsMax = 16;                       // most register-resident keys per thread
constexpr int kCachedMax = kSelThreads * kItemsMax; // 16384
constexpr int kRankMax = 4096;                      // largest k sorted into rank order
constexpr int kPackMax = 2048;                      // largest k emitted through the packed list in LDS
static_assert(kPackMax * (8 + 4) <= kHistWindow * 4, "the packed list reuses the window histogram's LDS");

template <typename V>
struct KeyOf;
template <>
struct KeyOf<float> {
  using K = uint32_t;
};
template <>
struct KeyOf<double> {
  using K = uint64_t;
};

// Group activation of eq. (6) for groups of eight: sum of the absolute values of the eight entries at src (32-
// or 64-byte aligned), added in index order in their own type; vector loads, nothing that waits in between.
__device__ __forceinline__ float group8_abs_sum(const float* __restrict__ src) {
  const float4 a = reinterpret_cast<const float4*>(src)[0], b = reinterpret_cast<const float4*>(src)[1];
  float s = fabsf(a.x);
  s += fabsf(a.y);
  s += fabsf(a.z);
  s += fabsf(a.w);
  s += fabsf(b.x);
  s += fabsf(b.y);
  s += fabsf(b.z);
  s += fabsf(b.w);
  return s;
}
__device__ __forceinline__ double group8_abs_sum(const double* __restrict__ src) {
  const double2* p = reinterpret_cast<const double2*>(src);
  const double2 a = p[0], b = p[1], c = p[2], d = p[3];
  double s = fabs(a.x);
  s += fabs(a.y);
  s += fabs(b.x);
  s += fabs(b.y);
  s += fabs(c.x);
  s += fabs(c.y);
  s += fabs(d.x);
  s += fabs(d.y);
  return s;
}

// Selection of row b by one whole workgroup.  dyn: rank order only, K keys[k] then int pos[k], int rank[k].
// win: kHistWindow words of LDS for the window histogram, or nullptr to go straight to range narrowing.
// ITEMS: keys a thread keeps in registers (rows of at most ITEMS * 1024 entries), or 0 to stream the row from
// memory on every pass.
template <typename V, int ITEMS, bool G8 = false>
__device__ __forceinline__ void select_row(const SelectParams& p, int b, SelShared& sh, unsigned long long* dyn,
                                           uint32_t* win) {
  using K = typename KeyOf<V>::K;
  __shared__ int tot_gt[kSelWaves], tot_eq[kSelWaves];

  // Everything the kernel needs first goes out in one batch of loads: the device-side count, the keys and the
  // index map.  The keys are laid out over the waves by the host-known bound of the count, so that their
  // addresses do not wait for the count itself.
  const int nload = p.n_dev ? p.n_cap : p.n;
  const int k = p.k;
  const V* vals = reinterpret_cast<const V*>(p.vals) + (size_t)b * p.stride;
  const int32_t* map = p.map ? p.map + (size_t)b * p.map_stride : nullptr;
  const int lane = lane_id(), w = wave_id();
  const int M = (((nload + kSelWaves - 1) / kSelWaves) + kWave - 1) / kWave * kWave;
  const int base = w * M;
  const int iters = M / kWave;

  auto to_key = [&](V v) -> K {
    if (p.relu) v = v > (V)0 ? v : (V)0;
    return order_key(v);
  };
  // entry i of the row: the value itself, or (G8, for SelectParams::group8) the group activation of the eight values
  // 8 i .. 8 i + 7.  A template parameter: the vector loads of the group form cost registers that the kernels with
  // 16 entries per thread do not have.
  auto load_key = [&](int i) -> K {
    if constexpr (G8) return to_key(group8_abs_sum(vals + (size_t)i * 8));
    else return to_key(vals[i]);
  };

  HIRE_TS(0);
  const int n_raw = p.n_dev ? *p.n_dev : p.n;
  // Small selections are emitted in two phases: the selected (position, key) pairs are first packed into LDS in
  // output order, then one thread per output translates the position and stores; the index map is then read for
  // the selected positions only.  Otherwise the map is fetched for every position with the keys, because a load
  // inside the emission loop would cost one memory round trip per trip.
  const bool packed = win != nullptr && !p.rank_order && p.bitmap == nullptr && k <= kPackMax;
  constexpr bool CACHED = ITEMS > 0;
  constexpr int kItems = CACHED ? ITEMS : 1;
  K regs[kItems];
  int mapped[kItems];
  if (CACHED) {
    V raw[kItems];
    if constexpr (!G8) {
#pragma unroll
      for (int e = 0; e < kItems; ++e) {  // clamped and unconditional, so that the loads do not wait for one another
        const int i = min(base + e * kWave + lane, nload - 1);
        raw[e] = vals[i];
        mapped[e] = (map && !p.rank_order && !packed) ? map[i] : base + e * kWave + lane;
      }
    } else {
#pragma unroll
      for (int e = 0; e < kItems; ++e) {
        const int i = min(base + e * kWave + lane, nload - 1);
        raw[e] = group8_abs_sum(vals + (size_t)i * 8);
        mapped[e] = (map && !p.rank_order && !packed) ? map[i] : base + e * kWave + lane;
      }
    }
    const int n_now = p.n_dev ? min(n_raw, p.n_cap) : p.n;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      const int i = base + e * kWave + lane;
      regs[e] = (e < iters && i < n_now) ? to_key(raw[e]) : (K)0;
    }
  }
  const int n = p.n_dev ? min(n_raw, p.n_cap) : p.n;
  HIRE_TS(9);
  // element visitor: f(e, i, key) for every owned, valid element in index order
  auto visit = [&](auto&& f) {
    if (CACHED) {
#pragma unroll
      for (int e = 0; e < kItems; ++e) {
        const int i = base + e * kWave + lane;
        if (e < iters && i < n) f(e, i, regs[e]);
      }
    } else {
      for (int e0 = 0; e0 < iters; e0 += 8) {  // eight clamped loads in flight, then their elements in index order
        K kk[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) kk[j] = load_key(min(base + (e0 + j) * kWave + lane, n - 1));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int i = base + (e0 + j) * kWave + lane;
          if (e0 + j < iters && i < n) f(e0 + j, i, kk[j]);
        }
      }
    }
  };

  // ---- the k-th largest key ----
  // First try: a fine histogram (2^14 order keys per bin) of the kHistWindow bins at and below the largest key,
  // built in LDS; the bin holding the k-th key follows from one walk, and the few keys inside it are ranked
  // directly.  Exact zeros are left out (after a ReLU they would all queue up on one counter).  When the window
  // does not answer - the k-th key lies below it or among the zeros, or its bin is crowded - the range narrowing
  // of select.h takes over.
  K T = 0;
  bool guided = false;
  if (win != nullptr) {
    const int tid = (int)threadIdx.x;
    K hi = 0;
    visit([&](int, int, K key) { hi = key > hi ? key : hi; });
    hi = wave_max(hi);
    __syncthreads();  // previous readers of red_a are done
    if (lane == 0) sh.red_a[w] = (unsigned long long)hi;
    for (int i = tid; i < kHistWindow; i += kSelThreads) win[i] = 0u;
    if (tid == 0) sh.list_n = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kSelWaves; ++u) hi = (K)sh.red_a[u] > hi ? (K)sh.red_a[u] : hi;
    HIRE_TS(30);
    const int top_bin = (int)hist_bin(hi);
    const int base_bin = (top_bin | 7) - (kHistWindow - 1);  // a multiple of 8: the walk reads aligned groups
    const K zero_key = order_key((V)0);
    visit([&](int, int, K key) {
      const int rel = (int)hist_bin(key) - base_bin;
      if (rel >= 0 && key != zero_key) atomicAdd(&win[rel], 1u);
    });
    __syncthreads();
    const BinWalk wk = walk_histogram<kSelThreads>(win - base_bin, (uint32_t)top_bin, k, sh);
    HIRE_TS(31);
    if (wk.found && wk.cnt <= kSelSmall) {
      visit([&](int, int, K key) {
        if ((int)hist_bin(key) == wk.bin && key != zero_key) {
          const int q = atomicAdd(&sh.list_n, 1);
          if (q < kSelSmall) sh.list_key[q] = (unsigned long long)key;
        }
      });
      __syncthreads();
      const int m = min(sh.list_n, kSelSmall), need = k - wk.above;
      if (tid < m) {
        const K mine = (K)sh.list_key[tid];
        int cg = 0, cge = 0;
        for (int u0 = 0; u0 < m; u0 += 8) {  // eight LDS reads in flight
          K other[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) other[j] = (K)sh.list_key[min(u0 + j, m - 1)];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            cg += (u0 + j < m) && other[j] > mine;
            cge += (u0 + j < m) && other[j] >= mine;
          }
        }
        if (cg < need && need <= cge) sh.bc_key = (unsigned long long)mine;  // equal keys write the same value
      }
      __syncthreads();
      T = (K)sh.bc_key;
      guided = true;
      HIRE_TS(32);
    } else if (tid == 0 && p.window_misses != nullptr) {
      atomicAdd(p.window_misses, 1u);
    }
  }
  if (!guided) T = wg_kth_largest<K>([&](auto&& f) { visit([&](int, int, K key) { f(key); }); }, n, k, sh);

  // ---- ordered counts of keys above / equal to the threshold, per wave ----
  int cnt_gt = 0, cnt_eq = 0;
  visit([&](int, int, K key) {
    cnt_gt += key > T;
    cnt_eq += key == T;
  });
  cnt_gt = wave_sum(cnt_gt);
  cnt_eq = wave_sum(cnt_eq);
  __syncthreads();
  if (lane == 0) {
    tot_gt[w] = cnt_gt;
    tot_eq[w] = cnt_eq;
  }
  __syncthreads();
  int run_gt = 0, run_eq = 0, all_gt = 0;
  for (int u = 0; u < kSelWaves; ++u) {
    if (u < w) {
      run_gt += tot_gt[u];
      run_eq += tot_eq[u];
    }
    all_gt += tot_gt[u];
  }
  HIRE_TS(7);
  const int need_eq = k - all_gt;  // ties at the threshold that are taken, lowest indices first

  // ---- emission in index order ----
  K* rk_key = reinterpret_cast<K*>(dyn);
  int* rk_pos = reinterpret_cast<int*>(rk_key + (p.rank_order ? k : 0));
  // packed mode: the window histogram's LDS is free by now; K keys[kPackMax] then int pos[kPackMax]
  K* pk_key = reinterpret_cast<K*>(win);
  int* pk_pos = reinterpret_cast<int*>(pk_key + kPackMax);
  if (packed) __syncthreads();  // every wave is done with the window histogram
  // one step of 64 consecutive positions per wave; uniform trip count per wave, so the ballots are safe
  auto emit_step = [&](int e, K key_in, int mi) {
    const int i = base + e * kWave + lane;
    const bool valid = i < n;
    const K key = valid ? key_in : (K)0;
    const bool gt = valid && key > T, eq = valid && key == T;
    const uint64_t mg = __ballot(gt), me = __ballot(eq);
    const int gt_before = run_gt + mask_prefix(mg), eq_before = run_eq + mask_prefix(me);
    const bool sel = gt || (eq && eq_before < need_eq);
    const int out = gt_before + min(eq_before, need_eq);
    run_gt += __popcll(mg);
    run_eq += __popcll(me);
    const V v = key_value(key);
    if (p.bitmap) {
      const uint64_t ms = __ballot(sel);
      if (lane == 0 && (uint32_t)ms) atomicOr(&p.bitmap[(base + e * kWave) >> 5], (uint32_t)ms);
      if (lane == 32 && (uint32_t)(ms >> 32)) atomicOr(&p.bitmap[((base + e * kWave) >> 5) + 1], (uint32_t)(ms >> 32));
    }
    if (sel) {
      if (p.rank_order) {
        rk_key[out] = key;
        rk_pos[out] = i;
      } else if (packed) {
        pk_pos[out] = i;
        pk_key[out] = key;
      } else {
        if (p.idx_out) p.idx_out[(size_t)b * k + out] = mi;
        if (p.pos_out) p.pos_out[(size_t)b * k + out] = i;
        if (p.val_out) p.val_out[(size_t)b * k + out] = (float)v;
      }
    }
  };
  if (CACHED) {
#pragma unroll
    for (int e = 0; e < kItems; ++e)  // unrolled: the register arrays are indexed statically
      if (e < iters) emit_step(e, regs[e], mapped[e]);
  } else {
    for (int e = 0; e < iters; ++e) {
      const int i = min(base + e * kWave + lane, n - 1);
      emit_step(e, load_key(i), (map && !p.rank_order) ? map[i] : base + e * kWave + lane);
    }
  }
  HIRE_TS(8);
  if (packed) {
    __syncthreads();
    for (int t = (int)threadIdx.x; t < k; t += kSelThreads) {
      const int i = pk_pos[t];
      if (p.idx_out) p.idx_out[(size_t)b * k + t] = map ? map[i] : i;
      if (p.pos_out) p.pos_out[(size_t)b * k + t] = i;
      if (p.val_out) p.val_out[(size_t)b * k + t] = (float)key_value(pk_key[t]);
    }
  }
  if (!p.rank_order) return;

  // ---- rank order: position of each selected entry among the k (value desc, index asc) ----
  constexpr int kPerThread = kRankMax / kSelThreads;
  int* rk_rank = rk_pos + k;  // small k: partial ranks from several threads per entry are added up here
  const bool spread = k <= kSelThreads / 2;
  if (spread)
    for (int t = (int)threadIdx.x; t < k; t += kSelThreads) rk_rank[t] = 0;
  __syncthreads();
  if (spread) {
    const int padded = (k + kWave - 1) / kWave * kWave;
    const int slices = kSelThreads / padded, group = kSelThreads / slices;
    const int per = (k + slices - 1) / slices;
    const int t = (int)threadIdx.x % group, sl = (int)threadIdx.x / group;
    if (t < k && sl < slices) {
      const K mine = rk_key[t];
      const int u_lo = sl * per, u_hi = min(k, u_lo + per);
      int rank = 0;
      for (int u0 = u_lo; u0 < u_hi; u0 += 8) {  // eight LDS reads in flight
        K other[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) other[j] = rk_key[min(u0 + j, k - 1)];
#pragma unroll
        for (int j = 0; j < 8; ++j)  // the list is in index order, so u < t is "lower index"
          rank += (u0 + j < u_hi) && ((other[j] > mine) || (other[j] == mine && u0 + j < t));
      }
      atomicAdd(&rk_rank[t], rank);
    }
    __syncthreads();
  }
  int my_rank[kPerThread];
  V my_val[kPerThread];
#pragma unroll
  for (int q = 0; q < kPerThread; ++q) {
    const int t = (int)threadIdx.x + q * kSelThreads;
    my_rank[q] = -1;
    my_val[q] = (V)0;
    if (t < k) {
      const K mine = rk_key[t];
      int rank = spread ? rk_rank[t] : 0;
      for (int u0 = 0; u0 < (spread ? 0 : k); u0 += 8) {  // eight LDS reads in flight
        K other[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) other[j] = rk_key[min(u0 + j, k - 1)];
#pragma unroll
        for (int j = 0; j < 8; ++j)  // the list is in index order, so u < t is "lower index"
          rank += (u0 + j < k) && ((other[j] > mine) || (other[j] == mine && u0 + j < t));
      }
      const int i = rk_pos[t];
      const V v = key_value(mine);
      if (p.idx_out) p.idx_out[(size_t)b * k + rank] = map ? map[i] : i;
      if (p.pos_out) p.pos_out[(size_t)b * k + rank] = i;
      if (p.val_out) p.val_out[(size_t)b * k + rank] = (float)v;
      my_rank[q] = rank;
      my_val[q] = v;
    }
  }
  HIRE_TS(34);
  if (!p.prob_out) return;
  // ---- softmax over the k survivors: exp(z - zmax) / sum; the sorted values reuse the key array ----
  __syncthreads();
  V* sorted = reinterpret_cast<V*>(dyn);
#pragma unroll
  for (int q = 0; q < kPerThread; ++q)
    if (my_rank[q] >= 0) sorted[my_rank[q]] = my_val[q];
  __syncthreads();
  const double zmax = (double)sorted[0];
  double part = 0.0;
  for (int t = (int)threadIdx.x; t < k; t += kSelThreads) part += exp((double)sorted[t] - zmax);
  part = wave_sum(part);
  if (lane == 0) sh.red_a[w] = (unsigned long long)__double_as_longlong(part);
  __syncthreads();
  double sum = 0.0;
  for (int u = 0; u < kSelWaves; ++u) sum += __longlong_as_double((long long)sh.red_a[u]);
  for (int t = (int)threadIdx.x; t < k; t += kSelThreads)
    p.prob_out[(size_t)b * k + t] = (float)(exp((double)sorted[t] - zmax) / sum);
  HIRE_TS(35);
}

template <typename V, int ITEMS, bool G8 = false>
__global__ __launch_bounds__(kSelThreads) void k_select(SelectParams p) {
  __shared__ SelShared sh;
  __shared__ uint32_t win[kHistWindow];
  extern __shared__ unsigned long long dyn[];
  select_row<V, ITEMS, G8>(p, (int)blockIdx.x, sh, dyn, win);
}

// ---------------------------------------------------------------------------
// Bitmap -> ascending index list, one workgroup.
template <int kPer>  // words per thread and round, loaded together
__device__ __forceinline__ void compact_bitmap_per(const uint32_t* bitmap, int words, int32_t* __restrict__ list_out,
                                                   int32_t* __restrict__ count_out, int32_t* __restrict__ count_out2,
                                                   uint32_t* zero_ptr, int zero_words, SelShared& sh) {
  const int tid = (int)threadIdx.x;
  if (zero_ptr)
    for (int i = tid; i < zero_words; i += kSelThreads) zero_ptr[i] = 0u;
  int base = 0;
  for (int r0 = 0; r0 < words; r0 += kSelThreads * kPer) {
    const int w0 = r0 + tid * kPer;
    uint32_t m[kPer];
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const uint32_t v = bitmap[min(w0 + j, words - 1)];  // clamped and unconditional: the loads go out together
      m[j] = w0 + j < words ? v : 0u;
      cnt += __popc(m[j]);
    }
    int total;
    const int incl = wg_scan_incl(cnt, sh, &total);
    int out = base + incl - cnt;
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      uint32_t mm = m[j];
      while (mm) {
        const int bit = __ffs((int)mm) - 1;
        list_out[out++] = (w0 + j) * 32 + bit;
        mm &= mm - 1;
      }
    }
    base += total;
  }
  if (tid == 0) {
    count_out[0] = base;
    if (count_out2) count_out2[0] = base;
  }
}

// A short bitmap spreads one word per thread, so that the list is written by many threads.
__device__ __forceinline__ void compact_bitmap(const uint32_t* bitmap, int words, int32_t* __restrict__ list_out,
                                               int32_t* __restrict__ count_out, int32_t* __restrict__ count_out2,
                                               uint32_t* zero_ptr, int zero_words, SelShared& sh) {
  if (words <= 2 * kSelThreads)
    compact_bitmap_per<1>(bitmap, words, list_out, count_out, count_out2, zero_ptr, zero_words, sh);
  else
    compact_bitmap_per<8>(bitmap, words, list_out, count_out, count_out2, zero_ptr, zero_words, sh);
}

__global__ __launch_bounds__(kSelThreads) void k_bitmap_compact(const uint32_t* bitmap, int words,
                                                                int32_t* __restrict__ list_out,
                                                                int32_t* __restrict__ count_out,
                                                                int32_t* __restrict__ count_out2, uint32_t* zero_ptr,
                                                                int zero_words) {
  __shared__ SelShared sh;
  compact_bitmap(bitmap, words, list_out, count_out, count_out2, zero_ptr, zero_words, sh);
}

// ---------------------------------------------------------------------------
// Histogram-guided selection over many workgroups.  Grid (ceil(N / 4096), B): every workgroup of token b
// repeats the short walk over b's histogram (largest key from the producers' per-workgroup maxima, then the
// window of bins below it) and so knows the bin that holds the k'-th largest key; its own 4096 keys then fall
// into three classes: above that bin (selected: bit set in the union bitmap), inside it (listed for the
// resolving kernel), below (dropped).
constexpr int kMarkKeys = 4;  // keys per thread

// Largest key of token b from the producers' per-workgroup maxima, to all threads.
__device__ __forceinline__ uint32_t token_top_key(const MultiRegion& mr, int b, int slots, SelShared& sh) {
  const int tid = (int)threadIdx.x;
  const uint4 mx = reinterpret_cast<const uint4*>(mr.wgmax + (size_t)b * kWgMaxSlots)[tid];
  uint32_t top = 0u;
  top = (4 * tid + 0 < slots && mx.x > top) ? mx.x : top;
  top = (4 * tid + 1 < slots && mx.y > top) ? mx.y : top;
  top = (4 * tid + 2 < slots && mx.z > top) ? mx.z : top;
  top = (4 * tid + 3 < slots && mx.w > top) ? mx.w : top;
  return wg_max_u32(top, sh);
}

// Counting pass for long rows, where one atomic per key from the producer would pile up on the few cache lines
// that hold the populated bins.  Grid (ceil(N / 16384), B).  Bins are 2^shift order keys wide (coarser than the
// producer-side histogram); only the kHistWindow bins at and below the largest key's are counted, first in LDS,
// then with one global atomic per populated bin.
constexpr int kCountKeys = 16;  // keys per thread

__global__ __launch_bounds__(kSelThreads) void k_count_f32(const float* __restrict__ keys, int B, int N, int slots,
                                                           int shift, int relu, MultiRegion mr) {
  __shared__ SelShared sh;
  __shared__ uint32_t cnt[kHistWindow];
  if (!multi_hist_ok(mr.hdr, B)) return;
  const int b = (int)blockIdx.y, tid = (int)threadIdx.x;
  const float* row = keys + (size_t)b * N;
  const int i0 = (int)blockIdx.x * (kSelThreads * kCountKeys);
  float v[kCountKeys];
#pragma unroll
  for (int e = 0; e < kCountKeys; ++e) v[e] = row[min(i0 + e * kSelThreads + tid, N - 1)];
  if (relu) {
#pragma unroll
    for (int e = 0; e < kCountKeys; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
  }
  for (int i = tid; i < kHistWindow; i += kSelThreads) cnt[i] = 0u;
  const int top_bin = (int)(token_top_key(mr, b, slots, sh) >> shift);  // barriers inside: cnt is cleared
  const int lo_bin = top_bin - (kHistWindow - 1);
#pragma unroll
  for (int e = 0; e < kCountKeys; ++e) {
    const int rel = (int)(order_key(v[e]) >> shift) - lo_bin;
    if (i0 + e * kSelThreads + tid < N && rel >= 0) atomicAdd(&cnt[rel], 1u);
  }
  __syncthreads();
  uint32_t* hist = mr.hist + (size_t)b * kHistStride + kHistWindow + lo_bin;  // lo_bin >= -kHistWindow + 1: the apron
  for (int i = tid; i < kHistWindow; i += kSelThreads) {
    const uint32_t c = cnt[i];
    if (c) atomicAdd(&hist[i], c);
  }
}

__global__ __launch_bounds__(kSelThreads) void k_mark_f32(const float* __restrict__ keys, int B, int N, int kprime,
                                                          int slots, int shift, int relu, MultiRegion mr,
                                                          uint32_t* __restrict__ bitmap, long long bitmap_stride) {
  __shared__ SelShared sh;
  const int b = (int)blockIdx.y, tid = (int)threadIdx.x, lane = lane_id();
  bitmap += (size_t)b * bitmap_stride;  // stride 0: one bitmap for the union of all rows
  const bool ok = multi_hist_ok(mr.hdr, B);
  if (!ok) {  // histograms not usable yet: the resolving kernel selects by streaming and stamps the region
    if (blockIdx.x == 0 && tid == 0) {
      mr.walk[4 * b + 0] = kprime;
      mr.walk[4 * b + 1] = 0;
      mr.walk[4 * b + 2] = 0;
    }
    return;
  }
  const float* row = keys + (size_t)b * N;
  const int i0 = (int)blockIdx.x * (kSelThreads * kMarkKeys);
  float v[kMarkKeys];
#pragma unroll
  for (int e = 0; e < kMarkKeys; ++e) v[e] = row[min(i0 + e * kSelThreads + tid, N - 1)];
  if (relu) {
#pragma unroll
    for (int e = 0; e < kMarkKeys; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
  }
  const uint32_t top_bin = token_top_key(mr, b, slots, sh) >> shift;
  const BinWalk wk = walk_histogram<kSelThreads>(mr.hist + (size_t)b * kHistStride + kHistWindow, top_bin, kprime, sh);
  if (blockIdx.x == 0 && tid == 0) {
    mr.walk[4 * b + 0] = kprime - wk.above;
    mr.walk[4 * b + 1] = wk.found ? 1 : 0;
    mr.walk[4 * b + 2] = (int)top_bin;
  }
  if (!wk.found) return;
#pragma unroll
  for (int e = 0; e < kMarkKeys; ++e) {
    const int i = i0 + e * kSelThreads + tid;
    const uint32_t okey = order_key(v[e]);
    const int bin = (int)(okey >> shift);
    const bool valid = i < N;
    const uint64_t ms = __ballot(valid && bin > wk.bin);
    const int wbase = (i0 + e * kSelThreads + (tid & ~63)) >> 5;
    if (lane == 0 && (uint32_t)ms) atomicOr(&bitmap[wbase], (uint32_t)ms);
    if (lane == 32 && (uint32_t)(ms >> 32)) atomicOr(&bitmap[wbase + 1], (uint32_t)(ms >> 32));
    const bool amb = valid && bin == wk.bin;
    const uint64_t ma = __ballot(amb);
    if (ma) {
      int base = 0;
      if (lane == 0) base = (int)atomicAdd(&mr.amb_n[b], (uint32_t)__popcll(ma));
      base = __builtin_amdgcn_readfirstlane(base);
      const int pos = base + mask_prefix(ma);
      if (amb && pos < kAmbCap) mr.amb[(size_t)b * kAmbCap + pos] = AmbEntry{okey, i};
    }
  }
}

// Second half, grid (1 + cleaners, B).  Workgroup (0, b) ranks the listed keys of token b's threshold bin by (key
// descending, index ascending) and sets the bits of the first `need`; a token whose histogram did not answer
// (region not stamped, threshold outside the window, list overflow) is selected by the streaming kernel's
// method instead.  Workgroups (c > 0, b) put a slice of token b's histogram back to all-zero: only the bins
// its keys touched, or everything when the region is not stamped yet.
constexpr int kCleanKeys = 4096;  // keys per cleaning workgroup

__global__ __launch_bounds__(kSelThreads) void k_resolve_compact(const float* __restrict__ keys, int B, int N, int kprime,
                                                                 int shift, int relu, MultiRegion mr, uint32_t* bitmap,
                                                                 long long bitmap_stride) {
  __shared__ SelShared sh;
  __shared__ AmbEntry amb_sh[kAmbCap];
  __shared__ int rank_sh[kAmbCap];
  const int b = (int)blockIdx.y, tid = (int)threadIdx.x;
  bitmap += (size_t)b * bitmap_stride;  // stride 0: one bitmap for the union of all rows
  HIRE_TS(40);
  const bool ok = multi_hist_ok(mr.hdr, B);
  uint32_t* hist = mr.hist + (size_t)b * kHistStride;
  const float* row = keys + (size_t)b * N;
  if (blockIdx.x == 0) {
    const int need = mr.walk[4 * b + 0];
    const bool found = mr.walk[4 * b + 1] != 0;
    const int m = (int)mr.amb_n[b];
    if (ok && found && m <= kAmbCap) {
      HIRE_TS(41);
      for (int t = tid; t < m; t += kSelThreads) amb_sh[t] = mr.amb[(size_t)b * kAmbCap + t];
      __syncthreads();
      HIRE_TS(42);
      // rank of every listed key among the m, the comparisons of one key spread over as many threads as fit
      // (a wave issues an instruction every few cycles only, so a lone thread's m-step loop is slow)
      const int padded = (m + kWave - 1) / kWave * kWave;
      const int slices = padded <= kSelThreads ? kSelThreads / padded : 1;
      const int per = (m + slices - 1) / slices;
      for (int t = tid; t < kAmbCap; t += kSelThreads) rank_sh[t] = 0;
      __syncthreads();
      for (int t0 = 0; t0 < m; t0 += kSelThreads / slices) {
        const int t = t0 + tid % (kSelThreads / slices), sl = tid / (kSelThreads / slices);
        if (t < m && sl < slices) {
          const AmbEntry mine = amb_sh[t];
          const int u_lo = sl * per, u_hi = min(m, u_lo + per);
          int rank = 0;
          for (int u0 = u_lo; u0 < u_hi; u0 += 8) {  // eight LDS reads in flight
            AmbEntry o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = amb_sh[min(u0 + j, m - 1)];
#pragma unroll
            for (int j = 0; j < 8; ++j)
              rank += (u0 + j < u_hi) && ((o[j].okey > mine.okey) || (o[j].okey == mine.okey && o[j].idx < mine.idx));
          }
          atomicAdd(&rank_sh[t], rank);
        }
      }
      __syncthreads();
      for (int t = tid; t < m; t += kSelThreads) {
        const int idx = amb_sh[t].idx;
        if (rank_sh[t] < need) atomicOr(&bitmap[idx >> 5], 1u << (idx & 31));
      }
    } else {
      SelectParams sp{};
      sp.vals = keys;
      sp.stride = N;
      sp.n = N;
      sp.n_cap = N;
      sp.k = kprime;
      sp.relu = relu;
      sp.bitmap = bitmap;
      select_row<float, 0>(sp, b, sh, nullptr, reinterpret_cast<uint32_t*>(amb_sh));  // the list's LDS is free here
      if (tid == 0 && ok) atomicAdd(&mr.hdr->fallbacks, 1u);
    }
    HIRE_TS(43);
    __syncthreads();  // every thread has read amb_n[b]
    if (tid == 0) mr.amb_n[b] = 0u;
    HIRE_TS(44);
  } else {
    const int c = (int)blockIdx.x - 1, nc = (int)gridDim.x - 1;
    if (ok && shift == kHistShift) {  // the producer counted every key
      for (int i = c * kSelThreads + tid; i < N; i += nc * kSelThreads)
        hist[kHistWindow + hist_bin(order_key(relu && row[i] < 0.0f ? 0.0f : row[i]))] = 0u;
    } else if (ok) {                  // the counting pass filled the window below the largest key only
      uint32_t* win = hist + kHistWindow + mr.walk[4 * b + 2] - (kHistWindow - 1);
      for (int i = c * kSelThreads + tid; i < kHistWindow; i += nc * kSelThreads) win[i] = 0u;
    } else {
      for (int i = c * kSelThreads + tid; i < kHistStride; i += nc * kSelThreads) hist[i] = 0u;
    }
  }
}

// ---------------------------------------------------------------------------
// topk_select on long rows: the same many-workgroup selection with a bitmap per row, framed by two small kernels.
// k_row_maxima (grid (ceil(N / 16384), B)) plays the producer: per-workgroup maxima of the keys, and it is the
// sequence's first kernel (clears the bitmaps, checks the layout signature).  k_emit_rows (one workgroup per row)
// turns the row's bitmap into the ascending index list with the values.
__global__ __launch_bounds__(kSelThreads) void k_row_maxima(const float* __restrict__ keys, int N, int relu, MultiRegion mr,
                                                            uint32_t* zero_ptr, long long zero_words, GeneralHeader* gh,
                                                            unsigned long long sig) {
  __shared__ SelShared sh;
  const long long gsz = (long long)gridDim.x * gridDim.y * kSelThreads;
  for (long long i = ((long long)blockIdx.y * gridDim.x + blockIdx.x) * kSelThreads + threadIdx.x; i < zero_words; i += gsz)
    zero_ptr[i] = 0u;
  if (blockIdx.x == 0 && blockIdx.y == 0) general_header_check(gh, sig);
  const int b = (int)blockIdx.y, tid = (int)threadIdx.x;
  const float* row = keys + (size_t)b * N;
  const int i0 = (int)blockIdx.x * (kSelThreads * kCountKeys);
  float v[kCountKeys];
#pragma unroll
  for (int e = 0; e < kCountKeys; ++e) v[e] = row[min(i0 + e * kSelThreads + tid, N - 1)];  // clamped: a row's own key
  uint32_t m = 0u;
#pragma unroll
  for (int e = 0; e < kCountKeys; ++e) {
    const uint32_t ok = order_key(relu && v[e] < 0.0f ? 0.0f : v[e]);
    m = ok > m ? ok : m;
  }
  m = wg_max_u32(m, sh);
  if (tid == 0) mr.wgmax[(size_t)b * kWgMaxSlots + blockIdx.x] = m;
}

__global__ __launch_bounds__(kSelThreads) void k_emit_rows(const float* __restrict__ keys, int B, int N, int k, int relu,
                                                           MultiRegion mr, const uint32_t* __restrict__ bitmaps,
                                                           int words, int32_t* __restrict__ idx_out,
                                                           float* __restrict__ val_out, int32_t* __restrict__ counts) {
  __shared__ SelShared sh;
  const int b = (int)blockIdx.x;
  int32_t* list = idx_out + (size_t)b * k;
  compact_bitmap(bitmaps + (size_t)b * words, words, list, counts + b, nullptr, nullptr, 0, sh);
  if (b == 0 && threadIdx.x == 0 && !multi_hist_ok(mr.hdr, B)) {  // the histograms were cleared by the kernel before
    mr.hdr->fallbacks = 0u;
    mr.hdr->stamps += 1u;
    mr.hdr->layout_b = (uint32_t)B;
    mr.hdr->cookie = kMultiCookie;
  }
  if (val_out == nullptr) return;
  __syncthreads();  // the list is this workgroup's own: visible after the barrier
  const float* row = keys + (size_t)b * N;
  for (int t0 = 0; t0 < k; t0 += kSelThreads * 4) {  // four index -> value chains in flight per thread
    int j[4];
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) j[u] = list[min(t0 + u * kSelThreads + (int)threadIdx.x, k - 1)];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = row[j[u]];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = t0 + u * kSelThreads + (int)threadIdx.x;
      if (t < k) val_out[(size_t)b * k + t] = relu && v[u] < 0.0f ? 0.0f : (v[u] == 0.0f ? 0.0f : v[u]);
    }
  }
}

// Third part for bitmaps too long for the gather kernels to compact themselves, one workgroup: the union bitmap
// becomes the ascending candidate list, and a region that was not stamped is now (its histograms were cleared by
// the kernel before).  A kernel of its own rather than the last workgroup of the previous one: device-scope
// fences inside a kernel cost a write-back of the whole L2 here.
__global__ __launch_bounds__(kSelThreads) void k_union_compact(int B, MultiRegion mr, const uint32_t* bitmap, int words,
                                                               int32_t* __restrict__ list_out,
                                                               int32_t* __restrict__ count_out,
                                                               int32_t* __restrict__ count_out2, uint32_t* zero_ptr,
                                                               int zero_words) {
  __shared__ SelShared sh;
  compact_bitmap(bitmap, words, list_out, count_out, count_out2, zero_ptr, zero_words, sh);
  if (threadIdx.x == 0 && !multi_hist_ok(mr.hdr, B)) {
    mr.hdr->fallbacks = 0u;
    mr.hdr->stamps += 1u;
    mr.hdr->layout_b = (uint32_t)B;
    mr.hdr->cookie = kMultiCookie;
  }
}

// ---------------------------------------------------------------------------
// The same selection for rows of non-negative values (scorer keys and activations after a ReLU) of at most 16384
// entries, in index order: the leaner machinery of fast_select.h.  The values' bit patterns are the keys, entries
// at and beyond the row's length are zeroed once, so no pass tests validity; the largest key's bin anchors a
// window histogram that is built in LDS, the walk proposes the threshold bin, two comparisons per key count what
// lies above it and find its own few keys, which every wave ranks for itself.  Selected positions go to a bitmap
// (the lanes that share a word fold their bits, one atomic per non-zero word) or, packed in LDS in output order,
// to the index / position / value outputs.  Irregular rows (all zero, threshold among the zeros, crowded bin) take the narrowing of
// select.h inside fast_select.
struct LeanShared {
  SelShared sh;
  uint32_t win[kWin];  // the window histogram; afterwards the row's bitmap, or the packed outputs
  int wave_cnt[kSelWaves];
  uint32_t wmax[kSelWaves];
  int band_n;
};

// The row's keys are in kr (loaded, masked beyond n): anchor, window histogram, selection of the k largest.
template <int TB, typename K, int LOADS, bool FR>
__device__ __forceinline__ Selection<K> lean_select(const KeyRegs<K, LOADS, kSelThreads, FR>& kr, const void* vals, int k,
                                                    LeanShared& L, uint32_t* window_misses) {
  using Keys = KeyRegs<K, LOADS, kSelThreads, FR>;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  {
    uint4* z = reinterpret_cast<uint4*>(L.win) + 2 * tid;
    z[0] = z[1] = make_uint4(0, 0, 0, 0);
  }
  K mx = 0;
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < Keys::PER; ++q) mx = kr.r[e][q] > mx ? kr.r[e][q] : mx;
  mx = wave_max(mx);
  if (lane == 0) L.wmax[w] = fine_bin(mx);
  __syncthreads();
  const uint32_t anchor = wave_max(lane < kSelWaves ? L.wmax[lane] : 0u);  // bin of the row's largest key
  HIRE_TS(TB + 1);
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < Keys::PER; ++q) {
      const uint32_t slot = anchor - fine_bin(kr.r[e][q]);
      if (kr.r[e][q] != (K)0 && slot < (uint32_t)kWin) atomicAdd(&L.win[slot], 1u);  // zeros are never counted
    }
  __syncthreads();
  WinRegs<kSelThreads> wr;
  wr.issue(L.win);
  HIRE_TS(TB + 2);
  // (the window's LDS is free again once the walk inside has passed its first barrier)
  const Selection<K> sel = fast_select<TB + 3>(kr, vals, k, wr, anchor, anchor != 0u, L.sh, L.wave_cnt, window_misses, 0,
                                               k, true);
  HIRE_TS(TB + 6);
  return sel;
}

// The selected entries, packed in LDS in output order, to the index / position / value outputs.
// emit_all(fn): calls fn(position, output slot, value as float) for every selected entry.  coeff (optional):
// coeff[position] receives the value as well (after the barrier, so nothing waits for those stores).
template <typename EmitAll>
__device__ __forceinline__ void lean_outputs(const SelectParams& p, int b, int k, LeanShared& L, EmitAll&& emit_all,
                                             double* coeff = nullptr) {
  const int tid = (int)threadIdx.x;
  int* pk_pos = reinterpret_cast<int*>(L.win);  // k <= kWin / 2
  float* pk_val = reinterpret_cast<float*>(L.win + kWin / 2);
  emit_all([&](int i, int out, float v) {
    pk_pos[out] = i;
    pk_val[out] = v;
  });
  __syncthreads();
  const int32_t* map = p.map ? p.map + (size_t)b * p.map_stride : nullptr;
  for (int t = tid; t < k; t += kSelThreads) {
    const int i = pk_pos[t];
    if (p.idx_out) p.idx_out[(size_t)b * k + t] = map ? map[i] : i;
    if (p.pos_out) p.pos_out[(size_t)b * k + t] = i;
    if (p.val_out) p.val_out[(size_t)b * k + t] = pk_val[t];
    if (coeff) coeff[i] = (double)pk_val[t];
  }
}

// One row: load, select, write the outputs.
template <int TB, typename V>
__device__ __forceinline__ void lean_row(const SelectParams& p, int b, const V* vals, LeanShared& L) {
  using K = typename KeyOf<V>::K;
  constexpr int LOADS = sizeof(V) == 4 ? 4 : 8;  // 16 waves x loads x 256 (128) keys = 16384
  using Keys = KeyRegs<K, LOADS, kSelThreads, sizeof(V) == 8>;  // the fp64 instance is short of registers
  static_assert(Keys::CAPACITY == kCachedMax, "rows of up to 16384 entries");
  const int cap = p.n_dev ? p.n_cap : p.n, k = p.k;
  const int n_raw = p.n_dev ? *p.n_dev : p.n;
  Keys kr;
  kr.issue_clamped(vals, cap);
  kr.finish();
  const int n = p.n_dev ? min(n_raw, p.n_cap) : p.n;
  kr.mask_beyond(n);
  const Selection<K> sel = lean_select<TB>(kr, vals, k, L, p.window_misses);
  if (p.bitmap != nullptr) {
    // A bitmap word covers 32 consecutive indices: the keys of 32 / PER neighbouring lanes of one load.  Those
    // lanes fold their bits together and one of them adds the word to the union: no ranks, no LDS, no barrier.
    constexpr int PER = Keys::PER, LPW = 32 / PER;
    const int lane = lane_id();
#pragma unroll
    for (int e = 0; e < LOADS; ++e) {
      uint32_t bits = 0u;
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        const bool take = sel.plain ? kr.r[e][q] >= sel.cut.key
                                    : (kr.valid(e, q) && cut_takes(sel.cut, kr.r[e][q], kr.index(e, q)));
        bits |= take ? 1u << q : 0u;
      }
      bits <<= (lane % LPW) * PER;
#pragma unroll
      for (int m = 1; m < LPW; m <<= 1) bits |= (uint32_t)__shfl_xor((int)bits, m);
      if (lane % LPW == 0 && bits != 0u) atomicOr(&p.bitmap[(kr.base + e * Keys::SPAN) / 32 + lane / LPW], bits);
    }
  }
  if (p.idx_out != nullptr || p.pos_out != nullptr || p.val_out != nullptr) {
    lean_outputs(p, b, k, L, [&](auto&& put) {
      fast_emit(kr, sel, 0, k, [&](int i, int out, K bits, int, int) {
        V v;
        __builtin_memcpy(&v, &bits, sizeof(V));
        put(i, out, (float)v);
      });
    });
  }
  HIRE_TS(TB + 7);
}

template <typename V>
__global__ __launch_bounds__(kSelThreads) void k_select_nonneg(SelectParams p) {
  __shared__ LeanShared L;
  constexpr int TB = sizeof(V) == 4 ? 10 : 40;  // stamps of the profiling build: the two instances apart
  HIRE_TS(TB);
  lean_row<TB, V>(p, (int)blockIdx.x, reinterpret_cast<const V*>(p.vals) + (size_t)blockIdx.x * p.stride, L);
}

// ---------------------------------------------------------------------------
// Filter and refine (SelectParams::refine_w): the row holds fp32 values within err_c |u| |x| of the activations
// (launch_gather_dot_bf16).  The kernel selects the k largest stored values, takes the band of non-zero entries
// within hw = 2 err_c xnorm[b] *wnorm_max of the k-th, recomputes those in fp64 (every wave its own entries) into
// refine_h and lists them (value, position) in LDS.  What lies above the band is larger than the true k-th
// activation, what lies below is smaller, so with A entries above the band the k - A largest listed ones
// complete the selection.  refine_h finally receives the value (as rounded to fp32, which is what the second
// layer uses) of every selected entry: the second layer reads its coefficients there.  If the list does not settle it (band reaching the zeros, more
// entries than the list holds, counts that do not fit), the row's remaining stored values are written to
// refine_h as well and the row is selected again there in fp64, as launch_select_f64 would.

// fp64 dot product of a bf16 row and a bf16 token by one wave: products exact in fp32, sums in fp64.
__device__ __forceinline__ double wave_row_dot_f64(const uint16_t* row, const uint16_t* tok, int d) {
  const int cpr = d / 8, lane = lane_id();
  const uint4* r4 = reinterpret_cast<const uint4*>(row);
  const uint4* t4 = reinterpret_cast<const uint4*>(tok);
  double acc = 0.0;
#pragma nounroll
  for (int c0 = 0; c0 < cpr; c0 += 4 * kWave) {
    uint4 wv[4], xv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int c = min(c0 + v * kWave + lane, cpr - 1);
      wv[v] = r4[c];
      xv[v] = t4[c];
    }
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (c0 + v * kWave + lane < cpr) {
        const uint32_t wd[4] = {wv[v].x, wv[v].y, wv[v].z, wv[v].w}, xd[4] = {xv[v].x, xv[v].y, xv[v].z, xv[v].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          acc += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
          acc += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
        }
      }
  }
  return wave_sum(acc);
}

// The same for up to four rows at once (the first nr count; the others must point at readable rows): all their
// loads of a 256-chunk slice are in flight together.
__device__ __forceinline__ void wave_rows_dot_f64(const uint16_t* const (&row)[4], int nr, const uint16_t* tok, int d,
                                                  double (&out)[4]) {
  const int cpr = d / 8, lane = lane_id();
  const uint4* t4 = reinterpret_cast<const uint4*>(tok);
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma nounroll
  for (int c0 = 0; c0 < cpr; c0 += 2 * kWave) {
    uint4 wv[4][2], xv[2];
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      const int c = min(c0 + v * kWave + lane, cpr - 1);
      xv[v] = t4[c];
#pragma unroll
      for (int u = 0; u < 4; ++u) wv[u][v] = reinterpret_cast<const uint4*>(row[u])[c];
    }
#pragma unroll
    for (int v = 0; v < 2; ++v)
      if (c0 + v * kWave + lane < cpr) {
        const uint32_t xd[4] = {xv[v].x, xv[v].y, xv[v].z, xv[v].w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (u < nr) {  // uniform
            const uint32_t wd[4] = {wv[u][v].x, wv[u][v].y, wv[u][v].z, wv[u][v].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              acc[u] += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
              acc[u] += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
            }
          }
        }
      }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) out[u] = wave_sum(acc[u]);
}

__global__ __launch_bounds__(kSelThreads) void k_select_refine(SelectParams p) {
  using K = uint32_t;
  constexpr int LOADS = 4, TB = 40;
  using Keys = KeyRegs<K, LOADS, kSelThreads>;
  constexpr int PER = Keys::PER;
  static_assert(Keys::CAPACITY == kCachedMax && LOADS * PER <= 32, "rows of up to 16384 entries, one bit per key of a lane");
  __shared__ LeanShared L;
  const int b = (int)blockIdx.x, tid = (int)threadIdx.x, lane = lane_id();
  const int w = __builtin_amdgcn_readfirstlane(wave_id());
  const int cap = p.n_dev ? p.n_cap : p.n, k = p.k;
  const float* vals = reinterpret_cast<const float*>(p.vals) + (size_t)b * p.stride;
  double* h = p.refine_h + (size_t)b * p.refine_h_stride;
  HIRE_TS(TB);
  const int n_raw = p.n_dev ? *p.n_dev : p.n;
  Keys kr;
  kr.issue_clamped(vals, cap);
  if (tid == 0) L.band_n = 0;
  kr.finish();
  const int n = p.n_dev ? min(n_raw, p.n_cap) : p.n;
  kr.mask_beyond(n);
  const Selection<K> sel0 = lean_select<TB>(kr, vals, k, L, p.window_misses);
  // the band around the k-th stored value, as bit patterns of non-negative floats (they order like the values);
  // its bounds are rounded outwards, zeros are never part of it; with k = n everything is selected anyway
  const double cut0 = (double)__uint_as_float(sel0.cut.key);
  const double hw = 2.0 * (double)p.err_c * (double)p.xnorm[b] * (double)__uint_as_float(*p.wnorm_max) * 1.000001;
  const double lo_v = cut0 - hw, hi_v = cut0 + hw;
  const float lo_f = __double2float_rd(lo_v), hi_f = __double2float_ru(hi_v);
  const K lo_k = lo_f > 0.0f ? __float_as_uint(lo_f) : 1u, hi_k = __float_as_uint(hi_f);
  const bool any = k < n && hi_k >= lo_k;
  const K width = any ? hi_k - lo_k : 0u;
  int gt = 0;
  uint32_t bits = 0u;  // bit e * PER + q: this lane's key (e, q) lies in the band
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const K key = kr.r[e][q];
      gt += key > hi_k ? 1 : 0;
      if (any && (K)(key - lo_k) <= width) bits |= 1u << (e * PER + q);
    }
  const int above = wave_sum(gt);
  __syncthreads();  // every wave has left the selection: its list in LDS and its counts are free
  if (lane == 0) L.wave_cnt[w] = above;
  HIRE_TS(49);
  unsigned long long* lkey = reinterpret_cast<unsigned long long*>(L.sh.hist);  // [kFastAmbCap] refined values
  int* lidx = reinterpret_cast<int*>(L.sh.hist + 2 * kFastAmbCap);              // [kFastAmbCap] their positions
  {
    const int32_t* map = p.map + (size_t)b * p.map_stride;
    const uint16_t* tok = p.refine_x + (size_t)b * p.refine_d;
    uint64_t owners = __ballot(bits != 0u);
    while (owners != 0ull) {  // uniform over the wave
      const int src = __builtin_ctzll(owners);
      owners &= owners - 1ull;
      uint32_t sb = (uint32_t)__builtin_amdgcn_readlane((int)bits, src);
      while (sb != 0u) {
        const int t = __builtin_ctz(sb);
        sb &= sb - 1u;
        const int pos = kr.base + (t / PER) * Keys::SPAN + src * PER + (t % PER);
        const int unit = map[pos];
        double s = wave_row_dot_f64(p.refine_w + (size_t)unit * p.refine_d, tok, p.refine_d);
        s = s > 0.0 ? s : 0.0;  // ReLU, and -0 -> +0
        if (lane == 0) {
          h[pos] = s;
          const int slot = atomicAdd(&L.band_n, 1);
          if (slot < kFastAmbCap) {
            lkey[slot] = (unsigned long long)__double_as_longlong(s);
            lidx[slot] = pos;
          }
        }
      }
    }
  }
  __syncthreads();
  HIRE_TS(50);
  const int pa = wave_scan_incl(lane < kSelWaves ? L.wave_cnt[lane] : 0);
  const int A = __builtin_amdgcn_readlane(pa, kSelWaves - 1), C = L.band_n;
  const int need = k - A;
  if (k >= n) {  // uniform: every entry of the row is selected, nothing was refined
    lean_outputs(p, b, k, L, [&](auto&& put) {
      fast_emit(kr, sel0, 0, k, [&](int i, int out, K key, int, int) { put(i, out, __uint_as_float(key)); });
    }, h);
    HIRE_TS(TB + 7);
    return;
  }
  bool settled = false;
  int first = 0, count = 0;
  uint32_t selbits = 0u;  // bit e * PER + q: this lane's band key (e, q) is selected
  if (lo_v > 0.0 && C <= kFastAmbCap && need >= 1 && need <= C) {  // uniform over the workgroup
    const int m = C;
    const unsigned long long mine_k = lane < m ? lkey[lane] : 0ull;
    const int mine_i = lane < m ? lidx[lane] : 0x7FFFFFFF;
    int rank = 0;  // listed entries ahead of this lane's (value descending, position ascending)
    for (int u = 0; u < m; ++u) {
      const unsigned long long ok = read_lane(mine_k, u);
      const int oi = __builtin_amdgcn_readlane(mine_i, u);
      rank += ranks_ahead((uint64_t)ok, oi, (uint64_t)mine_k, mine_i) ? 1 : 0;
    }
    const bool taken = lane < m && rank < need;
    const uint64_t last = __ballot(lane < m && rank == need - 1);  // exactly one lane
    const double cut = __longlong_as_double((long long)read_lane(mine_k, __builtin_ctzll(last)));
    if (cut > lo_v && cut < hi_v) {  // the true k-th activation lies inside the band
      settled = true;
      const int above_before = w > 0 ? __builtin_amdgcn_readlane(pa, w - 1) : 0;
      const int rel = mine_i - kr.base;  // position inside this wave's range, if 0 <= rel < len
      const bool here = taken && rel >= 0 && rel < kr.len;
      first = above_before + __popcll(__ballot(taken && rel < 0));
      count = above + __popcll(__ballot(here));
      uint64_t mine = __ballot(here);  // the selected listed entries of this wave's range: mark them at their owners
      while (mine != 0ull) {
        const int s = __builtin_ctzll(mine);
        mine &= mine - 1ull;
        const int r = __builtin_amdgcn_readlane(rel, s);
        const int e = r / Keys::SPAN, l = (r % Keys::SPAN) / PER, q = r % PER;
        if (lane == l) selbits |= 1u << (e * PER + q);
      }
    }
  }
  HIRE_TS(51);
  if (settled) {  // uniform over the workgroup
    lean_outputs(p, b, k, L, [&](auto&& put) {
      fast_emit_if(
          kr, first, count, 0, k,
          [&](int e, int q) { return kr.r[e][q] > hi_k || ((selbits >> (e * PER + q)) & 1u) != 0u; },
          [&](int i, int out, K key, int e, int q) {
            double v = (double)__uint_as_float(key);
            if (((selbits >> (e * PER + q)) & 1u) != 0u)
              v = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const unsigned long long*>(h + i),
                                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            put(i, out, (float)v);
          });
    }, h);
    HIRE_TS(TB + 7);
    return;
  }
  // not settled: the stored values outside the band join the refined ones, and the row is selected there
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < PER; ++q)
      if (kr.valid(e, q) && ((bits >> (e * PER + q)) & 1u) == 0u) h[kr.index(e, q)] = (double)__uint_as_float(kr.r[e][q]);
  if (tid == 0 && p.window_misses) atomicAdd(p.window_misses, 1u);
  __syncthreads();
  SelectParams p2 = p;
  p2.n_dev = nullptr;
  p2.n = n;
  p2.n_cap = n;
  lean_row<TB, double>(p2, b, h, L);
}


// ---------------------------------------------------------------------------
// Filter and refine for the classifier (Algorithm 1 with phi = identity, then eq. (2)): the row holds fp32 logits
// within err_c |w| |x| of the true ones.  With t~ the k-th largest stored value, every entry stored below
// t~ - 2 err_c |x| max|w| has a true logit below that of k others, so only the entries at or above that mark -
// k and a few - are recomputed in fp64 (a wave per row), ranked (value descending, position ascending) and the
// first k kept, in rank order, with the softmax over them.  (A lower bound of t~ serves as well.)  The entries go through an LDS list of kSmList; rows
// with more of them (many equal logits) take several rounds, each merged with the best k so far.
constexpr int kSmList = 1024;
static_assert(kSoftmaxRefineMaxRow / kSelThreads == 64, "one bit of a 64-bit mask per value of a thread");

// kSmItems: values per thread (rows of up to 1024 kSmItems entries)
template <int kSmItems>
__global__ __launch_bounds__(kSelThreads) void k_softmax_refine(SelectParams p) {
  __shared__ SelShared sh;
  __shared__ __align__(16) uint32_t win[kWin];  // window histogram of the stored values' fine bins; then the list
  static_assert(kSmList * (sizeof(int) + sizeof(double)) <= kWin * sizeof(uint32_t), "the list fits the window's memory");
  double* l_val = reinterpret_cast<double*>(win);
  int* l_pos = reinterpret_cast<int*>(win + 2 * kSmList);
  __shared__ int b_pos[2][kSoftmaxRefineMaxK];
  __shared__ double b_val[2][kSoftmaxRefineMaxK];
  __shared__ int l_n;
  const int b = (int)blockIdx.x, tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int k = p.k;
  const int n = p.n_dev ? min(*p.n_dev, p.n_cap) : p.n;
  const float* vals = reinterpret_cast<const float*>(p.vals) + (size_t)b * p.stride;
  const int32_t* map = p.map + (size_t)b * p.map_stride;
  // value i of thread t is entry t + 1024 i; order keys, 0 (below every number) past the row's end
  uint32_t key[kSmItems];
  static_assert(kSmItems % 16 == 0 && kSmItems <= 64, "whole batches of loads");
#pragma unroll
  for (int i0 = 0; i0 < kSmItems; i0 += 16) {
    float v[16];
    if (kSelThreads * i0 < n) {  // uniform: short rows skip the batches past their end
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = vals[min(tid + kSelThreads * (i0 + u), n - 1)];  // clamped, unconditional
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) key[i0 + u] = tid + kSelThreads * (i0 + u) < n ? order_key(v[u]) : 0u;
  }
  // A lower bound of the k-th largest stored value is enough (a lower mark only lists a few more entries): the
  // lower edge of the fine bin (2^14 consecutive order keys) that holds it, found by walking a window histogram of
  // the 8192 bins below the row's largest key; if fewer than k keys lie inside, the next 8192 bins, and so on.
  uint32_t mx = 0u;
#pragma unroll
  for (int i = 0; i < kSmItems; ++i) mx = key[i] > mx ? key[i] : mx;
  mx = wg_max_u32(mx, sh);
  int anchor = (int)(mx >> kFineShift), above = 0;
  uint32_t floor_key = 0u;  // 0: every entry of the row
  while (true) {  // uniform
    __syncthreads();  // the window's readers of the round before are done
    {
      uint4* z = reinterpret_cast<uint4*>(win) + 2 * tid;
      z[0] = z[1] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSmItems; ++i) {
      const uint32_t slot = (uint32_t)(anchor - (int)(key[i] >> kFineShift));
      if (key[i] != 0u && slot < (uint32_t)kWin) atomicAdd(&win[slot], 1u);
    }
    __syncthreads();
    const uint4 c0 = reinterpret_cast<const uint4*>(win)[2 * tid], c1 = reinterpret_cast<const uint4*>(win)[2 * tid + 1];
    const int c[8] = {(int)c0.x, (int)c0.y, (int)c0.z, (int)c0.w, (int)c1.x, (int)c1.y, (int)c1.z, (int)c1.w};
    int mine = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) mine += c[q];
    int total;
    const int incl = wg_scan_incl<kSelThreads>(mine, sh, &total);
    const int need = k - above;  // >= 1
    if (total >= need) {         // uniform: one thread holds the bin of the need-th key
      int run = incl - mine;
      if (run < need && need <= incl) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          if (run < need && need <= run + c[q]) sh.bc_bin = 8 * tid + q;
          run += c[q];
        }
      }
      __syncthreads();
      const int bin = anchor - sh.bc_bin;  // >= 0
      floor_key = bin > 0 ? (uint32_t)bin << kFineShift : 0u;
      break;
    }
    above += total;
    anchor -= kWin;
    if (anchor < 0) break;  // cannot happen with k <= n: every key lies in some window
  }
  const double mark = (floor_key != 0u ? (double)key_value(floor_key) : -__builtin_huge_val()) -
                      2.0 * (double)p.err_c * (double)p.xnorm[b] * (double)__uint_as_float(*p.wnorm_max) * 1.000001;
  const uint32_t mark_key = floor_key != 0u ? order_key(__double2float_rd(mark)) : 1u;
  unsigned long long pending = 0ull;  // bit i: value i has to be recomputed and has not been listed yet
#pragma unroll
  for (int i = 0; i < kSmItems; ++i)
    if (key[i] != 0u && key[i] >= mark_key) pending |= 1ull << i;
  const uint16_t* tok = p.refine_x + (size_t)b * p.refine_d;
  int have = 0, cur = 0;  // entries of the best list so far, and which of its two copies holds them
  while (true) {  // uniform
    __syncthreads();  // the list and the counters of the round before have been read
    if (tid == 0) l_n = 0;
    __syncthreads();
    const int room = kSmList - have;
    while (pending != 0ull) {
      const int i = __builtin_ctzll(pending);
      const int slot = atomicAdd(&l_n, 1);
      if (slot >= room) break;
      l_pos[slot] = tid + kSelThreads * i;
      pending &= pending - 1ull;
    }
    __syncthreads();
    const int listed = min(l_n, room);
    for (int e0 = w; e0 < listed; e0 += 4 * kSelWaves) {  // a wave per row, four rows in flight per wave
      const uint16_t* row[4];
      int nr = 0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * kSelWaves;
        if (e < listed) nr = u + 1;
        row[u] = p.refine_w + (size_t)map[l_pos[min(e, listed - 1)]] * p.refine_d;
      }
      double s4[4];
      wave_rows_dot_f64(row, nr, tok, p.refine_d, s4);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (lane == 0 && u < nr) l_val[e0 + u * kSelWaves] = s4[u] == 0.0 ? 0.0 : s4[u];  // -0 -> +0
    }
    // the best so far join the list, then every entry is ranked among all of them
    for (int t = tid; t < have; t += kSelThreads) {
      l_pos[listed + t] = b_pos[cur][t];
      l_val[listed + t] = b_val[cur][t];
    }
    __syncthreads();
    const int m = listed + have;
    if (tid < m) {
      const double mine = l_val[tid];
      const int mine_pos = l_pos[tid];
      int rank = 0;
      for (int u0 = 0; u0 < m; u0 += 8) {  // eight LDS reads in flight
        double ov[8];
        int op[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          ov[j] = l_val[min(u0 + j, m - 1)];
          op[j] = l_pos[min(u0 + j, m - 1)];
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          rank += (u0 + j < m) && (ov[j] > mine || (ov[j] == mine && op[j] < mine_pos));
      }
      if (rank < k) {
        b_pos[cur ^ 1][rank] = mine_pos;
        b_val[cur ^ 1][rank] = mine;
      }
    }
    have = min(k, m);
    cur ^= 1;
    if (!__syncthreads_or(pending != 0ull)) break;
  }
  // the k survivors in rank order; softmax: exp(z - zmax) / sum
  const double zmax = b_val[cur][0];
  double part = 0.0;
  for (int t = tid; t < k; t += kSelThreads) part += exp(b_val[cur][t] - zmax);
  part = wave_sum(part);
  if (lane == 0) sh.red_a[w] = (unsigned long long)__double_as_longlong(part);
  __syncthreads();
  double sum = 0.0;
  for (int u = 0; u < kSelWaves; ++u) sum += __longlong_as_double((long long)sh.red_a[u]);
  for (int t = tid; t < k; t += kSelThreads) {
    const double z = b_val[cur][t];
    if (p.idx_out) p.idx_out[(size_t)b * k + t] = map[b_pos[cur][t]];
    if (p.val_out) p.val_out[(size_t)b * k + t] = (float)z;
    if (p.prob_out) p.prob_out[(size_t)b * k + t] = (float)(exp(z - zmax) / sum);
  }
}

hipError_t launch_softmax_refine(const SelectParams& p, int B, hipStream_t s) {
  const int cap = p.n_dev ? p.n_cap : p.n;
  if (cap < 1 || cap > kSoftmaxRefineMaxRow || p.k < 1 || p.k > kSoftmaxRefineMaxK || !p.refine_w || !p.refine_x ||
      p.refine_d % 8 != 0 || !p.map || !p.xnorm || !p.wnorm_max || !p.vals)
    return hipErrorInvalidValue;
  if (cap <= 16 * kSelThreads) return launch(k_softmax_refine<16>, dim3(B), dim3(kSelThreads), 0, s, p);
  if (cap <= 32 * kSelThreads) return launch(k_softmax_refine<32>, dim3(B), dim3(kSelThreads), 0, s, p);
  return launch(k_softmax_refine<64>, dim3(B), dim3(kSelThreads), 0, s, p);
}

// ---------------------------------------------------------------------------
template <typename V>
static bool select_is_lean(const SelectParams& p) {
  const int cap = p.n_dev ? p.n_cap : p.n;
  return p.nonneg && !p.rank_order && !p.group8 && !p.relu && cap > kSelThreads && cap <= kCachedMax &&
         p.k <= kWin / 2 && reinterpret_cast<uintptr_t>(p.vals) % 16 == 0 && (p.stride * (long long)sizeof(V)) % 16 == 0;
}
bool select_refine_supported(const SelectParams& p) {
  return select_is_lean<float>(p) && p.bitmap == nullptr && reinterpret_cast<uintptr_t>(p.refine_h) % 16 == 0 &&
         (p.refine_h_stride * (long long)sizeof(double)) % 16 == 0 && p.refine_d % 8 == 0;
}
hipError_t launch_select_refine(const SelectParams& p, int B, hipStream_t s) {
  if (!select_refine_supported(p) || !p.refine_w || !p.refine_x || !p.refine_h || !p.map || !p.xnorm || !p.wnorm_max)
    return hipErrorInvalidValue;
  return launch(k_select_refine, dim3(B), dim3(kSelThreads), 0, s, p);
}

template <typename V>
static hipError_t launch_select(const SelectParams& p, int B, hipStream_t s) {
  size_t lds = 0;
  if (p.rank_order) lds = (size_t)p.k * (sizeof(typename KeyOf<V>::K) + 2 * sizeof(int));
  const int cap = p.n_dev ? p.n_cap : p.n;
  if (select_is_lean<V>(p)) return launch(k_select_nonneg<V>, dim3(B), dim3(kSelThreads), 0, s, p);
  if (p.refine_w != nullptr) return hipErrorInvalidValue;  // launch_select_refine's business
  if (p.group8) {  // rows of at most kSelectGroup8Max groups
    if (cap <= kSelThreads) return launch(k_select<V, 1, true>, dim3(B), dim3(kSelThreads), lds, s, p);
    if (cap <= 4 * kSelThreads) return launch(k_select<V, 4, true>, dim3(B), dim3(kSelThreads), lds, s, p);
    return hipErrorInvalidValue;
  }
  if (cap <= kSelThreads) return launch(k_select<V, 1>, dim3(B), dim3(kSelThreads), lds, s, p);
  if (cap <= 4 * kSelThreads) return launch(k_select<V, 4>, dim3(B), dim3(kSelThreads), lds, s, p);
  if (cap <= kCachedMax) return launch(k_select<V, kItemsMax>, dim3(B), dim3(kSelThreads), lds, s, p);
  return launch(k_select<V, 0>, dim3(B), dim3(kSelThreads), lds, s, p);
}

hipError_t launch_select_f32(const SelectParams& p, int B, hipStream_t s) { return launch_select<float>(p, B, s); }
hipError_t launch_select_f64(const SelectParams& p, int B, hipStream_t s) { return launch_select<double>(p, B, s); }

size_t multi_body_bytes_host(int B) { return multi_body_bytes(B); }
size_t general_fallbacks_offset(int which) {
  switch (which) {
    case 0: return offsetof(GeneralHeader, multi) + offsetof(MultiHeader, fallbacks);
    case 1: return offsetof(GeneralHeader, window_misses);
    default: return offsetof(GeneralHeader, multi) + offsetof(MultiHeader, stamps);
  }
}

bool multi_producer_counts(int N, int B) { return (long long)N * B <= kDirectCountMaxKeys; }
int multi_hist_shift(int N, int B) { return multi_producer_counts(N, B) ? kHistShift : kCoarseShift; }

// Shared by the step (one union bitmap, keys already passed through phi) and topk_select on long rows (a bitmap per
// row, ReLU applied on the fly, always counted by the pass of its own).
static hipError_t mark_rows(const float* keys, int B, int N, int k, int slots, bool own_count, int relu,
                            const MultiRegion& mr, uint32_t* bitmap, long long bitmap_stride, hipStream_t s) {
  const int shift = own_count ? kCoarseShift : kHistShift;
  if (own_count) {
    const int chunks = (N + kSelThreads * kCountKeys - 1) / (kSelThreads * kCountKeys);
    const hipError_t e = launch(k_count_f32, dim3(chunks, B), dim3(kSelThreads), 0, s, keys, B, N, slots, shift, relu, mr);
    if (e != hipSuccess) return e;
  }
  const int chunks = (N + kSelThreads * kMarkKeys - 1) / (kSelThreads * kMarkKeys);
  return launch(k_mark_f32, dim3(chunks, B), dim3(kSelThreads), 0, s, keys, B, N, k, slots, shift, relu, mr, bitmap,
                bitmap_stride);
}

static hipError_t resolve_rows(const float* keys, int B, int N, int k, bool own_count, int relu, const MultiRegion& mr,
                               uint32_t* bitmap, long long bitmap_stride, hipStream_t s) {
  // per-key cleaning spreads over up to 64 workgroups; the window of the counting pass needs few
  const int cleaners = own_count ? 2 : min(64, (N + kCleanKeys - 1) / kCleanKeys);
  return launch(k_resolve_compact, dim3(1 + cleaners, B), dim3(kSelThreads), 0, s, keys, B, N, k,
                own_count ? kCoarseShift : kHistShift, relu, mr, bitmap, bitmap_stride);
}

hipError_t launch_mark_f32(const float* keys, int B, int N, int kprime, int slots, const HistRefs& hr, uint32_t* bitmap,
                           hipStream_t s) {
  return mark_rows(keys, B, N, kprime, slots, !multi_producer_counts(N, B), 0, multi_of(hr, B), bitmap, 0, s);
}

hipError_t launch_resolve_compact(const float* keys, int B, int N, int kprime, const HistRefs& hr, uint32_t* bitmap,
                                  int words, int32_t* list_out, int32_t* count_out, int32_t* count_out2,
                                  uint32_t* zero_ptr, int zero_words, hipStream_t s) {
  const MultiRegion mr = multi_of(hr, B);
  const hipError_t e = resolve_rows(keys, B, N, kprime, !multi_producer_counts(N, B), 0, mr, bitmap, 0, s);
  if (e != hipSuccess || list_out == nullptr) return e;  // no list wanted: the gather compacts the bitmap itself
  return launch(k_union_compact, dim3(1), dim3(kSelThreads), 0, s, B, mr, bitmap, words, list_out, count_out,
                count_out2, zero_ptr, zero_words);
}

size_t topk_long_workspace_bytes(int B, int N) {
  const size_t words = (size_t)(N + 31) / 32 + 2;
  return multi_body_bytes(B) + (B * words * 4 + 255) / 256 * 256 + ((size_t)B * 4 + 255) / 256 * 256;
}

hipError_t launch_topk_long(const float* scores, int B, int N, int k, int relu, int32_t* idx_out, float* val_out,
                            void* general_header, void* body, unsigned long long sig, hipStream_t s) {
  const int words = (N + 31) / 32 + 2;
  const MultiRegion mr = carve_multi(&static_cast<GeneralHeader*>(general_header)->multi, body, B);
  char* after = static_cast<char*>(body) + multi_body_bytes(B);
  uint32_t* bitmaps = reinterpret_cast<uint32_t*>(after);
  int32_t* counts = reinterpret_cast<int32_t*>(after + ((size_t)B * words * 4 + 255) / 256 * 256);
  const int chunks = (N + kSelThreads * kCountKeys - 1) / (kSelThreads * kCountKeys);
  if (chunks > kWgMaxSlots) return hipErrorInvalidValue;
  hipError_t e = launch(k_row_maxima, dim3(chunks, B), dim3(kSelThreads), 0, s, scores, N, relu, mr, bitmaps,
                        (long long)B * words, static_cast<GeneralHeader*>(general_header), sig);
  if (e != hipSuccess) return e;
  if ((e = mark_rows(scores, B, N, k, chunks, true, relu, mr, bitmaps, words, s)) != hipSuccess) return e;
  if ((e = resolve_rows(scores, B, N, k, true, relu, mr, bitmaps, words, s)) != hipSuccess) return e;
  return launch(k_emit_rows, dim3(B), dim3(kSelThreads), 0, s, scores, B, N, k, relu, mr, bitmaps, words, idx_out, val_out,
                counts);
}

hipError_t launch_bitmap_compact(const uint32_t* bitmap, int words, int32_t* list_out, int32_t* count_out,
                                 int32_t* count_out2, uint32_t* zero_ptr, int zero_words, hipStream_t s) {
  return launch(k_bitmap_compact, dim3(1), dim3(kSelThreads), 0, s, bitmap, words, list_out, count_out,
                     count_out2, zero_ptr, zero_words);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_select(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
