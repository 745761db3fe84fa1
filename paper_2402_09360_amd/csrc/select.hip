// Exact top-k selection kernels (TopInd_k / Top_k of arXiv 2402.09360 Sec. 3.1,
// used on both lines of Algorithm 1) and the bitmap compaction that forms the
// batch union of Sec. 3.4.1.
//
// One 1024-thread workgroup per score row.  Wave w owns the contiguous index
// range [w*M, (w+1)*M), M a multiple of 64, and walks it 64 at a time, so a
// wave ballot is a 64-bit slice of the selection mask in index order: ordered
// output positions come from popcounts, no sorting, and ties at the threshold
// go to the lowest indices by construction.
#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kItems = 16;                          // register-resident keys per thread
constexpr int kCachedMax = kSelThreads * kItems;    // 16384
constexpr int kRankMax = 4096;                      // largest k sorted into rank order

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

template <typename V, bool CACHED>
__global__ __launch_bounds__(kSelThreads) void k_select(SelectParams p) {
  using K = typename KeyOf<V>::K;
  __shared__ SelShared sh;
  __shared__ int tot_gt[kSelWaves], tot_eq[kSelWaves];
  extern __shared__ unsigned long long dyn[];  // rank order only: K keys[k], then int pos[k]

  const int b = (int)blockIdx.x;
  const int n = p.n_dev ? min(*p.n_dev, p.n_cap) : p.n;
  const int k = p.k;
  const V* vals = reinterpret_cast<const V*>(p.vals) + (size_t)b * p.stride;
  const int lane = lane_id(), w = wave_id();
  const int M = (((n + kSelWaves - 1) / kSelWaves) + kWave - 1) / kWave * kWave;
  const int base = w * M;
  const int iters = M / kWave;

  auto load_key = [&](int i) -> K {
    V v = vals[i];
    if (p.relu) v = v > (V)0 ? v : (V)0;
    return order_key(v);
  };

  HIRE_TS(0);
  K regs[kItems];
  if (CACHED) {
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      const int i = base + e * kWave + lane;
      regs[e] = (e < iters && i < n) ? load_key(i) : (K)0;
    }
  }
  // element visitor: f(e, i, key) for every owned, valid element in index order
  auto visit = [&](auto&& f) {
    if (CACHED) {
#pragma unroll
      for (int e = 0; e < kItems; ++e) {
        const int i = base + e * kWave + lane;
        if (e < iters && i < n) f(e, i, regs[e]);
      }
    } else {
      for (int e = 0; e < iters; ++e) {
        const int i = base + e * kWave + lane;
        if (i < n) f(e, i, load_key(i));
      }
    }
  };

  const K T = wg_kth_largest<K>([&](auto&& f) { visit([&](int, int, K key) { f(key); }); }, n, k, sh);

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
  float* coef = p.coef ? p.coef + (size_t)b * p.coef_stride : nullptr;
  for (int e = 0; e < iters; ++e) {  // uniform trip count per wave: ballots are safe
    const int i = base + e * kWave + lane;
    const bool valid = i < n;
    K key = 0;
    if (CACHED) {
      // regs[] is indexed with a loop-uniform e; select without dynamic register indexing
#pragma unroll
      for (int q = 0; q < kItems; ++q)
        if (q == e) key = regs[q];
    } else if (valid) {
      key = load_key(i);
    }
    const bool gt = valid && key > T, eq = valid && key == T;
    const uint64_t mg = __ballot(gt), me = __ballot(eq);
    const int gt_before = run_gt + mask_prefix(mg), eq_before = run_eq + mask_prefix(me);
    const bool sel = gt || (eq && eq_before < need_eq);
    const int out = gt_before + min(eq_before, need_eq);
    run_gt += __popcll(mg);
    run_eq += __popcll(me);
    const V v = key_value(key);
    if (coef && valid) coef[i] = sel ? (float)v : 0.0f;
    if (p.bitmap) {
      const uint64_t ms = __ballot(sel);
      if (lane == 0 && (uint32_t)ms) atomicOr(&p.bitmap[(base + e * kWave) >> 5], (uint32_t)ms);
      if (lane == 32 && (uint32_t)(ms >> 32)) atomicOr(&p.bitmap[((base + e * kWave) >> 5) + 1], (uint32_t)(ms >> 32));
    }
    if (sel) {
      if (p.rank_order) {
        rk_key[out] = key;
        rk_pos[out] = i;
      } else {
        if (p.idx_out) p.idx_out[(size_t)b * k + out] = p.map ? p.map[i] : i;
        if (p.pos_out) p.pos_out[(size_t)b * k + out] = i;
        if (p.val_out) p.val_out[(size_t)b * k + out] = (float)v;
      }
    }
  }
  HIRE_TS(8);
  if (!p.rank_order) return;

  // ---- rank order: position of each selected entry among the k (value desc, index asc) ----
  __syncthreads();
  constexpr int kPerThread = kRankMax / kSelThreads;
  int my_rank[kPerThread];
  V my_val[kPerThread];
#pragma unroll
  for (int q = 0; q < kPerThread; ++q) {
    const int t = (int)threadIdx.x + q * kSelThreads;
    my_rank[q] = -1;
    my_val[q] = (V)0;
    if (t < k) {
      const K mine = rk_key[t];
      int rank = 0;
      for (int u = 0; u < k; ++u) {
        const K other = rk_key[u];
        rank += (other > mine) || (other == mine && u < t);  // list is in index order, so u < t is "lower index"
      }
      const int i = rk_pos[t];
      const V v = key_value(mine);
      if (p.idx_out) p.idx_out[(size_t)b * k + rank] = p.map ? p.map[i] : i;
      if (p.pos_out) p.pos_out[(size_t)b * k + rank] = i;
      if (p.val_out) p.val_out[(size_t)b * k + rank] = (float)v;
      my_rank[q] = rank;
      my_val[q] = v;
    }
  }
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
}

// ---------------------------------------------------------------------------
// Bitmap -> ascending index list, one workgroup.
__global__ __launch_bounds__(kSelThreads) void k_bitmap_compact(const uint32_t* __restrict__ bitmap, int words,
                                                                int32_t* __restrict__ list_out,
                                                                int32_t* __restrict__ count_out,
                                                                int32_t* __restrict__ count_out2, uint32_t* zero_ptr,
                                                                int zero_words) {
  __shared__ SelShared sh;
  const int tid = (int)threadIdx.x;
  if (zero_ptr)
    for (int i = tid; i < zero_words; i += kSelThreads) zero_ptr[i] = 0u;
  const int wpt = (words + kSelThreads - 1) / kSelThreads;
  const int w0 = tid * wpt, w1 = min(words, w0 + wpt);
  int cnt = 0;
  for (int q = w0; q < w1; ++q) cnt += __popc(bitmap[q]);
  const int incl = wg_scan_incl(cnt, sh);
  int out = incl - cnt;
  for (int q = w0; q < w1; ++q) {
    uint32_t m = bitmap[q];
    while (m) {
      const int bit = __ffs((int)m) - 1;
      list_out[out++] = q * 32 + bit;
      m &= m - 1;
    }
  }
  if (tid == kSelThreads - 1) {
    count_out[0] = incl;
    if (count_out2) count_out2[0] = incl;
  }
}

// ---------------------------------------------------------------------------
template <typename V>
static hipError_t launch_select(const SelectParams& p, int B, hipStream_t s) {
  size_t lds = 0;
  if (p.rank_order) lds = (size_t)p.k * (sizeof(typename KeyOf<V>::K) + sizeof(int));
  const int cap = p.n_dev ? p.n_cap : p.n;
  if (cap <= kCachedMax) return launch(k_select<V, true>, dim3(B), dim3(kSelThreads), lds, s, p);
  return launch(k_select<V, false>, dim3(B), dim3(kSelThreads), lds, s, p);
}

hipError_t launch_select_f32(const SelectParams& p, int B, hipStream_t s) { return launch_select<float>(p, B, s); }
hipError_t launch_select_f64(const SelectParams& p, int B, hipStream_t s) { return launch_select<double>(p, B, s); }

hipError_t launch_bitmap_compact(const uint32_t* bitmap, int words, int32_t* list_out, int32_t* count_out,
                                 int32_t* count_out2, uint32_t* zero_ptr, int zero_words, hipStream_t s) {
  return launch(k_bitmap_compact, dim3(1), dim3(kSelThreads), 0, s, bitmap, words, list_out, count_out,
                     count_out2, zero_ptr, zero_words);
}

}  // namespace hire
