// HiRE-Softmax for one token on a long vocabulary (arXiv 2402.09360, Sec. 3.3 with Algorithm 1, phi = identity,
// and eq. (2)): the two kernels that follow the int4 scorers (HiRE-Q, HiRE-LRQ) on the short kernel sequence.
//
// The scorer leaves the keys and, per workgroup (rows of at most 512 codes: per wave), the largest key of its rows
// (~62 of them for the int4 scorer on 256000 classes).  The k'-th largest of those maxima is a lower bound of the
// k'-th largest key (each maximum is a key of its own), so the keys at or above it are a superset of the shortlist,
// typically 15-20 % larger than k' (40 % with the 2048 per-wave maxima of the short-row scorer).  The bound need
// not be the k'-th maximum itself: the maxima are counted into a window of coarse bins in LDS - slot s counts bin
// anchor - s, the anchor an a-priori upper bound of every key (7 * 127 * codes per row * largest row scale), so no
// reduction comes first - and the lower edge t of the bin in which the running count from the top reaches k'
// serves.
//
//   k_sm1_gather  one workgroup per 2048 keys: counts the maxima and walks the window (every workgroup,
//                 redundantly), finds its own keys >= t, computes their exact logits <w_j, x> in fp64 (a wave per
//                 row) and leaves (key, index, logit) in the workgroup's own slots (4096 slots shared out evenly:
//                 32 for each of the 125 workgroups of a 256000-class vocabulary, three times the expected
//                 number) - no counter shared between workgroups, and the slots of all workgroups in
//                 order are in ascending class order.
//   k_sm1_final   one workgroup, the slots in its registers: drops the D = |superset| - k' smallest keys (ties lose
//                 by higher index) so that exactly Algorithm 1's shortlist remains, takes the k largest logits
//                 of it (ties to the lower index) in rank order and the softmax over them.
//
// Nothing is taken on trust: the final kernel counts the superset itself, and a superset of fewer than k' entries,
// a workgroup with more entries than slots or a window that did not answer (maxima
// below it: a zero token) make it select the shortlist from the keys directly (range narrowing over the whole row,
// then the logits row by row): slow, exact, and counted.
#include <cmath>

#include "hist.h"
#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kSm1Threads = 1024;
constexpr int kSm1Waves = kSm1Threads / kWave;
constexpr int kSm1KeysPerThread = 2;    // one token: 2048 keys per workgroup of k_sm1_gather
constexpr int kSm1KeysPerThreadB = 8;   // batches: 8192 (the grid has a token dimension as well)
constexpr int kSm1Keys = kSm1KeysPerThread * kSm1Threads;
constexpr int kSm1SlotsTotal = 4096;   // slots of all workgroups of k_sm1_gather together
constexpr int kSm1SlotsMax = 1024;     // ... of one workgroup at most
constexpr int kSm1ListCap = 2048;      // entries of the final kernel's lists: a shortlist fits
constexpr int kSm1SlotsPerThread = kSm1SlotsTotal / kSm1Threads;
constexpr int kSm1DropBins = 256;      // fine bins above the superset's lower edge in which the D-th smallest key is looked for
constexpr int kSm1AmbCap = 64;         // keys of the bin that holds it
constexpr int kSm1XChunks = 4;         // 16-byte chunks of the token per lane: d <= 2048
static_assert(kSm1MaxRow / kSm1Keys * 32 <= kSm1SlotsTotal, "at least 32 slots per workgroup");

// Slots per workgroup of k_sm1_gather (kpt keys per thread): an even share of the total.
inline int sm1_workgroups(int N, int kpt) { return (N + kpt * kSm1Threads - 1) / (kpt * kSm1Threads); }
inline int sm1_slots_per_wg(int N, int kpt = kSm1KeysPerThread) {
  const int n_wg = sm1_workgroups(N, kpt);
  return kSm1SlotsTotal / n_wg < kSm1SlotsMax ? kSm1SlotsTotal / n_wg : kSm1SlotsMax;
}
static_assert(kSm1WinBins == 2 * kSm1Threads, "two window bins per thread");

struct Sm1Entry {
  uint32_t okey;  // order key of the scorer key
  int32_t idx;    // class; -1: empty slot; -2 (slot 0 only): the workgroup had more entries than slots
  double z;       // <w_idx, x>
};
static_assert(sizeof(Sm1Entry) == 16, "one 16-byte store per entry");

// Token chunks of a lane (chunk lane + 64 u, clamped) for wave_dot.
__device__ __forceinline__ void sm1_load_token(const uint16_t* x, int c8, uint4 (&xv)[kSm1XChunks]) {
  const uint4* x4 = reinterpret_cast<const uint4*>(x);
#pragma unroll
  for (int u = 0; u < kSm1XChunks; ++u) xv[u] = x4[min(lane_id() + u * kWave, c8 - 1)];
}

// <row, x> by one wave: products exact in fp32, sums in fp64, lanes added by the wave's fixed tree.
__device__ __forceinline__ double sm1_wave_dot(const uint16_t* row, int c8, const uint4 (&xv)[kSm1XChunks]) {
  const uint4* r4 = reinterpret_cast<const uint4*>(row);
  const int lane = lane_id();
  uint4 wv[kSm1XChunks];
#pragma unroll
  for (int u = 0; u < kSm1XChunks; ++u) wv[u] = load_streaming(&r4[min(lane + u * kWave, c8 - 1)]);
  double acc = 0.0;
#pragma unroll
  for (int u = 0; u < kSm1XChunks; ++u)
    if (lane + u * kWave < c8) {
      const uint32_t wd[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w}, xd[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
        acc += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
      }
    }
  return wave_sum(acc);
}

// Exclusive prefix of one count per wave (in LDS, complete) for this wave, and the total.
__device__ __forceinline__ int sm1_wave_base(const int* wave_cnt, int* total) {
  const int lane = lane_id();
  const int p = wave_scan_incl(lane < kSm1Waves ? wave_cnt[lane] : 0);
  const int w = __builtin_amdgcn_readfirstlane(wave_id());
  *total = __builtin_amdgcn_readlane(p, kSm1Waves - 1);
  return w > 0 ? __builtin_amdgcn_readlane(p, w - 1) : 0;
}

// LOGITS = false (batches, launch_maxima_select): grid (workgroups, tokens), token b's keys, maxima and slots; the
// entries carry no logit.  KPT: keys per thread (key q of thread t is KPT * 1024 * workgroup + 1024 q + t).
template <bool LOGITS, int KPT>
__global__ __launch_bounds__(kSm1Threads) void k_sm1_gather(const float* __restrict__ keys, int N, int d, int sd,
                                                            int kprime, int n_max,
                                                            const uint32_t* __restrict__ smax_word,
                                                            const uint16_t* __restrict__ W,
                                                            const uint16_t* __restrict__ x, MultiRegion mr,
                                                            Sm1Entry* __restrict__ slots, int n_slots) {
  __shared__ uint32_t win[kSm1WinBins];
  constexpr int kCounts = KPT * kSm1Waves, kChunks = (kCounts + kWave - 1) / kWave;
  __shared__ int wave_tot[kSm1Waves], wave_cnt[kChunks * kWave];
  __shared__ int bc_slot;
  __shared__ int loc_t[kSm1SlotsMax];
  __shared__ uint32_t loc_key[kSm1SlotsMax];
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id(), b = (int)blockIdx.y;
  const int i0 = (int)blockIdx.x * (KPT * kSm1Threads) + tid, c8 = d / 8;  // this thread's keys: i0 + 1024 q
  keys += (size_t)b * N;
  slots += (size_t)b * gridDim.x * n_slots;
  HIRE_TS(20);
  // everything this workgroup needs before it can decide, in one batch of loads
  float key[KPT];
#pragma unroll
  for (int q = 0; q < KPT; ++q) key[q] = keys[min(i0 + q * kSm1Threads, N - 1)];
  const uint4 mx = reinterpret_cast<const uint4*>(mr.wgmax + (size_t)b * kWgMaxSlots)[tid];  // maxima 4 tid .. 4 tid + 3
  const float smax = __uint_as_float(*smax_word);
  uint4 xv[kSm1XChunks];
  if (LOGITS) sm1_load_token(x, c8, xv);
  reinterpret_cast<uint2*>(win)[tid] = make_uint2(0u, 0u);
  if (tid == 0) bc_slot = 0;
  __syncthreads();
  HIRE_TS(21);

  // ---- the maxima into the window; walk: the slot in which the running count, from the top, reaches k' ----
  const int anchor = sm1_anchor_bin(smax, sd);  // the keys come from rows of sd codes
  const uint32_t mv[4] = {mx.x, mx.y, mx.z, mx.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int slot = anchor - (int)(mv[q] >> kSm1Shift);
    if (4 * tid + q < n_max && slot >= 0 && slot < kSm1WinBins) atomicAdd(&win[slot], 1u);
  }
  __syncthreads();
  const uint2 hb = reinterpret_cast<const uint2*>(win)[tid];  // window slots 2 tid, 2 tid + 1
  const int s = (int)(hb.x + hb.y);
  const int incl = wave_scan_incl(s);
  if (lane == kWave - 1) wave_tot[w] = incl;
  __syncthreads();
  int total;
  const int run = sm1_wave_base(wave_tot, &total) + incl - s;
  const bool found = total >= kprime;  // the same in every workgroup: they all count the same maxima
  if (found && run < kprime && kprime <= run + s) bc_slot = run + (int)hb.x >= kprime ? 2 * tid : 2 * tid + 1;
  __syncthreads();
  const uint32_t okey_lb = (uint32_t)(anchor - bc_slot) << kSm1Shift;  // lower edge of that bin
  if (blockIdx.x == 0 && tid == 0) {
    mr.walk[4 * b + 1] = found ? 1 : 0;
    mr.walk[4 * b + 2] = (int)okey_lb;
  }
  HIRE_TS(22);

  // ---- this workgroup's keys at or above the edge, in index order (all of the first 1024, then the second) ----
  uint32_t okey[KPT];
  uint64_t ballot[KPT];
  if (kCounts % kWave != 0 && tid < kChunks * kWave) wave_cnt[tid] = 0;  // the scan below reads whole chunks of 64
#pragma unroll
  for (int q = 0; q < KPT; ++q) {
    okey[q] = order_key(key[q]);
    ballot[q] = __ballot(found && i0 + q * kSm1Threads < N && okey[q] >= okey_lb);
  }
  if (kCounts % kWave != 0) __syncthreads();
#pragma unroll
  for (int q = 0; q < KPT; ++q)
    if (lane == 0) wave_cnt[q * kSm1Waves + w] = __popcll(ballot[q]);
  __syncthreads();
  int n_loc = 0;
  {
    // prefix over the KPT * 16 counts (key round q of wave w at q * 16 + w), 64 at a time
    int p[kChunks], before[kChunks];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      p[c] = wave_scan_incl(wave_cnt[c * kWave + lane]);
      before[c] = n_loc;
      n_loc += __builtin_amdgcn_readlane(p[c], kWave - 1);
    }
    const int wv = __builtin_amdgcn_readfirstlane(w);
#pragma unroll
    for (int q = 0; q < KPT; ++q) {
      const int slot = q * kSm1Waves + wv;  // uniform over the wave
      const int c = slot / kWave, l = slot % kWave;
      const int pos = before[c] + (l > 0 ? __builtin_amdgcn_readlane(p[c], l - 1) : 0) + mask_prefix(ballot[q]);
      if (((ballot[q] >> lane) & 1ull) && pos < n_slots) {
        loc_t[pos] = tid + q * kSm1Threads;
        loc_key[pos] = okey[q];
      }
    }
  }
  __syncthreads();

  // ---- their logits, a wave per row; every slot of the workgroup is written ----
  Sm1Entry* mine = slots + (size_t)blockIdx.x * n_slots;
  const int n_take = min(n_loc, n_slots);
  for (int e0 = 0; e0 < n_slots; e0 += kSm1Waves) {
    const int e = e0 + w;  // uniform over the wave
    Sm1Entry out;
    out.okey = 0u;
    out.idx = -1;
    out.z = 0.0;
    if (e < n_take) {
      const int j = (int)blockIdx.x * (KPT * kSm1Threads) + loc_t[e];
      if (LOGITS) out.z = sm1_wave_dot(W + (size_t)j * d, c8, xv);
      out.okey = loc_key[e];
      out.idx = j;
    }
    if (e == 0 && n_loc > n_slots) out.idx = -2;
    if (lane == 0 && e < n_slots) mine[e] = out;
  }
  HIRE_TS(23);
}

constexpr int kSm1ZBins = 256;  // bins of the logit selection

struct Sm1Shared {
  SelShared sel;
  uint32_t l_okey[kSm1ListCap];  // a shortlist taken from the keys directly: keys, classes (ascending), logits; ...
  int32_t l_idx[kSm1ListCap];    // ... otherwise, and afterwards, the entries of the k-th logit's bin: classes ...
  double l_z[kSm1ListCap];       // ... and logits (as order keys)
  uint32_t drop_hist[kSm1DropBins];
  uint32_t amb_key[kSm1AmbCap];
  int32_t amb_idx[kSm1AmbCap];
  uint32_t z_hist[kSm1ZBins];
  unsigned long long sel_key[kSm1MaxK];  // the k selected (logit as order key, class), unordered
  int32_t sel_idx[kSm1MaxK];
  double sel_z[kSm1MaxK];                // their logits in rank order
  double wave_lo[kSm1Waves], wave_hi[kSm1Waves];
  int wave_cnt[kSm1Waves];
  int amb_n, zamb_n, sel_n;
};
static_assert(kWgMaxSlots == 4 * kSm1Threads, "four of the scorer's maxima per thread");
static_assert(kSm1MaxShortlist <= kSm1ListCap, "the shortlist fits the lists");

// The k' largest keys of a row straight from the keys, for a selection the maxima could not serve: the k'-th largest
// key by range narrowing over the whole row, then emit(key, index, place) for the keys above it and the
// lowest-indexed of the equal ones, in ascending index order (thread t owns a contiguous range of the row; place
// counts from 0).
template <typename Emit>
__device__ __forceinline__ void sm1_select_from_keys(const float* __restrict__ keys, int N, int kprime,
                                                     SelSharedT<kSm1Threads>& sel, Emit&& emit) {
  const int tid = (int)threadIdx.x;
  auto for_each = [&](auto&& f) {
    for (int i = tid; i < N; i += kSm1Threads) f(order_key(keys[i]));
  };
  const uint32_t cut = wg_kth_largest<uint32_t, kSm1Threads>(for_each, N, kprime, sel);
  const int per = (N + kSm1Threads - 1) / kSm1Threads;
  const int i0 = min(tid * per, N), i1 = min(i0 + per, N);
  int gt = 0, eq = 0;
  for (int i = i0; i < i1; ++i) {
    const uint32_t ok = order_key(keys[i]);
    gt += ok > cut;
    eq += ok == cut;
  }
  int tot_gt, tot_eq;
  wg_scan_incl(gt, sel, &tot_gt);
  const int eq_before = wg_scan_incl(eq, sel, &tot_eq) - eq;
  int take = min(max(kprime - tot_gt - eq_before, 0), eq);  // equal keys: the lowest indices first
  const int mine = gt + take;
  int out = wg_scan_incl(mine, sel) - mine;
  for (int i = i0; i < i1; ++i) {
    const uint32_t ok = order_key(keys[i]);
    bool in = ok > cut;
    if (ok == cut && take > 0) {
      in = true;
      --take;
    }
    if (in) emit(ok, i, out++);
  }
}

// The shortlist that way into the lists of sh, then the logits, a wave per row.
__device__ __noinline__ void sm1_shortlist_from_keys(const float* __restrict__ keys, int N, int d, int kprime,
                                                     const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                                     Sm1Shared& sh) {
  const int lane = lane_id(), w = wave_id();
  sm1_select_from_keys(keys, N, kprime, sh.sel, [&](uint32_t ok, int i, int place) {
    sh.l_okey[place] = ok;
    sh.l_idx[place] = i;
  });
  __syncthreads();
  uint4 xv[kSm1XChunks];
  sm1_load_token(x, d / 8, xv);
  for (int e = w; e < kprime; e += kSm1Waves) {
    const double z = sm1_wave_dot(W + (size_t)sh.l_idx[e] * d, d / 8, xv);
    if (lane == 0) sh.l_z[e] = z;
  }
  __syncthreads();
}

__global__ __launch_bounds__(kSm1Threads) void k_sm1_final(const float* __restrict__ keys, int N, int d, int k,
                                                           int kprime, const uint16_t* __restrict__ W,
                                                           const uint16_t* __restrict__ x, MultiRegion mr,
                                                           const Sm1Entry* __restrict__ slots, int n_slots,
                                                           int32_t* __restrict__ top_idx, float* __restrict__ top_prob,
                                                           float* __restrict__ top_logit,
                                                           int32_t* __restrict__ cand_idx,
                                                           int32_t* __restrict__ n_cand) {
  constexpr int E = kSm1SlotsPerThread;
  __shared__ Sm1Shared sh;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  // ---- the slots stay in registers: wave w holds slots 256 w .. 256 w + 255, round j the 64 from 256 w + 64 j
  // (a load instruction takes one contiguous KB), so (wave, round, lane) is ascending class order ----
  uint32_t okey[E];
  int32_t idx[E];
  double z[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int sl = w * (E * kWave) + j * kWave + lane;
    const uint4 v = reinterpret_cast<const uint4*>(slots)[min(sl, n_slots - 1)];
    okey[j] = v.x;
    idx[j] = sl < n_slots ? (int32_t)v.y : -1;
    z[j] = __hiloint2double((int)v.w, (int)v.z);
  }
  const bool answered = mr.walk[1] != 0;
  const uint32_t okey_lb = (uint32_t)mr.walk[2];
  HIRE_TS(30);
  if (tid < kSm1DropBins) sh.drop_hist[tid] = 0u;
  if (tid < kSm1ZBins) sh.z_hist[tid] = 0u;
  if (tid == 0) {
    sh.amb_n = 0;
    sh.zamb_n = 0;
    sh.sel_n = 0;
  }
  __syncthreads();

  // ---- phase 1: the superset counted; its keys into the bins above the bound; the range of its logits ----
  uint32_t keep = 0u;  // bit j: entry j is (still) part of the shortlist
  bool over = false;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    keep |= idx[j] >= 0 ? 1u << j : 0u;
    over |= idx[j] == -2;
  }
  const uint32_t bin_lb = okey_lb >> kHistShift;
  int rel[E];
  auto logit_range = [&](double& lo, double& hi) {  // over the kept entries, to all threads
    lo = INFINITY;
    hi = -INFINITY;
#pragma unroll
    for (int j = 0; j < E; ++j)
      if ((keep >> j) & 1u) {
        lo = fmin(lo, z[j]);
        hi = fmax(hi, z[j]);
      }
    auto lower = [](double a, double b) { return fmin(a, b); };
    auto upper = [](double a, double b) { return fmax(a, b); };
    lo = read_lane63(wave_prefix(lo, (double)INFINITY, lower));
    hi = read_lane63(wave_prefix(hi, (double)-INFINITY, upper));
    if (lane == 0) {
      sh.wave_lo[w] = lo;
      sh.wave_hi[w] = hi;
    }
    __syncthreads();
    lo = read_lane63(wave_prefix(lane < kSm1Waves ? sh.wave_lo[lane] : (double)INFINITY, (double)INFINITY, lower));
    hi = read_lane63(wave_prefix(lane < kSm1Waves ? sh.wave_hi[lane] : (double)-INFINITY, (double)-INFINITY, upper));
  };
#pragma unroll
  for (int j = 0; j < E; ++j) {
    rel[j] = (keep >> j) & 1u ? (int)min((okey[j] >> kHistShift) - bin_lb, (uint32_t)kSm1DropBins) : kSm1DropBins;
    if (answered && rel[j] < kSm1DropBins) atomicAdd(&sh.drop_hist[rel[j]], 1u);
  }
  {
    const int c = wave_sum(__popc(keep));
    const bool wave_over = __ballot(over) != 0ull;
    if (lane == 0) sh.wave_cnt[w] = wave_over ? -1 : c;
  }
  double z_lo, z_hi;
  logit_range(z_lo, z_hi);  // its barrier publishes the counts and the bins as well
  int n_s = 0;
  bool direct = !answered;  // uniform
  {
    const int c = lane < kSm1Waves ? sh.wave_cnt[lane] : 0;
    direct |= __ballot(c < 0) != 0ull;
    n_s = wave_sum(c);
    direct |= n_s < kprime;  // (at most kSm1SlotsTotal entries; the lists below hold the k' <= kSm1ListCap kept ones)
  }
  HIRE_TS(31);
  // logit bins: linear in the logit between the smallest and the largest, hence monotone
  double z_scale = z_hi > z_lo ? (double)(kSm1ZBins - 1) / (z_hi - z_lo) : 0.0;
  int zbin[E];
  auto count_logits = [&]() {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      zbin[j] = -1;
      if ((keep >> j) & 1u) {
        zbin[j] = min(max((int)((z[j] - z_lo) * z_scale), 0), kSm1ZBins - 1);
        atomicAdd(&sh.z_hist[zbin[j]], 1u);
      }
    }
  };

  // ---- phases 2 and 3: exactly the k' largest keys - the D smallest of the superset go ----
  uint64_t bal[E];  // the kept entries of every round, for the ordered output of the shortlist
  if (!direct) {
    const int D = n_s - kprime;
    int beta = -1, need_drop = 0;
    if (D > 0) {
      // every wave walks the 256 bins from the bottom: four bins per lane
      const uint4 hv = reinterpret_cast<const uint4*>(sh.drop_hist)[lane];
      const int c4[4] = {(int)hv.x, (int)hv.y, (int)hv.z, (int)hv.w};
      const int s4 = c4[0] + c4[1] + c4[2] + c4[3];
      const int incl = wave_scan_incl(s4);
      const uint64_t reach = __ballot(incl >= D);
      if (reach == 0ull) {  // uniform: the D-th smallest lies above the bins looked at
        direct = true;
      } else {
        const int L = __ffsll((long long)reach) - 1;
        int below = __builtin_amdgcn_readlane(incl - s4, L), cb = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = __builtin_amdgcn_readlane(c4[q], L);
          if (cb == 0 && below + c >= D) {
            beta = 4 * L + q;
            cb = c;
          }
          if (cb == 0) below += c;
        }
        need_drop = D - below;  // 1 .. cb of the bin's keys go
#pragma unroll
        for (int j = 0; j < E; ++j)
          if (rel[j] == beta) {
            const int a = atomicAdd(&sh.amb_n, 1);
            if (a < kSm1AmbCap) {
              sh.amb_key[a] = okey[j];
              sh.amb_idx[a] = idx[j];
            }
          }
      }
    }
    if (!direct) {
      count_logits();  // all of the superset; the entries that go are taken out again below
      __syncthreads();
      const int m = sh.amb_n;
      if (m > kSm1AmbCap) {  // uniform
        direct = true;
      } else {
#pragma unroll
        for (int j = 0; j < E; ++j) {
          bool goes = rel[j] < beta;
          if (rel[j] == beta) {
            int lower = 0;  // entries of the bin that go first: smaller key, or the same key at a higher index
            for (int u0 = 0; u0 < m; u0 += 8) {  // eight LDS reads in flight
              uint32_t ok[8];
              int32_t oi[8];
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                ok[q] = sh.amb_key[min(u0 + q, kSm1AmbCap - 1)];
                oi[q] = sh.amb_idx[min(u0 + q, kSm1AmbCap - 1)];
              }
#pragma unroll
              for (int q = 0; q < 8; ++q)
                lower += u0 + q < m && (ok[q] < okey[j] || (ok[q] == okey[j] && oi[q] > idx[j]));
            }
            goes = lower < need_drop;
          }
          if (goes) {
            keep &= ~(1u << j);
            atomicSub(&sh.z_hist[zbin[j]], 1u);
            zbin[j] = -1;
          }
        }
        int mine = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          bal[j] = __ballot((keep >> j) & 1u);
          mine += __popcll(bal[j]);
        }
        if (lane == 0) sh.wave_cnt[w] = mine;  // (read by everybody before the barrier above)
      }
    }
  }
  if (direct) {  // the shortlist from the keys themselves; the logit bins start again
    __syncthreads();
    if (tid < kSm1ZBins) sh.z_hist[tid] = 0u;
    sm1_shortlist_from_keys(keys, N, d, kprime, W, x, sh);
    keep = 0u;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int p = tid + j * kSm1Threads;
      if (p < kprime) {
        keep |= 1u << j;
        okey[j] = sh.l_okey[p];
        idx[j] = sh.l_idx[p];
        z[j] = sh.l_z[p];
      }
    }
    logit_range(z_lo, z_hi);  // its barrier: the list has been read by everybody (its memory is reused below)
    z_scale = z_hi > z_lo ? (double)(kSm1ZBins - 1) / (z_hi - z_lo) : 0.0;
    count_logits();
  }
  __syncthreads();
  HIRE_TS(32);
  if (tid == 0) {
    if (direct) atomicAdd(&mr.hdr->fallbacks, 1u);
    if (n_cand) n_cand[0] = kprime;
  }

  // ---- optional: the shortlist itself, ascending ----
  if (cand_idx != nullptr) {
    if (direct) {  // the list was the shortlist, in order
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if ((keep >> j) & 1u) cand_idx[tid + j * kSm1Threads] = idx[j];
    } else {
      int total;
      int at = sm1_wave_base(sh.wave_cnt, &total);
#pragma unroll
      for (int j = 0; j < E; ++j) {
        if ((keep >> j) & 1u) cand_idx[at + mask_prefix(bal[j])] = idx[j];
        at += __popcll(bal[j]);
      }
    }
  }

  // ---- phase 4: the bin of the k-th largest logit; every wave walks the bins from the top (lane l holds bins
  // 255 - 4 l .. 252 - 4 l) ----
  int beta, above;
  {
    const uint4 hv = reinterpret_cast<const uint4*>(sh.z_hist)[kWave - 1 - lane];
    const int c4[4] = {(int)hv.w, (int)hv.z, (int)hv.y, (int)hv.x};  // descending bins
    const int s4 = c4[0] + c4[1] + c4[2] + c4[3];
    const int incl = wave_scan_incl(s4);
    const uint64_t reach = __ballot(incl >= k);  // never empty: k' >= k entries were counted
    const int L = __ffsll((long long)reach) - 1;
    above = __builtin_amdgcn_readlane(incl - s4, L);
    beta = kSm1ZBins - 1 - 4 * L;
    bool hit = false;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = __builtin_amdgcn_readlane(c4[q], L);
      if (!hit && above + c >= k) {
        beta = kSm1ZBins - 1 - 4 * L - q;
        hit = true;
      }
      if (!hit) above += c;
    }
  }
  // the `above` entries of higher bins are selected; the bin's own entries are listed, the first k - above of them
  // in rank order follow
  unsigned long long* zamb_key = reinterpret_cast<unsigned long long*>(sh.l_z);
  int32_t* zamb_idx = sh.l_idx;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if (zbin[j] > beta) {
      const int a = atomicAdd(&sh.sel_n, 1);
      sh.sel_key[a] = order_key(z[j]);
      sh.sel_idx[a] = idx[j];
    } else if (zbin[j] == beta) {
      const int a = atomicAdd(&sh.zamb_n, 1);
      zamb_key[a] = order_key(z[j]);
      zamb_idx[a] = idx[j];
    }
  }
  __syncthreads();
  HIRE_TS(34);
  // ---- phase 5: rank order.  A higher bin means a strictly larger logit, so an entry of the higher bins is
  // ranked among those alone (sixteen threads share one entry, four comparisons each), and an entry of the k-th
  // logit's bin comes `above` places after its rank inside the bin ----
  auto put = [&](int rank, unsigned long long key, int32_t cls) {
    const double zt = key_value((uint64_t)key);
    top_idx[rank] = cls;
    if (top_logit) top_logit[rank] = (float)zt;
    sh.sel_z[rank] = zt;
  };
  {
    const int t = tid >> 4, part = tid & 15;
    const int last = max(above - 1, 0);
    const unsigned long long mk = sh.sel_key[min(t, last)];
    const int32_t mi = sh.sel_idx[min(t, last)];
    int ahead = 0;  // larger logit, or the same at a lower class
#pragma unroll
    for (int q = 0; q < kSm1MaxK / 16; ++q) {
      const int u = part * (kSm1MaxK / 16) + q;
      const unsigned long long ok = sh.sel_key[min(u, last)];
      const int32_t oi = sh.sel_idx[min(u, last)];
      ahead += u < above && (ok > mk || (ok == mk && oi < mi));
    }
    ahead += dpp_move<0x111, 0xF>(0, ahead);  // row_shr:1
    ahead += dpp_move<0x112, 0xF>(0, ahead);  // row_shr:2
    ahead += dpp_move<0x114, 0xF>(0, ahead);  // row_shr:4
    ahead += dpp_move<0x118, 0xF>(0, ahead);  // row_shr:8: lane 15 of the row holds the entry's rank
    if (part == 15 && t < above) put(ahead, mk, mi);
  }
  {
    const int m = sh.zamb_n, need = k - above;  // 1 <= need <= m
    for (int t = tid; t < m; t += kSm1Threads) {  // usually a handful of entries: the first wave only
      const unsigned long long mk = zamb_key[t];
      const int32_t mi = zamb_idx[t];
      int ahead = 0;
      for (int u0 = 0; u0 < m; u0 += 8) {  // eight LDS reads in flight
        unsigned long long ok[8];
        int32_t oi[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          ok[q] = zamb_key[min(u0 + q, m - 1)];
          oi[q] = zamb_idx[min(u0 + q, m - 1)];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) ahead += u0 + q < m && (ok[q] > mk || (ok[q] == mk && oi[q] < mi));
      }
      if (ahead < need) put(above + ahead, mk, mi);
    }
  }
  __syncthreads();
  HIRE_TS(35);
  // ---- eq. (2): softmax over the k selected, exp(z - zmax) / sum ----
  if (w == 0) {
    const double zmax = sh.sel_z[0];
    const double ez = lane < k ? exp(sh.sel_z[min(lane, k - 1)] - zmax) : 0.0;
    const double sum = wave_sum(ez);
    if (lane < k) top_prob[lane] = (float)(ez / sum);
  }
  HIRE_TS(36);
}

// Batches (launch_maxima_select): one workgroup per token takes the token's slots (keys and classes, no logits),
// drops the surplus keys exactly as k_sm1_final does and sets the bits of the k' that remain in the union bitmap;
// a token the maxima could not serve is selected from its keys directly.
struct MaxShared {
  SelShared sel;
  uint32_t drop_hist[kSm1DropBins];
  uint32_t amb_key[kSm1AmbCap];
  int32_t amb_idx[kSm1AmbCap];
  int wave_cnt[kSm1Waves];
  int amb_n;
};

__global__ __launch_bounds__(kSm1Threads) void k_max_resolve(const float* __restrict__ keys, int N, int kprime,
                                                             MultiRegion mr, const Sm1Entry* __restrict__ slots,
                                                             int n_slots, uint32_t* __restrict__ bitmap) {
  constexpr int E = kSm1SlotsPerThread;
  __shared__ MaxShared sh;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id(), b = (int)blockIdx.x;
  keys += (size_t)b * N;
  slots += (size_t)b * n_slots;
  uint32_t okey[E];
  int32_t idx[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int sl = w * (E * kWave) + j * kWave + lane;
    const uint2 v = *reinterpret_cast<const uint2*>(slots + min(sl, n_slots - 1));
    okey[j] = v.x;
    idx[j] = sl < n_slots ? (int32_t)v.y : -1;
  }
  const bool answered = mr.walk[4 * b + 1] != 0;
  const uint32_t okey_lb = (uint32_t)mr.walk[4 * b + 2];
  if (tid < kSm1DropBins) sh.drop_hist[tid] = 0u;
  if (tid == 0) sh.amb_n = 0;
  __syncthreads();
  uint32_t keep = 0u;
  bool over = false;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    keep |= idx[j] >= 0 ? 1u << j : 0u;
    over |= idx[j] == -2;
  }
  const uint32_t bin_lb = okey_lb >> kHistShift;
  int rel[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    rel[j] = (keep >> j) & 1u ? (int)min((okey[j] >> kHistShift) - bin_lb, (uint32_t)kSm1DropBins) : kSm1DropBins;
    if (answered && rel[j] < kSm1DropBins) atomicAdd(&sh.drop_hist[rel[j]], 1u);
  }
  {
    const int c = wave_sum(__popc(keep));
    const bool wave_over = __ballot(over) != 0ull;
    if (lane == 0) sh.wave_cnt[w] = wave_over ? -1 : c;
  }
  __syncthreads();
  int n_s = 0;
  bool direct = !answered;  // uniform
  {
    const int c = lane < kSm1Waves ? sh.wave_cnt[lane] : 0;
    direct |= __ballot(c < 0) != 0ull;
    n_s = wave_sum(c);
    direct |= n_s < kprime;
  }
  if (!direct) {
    const int D = n_s - kprime;
    int beta = -1, need_drop = 0;
    if (D > 0) {  // every wave walks the 256 bins from the bottom: four bins per lane
      const uint4 hv = reinterpret_cast<const uint4*>(sh.drop_hist)[lane];
      const int c4[4] = {(int)hv.x, (int)hv.y, (int)hv.z, (int)hv.w};
      const int s4 = c4[0] + c4[1] + c4[2] + c4[3];
      const int incl = wave_scan_incl(s4);
      const uint64_t reach = __ballot(incl >= D);
      if (reach == 0ull) {  // uniform: the D-th smallest lies above the bins looked at
        direct = true;
      } else {
        const int L = __ffsll((long long)reach) - 1;
        int below = __builtin_amdgcn_readlane(incl - s4, L), cb = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int c = __builtin_amdgcn_readlane(c4[q], L);
          if (cb == 0 && below + c >= D) {
            beta = 4 * L + q;
            cb = c;
          }
          if (cb == 0) below += c;
        }
        need_drop = D - below;
#pragma unroll
        for (int j = 0; j < E; ++j)
          if (rel[j] == beta) {
            const int a = atomicAdd(&sh.amb_n, 1);
            if (a < kSm1AmbCap) {
              sh.amb_key[a] = okey[j];
              sh.amb_idx[a] = idx[j];
            }
          }
      }
    }
    if (!direct) {
      __syncthreads();
      const int m = sh.amb_n;
      if (m > kSm1AmbCap) {  // uniform
        direct = true;
      } else {
#pragma unroll
        for (int j = 0; j < E; ++j) {
          bool goes = rel[j] < beta;
          if (rel[j] == beta) {
            int lower = 0;  // entries of the bin that go first: smaller key, or the same key at a higher index
            for (int u0 = 0; u0 < m; u0 += 8) {
              uint32_t ok[8];
              int32_t oi[8];
#pragma unroll
              for (int q = 0; q < 8; ++q) {
                ok[q] = sh.amb_key[min(u0 + q, kSm1AmbCap - 1)];
                oi[q] = sh.amb_idx[min(u0 + q, kSm1AmbCap - 1)];
              }
#pragma unroll
              for (int q = 0; q < 8; ++q)
                lower += u0 + q < m && (ok[q] < okey[j] || (ok[q] == okey[j] && oi[q] > idx[j]));
            }
            goes = lower < need_drop;
          }
          if (((keep >> j) & 1u) && !goes) atomicOr(&bitmap[idx[j] >> 5], 1u << (idx[j] & 31));
        }
      }
    }
  }
  if (direct) {
    __syncthreads();
    sm1_select_from_keys(keys, N, kprime, sh.sel,
                         [&](uint32_t, int i, int) { atomicOr(&bitmap[i >> 5], 1u << (i & 31)); });
    if (tid == 0) atomicAdd(&mr.hdr->fallbacks, 1u);
  }
}

bool softmax_b1_supported(int N, int d, int k, int kprime) {
  return N > kSm1Keys && N <= kSm1MaxRow && d % 8 == 0 && d <= 64 * 8 * kSm1XChunks && k <= kSm1MaxK &&
         kprime <= kSm1MaxShortlist;
}

// Whether the sequence is worth taking (it is exact either way): n_max maxima bound the k'-th key only if there are
// more than k' of them, and a workgroup of k_sm1_gather that runs out of slots sends the whole step down the slow
// direct selection.  With q = k' / n_max the bound leaves about -n_max ln(1 - q) keys (1.15 k' at q = 1/4, 1.4 k' at
// 1/2), spread over the workgroups like a Poisson variable; the sequence is taken when the chance that any of
// them exceeds its slots is below 1e-4 per step (2e-7 for the int4 scorer at 256000 classes, k' = 1024).
static bool sm1_worthwhile(int N, int kprime, int n_max, int kpt) {
  if (n_max <= kprime) return false;
  const int n_wg = sm1_workgroups(N, kpt), c = sm1_slots_per_wg(N, kpt);
  const double q = (double)kprime / n_max;
  const double mean = -(double)n_max * std::log1p(-q) / n_wg;  // superset entries per workgroup
  if (mean >= c) return false;
  // P(X > c) for X ~ Poisson(mean): terms c + 1, c + 2, ... in log space
  double tail = 0.0;
  for (int j = c + 1; j < c + 400; ++j) tail += std::exp(j * std::log(mean) - mean - std::lgamma(j + 1.0));
  return tail * n_wg < 1e-4;
}
bool softmax_b1_worthwhile(int N, int kprime, int n_max) { return sm1_worthwhile(N, kprime, n_max, kSm1KeysPerThread); }
bool maxima_select_worthwhile(int N, int kprime, int n_max) {
  return sm1_worthwhile(N, kprime, n_max, kSm1KeysPerThreadB);
}

size_t softmax_b1_slot_bytes(int N) {
  return (size_t)((N + kSm1Keys - 1) / kSm1Keys) * sm1_slots_per_wg(N) * sizeof(Sm1Entry);
}

hipError_t launch_softmax_b1(const float* keys, int N, int d, int sd, int k, int kprime, int n_max, const void* q4,
                             const uint16_t* W, const uint16_t* x, const HistRefs& hr, void* slots, int32_t* top_idx,
                             float* top_prob, float* top_logit, int32_t* cand_idx, int32_t* n_cand, hipStream_t s) {
  const MultiRegion mr = multi_of(hr, 1);
  if (mr.wgmax == nullptr || n_max > kWgMaxSlots || !softmax_b1_supported(N, d, k, kprime))
    return hipErrorInvalidValue;
  const int n_wg = (N + kSm1Keys - 1) / kSm1Keys;
  const uint32_t* smax_word = static_cast<const uint32_t*>(q4) + (size_t)N * (sd / 8);  // behind the codes
  Sm1Entry* sl = static_cast<Sm1Entry*>(slots);
  if (const hipError_t e = launch(k_sm1_gather<true, kSm1KeysPerThread>, dim3(n_wg), dim3(kSm1Threads), 0, s, keys, N, d, sd, kprime, n_max, smax_word, W,
                                  x, mr, sl, sm1_slots_per_wg(N));
      e != hipSuccess)
    return e;
  return launch(k_sm1_final, dim3(1), dim3(kSm1Threads), 0, s, keys, N, d, k, kprime, W, x, mr,
                static_cast<const Sm1Entry*>(sl), n_wg * sm1_slots_per_wg(N), top_idx, top_prob, top_logit, cand_idx, n_cand);
}

bool maxima_select_supported(int N) { return N > kSm1KeysPerThreadB * kSm1Threads && N <= kSm1MaxRow; }

size_t maxima_select_slot_bytes(int B, int N) {  // (the one-token sequence's share is the larger of the two)
  return (size_t)B * kSm1SlotsTotal * sizeof(Sm1Entry);
}

hipError_t launch_maxima_select(const float* keys, int B, int N, int sd, int kprime, int n_max, const void* q4,
                                const HistRefs& hr, void* slots, uint32_t* bitmap, hipStream_t s) {
  const MultiRegion mr = multi_of(hr, B);
  if (mr.wgmax == nullptr || n_max > kWgMaxSlots || !maxima_select_supported(N)) return hipErrorInvalidValue;
  const int n_wg = sm1_workgroups(N, kSm1KeysPerThreadB), per_wg = sm1_slots_per_wg(N, kSm1KeysPerThreadB);
  const uint32_t* smax_word = static_cast<const uint32_t*>(q4) + (size_t)N * (sd / 8);  // behind the codes
  Sm1Entry* sl = static_cast<Sm1Entry*>(slots);
  if (const hipError_t e = launch(k_sm1_gather<false, kSm1KeysPerThreadB>, dim3(n_wg, B), dim3(kSm1Threads), 0, s, keys, N, 8, sd, kprime,
                                  n_max, smax_word, static_cast<const uint16_t*>(nullptr),
                                  static_cast<const uint16_t*>(nullptr), mr, sl, per_wg);
      e != hipSuccess)
    return e;
  return launch(k_max_resolve, dim3(B), dim3(kSm1Threads), 0, s, keys, N, kprime, mr, static_cast<const Sm1Entry*>(sl),
                n_wg * per_wg, bitmap);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_softmax_b1(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
