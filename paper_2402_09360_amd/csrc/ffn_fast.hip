// Batch-1 HiRE-FFN step in four kernels (arXiv 2402.09360, Algorithm 1 + eq. (4)),
// laid out so that no stage runs on a single workgroup:
//
//   k_fast_score   int8 token quantisation (redone by every workgroup, 4 KB), int4 scorer, keys to memory,
//                  a fine histogram of the keys (integer atomics, 2^18 bins over the top key bits, so that
//                  few keys share a counter) and each workgroup's largest key
//   k_fast_gather  every workgroup walks the 8192 histogram bins below the largest key, ranks the handful
//                  of keys of the threshold bin and so knows the exact k'-th key; the ascending candidate
//                  list follows from ballot prefix counts, each workgroup materialises only its own share
//                  and computes the exact pre-activations of those rows; histogram of h the same way
//   k_fast_w2      the same selection on h (exact top-k), then partial sums of h_j v_j for the workgroup's
//                  (row group, column slice); clears the key histogram bins that this step touched
//   k_fast_reduce  adds the row groups in a fixed order; clears the touched bins of the h histogram
//
// A kernel boundary is the cheapest device-wide synchronisation on this machine (a spinning grid barrier
// costs several microseconds per round with 256 workgroups), hence separate kernels instead of one
// persistent kernel.  Selection work is duplicated in every workgroup instead of being serialised in one.
//
// The histograms must be all zero when a step starts.  Every step restores that state and the last kernel
// stamps a cookie into the workspace; a workspace without the cookie (first use, arbitrary contents) runs
// one step on a slower histogram-free route while the last kernel clears the histograms.
#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kFineShift = 14;                    // fine bin = order key >> 14 (sign, exponent, 9 mantissa bits)
constexpr int kFineBins = 1 << (32 - kFineShift); // 262144
constexpr int kWindow = 8192;                     // bins walked below the largest key
constexpr int kHistWords = kWindow + kFineBins;   // leading kWindow words stay zero: windows may reach below bin 0
constexpr unsigned long long kCookie = 0x48695245464e4f4bull;
constexpr int kShareCap = 64;                     // rows one workgroup gathers at most
constexpr int kAmbCap = 64;                       // keys of the threshold bin ranked directly
constexpr int kMaxSlots = 2048;                   // per-workgroup maxima written by the producing kernel

__device__ __forceinline__ uint32_t fine_bin(uint32_t okey) { return okey >> kFineShift; }
__device__ __forceinline__ uint32_t fine_bin(uint64_t okey) {
  return order_key((float)key_value(okey)) >> kFineShift;  // fp64 -> fp32 rounding is monotone
}
__device__ __forceinline__ uint32_t fine_bin_of_value(double v) { return order_key((float)v) >> kFineShift; }

// Layout of the fast-path region at the head of the workspace.
struct FastRegion {
  unsigned long long cookie;
  uint32_t pad[62];
  uint32_t max1[kMaxSlots];  // largest key bin of each scorer workgroup
  uint32_t max2[kMaxSlots];  // largest h bin of each gather workgroup
  uint32_t hist1[kHistWords];
  uint32_t hist2[kHistWords];
};

// ---------------------------------------------------------------------------------------------------
// Kernel 1: scorer.
constexpr int kRPW = 4;  // rows per wave and pass

__global__ __launch_bounds__(256) void k_fast_score_int4(const uint4* __restrict__ q4, const float* __restrict__ scale,
                                                         const uint32_t* __restrict__ x, int N, int d,
                                                         float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                         FastRegion* __restrict__ fr) {
  extern __shared__ uint32_t lds[];  // raw token, d/2 dwords of bf16 pairs; then d/4 dwords of int8 quads
  __shared__ float red[4];
  __shared__ uint32_t wmax[4];
  uint32_t* xraw = lds;
  uint32_t* xq = lds + d / 2;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cpr = d / 32;
  const int total_waves = (int)gridDim.x * 4;
  const int gw = (int)blockIdx.x * 4 + w;

  // token first (loads return in order, and the token is needed first), then the first rows' weights
  float amax = 0.0f;
  for (int i = tid; i < d / 2; i += 256) {
    const uint32_t u = x[i];
    xraw[i] = u;
    amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(u)), fabsf(bf16_hi(u))));
  }
  const int cl = min(lane, cpr - 1);
  uint4 pre[kRPW];
#pragma unroll
  for (int rr = 0; rr < kRPW; ++rr) pre[rr] = q4[(size_t)min(gw * kRPW + rr, N - 1) * cpr + cl];
  const bool hist_ok = fr->cookie == kCookie;

  amax = wave_max(amax);
  if (lane == 0) red[w] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sx = __fdiv_rn(amax, 127.0f);
  if (amax == 0.0f) sx = 1.0f;
  for (int i = tid; i < d / 4; i += 256) {
    const uint32_t a = xraw[2 * i], b = xraw[2 * i + 1];
    const float f[4] = {bf16_lo(a), bf16_hi(a), bf16_lo(b), bf16_hi(b)};
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float r = rintf(__fdiv_rn(f[e], sx));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      packed |= ((uint32_t)(int)r & 0xFFu) << (8 * e);
    }
    xq[i] = packed;
  }
  __syncthreads();

  const uint4* xq4 = reinterpret_cast<const uint4*>(xq);
  uint32_t my_max = 0;
  for (int g = gw; g * kRPW < N; g += total_waves) {
    const int j0 = g * kRPW;
    int acc[kRPW];
#pragma unroll
    for (int rr = 0; rr < kRPW; ++rr) acc[rr] = 0;
    for (int c = lane; c < cpr; c += kWave) {
      uint4 wv[kRPW];
      if (g == gw && c == lane) {
#pragma unroll
        for (int rr = 0; rr < kRPW; ++rr) wv[rr] = pre[rr];
      } else {
#pragma unroll
        for (int rr = 0; rr < kRPW; ++rr) wv[rr] = q4[(size_t)min(j0 + rr, N - 1) * cpr + c];
      }
      const uint4 xa = xq4[2 * c], xb = xq4[2 * c + 1];
      const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xb.x, (int)xb.y, (int)xb.z, (int)xb.w};
#pragma unroll
      for (int rr = 0; rr < kRPW; ++rr) {
        const uint32_t wd[4] = {wv[rr].x, wv[rr].y, wv[rr].z, wv[rr].w};
        int a = acc[rr];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          a = __builtin_amdgcn_sdot4((int)(wd[t] & 0xF0F0F0F0u), xd[2 * t], a, false);
          a = __builtin_amdgcn_sdot4((int)((wd[t] << 4) & 0xF0F0F0F0u), xd[2 * t + 1], a, false);
        }
        acc[rr] = a;
      }
    }
    // four row sums (wave-uniform results); lanes 0, 16, 32, 48 take rows j0 + 0, 1, 2, 3
    const int t0 = wave_sum(acc[0]), t1 = wave_sum(acc[1]), t2 = wave_sum(acc[2]), t3 = wave_sum(acc[3]);
    const int s = (lane & 32) ? ((lane & 16) ? t3 : t2) : ((lane & 16) ? t1 : t0);
    const int j = j0 + (lane >> 4);
    if ((lane & 15) == 0 && j < N) {
      const int sum = s >> 4;  // every partial is a multiple of 16
      float key = (float)sum * scale[j];
      key = key > 0.0f ? key : 0.0f;  // ReLU, and -0 -> +0
      keys[j] = key;
      if (acc_out) acc_out[j] = sum;
      const uint32_t ok = order_key(key);
      if (ok != 0x80000000u) {  // zeros are never counted
        if (hist_ok) atomicAdd(&fr->hist1[kWindow + fine_bin(ok)], 1u);
        my_max = max(my_max, fine_bin(ok));
      }
    }
  }
  my_max = wave_max(my_max);
  if (lane == 0) wmax[w] = my_max;
  __syncthreads();
  if (tid == 0) fr->max1[blockIdx.x] = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));
}

// ---------------------------------------------------------------------------------------------------
// Register-resident keys of a 1024-thread workgroup.  Wave w owns the index range [w*M, (w+1)*M); one load
// brings PER consecutive values per lane (16 bytes), so element (load e, lane l, part q) has index
// w*M + e*64*PER + l*PER + q and a wave's ballots for fixed (e, q) are slices of the index order.
template <typename K>
struct KeyIO;
template <>
struct KeyIO<uint32_t> {
  static constexpr int PER = 4;
  using V = float;
  static __device__ __forceinline__ void unpack(const uint4& u, uint32_t* out) {
    out[0] = order_key(__uint_as_float(u.x));
    out[1] = order_key(__uint_as_float(u.y));
    out[2] = order_key(__uint_as_float(u.z));
    out[3] = order_key(__uint_as_float(u.w));
  }
};
template <>
struct KeyIO<uint64_t> {
  static constexpr int PER = 2;
  using V = double;
  static __device__ __forceinline__ void unpack(const uint4& u, uint64_t* out) {
    out[0] = order_key(__longlong_as_double((long long)(((uint64_t)u.y << 32) | u.x)));
    out[1] = order_key(__longlong_as_double((long long)(((uint64_t)u.w << 32) | u.z)));
  }
};

template <typename K, int LOADS>
struct KeyRegs {
  static constexpr int PER = KeyIO<K>::PER;
  K r[LOADS][PER];
  int base, n, loads_used;  // loads_used <= LOADS: the wave's range may be shorter than LOADS loads
  // vals must be readable up to the next multiple of 16 bytes past n values
  __device__ __forceinline__ void load(const void* vals, int n_) {
    n = n_;
    const int span = 64 * PER;
    const int M = (((n + kSelWaves - 1) / kSelWaves) + span - 1) / span * span;
    base = wave_id() * M;
    loads_used = M / span;
    const int last_vec = (n - 1) / PER;
    uint4 raw[LOADS];
#pragma unroll
    for (int e = 0; e < LOADS; ++e) {
      const int vec = min((base + e * span) / PER + lane_id(), last_vec);
      raw[e] = reinterpret_cast<const uint4*>(vals)[vec];
    }
#pragma unroll
    for (int e = 0; e < LOADS; ++e) KeyIO<K>::unpack(raw[e], r[e]);
  }
  __device__ __forceinline__ int index(int e, int q) const { return base + e * 64 * PER + lane_id() * PER + q; }
  __device__ __forceinline__ bool valid(int e, int q) const { return e < loads_used && index(e, q) < n; }
};

// Walks the kWindow histogram bins at and below `top_bin` from the top and returns, to all threads, the bin
// holding the need-th largest counted key, the number of counted keys above that bin and the bin's count.
// found == false if the window holds fewer than `need` keys.
struct BinWalk {
  int bin, above, cnt;
  bool found;
};
__device__ __forceinline__ BinWalk walk_histogram(const uint32_t* __restrict__ hist, uint32_t top_bin, int need,
                                                  SelShared& sh) {
  const int tid = (int)threadIdx.x;
  const int hi = (int)(top_bin | 7u);          // last bin of top_bin's aligned group of eight
  const int start = hi - 8 * tid - 7;          // this thread's eight bins, ascending; a multiple of 8, may be < 0
  const uint4* p = reinterpret_cast<const uint4*>(hist + kWindow + start);
  const uint4 h0 = p[0], h1 = p[1];
  const int c[8] = {(int)h1.w, (int)h1.z, (int)h1.y, (int)h1.x, (int)h0.w, (int)h0.z, (int)h0.y, (int)h0.x};
  int s = 0;
#pragma unroll
  for (int q = 0; q < 8; ++q) s += c[q];
  const int incl = wg_scan_incl(s, sh);
  const int excl = incl - s;
  if (tid == kSelThreads - 1) sh.bc_bin = -1;  // "not found" unless a thread below owns the crossing
  __syncthreads();
  if (excl < need && need <= incl) {
    int run = excl;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (run < need && need <= run + c[q]) {
        sh.bc_bin = start + 7 - q;
        sh.bc_above = run;
        sh.bc_cnt = c[q];
      }
      run += c[q];
    }
  }
  __syncthreads();
  BinWalk r;
  r.bin = sh.bc_bin;
  r.found = r.bin >= 0;
  r.above = sh.bc_above;
  r.cnt = sh.bc_cnt;
  return r;
}

// The need_total-th largest of the workgroup's register-resident keys (returned to all threads).
// Histogram route: walk the bins, then rank the few keys of the threshold bin directly.  Any irregularity
// (no valid histogram, window too short, crowded bin) takes the histogram-free narrowing of select.h, which
// re-reads the values from memory with rolled loops to keep the code small.
template <typename K, int LOADS>
__device__ K fast_threshold(const KeyRegs<K, LOADS>& kr, const void* vals, int need_total,
                            const uint32_t* __restrict__ hist, uint32_t top_bin, bool hist_ok, SelShared& sh) {
  constexpr int PER = KeyRegs<K, LOADS>::PER;
  using V = typename KeyIO<K>::V;
  const int tid = (int)threadIdx.x;
  if (hist_ok) {
    const BinWalk bw = walk_histogram(hist, top_bin, need_total, sh);
    if (bw.found && bw.cnt <= kAmbCap) {
      K* list = reinterpret_cast<K*>(sh.hist);
      if (tid == 0) sh.list_n = 0;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < LOADS; ++e)
#pragma unroll
        for (int q = 0; q < PER; ++q)
          if (kr.valid(e, q) && (int)fine_bin(kr.r[e][q]) == bw.bin) {
            const int p = atomicAdd(&sh.list_n, 1);
            if (p < kAmbCap) list[p] = kr.r[e][q];
          }
      __syncthreads();
      const int m = min(sh.list_n, kAmbCap), need = need_total - bw.above;
      if (tid < m) {
        const K mine = list[tid];
        int cg = 0, cge = 0;
        for (int u = 0; u < m; ++u) {
          const K other = list[u];
          cg += other > mine;
          cge += other >= mine;
        }
        if (cg < need && need <= cge) sh.bc_key = (unsigned long long)mine;
      }
      __syncthreads();
      return (K)sh.bc_key;
    }
  }
  __syncthreads();
  const V* v = reinterpret_cast<const V*>(vals);
  const int n = kr.n;
  return wg_kth_largest<K>(
      [&](auto&& f) {
#pragma unroll 1
        for (int i = tid; i < n; i += kSelThreads) f(order_key(v[i]));
      },
      n, need_total, sh);
}

// Ordered emission: calls emit(i, out, key) for every selected key whose rank `out` in ascending index order
// lies in [out_lo, out_hi).  Selected = key > T, or key == T among the first (k - #greater) such keys.
template <typename K, int LOADS, typename Emit>
__device__ __forceinline__ void fast_emit(const KeyRegs<K, LOADS>& kr, K T, int k, int out_lo, int out_hi,
                                          int* tot_gt, int* tot_eq, Emit&& emit) {
  constexpr int PER = KeyRegs<K, LOADS>::PER;
  const int lane = lane_id(), w = wave_id();
  int cnt_gt = 0, cnt_eq = 0;
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const bool valid = kr.valid(e, q);
      cnt_gt += __popcll(__ballot(valid && kr.r[e][q] > T));
      cnt_eq += __popcll(__ballot(valid && kr.r[e][q] == T));
    }
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
  const int need_eq = k - all_gt;
  // this wave's outputs are [first, last); most waves lie outside the wanted window and stop here
  {
    const int first = run_gt + min(run_eq, need_eq);
    const int last = run_gt + cnt_gt + min(run_eq + cnt_eq, need_eq);
    if (last <= out_lo || first >= out_hi) return;
  }
#pragma unroll
  for (int e = 0; e < LOADS; ++e) {
    uint64_t mg[PER], me[PER];
    int ngt = 0, neq = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const bool valid = kr.valid(e, q);
      mg[q] = __ballot(valid && kr.r[e][q] > T);
      me[q] = __ballot(valid && kr.r[e][q] == T);
      ngt += __popcll(mg[q]);
      neq += __popcll(me[q]);
    }
    const int first = run_gt + min(run_eq, need_eq);
    const int last = run_gt + ngt + min(run_eq + neq, need_eq);
    if (last > out_lo && first < out_hi) {  // wave-uniform
      // counts of flagged elements in lower lanes, then walk this lane's own PER elements in index order
      int g_before = run_gt, e_before = run_eq;
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        g_before += mask_prefix(mg[q]);
        e_before += mask_prefix(me[q]);
      }
#pragma unroll
      for (int q = 0; q < PER; ++q) {
        const bool gt = (mg[q] >> lane) & 1, eq = (me[q] >> lane) & 1;
        const bool sel = gt || (eq && e_before < need_eq);
        const int out = g_before + min(e_before, need_eq);
        if (sel && out >= out_lo && out < out_hi) emit(kr.index(e, q), out, kr.r[e][q]);
        g_before += gt;
        e_before += eq;
      }
    }
    run_gt += ngt;
    run_eq += neq;
  }
}

// Largest of the first `count` per-workgroup maxima, to all threads.
__device__ __forceinline__ uint32_t reduce_max_slots(const uint32_t* __restrict__ slots, int count, SelShared& sh) {
  uint32_t m = 0;
  for (int i = (int)threadIdx.x; i < count; i += kSelThreads) m = max(m, slots[i]);
  m = wave_max(m);
  __syncthreads();
  if (lane_id() == 0) sh.wave_tot[wave_id()] = (int)m;
  __syncthreads();
  m = 0;
#pragma unroll
  for (int u = 0; u < kSelWaves; ++u) m = max(m, (uint32_t)sh.wave_tot[u]);
  __syncthreads();
  return m;
}

// ---------------------------------------------------------------------------------------------------
// Kernel 2: exact k'-th key, this workgroup's share of the candidate list, exact pre-activations.
struct FastGatherParams {
  const float* keys;          // [N], readable to the next multiple of 4
  int N, kprime, d, score_blocks;
  FastRegion* fr;
  const uint16_t* W1;         // [N, d] bf16
  const uint4* x;             // token, d/8 uint4
  int32_t* cand;              // [kprime] ascending candidate list (workspace or caller's buffer)
  int32_t* n_cand;            // optional
  double* h;                  // [kprime]
};

__global__ __launch_bounds__(kSelThreads) void k_fast_gather(FastGatherParams p) {
  __shared__ SelShared sh;
  __shared__ int tot_gt[kSelWaves], tot_eq[kSelWaves];
  __shared__ int my_rows[kShareCap];
  __shared__ uint32_t wmax[kSelWaves];
  extern __shared__ uint4 xs[];  // token as raw bf16, d/8 uint4
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int G = (int)gridDim.x, g = (int)blockIdx.x;
  HIRE_TS(10);
  KeyRegs<uint32_t, 4> kr;
  kr.load(p.keys, p.N);
  for (int i = tid; i < p.d / 8; i += kSelThreads) xs[i] = p.x[i];
  const bool hist_ok = p.fr->cookie == kCookie;
  const uint32_t top = reduce_max_slots(p.fr->max1, p.score_blocks, sh);
  HIRE_TS(11);
  const uint32_t T = fast_threshold(kr, p.keys, p.kprime, p.fr->hist1, top, hist_ok, sh);
  HIRE_TS(12);

  const int share = (p.kprime + G - 1) / G;
  const int lo = min(p.kprime, g * share), hi = min(p.kprime, lo + share);
  fast_emit(kr, T, p.kprime, lo, hi, tot_gt, tot_eq, [&](int i, int out, uint32_t) { my_rows[out - lo] = i; });
  if (g == 0 && tid == 0 && p.n_cand) *p.n_cand = p.kprime;
  __syncthreads();
  HIRE_TS(13);

  const int cpr = p.d / 8;
  uint32_t my_max = 0;
  for (int r = w; r < hi - lo; r += kSelWaves) {
    const int j = my_rows[r];
    const uint4* row = reinterpret_cast<const uint4*>(p.W1 + (size_t)j * p.d);
    double acc = 0.0;
    for (int c0 = 0; c0 < cpr; c0 += 4 * kWave) {
      uint4 wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) wv[u] = row[min(c0 + u * kWave + lane, cpr - 1)];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + u * kWave + lane;
        if (c < cpr) {
          const uint4 xv = xs[c];
          const uint32_t wd[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w}, xd[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acc += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
            acc += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
          }
        }
      }
    }
    double s = wave_sum(acc);
    if (lane == 0) {
      s = s > 0.0 ? s : 0.0;  // ReLU, and -0 -> +0
      p.h[lo + r] = s;
      p.cand[lo + r] = j;
      if (s > 0.0) {
        const uint32_t b = fine_bin_of_value(s);
        if (hist_ok) atomicAdd(&p.fr->hist2[kWindow + b], 1u);
        my_max = max(my_max, b);
      }
    }
  }
  my_max = wave_max(my_max);
  if (lane == 0) wmax[w] = my_max;
  __syncthreads();
  if (tid == 0) {
    uint32_t m = 0;
    for (int u = 0; u < kSelWaves; ++u) m = max(m, wmax[u]);
    p.fr->max2[g] = m;
  }
  HIRE_TS(14);
}

// ---------------------------------------------------------------------------------------------------
// Kernel 3: exact top-k of h, then this workgroup's partial of sum_j h_j v_j.
struct FastW2Params {
  const double* h;       // [n], readable to the next multiple of 2
  int n, k, d, gather_blocks;
  FastRegion* fr;
  const int32_t* cand;   // [n] unit index of each position
  const uint16_t* W2;    // [N, d] bf16
  int32_t* topk_idx;     // optional [k]
  float* topk_val;       // optional [k]
  float* partial;        // [row_groups, d]
  int row_groups, col_slices;
  const float* keys;     // [N]: the bins of these keys are cleared in hist1
  int N;
};

constexpr int kFastCols = 512;

template <int LOADS>
__global__ __launch_bounds__(kSelThreads) void k_fast_w2(FastW2Params p) {
  __shared__ SelShared sh;
  __shared__ int tot_gt[kSelWaves], tot_eq[kSelWaves];
  __shared__ int my_unit[kShareCap];
  __shared__ float my_h[kShareCap];
  __shared__ float red[kSelWaves][kFastCols];
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cs = (int)blockIdx.x % p.col_slices, rg = (int)blockIdx.x / p.col_slices;
  KeyRegs<uint64_t, LOADS> kr;
  kr.load(p.h, p.n);
  const bool hist_ok = p.fr->cookie == kCookie;
  if (hist_ok) {  // the key histogram has served its purpose: clear the bins this step's keys touched
    for (int i = (int)blockIdx.x * kSelThreads + tid; i < p.N; i += (int)gridDim.x * kSelThreads)
      p.fr->hist1[kWindow + fine_bin(order_key(p.keys[i]))] = 0u;
  }
  const uint32_t top = reduce_max_slots(p.fr->max2, p.gather_blocks, sh);
  const uint64_t T = fast_threshold(kr, p.h, p.k, p.fr->hist2, top, hist_ok, sh);
  const int share = (p.k + p.row_groups - 1) / p.row_groups;
  const int lo = min(p.k, rg * share), hi = min(p.k, lo + share);
  fast_emit(kr, T, p.k, lo, hi, tot_gt, tot_eq, [&](int i, int out, uint64_t key) {
    const int unit = p.cand[i];
    const float hv = (float)key_value(key);
    my_unit[out - lo] = unit;
    my_h[out - lo] = hv;
    if (cs == 0) {
      if (p.topk_idx) p.topk_idx[out] = unit;
      if (p.topk_val) p.topk_val[out] = hv;
    }
  });
  __syncthreads();

  const int col0 = cs * kFastCols + lane * 8;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (col0 < p.d) {
    for (int r = w; r < hi - lo; r += kSelWaves) {
      const uint4 wv = *reinterpret_cast<const uint4*>(p.W2 + (size_t)my_unit[r] * p.d + col0);
      const float c = my_h[r];
      const float wf[8] = {bf16_lo(wv.x), bf16_hi(wv.x), bf16_lo(wv.y), bf16_hi(wv.y),
                           bf16_lo(wv.z), bf16_hi(wv.z), bf16_lo(wv.w), bf16_hi(wv.w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(c, wf[q], acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) red[w][lane * 8 + q] = acc[q];
  __syncthreads();
  if (tid < kFastCols) {
    const int col = cs * kFastCols + tid;
    if (col < p.d) {
      float s = 0.0f;
#pragma unroll
      for (int u = 0; u < kSelWaves; ++u) s += red[u][tid];
      p.partial[(size_t)rg * p.d + col] = s;
    }
  }
}

// Kernel 4: y = sum over row groups; restores the all-zero state of the h histogram.  On a workspace without
// the cookie, workgroup 0 clears both histograms completely and then stamps the cookie (after a barrier, so
// all of its threads have taken their decision; a workgroup that starts late and already sees the cookie only
// stores zeros into bins that are zero).
__global__ __launch_bounds__(256) void k_fast_reduce(const float* __restrict__ partial, int row_groups, int d,
                                                     float* __restrict__ y, FastRegion* __restrict__ fr,
                                                     const double* __restrict__ h, int n) {
  const int gid = (int)(blockIdx.x * blockDim.x + threadIdx.x), gsz = (int)(gridDim.x * blockDim.x);
  const bool hist_ok = fr->cookie == kCookie;
  if (gid < d) {
    float s = 0.0f;
#pragma unroll 8
    for (int g = 0; g < row_groups; ++g) s += partial[(size_t)g * d + gid];
    y[gid] = s;
  }
  if (hist_ok) {
    for (int i = gid; i < n; i += gsz) fr->hist2[kWindow + fine_bin_of_value(h[i])] = 0u;
  } else if (blockIdx.x == 0) {
    uint4* z1 = reinterpret_cast<uint4*>(fr->hist1);
    uint4* z2 = reinterpret_cast<uint4*>(fr->hist2);
    for (int i = (int)threadIdx.x; i < kHistWords / 4; i += (int)blockDim.x) {
      z1[i] = make_uint4(0, 0, 0, 0);
      z2[i] = make_uint4(0, 0, 0, 0);
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) fr->cookie = kCookie;
  }
}

// ---------------------------------------------------------------------------------------------------
size_t ffn_fast_region_bytes() { return sizeof(FastRegion); }

void ffn_fast_shape(int d, int k, int* row_groups, int* col_slices) {
  const int cs = (d + kFastCols - 1) / kFastCols;
  int rg = 256 / cs;
  const int by_rows = (k + 3) / 4;
  if (rg > by_rows) rg = by_rows;
  if (rg < 1) rg = 1;
  *row_groups = rg;
  *col_slices = cs;
}

bool ffn_fast_supported(int B, int N, int d, int k, int kprime) {
  if (!(B == 1 && N <= kSelThreads * 16 && kprime <= kSelThreads * 16 && d % 32 == 0 && d <= 8192)) return false;
  int rg, cs;
  ffn_fast_shape(d, k, &rg, &cs);
  return (k + rg - 1) / rg <= kShareCap;
}

hipError_t launch_ffn_fast(const FfnFastArgs& a, hipStream_t s) {
  hipError_t e;
  FastRegion* fr = reinterpret_cast<FastRegion*>(a.fast_region);
  const int groups = (a.N + kRPW - 1) / kRPW;
  const int score_blocks = min((groups + 3) / 4, kMaxSlots);
  {
    const size_t lds = (size_t)a.d * 2 + (size_t)a.d;
    e = launch(k_fast_score_int4, dim3(score_blocks), dim3(256), lds, s, reinterpret_cast<const uint4*>(a.q4),
               a.q4_scale, reinterpret_cast<const uint32_t*>(a.x), a.N, a.d, a.keys, a.scorer_acc, fr);
    if (e != hipSuccess) return e;
  }
  int G = (a.kprime + 7) / 8;
  G = max(1, min(G, 256));
  {
    FastGatherParams p{};
    p.keys = a.keys; p.N = a.N; p.kprime = a.kprime; p.d = a.d; p.score_blocks = score_blocks;
    p.fr = fr; p.W1 = a.w1u; p.x = reinterpret_cast<const uint4*>(a.x);
    p.cand = a.cand; p.n_cand = a.n_cand; p.h = a.h;
    e = launch(k_fast_gather, dim3(G), dim3(kSelThreads), (size_t)a.d * 2, s, p);
    if (e != hipSuccess) return e;
  }
  int rg, cs;
  ffn_fast_shape(a.d, a.k, &rg, &cs);
  {
    FastW2Params p{};
    p.h = a.h; p.n = a.kprime; p.k = a.k; p.d = a.d; p.gather_blocks = G; p.fr = fr; p.cand = a.cand; p.W2 = a.w2u;
    p.topk_idx = a.topk_idx; p.topk_val = a.topk_val; p.partial = a.partial; p.row_groups = rg; p.col_slices = cs;
    p.keys = a.keys; p.N = a.N;
    if (a.kprime <= kSelThreads * 4)
      e = launch(k_fast_w2<2>, dim3(rg * cs), dim3(kSelThreads), 0, s, p);
    else
      e = launch(k_fast_w2<8>, dim3(rg * cs), dim3(kSelThreads), 0, s, p);
    if (e != hipSuccess) return e;
  }
  return launch(k_fast_reduce, dim3((a.d + 255) / 256), dim3(256), 0, s, a.partial, rg, a.d, a.y, fr, a.h, a.kprime);
}

}  // namespace hire
