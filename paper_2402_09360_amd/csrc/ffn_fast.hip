// Batch-1 HiRE-FFN step in four kernels (arXiv 2402.09360, Algorithm 1 + eq. (4)),
// laid out so that no stage runs on a single workgroup:
//
//   k_fast_score   int8 token quantisation (redone by every workgroup, 4 KB), int4 scorer, keys to memory,
//                  a fine histogram of the keys (integer atomics, 2^17 bins over the top key bits, so that
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
// The selecting workgroups have sixteen waves: a wave issues one instruction every few cycles whatever its
// neighbours do, so the per-key work is spread as thin as the workgroup size allows, and the fixed parts
// (scans, broadcasts) avoid LDS round trips per wave by reading all wave totals in one vector access.
//
// ReLU makes every key and every h non-negative, so their IEEE bit patterns already order like the numbers
// and are used as integer keys directly.
//
// The histograms must be all zero when a step starts.  Every step restores that state and the last kernel
// stamps a cookie into the workspace; a workspace without the cookie (first use, arbitrary contents) runs
// one step on a slower histogram-free route while the last kernel clears the histograms.
#include "hist.h"
#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kFT = 1024;                         // threads of the selecting workgroups
constexpr int kFW = kFT / kWave;                  // their waves
using FastShared = SelSharedT<kFT>;

constexpr int kFineShift = 14;                    // fine bin = bits >> 14 (exponent and 9 mantissa bits of an fp32)
constexpr int kFineBins = 1 << (31 - kFineShift); // 131072 bins for non-negative values
constexpr int kWindow = kHistWindow;               // bins walked below the largest key (walk_histogram in hist.h)
constexpr int kHistWords = kWindow + kFineBins;   // leading kWindow words stay zero: windows may reach below bin 0
constexpr unsigned long long kCookie = 0x48695245464e4f4bull;
constexpr int kShareCap = 64;                     // rows one workgroup handles at most
constexpr int kFastAmbCap = 64;                   // keys of the threshold bin ranked directly
constexpr int kMaxSlots = 2048;                   // per-workgroup maxima written by the producing kernel

__device__ __forceinline__ uint32_t fine_bin(uint32_t bits) { return bits >> kFineShift; }
__device__ __forceinline__ uint32_t fine_bin(uint64_t bits) {  // fp64 -> fp32 rounding is monotone
  return __float_as_uint((float)__longlong_as_double((long long)bits)) >> kFineShift;
}

// Layout of the fast-path region at the head of the workspace.
struct FastRegion {
  unsigned long long cookie;
  uint32_t fallbacks[2];     // steps whose k'-th key / k-th h were found without the histogram (statistics)
  uint32_t pad[60];
  uint32_t max1[kMaxSlots];  // largest key bin of each scorer workgroup
  uint32_t max2[kMaxSlots];  // largest h bin of each gather workgroup
  uint32_t hist1[kHistWords];
  uint32_t hist2[kHistWords];
};

// ---------------------------------------------------------------------------------------------------
// Kernel 1: scorer.
constexpr int kRPW = 4;     // rows per wave and pass
constexpr int kST = 1024;   // threads per scorer workgroup: one workgroup per CU, the token is quantised once per CU
constexpr int kSW = kST / kWave;

__global__ __launch_bounds__(kST) void k_fast_score_int4(const uint4* __restrict__ q4, const float* __restrict__ scale,
                                                         const uint32_t* __restrict__ x, int N, int d,
                                                         float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                         FastRegion* __restrict__ fr,
                                                         unsigned long long* __restrict__ clocks,
                                                         float* __restrict__ gkeys) {
  // gkeys != nullptr (group-sparse step, groups of eight adjacent units, eq. (6)): what is handed on, counted in
  // the histogram and maximised is the group activation gkeys[J] = sum_{l<8} |key[8J + l]| (fp32, unit order)
  // instead of the unit keys; a workgroup's 64 consecutive rows are eight whole groups.
  extern __shared__ uint32_t lds[];  // raw token, d/2 dwords of bf16 pairs; then d/4 dwords of int8 quads
  __shared__ float red[kSW];
  __shared__ float unit_keys[kSW * kRPW];
  if (clocks && threadIdx.x == 0) clocks[2 * blockIdx.x] = wall_clock64();
  __shared__ uint32_t wmax[kSW];
  uint32_t* xraw = lds;
  uint32_t* xq = lds + d / 2;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cpr = d / 32;
  const int total_waves = (int)gridDim.x * kSW;
  const int gw = (int)blockIdx.x * kSW + w;

  // token first (loads return in order, and the token is needed first), then the first rows' weights and
  // scales: all of these loads are in flight together
  const bool hist_ok = fr->cookie == kCookie;
  const uint4* x4 = reinterpret_cast<const uint4*>(x);
  const int xvecs = d / 8;
  const uint4 xv0 = x4[min(tid, xvecs - 1)];
  const int cl = min(lane, cpr - 1);
  uint4 pre[kRPW];
#pragma unroll
  for (int rr = 0; rr < kRPW; ++rr) pre[rr] = load_streaming(&q4[(size_t)min(gw * kRPW + rr, N - 1) * cpr + cl]);
  const float pre_scale = scale[min(gw * kRPW + (lane >> 4), N - 1)];
  float amax = 0.0f;
  for (int i = tid; i < xvecs; i += kST) {
    const uint4 u = i == tid ? xv0 : x4[i];
    reinterpret_cast<uint4*>(xraw)[i] = u;
    const uint32_t ud[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(ud[q])), fabsf(bf16_hi(ud[q]))));
  }
  amax = wave_max(amax);
  if (lane == 0) red[w] = amax;
  __syncthreads();
  amax = wave_max(lane < kSW ? red[lane] : 0.0f);
  float sx = __fdiv_rn(amax, 127.0f);
  if (amax == 0.0f) sx = 1.0f;
  for (int i = tid; i < d / 4; i += kST) {
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
        for (int rr = 0; rr < kRPW; ++rr) wv[rr] = load_streaming(&q4[(size_t)min(j0 + rr, N - 1) * cpr + c]);
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
      float key = (float)sum * (g == gw ? pre_scale : scale[j]);
      key = key > 0.0f ? key : 0.0f;  // ReLU, and -0 -> +0
      if (acc_out) acc_out[j] = sum;
      if (gkeys != nullptr) {
        unit_keys[w * kRPW + (lane >> 4)] = key;  // one pass per workgroup here (N <= 64 * gridDim.x)
      } else {
        keys[j] = key;
        const uint32_t bits = __float_as_uint(key);
        if (bits != 0u) {  // zeros are never counted
          if (hist_ok) atomicAdd(&fr->hist1[kWindow + fine_bin(bits)], 1u);
          my_max = max(my_max, fine_bin(bits));
        }
      }
    }
  }
  if (gkeys != nullptr) {
    __syncthreads();
    const int J = (int)blockIdx.x * (kSW * kRPW / 8) + tid;
    if (tid < kSW * kRPW / 8 && J * 8 < N) {
      float sum = 0.0f;
#pragma unroll
      for (int l = 0; l < 8; ++l) sum += fabsf(unit_keys[tid * 8 + l]);
      gkeys[J] = sum;
      const uint32_t bits = __float_as_uint(sum);
      if (bits != 0u) {
        if (hist_ok) atomicAdd(&fr->hist1[kWindow + fine_bin(bits)], 1u);
        my_max = max(my_max, fine_bin(bits));
      }
    }
  }
  my_max = wave_max(my_max);
  if (lane == 0) wmax[w] = my_max;
  __syncthreads();
  if (w == 0) {
    const uint32_t m = wave_max(lane < kSW ? wmax[lane] : 0u);
    if (lane == 0) {
      fr->max1[blockIdx.x] = m;
      if (clocks) clocks[2 * blockIdx.x + 1] = wall_clock64();
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Register-resident non-negative keys of a kFT-thread workgroup, as raw IEEE bits.  Wave w owns the index
// range [w*M, (w+1)*M); one load brings PER consecutive values per lane (16 bytes), so element (load e, lane
// l, part q) has index w*M + e*64*PER + l*PER + q and a wave's ballots for fixed (e, q) are slices of the
// index order.
template <typename K>
struct KeyIO;
template <>
struct KeyIO<uint32_t> {
  static constexpr int PER = 4;
  using V = float;
  static __device__ __forceinline__ void unpack(const uint4& u, uint32_t* out) {
    out[0] = u.x;
    out[1] = u.y;
    out[2] = u.z;
    out[3] = u.w;
  }
  static __device__ __forceinline__ uint32_t to_order_key(uint32_t bits) { return bits | 0x80000000u; }
  static __device__ __forceinline__ uint32_t from_order_key(uint32_t key) { return key & 0x7FFFFFFFu; }
};
template <>
struct KeyIO<uint64_t> {
  static constexpr int PER = 2;
  using V = double;
  static __device__ __forceinline__ void unpack(const uint4& u, uint64_t* out) {
    out[0] = ((uint64_t)u.y << 32) | u.x;
    out[1] = ((uint64_t)u.w << 32) | u.z;
  }
  static __device__ __forceinline__ uint64_t to_order_key(uint64_t bits) { return bits | 0x8000000000000000ull; }
  static __device__ __forceinline__ uint64_t from_order_key(uint64_t key) { return key & 0x7FFFFFFFFFFFFFFFull; }
};

template <typename K, int LOADS>
struct KeyRegs {
  static constexpr int PER = KeyIO<K>::PER;
  K r[LOADS][PER];
  uint4 raw[LOADS];
  int base, n, loads_used;  // loads_used <= LOADS: the wave's range may be shorter than LOADS loads
  // Starts the loads; vals must be readable up to the next multiple of 16 bytes past n values.
  __device__ __forceinline__ void issue(const void* vals, int n_) {
    n = n_;
    const int span = 64 * PER;
    const int M = (((n + kFW - 1) / kFW) + span - 1) / span * span;
    base = wave_id() * M;
    loads_used = M / span;
    const int last_vec = (n - 1) / PER;
#pragma unroll
    for (int e = 0; e < LOADS; ++e) {
      const int vec = min((base + e * span) / PER + lane_id(), last_vec);
      raw[e] = reinterpret_cast<const uint4*>(vals)[vec];
    }
  }
  __device__ __forceinline__ void finish() {
#pragma unroll
    for (int e = 0; e < LOADS; ++e) KeyIO<K>::unpack(raw[e], r[e]);
  }
  __device__ __forceinline__ int index(int e, int q) const { return base + e * 64 * PER + lane_id() * PER + q; }
  __device__ __forceinline__ bool valid(int e, int q) const { return e < loads_used && index(e, q) < n; }
};

// What the selection needs to know about the threshold: selected = key >= t_ge, plus the first need_eq keys
// equal to t_eq in index order (need_eq == 0 when every key equal to the k-th is taken).
template <typename K>
struct Threshold {
  K t_ge, t_eq;
  int need_eq;
};


// The need_total-th largest of the workgroup's register-resident keys.  Histogram route: walk the bins, then
// rank the few keys of the threshold bin directly.  Any irregularity (no valid histogram, window too short,
// crowded bin) takes the histogram-free narrowing of select.h, which re-reads the values from memory with
// rolled loops to keep the code small.
template <typename K, int LOADS>
__device__ Threshold<K> fast_threshold(const KeyRegs<K, LOADS>& kr, const void* vals, int need_total,
                                       const uint32_t* __restrict__ hist, uint32_t top_bin, bool hist_ok,
                                       FastShared& sh, uint32_t* fallback_counter) {
  constexpr int PER = KeyRegs<K, LOADS>::PER;
  const int tid = (int)threadIdx.x;
  Threshold<K> th;
  if (hist_ok) {
    if (tid == 0) sh.list_n = 0;  // ordered before its use by the barriers of the walk
    const BinWalk bw = walk_histogram<kFT>(hist + kWindow, top_bin, need_total, sh);
    HIRE_TS(20);
    if (bw.found && bw.cnt <= kFastAmbCap) {
      K* list = reinterpret_cast<K*>(sh.hist);
#pragma unroll
      for (int e = 0; e < LOADS; ++e)
#pragma unroll
        for (int q = 0; q < PER; ++q)
          if (kr.valid(e, q) && (int)fine_bin(kr.r[e][q]) == bw.bin) {
            const int p = atomicAdd(&sh.list_n, 1);
            if (p < kFastAmbCap) list[p] = kr.r[e][q];
          }
      __syncthreads();
      HIRE_TS(21);
      const int m = min(sh.list_n, kFastAmbCap), need = need_total - bw.above;
      if (tid < kWave) {  // wave 0 ranks the at most 64 keys among themselves, one key per lane
        const K mine = tid < m ? list[tid] : (K)0;
        int cg = 0, cge = 0;
        for (int u = 0; u < m; ++u) {
          const K other = read_lane(mine, u);
          cg += other > mine;
          cge += other >= mine;
        }
        if (tid < m && cg < need && need <= cge) {  // equal keys write the same values
          sh.bc_key = (unsigned long long)mine;
          sh.bc_cnt = need - cg == cge - cg ? 0 : need - cg;  // 0: every key equal to the threshold is taken
        }
      }
      __syncthreads();
      th.t_eq = (K)sh.bc_key;
      th.need_eq = sh.bc_cnt;
      th.t_ge = th.need_eq == 0 ? th.t_eq : th.t_eq + 1;
      return th;
    }
  }
  __syncthreads();
  if (fallback_counter && blockIdx.x == 0 && tid == 0) atomicAdd(fallback_counter, 1u);
  using V = typename KeyIO<K>::V;
  const V* v = reinterpret_cast<const V*>(vals);
  const int n = kr.n;
  const K key = wg_kth_largest<K>(
      [&](auto&& f) {
#pragma unroll 1
        for (int i = tid; i < n; i += kFT) {
          K bits;
          __builtin_memcpy(&bits, &v[i], sizeof(K));
          f(KeyIO<K>::to_order_key(bits));
        }
      },
      n, need_total, sh);
  th.t_eq = KeyIO<K>::from_order_key(key);
  th.t_ge = th.t_eq + 1;
  th.need_eq = -1;  // unknown: counted by the emission
  return th;
}

// Ordered emission: calls emit(i, out, key) for every selected key whose rank `out` in ascending index order
// lies in [out_lo, out_hi).
template <typename K, int LOADS, typename Emit>
__device__ __forceinline__ void fast_emit(const KeyRegs<K, LOADS>& kr, Threshold<K> th, int k, int out_lo, int out_hi,
                                          int* tot_gt, int* tot_eq, Emit&& emit) {
  constexpr int PER = KeyRegs<K, LOADS>::PER;
  const int lane = lane_id(), w = __builtin_amdgcn_readfirstlane(wave_id());
  const bool ties = th.need_eq != 0;  // uniform
  int cnt_gt = 0, cnt_eq = 0;
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const bool valid = kr.valid(e, q);
      cnt_gt += __popcll(__ballot(valid && kr.r[e][q] >= th.t_ge));
      if (ties) cnt_eq += __popcll(__ballot(valid && kr.r[e][q] == th.t_eq));
    }
  HIRE_TS(22);
  __syncthreads();
  if (lane == 0) {
    tot_gt[w] = cnt_gt;
    tot_eq[w] = cnt_eq;
  }
  __syncthreads();
  HIRE_TS(23);
  const int pg = wave_scan_incl(lane < kFW ? tot_gt[lane] : 0), pe = wave_scan_incl(lane < kFW ? tot_eq[lane] : 0);
  int run_gt = w > 0 ? __builtin_amdgcn_readlane(pg, w - 1) : 0;
  int run_eq = w > 0 ? __builtin_amdgcn_readlane(pe, w - 1) : 0;
  const int all_gt = __builtin_amdgcn_readlane(pg, kFW - 1);
  const int need_eq = ties ? k - all_gt : 0;
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
      mg[q] = __ballot(valid && kr.r[e][q] >= th.t_ge);
      me[q] = ties ? __ballot(valid && kr.r[e][q] == th.t_eq) : 0ull;
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
  double* h;                  // [kprime << gs]
  // gs = 3 (group-sparse step): keys are group activations, N and kprime count groups of eight units, cand lists
  // groups; h holds the eight units of every candidate group and hg[kprime] their exact group activations
  // sum_l |h|, which are what is counted in the histogram and ranked by the next kernel.  gs = 0: units.
  int gs;
  double* hg;
  // CommonPath (eq. (7)): workgroups sparse_blocks .. gridDim.x - 1 skip the selection and compute the
  // activations of the m1 dense units, one row of Wd per wave: hd[r] = relu(<Wd[r, :], x>).  m1 = 0: none.
  int sparse_blocks;
  const uint16_t* Wd;
  int m1;
  double* hd;
};

constexpr int kGatherRows = 1;  // rows a wave has in flight

__global__ __launch_bounds__(kFT) void k_fast_gather(FastGatherParams p) {
  __shared__ FastShared sh;
  __shared__ int tot_gt[kFW], tot_eq[kFW];
  __shared__ int my_rows[kShareCap];
  __shared__ uint32_t wmax[kFW];
  __shared__ double unit_h[kShareCap];  // group-sparse: the units' activations of this workgroup's (<= 8) groups
  extern __shared__ float xtok[];  // token as fp32, d floats
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int G = p.sparse_blocks, g = (int)blockIdx.x;
  if (g >= G) {  // dense common-path units: token into LDS, then one row per wave
    const int xv = p.d / 8;
    for (int i = tid; i < xv; i += kFT) {
      const uint4 u = p.x[i];
      const float f[8] = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y),
                          bf16_lo(u.z), bf16_hi(u.z), bf16_lo(u.w), bf16_hi(u.w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) xtok[8 * i + q] = f[q];
    }
    __syncthreads();
    const int r = (g - G) * kFW + w;
    if (r >= p.m1) return;
    const uint4* row = reinterpret_cast<const uint4*>(p.Wd + (size_t)r * p.d);
    double acc = 0.0;
    for (int c0 = 0; c0 < xv; c0 += 4 * kWave) {
      uint4 wv[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) wv[v] = load_streaming(&row[min(c0 + v * kWave + lane, xv - 1)]);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = c0 + v * kWave + lane;
        if (c < xv) {
          const float4 xa = reinterpret_cast<const float4*>(xtok)[2 * c], xb = reinterpret_cast<const float4*>(xtok)[2 * c + 1];
          const float xf[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
          const uint32_t wd[4] = {wv[v].x, wv[v].y, wv[v].z, wv[v].w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acc += (double)(bf16_lo(wd[q]) * xf[2 * q]);
            acc += (double)(bf16_hi(wd[q]) * xf[2 * q + 1]);
          }
        }
      }
    }
    double sd = wave_sum(acc);
    sd = sd > 0.0 ? sd : 0.0;
    if (lane == 0) p.hd[r] = sd;
    return;
  }
  HIRE_TS(10);
  // every load that does not depend on another is started here, before the first wait
  const bool hist_ok = p.fr->cookie == kCookie;
  KeyRegs<uint32_t, 4> kr;
  kr.issue(p.keys, p.N);
  const int xvecs = p.d / 8;
  const uint4 xv0 = p.x[min(tid, xvecs - 1)];
  const uint32_t m = p.fr->max1[min(tid, p.score_blocks - 1)];  // score_blocks <= kFT
  for (int i = tid; i < xvecs; i += kFT) {
    const uint4 u = i == tid ? xv0 : p.x[i];
    const float f[8] = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y),
                        bf16_lo(u.z), bf16_hi(u.z), bf16_lo(u.w), bf16_hi(u.w)};
#pragma unroll
    for (int q = 0; q < 8; ++q) xtok[8 * i + q] = f[q];
  }
  HIRE_TS(15);
  const uint32_t top = wg_max_u32(m, sh);
  HIRE_TS(16);
  kr.finish();
  HIRE_TS(11);
  const Threshold<uint32_t> th = fast_threshold(kr, p.keys, p.kprime, p.fr->hist1, top, hist_ok, sh, &p.fr->fallbacks[0]);
  HIRE_TS(12);

  const int share = (p.kprime + G - 1) / G;
  const int lo = min(p.kprime, g * share), hi = min(p.kprime, lo + share);
  fast_emit(kr, th, p.kprime, lo, hi, tot_gt, tot_eq, [&](int i, int out, uint32_t) { my_rows[out - lo] = i; });
  if (g == 0 && tid == 0 && p.n_cand) *p.n_cand = p.kprime;
  __syncthreads();
  HIRE_TS(13);

  const int gs = p.gs, gmask = (1 << gs) - 1;
  const int cpr = p.d / 8, cnt = (hi - lo) << gs;  // rows of this workgroup
  uint32_t my_max = 0;
  for (int r0 = w; r0 < cnt; r0 += kFW * kGatherRows) {
    const uint4* row[kGatherRows];
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u) {
      const int r = min(r0 + kFW * u, cnt - 1);
      row[u] = reinterpret_cast<const uint4*>(p.W1 + (((size_t)my_rows[r >> gs] << gs) + (r & gmask)) * p.d);
    }
    double acc[kGatherRows];
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u) acc[u] = 0.0;
    for (int c0 = 0; c0 < cpr; c0 += 4 * kWave) {
      uint4 wv[kGatherRows][4];
#pragma unroll
      for (int u = 0; u < kGatherRows; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) wv[u][v] = load_streaming(&row[u][min(c0 + v * kWave + lane, cpr - 1)]);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = c0 + v * kWave + lane;
        if (c < cpr) {
          const float4 xa = reinterpret_cast<const float4*>(xtok)[2 * c], xb = reinterpret_cast<const float4*>(xtok)[2 * c + 1];
          const float xf[8] = {xa.x, xa.y, xa.z, xa.w, xb.x, xb.y, xb.z, xb.w};
#pragma unroll
          for (int u = 0; u < kGatherRows; ++u) {
            const uint32_t wd[4] = {wv[u][v].x, wv[u][v].y, wv[u][v].z, wv[u][v].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              acc[u] += (double)(bf16_lo(wd[q]) * xf[2 * q]);
              acc[u] += (double)(bf16_hi(wd[q]) * xf[2 * q + 1]);
            }
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u) {
      double s = wave_sum(acc[u]);
      const int r = r0 + kFW * u;
      if (lane == 0 && r < cnt) {
        s = s > 0.0 ? s : 0.0;  // ReLU, and -0 -> +0
        p.h[((size_t)lo << gs) + r] = s;
        if ((r & gmask) == 0) p.cand[lo + (r >> gs)] = my_rows[r >> gs];
        if (gs != 0) {
          unit_h[r] = s;
        } else if (s > 0.0) {
          const uint32_t b = fine_bin((uint64_t)__double_as_longlong(s));
          if (hist_ok) atomicAdd(&p.fr->hist2[kWindow + b], 1u);
          my_max = max(my_max, b);
        }
      }
    }
  }
  if (gs != 0) {  // exact group activations, units added in order
    __syncthreads();
    if (tid < hi - lo) {
      double e = 0.0;
      for (int l = 0; l <= gmask; ++l) e += fabs(unit_h[(tid << gs) + l]);
      p.hg[lo + tid] = e;
      if (e > 0.0) {
        const uint32_t b = fine_bin((uint64_t)__double_as_longlong(e));
        if (hist_ok) atomicAdd(&p.fr->hist2[kWindow + b], 1u);
        my_max = max(my_max, b);
      }
    }
  }
  my_max = wave_max(my_max);
  if (lane == 0) wmax[w] = my_max;
  __syncthreads();
  if (tid == 0) {
    uint32_t mm = 0;
    for (int u = 0; u < kFW; ++u) mm = max(mm, wmax[u]);
    p.fr->max2[g] = mm;
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
  // gs = 3 (group-sparse step): h holds exact group activations, n and k count groups, cand lists groups, keys /
  // N are the group keys; unit_h[n << gs] holds the units' activations (the second layer's coefficients) and
  // topk_val receives the eight of every selected group.  gs = 0: units, unit_h unused.
  int gs;
  const double* unit_h;
  // CommonPath (eq. (7)): row groups row_groups .. row_groups + dense_groups - 1 (times the column slices) add
  // the m1 dense units, 64 rows each: partial += fl32(hd[r]) * W2d[r, :].  dense_groups = 0: none.
  int dense_groups;
  const uint16_t* W2d;
  const double* hd;
  int m1;
};

constexpr int kFastCols = 512;
constexpr int kW2Rows = 4;  // rows a wave has in flight

__global__ __launch_bounds__(kFT) void k_fast_w2(FastW2Params p) {
  __shared__ FastShared sh;
  __shared__ int tot_gt[kFW], tot_eq[kFW];
  __shared__ int my_unit[kShareCap];
  __shared__ int my_pos[kShareCap];
  __shared__ float my_h[kShareCap * 8];
  __shared__ float red[kFW][kFastCols];
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cs = (int)blockIdx.x % p.col_slices, rg = (int)blockIdx.x / p.col_slices;
  const bool dense = rg >= p.row_groups;  // uniform over the workgroup
  int gs = p.gs, cnt;
  const uint16_t* W2 = p.W2;
  if (dense) {  // no selection: this group's 64 (or fewer) dense rows with their activations as coefficients
    const int r0 = (rg - p.row_groups) * kShareCap;
    cnt = min(kShareCap, p.m1 - r0);
    if (tid < cnt) {
      my_unit[tid] = r0 + tid;
      my_h[tid] = (float)p.hd[r0 + tid];
    }
    gs = 0;
    W2 = p.W2d;
    __syncthreads();
  } else {
  const bool hist_ok = p.fr->cookie == kCookie;
  KeyRegs<uint64_t, 2> kr;
  kr.issue(p.h, p.n);
  const uint32_t m0 = p.fr->max2[min(tid, p.gather_blocks - 1)];  // gather_blocks <= 256
  const int gid = (int)blockIdx.x * kFT + tid, gsz = p.row_groups * p.col_slices * kFT;  // the selecting workgroups
  const float key0 = p.keys[min(gid, p.N - 1)];
  if (hist_ok) {  // the key histogram has served its purpose: clear the bins this step's keys touched
    if (gid < p.N) p.fr->hist1[kWindow + fine_bin(__float_as_uint(key0))] = 0u;
    for (int i = gid + gsz; i < p.N; i += gsz) p.fr->hist1[kWindow + fine_bin(__float_as_uint(p.keys[i]))] = 0u;
  }
  const uint32_t top = wg_max_u32(m0, sh);
  kr.finish();
  const Threshold<uint64_t> th = fast_threshold(kr, p.h, p.k, p.fr->hist2, top, hist_ok, sh, &p.fr->fallbacks[1]);
  const int share = (p.k + p.row_groups - 1) / p.row_groups;
  const int lo = min(p.k, rg * share), hi = min(p.k, lo + share);
  fast_emit(kr, th, p.k, lo, hi, tot_gt, tot_eq, [&](int i, int out, uint64_t bits) {
    const int unit = p.cand[i];
    const float hv = (float)__longlong_as_double((long long)bits);
    my_unit[out - lo] = unit;
    my_pos[out - lo] = i;
    if (p.gs == 0) my_h[out - lo] = hv;
    if (cs == 0) {
      if (p.topk_idx) p.topk_idx[out] = unit;
      if (p.topk_val && p.gs == 0) p.topk_val[out] = hv;
    }
  });
  __syncthreads();
  cnt = (hi - lo) << gs;  // rows of this workgroup
  if (gs != 0) {  // the coefficients of the selected groups' units
    const int gmask = (1 << gs) - 1;
    for (int r = tid; r < cnt; r += kFT) {
      const float hv = (float)p.unit_h[((size_t)my_pos[r >> gs] << gs) + (r & gmask)];
      my_h[r] = hv;
      if (cs == 0 && p.topk_val) p.topk_val[((size_t)lo << gs) + r] = hv;
    }
    __syncthreads();
  }
  }  // selecting workgroups

  const int gmask = (1 << gs) - 1;
  const int col0 = min(cs * kFastCols + lane * 8, p.d - 8);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int r0 = w; r0 < cnt; r0 += kFW * kW2Rows) {
    uint4 wv[kW2Rows];
#pragma unroll
    for (int u = 0; u < kW2Rows; ++u) {
      const int r = min(r0 + kFW * u, cnt - 1);
      wv[u] = load_streaming(reinterpret_cast<const uint4*>(
          W2 + (((size_t)my_unit[r >> gs] << gs) + (r & gmask)) * p.d + col0));
    }
#pragma unroll
    for (int u = 0; u < kW2Rows; ++u) {
      const int r = r0 + kFW * u;
      const float c = r < cnt ? my_h[r] : 0.0f;
      const float wf[8] = {bf16_lo(wv[u].x), bf16_hi(wv[u].x), bf16_lo(wv[u].y), bf16_hi(wv[u].y),
                           bf16_lo(wv[u].z), bf16_hi(wv[u].z), bf16_lo(wv[u].w), bf16_hi(wv[u].w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(c, wf[q], acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) red[w][lane * 8 + q] = acc[q];
  __syncthreads();
  for (int c = tid; c < kFastCols; c += kFT) {
    const int col = cs * kFastCols + c;
    if (col < p.d) {
      float t = 0.0f;
#pragma unroll
      for (int u = 0; u < kFW; ++u) t += red[u][c];
      p.partial[(size_t)rg * p.d + col] = t;
    }
  }
}

// Kernel 4: y = sum over row groups; restores the all-zero state of the h histogram.  On a workspace without
// the cookie, workgroup 0 clears both histograms completely and then stamps the cookie (after a barrier, so
// all of its threads have taken their decision; a workgroup that starts late and already sees the cookie only
// stores zeros into bins that are zero).
constexpr int kRedCols = 64;  // columns per workgroup of the final reduction

__global__ __launch_bounds__(256) void k_fast_reduce(const float* __restrict__ partial, int row_groups, int d,
                                                     float* __restrict__ y, FastRegion* __restrict__ fr,
                                                     const double* __restrict__ h, int n) {
  __shared__ float part[4][kRedCols];
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int gid = (int)(blockIdx.x * blockDim.x + threadIdx.x), gsz = (int)(gridDim.x * blockDim.x);
  const bool hist_ok = fr->cookie == kCookie;
  const double h0 = h[min(gid, n - 1)];
  // wave w adds row groups w, w+4, ... for this workgroup's 64 columns, sixteen loads in flight at a time
  const int col = (int)blockIdx.x * kRedCols + lane;
  const int colc = min(col, d - 1);
  float s = 0.0f;
  for (int g0 = w; g0 < row_groups; g0 += 4 * 16) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = partial[(size_t)min(g0 + 4 * u, row_groups - 1) * d + colc];
#pragma unroll
    for (int u = 0; u < 16; ++u) s += (g0 + 4 * u < row_groups) ? v[u] : 0.0f;
  }
  part[w][lane] = s;
  __syncthreads();
  if (tid < kRedCols && col < d) y[col] = ((part[0][tid] + part[1][tid]) + part[2][tid]) + part[3][tid];
  if (hist_ok) {
    if (gid < n) fr->hist2[kWindow + fine_bin((uint64_t)__double_as_longlong(h0))] = 0u;
    for (int i = gid + gsz; i < n; i += gsz) fr->hist2[kWindow + fine_bin((uint64_t)__double_as_longlong(h[i]))] = 0u;
  } else if (blockIdx.x == 0) {
    uint4* z1 = reinterpret_cast<uint4*>(fr->hist1);
    uint4* z2 = reinterpret_cast<uint4*>(fr->hist2);
    for (int i = tid; i < kHistWords / 4; i += (int)blockDim.x) {
      z1[i] = make_uint4(0, 0, 0, 0);
      z2[i] = make_uint4(0, 0, 0, 0);
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      fr->fallbacks[0] = fr->fallbacks[1] = 0u;
      fr->cookie = kCookie;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
size_t ffn_fast_region_bytes() { return sizeof(FastRegion); }
size_t ffn_fast_fallbacks_offset() { return offsetof(FastRegion, fallbacks); }
int ffn_fast_score_blocks(int N) { return min(((N + kRPW - 1) / kRPW + kSW - 1) / kSW, kFT); }

void ffn_fast_shape(int d, int k, int* row_groups, int* col_slices) {
  const int cs = (d + kFastCols - 1) / kFastCols;
  int rg = 256 / cs;
  const int by_rows = (k + 3) / 4;
  if (rg > by_rows) rg = by_rows;
  if (rg < 1) rg = 1;
  *row_groups = rg;
  *col_slices = cs;
}

// Group-sparse step with groups of eight: N, k, k' count units.  The selections see N/8, k'/8 and k/8 entries; a
// workgroup of the gather takes at most kShareCap / 8 groups (its units' activations pass through LDS).
bool ffn_fast_group8_supported(int B, int N, int d, int k, int kprime) {
  if (!(B == 1 && N % 8 == 0 && k % 8 == 0 && kprime % 8 == 0 && N <= 16384 && d % 32 == 0 && d >= 64 && d <= 8192))
    return false;
  const int kpg = kprime / 8, G = max(1, min(kpg, 256));
  if ((kpg + G - 1) / G > kShareCap / 8) return false;
  // second layer: a workgroup keeps the coefficients of at most kShareCap groups
  const int cs = (d + kFastCols - 1) / kFastCols, kg = k / 8, rg = max(1, min(256 / cs, kg));
  return (kg + rg - 1) / rg <= kShareCap;
}

// Row groups (of kShareCap rows) the m1 dense common-path units add to the second-layer kernel.
int ffn_fast_dense_groups(int m1) { return (m1 + kShareCap - 1) / kShareCap; }

bool ffn_fast_supported(int B, int N, int d, int k, int kprime) {
  // register capacity of the selecting workgroups: 16 waves x 4 loads x 256 keys, 16 waves x 2 loads x 128 h
  if (!(B == 1 && N <= 16384 && kprime <= 4096 && d % 32 == 0 && d >= 64 && d <= 8192)) return false;
  int rg, cs;
  ffn_fast_shape(d, k, &rg, &cs);
  return (k + rg - 1) / rg <= kShareCap;
}

hipError_t launch_ffn_fast(const FfnFastArgs& a, hipStream_t s) {
  hipError_t e;
  FastRegion* fr = reinterpret_cast<FastRegion*>(a.fast_region);
  auto mark = [&](int i) -> hipError_t { return a.stage_events ? hipEventRecord(a.stage_events[i], s) : hipSuccess; };
  if ((e = mark(0)) != hipSuccess) return e;
  const int score_blocks = ffn_fast_score_blocks(a.N);  // <= kFT: the next kernel reads one maximum per thread
  const int gs = a.gs;  // 0, or 3 for groups of eight units
  // what the selections rank: units with their keys and activations, or groups with their summed ones
  const int n_sel = a.N >> gs, kp_sel = a.kprime >> gs, k_sel = a.k >> gs;
  const float* sel_keys = gs ? a.gkeys : a.keys;
  const double* sel_h = gs ? a.hg : a.h;
  {
    const size_t lds = (size_t)a.d * 2 + (size_t)a.d;
    e = launch(k_fast_score_int4, dim3(score_blocks), dim3(kST), lds, s, reinterpret_cast<const uint4*>(a.q4),
               a.q4_scale, reinterpret_cast<const uint32_t*>(a.x), a.N, a.d, a.keys, a.scorer_acc, fr, a.scorer_clocks,
               gs ? a.gkeys : static_cast<float*>(nullptr));
    if (e != hipSuccess) return e;
    if ((e = mark(1)) != hipSuccess) return e;
  }
  int G = gs ? kp_sel : (a.kprime + 7) / 8;  // a workgroup takes about eight rows: eight units or one group
  G = max(1, min(G, 256));
  {
    FastGatherParams p{};
    p.keys = sel_keys; p.N = n_sel; p.kprime = kp_sel; p.d = a.d; p.score_blocks = score_blocks;
    p.fr = fr; p.W1 = a.w1u; p.x = reinterpret_cast<const uint4*>(a.x);
    p.cand = a.cand; p.n_cand = a.n_cand; p.h = a.h; p.gs = gs; p.hg = a.hg;
    p.sparse_blocks = G; p.Wd = a.dense_w1u; p.m1 = a.m1; p.hd = a.h_dense;
    const int dense_blocks = (a.m1 + kFW - 1) / kFW;  // one dense row per wave
    e = launch(k_fast_gather, dim3(G + dense_blocks), dim3(kFT), (size_t)a.d * 4, s, p);
    if (e != hipSuccess) return e;
    if ((e = mark(2)) != hipSuccess) return e;
  }
  int rg, cs;
  ffn_fast_shape(a.d, a.k, &rg, &cs);
  if (gs) rg = max(1, min(256 / cs, k_sel));  // one or two groups (8 or 16 rows) per workgroup
  const int dense_groups = ffn_fast_dense_groups(a.m1);
  {
    FastW2Params p{};
    p.h = sel_h; p.n = kp_sel; p.k = k_sel; p.d = a.d; p.gather_blocks = G; p.fr = fr; p.cand = a.cand; p.W2 = a.w2u;
    p.topk_idx = a.topk_idx; p.topk_val = a.topk_val; p.partial = a.partial; p.row_groups = rg; p.col_slices = cs;
    p.keys = sel_keys; p.N = n_sel; p.gs = gs; p.unit_h = a.h;
    p.dense_groups = dense_groups; p.W2d = a.dense_w2u; p.hd = a.h_dense; p.m1 = a.m1;
    e = launch(k_fast_w2, dim3((rg + dense_groups) * cs), dim3(kFT), 0, s, p);
    if (e != hipSuccess) return e;
    if ((e = mark(3)) != hipSuccess) return e;
  }
  e = launch(k_fast_reduce, dim3((a.d + kRedCols - 1) / kRedCols), dim3(256), 0, s, a.partial, rg + dense_groups, a.d,
             a.y, fr, sel_h, kp_sel);
  if (e != hipSuccess) return e;
  return mark(4);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_fast(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
