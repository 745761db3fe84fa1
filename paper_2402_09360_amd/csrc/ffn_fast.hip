// Batch-1 HiRE-FFN step in three kernels (arXiv 2402.09360, Algorithm 1 + eq. (4)),
// laid out so that no stage runs on a single workgroup:
//
//   k_fast_score   int8 token quantisation (redone by every workgroup, 4 KB), int4 scorer, keys to memory and
//                  a fine histogram of the keys (integer atomics; a bin is 2^14 consecutive fp32 bit patterns,
//                  i.e. exponent and nine mantissa bits, so that few keys share a counter)
//   k_fast_gather  every workgroup walks the histogram from the top, ranks the handful of keys of the
//                  threshold bin and so knows the exact k'-th key; the ascending candidate list follows from
//                  prefix counts, each workgroup materialises only its own share and computes the exact
//                  pre-activations of those rows; histogram of h the same way
//   k_fast_w2      the same selection on h (exact top-k), then sum_j h_j v_j over all selected rows for the
//                  workgroup's 64 columns, reduced inside the workgroup in a fixed order: y itself, no
//                  kernel follows.  Clears the key histogram (the next step's scorer kernel clears the h
//                  histogram, which nobody reads in between).
//   k_fast_reduce  only for steps whose second layer runs in several row groups (more than 1024 selected
//                  rows, or dense common-path units): adds the groups' partial rows in a fixed order
//
// A kernel boundary is the cheapest device-wide synchronisation on this machine (a spinning grid barrier
// costs several microseconds per round with 256 workgroups), hence separate kernels instead of one
// persistent kernel.  Selection work is duplicated in every workgroup instead of being serialised in one.
// What the selecting heads cost is their chain of dependent memory round trips (~1 us each) and their serial
// sections: a SIMD issues one vector instruction every four cycles, so with sixteen waves on a CU each wave
// gets one every ~16 cycles and a section of a hundred instructions takes 0.7 us.  Hence
//
//  * the gather runs sixteen waves per workgroup (four keys per lane, one row in flight per wave) and the
//    second layer eight: fewer waves per workgroup were measured slower for the same work (the serial sections
//    of a lone wave run at 10 to 15 cycles per instruction);
//  * The histograms are windows of 8192 bins at FIXED addresses: slot s counts the keys of bin anchor - s.
//    The anchors are rigorous upper bounds of the keys and of the activations that the scorer kernel derives
//    from the quantised token alone (sum |xq|) and the layer's largest row scale (kept behind the packed int4
//    codes), so every workgroup of every kernel knows them without waiting for any maximum, and a consumer
//    requests its histogram window together with its keys as its very first instructions.
//  * Key arrays are zero-padded to whole 16-byte vectors and lanes beyond the end read a vector of zeros, so
//    the passes over the register-resident keys need no validity tests: every comparison is against a
//    positive threshold.
//
// ReLU makes every key and every h non-negative, so their IEEE bit patterns already order like the numbers
// and are used as integer keys directly.
//
// The key histogram must be all zero when a step starts.  The second-layer kernel of every step leaves it so
// and stamps a cookie into the workspace; on a workspace without the cookie (first use, arbitrary contents) the
// first selection of one step takes a slower histogram-free route.  The h histogram is cleared by the scorer
// kernel of the step that uses it.  No kernel waits for, or counts, the workgroups of another.
#include "fast_select.h"
#include "kernels.h"

namespace hire {

constexpr unsigned long long kCookie = 0x48695245464e4f4cull;
constexpr int kShareCap = 64;                     // rows one gather workgroup handles at most

// Layout of the fast-path region at the head of the workspace.
struct FastRegion {
  unsigned long long cookie;
  uint32_t fallbacks[2];     // steps whose k'-th key / k-th h were found without the histogram (statistics)
  uint32_t pad1;
  uint32_t anchor1, anchor2; // top bins of the two windows for the running step, written by the scorer kernel
  uint32_t pad0;
  uint32_t zeros[8];         // stays zero: what lanes beyond the end of a key array load
  uint32_t pad[48];
  uint32_t hist1[kWin];      // slot s: scorer keys in fine bin anchor1 - s
  uint32_t hist2[kWin];      // slot s: activations in fine bin anchor2 - s
};
static_assert(offsetof(FastRegion, zeros) == 32 && offsetof(FastRegion, hist1) == 256, "region layout");

// ---------------------------------------------------------------------------------------------------
// Kernel 1: scorer.
constexpr int kRPW = 4;     // rows per wave and pass
constexpr int kST = 1024;   // threads per scorer workgroup: one workgroup per CU, the token is quantised once per CU
constexpr int kSW = kST / kWave;

// LRQ (the int4 low-rank scorer's second product): the "token" is the fp32 intermediate t of the first product,
// rounded to bf16 here as it is loaded, the rows are those of the int4 copy of Z2, and the activations' bound comes
// from the real token's norm and the layer's largest row norm (xn, xn_d, umax) instead of from the int4 codes.
template <bool LRQ>
__global__ __launch_bounds__(kST) void k_fast_score_int4(const uint4* __restrict__ q4, const float* __restrict__ scale,
                                                         const uint32_t* __restrict__ x, int N, int d,
                                                         float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                         FastRegion* __restrict__ fr,
                                                         unsigned long long* __restrict__ clocks,
                                                         float* __restrict__ gkeys, const uint4* __restrict__ xn,
                                                         int xn_d, const float* __restrict__ umax) {
  // gkeys != nullptr (group-sparse step, groups of eight adjacent units, eq. (6)): what is handed on and counted
  // in the histogram is the group activation gkeys[J] = sum_{l<8} |key[8J + l]| (fp32, unit order) instead of
  // the unit keys; a workgroup's 64 consecutive rows are eight whole groups.
  extern __shared__ uint32_t lds[];  // raw token, d/2 dwords of bf16 pairs; then d/4 dwords of int8 quads
  __shared__ float red[kSW];
  __shared__ int isum[kSW];
  __shared__ float unit_keys[kSW * kRPW];
  if (clocks && threadIdx.x == 0) clocks[2 * blockIdx.x] = wall_clock64();
  HIRE_TS(30);
  uint32_t* xraw = lds;
  uint32_t* xq = lds + d / 2;
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cpr = d / 32;
  const int total_waves = (int)gridDim.x * kSW;
  const int gw = (int)blockIdx.x * kSW + w;

  // token first (loads return in order, and the token is needed first), then the first rows' weights and
  // scales: all of these loads are in flight together
  const bool hist_ok = fr->cookie == kCookie;
  const float smax = __uint_as_float(q4[(size_t)N * cpr].x);  // largest row scale, kept behind the codes
  // the window of the activations, filled by the next kernel, starts from zero (its last reader was the step before)
  for (int i = (int)blockIdx.x * kST + tid; i < kWin; i += (int)gridDim.x * kST) fr->hist2[i] = 0u;
  const uint4* x4 = reinterpret_cast<const uint4*>(x);
  const int xvecs = d / 8;
  // eight token values as bf16 pairs: as they are, or (LRQ) two vectors of four floats rounded to nearest even
  auto token_vec = [&](int i) -> uint4 {
    if constexpr (!LRQ) {
      return x4[i];
    } else {
      const uint4 a = x4[2 * i], b = x4[2 * i + 1];
      auto rne = [](uint32_t u) { return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16; };
      return make_uint4(rne(a.x) | (rne(a.y) << 16), rne(a.z) | (rne(a.w) << 16), rne(b.x) | (rne(b.y) << 16),
                        rne(b.z) | (rne(b.w) << 16));
    }
  };
  const uint4 xv0 = token_vec(min(tid, xvecs - 1));
  const int cl = min(lane, cpr - 1);
  uint4 pre[kRPW];
#pragma unroll
  for (int rr = 0; rr < kRPW; ++rr) pre[rr] = load_streaming(&q4[(size_t)min(gw * kRPW + rr, N - 1) * cpr + cl]);
  const float pre_scale = scale[min(gw * kRPW + (lane >> 4), N - 1)];
  float amax = 0.0f;
  for (int i = tid; i < xvecs; i += kST) {
    const uint4 u = i == tid ? xv0 : token_vec(i);
    reinterpret_cast<uint4*>(xraw)[i] = u;
    const uint32_t ud[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(ud[q])), fabsf(bf16_hi(ud[q]))));
  }
  amax = wave_max(amax);
  if (lane == 0) red[w] = amax;
  __syncthreads();
  HIRE_TS(31);
  amax = wave_max(lane < kSW ? red[lane] : 0.0f);
  float sx = __fdiv_rn(amax, 127.0f);
  if (amax == 0.0f) sx = 1.0f;
  int sabs = 0;  // this thread's share of sum |xq|
  for (int i = tid; i < d / 4; i += kST) {
    const uint32_t a = xraw[2 * i], b = xraw[2 * i + 1];
    const float f[4] = {bf16_lo(a), bf16_hi(a), bf16_lo(b), bf16_hi(b)};
    uint32_t packed = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float r = rintf(__fdiv_rn(f[e], sx));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      sabs += (int)fabsf(r);
      packed |= ((uint32_t)(int)r & 0xFFu) << (8 * e);
    }
    xq[i] = packed;
  }
  sabs = wave_sum(sabs);
  if (lane == 0) isum[w] = sabs;
  __syncthreads();
  HIRE_TS(32);
  // Upper bounds that hold for every unit of the layer, from the token alone.  With codes |q| <= 7, |xq| <= 127:
  //   key_j = fl(fl(acc_j) s_j) <= fl(7 sum|xq| smax)                       (rounding is monotone; 7 sum|xq| < 2^24)
  //   <u_j, x> = s_j sx sum (q + dq)(xq + dx), |dq|, |dx| <= 1/2 (+ rounding of the two divisions)
  //           <= smax sx (7.5 sum|xq| + 3.75 d + ...), taken with a margin that also covers the fp32 arithmetic
  // The group activations of eq. (6) are sums of eight such terms.
  const int sumabs = wave_sum(lane < kSW ? isum[lane] : 0);
  const float group_factor = gkeys != nullptr ? 8.001f : 1.0f;
  const float bound1 = (float)(7 * sumabs) * smax * group_factor;
  float bound2 = smax * sx * (7.6f * (float)sumabs + 3.8f * (float)d + 1.0f) * 1.01f * group_factor;
  if constexpr (LRQ) {  // Cauchy-Schwarz: <u_j, x> <= |u_j| |x|, both rounded up by more than their error
    float xsq = 0.0f;
    for (int i = tid; i < xn_d / 8; i += kST) {
      const uint4 u = xn[i];
      const uint32_t ud[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = bf16_lo(ud[q]), b = bf16_hi(ud[q]);
        xsq = fmaf(a, a, xsq);
        xsq = fmaf(b, b, xsq);
      }
    }
    xsq = wave_sum(xsq);
    __syncthreads();  // red's readers above are done
    if (lane == 0) red[w] = xsq;
    __syncthreads();
    xsq = wave_sum(lane < kSW ? red[lane] : 0.0f);
    bound2 = sqrtf(xsq * (1.0f + (float)xn_d * 0x1p-22f)) * 1.0001f * umax[0] * 1.0001f;
  }
  const uint32_t anchor1 = fine_bin(__float_as_uint(bound1)), anchor2 = fine_bin(__float_as_uint(bound2));
  if (blockIdx.x == 0 && tid == 0) {
    fr->anchor1 = anchor1;
    fr->anchor2 = anchor2;
  }
  {  // zero padding of the handed-on key array up to a whole 16-byte vector
    float* arr = gkeys != nullptr ? gkeys : keys;
    const int n = gkeys != nullptr ? N / 8 : N;
    if (blockIdx.x == 0 && tid < ((4 - (n & 3)) & 3)) arr[n + tid] = 0.0f;
  }
  auto count_key = [&](float key) {
    const uint32_t bits = __float_as_uint(key);
    const uint32_t slot = anchor1 - fine_bin(bits);  // keys lie at or below the anchor; zeros are never counted
    if (hist_ok && bits != 0u && slot < (uint32_t)kWin) atomicAdd(&fr->hist1[slot], 1u);
  };

  const uint4* xq4 = reinterpret_cast<const uint4*>(xq);
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
    HIRE_TS(33);
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
        count_key(key);
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
      count_key(sum);
    }
  }
  HIRE_TS(34);
  if (clocks) {
    __syncthreads();
    if (tid == 0) clocks[2 * blockIdx.x + 1] = wall_clock64();
  }
}

// ---------------------------------------------------------------------------------------------------
// Kernel 1 for the low-rank scorer (HiRE-LR, Sec. 3.2): keys[j] = relu(<Z2[j, :], t>) in fp64 with
// t = bf16(Z1^T x).  The slices of Z1^T x come from k_lr_project; every workgroup adds them itself, in slice
// order, and rounds once (what k_lr_reduce does), so no kernel of one workgroup runs in between.  The anchors are
// Cauchy-Schwarz bounds: key_j <= |Z2_j| |t| and <u_j, x> <= |u_j| |x| with the layer's largest row norms
// (bounds[1], bounds[0]: upper bounds, prepared once per layer) and the norms of t and x formed here in fp32 and
// rounded up by more than their own error.  ROW_LANES lanes share a row as in k_lr_score_b1.
template <int ROW_LANES>
__global__ __launch_bounds__(kST) void k_fast_score_lr(const double* __restrict__ partial, int slices,
                                                       const uint16_t* __restrict__ z2, const uint4* __restrict__ x,
                                                       int N, int d, int r, const float* __restrict__ bounds,
                                                       double* __restrict__ keys, FastRegion* __restrict__ fr) {
  __shared__ uint4 ts[128];  // t as raw bf16: r <= 1024
  __shared__ float red_t[kSW], red_x[kSW];
  constexpr int kRows = kWave / ROW_LANES;  // rows per wave and trip
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int sub = lane % ROW_LANES, rw = lane / ROW_LANES;
  const int cpr = r / 8;
  HIRE_TS(30);
  const bool hist_ok = fr->cookie == kCookie;
  const float umax = bounds[0], zmax = bounds[1];
  for (int i = (int)blockIdx.x * kST + tid; i < kWin; i += (int)gridDim.x * kST) fr->hist2[i] = 0u;
  float tsq = 0.0f, xsq = 0.0f;
  uint16_t* t16 = reinterpret_cast<uint16_t*>(ts);
  for (int p = tid; p < r; p += kST) {
    double tot = 0.0;
    for (int s0 = 0; s0 < slices; s0 += 8) {  // eight loads in flight; added in slice order
      double v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = partial[(size_t)min(s0 + j, slices - 1) * r + p];
#pragma unroll
      for (int j = 0; j < 8; ++j) tot += s0 + j < slices ? v[j] : 0.0;
    }
    const uint16_t tb = f64_to_bf16_rne(tot);
    t16[p] = tb;
    const float tf = bf16_to_f32(tb);
    tsq = fmaf(tf, tf, tsq);
  }
  for (int i = tid; i < d / 8; i += kST) {
    const uint4 u = x[i];
    const uint32_t ud[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float a = bf16_lo(ud[q]), b = bf16_hi(ud[q]);
      xsq = fmaf(a, a, xsq);
      xsq = fmaf(b, b, xsq);
    }
  }
  tsq = wave_sum(tsq);
  xsq = wave_sum(xsq);
  if (lane == 0) {
    red_t[w] = tsq;
    red_x[w] = xsq;
  }
  __syncthreads();
  HIRE_TS(32);
  tsq = wave_sum(lane < kSW ? red_t[lane] : 0.0f);
  xsq = wave_sum(lane < kSW ? red_x[lane] : 0.0f);
  const float tnorm = sqrtf(tsq * (1.0f + (float)r * 0x1p-22f)) * 1.0001f;
  const float xnorm = sqrtf(xsq * (1.0f + (float)d * 0x1p-22f)) * 1.0001f;
  const float bound1 = tnorm * zmax * 1.0001f, bound2 = xnorm * umax * 1.0001f;
  const uint32_t anchor1 = fine_bin(__float_as_uint(bound1)), anchor2 = fine_bin(__float_as_uint(bound2));
  if (blockIdx.x == 0 && tid == 0) {
    fr->anchor1 = anchor1;
    fr->anchor2 = anchor2;
    if (N & 1) keys[N] = 0.0;  // zero padding of the handed-on key array up to a whole 16-byte vector
  }
  const int total = (int)gridDim.x * kSW * kRows;
  for (int j0 = ((int)blockIdx.x * kSW + w) * kRows; j0 < N; j0 += total) {
    const int j = j0 + rw;
    const uint4* row = reinterpret_cast<const uint4*>(z2 + (size_t)min(j, N - 1) * r);
    double acc = 0.0;
    for (int c0 = 0; c0 < cpr; c0 += ROW_LANES) {
      const int c = c0 + sub;
      const uint4 wv = row[min(c, cpr - 1)];
      const uint4 tv = ts[min(c, cpr - 1)];
      const uint32_t keep = c < cpr ? 0xFFFFFFFFu : 0u;
      const uint32_t wd[4] = {wv.x & keep, wv.y & keep, wv.z & keep, wv.w & keep};
      const uint32_t td[4] = {tv.x, tv.y, tv.z, tv.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc += (double)(bf16_lo(wd[q]) * bf16_lo(td[q]));
        acc += (double)(bf16_hi(wd[q]) * bf16_hi(td[q]));
      }
    }
    double s;
    if constexpr (ROW_LANES == kWave) {
      s = wave_sum(acc);
    } else {  // prefix sum along the 16 lanes of a DPP row: the row's last lane holds its total
      auto add = [](double a, double b) { return a + b; };
      s = acc;
      s = add(s, dpp_move<0x111, 0xF>(0.0, s));
      s = add(s, dpp_move<0x112, 0xF>(0.0, s));
      s = add(s, dpp_move<0x114, 0xF>(0.0, s));
      s = add(s, dpp_move<0x118, 0xF>(0.0, s));
    }
    if (sub == ROW_LANES - 1 && j < N) {
      s = s > 0.0 ? s : 0.0;  // ReLU, and -0 -> +0
      keys[j] = s;
      const uint32_t slot = anchor1 - fine_bin((uint64_t)__double_as_longlong(s));  // keys lie at or below the anchor
      if (hist_ok && s > 0.0 && slot < (uint32_t)kWin) atomicAdd(&fr->hist1[slot], 1u);  // zeros are never counted
    }
  }
  HIRE_TS(34);
}

// ---------------------------------------------------------------------------------------------------
// Kernel 2: exact k'-th key, this workgroup's share of the candidate list, exact pre-activations.
// Sixteen waves per workgroup, sixteen keys per lane.  K: the keys' bit patterns, 32 bits for the int4 scorer's
// fp32 keys, 64 for the low-rank scorer's fp64 ones.
constexpr int kGT = 1024;  // smaller workgroups were measured: slower (fewer waves to hide each phase's latency)
constexpr int kGW = kGT / kWave;
constexpr int kGatherLoads = 64 / kGW;    // waves x loads x 256 keys = 16384
constexpr int kGatherRows = 16 / kGW;     // rows a wave has in flight: sixteen per workgroup
using GatherShared = SelSharedT<kGT>;
template <typename K>
using GatherKeys = KeyRegs<K, kGatherLoads * (int)(sizeof(K) / 4), kGT>;  // 16384 keys either way

struct FastGatherParams {
  const void* keys;           // [N] fp32 (fp64), zero up to the next multiple of 4 (2)
  int N, kprime, d;
  FastRegion* fr;
  const uint16_t* W1;         // [N, d] bf16
  const uint4* x;             // token, d/8 uint4
  int32_t* cand;              // [kprime] ascending candidate list in the workspace (read back by the next kernel)
  int32_t* cand_out;          // optional: the caller's copy
  int32_t* n_cand;            // optional
  double* h;                  // [kprime << gs] (+ zero padding to a multiple of 2 when gs = 0)
  // gs = 3 (group-sparse step): keys are group activations, N and kprime count groups of eight units, cand lists
  // groups; h holds the eight units of every candidate group and hg[kprime] their exact group activations
  // sum_l |h|, which are what is counted in the histogram and ranked by the next kernel.  gs = 0: units.
  int gs;
  double* hg;
  // CommonPath (eq. (7)): workgroups sparse_blocks .. gridDim.x - 1 skip the selection and compute the
  // activations of the m1 dense units, kGW * kGatherRows rows per workgroup: hd[r] = relu(<Wd[r, :], x>).
  int sparse_blocks;
  const uint16_t* Wd;
  int m1;
  double* hd;
};

// relu(<row_u, x>) for up to kGatherRows rows per wave at once, the token as fp32 in LDS: sixteen bytes per lane
// and load, all loads of the rows' 256-chunk slice in flight together; every bf16 product is exact in fp32 and
// the sums run in fp64.  Only the first nr rows (uniform over the wave) are computed; the others must point at
// row 0, whose loads they repeat.
__device__ __forceinline__ void rows_dot_relu(const uint4* const (&row)[kGatherRows], int nr,
                                              const float* __restrict__ xtok, int cpr, double (&out)[kGatherRows]) {
  const int lane = lane_id();
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
          if (u < nr) {
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
  }
#pragma unroll
  for (int u = 0; u < kGatherRows; ++u) {
    const double s = wave_sum(acc[u]);
    out[u] = s > 0.0 ? s : 0.0;  // ReLU, and -0 -> +0
  }
}

__device__ __forceinline__ void token_to_lds(const uint4* __restrict__ x, int xvecs, float* xtok) {
  const int tid = (int)threadIdx.x;
  const uint4 xv0 = x[min(tid, xvecs - 1)];
  for (int i = tid; i < xvecs; i += kGT) {
    const uint4 u = i == tid ? xv0 : x[i];
    const float f[8] = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y),
                        bf16_lo(u.z), bf16_hi(u.z), bf16_lo(u.w), bf16_hi(u.w)};
#pragma unroll
    for (int q = 0; q < 8; ++q) xtok[8 * i + q] = f[q];
  }
}

template <typename K>
__global__ __launch_bounds__(kGT) void k_fast_gather(FastGatherParams p) {
  __shared__ GatherShared sh;
  __shared__ int wave_cnt[kGW];
  __shared__ int my_rows[kShareCap];
  __shared__ double unit_h[kShareCap];  // group-sparse: the units' activations of this workgroup's (<= 8) groups
  extern __shared__ float xtok[];  // token as fp32, d floats
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int G = p.sparse_blocks, g = (int)blockIdx.x;
  const int xvecs = p.d / 8;
  if (g >= G) {  // dense common-path units: token into LDS, then kGatherRows rows per wave
    token_to_lds(p.x, xvecs, xtok);
    __syncthreads();
    const int r0 = (g - G) * (kGW * kGatherRows);
    const int have = min(kGW * kGatherRows, p.m1 - r0);
    if (w >= have) return;
    const uint4* row[kGatherRows];
    double sd[kGatherRows];
    const int nr = (have - w + kGW - 1) / kGW;  // rows w, w + kGW, ... below have
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u)
      row[u] = reinterpret_cast<const uint4*>(p.Wd + (size_t)(r0 + (u < nr ? w + kGW * u : w)) * p.d);
    rows_dot_relu(row, nr, xtok, xvecs, sd);
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u)
      if (lane == 0 && w + kGW * u < have) p.hd[r0 + w + kGW * u] = sd[u];
    return;
  }
  HIRE_TS(10);
  // every load of the selection goes out here, before the first wait
  const bool hist_ok = p.fr->cookie == kCookie;
  const uint32_t anchor1 = p.fr->anchor1, anchor2 = p.fr->anchor2;
  WinRegs<kGT> wr;
  wr.issue(p.fr->hist1);
  GatherKeys<K> kr;
  kr.issue(p.keys, p.N, p.fr->zeros);
  token_to_lds(p.x, xvecs, xtok);
  kr.finish();
  HIRE_TS(11);
#ifdef HIRE_TIMESTAMPS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // profiling build only: when has everything requested arrived?
  HIRE_TS(18);
#endif
  const int share = (p.kprime + G - 1) / G;
  const int lo = min(p.kprime, g * share), hi = min(p.kprime, lo + share);
  const Selection<K> sel = fast_select<15>(
      kr, p.keys, p.kprime, wr, anchor1, hist_ok, sh, wave_cnt,
      hist_ok ? &p.fr->fallbacks[0] : static_cast<uint32_t*>(nullptr),  // a fresh workspace's first step is not counted
      lo, hi);
  HIRE_TS(12);

  fast_emit(kr, sel, lo, hi, [&](int i, int out, K, int, int) { my_rows[out - lo] = i; });
  __syncthreads();  // my_rows, and the token in LDS (no global store is pending here: a barrier would wait for it)
  HIRE_TS(13);

  const int gs = p.gs, gmask = (1 << gs) - 1;
  const int cnt = (hi - lo) << gs;  // rows of this workgroup
  auto count_h = [&](double v) {  // the scorer kernel of this step has cleared the window
    if (v > 0.0) {
      const uint32_t slot = anchor2 - fine_bin((uint64_t)__double_as_longlong(v));  // v lies at or below the anchor
      if (slot < (uint32_t)kWin) atomicAdd(&p.fr->hist2[slot], 1u);
    }
  };
  for (int r0 = 0; r0 < cnt; r0 += kGW * kGatherRows) {  // one trip unless groups are gathered
    if (r0 + w >= cnt) break;                             // uniform over the wave
    const uint4* row[kGatherRows];
    double s[kGatherRows];
    const int nr = min(kGatherRows, (cnt - r0 - w + kGW - 1) / kGW);  // rows r0 + w, r0 + w + kGW, ... below cnt
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u) {
      const int r = r0 + w + (u < nr ? kGW * u : 0);
      const size_t unit = ((size_t)my_rows[r >> gs] << gs) + (r & gmask);
      row[u] = reinterpret_cast<const uint4*>(p.W1 + unit * p.d);
    }
    rows_dot_relu(row, nr, xtok, xvecs, s);
#pragma unroll
    for (int u = 0; u < kGatherRows; ++u) {
      const int r = r0 + w + kGW * u;
      if (lane == 0 && r < cnt) {
        p.h[((size_t)lo << gs) + r] = s[u];
        if ((r & gmask) == 0) {
          p.cand[lo + (r >> gs)] = my_rows[r >> gs];
          if (p.cand_out) p.cand_out[lo + (r >> gs)] = my_rows[r >> gs];
        }
        if (gs != 0) {
          unit_h[r] = s[u];
        } else {
          count_h(s[u]);
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
      count_h(e);
    }
  }
  if (g == 0 && tid == 0) {
    if (p.n_cand) *p.n_cand = p.kprime;
    if (p.kprime & 1) (p.gs != 0 ? p.hg : p.h)[p.kprime] = 0.0;  // zero padding of what the next kernel ranks
  }
  HIRE_TS(14);
}

// ---------------------------------------------------------------------------------------------------
// Kernel 3: exact top-k of h, then sum_j h_j v_j over the selected rows for this workgroup's 32 columns.
// A workgroup reads a 64-byte slice of every selected row (four lanes per row, sixteen rows per wave and load,
// all loads of a wave in flight together) and reduces inside itself in a fixed order, so with one row group
// the result is y itself and no kernel follows.  Steps with more than kRowsCap selected rows, and the dense
// common-path units, add row groups whose partial rows k_fast_reduce sums.
constexpr int kWT = 512;
constexpr int kWW = kWT / kWave;
constexpr int kW2Loads = 32 / kWW;   // waves x loads x 128 activations = 4096
using W2Shared = SelSharedT<kWT>;
using W2Keys = KeyRegs<uint64_t, kW2Loads, kWT>;
static_assert(GatherKeys<uint32_t>::CAPACITY >= 16384 && GatherKeys<uint64_t>::CAPACITY >= 16384 && W2Keys::CAPACITY >= 4096, "register capacity of the selecting workgroups");

struct FastW2Params {
  const double* h;       // [n], zero up to the next multiple of 2
  int n, k, d;
  FastRegion* fr;
  const int32_t* cand;   // [n] unit index of each position, readable to the next multiple of 2
  const uint16_t* W2;    // [N, d] bf16
  int32_t* topk_idx;     // optional [k]
  float* topk_val;       // optional [k]
  float* out;            // row_groups + dense_groups == 1: y [d]; otherwise partial [row_groups + dense_groups, d]
  int row_groups, col_slices;
  // gs = 3 (group-sparse step): h holds exact group activations, n and k count groups, cand lists groups;
  // unit_h[n << gs] holds the units' activations (the second layer's coefficients) and topk_val receives the
  // eight of every selected group.  gs = 0: units, unit_h unused.
  int gs;
  const double* unit_h;
  // CommonPath (eq. (7)): row groups row_groups .. row_groups + dense_groups - 1 (times the column slices) add
  // the m1 dense units, kRowsCap rows each: out += fl32(hd[r]) * W2d[r, :].  dense_groups = 0: none.
  int dense_groups;
  const uint16_t* W2d;
  const double* hd;
  int m1;
};

constexpr int kSliceCols = 32;  // columns per workgroup: 64 bytes of a row
constexpr int kRowsCap = 1024;    // rows per workgroup
constexpr int kRowLanes = kSliceCols / 8;        // lanes that share a row: 16 bytes each
constexpr int kRowsPerLoad = kWave / kRowLanes;  // rows a wave covers with one load instruction
constexpr int kW2Batch = 8;       // loads a lane has in flight

// Column slice of a workgroup: slices 2i and 2i+1 are the two halves of the same 128-byte lines; they go to
// workgroups b and b + 8, which the dispatcher places on the same die (workgroups go round the eight dies),
// so that the second half of a line is found in that die's L2.
__device__ __forceinline__ int slice_of(int b, int slices) {
  if (kSliceCols != 32 || slices % 16 != 0) return b;
  return 2 * (b % 8) + (b / 8) % 2 + 16 * (b / 16);
}

__global__ __launch_bounds__(kWT) void k_fast_w2(FastW2Params p) {
  __shared__ W2Shared sh;
  __shared__ int wave_cnt[kWW];
  __shared__ int my_unit[kRowsCap];
  __shared__ float my_h[kRowsCap];
  __shared__ int grp_unit[kRowsCap / 8], grp_pos[kRowsCap / 8];  // group-sparse: the selected groups
  __shared__ float red[kWW * kRowsPerLoad][kSliceCols];
  __shared__ float red2[kWW][kSliceCols];
  const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const int cs = slice_of((int)blockIdx.x % p.col_slices, p.col_slices), rg = (int)blockIdx.x / p.col_slices;
  const bool dense = rg >= p.row_groups;  // uniform over the workgroup
  const int n_selecting = p.row_groups * p.col_slices;
  int cnt, lo = 0, hi = 0;
  const uint16_t* W2 = p.W2;
  if (dense) {  // no selection: this group's dense rows with their activations as coefficients
    const int r0 = (rg - p.row_groups) * kRowsCap;
    cnt = min(kRowsCap, p.m1 - r0);
    for (int i = tid; i < cnt; i += kWT) {
      my_unit[i] = r0 + i;
      my_h[i] = (float)p.hd[r0 + i];
    }
    W2 = p.W2d;
    __syncthreads();
  } else {
    HIRE_TS(24);
    const uint32_t anchor2 = p.fr->anchor2;
    WinRegs<kWT> wr;
    wr.issue(p.fr->hist2);
    W2Keys kr;
    kr.issue(p.h, p.n, p.fr->zeros);
    // unit index of each of this thread's positions: position (e, lane, q) is 2 * (vector index) + q
    int2 cu[kW2Loads];
#pragma unroll
    for (int e = 0; e < kW2Loads; ++e) {
      const int vec = min((kr.base + e * W2Keys::SPAN) / 2 + lane, (p.n - 1) / 2);
      cu[e] = reinterpret_cast<const int2*>(p.cand)[vec];
    }
    kr.finish();
    // the activations' window is valid on any workspace: this step's scorer kernel cleared it, its gather filled it
    const int share = min(kRowsCap >> p.gs, (p.k + p.row_groups - 1) / p.row_groups);
    lo = min(p.k, rg * share);
    hi = min(p.k, lo + share);
    const Selection<uint64_t> sel = fast_select<20>(kr, p.h, p.k, wr, anchor2, true, sh, wave_cnt,
                                                    &p.fr->fallbacks[1], lo, hi);
    HIRE_TS(25);
    // into LDS only: a global store here would be waited for by the barrier that follows
    fast_emit(kr, sel, lo, hi, [&](int i, int out, uint64_t bits, int e, int q) {
      const int unit = q ? cu[e].y : cu[e].x;
      if (p.gs == 0) {
        my_unit[out - lo] = unit;
        my_h[out - lo] = (float)__longlong_as_double((long long)bits);
      } else {
        grp_unit[out - lo] = unit;
        grp_pos[out - lo] = i;
      }
    });
    __syncthreads();
    cnt = (hi - lo) << p.gs;  // rows of this workgroup
    if (p.gs != 0) {  // the selected groups' units and their coefficients
      const int gmask = (1 << p.gs) - 1;
      for (int r = tid; r < cnt; r += kWT) {
        const float hv = (float)p.unit_h[((size_t)grp_pos[r >> p.gs] << p.gs) + (r & gmask)];
        my_unit[r] = (grp_unit[r >> p.gs] << p.gs) + (r & gmask);
        my_h[r] = hv;
      }
      __syncthreads();
    }
    HIRE_TS(26);
  }

  // rows r = (step * kWW + w) * kRowsPerLoad + slot for this lane's slot; eight columns per lane
  const int slot = lane / kRowLanes, part = lane % kRowLanes;
  const int col = cs * kSliceCols + part * 8;
  const int colc = min(col, p.d - 8);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  constexpr int kStride = kWW * kRowsPerLoad;  // rows the workgroup covers per load of every wave
  for (int r0 = w * kRowsPerLoad + slot; r0 < cnt; r0 += kStride * kW2Batch) {
    uint4 wv[kW2Batch];
    float cf[kW2Batch];
#pragma unroll
    for (int u = 0; u < kW2Batch; ++u) {
      const int r = r0 + kStride * u, rc = min(r, cnt - 1);
      wv[u] = load_streaming(reinterpret_cast<const uint4*>(W2 + (size_t)my_unit[rc] * p.d + colc));
      cf[u] = r < cnt ? my_h[rc] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kW2Batch; ++u) {
      const float wf[8] = {bf16_lo(wv[u].x), bf16_hi(wv[u].x), bf16_lo(wv[u].y), bf16_hi(wv[u].y),
                           bf16_lo(wv[u].z), bf16_hi(wv[u].z), bf16_lo(wv[u].w), bf16_hi(wv[u].w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(cf[u], wf[q], acc[q]);
    }
  }
  HIRE_TS(27);
  // fixed-order reduction: the (wave, slot) partial rows -> one per wave -> 1
  {
    float4* dst = reinterpret_cast<float4*>(&red[w * kRowsPerLoad + slot][part * 8]);
    dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
  __syncthreads();
  if (tid < kWW * kSliceCols) {
    const int c = tid % kSliceCols, j = tid / kSliceCols;  // j < kWW
    float t = 0.0f;
#pragma unroll
    for (int u = 0; u < kRowsPerLoad; ++u) t += red[j * kRowsPerLoad + u][c];
    red2[j][c] = t;
  }
  __syncthreads();
  if (tid < kSliceCols) {
    const int c = cs * kSliceCols + tid;
    if (c < p.d) {
      float t = 0.0f;
#pragma unroll
      for (int u = 0; u < kWW; ++u) t += red2[u][tid];
      p.out[(size_t)(p.row_groups + p.dense_groups == 1 ? 0 : rg) * p.d + c] = t;
    }
  }
  HIRE_TS(28);
  if (dense) return;
  if (cs == 0) {  // the selected entries and their activations, in the order of the second layer's rows
    if (p.topk_idx)
      for (int j = tid; j < hi - lo; j += kWT) p.topk_idx[lo + j] = p.gs == 0 ? my_unit[j] : grp_unit[j];
    if (p.topk_val)
      for (int r = tid; r < cnt; r += kWT) p.topk_val[((size_t)lo << p.gs) + r] = my_h[r];
  }
  // The key histogram has served its purpose: the selecting workgroups clear it between them and say so in the
  // cookie (the same value from each; the next kernel that looks at either starts after this one has ended).
  for (int i = (int)blockIdx.x * kWT + tid; i < kWin; i += n_selecting * kWT) p.fr->hist1[i] = 0u;
  if (tid == 0) p.fr->cookie = kCookie;
}

// Kernel 4 (only when the second layer ran in several row groups): y = their sum, in order.
__global__ __launch_bounds__(256) void k_fast_reduce(const float* __restrict__ partial, int groups, int d,
                                                     float* __restrict__ y) {
  const int col = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  const int colc = min(col, d - 1);
  float s = 0.0f;
  for (int g0 = 0; g0 < groups; g0 += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)min(g0 + u, groups - 1) * d + colc];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += g0 + u < groups ? v[u] : 0.0f;
  }
  if (col < d) y[col] = s;
}

// ---------------------------------------------------------------------------------------------------
size_t ffn_fast_region_bytes() { return sizeof(FastRegion); }
size_t ffn_fast_fallbacks_offset() { return offsetof(FastRegion, fallbacks); }
void ffn_fast_state_layout(size_t* cookie_off, unsigned long long* cookie, size_t* hist1_off, size_t* hist2_off,
                           size_t* hist_words) {
  *cookie_off = offsetof(FastRegion, cookie);
  *cookie = kCookie;
  *hist1_off = offsetof(FastRegion, hist1);
  *hist2_off = offsetof(FastRegion, hist2);
  *hist_words = kWin;
}
int ffn_fast_score_blocks(int N) { return min(((N + kRPW - 1) / kRPW + kSW - 1) / kSW, 1024); }

// Row groups and column slices of the second-layer kernel for `rows` selected rows (units).
void ffn_fast_shape(int d, int rows, int* row_groups, int* col_slices) {
  *col_slices = (d + kSliceCols - 1) / kSliceCols;
  *row_groups = max(1, (rows + kRowsCap - 1) / kRowsCap);
}

// Group-sparse step with groups of eight: N, k, k' count units.  The selections see N/8, k'/8 and k/8 entries; a
// workgroup of the gather takes at most kShareCap / 8 groups (its units' activations pass through LDS).
bool ffn_fast_group8_supported(int B, int N, int d, int k, int kprime) {
  if (!(B == 1 && N % 8 == 0 && k % 8 == 0 && kprime % 8 == 0 && N <= GatherKeys<uint32_t>::CAPACITY && d % 32 == 0 && d >= 64 &&
        d <= 8192))
    return false;
  const int kpg = kprime / 8, G = max(1, min(kpg, 256));
  return (kpg + G - 1) / G <= kShareCap / 8;
}

// Row groups (of kRowsCap rows) the m1 dense common-path units add to the second-layer kernel.
int ffn_fast_dense_groups(int m1) { return (m1 + kRowsCap - 1) / kRowsCap; }

// Floats of partial rows the step needs (0: the second-layer kernel writes y itself).
size_t ffn_fast_partial_floats(int d, int k, int m1) {
  int rg, cs;
  ffn_fast_shape(d, k, &rg, &cs);
  const int groups = rg + ffn_fast_dense_groups(m1);
  return groups > 1 ? (size_t)groups * d : 0;
}

bool ffn_fast_supported(int B, int N, int d, int k, int kprime) {
  return B == 1 && N <= GatherKeys<uint32_t>::CAPACITY && kprime <= W2Keys::CAPACITY && d % 32 == 0 && d >= 64 && d <= 8192 &&
         k >= 1;
}

hipError_t launch_ffn_fast(const FfnFastArgs& a, hipStream_t s) {
  hipError_t e;
  FastRegion* fr = reinterpret_cast<FastRegion*>(a.fast_region);
  auto mark = [&](int i) -> hipError_t { return a.stage_events ? hipEventRecord(a.stage_events[i], s) : hipSuccess; };
  if ((e = mark(0)) != hipSuccess) return e;
  const int score_blocks = ffn_fast_score_blocks(a.N);
  const int gs = a.gs;  // 0, or 3 for groups of eight units
  // what the selections rank: units with their keys and activations, or groups with their summed ones
  const int n_sel = a.N >> gs, kp_sel = a.kprime >> gs, k_sel = a.k >> gs;
  const bool lowrank = a.lowrank;
  const void* sel_keys = lowrank ? static_cast<const void*>(a.keys64) : (gs ? a.gkeys : a.keys);
  const double* sel_h = gs ? a.hg : a.h;
  if (lowrank) {
    if (gs != 0 || a.m1 != 0 || a.r < 8 || a.r > 1024 || a.r % 8 != 0) return hipErrorInvalidValue;
    e = launch_lr_project(static_cast<const uint16_t*>(a.lr_a), a.x, 1, a.d, a.r, nullptr, a.t_partial, nullptr, 0, nullptr,
                          0ull, s);
    if (e != hipSuccess) return e;
    const int slices = lr_project_slices(a.d);
    const uint4* x4 = reinterpret_cast<const uint4*>(a.x);
    if (a.r <= 128)
      e = launch(k_fast_score_lr<16>, dim3(score_blocks), dim3(kST), 0, s, a.t_partial, slices,
                 static_cast<const uint16_t*>(a.lr_b), x4, a.N, a.d, a.r, a.norm_bounds, a.keys64, fr);
    else
      e = launch(k_fast_score_lr<kWave>, dim3(score_blocks), dim3(kST), 0, s, a.t_partial, slices,
                 static_cast<const uint16_t*>(a.lr_b), x4, a.N, a.d, a.r, a.norm_bounds, a.keys64, fr);
    if (e != hipSuccess) return e;
    if ((e = mark(1)) != hipSuccess) return e;
  } else if (a.lrq) {
    // first product: the r rows of the int4 copy of Z1^T against the token (no phi), fp32 intermediate; then the
    // scorer kernel on the int4 copy of Z2 with that intermediate as its token
    if (gs != 0 || a.m1 != 0 || a.r < 32 || a.r > 8192 || a.r % 32 != 0) return hipErrorInvalidValue;
    e = launch_scorer_int4_fused(reinterpret_cast<const uint32_t*>(a.lr_a), a.lr_a_scale, a.x, false, a.r, a.d, 0,
                                 a.keys_t, nullptr, HistRefs{nullptr, nullptr}, nullptr, 0, 0ull, s);
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)a.r * 2 + (size_t)a.r;
    e = launch(k_fast_score_int4<true>, dim3(score_blocks), dim3(kST), lds, s, reinterpret_cast<const uint4*>(a.lr_b),
               a.lr_b_scale, reinterpret_cast<const uint32_t*>(a.keys_t), a.N, a.r, a.keys, static_cast<int32_t*>(nullptr),
               fr, a.scorer_clocks, static_cast<float*>(nullptr), reinterpret_cast<const uint4*>(a.x), a.d,
               a.norm_bounds);
    if (e != hipSuccess) return e;
    if ((e = mark(1)) != hipSuccess) return e;
  } else {
    const size_t lds = (size_t)a.d * 2 + (size_t)a.d;
    e = launch(k_fast_score_int4<false>, dim3(score_blocks), dim3(kST), lds, s, reinterpret_cast<const uint4*>(a.q4),
               a.q4_scale, reinterpret_cast<const uint32_t*>(a.x), a.N, a.d, a.keys, a.scorer_acc, fr, a.scorer_clocks,
               gs ? a.gkeys : static_cast<float*>(nullptr), static_cast<const uint4*>(nullptr), 0,
               static_cast<const float*>(nullptr));
    if (e != hipSuccess) return e;
    if ((e = mark(1)) != hipSuccess) return e;
  }
  int G = gs ? kp_sel : (a.kprime + 7) / 8;  // a workgroup takes about eight rows: eight units or one group
  G = max(1, min(G, 256));
  {
    FastGatherParams p{};
    p.keys = sel_keys; p.N = n_sel; p.kprime = kp_sel; p.d = a.d;
    p.fr = fr; p.W1 = a.w1u; p.x = reinterpret_cast<const uint4*>(a.x);
    p.cand = a.cand; p.cand_out = a.cand_out; p.n_cand = a.n_cand; p.h = a.h; p.gs = gs; p.hg = a.hg;
    p.sparse_blocks = G; p.Wd = a.dense_w1u; p.m1 = a.m1; p.hd = a.h_dense;
    const int dense_blocks = (a.m1 + kGW * kGatherRows - 1) / (kGW * kGatherRows);
    e = lowrank ? launch(k_fast_gather<uint64_t>, dim3(G + dense_blocks), dim3(kGT), (size_t)a.d * 4, s, p)
                : launch(k_fast_gather<uint32_t>, dim3(G + dense_blocks), dim3(kGT), (size_t)a.d * 4, s, p);
    if (e != hipSuccess) return e;
    if ((e = mark(2)) != hipSuccess) return e;
  }
  int rg, cs;
  ffn_fast_shape(a.d, a.k, &rg, &cs);
  const int dense_groups = ffn_fast_dense_groups(a.m1);
  const bool direct = rg + dense_groups == 1;  // the second-layer kernel writes y itself
  {
    FastW2Params p{};
    p.h = sel_h; p.n = kp_sel; p.k = k_sel; p.d = a.d; p.fr = fr; p.cand = a.cand; p.W2 = a.w2u;
    p.topk_idx = a.topk_idx; p.topk_val = a.topk_val; p.out = direct ? a.y : a.partial; p.row_groups = rg;
    p.col_slices = cs;
    p.gs = gs; p.unit_h = a.h;
    p.dense_groups = dense_groups; p.W2d = a.dense_w2u; p.hd = a.h_dense; p.m1 = a.m1;
    e = launch(k_fast_w2, dim3((rg + dense_groups) * cs), dim3(kWT), 0, s, p);
    if (e != hipSuccess) return e;
    if ((e = mark(3)) != hipSuccess) return e;
  }
  if (!direct) {
    e = launch(k_fast_reduce, dim3((a.d + 255) / 256), dim3(256), 0, s, a.partial, rg + dense_groups, a.d, a.y);
    if (e != hipSuccess) return e;
  }
  return mark(4);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_fast(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
