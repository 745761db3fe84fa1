// HiRE-FFN with the distributed approximate top-k of arXiv 2402.09360, Algorithm 2 (DA-TOP-k), with every
// "machine" of the algorithm a workgroup of one GPU: the hidden units are cut into s contiguous shards, shard i
// runs Algorithm 1 on its own N/s units with the quotas k'/s and k/s, and the shards' second-layer contributions
// are summed (eq. (4)).  No threshold has to be agreed on across the device, so a whole step is one kernel with
// no dependency between workgroups plus a small reduction:
//
//   k_ffn_shard   one workgroup per shard: int8 token -> integer scores of the shard's rows (int4 codes, dot4)
//                 -> keys in LDS -> top k'/s by rank counting -> (batch) union -> exact fp64 pre-activations of
//                 the shortlisted rows -> top k/s -> fp32 partial output row of the shard
//   k_shard_reduce  y[b] = sum over shards of the partial rows, in a fixed order
//
// A shard is small (64 units at s = 256 for d_ff = 16384), so both selections are done by counting, for every
// entry, how many entries beat it (larger value, or equal value and lower index): exact, tie rule included,
// and a few LDS reads per thread.  Each phase issues all of its row loads before it uses any of them, spread over
// the workgroup's 16 waves: four packed int4 rows per wave while scoring, one bf16 row per wave in the exact
// stage, four per thread in the second layer.
//
// Batches are handled token after token (tokens staged in LDS one at a time, rows re-read through the caches):
// correct for any batch size, tuned for one token.
#include "device_utils.h"
#include "kernels.h"
#include "select.h"

namespace hire {

// 16 waves per workgroup: with one workgroup per CU every phase is bound by how many waves issue instructions
// and hold loads in flight, not by registers or LDS.
constexpr int kShThreads = 1024;
constexpr int kShWaves = kShThreads / kWave;

__device__ __forceinline__ float shard_block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if (lane_id() == 0) red[wave_id()] = v;
  __syncthreads();
  float m = red[0];
#pragma unroll
  for (int u = 1; u < kShWaves; ++u) m = fmaxf(m, red[u]);
  return m;
}

// flag[i] = 1 for the `want` entries of v[0..n) that rank first by (value descending, index ascending).
// v is padded to a multiple of four entries with values below every real one (the values here are >= 0), so that
// the inner loop reads four entries at a time and the reads pipeline.  Short rows are shared out: with n <= 512
// several threads count over a part of the row each for every entry and add their counts in beat[], which must
// hold n zeros on entry and is left zeroed.  or_into: keep flags that are already set (union
// over tokens).  Ends with a barrier.
template <typename T>
__device__ __forceinline__ void rank_flags(const T* v, int n, int want, int* flag, int* beat, bool or_into) {
  const int tid = (int)threadIdx.x;
  if (n <= kShThreads / 2) {
    int shift = 6;
    while ((1 << shift) < n) ++shift;
    const int parts = kShThreads >> shift;
    const int i = tid & ((1 << shift) - 1), part = tid >> shift;
    const int per = (((n + parts - 1) / parts) + 3) & ~3;  // whole groups of four per part
    const int lo = part * per, hi = min(lo + per, (n + 3) & ~3);
    if (i < n) {
      const T vi = v[i];
      int cnt = 0;
      for (int j0 = lo; j0 < hi; j0 += 4) {
        T vj[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) vj[u] = v[j0 + u];
#pragma unroll
        for (int u = 0; u < 4; ++u) cnt += (vj[u] > vi || (vj[u] == vi && j0 + u < i)) ? 1 : 0;
      }
      if (cnt) atomicAdd(&beat[i], cnt);
    }
    __syncthreads();
    if (tid < n) {
      const int f = beat[tid] < want ? 1 : 0;
      beat[tid] = 0;
      flag[tid] = or_into ? (flag[tid] | f) : f;
    }
    __syncthreads();
    return;
  }
  for (int i = tid; i < n; i += kShThreads) {
    const T vi = v[i];
    int cnt = 0;
    for (int j0 = 0; j0 < n; j0 += 4) {
      T vj[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) vj[u] = v[j0 + u];
#pragma unroll
      for (int u = 0; u < 4; ++u) cnt += (vj[u] > vi || (vj[u] == vi && j0 + u < i)) ? 1 : 0;
    }
    const int f = cnt < want ? 1 : 0;
    flag[i] = or_into ? (flag[i] | f) : f;
  }
  __syncthreads();
}

// The same selection for a row of at most 64 entries by ONE wave (lane i counts for entry i; the other waves wait
// at the caller's barrier and leave it the instruction issue): returns the selected entries as a bit mask.
template <typename T>
__device__ __forceinline__ uint64_t wave_rank_mask(const T* v, int n, int want) {
  const int i = lane_id();
  const T vi = v[min(i, n - 1)];
  int cnt = 0;
  for (int j0 = 0; j0 < n; j0 += 4) {
    T vj[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) vj[u] = v[j0 + u];
#pragma unroll
    for (int u = 0; u < 4; ++u) cnt += (vj[u] > vi || (vj[u] == vi && j0 + u < i)) ? 1 : 0;
  }
  return __ballot(i < n && cnt < want);
}

// list[0..) = the indices i < n with flag[i] set, ascending; returns how many (to every thread).  256 entries per
// round of kShThreads entries: ballot and lane prefix inside a wave, the waves' counts through LDS.  Ends with a
// barrier.
__device__ __forceinline__ int compact_flags(const int* flag, int n, int* list, int* wave_cnt) {
  const int lane = lane_id(), w = wave_id();
  if (n <= kWave) {  // one wave does it
    if (w == 0) {
      const bool f = lane < n && flag[lane] != 0;
      const uint64_t mask = __ballot(f);
      if (f) list[mask_prefix(mask)] = lane;
      if (lane == 0) wave_cnt[0] = __popcll(mask);
    }
    __syncthreads();
    return wave_cnt[0];
  }
  int base = 0;
  for (int i0 = 0; i0 < n; i0 += kShThreads) {
    const int i = i0 + (int)threadIdx.x;
    const bool f = i < n && flag[i] != 0;
    const uint64_t mask = __ballot(f);
    if (lane == 0) wave_cnt[w] = __popcll(mask);
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int u = 0; u < kShWaves; ++u) {
      const int c = wave_cnt[u];
      off += u < w ? c : 0;
      tot += c;
    }
    if (f) list[base + off + mask_prefix(mask)] = i;
    base += tot;
    __syncthreads();
  }
  return base;
}

// CH: 16-byte chunks of a packed int4 row per lane (d <= 2048 * CH).
template <int CH>
__global__ __launch_bounds__(kShThreads) void k_ffn_shard(
    const uint4* __restrict__ q4, const float* __restrict__ scale, const uint16_t* __restrict__ w1u,
    const uint16_t* __restrict__ w2u, const uint16_t* __restrict__ x, int B, int N, int d, int Ls, int kps, int ks,
    int cap, float* __restrict__ partial, int32_t* __restrict__ topk_idx, float* __restrict__ topk_val,
    int32_t* __restrict__ cand, int32_t* __restrict__ n_cand, int32_t* __restrict__ acc_out) {
  constexpr int kRowsPerWave = 4 / CH;   // packed rows a wave has in flight while scoring
  constexpr int kExactRows = 1;          // bf16 rows a wave has in flight in the exact stage
  constexpr int kXch = 4 * CH;           // 16-byte chunks of a bf16 row per lane
  extern __shared__ uint4 lds[];
  __shared__ float red[kShWaves];
  __shared__ int wave_cnt[kShWaves];
  const int cpr = d / 32, c8 = d / 8;
  uint4* xb = lds;                                   // [d/8]  token, raw bf16
  uint4* xq = xb + c8;                               // [d/16] token, int8
  const int Lp = (Ls + 3) & ~3;                      // padded to whole groups of four for the rank counting
  double* hv = reinterpret_cast<double*>(xq + d / 16);  // [Lp] exact pre-activations of the union
  float* keys = reinterpret_cast<float*>(hv + Lp);   // [Lp]
  int* uflag = reinterpret_cast<int*>(keys + Lp);    // [Ls] unit is in the union
  int* ulist = uflag + Ls;                           // [Ls] the union, ascending local unit numbers
  int* sflag = ulist + Ls;                           // [Ls] union entry is selected for the token
  int* spos = sflag + Ls;                            // [Ls] the selected union entries, ascending
  int* beat = spos + Ls;                             // [Ls] rank counters of short rows, zero between uses
  const int sh = (int)blockIdx.x, tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const size_t unit0 = (size_t)sh * Ls;

  // token b into LDS: raw bf16 and, for the scorer, int8 with the per-token scale amax / 127
  // In three steps, so that the packed rows of the first scoring trip can be requested between them: loads
  // return in issue order, so the token must not queue behind the rows, and the rows should fly while the token
  // is quantised.
  constexpr int kXreg = (2048 * CH / 8 + kShThreads - 1) / kShThreads;  // 16-byte chunks of the token per thread
  uint4 xreg[kXreg];
  auto request_token = [&](int b) {
    const uint4* xr = reinterpret_cast<const uint4*>(x + (size_t)b * d);
#pragma unroll
    for (int u = 0; u < kXreg; ++u) xreg[u] = xr[min(tid + u * kShThreads, c8 - 1)];
  };
  auto token_to_lds = [&]() -> float {  // returns this thread's share of max |x_i|
    float amax = 0.0f;
#pragma unroll
    for (int u = 0; u < kXreg; ++u) {
      const int c = tid + u * kShThreads;
      if (c >= c8) continue;
      const uint4 v = xreg[u];
      xb[c] = v;
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(wd[q])), fabsf(bf16_hi(wd[q]))));
    }
    return amax;
  };
  auto quantise_token = [&](float amax) {
    amax = shard_block_max(amax, red);  // its barriers also publish xb
    float sx = __fdiv_rn(amax, 127.0f);
    if (amax == 0.0f) sx = 1.0f;
    auto code = [&](float f) -> uint32_t {
      float r = rintf(__fdiv_rn(f, sx));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      return (uint32_t)((int)r) & 0xFFu;
    };
    for (int c = tid; c < c8; c += kShThreads) {
      const uint4 v = xb[c];
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
      uint2 o;
      o.x = code(bf16_lo(wd[0])) | code(bf16_hi(wd[0])) << 8 | code(bf16_lo(wd[1])) << 16 | code(bf16_hi(wd[1])) << 24;
      o.y = code(bf16_lo(wd[2])) | code(bf16_hi(wd[2])) << 8 | code(bf16_lo(wd[3])) << 16 | code(bf16_hi(wd[3])) << 24;
      reinterpret_cast<uint2*>(xq)[c] = o;
    }
    __syncthreads();
  };

  HIRE_TS(0);
  for (int i = tid; i < Ls; i += kShThreads) {
    uflag[i] = 0;
    beat[i] = 0;
  }
  if (tid < Lp - Ls) keys[Ls + tid] = -1.0f;  // padding ranks below every key (keys are >= 0 after the ReLU)

  uint4 wv[kRowsPerWave][CH];
  const uint4* q4s = q4 + unit0 * cpr;  // the shard's packed rows; offsets inside a shard fit 32 bits
  auto fetch_packed = [&](int r0) {
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {  // clamped and unconditional: one batch of loads
      const int row = min(r0 + rr, Ls - 1) * cpr;
#pragma unroll
      for (int u = 0; u < CH; ++u) wv[rr][u] = load_streaming(&q4s[row + min(lane + u * kWave, cpr - 1)]);
    }
  };

  // ---- every token's shortlist of k'/s units, marked in the union flags ----
  for (int b = 0; b < B; ++b) {
    const int first = w * kRowsPerWave;
    request_token(b);
    const float amax = token_to_lds();
    __builtin_amdgcn_sched_barrier(0);
    if (first < Ls) fetch_packed(first);  // in flight while the token is quantised
    __builtin_amdgcn_sched_barrier(0);
    quantise_token(amax);
    HIRE_TS(1);
    for (int r0 = first; r0 < Ls; r0 += kShWaves * kRowsPerWave) {
      if (r0 != first) fetch_packed(r0);
      int acc[kRowsPerWave];
#pragma unroll
      for (int rr = 0; rr < kRowsPerWave; ++rr) acc[rr] = 0;
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int c = lane + u * kWave;
        if (c < cpr) {
          const uint4 xa = xq[2 * c], xc = xq[2 * c + 1];
          const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
#pragma unroll
          for (int rr = 0; rr < kRowsPerWave; ++rr) {
            const uint32_t wd[4] = {wv[rr][u].x, wv[rr][u].y, wv[rr][u].z, wv[rr][u].w};
            int a = acc[rr];
#pragma unroll
            for (int t = 0; t < 4; ++t) {  // a byte holds two codes: 16 * code from the high nibble, then the low one
              a = __builtin_amdgcn_sdot4((int)(wd[t] & 0xF0F0F0F0u), xd[2 * t], a, false);
              a = __builtin_amdgcn_sdot4((int)((wd[t] << 4) & 0xF0F0F0F0u), xd[2 * t + 1], a, false);
            }
            acc[rr] = a;
          }
        }
      }
      int mine = 0;
#pragma unroll
      for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int sum = wave_sum(acc[rr]) >> 4;  // every partial is a multiple of 16
        mine = lane == rr ? sum : mine;
      }
      if (lane < kRowsPerWave && r0 + lane < Ls) {
        const size_t j = unit0 + r0 + lane;
        float key = (float)mine * scale[j];
        key = key > 0.0f ? key : 0.0f;  // phi = ReLU; also turns -0 into +0
        keys[r0 + lane] = key;
        if (acc_out) acc_out[(size_t)b * N + j] = mine;
      }
    }
    __syncthreads();
    HIRE_TS(2);
    rank_flags<float>(keys, Ls, kps, uflag, beat, true);
    HIRE_TS(3);
  }
  const int n_u = compact_flags(uflag, Ls, ulist, wave_cnt);
  if (cand != nullptr)
    for (int t = tid; t < n_u; t += kShThreads) cand[(size_t)sh * cap + t] = (int32_t)unit0 + ulist[t];
  if (n_cand != nullptr && tid == 0) n_cand[sh] = n_u;
  HIRE_TS(4);

  // ---- per token: exact pre-activations on the union, top k/s, partial second-layer row ----
  const uint4* w1s = reinterpret_cast<const uint4*>(w1u + unit0 * d);  // the shard's rows, 16-byte chunks
  for (int b = 0; b < B; ++b) {
    if (B > 1) {
      request_token(b);
      token_to_lds();
      __syncthreads();
    }
    for (int t0 = w * kExactRows; t0 < n_u; t0 += kShWaves * kExactRows) {
      uint4 ev[kExactRows][kXch];
#pragma unroll
      for (int rr = 0; rr < kExactRows; ++rr) {
        const int row = ulist[min(t0 + rr, n_u - 1)] * c8;
#pragma unroll
        for (int u = 0; u < kXch; ++u) ev[rr][u] = load_streaming(&w1s[row + min(lane + u * kWave, c8 - 1)]);
      }
      double acc[kExactRows];
#pragma unroll
      for (int rr = 0; rr < kExactRows; ++rr) acc[rr] = 0.0;
#pragma unroll
      for (int u = 0; u < kXch; ++u) {
        const int c = lane + u * kWave;
        if (c < c8) {
          const uint4 xv = xb[c];
          const uint32_t xd[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
          for (int rr = 0; rr < kExactRows; ++rr) {
            const uint32_t wd[4] = {ev[rr][u].x, ev[rr][u].y, ev[rr][u].z, ev[rr][u].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // bf16 x bf16 is exact in fp32; the sum runs in fp64
              acc[rr] += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
              acc[rr] += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
            }
          }
        }
      }
#pragma unroll
      for (int rr = 0; rr < kExactRows; ++rr) {
        double s = wave_sum(acc[rr]);
        s = s > 0.0 ? s : 0.0;
        if (lane == 0 && t0 + rr < n_u) hv[t0 + rr] = s;
      }
    }
    HIRE_TS(5);
    if (tid < ((n_u + 3) & ~3) - n_u) hv[n_u + tid] = -1.0;  // padding ranks below every activation (>= 0)
    __syncthreads();
    if (n_u <= kWave) {
      if (w == 0) {
        const uint64_t m = wave_rank_mask<double>(hv, n_u, ks);
        if ((m >> lane) & 1) spos[mask_prefix(m)] = lane;
      }
      __syncthreads();
    } else {
      rank_flags<double>(hv, n_u, ks, sflag, beat, false);
      compact_flags(sflag, n_u, spos, wave_cnt);  // exactly ks entries
    }
    HIRE_TS(6);
    for (int t = tid; t < ks; t += kShThreads) {
      const size_t o = (size_t)b * ((size_t)ks * gridDim.x) + (size_t)sh * ks + t;
      if (topk_idx) topk_idx[o] = (int32_t)unit0 + ulist[spos[t]];
      if (topk_val) topk_val[o] = (float)hv[spos[t]];
    }
    // second layer: every thread owns eight columns; four rows in flight, added in selection order
    for (int col = tid * 8; col < d; col += kShThreads * 8) {
      float a[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) a[q] = 0.0f;
      for (int t0 = 0; t0 < ks; t0 += 4) {
        uint4 rv[4];
        float cf[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int p = spos[min(t0 + u, ks - 1)];
          rv[u] = load_streaming(reinterpret_cast<const uint4*>(w2u + unit0 * d) + (ulist[p] * c8 + (col >> 3)));
          cf[u] = t0 + u < ks ? (float)hv[p] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float wf[8] = {bf16_lo(rv[u].x), bf16_hi(rv[u].x), bf16_lo(rv[u].y), bf16_hi(rv[u].y),
                               bf16_lo(rv[u].z), bf16_hi(rv[u].z), bf16_lo(rv[u].w), bf16_hi(rv[u].w)};
#pragma unroll
          for (int q = 0; q < 8; ++q) a[q] = fmaf(cf[u], wf[q], a[q]);
        }
      }
      float4* out = reinterpret_cast<float4*>(partial + ((size_t)sh * B + b) * d + col);
      out[0] = make_float4(a[0], a[1], a[2], a[3]);
      out[1] = make_float4(a[4], a[5], a[6], a[7]);
    }
    HIRE_TS(7);
    __syncthreads();  // hv, the flags and the token are reused by the next token
  }
}

// y[b, col] = sum over the shards of partial[shard, b, col]: 64 columns per workgroup, the shards in four
// contiguous quarters (one per wave, 16 loads in flight), the quarters added in order.
__global__ __launch_bounds__(kShThreads) void k_shard_reduce(const float* __restrict__ partial, int shards, int B,
                                                             int d, float* __restrict__ y) {
  __shared__ float red[4][kWave];
  const int lane = lane_id(), q = wave_id(), b = (int)blockIdx.y;
  const int col = min((int)blockIdx.x * kWave + lane, d - 1);
  const int per = (shards + 3) / 4;
  const int lo = q * per, hi = min(shards, lo + per);
  float s = 0.0f;
  for (int s0 = lo; s0 < hi; s0 += 16) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = partial[((size_t)min(s0 + u, shards - 1) * B + b) * d + col];
#pragma unroll
    for (int u = 0; u < 16; ++u) s += s0 + u < hi ? v[u] : 0.0f;
  }
  red[q][lane] = s;
  __syncthreads();
  if (q == 0 && (int)blockIdx.x * kWave + lane < d)
    y[(size_t)b * d + col] = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
}

bool ffn_shard_supported(int N, int d, int shards) {
  return shards >= 1 && N % shards == 0 && N / shards <= kShardMaxUnits && d % 32 == 0 && d >= 32 && d <= 8192;
}

size_t ffn_shard_partial_floats(int B, int d, int shards) { return (size_t)shards * B * d; }

hipError_t launch_ffn_shard(const FfnShardArgs& a, hipStream_t s) {
  const int Ls = a.N / a.shards, kps = a.kprime / a.shards, ks = a.k / a.shards;
  const int cap = (int)((long long)a.B * kps < (long long)Ls ? a.B * kps : Ls);
  const size_t lds = (size_t)a.d * 3 + (size_t)((Ls + 3) & ~3) * (8 + 4) + (size_t)Ls * (5 * 4);
  const uint4* q = reinterpret_cast<const uint4*>(a.q4);
  const dim3 grid(a.shards), block(kShThreads);
  hipError_t e;
  if (a.d <= 2048)
    e = launch(k_ffn_shard<1>, grid, block, lds, s, q, a.q4_scale, a.w1u, a.w2u, a.x, a.B, a.N, a.d, Ls, kps, ks, cap,
               a.partial, a.topk_idx, a.topk_val, a.cand, a.n_cand, a.scorer_acc);
  else if (a.d <= 4096)
    e = launch(k_ffn_shard<2>, grid, block, lds, s, q, a.q4_scale, a.w1u, a.w2u, a.x, a.B, a.N, a.d, Ls, kps, ks, cap,
               a.partial, a.topk_idx, a.topk_val, a.cand, a.n_cand, a.scorer_acc);
  else
    e = launch(k_ffn_shard<4>, grid, block, lds, s, q, a.q4_scale, a.w1u, a.w2u, a.x, a.B, a.N, a.d, Ls, kps, ks, cap,
               a.partial, a.topk_idx, a.topk_val, a.cand, a.n_cand, a.scorer_acc);
  return e;
}

hipError_t launch_ffn_shard_reduce(const FfnShardArgs& a, hipStream_t s) {
  return launch(k_shard_reduce, dim3((a.d + kWave - 1) / kWave, a.B), dim3(kShThreads), 0, s, a.partial, a.shards, a.B,
                a.d, a.y);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_shard(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
