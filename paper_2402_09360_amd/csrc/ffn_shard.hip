// HiRE-FFN with the distributed approximate top-k of arXiv 2402.09360, Algorithm 2 (DA-TOP-k), with every
// "machine" of the algorithm a workgroup of one GPU: the hidden units are cut into s contiguous shards, shard i
// runs Algorithm 1 on its own N/s units with the quotas k'/s and k/s (rounded up), and the shards' second-layer contributions
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
// Batches are taken in bundles of up to four tokens that share every loaded row; larger batches run bundle after
// bundle (rows re-read through the caches) with the union flags carried along: correct for any batch size, tuned
// for one to four tokens.
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

// CH: 16-byte chunks of a packed int4 row per lane (d <= 2048 * CH).  The batch is taken BT tokens at a time: the
// tokens of such a bundle sit in LDS side by side and every row that is loaded - packed for the scores, bf16 for
// the exact stage - is used for all of them before the next bundle re-reads it.
template <int CH, int BT>
__global__ __launch_bounds__(kShThreads) void k_ffn_shard(
    const uint4* __restrict__ q4, const float* __restrict__ scale, const uint16_t* __restrict__ w1u,
    const uint16_t* __restrict__ w2u, const uint16_t* __restrict__ x, int B, int N, int d, int Ls, int kps, int ks,
    int cap, float* __restrict__ partial, int32_t* __restrict__ topk_idx, float* __restrict__ topk_val,
    int32_t* __restrict__ cand, int32_t* __restrict__ n_cand, int32_t* __restrict__ acc_out) {
  constexpr int kRowsPerWave = BT >= 4 ? 2 : 4 / CH;  // packed rows a wave has in flight while scoring (registers)
  constexpr int kXch = 4 * CH;           // 16-byte chunks of a bf16 row per lane
  extern __shared__ uint4 lds[];
  __shared__ uint32_t amax_sh[BT];
  __shared__ int wave_cnt[kShWaves];
  const int cpr = d / 32, c8 = d / 8, c16 = d / 16;
  const int Lp = (Ls + 3) & ~3;                      // padded to whole groups of four for the rank counting
  uint4* xb = lds;                                   // [BT][d/8]  tokens, raw bf16
  uint4* xq = xb + BT * c8;                          // [BT][d/16] tokens, int8
  double* hv = reinterpret_cast<double*>(xq + BT * c16);  // [BT][Lp] exact pre-activations on the union
  float* keys = reinterpret_cast<float*>(hv + BT * Lp);   // [BT][Lp]
  int* uflag = reinterpret_cast<int*>(keys + BT * Lp);    // [Ls] unit is in the union
  int* ulist = uflag + Ls;                           // [Ls] the union, ascending local unit numbers
  int* sflag = ulist + Ls;                           // [Ls] union entry is selected for the token
  int* spos = sflag + Ls;                            // [BT][Ls] every token's selected union entries, ascending
  int* beat = spos + BT * Ls;                        // [Ls] rank counters of short rows, zero between uses
  const int sh = (int)blockIdx.x, tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  const size_t unit0 = (size_t)sh * Ls;

  // Tokens b0 .. b0 + BT - 1 (clamped to the batch: the spare slots of the last bundle repeat its last token and
  // their results are dropped) into LDS: raw bf16 and, for the scorer, int8 with the per-token scale amax / 127.
  // The bundle's 16-byte chunks are dealt out flat over the threads.  In three steps, so that the packed rows of
  // the first scoring trip can be requested between them: loads return in issue order, so the tokens must not
  // queue behind the rows, and the rows should fly while the tokens are quantised.
  constexpr int kXreg = (BT * 2048 * CH / 8 + kShThreads - 1) / kShThreads;  // chunks of the bundle per thread
  uint4 xreg[kXreg];
  int xbb[kXreg], xc[kXreg];  // the token of the bundle and the chunk of it that this thread stages
#pragma unroll
  for (int u = 0; u < kXreg; ++u) {
    const int idx = min(tid + u * kShThreads, BT * c8 - 1);
    xbb[u] = BT == 1 ? 0 : idx / c8;  // one division per thread and kernel: instructions are dear with 16 waves
    xc[u] = idx - xbb[u] * c8;
  }
  auto request_tokens = [&](int b0) {
#pragma unroll
    for (int u = 0; u < kXreg; ++u)
      xreg[u] = reinterpret_cast<const uint4*>(x)[min(b0 + xbb[u], B - 1) * c8 + xc[u]];
  };
  // with want_amax: max |x_i| of every token into amax_sh (as bits; zero on entry, see quantise_tokens)
  auto tokens_to_lds = [&](bool want_amax) {
#pragma unroll
    for (int u = 0; u < kXreg; ++u) {
      const int idx = tid + u * kShThreads;
      if (idx >= BT * c8) continue;
      const uint4 v = xreg[u];
      xb[idx] = v;
      if (want_amax) {
        const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
        float amax = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(wd[q])), fabsf(bf16_hi(wd[q]))));
        // non-negative floats order like their bits; a wave whose chunks all belong to one token (the usual
        // case) sends one atomic
        if (c8 % kWave == 0) {
          amax = wave_max(amax);
          if (lane == 0) atomicMax(&amax_sh[xbb[u]], __float_as_uint(amax));
        } else {
          atomicMax(&amax_sh[xbb[u]], __float_as_uint(amax));
        }
      }
    }
  };
  auto quantise_tokens = [&]() {
    __syncthreads();  // amax_sh and xb are complete
#pragma unroll
    for (int u = 0; u < kXreg; ++u) {
      const int idx = tid + u * kShThreads;
      if (idx >= BT * c8) continue;
      const float m = __uint_as_float(amax_sh[xbb[u]]);
      float sx = __fdiv_rn(m, 127.0f);
      if (m == 0.0f) sx = 1.0f;
      auto code = [&](float f) -> uint32_t {
        float r = rintf(__fdiv_rn(f, sx));
        r = fminf(fmaxf(r, -127.0f), 127.0f);
        return (uint32_t)((int)r) & 0xFFu;
      };
      const uint4 v = xreg[u];
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
      uint2 o;
      o.x = code(bf16_lo(wd[0])) | code(bf16_hi(wd[0])) << 8 | code(bf16_lo(wd[1])) << 16 | code(bf16_hi(wd[1])) << 24;
      o.y = code(bf16_lo(wd[2])) | code(bf16_hi(wd[2])) << 8 | code(bf16_lo(wd[3])) << 16 | code(bf16_hi(wd[3])) << 24;
      reinterpret_cast<uint2*>(xq)[idx] = o;  // [BT][d/16] uint4 = [BT][d/8] uint2
    }
    __syncthreads();
    if (tid < BT) amax_sh[tid] = 0u;  // for the next bundle; the barriers of the scoring that follows publish it
  };

  // the first bundle's loads go out before anything else is computed: with 16 waves on the CU every instruction
  // in front of them delays them by several nanoseconds
  HIRE_TS(0);
  request_tokens(0);
  __builtin_amdgcn_sched_barrier(0);
  if (tid < BT) amax_sh[tid] = 0u;
  __syncthreads();  // (waits for the tokens as well, which everything below needs anyway)
  for (int i = tid; i < Ls; i += kShThreads) {
    uflag[i] = 0;
    beat[i] = 0;
  }
  if (tid < BT * (Lp - Ls))  // padding ranks below every key (keys are >= 0 after the ReLU)
    keys[(tid / (Lp - Ls)) * Lp + Ls + tid % (Lp - Ls)] = -1.0f;

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
  for (int b0 = 0; b0 < B; b0 += BT) {
    const int nb = min(BT, B - b0);
    const int first = w * kRowsPerWave;
    if (b0 > 0) request_tokens(b0);
    tokens_to_lds(true);
    __builtin_amdgcn_sched_barrier(0);
    if (first < Ls) fetch_packed(first);  // in flight while the tokens are quantised
    __builtin_amdgcn_sched_barrier(0);
    quantise_tokens();
    HIRE_TS(1);
    for (int r0 = first; r0 < Ls; r0 += kShWaves * kRowsPerWave) {
      if (r0 != first) fetch_packed(r0);
      int acc[BT][kRowsPerWave];
#pragma unroll
      for (int bb = 0; bb < BT; ++bb)
#pragma unroll
        for (int rr = 0; rr < kRowsPerWave; ++rr) acc[bb][rr] = 0;
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int c = lane + u * kWave;
        if (c < cpr) {
#pragma unroll
          for (int bb = 0; bb < BT; ++bb) {
            const uint4 xa = xq[bb * c16 + 2 * c], xc = xq[bb * c16 + 2 * c + 1];
            const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w,
                               (int)xc.x, (int)xc.y, (int)xc.z, (int)xc.w};
#pragma unroll
            for (int rr = 0; rr < kRowsPerWave; ++rr) {
              const uint32_t wd[4] = {wv[rr][u].x, wv[rr][u].y, wv[rr][u].z, wv[rr][u].w};
              int a = acc[bb][rr];
#pragma unroll
              for (int t = 0; t < 4; ++t) {  // a byte holds two codes: 16 * code from the high nibble, then the low one
                a = __builtin_amdgcn_sdot4((int)(wd[t] & 0xF0F0F0F0u), xd[2 * t], a, false);
                a = __builtin_amdgcn_sdot4((int)((wd[t] << 4) & 0xF0F0F0F0u), xd[2 * t + 1], a, false);
              }
              acc[bb][rr] = a;
            }
          }
        }
      }
#pragma unroll
      for (int bb = 0; bb < BT; ++bb) {
        int mine = 0;
#pragma unroll
        for (int rr = 0; rr < kRowsPerWave; ++rr) {
          const int sum = wave_sum(acc[bb][rr]) >> 4;  // every partial is a multiple of 16
          mine = lane == rr ? sum : mine;
        }
        if (lane < kRowsPerWave && r0 + lane < Ls && bb < nb) {
          const size_t j = unit0 + r0 + lane;
          float key = (float)mine * scale[j];
          key = key > 0.0f ? key : 0.0f;  // phi = ReLU; also turns -0 into +0
          keys[bb * Lp + r0 + lane] = key;
          if (acc_out) acc_out[(size_t)(b0 + bb) * N + j] = mine;
        }
      }
    }
    __syncthreads();
    HIRE_TS(2);
    for (int bb = 0; bb < nb; ++bb) rank_flags<float>(keys + bb * Lp, Ls, kps, uflag, beat, true);
    HIRE_TS(3);
  }
  const int n_u = compact_flags(uflag, Ls, ulist, wave_cnt);
  if (cand != nullptr)
    for (int t = tid; t < n_u; t += kShThreads) cand[(size_t)sh * cap + t] = (int32_t)unit0 + ulist[t];
  if (n_cand != nullptr && tid == 0) n_cand[sh] = n_u;
  HIRE_TS(4);

  // ---- per token: exact pre-activations on the union, top k/s, partial second-layer row ----
  const uint4* w1s = reinterpret_cast<const uint4*>(w1u + unit0 * d);  // the shard's rows, 16-byte chunks
  const uint4* w2s = reinterpret_cast<const uint4*>(w2u + unit0 * d);
  const int n_up = (n_u + 3) & ~3;
  for (int b0 = 0; b0 < B; b0 += BT) {
    const int nb = min(BT, B - b0);
    if (B > BT) {  // a single bundle is still in LDS
      request_tokens(b0);
      tokens_to_lds(false);
      __syncthreads();
    }
    for (int t0 = w; t0 < n_u; t0 += kShWaves) {  // one bf16 row per wave in flight, used for every token
      uint4 ev[kXch];
      const int row = ulist[t0] * c8;
#pragma unroll
      for (int u = 0; u < kXch; ++u) ev[u] = load_streaming(&w1s[row + min(lane + u * kWave, c8 - 1)]);
      double acc[BT];
#pragma unroll
      for (int bb = 0; bb < BT; ++bb) acc[bb] = 0.0;
#pragma unroll
      for (int u = 0; u < kXch; ++u) {
        const int c = lane + u * kWave;
        if (c < c8) {
          const uint32_t wd[4] = {ev[u].x, ev[u].y, ev[u].z, ev[u].w};
          // the row's values widened once and used for every token; an fp64 FMA of two bf16 values rounds once,
          // exactly like adding their (exact) fp32 product
          double wdv[8];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            wdv[2 * q] = (double)bf16_lo(wd[q]);
            wdv[2 * q + 1] = (double)bf16_hi(wd[q]);
          }
#pragma unroll
          for (int bb = 0; bb < BT; ++bb) {
            const uint4 xv = xb[bb * c8 + c];
            const uint32_t xd[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              acc[bb] = fma(wdv[2 * q], (double)bf16_lo(xd[q]), acc[bb]);
              acc[bb] = fma(wdv[2 * q + 1], (double)bf16_hi(xd[q]), acc[bb]);
            }
          }
        }
      }
#pragma unroll
      for (int bb = 0; bb < BT; ++bb) {
        double s = wave_sum(acc[bb]);
        s = s > 0.0 ? s : 0.0;
        if (lane == 0) hv[bb * Lp + t0] = s;
      }
    }
    HIRE_TS(5);
    if (tid < BT * (n_up - n_u))  // padding ranks below every activation (>= 0)
      hv[(tid / (n_up - n_u)) * Lp + n_u + tid % (n_up - n_u)] = -1.0;
    __syncthreads();
    // the k/s survivors of every token of the bundle: spos[bb][0 .. ks)
    if (n_u <= kWave) {  // one wave per token, no barrier in between
      if (w < nb) {
        const uint64_t m = wave_rank_mask<double>(hv + w * Lp, n_u, ks);
        if ((m >> lane) & 1) spos[w * Ls + mask_prefix(m)] = lane;
      }
      __syncthreads();
    } else {
      for (int bb = 0; bb < nb; ++bb) {
        rank_flags<double>(hv + bb * Lp, n_u, ks, sflag, beat, false);
        compact_flags(sflag, n_u, spos + bb * Ls, wave_cnt);  // exactly ks entries
      }
    }
    HIRE_TS(6);
    for (int i = tid; i < nb * ks; i += kShThreads) {
      const int bb = i / ks, t = i - bb * ks, p = spos[bb * Ls + t];
      const size_t o = (size_t)(b0 + bb) * ((size_t)ks * gridDim.x) + (size_t)sh * ks + t;
      if (topk_idx) topk_idx[o] = (int32_t)unit0 + ulist[p];
      if (topk_val) topk_val[o] = (float)hv[bb * Lp + p];
    }
    // second layer: an item is eight columns of one token; four rows in flight, added in selection order
#pragma unroll
    for (int u = 0; u < kXreg; ++u) {  // the flat item numbering of the token staging
      const int bb = xbb[u], cc = xc[u];
      if (tid + u * kShThreads >= nb * c8) continue;
      const int* sp = spos + bb * Ls;
      const double* hb = hv + bb * Lp;
      float a[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) a[q] = 0.0f;
      for (int t0 = 0; t0 < ks; t0 += 4) {
        uint4 rv[4];
        float cf[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int p = sp[min(t0 + u, ks - 1)];
          rv[u] = load_streaming(&w2s[ulist[p] * c8 + cc]);
          cf[u] = t0 + u < ks ? (float)hb[p] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float wf[8] = {bf16_lo(rv[u].x), bf16_hi(rv[u].x), bf16_lo(rv[u].y), bf16_hi(rv[u].y),
                               bf16_lo(rv[u].z), bf16_hi(rv[u].z), bf16_lo(rv[u].w), bf16_hi(rv[u].w)};
#pragma unroll
          for (int q = 0; q < 8; ++q) a[q] = fmaf(cf[u], wf[q], a[q]);
        }
      }
      float4* out = reinterpret_cast<float4*>(partial + ((size_t)sh * B + b0 + bb) * d + cc * 8);
      out[0] = make_float4(a[0], a[1], a[2], a[3]);
      out[1] = make_float4(a[4], a[5], a[6], a[7]);
    }
    HIRE_TS(7);
    __syncthreads();  // hv, spos and the tokens are reused by the next bundle
  }
}

// y[b, col] = sum over the shards of partial[shard, b, col]: 64 columns per workgroup, the shards in four
// contiguous quarters (one per wave, 16 loads in flight), the quarters added in order.
constexpr int kShRedThreads = 256;  // four waves, one quarter of the shards each
__global__ __launch_bounds__(kShRedThreads) void k_shard_reduce(const float* __restrict__ partial, int shards, int B,
                                                                int d, float* __restrict__ y) {
  constexpr int kQuarters = kShRedThreads / kWave;
  static_assert(kQuarters == 4, "one row of red per wave of the workgroup");
  __shared__ float red[kQuarters][kWave];
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

template <int CH, int BT>
static hipError_t shard_launch(const FfnShardArgs& a, hipStream_t s) {
  // quotas that do not divide are rounded up (Algorithm 2 keeps ceil(k'/s), then ceil(k/s) per machine); since s
  // divides N and k <= k' <= N, ks <= kps <= Ls always holds
  const int Ls = a.N / a.shards, kps = (a.kprime + a.shards - 1) / a.shards, ks = (a.k + a.shards - 1) / a.shards;
  const int cap = (int)((long long)a.B * kps < (long long)Ls ? a.B * kps : Ls);
  const size_t lds = (size_t)BT * ((size_t)a.d * 3 + (size_t)((Ls + 3) & ~3) * (8 + 4)) + (size_t)Ls * ((4 + BT) * 4);
  static std::atomic<size_t> raised_to{0};  // bundles of several tokens with long shards pass the default limit
  if (const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(k_ffn_shard<CH, BT>), lds, raised_to);
      e != hipSuccess)
    return e;
  return launch(k_ffn_shard<CH, BT>, dim3(a.shards), dim3(kShThreads), lds, s, reinterpret_cast<const uint4*>(a.q4),
                a.q4_scale, a.w1u, a.w2u, a.x, a.B, a.N, a.d, Ls, kps, ks, cap, a.partial, a.topk_idx, a.topk_val,
                a.cand, a.n_cand, a.scorer_acc);
}

// Tokens side by side: as many as LDS (under 64 KB) and registers take; one token runs the leaner single variant.
hipError_t launch_ffn_shard(const FfnShardArgs& a, hipStream_t s) {
  if (a.d <= 2048) return a.B == 1 ? shard_launch<1, 1>(a, s) : shard_launch<1, 4>(a, s);
  if (a.d <= 4096) return a.B == 1 ? shard_launch<2, 1>(a, s) : shard_launch<2, 2>(a, s);
  return shard_launch<4, 1>(a, s);
}

hipError_t launch_ffn_shard_reduce(const FfnShardArgs& a, hipStream_t s) {
  return launch(k_shard_reduce, dim3((a.d + kWave - 1) / kWave, a.B), dim3(kShRedThreads), 0, s, a.partial, a.shards,
                a.B, a.d, a.y);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_shard(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
