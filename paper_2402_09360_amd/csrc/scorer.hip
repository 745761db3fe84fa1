// Compressed scorers of HiRE (arXiv 2402.09360, Algorithm 1 line 1, Sec. 3.2):
//   HiRE-Q : int4 copy of Z times int8 activations, int32 accumulation
//   HiRE-LR: Z1 Z2^T in bf16 with wide accumulation
// plus the one-off int4 packing of a weight matrix.
//
// Packed int4 layout (per row, cols/8 dwords): dword u holds codes 8u..8u+7;
// byte b of the dword carries code 8u+b in its high nibble and code 8u+4+b in
// its low nibble.  `w & 0xF0F0F0F0` and `(w << 4) & 0xF0F0F0F0` are then four
// signed bytes each, equal to 16*code, lined up with two consecutive dwords
// of int8 activations: two v_dot4 per dword, and one exact >> 4 at the end.
#include "device_utils.h"
#include "hist.h"
#include "kernels.h"

namespace hire {

__device__ __forceinline__ void zero_slice(uint32_t* p, int words) {
  if (p == nullptr) return;
  const int stride = (int)(gridDim.x * blockDim.x);
  for (int i = (int)(blockIdx.x * blockDim.x + threadIdx.x); i < words; i += stride) p[i] = 0u;
}

// Block-wide max of non-negative floats (256 threads).
__device__ __forceinline__ float block_max_256(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if (lane_id() == 0) red[wave_id()] = v;
  __syncthreads();
  float m = red[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) m = fmaxf(m, red[w]);
  return m;
}

// ---------------------------------------------------------------------------
// int4 packing: one block per row.
// max_scale: one word behind the codes that ends up holding the largest scale of any row that is not all zero (as
// float bits, which order like the positive numbers themselves); cleared before this kernel runs.
__global__ __launch_bounds__(256) void k_pack_int4(const uint16_t* __restrict__ w, int cols, uint32_t* __restrict__ q4,
                                                   float* __restrict__ scale, uint32_t* __restrict__ max_scale) {
  __shared__ float red[4];
  const int j = (int)blockIdx.x;
  const uint16_t* row = w + (size_t)j * cols;
  float amax = 0.0f;
  for (int i = (int)threadIdx.x; i < cols; i += 256) amax = fmaxf(amax, fabsf(bf16_to_f32(row[i])));
  amax = block_max_256(amax, red);
  float s = __fdiv_rn(amax, 7.0f);
  if (amax == 0.0f) s = 1.0f;
  if (threadIdx.x == 0) {
    scale[j] = s;
    if (amax != 0.0f) atomicMax(max_scale, __float_as_uint(s));
  }
  uint32_t* out = q4 + (size_t)j * (cols / 8);
  for (int u = (int)threadIdx.x; u < cols / 8; u += 256) {
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float r = rintf(__fdiv_rn(bf16_to_f32(row[8 * u + e]), s));
      r = fminf(fmaxf(r, -7.0f), 7.0f);
      const uint32_t nib = (uint32_t)((int)r) & 0xFu;
      const int byte = e & 3, high = e < 4;
      word |= nib << (8 * byte + (high ? 4 : 0));
    }
    out[u] = word;
  }
}

__global__ __launch_bounds__(256) void k_unpack_int4(const uint32_t* __restrict__ q4, int cols,
                                                     int8_t* __restrict__ codes) {
  const int j = (int)blockIdx.x;
  const uint32_t* in = q4 + (size_t)j * (cols / 8);
  int8_t* out = codes + (size_t)j * cols;
  for (int u = (int)threadIdx.x; u < cols / 8; u += 256) {
    const uint32_t word = in[u];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int byte = e & 3, high = e < 4;
      const uint32_t nib = (word >> (8 * byte + (high ? 4 : 0))) & 0xFu;
      out[8 * u + e] = (int8_t)((int)(nib << 28) >> 28);
    }
  }
}

// ---------------------------------------------------------------------------
// Per-token int8 activations: one block per token.
__global__ __launch_bounds__(256) void k_quantize_tokens(const uint16_t* __restrict__ x, int d, int8_t* __restrict__ xq,
                                                         float* __restrict__ sx, uint32_t* zero_ptr, int zero_words,
                                                         GeneralHeader* gh, unsigned long long sig) {
  __shared__ float red[4];
  zero_slice(zero_ptr, zero_words);
  if (blockIdx.x == 0) general_header_check(gh, sig);
  const int b = (int)blockIdx.x;
  const uint4* row = reinterpret_cast<const uint4*>(x + (size_t)b * d);  // d is a multiple of 32: whole 16-byte chunks
  const int chunks = d / 8;
  float amax = 0.0f;
  for (int c = (int)threadIdx.x; c < chunks; c += 256) {
    const uint4 v = row[c];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(w[q])), fabsf(bf16_hi(w[q]))));
  }
  amax = block_max_256(amax, red);
  float s = __fdiv_rn(amax, 127.0f);
  if (amax == 0.0f) s = 1.0f;
  if (threadIdx.x == 0) sx[b] = s;
  auto code = [&](float f) -> uint32_t {
    float r = rintf(__fdiv_rn(f, s));
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (uint32_t)((int)r) & 0xFFu;
  };
  for (int c = (int)threadIdx.x; c < chunks; c += 256) {
    const uint4 v = row[c];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint2 o;
    o.x = code(bf16_lo(w[0])) | code(bf16_hi(w[0])) << 8 | code(bf16_lo(w[1])) << 16 | code(bf16_hi(w[1])) << 24;
    o.y = code(bf16_lo(w[2])) | code(bf16_hi(w[2])) << 8 | code(bf16_lo(w[3])) << 16 | code(bf16_hi(w[3])) << 24;
    reinterpret_cast<uint2*>(xq + (size_t)b * d)[c] = o;
  }
}

// ---------------------------------------------------------------------------
// int4 x int8 scorer.  A wave owns RPW consecutive rows at a time; lane l
// handles the 16-byte chunks l, l+64, ... of each row (one chunk = 32 codes).
// The token tile's int8 activations sit in LDS.  With a histogram region the epilogue also counts every key
// into its token's fine histogram and leaves the workgroup's largest key per token behind: what the
// selection kernels need to find the k'-th largest key without a pass of their own.
constexpr int kScorerRPW = 4;

template <int BT>
__global__ __launch_bounds__(256) void k_scorer_int4(const uint4* __restrict__ q4, const float* __restrict__ scale,
                                                     const int8_t* __restrict__ xq, int B, int N, int d, int relu,
                                                     float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                     MultiRegion mr) {
  extern __shared__ uint4 xs[];  // [BT][d/16] : token tile, 16 int8 per uint4
  __shared__ uint32_t wmax_sh[4][BT];
  const bool hist_on = mr.hist != nullptr && multi_hist_ok(mr.hdr, B);
  const int cpr = d / 32;        // 16-byte chunks per packed row
  const int xv = d / 16;         // uint4 per token row of xq
  const int lane = lane_id();
  const int waves_per_block = (int)(blockDim.x >> 6);
  const int total_waves = (int)gridDim.x * waves_per_block;
  for (int b0 = 0; b0 < B; b0 += BT) {
    __syncthreads();
    for (int i = (int)threadIdx.x; i < BT * xv; i += (int)blockDim.x) {
      const int bb = i / xv, c = i - bb * xv;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (b0 + bb < B) v = reinterpret_cast<const uint4*>(xq + (size_t)(b0 + bb) * d)[c];
      xs[i] = v;
    }
    __syncthreads();
    uint32_t wmax[BT];
#pragma unroll
    for (int bb = 0; bb < BT; ++bb) wmax[bb] = 0u;
    for (int g = (int)blockIdx.x * waves_per_block + wave_id(); g * kScorerRPW < N; g += total_waves) {
      const int j0 = g * kScorerRPW;
      int acc[kScorerRPW][BT];
#pragma unroll
      for (int rr = 0; rr < kScorerRPW; ++rr)
#pragma unroll
        for (int bb = 0; bb < BT; ++bb) acc[rr][bb] = 0;
      for (int c = lane; c < cpr; c += kWave) {
        uint4 wv[kScorerRPW];
#pragma unroll
        for (int rr = 0; rr < kScorerRPW; ++rr) {
          const int j = min(j0 + rr, N - 1);
          wv[rr] = q4[(size_t)j * cpr + c];
        }
#pragma unroll
        for (int bb = 0; bb < BT; ++bb) {
          const uint4 xa = xs[bb * xv + 2 * c], xb = xs[bb * xv + 2 * c + 1];
          const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xb.x, (int)xb.y, (int)xb.z, (int)xb.w};
#pragma unroll
          for (int rr = 0; rr < kScorerRPW; ++rr) {
            const uint32_t wd[4] = {wv[rr].x, wv[rr].y, wv[rr].z, wv[rr].w};
            int a = acc[rr][bb];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const int hi = (int)(wd[t] & 0xF0F0F0F0u);
              const int lo = (int)((wd[t] << 4) & 0xF0F0F0F0u);
              a = __builtin_amdgcn_sdot4(hi, xd[2 * t], a, false);
              a = __builtin_amdgcn_sdot4(lo, xd[2 * t + 1], a, false);
            }
            acc[rr][bb] = a;
          }
        }
      }
#pragma unroll
      for (int rr = 0; rr < kScorerRPW; ++rr)
#pragma unroll
        for (int bb = 0; bb < BT; ++bb) {
          const int sum = wave_sum(acc[rr][bb]) >> 4;  // every partial is a multiple of 16
          const int j = j0 + rr, b = b0 + bb;
          if (lane == 0 && j < N && b < B) {
            float key = (float)sum * scale[j];
            if (relu) key = key > 0.0f ? key : 0.0f;
            if (key == 0.0f) key = 0.0f;
            keys[(size_t)b * N + j] = key;
            if (acc_out) acc_out[(size_t)b * N + j] = sum;
            const uint32_t ok = order_key(key);
            wmax[bb] = ok > wmax[bb] ? ok : wmax[bb];
            // ReLU zeros stay uncounted: they would all queue up on one counter, and a threshold among them
            // is the streaming selection's case anyway
            if (hist_on && !(relu && key == 0.0f))
              atomicAdd(&mr.hist[(size_t)b * kHistStride + kHistWindow + hist_bin(ok)], 1u);
          }
        }
    }
    if (mr.wgmax != nullptr) {
      if (lane == 0) {
#pragma unroll
        for (int bb = 0; bb < BT; ++bb) wmax_sh[wave_id()][bb] = wmax[bb];
      }
      __syncthreads();
      const int bb = (int)threadIdx.x;
      if (bb < BT && b0 + bb < B) {
        uint32_t m = 0u;
        for (int w = 0; w < waves_per_block; ++w) m = wmax_sh[w][bb] > m ? wmax_sh[w][bb] : m;
        mr.wgmax[(size_t)(b0 + bb) * kWgMaxSlots + blockIdx.x] = m;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// The same for one token and rows of at most 64 * CH 16-byte chunks (d <= 2048 * CH), software-pipelined: a wave
// holds two sets of four rows in registers and issues the loads of the next set before it reduces the current
// one, so that its memory latency overlaps its own arithmetic as well as other waves'.  Lanes 0..3 finish one row
// each (key, store, histogram atomic), so the four keys leave as one 16-byte store.  The kernel is the first of
// its step: every workgroup quantises the token into LDS itself (4 KB of bf16 from L2 is cheaper than a kernel of
// its own), and together they clear the words at zero_ptr and check the workspace's layout signature.
template <int CH>
__global__ __launch_bounds__(256) void k_scorer_int4_b1(const uint4* __restrict__ q4, const float* __restrict__ scale,
                                                        const uint16_t* __restrict__ x, int N, int d, int relu,
                                                        float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                        MultiRegion mr, uint32_t* zero_ptr, int zero_words,
                                                        GeneralHeader* gh, unsigned long long sig) {
  extern __shared__ uint4 xs[];  // [d/16] token, 16 int8 per uint4
  __shared__ uint32_t wmax_sh[4];
  __shared__ float red[4];
  zero_slice(zero_ptr, zero_words);
  if (blockIdx.x == 0) general_header_check(gh, sig);
  const int cpr = d / 32;
  const int lane = lane_id();
  const int total_waves = (int)gridDim.x * 4;
  const bool hist_on = mr.hist != nullptr && multi_hist_ok(mr.hdr, 1);
  const int groups = (N + kScorerRPW - 1) / kScorerRPW;

  auto fetch = [&](int g, uint4 (&wv)[kScorerRPW][CH]) {
#pragma unroll
    for (int rr = 0; rr < kScorerRPW; ++rr) {
      const uint4* row = q4 + (size_t)min(g * kScorerRPW + rr, N - 1) * cpr;
#pragma unroll
      for (int u = 0; u < CH; ++u) wv[rr][u] = load_streaming(&row[min(lane + u * kWave, cpr - 1)]);  // clamped, unconditional
    }
  };
  uint32_t wmax = 0u;
  auto finish = [&](int g, const uint4 (&wv)[kScorerRPW][CH]) {
    int acc[kScorerRPW];
#pragma unroll
    for (int rr = 0; rr < kScorerRPW; ++rr) acc[rr] = 0;
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const int c = lane + u * kWave;
      if (c < cpr) {
        const uint4 xa = xs[2 * c], xb = xs[2 * c + 1];
        const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xb.x, (int)xb.y, (int)xb.z, (int)xb.w};
#pragma unroll
        for (int rr = 0; rr < kScorerRPW; ++rr) {
          const uint32_t wd[4] = {wv[rr][u].x, wv[rr][u].y, wv[rr][u].z, wv[rr][u].w};
          int a = acc[rr];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            a = __builtin_amdgcn_sdot4((int)(wd[t] & 0xF0F0F0F0u), xd[2 * t], a, false);
            a = __builtin_amdgcn_sdot4((int)((wd[t] << 4) & 0xF0F0F0F0u), xd[2 * t + 1], a, false);
          }
          acc[rr] = a;
        }
      }
    }
    int mine = 0;
#pragma unroll
    for (int rr = 0; rr < kScorerRPW; ++rr) {
      const int sum = wave_sum(acc[rr]) >> 4;  // every partial is a multiple of 16
      mine = lane == rr ? sum : mine;
    }
    const int j = g * kScorerRPW + lane;
    if (lane < kScorerRPW && j < N) {
      float key = (float)mine * scale[j];
      if (relu) key = key > 0.0f ? key : 0.0f;
      if (key == 0.0f) key = 0.0f;
      keys[j] = key;
      if (acc_out) acc_out[j] = mine;
      const uint32_t ok = order_key(key);
      wmax = ok > wmax ? ok : wmax;
      if (hist_on && !(relu && key == 0.0f)) atomicAdd(&mr.hist[kHistWindow + hist_bin(ok)], 1u);
    }
  };

  uint4 wa[kScorerRPW][CH], wb[kScorerRPW][CH];
  int g = (int)blockIdx.x * 4 + wave_id();
  if (g < groups) fetch(g, wa);  // in flight while the token is quantised
  {
    const uint4* xr = reinterpret_cast<const uint4*>(x);  // d is a multiple of 32: whole 16-byte chunks of 8 bf16
    const int chunks = d / 8;
    float amax = 0.0f;
    for (int c = (int)threadIdx.x; c < chunks; c += 256) {
      const uint4 v = xr[c];
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(wd[q])), fabsf(bf16_hi(wd[q]))));
    }
    amax = block_max_256(amax, red);
    float sx = __fdiv_rn(amax, 127.0f);
    if (amax == 0.0f) sx = 1.0f;
    auto code = [&](float f) -> uint32_t {
      float r = rintf(__fdiv_rn(f, sx));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      return (uint32_t)((int)r) & 0xFFu;
    };
    for (int c = (int)threadIdx.x; c < chunks; c += 256) {
      const uint4 v = xr[c];
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
      uint2 o;
      o.x = code(bf16_lo(wd[0])) | code(bf16_hi(wd[0])) << 8 | code(bf16_lo(wd[1])) << 16 | code(bf16_hi(wd[1])) << 24;
      o.y = code(bf16_lo(wd[2])) | code(bf16_hi(wd[2])) << 8 | code(bf16_lo(wd[3])) << 16 | code(bf16_hi(wd[3])) << 24;
      reinterpret_cast<uint2*>(xs)[c] = o;
    }
    __syncthreads();
  }
  while (g < groups) {
    const int g1 = g + total_waves, g2 = g1 + total_waves;
    fetch(min(g1, groups - 1), wb);
    __builtin_amdgcn_sched_barrier(0);
    finish(g, wa);
    __builtin_amdgcn_sched_barrier(0);
    if (g1 >= groups) break;
    fetch(min(g2, groups - 1), wa);
    __builtin_amdgcn_sched_barrier(0);
    finish(g1, wb);
    __builtin_amdgcn_sched_barrier(0);
    g = g2;
  }
  if (mr.wgmax == nullptr) return;
  wmax = wave_max(wmax);
  if (lane == 0) wmax_sh[wave_id()] = wmax;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t m = 0u;
    for (int w = 0; w < 4; ++w) m = wmax_sh[w] > m ? wmax_sh[w] : m;
    mr.wgmax[blockIdx.x] = m;
  }
}

// ---------------------------------------------------------------------------
// Low-rank scorer, stage 1: t[b,p] = bf16(sum_i Z1[i,p] x[b,i]).  Z1 is [d, r] row-major, so the sum runs down
// the rows.  grid (slices of kLrSliceRows rows, tokens): a workgroup adds its slice for one token in fp64 - thread
// (row lane, chunk) owns 8 columns of every row-lane-th row - folds the row lanes through LDS in a fixed order
// and writes one partial row; k_lr_reduce adds the slices in a fixed order and rounds to bf16.
constexpr int kLrSliceRows = 64;

__global__ __launch_bounds__(256) void k_lr_project(const uint16_t* __restrict__ z1, const uint16_t* __restrict__ x,
                                                    int d, int r, double* __restrict__ partial, uint32_t* zero_ptr,
                                                    int zero_words, GeneralHeader* gh, unsigned long long sig) {
  extern __shared__ double part[];  // [row lanes][r]
  zero_slice(zero_ptr, zero_words);
  if (blockIdx.x == 0 && blockIdx.y == 0) general_header_check(gh, sig);
  const int b = (int)blockIdx.y, sl = (int)blockIdx.x, slices = (int)gridDim.x;
  const int chunks = r / 8;              // 16-byte chunks per row of Z1
  const int lanes = 256 / chunks;        // row lanes; threads past lanes * chunks idle
  const int tid = (int)threadIdx.x;
  const int rl = tid / chunks, c = tid - rl * chunks;
  const int i0 = sl * kLrSliceRows, i1 = min(d, i0 + kLrSliceRows);
  const uint16_t* xr = x + (size_t)b * d;
  double acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) acc[q] = 0.0;
  if (rl < lanes) {
    for (int i = i0 + rl; i < i1; i += lanes) {
      const uint4 v = reinterpret_cast<const uint4*>(z1 + (size_t)i * r)[c];
      const float xi = bf16_to_f32(xr[i]);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[2 * q] += (double)(bf16_lo(w[q]) * xi);       // a product of two bf16 is exact in fp32
        acc[2 * q + 1] += (double)(bf16_hi(w[q]) * xi);
      }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) part[(size_t)rl * r + c * 8 + q] = acc[q];
  }
  __syncthreads();
  for (int p = tid; p < r; p += 256) {
    double tot = 0.0;
    for (int u = 0; u < lanes; ++u) tot += part[(size_t)u * r + p];
    partial[((size_t)b * slices + sl) * r + p] = tot;
  }
}

__global__ __launch_bounds__(256) void k_lr_reduce(const double* __restrict__ partial, int slices, int r,
                                                   uint16_t* __restrict__ t) {
  const int b = (int)blockIdx.x;
  for (int p = (int)threadIdx.x; p < r; p += 256) {
    double tot = 0.0;
    for (int s0 = 0; s0 < slices; s0 += 8) {  // eight loads in flight; added in slice order
      double v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = partial[((size_t)b * slices + min(s0 + j, slices - 1)) * r + p];
#pragma unroll
      for (int j = 0; j < 8; ++j) tot += s0 + j < slices ? v[j] : 0.0;
    }
    t[(size_t)b * r + p] = f64_to_bf16_rne(tot);
  }
}

// Low-rank scorer, stage 2, one token: key[j] = phi(<Z2[j,:], t>).  ROW_LANES lanes share a row (16 when a row
// is at most 16 chunks of 16 bytes - four rows per wave - else the whole wave); the lanes' partial sums are
// folded along the DPP row (or the wave), and the last lane of each group stores the row's key.
template <int ROW_LANES>
__global__ __launch_bounds__(256) void k_lr_score_b1(const uint16_t* __restrict__ z2, const uint16_t* __restrict__ t,
                                                     int N, int r, int relu, double* __restrict__ keys) {
  extern __shared__ uint4 xs[];  // t as raw bf16, [r/8] uint4
  constexpr int kRows = kWave / ROW_LANES;  // rows per wave and trip
  const int cpr = r / 8;
  const int lane = lane_id(), sub = lane % ROW_LANES, rw = lane / ROW_LANES;
  for (int i = (int)threadIdx.x; i < cpr; i += 256) xs[i] = reinterpret_cast<const uint4*>(t)[i];
  __syncthreads();
  const int total = (int)gridDim.x * 4 * kRows;
  for (int j0 = ((int)blockIdx.x * 4 + wave_id()) * kRows; j0 < N; j0 += total) {
    const int j = j0 + rw;
    const uint4* row = reinterpret_cast<const uint4*>(z2 + (size_t)min(j, N - 1) * r);
    double acc = 0.0;
    for (int c0 = 0; c0 < cpr; c0 += ROW_LANES) {
      const int c = c0 + sub;
      const uint4 wv = row[min(c, cpr - 1)];
      const uint4 tv = xs[min(c, cpr - 1)];
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
      if (relu) s = s > 0.0 ? s : 0.0;
      if (s == 0.0) s = 0.0;
      keys[j] = s;
    }
  }
}

__global__ void k_clear_words(uint32_t* p, int words) { zero_slice(p, words); }

// Plain copy, 16 bytes per thread and iteration: the reference point for calibrating HBM traffic counters.
__global__ __launch_bounds__(256) void k_plain_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
size_t general_header_bytes() { return sizeof(GeneralHeader); }

unsigned long long layout_signature(int scorer_kind, int B, int d, int N, int r, int k, int kprime, int ffn) {
  unsigned long long h = 0x9E3779B97F4A7C15ull;
  const int v[8] = {scorer_kind, B, d, N, r, k, kprime, ffn};
  for (int i = 0; i < 8; ++i) {
    h ^= (unsigned long long)(unsigned)v[i] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2);
    h *= 0xBF58476D1CE4E5B9ull;
  }
  return h | 1ull;  // never the cleared header's zero
}

hipError_t launch_clear_words(uint32_t* p, int words, hipStream_t s) {
  return launch(k_clear_words, dim3((words + 255) / 256), dim3(256), 0, s, p, words);
}

hipError_t launch_plain_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  return launch(k_plain_copy, dim3(4096), dim3(256), 0, s, static_cast<const uint4*>(src), static_cast<uint4*>(dst),
                bytes / 16);
}

hipError_t launch_pack_int4(const uint16_t* w, int rows, int cols, uint32_t* q4, float* scale, hipStream_t s) {
  uint32_t* trailer = q4 + (size_t)rows * (cols / 8);
  if (const hipError_t e = launch_clear_words(trailer, (int)(kPackTrailerBytes / 4), s); e != hipSuccess) return e;
  return launch(k_pack_int4, dim3(rows), dim3(256), 0, s, w, cols, q4, scale, trailer);
}

hipError_t launch_unpack_int4(const uint32_t* q4, int rows, int cols, int8_t* codes, hipStream_t s) {
  return launch(k_unpack_int4, dim3(rows), dim3(256), 0, s, q4, cols, codes);
}

hipError_t launch_quantize_tokens(const uint16_t* x, int B, int d, int8_t* xq, float* sx, uint32_t* zero_ptr,
                                  int zero_words, void* general_header, unsigned long long sig, hipStream_t s) {
  return launch(k_quantize_tokens, dim3(B), dim3(256), 0, s, x, d, xq, sx, zero_ptr, zero_words,
                static_cast<GeneralHeader*>(general_header), sig);
}

template <int BT>
static hipError_t scorer_int4_bt(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d,
                                 int relu, float* keys, int32_t* acc, const MultiRegion& mr, hipStream_t s) {
  const int blocks = scorer_int4_blocks(N);
  const size_t lds = (size_t)BT * d;
  return launch(k_scorer_int4<BT>, dim3(blocks), dim3(256), lds, s, reinterpret_cast<const uint4*>(q4), scale, xq,
                     B, N, d, relu, keys, acc, mr);
}

int scorer_int4_blocks(int N) {
  const int groups = (N + kScorerRPW - 1) / kScorerRPW;
  static_assert(kWgMaxSlots >= 4096, "one maximum slot per scorer workgroup (short rows: 4 x 512 waves)");
  return min((groups + 3) / 4, 4096);
}

hipError_t launch_scorer_int4(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d, int relu,
                              float* keys, int32_t* acc, const HistRefs& hr, hipStream_t s) {
  MultiRegion mr = multi_of(hr, B);
  if (!multi_producer_counts(N, B)) mr.hist = nullptr;  // then the selection counts in a pass of its own
  if (B == 1) return scorer_int4_bt<1>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
  return hipErrorInvalidValue;  // batches score on the matrix cores (scorer_mfma.hip)
}

bool scorer_int4_fused_supported(int d) { return d <= 8192; }

// The same for short rows (d <= 32 * LPR; the int4 low-rank scorer's second product has rows of r codes): LPR
// lanes share a row, so one load instruction of a wave covers 64 / LPR consecutive rows - one contiguous KB when
// a row is exactly LPR chunks - instead of leaving most lanes on clamped duplicates.  The row sums form inside the
// 16-lane DPP rows and land in the last lane of each row's group.
// XF32: the token comes as fp32 (the first product of the int4 low-rank scorer) and is rounded to bf16, nearest
// even, before it is quantised - the separate conversion pass folded in.
template <int LPR, bool XF32>
__global__ __launch_bounds__(256) void k_scorer_int4_b1_short(const uint4* __restrict__ q4,
                                                              const float* __restrict__ scale,
                                                              const void* __restrict__ x, int N, int d, int relu,
                                                              float* __restrict__ keys, int32_t* __restrict__ acc_out,
                                                              MultiRegion mr, uint32_t* zero_ptr, int zero_words,
                                                              GeneralHeader* gh, unsigned long long sig) {
  static_assert(LPR == 4 || LPR == 16, "lanes per row");
  constexpr int kRowsPerLoad = kWave / LPR;
  constexpr int kLoads = 8;  // load instructions a wave has in flight
  constexpr int kRowsPerTrip = kRowsPerLoad * kLoads;
  extern __shared__ uint4 xs[];  // [d/16] token, 16 int8 per uint4
  __shared__ float red[4];
  zero_slice(zero_ptr, zero_words);
  if (blockIdx.x == 0) general_header_check(gh, sig);
  const int cpr = d / 32;
  const int lane = lane_id(), sub = lane % LPR, rsub = lane / LPR;
  const bool hist_on = mr.hist != nullptr && multi_hist_ok(mr.hdr, 1);
  const int csub = min(sub, cpr - 1);
  const int trips = (N + kRowsPerTrip - 1) / kRowsPerTrip, stride = (int)gridDim.x * 4;
  auto fetch = [&](int trip, uint4 (&wv)[kLoads], float (&sc)[kLoads]) {
    const int j0 = trip * kRowsPerTrip + rsub;
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {  // clamped and unconditional: one batch of loads, the row scales with them
      const int jc = min(j0 + u * kRowsPerLoad, N - 1);
      wv[u] = load_streaming(&q4[(size_t)jc * cpr + csub]);
      sc[u] = scale[jc];
    }
  };
  uint4 wa[kLoads], wb[kLoads];
  float sa[kLoads], sb[kLoads];
  int trip = (int)blockIdx.x * 4 + wave_id();
  // the token's loads first, the first rows behind them (loads return in issue order), then the token's arithmetic
  // while the rows fly; d <= 512, so a thread holds at most one chunk of eight token values
  const int c = (int)threadIdx.x;
  const bool mine = c < d / 8;
  const int cc = mine ? c : 0;
  float4 tok_a = make_float4(0.f, 0.f, 0.f, 0.f), tok_b = tok_a;
  uint4 tok_h = make_uint4(0, 0, 0, 0);
  if (XF32) {
    tok_a = reinterpret_cast<const float4*>(x)[2 * cc];
    tok_b = reinterpret_cast<const float4*>(x)[2 * cc + 1];
  } else {
    tok_h = reinterpret_cast<const uint4*>(x)[cc];
  }
  __builtin_amdgcn_sched_barrier(0);
  if (trip < trips) fetch(trip, wa, sa);
  __builtin_amdgcn_sched_barrier(0);
  {  // the token as int8, scale amax / 127
    float xf[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) xf[q] = 0.0f;
    if (mine) {
      if (XF32) {
        const float4 a = tok_a, b = tok_b;
        const float raw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int q = 0; q < 8; ++q) {  // to bf16, round to nearest even (finite values)
          const uint32_t u = __float_as_uint(raw[q]);
          xf[q] = __uint_as_float((u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u);
        }
      } else {
        const uint4 v = tok_h;
        const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          xf[2 * q] = bf16_lo(wd[q]);
          xf[2 * q + 1] = bf16_hi(wd[q]);
        }
      }
    }
    float amax = 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q) amax = fmaxf(amax, fabsf(xf[q]));
    amax = block_max_256(amax, red);
    float sx = __fdiv_rn(amax, 127.0f);
    if (amax == 0.0f) sx = 1.0f;
    auto code = [&](float f) -> uint32_t {
      float r = rintf(__fdiv_rn(f, sx));
      r = fminf(fmaxf(r, -127.0f), 127.0f);
      return (uint32_t)((int)r) & 0xFFu;
    };
    if (mine) {
      uint2 o;
      o.x = code(xf[0]) | code(xf[1]) << 8 | code(xf[2]) << 16 | code(xf[3]) << 24;
      o.y = code(xf[4]) | code(xf[5]) << 8 | code(xf[6]) << 16 | code(xf[7]) << 24;
      reinterpret_cast<uint2*>(xs)[c] = o;
    }
    __syncthreads();
  }
  const uint4 xa = xs[2 * csub], xb = xs[2 * csub + 1];
  const int xd[8] = {(int)xa.x, (int)xa.y, (int)xa.z, (int)xa.w, (int)xb.x, (int)xb.y, (int)xb.z, (int)xb.w};
  const uint32_t keep = sub < cpr ? 0xFFFFFFFFu : 0u;  // lanes past the row's end contribute zeros
  uint32_t wmax = 0u;
  auto finish = [&](int trip, const uint4 (&wv)[kLoads], const float (&sc)[kLoads]) {
    const int j0 = trip * kRowsPerTrip + rsub;
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
      const uint32_t wd[4] = {wv[u].x & keep, wv[u].y & keep, wv[u].z & keep, wv[u].w & keep};
      int a = 0;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        a = __builtin_amdgcn_sdot4((int)(wd[t] & 0xF0F0F0F0u), xd[2 * t], a, false);
        a = __builtin_amdgcn_sdot4((int)((wd[t] << 4) & 0xF0F0F0F0u), xd[2 * t + 1], a, false);
      }
      a += dpp_move<0x111, 0xF>(0, a);  // row_shr:1
      a += dpp_move<0x112, 0xF>(0, a);  // row_shr:2
      if (LPR == 16) {
        a += dpp_move<0x114, 0xF>(0, a);  // row_shr:4
        a += dpp_move<0x118, 0xF>(0, a);  // row_shr:8
      }
      const int j = j0 + u * kRowsPerLoad;
      if (sub == LPR - 1 && j < N) {
        const int sum = a >> 4;  // every partial is a multiple of 16
        float key = (float)sum * sc[u];
        if (relu) key = key > 0.0f ? key : 0.0f;
        if (key == 0.0f) key = 0.0f;
        keys[j] = key;
        if (acc_out) acc_out[j] = sum;
        const uint32_t ok = order_key(key);
        wmax = ok > wmax ? ok : wmax;
        if (hist_on && !(relu && key == 0.0f)) atomicAdd(&mr.hist[kHistWindow + hist_bin(ok)], 1u);
      }
    }
  };
  // two register sets in turn, as in the full-row kernel
  while (trip < trips) {
    const int t1 = trip + stride, t2 = t1 + stride;
    fetch(min(t1, trips - 1), wb, sb);
    __builtin_amdgcn_sched_barrier(0);
    finish(trip, wa, sa);
    __builtin_amdgcn_sched_barrier(0);
    if (t1 >= trips) break;
    fetch(min(t2, trips - 1), wa, sa);
    __builtin_amdgcn_sched_barrier(0);
    finish(t1, wb, sb);
    __builtin_amdgcn_sched_barrier(0);
    trip = t2;
  }
  if (mr.wgmax == nullptr) return;
  // one maximum per wave (scorer_int4_fused_maxima): with at most 512 workgroups the finer grain is what lets
  // launch_softmax_b1 bound the k'-th key from the maxima
  wmax = wave_max(wmax);
  if (lane == 0) mr.wgmax[blockIdx.x * 4 + wave_id()] = wmax;
}

// Workgroups of the batch-1 scorer kernels.  Short rows: at most 512 workgroups, so that on a long matrix the token
// staging of a workgroup is spread over several trips.
int scorer_int4_fused_blocks(int N, int d) {
  if (d > 512) return scorer_int4_blocks(N);
  const int rows_per_trip = d <= 128 ? 128 : 32;
  const int trips = (N + rows_per_trip - 1) / rows_per_trip;
  return max(1, min((trips + 3) / 4, 512));  // one trip per wave until 512 workgroups are out, then several
}

// Maxima the kernels leave for the selections that follow: one per workgroup, or (short rows) one per wave.
int scorer_int4_fused_maxima(int N, int d) {
  return d > 512 ? scorer_int4_fused_blocks(N, d) : 4 * scorer_int4_fused_blocks(N, d);
}

bool scorer_int4_fused_takes_f32(int d) { return d <= 512; }

hipError_t launch_scorer_int4_fused(const uint32_t* q4, const float* scale, const void* x, bool x_is_f32, int N, int d,
                                    int relu, float* keys, int32_t* acc, const HistRefs& hr, uint32_t* zero_ptr,
                                    int zero_words, unsigned long long sig, hipStream_t s) {
  if (x_is_f32 && !scorer_int4_fused_takes_f32(d)) return hipErrorInvalidValue;
  MultiRegion mr = multi_of(hr, 1);
  if (!multi_producer_counts(N, 1)) mr.hist = nullptr;
  GeneralHeader* gh = static_cast<GeneralHeader*>(hr.header);
  const dim3 grid(scorer_int4_fused_blocks(N, d));
  const uint4* q = reinterpret_cast<const uint4*>(q4);
  if (d <= 128) {
    if (x_is_f32)
      return launch(k_scorer_int4_b1_short<4, true>, grid, dim3(256), (size_t)d, s, q, scale, x, N, d, relu, keys, acc,
                    mr, zero_ptr, zero_words, gh, sig);
    return launch(k_scorer_int4_b1_short<4, false>, grid, dim3(256), (size_t)d, s, q, scale, x, N, d, relu, keys, acc,
                  mr, zero_ptr, zero_words, gh, sig);
  }
  if (d <= 512) {
    if (x_is_f32)
      return launch(k_scorer_int4_b1_short<16, true>, grid, dim3(256), (size_t)d, s, q, scale, x, N, d, relu, keys, acc,
                    mr, zero_ptr, zero_words, gh, sig);
    return launch(k_scorer_int4_b1_short<16, false>, grid, dim3(256), (size_t)d, s, q, scale, x, N, d, relu, keys, acc,
                  mr, zero_ptr, zero_words, gh, sig);
  }
  const uint16_t* xb = static_cast<const uint16_t*>(x);
  if (d <= 2048)
    return launch(k_scorer_int4_b1<1>, grid, dim3(256), (size_t)d, s, q, scale, xb, N, d, relu, keys, acc, mr, zero_ptr,
                  zero_words, gh, sig);
  if (d <= 4096)
    return launch(k_scorer_int4_b1<2>, grid, dim3(256), (size_t)d, s, q, scale, xb, N, d, relu, keys, acc, mr, zero_ptr,
                  zero_words, gh, sig);
  return launch(k_scorer_int4_b1<4>, grid, dim3(256), (size_t)d, s, q, scale, xb, N, d, relu, keys, acc, mr, zero_ptr,
                zero_words, gh, sig);
}

// fp32 -> bf16, round to nearest even (finite inputs): the int4 low-rank scorer's intermediate as the bf16
// activation its second product quantises.
__global__ __launch_bounds__(256) void k_f32_to_bf16(const float* __restrict__ in, int n, uint16_t* __restrict__ out) {
  const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
  if (i >= n) return;
  const uint32_t u = __float_as_uint(in[i]);
  out[i] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

hipError_t launch_f32_to_bf16(const float* in, int n, uint16_t* out, hipStream_t s) {
  return launch(k_f32_to_bf16, dim3((n + 255) / 256), dim3(256), 0, s, in, n, out);
}

int lr_project_slices(int d) { return (d + kLrSliceRows - 1) / kLrSliceRows; }

hipError_t launch_lr_project(const uint16_t* z1, const uint16_t* x, int B, int d, int r, uint16_t* t, double* partial,
                             uint32_t* zero_ptr, int zero_words, void* general_header, unsigned long long sig,
                             hipStream_t s) {
  const int slices = lr_project_slices(d);
  const size_t lds = (size_t)(256 / (r / 8)) * r * sizeof(double);
  const hipError_t e = launch(k_lr_project, dim3(slices, B), dim3(256), lds, s, z1, x, d, r, partial, zero_ptr,
                              zero_words, static_cast<GeneralHeader*>(general_header), sig);
  if (e != hipSuccess || t == nullptr) return e;  // no t: the caller adds the slices itself
  return launch(k_lr_reduce, dim3(B), dim3(256), 0, s, partial, slices, r, t);
}

// Largest row norm of a bf16 matrix, rounded up: one wave per row, fp32 sum of squares (its relative error is at
// most cols 2^-23), atomic max on the float's bits (out cleared beforehand).
__global__ __launch_bounds__(256) void k_row_norm_max(const uint16_t* __restrict__ W, int rows, int cols,
                                                      uint32_t* __restrict__ out) {
  const int lane = lane_id(), cpr = cols / 8;
  float best = 0.0f;
  for (int j = (int)blockIdx.x * 4 + wave_id(); j < rows; j += (int)gridDim.x * 4) {
    const uint4* row = reinterpret_cast<const uint4*>(W + (size_t)j * cols);
    float acc = 0.0f;
    for (int c = lane; c < cpr; c += kWave) {
      const uint4 v = row[c];
      const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float a = bf16_lo(wd[q]), b = bf16_hi(wd[q]);
        acc = fmaf(a, a, acc);
        acc = fmaf(b, b, acc);
      }
    }
    acc = wave_sum(acc);
    best = fmaxf(best, sqrtf(acc * (1.0f + (float)cols * 0x1p-22f)) * 1.0001f);
  }
  if (lane == 0 && best > 0.0f) atomicMax(out, __float_as_uint(best));
}

hipError_t launch_row_norm_max(const uint16_t* W, int rows, int cols, float* out, hipStream_t s) {
  hipError_t e = launch_clear_words(reinterpret_cast<uint32_t*>(out), 1, s);
  if (e != hipSuccess) return e;
  return launch(k_row_norm_max, dim3(max(1, min((rows + 3) / 4, 2048))), dim3(256), 0, s, W, rows, cols,
                reinterpret_cast<uint32_t*>(out));
}

hipError_t launch_lr_score(const uint16_t* z2, const uint16_t* t, int N, int r, int relu, double* keys, hipStream_t s) {
  const dim3 grid(max(1, min((N + 15) / 16, 4096)));
  const size_t lds = (size_t)r * 2;
  if (r <= 128) return launch(k_lr_score_b1<16>, grid, dim3(256), lds, s, z2, t, N, r, relu, keys);
  return launch(k_lr_score_b1<kWave>, grid, dim3(256), lds, s, z2, t, N, r, relu, keys);
}

}  // namespace hire
