// Exact pre-activations on the candidate union for batches (arXiv 2402.09360, Algorithm 1 line 2):
//   h[b, t] = phi(<z_{U[t]}, x_b>),  t < |U|,
// on the fp64 matrix cores.  A workgroup owns 16 candidate rows and 16 tokens and accumulates their 16 x 16
// tile with 16x16x4 MFMAs: tokens are the A matrix, candidate rows the B matrix, so lane l of the result holds
// candidate l % 16 for tokens l / 16 + 4 r, r = 0..3.  Every lane converts its own bf16 operands: lane (j, g)
// reads 16-byte chunks 4 * it + g of candidate row j and of token j - no sharing between lanes, hence no LDS
// staging - and feeds the eight values of a chunk to eight consecutive MFMAs.  Which position of the row goes
// to which MFMA is free as long as both operands agree, since the order of a sum's terms is.
//
// The four waves of the workgroup split the row's chunks between them (a union of a few thousand rows gives
// too few tiles to occupy the machine otherwise) and add their partial tiles through LDS in a fixed order.
//
// fp64 accumulation of products that are exact (bf16 x bf16 fits fp32, let alone fp64) keeps the ranking that
// follows independent of the summation order up to the last bits of a double.
#include "device_utils.h"
#include "hist.h"
#include "kernels.h"

namespace hire {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kGmBatch = 2;  // 16-byte chunks per lane in flight for each operand

// TOK: tokens per tile.  16: the 16x16x4 MFMA as described.  4 (batches of at most four): the 4x4x4 MFMA of four
// independent blocks - lane l then holds candidate l % 16 (block l / 4 % 4, column l % 4) and K group l / 16 on
// the weight side as before, token l % 4 on the token side, and the result for candidate l % 16 and token l / 16 -
// a quarter of the matrix-core time of a 16-token tile that is three quarters padding.
// gs > 0 (group-sparse FFN, eq. (6)): list entries are groups of 2^gs <= 16 adjacent rows, a tile covers 16 >> gs
// of them, and the result of row l of entry e goes to column e * 2^gs + l of h.  Counts stay in entries.
template <int TOK>
__global__ __launch_bounds__(256) void k_gather_dot_mfma(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                                         int B, int d, const int32_t* __restrict__ list, int n_host,
                                                         const int32_t* __restrict__ n_dev, int n_cap, int relu,
                                                         double* __restrict__ h, long long stride_h,
                                                         GatherUnion un, int gs) {
  constexpr int kAcc = TOK == 16 ? 4 : 1;  // result values per lane
  __shared__ double red[3][kAcc][kWave];
  __shared__ SelSharedT<256> sh;
  __shared__ int32_t rows_sh[16];
  HIRE_TS(50);
  const int tile = (int)blockIdx.x;
  const int lane = lane_id(), w = wave_id(), jl = lane & 15, g = lane >> 4;
  const int ept = 16 >> gs, e0 = tile * ept;  // entries per tile, the tile's first entry
  int n;                                      // entries
  if (un.bitmap != nullptr) {  // the workgroup finds its candidates in the union bitmap itself
    n = un.words <= 4 * 64 * kLocateStepsShort ? union_locate<256, kLocateStepsShort>(un.bitmap, un.words, sh, e0, ept, rows_sh)
                                               : union_locate<256>(un.bitmap, un.words, sh, e0, ept, rows_sh);
    n = min(n, n_cap);
    if (blockIdx.y == 0) {
      if (tile == 0) publish_union(un, n);
      const int t = (int)threadIdx.x;
      if (t < ept && e0 + t < n) un.list_out[e0 + t] = rows_sh[t];
    }
  } else {
    n = n_dev ? min(*n_dev, n_cap) : n_host;
  }
  n <<= gs;  // rows from here on
  HIRE_TS(51);
  const int tok = (int)blockIdx.y * TOK + (TOK == 16 ? jl : (jl & 3));
  const bool live = tile * 16 < n;  // uniform over the workgroup
  const int t_idx = tile * 16 + jl;
  v4d acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = acc0;  // two independent chains (16 tokens)
  double sacc0 = 0.0, sacc1 = 0.0;                 // the same for 4 tokens
  if (live) {
    const int cpr = d / 8;  // 16-byte chunks per row
    const int tc = min(t_idx, n - 1);
    const int te = tc >> gs;  // the row's entry
    const int cand = ((un.bitmap != nullptr ? rows_sh[te - e0] : (list != nullptr ? list[te] : te)) << gs) +
                     (tc & ((1 << gs) - 1));
    const uint4* wrow = reinterpret_cast<const uint4*>(W + (size_t)cand * d);
    const uint4* xrow = reinterpret_cast<const uint4*>(x + (size_t)min(tok, B - 1) * d);
    const int nit = (cpr + 3) / 4;
    const int per_wave = (nit + 3) / 4;
    const int it_lo = w * per_wave, it_hi = min(nit, it_lo + per_wave);

    auto fetch = [&](int it0, uint4 (&wv)[kGmBatch], uint4 (&tv)[kGmBatch]) {
#pragma unroll
      for (int u = 0; u < kGmBatch; ++u) {
        const int c = (it0 + u) * 4 + g;
        const int cc = min(c, cpr - 1);
        // clamped and unconditional: the loads of a batch must not wait for one another.  Plain loads: consecutive
        // loads share cache lines (64 bytes of a row each)
        wv[u] = wrow[cc];
        tv[u] = xrow[cc];
      }
    };

    auto mac = [&](int it0, const uint4 (&wv)[kGmBatch], const uint4 (&tv)[kGmBatch]) {
#pragma unroll
      for (int u = 0; u < kGmBatch; ++u) {
        // past the wave's share or the row's end: zero weights, the product vanishes whatever the token holds
        const uint32_t keep = (it0 + u < it_hi && (it0 + u) * 4 + g < cpr) ? 0xFFFFFFFFu : 0u;
        const uint32_t wd[4] = {wv[u].x & keep, wv[u].y & keep, wv[u].z & keep, wv[u].w & keep};
        const uint32_t td[4] = {tv[u].x, tv[u].y, tv[u].z, tv[u].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if constexpr (TOK == 16) {
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)bf16_lo(td[q]), (double)bf16_lo(wd[q]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)bf16_hi(td[q]), (double)bf16_hi(wd[q]), acc1, 0, 0, 0);
          } else {
            sacc0 = __builtin_amdgcn_mfma_f64_4x4x4f64((double)bf16_lo(td[q]), (double)bf16_lo(wd[q]), sacc0, 0, 0, 0);
            sacc1 = __builtin_amdgcn_mfma_f64_4x4x4f64((double)bf16_hi(td[q]), (double)bf16_hi(wd[q]), sacc1, 0, 0, 0);
          }
        }
      }
    };

    // two register sets in turn: the loads of the next batch are issued before the current one is consumed (the
    // scheduling barriers keep the compiler from sinking them to their first use)
    uint4 wa[kGmBatch], ta[kGmBatch], wb[kGmBatch], tb[kGmBatch];
    fetch(it_lo, wa, ta);
    HIRE_TS(52);
    for (int it0 = it_lo; it0 < it_hi; it0 += 2 * kGmBatch) {
      fetch(it0 + kGmBatch, wb, tb);
      __builtin_amdgcn_sched_barrier(0);
      mac(it0, wa, ta);
      __builtin_amdgcn_sched_barrier(0);
      fetch(it0 + 2 * kGmBatch, wa, ta);
      __builtin_amdgcn_sched_barrier(0);
      mac(it0 + kGmBatch, wb, tb);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  HIRE_TS(53);
  double acc[kAcc];
  if constexpr (TOK == 16) {
    const v4d a = acc0 + acc1;
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = a[r];
  } else {
    acc[0] = sacc0 + sacc1;
  }
  if (w > 0) {
#pragma unroll
    for (int r = 0; r < kAcc; ++r) red[w - 1][r][lane] = acc[r];
  }
  __syncthreads();
  if (w > 0) return;
#pragma unroll
  for (int r = 0; r < kAcc; ++r) {
    // 16-token tiles interleave the rows over the lane groups; a 4-token tile has token l / 16 in lane l
    const int tk = (int)blockIdx.y * TOK + g + 4 * r;
    double s = ((acc[r] + red[0][r][lane]) + red[1][r][lane]) + red[2][r][lane];
    if (relu) s = s > 0.0 ? s : 0.0;
    if (s == 0.0) s = 0.0;
    const bool valid = live && tk < B && t_idx < n;
    if (valid) h[(size_t)tk * stride_h + t_idx] = s;
  }
  HIRE_TS(54);
}

static int gather_mfma_tiles(int cap, int gs) { return max(1, (int)((((long long)cap << gs) + 15) / 16)); }

hipError_t launch_gather_dot_mfma(const uint16_t* W, const uint16_t* x, int B, int d, const int32_t* list, int n,
                                  const int32_t* n_dev, int n_cap, int relu, double* h, long long stride_h,
                                  const HistRefs& hr, const UnionRefs* un, int gs, hipStream_t s) {
  const int cap = n_dev ? n_cap : n;
  const GatherUnion u = make_gather_union(un, hr, B);
  if (B <= 4)
    return launch(k_gather_dot_mfma<4>, dim3(gather_mfma_tiles(cap, gs), 1), dim3(256), 0, s, W, x, B, d,
                  u.bitmap ? nullptr : list, n, n_dev, cap, relu, h, stride_h, u, gs);
  return launch(k_gather_dot_mfma<16>, dim3(gather_mfma_tiles(cap, gs), (B + 15) / 16), dim3(256), 0, s, W, x, B, d,
                u.bitmap ? nullptr : list, n, n_dev, cap, relu, h, stride_h, u, gs);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_gather(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
