// Exact pre-activations on the candidate union for batches (arXiv 2402.09360, Algorithm 1 line 2):
//   h[b, t] = phi(<z_{U[t]}, x_b>),  t < |U|,
// on the fp64 matrix cores.  A wave owns 16 candidate rows and 16 tokens and accumulates their 16 x 16 tile
// with 16x16x4 MFMAs: tokens are the A matrix, candidate rows the B matrix, so lane l of the result holds
// candidate l % 16 for tokens l / 16 + 4 r, r = 0..3.  Every lane converts its own bf16 operands: lane (j, g)
// reads the 16-byte chunks 4 * it + g of candidate row j and of token j - no sharing between lanes, hence no
// LDS - and feeds the eight values of a chunk to eight consecutive MFMAs.  Which position of the row goes to
// which MFMA is free as long as both operands agree, since the order of a sum's terms is.
//
// fp64 accumulation of products that are exact (bf16 x bf16 fits fp32, let alone fp64) keeps the ranking that
// follows independent of the summation order up to the last bits of a double.
#include "device_utils.h"
#include "kernels.h"

namespace hire {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kGmBatch = 8;  // 16-byte chunks per lane in flight for each operand

__global__ __launch_bounds__(256) void k_gather_dot_mfma(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                                         int B, int d, const int32_t* __restrict__ list, int n_host,
                                                         const int32_t* __restrict__ n_dev, int n_cap, int relu,
                                                         double* __restrict__ h, long long stride_h) {
  const int n = n_dev ? min(*n_dev, n_cap) : n_host;
  const int tile = (int)blockIdx.x * 4 + wave_id();
  if (tile * 16 >= n) return;  // whole waves leave; no barriers in this kernel
  const int lane = lane_id(), jl = lane & 15, g = lane >> 4;
  const int t_idx = tile * 16 + jl;
  const int tok = (int)blockIdx.y * 16 + jl;
  const int cpr = d / 8;  // 16-byte chunks per row
  const uint4* wrow = reinterpret_cast<const uint4*>(W + (size_t)list[min(t_idx, n - 1)] * d);
  const uint4* xrow = reinterpret_cast<const uint4*>(x + (size_t)min(tok, B - 1) * d);
  const int nit = (cpr + 3) / 4;

  auto fetch = [&](int it0, uint4 (&wv)[kGmBatch], uint4 (&tv)[kGmBatch]) {
#pragma unroll
    for (int u = 0; u < kGmBatch; ++u) {
      const int c = (it0 + u) * 4 + g;
      const int cc = min(c, cpr - 1);
      wv[u] = wrow[cc];
      tv[u] = xrow[cc];
      if (c >= cpr) wv[u] = make_uint4(0, 0, 0, 0);  // zero weights: the product vanishes whatever the token holds
    }
  };

  v4d acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
  uint4 wv[kGmBatch], tv[kGmBatch], wn[kGmBatch], tn[kGmBatch];
  fetch(0, wv, tv);
  for (int it0 = 0; it0 < nit; it0 += kGmBatch) {
    fetch(it0 + kGmBatch, wn, tn);  // clamped: past the end it re-reads the last chunk and zeroes it
#pragma unroll
    for (int u = 0; u < kGmBatch; ++u) {
      const uint32_t wd[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
      const uint32_t td[4] = {tv[u].x, tv[u].y, tv[u].z, tv[u].w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)bf16_lo(td[q]), (double)bf16_lo(wd[q]), acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)bf16_hi(td[q]), (double)bf16_hi(wd[q]), acc1, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kGmBatch; ++u) {
      wv[u] = wn[u];
      tv[u] = tn[u];
    }
  }
  if (t_idx >= n) return;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int tk = (int)blockIdx.y * 16 + g + 4 * r;  // fp64 tiles interleave the rows over the lane groups
    if (tk >= B) continue;
    double s = acc0[r] + acc1[r];
    if (relu) s = s > 0.0 ? s : 0.0;
    if (s == 0.0) s = 0.0;
    h[(size_t)tk * stride_h + t_idx] = s;
  }
}

hipError_t launch_gather_dot_mfma(const uint16_t* W, const uint16_t* x, int B, int d, const int32_t* list, int n,
                                  const int32_t* n_dev, int n_cap, int relu, double* h, long long stride_h,
                                  hipStream_t s) {
  const int cap = n_dev ? n_cap : n;
  const int blocks = max(1, (cap + 63) / 64);
  return launch(k_gather_dot_mfma, dim3(blocks, (B + 15) / 16), dim3(256), 0, s, W, x, B, d, list, n, n_dev, n_cap,
                relu, h, stride_h);
}

}  // namespace hire
