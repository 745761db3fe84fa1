// HiRE-Q scorer for batches (arXiv 2402.09360, Algorithm 1 line 1 with the int4 Zapprox of Sec. 3.2) on the
// int8 matrix cores: acc[b, j] = sum_i q_j[i] xq[b, i] as 16x16x64 MFMA tiles, 16 tokens by 16 weight rows.
//
// A wave owns 16 consecutive rows of the packed int4 matrix - one contiguous block of memory - and keeps a
// K segment of it in registers while it runs over the token tiles, so the weights cross HBM once whatever
// the batch size.  The packed layout (scorer.hip) turns one dword into two registers of four signed bytes
// equal to 16*code with two ANDs and a shift; these feed the MFMA directly and the sums are shifted back by
// four bits at the end (every partial is a multiple of 16, so this is exact).  Which 16 of a segment's codes a
// lane contributes to which MFMA does not matter as long as its token operand holds the activations of the
// same 16 positions: a dot product does not care about the order of its terms.
//
// Operand roles: tokens are the A matrix (rows), weights the B matrix (columns), so lane l of the result holds
// weight row l % 16 for tokens 4 * (l / 16) .. + 3, and the 16 lanes of a DPP row store 16 consecutive keys
// of one token.
#include "device_utils.h"
#include "hist.h"
#include "kernels.h"

namespace hire {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kMfmaWaves = 4;          // waves (16-row tiles) per workgroup
constexpr int kMfmaRows = 16 * kMfmaWaves;

// CT: token tiles of 16 (batch <= 16 * CT).  KI: 16-byte weight chunks a lane holds per K segment; a segment
// covers KI * 128 codes.
template <int CT, int KI>
__global__ __launch_bounds__(64 * kMfmaWaves) void k_scorer_int4_mfma(const uint4* __restrict__ q4,
                                                                      const float* __restrict__ scale,
                                                                      const int8_t* __restrict__ xq, int B, int N, int d,
                                                                      int relu, float* __restrict__ keys,
                                                                      int32_t* __restrict__ acc_out, MultiRegion mr) {
  constexpr int kTok = 16 * CT;
  constexpr int kSegQ = KI * 8;        // uint4 (16 int8) per token and segment
  constexpr int kStride = kSegQ + 1;   // padded: the 16 token rows a DPP row reads land in different banks
  extern __shared__ uint4 xs[];        // [kTok][kStride]
  const int lane = lane_id(), w = wave_id(), jl = lane & 15, g = lane >> 4;
  const int cpr = d / 32;              // 16-byte chunks per packed row
  const int xv = d / 16;               // uint4 per token
  const int nseg = (cpr + KI * 4 - 1) / (KI * 4);
  const bool hist_on = mr.hist != nullptr && multi_hist_ok(mr.hdr, B);
  uint32_t wmax[CT][4];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 4; ++r) wmax[ct][r] = 0u;

  // Weights of one K segment of the wave's 16 rows.  Clamped and unconditional: the loads must not wait for one
  // another.  Plain loads: a load covers half a cache line per row, the next one the other half, so the line has
  // to stay (streaming loads cost 7 % here).
  uint4 wv[KI];
  auto load_weights = [&](int tile, int seg) {
    const uint4* wrow = q4 + (size_t)min(tile * kMfmaRows + w * 16 + jl, N - 1) * cpr;
#pragma unroll
    for (int it = 0; it < KI; ++it) wv[it] = wrow[min(seg * KI * 4 + it * 4 + g, cpr - 1)];
  };
  for (int tile = (int)blockIdx.x; tile * kMfmaRows < N; tile += (int)gridDim.x) {
    const int j0 = tile * kMfmaRows + w * 16;
    const int j = j0 + jl;
    const float sj = scale[min(j, N - 1)];
    v4i acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = v4i{0, 0, 0, 0};
    for (int seg = 0; seg < nseg; ++seg) {
      // issued first, the weights fly while the token tile is staged
      load_weights(tile, seg);
      if (nseg > 1 || tile == (int)blockIdx.x) {
        __syncthreads();  // readers of the previous tile are done
        // eight loads per thread go out together (clamped and unconditional, zeroed where they do not count when
        // they are stored): a loop with one load per trip would pay a round trip to L2 per trip
        // (with one stage per workgroup - up to 32 tokens - that round trip is paid once and the registers of a
        // batch would cost a resident workgroup: one load per trip there)
        constexpr int kStageBatch = CT >= 4 ? 8 : 1, kStageStep = 64 * kMfmaWaves;
        for (int i0 = (int)threadIdx.x; i0 < kTok * kSegQ; i0 += kStageStep * kStageBatch) {
          uint4 v[kStageBatch];
#pragma unroll
          for (int u = 0; u < kStageBatch; ++u) {
            const int i = min(i0 + u * kStageStep, kTok * kSegQ - 1);
            const int t = i / kSegQ, q = i - t * kSegQ;
            v[u] = reinterpret_cast<const uint4*>(xq + (size_t)min(t, B - 1) * d)[min(seg * kSegQ + q, xv - 1)];
          }
#pragma unroll
          for (int u = 0; u < kStageBatch; ++u) {
            const int i = i0 + u * kStageStep;
            if (i < kTok * kSegQ) {
              const int t = i / kSegQ, q = i - t * kSegQ;
              const bool counts = t < B && seg * kSegQ + q < xv;
              xs[t * kStride + q] = counts ? v[u] : make_uint4(0, 0, 0, 0);
            }
          }
        }
        __syncthreads();
      }
#pragma unroll
      for (int it = 0; it < KI; ++it) {
        const uint32_t keep = seg * KI * 4 + it * 4 + g < cpr ? 0xFFFFFFFFu : 0u;  // past the row's end: zeros
        const uint32_t wd[4] = {wv[it].x & keep, wv[it].y & keep, wv[it].z & keep, wv[it].w & keep};
        v4i wa, wb;
        wa[0] = (int)(wd[0] & 0xF0F0F0F0u);
        wa[1] = (int)((wd[0] << 4) & 0xF0F0F0F0u);
        wa[2] = (int)(wd[1] & 0xF0F0F0F0u);
        wa[3] = (int)((wd[1] << 4) & 0xF0F0F0F0u);
        wb[0] = (int)(wd[2] & 0xF0F0F0F0u);
        wb[1] = (int)((wd[2] << 4) & 0xF0F0F0F0u);
        wb[2] = (int)(wd[3] & 0xF0F0F0F0u);
        wb[3] = (int)((wd[3] << 4) & 0xF0F0F0F0u);
        const int q = 2 * (it * 4 + g);  // the chunk's 32 codes meet token bytes 16q .. 16q + 31 of the segment
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const uint4 ta = xs[(ct * 16 + jl) * kStride + q], tb = xs[(ct * 16 + jl) * kStride + q + 1];
          const v4i va = {(int)ta.x, (int)ta.y, (int)ta.z, (int)ta.w};
          const v4i vb = {(int)tb.x, (int)tb.y, (int)tb.z, (int)tb.w};
          acc[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(va, wa, acc[ct], 0, 0, 0);
          acc[ct] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vb, wb, acc[ct], 0, 0, 0);
        }
      }
    }
    // epilogue: this lane holds row j for tokens ct*16 + 4g + r
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = ct * 16 + 4 * g + r;
        const int sum = acc[ct][r] >> 4;
        if (t < B && j < N) {
          float key = (float)sum * sj;
          if (relu) key = key > 0.0f ? key : 0.0f;
          if (key == 0.0f) key = 0.0f;
          keys[(size_t)t * N + j] = key;
          if (acc_out) acc_out[(size_t)t * N + j] = sum;
          const uint32_t ok = order_key(key);
          wmax[ct][r] = ok > wmax[ct][r] ? ok : wmax[ct][r];
          if (hist_on && !(relu && key == 0.0f))
            atomicAdd(&mr.hist[(size_t)t * kHistStride + kHistWindow + hist_bin(ok)], 1u);
        }
      }
  }
  if (mr.wgmax == nullptr) return;
  // largest key per token and wave (scorer_mfma_maxima per token): across the 16 lanes of each DPP row
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      uint32_t v = wmax[ct][r];
      auto mx = [](uint32_t a, uint32_t b) { return b > a ? b : a; };
      v = mx(v, dpp_move<0x111, 0xF>(0u, v));
      v = mx(v, dpp_move<0x112, 0xF>(0u, v));
      v = mx(v, dpp_move<0x114, 0xF>(0u, v));
      v = mx(v, dpp_move<0x118, 0xF>(0u, v));
      const int t = ct * 16 + 4 * g + r;
      if (jl == 15 && t < B) mr.wgmax[(size_t)t * kWgMaxSlots + blockIdx.x * kMfmaWaves + w] = v;
    }
}

// Three workgroups per CU (what registers and LDS allow to be resident), each running over several tiles: the token
// tile is staged once per workgroup.  Measured on the vocabulary matrix at batch 16: 70 us with one workgroup per
// tile, 56 us with 768 workgroups; requesting the next tile's weights ahead of the epilogue made it slower (69 us).
int scorer_mfma_blocks(int N) { return min((N + kMfmaRows - 1) / kMfmaRows, 768); }
int scorer_mfma_maxima(int N) { return kMfmaWaves * scorer_mfma_blocks(N); }
static_assert(kMfmaWaves * 768 <= kWgMaxSlots, "one maximum slot per wave of the scorer");

template <int CT, int KI>
static hipError_t scorer_mfma_launch(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d,
                                     int relu, float* keys, int32_t* acc, const MultiRegion& mr, hipStream_t s) {
  const size_t lds = (size_t)16 * CT * (KI * 8 + 1) * sizeof(uint4);
  auto kernel = k_scorer_int4_mfma<CT, KI>;
  static std::atomic<size_t> raised_to{0};
  if (const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kernel), lds, raised_to); e != hipSuccess)
    return e;
  return launch(kernel, dim3(scorer_mfma_blocks(N)), dim3(64 * kMfmaWaves), lds, s,
                reinterpret_cast<const uint4*>(q4), scale, xq, B, N, d, relu, keys, acc, mr);
}

hipError_t launch_scorer_int4_mfma(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d,
                                   int relu, float* keys, int32_t* acc, const HistRefs& hr, hipStream_t s) {
  MultiRegion mr = multi_of(hr, B);
  if (!multi_producer_counts(N, B)) mr.hist = nullptr;  // then the selection counts in a pass of its own
  if (d <= 128) {  // short rows (the int4 low-rank scorer's second product): K segments no longer than a row
    if (B <= 16) return scorer_mfma_launch<1, 1>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
    if (B <= 32) return scorer_mfma_launch<2, 1>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
    return scorer_mfma_launch<4, 1>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
  }
  if (d <= 512) {
    if (B <= 16) return scorer_mfma_launch<1, 4>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
    if (B <= 32) return scorer_mfma_launch<2, 4>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
    return scorer_mfma_launch<4, 4>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
  }
  if (B <= 16) return scorer_mfma_launch<1, 16>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
  if (B <= 32) return scorer_mfma_launch<2, 16>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
  return scorer_mfma_launch<4, 16>(q4, scale, xq, B, N, d, relu, keys, acc, mr, s);
}

}  // namespace hire
