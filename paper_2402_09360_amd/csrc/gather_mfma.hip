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

// ---------------------------------------------------------------------------------------------------
// Filter stage of the exact pre-activations for batches (filter and refine): the same tile on the bf16 matrix
// cores, 50 times the fp64 rate, so the stage is a read of the candidate rows.  Tokens are the A matrix,
// candidate rows the B matrix of a 16x16x32 MFMA: lane (j, g) feeds 16-byte chunk 4 it + g of token j and of
// candidate j as they come from memory, no conversion; result value i of lane l belongs to token 4 (l / 16) + i
// and candidate l % 16.  The K range is split over the four waves as above.
//
// What is stored is not the activation but a value within a proven distance of it.  Every MFMA (with more than
// 32 tokens, where the fp64 additions pace the kernel: every second one) starts from a zero accumulator, so a
// segment is the sum of S = 32 (64) products, each exact in fp32, after at most S roundings, each bounded - whether the hardware rounds to nearest, truncates, or aligns the products to the
// largest before adding - by 2^-23 of a running sum that never exceeds the segment's sum of |u_i x_i|.  The
// segments are added in fp64, whose own error is below 2^-40 of the same sums, and the total is rounded to fp32
// (2^-24 of it).  Hence, with a factor two of margin and Cauchy-Schwarz:
//   |stored - <u_j, x_b>| <= delta(b, j) = S 2^-22 |u_j| |x_b| = 2^-17 (2^-16) |u_j| |x_b|,   whatever d.
// The squared norms are the diagonals of two more MFMA chains (rows times rows, tokens times tokens; sums of
// non-negative terms, so their d roundings cost at most d 2^-23 relatively: rounded up by more than that).
// Stored per (token, candidate), as fp32 - with phi = identity (RELU false: the classifier) the sum itself; with
// the ReLU: the sum if it is positive (never rounded to zero); the smallest
// positive float if it lies in (-2 delta, 0], where the true activation may still be positive; exactly 0 below
// that, where the true activation is exactly 0.  The selection (k_select_refine) recomputes in fp64 the entries
// whose stored value lies within 2 max_j delta(b, j) of the k-th largest stored value and selects on the result:
// the selected set is that of the fp64 values.  xnorm[b] receives an upper bound of |x_b| (tile 0), *wnorm_max (float bits, atomic
// max, cleared by the step's first kernel) one of the largest |u_j| over the candidates.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& u) {
  bf16x8 v;
  __builtin_memcpy(&v, &u, sizeof(v));
  return v;
}
__device__ __forceinline__ float pick4(const f32x4& v, int i) {
  return i == 0 ? v[0] : (i == 1 ? v[1] : (i == 2 ? v[2] : v[3]));
}

// profiling build: the same stamps for the grid's last workgroup, four slots further on
#ifdef HIRE_TIMESTAMPS
#define HIRE_TS_BOTH(i)                                                              \
  do {                                                                               \
    HIRE_TS(i);                                                                      \
    if (threadIdx.x == 0 && blockIdx.x == gridDim.x - 1 && blockIdx.y == 0) {        \
      hire_ts[(i) + 4] = wall_clock64();                                             \
      hire_ts[64 + (i) + 4] = clock64();                                             \
    }                                                                                \
  } while (0)
#else
#define HIRE_TS_BOTH(i) ((void)0)
#endif

constexpr int kWaveLocateWords = 512;

// The indices of the set bits with ranks [r0, r0 + R) of a bitmap of at most 512 words, found by one wave on its
// own (lane l holds words 8 l .. 8 l + 7, requested by issue()): no barrier, so loads issued after the bitmap's
// stay in flight meanwhile.  out[r - r0] receives the index of rank r (this wave's LDS); returns the number of set bits.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct WaveBitmap {
  uint4 lo, hi;
  __device__ __forceinline__ void issue(const uint32_t* __restrict__ bitmap, int words) {
    const uint4* b4 = reinterpret_cast<const uint4*>(bitmap);
    const int last_vec = (words - 1) / 4, lane = lane_id();
    lo = b4[min(2 * lane, last_vec)];
    hi = b4[min(2 * lane + 1, last_vec)];
  }
};
__device__ __forceinline__ int wave_locate(const WaveBitmap& wb, int words, int r0, int R, int32_t* out) {
  const int lane = lane_id();
  const uint4 lo = wb.lo, hi = wb.hi;
  uint32_t m[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  int c = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    m[i] = 8 * lane + i < words ? m[i] : 0u;  // clamped loads repeat words, the last vector may reach past the bitmap
    c += __popc(m[i]);
  }
  const int incl = wave_scan_incl(c);
  const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
  // lane j resolves rank r0 + j (R <= 64): the lane that holds it by bisection over the lanes' running counts, the
  // word among that lane's eight, the bit inside the word by bisection over its halves
  const int r = r0 + lane;
  int lo_l = 0, hi_l = kWave - 1;
#pragma unroll
  for (int st = 0; st < 6; ++st) {
    const int mid = (lo_l + hi_l) >> 1;
    const int v = __shfl(incl, mid);
    if (v > r) hi_l = mid;
    else lo_l = mid + 1;
  }
  const int owner = min(lo_l, kWave - 1);
  int rem = r - __shfl(incl - c, owner);  // which of the owner's bits
  uint32_t word = 0u;
  int widx = 0;
  bool found = false;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t wi = (uint32_t)__shfl((int)m[i], owner);
    const int pc = __popc(wi);
    if (!found && rem < pc) {
      word = wi;
      widx = i;
      found = true;
    }
    if (!found) rem -= pc;
  }
  int pos = 0;
#pragma unroll
  for (int sh = 16; sh >= 1; sh >>= 1) {
    const int below = __popc(word & (((1u << sh) - 1u) << pos));
    if (rem >= below) {
      rem -= below;
      pos += sh;
    }
  }
  if (lane < R && r < total && found) out[lane] = (8 * owner + widx) * 32 + pos;
  wave_lds_fence();
  return total;
}

// Operands pass through LDS: a lane of the matrix cores wants 16 bytes of each of 16 different rows, which as a
// global load touches 16 cache lines per quarter wave; instead every load instruction brings 1 KiB of one row
// (lane l its chunk l) and an LDS slab of 16 rows (row stride 1040 bytes: conflict-free 16-byte reads down a
// column) turns them round.  A workgroup of NWV waves owns 16 NWV candidates, 16 per wave, and all of the batch's
// tokens (TT tiles of 16); K goes by in passes of 64 chunks (512 elements).  Per pass the waves stage the tokens' slab
// together; every wave stages its own candidates' slab, whose loads for the next pass are requested before the
// matrix cores start on this one, so that candidate rows are in flight all the time.  The barriers between the
// phases wait for LDS only, not for those loads.
constexpr int kSlabChunks = 64;                          // 16-byte chunks of a row per pass: one per lane
constexpr int kSlabRowBytes = kSlabChunks * 16 + 16;     // padded
constexpr int kSlabBytes = 16 * kSlabRowBytes;           // 16 rows
constexpr int kSlabSteps = kSlabChunks / 4;              // MFMA steps per pass
static_assert(sizeof(SelSharedT<256>) <= 4 * (size_t)kSlabBytes, "the long-bitmap search borrows the slabs' memory");

// Workgroup barrier that orders LDS traffic only: global loads stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int TT, int NWV, int TSPLIT, bool RELU>
__global__ __launch_bounds__(64 * NWV * TSPLIT) void k_gather_dot_bf16(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                                         int B, int d, const int32_t* __restrict__ list, int n_host,
                                                         const int32_t* __restrict__ n_dev, int n_cap,
                                                         float* __restrict__ h, long long stride_h, GatherUnion un,
                                                         float* __restrict__ xnorm, uint32_t* __restrict__ wnorm_max,
                                                         float err_c) {
  // NWV groups of 16 candidates, each shared by TSPLIT waves that take TT / TSPLIT of the token tiles (and
  // 16 / TSPLIT of the group's rows when its slab is staged)
  constexpr int NW = NWV * TSPLIT, TTW = TT / TSPLIT, RPW = 16 / TSPLIT;
  static_assert(TT <= NWV && 16 * TT % NW == 0 && TT % TSPLIT == 0 && 16 % TSPLIT == 0,
                "one wave per token tile for the norms, equal shares of the tokens' and candidates' rows");
  constexpr int kTile = 16 * NWV;  // candidates of the workgroup
  extern __shared__ __align__(16) unsigned char lds[];  // NWV candidate slabs (one per wave), then TT token slabs
  __shared__ float xsq[TT][16];
  __shared__ float wmx[NW];
  __shared__ int32_t rows_sh[kTile];  // the tile's candidates
  __shared__ int n_sh;
  const int tile = (int)blockIdx.x;
  const int lane = lane_id(), jl = lane & 15, g = lane >> 4;
  // known to be uniform: a matrix-core instruction must never sit behind a branch that is lowered to lane masking
  const int w = __builtin_amdgcn_readfirstlane(wave_id());
  const int e0 = tile * kTile;
  const int cpr = d / 8;  // 16-byte chunks per row
  HIRE_TS_BOTH(55);
  // The tile's candidates: wave 0 finds them in a short bitmap on its own, a long bitmap takes the whole
  // workgroup, a list is read.
  const bool in_wave = un.bitmap != nullptr && un.words <= kWaveLocateWords;
  if (in_wave) {
    if (w == 0) {
      WaveBitmap wb;
      wb.issue(un.bitmap, un.words);
      const int total = wave_locate(wb, un.words, e0, kTile, rows_sh);
      if (lane == 0) n_sh = total;
    }
  } else if (un.bitmap != nullptr) {
    const int total = union_locate<64 * NW>(un.bitmap, un.words, *reinterpret_cast<SelSharedT<64 * NW>*>(lds), e0, kTile, rows_sh);
    if (threadIdx.x == 0) n_sh = total;
  } else {
    const int total = n_dev ? *n_dev : n_host;
    const int t = (int)threadIdx.x;
    if (t < kTile) rows_sh[t] = list != nullptr ? list[min(e0 + t, max(min(total, n_cap), 1) - 1)] : e0 + t;
    if (t == 0) n_sh = total;
  }
  __syncthreads();
  const int n = min(n_sh, n_cap);
  if (un.bitmap != nullptr) {
    if (tile == 0) publish_union(un, n);
    const int t = (int)threadIdx.x;
    if (t < kTile && e0 + t < n) un.list_out[e0 + t] = rows_sh[t];
  }
  HIRE_TS_BOTH(56);
  if (e0 >= n) return;  // uniform over the workgroup
  const int cw = w % NWV, tsp = w / NWV;  // candidate group, share of the token tiles (uniform)
  const int tt0 = tsp * TTW;
  unsigned char* wslab = lds + cw * kSlabBytes;
  unsigned char* xslab = lds + NWV * kSlabBytes;
  const unsigned char* wcol = wslab + jl * kSlabRowBytes + 16 * g;  // this lane's operand of step u: + 64 u
  const unsigned char* xcol = xslab + jl * kSlabRowBytes + 16 * g;  // ... of token tile tt: + tt * kSlabBytes
  double acc[TTW][4];
#pragma unroll
  for (int tt = 0; tt < TTW; ++tt)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[tt][r] = 0.0;
  const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
  f32x4 accw = zero, accx = zero;  // rows times rows (this wave's 16), tokens times tokens (one tile, for some waves)
  // A pass's operands in registers: this wave's 16 candidate rows (one register per row) and its share of the
  // tokens' rows (rows w, w + NWV, ... of the 16 TT; tokens past the batch are zeros), all requested together.
  // DEPTH such sets are in flight; with many token tiles (little register space, long matrix-core phases) the
  // tokens are requested at the start of their own pass instead.
  constexpr int DEPTH = TTW <= 2 ? 2 : 1;
  constexpr bool kTokensAhead = TTW <= 2;
  constexpr int kLdsBatch = TTW == 1 ? 4 : 2;
  constexpr int kSegSteps = filter_segment_steps(16 * TT);
  static_assert(kLdsBatch % kSegSteps == 0 && kSlabSteps % kLdsBatch == 0, "whole segments per batch");
  struct Operands {
    uint4 wv[RPW];
    uint4 xv[16 * TT / NW];
  };
  auto request_tokens = [&](int cs, Operands& o) {
    const int nch = min(kSlabChunks, cpr - cs);
#pragma unroll
    for (int i = 0; i < 16 * TT / NW; ++i) {
      const int row = w + NW * i;
      o.xv[i] = make_uint4(0, 0, 0, 0);
      if (lane < nch && row < B) o.xv[i] = reinterpret_cast<const uint4*>(x + (size_t)row * d)[cs + lane];
    }
  };
  auto request = [&](int cs, Operands& o) {
    const int nch = min(kSlabChunks, cpr - cs);
#pragma unroll
    for (int r = 0; r < RPW; ++r) {
      o.wv[r] = make_uint4(0, 0, 0, 0);
      const int cand = __builtin_amdgcn_readfirstlane(rows_sh[min(e0 + 16 * cw + tsp * RPW + r, n - 1) - e0]);  // scalar address
      if (lane < nch) o.wv[r] = reinterpret_cast<const uint4*>(W + (size_t)cand * d)[cs + lane];
    }
    if (kTokensAhead) request_tokens(cs, o);
  };
  // One pass: the operands go to LDS, their registers are asked to fetch the pass DEPTH further on, the matrix
  // cores work.
  auto run_pass = [&](int cs, Operands& o) {
    const int nch = min(kSlabChunks, cpr - cs), steps = (nch + 3) / 4;  // uniform
    [[maybe_unused]] const int ts0 = 1 + 6 * min(cs / kSlabChunks, 7);  // profiling build: six stamps per pass
    HIRE_TS(ts0);
    if (!kTokensAhead) request_tokens(cs, o);
#pragma unroll
    for (int i = 0; i < 16 * TT / NW; ++i)
      *reinterpret_cast<uint4*>(xslab + (w + NW * i) * kSlabRowBytes + 16 * lane) = o.xv[i];
    HIRE_TS(ts0 + 1);
#pragma unroll
    for (int r = 0; r < RPW; ++r)
      *reinterpret_cast<uint4*>(wslab + (tsp * RPW + r) * kSlabRowBytes + 16 * lane) = o.wv[r];
    HIRE_TS(ts0 + 2);
    if (cs + DEPTH * kSlabChunks < cpr) request(cs + DEPTH * kSlabChunks, o);  // in flight while the matrix cores work
    lds_barrier();
    HIRE_TS(ts0 + 3);
    // operands come from LDS kLdsBatch steps at a time: one wait for their latency, not one per step
#pragma unroll
    for (int u0 = 0; u0 < kSlabSteps; u0 += kLdsBatch) {
      if (u0 < steps) {  // uniform; steps past the row's end inside a batch multiply zeros
        bf16x8 wk[kLdsBatch], tk[TTW][kLdsBatch];
#pragma unroll
        for (int v = 0; v < kLdsBatch; ++v) {
          wk[v] = as_bf16x8(*reinterpret_cast<const uint4*>(wcol + 64 * (u0 + v)));
#pragma unroll
          for (int tt = 0; tt < TTW; ++tt)
            tk[tt][v] = as_bf16x8(*reinterpret_cast<const uint4*>(xcol + (tt0 + tt) * kSlabBytes + 64 * (u0 + v)));
        }
        // kSegSteps steps (32 products each) per fp32 segment; the segments of a batch are started side by side so
        // that no matrix-core instruction waits for the one issued just before it
        constexpr int kSeg = kLdsBatch / kSegSteps;
#pragma unroll
        for (int v = 0; v < kLdsBatch; ++v) accw = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wk[v], wk[v], accw, 0, 0, 0);
        f32x4 part[TTW][kSeg];
#pragma unroll
        for (int tt = 0; tt < TTW; ++tt)
#pragma unroll
          for (int q = 0; q < kSeg; ++q)
            part[tt][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[tt][kSegSteps * q], wk[kSegSteps * q], zero, 0, 0, 0);
#pragma unroll
        for (int st = 1; st < kSegSteps; ++st)
#pragma unroll
          for (int tt = 0; tt < TTW; ++tt)
#pragma unroll
            for (int q = 0; q < kSeg; ++q)
              part[tt][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[tt][kSegSteps * q + st], wk[kSegSteps * q + st],
                                                                    part[tt][q], 0, 0, 0);
#pragma unroll
        for (int tt = 0; tt < TTW; ++tt) {
          if ((tt0 + tt) % NWV == cw) {  // uniform: token tile t's norms are formed by the wave of group t % NWV that has it
#pragma unroll
            for (int v = 0; v < kLdsBatch; ++v)
              accx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[tt][v], tk[tt][v], accx, 0, 0, 0);
          }
#pragma unroll
          for (int q = 0; q < kSeg; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[tt][r] += (double)part[tt][q][r];
        }
      }
    }
    HIRE_TS(ts0 + 4);
    lds_barrier();  // the slabs are read before they are filled again
    HIRE_TS(ts0 + 5);
  };
  Operands op[DEPTH];
#pragma unroll
  for (int q = 0; q < DEPTH; ++q)
    if (q * kSlabChunks < cpr) request(q * kSlabChunks, op[q]);
#pragma nounroll
  for (int cs = 0; cs < cpr; cs += DEPTH * kSlabChunks) {
#pragma unroll
    for (int q = 0; q < DEPTH; ++q)
      if (cs + q * kSlabChunks < cpr) run_pass(cs + q * kSlabChunks, op[q]);  // uniform
  }
  HIRE_TS_BOTH(57);
  // entry (i, i) of a 16 x 16 result sits in value i % 4 of lane 16 (i / 4) + i
  const float up = 1.0f + (float)d * 0x1p-22f;  // more than the relative error of the norms' sums
  if (cw < TT && cw / TTW == tsp && (jl >> 2) == g) xsq[cw][jl] = pick4(accx, jl & 3);
  float wn2 = (jl >> 2) == g ? pick4(accw, jl & 3) : 0.0f;  // |u_jl|^2 sits in lane 16 (jl / 4) + jl: to all four
  wn2 = fmaxf(wn2, __shfl_xor(wn2, 16));
  wn2 = fmaxf(wn2, __shfl_xor(wn2, 32));
  const float wnorm = sqrtf(wn2 * up) * 1.0001f;
  const int t_idx = e0 + 16 * cw + jl;
  {
    float m = t_idx < n ? wnorm : 0.0f;
    m = fmaxf(m, __shfl_xor(m, 1));
    m = fmaxf(m, __shfl_xor(m, 2));
    m = fmaxf(m, __shfl_xor(m, 4));
    m = fmaxf(m, __shfl_xor(m, 8));
    if (lane == 0) wmx[w] = m;
  }
  __syncthreads();
  // what the maximum holds so far: requested before the stores below, looked at after them (and after the
  // barrier, which would wait for it)
  uint32_t seen_max = 0u;
  if (w == 0 && lane == 0) seen_max = *reinterpret_cast<volatile uint32_t*>(wnorm_max);
#pragma unroll
  for (int tt = 0; tt < TTW; ++tt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int tl = 4 * g + r, tk = 16 * (tt0 + tt) + tl;
      const float xnrm = sqrtf(xsq[tt0 + tt][tl] * up) * 1.0001f;
      const double s = acc[tt][r];
      const double delta = (double)(err_c * wnorm * xnrm);
      const float tiny = __uint_as_float(1u);  // the smallest positive float
      float v = (float)s;  // phi = identity (the classifier): the sum itself
      if constexpr (RELU) {
        v = 0.0f;
        if (s > 0.0) v = fmaxf((float)s, tiny);
        else if (s > -2.0 * delta) v = tiny;  // the true activation may still be positive
      }
      if (tk < B && t_idx < n) h[(size_t)tk * stride_h + t_idx] = v;
    }
  if (w == 0) {  // one atomic per workgroup at most
    float m = wmx[0];
#pragma unroll
    for (int q = 1; q < NW; ++q) m = fmaxf(m, wmx[q]);
    // most workgroups found a maximum at least as large already there and skip the atomic
    if (lane == 0 && __float_as_uint(m) > seen_max) atomicMax(wnorm_max, __float_as_uint(m));
  }
  if (tile == 0 && w == 0) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
      if (lane < 16 && 16 * tt + lane < B) xnorm[16 * tt + lane] = sqrtf(xsq[tt][lane] * up) * 1.0001f;
  }
  HIRE_TS_BOTH(58);
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

hipError_t launch_gather_dot_bf16(const uint16_t* W, const uint16_t* x, int B, int d, const int32_t* list,
                                  const int32_t* n_dev, int n_cap, float* h, long long stride_h, const HistRefs& hr,
                                  const UnionRefs* un, int n_rows, int relu, float* xnorm, uint32_t* wnorm_max,
                                  hipStream_t s) {
  GatherUnion u = make_gather_union(un, hr, B);
  u.words = min(u.words, (n_rows + 31) / 32);  // the bitmap's padding words hold no bits
  if (B < 1 || B > 64) return hipErrorInvalidValue;
  static std::atomic<size_t> raised_to[8] = {};
  auto go = [&](auto kernel, int tt, int nwv, int tsplit, std::atomic<size_t>& raised) {
    const size_t lds = (size_t)(nwv + tt) * kSlabBytes;
    if (const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kernel), lds, raised); e != hipSuccess)
      return e;
    const int tile = 16 * nwv;
    return launch(kernel, dim3(max(1, (n_cap + tile - 1) / tile)), dim3(64 * nwv * tsplit), lds, s, W, x, B, d,
                  u.bitmap ? nullptr : list, 0, n_dev, n_cap, h, stride_h, u, xnorm, wnorm_max, gather_filter_error(B));
  };
  // few tokens: small workgroups, so that every compute unit holds several and has enough loads in flight;
  // beyond 32 tokens two waves share a group of candidates, two token tiles each: the fp64 additions that pace
  // the passes are spread over twice the waves
  const bool small = B <= 16 && (u.bitmap == nullptr || u.words <= kWaveLocateWords);
  if (relu) {
    if (small) return go(k_gather_dot_bf16<1, 2, 1, true>, 1, 2, 1, raised_to[0]);
    if (B <= 16) return go(k_gather_dot_bf16<1, 4, 1, true>, 1, 4, 1, raised_to[1]);
    if (B <= 32) return go(k_gather_dot_bf16<2, 4, 1, true>, 2, 4, 1, raised_to[2]);
    return go(k_gather_dot_bf16<4, 4, 2, true>, 4, 4, 2, raised_to[3]);
  }
  if (small) return go(k_gather_dot_bf16<1, 2, 1, false>, 1, 2, 1, raised_to[4]);
  if (B <= 16) return go(k_gather_dot_bf16<1, 4, 1, false>, 1, 4, 1, raised_to[5]);
  if (B <= 32) return go(k_gather_dot_bf16<2, 4, 1, false>, 2, 4, 1, raised_to[6]);
  return go(k_gather_dot_bf16<4, 4, 2, false>, 4, 4, 2, raised_to[7]);
}

}  // namespace hire

#ifdef HIRE_TIMESTAMPS
extern "C" int hire_debug_timestamps_gather(unsigned long long* host64) {
  return (int)hipMemcpyFromSymbol(host64, HIP_SYMBOL(hire_ts), sizeof(hire_ts));
}
#endif
