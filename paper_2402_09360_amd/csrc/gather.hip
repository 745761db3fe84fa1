// Exact stage of HiRE (arXiv 2402.09360, Algorithm 1 line 2 and eq. (4)):
//   gather_dot    h[b,t] = phi(<z_{U[t]}, x_b>) over the candidate rows only
//   w2_tokens     y_b    = sum_{j in S_b} h[b,j] v_j over the selected rows only
// Rows are unit-major, so every gathered row is one contiguous run of 2*d bytes
// read with 16-byte loads.
//
// gather_dot accumulates in fp64: a bf16*bf16 product is exact in fp32, and
// fp64 sums of such products differ between summation orders only in the last
// bits, which keeps the top-k decision that follows independent of the order.
#include "device_utils.h"
#include "hist.h"
#include "kernels.h"

namespace hire {

// One token: a wave per candidate row, the token in LDS as raw bf16.  The candidates come either as a list
// (list != nullptr, count from n_dev or n_host) or as the union bitmap, which every workgroup compacts for its
// own contiguous share of ranks (union_locate); it then also writes that share of the ascending candidate list,
// and workgroup 0 the count.
// gs > 0 (group-sparse FFN, eq. (6)): the candidates are groups of 2^gs adjacent rows; entry e of the list stands
// for rows list[e] * 2^gs + l, l < 2^gs, whose results go to h[e * 2^gs + l].  Counts and capacities stay in
// entries.
__global__ __launch_bounds__(256) void k_gather_dot(const uint16_t* __restrict__ W, const uint16_t* __restrict__ x,
                                                    int d, const int32_t* __restrict__ list, int n_host,
                                                    const int32_t* __restrict__ n_dev, int n_cap, int relu,
                                                    double* __restrict__ h, GatherUnion un, int share, int gs) {
  extern __shared__ uint4 xs[];  // [d/8] raw bf16 token, then (bitmap mode) the indices of the workgroup's ranks
  __shared__ SelSharedT<256> sh;
  const int cpr = d / 8;         // 16-byte chunks per row
  const int lane = lane_id();
  for (int i = (int)threadIdx.x; i < cpr; i += 256) xs[i] = reinterpret_cast<const uint4*>(x)[i];
  // ranks of this workgroup: a contiguous share of the capacity
  const int r0 = (int)blockIdx.x * share;
  const int gmask = (1 << gs) - 1;
  int n;
  const int32_t* rows;  // indices of ranks r0 ..
  if (un.bitmap != nullptr) {
    int32_t* mine = reinterpret_cast<int32_t*>(xs + cpr);
    n = un.words <= 4 * 64 * kLocateStepsShort ? union_locate<256, kLocateStepsShort>(un.bitmap, un.words, sh, r0, share, mine)
                                               : union_locate<256>(un.bitmap, un.words, sh, r0, share, mine);
    n = min(n, n_cap);
    if (blockIdx.x == 0) publish_union(un, n);
    for (int t = (int)threadIdx.x; t < share && r0 + t < n; t += 256) un.list_out[r0 + t] = mine[t];
    rows = mine;
  } else {
    n = n_dev ? min(*n_dev, n_cap) : n_host;
    rows = list ? list + r0 : nullptr;  // no list: entry e is row e itself
    __syncthreads();
  }
  for (int t = wave_id(); t < (share << gs) && r0 + (t >> gs) < n; t += 4) {
    const int entry = rows ? rows[t >> gs] : r0 + (t >> gs);
    const uint4* row = reinterpret_cast<const uint4*>(W + (((size_t)entry << gs) + (t & gmask)) * d);
    double acc = 0.0;
#pragma unroll 4
    for (int c = lane; c < cpr; c += kWave) {
      const uint4 wv = load_streaming(&row[c]);
      const uint32_t wd[4] = {wv.x, wv.y, wv.z, wv.w};
      const uint4 xv = xs[c];
      const uint32_t xd[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc += (double)(bf16_lo(wd[q]) * bf16_lo(xd[q]));
        acc += (double)(bf16_hi(wd[q]) * bf16_hi(xd[q]));
      }
    }
    double s = wave_sum(acc);
    if (relu) s = s > 0.0 ? s : 0.0;
    if (s == 0.0) s = 0.0;
    if (lane == 0) h[((size_t)r0 << gs) + t] = s;
  }
}

// ---------------------------------------------------------------------------
// Second layer, token by token: y_b = sum_{i < k} fl32(h[b, pos[b, i]]) * W2[map[pos[b, i]], :].
// grid = (column slices of 512, row groups, tokens).  Wave w of a block takes batches of eight of its row
// group's entries: the eight positions, row numbers and coefficients are fetched by eight lanes and handed
// round as wave-uniform values, so the eight row loads (16 bytes per lane, 8 columns) are in flight together
// instead of each waiting for its own index chain.  The four waves are summed through LDS in a fixed order and
// the block writes one partial row; k_w2_reduce then adds the groups in a fixed order.  Rows chosen by several
// tokens are read once per token; the repeats are served by the caches.
// gs > 0 (group-sparse FFN): pos lists k >> gs selected groups per token; entry e < k is unit e % 2^gs of group
// e >> gs, its row map[pos] * 2^gs + l and its coefficient h[pos * 2^gs + l].  val_out (optional): the k
// coefficients in entry order, as fp32.
constexpr int kW2Cols = 512;
constexpr int kW2Batch = 8;

__global__ __launch_bounds__(256) void k_w2_tokens(const uint16_t* __restrict__ W2, int d, int k,
                                                   const int32_t* __restrict__ pos, const int32_t* __restrict__ map,
                                                   const double* __restrict__ h, long long h_stride,
                                                   float* __restrict__ partial, int gs,
                                                   float* __restrict__ val_out) {
  __shared__ float red[4][kW2Cols];
  const int groups = (int)gridDim.y, g = (int)blockIdx.y, b = (int)blockIdx.z, B = (int)gridDim.z;
  const int rpg = (k + groups - 1) / groups;
  const int p0 = g * rpg, p1 = min(k, p0 + rpg);
  const int lane = lane_id(), w = wave_id();
  const int col0 = (int)blockIdx.x * kW2Cols + lane * 8;
  const int colc = min(col0, d - 8);  // d is a multiple of 8
  float acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
  // wave w owns entries p0 + w*kW2Batch + [0, kW2Batch), then strides by four batches
  for (int pb = p0 + w * kW2Batch; pb < p1; pb += 4 * kW2Batch) {
    const int pe = min(pb + (lane & (kW2Batch - 1)), p1 - 1);
    const int l = pe & ((1 << gs) - 1);
    const int ps = pos ? pos[(size_t)b * (k >> gs) + (pe >> gs)] : pe >> gs;  // no list: all k entries in order
    const int row = ((map ? map[ps] : ps) << gs) + l;
    const float c = (float)h[(size_t)b * h_stride + ((size_t)ps << gs) + l];
    if (val_out != nullptr && blockIdx.x == 0 && lane < kW2Batch && pb + lane < p1) val_out[(size_t)b * k + pe] = c;
    uint4 wv[kW2Batch];
#pragma unroll
    for (int u = 0; u < kW2Batch; ++u) {
      const int ru = __builtin_amdgcn_readlane(row, u);
      wv[u] = *reinterpret_cast<const uint4*>(W2 + (size_t)ru * d + colc);
    }
#pragma unroll
    for (int u = 0; u < kW2Batch; ++u) {
      float cu = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c), u));
      if (pb + u >= p1) cu = 0.0f;
      const float wf[8] = {bf16_lo(wv[u].x), bf16_hi(wv[u].x), bf16_lo(wv[u].y), bf16_hi(wv[u].y),
                           bf16_lo(wv[u].z), bf16_hi(wv[u].z), bf16_lo(wv[u].w), bf16_hi(wv[u].w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(cu, wf[q], acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) red[w][lane * 8 + q] = acc[q];
  __syncthreads();
  // 256 threads, 512 columns: two columns each, waves added in order 0..3
  for (int c = (int)threadIdx.x; c < kW2Cols; c += 256) {
    const int col = (int)blockIdx.x * kW2Cols + c;
    if (col < d) partial[((size_t)g * B + b) * d + col] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
  }
}

// The same product for plain units (no groups), one kernel: a workgroup owns 64 columns (128 bytes of every
// selected row) of one token and all of its k rows, so it writes y itself and nothing has to be reduced across
// workgroups.  The token's rows and coefficients go to LDS first (two dependent loads per entry, all in flight
// together); then eight lanes share a row, a wave reads eight rows per instruction and has eight instructions in
// flight; the lanes' sums are folded by a fixed shuffle tree, the waves' through LDS in wave order.
constexpr int kW2dMaxK = 4096;

// LPR: lanes per row (8 columns each)
template <int LPR>
__global__ __launch_bounds__(256) void k_w2_direct(const uint16_t* __restrict__ W2, int d, int k,
                                                   const int32_t* __restrict__ pos, const int32_t* __restrict__ map,
                                                   const double* __restrict__ h, long long h_stride,
                                                   float* __restrict__ y, float* __restrict__ val_out) {
  __shared__ int32_t rows_l[kW2dMaxK];
  __shared__ float coef_l[kW2dMaxK];
  constexpr int kW2dCols = 8 * LPR, RPI = kWave / LPR;  // columns of the workgroup, rows per wave and instruction
  __shared__ float red[4][kW2dCols];
  const int b = (int)blockIdx.y, tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
  for (int t0 = tid; t0 < k; t0 += 4 * 256) {  // four entries per thread in flight
    int ps[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ps[u] = pos ? pos[(size_t)b * k + min(t0 + u * 256, k - 1)] : min(t0 + u * 256, k - 1);
    int row[4];
    double hv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      row[u] = map ? map[ps[u]] : ps[u];
      hv[u] = h[(size_t)b * h_stride + ps[u]];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = t0 + u * 256;
      if (t < k) {
        rows_l[t] = row[u];
        coef_l[t] = (float)hv[u];
        if (val_out != nullptr && blockIdx.x == 0) val_out[(size_t)b * k + t] = (float)hv[u];
      }
    }
  }
  __syncthreads();
  const int sub = lane % LPR, rw = lane / LPR;
  const int col0 = (int)blockIdx.x * kW2dCols + sub * 8;
  const int colc = min(col0, d - 8);  // d is a multiple of 8
  float acc[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) acc[q] = 0.0f;
  for (int tb = w * RPI + rw; tb < k; tb += 8 * 4 * RPI) {  // lane's rows tb, tb + 4 RPI, ...: eight in flight
    uint4 wv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = min(tb + u * 4 * RPI, k - 1);
      wv[u] = *reinterpret_cast<const uint4*>(W2 + (size_t)rows_l[t] * d + colc);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = tb + u * 4 * RPI;
      const float c = t < k ? coef_l[t] : 0.0f;
      const float wf[8] = {bf16_lo(wv[u].x), bf16_hi(wv[u].x), bf16_lo(wv[u].y), bf16_hi(wv[u].y),
                           bf16_lo(wv[u].z), bf16_hi(wv[u].z), bf16_lo(wv[u].w), bf16_hi(wv[u].w)};
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = fmaf(c, wf[q], acc[q]);
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) {  // the row lanes of a column chunk
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) acc[q] += __shfl_xor(acc[q], m);
  }
  if (rw == 0) {
#pragma unroll
    for (int q = 0; q < 8; ++q) red[w][sub * 8 + q] = acc[q];
  }
  __syncthreads();
  if (tid < kW2dCols) {
    const int col = (int)blockIdx.x * kW2dCols + tid;
    if (col < d) y[(size_t)b * d + col] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
  }
}

// accumulate: add to what y holds (the dense common path on top of the sparse part).
__global__ __launch_bounds__(256) void k_w2_reduce(const float* __restrict__ partial, int groups, int B, int d,
                                                   float* __restrict__ y, int accumulate) {
  const int col = (int)(blockIdx.x * blockDim.x + threadIdx.x), b = (int)blockIdx.y;
  if (col >= d) return;
  float s = 0.0f;
  for (int g0 = 0; g0 < groups; g0 += 8) {  // eight loads in flight; added in group order
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = partial[((size_t)min(g0 + j, groups - 1) * B + b) * d + col];
#pragma unroll
    for (int j = 0; j < 8; ++j) s += g0 + j < groups ? v[j] : 0.0f;
  }
  y[(size_t)b * d + col] = accumulate ? y[(size_t)b * d + col] + s : s;
}

// ---------------------------------------------------------------------------
// Group sums (eq. (6)): out[b, J] = sum_{l < 2^gs} |in[b, J * 2^gs + l]|, added in index order in the type of
// the input, for J < n (n from n_dev if given).
template <typename T>
__global__ __launch_bounds__(256) void k_group_sums(const T* __restrict__ in, long long stride_in, int n_host,
                                                    const int32_t* __restrict__ n_dev, int n_cap, int gs,
                                                    T* __restrict__ out, long long stride_out) {
  const int n = n_dev ? min(*n_dev, n_cap) : n_host;
  const int J = (int)(blockIdx.x * blockDim.x + threadIdx.x), b = (int)blockIdx.y;
  if (J >= n) return;
  const T* src = in + (size_t)b * stride_in + ((size_t)J << gs);
  T sum = (T)0;
  for (int l0 = 0; l0 < (1 << gs); l0 += 4) {  // group sizes 1, 2 or a multiple of 4
    T v[4];
#pragma unroll
    for (int l = 0; l < 4; ++l) v[l] = src[min(l0 + l, (1 << gs) - 1)];
#pragma unroll
    for (int l = 0; l < 4; ++l)
      if (l0 + l < (1 << gs)) sum += v[l] < (T)0 ? -v[l] : v[l];
  }
  out[(size_t)b * stride_out + J] = sum;
}

template <typename T>
static hipError_t group_sums(const T* in, int B, long long stride_in, int n, const int32_t* n_dev, int n_cap, int gs,
                             T* out, long long stride_out, hipStream_t s) {
  const int cap = n_dev ? n_cap : n;
  return launch(k_group_sums<T>, dim3((cap + 255) / 256, B), dim3(256), 0, s, in, stride_in, n, n_dev, n_cap, gs, out,
                stride_out);
}
hipError_t launch_group_sums_f32(const float* in, int B, long long stride_in, int n, int gs, float* out,
                                 long long stride_out, hipStream_t s) {
  return group_sums<float>(in, B, stride_in, n, nullptr, n, gs, out, stride_out, s);
}
hipError_t launch_group_sums_f64(const double* in, int B, long long stride_in, int n, const int32_t* n_dev, int n_cap,
                                 int gs, double* out, long long stride_out, hipStream_t s) {
  return group_sums<double>(in, B, stride_in, n, n_dev, n_cap, gs, out, stride_out, s);
}

// Entries per workgroup: about four rows (one per wave), more once 2048 workgroups no longer cover the list.
static int gather_dot_share(int cap, int gs) { return max(max(1, 4 >> gs), (cap + 2047) / 2048); }

bool union_in_gather(int words) { return words <= kUnionLocateMaxWords; }

hipError_t launch_gather_dot(const uint16_t* W, const uint16_t* x, int d, const int32_t* list, int n,
                             const int32_t* n_dev, int n_cap, int relu, double* h, const HistRefs& hr,
                             const UnionRefs* un, int gs, hipStream_t s) {
  const int cap = n_dev ? n_cap : n;
  const GatherUnion u = make_gather_union(un, hr, 1);
  const int share = gather_dot_share(cap, gs);
  const int blocks = max(1, (cap + share - 1) / share);
  size_t lds = (size_t)d * 2;
  if (u.bitmap) lds += (size_t)share * 4;
  return launch(k_gather_dot, dim3(blocks), dim3(256), lds, s, W, x, d, u.bitmap ? nullptr : list, n, n_dev, cap, relu, h,
                u, share, gs);
}

// Row groups per token: enough workgroups to fill the machine, at least a few batches of rows each.
int w2_groups(int k, int B, int d) {
  const int slices = (d + kW2Cols - 1) / kW2Cols;
  int g = 1024 / (slices * B);
  const int by_rows = (k + 4 * kW2Batch - 1) / (4 * kW2Batch);
  if (g > by_rows) g = by_rows;
  if (g > 64) g = 64;
  if (g < 1) g = 1;
  return g;
}

hipError_t launch_w2_tokens(const uint16_t* W2, int d, int B, int k, const int32_t* pos, const int32_t* map,
                            const double* h, long long h_stride, float* partial, float* y, int gs, float* val_out,
                            int accumulate, hipStream_t s) {
  // many tokens, plain units: one kernel, no partial sums (256 columns per workgroup still make 8 B workgroups)
  if (gs == 0 && !accumulate && k <= kW2dMaxK && d % 256 == 0 && B >= 32)
    return launch(k_w2_direct<32>, dim3(d / 256, B), dim3(256), 0, s, W2, d, k, pos, map, h, h_stride, y, val_out);
  const int groups = w2_groups(k, B, d);
  const int slices = (d + kW2Cols - 1) / kW2Cols;
  hipError_t e = launch(k_w2_tokens, dim3(slices, groups, B), dim3(256), 0, s, W2, d, k, pos, map, h, h_stride,
                        partial, gs, val_out);
  if (e != hipSuccess) return e;
  return launch(k_w2_reduce, dim3((d + 255) / 256, B), dim3(256), 0, s, partial, groups, B, d, y, accumulate);
}

}  // namespace hire
