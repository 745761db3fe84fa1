// Fine key histograms that guide the exact selections: one counter per 2^14 consecutive order keys (sign,
// exponent and the top nine mantissa bits of an fp32), filled with integer atomics by the kernel that produces
// the keys, walked from the largest key downwards by the kernels that select.  With ~one key per counter the
// atomics do not queue up behind one another (same-address atomics complete at ~30 ns each on this machine),
// and the bin that holds the k-th largest key contains only a handful of keys, which are ranked directly.
#pragma once

#include "kernels.h"
#include "select.h"

namespace hire {

constexpr int kHistShift = 14;
constexpr int kHistWindow = 8192;                    // bins walked at and below the largest key (16 octaves)
constexpr int kHistBins = 1 << (32 - kHistShift);    // 262144: all order keys
constexpr int kHistStride = kHistWindow + kHistBins; // words per histogram; the first kHistWindow words stay zero
                                                     // so that a window may reach below bin 0

__device__ __forceinline__ uint32_t hist_bin(uint32_t okey) { return okey >> kHistShift; }
__device__ __forceinline__ uint32_t hist_bin(uint64_t okey) {  // fp64 -> fp32 rounding is monotone
  return order_key((float)key_value(okey)) >> kHistShift;
}

// Walks the kHistWindow bins at and below `top_bin` from the top.  found == false if the window holds fewer
// than `need` keys; otherwise the bin holding the need-th largest counted key, the number of counted keys above
// that bin and the bin's own count, to all NT threads.  hist points at the histogram's bin 0 (after the apron).
struct BinWalk {
  int bin, above, cnt;
  bool found;
};
// FRESH: the workgroup has not used sh.wave_tot yet (or is past a barrier since), so the scan need not wait for
// earlier readers.
template <int NT, bool FRESH = false>
__device__ __forceinline__ BinWalk walk_histogram(const uint32_t* __restrict__ hist, uint32_t top_bin, int need,
                                                  SelSharedT<NT>& sh) {
  constexpr int kPer = kHistWindow / NT;
  static_assert(kPer % 4 == 0, "whole 16-byte loads per thread");
  const int tid = (int)threadIdx.x;
  const int hi = (int)(top_bin | 7u);            // last bin of top_bin's aligned group of eight
  const int start = hi - kPer * (tid + 1) + 1;   // this thread's bins, ascending; a multiple of 8, may be < 0
  const uint4* p = reinterpret_cast<const uint4*>(hist + start);
  uint4 hv[kPer / 4];
#pragma unroll
  for (int u = 0; u < kPer / 4; ++u) hv[u] = p[u];
  int c[kPer], s = 0;  // c[q] = count of bin start + kPer-1 - q (descending)
#pragma unroll
  for (int u = 0; u < kPer / 4; ++u) {
    const int o = kPer - 4 - 4 * u;
    c[o + 3] = (int)hv[u].x;
    c[o + 2] = (int)hv[u].y;
    c[o + 1] = (int)hv[u].z;
    c[o + 0] = (int)hv[u].w;
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) s += c[q];
  int total;
  const int incl = wg_scan_incl<NT, FRESH>(s, sh, &total);
  BinWalk r;
  r.found = total >= need;  // uniform
  r.bin = r.above = r.cnt = 0;
  if (!r.found) return r;
  int run = incl - s;
  if (run < need && need <= incl) {
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      if (run < need && need <= run + c[q]) {
        sh.bc_bin = start + kPer - 1 - q;
        sh.bc_above = run;
        sh.bc_cnt = c[q];
      }
      run += c[q];
    }
  }
  __syncthreads();
  r.bin = sh.bc_bin;
  r.above = sh.bc_above;
  r.cnt = sh.bc_cnt;
  return r;
}

// A step with more keys than this (batch x row length) is not counted by the producer of the keys - one atomic
// per key: the device retires about 13 G of them per second, so 131 K keys add 10 us to a scorer kernel - but by
// a pass of its own with bins 2^kCoarseShift keys wide, aggregated in LDS first (a tenth of the atomics).
constexpr int kDirectCountMaxKeys = 65536;
constexpr int kCoarseShift = 15;

// ---- per-token histograms of the general route ---------------------------------------------------------
constexpr int kWgMaxSlots = 4096;  // per-workgroup maxima a key-producing kernel may write per token
constexpr int kAmbCap = 4096;      // keys of the threshold bin kept per token
constexpr unsigned long long kMultiCookie = 0x48695245484953ull;

struct MultiHeader {
  unsigned long long cookie;
  uint32_t layout_b;  // batch size the region was last laid out and cleaned for
  uint32_t stamps;    // times the region was found unstamped, cleared and stamped since the workspace was initialised
  uint32_t fallbacks; // tokens that took the streaming selection since the region was stamped
  uint32_t pad[59];
};
struct AmbEntry {
  uint32_t okey;
  int32_t idx;
};
struct MultiRegion {
  MultiHeader* hdr;
  int32_t* walk;     // [B][4]: need inside the threshold bin, found flag, bin of the largest key
  uint32_t* amb_n;   // [B]
  uint32_t* wgmax;   // [B][kWgMaxSlots]
  AmbEntry* amb;     // [B][kAmbCap]
  uint32_t* hist;    // [B][kHistStride]
};
inline size_t multi_body_bytes(int B) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  return up((size_t)B * 16) + up((size_t)B * 4) + up((size_t)B * kWgMaxSlots * 4) +
         up((size_t)B * kAmbCap * sizeof(AmbEntry)) + up((size_t)B * kHistStride * 4);
}
__host__ __device__ inline MultiRegion carve_multi(MultiHeader* hdr, void* body, int B) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  char* p = static_cast<char*>(body);
  MultiRegion r;
  r.hdr = hdr;
  r.walk = reinterpret_cast<int32_t*>(p);
  p += up((size_t)B * 16);
  r.amb_n = reinterpret_cast<uint32_t*>(p);
  p += up((size_t)B * 4);
  r.wgmax = reinterpret_cast<uint32_t*>(p);
  p += up((size_t)B * kWgMaxSlots * 4);
  r.amb = reinterpret_cast<AmbEntry*>(p);
  p += up((size_t)B * kAmbCap * sizeof(AmbEntry));
  r.hist = reinterpret_cast<uint32_t*>(p);
  return r;
}
// True when the histograms of this layout are known to be all zero between steps.
__device__ __forceinline__ bool multi_hist_ok(const MultiHeader* h, int B) {
  return h->cookie == kMultiCookie && h->layout_b == (uint32_t)B;
}


// ---- one token on a long vocabulary (softmax_b1.hip) ------------------------------------------------------
// A window of kSm1WinBins coarse bins (2^kSm1Shift order keys each, 16 octaves) below sm1_anchor_bin, which bounds
// every key a priori: |sum of code * xq| <= 7 * 127 * d exactly in fp32, times the largest row scale, and
// rounding is monotone.
constexpr int kSm1Shift = 16;
constexpr int kSm1WinBins = 2048;
constexpr int kSm1MaxRow = 262144;      // longest vocabulary of the short sequence
constexpr int kSm1MaxShortlist = 1536;  // largest k'
constexpr int kSm1MaxK = 64;            // largest k
__device__ __forceinline__ int sm1_anchor_bin(float smax, int d) {
  return (int)(order_key((float)(889 * d) * smax) >> kSm1Shift);
}

// ---- the general route's header: fixed place in the workspace, cleared by the workspace initialisation ----
// layout_sig names the workspace layout (batch size, shapes, k, k') the cookie was given under; the first
// kernel of a step drops the cookie when it finds another one, because the histograms then lie elsewhere.
struct GeneralHeader {
  MultiHeader multi;
  unsigned long long layout_sig;
  uint32_t window_misses;  // single-workgroup selections whose window histogram did not answer (testing aid)
  uint32_t pad[61];
};
static_assert(sizeof(GeneralHeader) == 512, "header size");

__host__ __device__ inline MultiRegion multi_of(const HistRefs& hr, int B) {
  if (!hr.header || !hr.multi_body) return MultiRegion{};
  return carve_multi(&static_cast<GeneralHeader*>(hr.header)->multi, hr.multi_body, B);
}
// Called by workgroup 0 of a step's first kernel.
__device__ __forceinline__ void general_header_check(GeneralHeader* gh, unsigned long long sig) {
  if (gh == nullptr || gh->layout_sig == sig) return;  // uniform
  const int tid = (int)threadIdx.x;
  if (tid == 0) {
    gh->multi.cookie = 0ull;
    gh->window_misses = 0u;
  }
  __syncthreads();  // every thread has compared before the signature changes
  if (tid == 0) gh->layout_sig = sig;
}

// ---- the candidate union as a bitmap, compacted by its consumers (union_locate in select.h) ----------------
struct GatherUnion {
  const uint32_t* bitmap;  // nullptr: take the list
  int words;
  int32_t* list_out;       // ascending candidates
  int32_t* count_out;      // device count read by the kernels that follow
  int32_t* count_out2;     // optional: the caller's copy
  MultiHeader* stamp;      // optional: key-histogram header to stamp once its histograms are known to be clear
  int stamp_b;
};

__device__ __forceinline__ void publish_union(const GatherUnion& u, int total) {
  if (threadIdx.x != 0) return;
  u.count_out[0] = total;
  if (u.count_out2) u.count_out2[0] = total;
  if (u.stamp != nullptr && !multi_hist_ok(u.stamp, u.stamp_b)) {
    u.stamp->fallbacks = 0u;
    u.stamp->stamps += 1u;
    u.stamp->layout_b = (uint32_t)u.stamp_b;
    u.stamp->cookie = kMultiCookie;
  }
}

inline GatherUnion make_gather_union(const UnionRefs* un, const HistRefs& hr, int B) {
  GatherUnion u{};
  if (un != nullptr && un->bitmap != nullptr && un->words <= kUnionLocateMaxWords) {
    u.bitmap = un->bitmap;
    u.words = un->words;
    u.list_out = un->list_out;
    u.count_out = un->count_out;
    u.count_out2 = un->count_out2;
    if (un->stamp_keys && hr.header && hr.multi_body) u.stamp = &static_cast<GeneralHeader*>(hr.header)->multi;
    u.stamp_b = B;
  }
  return u;
}

}  // namespace hire
