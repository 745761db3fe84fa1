// Exact selection of the largest keys of a workgroup's register-resident, non-negative keys (TopInd_k of
// arXiv 2402.09360 Sec. 3.1, both lines of Algorithm 1), guided by a window histogram: shared by the batch-1
// FFN kernels (histograms filled by the producing kernel, in the workspace) and by the per-token selection of
// the general route (histogram built in LDS).
//
// A fine bin is 2^14 consecutive fp32 bit patterns (exponent and nine mantissa bits), so few keys share a
// counter; a window histogram holds the 8192 bins (16 octaves) at and below an anchor bin, slot s counting the
// keys of bin anchor - s.  Non-negative IEEE values order like their bit patterns, which are used as integer
// keys directly; key arrays are zero-padded (or masked to zero) beyond their end, so that the passes over the
// registers need no validity tests: every comparison is against a positive threshold.
#pragma once

#include "select.h"

namespace hire {

constexpr int kFineShift = 14;                    // fine bin = bits >> 14 (exponent and 9 mantissa bits of an fp32)
constexpr int kWin = 8192;                        // bins of a window histogram (16 octaves below its anchor)
constexpr int kFastAmbCap = 64;                   // keys of the threshold bin ranked directly
static_assert(kFastAmbCap <= kWave, "the threshold bin's keys are ranked one per lane");

__device__ __forceinline__ uint32_t fine_bin(uint32_t bits) { return bits >> kFineShift; }
__device__ __forceinline__ uint32_t fine_bin(uint64_t bits) {  // fp64 -> fp32 rounding is monotone
  return __float_as_uint((float)__longlong_as_double((long long)bits)) >> kFineShift;
}

// Smallest key of fine bin b >= 1 in the key type's own bit patterns: key >= bin_floor(b) <=> fine_bin(key) >= b.
template <typename K>
__device__ __forceinline__ K bin_floor(uint32_t b);
template <>
__device__ __forceinline__ uint32_t bin_floor<uint32_t>(uint32_t b) { return b << kFineShift; }
template <>
__device__ __forceinline__ uint64_t bin_floor<uint64_t>(uint32_t b) {
  // A double rounds (to nearest, ties to even) to the float F = bits(b << 14) or above exactly when it is at or
  // above the midpoint between F and the float before it: F's last mantissa bit is zero, so the tie goes up.
  const double f = (double)__uint_as_float(b << kFineShift), before = (double)__uint_as_float((b << kFineShift) - 1u);
  return (uint64_t)__double_as_longlong(0.5 * (before + f));
}

// ---------------------------------------------------------------------------------------------------
// Register-resident non-negative keys of an NT-thread workgroup, as raw IEEE bits.  Wave w owns the index
// range [w*M, (w+1)*M); one load brings PER consecutive values per lane (16 bytes), so element (load e, lane
// l, part q) has index w*M + e*64*PER + l*PER + q.  Lanes whose vector starts at or beyond n load zeros; the
// array itself must be zero from n up to the next multiple of PER.
template <typename K>
struct KeyIO;
template <>
struct KeyIO<uint32_t> {
  static constexpr int PER = 4;
  using V = float;
  static __device__ __forceinline__ void unpack(const uint4& u, uint32_t* out) {
    out[0] = u.x;
    out[1] = u.y;
    out[2] = u.z;
    out[3] = u.w;
  }
  static __device__ __forceinline__ uint32_t to_order_key(uint32_t bits) { return bits | 0x80000000u; }
  static __device__ __forceinline__ uint32_t from_order_key(uint32_t key) { return key & 0x7FFFFFFFu; }
};
template <>
struct KeyIO<uint64_t> {
  static constexpr int PER = 2;
  using V = double;
  static __device__ __forceinline__ void unpack(const uint4& u, uint64_t* out) {
    out[0] = ((uint64_t)u.y << 32) | u.x;
    out[1] = ((uint64_t)u.w << 32) | u.z;
  }
  static __device__ __forceinline__ uint64_t to_order_key(uint64_t bits) { return bits | 0x8000000000000000ull; }
  static __device__ __forceinline__ uint64_t from_order_key(uint64_t key) { return key & 0x7FFFFFFFFFFFFFFFull; }
};

// FRESH: index() is computed anew at every use instead of being kept in registers from the first use on (for
// kernels short of registers).
template <typename K, int LOADS, int NT, bool FRESH = false>
struct KeyRegs {
  static constexpr int PER = KeyIO<K>::PER;
  static constexpr int SPAN = kWave * PER;  // keys per load of a wave
  static constexpr int NW = NT / kWave;
  static constexpr int CAPACITY = NW * LOADS * SPAN;
  K r[LOADS][PER];
  int base, len, n;  // the wave's index range is [base, base + len)
  // Starts the loads (into r, still packed); finish() unpacks in place.
  uint4 raw[LOADS];
  __device__ __forceinline__ void issue(const void* vals, int n_, const uint32_t* zeros16) {
    n = n_;
    const int M = (((n + NW - 1) / NW) + SPAN - 1) / SPAN * SPAN;  // <= LOADS * SPAN
    len = M;
    base = wave_id() * M;
    const int vecs = (n + PER - 1) / PER;
    const uint4* v4 = reinterpret_cast<const uint4*>(vals);
    const uint4* z4 = reinterpret_cast<const uint4*>(zeros16);
#pragma unroll
    for (int e = 0; e < LOADS; ++e) {
      const int vec = (base + e * SPAN) / PER + lane_id();
      raw[e] = *(e * SPAN < M && vec < vecs ? v4 + vec : z4);
    }
  }
  // The same for an array whose valid length is not known yet: cap values are readable (cap >= 1), the loads
  // stay inside them, and mask_beyond() zeroes what lies at and beyond the length once it is known.
  __device__ __forceinline__ void issue_clamped(const void* vals, int cap) {
    n = cap;
    const int M = (((cap + NW - 1) / NW) + SPAN - 1) / SPAN * SPAN;
    len = M;
    base = wave_id() * M;
    const int last_vec = (cap - 1) / PER;
    const uint4* v4 = reinterpret_cast<const uint4*>(vals);
#pragma unroll
    for (int e = 0; e < LOADS; ++e) raw[e] = v4[min((base + e * SPAN) / PER + lane_id(), last_vec)];
  }
  __device__ __forceinline__ void finish() {
#pragma unroll
    for (int e = 0; e < LOADS; ++e) KeyIO<K>::unpack(raw[e], r[e]);
  }
  __device__ __forceinline__ void mask_beyond(int n_) {
    n = n_;
#pragma unroll
    for (int e = 0; e < LOADS; ++e)
#pragma unroll
      for (int q = 0; q < PER; ++q)
        if (!(e * SPAN < len && index(e, q) < n_)) r[e][q] = (K)0;
  }
  __device__ __forceinline__ int index(int e, int q) const {
    int b = base + lane_id() * PER;
    if constexpr (FRESH) asm volatile("" : "+v"(b));  // opaque: not merged with the same sum computed elsewhere
    return b + e * SPAN + q;
  }
  __device__ __forceinline__ bool valid(int e, int q) const { return e * SPAN < len && index(e, q) < n; }
};

// A window histogram, walked from the top: thread t holds slots VEC*4*t .. VEC*4*(t+1) - 1 (requested by the
// caller as its first loads).  found == false if the window holds fewer than `need` keys; otherwise the slot
// holding the need-th largest counted key, to all threads.
struct WinWalk {
  int slot;
  bool found;
};
template <int NT>
struct WinRegs {
  static constexpr int VEC = kWin / NT / 4;  // 16-byte loads of counters per thread
  static_assert(VEC >= 1 && VEC * 4 * NT == kWin, "whole vectors of counters per thread");
  uint4 v[VEC];
  __device__ __forceinline__ void issue(const uint32_t* hist) {  // global memory or LDS
    const uint4* p = reinterpret_cast<const uint4*>(hist) + VEC * threadIdx.x;
#pragma unroll
    for (int u = 0; u < VEC; ++u) v[u] = p[u];
  }
};
template <int NT>
__device__ __forceinline__ WinWalk walk_window(const WinRegs<NT>& wr, int need, SelSharedT<NT>& sh) {
  constexpr int VEC = WinRegs<NT>::VEC;
  const int tid = (int)threadIdx.x;
  int sv[VEC], s = 0;
#pragma unroll
  for (int u = 0; u < VEC; ++u) {
    sv[u] = (int)(wr.v[u].x + wr.v[u].y + wr.v[u].z + wr.v[u].w);
    s += sv[u];
  }
  int total;
  const int incl = wg_scan_incl<NT, true>(s, sh, &total);
  WinWalk r;
  r.found = total >= need;  // uniform
  r.slot = 0;
  if (!r.found) return r;
  int run = incl - s;
  if (run < need && need <= incl) {  // one thread of the workgroup
#pragma unroll
    for (int u = 0; u < VEC; ++u) {
      if (run < need && need <= run + sv[u]) {
        const int c[4] = {(int)wr.v[u].x, (int)wr.v[u].y, (int)wr.v[u].z, (int)wr.v[u].w};
        int rr = run;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (rr < need && need <= rr + c[q]) sh.bc_bin = (VEC * tid + u) * 4 + q;
          rr += c[q];
        }
      }
      run += sv[u];
    }
  }
  __syncthreads();
  r.slot = sh.bc_bin;
  return r;
}

// Where the selection cuts the order (key descending, index ascending): an entry is selected iff its key is
// larger than `key`, or equal to it with an index of at most `idx`.  One rule covers ties at the boundary.
template <typename K>
struct Cut {
  K key;
  int idx;
};
template <typename K>
__device__ __forceinline__ bool cut_takes(const Cut<K>& c, K key, int idx) {
  return key > c.key || (key == c.key && idx <= c.idx);
}

// What a wave knows after the selection: the cut, the rank (in ascending index order) of its first selected
// key and how many of its keys are selected.  plain: every key equal to the cut's is selected and the cut's key
// is positive, so "selected" is key >= cut.key and the zero padding needs no test.  A wave that the caller's
// window of ranks cannot meet leaves the selection early with first/count bounding its ranks and no cut.
template <typename K>
struct Selection {
  Cut<K> cut;
  int first, count;
  bool plain;
};

// One entry of the threshold bin ahead of another in the order (key descending, index ascending).
__device__ __forceinline__ bool ranks_ahead(uint32_t ok, int oi, uint32_t mk, int mi) {
  // one 64-bit comparison: key in the upper half, complemented index in the lower
  return (((uint64_t)ok << 32) | (uint32_t)~oi) > (((uint64_t)mk << 32) | (uint32_t)~mi);
}
__device__ __forceinline__ bool ranks_ahead(uint64_t ok, int oi, uint64_t mk, int mi) {
  return ok > mk || (ok == mk && oi < mi);
}

// Selects the need_total largest of the workgroup's register-resident keys (ties to the lower index).
// Histogram route: the walk over the window proposes the bin of the need_total-th key; one pass over the
// registers counts each wave's keys above that bin and lists the bin's own few keys with their indices; every
// wave then ranks that list itself (no further barrier) and so knows the cut and, from the waves' counts, the
// rank of its own first selected key.  The histogram only proposes the bin: the counts that decide are taken
// from the keys, so the result does not depend on the histogram being right.  Any irregularity (no valid
// histogram, fewer than need_total keys inside the window, crowded bin, a proposed bin that the keys' own counts
// do not confirm) takes the histogram-free narrowing of select.h, which re-reads the values from memory with
// rolled loops to keep the code small, and then finds the index of the last selected key among those equal to
// the threshold.
// wave_cnt: LDS int[NT / 64].  All threads of the workgroup call this.  [out_lo, out_hi): the ranks the caller
// will emit.  fallback_counter (optional) counts the selections that took the narrowing: of workgroup 0 (all
// workgroups select the same keys) or, count_every_workgroup, of every one.  TS: first of three phase stamps of
// the profiling build.
template <int TS, typename K, int LOADS, int NT, bool FR>
__device__ __forceinline__ Selection<K> fast_select(const KeyRegs<K, LOADS, NT, FR>& kr, const void* vals,
                                                           int need_total, const WinRegs<NT>& wr, uint32_t anchor,
                                                           bool hist_ok, SelSharedT<NT>& sh, int* wave_cnt,
                                                           uint32_t* fallback_counter, int out_lo, int out_hi,
                                                           bool count_every_workgroup = false) {
  constexpr int PER = KeyRegs<K, LOADS, NT, FR>::PER;
  constexpr int NW = NT / kWave;
  const int tid = (int)threadIdx.x, lane = lane_id();
  const int w = __builtin_amdgcn_readfirstlane(wave_id());
  Selection<K> out;
  K* lkey = reinterpret_cast<K*>(sh.hist);                        // [kFastAmbCap] keys of the threshold bin
  int* lidx = reinterpret_cast<int*>(sh.hist + 2 * kFastAmbCap);  // [kFastAmbCap] their indices
  if (hist_ok) {
    if (tid == 0) sh.list_n = 0;  // ordered before its use by the barriers of the walk
    const WinWalk bw = walk_window<NT>(wr, need_total, sh);
    HIRE_TS(TS);
    const uint32_t bin = anchor - (uint32_t)bw.slot;  // bin >= 1 wherever a key was counted
    if (bw.found && bin >= 1u && bin <= anchor) {  // uniform
      const K lo = bin_floor<K>(bin), up = bin_floor<K>(bin + 1u), width = up - lo;
      // Two comparisons per key, each added into a per-lane counter through the carry input (no mask stays alive,
      // no scalar work per key); one wave sum at the end.
      int ge_up = 0, ge_lo = 0;
#pragma unroll
      for (int e = 0; e < LOADS; ++e)
#pragma unroll
        for (int q = 0; q < PER; ++q) {
          ge_up += kr.r[e][q] >= up ? 1 : 0;
          ge_lo += kr.r[e][q] >= lo ? 1 : 0;
        }
      const int above = wave_sum(ge_up);
      if (ge_lo != ge_up) {  // this lane holds keys of the bin: few lanes of few waves
        K lo2 = lo;
        asm volatile("" : "+v"(lo2));  // compared afresh: nothing of the pass above is kept for this
#pragma unroll
        for (int e = 0; e < LOADS; ++e)
#pragma unroll
          for (int q = 0; q < PER; ++q)
            if ((K)(kr.r[e][q] - lo2) < width) {
              const int p = atomicAdd(&sh.list_n, 1);
              if (p < kFastAmbCap) {
                lkey[p] = kr.r[e][q];
                lidx[p] = kr.index(e, q);
              }
            }
      }
      if (lane == 0) wave_cnt[w] = above;
      __syncthreads();
      HIRE_TS(TS + 1);
      // What the histogram said is checked against the keys themselves: with A keys above the bin and C inside it
      // (both counted from the registers), the need_total-th largest key lies in the bin iff A < need_total <= A + C.
      const int pa = wave_scan_incl(lane < NW ? wave_cnt[lane] : 0);
      const int A = __builtin_amdgcn_readlane(pa, NW - 1), C = sh.list_n;
      if (C <= kFastAmbCap && A < need_total && need_total <= A + C) {  // uniform over the workgroup
        const int above_before = w > 0 ? __builtin_amdgcn_readlane(pa, w - 1) : 0;
        if (above_before + above + C <= out_lo || above_before >= out_hi) {
          // whatever the bin's keys turn out to be, this wave's ranks miss the caller's window: no ranking
          out.cut.key = 0;
          out.cut.idx = 0;
          out.plain = true;
          out.first = above_before;
          out.count = 0;
          return out;
        }
        const int m = C, need = need_total - A;  // 1 <= need <= m <= 64
        const K mine_k = lane < m ? lkey[lane] : (K)0;
        const int mine_i = lane < m ? lidx[lane] : 0x7FFFFFFF;
        int rank = 0;  // entries of the bin ahead of this lane's
        for (int u = 0; u < m; ++u) {
          const K ok = read_lane(mine_k, u);
          const int oi = __builtin_amdgcn_readlane(mine_i, u);
          rank += ranks_ahead(ok, oi, mine_k, mine_i) ? 1 : 0;
        }
        const bool sel = lane < m && rank < need;
        const uint64_t last = __ballot(lane < m && rank == need - 1);  // exactly one lane
        const int src = __builtin_ctzll(last);
        out.cut.key = read_lane(mine_k, src);
        out.cut.idx = __builtin_amdgcn_readlane(mine_i, src);
        out.plain = __ballot(lane < m && !sel && mine_k == out.cut.key) == 0ull;
        const int rel = mine_i - kr.base;  // position inside this wave's range, if 0 <= rel < len
        const bool mine_here = sel && rel >= 0 && rel < kr.len;
        out.first = above_before + __popcll(__ballot(sel && rel < 0));
        out.count = above + __popcll(__ballot(mine_here));
        HIRE_TS(TS + 2);
        return out;
      }
    }
  }
  __syncthreads();
  if (fallback_counter && (blockIdx.x == 0 || count_every_workgroup) && tid == 0) atomicAdd(fallback_counter, 1u);
  using V = typename KeyIO<K>::V;
  const V* v = reinterpret_cast<const V*>(vals);
  const int n = kr.n;
  const K okey = wg_kth_largest<K>(
      [&](auto&& f) {
#pragma unroll 1
        for (int i = tid; i < n; i += NT) {
          K bits;
          __builtin_memcpy(&bits, &v[i], sizeof(K));
          f(KeyIO<K>::to_order_key(bits));
        }
      },
      n, need_total, sh);
  const K t = KeyIO<K>::from_order_key(okey);
  // keys above the threshold and equal to it, per wave; then the index of the last selected one among the equal
  int gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < LOADS; ++e)
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const bool valid = kr.valid(e, q);
      gt += __popcll(__ballot(valid && kr.r[e][q] > t));
      eq += __popcll(__ballot(valid && kr.r[e][q] == t));
    }
  __syncthreads();  // the narrowing's last readers of wave_tot are done
  if (lane == 0) {
    wave_cnt[w] = gt;
    sh.wave_tot[w] = eq;
  }
  __syncthreads();
  const int pg = wave_scan_incl(lane < NW ? wave_cnt[lane] : 0), pe = wave_scan_incl(lane < NW ? sh.wave_tot[lane] : 0);
  const int gt_before = w > 0 ? __builtin_amdgcn_readlane(pg, w - 1) : 0;
  const int eq_before = w > 0 ? __builtin_amdgcn_readlane(pe, w - 1) : 0;
  const int need_eq = need_total - __builtin_amdgcn_readlane(pg, NW - 1);  // >= 1: the threshold itself is selected
  if (eq_before < need_eq && need_eq <= eq_before + eq) {  // uniform over the wave; true for exactly one wave
    int run = eq_before;
#pragma unroll
    for (int e = 0; e < LOADS; ++e) {
      int c = 0;
#pragma unroll
      for (int q = 0; q < PER; ++q) c += (kr.valid(e, q) && kr.r[e][q] == t) ? 1 : 0;
      const int incl = wave_scan_incl(c);
      const int tot = __builtin_amdgcn_readlane(incl, kWave - 1);
      if (run < need_eq && need_eq <= run + tot) {
        int pos = run + incl - c;  // equal keys before this lane's
#pragma unroll
        for (int q = 0; q < PER; ++q)
          if (kr.valid(e, q) && kr.r[e][q] == t) {
            if (++pos == need_eq) sh.bc_bin = kr.index(e, q);
          }
      }
      run += tot;
    }
  }
  __syncthreads();
  out.cut.key = t;
  out.cut.idx = sh.bc_bin;
  out.plain = false;
  out.first = gt_before + min(eq_before, need_eq);
  out.count = gt + (min(eq_before + eq, need_eq) - min(eq_before, need_eq));
  return out;
}

// Ordered emission: calls emit(i, rank, key, e, q) for every key with take(e, q) whose rank in ascending index
// order lies in [out_lo, out_hi); first / count: the rank of the wave's first such key and their number.  Only the
// waves whose own ranks meet that window do any work.
template <typename K, int LOADS, int NT, bool FR, typename Take, typename Emit>
__device__ __forceinline__ void fast_emit_if(const KeyRegs<K, LOADS, NT, FR>& kr, int first, int count, int out_lo,
                                             int out_hi, Take&& take_fn, Emit&& emit) {
  constexpr int PER = KeyRegs<K, LOADS, NT, FR>::PER;
  if (first + count <= out_lo || first >= out_hi) return;  // uniform over the wave
  int run = first;
#pragma unroll
  for (int e = 0; e < LOADS; ++e) {
    // ranks inside this load follow (lane, part): selected keys of lower lanes, then this lane's lower parts.
    // Ballots and mask counts instead of a scan across lanes: independent instructions, no chain of lane shifts.
    bool take[PER];
    int before = 0, tot = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      take[q] = take_fn(e, q);
      const uint64_t m = __ballot(take[q]);
      before += mask_prefix(m);
      tot += __popcll(m);
    }
    if (run + tot > out_lo && run < out_hi) {  // uniform
      int pos = run + before;
#pragma unroll
      for (int q = 0; q < PER; ++q)
        if (take[q]) {
          if (pos >= out_lo && pos < out_hi) emit(kr.index(e, q), pos, kr.r[e][q], e, q);
          ++pos;
        }
    }
    run += tot;
  }
}

// The same for a selection: the keys that its cut takes.
template <typename K, int LOADS, int NT, bool FR, typename Emit>
__device__ __forceinline__ void fast_emit(const KeyRegs<K, LOADS, NT, FR>& kr, const Selection<K>& s, int out_lo,
                                          int out_hi, Emit&& emit) {
  fast_emit_if(
      kr, s.first, s.count, out_lo, out_hi,
      [&](int e, int q) {
        return s.plain ? kr.r[e][q] >= s.cut.key : (kr.valid(e, q) && cut_takes(s.cut, kr.r[e][q], kr.index(e, q)));
      },
      emit);
}

}  // namespace hire
