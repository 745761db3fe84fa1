// C ABI of libhire (declared in include/hire.h): argument validation, workspace
// carving and the kernel sequence of one HiRE-FFN / HiRE-Softmax decode step.
#include "../../include/hire.h"

#include "kernels.h"

#include <atomic>
#include <vector>

// Scratch memory of hire_ffn_step_static: one array per GPU the library runs on, held until the process ends,
// all zero when the code object is loaded (which is the state hire_workspace_init gives a workspace).  In host
// code this name only stands for the symbol; the memory is reached through the per-device address that
// hipGetSymbolAddress returns (static_scratch below), never through the name.
static __device__ __align__(256) unsigned char scratch[HIRE_STATIC_SCRATCH_BYTES];

namespace {

using namespace hire;

constexpr size_t kAlign = 256;
constexpr int kSingleWgMaxRow = 32768;  // up to this row length one workgroup per token selects the k' keys
constexpr int kMfmaMinBatch = 2;  // from this batch size on the scorer and the gather run on the matrix cores
constexpr int kFilterMinBatch = 16;  // filter and refine pays from here on (the fp64 tile count grows with the batch)
constexpr int kCounters = 64;     // int32 counters behind the union bitmap, cleared with it by a step's first kernel
constexpr int kCntWnormMax = 8;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Bump allocator over the caller's workspace; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off = align_up(off + count * sizeof(T));
    return p;
  }
};

struct StepBuffers {
  void* fast_region;  // fixed offset 0: cookie, maxima and histograms of the batch-1 four-kernel route
  HistRefs hist;      // general route: header at a fixed offset after the fast region; key histograms (long rows)
  uint32_t* window_misses;  // counter inside the header
  unsigned long long sig;  // names this layout
  int8_t* xq;
  float* sx;
  uint16_t* t;       // low-rank intermediate, bf16 [B, r]
  float* keys_t;     // int4 low-rank scorer: the intermediate before rounding, fp32 [B, r]
  double* t_partial; // its per-slice partial sums
  void* keys;        // fp32 or fp64 [B, N]
  void* gkeys;       // group-sparse: summed absolute keys, same type, [B, N >> gs]
  double* hg;        // group-sparse: summed absolute exact activations [B, cap_u]
  uint32_t* bitmap;  // candidate union bitmap, then (after it) the counters
  int32_t* counters; // [0] = |U|
  int32_t* cand;     // U
  double* h;         // [B, cap_u]
  int32_t* pos;      // [B,k] positions inside U of every token's selected units
  int32_t* sel_idx;  // [B,k] when the caller does not ask for topk_idx
  float* partial;    // second-layer partial sums
  // filter and refine of the exact stage (batches): upper bounds of the tokens' norms, the fp32 stored values
  float* xnorm;      // [B]
  float* hf;         // [B, hf_stride]
  int hf_stride;
  void* sm1_slots;   // long rows: slots of the keys at or above the bound from the scorer's maxima
  bool sm1_ok;       // ... which this layout has
  bool max_ok;       // long rows: slots for the selection of k' from the scorer's maxima
  int words, cap_u, zero_words;
  size_t bytes;
};

// gs > 0: group-sparse FFN with groups of 2^gs units; the selections, the bitmap, the union and cap_u then count
// groups, while keys and h keep one value per unit.
StepBuffers carve(void* ws, int scorer_kind, int B, int d, int N, int r, int k, int kprime, bool ffn, int gs = 0) {
  StepBuffers s{};
  Carver c(ws);
  const int Ns = N >> gs, kps = kprime >> gs;
  s.cap_u = (int)((long long)B * kps < (long long)Ns ? B * kps : Ns);
  s.words = (Ns + 31) / 32 + 2;
  s.fast_region = c.take<char>(ffn_fast_region_bytes());
  s.hist.header = c.take<char>(general_header_bytes());
  s.sig = layout_signature(scorer_kind, B, d, N, r, k, kprime, (ffn ? 1 : 0) + 16 * gs);
  s.window_misses = s.hist.header ? reinterpret_cast<uint32_t*>(static_cast<char*>(s.hist.header) +
                                                                 general_fallbacks_offset(1))
                                  : nullptr;
  const bool int4_like = scorer_kind == HIRE_SCORER_INT4 || scorer_kind == HIRE_SCORER_LRQ;
  if (int4_like && N > kSingleWgMaxRow && gs == 0) s.hist.multi_body = c.take<char>(multi_body_bytes_host(B));
  if (int4_like) {
    s.xq = c.take<int8_t>((size_t)B * (d > r ? d : r));
    s.sx = c.take<float>(B);
    s.keys = c.take<float>((size_t)B * N + 4);
    if (gs > 0) s.gkeys = c.take<float>((size_t)B * Ns + 4);
    if (scorer_kind == HIRE_SCORER_LRQ) {
      s.keys_t = c.take<float>((size_t)B * r + 4);
      s.t = c.take<uint16_t>((size_t)B * r);
    }
  } else {
    s.t = c.take<uint16_t>((size_t)B * r);
    s.t_partial = c.take<double>((size_t)B * lr_project_slices(d) * r);
    s.keys = c.take<double>((size_t)B * N);
    if (gs > 0) s.gkeys = c.take<double>((size_t)B * Ns);
  }
  // bitmap and counters are contiguous so that one pass clears both.  counters[0] = |U|, [kCntWnormMax] = largest
  // candidate row norm of the filter stage (float bits)
  s.bitmap = c.take<uint32_t>((size_t)s.words + kCounters);
  s.counters = s.bitmap ? reinterpret_cast<int32_t*>(s.bitmap + s.words) : nullptr;
  s.zero_words = s.words + kCounters;
  s.cand = c.take<int32_t>(s.cap_u);
  s.h = c.take<double>(((size_t)B * s.cap_u << gs) + 2);
  if (gs > 0) s.hg = c.take<double>((size_t)B * s.cap_u + 2);
  if (B >= kFilterMinBatch && gs == 0 && (ffn || s.cap_u <= kSoftmaxRefineMaxRow)) {
    s.xnorm = c.take<float>(HIRE_MAX_BATCH);
    s.hf_stride = (s.cap_u + 3) / 4 * 4;  // rows start at multiples of 16 bytes
    s.hf = c.take<float>((size_t)B * s.hf_stride);
  }
  s.sm1_ok = !ffn && B == 1 && gs == 0 && int4_like && N > kSingleWgMaxRow && softmax_b1_supported(N, d, 1, 1);
  s.max_ok = gs == 0 && int4_like && N > kSingleWgMaxRow && maxima_select_supported(N);
  if (s.sm1_ok || s.max_ok) s.sm1_slots = c.take<char>(maxima_select_slot_bytes(B, N));
  if (ffn) {
    s.pos = c.take<int32_t>((size_t)B * k);
    s.sel_idx = c.take<int32_t>((size_t)B * k);
    size_t partial = (size_t)w2_groups(k, B, d) * B * d;
    const bool fast = gs == 3 ? ffn_fast_group8_supported(B, N, d, k, kprime)
                              : (gs == 0 && ffn_fast_supported(B, N, d, k, kprime));
    if (fast && ffn_fast_partial_floats(d, k, 0) > partial) partial = ffn_fast_partial_floats(d, k, 0);
    s.partial = c.take<float>(partial);
  }
  s.bytes = c.off;
  return s;
}

int check_common(int d, int N, int B, int k, int kprime, int scorer_kind, const void* q4, const float* q4_scale,
                 const void* lr_a, const void* lr_b, int r, const float* lr_a_scale, const float* lr_b_scale,
                 const void* W, const void* x) {
  if (d < 32 || d % 8 != 0 || N < 1 || B < 1 || B > HIRE_MAX_BATCH) return HIRE_EINVAL;
  if (k < 1 || k > kprime || kprime > N) return HIRE_EINVAL;
  if (!W || !x || !aligned(W, 256) || !aligned(x, 16)) return HIRE_EINVAL;
  if (scorer_kind == HIRE_SCORER_INT4) {
    if (d % 32 != 0 || !q4 || !q4_scale || !aligned(q4, 256)) return HIRE_EINVAL;
  } else if (scorer_kind == HIRE_SCORER_LRQ) {
    if (d % 32 != 0 || r < 32 || r % 32 != 0 || r > 1024 || !lr_a || !lr_b || !lr_a_scale || !lr_b_scale ||
        !aligned(lr_a, 256) || !aligned(lr_b, 256))
      return HIRE_EINVAL;
  } else if (scorer_kind == HIRE_SCORER_LOWRANK) {
    if (r < 8 || r % 8 != 0 || r > 1024 || !lr_a || !lr_b || !aligned(lr_a, 16) || !aligned(lr_b, 256))
      return HIRE_EINVAL;
  } else {
    return HIRE_EINVAL;
  }
  return HIRE_OK;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

#define HIRE_TRY(expr)                 \
  do {                                 \
    const hipError_t e_ = (expr);      \
    if (e_ != hipSuccess) {            \
      g_last_hip_error = e_;           \
      return HIRE_ELAUNCH;             \
    }                                  \
  } while (0)

// Optional stage timing: when the caller has handed over events, event i is recorded on the stream in front of
// stage i and one more after the last stage.
thread_local hipEvent_t* g_stage_events = nullptr;
thread_local int g_force_generic = 0;
thread_local int g_force_exact_stage = 0;  // testing: batches compute every candidate's activation in fp64
thread_local unsigned long long* g_scorer_clocks = nullptr;  // testing: route every step through the general multi-kernel path

#define HIRE_STAGE(i, st)                                             \
  do {                                                                \
    if (g_stage_events) HIRE_TRY(hipEventRecord(g_stage_events[i], st)); \
  } while (0)

// Steps 1-3 of a step, shared by FFN and softmax: scorer, per-token top-k', union, exact scores on the union.
struct ScorerRefs {
  int kind;
  const void* q4;
  const float* q4_scale;
  const void* lr_a;
  const void* lr_b;
  int r;
  const float* lr_a_scale;
  const float* lr_b_scale;
};
template <typename Layer>
ScorerRefs scorer_of(const Layer* L) {
  return ScorerRefs{L->scorer_kind, L->q4, L->q4_scale, L->lr_a, L->lr_b, L->r, L->lr_a_scale, L->lr_b_scale};
}

// filter: the exact stage writes the fast bf16 approximations (launch_gather_dot_bf16) instead of the fp64
// activations; the caller then refines around the selection threshold.
// maxima_out (one token, int4 scorers): return after the scorer, with the number of maxima it left.
int run_front(const StepBuffers& s, const ScorerRefs& sc, const void* W, const void* x, int B, int d, int N,
              int kprime, int relu, int32_t* cand_out, int32_t* n_cand, int32_t* scorer_acc, hipStream_t st,
              int gs = 0, bool filter = false, int* maxima_out = nullptr) {
  const int scorer_kind = sc.kind, r = sc.r;
  const void* lr_a = sc.lr_a;
  const void* lr_b = sc.lr_b;
  const uint16_t* xb = static_cast<const uint16_t*>(x);
  // what the int4 scorer and its token quantisation work on: the layer's own int4 copy and the token, or
  // (int4 low-rank scorer) the int4 copy of Z2 and the r-vector t
  const bool lrq = scorer_kind == HIRE_SCORER_LRQ;
  const bool int4_like = scorer_kind == HIRE_SCORER_INT4 || lrq;
  const void* q4 = lrq ? sc.lr_b : sc.q4;
  const float* q4_scale = lrq ? sc.lr_b_scale : sc.q4_scale;
  const uint16_t* tok = lrq ? s.t : xb;
  const int sd = lrq ? r : d;
  // what is ranked: units, or groups of 2^gs units by their summed absolute keys.  Groups of eight are summed by
  // the selection as it loads the keys; other sizes by a kernel of their own.
  const int Ns = N >> gs;
  const bool in_select = gs == 3 && Ns <= kSelectGroup8Max;
  SelectParams sp{};
  sp.group8 = in_select ? 1 : 0;
  sp.stride = in_select ? N : Ns;
  sp.n = Ns;
  sp.n_cap = Ns;
  sp.k = kprime >> gs;
  sp.relu = 0;  // the scorers already applied phi
  sp.nonneg = relu;  // phi = ReLU (and sums of absolute values): nothing negative is ranked
  sp.bitmap = s.bitmap;
  sp.vals = (gs > 0 && !in_select) ? s.gkeys : s.keys;
  int32_t* cand = cand_out ? cand_out : s.cand;
  // short bitmaps are compacted by the gather kernel itself; long ones by a kernel of their own
  const bool in_gather = union_in_gather(s.words);
  const bool many_wg = int4_like && N > kSingleWgMaxRow && gs == 0;  // long rows: key histograms
  UnionRefs un{s.bitmap, s.words, cand, s.counters, n_cand, many_wg};
  sp.window_misses = s.window_misses;
  HIRE_STAGE(0, st);
  bool t_is_f32 = false;
  if (lrq) {
    // first product of the int4 low-rank scorer: t = bf16(float(Z1q^T xq) * s1), the r rows of Z1^T scored like
    // any int4 matrix (no phi), then rounded to the bf16 activation the second product quantises
    const HistRefs header_only{s.hist.header, nullptr};
    const uint32_t* qa = static_cast<const uint32_t*>(lr_a);
    if (B == 1 && scorer_int4_fused_supported(d)) {
      HIRE_TRY(launch_scorer_int4_fused(qa, sc.lr_a_scale, xb, false, r, d, 0, s.keys_t, nullptr, header_only, s.bitmap,
                                        s.zero_words, s.sig, st));
    } else {
      HIRE_TRY(launch_quantize_tokens(xb, B, d, s.xq, s.sx, s.bitmap, s.zero_words, s.hist.header, s.sig, st));
      if (B >= kMfmaMinBatch)
        HIRE_TRY(launch_scorer_int4_mfma(qa, sc.lr_a_scale, s.xq, B, r, d, 0, s.keys_t, nullptr, header_only, st));
      else
        HIRE_TRY(launch_scorer_int4(qa, sc.lr_a_scale, s.xq, B, r, d, 0, s.keys_t, nullptr, header_only, st));
    }
    // the second product's batch-1 kernel for short rows rounds the intermediate itself
    t_is_f32 = B == 1 && scorer_int4_fused_supported(r) && scorer_int4_fused_takes_f32(r);
    if (!t_is_f32) HIRE_TRY(launch_f32_to_bf16(s.keys_t, B * r, s.t, st));
  }
  if (int4_like) {
    const bool fused = B == 1 && scorer_int4_fused_supported(sd);  // the scorer quantises the token itself
    if (!fused)
      HIRE_TRY(launch_quantize_tokens(tok, B, sd, s.xq, s.sx, s.bitmap, s.zero_words, s.hist.header, s.sig, st));
    HIRE_STAGE(1, st);
    int slots;
    if (fused) {
      HIRE_TRY(launch_scorer_int4_fused(static_cast<const uint32_t*>(q4), q4_scale,
                                        t_is_f32 ? static_cast<const void*>(s.keys_t) : static_cast<const void*>(tok),
                                        t_is_f32, N, sd, relu,
                                        static_cast<float*>(s.keys), scorer_acc, s.hist, s.bitmap, s.zero_words, s.sig,
                                        st));
      slots = scorer_int4_fused_maxima(N, sd);
    } else if (B >= kMfmaMinBatch) {
      HIRE_TRY(launch_scorer_int4_mfma(static_cast<const uint32_t*>(q4), q4_scale, s.xq, B, N, sd, relu,
                                       static_cast<float*>(s.keys), scorer_acc, s.hist, st));
      slots = scorer_mfma_maxima(N);
    } else {
      HIRE_TRY(launch_scorer_int4(static_cast<const uint32_t*>(q4), q4_scale, s.xq, B, N, sd, relu,
                                  static_cast<float*>(s.keys), scorer_acc, s.hist, st));
      slots = scorer_int4_blocks(N);
    }
    HIRE_STAGE(2, st);
    if (maxima_out != nullptr) {
      *maxima_out = slots;
      return fused ? HIRE_OK : HIRE_EINVAL;
    }
    if (gs > 0 && !in_select)
      HIRE_TRY(launch_group_sums_f32(static_cast<const float*>(s.keys), B, N, Ns, gs, static_cast<float*>(s.gkeys), Ns,
                                     st));
    if (many_wg && B >= 2 && s.max_ok && in_gather && maxima_select_worthwhile(N, kprime, slots) && !g_force_generic) {
      // long rows, batches: every token's k' largest keys from the bound that the scorer's maxima give (no key
      // histogram is filled or read, so none is stamped clean either)
      HIRE_TRY(launch_maxima_select(static_cast<const float*>(s.keys), B, N, sd, kprime, slots, q4, s.hist, s.sm1_slots,
                                    s.bitmap, st));
      HIRE_STAGE(3, st);
      un.stamp_keys = false;
    } else if (many_wg) {
      HIRE_TRY(launch_mark_f32(static_cast<const float*>(s.keys), B, N, kprime, slots, s.hist, s.bitmap, st));
      HIRE_STAGE(3, st);
      HIRE_TRY(launch_resolve_compact(static_cast<const float*>(s.keys), B, N, kprime, s.hist, s.bitmap, s.words,
                                      in_gather ? nullptr : cand, s.counters, n_cand, nullptr, 0, st));
    } else {
      HIRE_TRY(launch_select_f32(sp, B, st));
      HIRE_STAGE(3, st);
      if (!in_gather) HIRE_TRY(launch_bitmap_compact(s.bitmap, s.words, cand, s.counters, n_cand, nullptr, 0, st));
    }
  } else {
    HIRE_TRY(launch_lr_project(static_cast<const uint16_t*>(lr_a), xb, B, d, r, s.t, s.t_partial, s.bitmap, s.zero_words,
                               s.hist.header, s.sig, st));
    HIRE_STAGE(1, st);
    if (B >= kMfmaMinBatch)  // the same contraction as the exact stage, over all rows of Z2 with t as the tokens
      HIRE_TRY(launch_gather_dot_mfma(static_cast<const uint16_t*>(lr_b), s.t, B, r, nullptr, N, nullptr, N, relu,
                                      static_cast<double*>(s.keys), N, s.hist, nullptr, 0, st));
    else
      HIRE_TRY(launch_lr_score(static_cast<const uint16_t*>(lr_b), s.t, N, r, relu, static_cast<double*>(s.keys), st));
    HIRE_STAGE(2, st);
    if (gs > 0 && !in_select)
      HIRE_TRY(launch_group_sums_f64(static_cast<const double*>(s.keys), B, N, Ns, nullptr, Ns, gs,
                                     static_cast<double*>(s.gkeys), Ns, st));
    HIRE_TRY(launch_select_f64(sp, B, st));
    HIRE_STAGE(3, st);
    if (!in_gather) HIRE_TRY(launch_bitmap_compact(s.bitmap, s.words, cand, s.counters, n_cand, nullptr, 0, st));
  }
  HIRE_STAGE(4, st);
  if (filter)
    HIRE_TRY(launch_gather_dot_bf16(static_cast<const uint16_t*>(W), xb, B, d, cand, s.counters, s.cap_u, s.hf,
                                    s.hf_stride, s.hist, in_gather ? &un : nullptr, N, relu, s.xnorm,
                                    reinterpret_cast<uint32_t*>(s.counters + kCntWnormMax), st));
  else if (B >= kMfmaMinBatch)
    HIRE_TRY(launch_gather_dot_mfma(static_cast<const uint16_t*>(W), xb, B, d, cand, 0, s.counters, s.cap_u, relu, s.h,
                                    (long long)s.cap_u << gs, s.hist, in_gather ? &un : nullptr, gs, st));
  else
    HIRE_TRY(launch_gather_dot(static_cast<const uint16_t*>(W), xb, d, cand, 0, s.counters, s.cap_u, relu, s.h,
                               s.hist, in_gather ? &un : nullptr, gs, st));
  return HIRE_OK;
}

}  // namespace

extern "C" {

int hire_version(void) { return 100; }

const char* hire_strerror(int code) {
  switch (code) {
    case HIRE_OK: return "ok";
    case HIRE_EINVAL: return "invalid argument";
    case HIRE_ENOSPC: return "workspace too small";
    case HIRE_EUNSUPPORTED: return "unsupported combination";
    case HIRE_ELAUNCH: return "kernel launch failed";
    default: return "unknown error";
  }
}

int hire_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || workspace_bytes < kAlign || !aligned(workspace, 256)) return HIRE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  HIRE_TRY(launch_clear_words(static_cast<uint32_t*>(workspace), (int)(kAlign / 4), st));
  const size_t second = align_up(ffn_fast_region_bytes());  // header of the general route's histograms
  if (workspace_bytes >= second + general_header_bytes())
    HIRE_TRY(launch_clear_words(reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + second),
                                (int)(general_header_bytes() / 4), st));
  return HIRE_OK;
}

int hire_debug_fast_fallbacks(const void* workspace, uint32_t* host_out2, void* stream) {
  if (!workspace || !host_out2) return HIRE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  HIRE_TRY(hipMemcpyAsync(host_out2, static_cast<const char*>(workspace) + ffn_fast_fallbacks_offset(),
                          2 * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
  HIRE_TRY(hipStreamSynchronize(st));
  return HIRE_OK;
}

int hire_debug_fast_state(const void* workspace, uint32_t* host_out3, void* stream) {
  if (!workspace || !host_out3) return HIRE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  size_t cookie_off, h1, h2, words;
  unsigned long long want = 0, cookie = 0;
  ffn_fast_state_layout(&cookie_off, &want, &h1, &h2, &words);
  const char* base = static_cast<const char*>(workspace);
  std::vector<uint32_t> host(2 * words);
  HIRE_TRY(hipMemcpyAsync(&cookie, base + cookie_off, sizeof(cookie), hipMemcpyDeviceToHost, st));
  HIRE_TRY(hipMemcpyAsync(host.data(), base + h1, words * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
  HIRE_TRY(hipMemcpyAsync(host.data() + words, base + h2, words * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
  HIRE_TRY(hipStreamSynchronize(st));
  host_out3[0] = cookie == want ? 1u : 0u;
  host_out3[1] = host_out3[2] = 0u;
  for (size_t i = 0; i < words; ++i) {
    host_out3[1] += host[i] != 0u ? 1u : 0u;
    host_out3[2] += host[words + i];
  }
  return HIRE_OK;
}

int hire_debug_general_fallbacks(const void* workspace, uint32_t* host_out3, void* stream) {
  if (!workspace || !host_out3) return HIRE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const char* hdr = static_cast<const char*>(workspace) + align_up(ffn_fast_region_bytes());
  for (int i = 0; i < 3; ++i)
    HIRE_TRY(hipMemcpyAsync(host_out3 + i, hdr + general_fallbacks_offset(i), sizeof(uint32_t), hipMemcpyDeviceToHost,
                            st));
  HIRE_TRY(hipStreamSynchronize(st));
  return HIRE_OK;
}

int hire_debug_plain_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned(src, 16) || !aligned(dst, 16)) return HIRE_EINVAL;
  HIRE_TRY(launch_plain_copy(src, dst, bytes, static_cast<hipStream_t>(stream)));
  return HIRE_OK;
}

int hire_lr_prepare(const hire_ffn_layer* L, float* bounds2_out, void* stream) {
  const bool lrq = L && L->scorer_kind == HIRE_SCORER_LRQ;
  if (!L || !bounds2_out || (L->scorer_kind != HIRE_SCORER_LOWRANK && !lrq) || !L->w1u || !L->lr_b || L->d_ff < 1 ||
      L->d_model < 8 || L->d_model % 8 != 0 || L->r < 8 || L->r % 8 != 0 || !aligned(L->w1u, 16) ||
      !aligned(L->lr_b, 16) || !aligned(bounds2_out, 4))
    return HIRE_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  HIRE_TRY(launch_row_norm_max(static_cast<const uint16_t*>(L->w1u), L->d_ff, L->d_model, bounds2_out, st));
  if (lrq)  // the int4 copy of Z2 bounds its own keys (largest row scale, kept behind its codes)
    HIRE_TRY(launch_clear_words(reinterpret_cast<uint32_t*>(bounds2_out + 1), 1, st));
  else
    HIRE_TRY(launch_row_norm_max(static_cast<const uint16_t*>(L->lr_b), L->d_ff, L->r, bounds2_out + 1, st));
  return HIRE_OK;
}

int hire_debug_filter_stage(const void* W, const void* x, int B, int d, int rows, const int32_t* rows_dev, float* stored,
                            float* xnorm, uint32_t* wnorm_max, float* err_c, void* stream) {
  if (!W || !x || !rows_dev || !stored || !xnorm || !wnorm_max || !err_c || B < 1 || B > HIRE_MAX_BATCH || rows < 1 ||
      d < 8 || d % 8 != 0 || !aligned(W, 16) || !aligned(x, 16))
    return HIRE_EINVAL;
  *err_c = gather_filter_error(B);
  HIRE_TRY(launch_gather_dot_bf16(static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(x), B, d, nullptr,
                                  rows_dev, rows, stored, rows, HistRefs{}, nullptr, rows, 1, xnorm, wnorm_max,
                                  static_cast<hipStream_t>(stream)));
  return HIRE_OK;
}

int hire_set_scorer_clocks(void* device_buf, size_t bytes) {
  if (device_buf && (bytes < 2 * 1024 * sizeof(unsigned long long) || !aligned(device_buf, 8))) return HIRE_EINVAL;
  g_scorer_clocks = static_cast<unsigned long long*>(device_buf);
  return HIRE_OK;
}

int hire_ffn_scorer_workgroups(int d_ff) { return d_ff > 0 ? ffn_fast_score_blocks(d_ff) : 0; }

void hire_force_generic_path(int on) { g_force_generic = on; }

void hire_force_exact_stage(int on) { g_force_exact_stage = on; }

void hire_set_stage_events(void** events) { g_stage_events = reinterpret_cast<hipEvent_t*>(events); }

const char* hire_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

size_t hire_pack_int4_bytes(int rows, int cols) {
  if (rows < 1 || cols < 32 || cols % 32 != 0) return 0;
  return (size_t)rows * (size_t)(cols / 2) + kPackTrailerBytes;
}

int hire_pack_int4(const void* w_bf16, int rows, int cols, void* q4_out, float* scale_out, void* stream) {
  if (!w_bf16 || !q4_out || !scale_out || rows < 1 || cols < 32 || cols % 32 != 0) return HIRE_EINVAL;
  if (!aligned(q4_out, 16)) return HIRE_EINVAL;
  HIRE_TRY(launch_pack_int4(static_cast<const uint16_t*>(w_bf16), rows, cols, static_cast<uint32_t*>(q4_out),
                            scale_out, static_cast<hipStream_t>(stream)));
  return HIRE_OK;
}

int hire_unpack_int4(const void* q4, int rows, int cols, int8_t* codes_out, void* stream) {
  if (!q4 || !codes_out || rows < 1 || cols < 32 || cols % 32 != 0) return HIRE_EINVAL;
  HIRE_TRY(launch_unpack_int4(static_cast<const uint32_t*>(q4), rows, cols, codes_out,
                              static_cast<hipStream_t>(stream)));
  return HIRE_OK;
}

size_t hire_ffn_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime) {
  if (!L || L->d_model < 32 || L->d_ff < 1 || B < 1 || B > HIRE_MAX_BATCH || k < 1 || k > kprime || kprime > L->d_ff)
    return 0;
  return carve(nullptr, L->scorer_kind, B, L->d_model, L->d_ff, L->r, k, kprime, true).bytes;
}

size_t hire_softmax_workspace_bytes(const hire_softmax_layer* L, int B, int k, int kprime) {
  if (!L || L->d_model < 32 || L->vocab < 1 || B < 1 || B > HIRE_MAX_BATCH || k < 1 || k > kprime ||
      kprime > L->vocab)
    return 0;
  return carve(nullptr, L->scorer_kind, B, L->d_model, L->vocab, L->r, k, kprime, false).bytes;
}

// Long rows in index order go through the many-workgroup selection, which keeps histograms in the workspace.
// Rank order on such rows: the same selection in index order into the workspace, then the k survivors of every row
// are ranked by the single-workgroup kernel (positions there are in index order, so ties still go to the lower
// index).
static bool topk_long_route(int N, int /*flags*/) { return N > kSingleWgMaxRow; }
static size_t topk_rank_tmp_bytes(int B, int k, int flags) {
  return (flags & HIRE_ORDER_RANK) ? 2 * align_up((size_t)B * k * sizeof(int32_t)) : 0;
}

size_t hire_topk_workspace_bytes(int B, int N, int k, int flags) {
  if (B < 1 || N < 1 || k < 1 || k > N) return 0;
  if (!topk_long_route(N, flags)) return kAlign;  // LDS and registers only; a token amount keeps the pointer non-null
  // the header sits where the step workspaces have it, so that one initialisation routine serves all
  return align_up(ffn_fast_region_bytes()) + align_up(general_header_bytes()) +
         align_up(topk_long_workspace_bytes(B, N)) + topk_rank_tmp_bytes(B, k, flags);
}

int hire_ffn_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, float* y, int32_t* topk_idx,
                  float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc, void* workspace,
                  size_t workspace_bytes, void* stream) {
  if (!L || !y || !workspace) return HIRE_EINVAL;
  const int d = L->d_model, N = L->d_ff;
  int rc = check_common(d, N, B, k, kprime, L->scorer_kind, L->q4, L->q4_scale, L->lr_a, L->lr_b, L->r, L->lr_a_scale,
                        L->lr_b_scale, L->w1u, x);
  if (rc != HIRE_OK) return rc;
  if (!L->w2u || !aligned(L->w2u, 256) || !aligned(workspace, 256) || !aligned(y, 16)) return HIRE_EINVAL;
  if (scorer_acc && L->scorer_kind != HIRE_SCORER_INT4) return HIRE_EINVAL;
  const StepBuffers s = carve(workspace, L->scorer_kind, B, d, N, L->r, k, kprime, true);
  if (workspace_bytes < s.bytes) return HIRE_ENOSPC;
  hipStream_t st = static_cast<hipStream_t>(stream);

  const bool fast_int4 = L->scorer_kind == HIRE_SCORER_INT4;
  const bool fast_lr = L->scorer_kind == HIRE_SCORER_LOWRANK && L->row_norm_bounds != nullptr && L->r <= 1024;
  const bool fast_lrq = L->scorer_kind == HIRE_SCORER_LRQ && L->row_norm_bounds != nullptr && L->r <= 8192 &&
                        scorer_int4_fused_supported(d);
  if ((fast_int4 || fast_lr || fast_lrq) && ffn_fast_supported(B, N, d, k, kprime) && !g_force_generic) {
    FfnFastArgs a{};
    a.N = N; a.d = d; a.k = k; a.kprime = kprime;
    a.q4 = L->q4; a.q4_scale = L->q4_scale;
    a.lowrank = fast_lr;
    a.lrq = fast_lrq;
    if (fast_lr || fast_lrq) {
      a.lr_a = L->lr_a; a.lr_b = L->lr_b; a.r = L->r; a.norm_bounds = L->row_norm_bounds;
      a.t_partial = s.t_partial; a.keys64 = static_cast<double*>(s.keys);
      a.lr_a_scale = L->lr_a_scale; a.lr_b_scale = L->lr_b_scale; a.keys_t = s.keys_t;
    }
    a.w1u = static_cast<const uint16_t*>(L->w1u); a.w2u = static_cast<const uint16_t*>(L->w2u);
    a.x = static_cast<const uint16_t*>(x); a.y = y;
    a.topk_idx = topk_idx; a.topk_val = topk_val;
    a.cand = s.cand; a.cand_out = cand_idx; a.n_cand = n_cand; a.scorer_acc = scorer_acc;
    a.fast_region = s.fast_region;
    a.keys = static_cast<float*>(s.keys); a.h = s.h; a.partial = s.partial;
    a.stage_events = g_stage_events;
    a.scorer_clocks = g_scorer_clocks;
    HIRE_TRY(launch_ffn_fast(a, st));
    return HIRE_OK;
  }

  // step 4: exact top-k of h over U for every token
  SelectParams sp{};
  sp.vals = s.h;
  sp.stride = s.cap_u;
  sp.n_dev = s.counters;
  sp.n_cap = s.cap_u;
  sp.k = k;
  sp.idx_out = topk_idx ? topk_idx : s.sel_idx;
  sp.val_out = topk_val;
  sp.pos_out = s.pos;
  sp.nonneg = 1;  // activations after the ReLU
  sp.window_misses = s.window_misses;
  // Batches: filter and refine.  The exact stage runs on the bf16 matrix cores and stores fp32 values within a
  // proven distance of the activations; the selection finds the k-th largest stored value of every token,
  // recomputes in fp64 the entries within twice that distance of it and selects on the result.  Whatever lies
  // outside that band is on the same side of the threshold in fp64 as its stored value, so the selected sets are
  // those of the fp64 activations.
  SelectParams fr = sp;
  fr.vals = s.hf;
  fr.stride = s.hf_stride;
  fr.refine_w = static_cast<const uint16_t*>(L->w1u);
  fr.refine_x = static_cast<const uint16_t*>(x);
  fr.refine_d = d;
  fr.refine_h = s.h;
  fr.refine_h_stride = s.cap_u;
  fr.xnorm = s.xnorm;
  fr.wnorm_max = reinterpret_cast<const uint32_t*>(s.counters + kCntWnormMax);
  fr.err_c = gather_filter_error(B);
  const bool filter = B >= kFilterMinBatch && s.hf != nullptr && select_refine_supported(fr) && !g_force_exact_stage;
  rc = run_front(s, scorer_of(L), L->w1u, x, B, d, N, kprime, 1, cand_idx, n_cand, scorer_acc, st, 0, filter);
  if (rc != HIRE_OK) return rc;
  const int32_t* cand = cand_idx ? cand_idx : s.cand;
  sp.map = fr.map = cand;
  HIRE_STAGE(5, st);
  if (filter)
    HIRE_TRY(launch_select_refine(fr, B, st));
  else
    HIRE_TRY(launch_select_f64(sp, B, st));
  HIRE_STAGE(6, st);

  // step 5: second layer over each token's selected rows
  HIRE_TRY(launch_w2_tokens(static_cast<const uint16_t*>(L->w2u), d, B, k, s.pos, cand, s.h, s.cap_u, s.partial, y,
                            0, nullptr, 0, st));
  HIRE_STAGE(7, st);
  return HIRE_OK;
}

// Address of the calling thread's current device's copy of `scratch`, looked up once per device.
static int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> ptr_of_device[kMaxDevices];
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    g_last_hip_error = e != hipSuccess ? e : hipErrorInvalidDevice;
    return HIRE_ELAUNCH;
  }
  void* p = ptr_of_device[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      g_last_hip_error = e != hipSuccess ? e : hipErrorInvalidSymbol;
      return HIRE_ELAUNCH;
    }
    ptr_of_device[dev].store(p, std::memory_order_release);  // threads that race here store the same address
  }
  *out = p;
  return HIRE_OK;
}

int hire_ffn_step_static(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, float* y, int32_t* topk_idx,
                         float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc, void* stream) {
  const size_t need = hire_ffn_workspace_bytes(L, B, k, kprime);
  if (need == 0) return HIRE_EINVAL;
  if (need > (size_t)HIRE_STATIC_SCRATCH_BYTES) return HIRE_ENOSPC;
  void* ws = nullptr;
  if (const int rc = static_scratch(&ws); rc != HIRE_OK) return rc;
  return hire_ffn_step(L, x, B, k, kprime, y, topk_idx, topk_val, cand_idx, n_cand, scorer_acc, ws,
                       (size_t)HIRE_STATIC_SCRATCH_BYTES, stream);
}

static int group_shift(int group) {
  for (int gs = 0; gs <= 4; ++gs)
    if (group == 1 << gs) return gs;
  return -1;
}

static int check_group(const hire_ffn_layer* L, int B, int k, int kprime, int group) {
  const int gs = group_shift(group);
  if (!L || gs < 0 || L->d_ff < 1 || L->d_ff % group || k % group || kprime % group) return -1;
  if ((L->d_ff >> gs) > kSingleWgMaxRow) return -1;
  if (L->d_model < 32 || B < 1 || B > HIRE_MAX_BATCH || k < 1 || k > kprime || kprime > L->d_ff) return -1;
  return gs;
}

size_t hire_ffn_group_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime, int group) {
  const int gs = check_group(L, B, k, kprime, group);
  if (gs < 0) return 0;
  return carve(nullptr, L->scorer_kind, B, L->d_model, L->d_ff, L->r, k, kprime, true, gs).bytes;
}

// Dense common-path units riding along with a group-sparse step (eq. (7)).  folded is set when the step's own
// launches have added them to y; otherwise the caller adds them with kernels of their own.
struct DenseRefs {
  const uint16_t* w1u;
  const uint16_t* w2u;
  int m1;
  double* h;          // [m1] workspace
  float* fast_partial; // ffn_fast_partial_floats(d, k, m1) floats
  bool folded;
};

static int ffn_group_step_impl(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, int group, float* y,
                               int32_t* topk_group, float* topk_val, int32_t* cand_group, int32_t* n_cand,
                               int32_t* scorer_acc, void* workspace, size_t workspace_bytes, void* stream,
                               DenseRefs* dense) {
  if (!L || !y || !workspace) return HIRE_EINVAL;
  const int d = L->d_model, N = L->d_ff;
  int rc = check_common(d, N, B, k, kprime, L->scorer_kind, L->q4, L->q4_scale, L->lr_a, L->lr_b, L->r, L->lr_a_scale,
                        L->lr_b_scale, L->w1u, x);
  if (rc != HIRE_OK) return rc;
  if (!L->w2u || !aligned(L->w2u, 256) || !aligned(workspace, 256) || !aligned(y, 16)) return HIRE_EINVAL;
  if (scorer_acc && L->scorer_kind != HIRE_SCORER_INT4) return HIRE_EINVAL;
  const int gs = group_shift(group);
  if (gs < 0 || N % group || k % group || kprime % group) return HIRE_EINVAL;
  if ((N >> gs) > kSingleWgMaxRow) return HIRE_EUNSUPPORTED;
  const StepBuffers s = carve(workspace, L->scorer_kind, B, d, N, L->r, k, kprime, true, gs);
  if (workspace_bytes < s.bytes) return HIRE_ENOSPC;
  hipStream_t st = static_cast<hipStream_t>(stream);

  if (L->scorer_kind == HIRE_SCORER_INT4 && gs == 3 && ffn_fast_group8_supported(B, N, d, k, kprime) &&
      !g_force_generic) {  // batch 1, groups of eight: the four-kernel route on group activations
    FfnFastArgs a{};
    a.N = N; a.d = d; a.k = k; a.kprime = kprime;
    a.q4 = L->q4; a.q4_scale = L->q4_scale;
    a.w1u = static_cast<const uint16_t*>(L->w1u); a.w2u = static_cast<const uint16_t*>(L->w2u);
    a.x = static_cast<const uint16_t*>(x); a.y = y;
    a.topk_idx = topk_group; a.topk_val = topk_val;
    a.cand = s.cand; a.cand_out = cand_group; a.n_cand = n_cand; a.scorer_acc = scorer_acc;
    a.fast_region = s.fast_region;
    a.keys = static_cast<float*>(s.keys); a.h = s.h; a.partial = s.partial;
    a.gs = 3; a.gkeys = static_cast<float*>(s.gkeys); a.hg = s.hg;
    if (dense != nullptr && dense->m1 > 0) {
      a.dense_w1u = dense->w1u; a.dense_w2u = dense->w2u; a.m1 = dense->m1; a.h_dense = dense->h;
      a.partial = dense->fast_partial;
      dense->folded = true;
    }
    a.stage_events = g_stage_events;
    a.scorer_clocks = g_scorer_clocks;
    HIRE_TRY(launch_ffn_fast(a, st));
    return HIRE_OK;
  }

  // scorer, group sums of its keys, top k'/g groups per token, union, exact activations of the union's units
  rc = run_front(s, scorer_of(L), L->w1u, x, B, d, N, kprime, 1, cand_group, n_cand, scorer_acc, st, gs);
  if (rc != HIRE_OK) return rc;
  const int32_t* cand = cand_group ? cand_group : s.cand;
  HIRE_STAGE(5, st);

  // exact group activations and the top k/g groups of every token
  // (groups of eight: summed by the selection as it loads h; other sizes by a kernel of their own)
  const bool in_select = gs == 3 && s.cap_u <= kSelectGroup8Max;
  const double* ranked = s.h;
  if (gs > 0 && !in_select) {
    HIRE_TRY(launch_group_sums_f64(s.h, B, (long long)s.cap_u << gs, 0, s.counters, s.cap_u, gs, s.hg, s.cap_u, st));
    ranked = s.hg;
  }
  SelectParams sp{};
  sp.vals = ranked;
  sp.group8 = in_select ? 1 : 0;
  sp.stride = in_select ? ((long long)s.cap_u << gs) : s.cap_u;
  sp.n_dev = s.counters;
  sp.n_cap = s.cap_u;
  sp.k = k >> gs;
  sp.idx_out = topk_group ? topk_group : s.sel_idx;
  sp.map = cand;
  sp.pos_out = s.pos;
  sp.nonneg = 1;  // activations after the ReLU, or sums of their absolute values
  sp.window_misses = s.window_misses;
  HIRE_TRY(launch_select_f64(sp, B, st));
  HIRE_STAGE(6, st);

  // second layer over the units of each token's groups; it also hands out their activations
  HIRE_TRY(launch_w2_tokens(static_cast<const uint16_t*>(L->w2u), d, B, k, s.pos, cand, s.h, (long long)s.cap_u << gs,
                            s.partial, y, gs, topk_val, 0, st));
  HIRE_STAGE(7, st);
  return HIRE_OK;
}

int hire_ffn_group_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, int group, float* y,
                        int32_t* topk_group, float* topk_val, int32_t* cand_group, int32_t* n_cand,
                        int32_t* scorer_acc, void* workspace, size_t workspace_bytes, void* stream) {
  return ffn_group_step_impl(L, x, B, k, kprime, group, y, topk_group, topk_val, cand_group, n_cand, scorer_acc,
                             workspace, workspace_bytes, stream, nullptr);
}

// CommonPath: the group-sparse step's workspace, then the dense units' activations and partial rows.
struct CommonBuffers {
  size_t sparse_bytes;
  double* h;       // [B, m1]
  float* partial;  // [w2_groups(m1, B, d), B, d]
  float* fast_partial;  // batch 1: the four-kernel route's partial rows, sparse and dense row groups together
  size_t bytes;
};
static CommonBuffers carve_common(void* ws, const hire_ffn_layer* L, int m1, int B, int k, int kprime, int gs) {
  CommonBuffers c{};
  c.sparse_bytes = align_up(carve(nullptr, L->scorer_kind, B, L->d_model, L->d_ff, L->r, k, kprime, true, gs).bytes);
  Carver cv(ws);
  cv.take<char>(c.sparse_bytes);
  c.h = cv.take<double>((size_t)B * m1 + 2);
  c.partial = cv.take<float>((size_t)w2_groups(m1 > 0 ? m1 : 1, B, L->d_model) * B * L->d_model);
  if (B == 1) c.fast_partial = cv.take<float>(ffn_fast_partial_floats(L->d_model, k, m1));
  c.bytes = cv.off;
  return c;
}

size_t hire_ffn_commonpath_workspace_bytes(const hire_ffn_layer* L, int m1, int B, int k, int kprime, int group) {
  const int gs = check_group(L, B, k, kprime, group);
  if (gs < 0 || m1 < 0) return 0;
  return carve_common(nullptr, L, m1, B, k, kprime, gs).bytes;
}

int hire_ffn_commonpath_step(const hire_ffn_layer* L, const void* dense_w1u, const void* dense_w2u, int m1,
                             const void* x, int B, int k, int kprime, int group, float* y, int32_t* topk_group,
                             float* topk_val, int32_t* cand_group, int32_t* n_cand, int32_t* scorer_acc,
                             void* workspace, size_t workspace_bytes, void* stream) {
  if (!L || m1 < 0) return HIRE_EINVAL;
  if (m1 > 0 && (!dense_w1u || !dense_w2u || !aligned(dense_w1u, 256) || !aligned(dense_w2u, 256))) return HIRE_EINVAL;
  const int gs = group_shift(group);
  if (gs < 0) return HIRE_EINVAL;
  const size_t need = hire_ffn_commonpath_workspace_bytes(L, m1, B, k, kprime, group);
  if (need != 0 && workspace_bytes < need) return HIRE_ENOSPC;
  // the sparse units first: it validates the shared arguments and writes y; at batch 1 with groups of eight its
  // own launches take the dense units along
  CommonBuffers c{};
  DenseRefs dense{};
  if (need != 0 && m1 > 0) {
    c = carve_common(workspace, L, m1, B, k, kprime, gs);
    dense = DenseRefs{static_cast<const uint16_t*>(dense_w1u), static_cast<const uint16_t*>(dense_w2u), m1, c.h,
                      c.fast_partial, false};
  }
  int rc = ffn_group_step_impl(L, x, B, k, kprime, group, y, topk_group, topk_val, cand_group, n_cand, scorer_acc,
                               workspace, workspace_bytes, stream, (need != 0 && m1 > 0 && B == 1) ? &dense : nullptr);
  if (rc != HIRE_OK || m1 == 0 || dense.folded) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int d = L->d_model;
  const uint16_t* xb = static_cast<const uint16_t*>(x);
  const HistRefs none{};
  // dense units: every row's activation, then the second layer over all of them, added onto y
  if (B >= kMfmaMinBatch)
    HIRE_TRY(launch_gather_dot_mfma(static_cast<const uint16_t*>(dense_w1u), xb, B, d, nullptr, m1, nullptr, m1, 1, c.h,
                                    m1, none, nullptr, 0, st));
  else
    HIRE_TRY(launch_gather_dot(static_cast<const uint16_t*>(dense_w1u), xb, d, nullptr, m1, nullptr, m1, 1, c.h, none,
                               nullptr, 0, st));
  HIRE_TRY(launch_w2_tokens(static_cast<const uint16_t*>(dense_w2u), d, B, m1, nullptr, nullptr, c.h, m1, c.partial, y,
                            0, nullptr, 1, st));
  return HIRE_OK;
}

// The partial rows sit behind the places of the two route headers, so that a workspace shared with the other
// entry points keeps their headers intact.
static size_t shard_partial_offset() { return align_up(ffn_fast_region_bytes()) + align_up(general_header_bytes()); }

static bool shard_args_ok(const hire_ffn_layer* L, int B, int k, int kprime, int shards) {
  if (!L || L->d_model < 32 || L->d_ff < 1 || B < 1 || B > HIRE_MAX_BATCH || k < 1 || k > kprime || kprime > L->d_ff)
    return false;
  return shards >= 1 && L->d_ff % shards == 0;
}

size_t hire_ffn_shard_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime, int shards) {
  if (!shard_args_ok(L, B, k, kprime, shards) || !ffn_shard_supported(L->d_ff, L->d_model, shards)) return 0;
  return shard_partial_offset() + align_up(ffn_shard_partial_floats(B, L->d_model, shards) * sizeof(float));
}

int hire_ffn_shard_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, int shards, float* y,
                        int32_t* topk_idx, float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc,
                        void* workspace, size_t workspace_bytes, void* stream) {
  if (!L || !y || !workspace) return HIRE_EINVAL;
  const int d = L->d_model, N = L->d_ff;
  if (L->scorer_kind != HIRE_SCORER_INT4) return HIRE_EUNSUPPORTED;
  int rc = check_common(d, N, B, k, kprime, L->scorer_kind, L->q4, L->q4_scale, L->lr_a, L->lr_b, L->r, L->lr_a_scale,
                        L->lr_b_scale, L->w1u, x);
  if (rc != HIRE_OK) return rc;
  if (!L->w2u || !aligned(L->w2u, 256) || !aligned(workspace, 256) || !aligned(y, 16)) return HIRE_EINVAL;
  if (!shard_args_ok(L, B, k, kprime, shards)) return HIRE_EINVAL;
  if (!ffn_shard_supported(N, d, shards)) return HIRE_EUNSUPPORTED;
  if (workspace_bytes < hire_ffn_shard_workspace_bytes(L, B, k, kprime, shards)) return HIRE_ENOSPC;
  FfnShardArgs a{};
  a.N = N; a.d = d; a.B = B; a.k = k; a.kprime = kprime; a.shards = shards;
  a.q4 = L->q4; a.q4_scale = L->q4_scale;
  a.w1u = static_cast<const uint16_t*>(L->w1u); a.w2u = static_cast<const uint16_t*>(L->w2u);
  a.x = static_cast<const uint16_t*>(x); a.y = y;
  a.topk_idx = topk_idx; a.topk_val = topk_val; a.cand = cand_idx; a.n_cand = n_cand; a.scorer_acc = scorer_acc;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + shard_partial_offset());
  hipStream_t st = static_cast<hipStream_t>(stream);
  HIRE_STAGE(0, st);
  HIRE_TRY(launch_ffn_shard(a, st));
  HIRE_STAGE(1, st);
  HIRE_TRY(launch_ffn_shard_reduce(a, st));
  HIRE_STAGE(2, st);
  return HIRE_OK;
}

int hire_softmax_step(const hire_softmax_layer* L, const void* x, int B, int k, int kprime, int32_t* top_idx,
                      float* top_prob, float* top_logit, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!L || !top_idx || !top_prob || !workspace) return HIRE_EINVAL;
  const int d = L->d_model, N = L->vocab;
  int rc = check_common(d, N, B, k, kprime, L->scorer_kind, L->q4, L->q4_scale, L->lr_a, L->lr_b, L->r, L->lr_a_scale,
                        L->lr_b_scale, L->w, x);
  if (rc != HIRE_OK) return rc;
  if (k > HIRE_MAX_RANK_ORDER_K) return HIRE_EUNSUPPORTED;
  if (!aligned(workspace, 256)) return HIRE_EINVAL;
  if (scorer_acc && L->scorer_kind != HIRE_SCORER_INT4) return HIRE_EINVAL;
  const StepBuffers s = carve(workspace, L->scorer_kind, B, d, N, L->r, k, kprime, false);
  if (workspace_bytes < s.bytes) return HIRE_ENOSPC;
  hipStream_t st = static_cast<hipStream_t>(stream);

  // Batches: filter and refine as in the FFN step - fp32 logits with a proven error from the bf16 matrix cores,
  // fp64 only for the entries that can still be among the k largest.
  const bool filter = B >= kFilterMinBatch && s.hf != nullptr && s.cap_u <= kSoftmaxRefineMaxRow &&
                      k <= kSoftmaxRefineMaxK && d % 8 == 0 && !g_force_exact_stage;
  // One token on a long vocabulary: the scorer (both int4 kinds), the exact logits of a superset of the shortlist
  // (from the scorer's maxima), and the final selections with the softmax.
  const bool lrq = L->scorer_kind == HIRE_SCORER_LRQ;
  const int sd = lrq ? L->r : d;  // codes per row of the matrix that produces the keys
  if (s.sm1_ok && scorer_int4_fused_supported(sd) && (!lrq || scorer_int4_fused_supported(d)) &&
      softmax_b1_supported(N, d, k, kprime) && softmax_b1_worthwhile(N, kprime, scorer_int4_fused_maxima(N, sd)) &&
      !g_force_generic) {
    int n_max = 0;
    rc = run_front(s, scorer_of(L), L->w, x, B, d, N, kprime, 0, cand_idx, n_cand, scorer_acc, st, 0, false, &n_max);
    if (rc != HIRE_OK) return rc;
    HIRE_STAGE(3, st);
    HIRE_STAGE(4, st);
    HIRE_TRY(launch_softmax_b1(static_cast<const float*>(s.keys), N, d, sd, k, kprime, n_max, lrq ? L->lr_b : L->q4,
                               static_cast<const uint16_t*>(L->w), static_cast<const uint16_t*>(x), s.hist,
                               s.sm1_slots, top_idx, top_prob, top_logit, cand_idx, n_cand, st));
    HIRE_STAGE(5, st);
    HIRE_STAGE(6, st);
    return HIRE_OK;
  }
  rc = run_front(s, scorer_of(L), L->w, x, B, d, N, kprime, 0, cand_idx, n_cand, scorer_acc, st, 0, filter);
  if (rc != HIRE_OK) return rc;
  HIRE_STAGE(5, st);

  SelectParams sp{};
  sp.vals = s.h;
  sp.stride = s.cap_u;
  sp.n_dev = s.counters;
  sp.n_cap = s.cap_u;
  sp.k = k;
  sp.rank_order = 1;
  sp.idx_out = top_idx;
  sp.val_out = top_logit;
  sp.prob_out = top_prob;
  sp.map = cand_idx ? cand_idx : s.cand;
  sp.window_misses = s.window_misses;
  if (filter) {
    sp.vals = s.hf;
    sp.stride = s.hf_stride;
    sp.refine_w = static_cast<const uint16_t*>(L->w);
    sp.refine_x = static_cast<const uint16_t*>(x);
    sp.refine_d = d;
    sp.xnorm = s.xnorm;
    sp.wnorm_max = reinterpret_cast<const uint32_t*>(s.counters + kCntWnormMax);
    sp.err_c = gather_filter_error(B);
    HIRE_TRY(launch_softmax_refine(sp, B, st));
  } else {
    HIRE_TRY(launch_select_f64(sp, B, st));
  }
  HIRE_STAGE(6, st);
  return HIRE_OK;
}

int topk_select(const float* scores, int B, int N, int k, int flags, int32_t* idx_out, float* val_out, void* workspace,
                size_t workspace_bytes, void* stream) {
  if (!scores || !idx_out || B < 1 || N < 1 || k < 1 || k > N) return HIRE_EINVAL;
  if ((flags & HIRE_ORDER_RANK) && k > HIRE_MAX_RANK_ORDER_K) return HIRE_EUNSUPPORTED;
  if (topk_long_route(N, flags)) {
    if (!workspace || !aligned(workspace, 256)) return HIRE_EINVAL;
    if (workspace_bytes < hire_topk_workspace_bytes(B, N, k, flags)) return HIRE_ENOSPC;
    char* base = static_cast<char*>(workspace) + align_up(ffn_fast_region_bytes());
    char* body = base + align_up(general_header_bytes());
    const bool rank = (flags & HIRE_ORDER_RANK) != 0;
    int32_t* idx_tmp = reinterpret_cast<int32_t*>(body + align_up(topk_long_workspace_bytes(B, N)));
    float* val_tmp = reinterpret_cast<float*>(reinterpret_cast<char*>(idx_tmp) +
                                              align_up((size_t)B * k * sizeof(int32_t)));
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIRE_TRY(launch_topk_long(scores, B, N, k, (flags & HIRE_RELU) ? 1 : 0, rank ? idx_tmp : idx_out,
                              rank ? val_tmp : val_out, base, body,
                              layout_signature(2 /* neither scorer: a bare selection */, B, 0, N, 0, k, 0, flags), st));
    if (rank) {  // all k entries of the index-ordered list, in rank order
      SelectParams sp{};
      sp.vals = val_tmp;  // max(., 0) already applied where asked for
      sp.stride = k;
      sp.n = k;
      sp.n_cap = k;
      sp.k = k;
      sp.rank_order = 1;
      sp.idx_out = idx_out;
      sp.val_out = val_out;
      sp.map = idx_tmp;
      sp.map_stride = k;
      HIRE_TRY(launch_select_f32(sp, B, st));
    }
    return HIRE_OK;
  }
  SelectParams sp{};
  sp.vals = scores;
  sp.stride = N;
  sp.n = N;
  sp.n_cap = N;
  sp.k = k;
  sp.relu = (flags & HIRE_RELU) ? 1 : 0;
  sp.rank_order = (flags & HIRE_ORDER_RANK) ? 1 : 0;
  sp.idx_out = idx_out;
  sp.val_out = val_out;
  HIRE_TRY(launch_select_f32(sp, B, static_cast<hipStream_t>(stream)));
  return HIRE_OK;
}

}  // extern "C"
