// Host-side launch interface of the HiRE kernels (internal to libhire).
// Every launcher enqueues on `stream` and returns the HIP launch status.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace hire {

// Launch and report this launch's status only: the sticky "last error" is cleared first, because other users
// of the runtime in the same process (PyTorch) may have left an unrelated one behind.
template <typename... Params, typename... Args>
inline hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         Args... args) {
  (void)hipGetLastError();
  kernel<<<grid, block, lds, stream>>>(args...);
  return hipGetLastError();
}

// Dynamic LDS beyond the default limit needs the kernel's attribute raised before the launch.  `raised_to` is a
// counter of the call site's own (one per kernel instantiation): the attribute is set again only when a launch
// asks for more than any before it.  Threads that race here set the same attribute twice, which is harmless.
constexpr size_t kDefaultDynamicLds = 48 * 1024;
inline hipError_t ensure_dynamic_lds(const void* kernel, size_t lds, std::atomic<size_t>& raised_to) {
  if (lds <= kDefaultDynamicLds || raised_to.load(std::memory_order_acquire) >= lds) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e == hipSuccess) raised_to.store(lds, std::memory_order_release);
  return e;
}

// Places of the general route's histograms in the caller's workspace (any may be null: no histograms).
struct HistRefs {
  void* header;      // general_header_bytes() at a fixed place, cleared by the workspace initialisation
  void* multi_body;  // multi_body_bytes_host(B): per-token histograms of the scorer keys (long rows)
};
size_t general_header_bytes();
unsigned long long layout_signature(int scorer_kind, int B, int d, int N, int r, int k, int kprime, int ffn);

// ---- scorer.hip ------------------------------------------------------------
// The packed blob is rows * cols / 2 bytes of codes followed by kPackTrailerBytes: the first trailer word holds the
// largest row scale (float bits; all-zero rows left out), which the batch-1 FFN scorer turns into an upper bound
// of every key of a step; the rest is zero.
constexpr size_t kPackTrailerBytes = 64;
hipError_t launch_pack_int4(const uint16_t* w, int rows, int cols, uint32_t* q4, float* scale, hipStream_t s);
hipError_t launch_unpack_int4(const uint32_t* q4, int rows, int cols, int8_t* codes, hipStream_t s);

// x bf16 [B,d] -> xq int8 [B,d], sx fp32 [B]; also clears `zero_words` 32-bit words at zero_ptr.  As a step's
// first kernel it checks the general header (optional) against the layout signature.
hipError_t launch_quantize_tokens(const uint16_t* x, int B, int d, int8_t* xq, float* sx, uint32_t* zero_ptr,
                                  int zero_words, void* general_header, unsigned long long sig, hipStream_t s);

// One token (B == 1): keys[j] = phi(float(sum_i q[j,i] xq[i]) * scale[j]); acc (optional) gets the integer sums.
// With histogram places the kernel also leaves the key counts and the per-workgroup maxima for launch_mark_f32.
hipError_t launch_scorer_int4(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d, int relu,
                              float* keys, int32_t* acc, const HistRefs& hr, hipStream_t s);
int scorer_int4_blocks(int N);
// The same as a step's first kernel, for rows of at most 8192 codes: quantises the token itself (x bf16 [d]),
// clears zero_words words at zero_ptr and checks the general header against the layout signature.
bool scorer_int4_fused_supported(int d);
// out[i] = bf16(in[i]), round to nearest even, i < n.
hipError_t launch_f32_to_bf16(const float* in, int n, uint16_t* out, hipStream_t s);
hipError_t launch_scorer_int4_fused(const uint32_t* q4, const float* scale, const void* x, bool x_is_f32, int N, int d,
                                    int relu, float* keys, int32_t* acc, const HistRefs& hr, uint32_t* zero_ptr,
                                    int zero_words, unsigned long long sig, hipStream_t s);
// x_is_f32: the token is fp32 [d] and is rounded to bf16 (nearest even) before it is quantised; only for rows the
// short-row kernels take (scorer_int4_fused_takes_f32(d)).
bool scorer_int4_fused_takes_f32(int d);
int scorer_int4_fused_blocks(int N, int d);  // workgroups launch_scorer_int4_fused uses
int scorer_int4_fused_maxima(int N, int d);  // maxima it leaves per token: one per workgroup, short rows one per wave
// The same on the int8 matrix cores, for batches (scorer_mfma.hip); B <= 64.
hipError_t launch_scorer_int4_mfma(const uint32_t* q4, const float* scale, const int8_t* xq, int B, int N, int d,
                                   int relu, float* keys, int32_t* acc, const HistRefs& hr, hipStream_t s);
int scorer_mfma_blocks(int N);
int scorer_mfma_maxima(int N);  // maxima it leaves per token: one per wave

// t[b,:] = bf16(Z1^T x_b); also clears zero_words words at zero_ptr and, as a step's first kernel, checks the
// general header (optional) against the layout signature.
// partial: fp64 [B, lr_project_slices(d), r] scratch.
int lr_project_slices(int d);
hipError_t launch_lr_project(const uint16_t* z1, const uint16_t* x, int B, int d, int r, uint16_t* t, double* partial,
                             uint32_t* zero_ptr, int zero_words, void* general_header, unsigned long long sig,
                             hipStream_t s);
// One token: keys[j] = phi(<Z2[j,:], t>) in fp64.  Batches run launch_gather_dot_mfma over all rows instead.
// *out = an upper bound of the largest row norm of the bf16 matrix W [rows, cols] (cols a multiple of 8).
hipError_t launch_row_norm_max(const uint16_t* W, int rows, int cols, float* out, hipStream_t s);
hipError_t launch_lr_score(const uint16_t* z2, const uint16_t* t, int N, int r, int relu, double* keys, hipStream_t s);

// Clears `words` 32-bit words.
hipError_t launch_clear_words(uint32_t* p, int words, hipStream_t s);

// Plain device-to-device copy of `bytes` (multiple of 16).
hipError_t launch_plain_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

// ---- select.hip ------------------------------------------------------------
struct SelectParams {
  const void* vals;         // float or double [B, stride]
  long long stride;
  int n;                    // number of entries per row when n_dev == nullptr
  const int32_t* n_dev;     // device-side count (overrides n); n_cap bounds it
  int n_cap;                // host upper bound of n (chooses the register-resident or the streaming variant)
  int k;
  int relu;                 // rank max(v, 0)
  int rank_order;           // outputs in rank order instead of ascending index
  int32_t* idx_out;         // [B,k] selected indices (through map if given), optional
  float* val_out;           // [B,k] selected values, optional
  const int32_t* map;       // optional translation of positions to indices for idx_out
  long long map_stride;     // row b uses map + b * map_stride (0: one map for all rows)
  int32_t* pos_out;         // [B,k] selected positions (no map), optional
  float* prob_out;          // [B,k] softmax over the selected values (rank order only), optional
  uint32_t* bitmap;         // optional: bit i set (atomic or) for every selected position of any row
  uint32_t* window_misses;  // optional device counter: rows whose window histogram did not give the k-th largest
  // Filter and refine (launch_select_refine only): vals are fp32 rows written by launch_gather_dot_bf16, within
  // err_c |u| |x| of the activations; map lists the rows' units.  The kernel recomputes in fp64
  // (relu(<refine_w[map[i], :], refine_x[b, :]>)) every non-zero entry within 2 * err_c * xnorm[b] * *wnorm_max of the
  // k-th largest stored value and selects on the result.  refine_h [B, refine_h_stride] (fp64) receives the value
  // of every selected entry (and of others): the second layer reads its coefficients there.
  const uint16_t* refine_w;  // bf16 [rows, refine_d]
  const uint16_t* refine_x;  // bf16 [B, refine_d]
  int refine_d;
  double* refine_h;
  long long refine_h_stride;
  const float* xnorm;
  const uint32_t* wnorm_max;
  float err_c;
  int nonneg;               // != 0: every value is known to be >= 0 (keys and activations after a ReLU); such rows
                            // of 1025..16384 entries in index order take a leaner kernel
  int group8;               // != 0 (rows of at most kSelectGroup8Max entries): entry i is the sum of |vals[8 i + l]|,
                            // l < 8, added in index order in the values'
                            // type (group activations of eq. (6)); stride counts values, n / n_dev / n_cap entries
};
constexpr int kSelectGroup8Max = 4096;
hipError_t launch_select_f32(const SelectParams& p, int B, hipStream_t s);
// The k largest of every row of scores [B, N] in ascending index order, selected by many workgroups per row
// through key histograms (for long rows).  general_header: general_header_bytes() cleared by the workspace
// initialisation; body: topk_long_workspace_bytes(B, N).  N <= 16384 * 4096.
size_t topk_long_workspace_bytes(int B, int N);
hipError_t launch_topk_long(const float* scores, int B, int N, int k, int relu, int32_t* idx_out, float* val_out,
                            void* general_header, void* body, unsigned long long sig, hipStream_t s);
hipError_t launch_select_f64(const SelectParams& p, int B, hipStream_t s);
// Filter and refine: see SelectParams.  Rows of 1025..16384 fp32 entries, k <= 4096, 16-byte aligned rows.
bool select_refine_supported(const SelectParams& p);
hipError_t launch_select_refine(const SelectParams& p, int B, hipStream_t s);
// The same for the classifier (phi = identity, signed values, rank order, softmax over the k survivors): every
// entry within 2 * err_c * xnorm[b] * *wnorm_max below the k-th largest stored value is recomputed in fp64 and the k
// largest of those are returned in rank order (idx_out through map, val_out, prob_out).  Rows of at most
// kSoftmaxRefineMaxRow fp32 entries, k <= kSoftmaxRefineMaxK.
constexpr int kSoftmaxRefineMaxRow = 65536, kSoftmaxRefineMaxK = 512;
hipError_t launch_softmax_refine(const SelectParams& p, int B, hipStream_t s);

// HiRE-Softmax for one token after launch_scorer_int4_fused on a long vocabulary (key histograms present): from the
// scorer's per-workgroup maxima (n_max of them) a lower bound of the k'-th largest key, exact logits of the keys at
// or above it (a superset of the shortlist), then Algorithm 1's shortlist, the k largest logits in rank order
// (top_idx, optional top_logit) and their softmax (top_prob); optional cand_idx (the k' shortlisted classes,
// ascending) and n_cand.  q4: the packed codes the keys were scored with, rows of sd codes (their trailer bounds the
// keys); slots: softmax_b1_slot_bytes(N) of scratch.
bool softmax_b1_supported(int N, int d, int k, int kprime);
bool softmax_b1_worthwhile(int N, int kprime, int n_max);  // enough maxima and slots for the bound to serve
size_t softmax_b1_slot_bytes(int N);
hipError_t launch_softmax_b1(const float* keys, int N, int d, int sd, int k, int kprime, int n_max, const void* q4,
                             const uint16_t* W, const uint16_t* x, const HistRefs& hr, void* slots, int32_t* top_idx,
                             float* top_prob, float* top_logit, int32_t* cand_idx, int32_t* n_cand, hipStream_t s);

// The same bound from the scorer's maxima for batches, long rows (maxima_select_supported): for every token the keys
// at or above its bound, then exactly its k' largest keys (ties to the lower index) as bits of the union bitmap
// (which must be clear).  Replaces launch_mark_f32 + launch_resolve_compact; takes no histogram and leaves none.
// slots: maxima_select_slot_bytes(B, N) of scratch.  maxima_select_worthwhile says whether the bound will serve.
bool maxima_select_supported(int N);
bool maxima_select_worthwhile(int N, int kprime, int n_max);
size_t maxima_select_slot_bytes(int B, int N);
hipError_t launch_maxima_select(const float* keys, int B, int N, int sd, int kprime, int n_max, const void* q4,
                                const HistRefs& hr, void* slots, uint32_t* bitmap, hipStream_t s);

// Ascending list of the set bits of bitmap[0..words): list_out, count to count_out[0] and (optional) count_out2[0].
// Also clears zero_words words at zero_ptr (may be nullptr).
hipError_t launch_bitmap_compact(const uint32_t* bitmap, int words, int32_t* list_out, int32_t* count_out,
                                 int32_t* count_out2, uint32_t* zero_ptr, int zero_words, hipStream_t s);

// Histogram-guided top-k' of every token's keys and their union, for keys whose producer has filled the
// key histograms:
// launch_mark_f32 sets the bits of all keys above the threshold bin and lists the keys inside it;
// launch_resolve_compact ranks those, falls back to a streaming selection for tokens whose histogram did not
// answer, restores the region to all-zero and (list_out != nullptr) turns the bitmap into the ascending list.
size_t multi_body_bytes_host(int B);
int multi_hist_shift(int N, int B);  // == the producer-side bin width exactly when the producer counts the keys
bool multi_producer_counts(int N, int B);
// uint32 counters inside the general header: 0 streaming k' selections of the many-workgroup route, 1 window
// misses of single-workgroup selections, 2 stampings of the key histograms
size_t general_fallbacks_offset(int which);
hipError_t launch_mark_f32(const float* keys, int B, int N, int kprime, int slots, const HistRefs& hr, uint32_t* bitmap,
                           hipStream_t s);
hipError_t launch_resolve_compact(const float* keys, int B, int N, int kprime, const HistRefs& hr, uint32_t* bitmap,
                                  int words, int32_t* list_out, int32_t* count_out, int32_t* count_out2,
                                  uint32_t* zero_ptr, int zero_words, hipStream_t s);

// ---- gather.hip, gather_mfma.hip ---------------------------------------------
// The candidate union handed over as a bitmap: the gather kernels then compact it themselves (every workgroup for
// its own share of ranks), write the ascending list and the count, and stamp the key histograms' header on a
// fresh workspace; no compaction kernel runs in between.  Only for bitmaps of at most kUnionLocateMaxWords words
// (union_in_gather); longer ones go through launch_bitmap_compact and the list.
constexpr int kUnionLocateMaxWords = 8192;
struct UnionRefs {
  const uint32_t* bitmap;
  int words;
  int32_t* list_out;
  int32_t* count_out;
  int32_t* count_out2;  // optional
  bool stamp_keys;      // the key histograms were cleared by the kernel before: stamp their header
};
bool union_in_gather(int words);

// One token: h[t] = phi(<W[list[t], :], x>) for t < n (n from n_dev if given), fp64 accumulation.
// list == nullptr without a union bitmap: row t itself.
// gs > 0 (both gathers): list entries are groups of 2^gs adjacent rows (2^gs <= 16); entry e, row l of the group
// -> W row list[e] * 2^gs + l -> h column e * 2^gs + l.  n, n_dev and n_cap count entries.
hipError_t launch_gather_dot(const uint16_t* W, const uint16_t* x, int d, const int32_t* list, int n,
                             const int32_t* n_dev, int n_cap, int relu, double* h, const HistRefs& hr,
                             const UnionRefs* un, int gs, hipStream_t s);
// Batches, on the fp64 matrix cores: h[b*stride_h + t].  list == nullptr without a union bitmap: row t itself
// (all n rows in order).
hipError_t launch_gather_dot_mfma(const uint16_t* W, const uint16_t* x, int B, int d, const int32_t* list, int n,
                                  const int32_t* n_dev, int n_cap, int relu, double* h, long long stride_h,
                                  const HistRefs& hr, const UnionRefs* un, int gs, hipStream_t s);

// Filter stage of the exact pre-activations for batches: h[b*stride_h + t] = a value within
// gather_filter_error(B) * |u_{list[t]}| * |x_b| of relu(<u_{list[t]}, x_b>) (bf16 matrix cores, fp32 segments of 32 or 64 products;
// see the kernel for what exactly is stored), xnorm[b] = |x_b|, *wnorm_max = max_t |u_{list[t]}| as float bits
// (atomic max: cleared before the step).  n_dev / n_cap as above; rows only (no groups); n_rows: rows of W (what
// the union bitmap spans).
constexpr int filter_segment_steps(int B) { return B > 32 ? 2 : 1; }  // 32-product MFMA steps per fp32 segment
inline float gather_filter_error(int B) { return (float)filter_segment_steps(B) * 0x1p-17f; }
hipError_t launch_gather_dot_bf16(const uint16_t* W, const uint16_t* x, int B, int d, const int32_t* list,
                                  const int32_t* n_dev, int n_cap, float* h, long long stride_h, const HistRefs& hr,
                                  const UnionRefs* un, int n_rows, int relu, float* xnorm, uint32_t* wnorm_max,
                                  hipStream_t s);

// out[b*stride_out + J] = sum_{l < 2^gs} |in[b*stride_in + J*2^gs + l]| for J < n, added in index order in the
// input's type (the group activations of eq. (6)).
hipError_t launch_group_sums_f32(const float* in, int B, long long stride_in, int n, int gs, float* out,
                                 long long stride_out, hipStream_t s);
hipError_t launch_group_sums_f64(const double* in, int B, long long stride_in, int n, const int32_t* n_dev, int n_cap,
                                 int gs, double* out, long long stride_out, hipStream_t s);

// y[b,:] = sum_{i < k} fl32(h[b*h_stride + pos[b*k + i]]) * W2[map[pos[b*k + i]], :]; deterministic two-stage
// reduction.  partial: fp32 [w2_groups(k, B, d), B, d] scratch.
// gs > 0: pos is [B, k >> gs] groups; entry i < k is unit i % 2^gs of group i >> gs (row map[pos] * 2^gs + l,
// coefficient h[pos * 2^gs + l]).  val_out (optional): fp32 [B, k] coefficients in entry order.
// pos == nullptr: entries 0 .. k-1 in order for every token.  accumulate != 0: y += the sum instead of y = it.
int w2_groups(int k, int B, int d);
hipError_t launch_w2_tokens(const uint16_t* W2, int d, int B, int k, const int32_t* pos, const int32_t* map,
                            const double* h, long long h_stride, float* partial, float* y, int gs, float* val_out,
                            int accumulate, hipStream_t s);

// ---- ffn_fast.hip ----------------------------------------------------------
// Batch-1 FFN step in three kernels; see the file header.  All pointers device.
struct FfnFastArgs {
  int N, d, k, kprime;
  const void* q4;
  const float* q4_scale;
  const uint16_t* w1u;
  const uint16_t* w2u;
  const uint16_t* x;
  float* y;
  int32_t* topk_idx;   // optional
  float* topk_val;     // optional
  int32_t* cand;       // [kprime] workspace, padded to a multiple of 2
  int32_t* cand_out;   // optional: the caller's copy of the candidate list
  int32_t* n_cand;     // optional
  int32_t* scorer_acc; // optional
  // workspace
  void* fast_region;   // ffn_fast_region_bytes() bytes at the head of the workspace (cookie, maxima, histograms)
  float* keys;         // [N] padded to a multiple of 4
  double* h;           // [kprime] padded to a multiple of 2
  float* partial;      // ffn_fast_partial_floats(d, k, m1) floats (none needed when that is 0)
  // group-sparse step with groups of eight units (gs = 3; 0 otherwise): N, k, kprime still count units; cand,
  // n_cand and topk_idx are in groups, topk_val and h per unit
  int gs;
  float* gkeys;        // gs = 3: [N/8] padded to a multiple of 4
  double* hg;          // gs = 3: [kprime/8] padded to a multiple of 2
  // CommonPath (eq. (7)): m1 dense units next to the sparse ones, folded into the gather and second-layer
  // launches as extra workgroups (m1 = 0: none).
  const uint16_t* dense_w1u;  // [m1, d]
  const uint16_t* dense_w2u;  // [m1, d]
  int m1;
  double* h_dense;            // [m1] workspace
  // Low-rank scorer (lowrank; otherwise the int4 one): keys are fp64 (keys64, [N] padded to
  // a multiple of 2), t_partial holds lr_project_slices(d) * r doubles, norm_bounds the two row-norm bounds of
  // hire_lr_prepare.  Plain units only (gs = 0, m1 = 0).
  bool lowrank;
  const void* lr_a;
  const void* lr_b;
  int r;
  const float* norm_bounds;
  double* t_partial;
  double* keys64;
  // int4 low-rank scorer (lrq): lr_a / lr_b are the packed blobs of Z1 transposed and Z2 with their scales, keys_t
  // r + 4 floats for the intermediate; the keys are fp32 (keys); norm_bounds[0] bounds the rows of w1u
  bool lrq;
  const float* lr_a_scale;
  const float* lr_b_scale;
  float* keys_t;
  hipEvent_t* stage_events;  // optional: 5 events recorded around the four kernels
  unsigned long long* scorer_clocks;  // optional: start/end wall clock (100 MHz ticks) of every scorer workgroup
};
size_t ffn_fast_region_bytes();
int ffn_fast_score_blocks(int N);
size_t ffn_fast_fallbacks_offset();  // two uint32 counters inside the region
// Where the region keeps its cookie (and the value that says "key histogram all zero") and its two histograms.
void ffn_fast_state_layout(size_t* cookie_off, unsigned long long* cookie, size_t* hist1_off, size_t* hist2_off,
                           size_t* hist_words);
bool ffn_fast_supported(int B, int N, int d, int k, int kprime);
bool ffn_fast_group8_supported(int B, int N, int d, int k, int kprime);  // the same route for groups of eight units
int ffn_fast_dense_groups(int m1);
void ffn_fast_shape(int d, int rows, int* row_groups, int* col_slices);
size_t ffn_fast_partial_floats(int d, int k, int m1);
hipError_t launch_ffn_fast(const FfnFastArgs& a, hipStream_t s);

// ---- ffn_shard.hip -----------------------------------------------------------
// HiRE-FFN step with Algorithm 2's sharded approximate top-k, one workgroup per shard; see the file header.
// Requires ffn_shard_supported(N, d, shards); quotas ceil(k'/shards), ceil(k/shards).  All pointers device.
constexpr int kShardMaxUnits = 1024;  // units per shard
struct FfnShardArgs {
  int N, d, B, k, kprime, shards;
  const void* q4;
  const float* q4_scale;
  const uint16_t* w1u;
  const uint16_t* w2u;
  const uint16_t* x;
  float* y;
  int32_t* topk_idx;    // optional [B, shards*ceil(k/shards)]
  float* topk_val;      // optional [B, shards*ceil(k/shards)]
  int32_t* cand;        // optional [shards, min(B*ceil(k'/shards), N/shards)]
  int32_t* n_cand;      // optional [shards]
  int32_t* scorer_acc;  // optional [B, N]
  float* partial;       // workspace: ffn_shard_partial_floats(B, d, shards) floats
};
bool ffn_shard_supported(int N, int d, int shards);
size_t ffn_shard_partial_floats(int B, int d, int shards);
hipError_t launch_ffn_shard(const FfnShardArgs& a, hipStream_t s);         // the shards' partial rows
hipError_t launch_ffn_shard_reduce(const FfnShardArgs& a, hipStream_t s);  // y = their sum

}  // namespace hire
