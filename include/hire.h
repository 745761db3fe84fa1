/*
 * hire.h -- C ABI of libhire: the HiRE decode-step hot path on one MI355X (gfx950).
 *
 * HiRE (arXiv 2402.09360, Algorithm 1): a cheap compressed scorer ranks all
 * rows of a weight matrix Z, the top-k' rows form a candidate set S' (unioned
 * over the batch, Sec. 3.4.1 "dynamic overlap"), the exact bf16 computation is
 * done on the gathered candidate rows only, and the exact top-k is taken among
 * them.  Applied to the FFN (Sec. 3.4, eq. (4)) and to the softmax/classifier
 * layer (Sec. 3.3, eq. (2)).
 *
 * General rules, valid for every entry point below:
 *   - Every pointer is a DEVICE pointer owned by the caller unless it is one
 *     of the two layer descriptor structs, which are HOST structs holding
 *     device pointers.  The library allocates nothing and frees nothing.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No entry point synchronises.
 *   - All matrices are row-major and "unit-major": row j is the vector of
 *     hidden unit / class j (u_j, v_j or the class row).  bf16 is the usual
 *     upper half of an IEEE binary32.
 *   - Weight matrices, packed int4 blobs and the workspace must be 256-byte
 *     aligned; x and the outputs 16-byte aligned.
 *   - Return value: HIRE_OK, or a negative code.  Argument errors are found
 *     on the host before anything is enqueued.  Errors inside a kernel
 *     (e.g. a NaN input, which is unsupported) are not reported.
 *   - Calls that share a workspace must be ordered on one stream.
 *   - Ties are always broken toward the lower index; -0.0 ranks as +0.0.
 *
 * Testing and measurement aids (stage events, route switches, counters of the slower exact routes, the inverse of
 * the int4 packing, a calibration copy) are declared in hire_debug.h and are not part of the product interface.
 */
#ifndef HIRE_H
#define HIRE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HIRE_OK 0
#define HIRE_EINVAL (-1)       /* bad shape, k > k', k' > N, B out of range, null or misaligned pointer */
#define HIRE_ENOSPC (-2)       /* workspace smaller than hire_*_workspace_bytes reports */
#define HIRE_EUNSUPPORTED (-3) /* a combination this build does not implement */
#define HIRE_ELAUNCH (-4)      /* the HIP runtime refused a launch */

#define HIRE_SCORER_INT4 0    /* HiRE-Q, Sec. 3.2 */
#define HIRE_SCORER_LOWRANK 1 /* HiRE-LR, Sec. 3.2 */
#define HIRE_SCORER_LRQ 2     /* HiRE-LRQ, Sec. 4.1: the low-rank factors themselves in int4.  The paper gives no
                                 detail; here the scorer is two chained HiRE-Q products:
                                   xq = int8(x);  t_p = float(sum_i q1[p,i] xq[i]) * s1[p], stored as bf16;
                                   tq = int8(t);  key_j = phi(float(sum_p q2[j,p] tq[p]) * s2[j])
                                 with q1/s1 the int4 copy of Z1 transposed ([r, d_model] rows) and q2/s2 that of
                                 Z2 ([rows, r]); both per-token scales are positive constants and are left out. */

/* topk_select flags */
#define HIRE_RELU 1        /* rank max(score, 0) instead of score */
#define HIRE_ORDER_RANK 2  /* output by (value descending, index ascending); default: ascending index */

#define HIRE_MAX_BATCH 64
#define HIRE_MAX_RANK_ORDER_K 4096 /* largest k that HIRE_ORDER_RANK / the softmax step sort */

/* One FFN layer (eq. (3)/(4): FF(x) = sum_j relu(<u_j,x>) v_j), unit-major. */
typedef struct hire_ffn_layer {
  int d_model;            /* d; multiple of 32 (int4 scorer) and of 8 */
  int d_ff;               /* m = number of hidden units */
  const void* w1u;        /* bf16 [d_ff, d_model], row j = u_j */
  const void* w2u;        /* bf16 [d_ff, d_model], row j = v_j */
  int scorer_kind;        /* HIRE_SCORER_INT4, HIRE_SCORER_LOWRANK or HIRE_SCORER_LRQ */
  const void* q4;         /* INT4: blob written by hire_pack_int4 for w1u */
  const float* q4_scale;  /* INT4: fp32 [d_ff] row scales from hire_pack_int4 */
  const void* lr_a;       /* LOWRANK: Z1, bf16 [d_model, r].  LRQ: blob written by hire_pack_int4 for Z1
                             transposed (rows = r, cols = d_model), 256-byte aligned */
  const void* lr_b;       /* LOWRANK: Z2, bf16 [d_ff, r] (row j = unit j's r-vector).  LRQ: blob written by
                             hire_pack_int4 for Z2 (rows = d_ff, cols = r) */
  int r;                  /* LOWRANK: rank, multiple of 8, <= 1024.  LRQ: multiple of 32, <= 1024 */
  const float* lr_a_scale; /* LRQ: fp32 [r] row scales of lr_a; otherwise unused */
  const float* lr_b_scale; /* LRQ: fp32 [d_ff] row scales of lr_b; otherwise unused */
  const float* row_norm_bounds; /* LOWRANK and LRQ, optional (may be NULL): DEVICE fp32 [2] written by hire_lr_prepare
                             for this layer.  With it a batch-1 step of a layer of at most 16384 units takes the same
                             short kernel sequence as with the int4 scorer; the results do not depend on it. */
} hire_ffn_layer;

/* The classifier of eq. (1): logits = W x, one row per class. */
typedef struct hire_softmax_layer {
  int d_model;
  int vocab;              /* c */
  const void* w;          /* bf16 [vocab, d_model] */
  int scorer_kind;
  const void* q4;
  const float* q4_scale;  /* fp32 [vocab] */
  const void* lr_a;       /* bf16 [d_model, r]; LRQ: int4 blob of Z1 transposed, as in hire_ffn_layer */
  const void* lr_b;       /* bf16 [vocab, r]; LRQ: int4 blob of Z2 */
  int r;
  const float* lr_a_scale; /* LRQ: fp32 [r] */
  const float* lr_b_scale; /* LRQ: fp32 [vocab] */
} hire_softmax_layer;

/* Library version (major*10000 + minor*100 + patch). */
int hire_version(void);

/* Static text for a return code. */
const char* hire_strerror(int code);

/* Text of the HIP runtime error behind the calling thread's most recent HIRE_ELAUNCH. */
const char* hire_last_launch_error(void);

/* HiRE-Q preparation (Sec. 3.2: Zapprox is an int4 copy of Z; the paper names
 * no quantiser, this one is symmetric with one scale per row).
 * For every row j of w_bf16 [rows, cols]: amax = max|w_ji|, scale_j = amax/7
 * (fp32 division; 1 if the row is all zero), code_ji = clamp(rint(w_ji /
 * scale_j), -7, 7) with fp32 division and round-half-even.  The codes are
 * written to q4_out in the library's packed layout (hire_pack_int4_bytes
 * bytes, opaque: the codes, then a short trailer that holds the largest row
 * scale, from which the batch-1 FFN step bounds its scorer keys), scales to
 * scale_out [rows].  cols must be a multiple of 32.  A blob must be passed to
 * the steps whole and unchanged.  Not part of the timed step. */
size_t hire_pack_int4_bytes(int rows, int cols);
int hire_pack_int4(const void* w_bf16, int rows, int cols, void* q4_out, float* scale_out, void* stream);

/* HiRE-LR / HiRE-LRQ preparation (Sec. 3.2), optional and not part of the timed step: bounds2_out (DEVICE fp32 [2])
 * receives upper bounds of the largest row norm of L->w1u and (LOWRANK; 0 for LRQ, whose int4 copy of Z2 carries its
 * own bound) of L->lr_b (fp32 sums of squares, rounded up by more than their error).  Cauchy-Schwarz with the norms of the token and of Z1^T x then bounds every activation and every scorer
 * key of a step before it is computed, which the batch-1 kernels use to place their histograms.  L must be a
 * HIRE_SCORER_LOWRANK or HIRE_SCORER_LRQ layer; its row_norm_bounds field is not read here.  The values must be recomputed when
 * w1u or lr_b change.  Returns HIRE_EINVAL for a NULL or misaligned argument or another scorer kind. */
int hire_lr_prepare(const hire_ffn_layer* L, float* bounds2_out, void* stream);

/* Must be called once on a workspace after its memory was allocated (or reused for anything else) and before
 * the first step that uses it: clears the marker at the head of the workspace that tells the batch-1 FFN
 * kernels whether their key histogram is in the clean state the previous step left.  Steps keep that state
 * consistent among themselves afterwards. */
int hire_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* Workspace sizes in bytes for one step with the given batch / k / k'.  0 when the sizes are invalid (B outside
 * 1..HIRE_MAX_BATCH, k < 1, k > k', k' beyond the rows); the layer's pointers and its scorer's rank are checked by the
 * step itself, which returns HIRE_EINVAL for them whatever workspace it is given. */
size_t hire_ffn_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime);
size_t hire_softmax_workspace_bytes(const hire_softmax_layer* L, int B, int k, int kprime);
size_t hire_topk_workspace_bytes(int B, int N, int k, int flags);

/* HiRE-FFN decode step for B tokens (Sec. 3.4 + Algorithm 1 + Sec. 3.4.1 + eq. (4)):
 *   1. scorer keys relu(Zapprox^T x_b) for all d_ff units
 *        INT4:    x_b -> int8 per token (scale amax/127), integer dot with the
 *                 int4 codes (int32, exact), key = float(acc) * scale_j (one
 *                 fp32 multiply), relu
 *        LOWRANK: t = Z1^T x_b rounded to bf16, key = relu(<Z2[j,:], t>)
 *        LRQ:     the two chained int4 products described at HIRE_SCORER_LRQ
 *   2. S'_b = the k' largest keys of token b; U = union over b, ascending
 *   3. h[b,j] = relu(<u_j, x_b>) for j in U (bf16 inputs, wide accumulation)
 *   4. S_b = the k largest h[b,.] over U
 *   5. y_b = sum_{j in S_b} h[b,j] v_j
 * x: bf16 [B, d_model].  y: fp32 [B, d_model].
 * Optional outputs (NULL to skip): topk_idx int32 [B,k] = S_b ascending;
 * topk_val fp32 [B,k] = h in the same order; cand_idx int32 [min(B*k', d_ff)]
 * = U ascending (entries past |U| are left untouched); n_cand = |U| (one
 * int32); scorer_acc int32 [B, d_ff] = the integer scores (INT4 only).
 * Requires 1 <= k <= k' <= d_ff, 1 <= B <= HIRE_MAX_BATCH. */
int hire_ffn_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, float* y, int32_t* topk_idx,
                  float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc, void* workspace,
                  size_t workspace_bytes, void* stream);

/* hire_ffn_step for callers that cannot allocate device memory or hand over a workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same computation with the same
 * arguments, outputs and errors as hire_ffn_step, except that the scratch memory is a statically allocated device
 * array inside the library (HIRE_STATIC_SCRATCH_BYTES, one per GPU the library runs on, held until the process
 * ends) instead of the caller's workspace.  The call allocates and frees nothing, on the host or on the device.
 *   - Steps that would need a larger workspace (hire_ffn_workspace_bytes(L, B, k, kprime) beyond
 *     HIRE_STATIC_SCRATCH_BYTES; the ~1B layer shape fits up to batch 16) return HIRE_ENOSPC, nothing enqueued.
 *   - The array belongs to the device that is current when the call is made; its address is looked up on the
 *     first call on that device (no work is enqueued for that, but make that first call outside a capture).
 *   - All calls on one GPU share that GPU's array, which keeps what the last call left there (the steps keep it
 *     consistent among themselves, as they do with a workspace).  Calls that overlap in time on one GPU, on
 *     different streams or from different threads, race on it: order them on one stream. */
#define HIRE_STATIC_SCRATCH_BYTES (8u << 20)
int hire_ffn_step_static(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, float* y, int32_t* topk_idx,
                         float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc, void* stream);

/* Group-sparse HiRE-FFN decode step (Sec. 3.4, eq. (6), with Algorithm 1 and Sec. 3.4.1): the d_ff hidden units
 * form d_ff/group groups of `group` adjacent units, and whole groups are shortlisted, selected and used.  k and k'
 * still count units: k'/group groups are shortlisted per token and k/group survive.
 *   1. scorer keys as in hire_ffn_step; Phi[b,J] = sum_{l<group} |key[b, group*J + l]|, added in unit order in the
 *      keys' own precision (fp32 for INT4, fp64 for LOWRANK)
 *   2. S'_b = the k'/group groups with the largest Phi[b,.]; U = their union over the batch, ascending
 *   3. h[b,j] = relu(<u_j, x_b>) for every unit j of every group in U
 *   4. E[b,J] = sum_l |h[b, group*J + l]|;  S_b = the k/group groups of U with the largest E[b,.]
 *   5. y_b = sum_{J in S_b} sum_{l<group} h[b, group*J + l] v_{group*J + l}
 * Ties go to the lower group index.  group is 1, 2, 4, 8 or 16 and divides d_ff, k and k'; d_ff/group <= 32768
 * (otherwise HIRE_EUNSUPPORTED).  group = 1 computes what hire_ffn_step computes.
 * Optional outputs (NULL to skip): topk_group int32 [B, k/group] = S_b ascending; topk_val fp32 [B, k] = h of the
 * units of those groups, group by group in the same order; cand_group int32 [min(B*k'/group, d_ff/group)] = U
 * ascending; n_cand = |U| in groups; scorer_acc int32 [B, d_ff] (INT4 only).
 * workspace: hire_ffn_group_workspace_bytes(L, B, k, kprime, group) bytes (0 on invalid arguments), 256-byte
 * aligned, passed through hire_workspace_init once.  Errors as for hire_ffn_step. */
size_t hire_ffn_group_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime, int group);
int hire_ffn_group_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, int group, float* y,
                        int32_t* topk_group, float* topk_val, int32_t* cand_group, int32_t* n_cand,
                        int32_t* scorer_acc, void* workspace, size_t workspace_bytes, void* stream);

/* CommonPath FFN decode step (Sec. 3.4.1, static overlap, eq. (7)): m1 hidden units that every token uses, as in a
 * dense layer, next to the group-sparse HiRE step on the layer's other d_ff units:
 *   y_b = sum_{j<m1} relu(<u^d_j, x_b>) v^d_j  +  (y_b of hire_ffn_group_step on L)
 * dense_w1u, dense_w2u: bf16 [m1, d_model], row j = u^d_j, v^d_j, 256-byte aligned (ignored when m1 = 0, which
 * makes this hire_ffn_group_step).  All other arguments, the optional outputs (indices count inside L's units) and
 * the errors as for hire_ffn_group_step.  workspace: hire_ffn_commonpath_workspace_bytes(...) bytes (0 on invalid
 * arguments), 256-byte aligned, passed through hire_workspace_init once. */
size_t hire_ffn_commonpath_workspace_bytes(const hire_ffn_layer* L, int m1, int B, int k, int kprime, int group);
int hire_ffn_commonpath_step(const hire_ffn_layer* L, const void* dense_w1u, const void* dense_w2u, int m1,
                             const void* x, int B, int k, int kprime, int group, float* y, int32_t* topk_group,
                             float* topk_val, int32_t* cand_group, int32_t* n_cand, int32_t* scorer_acc,
                             void* workspace, size_t workspace_bytes, void* stream);

/* HiRE-FFN decode step with the distributed approximate top-k of Algorithm 2 (DA-TOP-k), every "machine" of the
 * algorithm being a part of this one GPU: the d_ff hidden units are cut into `shards` contiguous shards of
 * d_ff/shards units, and shard i runs steps 1-5 of hire_ffn_step on its own units with the quotas
 * q' = ceil(k'/shards) and q = ceil(k/shards) (Algorithm 2 rounds a quota that does not divide up, so the step then
 * keeps shards*q >= k units per token; per-shard candidate union across the batch); y_b is the sum of the shards'
 * contributions.  The result is not that of hire_ffn_step unless shards = 1: no threshold is agreed on across shards.
 * INT4 scorer only.  shards divides d_ff (else HIRE_EINVAL); d_ff/shards <= 1024 and d_model <= 8192 (else
 * HIRE_EUNSUPPORTED; 256 shards suit d_ff = 16384).
 * Optional outputs (NULL to skip): topk_idx int32 [B, shards*q]: shard after shard, q ascending unit indices each
 * (hence ascending overall); topk_val fp32 [B, shards*q] same order; cand_idx int32 [shards, cap], cap =
 * min(B*q', d_ff/shards): row i holds shard i's candidate union ascending, n_cand[i] entries valid;
 * n_cand int32 [shards]; scorer_acc int32 [B, d_ff].
 * workspace: hire_ffn_shard_workspace_bytes(...) bytes (0 on invalid or unsupported arguments), 256-byte aligned;
 * no initialisation needed, and hire_workspace_init does no harm. */
size_t hire_ffn_shard_workspace_bytes(const hire_ffn_layer* L, int B, int k, int kprime, int shards);
int hire_ffn_shard_step(const hire_ffn_layer* L, const void* x, int B, int k, int kprime, int shards, float* y,
                        int32_t* topk_idx, float* topk_val, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc,
                        void* workspace, size_t workspace_bytes, void* stream);

/* HiRE-Softmax decode step (Sec. 3.3 + Algorithm 1 with phi = identity + eq. (2)):
 * steps 1-3 as above with signed keys and logits z[b,j] = <w_j, x_b>; then the
 * k largest logits of each token in rank order and the softmax over those k
 * (eq. (2): renormalising the top-k of the full softmax equals the softmax of
 * the top-k logits).
 * top_idx int32 [B,k] (logit descending, index ascending), top_prob fp32
 * [B,k]; optional top_logit fp32 [B,k], cand_idx [min(B*k', vocab)], n_cand,
 * scorer_acc int32 [B, vocab].  Requires k <= HIRE_MAX_RANK_ORDER_K. */
int hire_softmax_step(const hire_softmax_layer* L, const void* x, int B, int k, int kprime, int32_t* top_idx,
                      float* top_prob, float* top_logit, int32_t* cand_idx, int32_t* n_cand, int32_t* scorer_acc,
                      void* workspace, size_t workspace_bytes, void* stream);

/* TopInd_k / Top_k of Sec. 3.1 on a batch of score rows: for each of the B
 * rows of scores fp32 [B, N] the indices of the k largest entries (after
 * max(.,0) if HIRE_RELU), ties to the lower index.  idx_out int32 [B,k] in
 * ascending index order, or in rank order with HIRE_ORDER_RANK (then k <=
 * HIRE_MAX_RANK_ORDER_K); val_out (optional) fp32 [B,k] the ranked values in
 * the same order.  Requires 1 <= k <= N, B >= 1.  workspace: hire_topk_workspace_bytes(B, N, k, flags) bytes,
 * 256-byte aligned, passed through hire_workspace_init once: rows longer than 32768 are selected by many
 * workgroups per row through histograms kept there (HIRE_ENOSPC if it is smaller), and for rank order the k
 * survivors, staged there in index order, are then ranked; shorter rows use one workgroup per row and no
 * workspace memory. */
int topk_select(const float* scores, int B, int N, int k, int flags, int32_t* idx_out, float* val_out,
                void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HIRE_H */
