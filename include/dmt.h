/*
 * dmt.h - C ABI of libdmt: one GPU's share of the tower-decomposed sparse step
 * of Disaggregated Multi-Tower (DMT, arXiv 2403.00877), for AMD MI355X (gfx950).
 *
 * The library runs three operations, each as hand-written HIP kernels:
 *   dmt_tower_lookup_fwd         tower-local sum-pooled embedding lookup whose
 *                                store already has the layout SPTT's steps c-e
 *                                produce (paper Sec. 2.2 step b, Sec. 3.1.1)
 *   dmt_tower_module_fwd         the per-tower Tower Module that shrinks that
 *                                payload (paper Sec. 3.2, Sec. 4 Listings 1-2)
 *   dmt_tower_lookup_bwd_update  gradients to the activated rows only (paper
 *                                Sec. 2.2): stable sort by row id, segment
 *                                reduce, one deterministic rowwise-Adagrad
 *                                write per row
 * and, between the last two in a training step,
 *   dmt_tower_module_fwd_keep    the same forward, keeping what its backward needs
 *   dmt_tower_module_bwd         the Tower Module's backward, whose dL/d(pooled)
 *                                is what dmt_tower_lookup_bwd_update consumes
 * Beside the step, the Tower Partitioner that decides which table goes to which
 * tower (paper Sec. 3.3):
 *   dmt_tp_interaction           feature interaction matrix of a batch of pooled
 *                                embeddings (device)
 *   dmt_tp_embed, dmt_tp_kmeans  distance embedding by Adam and constrained
 *                                K-means (host; they touch |F| x |F| numbers)
 * and SPTT's data-shuffle steps c and e in explicit form (paper Sec. 3.1.1):
 *   dmt_sptt_peer_permute, dmt_sptt_shuffle   block transposes in device memory
 *   dmt_sptt_peer_permute_ids    step c moved in front of step b (paper Sec.
 *                                3.1.3): the same permute on the jagged ids
 * For callers that can neither allocate nor hand over a workspace:
 *   dmt_tower_lookup_bwd_update_noalloc   the update on a scratch array that
 *                                lives inside the library
 *
 * Conventions
 *  - C linkage, no exceptions cross the boundary; every call returns dmt_status.
 *  - "dev" pointers are device memory owned by the CALLER (e.g. PyTorch
 *    tensors); "host" pointers are ordinary host memory, read during the call
 *    only.  The library owns nothing but the plan object and the small device
 *    tables dmt_plan_bind creates.
 *  - The dmt_tower_* calls validate on the host first (null pointers,
 *    sizes against the plan, supported dtypes / widths) and return
 *    DMT_EINVAL / DMT_ENOTSUP without launching anything; then they enqueue
 *    kernels on `stream` (a hipStream_t, NULL = default stream) and return
 *    without synchronising and without allocating device memory.  Scratch
 *    memory is the caller's `workspace`, sized by the dmt_*_workspace_bytes
 *    functions.  (The Tower Module calls build short descriptor lists on the
 *    host; if that allocation fails they return DMT_ENOMEM.)
 *  - Ids out of range [0, rows_f) are never dereferenced: the kernels skip them
 *    and record the smallest offending position; dmt_last_device_error
 *    synchronises the stream and reports it as DMT_EBOUNDS.  Offsets that do
 *    not tile [0, nnz) make the update touch no row at all; the same call
 *    reports them as DMT_EINVAL with the first offending bag.
 *  - Enumerations are passed by value as int32_t, so that a value outside the
 *    enumeration reaches the library's own check.
 *  - Jagged input is feature-major CSR: bag (f, b) of table f and sample b owns
 *    indices[offsets[f*B + b] .. offsets[f*B + b + 1]); offsets has
 *    num_tables*B + 1 entries, offsets[0] = 0, offsets[num_tables*B] = nnz.
 *  - Tower-major pooled layout: towers one after another, each a row-major
 *    [B][W_t] block, W_t = sum of the dims of the tower's tables; inside a row
 *    the tables appear in ascending table id.  With equal dims N this is the
 *    paper's `embs` of shape (B, |F|, N) per tower (Sec. 4).
 *  - Calls that share a plan, a workspace or tables must be ordered by the
 *    caller (same stream, or events).
 */
#ifndef DMT_H_
#define DMT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DMT_OK = 0,
  DMT_EINVAL = 1,   /* bad argument (null, negative, exceeds the plan's maxima) */
  DMT_ENOTSUP = 2,  /* valid but not supported by these kernels                 */
  DMT_EBOUNDS = 3,  /* an id outside its table was seen on the device           */
  DMT_ENOMEM = 4,   /* host allocation failed / workspace too small             */
  DMT_EHIP = 5      /* a HIP runtime call failed                                */
} dmt_status;

/* Element types.  Across the boundary a type (like every other enumeration here) travels as
 * an int32_t holding one of these values, so that a value outside the list is an argument the
 * call can reject (DMT_EINVAL) instead of an invalid enum object. */
typedef enum { DMT_F32 = 0, DMT_F16 = 1, DMT_BF16 = 2 } dmt_dtype;

typedef enum {
  DMT_TM_LINEAR = 0,       /* y = W x + b            (Listing 1 with c = 0)                      */
  DMT_TM_LINEAR_RELU = 1,  /* y = max(0, W x + b)                                                 */
  DMT_TM_DOT_LINEAR = 2,   /* z = [pairwise dots (i<j) | x], y = W z + b  (Sec. 3.2, Sec. 4)      */
  DMT_TM_CROSS_LINEAR = 3, /* x_{l+1} = x0 * (W_l x_l + b_l) + x_l, y = W x_L + b  (Listing 2)    */
  DMT_TM_DLRM = 4,         /* y = [W x + b | W_f x_0 + b_f | ... | W_f x_{F-1} + b_f]: the flat
                              projection next to ONE projection shared by every feature's
                              embedding x_f  (Listing 1 with c > 0)                                */
  DMT_TM_CROSS_LOWRANK_LINEAR = 5 /* x_{l+1} = x0 * (U_l (V_l x_l) + b_l) + x_l, y = W x_L + b:
                              Listing 2 with DCN-v2's low-rank cross layer                         */
} dmt_tm_kind;

#define DMT_MAX_CROSS_LAYERS 4
#define DMT_MAX_TOWERS 64
#define DMT_MAX_TABLES 4096

typedef struct dmt_plan dmt_plan; /* opaque, library-owned */

/* Human-readable name of a status code (static string). */
const char* dmt_status_str(int32_t status);

/*
 * Describe the model's sparse side (paper Sec. 2.1: one table per sparse
 * feature; Sec. 3.1: features pre-partitioned into towers).  Host-only: no
 * device is touched.
 *   rows, dims       host [num_tables]: rows and embedding dim of each table.
 *                    dims[f] * sizeof(element) must be a multiple of 16 bytes
 *                    and at most 1024 bytes.
 *   table_dtype      element type of every table.
 *   table_to_tower   host [num_tables], values in [0, num_towers); every tower
 *                    needs at least one table.  A table's slot inside its tower
 *                    is its rank among the tower's tables by ascending id.
 *   max_batch, max_nnz  upper bounds later calls are checked against.
 * The sum of all rows must stay below 2^31 (rows are numbered globally inside
 * the backward sort, in 31 bits of a 32-bit key).
 */
dmt_status dmt_plan_create(dmt_plan** out, int32_t num_tables, const int64_t* rows,
                           const int32_t* dims, int32_t table_dtype, int32_t num_towers,
                           const int32_t* table_to_tower, int64_t max_batch, int64_t max_nnz);

void dmt_plan_destroy(dmt_plan* plan);

/*
 * Element offsets of the tower-major pooled tensor for batch size B (host-only):
 *   tower_base  host out [num_towers + 1]: first element of each tower's block;
 *               tower_base[num_towers] is the tensor's total element count
 *   tower_width host out [num_towers]: W_t
 *   col_off     host out [num_tables]: first column of each table inside its
 *               tower's rows
 * Any output pointer may be NULL.
 */
dmt_status dmt_plan_layout(const dmt_plan* plan, int64_t B, int64_t* tower_base,
                           int32_t* tower_width, int32_t* col_off);

/*
 * Attach the tables (and optionally the optimizer state) and upload the plan's
 * small lookup tables to the current device.  Synchronous; call once before
 * the dmt_tower_* calls and again whenever a pointer changes.
 *   tables  host [num_tables] of dev pointers; table f is row-major
 *           [rows[f]][dims[f]] of table_dtype, 16-byte aligned, row stride
 *           dims[f] elements.
 *   adagrad_state  host [num_tables] of dev float pointers ([rows[f]] each), or
 *           NULL when the backward is not used.
 */
dmt_status dmt_plan_bind(dmt_plan* plan, const void* const* tables, float* const* adagrad_state);

/*
 * Row-wise shards (paper Sec. 3.1.3: a table too large for one GPU is split by rows inside
 * its tower, and step d becomes a ReduceScatter that adds the shards' partial pools).  After
 * this call table f of the plan stands for rows [row_begin[f], row_begin[f] + rows[f]) of a
 * larger table: `indices` keep carrying ids of the whole table, ids outside the local rows
 * belong to other shards and are skipped without being reported, dmt_tower_lookup_fwd writes
 * the PARTIAL pool of the local rows (the caller's reduction over the shards gives the pooled
 * embedding), and dmt_tower_lookup_bwd_update updates the local rows only, each exactly as
 * the unsharded table's row would be.
 *   row_begin   host [num_tables], >= 0, row_begin[f] + rows[f] <= 2^31
 * May be called before or after dmt_plan_bind (it synchronises then); not while kernels of
 * this plan are in flight.
 */
dmt_status dmt_plan_set_row_shards(dmt_plan* plan, const int64_t* row_begin);

/*
 * Tower-local pooled lookup, forward (paper Sec. 2.2 step b with the layout of
 * Sec. 3.1.1 steps c-e fused into the store).
 *   pooled_out[tower_base[t] + b*W_t + col_off[f] + d]
 *        = sum over j in bag (f, b) of table_f[indices[j]][d]
 * accumulated in float32, rounded once to out_dtype.  An empty bag gives
 * zeros; an id occurring twice in a bag is added twice.
 *   indices  dev int32 [nnz]; offsets dev int64 [num_tables*B + 1]
 *   pooled_out dev, tower_base[num_towers] elements of out_dtype, 16-byte aligned
 */
dmt_status dmt_tower_lookup_fwd(const dmt_plan* plan, const int32_t* indices,
                                const int64_t* offsets, int64_t B, int64_t nnz,
                                void* pooled_out, int32_t out_dtype, void* stream);

/*
 * Per-tower Tower-Module parameters (paper Sec. 4).  All weights are dev
 * pointers of the dtype passed to dmt_tower_module_fwd, row-major [out][in];
 * biases are dev [out] of the same dtype.
 *   LINEAR / LINEAR_RELU : w_proj [out_dim][W_t]
 *   DOT_LINEAR  : the tower's tables must share one dim n; with nf tables the
 *                 projection input is [nf(nf-1)/2 dots, (i,j) row-major, i<j |
 *                 the W_t pooled values]; w_proj [out_dim][nf(nf-1)/2 + W_t]
 *   CROSS_LINEAR: num_cross_layers full-rank layers w_cross[l] [W_t][W_t],
 *                 b_cross[l] [W_t], then w_proj [out_dim][W_t]
 *   DLRM        : the tower's nf tables must share one dim n.  feat_out = c D
 *                 outputs per feature from the shared layer w_cross[0] [feat_out][n],
 *                 b_cross[0] [feat_out]; the first out_dim - nf * feat_out (>= 1)
 *                 outputs from w_proj [out_dim - nf * feat_out][W_t], b_proj.
 *                 num_cross_layers is ignored.
 *   CROSS_LOWRANK_LINEAR: num_cross_layers <= DMT_MAX_CROSS_LAYERS / 2 layers of rank
 *                 feat_out = r (a multiple of 8 for the 16-bit types): w_cross[2 l] = V_l
 *                 [r][W_t], w_cross[2 l + 1] = U_l [W_t][r], b_cross[l] [W_t]; then
 *                 w_proj [out_dim][W_t]
 */
typedef struct {
  int32_t kind;              /* dmt_tm_kind */
  int32_t out_dim;           /* O_t */
  int32_t num_cross_layers;  /* CROSS_LINEAR (<= DMT_MAX_CROSS_LAYERS) and
                                CROSS_LOWRANK_LINEAR (half as many) only */
  int32_t feat_out;          /* DLRM: outputs of the per-feature layer (c D);
                                CROSS_LOWRANK_LINEAR: the rank r */
  const void* w_proj;
  const void* b_proj;
  const void* w_cross[DMT_MAX_CROSS_LAYERS];
  const void* b_cross[DMT_MAX_CROSS_LAYERS];
} dmt_tm_params;

/* Bytes of scratch dmt_tower_module_fwd needs for these towers at batch B
 * (0 is possible).  Host-only. */
size_t dmt_tm_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower, int64_t B);

/*
 * Tower Module forward (paper Sec. 3.2: D = TM(V) with |D| < |V|, applied to
 * what step e leaves on the GPU).  For every tower t:
 *   tm_out block t = TM_t(pooled block t), row-major [B][O_t], towers one after
 *   another (block t starts at element B * sum_{t' < t} O_t').
 * dtype is the type of pooled, weights, biases and tm_out alike: DMT_BF16 /
 * DMT_F16 run on MFMA with float32 accumulation (cross-layer intermediates are
 * kept in that 16-bit type); DMT_F32 runs in plain float32 arithmetic.
 *   per_tower  host [num_towers]
 *   workspace  dev, at least dmt_tm_workspace_bytes, 256-byte aligned (may be
 *              NULL when that is 0)
 */
dmt_status dmt_tower_module_fwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                const void* pooled, int64_t B, void* tm_out, int32_t dtype,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Training forward: dmt_tower_module_fwd that also keeps, in `kept`, what the
 * backward would otherwise recompute: x_{l+1} and u_l = W_l x_l + b_l of every
 * cross layer, full-rank or low-rank (paper Listing 2), each [B][W_t] in
 * `dtype`; the pairwise dot terms of a dot-product tower, [B][F_t (F_t - 1) / 2
 * rounded up to 8] in `dtype`, and its projection weights repacked to match
 * (so the weights must not change between this call and the backward).  tm_out is bit for bit that of
 * dmt_tower_module_fwd.  Towers of the other kinds keep nothing (their backward
 * needs only the pooled values).
 *   kept  dev, at least dmt_tm_kept_bytes(plan, per_tower, B, dtype), 256-byte
 *         aligned, caller-owned; pass the same buffer, unchanged, to
 *         dmt_tower_module_bwd.  May be NULL when that size is 0.
 */
size_t dmt_tm_kept_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower, int64_t B,
                         int32_t dtype);
dmt_status dmt_tower_module_fwd_keep(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                     const void* pooled, int64_t B, void* tm_out, int32_t dtype,
                                     void* kept, size_t kept_bytes, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * Parameter gradients of one tower's Tower Module, all dev float32, row-major,
 * shaped like the parameters themselves (dw_proj [O_t][K_t] with K_t the row
 * length of w_proj; dw_cross[l] [W_t][W_t]; the db_* vectors; for a DLRM tower
 * dw_proj has the flat layer's out_dim - nf * feat_out rows and dw_cross[0] /
 * db_cross[0] receive the shared per-feature layer's [feat_out][n] / [feat_out];
 * for a low-rank cross tower dw_cross[2 l] / dw_cross[2 l + 1] are dV_l / dU_l).
 * Every array is overwritten, not accumulated into.  Caller-owned.
 */
typedef struct {
  float* dw_proj;
  float* db_proj;
  float* dw_cross[DMT_MAX_CROSS_LAYERS];
  float* db_cross[DMT_MAX_CROSS_LAYERS];
} dmt_tm_grads;

/* Bytes of scratch dmt_tower_module_bwd needs for these towers at batch B.  Host-only. */
size_t dmt_tm_bwd_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower, int64_t B);

/*
 * Tower Module backward: the chain rule through the forms of paper Sec. 3.2 /
 * Sec. 4 (Listings 1 and 2), from dL/d(tm_out) to dL/d(pooled) and to the
 * gradients of every weight and bias.  grad_pooled is exactly what
 * dmt_tower_lookup_bwd_update consumes, so the two calls chain without a copy.
 *   linear(+ReLU)  dpre = grad_tm_out (where tm_out > 0 under ReLU);
 *                  grad_pooled = dpre W, dW = dpre^T x, db = sum_b dpre
 *   dot + linear   dz = dy W over z = [dot terms | x]; dW = dy^T z; the flat part
 *                  of dz passes to x and each term (i, j) adds dz_ij x_j to dx_i
 *                  and dz_ij x_i to dx_j
 *   DLRM           both layers are linear layers of their own: the shared per-feature
 *                  layer's gradients are sums over the batch and over the features,
 *                  and grad_pooled adds both paths
 *   cross + linear layers taken from the last to the first with
 *                  du_l = dx_{l+1} * x0, dx0 += dx_{l+1} * u_l, dW_l = du_l^T x_l,
 *                  db_l = sum_b du_l, dx_l = du_l W_l + dx_{l+1};
 *                  grad_pooled = dx_0 + dx0
 *   low-rank cross the same with t_l = V_l x_l, u_l = U_l t_l + b_l: dU_l = du_l^T t_l,
 *                  dt_l = du_l U_l, dV_l = dt_l^T x_l, dx_l = dt_l V_l + dx_{l+1}
 * The forward's intermediates are recomputed (dot terms; u_l and x_l of the cross
 * layers) unless `kept` hands over what dmt_tower_module_fwd_keep stored for
 * the same plan, towers, B and dtype.
 * For DMT_BF16 / DMT_F16 every contraction runs on MFMA with float32
 * accumulation over operands rounded once to that 16-bit type (dpre, du_l, u_l,
 * x_l); gradients between layers and all outputs stay float32.  Bias gradients
 * are fixed-order sums of those rounded operands, so results repeat bit for bit.
 * DMT_F32 runs in plain float32 arithmetic.
 *   per_tower    host [num_towers], as passed to the forward
 *   pooled       dev, the forward's input;  tm_out dev, the forward's output
 *                (read only by LINEAR_RELU towers, may be NULL when there are none)
 *   grad_tm_out  dev float32, laid out like tm_out
 *   grad_pooled  dev float32 out, tower-major like pooled, 16-byte aligned
 *   grads        host [num_towers]; entries a tower's kind does not have are ignored
 *   kept         NULL, or dev as filled by dmt_tower_module_fwd_keep (kept_bytes its size)
 *   workspace    dev, at least dmt_tm_bwd_workspace_bytes (which assumes kept = NULL;
 *                less is used with it), 256-byte aligned
 */
dmt_status dmt_tower_module_bwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                const void* pooled, const void* tm_out, int64_t B,
                                const float* grad_tm_out, int32_t dtype, float* grad_pooled,
                                const dmt_tm_grads* grads, const void* kept, size_t kept_bytes,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Optional outputs of the backward's integer stages, for parity checks.  Any
 * pointer may be NULL.  All dev.  A lookup whose id is outside its table sorts
 * behind its table's valid lookups, shows as key -1 in sorted_keys, starts no run
 * (it lies inside the extent of the run before it) and is not counted. */
typedef struct {
  int64_t* sorted_keys;  /* [nnz]  (table << 32 | row), ascending, stable           */
  int32_t* sorted_bag;   /* [nnz]  bag id f*B + b of each sorted lookup              */
  int64_t* unique_keys;  /* [nnz]  first num_unique entries valid                    */
  int64_t* seg_off;      /* [nnz + 1] run starts; seg_off[num_unique] = nnz          */
  int64_t* num_unique;   /* [1]                                                      */
} dmt_bwd_debug;

/* Bytes of scratch dmt_tower_lookup_bwd_update needs for (B, nnz).  Host-only. */
size_t dmt_bwd_workspace_bytes(const dmt_plan* plan, int64_t B, int64_t nnz);

/*
 * Backward of the pooled lookup fused with a rowwise-Adagrad step on the
 * activated rows (paper Sec. 2.2: only the rows a batch touched receive
 * gradients).  For every distinct (table f, row r) among the lookups:
 *   G      = sum over all lookups of (f, r) of grad_pooled[bag's slice]   (float32,
 *            fixed order: ascending bag, so results repeat bit for bit)
 *   state[f][r] += mean_d(G[d]^2)
 *   table_f[r][d] -= lr * G[d] / (sqrt(state[f][r]) + eps)   (rounded once to the
 *            table dtype, one writer per row, no atomics)
 * Rows no lookup touched, and their states, are not written.
 * `offsets` must tile [0, nnz): offsets[0] = 0, ascending, offsets[num_tables*B] = nnz.  This
 * is checked on the device; when it does not hold no row and no state is written and
 * dmt_last_device_error returns DMT_EINVAL.
 *   grad_pooled  dev float32, tower-major like pooled_out
 *   workspace    dev, at least dmt_bwd_workspace_bytes(plan, B, nnz), 256-byte aligned
 *   dbg          NULL or where to export the sorted / deduplicated keys
 * Requires dmt_plan_bind with a non-NULL adagrad_state.
 */
dmt_status dmt_tower_lookup_bwd_update(const dmt_plan* plan, const int32_t* indices,
                                       const int64_t* offsets, int64_t B, int64_t nnz,
                                       const float* grad_pooled, float lr, float eps,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       const dmt_bwd_debug* dbg);

/*
 * dmt_tower_lookup_bwd_update for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving / training loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical table and state updates,
 * but the scratch memory is an array of DMT_BWD_NOALLOC_SCRATCH_BYTES bytes inside the library
 * (one copy on every GPU the library runs on, held until the process ends) and there are no
 * parity exports.  The call allocates nothing on host or device; the first call on a device
 * looks up the array's address there.
 *   DMT_ENOMEM  dmt_bwd_workspace_bytes(plan, B, nnz) exceeds the array (about 28 bytes per
 *               lookup at dim 128: roughly 1.1 million lookups); nothing is launched
 * All calls on one GPU share that GPU's array, whatever their plan or stream: calls that
 * overlap in time on one GPU race and must be ordered by the caller.  The array keeps the
 * previous call's contents; no kernel of the update reads scratch it has not written in the
 * same call, so nothing needs clearing between calls.
 */
#define DMT_BWD_NOALLOC_SCRATCH_BYTES (32u << 20)
size_t dmt_bwd_noalloc_scratch_bytes(void);
dmt_status dmt_tower_lookup_bwd_update_noalloc(const dmt_plan* plan, const int32_t* indices,
                                               const int64_t* offsets, int64_t B, int64_t nnz,
                                               const float* grad_pooled, float lr, float eps,
                                               void* stream);

/*
 * Tower Partitioner (paper Sec. 3.3): a balanced feature -> tower map learned from the
 * embeddings a model produces.  Three calls, one per stage; the caller moves the small
 * |F| x |F| matrix from the device to the host between the first and the second.
 *
 * Stage 1, on the device.  interaction[i][j] = | mean over the batch of the cosine between the
 * pooled embeddings of features i and j | (the cosine kernel on normalised embeddings, the
 * batch form mean(R R^T, dim = 0), then the absolute value).  A zero embedding has no
 * direction and counts as cosine 0.
 *   plan          any bound plan whose tables all have the same dim N, N % 8 == 0, N <= 512
 *                 (else DMT_ENOTSUP); typically one tower holding every table
 *   pooled        dev, the tower-major tensor dmt_tower_lookup_fwd wrote for this plan and B
 *   interaction   dev out, float32 [F][F] in table order, exactly symmetric
 *   workspace     dev, at least dmt_tp_workspace_bytes(plan, B), 16-byte aligned
 * 16-bit embeddings are contracted as they are (their products are exact in float32) and the
 * cosines formed in float32; float32 embeddings are normalised and rounded to float16 first,
 * so that an entry can differ from the exact value by up to 2^-10.
 */
size_t dmt_tp_workspace_bytes(const dmt_plan* plan, int64_t B);

dmt_status dmt_tp_interaction(const dmt_plan* plan, const void* pooled, int64_t B,
                              int32_t pooled_dtype, float* interaction, void* workspace,
                              size_t workspace_bytes, void* stream);

typedef enum {
  DMT_TP_DIVERSE = 0,   /* D = I: features that differ share a tower    */
  DMT_TP_COHERENT = 1   /* D = 1 - I: features that agree share a tower */
} dmt_tp_strategy;

/*
 * Stage 2, on the host, float64.  D = f(I) by `strategy`, then coordinates x_i in R^n that
 * minimise  sum over i, over j < i, of (||x_i - x_j||_2 - D(i, j))^2  by `steps` iterations of
 * Adam (beta1 0.9, beta2 0.999, epsilon 1e-8, bias-corrected) with step size lr from x0.
 * Only the entries of `interaction` below the diagonal are read.
 *   interaction   host, float32 [F][F]
 *   x0, x         host, float64 [F][n]: start (the method's random draw, supplied by the
 *                 caller) and result; may be the same buffer
 *   stress        host out or NULL: the objective at x
 */
dmt_status dmt_tp_embed(const float* interaction, int32_t F, int32_t strategy, int32_t n,
                        int32_t steps, double lr, const double* x0, double* x, double* stress);

/*
 * Stage 3, on the host, float64.  Constrained K-means (Bradley, Bennett and Demiriz 2000) of
 * the F points x into T groups: the assignment step is the minimum-cost assignment under
 * bounds on the group sizes, the update step moves every centre to its group's mean; it stops
 * when an assignment repeats, or after max_iter assignment steps.  The bounds make the
 * largest group at most `ratio` times the smallest: every group holds at least
 * smin = min(ceil(F / (T - 1 + ratio)), floor(F / T)) and at most
 * max(floor(ratio * smin), ceil(F / T)) points (ratio 1: sizes floor(F / T) and ceil(F / T)).
 *   centres0        host, float64 [T][n], the start centres (supplied by the caller)
 *   table_to_tower  host out, int32 [F]: group of each feature, usable as dmt_plan_create's map
 *   centres         host out [T][n] or NULL;  iterations  host out or NULL
 * DMT_EINVAL unless 1 <= T <= F, ratio >= 1, max_iter >= 1; DMT_ENOTSUP when T times the
 * upper size bound exceeds 4096 (the assignment step is cubic in it).
 */
dmt_status dmt_tp_kmeans(const double* x, int32_t F, int32_t n, int32_t T, double ratio,
                         const double* centres0, int32_t max_iter, int32_t* table_to_tower,
                         double* centres, int32_t* iterations);

/*
 * SPTT's data-shuffle steps inside one GPU's memory (paper Sec. 3.1.1, steps c and e), in
 * their explicit form.  (The training step above does not need them: dmt_tower_lookup_fwd
 * already stores in the layout they lead to.  They serve a deployment in which step d's
 * intra-host exchange runs between them.)  G ranks, L per host, T = G / L hosts.  A block is
 * `block_bytes` contiguous bytes (a multiple of 16): the embeddings of one feature for one
 * rank's samples.  `in` and `out` are dev, 16-byte aligned, distinct buffers of equal size.
 *
 * Peer order: all ranks sorted by (g % L, g / L), so that peers (ranks with equal g % L) are
 * adjacent and ordered by host; G = 4, L = 2 gives (0, 2, 1, 3).  (The walk-through prints the
 * key (g % T, g / L), which equals this one in its example, T = L = 2, and fails to bring
 * peers together otherwise.)  order: host out [G], order[k] = rank at position k.
 */
dmt_status dmt_sptt_peer_order(int32_t G, int32_t L, int32_t* order);

/* Step c, peer permute: in [features][G][block] in rank order -> out[f][k] = in[f][order[k]]. */
dmt_status dmt_sptt_peer_permute(const void* in, void* out, int64_t features, int32_t G, int32_t L,
                                 int64_t block_bytes, void* stream);

/*
 * Step c moved in front of step b (paper Sec. 3.1.3: steps b and c may be swapped so that the
 * shuffle acts on the smaller object): the peer permute on the sparse inputs.  `indices` /
 * `offsets` are a jagged batch as everywhere in this library, for `features` local features and
 * B = G * B_l samples, the samples of rank g being bags g * B_l .. (g + 1) * B_l - 1 of every
 * feature.  The output is the same batch with every feature's G blocks of B_l bags in peer
 * order (out block k of a feature = in block order[k]); a lookup on it yields, block for block,
 * what dmt_sptt_peer_permute makes of the lookup on the input.
 *   indices dev int32 [nnz], offsets dev int64 [features * G * B_l + 1] (tiling [0, nnz));
 *   out_indices / out_offsets dev, same sizes, distinct from the inputs
 * DMT_ENOTSUP for G > 1024 or features * G > 65535.  Offsets outside [0, nnz] are clamped: the
 * copies stay in bounds whatever they hold.
 */
dmt_status dmt_sptt_peer_permute_ids(const int32_t* indices, const int64_t* offsets,
                                     int64_t features, int32_t G, int32_t L, int64_t B_l,
                                     int64_t nnz, int32_t* out_indices, int64_t* out_offsets,
                                     void* stream);

/* Step e: in [features][peers][block] -> out [peers][features][block], i.e. the 2-D arrangement
 * (features, peers) transposed and flattened as (peers x features). */
dmt_status dmt_sptt_shuffle(const void* in, void* out, int64_t features, int64_t peers,
                            int64_t block_bytes, void* stream);

/*
 * Synchronise `stream` and report what the kernels since the last call found wrong with
 * their jagged input.  Clears the record.
 *   DMT_EINVAL   the backward saw `offsets` that do not tile [0, nnz) (first entry not 0, a
 *                descending pair, an entry outside [0, nnz], last entry not nnz);
 *                *bad_position = the first such bag.  That call updated no row.
 *   DMT_EBOUNDS  an id outside its table; *bad_position = smallest offending position in
 *                `indices`.  Such lookups were skipped, everything else was done.
 *   DMT_OK       neither; *bad_position = -1.
 */
dmt_status dmt_last_device_error(const dmt_plan* plan, void* stream, int64_t* bad_position);

/*
 * Kernel timing for benchmarks: HIP events recorded on the caller's stream
 * right before and after the launches of the selected kernel families.  Off by
 * default; the events cost about a microsecond each, so select only what is
 * being measured.
 */
typedef enum {
  DMT_K_LOOKUP_FWD = 0,        /* gather + pool + tower-major store           */
  DMT_K_TM_DOTS = 1,           /* pairwise dot terms                          */
  DMT_K_TM_PACK = 2,           /* projection-weight repack for the dot TM     */
  DMT_K_TM_GEMM = 3,           /* grouped contraction (cross layers, linears) */
  DMT_K_BWD_KEYS = 4,          /* key build                                   */
  DMT_K_BWD_SORT_HIST = 5,     /* radix pass: per-block digit histogram       */
  DMT_K_BWD_SORT_SCAN = 6,     /* radix pass: digit offsets                   */
  DMT_K_BWD_SORT_SCATTER = 7,  /* radix pass: stable scatter                  */
  DMT_K_BWD_HEADS = 8,         /* run heads -> segment offsets                */
  DMT_K_BWD_REDUCE_UPDATE = 9, /* segment reduce + rowwise Adagrad            */
  DMT_K_BWD_FIXUP = 10,        /* rows whose run spans reduce tiles           */
  DMT_K_TM_BWD_GEMM = 11,      /* Tower Module backward: grouped contractions */
  DMT_K_TM_BWD_AUX = 12,       /* ... its elementwise / transpose / sum steps */
  DMT_K_TP_GRAM = 13,          /* Tower Partitioner: normalise + Gram tiles   */
  DMT_K_TP_FINISH = 14,        /* ... slice sum, mean, absolute value         */
  DMT_K_COUNT = 15
} dmt_kernel_id;

const char* dmt_kernel_name(int32_t kernel_id);

/* Select the kernel families to time (bit i = dmt_kernel_id i); 0 turns timing
 * off.  Pending measurements are dropped. */
dmt_status dmt_profile_enable(dmt_plan* plan, uint32_t kernel_mask);

/* Synchronise `stream`, add up the event pairs recorded since the last read:
 * total_ms and launches are host out [DMT_K_COUNT]; then reset. */
dmt_status dmt_profile_read(dmt_plan* plan, void* stream, double* total_ms, int64_t* launches);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers
 * 16-byte aligned) by a grid-stride kernel named dmt_copy_kernel.  It exists so
 * that hardware byte counters can be calibrated against a kernel whose traffic
 * is known exactly: `bytes` read and `bytes` written.
 */
dmt_status dmt_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/*
 * Plain gather of n rows of `row_bytes` bytes (a power of two, 16 ... 1024) by id from a
 * row-major table of `rows` rows, by a kernel named dmt_gather_kernel that does nothing else
 * (eight row reads in flight per wave).  It exists so that the rate of the lookup and update
 * kernels, whose traffic is rows at random addresses, can be set against what such reads reach
 * on the machine at hand, from a table that fits the L2, the Infinity Cache, or neither.
 *   table dev [rows][row_bytes], 16-byte aligned; ids dev int32 [n] (an id outside [0, rows)
 *   reads row 0); out dev, DMT_CALIBRATION_GATHER_BLOCKS * 256 * 16 bytes, 16-byte aligned (one
 *   folded word per thread, written so that the reads cannot be optimised away).
 * Traffic: n * row_bytes bytes of rows and 4 n bytes of ids read.
 */
#define DMT_CALIBRATION_GATHER_BLOCKS 2048
dmt_status dmt_calibration_gather(const void* table, int64_t rows, int32_t row_bytes,
                                  const int32_t* ids, int64_t n, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DMT_H_ */
