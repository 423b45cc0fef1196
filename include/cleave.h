/*
 * cleave.h -- C ABI of the MI355X sub-GEMM task library.
 *
 * The library implements the compute path of Cleave's parameter-server
 * training scheme on one GPU:
 *
 *   plan     Task generation (paper Sec. 3.2 "Seamless training"; Sec. 4.1
 *            "Search space of GEMM"): a GEMM  O = op(A) . op(B)  with
 *            op(A) of size M x K and op(B) of size K x N is cut into row
 *            blocks of A and column blocks of B; one task is one (row block,
 *            column block) pair and produces the matching block of O.  The
 *            blocks cover O exactly once, without redundant work (Sec. 4.1,
 *            coverage constraint) and no task is empty (Sec. 4.1, zero-task
 *            constraint).  In addition the inner dimension is cut into S
 *            contiguous chunks ("K-split"), so a task is (tile, chunk) and
 *            yields a partial block; S = 1 is the paper's own case.
 *   execute  Sub-GEMM execution (Sec. 4.1, computation-cost term: a task
 *            costs 2 * m_len * n_len * k_len flops): every task reads its
 *            rows of op(A) and columns of op(B) and stores an fp32 partial
 *            block.  Re-executing a task (Sec. 4.2 churn recovery: lost
 *            shards are issued again) gives bitwise identical output.
 *   reduce   Parameter-server aggregation (Sec. 3.2: the PS aggregates the
 *            computed outputs): the S partial blocks of every tile are summed
 *            in ascending chunk order, ((P0 + P1) + P2) + ..., in fp32, and
 *            written into the full output C.
 *
 * Conventions
 *   - Every function returns CLEAVE_OK (0) or a negative cleave_status; no
 *     exception or abort crosses this boundary.  On error, output arguments
 *     are left untouched.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory of the current device, owned by the caller.  The library
 *     never allocates, frees or retains A, B, partials or C.
 *   - Matrices are row-major with a leading dimension in elements.
 *       transA = 0: A is stored M x K (lda >= K); transA = 1: A is stored
 *       K x M (lda >= M) and read as its transpose, without a copy.
 *       transB = 0: B is stored K x N (ldb >= N); transB = 1: B is stored
 *       N x K (ldb >= K).  (Forward X.W is (0,0); dX = dY.W^T is (0,1);
 *       dW = X^T.dY is (1,0).)
 *   - execute and reduce enqueue work on the given HIP stream (a hipStream_t
 *     passed as void*, NULL = the default stream) and return without waiting
 *     for it.  The first execute/reduce of a plan on a device uploads the
 *     plan's tables with a blocking copy and allocates everything later calls
 *     need (including the work-list memory of subset launches);
 *     cleave_plan_upload does that ahead of time.  After it, execute and
 *     reduce allocate nothing.
 */
#ifndef CLEAVE_H
#define CLEAVE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CLEAVE_OK = 0,
  CLEAVE_EINVAL = -1, /* bad size, edge list, split count, pointer, leading dimension, enum */
  CLEAVE_ENOMEM = -2, /* host or device allocation of plan tables failed */
  CLEAVE_EHIP = -3,   /* a HIP runtime call failed; see cleave_last_hip_error */
  CLEAVE_ELIMIT = -4  /* the request exceeds a fixed limit of the entry point */
} cleave_status;

typedef enum { CLEAVE_F32 = 0, CLEAVE_BF16 = 1 } cleave_dtype;

/* One sub-GEMM task: 64-byte POD, same bytes on host and device.
 * Ranges are half-open and refer to the logical op(A) . op(B). */
typedef struct {
  uint32_t gemm_id;      /* caller's label for the GEMM this plan belongs to */
  uint32_t tile_id;      /* index of the output tile, canonical order */
  uint32_t m0, m_len;    /* rows of op(A) / of the output tile */
  uint32_t n0, n_len;    /* columns of op(B) / of the output tile */
  uint32_t k0, k_len;    /* chunk of the inner dimension */
  uint32_t ksplit_idx;   /* s: which chunk */
  uint32_t ksplit_cnt;   /* S: chunks of this tile */
  uint64_t partial_off;  /* element offset of this task's m_len x n_len fp32 block */
  uint32_t flags;        /* 0 */
  uint32_t reserved[3];  /* 0 */
} cleave_task;

typedef struct cleave_plan cleave_plan; /* opaque, host-owned */

/* ---- plan --------------------------------------------------------------
 * Canonical task order: tile rows outermost, tile columns next, chunk index s
 * innermost; tile_id is the running tile index; partial_off is the running
 * sum of m_len*n_len, so a tile's S blocks are adjacent and each block is a
 * contiguous row-major m_len x n_len array.
 * Chunks: kc = ceil(K/S); chunk s = [s*kc, min((s+1)*kc, K)); a split with
 * (S-1)*kc >= K (an empty chunk) is CLEAVE_EINVAL.
 */

/* Uniform tiling: ceil(M/tile_m) x ceil(N/tile_n) tiles, the last row and
 * column of tiles clipped (never padded).  All arguments host values; *out is
 * a new plan the caller destroys with cleave_plan_destroy.
 * CLEAVE_EINVAL: a non-positive size, a dimension above 2^31-1, an empty
 * chunk, out == NULL, or a plan whose 32-bit indices would wrap (more than
 * 2^32-1 tasks, or a single tile of more than 2^32-1 128 x 128 sub-tiles). */
int cleave_plan_uniform(int64_t M, int64_t N, int64_t K, int64_t tile_m, int64_t tile_n,
                        int32_t ksplit, uint32_t gemm_id, cleave_plan** out);

/* Explicit (heterogeneous) tiling: n_bands row bands of heights band_h[b]
 * (sum M); band b is cut into n_cols[b] columns whose widths are listed
 * consecutively in col_w (each band's widths sum to N); ksplit_per_tile has
 * one S per tile in band-major order.  All arrays are host memory, read only
 * during the call.  CLEAVE_EINVAL as above, or lists that do not sum to M / N,
 * or an empty band / column. */
int cleave_plan_explicit(int64_t M, int64_t N, int64_t K, int32_t n_bands, const int64_t* band_h,
                         const int32_t* n_cols, const int64_t* col_w,
                         const int32_t* ksplit_per_tile, uint32_t gemm_id, cleave_plan** out);

/* A batch of n_batch independent GEMMs of one shape M x N x K in one task
 * list (paper Sec. 3.1, table of GEMM shapes: the attention-score products
 * Q K^T are 1024 x 128 x 1024, one per sequence and head, and share a DAG
 * level).  Member g contributes the uniform plan of a single GEMM with
 * gemm_id = g: tile ids restart at 0, partial offsets run on through the whole
 * list.  The plan is used with cleave_execute_batched / cleave_reduce_batched
 * (members addressed by strides) or cleave_execute_grouped /
 * cleave_reduce_grouped (one pointer per member); the plain calls return
 * CLEAVE_EINVAL on it, and the batched and grouped calls on a plain plan.  CLEAVE_EINVAL as for cleave_plan_uniform, or n_batch < 1. */
int cleave_plan_batched(int64_t M, int64_t N, int64_t K, int64_t tile_m, int64_t tile_n,
                        int32_t ksplit, int64_t n_batch, cleave_plan** out);

int64_t cleave_plan_num_tasks(const cleave_plan* plan);
int64_t cleave_plan_num_tiles(const cleave_plan* plan);
/* Host array of num_tasks records; borrowed, valid until cleave_plan_destroy. */
const cleave_task* cleave_plan_tasks(const cleave_plan* plan);
/* Number of fp32 elements the caller must provide as `partials`. */
int64_t cleave_plan_partial_elems(const cleave_plan* plan);
/* M, N, K of the plan into dims[0..2] (host). */
int cleave_plan_dims(const cleave_plan* plan, int64_t* dims);
/* Copies the plan's tables to the current device now (blocking). */
int cleave_plan_upload(cleave_plan* plan);
/* Frees host and device tables.  NULL is allowed.  Work already enqueued that
 * uses the plan must have finished. */
void cleave_plan_destroy(cleave_plan* plan);

/* ---- execute -------------------------------------------------------------
 * Runs the tasks task_ids[0..n_ids) (host array of indices into the plan's
 * task list, any order, CLEAVE_EINVAL on an index out of range or a repeated
 * index) or, with task_ids == NULL and n_ids == 0, all tasks.  Writes exactly
 * the partial blocks of those tasks into `partials` (device, fp32,
 * cleave_plan_partial_elems elements) and nothing else.
 * A, B: device, dtype elements (4-byte aligned for F32, 2-byte for BF16; rows
 * that start on 16-byte boundaries and inner chunks that are multiples of 16
 * bytes take the fast path, anything else a slower guarded path).
 * The bits of a task's block depend only on its record, the operands and
 * dtype/layout -- not on which other tasks run in the same call.
 * A call with task_ids is stream-ordered like any other: the task indices
 * travel in kernel arguments, the subset's work list is written on the device
 * into memory the plan set aside when its tables were uploaded, and nothing
 * is allocated, copied or waited for on the host.  Such calls may be issued
 * on several streams and from several threads at once (the plan serialises
 * its own bookkeeping) and may be captured into a HIP graph:
 *   - outside capture, a call reuses work-list memory of an earlier subset
 *     call of the same plan only after that call's kernels have finished; the
 *     host waits only in the corner case that more than two full task lists'
 *     worth of subset work of one plan is still in flight;
 *   - under stream capture, the call's work-list memory stays reserved until
 *     the plan is destroyed (the graph may be replayed at any time); the
 *     memory set aside for captured calls holds one full task list's worth of
 *     work items (every task listed once, over all captured calls of the
 *     plan, always fits), beyond that CLEAVE_ENOMEM.  The plan's tables must
 *     have been uploaded before capture begins (cleave_plan_upload or any
 *     earlier call).
 */
int cleave_execute(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                   const void* A, int64_t lda, int transA,
                   const void* B, int64_t ldb, int transB,
                   int dtype, float* partials, void* hip_stream);

/* cleave_execute for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same result bits as cleave_execute, but the call never
 * allocates or frees anything on the device or through the HIP runtime:
 *   - the plan's tables must already be on the current device
 *     (cleave_plan_upload, or any earlier execute / reduce of the plan);
 *     otherwise CLEAVE_EINVAL -- this call does not upload;
 *   - the work list of a subset (task_ids != NULL) is written into a fixed
 *     768 KB array that is part of the library's code object (one copy per
 *     GPU, held until the process ends) instead of plan-owned memory; a subset
 *     whose tasks are cut into more than 16384 work items (256 x 256 or
 *     128 x 128 sub-tiles of the tasks' blocks) is refused with CLEAVE_ELIMIT
 *     and nothing is enqueued;
 *   - every call on a GPU uses that GPU's one array, from its start: two
 *     subset calls that may run at the same time on one GPU (different
 *     streams, or threads) race and must be ordered by the caller; calls on
 *     one stream are ordered by the stream.  No state is carried from call to
 *     call: the array is overwritten by each call that uses it.
 * With task_ids == NULL the whole plan runs (no work list is written). */
int cleave_execute_noalloc(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                           const void* A, int64_t lda, int transA,
                           const void* B, int64_t ldb, int transB,
                           int dtype, float* partials, void* hip_stream);

/* Batched form of cleave_execute for a plan made by cleave_plan_batched.
 * Member g = o * n_inner + i (0 <= i < n_inner, n_inner divides n_batch) reads
 * its operands as zero-copy views: its stored A starts a_outer * o + a_inner * i
 * elements after `A` and has leading dimension lda; B likewise.  Example, Q and
 * K stored token-major [tokens, heads * d]: n_inner = heads, a_outer = seq *
 * lda, a_inner = d, transB = 1 with the same strides for K.  Strides are
 * non-negative element counts; the caller guarantees that every view lies
 * inside its allocation.  Everything else as for cleave_execute. */
int cleave_execute_batched(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                           const void* A, int64_t lda, int transA, int64_t a_outer, int64_t a_inner,
                           const void* B, int64_t ldb, int transB, int64_t b_outer, int64_t b_inner,
                           int64_t n_inner, int dtype, float* partials, void* hip_stream);

/* Grouped form of cleave_execute: the same-shape GEMMs of one DAG level in one
 * launch (Sec. 4.1: the GEMMs of a level are independent and are dispatched
 * together, e.g. the Q, K and V projections).  plan: made by
 * cleave_plan_batched with n_batch <= 8 members; n_members: must equal
 * n_batch; A_list, B_list: host arrays of n_members device pointers (read
 * during the call only), member g multiplies A_list[g] by B_list[g]
 * (pointers may repeat: the projections of a level share their input).  All
 * members share lda, transA, ldb, transB and dtype.  partials: one workspace of
 * cleave_plan_partial_elems elements, member after member.  The bits of a
 * block are those a single-GEMM plan of the same tiling gives for that member.
 * CLEAVE_EINVAL: as for cleave_execute, a plain plan, more than 8 members,
 * n_members != n_batch, a null or misaligned member pointer. */
int cleave_execute_grouped(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                           int64_t n_members, const void* const* A_list, int64_t lda, int transA,
                           const void* const* B_list, int64_t ldb, int transB,
                           int dtype, float* partials, void* hip_stream);

/* Execute for plans without K-splits (every task covers the whole inner
 * dimension, as in the paper's own decomposition, Sec. 4.1): each block is
 * already the finished piece of the output, so it is written straight to its
 * place in C and no partial buffer or reduce call is needed (Sec. 3.2: the PS
 * only assembles the returned blocks).  The values are those cleave_execute
 * followed by cleave_reduce would give, bit for bit (fp32; bf16 = round to
 * nearest even of them).  Plain or batched plan: for a plain plan pass
 * n_inner = 0 and all strides 0; for a batched plan the strides are those of
 * cleave_execute_batched / cleave_reduce_batched.  C: device, out_dtype
 * elements, leading dimension ldc >= N.  task_ids as for cleave_execute.
 * CLEAVE_EINVAL: as for cleave_execute, or a task with a K-split. */
int cleave_execute_assemble(cleave_plan* plan, const int64_t* task_ids, int64_t n_ids,
                            const void* A, int64_t lda, int transA, int64_t a_outer, int64_t a_inner,
                            const void* B, int64_t ldb, int transB, int64_t b_outer, int64_t b_inner,
                            int64_t n_inner, int dtype,
                            void* C, int64_t ldc, int64_t c_outer, int64_t c_inner, int out_dtype,
                            void* hip_stream);

/* ---- reduce --------------------------------------------------------------
 * C[m0+i, n0+j] = ((P_0[i,j] + P_1[i,j]) + ...) + P_{S-1}[i,j] for every tile.
 * partials: device fp32, as written by cleave_execute.  C: device, M x N
 * row-major with leading dimension ldc (>= N), out_dtype CLEAVE_F32 or
 * CLEAVE_BF16 (round to nearest even of the fp32 sum).  With S = 1 the fp32
 * output is a bitwise copy of the single partial. */
int cleave_reduce(cleave_plan* plan, const float* partials, void* C, int64_t ldc,
                  int out_dtype, void* hip_stream);

/* Batched form of cleave_reduce: member g = o * n_inner + i writes its M x N
 * result c_outer * o + c_inner * i elements after `C`, leading dimension ldc. */
int cleave_reduce_batched(cleave_plan* plan, const float* partials, void* C, int64_t ldc,
                          int64_t c_outer, int64_t c_inner, int64_t n_inner,
                          int out_dtype, void* hip_stream);

/* Grouped form of cleave_reduce, the counterpart of cleave_execute_grouped:
 * member g's M x N result goes to C_list[g] (host array of n_members = n_batch
 * device pointers), all with leading dimension ldc and element type out_dtype. */
int cleave_reduce_grouped(cleave_plan* plan, const float* partials, int64_t n_members,
                          void* const* C_list, int64_t ldc, int out_dtype, void* hip_stream);

/* ---- aggregation feeding a PS-side streaming operator ---------------------
 * The paper keeps non-GEMM operators and the optimizer on the parameter
 * server (Sec. 4.1) and runs the optimizer per weight matrix right behind that
 * matrix's gradient GEMM (Sec. 6, "Optimizer step accounting and pipelining").
 * Both calls compute the same fixed-order sum as cleave_reduce and hand it to
 * the operator without storing it.  Single-GEMM plans, except where a grouped
 * form is declared.
 *
 * cleave_reduce_residual: C = sum + R.  R: device, M x N, element type and
 * leading dimension of C; R == C (in-place accumulation) is allowed. */
int cleave_reduce_residual(cleave_plan* plan, const float* partials, const void* R, void* C,
                           int64_t ldc, int out_dtype, void* hip_stream);

/* cleave_reduce_adam: the sum is the gradient g of an M x N weight; per element
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   w = w - lr ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay w )
 * in fp32 (Adam as published, decoupled weight decay).  w, m, v: device fp32,
 * M x N, leading dimension ld, updated in place; w_bf16: device bf16 copy of
 * the new weight, same layout, or NULL.  step counts from 1.  Memory traffic
 * per parameter: 4 S bytes of partials + 24 (+2) bytes of state -- the 26
 * bytes per parameter of the paper's optimizer term.
 * CLEAVE_EINVAL: NULL w/m/v, step < 1, beta outside [0, 1), negative eps, NaN. */
int cleave_reduce_adam(cleave_plan* plan, const float* partials, float* w, float* m, float* v,
                       void* w_bf16, int64_t ld, float lr, float beta1, float beta2, float eps,
                       float weight_decay, int64_t step, void* hip_stream);

/* Grouped form of cleave_reduce_adam: the weight-gradient GEMMs of one DAG level
 * (same shape; plan made by cleave_plan_batched, at most 8 members, executed
 * with cleave_execute_grouped) aggregated and applied in one launch.  w_list,
 * m_list, v_list: host arrays of n_members device pointers (fp32, M x N,
 * leading dimension ld, updated in place); w_bf16_list: likewise for the bf16
 * copies, or NULL for none.  Same arithmetic per element as cleave_reduce_adam:
 * member g's result is bit for bit what the single call gives for it.
 * CLEAVE_EINVAL: as for cleave_reduce_adam, a plain plan, n_members != n_batch,
 * a NULL or misaligned member pointer. */
int cleave_reduce_adam_grouped(cleave_plan* plan, const float* partials, int64_t n_members,
                               float* const* w_list, float* const* m_list, float* const* v_list,
                               void* const* w_bf16_list, int64_t ld,
                               float lr, float beta1, float beta2, float eps, float weight_decay,
                               int64_t step, void* hip_stream);

/* Workgroup loads of the fast kernel's schedule (host only; for inspection
 * and tests).  The fast bf16 kernel runs `grid` persistent workgroups over a
 * list of work items (sub-tiles of tasks); when the items' chunk lengths
 * differ -- heterogeneous tilings, Sec. 4.1 / Sec. 3.2 -- the library gives
 * every workgroup a run of items of nearly equal total cost (longest items
 * first, to the least-loaded workgroup, XCD-local where that costs nothing)
 * instead of every grid-th item.  list: 0 = the 256 x 256 class, 1 = the
 * 128 x 128 class, 2 = the all-small cut used when the large class has few
 * items.  balanced = 0: loads[b] under the every-grid-th rule; 1: under the
 * schedule the library uses (the same when all items are equal).  loads: host,
 * grid doubles, in units of one 64-element K step (an item costs its steps
 * plus 4.5 for its store phase).  CLEAVE_EINVAL: NULL, bad list, grid < 1. */
int cleave_plan_schedule_loads(const cleave_plan* plan, int list, int grid, int balanced,
                               double* loads);

/* ---- verify --------------------------------------------------------------
 * Check of returned partial blocks by random projection (paper Sec. 6,
 * "Robustness to poisoning attacks": r^T (A B) s = (A^T r)^T (B s), matrix-
 * vector work only).  For every task t of the plan, with A_blk = op(A)[m0:m0+
 * m_len, k0:k0+k_len], B_blk = op(B)[k0:k0+k_len, n0:n0+n_len], P_t the task's
 * block in `partials`, r_t = r[m0:m0+m_len] and s_t = s[n0:n0+n_len]:
 *     lhs[t]   = r_t^T P_t s_t
 *     rhs[t]   = (A_blk^T r_t)^T (B_blk s_t)
 *     scale[t] = (|A_blk|^T |r_t|)^T (|B_blk| |s_t|)
 *     accept[t] = 1 if |lhs[t] - rhs[t]| <= tol * scale[t], else 0
 * all sums carried in fp64 in a fixed order (exact, hence lhs == rhs for a
 * correct block, when all values are small integers).
 * A, B, lda, ldb, transA, transB, dtype, partials: as for cleave_execute (the
 * call only reads them).  r: device, M floats; s: device, N floats -- the
 * caller draws them afresh per check.  tol >= 0 (host value).  lhs, rhs,
 * scale: device, num_tasks doubles each, any of them may be NULL; accept:
 * device, num_tasks int32, required.  Asynchronous on hip_stream.  The first
 * call on a plan allocates device scratch owned by the plan (projections of
 * the operands per distinct row / column range of the tiling, per-item sums);
 * two verify calls on one plan must not overlap in time.
 * CLEAVE_EINVAL: NULL or misaligned pointer, bad enum, short leading
 * dimension, negative or NaN tol, or a batched plan (use the forms below). */
int cleave_verify(cleave_plan* plan,
                  const void* A, int64_t lda, int transA,
                  const void* B, int64_t ldb, int transB, int dtype,
                  const float* partials, const float* r, const float* s, double tol,
                  double* lhs, double* rhs, double* scale, int32_t* accept,
                  void* hip_stream);

/* cleave_verify and cleave_reduce in one pass over the partial blocks (Sec. 6
 * and Sec. 3.2: the parameter server checks the blocks the devices return and
 * aggregates them): every partial element is read once, for its check and for
 * the sum.  lhs, rhs, scale, accept: as cleave_verify defines them (rhs and
 * scale the same bits as cleave_verify's; lhs summed over shorter runs of rows,
 * hence equal up to fp64 rounding, exactly equal for small integers).  C, ldc,
 * out_dtype: as for cleave_reduce; C
 * is bit for bit what cleave_reduce writes -- the sum of all S blocks of a tile
 * whatever the verdicts, so a caller that finds a block rejected re-issues the
 * task and aggregates again.  Tiles with more than 8 splits make the call run
 * the two passes one after the other (same results).  Plain plans only.
 * Scratch and the no-overlap rule as for cleave_verify.
 * CLEAVE_EINVAL: as for cleave_verify and cleave_reduce. */
int cleave_verify_reduce(cleave_plan* plan,
                         const void* A, int64_t lda, int transA,
                         const void* B, int64_t ldb, int transB, int dtype,
                         const float* partials, const float* r, const float* s, double tol,
                         double* lhs, double* rhs, double* scale, int32_t* accept,
                         void* C, int64_t ldc, int out_dtype, void* hip_stream);

/* The same check for a plan made by cleave_plan_batched (the attention
 * products of Sec. 3.1's table, or the same-shape GEMMs of a DAG level): every
 * task of every member is checked against that member's operands.  Members are
 * addressed as in cleave_execute_batched (strides) or cleave_execute_grouped
 * (one pointer per member, at most 8).  r: n_batch x M floats, member g's probe
 * vector at r + g * M; s: n_batch x N floats likewise; lhs, rhs, scale, accept:
 * one entry per task of the batched task list.  Everything else, including the
 * scratch the first call allocates and the rule that verify calls on one plan
 * must not overlap, as for cleave_verify.  CLEAVE_EINVAL as for cleave_verify
 * and the corresponding execute call, or a plain plan. */
int cleave_verify_batched(cleave_plan* plan,
                          const void* A, int64_t lda, int transA, int64_t a_outer, int64_t a_inner,
                          const void* B, int64_t ldb, int transB, int64_t b_outer, int64_t b_inner,
                          int64_t n_inner, int dtype,
                          const float* partials, const float* r, const float* s, double tol,
                          double* lhs, double* rhs, double* scale, int32_t* accept,
                          void* hip_stream);
int cleave_verify_grouped(cleave_plan* plan, int64_t n_members,
                          const void* const* A_list, int64_t lda, int transA,
                          const void* const* B_list, int64_t ldb, int transB, int dtype,
                          const float* partials, const float* r, const float* s, double tol,
                          double* lhs, double* rhs, double* scale, int32_t* accept,
                          void* hip_stream);

/* ---- cost model and shard assignment (host only) -------------------------
 * Paper Sec. 4.1: a device d receives alpha rows of A (m x n) and beta columns
 * of B (n x q), b bytes per element, and returns the alpha x beta block:
 *   downlink (alpha n b + n beta b) / down_bw + down_lat,
 *   uplink   alpha beta b / up_bw + up_lat,   compute 2 alpha beta n / flops,
 * overlapped: the shard costs the maximum of the three; it must fit
 * alpha n b + n beta b + alpha beta b <= mem_bytes; a device is idle
 * (alpha = beta = 0, cost 0) or has both >= 1; a GEMM costs the maximum over
 * its devices.  Units: bytes/s, s, flop/s, bytes. */
typedef struct cleave_device {
  double down_bw, up_bw;     /* > 0 */
  double down_lat, up_lat;   /* >= 0 */
  double flops;              /* > 0 */
  double mem_bytes;          /* >= 0 */
} cleave_device;

/* Cost of one shard.  alpha_fetch <= alpha and beta_fetch <= beta are the rows
 * and columns the device still has to download (Sec. 4.2, churn recovery with
 * cached rows / columns); pass alpha, beta for a cold start.  Returns a
 * negative value on invalid arguments (NULL, non-positive rates, one of alpha
 * and beta zero, sizes above 2^24, elem_bytes above 16). */
double cleave_shard_cost(const cleave_device* dev, int64_t alpha, int64_t beta,
                         int64_t alpha_fetch, int64_t beta_fetch, int64_t n, int32_t elem_bytes);
/* 1 if the shard fits the device's memory, 0 if not, CLEAVE_EINVAL on invalid arguments. */
int cleave_shard_fits(const cleave_device* dev, int64_t alpha, int64_t beta, int64_t n,
                      int32_t elem_bytes);

/* Heterogeneous assignment of the m x q output of one GEMM (inner dimension n)
 * to at most n_devs devices, one shard per device, as a guillotine tiling:
 * row bands, each cut into columns.  A deterministic heuristic in place of
 * the paper's MILP (bisection on the target time; devices by descending
 * capacity; see scheduler.cpp).  Shard edges are multiples of `granule` except
 * for ragged rests.  Outputs, all host arrays the caller provides with room
 * for n_devs entries each: *n_bands, band_h[n_bands] (sum m), n_cols[n_bands],
 * col_w (widths of band 0, then band 1, ...; each band sums to q),
 * tile_device (same order: index into devs of the tile's owner), *cost = the
 * GEMM's cost under the model.  band_h / n_cols / col_w are the arguments of
 * cleave_plan_explicit (with one K-split entry of 1 per tile).
 * CLEAVE_EINVAL: NULL pointers, invalid device, non-positive or too large
 * sizes, or no cover exists within the devices' memory. */
int cleave_assign(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                  const cleave_device* devs, int32_t n_devs, int64_t granule,
                  int32_t* n_bands, int64_t* band_h, int32_t* n_cols, int64_t* col_w,
                  int32_t* tile_device, double* cost);

/* Churn re-solve (paper Sec. 4.2): the m x q rectangle is the unfinished output
 * of failed devices, starting at (row0, col0) of the GEMM's output; devs are
 * the survivors.  cached[4k .. 4k+3] = [row_lo, row_hi, col_lo, col_hi): the
 * rows of A and columns of B survivor k already holds (absolute indices; an
 * empty interval if none), which it does not download again; mem_used[k] =
 * bytes of its memory already taken (no cache replacement during a GEMM).
 * Same construction, outputs and errors as cleave_assign, with the cache-aware
 * downlink term; also CLEAVE_EINVAL for NULL / negative / inverted intervals. */
int cleave_reassign(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                    const cleave_device* devs, int32_t n_devs, int64_t granule,
                    int64_t row0, int64_t col0, const int64_t* cached, const double* mem_used,
                    int32_t* n_bands, int64_t* band_h, int32_t* n_cols, int64_t* col_w,
                    int32_t* tile_device, double* cost);

/* The churn re-solve with general cache sets (paper Sec. 4.2: binary cache
 * matrices R_s over the rows of A and C_s over the columns of B, one row per
 * device): survivor k holds the rows in the union of its n_row_iv[k] intervals
 * and the columns in the union of its n_col_iv[k] intervals.  row_iv lists the
 * devices' row intervals one after the other as pairs [lo, hi) (absolute
 * indices, per device ascending and disjoint), col_iv likewise; a device with
 * no cached rows has n_row_iv[k] = 0.  The downlink term of a shard counts
 * only the rows and columns outside the owner's sets.  Everything else as for
 * cleave_reassign, which is the special case of one interval each.
 * CLEAVE_EINVAL also for negative counts, unsorted or overlapping intervals. */
int cleave_reassign_sets(int64_t m, int64_t q, int64_t n, int32_t elem_bytes,
                         const cleave_device* devs, int32_t n_devs, int64_t granule,
                         int64_t row0, int64_t col0,
                         const int32_t* n_row_iv, const int64_t* row_iv,
                         const int32_t* n_col_iv, const int64_t* col_iv, const double* mem_used,
                         int32_t* n_bands, int64_t* band_h, int32_t* n_cols, int64_t* col_w,
                         int32_t* tile_device, double* cost);

/* ---- misc ----------------------------------------------------------------*/
const char* cleave_strerror(int status);
/* hipError_t value of the most recent CLEAVE_EHIP on this thread (0 if none). */
int cleave_last_hip_error(void);
/* Library ABI version (major*100 + minor). */
int cleave_version(void);
/* Name of the kernel variant the last cleave_execute of this plan chose for
 * its dominant launch (for profiling reports); static string, never NULL. */
const char* cleave_plan_last_kernel(const cleave_plan* plan);

#ifdef __cplusplus
}
#endif
#endif /* CLEAVE_H */
