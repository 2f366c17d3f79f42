/*
 * libosdp — operator-split linear layer of OSDP (arXiv 2209.13258) for AMD MI355X (gfx950).
 *
 * One GPU's share of a sharded-data-parallel step for one linear operator
 * Y[T x O] = X[T x I] . W[I x O] (no bias).  W is kept in an N-way shard-major
 * layout (Section 2.2: ZeRO/FSDP shard the model states over the N workers and
 * re-gather them for use).  Following Section 3.3 ("Operator Splitting") the
 * operator is cut into k slices that are gathered and processed one after
 * another, so that only a slice of gathered weight is live at a time: the
 * gathered-weight peak drops from size(MatMul) to size(MatMul)/slice_granularity.
 * By default the slices are column slices of W (output features):
 *
 *     forward  : Y[:, c0_j:c1_j]  = X . Ws_j                     (concatenate)
 *     backward : dW[:, c0_j:c1_j] = X^T . dY[:, c0_j:c1_j]       (concatenate)
 *                dX               = sum_j dY[:, c0_j:c1_j] . Ws_j^T   (sum)
 *
 * where Ws_j[I x w_j] is slice j gathered from the N shards into a staging
 * buffer.  All three recombine to exactly the unsplit product.
 *
 * A plan may instead cut an operator along W's rows (input features), which is
 * the scheme Section 3.3 prints: the input is cut along its last dimension, the
 * weight along its first, and the partial products are added up:
 *
 *     forward  : Y                = sum_j X[:, r0_j:r1_j] . Wr_j      (sum)
 *     backward : dW[r0_j:r1_j, :] = X[:, r0_j:r1_j]^T . dY            (concatenate)
 *                dX[:, r0_j:r1_j] = dY . Wr_j^T                       (concatenate)
 *
 * with Wr_j[h_j x O] the gathered row slice, r0_j = floor(j*I/k).  The staging
 * law is the same (size(MatMul)/k per live slice); the sum now sits in the
 * forward pass.
 *
 * Conventions
 *   - Plain C ABI: no C++ or framework types.  Every "device" pointer is a HIP
 *     device pointer on the current device; every "host" pointer is ordinary
 *     host memory that is only read during the call.
 *   - All matrices hold bf16 (IEEE binary32 upper half), row-major, with an
 *     explicit leading dimension counted in elements.  Products accumulate in
 *     fp32 on the matrix cores; outputs are rounded to bf16, nearest even.
 *   - Shard-major layout of W (and of dW): flat index f = r*O + c, shard
 *     length L = ceil(I*O/N); the element lives in buffer w_shards[f / L] at
 *     element offset f % L.  Each shard is its own allocation of L elements;
 *     the tail of the last shard is padding that is never read or written.
 *     When N divides I this is N row blocks of I/N rows.
 *   - Slice bounds: c0_j = floor(j*O/k), c1_j = floor((j+1)*O/k).  k = 0 means
 *     "no splitting" (the paper's granularity 0, Section 4.3) and equals k = 1.
 *   - The library never allocates device memory.  The caller owns all buffers,
 *     including the workspace; the library owns only a few HIP events (at most 64
 *     per calling host thread and device; a thread that ends hands its events to
 *     the threads that start later) and one fixed scratch array per device for
 *     osdp_split_linear_fwd_noalloc.
 *   - Threads: any host thread may call; calls from different threads share no
 *     state in the library.  Two calls that use the same workspace or outputs
 *     must be ordered by the caller's streams like any other GPU work.
 *   - Calls enqueue work and return.  When a call returns, synchronising
 *     stream_compute alone makes every output valid, and stream_copy has been
 *     ordered after the last use of the workspace.  Inputs must be ready on
 *     stream_compute when the call is made.
 *   - The forward, backward and gather calls can be captured into a HIP graph on
 *     stream_compute (after one eager call, which sets kernel attributes): they enqueue
 *     kernels and event records / waits only, and every use of stream_copy starts
 *     from and returns to stream_compute.  Not capturable: the profiling calls
 *     and osdp_granularity_measure, which synchronise.
 *   - Errors: arguments are validated before anything is enqueued, so every
 *     status except OSDP_ERR_HIP leaves the outputs untouched.
 *     osdp_last_error() gives a thread-local message for the last failure.
 *
 * Shapes the GPU kernels accept (else OSDP_ERR_UNSUPPORTED): I, O, every slice
 * bound c0_j (or r0_j), the shard length L and every leading dimension are multiples of
 * 8 elements (16-byte vectors); pointers are 16-byte aligned; N <= 64;
 * T, I, O < 2^31.
 */
#ifndef OSDP_H
#define OSDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OSDP_MAX_SHARDS 64
#define OSDP_API __attribute__((visibility("default")))

typedef enum {
  OSDP_OK = 0,
  OSDP_ERR_INVALID_ARG = -1, /* null pointer, non-positive size (T < 0), k > O, slice out of range, ld too small */
  OSDP_ERR_UNSUPPORTED = -2, /* legal problem the kernels or this entry point do not handle (alignment, N > 64) */
  OSDP_ERR_WORKSPACE = -3,   /* workspace_bytes smaller than osdp_split_linear_workspace_bytes says */
  OSDP_ERR_HIP = -4          /* a HIP runtime call failed; outputs are undefined */
} osdp_status;

/* One linear operator (the paper's operator i with its parallelism degree N,
 * Section 3) together with its slice granularity (Section 3.3). */
typedef struct {
  int64_t T; /* tokens: rows of X, Y, dY, dX.  0 is allowed: the
                forward call then does nothing, the backward call
                stores dW = 0 (an empty sum); X, Y, dY, dX may be
                NULL                                              */
  int64_t I; /* in-features: columns of X, rows of W               */
  int64_t O; /* out-features: columns of W, Y                      */
  int32_t N; /* shard count                                        */
  int32_t k; /* slice granularity; 0 == 1 == unsplit               */
} osdp_shape;

/* How the slice-sized staging area is used. */
typedef enum {
  OSDP_STAGING_AUTO = 0,   /* DOUBLE when two distinct streams are given and k > 1, else SINGLE */
  OSDP_STAGING_SINGLE = 1, /* one slot of one slice (size/k): gather and GEMM alternate, no overlap */
  OSDP_STAGING_DOUBLE = 2, /* two slots of one slice (2*size/k): gather j+1 overlaps GEMM j        */
  OSDP_STAGING_HALF = 3    /* two slots of half a slice (size/k in total): a slice is processed either as
                              two half-width sub-slices in a ring (the gather of one half rides along
                              with the GEMM of the other) or, when the library estimates that faster,
                              as one slice staged across both slots (the SINGLE schedule).  On one
                              GPU the ring seldom pays: half-width launches have half the output
                              tiles, and an overlapped gather costs the GEMM beside it what it saves */
} osdp_staging_mode;

/* Which dimension of W the k slices cut. */
typedef enum {
  OSDP_SPLIT_OUT_FEATURES = 0, /* columns of W: Y and dW concatenate, dX is summed                   */
  OSDP_SPLIT_IN_FEATURES = 1,  /* rows of W, the forward product's reduction dimension (Section 3.3
                                  as printed): Y is summed, dW and dX concatenate                     */
  OSDP_SPLIT_LONGER = 2,       /* whichever of the two is longer (columns when I == O): the fp32 partial
                                  sum is T x the other dimension, and measured on MI355X the longer cut
                                  is the faster one at every granularity                              */
  OSDP_SPLIT_PER_PASS = 3      /* columns in the forward pass, rows in the backward pass: Y, dX and dW are
                                  all concatenations, no fp32 partial sum exists in either pass; every
                                  slice is still size/k (the passes gather differently shaped slices of
                                  the same size).  Needs both I/k and O/k bounds on multiples of 8; not
                                  with slices in DP mode                                               */
} osdp_split_dim;

/* The per-operator execution plan (the paper's plan vector p over the n
 * operators, Section 3.1), extended by the slice granularity of each operator
 * (Section 3.3).  All arrays are host memory.  A NULL plan means "use
 * shape->k, every slice gathered (ZDP), OSDP_STAGING_AUTO". */
typedef struct {
  int32_t n_ops;            /* number of operators the arrays describe                         */
  const int32_t *k_per_op;  /* [n_ops] slice granularity; overrides shape->k for op_index      */
  const uint64_t *zdp_mask; /* [n_ops] or NULL (= every slice ZDP); bit j set: slice j is      */
                            /* sharded and gathered (ZDP mode), clear: slice j is replicated   */
                            /* (DP mode, Section 3.3: each slice may get its own mode) and is  */
                            /* used from the caller's replica: the _mixed entry points only.   */
  int32_t staging;          /* an osdp_staging_mode                                            */
  const uint8_t *split_dim_per_op; /* [n_ops] or NULL (= all OSDP_SPLIT_OUT_FEATURES): an       */
                            /* osdp_split_dim per operator                                     */
  const int32_t *staging_per_op;   /* [n_ops] or NULL (= `staging` for all): an                  */
                            /* osdp_staging_mode per operator                                  */
} osdp_plan;

/* Column range [*c0, *c1) of slice j for shape->O and shape->k. Host only. */
OSDP_API osdp_status osdp_slice_range(const osdp_shape *shape, int32_t slice_j, int64_t *c0, int64_t *c1);

/* Row range [*r0, *r1) of slice j when W is cut along its rows: r0 = floor(j*I/k). Host only. */
OSDP_API osdp_status osdp_row_slice_range(const osdp_shape *shape, int32_t slice_j, int64_t *r0, int64_t *r1);

/* Section 3.3, re-gathering of one slice: Ws_j[r, c] = W[r, c0_j + c].
 *   w_shards : host array of shape->N device pointers (bf16 shard buffers)
 *   staging  : device, dense row-major [I x w_j] bf16, >= I*w_j*2 bytes, written in full
 *   stream   : hipStream_t (NULL = default stream)
 * Pure copy: the result is bit-exact. */
OSDP_API osdp_status osdp_split_linear_gather_slice(const osdp_shape *shape, int32_t slice_j,
                                           const void *const *w_shards, void *staging,
                                           void *stream);

/* The same for a row slice (Section 3.3: the weight cut along its first dimension):
 * Wr_j[r, c] = W[r0_j + r, c].
 *   staging  : device, dense row-major [h_j x O] bf16, >= h_j*O*2 bytes, written in full
 * Row bounds must be multiples of 8. Pure copy: bit-exact. */
OSDP_API osdp_status osdp_split_linear_gather_row_slice(const osdp_shape *shape, int32_t slice_j,
                                               const void *const *w_shards, void *staging,
                                               void *stream);

/* Bytes of workspace a forward (is_bwd = 0) or backward (is_bwd != 0) call
 * needs, and how many of them hold gathered weights at the peak
 * (Section 3.3: size(MatMul)/slice_granularity per live slice).
 * Workspace layout: [staging slots][fp32 accumulator: T*I for dX, backward with column slices and more than
 * one dX launch; T*O for Y, forward with row slices and more than one launch][fp32 planes: forward with column
 * slices, T <= 4096 and I >= 16384, where the product is summed in parts of 8192 input features: parts x T x
 * (columns of the widest launch) x 4 bytes].
 * With OSDP_STAGING_AUTO the total covers both the one-stream and the two-stream call.
 * Either output pointer may be NULL. Host only. */
OSDP_API osdp_status osdp_split_linear_workspace_bytes(const osdp_shape *shape, const osdp_plan *plan,
                                              int32_t op_index, int32_t is_bwd, size_t *total,
                                              size_t *peak_weight_staging);

/* Section 3.3, forward of the split operator: for j = 0..k-1 gather slice j,
 * then Y[:, c0_j:c1_j] = X . Ws_j.
 *   X  : device [T x I], ldx >= I        Y : device [T x O], ldy >= O (every element written)
 *   w_shards : host array of N device pointers
 *   workspace: device, 256-byte aligned, >= osdp_split_linear_workspace_bytes(.., 0, ..)
 *   stream_compute : hipStream_t the GEMMs run on
 *   stream_copy    : hipStream_t the gathers may run on; NULL or == stream_compute = no overlap.
 *                    The library keeps a call on stream_compute alone when the copy stream could
 *                    not hide anything (launches that hold both slots; gathers too small to be
 *                    worth the cross-stream events).
 * With row slices (plan->split_dim_per_op): for j = 0..k-1 gather row slice j, then
 * Y += X[:, r0_j:r1_j] . Wr_j, the sum carried in fp32 (through the workspace between launches) in ascending
 * j and rounded to bf16 once.
 * Y is bit-identical for every k, staging mode and stream choice (row slices: when every slice height is a
 * multiple of 16).  With column slices, T <= 4096 and I >= 16384 (few output tiles per slice, a long reduction)
 * the product is the sum over min(I / 8192, 8) parts of the input features, each part accumulated on its own and
 * the parts added in ascending order in fp32 before the one rounding to bf16 (when that number of parts times 64
 * divides I): the unsplit operator (k = 1) is computed the same way, so this too is independent of k.  (Row slices always
 * continue one accumulator chain.) */
OSDP_API osdp_status osdp_split_linear_fwd(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                  const void *X, int64_t ldx, const void *const *w_shards,
                                  void *Y, int64_t ldy, void *workspace, size_t workspace_bytes,
                                  void *stream_compute, void *stream_copy);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): osdp_split_linear_fwd on one
 * stream, with the staging slots, the fp32 partial sum and the fp32 planes of a forward summed in parts kept in a fixed array of
 * OSDP_NOALLOC_SCRATCH_BYTES that is part of the library's device code (one copy per GPU, held
 * until the process ends).  Same arguments, layouts, results (bit for bit) and errors as
 * osdp_split_linear_fwd with stream_copy = NULL; nothing is allocated, no event is created.
 * OSDP_ERR_WORKSPACE, before anything is enqueued, when the plan needs more than the array holds
 * (what osdp_split_linear_workspace_bytes reports for the forward pass): raise k.
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (every byte a
 * call reads it has written first, so nothing needs clearing): calls on different streams or from
 * different threads that overlap in time on one GPU race and must be ordered by the caller. */
#define OSDP_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
OSDP_API osdp_status osdp_split_linear_fwd_noalloc(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                                   const void *X, int64_t ldx, const void *const *w_shards,
                                                   void *Y, int64_t ldy, void *stream);

/* Section 3.3 applied to the backward pass (the weights are gathered again,
 * Section 2.2): for j = 0..k-1, dW[:, c0_j:c1_j] = X^T . dY[:, c0_j:c1_j]
 * (written into dw_shards, same shard-major layout as W, overwritten), and
 * dX = sum_j dY[:, c0_j:c1_j] . Ws_j^T, accumulated in fp32 across the slices
 * in ascending j and rounded to bf16 once.  Slices that are staged together
 * (two slots) share one dW launch, and one dX pass when their widths are
 * multiples of 64; the fp32 partial sum goes through the workspace only
 * between passes.
 *   dY : device [T x O], lddy >= O       dX : device [T x I], lddx >= I
 *   dw_shards : host array of N device pointers, each L elements
 * With row slices: dW[r0_j:r1_j, :] = X[:, r0_j:r1_j]^T . dY and dX[:, r0_j:r1_j] = dY . Wr_j^T, no sum.
 * dW is bit-identical for every k and split dimension; dX is too when every slice width is a
 * multiple of 16 (row slices: always; with T <= 4096 and O >= 16384 their dX is summed in parts of 8192 output
 * features, like the forward product of column slices, whatever k). */
OSDP_API osdp_status osdp_split_linear_bwd(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                  const void *X, int64_t ldx, const void *dY, int64_t lddy,
                                  const void *const *w_shards, void *dX, int64_t lddx,
                                  void *const *dw_shards, void *workspace, size_t workspace_bytes,
                                  void *stream_compute, void *stream_copy);

/* ---- every slice in its own mode -------------------------------------------
 * Section 3.3, last paragraph: once an operator is cut into slices each slice
 * can be DP or ZDP on its own (the paper's example: 1 of 4 slices ZDP, 3 DP).
 * A ZDP slice (plan->zdp_mask bit set) is handled as above: gathered from the
 * shards into a staging slot before every use, its gradient written into
 * dw_shards.  A DP slice is replicated on every worker: it is read where it
 * lies in the caller's replica (no gather, no staging, so the gathered-weight
 * peak counts ZDP slices only) and its gradient is a plain array of the same
 * shape.
 *   w_dp  : host array of k device pointers; w_dp[j] (DP slices only; others
 *           ignored) is slice j, row-major bf16 with leading dimension ld_dp:
 *           [I x w_j] for column slices, [h_j x O] for row slices.  A full
 *           row-major copy of W serves with w_dp[j] = W + c0_j, ld_dp = O
 *           (row slices: W + r0_j*O).  May be NULL when no slice is DP.
 *   dw_dp : the same for the gradients (written, DP slices only).
 *   ld_dp : multiple of 8, >= the widest DP slice's columns.
 * The shard buffers keep the layout of the whole matrix, so a plan can change
 * a slice's mode without re-sharding; their elements inside DP slices are
 * never read, and dw_shards is not written there.  Everything else (shapes,
 * workspace from osdp_split_linear_workspace_bytes, streams, errors) as for
 * osdp_split_linear_fwd / _bwd, which these calls equal when every slice is
 * ZDP.  Results are bit-identical to the all-ZDP plan on the same weights. */
OSDP_API osdp_status osdp_split_linear_fwd_mixed(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                                 const void *X, int64_t ldx, const void *const *w_shards,
                                                 const void *const *w_dp, int64_t ld_dp, void *Y, int64_t ldy,
                                                 void *workspace, size_t workspace_bytes, void *stream_compute,
                                                 void *stream_copy);
OSDP_API osdp_status osdp_split_linear_bwd_mixed(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                                 const void *X, int64_t ldx, const void *dY, int64_t lddy,
                                                 const void *const *w_shards, const void *const *w_dp, int64_t ld_dp,
                                                 void *dX, int64_t lddx, void *const *dw_shards, void *const *dw_dp,
                                                 void *workspace, size_t workspace_bytes, void *stream_compute,
                                                 void *stream_copy);

/* ---- automatic slice granularity ------------------------------------------
 * Section 4.3 (effectiveness of operator splitting) observes that the best
 * granularity depends on the operator: small operators pay time for every extra
 * slice, large ones need many slices before the gathered-weight peak stops
 * falling, and leaves open how to suggest a granularity per operator from the
 * model description and the device.  Here: enumerate the (granularity, split
 * dimension, staging mode) combinations the kernels take for the operator's
 * shape, time each on this device with the operator's own buffers, and select
 * by a fixed rule. */

typedef struct {
  int32_t k;                  /* slice granularity, >= 1                                  */
  int32_t staging;            /* OSDP_STAGING_SINGLE, _DOUBLE or _HALF                    */
  int32_t split_dim;          /* an osdp_split_dim                                        */
  int32_t reserved;           /* 0                                                        */
  size_t peak_weight_staging; /* gathered-weight bytes live at the peak (Section 3.3 law) */
  size_t workspace;           /* workspace bytes that cover the forward and the backward  */
  double ms;                  /* one forward + backward in milliseconds; 0 = not measured */
} osdp_granularity_candidate;

/* Lists the combinations that osdp_split_linear_fwd / _bwd accept for this
 * shape (shape->k is ignored): for every k of k_list (host, n_k entries >= 1;
 * NULL = 1, 2, 3, 4, 6, 8, 12, 16), in the order given, for the column split,
 * the row split, then the per-pass split, for SINGLE, DOUBLE, HALF staging.  Combinations that
 * resolve to the same execution are listed once (k = 1: one SINGLE entry).
 * Writes at most `capacity` entries to out (ms = 0) and the full count to
 * *count; out may be NULL when capacity is 0. Host only. */
OSDP_API osdp_status osdp_granularity_candidates(const osdp_shape *shape, const int32_t *k_list, int32_t n_k,
                                                 osdp_granularity_candidate *out, int32_t capacity, int32_t *count);

/* Times every candidate on the current device: `warmup` untimed and `reps`
 * timed repetitions of osdp_split_linear_fwd followed by osdp_split_linear_bwd
 * with the candidate's plan, HIP events on stream_compute, and stores the mean
 * in cands[i].ms.  Buffers as for those two calls; workspace_bytes must cover
 * the largest candidate (OSDP_ERR_WORKSPACE otherwise, before anything runs).
 * Synchronises stream_compute once per candidate.  Y, dX and dW end up holding
 * the last candidate's (valid) results. */
OSDP_API osdp_status osdp_granularity_measure(const osdp_shape *shape, const void *X, int64_t ldx, const void *dY,
                                              int64_t lddy, const void *const *w_shards, void *Y, int64_t ldy,
                                              void *dX, int64_t lddx, void *const *dw_shards, void *workspace,
                                              size_t workspace_bytes, void *stream_compute, void *stream_copy,
                                              osdp_granularity_candidate *cands, int32_t n, int32_t warmup,
                                              int32_t reps);

/* The selection rule. Host only.  Among the measured candidates (ms > 0) whose
 * peak_weight_staging is at most staging_budget bytes and whose workspace (the
 * staging slots plus the fp32 partial sum) is at most workspace_budget bytes
 * (0 = no limit, each), let t* be the smallest ms.  Of those with ms <= (1 + max_slowdown) * t*, the one
 * with the smallest peak_weight_staging is chosen; ties go to the smaller ms,
 * then to the lower index.  max_slowdown = 0 picks the fastest candidate that
 * fits; a large max_slowdown picks the smallest peak whatever it costs in time
 * (the trade-off Section 4.3 leaves open).
 * OSDP_ERR_UNSUPPORTED when no measured candidate fits the budgets. */
OSDP_API osdp_status osdp_granularity_select(const osdp_granularity_candidate *cands, int32_t n,
                                             size_t staging_budget, size_t workspace_budget,
                                             double max_slowdown, int32_t *chosen);

/* ---- execution-plan search (host only) -------------------------------------
 * Section 3.1 (problem formulation and cost model), Section 3.2 (Profiler,
 * Search Engine, Scheduler) and Algorithm 1.  An "operator" here is whatever
 * unit gets its own mode: a whole operator, or one slice of a split operator
 * (Section 3.3), whose costs are the operator's divided by the granularity. */

typedef struct {
  double m_model; /* M_i^(model): bytes of model states (parameters and optimizer states)      */
  double m_act;   /* M_i^(act): activation bytes per sample                                    */
  double m_extra; /* M_i^(extra): other bytes (workspaces)                                     */
  double s_bytes; /* S_i: size of the operator's parameters, as counted by the collectives     */
  double gamma;   /* gamma_i: computation time per sample                                      */
} osdp_operator_cost;

typedef struct {
  int32_t N;      /* parallelism degree                                                        */
  int32_t b_max;  /* largest batch size to try; 0 = 65536                                      */
  double alpha;   /* network latency per communication step                                    */
  double beta;    /* transfer time per unit of s_bytes                                         */
  double m_limit; /* device memory limit, same unit as the m_* fields                          */
} osdp_device_info;

typedef struct {
  int32_t found;             /* 0: not even b = 1 has a plan within the memory limit           */
  int32_t b;                 /* chosen batch size                                              */
  double time_per_sample;    /* T(p, b) = (1/b) * sum_i T_i(p_i, b) of the chosen plan         */
  double memory;             /* M(p, b) of the chosen plan                                     */
  int32_t batch_sizes_tried; /* number of batch sizes that had a feasible plan                 */
  int32_t exact;             /* 1: proven optimal; 0: a search ran out of its node budget and  */
                             /* returned the best plan it had found                            */
  int32_t reserved;
  uint64_t plans_visited;    /* nodes of the search trees over all batch sizes                 */
} osdp_search_result;

/* The cost model of Section 3.1 for one plan: modes[i] = 0 (DP) or 1 (ZDP).
 *   M(p, b) = sum_i [ M_model_i (DP) or M_model_i / N (ZDP) ] + b * M_act_i + M_extra_i
 *   T(p, b) = (1/b) * sum_i [ 2 (DP) or 3 (ZDP) ] * (N-1) * (alpha + S_i/N * beta) + b * gamma_i
 * Sums run over the operators in order.  Either output may be NULL. */
OSDP_API osdp_status osdp_cost_model(const osdp_operator_cost *ops, int32_t n, const osdp_device_info *dev,
                                     const uint8_t *modes, int32_t b, double *memory, double *time_per_sample);

/* Algorithm 1.  For b = 1, 2, 3, ... a depth-first search over {DP, ZDP}^n,
 * pruned when the memory limit can no longer be met or the best time so far
 * can no longer be beaten, finds a fastest plan with M(p, b) <= m_limit; the
 * loop ends at the first b with no such plan (or after b_max); the (plan, b)
 * with the smallest time per sample is returned in modes[n] and *result (of
 * equally fast batch sizes the smaller).  The search is exact: the time is the
 * minimum over all 2^n plans up to the rounding of the sums (1e-12 relative);
 * when several plans reach it, which of them is returned is unspecified.
 * Operators with identical costs (repeated layers) are decided together, as
 * a count, and classes are explored cheapest-memory-first (extra time per
 * byte given back), which keeps models of hundreds of operators to
 * milliseconds; the worst case (all operators different, costs strongly
 * correlated) remains exponential, so each batch size's search stops after
 * 2e7 nodes and result->exact then reads 0. */
OSDP_API osdp_status osdp_plan_search(const osdp_operator_cost *ops, int32_t n, const osdp_device_info *dev,
                                      uint8_t *modes, osdp_search_result *result);

/* ---- test and debug switches ------------------------------------------------
 * Process-wide switches for tests and for hunting stream races; none of them
 * but "split_k" changes a result bit.  Initial values come from the environment variables
 * OSDP_DEBUG_<NAME IN CAPITALS>, read once when the library is first used.
 *   "gemm_generic"   0 | 1   1: every GEMM runs on the bounds-checked kernel
 *   "tile"          -1 .. 3  force tile shape 256x256, 256x128, 128x256, 128x128 where it divides the launch
 *   "deep"          -1 | 0   0: launches of at most one tile per CU keep the shallow LDS pipelines
 *   "split_launch"  -1 | 0   0: no launch is cut into whole rounds of large tiles + remainder
 *   "split_k"       -1 | 0   0: forward products are never summed in parts of the reduction (the one switch that
 *                            changes result bits: those of the products that are otherwise summed in parts)
 *   "four_wave"     -1 .. 1  0: 256x256 tiles always run on the eight-wave kernel; 1: on the four-wave kernel
 *                            whenever it takes the launch (K >= 192), also where the eight-wave one measured faster
 *   "persistent"    -1 .. 1  0: a launch of more 256x256 tiles than CUs keeps the four-wave kernel of one tile per
 *                            workgroup; otherwise one workgroup per CU walks through the tiles; 1: the walking
 *                            form also for launches of fewer tiles
 *   "fused_gather"  -1 | 0   0: every gather is a launch of its own (on stream_copy where the pipeline overlaps);
 *                            otherwise a GEMM launch takes the next slice's gather along wherever it can
 *   "fwd_pair"      -1 .. 1  0: the forward never runs two staged slices in one launch; 1: whenever it can
 *   "poison_staging" 0 | 1   1: a staging slot is filled with bf16 NaN patterns when a call starts and again as
 *                            soon as the last GEMM that reads its slice has been enqueued (on the compute
 *                            stream, ahead of the event that hands the slot to the next gather): a GEMM that
 *                            runs ahead of its gather, or a gather that lands on a slice still in use,
 *                            then shows up as NaN or wrong outputs instead of going unnoticed because the
 *                            stale bytes happened to be right.  Costs one fill per slot use.
 * -1 restores the library's own choice.  OSDP_ERR_INVALID_ARG for unknown names or values. */
OSDP_API osdp_status osdp_debug_option(const char *name, int32_t value);

/* ---- per-kernel timing (for benchmarks) --------------------------------- */

typedef enum {
  OSDP_KERNEL_GATHER = 0,
  OSDP_KERNEL_GEMM_FWD = 1,
  OSDP_KERNEL_GEMM_DW = 2,
  OSDP_KERNEL_GEMM_DX = 3,
  OSDP_KERNEL_GATHER_CARRIED = 4, /* gathers that ran inside a GEMM launch: launches and bytes only, their time is
                                     part of the GEMM launches that carried them */
  OSDP_KERNEL_GEMM_PERSISTENT = 5, /* the GEMM launches among kinds 1-3 that ran as the persistent kernel (one workgroup
                                      per CU walking through the tiles): a count only, time and flops are in their kinds */
  OSDP_KERNEL_KINDS = 6
} osdp_kernel_kind;

typedef struct {
  int64_t launches; /* kernel launches seen since osdp_profile_begin          */
  double ms;        /* sum of their durations, HIP events on the launch stream */
  double flops;     /* 2*M*N*K summed over GEMM launches                       */
  double bytes;     /* algorithmic bytes summed over launches: operands read once, output written once */
} osdp_kernel_stats;

/* Between begin and end every kernel launch of the calling thread is bracketed
 * by a pair of HIP events on its own stream (at most max_launches launches;
 * later ones are not timed).  osdp_profile_end synchronises the device and
 * fills stats[OSDP_KERNEL_KINDS]. Not for use inside hot loops one wants
 * undisturbed: the event records sit between the kernels. */
OSDP_API osdp_status osdp_profile_begin(int32_t max_launches);
OSDP_API osdp_status osdp_profile_end(osdp_kernel_stats *stats);

/* After osdp_profile_end: how the launches of the profiled region lay in time (all streams on one clock).
 *   span_ms           : first launch start to last launch end
 *   idle_ms           : the part of the span in which no kernel of the library ran (launch gaps, event handling)
 *   gather_exposed_ms : the time in which a gather kernel ran and no GEMM did, i.e. gather time that no GEMM hid
 *                       (gathers carried inside GEMM launches are not kernels of their own and do not appear here)
 * Any pointer may be NULL.  Host only. */
OSDP_API osdp_status osdp_profile_overlap(double *span_ms, double *idle_ms, double *gather_exposed_ms);

OSDP_API const char *osdp_strerror(osdp_status status);
OSDP_API const char *osdp_last_error(void);
OSDP_API const char *osdp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OSDP_H */
