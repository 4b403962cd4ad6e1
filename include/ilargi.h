/*
 * ilargi.h -- C ABI of the MI355X (gfx950) library for factorized linear algebra over a target
 * table that is never built:
 *
 *     T = I_1 D_1 M_1^T + ... + I_n D_n M_n^T                 (paper, Sec. 2.2, rewrite rule)
 *
 * D_k  source table k (the paper's S_k), r_k x c_k, float32, row-major, leading dimension c_k.
 * I_k  indicator matrix (paper, Def. 2), logically r_T x r_k binary with at most one 1 per row.
 *      Stored compressed as row_idx: int32[r_T], row_idx[i] = the row of D_k that feeds target row
 *      i, or -1 when target row i takes nothing from source k.  Never stored as a matrix.
 * M_k  mapping matrix (paper, Def. 1), c_T x c_k binary, at most one 1 per row and per column.
 *      Stored compressed as col_map: int32[c_k], col_map[j] = target column of source column j, or
 *      -1 when the column is dropped.  Different sources may map to the same target column; their
 *      contributions are summed, as the rewrite rule says.
 *
 * Conventions for every call
 *   - Matrices are dense float32, row-major, with no padding between rows.
 *   - "device" pointers are HIP device addresses valid on the current device; "host" pointers are
 *     ordinary process memory.  The library never takes ownership of caller memory.  A buffer with
 *     r_T rows may be NULL when r_T = 0 (it is empty); every other buffer must not be.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Operator calls only
 *     enqueue work on that stream and return; outputs are valid once the stream has reached that
 *     point.  ilargi_plan_create synchronizes the stream before it returns.
 *   - The library allocates no device memory.  All device state of a plan (inverse indices, column
 *     tables, intermediates, reduction partials) lives in the caller's workspace, whose size
 *     ilargi_plan_workspace_bytes reports.  Calls that share a plan must not overlap in time.
 *   - Every call returns an ilargi_status_t and never throws or aborts.  On an error detected
 *     before launch, outputs are untouched.  ilargi_last_error() gives a message for the last
 *     failure on the calling thread.
 *   - Floating-point results are deterministic: the same plan and inputs give the same bits on
 *     every run; no floating-point atomics are used.
 */
#ifndef ILARGI_H_
#define ILARGI_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ilargi_plan ilargi_plan_t; /* opaque; host object owned by the library */

typedef enum {
  ILARGI_OK = 0,
  ILARGI_ERR_NULL = 1,        /* a required pointer is NULL */
  ILARGI_ERR_SHAPE = 2,       /* negative or inconsistent sizes */
  ILARGI_ERR_COLMAP = 3,      /* col_map entry outside [-1, c_T) or two columns of one source share a target */
  ILARGI_ERR_INDEX_RANGE = 4, /* row_idx entry outside [-1, r_k) */
  ILARGI_ERR_WORKSPACE = 5,   /* workspace too small or misaligned, or cx / m above max_cx */
  ILARGI_ERR_UNSUPPORTED = 6, /* combination of arguments that has no kernel */
  ILARGI_ERR_DEVICE = 7       /* a HIP call failed */
} ilargi_status_t;

typedef enum {
  ILARGI_F32 = 0,            /* float32 operands, float32 accumulation */
  ILARGI_BF16_IN_F32_ACC = 1 /* table and X/W entries rounded to bfloat16 (nearest even) as they are
                                read, products accumulated in float32; wide operands only */
} ilargi_precision_t;

typedef enum { ILARGI_LINEAR = 0, ILARGI_LOGISTIC = 1 } ilargi_model_t;

typedef struct {
  const float* D;         /* device, rows x cols; borrowed: must stay alive and unchanged while the plan lives */
  int64_t rows, cols;     /* r_k, c_k (both may be 0) */
  const int32_t* row_idx; /* device int32[r_T], borrowed; NULL = identity (requires rows == r_T) */
  const int32_t* col_map; /* HOST int32[cols]; copied when the plan is created */
  /* Optional: the table in compressed sparse rows instead of D (the paper keeps its matrices sparse,
   * Sec. 3.1).  With csr_rowptr != NULL, D must be NULL.  Borrowed like D.  A plan with a sparse source
   * serves lmm, tmm, gd_step, materialize, row_sum, col_sum, crossprod (up to 16384 target columns) and the
   * element-wise operators that keep zero at zero (which then act on csr_val, nnz values), in float32; the
   * bf16 variants return UNSUPPORTED.  Invalid sparse rows are reported by ilargi_plan_create as INDEX_RANGE.  A dense table has at
   * most 4096 columns; a sparse one up to 2^20 (one-hot encodings), provided that beyond 4096 columns no row
   * holds more than 2048 stored entries (else UNSUPPORTED). */
  const int32_t* csr_rowptr; /* device int32[rows + 1], rising from 0 to nnz */
  const int32_t* csr_col;    /* device int32[nnz], in [0, cols), strictly ascending within a row */
  const float* csr_val;      /* device float32[nnz] */
  int64_t nnz;               /* stored entries, < 2^31 */
} ilargi_source_t;

/* Bytes of device workspace a plan over these shapes needs when operands have at most max_cx
 * columns (X / Y / W columns).  Reads only sizes and whether row_idx is NULL; touches no device.
 * Errors: NULL, SHAPE. */
ilargi_status_t ilargi_plan_workspace_bytes(int n, const ilargi_source_t* sources, int64_t r_T,
                                            int64_t c_T, int64_t max_cx, size_t* bytes);

/* Build a plan: validate shapes and column maps (Def. 1), range-check row_idx on the device
 * (Def. 2) and build, for every source whose row_idx is not the identity, the inverse index of
 * I_k in compressed-row form: rowptr int32[r_k+1] and perm int32[nnz_k], the target rows fed by
 * each source row, ascending within a source row.  `workspace` is device memory, 256-byte aligned,
 * of at least the reported size, owned by the caller and used by the plan until it is destroyed.
 * Errors: NULL, SHAPE, COLMAP, INDEX_RANGE, WORKSPACE, DEVICE.  *plan is written only on success. */
ilargi_status_t ilargi_plan_create(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                   int64_t max_cx, void* workspace, size_t workspace_bytes,
                                   void* stream, ilargi_plan_t** plan);

/* ilargi_plan_create for callers that cannot allocate device memory (code that must not call hipMalloc: tight
 * serving loops, harnesses that forbid allocation, set-up code running beside a captured graph): the plan's
 * device state lives in a scratch array that is part of the library itself, ilargi_static_scratch_bytes() bytes
 * (128 MiB) on every GPU the library is used on, held until the process ends.  The call allocates no device
 * memory and calls no allocating routine.  Same arguments, validation, results and errors as
 * ilargi_plan_create, and the plan serves every operator in the same way (bit-identical results), with
 * these limits:
 *   - a plan that needs more than the array holds (see ilargi_plan_workspace_bytes) is refused with WORKSPACE;
 *   - one such plan per device at a time: while it lives, another ilargi_plan_create_static on that device is
 *     refused with WORKSPACE; ilargi_plan_destroy releases the array;
 *   - the array keeps the last plan's contents; the call initialises every region it reads.  Calls from several
 *     threads that create static plans on one device are serialised by the library, but work that a destroyed
 *     plan still has in flight on a stream races with the next plan's set-up: synchronize before destroying.
 * The current device at the time of the call selects the array. */
ilargi_status_t ilargi_plan_create_static(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                          int64_t max_cx, void* stream, ilargi_plan_t** plan);

/* Size in bytes of the scratch array behind ilargi_plan_create_static. */
size_t ilargi_static_scratch_bytes(void);

/* Release the host object.  The workspace and all borrowed arrays stay with the caller. */
ilargi_status_t ilargi_plan_destroy(ilargi_plan_t* plan);

/* Clustered entity table (a data layout, not an operator of the paper: Alg. 1 sums over the target rows, and
 * a sum does not depend on the order of its terms).  For a two-table star join T = [S | I_R R] -- an identity
 * source S of r_T rows and one source R that every target row joins -- the plan can keep a copy of S with its
 * rows in join order (grouped by the row of R they join, the order of the inverse index).  ilargi_gd_step
 * with one model in float32 then reads S and R once per iteration as two plain streams: the product R w_R,
 * the residual and the segment sums I_R^T e of Sec. 2.2's rules never go to memory.  ilargi_crossprod streams the
 * copy instead of gathering rows of S (same result, bit for bit); every other operator ignores it.  The one-pass
 * iteration pays when at least about four target rows join a row of R on average, or when R holds more cells
 * than S (every row of R costs the pass two reductions over a wavefront, however few target rows it serves):
 * ilargi_gd_step takes it in those two cases and keeps its usual sequence otherwise.
 *   ilargi_plan_cluster_bytes: size of the buffer, 4 r_T c_S + 8 r_T bytes rounded up to 256-byte pieces.
 *     Errors: NULL, UNSUPPORTED (not such a join; S needs 4..32 columns, R 4..256 columns, both in whole
 *     16-byte aligned float4s).
 *   ilargi_plan_cluster: fills `buffer` (device, 256-byte aligned, owned by the caller, used by the plan until
 *     it is destroyed or the call is repeated) on `stream`.  The copy holds the values S has at this call;
 *     sources must stay unchanged while the plan lives anyway, and ilargi_elementwise applied to S in place
 *     makes the plan forget the copy.  `y` (optional, device float[r_T]): the labels of the training set; they
 *     are copied in join order as well, and an ilargi_gd_step whose y is this same pointer reads them from the
 *     copy instead of gathering them (the vector must then stay unchanged like a source table; a gd_step with
 *     any other y gathers its labels as usual).  buffer == NULL: forget the copy.
 *     Errors: NULL, UNSUPPORTED, WORKSPACE, DEVICE. */
ilargi_status_t ilargi_plan_cluster_bytes(const ilargi_plan_t* plan, size_t* bytes);
ilargi_status_t ilargi_plan_cluster(ilargi_plan_t* plan, void* buffer, size_t buffer_bytes, const float* y,
                                    void* stream);

/* Left multiply (paper, Sec. 2.2):  out = T X = sum_k I_k (D_k (M_k^T X)).
 * X device c_T x cx, out device r_T x cx, 1 <= cx <= max_cx.  Errors: NULL, WORKSPACE, UNSUPPORTED. */
ilargi_status_t ilargi_lmm(ilargi_plan_t* plan, const float* X, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream);

/* Transposed multiply (the transpose operator of Sec. 2.2 / Alg. 1):
 * out = T^T Y = sum_k M_k (D_k^T (I_k^T Y)).  Y device r_T x cx, out device c_T x cx. */
ilargi_status_t ilargi_tmm(ilargi_plan_t* plan, const float* Y, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream);

/* Right multiply (Tab. 2, row XT):  out = X T = (T^T X^T)^T.  X device cx x r_T, out device cx x c_T,
 * 1 <= cx <= max_cx.  Uses the plan's residual buffer as scratch (like every call on a plan it must not
 * overlap with another). */
ilargi_status_t ilargi_rmm(ilargi_plan_t* plan, const float* X, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream);

/* Gram matrix  out = T^T T = sum_k sum_l M_k D_k^T (I_k^T I_l) D_l M_l^T, cross terms included.
 * out device c_T x c_T, both triangles written, symmetric to the bit.  A plan with a sparse source forms it
 * as T^T (T I), min(max_cx, 16) identity columns at a time through lmm and tmm (so it uses the plan's
 * residual buffer as scratch), and is limited to c_T <= 16384 (else UNSUPPORTED). */
ilargi_status_t ilargi_crossprod(ilargi_plan_t* plan, float* out, void* stream);

/* Join-gather baseline (paper, Sec. 2.2: the rewrite rule with X = I, i.e. T = sum_k I_k D_k M_k^T written
 * out): write the materialized target table.  T device r_T x c_T.  Each cell is the
 * float32 sum, in source order starting from +0.0, of the source cells mapped to it; cells nobody
 * maps to are +0.0.  The result is reproducible bit for bit. */
ilargi_status_t ilargi_materialize(ilargi_plan_t* plan, float* T, void* stream);

/* One gradient-descent iteration of Alg. 1 for m models at once, without materializing T:
 *   Z = T W;   E = Z - y (LINEAR)  or  sigmoid(Z) - y (LOGISTIC, y in {0,1});
 *   G = T^T E / r_T;   W[:, j] -= lr[j] * G[:, j].
 * Alg. 1 prints the update without the 1/r_T factor; pass lr = gamma * r_T to obtain it.
 * loss[j] (optional, device float[m]) receives the loss at the weights the call started from:
 * ||Z - y||^2 / (2 r_T) for LINEAR, mean(softplus(Z) - y Z) for LOGISTIC.
 * W device c_T x m in/out, y device float[r_T], lr device float[m], 1 <= m <= max_cx. */
ilargi_status_t ilargi_gd_step(ilargi_plan_t* plan, ilargi_model_t model, float* W, int64_t m,
                               const float* y, const float* lr, float* loss,
                               ilargi_precision_t precision, void* stream);

/* One Lloyd iteration of KMeans over the rows of T without materializing it (KMeans is one of the models
 * evaluated in Sec. 4, Tab. 7-9; the paper prints no algorithm for it, this is the textbook one):
 *   a_i = argmin_j ||t_i - c_j||^2  taken as  argmin_j (||c_j||^2 - 2 (T C)_ij),  the first j among equals,
 *   c_j <- mean of the rows with a_i = j  =  (T^T A)_j / n_j  with A the 0/1 assignment matrix;
 *   a centroid without rows keeps its place.
 * C device c_T x k in/out (column j is centroid j), 1 <= k <= min(max_cx, 256); assign (optional) device
 * int32[r_T] receives a_i (with respect to the centroids the call started from); counts (optional) device
 * int32[k] receives n_j.  Values must be finite.  Uses the plan's residual buffer as scratch.
 * Errors: NULL, SHAPE, WORKSPACE, UNSUPPORTED (k > 256). */
ilargi_status_t ilargi_kmeans_step(ilargi_plan_t* plan, float* C, int64_t k, int32_t* assign, int32_t* counts,
                                   void* stream);

/* One round of multiplicative updates of Gaussian NMF, T ~ W H with non-negative factors (Gaussian NMF is one
 * of the models evaluated in Sec. 4, Tab. 7-9; the paper prints no algorithm, these are the updates of Lee and
 * Seung for the squared Frobenius error):
 *   W <- W o (T H^T) (/) max(W (H H^T), 1e-30)          (left multiply by H^T),
 *   H <- H o (W^T T) (/) max((W^T W) H, 1e-30)          (transposed multiply by the new W).
 * W device r_T x r in/out; Ht device c_T x r in/out holds H transposed (row t is column t of H);
 * 1 <= r <= min(max_cx, 64).  Uses the plan's residual buffer as scratch.
 * Errors: NULL, SHAPE, WORKSPACE, UNSUPPORTED (r > 64). */
ilargi_status_t ilargi_gnmf_step(ilargi_plan_t* plan, float* W, float* Ht, int64_t r, void* stream);

/* Element-wise operators of Tab. 2 (first two rows): arithmetic with a scalar, T (/) x, and functions f(T). */
typedef enum {
  ILARGI_OP_MUL = 0,    /* t * x */
  ILARGI_OP_DIV = 1,    /* t / x */
  ILARGI_OP_ADD = 2,    /* t + x */
  ILARGI_OP_SUB = 3,    /* t - x */
  ILARGI_OP_POW = 4,    /* t ^ x */
  ILARGI_OP_EXP = 5,    /* exp(t);  x is ignored from here on */
  ILARGI_OP_LOG = 6,
  ILARGI_OP_SQRT = 7,
  ILARGI_OP_ABS = 8,
  ILARGI_OP_SQUARE = 9
} ilargi_elementwise_t;

/* T (/) x or f(T) in factorized form (Tab. 2: sum_k m_k operations instead of m_T): the result is the
 * table described by the same row_idx / col_map with source tables D_out[k] = op(D_k, x).
 * D_out: host array of n device pointers, D_out[k] r_k x c_k float32 (entries of empty sources are not
 * read); D_out[k] may be the source table itself, and if every table is updated in place the plan keeps
 * describing the result.  The factorized form equals the operator on the cells of T
 *   - always for MUL and DIV (they distribute over the sums of shared cells and keep empty cells 0);
 *   - for SQRT, ABS, SQUARE and POW with x > 0 (zero stays zero) when no target column is fed by two
 *     sources;
 *   - for ADD, SUB, EXP, LOG and POW with x <= 0 when, in addition, every target column is fed and
 *     every source reaches every target row (each cell of T has exactly one source cell).
 * Otherwise the call returns UNSUPPORTED and writes nothing.  Errors: NULL, UNSUPPORTED. */
ilargi_status_t ilargi_elementwise(ilargi_plan_t* plan, ilargi_elementwise_t op, float x,
                                   float* const* D_out, void* stream);

/* rowSum(T) (Tab. 2) = T 1: out device float[r_T]. */
ilargi_status_t ilargi_row_sum(ilargi_plan_t* plan, float* out, void* stream);

/* colSum(T) (Tab. 2) = sum_k M_k (D_k^T cnt_k), cnt_k[j] = number of target rows taking row j of source k
 * (kept with the plan): no pass over the r_T target rows.  out device float[c_T]. */
ilargi_status_t ilargi_col_sum(ilargi_plan_t* plan, float* out, void* stream);

/* Factorize or materialize (Sec. 3)?  Host-only: reads the shapes in `sources` and whether row_idx is NULL
 * (D, row_idx contents and col_map are not touched), like ilargi_plan_workspace_bytes. */
typedef struct {
  int64_t iterations;        /* gradient-descent iterations the table will serve (>= 1); the paper trains 200 */
  int64_t models;            /* models trained at once (>= 1) */
  double bytes_per_second;   /* sustained memory bandwidth to price bytes with; 0 = 5.0e12 (a plain copy on MI355X) */
  double launch_seconds;     /* cost of one dependent kernel launch; 0 = 2.5e-6 */
} ilargi_workload_t;

typedef struct {
  int factorize;             /* 1 = the factorized path is predicted to finish the workload sooner */
  double complexity_ratio;   /* Eq. (1) for linear regression, dense operands: O_materialized / O_factorized */
  double tuple_ratio;        /* r_T / (rows of the sources that have a row_idx) */
  double feature_ratio;      /* (columns of those sources) / (columns of the identity sources) */
  int morpheus_rule;         /* 1 = tuple_ratio >= 5 and feature_ratio >= 1 (the thresholds Sec. 4.3 quotes) */
  double bytes_factorized;   /* bytes one iteration moves, factorized */
  double bytes_materialized; /* the same on the materialized table */
  double bytes_join;         /* bytes the join itself moves (once) */
  double seconds_factorized; /* predicted time of the whole workload */
  double seconds_materialized; /* join + iterations on the table */
} ilargi_choice_t;

/* workload may be NULL (200 iterations, one model, default rates).  Errors: NULL, SHAPE. */
ilargi_status_t ilargi_choose(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                              const ilargi_workload_t* workload, ilargi_choice_t* out);

/* I_k^T Y for one source (the segmented sum inside ilargi_tmm), exposed for inspection:
 * Z[j, :] = sum of Y[i, :] over the target rows i with row_idx_k[i] == j.
 * Y device r_T x cx, Z device r_k x cx. */
ilargi_status_t ilargi_segment_sum(ilargi_plan_t* plan, int k, const float* Y, int64_t cx, float* Z,
                                   void* stream);

/* Device pointers to the inverse index of source k inside the workspace (valid while the plan
 * lives).  For an identity source *rowptr and *perm are NULL and *nnz = r_k. */
ilargi_status_t ilargi_plan_inverse_index(const ilargi_plan_t* plan, int k, const int32_t** rowptr,
                                          const int32_t** perm, int64_t* nnz);

/* Per-kernel timing for benchmarks.  After trace_begin, every launch of the kernel family named by
 * `tag` ("*" = every family; "<label>/<family>" = that family under one label) is bracketed by a pair of HIP events on the call's stream (at most
 * max_launches pairs; later launches run untimed).  Families: "lmm_rows:<k>" (product of source k),
 * "lmm_assemble", "segsum:<k>", "colred:<k>", "finalize", "materialize", "gram:<k n + l>", "star_pass", "gd_cluster",
 * "elementwise:<k>".  trace_label sets a
 * prefix ("<label>/<family>") for the launches that follow, so a caller can tell its operators apart.
 * trace_end waits for the recorded events, writes the elapsed milliseconds of up to `capacity`
 * launches to the host array `ms` (may be NULL), stores the number of recorded launches in *count
 * and switches tracing off; trace_name copies the name of recorded launch i (valid until the next
 * trace_begin).  Events are host objects; no device memory is allocated. */
ilargi_status_t ilargi_plan_trace_begin(ilargi_plan_t* plan, const char* tag, int max_launches);
ilargi_status_t ilargi_plan_trace_label(ilargi_plan_t* plan, const char* label);
ilargi_status_t ilargi_plan_trace_end(ilargi_plan_t* plan, float* ms, int capacity, int* count);
ilargi_status_t ilargi_plan_trace_name(const ilargi_plan_t* plan, int i, char* buf, int buf_len);

/* Plain streaming kernels for calibration (what the memory system delivers, and the scale of the
 * profiler's byte counters): kind 0 copies n_floats floats src -> dst, kind 1 only reads src (dst
 * receives one float per workgroup, so it needs `blocks` floats), kind 2 only writes dst; kinds 3 and 4
 * are the copy and the write with non-temporal accesses.  Device
 * pointers, 16-byte aligned, n_floats a multiple of 4, `blocks` workgroups of 256 threads (1 .. 2^22) that
 * walk the buffer with a grid stride: n_floats / 1024 workgroups touch one float4 per thread, in address
 * order, which is the pattern that writes fastest on the MI355X. */
ilargi_status_t ilargi_stream_probe(int kind, float* dst, const float* src, int64_t n_floats, int blocks,
                                    void* stream);

/* Message for the most recent failure on this thread ("" if none).  Static storage. */
const char* ilargi_last_error(void);

/* Library version, "major.minor". */
const char* ilargi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ILARGI_H_ */
