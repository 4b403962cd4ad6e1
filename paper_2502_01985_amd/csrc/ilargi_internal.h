// Internal declarations shared by the translation units of libilargi (not installed).
#ifndef ILARGI_INTERNAL_H_
#define ILARGI_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ilargi.h"

namespace ilargi {

constexpr int kMaxPairLists = 4;     // pair lists of crossprod a plan holds (source pairs joined row by row)
constexpr int kMaxSources = 16;      // sources per plan (kernel argument arrays are this long)
constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kBlock = 256;          // threads per workgroup in the streaming kernels
constexpr int kNarrowCT = 4;         // operand columns one narrow (VALU) pass handles
constexpr int kColredBlocks = 1024;  // most row chunks (= partial results) of the D^T Z reduction
constexpr int kColredTarget = 512;   // row chunks aimed at: two workgroups per compute unit, eight loads in flight per lane
constexpr int kSparseBlockRows = 1024;   // rows a row block of the sparse row-wise product holds at most
constexpr int kSparseChunk = 4096;   // entries of a column one workgroup sums
constexpr int kSegSlices = 8;        // slices of target rows of the sliced segment sum (one per XCD and its L2)
constexpr int kSlLong = 256;         // ... runs of a (slice, source row) longer than this are cut into chunks
constexpr int kSlChunk = 1024;       // ... of this many entries, each summed by a whole workgroup
constexpr int kLongSeg = 2048;       // inverse-index segments longer than this are split ...
constexpr int kSegChunk = 2048;      // ... into chunks of this many entries
constexpr int kSortChunk = 2048;     // keys per workgroup in one radix pass
constexpr int kMaxLdsFloats = 4096;  // 16 KiB of LDS for the staged operand rows (also the column limit of a source)
constexpr int64_t kGramPartialFloats = 16ll << 20;

// Row gathers of per-source products:  out[i,:] += P_s[row_s(i), :]  (assembly step of Sec. 2.2).
struct GatherArgs {
  int n;
  const int32_t* idx[kMaxSources];  // NULL: identity on the first rows[s] target rows
  const float* P[kMaxSources];
  int64_t rows[kMaxSources];
  int ldp;
};

struct LmmArgs {
  const float* D;         // fused identity-prefix source (may be NULL)
  int64_t d_rows;         // target rows [0, d_rows) take row i of D
  int ck;                 // columns of D
  const int32_t* colmap;  // device int32[ck]
  const float* X;         // c_T x ldx
  int ldx, col0, ncols;   // operand columns [col0, col0 + ncols)
  float* out;             // r_out x ldo
  int ldo;
  int64_t r_out;
  int logL;               // lanes per row = 1 << logL
  GatherArgs g;
  // gradient-descent modes
  const float* y;         // labels, r_out
  float* loss_partial;    // narrow kernel: [gridDim.x][kNarrowCT]; matrix-core kernel: [gridDim.x][ld_loss]
  int ld_loss;
  int nt_out;             // store the output with non-temporal stores (large results nobody re-reads soon)
  float* scratch;         // optional device scratch of scratch_floats floats (the caller's, free for the launch)
  int64_t scratch_floats;
  float* grad_partial;    // optional partials of D^T e: narrow kernel [gridDim.x][ck][kNarrowCT],
                          // matrix-core kernel [gridDim.x][ck][ld_grad]
  int ld_grad;
};

// Tile shape of the matrix-core left multiply for a table with ck columns.
struct MfmaShape {
  int kp;            // ck rounded up to a multiple of 16
  int kc;            // table columns staged per step
  int lda;           // LDS row stride of the staged rows (floats)
  int rb;            // table rows per workgroup step
  size_t lds_bytes;
};

// A source table in compressed sparse rows with its column-sorted view (kernels_sparse.hip).
struct SparseArgs {
  const int32_t* rowptr;   // rows + 1
  const int32_t* col;      // nnz, strictly ascending within a row
  const float* val;        // nnz
  int64_t rows, nnz;
  int cols;
  const int32_t* colmap;   // device int32[cols]
  const int32_t* row_block;  // n_row_blocks + 1: runs of whole rows with at most sparse_row_block_cap(cols) entries
  int n_row_blocks;
  // column-sorted view, built with the plan
  const int32_t* csc_row;  // nnz: row of the p-th entry in column order
  const float* csc_val;    // nnz: its value
  const int32_t* chunk_beg, *chunk_end;   // n_chunks ranges of that order, each inside one column
  const int32_t* col_first_chunk;         // cols + 1
  int n_chunks;
};

// Gradient-descent pass over a two-table star join for a wide batch of models (kernels_star.hip).
struct StarArgs {
  const float* S;            // r_T x cs, row i of S is target row i
  int cs;
  const int32_t* s_colmap;   // device int32[cs]
  const float* W;            // c_T x ldw
  int ldw, m;
  float* PZ;                 // r_R x ldp: in  P = R W_R,  out  Z = segment sums of the residual
  int ldp;
  int64_t r_R;
  const int32_t* rowptr;     // r_R + 1: inverse index of the dimension table (every target row joins one row)
  const int32_t* perm;       // r_T
  const int32_t* idx;        // r_T: row of R each target row joins
  const float* y;            // r_T
  const float* Sp;           // NULL, or S with its rows in join order (Sp[p, :] = S[perm[p], :]) ...
  const int32_t* keys;       // ... with the row of R each of those rows joins, r_T ...
  const float* yp;           // ... and, if not NULL, their labels, r_T
  float* loss_partial;       // [gridDim.x][ld_loss]
  int ld_loss;
  float* grad_partial;       // [gridDim.x][cs][ld_grad] partials of S^T E
  int ld_grad;
};

// The entity table's share of the Gram matrix of a two-table star join, one pass in join order
// (kernels_gram_star.hip).
struct GramStarArgs {
  const float* S; int cs;            // r_T x cs, row i of S is target row i
  int64_t r_R;                       // rows of the dimension table
  const int32_t* rowptr;             // r_R + 1: inverse index of R (every target row joins one row)
  const int32_t* perm;               // r_T
  const int32_t* idx;                // r_T: row of R each target row joins
  const float* Sp;                   // NULL, or S with its rows in join order (Sp[p, :] = S[perm[p], :]): then a plain stream
  float* ss_partial;                 // [gridDim.x][cs][cs] partials of S^T S (upper-triangle 16 x 16 tiles)
  float* zc;                         // r_R x cs: rows of S summed per row of R
};

// Join-order transposed multiply of one joined source (kernels_tmm_join.hip).
struct TmmJoinArgs {
  const float* D; int ck;            // r_k x ck source table
  int64_t r_k;
  const int32_t* rowptr;             // r_k + 1: inverse index
  const int32_t* perm;               // target rows in source-row order
  const float* Y; int ldy, col0, c;  // operand columns [col0, col0 + c), c <= 16
  float* partial;                    // [gridDim.x][ck][c]
};

struct SegArgs {
  const int32_t* rowptr;   // r_k + 1
  const int32_t* perm;     // nnz
  const int32_t* chunk_seg, *chunk_beg, *chunk_end;  // long-segment chunks
  const int32_t* long_seg, *long_first;              // long segments and their chunk ranges
  int n_chunks, n_long;
  int64_t r_k;
  const float* Y;          // rows addressed through perm (and gidx if given)
  int ldy, col0, ncols;
  const int32_t* gidx;     // optional second-level gather: Y row = gidx[perm[p]] (skip if < 0)
  int64_t g_rows;          // with gidx == NULL and g_rows >= 0: rows >= g_rows are skipped
  float* Z;                // r_k x ldz
  int ldz, zcol0;
  float* chunk_partial;    // n_chunks x ncols
  int logG;                // lanes per segment in the narrow kernel
  const int32_t* block_first;  // join-order column reduce: workgroup b owns source rows [block_first[b], block_first[b + 1])
  // sliced form (large target tables): a second copy of the index ordered by (slice of target rows, source row)
  const int32_t* sl_rowptr;    // [kSegSlices * r_k + 1] entries of (slice x, source row j) are sl_perm[sl_rowptr[x r_k + j] ..)
  const int32_t* sl_perm;      // NULL: no sliced index
  const int32_t* sl_chunk0;    // [kSegSlices][r_k] first chunk record of a run longer than kSlLong, else -1
  const int32_t* sl_ch_beg, *sl_ch_end;   // [kSegSlices][sl_cap] chunk records: ranges of sl_perm
  const int32_t* sl_nchunk;    // [kSegSlices] their number
  float* sl_ch_partial;        // [kSegSlices][sl_cap][CT] chunk sums
  int sl_cap, sl_logG;
  float* Zs;                   // [kSegSlices][r_k][CT] per-slice sums of the short runs
};

// Plain per-source products P_k = D_k (M_k^T X) of several sources in one launch (kernels_lmm.hip).
constexpr int kRowdotMulti = 4;
struct RowdotArgs {
  const float* D; int ck; int64_t rows;
  const int32_t* colmap;
  const float* X; int ldx, col0, ncols;
  float* out; int ldo;
  int logL, vw;                // lanes per row (log2), floats per vector load (4 or 2)
};
struct RowdotMulti {
  int n;
  int first[kRowdotMulti + 1];
  RowdotArgs a[kRowdotMulti];
};

// Sliced segment sums of several sources in one launch (kernels_tmm.hip).
constexpr int kSegMulti = 4;
struct SegMulti {
  int n;
  int first[kSegMulti + 1];    // workgroups [first[q], first[q + 1]) of the sum kernel serve source q (multiples of kSegSlices)
  int cfirst[kSegMulti + 1];   // ... of the kernel that adds the per-slice sums
  SegArgs s[kSegMulti];
};

struct ColredArgs {
  const float* D;
  int64_t rows;
  int ck;
  const float* Z;          // rows x ldz
  int ldz, col0, ncols;
  float* partial;          // [nblocks][ck][kNarrowCT]
  int64_t rows_per_block;
  int vec;
};

// Shares of a narrow transposed multiply that run in one launch (kernels_tmm.hip).
constexpr int kTmmParts = 4;
struct TmmParts {
  int n;
  int first[kTmmParts + 1];   // workgroups [first[q], first[q + 1]) serve part q
  int join[kTmmParts];        // 1: join-order form (segment sums in LDS), 0: operand rows read from c.Z
  ColredArgs c[kTmmParts];
  SegArgs s[kTmmParts];       // inverse index and operand of the join-order form
};

struct FinSource {
  const int32_t* tcol2src;  // c_T
  const float* partial;     // [nblocks][ck][kNarrowCT]
  int nblocks, ck;
};

struct FinArgs {
  int n;
  FinSource s[kMaxSources];
  float* out;  // c_T x ldo (or W for the update mode)
  int ldo, col0, ncols;
  // update mode
  const float* lr;
  float inv_rT;
  const float* loss_partial;
  int n_loss_partial;
  float* loss;
  float loss_scale;
};

struct MatArgs {
  int n;
  const float* D[kMaxSources];
  const int32_t* idx[kMaxSources];
  const int32_t* tcol2src[kMaxSources];
  int64_t rows[kMaxSources];
  int ck[kMaxSources];
  float* T;
  int64_t r_T;
  int c_T;
  // optional tables for the vectorized form: per group of four target columns the feeding source slot
  // (-1: nobody) and its first source column; NULL when some group is fed irregularly
  const int32_t* gslot;
  const int32_t* gj0;
  int flat_ok;   // every fed group is four 16-byte-aligned values of its source (tables narrower than 4096 columns)
  // optional tables for the column form: for target column t the (up to two) feeding source slots
  // ct_slot[2t], ct_slot[2t+1] (-1: none) in source order and their source columns ct_j[2t], ct_j[2t+1];
  // NULL when some column has more than two feeders
  const int32_t* ct_slot;
  const int32_t* ct_j;
};

// Transposed reduction  C = sum_t w_t a_t^T b_t  on the matrix cores (see kernels_tred.hip).
struct TredArgs {
  const float* A; int lda, ca; const int32_t* ia; int64_t a_rows;   // row t of A = A[ia ? ia[t] : t]
  const float* B; int ldb, cb, bcol0; const int32_t* ib; int64_t b_rows;
  const int32_t* wptr;     // optional: w_t = wptr[t+1] - wptr[t]
  int64_t n_rows, rows_per_block;
  float* partial;          // [row chunk][ca][cb]
  int gx, gy;              // set by launch_tred: row chunks and output tiles of the launch (see tred_block_ids)
  int upper_only;          // A == B: only tiles touching the upper triangle are computed
};

struct ColAsmArgs {
  int n;
  const int32_t* tcol2src[kMaxSources];
  const float* G[kMaxSources];   // c_k x cx each; with nparts[k] > 1: that many such blocks, to be added in order
  int nparts[kMaxSources];       // (0 counts as 1)
  int ck[kMaxSources];
  int c_T, cx;
  float* out;                    // c_T x cx
  const float* lr;
  float inv_rT;
  const float* loss_partial;     // [n_loss_partial][cx]
  int n_loss_partial;
  float* loss;
  float loss_scale;
};

struct GramAsmPair { const float* block; int k, l, cb; };

// Records `msg` as the calling thread's last error (what ilargi_last_error returns) and returns `code`.
ilargi_status_t set_error(ilargi_status_t code, const char* msg);

// One gradient-descent iteration on a small two-table star join in a single workgroup (kernels_small.hip).
constexpr size_t kSmallGdMaxLds = 152 << 10;    // dynamic LDS the kernel may use (of the 160 KiB of a compute unit)
struct SmallStarArgs {
  const float* S; int cs;       // entity table r_T x cs: cs <= 16, a multiple of 4, 16-byte aligned
  const float* R; int cr, r_R;  // joined table (NULL: none), r_R <= 1024 rows, cr <= 16
  const int32_t* idx;           // r_T keys into R (-1: none)
  const int32_t* rowptr;        // inverse index of R
  const int32_t* perm;
  int nnz;
  const int32_t* tcol_s;        // device int32[c_T]: column of S feeding target column t, or -1
  const int32_t* tcol_r;
  int16_t colmap[2][16];        // target column of every column of S and of R, or -1
  int s_first;                  // S comes before R in the plan (order of the sums in shared target columns)
  float* W; int ldw, col;       // weight column `col` of the c_T x ldw matrix, updated in place
  const float* y; const float* lr; float* loss;
  int r_T, c_T;
  float inv_rT, loss_scale;
};
int small_star_max_rows(int nvs);
size_t small_star_lds_bytes(const SmallStarArgs& a);
hipError_t launch_small_star(const SmallStarArgs& a, int mode, hipStream_t st);

// Gradient-descent pass that joins the rows of its sources on the fly in target order (kernels_rowjoin.hip).
constexpr int kRowJoinSources = 3;
struct RowJoinArgs {
  int n;                                    // sources, 1 .. kRowJoinSources
  const float* D[kRowJoinSources];          // rows[s] x ck[s], 16-byte aligned, ck a multiple of 4, at most 64
  int ck[kRowJoinSources];
  int64_t rows[kRowJoinSources];
  const int32_t* idx[kRowJoinSources];      // r_T row indices (-1: none); NULL: identity on the first rows[s] target rows
  const int32_t* colmap[kRowJoinSources];   // device int32[ck]
  const float* W; int ldw, col;             // weight column `col` of the c_T x ldw matrix
  const float* y; int64_t r_T;
  float* loss_partial;                      // [gridDim.x][kNarrowCT]
  float* grad_partial[kRowJoinSources];     // [gridDim.x][ck][kNarrowCT] partials of D_s^T e
};
bool gd_rowjoin_supported(const RowJoinArgs& a);
hipError_t launch_gd_rowjoin(const RowJoinArgs& a, int mode, int max_grid, hipStream_t st, int* grid_out);

// Gradient-descent pass of one model over a two-table star join whose entity table is kept in join order
// (kernels_gd_cluster.hip): both tables are read once, no product, residual or segment sum is stored.
struct ClusterArgs {
  const float* Sp; int cs;                  // the entity table with its rows in join order, r_T x cs, 16-byte aligned
  const int32_t* keys;                      // int32[r_T], ascending: the row of the dimension table each of those rows joins
  const int32_t* perm;                      // int32[r_T]: its target row (where its label is)
  const float* R; int cr; int64_t r_R;      // dimension table, r_R x cr, 16-byte aligned, cr a multiple of 4, at most 256
  const int32_t* s_colmap;                  // device int32[cs], int32[cr]: target column of every table column (-1: none)
  const int32_t* r_colmap;
  const float* W; int ldw, col;             // weight column `col` of the c_T x ldw matrix
  const float* y; int64_t r_T;
  const float* yp;                          // the labels in join order, float[r_T], or NULL (then y is gathered through perm)
  float* loss_partial;                      // [gridDim.x][kNarrowCT]
  float* grad_partial_s;                    // [gridDim.x][cs][kNarrowCT] partials of S^T e
  float* grad_partial_r;                    // [gridDim.x][cr][kNarrowCT] partials of R^T (I_R^T e)
};
bool gd_cluster_supported(int cs, int cr);
// Sp[p, :] = S[perm[p], :], keys[p] = idx[perm[p]] and, with labels y, yp[p] = y[perm[p]] for p < r_T.
hipError_t launch_cluster_rows(const float* S, int cs, const int32_t* perm, const int32_t* idx, int64_t r_T, float* Sp,
                               int32_t* keys, const float* y, float* yp, hipStream_t st);
hipError_t launch_gd_cluster(const ClusterArgs& a, int mode, int max_grid, hipStream_t st, int* grid_out);

// ---- launchers (each enqueues on `st`; returns the HIP error of the launch) ----
hipError_t launch_check_idx(const int32_t* idx, int64_t r_T, int64_t r_k, int32_t* flags, hipStream_t st);
hipError_t launch_sort_by_source_row(const int32_t* idx, int64_t r_T, int64_t r_k, int32_t* keys_a,
                                     int32_t* vals_a, int32_t* keys_b, int32_t* vals_b, int32_t* hist,
                                     int32_t* rowptr, int32_t* perm, hipStream_t st);
size_t sort_hist_ints(int64_t r_T);
// In-place exclusive prefix sum of n integers on the device; `totals` is scratch of ceil(n / 1024) integers.
void launch_exclusive_scan(int32_t* a, int64_t n, int32_t* totals, hipStream_t st);

hipError_t launch_lmm_rows(const LmmArgs& a, int vec, int mode, hipStream_t st, int* grid_out);
// Assembly with one lane per target row (kernels_lmm_lane.hip): one operand column, identity source with short rows.
bool lmm_lane_supported(const LmmArgs& a, int vec, int mode, bool fuseg);
hipError_t launch_lmm_lane(const LmmArgs& a, int vec, int mode, hipStream_t st, int* grid_out);
// The streaming product kernel: dense table, at most four operand columns, rows of aligned vectors of vec = 4 or 2
// floats; the products of up to kRowdotMulti sources (same operand columns) can share one launch.
bool rowdot_supported(const LmmArgs& a, int vec);
hipError_t launch_rowdot_multi(const LmmArgs* a, const int* vec, int n, hipStream_t st);
int lmm_grid(int64_t r_out, int logL, bool fuseg);
bool lmm_can_fuse_gradient(int ck, int vec, int logL);
MfmaShape lmm_mfma_shape(int ck, int nt, bool gathers, bool bf16);
bool lmm_mfma_can_fuse_gradient(int ck, int ncols, bool bf16);
hipError_t launch_lmm_mfma(const LmmArgs& a, int vec, int mode, bool bf16, hipStream_t st, int* grid_out);
bool lmm_flat_pair_supported(const LmmArgs& a, int vec, bool fuseg);
hipError_t launch_lmm_flat_pair(const LmmArgs& a, int mode, bool fuseg, hipStream_t st, int* grid_out);
bool lmm_prod_f32_wide_supported(const LmmArgs& a, int vec, int mode);
hipError_t launch_lmm_prod_f32_wide(const LmmArgs& a, hipStream_t st);
bool lmm_prod_bf16_supported(const LmmArgs& a, int vec, int mode);
hipError_t launch_lmm_prod_bf16(const LmmArgs& a, hipStream_t st);
bool lmm_prod_stream_supported(const LmmArgs& a, int vec, int mode);
hipError_t launch_lmm_prod_stream(const LmmArgs& a, hipStream_t st);
bool lmm_flat_wide_supported(const LmmArgs& a, int vec, int mode);
hipError_t launch_lmm_flat_wide(const LmmArgs& a, hipStream_t st, int* grid_out);
bool gd_star_supported(int cs, int m);
hipError_t launch_gd_star(const StarArgs& a, int vec, int mode, bool bf16, int max_grid, hipStream_t st, int* grid_out);
hipError_t launch_csr_check(const SparseArgs& a, int32_t* flags, hipStream_t st);
hipError_t launch_csr_entry_rows(const SparseArgs& a, int32_t* entry_row, hipStream_t st);
hipError_t launch_csr_gather_rows(const int32_t* entry_row, const float* val, const int32_t* perm, int64_t nnz,
                                  int32_t* csc_row, float* csc_val, hipStream_t st);
int sparse_row_block_cap(int cols);
hipError_t launch_spmm_rows(const SparseArgs& a, const float* X, int ldx, int col0, int ncols, float* P, int ldp,
                            hipStream_t st);
hipError_t launch_spmm_t(const SparseArgs& a, const float* Z, int ldz, int col0, int ncols, float* partial, float* G,
                         hipStream_t st);
hipError_t launch_mat_scatter(const SparseArgs* sparse, const float* D, int64_t rows, int ck, const int32_t* colmap,
                              const int32_t* idx, int64_t ident_rows, float* T, int64_t r_T, int c_T, hipStream_t st);
hipError_t launch_segsum(const SegArgs& a, hipStream_t st);
// Builds the sliced copy of an inverse index (see SegArgs): sl_rowptr, sl_perm, the chunk records of long runs.
// src_beg: scratch of kSegSlices * r_k integers; scan_scratch: of (kSegSlices * r_k + 1) / 1024 + 1 integers.
hipError_t launch_build_sliced_index(const int32_t* rowptr, const int32_t* perm, int64_t r_k, int64_t nnz, int64_t slice_rows,
                                     int32_t* sl_rowptr, int32_t* sl_perm, int32_t* sl_chunk0, int32_t* ch_beg, int32_t* ch_end,
                                     int32_t* sl_nchunk, int cap, int32_t* src_beg, int32_t* scan_scratch, hipStream_t st);
int64_t segsum_sliced_chunk_cap(int64_t nnz);
// n <= kSegMulti sources with the same number of operand columns; their sums and the sums over slices run as one
// launch each.
hipError_t launch_segsum_sliced(const SegArgs* a, int n, hipStream_t st);
hipError_t launch_colred(const ColredArgs& a, int nblocks, hipStream_t st);
bool lmm_flat_supported(const LmmArgs& a, int vec, bool fuseg);
hipError_t launch_lmm_flat(const LmmArgs& a, int mode, bool fuseg, hipStream_t st, int* grid_out);
hipError_t launch_finalize(const FinArgs& a, int c_T, int mode, hipStream_t st);
int colred_step_rows(int ck, int vec);
bool tmm_part_supported(const ColredArgs& c, const SegArgs* s);
hipError_t launch_tmm_parts(const TmmParts& t, hipStream_t st);
hipError_t launch_materialize(const MatArgs& a, hipStream_t st);
hipError_t launch_gram_assemble(const GramAsmPair* pairs_dev, int npairs, const int32_t* const* tcol2src_dev,
                                int c_T, float* out, hipStream_t st);
bool tmm_join_supported(int ck, int c);
hipError_t launch_tmm_join(const TmmJoinArgs& a, int64_t partial_floats, hipStream_t st, int* grid_out);
bool gram_star_supported(int cs);
hipError_t launch_gram_star(const GramStarArgs& a, int vec, int max_grid, hipStream_t st, int* grid_out);
// Gram blocks of tables with at most 64 columns as streaming matrix-core kernels (kernels_gram_narrow.hip): the
// diagonal block of a table with 36..64 columns, and the block of two tables over a list of row pairs.
bool gram_narrow_supported(const TredArgs& a);
bool gram_pairs_supported(const TredArgs& a);
hipError_t launch_gram_narrow(TredArgs& a, float* partial, int64_t partial_floats, hipStream_t st, int* nch_out);
hipError_t launch_pair_list(const int32_t* idx_a, int64_t rows_a, const int32_t* idx_b, int64_t rows_b, int64_t r_T,
                            int32_t* scan, int32_t* totals, int32_t* list_a, int32_t* list_b, hipStream_t st);
bool gram_sym_supported(const TredArgs& a);
hipError_t launch_gram_sym(TredArgs& a, float* partial, int64_t partial_floats, float* block, hipStream_t st);
hipError_t launch_tred(const TredArgs& a, int nchunks, bool bf16, hipStream_t st);
// streaming column reduce over plain rows (kernels_wide_bf16.hip): a.partial receives a.gx blocks of ca x cb
bool tred_stream_supported(const TredArgs& a);
int tred_stream_grid(const TredArgs& a, int64_t partial_floats);
hipError_t launch_tred_stream(TredArgs& a, int grid, bool bf16, hipStream_t st);
void tred_occupancy(const TredArgs& a, bool bf16, int* slots, int* tiles);
// G = S^T Y for an identity source with rows of at most 16 float4 and 5..16 operand columns (kernels_colred_flat.hip).
struct ColredFlatArgs {
  const float* S; int64_t rows; int nvec;   // rows x (4 nvec), 16-byte aligned
  const float* Y; int ldy; int c;           // operand rows 0 .. rows - 1, columns 0 .. c - 1
  float* partial;                           // [workgroup][4 nvec][c]
};
bool colred_flat_supported(const float* S, int64_t cols, int c);
hipError_t launch_colred_flat(const ColredFlatArgs& a, int64_t partial_floats, hipStream_t st, int* grid_out);
// The flat column reduce of an identity source and the join-order pass of a joined source (nnz_j index entries) in one
// launch; *grid_f and *grid_j workgroups leave partial blocks in f.partial and j.partial.
bool tmm_pair_supported(const ColredFlatArgs& f, const TmmJoinArgs& j);
hipError_t launch_tmm_pair(const ColredFlatArgs& f, const TmmJoinArgs& j, int64_t nnz_j, int64_t room_f, int64_t room_j,
                           hipStream_t st, int* grid_f, int* grid_j);
// tcols > 0: the summed (elems / tcols) x tcols matrix is written transposed
hipError_t launch_tred_reduce(const float* partial, int nchunks, int64_t elems, float* block, hipStream_t st, int tcols = 0);
hipError_t launch_colasm(const ColAsmArgs& a, int mode, hipStream_t st);
hipError_t launch_probe(int kind, float* dst, const float* src, int64_t n_floats, int blocks, hipStream_t st);
hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st);
hipError_t launch_fill(float* p, int64_t n, float v, hipStream_t st);
hipError_t launch_transpose(const float* in, int64_t rows, int64_t cols, float* out, hipStream_t st);
hipError_t launch_eye_block(float* E, int64_t rows, int w, int64_t j0, hipStream_t st);   // columns j0.. of the identity
hipError_t launch_mirror_upper(float* G, int64_t n, hipStream_t st);                      // lower triangle := upper
constexpr int64_t kSparseGramMaxCols = 16384;   // crossprod over sparse sources: the c_T x c_T result stays below 1 GiB
constexpr int kSparseGramWidth = 16;            // identity columns multiplied through per round
hipError_t launch_fanout(const int32_t* rowptr, int64_t rows, float* cnt, hipStream_t st);
hipError_t launch_elementwise(int op, const float* in, float* out, int64_t n, float x, hipStream_t st);
// KMeans / Gaussian NMF row-local steps (kernels_models.hip)
constexpr int kKmeansMaxK = 256;
constexpr int kGnmfMaxRank = 64;
hipError_t launch_centroid_norm(const float* C, int64_t c_T, int k, float* cn, hipStream_t st);
hipError_t launch_kmeans_assign(float* P, const float* cn, int64_t r_T, int k, int32_t* assign, int32_t* counts_partial,
                                int64_t partial_ints, int32_t* counts, hipStream_t st);
hipError_t launch_kmeans_update(float* C, const float* G, const int32_t* counts, int64_t c_T, int k,
                                int32_t* counts_out, hipStream_t st);
hipError_t launch_gnmf_update(float* X, const float* P, const float* Q, int64_t rows, int k, float tiny,
                              float* gram_partial, int64_t partial_floats, int* nparts_out, hipStream_t st);

inline int ilog2_ceil(int64_t v) { int l = 0; while ((1ll << l) < v) ++l; return l; }

}  // namespace ilargi
#endif
