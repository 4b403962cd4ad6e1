// Source tables in compressed sparse rows (the paper keeps its matrices sparse, Sec. 3.1, and sweeps the sparsity
// of the tables, Tab. 3).  A sparse source D_k = (rowptr, col, val) takes part in the same operators:
//   P_k = D_k X_k        row-wise: a group of lanes walks the entries of a row, X_k sits in LDS;
//   G_k = D_k^T Z_k      column-wise over a column-sorted view built with the plan (the stable sort that builds
//                        the inverse index of a row index, applied to the column indices): entries of a column
//                        are summed in row order, long columns in chunks combined in chunk order - no atomics;
//   join-gather          one pass per source over the target rows, sources in order, so every cell receives
//                        its terms in the order the dense kernels use.
// Operands have at most four columns per pass, as in the narrow dense kernels.
#include <algorithm>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

// flags[0] |= 1 when rowptr is not a non-decreasing map onto [0, nnz], a column index is out of range or the
// column indices of a row do not ascend strictly (no cell twice).  The first pass only reads rowptr, so the
// second never follows a row pointer outside [0, nnz].
__global__ __launch_bounds__(kBlock) void csr_check_kernel(const int32_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ col, int64_t rows,
                                                           int64_t cols, int64_t nnz, int32_t* __restrict__ flags) {
  const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, nt = (int64_t)gridDim.x * blockDim.x;
  bool bad = false;
  for (int64_t r = t0; r < rows; r += nt) {
    const int64_t b = rowptr[r], e = rowptr[r + 1];
    if (b < 0 || e < b || e > nnz) { bad = true; continue; }
    for (int64_t p = b; p < e; ++p) bad |= col[p] < 0 || col[p] >= cols || (p > b && col[p] <= col[p - 1]);
  }
  if (t0 == 0) bad |= rowptr[0] != 0 || (int64_t)rowptr[rows] != nnz;
  if (bad) atomicOr(flags, 1);
}

// entry_row[e] = the row entry e belongs to.
__global__ __launch_bounds__(kBlock) void csr_entry_rows_kernel(const int32_t* __restrict__ rowptr, int64_t rows,
                                                                int32_t* __restrict__ entry_row) {
  const int lane = threadIdx.x % kWave;
  const int64_t w0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  const int64_t nw = (int64_t)gridDim.x * blockDim.x / kWave;
  for (int64_t r = w0; r < rows; r += nw)
    for (int e = rowptr[r] + lane; e < rowptr[r + 1]; e += kWave) entry_row[e] = (int32_t)r;
}

// Column-sorted view: csc_row[p] = entry_row[perm[p]], csc_val[p] = val[perm[p]] for the p-th entry in column order.
__global__ __launch_bounds__(kBlock) void csr_gather_rows_kernel(const int32_t* __restrict__ entry_row,
                                                                 const float* __restrict__ val,
                                                                 const int32_t* __restrict__ perm, int64_t nnz,
                                                                 int32_t* __restrict__ csc_row,
                                                                 float* __restrict__ csc_val) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += (int64_t)gridDim.x * blockDim.x) {
    const int32_t e = perm[p];
    csc_row[p] = entry_row[e];
    csc_val[p] = val[e];
  }
}

// P[r, col0 + c] = sum over the entries e of row r of val[e] * X[colmap[col[e]], col0 + c], c < CT.
// A workgroup owns a run of whole rows with at most `cap` stored entries (row_block table, built with the
// plan): it first copies their values and column indices to LDS with coalesced loads (all of a thread's loads
// in flight at once - rows are short, walking them one by one would leave the memory system idle), then
// 2^k lanes per row sum the row from LDS.  X_k (ck x CT) is staged in LDS through the column map.
// XG (tables too wide for that, e.g. one-hot encodings with tens of thousands of columns): the operand values
// are fetched per stored entry while the block is staged (column map, then operand, all loads of a thread in
// flight), and LDS holds the products val * x instead of values and column indices.
template <int CT, bool XG>
__global__ __launch_bounds__(kBlock) void spmm_rows_kernel(SparseArgs a, const float* __restrict__ X, int ldx,
                                                           int col0, int ncols, float* __restrict__ P, int ldp,
                                                           int cap) {
  extern __shared__ float lds[];
  float* Xs = lds;                                        // [cols][CT]   (not XG)
  float* valS = XG ? lds : lds + (size_t)a.cols * CT;     // [cap], XG: [cap][CT] products
  int* colS = reinterpret_cast<int*>(valS + (size_t)cap * (XG ? CT : 1));   // [cap] (not XG)
  int* rpS = XG ? colS : colS + cap;                      // [kSparseBlockRows + 1] row pointers of the block
  if constexpr (!XG) {
    for (int e = threadIdx.x; e < a.cols * CT; e += kBlock) {
      const int j = e / CT, c = e - j * CT;
      const int t = a.colmap[j];
      Xs[e] = (t >= 0 && c < ncols) ? X[(int64_t)t * ldx + col0 + c] : 0.0f;
    }
  }
  for (int blk = blockIdx.x; blk < a.n_row_blocks; blk += gridDim.x) {
    const int r_lo = a.row_block[blk], r_hi = a.row_block[blk + 1];
    const int e_lo = a.rowptr[r_lo], e_hi = a.rowptr[r_hi];
    const int ne = e_hi - e_lo, nr = r_hi - r_lo;
    __syncthreads();                                      // Xs ready; the previous block's entries are consumed
    constexpr int U = 8;
    for (int p0 = threadIdx.x; p0 < ne; p0 += U * kBlock) {
      float v[U];
      int cc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int p = p0 + u * kBlock;
        v[u] = p < ne ? a.val[e_lo + p] : 0.0f;
        cc[u] = p < ne ? a.col[e_lo + p] : 0;
      }
      if constexpr (XG) {
        int tc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) tc[u] = p0 + u * kBlock < ne ? a.colmap[cc[u]] : -1;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
          float xv[U];
#pragma unroll
          for (int u = 0; u < U; ++u) xv[u] = (tc[u] >= 0 && c < ncols) ? X[(int64_t)tc[u] * ldx + col0 + c] : 0.0f;
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int p = p0 + u * kBlock;
            if (p < ne) valS[(size_t)p * CT + c] = v[u] * xv[u];
          }
        }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int p = p0 + u * kBlock;
          if (p < ne) { valS[p] = v[u]; colS[p] = cc[u]; }
        }
      }
    }
    for (int g = threadIdx.x; g <= nr; g += kBlock) rpS[g] = a.rowptr[r_lo + g] - e_lo;
    __syncthreads();
    // lanes per row: about eight entries per lane (a wavefront instruction then serves up to 64 rows; with a
    // lane per entry most of the time goes into the cross-lane sums of short rows), at most a wavefront
    int logL = 0;
    while (logL < 6 && ((int64_t)nr << (logL + 3)) < ne) ++logL;
    const int L = 1 << logL, sub = threadIdx.x & (L - 1);
    for (int g = threadIdx.x >> logL; g < nr; g += kBlock >> logL) {
      const int r = r_lo + g;
      const int beg = rpS[g], end = rpS[g + 1];
      float acc[CT];
#pragma unroll
      for (int c = 0; c < CT; ++c) acc[c] = 0.0f;
      for (int p = beg + sub; p < end; p += L) {
        if constexpr (XG) {
#pragma unroll
          for (int c = 0; c < CT; ++c) acc[c] += valS[(size_t)p * CT + c];
        } else {
          const float v = valS[p];
          const float* x = Xs + colS[p] * CT;
#pragma unroll
          for (int c = 0; c < CT; ++c) acc[c] = fmaf(v, x[c], acc[c]);
        }
      }
      for (int off = L >> 1; off > 0; off >>= 1) {
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[c] += __shfl_xor(acc[c], off);
      }
      if (sub == 0) {
#pragma unroll
        for (int c = 0; c < CT; ++c)
          if (c < ncols) P[(int64_t)r * ldp + col0 + c] = acc[c];
      }
    }
  }
}

// One workgroup per chunk of a column (at most kSparseChunk entries of the column-sorted view):
// partial[chunk, c] = sum csc_val[p] * Z[csc_row[p], col0 + c], fixed tree.
template <int CT>
__global__ __launch_bounds__(kBlock) void spmm_t_partial_kernel(SparseArgs a, const float* __restrict__ Z, int ldz,
                                                                int col0, int ncols, float* __restrict__ partial) {
  __shared__ float red[kBlock / kWave][CT];
  const int chunk = blockIdx.x;
  const int beg = a.chunk_beg[chunk], end = a.chunk_end[chunk];
  float acc[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) acc[c] = 0.0f;
  // eight entries per thread at a time: values and rows first, then the gathered operand rows
  constexpr int U = 8;
  for (int p0 = beg + threadIdx.x; p0 < end; p0 += U * kBlock) {
    float v[U];
    int row[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int p = p0 + u * kBlock;
      v[u] = p < end ? a.csc_val[p] : 0.0f;
      row[u] = p < end ? a.csc_row[p] : 0;
    }
    float z[U][CT];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int c = 0; c < CT; ++c) z[u][c] = c < ncols ? Z[(int64_t)row[u] * ldz + col0 + c] : 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int c = 0; c < CT; ++c) acc[c] = fmaf(v[u], z[u][c], acc[c]);
  }
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    float s = acc[c];
    for (int off = kWave / 2; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if (threadIdx.x % kWave == 0) red[threadIdx.x / kWave][c] = s;
  }
  __syncthreads();
  if (threadIdx.x < CT) {
    float s = 0.0f;
    for (int w = 0; w < kBlock / kWave; ++w) s += red[w][threadIdx.x];
    partial[(int64_t)chunk * CT + threadIdx.x] = s;
  }
}

// G[j, c] = sum of the partials of column j's chunks, in chunk order (G laid out [cols][kNarrowCT]; columns the
// operand does not have are written as zero).
template <int CT>
__global__ __launch_bounds__(kBlock) void spmm_t_combine_kernel(SparseArgs a, const float* __restrict__ partial,
                                                                float* __restrict__ G) {
  for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < a.cols * kNarrowCT; e += gridDim.x * blockDim.x) {
    const int j = e / kNarrowCT, c = e - j * kNarrowCT;
    float s = 0.0f;
    if (c < CT)
      for (int ch = a.col_first_chunk[j]; ch < a.col_first_chunk[j + 1]; ++ch) s += partial[(int64_t)ch * CT + c];
    G[e] = s;
  }
}

// T[i, colmap[col[e]]] += val[e] over the entries e of the source row that target row i takes; one wavefront per
// target row.  Dense form of the same pass for tables given as D.
__global__ __launch_bounds__(kBlock) void mat_scatter_sparse_kernel(SparseArgs a, const int32_t* __restrict__ idx,
                                                                    int64_t ident_rows, float* __restrict__ T,
                                                                    int64_t r_T, int c_T) {
  const int lane = threadIdx.x % kWave;
  const int64_t w0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  const int64_t nw = (int64_t)gridDim.x * blockDim.x / kWave;
  for (int64_t i = w0; i < r_T; i += nw) {
    const int64_t r = idx ? (int64_t)idx[i] : (i < ident_rows ? i : -1);
    if (r < 0) continue;
    for (int e = a.rowptr[r] + lane; e < a.rowptr[r + 1]; e += kWave) {
      const int t = a.colmap[a.col[e]];
      if (t >= 0) T[i * c_T + t] += a.val[e];
    }
  }
}

__global__ __launch_bounds__(kBlock) void mat_scatter_dense_kernel(const float* __restrict__ D, int64_t rows, int ck,
                                                                   const int32_t* __restrict__ colmap,
                                                                   const int32_t* __restrict__ idx, int64_t ident_rows,
                                                                   float* __restrict__ T, int64_t r_T, int c_T) {
  const int lane = threadIdx.x % kWave;
  const int64_t w0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
  const int64_t nw = (int64_t)gridDim.x * blockDim.x / kWave;
  for (int64_t i = w0; i < r_T; i += nw) {
    const int64_t r = idx ? (int64_t)idx[i] : (i < ident_rows ? i : -1);
    if (r < 0) continue;
    for (int j = lane; j < ck; j += kWave) {
      const int t = colmap[j];
      if (t >= 0) T[i * c_T + t] += D[r * ck + j];
    }
  }
}

int grid_of(int64_t n, int per_block, int cap) {
  int64_t g = (n + per_block - 1) / per_block;
  return (int)(g < 1 ? 1 : (g > cap ? cap : g));
}

}  // namespace

hipError_t launch_csr_check(const SparseArgs& a, int32_t* flags, hipStream_t st) {
  csr_check_kernel<<<grid_of(a.rows + 1, kBlock, 4096), kBlock, 0, st>>>(a.rowptr, a.col, a.rows, a.cols, a.nnz, flags);
  return hipGetLastError();
}

hipError_t launch_csr_entry_rows(const SparseArgs& a, int32_t* entry_row, hipStream_t st) {
  if (a.rows <= 0 || a.nnz <= 0) return hipSuccess;
  csr_entry_rows_kernel<<<grid_of(a.rows, kBlock / kWave, 8192), kBlock, 0, st>>>(a.rowptr, a.rows, entry_row);
  return hipGetLastError();
}

hipError_t launch_csr_gather_rows(const int32_t* entry_row, const float* val, const int32_t* perm, int64_t nnz,
                                  int32_t* csc_row, float* csc_val, hipStream_t st) {
  if (nnz <= 0) return hipSuccess;
  csr_gather_rows_kernel<<<grid_of(nnz, kBlock, 8192), kBlock, 0, st>>>(entry_row, val, perm, nnz, csc_row, csc_val);
  return hipGetLastError();
}

hipError_t launch_spmm_rows(const SparseArgs& a, const float* X, int ldx, int col0, int ncols, float* P, int ldp,
                            hipStream_t st) {
  if (a.rows <= 0 || ncols <= 0 || a.n_row_blocks <= 0) return hipSuccess;
  const bool xg = a.cols > kMaxLdsFloats;                 // operand fetched per entry instead of staged
  const int fit = xg ? kNarrowCT : (a.cols * 4 <= kMaxLdsFloats ? 4 : (a.cols * 2 <= kMaxLdsFloats ? 2 : 1));
  if (ncols > fit) return hipErrorInvalidValue;
  const int ct = ncols <= 1 ? 1 : (ncols <= 2 ? 2 : 4);   // columns the kernel carries: the operand's, rounded up
  const int cap = sparse_row_block_cap(a.cols);
  const size_t lds_bytes = xg ? ((size_t)cap * ct + kSparseBlockRows + 1) * sizeof(float)
                              : ((size_t)a.cols * ct + 2 * (size_t)cap + kSparseBlockRows + 1) * sizeof(float);
  const int grid = std::min(a.n_row_blocks, 8192);
#define ILARGI_SPMM(C, G) spmm_rows_kernel<C, G><<<grid, kBlock, lds_bytes, st>>>(a, X, ldx, col0, ncols, P, ldp, cap)
  if (xg) { if (ct == 4) ILARGI_SPMM(4, true); else if (ct == 2) ILARGI_SPMM(2, true); else ILARGI_SPMM(1, true); }
  else { if (ct == 4) ILARGI_SPMM(4, false); else if (ct == 2) ILARGI_SPMM(2, false); else ILARGI_SPMM(1, false); }
#undef ILARGI_SPMM
  return hipGetLastError();
}

// Entries a row block holds at most: 2048, or a whole row of the widest table whose operand is staged in LDS.
// Wider tables keep 2048: their rows must not hold more stored entries than that (checked with the plan).
int sparse_row_block_cap(int cols) { return cols <= kMaxLdsFloats ? std::max(2048, cols) : 2048; }

hipError_t launch_spmm_t(const SparseArgs& a, const float* Z, int ldz, int col0, int ncols, float* partial, float* G,
                         hipStream_t st) {
  if (a.cols <= 0 || ncols <= 0 || ncols > kNarrowCT) return ncols > kNarrowCT ? hipErrorInvalidValue : hipSuccess;
  const int grid = grid_of((int64_t)a.cols * kNarrowCT, kBlock, 1024);
  if (ncols <= 1) {
    if (a.n_chunks > 0) spmm_t_partial_kernel<1><<<a.n_chunks, kBlock, 0, st>>>(a, Z, ldz, col0, ncols, partial);
    spmm_t_combine_kernel<1><<<grid, kBlock, 0, st>>>(a, partial, G);
  } else if (ncols <= 2) {
    if (a.n_chunks > 0) spmm_t_partial_kernel<2><<<a.n_chunks, kBlock, 0, st>>>(a, Z, ldz, col0, ncols, partial);
    spmm_t_combine_kernel<2><<<grid, kBlock, 0, st>>>(a, partial, G);
  } else {
    if (a.n_chunks > 0) spmm_t_partial_kernel<4><<<a.n_chunks, kBlock, 0, st>>>(a, Z, ldz, col0, ncols, partial);
    spmm_t_combine_kernel<4><<<grid, kBlock, 0, st>>>(a, partial, G);
  }
  return hipGetLastError();
}

hipError_t launch_mat_scatter(const SparseArgs* sparse, const float* D, int64_t rows, int ck, const int32_t* colmap,
                              const int32_t* idx, int64_t ident_rows, float* T, int64_t r_T, int c_T, hipStream_t st) {
  if (r_T <= 0) return hipSuccess;
  const int grid = grid_of(r_T, kBlock / kWave, 16384);
  if (sparse != nullptr) mat_scatter_sparse_kernel<<<grid, kBlock, 0, st>>>(*sparse, idx, ident_rows, T, r_T, c_T);
  else mat_scatter_dense_kernel<<<grid, kBlock, 0, st>>>(D, rows, ck, colmap, idx, ident_rows, T, r_T, c_T);
  return hipGetLastError();
}

}  // namespace ilargi
