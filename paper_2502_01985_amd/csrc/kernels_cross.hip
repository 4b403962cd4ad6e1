// Gram matrix  T^T T = sum_k sum_l M_k D_k^T (I_k^T I_l) D_l M_l^T  (the rewrite rule of Sec. 2.2 applied to
// both factors).  Each (k, l) block is a sum over rows t of  w_t * a_t^T b_t  where a_t, b_t are rows of two
// row-major matrices, optionally addressed through index vectors:
//   diagonal   a = b = D_k,            w_t = number of target rows fed by source row t   (I_k^T I_k is diagonal)
//   via sums   a = I_l^T (I_k D_k),    b = D_l          (rows of D_k summed per source row of l beforehand)
//   via pairs  a = D_k[row_idx_k[i]],  b = D_l[row_idx_l[i]]   over the target rows i that have both.
#include "ilargi_internal.h"

namespace ilargi {

namespace {

constexpr int kTile = 64;   // output tile edge
constexpr int kRows = 16;   // rows staged per step

__global__ __launch_bounds__(kBlock) void gram_kernel(GramArgs a) {
  __shared__ float As[kRows][kTile + 4];
  __shared__ float Bs[kRows][kTile + 4];
  const int tiles_b = (a.cb + kTile - 1) / kTile;
  const int ta = blockIdx.y / tiles_b, tb = blockIdx.y - ta * tiles_b;
  const int a0 = ta * kTile, b0 = tb * kTile;
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  const int64_t t_lo = (int64_t)blockIdx.x * a.rows_per_chunk;
  const int64_t t_hi = min(t_lo + a.rows_per_chunk, a.n_rows);
  float acc[4][4];
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[p][q] = 0.0f;

  for (int64_t t0 = t_lo; t0 < t_hi; t0 += kRows) {
#pragma unroll
    for (int q = 0; q < (kRows * kTile) / kBlock; ++q) {
      int e = tid + q * kBlock;
      int r = e / kTile, c = e - r * kTile;
      int64_t t = t0 + r;
      float va = 0.0f, vb = 0.0f;
      if (t < t_hi) {
        int64_t ra = a.ia ? (int64_t)a.ia[t] : (t < a.a_rows ? t : -1);
        int64_t rb = a.ib ? (int64_t)a.ib[t] : (t < a.b_rows ? t : -1);
        if (ra >= 0 && rb >= 0) {
          float w = a.wptr ? (float)(a.wptr[t + 1] - a.wptr[t]) : 1.0f;
          if (a0 + c < a.ca) va = w * a.A[ra * a.lda + a0 + c];
          if (b0 + c < a.cb) vb = a.B[rb * a.ldb + b0 + c];
        }
      }
      As[r][c] = va;
      Bs[r][c] = vb;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      float av[4], bv[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) av[p] = As[r][ty * 4 + p];
#pragma unroll
      for (int q = 0; q < 4; ++q) bv[q] = Bs[r][tx * 4 + q];
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[p][q] = fmaf(av[p], bv[q], acc[p][q]);
    }
    __syncthreads();
  }
  float* out = a.partial + (int64_t)blockIdx.x * a.ca * a.cb;
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int ja = a0 + ty * 4 + p, jb = b0 + tx * 4 + q;
      if (ja < a.ca && jb < a.cb) out[(int64_t)ja * a.cb + jb] = acc[p][q];
    }
}

__global__ __launch_bounds__(kBlock) void gram_reduce_kernel(const float* __restrict__ partial, int nchunks,
                                                             int64_t elems, float* __restrict__ block) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < elems;
       e += (int64_t)gridDim.x * blockDim.x) {
    float s = 0.0f;
    for (int c = 0; c < nchunks; ++c) s += partial[(int64_t)c * elems + e];
    block[e] = s;
  }
}

// out[ti, tj] = sum over block pairs (k <= l), in order, of the cells of block (k, l) that M_k and M_l send to
// (ti, tj), plus the mirrored cell for k < l.  A diagonal block is read from its upper triangle so that the
// result is symmetric bit for bit.
__global__ __launch_bounds__(kBlock) void gram_assemble_kernel(const GramAsmPair* __restrict__ pairs, int npairs,
                                                               const int32_t* const* __restrict__ tcol2src,
                                                               int c_T, float* __restrict__ out) {
  int64_t total = (int64_t)c_T * c_T;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
       e += (int64_t)gridDim.x * blockDim.x) {
    int ti = (int)(e / c_T), tj = (int)(e - (int64_t)ti * c_T);
    float acc = 0.0f;
    for (int p = 0; p < npairs; ++p) {
      GramAsmPair pr = pairs[p];
      const int32_t* mk = tcol2src[pr.k];
      const int32_t* ml = tcol2src[pr.l];
      if (pr.k == pr.l) {
        int j1 = mk[ti], j2 = mk[tj];
        if (j1 >= 0 && j2 >= 0) {
          int lo = j1 < j2 ? j1 : j2, hi = j1 < j2 ? j2 : j1;
          acc += pr.block[(int64_t)lo * pr.cb + hi];
        }
      } else {
        float s = 0.0f;
        bool any = false;
        int jk = mk[ti], jl = ml[tj];
        if (jk >= 0 && jl >= 0) { s = pr.block[(int64_t)jk * pr.cb + jl]; any = true; }
        int jk2 = mk[tj], jl2 = ml[ti];
        if (jk2 >= 0 && jl2 >= 0) {
          float v = pr.block[(int64_t)jk2 * pr.cb + jl2];
          // a + b == b + a, so the cell and its mirror image receive the same bits
          s = any ? s + v : v;
          any = true;
        }
        if (any) acc += s;
      }
    }
    out[e] = acc;
  }
}

}  // namespace

hipError_t launch_gram(const GramArgs& a, int nchunks, hipStream_t st) {
  if (a.ca <= 0 || a.cb <= 0 || nchunks <= 0) return hipSuccess;
  int tiles = ((a.ca + kTile - 1) / kTile) * ((a.cb + kTile - 1) / kTile);
  dim3 grid(nchunks, tiles);
  gram_kernel<<<grid, kBlock, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_gram_reduce(const float* partial, int nchunks, int64_t elems, float* block, hipStream_t st) {
  if (elems <= 0) return hipSuccess;
  int grid = (int)((elems + kBlock - 1) / kBlock);
  if (grid > 4096) grid = 4096;
  gram_reduce_kernel<<<grid, kBlock, 0, st>>>(partial, nchunks, elems, block);
  return hipGetLastError();
}

hipError_t launch_gram_assemble(const GramAsmPair* pairs_dev, int npairs, const int32_t* const* tcol2src_dev,
                                int c_T, float* out, hipStream_t st) {
  if (c_T <= 0) return hipSuccess;
  int64_t total = (int64_t)c_T * c_T;
  int grid = (int)((total + kBlock - 1) / kBlock);
  if (grid > 4096) grid = 4096;
  gram_assemble_kernel<<<grid, kBlock, 0, st>>>(pairs_dev, npairs, tcol2src_dev, c_T, out);
  return hipGetLastError();
}

}  // namespace ilargi
