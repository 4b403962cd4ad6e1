// Gram matrix  T^T T = sum_k sum_l M_k D_k^T (I_k^T I_l) D_l M_l^T  (the rewrite rule of Sec. 2.2 applied to
// both factors).  Each (k, l) block is a sum over rows t of  w_t * a_t^T b_t  where a_t, b_t are rows of two
// row-major matrices, optionally addressed through index vectors:
//   diagonal   a = b = D_k,            w_t = number of target rows fed by source row t   (I_k^T I_k is diagonal)
//   via sums   a = I_l^T (I_k D_k),    b = D_l          (rows of D_k summed per source row of l beforehand)
//   via pairs  a = D_k[row_idx_k[i]],  b = D_l[row_idx_l[i]]   over the target rows i that have both.
#include "ilargi_internal.h"

namespace ilargi {

namespace {

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
