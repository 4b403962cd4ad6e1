// Small kernels around the factorized operators for the two unsupervised models the paper evaluates next to the
// regressions (Sec. 5, Tab. 7-9): one Lloyd iteration of KMeans and one round of multiplicative updates of
// Gaussian NMF.  The passes over the source tables are the left multiply and the transposed multiply; what is
// left are row-local steps on r_T x k (or c_T x k) matrices with k small:
//   KMeans:  a_i = argmin_j (|c_j|^2 - 2 (T C)_ij)   (|t_i|^2 is the same for every j), the 0/1 assignment matrix
//            that the transposed multiply then turns into per-cluster sums, cluster sizes, and the division;
//   NMF:     X <- X o P / max(X Q, tiny)  row by row, with Q = H H^T (k x k) for X = W, P = T H^T and
//            Q = W^T W for X = H^T, P = T^T W.
// Rows are staged in LDS with coalesced loads (a thread then walks its own row at an odd stride, free of bank
// conflicts) and written back the same way.
#include <algorithm>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

// cn[j] = sum_t C[t][j]^2, one workgroup per centroid, partial sums combined in a fixed tree.
__global__ __launch_bounds__(kBlock) void centroid_norm_kernel(const float* __restrict__ C, int64_t c_T, int k,
                                                               float* __restrict__ cn) {
  __shared__ float red[kBlock];
  const int j = blockIdx.x;
  float acc = 0.0f;
  for (int64_t t = threadIdx.x; t < c_T; t += kBlock) {
    const float v = C[t * k + j];
    acc = fmaf(v, v, acc);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kBlock / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) cn[j] = red[0];
}

// P (r_T x k) holds T C on entry and the 0/1 assignment matrix on exit; assign[i] (optional) the chosen centroid;
// counts[j] (zeroed by the caller) the cluster sizes, gathered with integer atomics (exact in any order).
__global__ __launch_bounds__(kBlock) void kmeans_assign_kernel(float* __restrict__ P, const float* __restrict__ cn,
                                                               int64_t r_T, int k, int rows_pb,
                                                               int32_t* __restrict__ assign, int32_t* __restrict__ counts) {
  extern __shared__ float lds[];
  const int ld = k | 1;
  float* tile = lds;                                           // [rows_pb][ld]
  float* cns = tile + (size_t)rows_pb * ld;                    // [k]
  int* hist = reinterpret_cast<int*>(cns + k);                 // [k]
  const int tid = threadIdx.x;
  for (int j = tid; j < k; j += kBlock) { cns[j] = cn[j]; hist[j] = 0; }
  const int64_t ntiles = (r_T + rows_pb - 1) / rows_pb;
  for (int64_t tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
    const int64_t r0 = tl * rows_pb;
    const int nrow = (int)min((int64_t)rows_pb, r_T - r0);
    const int total = nrow * k;
    float* base = P + r0 * k;
    __syncthreads();                                           // the previous tile is stored; cns / hist are set
    for (int e = tid; e < total; e += kBlock) {
      const int r = e / k, c = e - r * k;
      tile[r * ld + c] = base[e];
    }
    __syncthreads();
    if (tid < nrow) {
      float* row = tile + tid * ld;
      int best = 0;
      float bv = cns[0] - 2.0f * row[0];
      for (int j = 1; j < k; ++j) {
        const float v = cns[j] - 2.0f * row[j];
        if (v < bv) { bv = v; best = j; }                      // strict: the first of equal minima stays
      }
      for (int j = 0; j < k; ++j) row[j] = j == best ? 1.0f : 0.0f;
      if (assign != nullptr) assign[r0 + tid] = best;
      atomicAdd(&hist[best], 1);
    }
    __syncthreads();
    for (int e = tid; e < total; e += kBlock) {
      const int r = e / k, c = e - r * k;
      base[e] = tile[r * ld + c];
    }
  }
  __syncthreads();
  for (int j = tid; j < k; j += kBlock)
    if (hist[j] != 0) atomicAdd(&counts[j], hist[j]);
}

// C[t][j] = G[t][j] / counts[j] for clusters that have rows; the others keep their centroid.
__global__ __launch_bounds__(kBlock) void kmeans_update_kernel(float* __restrict__ C, const float* __restrict__ G,
                                                               const int32_t* __restrict__ counts, int64_t c_T, int k,
                                                               int32_t* __restrict__ counts_out) {
  const int64_t total = c_T * k;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < total; e += (int64_t)gridDim.x * kBlock) {
    const int j = (int)(e % k);
    const int n = counts[j];
    if (n > 0) C[e] = G[e] / (float)n;
  }
  if (counts_out != nullptr && blockIdx.x == 0)
    for (int j = threadIdx.x; j < k; j += kBlock) counts_out[j] = counts[j];
}

// X[i][a] <- X[i][a] * P[i][a] / max(sum_b X[i][b] Q[b][a], tiny), rows staged in LDS.
__global__ __launch_bounds__(kBlock) void gnmf_update_kernel(float* __restrict__ X, const float* __restrict__ P,
                                                             const float* __restrict__ Q, int64_t rows, int k,
                                                             int rows_pb, float tiny) {
  extern __shared__ float lds[];
  const int ld = k | 1;
  float* xt = lds;                                             // [rows_pb][ld]
  float* pt = xt + (size_t)rows_pb * ld;                       // [rows_pb][ld]
  float* qs = pt + (size_t)rows_pb * ld;                       // [k][k]
  const int tid = threadIdx.x;
  for (int e = tid; e < k * k; e += kBlock) qs[e] = Q[e];
  const int64_t ntiles = (rows + rows_pb - 1) / rows_pb;
  for (int64_t tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
    const int64_t r0 = tl * rows_pb;
    const int nrow = (int)min((int64_t)rows_pb, rows - r0);
    const int total = nrow * k;
    float* xb = X + r0 * k;
    const float* pb = P + r0 * k;
    __syncthreads();
    for (int e = tid; e < total; e += kBlock) {
      const int r = e / k, c = e - r * k;
      xt[r * ld + c] = xb[e];
      pt[r * ld + c] = pb[e];
    }
    __syncthreads();
    if (tid < nrow) {
      const float* xr = xt + tid * ld;
      float* pr = pt + tid * ld;
      for (int a = 0; a < k; ++a) {
        float den = 0.0f;
        for (int b = 0; b < k; ++b) den = fmaf(xr[b], qs[b * k + a], den);
        pr[a] = xr[a] * pr[a] / fmaxf(den, tiny);              // the new value takes the place of the consumed product
      }
    }
    __syncthreads();
    for (int e = tid; e < total; e += kBlock) {
      const int r = e / k, c = e - r * k;
      xb[e] = pt[r * ld + c];
    }
  }
}

int tile_rows(int k, int tiles) {
  // rows of a workgroup's LDS tile: up to one per thread, within about 48 KB for all tiles
  const int ld = k | 1;
  int rows = (48 * 1024 / 4) / (ld * tiles);
  return std::max(8, std::min(kBlock, rows));
}

int tile_grid(int64_t rows, int rows_pb) {
  const int64_t ntiles = (rows + rows_pb - 1) / rows_pb;
  return (int)std::max<int64_t>(1, std::min<int64_t>(ntiles, 4096));
}

}  // namespace

hipError_t launch_centroid_norm(const float* C, int64_t c_T, int k, float* cn, hipStream_t st) {
  if (k <= 0) return hipSuccess;
  centroid_norm_kernel<<<k, kBlock, 0, st>>>(C, c_T, k, cn);
  return hipGetLastError();
}

hipError_t launch_kmeans_assign(float* P, const float* cn, int64_t r_T, int k, int32_t* assign, int32_t* counts,
                                hipStream_t st) {
  if (r_T <= 0 || k <= 0) return hipSuccess;
  const int rows_pb = tile_rows(k, 1);
  const size_t lds_bytes = ((size_t)rows_pb * (k | 1) + 2 * (size_t)k) * sizeof(float);
  kmeans_assign_kernel<<<tile_grid(r_T, rows_pb), kBlock, lds_bytes, st>>>(P, cn, r_T, k, rows_pb, assign, counts);
  return hipGetLastError();
}

hipError_t launch_kmeans_update(float* C, const float* G, const int32_t* counts, int64_t c_T, int k,
                                int32_t* counts_out, hipStream_t st) {
  if (k <= 0 || c_T <= 0) return hipSuccess;
  const int64_t total = c_T * k;
  const int grid = (int)std::max<int64_t>(1, std::min<int64_t>((total + kBlock - 1) / kBlock, 4096));
  kmeans_update_kernel<<<grid, kBlock, 0, st>>>(C, G, counts, c_T, k, counts_out);
  return hipGetLastError();
}

hipError_t launch_gnmf_update(float* X, const float* P, const float* Q, int64_t rows, int k, float tiny, hipStream_t st) {
  if (rows <= 0 || k <= 0) return hipSuccess;
  const int rows_pb = tile_rows(k, 2);
  const size_t lds_bytes = (2 * (size_t)rows_pb * (k | 1) + (size_t)k * k) * sizeof(float);
  gnmf_update_kernel<<<tile_grid(rows, rows_pb), kBlock, lds_bytes, st>>>(X, P, Q, rows, k, rows_pb, tiny);
  return hipGetLastError();
}

}  // namespace ilargi
