// Small kernels around the factorized operators for the two unsupervised models the paper evaluates next to the
// regressions (Sec. 4, Tab. 7-9): one Lloyd iteration of KMeans and one round of multiplicative updates of
// Gaussian NMF.  The passes over the source tables are the left multiply and the transposed multiply; what is
// left are row-local steps on r_T x k (or c_T x k) matrices with k small:
//   KMeans:  a_i = argmin_j (|c_j|^2 - 2 (T C)_ij)   (|t_i|^2 is the same for every j), the 0/1 assignment matrix
//            that the transposed multiply then turns into per-cluster sums, cluster sizes, and the division;
//   NMF:     X <- X o P / max(X Q, tiny)  row by row, with Q = H H^T (k x k) for X = W, P = T H^T and
//            Q = W^T W for X = H^T, P = T^T W.
// Rows are staged in LDS with coalesced loads (a thread then walks its own row at an odd stride, free of bank
// conflicts) and written back the same way.
#include <algorithm>
#include <cstdint>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

// e / k for 0 <= e < 2^17 and 1 <= k <= 256 through the float reciprocal: (e + 0.5) / k is at least 0.5 / k away
// from the next integer, far more than the rounding error of the product.
__device__ __forceinline__ int div_small(int e, float inv_k) { return (int)(((float)e + 0.5f) * inv_k); }

// Staging of a run of whole rows (total = rows * k floats, contiguous in memory) into an LDS tile of row stride
// ld and back.  With vec4 (base 16-byte aligned) a thread keeps four float4 loads in flight; the values of one
// float4 may straddle two rows of the tile.
__device__ __forceinline__ void stage_in(float* tile, const float* base, int total, int k, int ld, float inv_k,
                                         bool vec4, int tid) {
  int done = 0;
  if (vec4) {
    const int n4 = total / 4;
    const float4* b4 = reinterpret_cast<const float4*>(base);
    for (int e0 = tid; e0 < n4; e0 += 4 * kBlock) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = e0 + u * kBlock;
        v[u] = idx < n4 ? b4[idx] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = e0 + u * kBlock;
        if (idx < n4) {
          int r = div_small(4 * idx, inv_k), c = 4 * idx - r * k;
          const float w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            tile[r * ld + c] = w[q];
            if (++c == k) { c = 0; ++r; }
          }
        }
      }
    }
    done = n4 * 4;
  }
  for (int e = done + tid; e < total; e += kBlock) {
    const int r = div_small(e, inv_k), c = e - r * k;
    tile[r * ld + c] = base[e];
  }
}

__device__ __forceinline__ void stage_out(float* base, const float* tile, int total, int k, int ld, float inv_k,
                                          bool vec4, int tid) {
  int done = 0;
  if (vec4) {
    const int n4 = total / 4;
    float4* b4 = reinterpret_cast<float4*>(base);
    for (int idx = tid; idx < n4; idx += kBlock) {
      int r = div_small(4 * idx, inv_k), c = 4 * idx - r * k;
      float w[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        w[q] = tile[r * ld + c];
        if (++c == k) { c = 0; ++r; }
      }
      b4[idx] = make_float4(w[0], w[1], w[2], w[3]);
    }
    done = n4 * 4;
  }
  for (int e = done + tid; e < total; e += kBlock) {
    const int r = div_small(e, inv_k), c = e - r * k;
    base[e] = tile[r * ld + c];
  }
}

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
// counts_partial[blockIdx.x][j] the cluster sizes among the workgroup's rows (thousands of workgroups adding to the
// same k counters in memory would queue up behind each other; the sums are taken by kmeans_counts_kernel).
__global__ __launch_bounds__(kBlock) void kmeans_assign_kernel(float* __restrict__ P, const float* __restrict__ cn,
                                                               int64_t r_T, int k, int rows_pb, int vec4,
                                                               int32_t* __restrict__ assign, int32_t* __restrict__ counts_partial) {
  extern __shared__ float lds[];
  const int ld = k | 1;
  float* tile = lds;                                           // [rows_pb][ld]
  float* cns = tile + (size_t)rows_pb * ld;                    // [k]
  int* hist = reinterpret_cast<int*>(cns + k);                 // [k]
  const int tid = threadIdx.x;
  const float inv_k = 1.0f / (float)k;
  for (int j = tid; j < k; j += kBlock) { cns[j] = cn[j]; hist[j] = 0; }
  const int64_t ntiles = (r_T + rows_pb - 1) / rows_pb;
  for (int64_t tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
    const int64_t r0 = tl * rows_pb;
    const int nrow = (int)min((int64_t)rows_pb, r_T - r0);
    const int total = nrow * k;
    float* base = P + r0 * k;
    __syncthreads();                                           // the previous tile is stored; cns / hist are set
    stage_in(tile, base, total, k, ld, inv_k, vec4 != 0, tid);
    __syncthreads();
    int best = -1;
    if (tid < nrow) {
      float* row = tile + tid * ld;
      best = 0;
      float bv = cns[0] - 2.0f * row[0];
      for (int j = 1; j < k; ++j) {
        const float v = cns[j] - 2.0f * row[j];
        if (v < bv) { bv = v; best = j; }                      // strict: the first of equal minima stays
      }
      for (int j = 0; j < k; ++j) row[j] = j == best ? 1.0f : 0.0f;
      if (assign != nullptr) assign[r0 + tid] = best;
    }
    // cluster sizes of the tile: one count per wavefront and centroid instead of one atomic per row
    for (int j = 0; j < k; ++j) {
      const unsigned long long m = __ballot(best == j);
      if (tid % kWave == 0 && m != 0) atomicAdd(&hist[j], __popcll(m));
    }
    __syncthreads();
    stage_out(base, tile, total, k, ld, inv_k, vec4 != 0, tid);
  }
  __syncthreads();
  for (int j = tid; j < k; j += kBlock) counts_partial[(size_t)blockIdx.x * k + j] = hist[j];
}

// counts[j] = sum over the workgroups' shares, one workgroup per centroid.
__global__ __launch_bounds__(kBlock) void kmeans_counts_kernel(const int32_t* __restrict__ partial, int nparts, int k,
                                                               int32_t* __restrict__ counts) {
  __shared__ int red[kBlock];
  const int j = blockIdx.x;
  int acc = 0;
  for (int p = threadIdx.x; p < nparts; p += kBlock) acc += partial[(size_t)p * k + j];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kBlock / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) counts[j] = red[0];
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
// NT > 0 (= number of 16-column tiles of X): the workgroup also forms  X_new^T X_new  over its rows on the matrix
// cores and leaves it in gram_partial[blockIdx.x] (k x k); the caller adds the workgroups' shares in order.
// MFMA 16x16x4: a wavefront takes 64 rows of the LDS tile, four at a time as the K index; lane l supplies
// X_new[row l / 16][16 ta + l % 16] as A and X_new[row l / 16][16 tb + l % 16] as B of tile (ta, tb), ta <= tb.
typedef float v4f __attribute__((ext_vector_type(4)));

// KQ: the rank rounded up to 16 KQ, the compile-time length of a row's denominators (kept in registers).
template <int NT, int KQ>
__global__ __launch_bounds__(kBlock) void gnmf_update_kernel(float* __restrict__ X, const float* __restrict__ P,
                                                             const float* __restrict__ Q, int64_t rows, int k,
                                                             int rows_pb, int vec4, float tiny,
                                                             float* __restrict__ gram_partial) {
  extern __shared__ float lds[];
  const int ld = k | 1;
  float* xt = lds;                                             // [rows_pb][ld]
  float* pt = xt + (size_t)rows_pb * ld;                       // [rows_pb][ld]
  constexpr int KT = 16 * KQ;
  float* qs = pt + (size_t)rows_pb * ld;                       // [k][KT], zero beyond column k (16-byte aligned rows)
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const float inv_k = 1.0f / (float)k;
  for (int e = tid; e < k * KT; e += kBlock) {
    const int b = e / KT, a = e - b * KT;
    qs[e] = a < k ? Q[b * k + a] : 0.0f;
  }
  constexpr int NP = NT > 0 ? NT * (NT + 1) / 2 : 1;
  v4f gacc[NP];
#pragma unroll
  for (int u = 0; u < NP; ++u) gacc[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
  const int64_t ntiles = (rows + rows_pb - 1) / rows_pb;
  for (int64_t tl = blockIdx.x; tl < ntiles; tl += gridDim.x) {
    const int64_t r0 = tl * rows_pb;
    const int nrow = (int)min((int64_t)rows_pb, rows - r0);
    const int total = nrow * k;
    float* xb = X + r0 * k;
    const float* pb = P + r0 * k;
    __syncthreads();
    stage_in(xt, xb, total, k, ld, inv_k, vec4 != 0, tid);
    stage_in(pt, pb, total, k, ld, inv_k, vec4 != 0, tid);
    __syncthreads();
    if (tid < nrow) {
      const float* xr = xt + tid * ld;
      float* pr = pt + tid * ld;
      // den[a] = sum_b x[b] Q[b][a], b ascending: one read of x[b] and KT / 4 broadcast reads of Q's row per b
      float den[KT];
#pragma unroll
      for (int a = 0; a < KT; ++a) den[a] = 0.0f;
      for (int b = 0; b < k; ++b) {
        const float xv = xr[b];
        const float4* qrow = reinterpret_cast<const float4*>(qs + b * KT);
#pragma unroll
        for (int a4 = 0; a4 < KT / 4; ++a4) {
          const float4 qv = qrow[a4];
          den[4 * a4 + 0] = fmaf(xv, qv.x, den[4 * a4 + 0]);
          den[4 * a4 + 1] = fmaf(xv, qv.y, den[4 * a4 + 1]);
          den[4 * a4 + 2] = fmaf(xv, qv.z, den[4 * a4 + 2]);
          den[4 * a4 + 3] = fmaf(xv, qv.w, den[4 * a4 + 3]);
        }
      }
#pragma unroll
      for (int a = 0; a < KT; ++a)
        if (a < k) pr[a] = xr[a] * pr[a] / fmaxf(den[a], tiny);   // the new value takes the place of the consumed product
    }
    __syncthreads();
    stage_out(xb, pt, total, k, ld, inv_k, vec4 != 0, tid);
    if constexpr (NT > 0) {
      const int s = lane % 16, q = lane / 16;
      for (int rb = wave * kWave; rb < nrow; rb += kBlock) {    // (a tile has at most 256 rows: one turn)
        for (int rq = rb; rq < min(rb + kWave, nrow); rq += 4) {
          const int row = rq + q;
          float v[NT];
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const int c = 16 * t + s;
            v[t] = (row < nrow && c < k) ? pt[row * ld + c] : 0.0f;
          }
          int u = 0;
#pragma unroll
          for (int ta = 0; ta < NT; ++ta)
#pragma unroll
            for (int tb = ta; tb < NT; ++tb, ++u)
              gacc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(v[ta], v[tb], gacc[u], 0, 0, 0);
        }
      }
    }
  }
  if constexpr (NT > 0) {
    // the four wavefronts' shares added in wavefront order; tile (ta, tb), register r of lane (s, q) is element
    // (16 ta + 4 q + r, 16 tb + s)
    float* red = lds;                                          // [NP][16][16], inside the two row tiles
    const int s = lane % 16, q = lane / 16;
    for (int w = 0; w < kBlock / kWave; ++w) {
      __syncthreads();
      if (wave == w) {
#pragma unroll
        for (int u = 0; u < NP; ++u)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float* p = red + u * 256 + (4 * q + r) * 16 + s;
            if (w == 0) *p = gacc[u][r];
            else *p += gacc[u][r];
          }
      }
    }
    __syncthreads();
    float* gp = gram_partial + (size_t)blockIdx.x * k * k;
    for (int e = tid; e < k * k; e += kBlock) {
      const int a = div_small(e, inv_k), b = e - a * k;
      const int i = min(a, b), j = max(a, b);                  // mirrored from the tiles on or above the diagonal
      const int ta = i / 16, tb = j / 16;
      const int u = ta * NT - ta * (ta - 1) / 2 + (tb - ta);
      gp[e] = red[u * 256 + (i % 16) * 16 + (j % 16)];
    }
  }
}

int tile_rows(int k, int tiles) {
  // rows of a workgroup's LDS tile: up to one per thread, within about 48 KB for all tiles
  const int ld = k | 1;
  int rows = (48 * 1024 / 4) / (ld * tiles);
  return std::max(8, std::min(kBlock, rows / 4 * 4));       // a multiple of four: tiles start 16-byte aligned
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

// counts_partial holds partial_ints values: one row of k per workgroup; counts[j] receives the cluster sizes.
hipError_t launch_kmeans_assign(float* P, const float* cn, int64_t r_T, int k, int32_t* assign, int32_t* counts_partial,
                                int64_t partial_ints, int32_t* counts, hipStream_t st) {
  if (r_T <= 0 || k <= 0) return hipSuccess;
  const int rows_pb = tile_rows(k, 1);
  const size_t lds_bytes = ((size_t)rows_pb * (k | 1) + 2 * (size_t)k) * sizeof(float);
  const int vec4 = reinterpret_cast<uintptr_t>(P) % 16 == 0;
  const int grid = (int)std::min<int64_t>(std::min(tile_grid(r_T, rows_pb), 2048), partial_ints / k);
  if (grid < 1) return hipErrorInvalidValue;
  kmeans_assign_kernel<<<grid, kBlock, lds_bytes, st>>>(P, cn, r_T, k, rows_pb, vec4, assign, counts_partial);
  kmeans_counts_kernel<<<k, kBlock, 0, st>>>(counts_partial, grid, k, counts);
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

// gram_partial (optional, partial_floats long): receives one k x k share of X_new^T X_new per workgroup;
// *nparts_out tells how many.
hipError_t launch_gnmf_update(float* X, const float* P, const float* Q, int64_t rows, int k, float tiny,
                              float* gram_partial, int64_t partial_floats, int* nparts_out, hipStream_t st) {
  if (nparts_out) *nparts_out = 0;
  if (rows <= 0 || k <= 0) return hipSuccess;
  if (k > kGnmfMaxRank) return hipErrorInvalidValue;
  const int rows_pb = tile_rows(k, 2);
  const int kq = (k + 15) / 16;
  const size_t lds_bytes = (2 * (size_t)rows_pb * (k | 1) + (size_t)k * 16 * kq) * sizeof(float);
  int grid = tile_grid(rows, rows_pb);
  if (gram_partial != nullptr) {
    grid = (int)std::min<int64_t>(std::min(grid, 2048), partial_floats / ((int64_t)k * k));
    if (grid < 1) return hipErrorInvalidValue;
  }
  const int vec4 = reinterpret_cast<uintptr_t>(X) % 16 == 0 && reinterpret_cast<uintptr_t>(P) % 16 == 0;
  typedef void (*GnmfFn)(float*, const float*, const float*, int64_t, int, int, int, float, float*);
  GnmfFn fn;
  if (gram_partial != nullptr)
    fn = kq == 1 ? gnmf_update_kernel<1, 1> : (kq == 2 ? gnmf_update_kernel<2, 2> : (kq == 3 ? gnmf_update_kernel<3, 3> : gnmf_update_kernel<4, 4>));
  else
    fn = kq == 1 ? gnmf_update_kernel<0, 1> : (kq == 2 ? gnmf_update_kernel<0, 2> : (kq == 3 ? gnmf_update_kernel<0, 3> : gnmf_update_kernel<0, 4>));
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, X, P, Q, rows, k, rows_pb, vec4, tiny, gram_partial);
  if (nparts_out) *nparts_out = grid;
  return hipGetLastError();
}

}  // namespace ilargi
