// Join-gather baseline: the materialized target table  T = sum_k I_k D_k M_k^T  (Sec. 2.2 with X = I).
// Every cell is the float32 sum, in source order and starting from +0.0, of the source cells mapped to it,
// which makes the table reproducible bit for bit.
#include "ilargi_internal.h"

namespace ilargi {

namespace {

// One wavefront per target row, lanes across target columns.
__global__ __launch_bounds__(kBlock) void materialize_kernel(MatArgs a) {
  const int lane = threadIdx.x % kWave;
  const int64_t wave0 = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = (int64_t)gridDim.x * (kBlock / kWave);
  for (int64_t i = wave0; i < a.r_T; i += nwaves) {
    int64_t jrow[kMaxSources];
#pragma unroll
    for (int k = 0; k < kMaxSources; ++k) {
      if (k < a.n) {
        if (a.idx[k] != nullptr) jrow[k] = a.idx[k][i];
        else jrow[k] = (i < a.rows[k]) ? i : -1;
      }
    }
    for (int t = lane; t < a.c_T; t += kWave) {
      float acc = 0.0f;
#pragma unroll
      for (int k = 0; k < kMaxSources; ++k) {
        if (k < a.n) {
          int j = a.tcol2src[k][t];
          if (j >= 0 && jrow[k] >= 0) acc += a.D[k][jrow[k] * a.ck[k] + j];
        }
      }
      a.T[i * a.c_T + t] = acc;
    }
  }
}

}  // namespace

hipError_t launch_materialize(const MatArgs& a, hipStream_t st) {
  if (a.r_T <= 0 || a.c_T <= 0) return hipSuccess;
  int64_t grid = (a.r_T + (kBlock / kWave) - 1) / (kBlock / kWave);
  if (grid > 8192) grid = 8192;
  materialize_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace ilargi
