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

// Fast form for the usual schema: every aligned group of four target columns is either fed by four
// consecutive columns of one source or by nobody (gslot / gj0 tables, built with the plan).  A lane owns
// column groups lane, lane + 64, ... of its wavefront's row and stores them as float4.
constexpr int kMatRows = 4;   // rows in flight per wavefront
constexpr int kMatGroups = 4; // column groups per lane (target tables up to 1024 columns)

__global__ __launch_bounds__(kBlock) void materialize_vec4_kernel(MatArgs a) {
  __shared__ const float* sD[kMaxSources];
  __shared__ const int32_t* sIdx[kMaxSources];
  __shared__ int64_t sRows[kMaxSources];
  __shared__ int sCk[kMaxSources];
  if (threadIdx.x < kMaxSources) {
    int k = threadIdx.x;
    sD[k] = k < a.n ? a.D[k] : nullptr;
    sIdx[k] = k < a.n ? a.idx[k] : nullptr;
    sRows[k] = k < a.n ? a.rows[k] : 0;
    sCk[k] = k < a.n ? a.ck[k] : 0;
  }
  __syncthreads();
  const int lane = threadIdx.x % kWave;
  const int ngroups = a.c_T / 4;
  const float* dp[kMatGroups];
  const int32_t* ip[kMatGroups];
  int64_t rows[kMatGroups];
  int ck[kMatGroups];
  bool vec[kMatGroups];
#pragma unroll
  for (int q = 0; q < kMatGroups; ++q) {
    int g = lane + q * kWave;
    dp[q] = nullptr; ip[q] = nullptr; rows[q] = 0; ck[q] = 0; vec[q] = false;
    if (g < ngroups) {
      int slot = a.gslot[g];
      if (slot >= 0) {
        int j0 = a.gj0[g];
        dp[q] = sD[slot] + j0;
        ip[q] = sIdx[slot];
        rows[q] = sRows[slot];
        ck[q] = sCk[slot];
        vec[q] = (j0 % 4 == 0) && (ck[q] % 4 == 0) && (reinterpret_cast<uintptr_t>(sD[slot]) % 16 == 0);
      }
    }
  }
  const int64_t wave0 = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kMatRows;
  const int64_t stride = (int64_t)gridDim.x * (kBlock / kWave) * kMatRows;
  for (int64_t i0 = wave0; i0 < a.r_T; i0 += stride) {
    float4 v[kMatRows][kMatGroups];
#pragma unroll
    for (int u = 0; u < kMatRows; ++u) {
      int64_t i = i0 + u;
#pragma unroll
      for (int q = 0; q < kMatGroups; ++q) {
        v[u][q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (dp[q] != nullptr && i < a.r_T) {
          int64_t r = ip[q] != nullptr ? (int64_t)ip[q][i] : (i < rows[q] ? i : -1);
          if (r >= 0) {
            const float* src = dp[q] + r * ck[q];
            if (vec[q]) v[u][q] = *reinterpret_cast<const float4*>(src);
            else v[u][q] = make_float4(src[0], src[1], src[2], src[3]);
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kMatRows; ++u) {
      int64_t i = i0 + u;
      if (i >= a.r_T) break;
#pragma unroll
      for (int q = 0; q < kMatGroups; ++q) {
        int g = lane + q * kWave;
        if (g < ngroups) {
          // 0.0f + x: a source cell holding -0.0 becomes +0.0, as in the sum that defines the cell
          typedef float f4 __attribute__((ext_vector_type(4)));
          f4 o = {0.0f + v[u][q].x, 0.0f + v[u][q].y, 0.0f + v[u][q].z, 0.0f + v[u][q].w};
          // the table is written once and not read back here: keep it out of the caches' way
          __builtin_nontemporal_store(o, reinterpret_cast<f4*>(a.T + i * a.c_T + 4 * g));
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_materialize(const MatArgs& a, hipStream_t st) {
  if (a.r_T <= 0 || a.c_T <= 0) return hipSuccess;
  bool fast = a.gslot != nullptr && a.c_T % 4 == 0 && a.c_T <= 4 * kWave * kMatGroups &&
              reinterpret_cast<uintptr_t>(a.T) % 16 == 0;
  if (fast) {
    int64_t waves = (a.r_T + kMatRows - 1) / kMatRows;
    int64_t grid = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 65536) grid = 65536;
    materialize_vec4_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  } else {
    int64_t grid = (a.r_T + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 8192) grid = 8192;
    materialize_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace ilargi
