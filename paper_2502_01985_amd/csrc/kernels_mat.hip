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

// General form for tables whose columns have at most two feeding sources each (ct_slot / ct_j tables, built
// with the plan, list them in source order).  A wavefront writes four rows per step; its 64 lanes first fetch
// the 4 x 16 row indices (row u, source slot s) in one coalesced-by-source load and park them in LDS, then
// every lane copies its columns t = lane, lane + 64, ... of the four rows.
constexpr int kColBlock = 4;   // columns per lane held in registers (target tables up to 256 columns per pass)

__global__ __launch_bounds__(kBlock) void materialize_cols_kernel(MatArgs a) {
  __shared__ const float* sD[kMaxSources];
  __shared__ const int32_t* sIdx[kMaxSources];
  __shared__ int64_t sRows[kMaxSources];
  __shared__ int sCk[kMaxSources];
  __shared__ int sJ[kBlock / kWave][4][kMaxSources];
  if (threadIdx.x < kMaxSources) {
    int k = threadIdx.x;
    sD[k] = k < a.n ? a.D[k] : nullptr;
    sIdx[k] = k < a.n ? a.idx[k] : nullptr;
    sRows[k] = k < a.n ? a.rows[k] : 0;
    sCk[k] = k < a.n ? a.ck[k] : 0;
  }
  __syncthreads();
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t wave0 = ((int64_t)blockIdx.x * (kBlock / kWave) + wave) * 4;
  const int64_t stride = (int64_t)gridDim.x * (kBlock / kWave) * 4;
  const int ru = lane / kMaxSources, rs = lane % kMaxSources;   // (row of the step, source slot) this lane fetches
  for (int cb = 0; cb < a.c_T; cb += kWave * kColBlock) {
    // this lane's columns of the pass and their feeders
    const float* dp[kColBlock][2];
    int ck[kColBlock][2], slot[kColBlock][2];
#pragma unroll
    for (int q = 0; q < kColBlock; ++q) {
      const int t = cb + lane + q * kWave;
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        slot[q][f] = t < a.c_T ? a.ct_slot[2 * t + f] : -1;
        dp[q][f] = nullptr; ck[q][f] = 0;
        if (slot[q][f] >= 0) { dp[q][f] = sD[slot[q][f]] + a.ct_j[2 * t + f]; ck[q][f] = sCk[slot[q][f]]; }
      }
    }
    for (int64_t i0 = wave0; i0 < a.r_T; i0 += stride) {
      {
        const int64_t i = i0 + ru;
        int r = -1;
        if (rs < a.n && i < a.r_T) r = sIdx[rs] != nullptr ? sIdx[rs][i] : (i < sRows[rs] ? (int)i : -1);
        __builtin_amdgcn_wave_barrier();
        sJ[wave][ru][rs] = r;
        __builtin_amdgcn_wave_barrier();
      }
      float v[4][kColBlock][2];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int q = 0; q < kColBlock; ++q)
#pragma unroll
          for (int f = 0; f < 2; ++f) {
            v[u][q][f] = 0.0f;
            if (slot[q][f] >= 0) {
              const int r = sJ[wave][u][slot[q][f]];
              if (r >= 0) v[u][q][f] = dp[q][f][(int64_t)r * ck[q][f]];
            }
          }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int64_t i = i0 + u;
        if (i >= a.r_T) break;
#pragma unroll
        for (int q = 0; q < kColBlock; ++q) {
          const int t = cb + lane + q * kWave;
          if (t < a.c_T) {
            float acc = 0.0f + v[u][q][0];
            if (slot[q][1] >= 0 && sJ[wave][u][slot[q][1]] >= 0) acc += v[u][q][1];
            __builtin_nontemporal_store(acc, a.T + i * a.c_T + t);
          }
        }
      }
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

// The same table written as one flat stream of float4: element e is column group e % (c_T / 4) of row
// e / (c_T / 4).  A wavefront stores kFlatU runs of 64 consecutive float4, so every store instruction fills whole
// 128-byte lines whatever the row length (880-byte rows otherwise leave partial lines at both ends of each row).
// Needs every fed group to be four 16-byte-aligned source values (flat_ok).  The loop body has no branches: all
// row indices of a step are requested, then all source values, then all stores go out; elements nobody feeds
// read a dummy location and are replaced by zero.
constexpr int kFlatU = 4;
constexpr int kFlatMaxGroups = 1024;
typedef const int32_t __attribute__((address_space(1)))* GIntPtr;
typedef float mf4 __attribute__((ext_vector_type(4)));
typedef const mf4 __attribute__((address_space(1)))* GVecPtr;

__global__ __launch_bounds__(kBlock) void materialize_flat_kernel(MatArgs a, int64_t total) {
  __shared__ const float* sD[kMaxSources];
  __shared__ const int32_t* sIdx[kMaxSources];
  __shared__ int64_t sRows[kMaxSources];
  __shared__ int sCk[kMaxSources];
  __shared__ short gS[kFlatMaxGroups];
  __shared__ short gJ[kFlatMaxGroups];
  const int ngroups = a.c_T / 4;
  if (threadIdx.x < kMaxSources) {
    int k = threadIdx.x;
    sD[k] = k < a.n ? a.D[k] : nullptr;
    sIdx[k] = k < a.n ? a.idx[k] : nullptr;
    sRows[k] = k < a.n ? a.rows[k] : 0;
    sCk[k] = k < a.n ? a.ck[k] : 0;
  }
  for (int g = threadIdx.x; g < ngroups; g += kBlock) { gS[g] = (short)a.gslot[g]; gJ[g] = (short)a.gj0[g]; }
  __syncthreads();
  const int lane = threadIdx.x % kWave;
  const int32_t* dummy = a.gslot;                   // 16-byte aligned, at least four values long
  constexpr int64_t kRun = (int64_t)kWave * kFlatU;
  const int64_t wave0 = ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * kRun;
  const int64_t stride = (int64_t)gridDim.x * (kBlock / kWave) * kRun;
  for (int64_t c0 = wave0; c0 < total; c0 += stride) {
    const int64_t row0 = c0 / ngroups;
    const unsigned g0 = (unsigned)(c0 - row0 * ngroups);
    int64_t irow[kFlatU];
    int slot[kFlatU], joff[kFlatU], ridx[kFlatU];
    bool gathered[kFlatU];
#pragma unroll
    for (int u = 0; u < kFlatU; ++u) {
      const unsigned off = g0 + lane + u * kWave;
      const unsigned dr = off / (unsigned)ngroups;
      const int g = (int)(off - dr * (unsigned)ngroups);
      irow[u] = row0 + dr;
      const bool live = c0 + lane + u * kWave < total;
      slot[u] = live ? (int)gS[g] : -1;
      joff[u] = gJ[g];
      const int32_t* ip = slot[u] >= 0 ? sIdx[slot[u]] : nullptr;
      gathered[u] = ip != nullptr;
      ridx[u] = *(GIntPtr)(gathered[u] ? ip + irow[u] : dummy);
    }
    mf4 v[kFlatU];
    bool fed[kFlatU];
#pragma unroll
    for (int u = 0; u < kFlatU; ++u) {
      const int sl = max(slot[u], 0);
      const int64_t r = gathered[u] ? (int64_t)ridx[u] : (irow[u] < sRows[sl] ? irow[u] : -1);
      fed[u] = slot[u] >= 0 && r >= 0;
      const float* src = fed[u] ? sD[sl] + r * sCk[sl] + joff[u] : reinterpret_cast<const float*>(dummy);
      v[u] = *(GVecPtr)src;
    }
#pragma unroll
    for (int u = 0; u < kFlatU; ++u) {
      const int64_t e = c0 + lane + u * kWave;
      if (e < total) {
        // 0.0f + x: a source cell holding -0.0 becomes +0.0, as in the sum that defines the cell
        mf4 o = {0.0f + v[u].x, 0.0f + v[u].y, 0.0f + v[u].z, 0.0f + v[u].w};
        if (!fed[u]) o = (mf4){0.0f, 0.0f, 0.0f, 0.0f};
        // the table is written once and not read back here: keep it out of the caches' way
        __builtin_nontemporal_store(o, reinterpret_cast<mf4*>(a.T) + e);
      }
    }
  }
}

}  // namespace

hipError_t launch_materialize(const MatArgs& a, hipStream_t st) {
  if (a.r_T <= 0 || a.c_T <= 0) return hipSuccess;
  bool fast = a.gslot != nullptr && a.c_T % 4 == 0 && a.c_T <= 4 * kWave * kMatGroups &&
              reinterpret_cast<uintptr_t>(a.T) % 16 == 0;
  const int64_t total = a.r_T * (a.c_T / 4);
  if (fast && a.flat_ok && a.c_T / 4 <= kFlatMaxGroups && reinterpret_cast<uintptr_t>(a.gslot) % 16 == 0) {
    int64_t waves = (total + kWave * kFlatU - 1) / (kWave * kFlatU);
    int64_t grid = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 65536) grid = 65536;
    materialize_flat_kernel<<<(int)grid, kBlock, 0, st>>>(a, total);
  } else if (fast) {
    int64_t waves = (a.r_T + kMatRows - 1) / kMatRows;
    int64_t grid = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 65536) grid = 65536;
    materialize_vec4_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  } else if (a.ct_slot != nullptr) {
    int64_t waves = (a.r_T + 3) / 4;
    int64_t grid = (waves + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 65536) grid = 65536;
    materialize_cols_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  } else {
    int64_t grid = (a.r_T + (kBlock / kWave) - 1) / (kBlock / kWave);
    if (grid > 8192) grid = 8192;
    materialize_kernel<<<(int)grid, kBlock, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace ilargi
