// One gradient-descent pass (Alg. 1) over sources whose rows feed fewer than two target rows on average
// (union-style integration: every table row lands on one target row), one model per pass.
//
// For such sources fetching the table row of every target row costs about as much as streaming the table once,
// so the rows are joined on the fly in target order and used twice while they are in registers:
//   z_i = sum_k D_k[row_k(i), :] w_k          (left multiply, Sec. 2.2)
//   e_i = residual of Alg. 1,  loss
//   G_k += D_k[row_k(i), :]^T e_i             (transposed multiply, same rows)
// Every table is read once; P_k, the residual and Z_k never exist in memory.  The factorized sequence (product,
// assembly, segment sum, column reduce) reads every gathered table twice.
//
// A wavefront takes 64 target rows per step.  Lane (g, p) = (lane / 16, lane % 16) holds float4 number p of the
// rows g * 16 + it, it = 0 .. 15, of every source: a table row of up to 64 columns is one 256-byte access of 16
// lanes.  The 16 partial dot products of a lane are summed across its 16-lane row with a halving exchange of
// data-parallel-primitive moves (15 adds), after which lane l holds z of row l of the step; labels, loss and
// residual are handled with lane = row.  The residuals go back through 64 floats of LDS, and every lane
// multiplies the float4s it still holds by the residual of their row.  Wavefronts are autonomous.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

__device__ __forceinline__ void rj_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kRjWaves = kBlock / kWave;
constexpr int kRjIts = 16;                   // rows of a step held by one lane

// Value of `x` in the lane the control word names (all lanes active).
template <int CTRL>
__device__ __forceinline__ float rj_dpp(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
constexpr int kDppRowMirror = 0x140;         // lane l of a row of 16  <-  lane 15 - l
constexpr int kDppHalfMirror = 0x141;        // lane l of a half row of 8  <-  lane 7 - l
constexpr int kDppSwap2 = 0x4E;              // quad_perm [2, 3, 0, 1]
constexpr int kDppSwap1 = 0xB1;              // quad_perm [1, 0, 3, 2]

// d[it] of the 16 lanes of a row  ->  lane p of the row returns the sum of d[p] over the row.
// Halving exchange: at each level a lane keeps the half of its values whose index has the lane's own bit and
// hands the other half to its partner, whose own bit is the opposite one.
__device__ __forceinline__ float rj_row_transpose_sum(const float (&d)[kRjIts], int p) {
  const bool b3 = (p & 8) != 0, b2 = (p & 4) != 0, b1 = (p & 2) != 0, b0 = (p & 1) != 0;
  float e8[8], e4[4], e2[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) e8[i] = (b3 ? d[i + 8] : d[i]) + rj_dpp<kDppRowMirror>(b3 ? d[i] : d[i + 8]);
#pragma unroll
  for (int i = 0; i < 4; ++i) e4[i] = (b2 ? e8[i + 4] : e8[i]) + rj_dpp<kDppHalfMirror>(b2 ? e8[i] : e8[i + 4]);
#pragma unroll
  for (int i = 0; i < 2; ++i) e2[i] = (b1 ? e4[i + 2] : e4[i]) + rj_dpp<kDppSwap2>(b1 ? e4[i] : e4[i + 2]);
  return (b0 ? e2[1] : e2[0]) + rj_dpp<kDppSwap1>(b0 ? e2[0] : e2[1]);
}

template <int NS, int MODE>
__global__ __launch_bounds__(kBlock) void gd_rowjoin_kernel(RowJoinArgs a) {
  extern __shared__ __align__(16) float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int g = lane / 16, p = lane % 16;
  int* Is = reinterpret_cast<int*>(lds) + wave * ((NS + 1) * kWave);   // [NS][64] row indices of the step
  float* Es = reinterpret_cast<float*>(Is + NS * kWave);                // [64] residuals of the step

  // this lane's four weights of every source (zero where the source has no such column or feeds no target column)
  float4 w4[NS];
  bool colive[NS];
  const float* Dp[NS];
  const int32_t* gidx[NS];
  int64_t grows[NS];
  int ck[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    ck[s] = a.ck[s];
    colive[s] = 4 * p < ck[s];
    Dp[s] = a.D[s] + 4 * p;
    gidx[s] = a.idx[s];
    grows[s] = a.rows[s];
    float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (colive[s]) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int t = a.colmap[s][4 * p + c];
        if (t >= 0) w[c] = a.W[(int64_t)t * a.ldw + a.col];
      }
    }
    w4[s] = make_float4(w[0], w[1], w[2], w[3]);
  }
  const int64_t r_T = a.r_T;
  auto row_of = [&](int s, int64_t i) -> int {
    return gidx[s] != nullptr ? gidx[s][i] : (i < grows[s] ? (int)i : -1);
  };

  float4 acc[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) acc[s] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  float loss_local = 0.0f;

  const int64_t nchunks = (r_T + kWave - 1) / kWave;
  const int64_t cstride = (int64_t)gridDim.x * kRjWaves;
  int64_t chunk = (int64_t)blockIdx.x * kRjWaves + wave;
  int jn[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int64_t i = chunk * kWave + lane;
    jn[s] = (chunk < nchunks && i < r_T) ? row_of(s, i) : -1;
  }
  for (; chunk < nchunks; chunk += cstride) {
    const int64_t i = chunk * kWave + lane;
    const bool rowlive = i < r_T;
    rj_wave_sync();                                              // the previous step's indices and residuals are consumed
#pragma unroll
    for (int s = 0; s < NS; ++s) Is[s * kWave + lane] = jn[s];
    rj_wave_sync();
    const float yi = a.y[min(i, r_T - 1)];
    {
      const int64_t inext = i + cstride * kWave;
#pragma unroll
      for (int s = 0; s < NS; ++s) jn[s] = (chunk + cstride < nchunks && inext < r_T) ? row_of(s, inext) : -1;
    }
    // the rows of the step: every load goes out before the first value is used
    float4 v[NS][kRjIts];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      int jj[kRjIts];
#pragma unroll
      for (int q = 0; q < kRjIts / 4; ++q) {
        const int4 t = *reinterpret_cast<const int4*>(Is + s * kWave + g * 16 + 4 * q);
        jj[4 * q] = t.x; jj[4 * q + 1] = t.y; jj[4 * q + 2] = t.z; jj[4 * q + 3] = t.w;
      }
#pragma unroll
      for (int it = 0; it < kRjIts; ++it) {
        v[s][it] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (jj[it] >= 0 && colive[s]) v[s][it] = *reinterpret_cast<const float4*>(Dp[s] + (int64_t)jj[it] * ck[s]);
      }
    }
    float d[kRjIts];
#pragma unroll
    for (int it = 0; it < kRjIts; ++it) {
      float t = 0.0f;
#pragma unroll
      for (int s = 0; s < NS; ++s)
        t += fmaf(v[s][it].x, w4[s].x, fmaf(v[s][it].y, w4[s].y, fmaf(v[s][it].z, w4[s].z, v[s][it].w * w4[s].w)));
      d[it] = t;
    }
    const float z = rj_row_transpose_sum(d, p);                  // row g * 16 + p = lane of the step
    float r = 0.0f;
    if (rowlive) {
      if constexpr (MODE == 1) {
        r = z - yi;
        loss_local = fmaf(r, r, loss_local);
      } else {
        // one exponential serves the sigmoid and the softplus: e = exp(-|z|)
        const float e = __expf(-fabsf(z));
        const float inv = __frcp_rn(1.0f + e);
        r = (z >= 0.0f ? inv : e * inv) - yi;
        loss_local += fmaxf(z, 0.0f) + log1pf(e) - yi * z;
      }
    }
    Es[lane] = r;
    rj_wave_sync();
    float er[kRjIts];
#pragma unroll
    for (int q = 0; q < kRjIts / 4; ++q) {
      const float4 t = *reinterpret_cast<const float4*>(Es + g * 16 + 4 * q);
      er[4 * q] = t.x; er[4 * q + 1] = t.y; er[4 * q + 2] = t.z; er[4 * q + 3] = t.w;
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int it = 0; it < kRjIts; ++it) {
        acc[s].x = fmaf(v[s][it].x, er[it], acc[s].x);
        acc[s].y = fmaf(v[s][it].y, er[it], acc[s].y);
        acc[s].z = fmaf(v[s][it].z, er[it], acc[s].z);
        acc[s].w = fmaf(v[s][it].w, er[it], acc[s].w);
      }
  }

  // the workgroup's sums, in the fixed order (wavefront, row group)
  __syncthreads();
  float4* gs = reinterpret_cast<float4*>(lds);                   // [waves * 4][NS][16]
#pragma unroll
  for (int s = 0; s < NS; ++s) gs[((wave * 4 + g) * NS + s) * 16 + p] = acc[s];
  float* ls = lds + kRjWaves * 4 * NS * 16 * 4;                  // [256] loss terms
  ls[tid] = loss_local;
  __syncthreads();
  if (tid < NS * 16) {
    const int s = tid / 16, q = tid % 16;
    float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int u = 0; u < kRjWaves * 4; ++u) {
      const float4 x = gs[(u * NS + s) * 16 + q];
      t.x += x.x; t.y += x.y; t.z += x.z; t.w += x.w;
    }
    if (4 * q < a.ck[s]) {
      // records of kNarrowCT floats per (workgroup, table column); this pass fills the first
      float4* out = reinterpret_cast<float4*>(a.grad_partial[s]) + (int64_t)blockIdx.x * a.ck[s] + 4 * q;
      out[0] = make_float4(t.x, 0.0f, 0.0f, 0.0f);
      out[1] = make_float4(t.y, 0.0f, 0.0f, 0.0f);
      out[2] = make_float4(t.z, 0.0f, 0.0f, 0.0f);
      out[3] = make_float4(t.w, 0.0f, 0.0f, 0.0f);
    }
  }
  // loss: tree over the 256 lanes' terms
  for (int w = kBlock / 2; w >= 1; w >>= 1) {
    if (tid < w) ls[tid] += ls[tid + w];
    __syncthreads();
  }
  if (tid == 0) reinterpret_cast<float4*>(a.loss_partial)[blockIdx.x] = make_float4(ls[0], 0.0f, 0.0f, 0.0f);
}

typedef void (*RjFn)(RowJoinArgs);

RjFn rj_pick(int ns, int mode) {
  if (ns == 1) return mode == 1 ? gd_rowjoin_kernel<1, 1> : gd_rowjoin_kernel<1, 2>;
  if (ns == 2) return mode == 1 ? gd_rowjoin_kernel<2, 1> : gd_rowjoin_kernel<2, 2>;
  return mode == 1 ? gd_rowjoin_kernel<3, 1> : gd_rowjoin_kernel<3, 2>;
}

size_t rj_lds_bytes(int ns) {
  const size_t step = (size_t)kRjWaves * (ns + 1) * kWave * sizeof(float);
  const size_t fin = ((size_t)kRjWaves * 4 * ns * 16 * 4 + kBlock) * sizeof(float);
  return std::max(step, fin);
}

int rj_slots(RjFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static RjFn seen_fn[8];
  static int seen_slots[8];
  static int n_seen = 0;
  for (int i = 0; i < n_seen; ++i)
    if (seen_fn[i] == fn) return seen_slots[i];
  int dev = 0, cus = 256, per_cu = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    cus = prop.multiProcessorCount;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, lds_bytes) != hipSuccess ||
      per_cu < 1)
    per_cu = 1;
  if (n_seen < 8) { seen_fn[n_seen] = fn; seen_slots[n_seen] = per_cu * cus; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// One to three dense sources with 16-byte aligned rows of at most 64 columns.
bool gd_rowjoin_supported(const RowJoinArgs& a) {
  if (a.n < 1 || a.n > kRowJoinSources || a.r_T < 1) return false;
  for (int s = 0; s < a.n; ++s) {
    if (a.D[s] == nullptr || a.ck[s] < 4 || a.ck[s] > 64 || a.ck[s] % 4 != 0) return false;
    if (reinterpret_cast<uintptr_t>(a.D[s]) % 16 != 0) return false;
  }
  return true;
}

hipError_t launch_gd_rowjoin(const RowJoinArgs& a, int mode, int max_grid, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!gd_rowjoin_supported(a) || (mode != 1 && mode != 2) || max_grid < 1) return hipErrorInvalidValue;
  RjFn fn = rj_pick(a.n, mode);
  const size_t lds_bytes = rj_lds_bytes(a.n);
  const int64_t nchunks = (a.r_T + kWave - 1) / kWave;
  int64_t grid = (nchunks + kRjWaves - 1) / kRjWaves;
  grid = std::min<int64_t>(grid, rj_slots(fn, lds_bytes));        // one round of resident workgroups
  grid = std::min<int64_t>(grid, max_grid);                       // ... within the partial buffers
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a);
  return hipGetLastError();
}

}  // namespace ilargi
