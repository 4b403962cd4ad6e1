// Column reduce of the transposed multiply for an identity source with short rows and 5..16 operand columns
// (Sec. 2.2):  G = S^T Y  with S r x (4 nvec), nvec <= 16, and Y r x c.
// The matrix-core form of this contraction gives a 20-column table a 64-column tile (or 16-column tiles read one
// float per lane) and moves ~190 bytes per load instruction.  Here the table is read as a flat stream of float4:
// a wavefront instruction takes rpi = 64 / nvec whole rows (60 of 64 lanes for a 20-column table), lane l holds
// part l % nvec of row l / nvec - the same part for every step, so each lane keeps the 4 x c partial sums of its
// four table columns in registers (plain FMAs: 4 c per row, a few microseconds for a million rows).  The nvec lanes
// of a row read the same operand row (one request).  At the end the lanes that hold the same part are added in
// row order through LDS, then the wavefronts in order; per-workgroup partial blocks are summed afterwards in
// workgroup order.  No floating-point atomics.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

// CMAX: compile-time bound of the operand columns (8 or 16).  YV4: operand rows are whole, aligned float4s.
template <int CMAX, bool YV4>
__global__ __launch_bounds__(kBlock) void colred_flat_kernel(ColredFlatArgs a) {
  __shared__ float tile[kWave][4 * CMAX + 1];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int nvec = a.nvec;
  const int rpi = kWave / nvec;                                 // rows per wavefront step
  const bool active = lane < rpi * nvec;
  const int r = lane / nvec;
  float acc[4][CMAX];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int n = 0; n < CMAX; ++n) acc[e][n] = 0.0f;
  const int64_t nsteps = (a.rows + rpi - 1) / rpi;
  const int64_t stride = (int64_t)gridDim.x * (kBlock / kWave);
  const float4* S4 = reinterpret_cast<const float4*>(a.S);
  auto load = [&](int64_t step, float4& s, float (&y)[CMAX]) {
    const int64_t row = step * rpi + r;
    const bool live = active && step < nsteps && row < a.rows;
    s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
    for (int n = 0; n < CMAX; ++n) y[n] = 0.0f;
    if (live) {
      s = S4[step * rpi * nvec + lane];                         // = float4 number  row * nvec + part
      const float* yr = a.Y + row * a.ldy;
      if constexpr (YV4) {
#pragma unroll
        for (int j = 0; j < CMAX / 4; ++j) {
          if (4 * j < a.c) {
            const float4 v = *reinterpret_cast<const float4*>(yr + 4 * j);
            y[4 * j] = v.x; y[4 * j + 1] = v.y; y[4 * j + 2] = v.z; y[4 * j + 3] = v.w;
          }
        }
      } else {
#pragma unroll
        for (int n = 0; n < CMAX; ++n)
          if (n < a.c) y[n] = yr[n];
      }
    }
  };
  auto fma_row = [&](const float4& s, const float (&y)[CMAX]) {
#pragma unroll
    for (int n = 0; n < CMAX; ++n) {
      acc[0][n] = fmaf(s.x, y[n], acc[0][n]);
      acc[1][n] = fmaf(s.y, y[n], acc[1][n]);
      acc[2][n] = fmaf(s.z, y[n], acc[2][n]);
      acc[3][n] = fmaf(s.w, y[n], acc[3][n]);
    }
  };
  for (int64_t step = (int64_t)blockIdx.x * (kBlock / kWave) + wave; step < nsteps; step += 2 * stride) {
    float4 s0, s1;
    float y0[CMAX], y1[CMAX];
    load(step, s0, y0);                                         // two steps in flight
    load(step + stride, s1, y1);
    fma_row(s0, y0);
    fma_row(s1, y1);
  }
  // lanes with the same part, in row order; then the wavefronts in order
  const int outs = nvec * 4 * CMAX;                             // (part, component, operand column), at most 1024
  float tot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int w = 0; w < kBlock / kWave; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int n = 0; n < CMAX; ++n) tile[lane][e * CMAX + n] = acc[e][n];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int o = tid + k * kBlock;
      if (o < outs) {
        const int p = o / (4 * CMAX), en = o - p * (4 * CMAX);
        float sum = 0.0f;
        for (int rr = 0; rr < rpi; ++rr) sum += tile[rr * nvec + p][en];
        tot[k] += sum;
      }
    }
  }
  float* gp = a.partial + (int64_t)blockIdx.x * (4 * nvec) * a.c;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int o = tid + k * kBlock;
    if (o < outs) {
      const int p = o / (4 * CMAX), en = o - p * (4 * CMAX);
      const int e = en / CMAX, n = en - e * CMAX;
      if (n < a.c) gp[(4 * p + e) * a.c + n] = tot[k];
    }
  }
}

typedef void (*CfFn)(ColredFlatArgs);

}  // namespace

// Rows of 1..16 aligned float4, 5..16 operand columns.
bool colred_flat_supported(const float* S, int64_t cols, int c) {
  return S != nullptr && cols >= 4 && cols % 4 == 0 && cols <= 64 && reinterpret_cast<uintptr_t>(S) % 16 == 0 && c > kNarrowCT && c <= 16;
}

// partial: partial_floats long, one (4 nvec) x c block per workgroup; *grid_out workgroups were launched.
hipError_t launch_colred_flat(const ColredFlatArgs& a, int64_t partial_floats, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!colred_flat_supported(a.S, 4 * (int64_t)a.nvec, a.c) || a.rows <= 0) return hipErrorInvalidValue;
  const bool yv4 = a.c % 4 == 0 && a.ldy % 4 == 0 && reinterpret_cast<uintptr_t>(a.Y) % 16 == 0;
  CfFn fn;
  if (a.c <= 8) fn = yv4 ? colred_flat_kernel<8, true> : colred_flat_kernel<8, false>;
  else fn = yv4 ? colred_flat_kernel<16, true> : colred_flat_kernel<16, false>;
  static std::mutex cache_mutex;
  static CfFn seen_fn[4];
  static int seen_slots[4];
  static int n_seen = 0;
  int slots = 0;
  {
    std::lock_guard<std::mutex> lock(cache_mutex);
    for (int i = 0; i < n_seen; ++i)
      if (seen_fn[i] == fn) slots = seen_slots[i];
    if (slots == 0) {
      int dev = 0, cus = 256, per_cu = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, 0) != hipSuccess || per_cu < 1)
        per_cu = 1;
      slots = per_cu * cus;
      if (n_seen < 4) { seen_fn[n_seen] = fn; seen_slots[n_seen] = slots; ++n_seen; }
    }
  }
  const int rpi = kWave / a.nvec;
  const int64_t nsteps = (a.rows + rpi - 1) / rpi;
  int64_t gx = (nsteps + 2 * (kBlock / kWave) - 1) / (2 * (kBlock / kWave));
  gx = std::min<int64_t>(gx, std::min<int64_t>(slots, 1024));            // one round of resident workgroups
  gx = std::min<int64_t>(gx, partial_floats / ((int64_t)4 * a.nvec * a.c));
  if (gx < 1) return hipErrorInvalidValue;
  if (grid_out) *grid_out = (int)gx;
  hipLaunchKernelGGL(fn, dim3((unsigned)gx), dim3(kBlock), 0, st, a);
  return hipGetLastError();
}

}  // namespace ilargi
