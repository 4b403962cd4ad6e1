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
#include "colred_flat_body.h"

namespace ilargi {

namespace {

template <int CMAX, bool YV4>
__global__ __launch_bounds__(kBlock) void colred_flat_kernel(ColredFlatArgs a) {
  __shared__ float tile[colred_flat_lds_floats(CMAX)];
  colred_flat_body<CMAX, YV4>(a, tile, (int)blockIdx.x, (int)gridDim.x);
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
