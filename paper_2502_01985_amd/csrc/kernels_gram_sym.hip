// Diagonal block of the Gram matrix,  C = sum_t w_t d_t^T d_t  for one table D with at most 208 columns
// (the cofactor block D_k^T diag(fan-out) D_k of T^T T, Sec. 2.2 / crossprod), on the matrix cores.
//
// C is symmetric, so only the 16 x 16 tiles (ci, cj), ci <= cj, are formed: for 200 columns that is 91 tiles
// instead of the 169 of the full square.  A workgroup of sixteen wavefronts stages 32 whole rows in LDS (coalesced
// float4 loads, every value fetched once), and each wavefront owns up to six tiles: for a quad of rows it
// reads the 16 columns of tile-row ci (times the row weight) and of tile-column cj from LDS and issues one
// MFMA 16x16x4 per tile.  In that MFMA both operands have the same layout (lane 16 q + s holds row q, column
// s of the 16), which is why one staged copy serves both sides.  Workgroups own row chunks; their partial
// blocks are added afterwards in chunk order, so the result is reproducible.
#include <algorithm>
#include <type_traits>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kGsThreads = 1024;
constexpr int kGsRows = 32;      // rows staged per step
constexpr int kGsPW = 6;         // tiles per wavefront: 16 x 6 = 96 >= 91 tiles of a 208-column table
constexpr int kGsMaxTiles = 13;  // 16-column tiles per side

template <bool VEC4>
__global__ __launch_bounds__(kGsThreads) void gram_sym_kernel(TredArgs a, int ntile, int ldr) {
  extern __shared__ float lds[];
  float* Rs = lds;                       // [kGsRows][ldr]
  float* Ws = lds + kGsRows * ldr;       // [kGsRows] row weights (0 beyond the chunk)
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: the tile list lives in scalar registers
  const int s = lane % 16, q = lane / 16;
  // this wavefront's tiles: pairs (ci, cj), ci <= cj, numbered row by row
  // (slots beyond the last pair repeat tile (0, 0) and are not written: the inner loop stays free of branches)
  int ci[kGsPW], cj[kGsPW];
  bool live_tile[kGsPW];
  {
    int p = wave * kGsPW, i = 0;
    while (i < ntile && p >= ntile - i) { p -= ntile - i; ++i; }
    int j = i + p;
#pragma unroll
    for (int u = 0; u < kGsPW; ++u) {
      live_tile[u] = i < ntile;
      ci[u] = live_tile[u] ? i : 0;
      cj[u] = live_tile[u] ? j : 0;
      if (++j >= ntile) { ++i; j = i; }
    }
  }
  v4f acc[kGsPW];
#pragma unroll
  for (int u = 0; u < kGsPW; ++u) acc[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  const int64_t t_lo = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t t_hi = min(t_lo + a.rows_per_block, a.n_rows);
  const int width = ntile * 16;
  // staging slots of this thread: up to NV float4 (or scalars) of the 32 x width tile, the same every step;
  // the next step's values are fetched into registers while the matrix cores work on the current rows
  typedef typename std::conditional<VEC4, float4, float>::type SVal;
  constexpr int NV = VEC4 ? (kGsRows * kGsMaxTiles * 4 + kGsThreads - 1) / kGsThreads
                          : (kGsRows * kGsMaxTiles * 16 + kGsThreads - 1) / kGsThreads;
  const int spr = VEC4 ? width / 4 : width;   // slots per row
  const int live = VEC4 ? a.ca / 4 : a.ca;    // slots inside the table
  SVal sv[NV];
  float wv = 0.0f;
  auto fetch = [&](int64_t t0) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = tid + u * kGsThreads;
      const int r = e / spr, g = e - r * spr;
      const int64_t t = t0 + r;
      if constexpr (VEC4) sv[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      else sv[u] = 0.0f;
      if (r < kGsRows && t < t_hi && t < a.a_rows && g < live) {
        if constexpr (VEC4) sv[u] = *reinterpret_cast<const float4*>(a.A + t * a.lda + 4 * g);
        else sv[u] = a.A[t * a.lda + g];
      }
    }
    wv = 0.0f;
    if (tid < kGsRows && t0 + tid < t_hi) wv = a.wptr ? (float)(a.wptr[t0 + tid + 1] - a.wptr[t0 + tid]) : 1.0f;
  };
  fetch(t_lo);
  for (int64_t t0 = t_lo; t0 < t_hi; t0 += kGsRows) {
    __syncthreads();                     // the previous rows are consumed
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = tid + u * kGsThreads;
      const int r = e / spr, g = e - r * spr;
      if (r < kGsRows) {
        if constexpr (VEC4) *reinterpret_cast<float4*>(Rs + r * ldr + 4 * g) = sv[u];
        else Rs[r * ldr + g] = sv[u];
      }
    }
    if (tid < kGsRows) Ws[tid] = wv;
    __syncthreads();
    if (t0 + kGsRows < t_hi) fetch(t0 + kGsRows);
#pragma unroll 2
    for (int rq = 0; rq < kGsRows / 4; ++rq) {
      const float* row = Rs + (rq * 4 + q) * ldr + s;
      const float w = Ws[rq * 4 + q];
#pragma unroll
      for (int u = 0; u < kGsPW; ++u) {
        const float av = row[16 * ci[u]] * w;
        const float bv = row[16 * cj[u]];
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[u], 0, 0, 0);
      }
    }
  }
  // tile (ci, cj): register r of lane 16 q + s is C[16 ci + 4 q + r][16 cj + s]
  float* out = a.partial + (int64_t)blockIdx.x * a.ca * a.cb;
#pragma unroll
  for (int u = 0; u < kGsPW; ++u) {
    if (!live_tile[u]) continue;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = 16 * ci[u] + 4 * q + r, n = 16 * cj[u] + s;
      if (j < a.ca && n < a.cb) out[(int64_t)j * a.cb + n] = acc[u][r];
    }
  }
}

}  // namespace

// A == B without index vectors, at most 208 columns, enough tiles to occupy the wavefronts.
bool gram_sym_supported(const TredArgs& a) {
  return a.upper_only && a.A == a.B && a.ia == nullptr && a.ib == nullptr && a.ca == a.cb && a.lda == a.ldb &&
         a.bcol0 == 0 && a.ca > 64 && a.ca <= 16 * kGsMaxTiles;
}

// Splits the rows into chunks (one workgroup each, about one per compute unit, a multiple of the staging step,
// within the caller's partial buffer of partial_floats), sets a.rows_per_block and launches; the chunk count
// comes back for the ordered sum of the partial blocks.
hipError_t launch_gram_sym(TredArgs& a, int64_t partial_floats, hipStream_t st, int* nchunks_out) {
  if (nchunks_out) *nchunks_out = 0;
  if (!gram_sym_supported(a) || a.n_rows <= 0) return hipErrorInvalidValue;
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      return (int)prop.multiProcessorCount;
    return 256;
  }();
  int64_t nch = std::min<int64_t>(cus, partial_floats / ((int64_t)a.ca * a.cb));
  nch = std::max<int64_t>(1, std::min<int64_t>(nch, (a.n_rows + kGsRows - 1) / kGsRows));
  a.rows_per_block = ((a.n_rows + nch - 1) / nch + kGsRows - 1) / kGsRows * kGsRows;
  nch = (a.n_rows + a.rows_per_block - 1) / a.rows_per_block;
  const int ntile = (a.ca + 15) / 16;
  int ldr = ntile * 16;
  if (ldr % 32 == 0) ldr += 16;          // rows q and q + 1 of a quad on different LDS banks
  const bool vec4 = a.ca % 4 == 0 && a.lda % 4 == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0;
  const size_t lds_bytes = ((size_t)kGsRows * ldr + kGsRows) * sizeof(float);
  if (vec4) hipLaunchKernelGGL(gram_sym_kernel<true>, dim3((unsigned)nch), dim3(kGsThreads), lds_bytes, st, a, ntile, ldr);
  else hipLaunchKernelGGL(gram_sym_kernel<false>, dim3((unsigned)nch), dim3(kGsThreads), lds_bytes, st, a, ntile, ldr);
  if (nchunks_out) *nchunks_out = (int)nch;
  return hipGetLastError();
}

}  // namespace ilargi
