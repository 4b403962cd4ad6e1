// Diagonal block of the Gram matrix,  C = sum_t w_t d_t^T d_t  for one table D with at most 208 columns
// (the cofactor block D_k^T diag(fan-out) D_k of T^T T, Sec. 2.2 / crossprod), on the matrix cores.
//
// C is symmetric, so only the 16 x 16 tiles (ci, cj), ci <= cj, are formed: for 200 columns that is 91 tiles
// instead of the 169 of the full square.  A workgroup of sixteen wavefronts stages 32 whole rows in LDS (coalesced
// float4 loads, every value fetched once), and each wavefront owns up to six tiles: for a quad of rows it reads
// the 16 columns of tile-row ci (times the row weight) and of tile-column cj from LDS and issues one MFMA 16x16x4
// per tile.
// In that MFMA both operands have the same layout (lane 16 q + s holds row q, column s of the 16), which is why
// one staged copy serves both sides.  Workgroups own row chunks; each leaves its tiles packed (a tile's register r
// of all 64 lanes is one 256-byte run), and a second kernel adds the chunks in order and puts the sums in place.
#include <algorithm>
#include <type_traits>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kGsThreads = 1024;
constexpr int kGsRows = 32;      // rows staged per step
constexpr int kGsMaxTiles = 13;  // 16-column tiles of D
constexpr int kGsPW = 6;         // tiles per wavefront: 16 x 6 = 96 >= 91 tiles of a 208-column table
constexpr int kGsLdr = 16 * kGsMaxTiles;   // LDS row stride, a constant (208 = 6.5 x 32 banks: the four rows of a quad
                                           // fall on alternating halves of the banks) so that the row steps of the
                                           // unrolled inner loop become immediate offsets of the LDS reads

template <bool VEC4>
__global__ __launch_bounds__(kGsThreads) void gram_sym_kernel(TredArgs a, int ntile) {
  constexpr int PW = kGsPW;
  constexpr int ldr = kGsLdr;
  extern __shared__ float lds[];
  float* Rs = lds;                       // [kGsRows][ldr]
  float* Ws = lds + kGsRows * ldr;       // [kGsRows] row weights (0 beyond the chunk)
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: the tile list lives in scalar registers
  const int s = lane % 16, q = lane / 16;
  const int ntot = ntile * (ntile + 1) / 2;
  // this wavefront's tiles: the pairs (ci, cj), ci <= cj, numbered row by row; slots beyond the last tile repeat
  // tile (0, 0) and are not written: the inner loop stays free of branches
  int offa[PW], offb[PW];
  bool live_tile[PW];
  {
    int p = wave * PW, i = 0;
    while (i < ntile && p >= ntile - i) { p -= ntile - i; ++i; }
    int j = i + p;
#pragma unroll
    for (int u = 0; u < PW; ++u) {
      live_tile[u] = wave * PW + u < ntot;
      offa[u] = live_tile[u] ? 16 * i : 0;
      offb[u] = live_tile[u] ? 16 * j : 0;
      if (++j >= ntile) { ++i; j = i; }
    }
  }
  v4f acc[PW];
#pragma unroll
  for (int u = 0; u < PW; ++u) acc[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  const int64_t t_lo = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t t_hi = min(t_lo + a.rows_per_block, a.n_rows);
  const int width = ntile * 16;
  // staging slots of this thread: up to NV float4 (or scalars) of the 32 x width tile, the same every step;
  // the next step's values are fetched into registers while the matrix cores work on the current rows
  typedef typename std::conditional<VEC4, float4, float>::type SVal;
  constexpr int NV = VEC4 ? (kGsRows * kGsMaxTiles * 4 + kGsThreads - 1) / kGsThreads
                          : (kGsRows * kGsMaxTiles * 16 + kGsThreads - 1) / kGsThreads;
  const int spr = VEC4 ? width / 4 : width;          // slots per row
  const int live = VEC4 ? a.ca / 4 : a.ca;           // slots inside the table
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
  const float* pa[PW];
  const float* pb[PW];
#pragma unroll
  for (int u = 0; u < PW; ++u) {
    pa[u] = Rs + q * ldr + s + offa[u];
    pb[u] = Rs + q * ldr + s + offb[u];
  }
  const float* wq = Ws + q;
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
#pragma unroll
    for (int rq = 0; rq < kGsRows / 4; ++rq) {
      const float w = wq[rq * 4];
#pragma unroll
      for (int u = 0; u < PW; ++u) {
        // (pa[u], pb[u] are loop-invariant lane addresses; the row step is a compile-time offset)
        const float av = pa[u][rq * 4 * ldr] * w;
        const float bv = pb[u][rq * 4 * ldr];
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[u], 0, 0, 0);
      }
    }
  }
  // packed: tile t of this workgroup, register r, lane
  float* out = a.partial + (int64_t)blockIdx.x * ntot * 256;
#pragma unroll
  for (int u = 0; u < PW; ++u) {
    if (!live_tile[u]) continue;
    const int t = wave * PW + u;
#pragma unroll
    for (int r = 0; r < 4; ++r) out[(t * 4 + r) * kWave + lane] = acc[u][r];
  }
}

// Adds the chunks of one quarter tile (register r of a tile: 64 values) in order: sixteen thread groups stride the
// chunks, then the groups are added in order.  Tile t, register r, lane 16 q + s is element (4 q + r, s) of tile
// (ci, cj).
__global__ __launch_bounds__(kGsThreads) void gram_tile_reduce_kernel(const float* __restrict__ partial, int nchunks, int ntile,
                                                                      int ca, float* __restrict__ block) {
  __shared__ float red[16][kWave];
  const int ntot = ntile * (ntile + 1) / 2;
  const int t = blockIdx.x / 4, r = blockIdx.x % 4;
  const int lane = threadIdx.x % kWave, cg = threadIdx.x / kWave;
  const float* src = partial + ((int64_t)t * 4 + r) * kWave + lane;
  const int64_t stride = (int64_t)ntot * 256;
  float acc = 0.0f;
  int c = cg;
  for (; c + 3 * 16 < nchunks; c += 4 * 16) {
    const float v0 = src[(int64_t)c * stride], v1 = src[(int64_t)(c + 16) * stride];
    const float v2 = src[(int64_t)(c + 32) * stride], v3 = src[(int64_t)(c + 48) * stride];
    acc += v0; acc += v1; acc += v2; acc += v3;
  }
  for (; c < nchunks; c += 16) acc += src[(int64_t)c * stride];
  red[cg][lane] = acc;
  __syncthreads();
  if (threadIdx.x < kWave) {
    float sum = 0.0f;
#pragma unroll
    for (int g = 0; g < 16; ++g) sum += red[g][lane];
    const int s = lane % 16, q = lane / 16;
    int p = t, i = 0;
    while (p >= ntile - i) { p -= ntile - i; ++i; }
    const int j = 16 * i + 4 * q + r, n = 16 * (i + p) + s;
    if (j < ca && n < ca) block[(int64_t)j * ca + n] = sum;
  }
}

}  // namespace

// A == B without index vectors, at most 208 columns, enough tiles to occupy the wavefronts.
bool gram_sym_supported(const TredArgs& a) {
  return a.upper_only && a.A == a.B && a.ia == nullptr && a.ib == nullptr && a.ca == a.cb && a.lda == a.ldb &&
         a.bcol0 == 0 && a.ca > 64 && a.ca <= 16 * kGsMaxTiles;
}

// Splits the rows into chunks (one workgroup each, about one per compute unit, a multiple of the staging step,
// within the caller's partial buffer of partial_floats), launches the tile kernel and the ordered sum of the
// chunks.  block receives the upper-triangle tiles of D^T diag(w) D (ca x ca).
hipError_t launch_gram_sym(TredArgs& a, float* partial, int64_t partial_floats, float* block, hipStream_t st) {
  if (!gram_sym_supported(a) || a.n_rows <= 0) return hipErrorInvalidValue;
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      return (int)prop.multiProcessorCount;
    return 256;
  }();
  const int ntile = (a.ca + 15) / 16;
  const int ntot = ntile * (ntile + 1) / 2;
  int64_t nch = std::min<int64_t>(cus, partial_floats / ((int64_t)ntot * 256));
  if (nch < 1) return hipErrorInvalidValue;
  nch = std::max<int64_t>(1, std::min<int64_t>(nch, (a.n_rows + kGsRows - 1) / kGsRows));
  a.rows_per_block = ((a.n_rows + nch - 1) / nch + kGsRows - 1) / kGsRows * kGsRows;
  nch = (a.n_rows + a.rows_per_block - 1) / a.rows_per_block;
  a.partial = partial;
  constexpr int ldr = kGsLdr;
  const bool vec4 = a.ca % 4 == 0 && a.lda % 4 == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0;
  const size_t lds_bytes = ((size_t)kGsRows * ldr + kGsRows) * sizeof(float);
  if (vec4) hipLaunchKernelGGL(gram_sym_kernel<true>, dim3((unsigned)nch), dim3(kGsThreads), lds_bytes, st, a, ntile);
  else hipLaunchKernelGGL(gram_sym_kernel<false>, dim3((unsigned)nch), dim3(kGsThreads), lds_bytes, st, a, ntile);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  gram_tile_reduce_kernel<<<4 * ntot, kGsThreads, 0, st>>>(partial, (int)nch, ntile, a.ca, block);
  return hipGetLastError();
}

}  // namespace ilargi
