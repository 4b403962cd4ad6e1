// Per-source product of the left multiply for operands of 5..16 columns (Sec. 2.2):
//   P = D X_D,   D r x ck (ck <= 256, 16-byte aligned rows),  X_D = the rows of X the column map selects
// as a streaming kernel: the table goes from memory straight into the A operands of the matrix cores, no LDS
// staging of table rows and no barrier after the operand is in place.
//
// A wavefront owns 16 table rows at a time.  Lane (li, q) = (lane % 16, lane / 16) loads the float4 at columns
// 16 s + 4 q .. + 3 of row li for every step s: the four values are the A operand (row li, K slot q) of four
// 16x16x4 products whose B operand is X_D[16 s + 4 q + e][n = li], e = 0..3 (the summation index of a product is
// free to be dealt to the K slots in any order, as long as A and B agree).  All loads of a tile are issued before
// the first product, and before the operand is staged, so a wavefront has its whole tile (up to 13 KiB) in flight;
// enough wavefronts are resident that the whole table is requested within the first microseconds.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int kPsWaves = kBlock / kWave;

// NST: compile-time bound of the 16-column steps of a table row.
template <int NST>
__global__ __launch_bounds__(kBlock) void lmm_prod_stream_kernel(LmmArgs a, int nst) {
  extern __shared__ __align__(16) float lds[];       // Xs [4 nst][16][4]: X_D[4 g + e][n] at (g * 16 + n) * 4 + e
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int64_t tstride = (int64_t)gridDim.x * kPsWaves;
  int64_t tile = (int64_t)blockIdx.x * kPsWaves + wave;
  const int ck = a.ck;

  float4 av[NST];
  auto fetch = [&](int64_t t) {
    const int64_t row = t * 16 + li;
    const float* rp = a.D + row * ck + 4 * q;
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      av[s] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (s < nst && t < ntiles && row < a.d_rows && 16 * s + 4 * q < ck) av[s] = *reinterpret_cast<const float4*>(rp + 16 * s);
    }
  };
  fetch(tile);
  // the operand: every column-map load of a thread first, then every operand load (two round trips in all, under
  // the first tile's loads); element e = 16 k + n, one per thread and step
  {
    int tc[NST];
#pragma unroll
    for (int u = 0; u < NST; ++u) {
      const int k = (tid + u * kBlock) / 16;
      tc[u] = (u < nst && k < ck) ? a.colmap[k] : -1;
    }
    float xv[NST];
#pragma unroll
    for (int u = 0; u < NST; ++u) {
      const int n = (tid + u * kBlock) % 16;
      xv[u] = (tc[u] >= 0 && n < a.ncols) ? a.X[(int64_t)tc[u] * a.ldx + a.col0 + n] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < NST; ++u) {
      const int e = tid + u * kBlock;
      const int k = e / 16, n = e % 16;
      if (u < nst) lds[((k >> 2) * 16 + n) * 4 + (k & 3)] = xv[u];
    }
  }
  __syncthreads();
  for (; tile < ntiles; tile += tstride) {
    v4f acc = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      if (s < nst) {
        const float4 bv = *reinterpret_cast<const float4*>(lds + ((4 * s + q) * 16 + li) * 4);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s].x, bv.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s].y, bv.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s].z, bv.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s].w, bv.w, acc, 0, 0, 0);
      }
    }
    const int64_t row0 = tile * 16;
    fetch(tile + tstride);
    // register r of lane (li, q) = P[row 4 q + r][column li]
    if (li < a.ncols) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t row = row0 + 4 * q + r;
        if (row < a.r_out) {
          float* op = a.out + row * a.ldo + a.col0 + li;
          if (a.nt_out) __builtin_nontemporal_store(acc[r], op);
          else *op = acc[r];
        }
      }
    }
  }
}

// Tables wider than 256 columns (up to 1024): the same product in chunks of 256 columns.  A wavefront walks the
// (tile, chunk) pairs of its tiles in order, one accumulator per tile; the whole operand (ck x 16) stays in LDS.
constexpr int kPsChunk = 16;         // 16-column steps per chunk

__global__ __launch_bounds__(kBlock) void lmm_prod_stream_chunked_kernel(LmmArgs a, int nst) {
  extern __shared__ __align__(16) float lds[];       // Xs [4 nst][16][4]
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int64_t tstride = (int64_t)gridDim.x * kPsWaves;
  const int nchunks = (nst + kPsChunk - 1) / kPsChunk;
  const int ck = a.ck;
  float4 av[kPsChunk];
  auto fetch = [&](int64_t t, int kc) {
    const int64_t row = min(t * 16 + li, a.d_rows - 1);       // clamped; rows beyond the table are never stored
    const float* rp = a.D + row * ck + 4 * q;
#pragma unroll
    for (int s = 0; s < kPsChunk; ++s) {
      const int col = 16 * (kc * kPsChunk + s) + 4 * q;
      const float4 v = *reinterpret_cast<const float4*>(rp + min(col, ck - 4) - 4 * q);
      av[s] = (col < ck && t < ntiles) ? v : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
  };
  int64_t tile = (int64_t)blockIdx.x * kPsWaves + wave;
  fetch(min(tile, ntiles - 1), 0);
  for (int e = tid; e < 16 * nst * 16; e += kBlock) {         // element e = 16 k + n
    const int k = e / 16, n = e % 16;
    const int t = k < ck ? a.colmap[k] : -1;
    lds[((k >> 2) * 16 + n) * 4 + (k & 3)] = (t >= 0 && n < a.ncols) ? a.X[(int64_t)t * a.ldx + a.col0 + n] : 0.0f;
  }
  __syncthreads();
  for (; tile < ntiles; tile += tstride) {
    v4f acc = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
    for (int kc = 0; kc < nchunks; ++kc) {
      float4 ac[kPsChunk];
#pragma unroll
      for (int s = 0; s < kPsChunk; ++s) ac[s] = av[s];
      // the next chunk of this tile, or the first chunk of the wavefront's next tile
      if (kc + 1 < nchunks) fetch(tile, kc + 1);
      else fetch(min(tile + tstride, ntiles - 1), 0);
#pragma unroll
      for (int s = 0; s < kPsChunk; ++s) {
        const int step = min(kc * kPsChunk + s, nst - 1);     // (steps beyond the table multiply zeros)
        const float4 bv = *reinterpret_cast<const float4*>(lds + ((4 * step + q) * 16 + li) * 4);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[s].x, bv.x, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[s].y, bv.y, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[s].z, bv.z, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[s].w, bv.w, acc, 0, 0, 0);
      }
    }
    const int64_t row0 = tile * 16;
    if (li < a.ncols) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t row = row0 + 4 * q + r;
        if (row < a.r_out) {
          float* op = a.out + row * a.ldo + a.col0 + li;
          if (a.nt_out) __builtin_nontemporal_store(acc[r], op);
          else *op = acc[r];
        }
      }
    }
  }
}

typedef void (*PsFn)(LmmArgs, int);

int ps_slots(PsFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static PsFn seen_fn[32];
  static size_t seen_lds[32];
  static int seen_slots[32];
  static int n_seen = 0;
  for (int i = 0; i < n_seen; ++i)
    if (seen_fn[i] == fn && seen_lds[i] == lds_bytes) return seen_slots[i];
  int dev = 0, cus = 256, per_cu = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    cus = prop.multiProcessorCount;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, lds_bytes) != hipSuccess ||
      per_cu < 1)
    per_cu = 1;
  if (n_seen < 32) { seen_fn[n_seen] = fn; seen_lds[n_seen] = lds_bytes; seen_slots[n_seen] = per_cu * cus; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// A dense table with 16-byte aligned rows of at most 1024 columns (more than 256: in chunks), a result of at most 16
// columns, no gathers and no epilogue.
bool lmm_prod_stream_supported(const LmmArgs& a, int vec, int mode) {
  if (mode != 0 || a.D == nullptr || vec != 4 || a.ck < 4 || a.ck % 4 != 0 || a.ck > 1024) return false;
  if (a.g.n != 0 || a.grad_partial != nullptr || a.ncols < 1 || a.ncols > 16 || a.d_rows < 1) return false;
  if (reinterpret_cast<uintptr_t>(a.D) % 16 != 0 || a.d_rows < a.r_out) return false;
  return true;
}

hipError_t launch_lmm_prod_stream(const LmmArgs& a, hipStream_t st) {
  if (!lmm_prod_stream_supported(a, 4, 0)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nst = (a.ck + 15) / 16;
  if (nst > 16) {
    const size_t lds_bytes = (size_t)16 * nst * 16 * sizeof(float);
    const int64_t ntiles = (a.r_out + 15) / 16;
    int64_t grid = (ntiles + kPsWaves - 1) / kPsWaves;
    grid = std::min<int64_t>(grid, ps_slots(lmm_prod_stream_chunked_kernel, lds_bytes));
    hipLaunchKernelGGL(lmm_prod_stream_chunked_kernel, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, nst);
    return hipGetLastError();
  }
  PsFn fn = nst <= 2 ? lmm_prod_stream_kernel<2>
          : nst <= 4 ? lmm_prod_stream_kernel<4>
          : nst <= 8 ? lmm_prod_stream_kernel<8>
          : nst <= 13 ? lmm_prod_stream_kernel<13> : lmm_prod_stream_kernel<16>;
  const size_t lds_bytes = (size_t)16 * nst * 16 * sizeof(float);
  const int64_t ntiles = (a.r_out + 15) / 16;
  int64_t grid = (ntiles + kPsWaves - 1) / kPsWaves;
  grid = std::min<int64_t>(grid, ps_slots(fn, lds_bytes));      // one round of resident workgroups
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, nst);
  return hipGetLastError();
}

}  // namespace ilargi
