// Assembly pass of the left multiply for operands of 8, 12 or 16 columns over an identity source with short rows
// (at most 32 columns, float4-aligned):
//   out[i, :] = D[i, :] X_D + sum_s P_s[row_idx_s[i], :]          (paper, Sec. 2.2)
// Per target row this moves 4 c_D + 4 + 8 c bytes and needs c_D c multiply-adds: bandwidth-bound by a wide margin
// (c_D c / 2 flops per moved float at most), so the products are plain FMAs and the kernel is shaped around its
// three memory streams.  Wavefronts are autonomous (no workgroup barrier after the operand is staged):
//   - the table is read as one flat stream of float4, 64 rows per step, the next step's rows already in flight;
//     the rows pass through a wavefront-private LDS tile because the product wants them in another mapping;
//   - lane (r, g) = (lane / 4 + 16 q, lane % 4), q = 0..3, forms columns 4 g .. 4 g + 3 of four rows: it gathers
//     its float4 of every joined product row (the four lanes of a row fetch one contiguous row of P) and stores its
//     float4 of the result, so every store instruction of the wavefront writes 16 whole rows, 64 c bytes in a run;
//   - operand values X_D come from a workgroup-wide LDS copy, four consecutive columns per 128-bit read.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

__device__ __forceinline__ void fw_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kFwGather = 3;                 // gathered sources
constexpr int kFwWaves = kBlock / kWave;
constexpr int kFwN = 16;                     // operand columns of the staged operand (zero beyond ncols)

typedef float nt4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int64_t fw_gather_row(const GatherArgs& g, int s, int64_t i) {
  if (g.idx[s] != nullptr) return g.idx[s][i];
  return i < g.rows[s] ? i : -1;
}

// NVT: compile-time bound of nvec = ck / 4.  stride: floats between rows of the wavefront's tile.
template <int NVT>
__global__ __launch_bounds__(kBlock) void lmm_flat_wide_kernel(LmmArgs a, int stride, int wave_floats) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int nvec = a.ck / 4;
  float* Xs = lds;                                             // [ck][16]
  float* Ss = lds + (size_t)4 * NVT * kFwN + (size_t)wave * wave_floats;   // [64][stride] this wavefront's rows
  int* Is = reinterpret_cast<int*>(Ss + kWave * stride);       // [kFwGather][64] row indices of the step
  const int g4 = lane % 4, rl = lane / 4;                      // output columns 4 g4 .., rows rl + 16 q
  const bool col_live = 4 * g4 < a.ncols;
  const int64_t nchunks = (a.r_out + kWave - 1) / kWave;
  const int64_t cstride = (int64_t)gridDim.x * kFwWaves;
  int64_t chunk = (int64_t)blockIdx.x * kFwWaves + wave;

  float4 v[NVT], vn[NVT];
  auto load_chunk = [&](int64_t ch, float4 (&dst)[NVT]) {
    const int64_t r0 = ch * kWave;
    const float4* b4 = reinterpret_cast<const float4*>(a.D + r0 * a.ck);
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      const int e = u * kWave + lane;
      dst[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (u < nvec && ch < nchunks && r0 + e / nvec < a.d_rows) dst[u] = b4[e];
    }
  };
  int jn[kFwGather];
  auto load_idx = [&](int64_t ch) {
    const int64_t i = ch * kWave + lane;
#pragma unroll
    for (int s = 0; s < kFwGather; ++s)
      jn[s] = (s < a.g.n && ch < nchunks && i < a.r_out) ? (int)fw_gather_row(a.g, s, i) : -1;
  };
  // the first step's rows and indices are requested before anything else, so that they travel while the operand
  // is staged: column-map entries first, then the operand values they name (two round trips for all of a thread's
  // elements together)
  load_chunk(chunk, vn);
  load_idx(chunk);
  {
    constexpr int U = (4 * NVT * kFwN + kBlock - 1) / kBlock;
    int tc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = (tid + u * kBlock) / kFwN;
      tc[u] = j < a.ck ? a.colmap[j] : -1;
    }
    float xv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int n = (tid + u * kBlock) % kFwN;
      xv[u] = (tc[u] >= 0 && n < a.ncols) ? a.X[(int64_t)tc[u] * a.ldx + a.col0 + n] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (tid + u * kBlock < a.ck * kFwN) Xs[tid + u * kBlock] = xv[u];
  }
  __syncthreads();
  for (; chunk < nchunks; chunk += cstride) {
    const int64_t row0 = chunk * kWave;
#pragma unroll
    for (int u = 0; u < NVT; ++u) v[u] = vn[u];
    fw_wave_sync();                                            // the previous step's tile is consumed
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      if (u < nvec) {
        const int e = u * kWave + lane;
        const int r = e / nvec, part = e - r * nvec;
        *reinterpret_cast<float4*>(Ss + r * stride + 4 * part) = v[u];
      }
    }
#pragma unroll
    for (int s = 0; s < kFwGather; ++s)
      if (s < a.g.n) Is[s * kWave + lane] = jn[s];
    fw_wave_sync();
    load_chunk(chunk + cstride, vn);                           // next step's rows and indices go out now
    load_idx(chunk + cstride);
    // gathered product rows of this step
    float4 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
    for (int s = 0; s < kFwGather; ++s) {
      if (s < a.g.n) {
        float4 p[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = Is[s * kWave + rl + 16 * q];
          p[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
          if (j >= 0 && col_live) p[q] = *reinterpret_cast<const float4*>(a.g.P[s] + (int64_t)j * a.g.ldp + a.col0 + 4 * g4);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) { acc[q].x += p[q].x; acc[q].y += p[q].y; acc[q].z += p[q].z; acc[q].w += p[q].w; }
      }
    }
    // the identity source's product: four rows x four columns per lane
    for (int j4 = 0; j4 < nvec; ++j4) {
      float4 x[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = *reinterpret_cast<const float4*>(Xs + (4 * j4 + e) * kFwN + 4 * g4);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 d = *reinterpret_cast<const float4*>(Ss + (rl + 16 * q) * stride + 4 * j4);
        acc[q].x = fmaf(d.x, x[0].x, fmaf(d.y, x[1].x, fmaf(d.z, x[2].x, fmaf(d.w, x[3].x, acc[q].x))));
        acc[q].y = fmaf(d.x, x[0].y, fmaf(d.y, x[1].y, fmaf(d.z, x[2].y, fmaf(d.w, x[3].y, acc[q].y))));
        acc[q].z = fmaf(d.x, x[0].z, fmaf(d.y, x[1].z, fmaf(d.z, x[2].z, fmaf(d.w, x[3].z, acc[q].z))));
        acc[q].w = fmaf(d.x, x[0].w, fmaf(d.y, x[1].w, fmaf(d.z, x[2].w, fmaf(d.w, x[3].w, acc[q].w))));
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t i = row0 + rl + 16 * q;
      if (i < a.r_out && col_live) {
        float* op = a.out + i * a.ldo + a.col0 + 4 * g4;
        if (a.nt_out) {
          nt4f t = {acc[q].x, acc[q].y, acc[q].z, acc[q].w};
          __builtin_nontemporal_store(t, reinterpret_cast<nt4f*>(op));
        } else {
          *reinterpret_cast<float4*>(op) = acc[q];
        }
      }
    }
  }
}

typedef void (*FwFn)(LmmArgs, int, int);

int fw_nvt(int nvec) { return nvec <= 4 ? 4 : (nvec == 5 ? 5 : 8); }

int fw_slots(FwFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static FwFn seen_fn[16];
  static size_t seen_lds[16];
  static int seen_slots[16];
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
  if (n_seen < 16) { seen_fn[n_seen] = fn; seen_lds[n_seen] = lds_bytes; seen_slots[n_seen] = per_cu * cus; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// Identity source with float4-aligned rows of at most 8 float4, a result of 8, 12 or 16 columns whose rows (and
// those of the gathered products) are whole aligned float4s, at most three gathered sources, no epilogue.
bool lmm_flat_wide_supported(const LmmArgs& a, int vec, int mode) {
  if (mode != 0 || a.D == nullptr || vec != 4 || a.ck < 4 || a.ck % 4 != 0 || a.ck > 32 || a.g.n > kFwGather) return false;
  if (a.ncols < 8 || a.ncols > kFwN || a.ncols % 4 != 0 || a.col0 % 4 != 0 || a.ldo % 4 != 0) return false;
  if (reinterpret_cast<uintptr_t>(a.out) % 16 != 0 || a.grad_partial != nullptr) return false;
  for (int s = 0; s < a.g.n; ++s)
    if (a.g.ldp % 4 != 0 || reinterpret_cast<uintptr_t>(a.g.P[s]) % 16 != 0) return false;
  return true;
}

hipError_t launch_lmm_flat_wide(const LmmArgs& a, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!lmm_flat_wide_supported(a, 4, 0)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nvec = a.ck / 4;
  const int nvt = fw_nvt(nvec);
  const int stride = (nvec % 2 == 1) ? a.ck : a.ck + 4;         // an odd number of float4: rows spread over the banks
  int wave_floats = kWave * stride + kFwGather * kWave;
  wave_floats = (wave_floats + 3) / 4 * 4;
  const size_t lds_bytes = ((size_t)4 * nvt * kFwN + (size_t)kFwWaves * wave_floats) * sizeof(float);
  FwFn fn = nvt == 4 ? lmm_flat_wide_kernel<4> : (nvt == 5 ? lmm_flat_wide_kernel<5> : lmm_flat_wide_kernel<8>);
  const int64_t nchunks = (a.r_out + kWave - 1) / kWave;
  int64_t grid = (nchunks + kFwWaves - 1) / kFwWaves;
  grid = std::min<int64_t>(grid, fw_slots(fn, lds_bytes));       // one round of resident workgroups
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, stride, wave_floats);
  return hipGetLastError();
}

}  // namespace ilargi
