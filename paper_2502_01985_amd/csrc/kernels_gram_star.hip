// Gram matrix of a two-table star join  T = [S | I_R R]  (crossprod, the rewrite of Sec. 2.2 on both factors):
// what the entity table contributes,
//   S^T S              and          Zc = I_R^T S   (rows of S summed per row of R; then S^T (I_R R) = Zc^T R),
// in ONE pass over S in join order.  As in the join-order gradient pass, a wavefront owns 16 rows of R and all
// target rows that join them (inverse index).  For every 16 staged rows of S the same LDS values serve as
//   A and B of  S^T S              (tile (i, j): A = columns 16 i.., B = columns 16 j.. of rows 4 q + r),
//   B of        Zc += Ind^T S      (A = 1 where row 4 q + r joins row li of the tile of R, else 0: exact sums).
// S is read once; the kernel keeps few registers, so that many wavefronts cover the latency of the gathered rows.
// S has at most 32 columns.  Per-workgroup partial blocks of S^T S are added afterwards in workgroup order, so the
// result is reproducible.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void gs_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kGsST = 32;            // target rows a wavefront stages at a time
constexpr int kGsJS = 2;             // 16-column tiles of S
constexpr int kGsLda = 36;           // LDS row stride of the staged rows of S
constexpr int kGsWavesPerBlock = kBlock / kWave;

template <bool VEC4>
__global__ __launch_bounds__(kBlock) void gram_star_kernel(GramStarArgs a, int rtiles) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  float* wbase = lds + (size_t)wave * (kGsST * kGsLda + 2 * kGsST + 32);
  float* As = wbase;                                          // [ST][lda] staged rows of S (zero beyond cs)
  int* iS = reinterpret_cast<int*>(As + kGsST * kGsLda);      // [ST] target row of each staged row
  int* jS = iS + kGsST;                                       // [ST] row of the R tile it joins (-1: none)
  int* rpS = jS + kGsST;                                      // [17] row pointers of the tile of R

  v4f sacc[3];                                                // S^T S tiles (0,0), (0,1), (1,1)
#pragma unroll
  for (int u = 0; u < 3; ++u) sacc[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  typedef typename std::conditional<VEC4, float4, float>::type SVal;
  constexpr int NV = VEC4 ? kGsST * 8 / kWave : kGsST * 32 / kWave;   // staging slots of a lane (32 columns per row)
  constexpr int gslots = VEC4 ? 8 : 32;
  const int glive = VEC4 ? a.cs / 4 : a.cs;
  const bool two = a.cs > 16;                                 // a second 16-column tile of S exists
  const float* Sb = a.Sp != nullptr ? a.Sp : a.S;

  for (int rt = blockIdx.x * kGsWavesPerBlock + wave; rt < rtiles; rt += gridDim.x * kGsWavesPerBlock) {
    const int64_t jb = (int64_t)rt * 16;
    const int p_begin = a.rowptr[jb];
    const int p_end = a.rowptr[min(jb + 16, a.r_R)];
    v4f zacc[kGsJS];
#pragma unroll
    for (int jt = 0; jt < kGsJS; ++jt) zacc[jt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
    // which row of the tile the p-th entry of the inverse index joins follows from the row pointers (the entries
    // of a row are consecutive): no need to gather the row index of every target row
    gs_wave_sync();
    if (lane <= 16) rpS[lane] = a.rowptr[min(jb + lane, a.r_R)];
    gs_wave_sync();
    auto joined = [&](int p) {
      int j = 0;
#pragma unroll
      for (int k = 1; k < 16; ++k) j += p >= rpS[k] ? 1 : 0;
      return j;
    };

    // the row of the table entry p of the inverse index stands for: its target row, or, in the join-ordered copy, p
    auto row_at = [&](int p) { return a.Sp != nullptr ? p : a.perm[p]; };
    int pi = (lane < kGsST && p_begin + lane < p_end) ? row_at(p_begin + lane) : -1;
    int pi_next = (lane < kGsST && p_begin + kGsST + lane < p_end) ? row_at(p_begin + kGsST + lane) : -1;
    int jl = pi >= 0 ? joined(p_begin + lane) : -1;
    gs_wave_sync();                                           // the previous tile's batches are consumed
    if (lane < kGsST) iS[lane] = pi;
    gs_wave_sync();
    SVal sv[NV];
    auto load_rows = [&](int cnt_rows) {
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int e = lane + u * kWave;
        const int r = e / gslots, g = e - r * gslots;
        if constexpr (VEC4) sv[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        else sv[u] = 0.0f;
        if (r < cnt_rows && g < glive) {
          const int64_t row = iS[r];
          if constexpr (VEC4) sv[u] = *reinterpret_cast<const float4*>(Sb + row * a.cs + 4 * g);
          else sv[u] = Sb[row * a.cs + g];
        }
      }
    };
    load_rows(min(kGsST, p_end - p_begin));
    for (int p0 = p_begin; p0 < p_end; p0 += kGsST) {
      const int cnt = min(kGsST, p_end - p0);
      const int cnt_next = max(0, min(kGsST, p_end - p0 - kGsST));
      gs_wave_sync();                                         // the previous batch is consumed
      if (lane < kGsST) { jS[lane] = jl; iS[lane] = pi_next; }
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int e = lane + u * kWave;
        const int r = e / gslots, g = e - r * gslots;
        if constexpr (VEC4) *reinterpret_cast<float4*>(As + r * kGsLda + 4 * g) = sv[u];
        else As[r * kGsLda + g] = sv[u];
      }
      gs_wave_sync();
      pi = pi_next;
      pi_next = (lane < kGsST && p0 + 2 * kGsST + lane < p_end) ? row_at(p0 + 2 * kGsST + lane) : -1;
      jl = pi >= 0 ? joined(p0 + kGsST + lane) : -1;
      load_rows(cnt_next);

      for (int t = 0; 16 * t < cnt; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = t * 16 + 4 * q + r;                 // rows beyond the batch hold zeros and join nothing
          const float a0 = As[row * kGsLda + li];
          const float ind = jS[row] == li ? 1.0f : 0.0f;
          sacc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, a0, sacc[0], 0, 0, 0);
          zacc[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(ind, a0, zacc[0], 0, 0, 0);
          if (two) {
            const float a1 = As[row * kGsLda + 16 + li];
            sacc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, a1, sacc[1], 0, 0, 0);
            sacc[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, a1, sacc[2], 0, 0, 0);
            zacc[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(ind, a1, zacc[1], 0, 0, 0);
          }
        }
      }
    }
    // Zc tile: register r of lane (li, q) is Zc[row 4 q + r of the tile][column 16 jt + li]
#pragma unroll
    for (int jt = 0; jt < kGsJS; ++jt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t j = jb + 4 * q + r;
        const int c = jt * 16 + li;
        if (j < a.r_R && c < a.cs) a.zc[j * a.cs + c] = zacc[jt][r];
      }
  }

  // the four wavefronts' shares of S^T S, added in wavefront order in LDS
  float* red = lds;                                           // [3][16][16]
  auto reduce_store = [&](const v4f& v, int w, int slot) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float* p = red + slot * 256 + (4 * q + r) * 16 + li;
      if (w == 0) *p = v[r];
      else *p += v[r];
    }
  };
  for (int w = 0; w < kGsWavesPerBlock; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int u = 0; u < 3; ++u) reduce_store(sacc[u], w, u);
    }
  }
  __syncthreads();
  // S^T S partial (upper-triangle tiles only; the caller reads the upper triangle)
  float* ss = a.ss_partial + (int64_t)blockIdx.x * a.cs * a.cs;
  for (int e = tid; e < 3 * 256; e += kBlock) {
    const int u = e / 256, i = (e % 256) / 16, j = e % 16;
    const int row = (u == 2 ? 16 : 0) + i, col = (u == 0 ? 0 : 16) + j;
    if (row < a.cs && col < a.cs) ss[row * a.cs + col] = red[e];
  }
}

typedef void (*GramStarFn)(GramStarArgs, int);

}  // namespace

bool gram_star_supported(int cs) { return cs >= 1 && cs <= 16 * kGsJS; }

// max_grid: the caller's bound on workgroups (sizes of the partial buffers).
hipError_t launch_gram_star(const GramStarArgs& a, int vec, int max_grid, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!gram_star_supported(a.cs) || a.r_R <= 0 || max_grid < 1) return hipErrorInvalidValue;
  const int rtiles = (int)((a.r_R + 15) / 16);
  GramStarFn fn = vec == 4 ? gram_star_kernel<true> : gram_star_kernel<false>;
  size_t lds_floats = (size_t)kGsWavesPerBlock * (kGsST * kGsLda + 2 * kGsST + 32);
  lds_floats = std::max(lds_floats, (size_t)3 * 256);
  const size_t lds_bytes = lds_floats * sizeof(float);
  static std::mutex cache_mutex;
  static int slots = 0;
  {
    std::lock_guard<std::mutex> lock(cache_mutex);
    if (slots == 0) {
      int dev = 0, cus = 256, per_cu = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(gram_star_kernel<true>), kBlock,
                                                       lds_bytes) != hipSuccess || per_cu < 1)
        per_cu = 1;
      slots = per_cu * cus;
    }
  }
  int64_t gx = (rtiles + kGsWavesPerBlock - 1) / kGsWavesPerBlock;
  gx = std::min<int64_t>(gx, std::min<int64_t>(slots, max_grid));     // one round of resident workgroups
  if (grid_out) *grid_out = (int)gx;
  hipLaunchKernelGGL(fn, dim3((unsigned)gx), dim3(kBlock), lds_bytes, st, a, rtiles);
  return hipGetLastError();
}

}  // namespace ilargi
