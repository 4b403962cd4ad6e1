// One gradient-descent iteration of Alg. 1 for one model on a SMALL two-table star join T = [S | I_R R] (or a
// single table S), in a single launch of a single workgroup.  A schema of a few hundred KiB is bound by the
// latency of dependent launches and cache round trips, not by bandwidth: the factorized iteration otherwise
// takes five launches.  Here every global load of the iteration is requested at the start and the tables stay in
// registers (the entity table: up to 16 float4 per thread), so the whole iteration costs one round trip:
//
//   P = R (M_R^T w)                          thread per row of R                (Sec. 2.2, left multiply)
//   z_i = S[i] . w_S + P[row_idx[i]],  e_i   thread per target row              (assembly, residual of Alg. 1)
//   Z = I_R^T e                              thread per row of R, entries of the inverse index in order (LDS)
//   G_R = R^T Z,  G_S = S^T e                per-thread products added in a fixed order: butterfly inside the
//                                            wavefronts, wavefronts in order
//   w  -= lr * (M_S G_S + M_R G_R) / r_T     thread per target column, sources in plan order
#include <algorithm>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

constexpr int kSmallThreads = 1024;
constexpr int kSmallWaves = kSmallThreads / kWave;

__device__ __forceinline__ float small_sigmoid(float z) {
  if (z >= 0.0f) return 1.0f / (1.0f + __expf(-z));
  float e = __expf(z);
  return e / (1.0f + e);
}

__device__ __forceinline__ float small_softplus(float z) { return fmaxf(z, 0.0f) + log1pf(__expf(-fabsf(z))); }

constexpr int kSmallRowVecs = 16;          // float4 of the entity table a thread keeps in registers

template <int NV>
__device__ __forceinline__ float small_dot(const float4 (&v)[NV], const float* wk) {
  float acc = 0.0f;
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const float4 w = reinterpret_cast<const float4*>(wk)[q];
    acc = fmaf(v[q].x, w.x, fmaf(v[q].y, w.y, fmaf(v[q].z, w.z, fmaf(v[q].w, w.w, acc))));
  }
  return acc;
}

// NVS: float4 per row of the entity table S (row i = target row i); NVR: float4 per row of the joined table R
// (0: there is none).  MODE 1: linear regression, MODE 2: logistic regression.
// Every global load of the iteration is requested at the start, in one round trip: a thread's rows of S (up to
// 16 / NVS, rows tid + 1024 u), their labels and keys, its row of R with its two row pointers, its share of the
// inverse index (copied to LDS) and the weights.  The rest of the iteration works on registers and LDS.
template <int NVS, int NVR, int MODE>
__global__ __launch_bounds__(kSmallThreads) void small_star_kernel(SmallStarArgs a) {
  constexpr int UI = kSmallRowVecs / NVS;
  constexpr int NR = NVR > 0 ? NVR : 1;
  extern __shared__ float lds[];
  float* wk = lds;                                   // [2][16] the weights in source-column order (S, then R)
  float* gl = wk + 32;                               // [2][16] gradient blocks
  float* pz = gl + 32 + 33 * kWave;                  // [1024] products of R (after the [33][64] second-stage sums)
  float* es = pz + kSmallThreads;                    // [r_T] residual
  int* pl = reinterpret_cast<int*>(es + a.r_T);      // [nnz] inverse index entries
  const int tid = threadIdx.x;

  float4 sv[UI][NVS];
  float yv[UI];
  int jr[UI];
#pragma unroll
  for (int u = 0; u < UI; ++u) {
    const int i = tid + u * kSmallThreads;
    const bool live = i < a.r_T;
#pragma unroll
    for (int q = 0; q < NVS; ++q)
      sv[u][q] = (live && q < a.cs / 4) ? reinterpret_cast<const float4*>(a.S + (int64_t)i * a.cs)[q] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    yv[u] = live ? a.y[i] : 0.0f;
    jr[u] = (NVR > 0 && live) ? a.idx[i] : -1;
  }
  float4 rv[NR];
  int rp0 = 0, rp1 = 0;
  if constexpr (NVR > 0) {
    const bool live = tid < a.r_R;
#pragma unroll
    for (int q = 0; q < NVR; ++q)
      rv[q] = (live && q < a.cr / 4) ? reinterpret_cast<const float4*>(a.R + (int64_t)tid * a.cr)[q] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (live) { rp0 = a.rowptr[tid]; rp1 = a.rowptr[tid + 1]; }
    int pv[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int p = tid + u * kSmallThreads;
      pv[u] = p < a.nnz ? a.perm[p] : 0;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int p = tid + u * kSmallThreads;
      if (p < a.nnz) pl[p] = pv[u];
    }
  }
  float wold = 0.0f;
  int tcs = -1, tcr = -1;
  if (tid < a.c_T) {
    wold = a.W[(int64_t)tid * a.ldw + a.col];
    tcs = a.tcol_s[tid];
    if constexpr (NVR > 0) tcr = a.tcol_r[tid];
  }
  if (tid < 32) {
    const int k = tid / 16, j = tid % 16;
    const int t = a.colmap[k][j];
    wk[tid] = t >= 0 ? a.W[(int64_t)t * a.ldw + a.col] : 0.0f;
  }
  __syncthreads();

  // P = R w_R  (Sec. 2.2: the per-source product)
  if constexpr (NVR > 0) {
    if (tid < a.r_R) pz[tid] = small_dot<NVR>(rv, wk + 16);
    __syncthreads();
  }
  // assembly, residual and loss of Alg. 1
  float ev[UI];
  float loss_local = 0.0f;
#pragma unroll
  for (int u = 0; u < UI; ++u) {
    const int i = tid + u * kSmallThreads;
    ev[u] = 0.0f;
    if (i < a.r_T) {
      float z = small_dot<NVS>(sv[u], wk);
      if (jr[u] >= 0) z += pz[jr[u]];
      if constexpr (MODE == 1) {
        ev[u] = z - yv[u];
        loss_local = fmaf(ev[u], ev[u], loss_local);
      } else {
        ev[u] = small_sigmoid(z) - yv[u];
        loss_local += small_softplus(z) - yv[u] * z;
      }
      es[i] = ev[u];
    }
  }
  __syncthreads();
  // Z = I_R^T e (entries of a row in index order) and this thread's terms of R^T Z, S^T e and the loss
  constexpr int NVALS = 4 * (NVS + NVR) + 1;
  float vals[NVALS];
  {
    float4 accs[NVS];
#pragma unroll
    for (int q = 0; q < NVS; ++q) accs[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
    for (int u = 0; u < UI; ++u)
#pragma unroll
      for (int q = 0; q < NVS; ++q) {
        accs[q].x = fmaf(sv[u][q].x, ev[u], accs[q].x); accs[q].y = fmaf(sv[u][q].y, ev[u], accs[q].y);
        accs[q].z = fmaf(sv[u][q].z, ev[u], accs[q].z); accs[q].w = fmaf(sv[u][q].w, ev[u], accs[q].w);
      }
#pragma unroll
    for (int q = 0; q < NVS; ++q) { vals[4 * q] = accs[q].x; vals[4 * q + 1] = accs[q].y; vals[4 * q + 2] = accs[q].z; vals[4 * q + 3] = accs[q].w; }
  }
  if constexpr (NVR > 0) {
    float zr = 0.0f;
    for (int p = rp0; p < rp1; ++p) zr += es[pl[p]];
#pragma unroll
    for (int q = 0; q < NVR; ++q) {
      vals[4 * (NVS + q)] = rv[q].x * zr; vals[4 * (NVS + q) + 1] = rv[q].y * zr;
      vals[4 * (NVS + q) + 2] = rv[q].z * zr; vals[4 * (NVS + q) + 3] = rv[q].w * zr;
    }
  }
  vals[NVALS - 1] = loss_local;
  __syncthreads();                                   // es, pz and pl are dead: their LDS serves the sums
  // workgroup sums in a fixed order through LDS: red[v][t] <- value v of thread t; thread (v, part) adds the
  // entries part, part + 64, ...; then thread v adds the 64 parts in order
  float* red = pz;                                   // [NVALS][1024]
  float* red2 = gl + 32;                             // [NVALS][64]
#pragma unroll
  for (int v = 0; v < NVALS; ++v) red[v * kSmallThreads + tid] = vals[v];
  __syncthreads();
  for (int v = tid / kWave; v < NVALS; v += kSmallWaves) {
    const int part = tid % kWave;
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < kSmallThreads / kWave; ++k) sum += red[v * kSmallThreads + part + kWave * k];
    red2[v * kWave + part] = sum;
  }
  __syncthreads();
  if (tid < NVALS) {
    float sum = 0.0f;
    for (int k = 0; k < kWave; ++k) sum += red2[tid * kWave + k];
    if (tid < 4 * NVS) gl[tid] = sum;                                  // column tid of S
    else if (tid < NVALS - 1) gl[16 + tid - 4 * NVS] = sum;            // column tid - 4 NVS of R
    else if (a.loss != nullptr) a.loss[a.col] = sum * a.loss_scale;    // loss at the weights the iteration started from
  }
  __syncthreads();
  // column scatter through the maps, sources in their order in the plan, and the update of Alg. 1
  if (tid < a.c_T && (tcs >= 0 || tcr >= 0)) {
    float g = 0.0f;
    if (a.s_first) { if (tcs >= 0) g += gl[tcs]; if (tcr >= 0) g += gl[16 + tcr]; }
    else { if (tcr >= 0) g += gl[16 + tcr]; if (tcs >= 0) g += gl[tcs]; }
    a.W[(int64_t)tid * a.ldw + a.col] = wold - a.lr[a.col] * (g * a.inv_rT);
  }
}

typedef void (*SmallFn)(SmallStarArgs);

template <int NVS, int NVR>
SmallFn small_pick_mode(int mode) { return mode == 1 ? small_star_kernel<NVS, NVR, 1> : small_star_kernel<NVS, NVR, 2>; }

template <int NVS>
SmallFn small_pick_r(int nvr, int mode) {
  switch (nvr) {
    case 0: return small_pick_mode<NVS, 0>(mode);
    case 1: return small_pick_mode<NVS, 1>(mode);
    case 2: return small_pick_mode<NVS, 2>(mode);
    case 3: return small_pick_mode<NVS, 3>(mode);
    default: return small_pick_mode<NVS, 4>(mode);
  }
}

}  // namespace

// Rows of the entity table a thread can keep in registers when its rows have nvs float4.
int small_star_max_rows(int nvs) { return kSmallThreads * (kSmallRowVecs / nvs); }

size_t small_star_lds_bytes(const SmallStarArgs& a) {
  // weights and gradient blocks, second-stage sums, then the larger of (products, residual, index entries) and the
  // per-thread terms of the final sums, which reuse that space
  const size_t work = (size_t)kSmallThreads + a.r_T + a.nnz;
  const size_t sums = (size_t)(a.cs + (a.R != nullptr ? a.cr : 0) + 1) * kSmallThreads;
  return sizeof(float) * (64 + 33 * kWave + std::max(work, sums));
}

hipError_t launch_small_star(const SmallStarArgs& a, int mode, hipStream_t st) {
  const int nvs = a.cs / 4, nvr = a.R != nullptr ? a.cr / 4 : 0;
  const size_t lds = small_star_lds_bytes(a);
  if (nvs < 1 || nvs > 4 || nvr > 4 || a.r_T > small_star_max_rows(nvs) || a.r_R > kSmallThreads ||
      a.nnz > 16 * kSmallThreads || a.c_T > kSmallThreads || lds > kSmallGdMaxLds)
    return hipErrorInvalidValue;
  SmallFn fn = nvs == 1 ? small_pick_r<1>(nvr, mode) : nvs == 2 ? small_pick_r<2>(nvr, mode)
             : nvs == 3 ? small_pick_r<3>(nvr, mode) : small_pick_r<4>(nvr, mode);
  if (lds > (64 << 10)) {
    // more dynamic LDS than a kernel may use by default
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(fn, dim3(1), dim3(kSmallThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace ilargi
