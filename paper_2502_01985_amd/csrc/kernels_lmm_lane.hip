// Assembly pass of the left multiply for ONE operand column over an identity source with short, 8-byte aligned rows
// (a number of columns that is 2 modulo 4, such as the 10-column entity table of the three-dimension benchmark), one
// lane per pair of target rows (the kernel is written for RPL rows per lane; RPL = 2 is what is built):
//   out[i] = D[i, :] x_D + sum_s P_s[row_idx_s[i]]                (paper, Sec. 2.2)
// with the residual and loss of Alg. 1 as epilogue (MODE 1 linear, MODE 2 logistic) and this workgroup's share of
// D^T e, the identity source's block of the gradient.
//
// A wavefront step covers 64 units (a unit = RPL consecutive rows = NV aligned float4): one contiguous run of
// memory that the wavefront reads as a flat stream of float4 (lane l takes float4 64 u + l: whole cache lines per
// instruction), writes to a private LDS tile and reads back transposed, lane l the NV float4 of unit l (a stride of
// NV float4 between lanes, conflict-free for the odd NV of 8-byte aligned rows).  From there on a row lives in one
// lane: the dot product with the operand (uniform values), the gathered product values, the epilogue and the
// gradient terms are plain per-lane arithmetic without partial sums through LDS or cross-lane exchange.
// The loop is branch-free for whole steps: every address is clamped to the table instead of guarded, lanes beyond the
// end contribute zeros, and only the store is predicated.  Requests run one step ahead (row indices two): at the top
// of a step everything it consumes was requested a whole step earlier (requesting the table rows two steps ahead
// measured the same).  Wavefronts are autonomous; the per-lane
// gradient and loss sums meet once, at the end, in a fixed order.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kLaneGather = 3;                 // gathered sources
constexpr int kLaneWaves = kBlock / kWave;

__device__ __forceinline__ void lane_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float lane_uniform(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}

// RPL rows per lane (1: rows of whole float4, 2: rows of an odd number of float2), NV float4 per unit.
template <int RPL, int NV, int MODE>
__global__ __launch_bounds__(kBlock) void lmm_lane_kernel(LmmArgs a) {
  constexpr int CK = 4 * NV / RPL;                              // columns of the table
  extern __shared__ v4f lds4[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  v4f* tile = lds4 + (size_t)wave * kWave * NV;

  float w[CK];                                                  // operand values, the same in every lane
#pragma unroll
  for (int j = 0; j < CK; ++j) {
    const int t = a.colmap[j];
    w[j] = lane_uniform(t >= 0 ? a.X[(int64_t)t * a.ldx + a.col0] : 0.0f);
  }
  const int ng = a.g.n;
  const int32_t* gidx[kLaneGather];
  const float* gP[kLaneGather];
#pragma unroll
  for (int s = 0; s < kLaneGather; ++s) {
    gidx[s] = s < ng ? a.g.idx[s] : nullptr;
    gP[s] = s < ng ? a.g.P[s] + a.col0 : nullptr;
  }
  const int64_t ldp = a.g.ldp;
  const int64_t nunits = a.r_out / RPL;                         // r_out is a multiple of RPL
  const int64_t nchunks = (nunits + kWave - 1) / kWave;
  const int64_t last_f4 = nunits * NV - 1;
  const v4f* D4 = reinterpret_cast<const v4f*>(a.D);
  const int64_t cstride = (int64_t)gridDim.x * kLaneWaves;
  int64_t chunk = (int64_t)blockIdx.x * kLaneWaves + wave;

  auto load_rows = [&](int64_t ch, v4f (&dst)[NV]) {
    const int64_t base = ch * (kWave * NV) + lane;
#pragma unroll
    for (int u = 0; u < NV; ++u) dst[u] = D4[min(base + u * kWave, last_f4)];
  };
  auto load_idx = [&](int64_t ch, int (&j)[kLaneGather][RPL]) {
    const int64_t unit = min(ch * kWave + lane, nunits - 1);
#pragma unroll
    for (int s = 0; s < kLaneGather; ++s) {
#pragma unroll
      for (int h = 0; h < RPL; ++h) j[s][h] = -1;
      if (s < ng) {
        if constexpr (RPL == 2) {
          const int2 t = *reinterpret_cast<const int2*>(gidx[s] + 2 * unit);
          j[s][0] = t.x; j[s][1] = t.y;
        } else {
          j[s][0] = gidx[s][unit];
        }
      }
    }
  };
  auto load_y = [&](int64_t ch, float (&y)[RPL]) {
    if constexpr (MODE != 0) {
      const int64_t unit = min(ch * kWave + lane, nunits - 1);
      if constexpr (RPL == 2) {
        const float2 t = *reinterpret_cast<const float2*>(a.y + 2 * unit);
        y[0] = t.x; y[1] = t.y;
      } else {
        y[0] = a.y[unit];
      }
    } else {
#pragma unroll
      for (int h = 0; h < RPL; ++h) y[h] = 0.0f;
    }
  };
  // a missing key reads row 0; its value is dropped when it is used
  auto gather = [&](const int (&j)[kLaneGather][RPL], float (&p)[kLaneGather][RPL]) {
#pragma unroll
    for (int s = 0; s < kLaneGather; ++s) {
#pragma unroll
      for (int h = 0; h < RPL; ++h) p[s][h] = 0.0f;
      if (s < ng) {
#pragma unroll
        for (int h = 0; h < RPL; ++h) p[s][h] = gP[s][(int64_t)max(j[s][h], 0) * ldp];
      }
    }
  };

  float gacc[CK];
#pragma unroll
  for (int j = 0; j < CK; ++j) gacc[j] = 0.0f;
  float loss_local = 0.0f;

  v4f vn[NV];
  int jc[kLaneGather][RPL], jn[kLaneGather][RPL];
  float pn[kLaneGather][RPL], yn[RPL];
  load_idx(chunk, jc);
  load_rows(chunk, vn);
  load_y(chunk, yn);
  load_idx(chunk + cstride, jn);
  gather(jc, pn);
  for (; chunk < nchunks; chunk += cstride) {
    // this step's values (all requested a step ago) leave the request registers
    float pc[kLaneGather][RPL], yc[RPL];
#pragma unroll
    for (int s = 0; s < kLaneGather; ++s)
#pragma unroll
      for (int h = 0; h < RPL; ++h) pc[s][h] = jc[s][h] >= 0 ? pn[s][h] : 0.0f;
#pragma unroll
    for (int h = 0; h < RPL; ++h) yc[h] = yn[h];
    lane_wave_sync();                                           // the previous step's tile is consumed
#pragma unroll
    for (int u = 0; u < NV; ++u) tile[u * kWave + lane] = vn[u];
    lane_wave_sync();
    // the next step's requests
#pragma unroll
    for (int s = 0; s < kLaneGather; ++s)
#pragma unroll
      for (int h = 0; h < RPL; ++h) jc[s][h] = jn[s][h];
    gather(jc, pn);
    load_y(chunk + cstride, yn);
    load_idx(chunk + 2 * cstride, jn);
    load_rows(chunk + cstride, vn);
    // lane = unit
    float f[4 * NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const v4f t = tile[lane * NV + k];
      f[4 * k] = t[0]; f[4 * k + 1] = t[1]; f[4 * k + 2] = t[2]; f[4 * k + 3] = t[3];
    }
    const int64_t unit = chunk * kWave + lane;
    const bool live = unit < nunits;
    float r[RPL];
#pragma unroll
    for (int h = 0; h < RPL; ++h) {
      float z0 = 0.0f, z1 = 0.0f;                               // two chains
#pragma unroll
      for (int j = 0; j < CK; j += 2) {
        z0 = fmaf(f[h * CK + j], w[j], z0);
        if (j + 1 < CK) z1 = fmaf(f[h * CK + j + 1], w[j + 1], z1);
      }
      float zz = z0 + z1;
#pragma unroll
      for (int s = 0; s < kLaneGather; ++s) zz += pc[s][h];
      if constexpr (MODE == 0) {
        r[h] = zz;
      } else if constexpr (MODE == 1) {
        r[h] = live ? zz - yc[h] : 0.0f;
        loss_local = fmaf(r[h], r[h], loss_local);
      } else {
        // one exponential serves the sigmoid and the softplus: e = exp(-|z|)
        const float e = __expf(-fabsf(zz));
        const float inv = __builtin_amdgcn_rcpf(1.0f + e);
        const float sg = zz >= 0.0f ? inv : e * inv;
        r[h] = live ? sg - yc[h] : 0.0f;
        loss_local += live ? fmaxf(zz, 0.0f) + __logf(1.0f + e) - yc[h] * zz : 0.0f;
      }
    }
    if (live) {
      float* op = a.out + unit * RPL * a.ldo + a.col0;
      if (a.ldo == 1 && RPL == 2) {
        typedef float v2f __attribute__((ext_vector_type(2)));
        const v2f t = {r[0], r[RPL - 1]};
        if (a.nt_out) __builtin_nontemporal_store(t, reinterpret_cast<v2f*>(op));
        else *reinterpret_cast<v2f*>(op) = t;
      } else {
#pragma unroll
        for (int h = 0; h < RPL; ++h) {
          if (a.nt_out) __builtin_nontemporal_store(r[h], op + (int64_t)h * a.ldo);
          else op[(int64_t)h * a.ldo] = r[h];
        }
      }
    }
    if constexpr (MODE != 0) {
#pragma unroll
      for (int h = 0; h < RPL; ++h)
#pragma unroll
        for (int j = 0; j < CK; ++j) gacc[j] = fmaf(f[h * CK + j], r[h], gacc[j]);
    }
  }

  if constexpr (MODE != 0) {
    // lanes by a fixed butterfly, then the wavefronts in order
    __syncthreads();
    float* red = reinterpret_cast<float*>(lds4);               // [waves][CK + 1]
#pragma unroll
    for (int j = 0; j <= CK; ++j) {
      float s = j < CK ? gacc[j < CK ? j : 0] : loss_local;
      for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      if (lane == 0) red[wave * (CK + 1) + j] = s;
    }
    __syncthreads();
    if (tid <= CK) {
      float s = 0.0f;
      for (int wv = 0; wv < kLaneWaves; ++wv) s += red[wv * (CK + 1) + tid];
      if (tid < CK) a.grad_partial[((int64_t)blockIdx.x * CK + tid) * kNarrowCT] = s;
      else a.loss_partial[(int64_t)blockIdx.x * kNarrowCT] = s;
    }
  }
}

typedef void (*LaneFn)(LmmArgs);

template <int RPL, int NV>
LaneFn pick_lane(int mode) {
  return mode == 0 ? lmm_lane_kernel<RPL, NV, 0> : (mode == 1 ? lmm_lane_kernel<RPL, NV, 1> : lmm_lane_kernel<RPL, NV, 2>);
}

// Built for rows of 6, 10 and 14 columns (pairs of 8-byte aligned rows).  For rows of whole float4 the same kernel
// (RPL = 1) measured 2 us faster than the flat-stream assembly on tables that sit in the last-level cache and 2 us
// slower on tables that come from memory, so those keep the flat-stream kernel.
LaneFn lane_fn(int rpl, int nv, int mode) {
  if (rpl != 2) return nullptr;
  switch (nv) {
    case 3: return pick_lane<2, 3>(mode);
    case 5: return pick_lane<2, 5>(mode);
    case 7: return pick_lane<2, 7>(mode);
    default: return nullptr;
  }
}

int lane_slots(LaneFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static LaneFn seen_fn[64];
  static int seen_slots[64];
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
  if (n_seen < 64) { seen_fn[n_seen] = fn; seen_slots[n_seen] = per_cu * cus; ++n_seen; }
  return per_cu * cus;
}

void lane_shape(const LmmArgs& a, int vec, int* rpl, int* nv) {
  *rpl = (vec == 2 && a.ck % 4 == 2) ? 2 : 1;
  *nv = *rpl * a.ck / 4;
}

}  // namespace

// One operand column; the identity source covers every target row (d_rows == r_out, an even number); rows of 6, 10
// or 14 columns (vec 2) on a 16-byte aligned base; one to three
// sources gathered through row indices (8-byte aligned when a lane takes two rows); with a gradient-descent mode the
// fused gradient is part of the kernel.
bool lmm_lane_supported(const LmmArgs& a, int vec, int mode, bool fuseg) {
  if (a.D == nullptr || a.ncols != 1 || a.g.n < 1 || a.g.n > kLaneGather || a.r_out <= 0 || a.d_rows != a.r_out) return false;
  if ((mode != 0) != fuseg) return false;
  if (mode != 0 && (a.y == nullptr || a.loss_partial == nullptr || a.grad_partial == nullptr)) return false;
  if (reinterpret_cast<uintptr_t>(a.D) % 16 != 0) return false;
  if (!((vec == 4 && a.ck % 4 == 0) || (vec == 2 && a.ck % 4 == 2))) return false;
  int rpl, nv;
  lane_shape(a, vec, &rpl, &nv);
  if (lane_fn(rpl, nv, mode) == nullptr || a.r_out % rpl != 0) return false;
  for (int s = 0; s < a.g.n; ++s) {
    if (a.g.idx[s] == nullptr) return false;
    if (rpl == 2 && reinterpret_cast<uintptr_t>(a.g.idx[s]) % 8 != 0) return false;
  }
  if (rpl == 2 && mode != 0 && reinterpret_cast<uintptr_t>(a.y) % 8 != 0) return false;
  if (rpl == 2 && a.ldo == 1 && reinterpret_cast<uintptr_t>(a.out + a.col0) % 8 != 0) return false;
  return true;
}

hipError_t launch_lmm_lane(const LmmArgs& a, int vec, int mode, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!lmm_lane_supported(a, vec, mode, mode != 0)) return hipErrorInvalidValue;
  int rpl, nv;
  lane_shape(a, vec, &rpl, &nv);
  LaneFn fn = lane_fn(rpl, nv, mode);
  size_t lds_bytes = (size_t)kLaneWaves * kWave * nv * sizeof(v4f);
  lds_bytes = std::max(lds_bytes, (size_t)kLaneWaves * (a.ck + 1) * sizeof(float));
  const int64_t nchunks = (a.r_out / rpl + kWave - 1) / kWave;
  int64_t grid = (nchunks + kLaneWaves - 1) / kLaneWaves;
  int64_t cap = lane_slots(fn, lds_bytes);
  if (mode != 0) cap = std::min<int64_t>(cap, kColredBlocks);
  if (grid > cap) grid = cap;
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a);
  return hipGetLastError();
}

}  // namespace ilargi
