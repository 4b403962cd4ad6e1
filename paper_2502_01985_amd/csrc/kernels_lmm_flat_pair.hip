// Assembly pass of the left multiply for narrow operands over an identity source whose rows are only 8-byte aligned
// (a number of columns that is 2 modulo 4, such as the 10-column entity table of the three-dimension benchmark):
//   out[i, :] = D[i, :] X_D + sum_s P_s[row_idx_s[i], :]          (paper, Sec. 2.2)
// with the residual and loss of Alg. 1 as epilogue and, with FUSEG, this workgroup's share of D^T E.
//
// Two consecutive rows of such a table are together a whole number of float4s that starts on a 16-byte boundary,
// so the table is read as a flat stream of float4 exactly like a table of r / 2 rows and 2 c columns ("pairs"),
// every lane busy, where a power-of-two group of lanes per 40-byte row leaves 3 of 8 idle and loads 8 bytes per
// lane.  Virtual column v of a pair is column v % c of its first (v < c) or second row: every float4 contributes to
// two partial dot products (with operand vectors that are zero in the other row's slots), lane l then finishes
// pair l of the step, i.e. the target rows 2 l and 2 l + 1: indices, gathered product rows, labels and output are
// accessed as neighbouring pairs.  For the gradient block the virtual columns v and v + c are added at the end.
// The table must have an even number of rows.  Wavefronts are autonomous: no workgroup barrier inside the loop.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

__device__ __forceinline__ void pair_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kPairGather = 3;                 // gathered sources
constexpr int kPairWaves = kBlock / kWave;

// NVT: compile-time bound of nvec = 2 ck / 4 (float4 per pair of rows).  wave_floats: LDS floats of one wavefront.
template <int NVT, int CT, int MODE, bool FUSEG>
__global__ __launch_bounds__(kBlock) void lmm_flat_pair_kernel(LmmArgs a, int wave_floats) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int ck2 = 2 * a.ck;
  const int nvec = ck2 / 4;
  const int ldp = nvec | 1;                                    // odd row stride of the partial-dot tiles
  float4* XsA = reinterpret_cast<float4*>(lds);                // [nvec][CT] operand values for the first row of a pair
  float4* XsB = XsA + NVT * CT;                                // [nvec][CT] ... for the second row
  float* wbase = lds + 8 * NVT * CT + (size_t)wave * wave_floats;
  float* PdA = wbase;                                          // [CT][64 * ldp] partial dot products, first rows
  float* PdB = PdA + CT * kWave * ldp;                         // ... second rows
  float* Es = PdB + CT * kWave * ldp;                          // [CT][2][64] residuals by pair (FUSEG)
  for (int e = tid; e < nvec * CT; e += kBlock) {
    const int part = e / CT, n = e - part * CT;
    float xa[4] = {0.0f, 0.0f, 0.0f, 0.0f}, xb[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (n < a.ncols) {
      for (int c = 0; c < 4; ++c) {
        const int v = 4 * part + c;
        const int j = v < a.ck ? v : v - a.ck;
        const int t = a.colmap[j];
        const float x = t >= 0 ? a.X[(int64_t)t * a.ldx + a.col0 + n] : 0.0f;
        if (v < a.ck) xa[c] = x; else xb[c] = x;
      }
    }
    XsA[e] = make_float4(xa[0], xa[1], xa[2], xa[3]);
    XsB[e] = make_float4(xb[0], xb[1], xb[2], xb[3]);
  }
  __syncthreads();

  // float4 number 64 u + lane of a step: its pair, its part of the pair, which of its slots belong to the first row
  int row_u[NVT], part_u[NVT];
#pragma unroll
  for (int u = 0; u < NVT; ++u) {
    const int e = u * kWave + lane;
    row_u[u] = u < nvec ? e / nvec : 0;
    part_u[u] = u < nvec ? e - row_u[u] * nvec : 0;
  }
  float loss_local[CT];
#pragma unroll
  for (int n = 0; n < CT; ++n) loss_local[n] = 0.0f;
  float4 gacc[FUSEG ? NVT : 1][CT];
#pragma unroll
  for (int u = 0; u < (FUSEG ? NVT : 1); ++u)
#pragma unroll
    for (int n = 0; n < CT; ++n) gacc[u][n] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

  const int64_t npairs = (a.r_out + 1) / 2;
  const int64_t nchunks = (npairs + kWave - 1) / kWave;
  const int64_t cstride = (int64_t)gridDim.x * kPairWaves;
  int64_t chunk = (int64_t)blockIdx.x * kPairWaves + wave;
  // the gathered sources' pointers, read from the kernel arguments once
  const int32_t* gidx[kPairGather];
  const float* gP[kPairGather];
  int64_t grows[kPairGather];
#pragma unroll
  for (int s = 0; s < kPairGather; ++s) {
    gidx[s] = s < a.g.n ? a.g.idx[s] : nullptr;
    gP[s] = s < a.g.n ? a.g.P[s] + a.col0 : nullptr;
    grows[s] = s < a.g.n ? a.g.rows[s] : 0;
  }
  const int ng = a.g.n, ldp_g = a.g.ldp;
  const int64_t r_out = a.r_out;
  int jn[kPairGather][2];
  auto load_idx = [&](int64_t ch) {
    const int64_t i = 2 * (ch * kWave + lane);
#pragma unroll
    for (int s = 0; s < kPairGather; ++s) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const bool in = s < ng && ch < nchunks && i + h < r_out;
        int j = -1;
        if (in) j = gidx[s] != nullptr ? gidx[s][i + h] : (i + h < grows[s] ? (int)(i + h) : -1);
        jn[s][h] = j;
      }
    }
  };
  float4 v[NVT], vn[NVT];
  auto load_chunk = [&](int64_t ch, float4 (&dst)[NVT]) {
    const int64_t p0 = ch * kWave;                             // first pair of the step
    const float4* b4 = reinterpret_cast<const float4*>(a.D + 2 * p0 * a.ck);
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      dst[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (u < nvec && ch < nchunks && 2 * (p0 + row_u[u]) < a.d_rows) dst[u] = b4[u * kWave + lane];
    }
  };
  load_idx(chunk);
  load_chunk(chunk, vn);
  for (; chunk < nchunks; chunk += cstride) {
    const int64_t i0 = 2 * (chunk * kWave + lane);            // this lane's two target rows: i0, i0 + 1
    const bool live0 = i0 < a.r_out, live1 = i0 + 1 < a.r_out;
#pragma unroll
    for (int u = 0; u < NVT; ++u) v[u] = vn[u];
    load_chunk(chunk + cstride, vn);
    // gathered product rows of this step (indices were prefetched), labels, next step's indices
    float gsum[2][CT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int n = 0; n < CT; ++n) gsum[h][n] = 0.0f;
#pragma unroll
    for (int s = 0; s < kPairGather; ++s) {
      if (s < ng) {
        // branch-free: a missing key reads row 0 and contributes nothing
        float pv[2][CT];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const float* p = gP[s] + (int64_t)max(jn[s][h], 0) * ldp_g;
#pragma unroll
          for (int n = 0; n < CT; ++n) pv[h][n] = n < a.ncols ? p[n] : 0.0f;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int n = 0; n < CT; ++n) gsum[h][n] += jn[s][h] >= 0 ? pv[h][n] : 0.0f;
      }
    }
    float yi[2] = {0.0f, 0.0f};
    if constexpr (MODE != 0) {
      yi[0] = a.y[min(i0, r_out - 1)];
      yi[1] = a.y[min(i0 + 1, r_out - 1)];
    }
    load_idx(chunk + cstride);
    // partial dot products into the tiles
    pair_wave_sync();                                          // the previous step's tiles are consumed
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      if (u < nvec) {
#pragma unroll
        for (int n = 0; n < CT; ++n) {
          const float4 xa = XsA[part_u[u] * CT + n], xb = XsB[part_u[u] * CT + n];
          PdA[n * kWave * ldp + row_u[u] * ldp + part_u[u]] =
              fmaf(v[u].x, xa.x, fmaf(v[u].y, xa.y, fmaf(v[u].z, xa.z, v[u].w * xa.w)));
          PdB[n * kWave * ldp + row_u[u] * ldp + part_u[u]] =
              fmaf(v[u].x, xb.x, fmaf(v[u].y, xb.y, fmaf(v[u].z, xb.z, v[u].w * xb.w)));
        }
      }
    }
    pair_wave_sync();
    // lane = pair: sums of the two rows' partials, epilogue, stores
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float z[2] = {0.0f, 0.0f};
      const float* pa = PdA + n * kWave * ldp + lane * ldp;
      const float* pb = PdB + n * kWave * ldp + lane * ldp;
      for (int p = 0; p < nvec; ++p) { z[0] += pa[p]; z[1] += pb[p]; }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float zz = z[h] + gsum[h][n];
        float r = zz;
        const bool live = h == 0 ? live0 : live1;
        if (live && n < a.ncols) {
          if constexpr (MODE == 1) {
            r = zz - yi[h];
            loss_local[n] = fmaf(r, r, loss_local[n]);
          } else if constexpr (MODE == 2) {
            // one exponential serves the sigmoid and the softplus: e = exp(-|z|)
            const float e = __expf(-fabsf(zz));
            const float inv = __frcp_rn(1.0f + e);
            r = (zz >= 0.0f ? inv : e * inv) - yi[h];
            loss_local[n] += fmaxf(zz, 0.0f) + log1pf(e) - yi[h] * zz;
          }
          float* op = a.out + (i0 + h) * a.ldo + a.col0 + n;
          if (a.nt_out) __builtin_nontemporal_store(r, op);
          else *op = r;
        } else {
          r = 0.0f;
        }
        if constexpr (FUSEG) Es[(n * 2 + h) * kWave + lane] = r;
      }
    }
    if constexpr (FUSEG) {
      pair_wave_sync();
      // D^T E: every lane multiplies the float4s it still holds by the residual of the row each slot belongs to
#pragma unroll
      for (int u = 0; u < NVT; ++u) {
        if (u < nvec) {
          const int v0 = 4 * part_u[u];
#pragma unroll
          for (int n = 0; n < CT; ++n) {
            const float ea = Es[(n * 2) * kWave + row_u[u]], eb = Es[(n * 2 + 1) * kWave + row_u[u]];
            gacc[u][n].x = fmaf(v[u].x, v0 < a.ck ? ea : eb, gacc[u][n].x);
            gacc[u][n].y = fmaf(v[u].y, v0 + 1 < a.ck ? ea : eb, gacc[u][n].y);
            gacc[u][n].z = fmaf(v[u].z, v0 + 2 < a.ck ? ea : eb, gacc[u][n].z);
            gacc[u][n].w = fmaf(v[u].w, v0 + 3 < a.ck ? ea : eb, gacc[u][n].w);
          }
        }
      }
    }
  }

  __syncthreads();                                             // every wavefront is done with its tiles
  float* blk = lds + 8 * NVT * CT;                             // the wavefronts' LDS, free for the block's sums
  if constexpr (MODE != 0) {
    float* lsum = blk;                                         // [waves][CT]
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float s = loss_local[n];
      for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      if (lane == 0) lsum[wave * CT + n] = s;
    }
    __syncthreads();
    if (tid < CT) {
      float s = 0.0f;
      for (int w = 0; w < kPairWaves; ++w) s += lsum[w * CT + tid];
      a.loss_partial[(int64_t)blockIdx.x * kNarrowCT + tid] = s;
    }
    __syncthreads();
  }
  if constexpr (FUSEG) {
    // virtual column 4 part + c, operand column n: every (load u, lane l) with (64 u + l) % nvec == part contributes;
    // they are added in the order u, l for each wavefront, then the wavefronts in order, then columns v and v + ck
    float* gw = wbase;                                         // [NVT][64][CT] float4 of this wavefront
#pragma unroll
    for (int u = 0; u < NVT; ++u)
      if (u < nvec) {
#pragma unroll
        for (int n = 0; n < CT; ++n) reinterpret_cast<float4*>(gw)[(u * kWave + lane) * CT + n] = gacc[u][n];
      }
    pair_wave_sync();
    float mine = 0.0f;
    const int outs = ck2 * CT;                                 // at most 64
    if (lane < outs) {
      const int j = lane / CT, n = lane - j * CT;
      const int part = j / 4, c = j - part * 4;
      float m0 = 0.0f, m1 = 0.0f, m2 = 0.0f, m3 = 0.0f;
      for (int u = 0; u < nvec; ++u) {
        int l0 = (part - (u * kWave) % nvec) % nvec;
        if (l0 < 0) l0 += nvec;
        const float* col = gw + (size_t)(u * kWave * CT + n) * 4 + c;
        int l = l0;
        for (; l + 3 * nvec < kWave; l += 4 * nvec) {
          m0 += col[(size_t)l * CT * 4];
          m1 += col[(size_t)(l + nvec) * CT * 4];
          m2 += col[(size_t)(l + 2 * nvec) * CT * 4];
          m3 += col[(size_t)(l + 3 * nvec) * CT * 4];
        }
        for (; l < kWave; l += nvec) m0 += col[(size_t)l * CT * 4];
      }
      mine = (m0 + m1) + (m2 + m3);
    }
    __syncthreads();                                           // all wavefronts have read their own tiles
    float* gb = blk;                                           // [waves][outs]
    if (lane < outs) gb[wave * outs + lane] = mine;
    __syncthreads();
    if (tid < a.ck * CT) {
      const int j = tid / CT, n = tid - j * CT;
      float s = 0.0f;
      for (int w = 0; w < kPairWaves; ++w) s += gb[w * outs + j * CT + n];
      for (int w = 0; w < kPairWaves; ++w) s += gb[w * outs + (j + a.ck) * CT + n];
      a.grad_partial[((int64_t)blockIdx.x * a.ck + j) * kNarrowCT + n] = s;
    }
  }
}

typedef void (*PairFn)(LmmArgs, int);

template <int NVT, int CT>
PairFn pick_pair(int mode, bool fuseg) {
  if constexpr (NVT * CT <= 8) {
    if (fuseg) return mode == 1 ? lmm_flat_pair_kernel<NVT, CT, 1, true> : lmm_flat_pair_kernel<NVT, CT, 2, true>;
  }
  if (mode == 0) return lmm_flat_pair_kernel<NVT, CT, 0, false>;
  return mode == 1 ? lmm_flat_pair_kernel<NVT, CT, 1, false> : lmm_flat_pair_kernel<NVT, CT, 2, false>;
}

int pair_nvt(int nvec) { return nvec <= 3 ? 3 : (nvec <= 5 ? 5 : (nvec <= 7 ? 7 : 16)); }

int pair_slots(PairFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static PairFn seen_fn[64];
  static size_t seen_lds[64];
  static int seen_slots[64];
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
  if (n_seen < 64) { seen_fn[n_seen] = fn; seen_lds[n_seen] = lds_bytes; seen_slots[n_seen] = per_cu * cus; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// Identity source with an even number of rows of 2 (mod 4) columns, 8-byte aligned rows on a 16-byte aligned base,
// at most three gathered sources, and few enough (float4 per pair) x (operand columns) for the variant.
bool lmm_flat_pair_supported(const LmmArgs& a, int vec, bool fuseg) {
  if (a.D == nullptr || vec != 2 || a.ck < 2 || a.ck % 4 != 2 || a.d_rows % 2 != 0 || a.g.n > kPairGather || a.ncols < 1 ||
      a.ncols > kNarrowCT || reinterpret_cast<uintptr_t>(a.D) % 16 != 0)
    return false;
  const int nvec = a.ck / 2;
  const int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  const int nvt = pair_nvt(nvec);
  if (nvec > 16 || nvt * ct > 16) return false;
  if (fuseg && (nvt * ct > 8 || 2 * a.ck * ct > kWave)) return false;
  return true;
}

hipError_t launch_lmm_flat_pair(const LmmArgs& a, int mode, bool fuseg, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!lmm_flat_pair_supported(a, 2, fuseg)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nvec = a.ck / 2;
  const int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  const int nvt = pair_nvt(nvec);
  const int ldp = nvec | 1;
  int wave_floats = 2 * ct * kWave * ldp + 2 * ct * kWave;
  if (fuseg) wave_floats = std::max(wave_floats, nvt * kWave * ct * 4);
  wave_floats = (wave_floats + 3) / 4 * 4;
  const size_t lds_bytes = ((size_t)8 * nvt * ct + (size_t)kPairWaves * wave_floats) * sizeof(float);
  const int64_t nchunks = ((a.r_out + 1) / 2 + kWave - 1) / kWave;
  int64_t grid = (nchunks + kPairWaves - 1) / kPairWaves;
  PairFn fn = nullptr;
  if (nvt == 3) fn = ct == 1 ? pick_pair<3, 1>(mode, fuseg) : (ct == 2 ? pick_pair<3, 2>(mode, fuseg) : pick_pair<3, 4>(mode, fuseg));
  else if (nvt == 5) fn = ct == 1 ? pick_pair<5, 1>(mode, fuseg) : pick_pair<5, 2>(mode, fuseg);
  else if (nvt == 7) fn = ct == 1 ? pick_pair<7, 1>(mode, fuseg) : pick_pair<7, 2>(mode, fuseg);
  else fn = pick_pair<16, 1>(mode, fuseg);
  int64_t cap = pair_slots(fn, lds_bytes);
  if (fuseg || mode != 0) cap = std::min<int64_t>(cap, kColredBlocks);
  if (grid > cap) grid = cap;
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, wave_floats);
  return hipGetLastError();
}

}  // namespace ilargi
