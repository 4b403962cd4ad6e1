// Assembly pass of the left multiply for narrow operands (at most four columns) over an identity source with
// short rows (at most 64 columns, float4-aligned):
//   out[i, :] = D[i, :] X_D + sum_s P_s[row_idx_s[i], :]          (paper, Sec. 2.2)
// with the residual and loss of Alg. 1 as epilogue (MODE 1 linear, MODE 2 logistic) and, with FUSEG, this
// workgroup's share of D^T E (the identity source's block of the gradient) from the table values still in
// registers.
//
// The table is read as one flat stream of float4: a wavefront takes 64 rows = nvec wavefront loads of 64
// consecutive float4, every lane busy whatever the row length (a 20-column table has 5 float4 per row; giving a
// row a power-of-two group of lanes leaves 3 lanes of 8 idle).  Lane l of load u holds float4 number 64 u + l of
// the chunk, i.e. part (64 u + l) % nvec of row (64 u + l) / nvec - the same part for every chunk, so its operand
// values are looked up once per chunk from a small LDS table.  Each lane writes its partial dot products to a
// wavefront-private LDS tile; then lane r adds up the nvec partials of row r and continues in "row mapping":
// row indices, gathered product rows, labels and the output are all accessed with lane = row, fully coalesced.
// Wavefronts are autonomous: no workgroup barrier inside the loop.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

__device__ __forceinline__ void flat_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kFlatGather = 3;                 // gathered sources (their row indices are prefetched a chunk ahead)
constexpr int kFlatWaves = kBlock / kWave;

// NVT: compile-time bound of nvec = ck / 4.  wave_floats: LDS floats of one wavefront.
template <int NVT, int CT, int MODE, bool FUSEG>
__global__ __launch_bounds__(kBlock) void lmm_flat_kernel(LmmArgs a, int wave_floats) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int nvec = a.ck / 4;
  const int ldp = nvec | 1;                                    // odd row stride of the partial-dot tile
  float4* Xs4 = reinterpret_cast<float4*>(lds);                // [nvec][CT]
  float* wbase = lds + 4 * NVT * CT + (size_t)wave * wave_floats;
  float* Pd = wbase;                                           // [CT][64 * ldp] partial dot products
  float* Es = Pd + CT * kWave * ldp;                           // [CT][64] residuals by row (FUSEG)
  // float4 number 64 u + lane of a chunk: its row, its part of the row, its place in the partial-dot tile
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

  const int64_t nchunks = (a.r_out + kWave - 1) / kWave;
  const int64_t cstride = (int64_t)gridDim.x * kFlatWaves;
  int64_t chunk = (int64_t)blockIdx.x * kFlatWaves + wave;
  // the gathered sources' pointers, read from the kernel arguments once
  const int32_t* gidx[kFlatGather];
  const float* gP[kFlatGather];
  int64_t grows[kFlatGather];
#pragma unroll
  for (int s = 0; s < kFlatGather; ++s) {
    gidx[s] = s < a.g.n ? a.g.idx[s] : nullptr;
    gP[s] = s < a.g.n ? a.g.P[s] + a.col0 : nullptr;
    grows[s] = s < a.g.n ? a.g.rows[s] : 0;
  }
  const int ng = a.g.n, ldp_g = a.g.ldp;
  const int64_t r_out = a.r_out;
  auto gather_row = [&](int s, int64_t i) -> int {
    return gidx[s] != nullptr ? gidx[s][i] : (i < grows[s] ? (int)i : -1);
  };
  int jn[kFlatGather];
#pragma unroll
  for (int s = 0; s < kFlatGather; ++s) {
    const int64_t i = chunk * kWave + lane;
    jn[s] = (s < ng && chunk < nchunks && i < r_out) ? gather_row(s, i) : -1;
  }
  // the chunk of the table, flat; the next chunk is requested before the current one is used, so that a
  // wavefront always has a chunk in flight
  float4 v[NVT], vn[NVT];
  auto load_chunk = [&](int64_t ch, float4 (&dst)[NVT]) {
    const int64_t r0 = ch * kWave;
    const float4* b4 = reinterpret_cast<const float4*>(a.D + r0 * a.ck);
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      dst[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (u < nvec && ch < nchunks && r0 + row_u[u] < a.d_rows) dst[u] = b4[u * kWave + lane];
    }
  };
  load_chunk(chunk, vn);
  // the operand is staged while the first chunk and its row indices travel
  for (int e = tid; e < nvec * CT; e += kBlock) {
    const int part = e / CT, n = e - part * CT;
    float4 x = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (n < a.ncols) {
      const int t0 = a.colmap[4 * part], t1 = a.colmap[4 * part + 1], t2 = a.colmap[4 * part + 2], t3 = a.colmap[4 * part + 3];
      if (t0 >= 0) x.x = a.X[(int64_t)t0 * a.ldx + a.col0 + n];
      if (t1 >= 0) x.y = a.X[(int64_t)t1 * a.ldx + a.col0 + n];
      if (t2 >= 0) x.z = a.X[(int64_t)t2 * a.ldx + a.col0 + n];
      if (t3 >= 0) x.w = a.X[(int64_t)t3 * a.ldx + a.col0 + n];
    }
    Xs4[e] = x;
  }
  __syncthreads();
  for (; chunk < nchunks; chunk += cstride) {
    const int64_t row0 = chunk * kWave;
    const int64_t i = row0 + lane;
    const bool rowlive = i < a.r_out;
#pragma unroll
    for (int u = 0; u < NVT; ++u) v[u] = vn[u];
    load_chunk(chunk + cstride, vn);
    // row mapping: gathered product rows of this chunk (indices were prefetched), labels, next chunk's indices
    float gsum[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) gsum[n] = 0.0f;
#pragma unroll
    for (int s = 0; s < kFlatGather; ++s) {
      if (s < ng) {
        // branch-free: a missing key reads row 0 and contributes nothing
        const float* p = gP[s] + (int64_t)max(jn[s], 0) * ldp_g;
        float pv[CT];
#pragma unroll
        for (int n = 0; n < CT; ++n) pv[n] = n < a.ncols ? p[n] : 0.0f;
#pragma unroll
        for (int n = 0; n < CT; ++n) gsum[n] += jn[s] >= 0 ? pv[n] : 0.0f;
      }
    }
    float yi = 0.0f;
    if constexpr (MODE != 0) yi = a.y[min(i, r_out - 1)];
    {
      const int64_t inext = i + cstride * kWave;
#pragma unroll
      for (int s = 0; s < kFlatGather; ++s)
        jn[s] = (s < ng && chunk + cstride < nchunks && inext < r_out) ? gather_row(s, inext) : -1;
    }
    // partial dot products into the tile
    flat_wave_sync();                                          // the previous chunk's tile is consumed
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      if (u < nvec) {
#pragma unroll
        for (int n = 0; n < CT; ++n) {
          const float4 x = Xs4[part_u[u] * CT + n];
          Pd[n * kWave * ldp + row_u[u] * ldp + part_u[u]] =
              fmaf(v[u].x, x.x, fmaf(v[u].y, x.y, fmaf(v[u].z, x.z, v[u].w * x.w)));
        }
      }
    }
    flat_wave_sync();
    // lane = row: sum of the row's partials, epilogue, store
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float z = 0.0f;
      const float* pr = Pd + n * kWave * ldp + lane * ldp;
      for (int p = 0; p < nvec; ++p) z += pr[p];
      z += gsum[n];
      float r = z;
      if (rowlive && n < a.ncols) {
        if constexpr (MODE == 1) {
          r = z - yi;
          loss_local[n] = fmaf(r, r, loss_local[n]);
        } else if constexpr (MODE == 2) {
          // one exponential serves the sigmoid and the softplus: e = exp(-|z|)
          const float e = __expf(-fabsf(z));
          const float inv = __frcp_rn(1.0f + e);
          r = (z >= 0.0f ? inv : e * inv) - yi;
          loss_local[n] += fmaxf(z, 0.0f) + log1pf(e) - yi * z;
        }
        float* op = a.out + i * a.ldo + a.col0 + n;
        if (a.nt_out) __builtin_nontemporal_store(r, op);
        else *op = r;
      } else {
        r = 0.0f;
      }
      if constexpr (FUSEG) Es[n * kWave + lane] = r;
    }
    if constexpr (FUSEG) {
      flat_wave_sync();
      // D^T E: every lane multiplies the float4s it still holds by the residual of their row
#pragma unroll
      for (int u = 0; u < NVT; ++u) {
        if (u < nvec) {
#pragma unroll
          for (int n = 0; n < CT; ++n) {
            const float er = Es[n * kWave + row_u[u]];
            gacc[u][n].x = fmaf(v[u].x, er, gacc[u][n].x);
            gacc[u][n].y = fmaf(v[u].y, er, gacc[u][n].y);
            gacc[u][n].z = fmaf(v[u].z, er, gacc[u][n].z);
            gacc[u][n].w = fmaf(v[u].w, er, gacc[u][n].w);
          }
        }
      }
    }
  }

  __syncthreads();                                             // every wavefront is done with its tiles
  float* blk = lds + 4 * NVT * CT;                             // the wavefronts' LDS, free for the block's sums
  if constexpr (MODE != 0) {
    // loss of this workgroup: butterfly inside each wavefront, then the wavefronts in order
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
      for (int w = 0; w < kFlatWaves; ++w) s += lsum[w * CT + tid];
      a.loss_partial[(int64_t)blockIdx.x * kNarrowCT + tid] = s;
    }
    __syncthreads();
  }
  if constexpr (FUSEG) {
    // column 4 part + c of the table, operand column n: every (load u, lane l) with (64 u + l) % nvec == part
    // contributes; they are added in the order u, l for each wavefront, then the wavefronts in order
    float* gw = wbase;                                         // [NVT][64][CT] float4 of this wavefront
#pragma unroll
    for (int u = 0; u < NVT; ++u)
      if (u < nvec) {
#pragma unroll
        for (int n = 0; n < CT; ++n) reinterpret_cast<float4*>(gw)[(u * kWave + lane) * CT + n] = gacc[u][n];
      }
    flat_wave_sync();
    float mine = 0.0f;
    const int outs = a.ck * CT;                                // at most 64
    if (lane < outs) {
      const int j = lane / CT, n = lane - j * CT;
      const int part = j / 4, c = j - part * 4;
      // four interleaved chains (a fixed order all the same) so that the LDS reads overlap
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
    if (tid < outs) {
      float s = 0.0f;
      for (int w = 0; w < kFlatWaves; ++w) s += gb[w * outs + tid];
      const int j = tid / CT, n = tid - j * CT;
      a.grad_partial[((int64_t)blockIdx.x * a.ck + j) * kNarrowCT + n] = s;
    }
  }
}

typedef void (*FlatFn)(LmmArgs, int);

template <int NVT, int CT>
FlatFn pick_flat(int mode, bool fuseg) {
  if constexpr (NVT * CT <= 8) {
    if (fuseg) return mode == 1 ? lmm_flat_kernel<NVT, CT, 1, true> : lmm_flat_kernel<NVT, CT, 2, true>;
  }
  if (mode == 0) return lmm_flat_kernel<NVT, CT, 0, false>;
  return mode == 1 ? lmm_flat_kernel<NVT, CT, 1, false> : lmm_flat_kernel<NVT, CT, 2, false>;
}

// Compile-time bound of the float4 per row that serves a table (5 = the 20-column entity table of the benchmark).
int flat_nvt(int nvec) { return nvec <= 4 ? 4 : (nvec == 5 ? 5 : (nvec <= 8 ? 8 : 16)); }

// Workgroups of a variant the device holds at once (cached: the query costs more than a launch).
int flat_slots(FlatFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static FlatFn seen_fn[64];
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

// Identity source with float4-aligned rows of at most 16 float4, at most three gathered sources, and few enough
// (float4 per row) x (operand columns) for the register and LDS budget of the variant.
bool lmm_flat_supported(const LmmArgs& a, int vec, bool fuseg) {
  if (a.D == nullptr || vec != 4 || a.ck < 4 || a.ck % 4 != 0 || a.g.n > kFlatGather || a.ncols < 1 || a.ncols > kNarrowCT) return false;
  const int nvec = a.ck / 4;
  const int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  const int nvt = flat_nvt(nvec);
  if (nvec > 16 || nvt * ct > 16) return false;
  if (fuseg && (nvt * ct > 8 || a.ck * ct > kWave)) return false;
  return true;
}

hipError_t launch_lmm_flat(const LmmArgs& a, int mode, bool fuseg, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!lmm_flat_supported(a, 4, fuseg)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nvec = a.ck / 4;
  const int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  const int nvt = flat_nvt(nvec);
  const int ldp = nvec | 1;
  int wave_floats = ct * kWave * ldp + ct * kWave;
  if (fuseg) wave_floats = std::max(wave_floats, nvt * kWave * ct * 4);
  wave_floats = (wave_floats + 3) / 4 * 4;                       // float4 alignment of the wavefronts' tiles
  const size_t lds_bytes = ((size_t)4 * nvt * ct + (size_t)kFlatWaves * wave_floats) * sizeof(float);
  const int64_t nchunks = (a.r_out + kWave - 1) / kWave;
  int64_t grid = (nchunks + kFlatWaves - 1) / kFlatWaves;
  FlatFn fn = nullptr;
  if (nvt == 4) fn = ct == 1 ? pick_flat<4, 1>(mode, fuseg) : (ct == 2 ? pick_flat<4, 2>(mode, fuseg) : pick_flat<4, 4>(mode, fuseg));
  else if (nvt == 5) fn = ct == 1 ? pick_flat<5, 1>(mode, fuseg) : pick_flat<5, 2>(mode, fuseg);
  else if (nvt == 8) fn = ct == 1 ? pick_flat<8, 1>(mode, fuseg) : pick_flat<8, 2>(mode, fuseg);
  else fn = pick_flat<16, 1>(mode, fuseg);
  // one round of resident workgroups (every wavefront walks its share of the chunks), within the partial buffers
  int64_t cap = flat_slots(fn, lds_bytes);
  if (fuseg || mode != 0) cap = std::min<int64_t>(cap, kColredBlocks);
  if (grid > cap) grid = cap;
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, wave_floats);
  return hipGetLastError();
}

}  // namespace ilargi
