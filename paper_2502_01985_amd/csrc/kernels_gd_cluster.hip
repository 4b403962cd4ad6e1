// One gradient-descent pass (Alg. 1) of one model over a two-table star join  T = [S | I_R R]  whose entity table S
// is kept in JOIN ORDER (a copy Sp with the rows grouped by the row of R they join, made once for the plan):
//
//   z_t = Sp[t, :] w_S + R[key_t, :] w_R        (left multiply, Sec. 2.2)
//   e_t = residual of Alg. 1,  loss
//   G_S += Sp[t, :]^T e_t,   G_R += R[j, :]^T (sum of e_t over the rows t with key_t = j)      (transposed multiply)
//
// Rows that join the same row of R are neighbours in Sp, so both tables are plain streams: R is read ONCE per
// iteration (the factorized sequence reads it for the product and again for the column reduce), and the product
// R w_R, the residual and the segment sums I_R^T e never exist in memory.  The only gather left is the label of a
// row (4 bytes at its target row).
//
// A wavefront takes 64 consecutive rows of Sp as a flat stream of float4 (every lane busy whatever the row length;
// partial dot products meet in a wavefront-private LDS tile, then lane = row).  Their keys are an ascending run
// jlo .. jhi of rows of R; lane l holds the float4 number l of each of those rows (a row of up to 256 columns is
// one coalesced access), four rows at a time.  Pass 1 forms the four dot products with w_R (butterfly over the
// wavefront) and hands each to the lanes whose key matches; after the residuals, pass 2 adds up the residuals of
// each key over the wavefront (the wavefront's share of that segment sum; shares of a segment that spans several
// wavefronts add up in G_R because the product is linear) and multiplies the row, still in registers for the first
// eight rows of the run, by it.  Wavefronts are autonomous; sums are formed in a fixed order, so results repeat bit
// for bit.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

__device__ __forceinline__ void gc_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kGcWaves = kBlock / kWave;

// Value of `x` in the lane the data-parallel-primitive control word names (all lanes active).
template <int CTRL>
__device__ __forceinline__ float gc_dpp(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
constexpr int kGcSwap1 = 0xB1;               // quad_perm [1, 0, 3, 2]: lane l <- lane l ^ 1
constexpr int kGcSwap2 = 0x4E;               // quad_perm [2, 3, 0, 1]: lane l <- lane l ^ 2
constexpr int kGcHalfMirror = 0x141;         // lane l of a half row of 8  <-  lane 7 - l
constexpr int kGcRowMirror = 0x140;          // lane l of a row of 16  <-  lane 15 - l
constexpr int kGcSwizzleXor16 = 0x401F;      // ds_swizzle, bit mode: and 0x1F, or 0, xor 0x10

// Sums of four values over the 64 lanes, the same bits in every lane: at every level a lane and its partner add the
// same two numbers (a + b == b + a), and the two halves of the wavefront are added lower + upper by every lane.
__device__ __forceinline__ void gc_wave_sum4(float (&d)[4]) {
#pragma unroll
  for (int b = 0; b < 4; ++b) d[b] += gc_dpp<kGcSwap1>(d[b]);
#pragma unroll
  for (int b = 0; b < 4; ++b) d[b] += gc_dpp<kGcSwap2>(d[b]);
#pragma unroll
  for (int b = 0; b < 4; ++b) d[b] += gc_dpp<kGcHalfMirror>(d[b]);      // the other quad of the half row (all its lanes agree)
#pragma unroll
  for (int b = 0; b < 4; ++b) d[b] += gc_dpp<kGcRowMirror>(d[b]);       // the other half of the row
#pragma unroll
  for (int b = 0; b < 4; ++b)
    d[b] += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, d[b]), kGcSwizzleXor16));
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, d[b]), 0));
    const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, d[b]), 32));
    d[b] = lo + hi;
  }
}

// NVT = cs / 4, the float4s of a row of S.  MODE 1 linear, 2 logistic.  wave_floats: LDS floats of one wavefront.
template <int NVT, int MODE>
__global__ __launch_bounds__(kBlock) void gd_cluster_kernel(ClusterArgs a, int wave_floats) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // uniform: chunk numbers and key runs live in scalar registers
  constexpr int nvec = NVT;
  constexpr int ldp = nvec | 1;                                    // odd row stride of the partial-dot tile
  float4* Xs4 = reinterpret_cast<float4*>(lds);                // [NVT] weights of the columns of S
  float* wbase = lds + 4 * NVT + (size_t)wave * wave_floats;
  float* Pd = wbase;                                           // [64 * ldp] partial dot products
  float* Es = Pd + kWave * ldp;                                // [64] residuals by row
  int row_u[NVT], part_u[NVT];
#pragma unroll
  for (int u = 0; u < NVT; ++u) {
    const int e = u * kWave + lane;
    row_u[u] = u < nvec ? e / nvec : 0;
    part_u[u] = u < nvec ? e - row_u[u] * nvec : 0;
  }
  const int nvr = a.cr / 4;
  const bool rlive = lane < nvr;
  const int jmax = (int)a.r_R - 1;
  float4 wr = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

  float loss_local = 0.0f;
  float4 gacc[NVT];
#pragma unroll
  for (int u = 0; u < NVT; ++u) gacc[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  float4 gR = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

  const int64_t r_T = a.r_T;
  const int64_t nchunks = (r_T + kWave - 1) / kWave;
  const int64_t cstride = (int64_t)gridDim.x * kGcWaves;
  int64_t chunk = (int64_t)blockIdx.x * kGcWaves + wave;
  // The loop is free of branches around its loads (addresses are clamped into the buffers, values that must not
  // count are zeroed by a select), and everything a chunk consumes -- its rows of S, its keys, target rows and
  // labels, the first eight rows of its run of R -- is requested in one group a chunk earlier, right after the
  // previous group has arrived: a wavefront then computes a whole chunk without waiting for memory.  The run of R
  // needs the keys, so the keys are requested two chunks ahead.
  const int64_t last4 = r_T * nvec - 1;                        // last float4 of Sp
  auto load_chunk = [&](int64_t ch, float4 (&dst)[NVT]) {
    const int64_t f0 = ch * kWave * nvec + lane;
    const float4* b4 = reinterpret_cast<const float4*>(a.Sp);
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      const int64_t f = f0 + u * kWave;
      const float4 x = b4[min(f, last4)];
      const bool ok = u < nvec && f <= last4;
      dst[u] = make_float4(ok ? x.x : 0.0f, ok ? x.y : 0.0f, ok ? x.z : 0.0f, ok ? x.w : 0.0f);
    }
  };
  // labels: kept in join order with the copy of S (then a row's label sits at its own index and the target rows are
  // not needed: the second index stream rereads the keys, which hit), else gathered from the target rows
  const float* ylab = a.yp != nullptr ? a.yp : a.y;
  const int32_t* pidx = a.yp != nullptr ? a.keys : a.perm;
  auto load_keys = [&](int64_t ch, int& k, int& p) {
    const int64_t i = ch * kWave + lane;
    const int64_t ic = min(i, r_T - 1);
    const int kk = a.keys[ic], pp = pidx[ic];
    k = i < r_T ? kk : -1;
    p = i < r_T ? (a.yp != nullptr ? (int)ic : pp) : 0;
  };
  // the run of rows of R a chunk joins (keys ascend; clamped to the table whatever the key buffer holds); jhi < jlo
  // for a chunk beyond the table
  auto run_of = [&](int64_t ch, int k, int& jlo, int& jhi) {
    const int64_t left = r_T - ch * kWave;
    const int nlive = (int)min((int64_t)kWave, max(left, (int64_t)1));
    const int lo = min(max(__builtin_amdgcn_readlane(k, 0), 0), jmax);
    const int hi = min(max(__builtin_amdgcn_readlane(k, nlive - 1), lo), jmax);
    jlo = lo;
    jhi = left > 0 ? hi : lo - 1;
  };
  // four rows j0 .. j0 + 3 of R (zero beyond jhi and beyond the table's columns)
  const float4* R4 = reinterpret_cast<const float4*>(a.R) + min(lane, nvr - 1);
  auto load_rows = [&](int j0, int jhi, float4 (&r)[4]) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const float4 x = R4[(int64_t)min(j0 + b, max(jhi, 0)) * nvr];        // (beyond the run: its last row again, a cache hit)
      const bool ok = rlive && j0 + b <= jhi;
      r[b] = make_float4(ok ? x.x : 0.0f, ok ? x.y : 0.0f, ok ? x.z : 0.0f, ok ? x.w : 0.0f);
    }
  };
  // pass 1: their products with w_R, handed to the lanes whose key matches
  auto dots = [&](const float4 (&r)[4], int j0, int kj, float& pl) {
    float d[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) d[b] = fmaf(r[b].x, wr.x, fmaf(r[b].y, wr.y, fmaf(r[b].z, wr.z, r[b].w * wr.w)));
    gc_wave_sum4(d);
#pragma unroll
    for (int b = 0; b < 4; ++b) pl += kj == j0 + b ? d[b] : 0.0f;
  };
  // pass 2: the wavefront's residuals per key, times the row
  auto axpy = [&](const float4 (&r)[4], int j0, int kj, float e) {
    float z[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) z[b] = kj == j0 + b ? e : 0.0f;
    gc_wave_sum4(z);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      gR.x = fmaf(r[b].x, z[b], gR.x);
      gR.y = fmaf(r[b].y, z[b], gR.y);
      gR.z = fmaf(r[b].z, z[b], gR.z);
      gR.w = fmaf(r[b].w, z[b], gR.w);
    }
  };

  // the first chunk's group, and the keys of the second
  float4 v[NVT], vn[NVT], rk0[4], rk1[4], rn0[4], rn1[4];
  int kn, pn, kn2, pn2, jlo_n, jhi_n;
  load_keys(chunk, kn, pn);
  load_keys(chunk + cstride, kn2, pn2);
  load_chunk(chunk, vn);
  run_of(chunk, kn, jlo_n, jhi_n);
  load_rows(jlo_n, jhi_n, rn0);
  load_rows(jlo_n + 4, jhi_n, rn1);
  float yn = ylab[pn];
  // the weights are looked up while the first group travels
  // this lane's four columns of R and their weights
  if (rlive) {
    float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int t = a.r_colmap[4 * lane + c];
      if (t >= 0) w[c] = a.W[(int64_t)t * a.ldw + a.col];
    }
    wr = make_float4(w[0], w[1], w[2], w[3]);
  }
  if (tid < nvec) {
    float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int t = a.s_colmap[4 * tid + c];
      if (t >= 0) w[c] = a.W[(int64_t)t * a.ldw + a.col];
    }
    Xs4[tid] = make_float4(w[0], w[1], w[2], w[3]);
  }
  __syncthreads();

  for (; chunk < nchunks; chunk += cstride) {
    const int64_t i = chunk * kWave + lane;
    const bool rowlive = i < r_T;
    // the group requested a chunk ago
#pragma unroll
    for (int u = 0; u < NVT; ++u) v[u] = vn[u];
#pragma unroll
    for (int b = 0; b < 4; ++b) { rk0[b] = rn0[b]; rk1[b] = rn1[b]; }
    const int kj = kn;
    const float yi = yn;
    const int jlo = jlo_n, jhi = jhi_n;
    // the next chunk's group; the keys of the chunk after it
    kn = kn2; pn = pn2;
    load_chunk(chunk + cstride, vn);
    run_of(chunk + cstride, kn, jlo_n, jhi_n);
    load_rows(jlo_n, jhi_n, rn0);
    load_rows(jlo_n + 4, jhi_n, rn1);
    yn = ylab[pn];
    load_keys(chunk + 2 * cstride, kn2, pn2);
    // partial dot products of the rows of S into the tile
    gc_wave_sync();                                            // the previous chunk's tile is consumed
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      if (u < nvec) {
        const float4 x = Xs4[part_u[u]];
        Pd[row_u[u] * ldp + part_u[u]] = fmaf(v[u].x, x.x, fmaf(v[u].y, x.y, fmaf(v[u].z, x.z, v[u].w * x.w)));
      }
    }
    gc_wave_sync();
    float pl = 0.0f;
    dots(rk0, jlo, kj, pl);
    dots(rk1, jlo + 4, kj, pl);
    for (int j0 = jlo + 8; j0 <= jhi; j0 += 4) {               // (runs of more than eight rows: fan-out below eight)
      float4 r[4];
      load_rows(j0, jhi, r);
      dots(r, j0, kj, pl);
    }
    // lane = row: sum of the row's partials, residual, loss
    float z = 0.0f;
    {
      const float* pr = Pd + lane * ldp;
#pragma unroll
      for (int p = 0; p < NVT; ++p) z += p < nvec ? pr[p] : 0.0f;
    }
    z += pl;
    float r_e = 0.0f;
    if constexpr (MODE == 1) {
      r_e = rowlive ? z - yi : 0.0f;
      loss_local = fmaf(r_e, r_e, loss_local);
    } else {
      // one exponential serves the sigmoid and the softplus: e = exp(-|z|)
      const float e = __expf(-fabsf(z));
      const float inv = __frcp_rn(1.0f + e);
      r_e = rowlive ? (z >= 0.0f ? inv : e * inv) - yi : 0.0f;
      loss_local += rowlive ? fmaxf(z, 0.0f) + log1pf(e) - yi * z : 0.0f;
    }
    Es[lane] = r_e;
    gc_wave_sync();
    // S^T e: every lane multiplies the float4s it still holds by the residual of their row
#pragma unroll
    for (int u = 0; u < NVT; ++u) {
      if (u < nvec) {
        const float er = Es[row_u[u]];
        gacc[u].x = fmaf(v[u].x, er, gacc[u].x);
        gacc[u].y = fmaf(v[u].y, er, gacc[u].y);
        gacc[u].z = fmaf(v[u].z, er, gacc[u].z);
        gacc[u].w = fmaf(v[u].w, er, gacc[u].w);
      }
    }
    axpy(rk0, jlo, kj, r_e);
    axpy(rk1, jlo + 4, kj, r_e);
    for (int j0 = jlo + 8; j0 <= jhi; j0 += 4) {
      float4 r[4];
      load_rows(j0, jhi, r);
      axpy(r, j0, kj, r_e);
    }
  }

  __syncthreads();                                             // every wavefront is done with its tiles
  float* blk = lds + 4 * NVT;                                  // the wavefronts' LDS, free for the block's sums
  {
    // loss of this workgroup: butterfly inside each wavefront, then the wavefronts in order
    float s = loss_local;
    for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
    if (lane == 0) blk[wave] = s;
    __syncthreads();
    if (tid == 0) {
      float t = 0.0f;
      for (int w = 0; w < kGcWaves; ++w) t += blk[w];
      reinterpret_cast<float4*>(a.loss_partial)[blockIdx.x] = make_float4(t, 0.0f, 0.0f, 0.0f);
    }
    __syncthreads();
  }
  {
    // column 4 part + c of S: every (load u, lane l) with (64 u + l) % nvec == part contributes; they are added
    // in the order u, l for each wavefront, then the wavefronts in order
    float* gw = wbase;                                         // [NVT][64] float4 of this wavefront
#pragma unroll
    for (int u = 0; u < NVT; ++u)
      if (u < nvec) reinterpret_cast<float4*>(gw)[u * kWave + lane] = gacc[u];
    gc_wave_sync();
    float mine = 0.0f;
    if (lane < a.cs) {
      const int part = lane / 4, c = lane - part * 4;
      float m0 = 0.0f, m1 = 0.0f, m2 = 0.0f, m3 = 0.0f;
      for (int u = 0; u < nvec; ++u) {
        int l0 = (part - (u * kWave) % nvec) % nvec;
        if (l0 < 0) l0 += nvec;
        const float* col = gw + (size_t)(u * kWave) * 4 + c;
        int l = l0;
        for (; l + 3 * nvec < kWave; l += 4 * nvec) {
          m0 += col[(size_t)l * 4];
          m1 += col[(size_t)(l + nvec) * 4];
          m2 += col[(size_t)(l + 2 * nvec) * 4];
          m3 += col[(size_t)(l + 3 * nvec) * 4];
        }
        for (; l < kWave; l += nvec) m0 += col[(size_t)l * 4];
      }
      mine = (m0 + m1) + (m2 + m3);
    }
    __syncthreads();                                           // all wavefronts have read their own tiles
    float* gb = blk;                                           // [waves][cs]
    if (lane < a.cs) gb[wave * a.cs + lane] = mine;
    __syncthreads();
    if (tid < a.cs) {
      float s = 0.0f;
      for (int w = 0; w < kGcWaves; ++w) s += gb[w * a.cs + tid];
      reinterpret_cast<float4*>(a.grad_partial_s)[(int64_t)blockIdx.x * a.cs + tid] = make_float4(s, 0.0f, 0.0f, 0.0f);
    }
    __syncthreads();
  }
  {
    // columns 4 l .. 4 l + 3 of R: the wavefronts in order
    float4* gr = reinterpret_cast<float4*>(blk);               // [waves][64]
    gr[wave * kWave + lane] = gR;
    __syncthreads();
    if (tid < nvr) {
      float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      for (int w = 0; w < kGcWaves; ++w) {
        const float4 x = gr[w * kWave + tid];
        t.x += x.x; t.y += x.y; t.z += x.z; t.w += x.w;
      }
      float4* out = reinterpret_cast<float4*>(a.grad_partial_r) + (int64_t)blockIdx.x * a.cr + 4 * tid;
      out[0] = make_float4(t.x, 0.0f, 0.0f, 0.0f);
      out[1] = make_float4(t.y, 0.0f, 0.0f, 0.0f);
      out[2] = make_float4(t.z, 0.0f, 0.0f, 0.0f);
      out[3] = make_float4(t.w, 0.0f, 0.0f, 0.0f);
    }
  }
}

// Sp[p, :] = S[perm[p], :] as float4, keys[p] = idx[perm[p]], yp[p] = y[perm[p]] (when labels are given).
__global__ __launch_bounds__(kBlock) void cluster_rows_kernel(const float4* __restrict__ S4, int nvec, const int32_t* __restrict__ perm,
                                                             const int32_t* __restrict__ idx, int64_t r_T,
                                                             float4* __restrict__ Sp4, int32_t* __restrict__ keys,
                                                             const float* __restrict__ y, float* __restrict__ yp) {
  const int64_t total = r_T * nvec;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < total; e += (int64_t)gridDim.x * kBlock) {
    const int64_t p = e / nvec;
    const int g = (int)(e - p * nvec);
    const int64_t t = perm[p];
    Sp4[e] = S4[t * nvec + g];
    if (g == 0) {
      keys[p] = idx[t];
      if (y != nullptr) yp[p] = y[t];
    }
  }
}

typedef void (*GcFn)(ClusterArgs, int);

template <int MODE>
GcFn gc_pick(int nvec) {
  switch (nvec) {
    case 1: return gd_cluster_kernel<1, MODE>;
    case 2: return gd_cluster_kernel<2, MODE>;
    case 3: return gd_cluster_kernel<3, MODE>;
    case 4: return gd_cluster_kernel<4, MODE>;
    case 5: return gd_cluster_kernel<5, MODE>;
    case 6: return gd_cluster_kernel<6, MODE>;
    case 7: return gd_cluster_kernel<7, MODE>;
    default: return gd_cluster_kernel<8, MODE>;
  }
}

int gc_slots(GcFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;
  std::lock_guard<std::mutex> lock(cache_mutex);
  static GcFn seen_fn[16];
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

// Entity table of 4 .. 32 columns, dimension table of 4 .. 256 columns, both in whole float4s.
bool gd_cluster_supported(int cs, int cr) {
  return cs >= 4 && cs % 4 == 0 && cs <= 32 && cr >= 4 && cr % 4 == 0 && cr <= 4 * kWave;
}

hipError_t launch_cluster_rows(const float* S, int cs, const int32_t* perm, const int32_t* idx, int64_t r_T, float* Sp,
                               int32_t* keys, const float* y, float* yp, hipStream_t st) {
  if (S == nullptr || perm == nullptr || idx == nullptr || Sp == nullptr || keys == nullptr || cs < 4 || cs % 4 != 0 ||
      (y != nullptr && yp == nullptr) ||
      reinterpret_cast<uintptr_t>(S) % 16 != 0 || reinterpret_cast<uintptr_t>(Sp) % 16 != 0)
    return hipErrorInvalidValue;
  if (r_T <= 0) return hipSuccess;
  const int nvec = cs / 4;
  const int64_t total = r_T * nvec;
  const int grid = (int)std::min<int64_t>((total + kBlock - 1) / kBlock, 8192);
  hipLaunchKernelGGL(cluster_rows_kernel, dim3((unsigned)grid), dim3(kBlock), 0, st, reinterpret_cast<const float4*>(S), nvec, perm,
                     idx, r_T, reinterpret_cast<float4*>(Sp), keys, y, yp);
  return hipGetLastError();
}

hipError_t launch_gd_cluster(const ClusterArgs& a, int mode, int max_grid, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!gd_cluster_supported(a.cs, a.cr) || (mode != 1 && mode != 2) || max_grid < 1 || a.r_T < 1 || a.r_R < 1) return hipErrorInvalidValue;
  if (a.Sp == nullptr || a.keys == nullptr || a.perm == nullptr || a.R == nullptr || (a.y == nullptr && a.yp == nullptr) || a.W == nullptr)
    return hipErrorInvalidValue;
  if (reinterpret_cast<uintptr_t>(a.Sp) % 16 != 0 || reinterpret_cast<uintptr_t>(a.R) % 16 != 0) return hipErrorInvalidValue;
  const int nvec = a.cs / 4;
  const int nvt = nvec;
  const int ldp = nvec | 1;
  int wave_floats = std::max(kWave * ldp + kWave, nvt * kWave * 4);
  wave_floats = (wave_floats + 3) / 4 * 4;
  const size_t lds_bytes = ((size_t)4 * nvt + (size_t)kGcWaves * wave_floats) * sizeof(float);
  GcFn fn = mode == 1 ? gc_pick<1>(nvec) : gc_pick<2>(nvec);
  const int64_t nchunks = (a.r_T + kWave - 1) / kWave;
  int64_t grid = (nchunks + kGcWaves - 1) / kGcWaves;
  grid = std::min<int64_t>(grid, gc_slots(fn, lds_bytes));         // one round of resident workgroups
  grid = std::min<int64_t>(grid, max_grid);                        // ... within the partial buffers
  if (grid_out) *grid_out = (int)grid;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(kBlock), lds_bytes, st, a, wave_floats);
  return hipGetLastError();
}

}  // namespace ilargi
