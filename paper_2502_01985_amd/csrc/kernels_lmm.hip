// Left multiply  T X = sum_k I_k (D_k (M_k^T X))  (paper, Sec. 2.2) for narrow operands (<= 4 columns per pass).
//
// One kernel serves both steps of the rewrite:
//   * the per-source product  P_k = D_k X_k  with  X_k = M_k^T X  (row select through col_map, staged in LDS);
//   * the assembly  out[i,:] = D_S[i,:] X_S + sum_k P_k[row_idx_k[i], :]  where the product of the source that
//     is the identity on the target rows is fused into the pass that gathers the other sources' rows.
// In the gradient-descent modes the assembled value becomes the residual of Alg. 1 before it is stored, and the
// identity source's share of the gradient,  D_S^T e, is accumulated from the table values still in registers.
//
// A workgroup handles up to 256 consecutive target rows per step, in two thread mappings that meet in LDS:
//   dot mapping     a row of D is read by L = 2^logL adjacent lanes (float4 each), so a wavefront load is one
//                   contiguous span of 64/L rows; the lanes of a row combine with an xor butterfly;
//   row mapping     thread t owns row t of the step: it loads row_idx (coalesced), gathers the P_k rows, adds
//                   the dot product from LDS, applies the epilogue and stores (coalesced).
// The row indices of the next step are prefetched while the current step computes.
#include <cstring>
#include <type_traits>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

template <int VEC> __device__ __forceinline__ void load_vec(const float* p, float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else if constexpr (VEC == 2) {
    float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  } else {
    v[0] = *p;
  }
}

__device__ __forceinline__ float sigmoidf_stable(float z) {
  if (z >= 0.0f) return 1.0f / (1.0f + __expf(-z));
  float e = __expf(z);
  return e / (1.0f + e);
}

__device__ __forceinline__ float softplusf_stable(float z) {
  return fmaxf(z, 0.0f) + log1pf(__expf(-fabsf(z)));
}

constexpr int kUnroll = 8;     // rows per lane group and step
constexpr int kPrefetch = 3;   // gathered sources whose row indices are prefetched one step ahead

__device__ __forceinline__ int64_t gather_row(const GatherArgs& g, int s, int64_t i) {
  if (g.idx[s] != nullptr) return g.idx[s][i];
  return i < g.rows[s] ? i : -1;
}

// MODE 0: store the product.  MODE 1: linear residual z - y.  MODE 2: logistic residual sigmoid(z) - y.
// FUSEG: also accumulate this workgroup's partial of D^T e (needs every row to fit one load per lane).
template <int VEC, int CT, int MODE, bool FUSEG>
__global__ __launch_bounds__(kBlock) void lmm_rows_kernel(LmmArgs a) {
  __shared__ float Xs[kMaxLdsFloats];           // [ck][CT]
  __shared__ float zbuf[2][kBlock * CT];        // dot products (then residuals) of the step's rows, ping-pong
  const int tid = threadIdx.x;
  for (int e = tid; e < a.ck * CT; e += kBlock) {
    int j = e / CT, n = e - j * CT;
    int t = a.colmap[j];
    Xs[e] = (t >= 0 && n < a.ncols) ? a.X[(int64_t)t * a.ldx + a.col0 + n] : 0.0f;
  }
  __syncthreads();

  const int L = 1 << a.logL;
  const int lig = tid & (L - 1);
  const int gid = tid >> a.logL;
  const int gpb = kBlock >> a.logL;                         // row groups per workgroup
  const int U = min(kUnroll, kBlock / gpb);                 // rows per group and step
  const int rpi = gpb * U;                                  // rows per step (<= 256)
  const int nvec = a.ck / VEC;
  const int64_t stride = (int64_t)gridDim.x * rpi;
  float loss_local[CT];
  float gacc[VEC][CT];
#pragma unroll
  for (int n = 0; n < CT; ++n) loss_local[n] = 0.0f;
#pragma unroll
  for (int e = 0; e < VEC; ++e)
#pragma unroll
    for (int n = 0; n < CT; ++n) gacc[e][n] = 0.0f;

  int64_t jn[kPrefetch];
  {
    int64_t i = (int64_t)blockIdx.x * rpi + tid;
#pragma unroll
    for (int s = 0; s < kPrefetch; ++s) jn[s] = (s < a.g.n && tid < rpi && i < a.r_out) ? gather_row(a.g, s, i) : -1;
  }

  int it = 0;
  for (int64_t base = (int64_t)blockIdx.x * rpi; base < a.r_out; base += stride, ++it) {
    float* zb = zbuf[it & 1];
    // ---- dot mapping: issue the table loads first
    float v[kUnroll][VEC];
    float acc[kUnroll][CT];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
      for (int n = 0; n < CT; ++n) acc[u][n] = 0.0f;
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[u][e] = 0.0f;
    }
    const bool single = nvec <= L;
    if (a.D != nullptr && single) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        int64_t i = base + (int64_t)u * gpb + gid;
        if (u < U && i < a.d_rows && lig < nvec) load_vec<VEC>(a.D + i * a.ck + lig * VEC, v[u]);
      }
    }
    // ---- row mapping: gathers of this step (indices were prefetched), then the next step's indices
    const int64_t irow = base + tid;
    const bool rowlive = tid < rpi && irow < a.r_out;
    float gsum[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) gsum[n] = 0.0f;
    if (rowlive) {
#pragma unroll
      for (int s = 0; s < kPrefetch; ++s) {
        if (s < a.g.n && jn[s] >= 0) {
          const float* p = a.g.P[s] + jn[s] * a.g.ldp + a.col0;
#pragma unroll
          for (int n = 0; n < CT; ++n)
            if (n < a.ncols) gsum[n] += p[n];
        }
      }
      for (int s = kPrefetch; s < a.g.n; ++s) {
        int64_t j = gather_row(a.g, s, irow);
        if (j >= 0) {
          const float* p = a.g.P[s] + j * a.g.ldp + a.col0;
#pragma unroll
          for (int n = 0; n < CT; ++n)
            if (n < a.ncols) gsum[n] += p[n];
        }
      }
    }
    float yi = 0.0f;
    if constexpr (MODE != 0) {
      if (rowlive) yi = a.y[irow];
    }
    {
      int64_t inext = irow + stride;
#pragma unroll
      for (int s = 0; s < kPrefetch; ++s)
        jn[s] = (s < a.g.n && tid < rpi && inext < a.r_out) ? gather_row(a.g, s, inext) : -1;
    }
    // ---- dot products
    if (a.D != nullptr) {
      if (single) {
        if (lig < nvec) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            float xv[CT];
#pragma unroll
            for (int n = 0; n < CT; ++n) xv[n] = Xs[(lig * VEC + e) * CT + n];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
              for (int n = 0; n < CT; ++n) acc[u][n] = fmaf(v[u][e], xv[n], acc[u][n]);
          }
        }
      } else {
        for (int t = lig; t < nvec; t += L) {
#pragma unroll
          for (int u = 0; u < kUnroll; ++u) {
            int64_t i = base + (int64_t)u * gpb + gid;
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[u][e] = 0.0f;
            if (u < U && i < a.d_rows) load_vec<VEC>(a.D + i * a.ck + t * VEC, v[u]);
          }
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            float xv[CT];
#pragma unroll
            for (int n = 0; n < CT; ++n) xv[n] = Xs[(t * VEC + e) * CT + n];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
#pragma unroll
              for (int n = 0; n < CT; ++n) acc[u][n] = fmaf(v[u][e], xv[n], acc[u][n]);
          }
        }
      }
      for (int m = L >> 1; m >= 1; m >>= 1) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
          for (int n = 0; n < CT; ++n) acc[u][n] += __shfl_xor(acc[u][n], m);
      }
    }
    if (lig == 0) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (u < U) {
#pragma unroll
          for (int n = 0; n < CT; ++n) zb[(u * gpb + gid) * CT + n] = acc[u][n];
        }
    }
    __syncthreads();
    // ---- row mapping: epilogue and store
    if (rowlive) {
#pragma unroll
      for (int n = 0; n < CT; ++n) {
        if (n < a.ncols) {
          float z = zb[tid * CT + n] + gsum[n];
          float r = z;
          if constexpr (MODE == 1) {
            r = z - yi;
            loss_local[n] = fmaf(r, r, loss_local[n]);
          } else if constexpr (MODE == 2) {
            r = sigmoidf_stable(z) - yi;
            loss_local[n] += softplusf_stable(z) - yi * z;
          }
          float* op = a.out + irow * a.ldo + a.col0 + n;
          if (a.nt_out) __builtin_nontemporal_store(r, op);
          else *op = r;
          if constexpr (FUSEG) zb[tid * CT + n] = r;
        } else if constexpr (FUSEG) {
          zb[tid * CT + n] = 0.0f;
        }
      }
    } else if constexpr (FUSEG) {
      if (tid < rpi) {
#pragma unroll
        for (int n = 0; n < CT; ++n) zb[tid * CT + n] = 0.0f;
      }
    }
    if constexpr (FUSEG) {
      __syncthreads();
      // gradient share of the fused source: table values are still in registers (single-load rows only)
      if (lig < nvec) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
          if (u < U) {
#pragma unroll
            for (int n = 0; n < CT; ++n) {
              float r = zb[(u * gpb + gid) * CT + n];
#pragma unroll
              for (int e = 0; e < VEC; ++e) gacc[e][n] = fmaf(v[u][e], r, gacc[e][n]);
            }
          }
      }
    }
  }

  if constexpr (MODE != 0) {
    // loss of this workgroup: butterfly inside each wavefront, then the four wavefronts in order
    __shared__ float lsum[kBlock / kWave][CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float s = loss_local[n];
      for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
      if ((tid % kWave) == 0) lsum[tid / kWave][n] = s;
    }
    __syncthreads();
    if (tid < CT) {
      float s = 0.0f;
      for (int w = 0; w < kBlock / kWave; ++w) s += lsum[w][tid];
      a.loss_partial[(int64_t)blockIdx.x * kNarrowCT + tid] = s;
    }
  }
  if constexpr (FUSEG) {
    // column j of the table, operand column n: add the lane groups of the workgroup in a fixed order
    __shared__ float red[VEC * CT][kBlock];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < VEC; ++e)
#pragma unroll
      for (int n = 0; n < CT; ++n) red[e * CT + n][tid] = gacc[e][n];
    __syncthreads();
    for (int o = tid; o < a.ck * CT; o += kBlock) {
      int j = o / CT, n = o - j * CT;
      int jl = j / VEC, e = j - jl * VEC;
      float s = 0.0f;
      for (int g = 0; g < gpb; ++g) s += red[e * CT + n][g * L + jl];
      a.grad_partial[((int64_t)blockIdx.x * a.ck + j) * kNarrowCT + n] = s;
    }
  }
}

template <int VEC, int CT>
hipError_t launch_mode(const LmmArgs& a, int mode, bool fuseg, int grid, size_t lds, hipStream_t st) {
  if (fuseg) {
    if (mode == 1) lmm_rows_kernel<VEC, CT, 1, true><<<grid, kBlock, lds, st>>>(a);
    else lmm_rows_kernel<VEC, CT, 2, true><<<grid, kBlock, lds, st>>>(a);
  } else {
    switch (mode) {
      case 0: lmm_rows_kernel<VEC, CT, 0, false><<<grid, kBlock, lds, st>>>(a); break;
      case 1: lmm_rows_kernel<VEC, CT, 1, false><<<grid, kBlock, lds, st>>>(a); break;
      default: lmm_rows_kernel<VEC, CT, 2, false><<<grid, kBlock, lds, st>>>(a); break;
    }
  }
  return hipGetLastError();
}

// Plain product  P = D (M^T X)  for at most four operand columns, rows of at most 64 aligned vectors of VW = 4 or 2
// floats: the role of the kernel above without gathers and epilogues, as a streaming kernel without LDS or
// workgroup barriers.
// L = 2^k >= ck / VW lanes share a row (a wavefront load covers 64 / L whole rows), eight loads per lane are in
// flight, each lane keeps its operand values in registers.  The eight partial sums of a lane are reduced across
// the L lanes with a butterfly that halves the number of live values at each of its first three steps (a lane
// pair exchanges one half of the values each way), ten shuffles per operand column instead of forty-eight.
// Several sources may share a launch: workgroup `bid` of the `nblocks` that serve this source.
constexpr int kDotU = 8;

template <int CT, int VW>
__device__ __forceinline__ void lmm_rowdot_body(const RowdotArgs& a, int bid, int nblocks) {
  typedef typename std::conditional<VW == 4, float4, float2>::type Vec;
  const int logL = a.logL;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int L = 1 << logL;                                   // 8 <= L <= 64
  const int cg = lane & (L - 1);                             // vector column group of this lane
  const int sub = lane >> logL;                              // row of the wavefront load
  const int rp = kWave >> logL;                              // rows per wavefront load
  const int nvec = a.ck / VW;
  float x[CT][VW];
#pragma unroll
  for (int n = 0; n < CT; ++n)
#pragma unroll
    for (int e = 0; e < VW; ++e) x[n][e] = 0.0f;
  if (cg < nvec) {
    int t[VW];
#pragma unroll
    for (int e = 0; e < VW; ++e) t[e] = a.colmap[VW * cg + e];
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      if (n < a.ncols) {
#pragma unroll
        for (int e = 0; e < VW; ++e) x[n][e] = t[e] >= 0 ? a.X[(int64_t)t[e] * a.ldx + a.col0 + n] : 0.0f;
      }
    }
  }
  const int64_t rows_per_step = (int64_t)rp * kDotU;
  const int64_t wave0 = ((int64_t)bid * (kBlock / kWave) + tid / kWave) * rows_per_step;
  const int64_t stride = (int64_t)nblocks * (kBlock / kWave) * rows_per_step;
  // which of the eight rows of a step this lane reports after the reduction: bits of the lane number at the
  // three halving steps (offsets L/2, L/4, L/8)
  const int o1 = L >> 1, o2 = L >> 2, o3 = L >> 3;
  const bool h1 = (cg & o1) != 0, h2 = (cg & o2) != 0, h3 = (cg & o3) != 0;
  const int urow = (h1 ? 4 : 0) + (h2 ? 2 : 0) + (h3 ? 1 : 0);
  for (int64_t base = wave0; base < a.rows; base += stride) {
    float v[kDotU][VW];
#pragma unroll
    for (int u = 0; u < kDotU; ++u) {
      const int64_t i = base + (int64_t)u * rp + sub;
#pragma unroll
      for (int e = 0; e < VW; ++e) v[u][e] = 0.0f;
      if (cg < nvec && i < a.rows) {
        const Vec t = *reinterpret_cast<const Vec*>(a.D + i * a.ck + VW * cg);
        v[u][0] = t.x; v[u][1] = t.y;
        if constexpr (VW == 4) { v[u][2] = t.z; v[u][3] = t.w; }
      }
    }
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float s8[kDotU];
#pragma unroll
      for (int u = 0; u < kDotU; ++u) {
        if constexpr (VW == 4)
          s8[u] = fmaf(v[u][0], x[n][0], fmaf(v[u][1], x[n][1], fmaf(v[u][2], x[n][2], v[u][3] * x[n][3])));
        else
          s8[u] = fmaf(v[u][0], x[n][0], v[u][1] * x[n][1]);
      }
      // offset L/2: the lower lane of a pair keeps rows 0..3, the upper one rows 4..7
      float s4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float keep = h1 ? s8[4 + j] : s8[j];
        const float send = h1 ? s8[j] : s8[4 + j];
        s4[j] = keep + __shfl_xor(send, o1);
      }
      float s2[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float keep = h2 ? s4[2 + j] : s4[j];
        const float send = h2 ? s4[j] : s4[2 + j];
        s2[j] = keep + __shfl_xor(send, o2);
      }
      float s1;
      {
        const float keep = h3 ? s2[1] : s2[0];
        const float send = h3 ? s2[0] : s2[1];
        s1 = keep + __shfl_xor(send, o3);
      }
      for (int o = o3 >> 1; o >= 1; o >>= 1) s1 += __shfl_xor(s1, o);
      // lanes whose low bits (below L/8) are zero hold the sum of row `urow` of their wavefront-load row `sub`
      const int64_t i = base + (int64_t)urow * rp + sub;
      if ((cg & (o3 - 1)) == 0 && n < a.ncols && i < a.rows) a.out[i * a.ldo + a.col0 + n] = s1;
    }
  }
}

// Workgroups [first[q], first[q + 1]) serve source q.
template <int CT>
__global__ __launch_bounds__(kBlock) void lmm_rowdot_kernel(RowdotMulti m) {
  int q = 0;
  while (q + 1 < m.n && (int)blockIdx.x >= m.first[q + 1]) ++q;
  const int bid = (int)blockIdx.x - m.first[q], nblocks = m.first[q + 1] - m.first[q];
  if (m.a[q].vw == 4) lmm_rowdot_body<CT, 4>(m.a[q], bid, nblocks);
  else lmm_rowdot_body<CT, 2>(m.a[q], bid, nblocks);
}

template <int VEC>
hipError_t launch_ct(const LmmArgs& a, int mode, bool fuseg, int grid, hipStream_t st) {
  int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  size_t lds = 0;
  switch (ct) {
    case 1: return launch_mode<VEC, 1>(a, mode, fuseg, grid, lds, st);
    case 2: return launch_mode<VEC, 2>(a, mode, fuseg, grid, lds, st);
    default: return launch_mode<VEC, 4>(a, mode, fuseg, grid, lds, st);
  }
}

}  // namespace

// Dense table, at most four operand columns, rows of at most 64 aligned vectors of 4 (or, with vec == 2, 2) floats.
bool rowdot_supported(const LmmArgs& a, int vec) {
  if (a.D == nullptr || a.g.n != 0 || a.ncols < 1 || a.ncols > kNarrowCT || a.r_out <= 0) return false;
  if (vec == 4) return a.ck >= 4 && a.ck <= 256 && a.ck % 4 == 0 && reinterpret_cast<uintptr_t>(a.D) % 16 == 0;
  if (vec == 2) return a.ck >= 2 && a.ck <= 128 && a.ck % 2 == 0 && reinterpret_cast<uintptr_t>(a.D) % 8 == 0;
  return false;
}

// The products of n <= kRowdotMulti sources (same operand columns) in one launch; vec[q] = 4 or 2 (NULL: all 4).
hipError_t launch_rowdot_multi(const LmmArgs* a, const int* vec, int n, hipStream_t st) {
  if (n < 1 || n > kRowdotMulti) return hipErrorInvalidValue;
  RowdotMulti m;
  memset(&m, 0, sizeof(m));
  m.n = n;
  // at most `cap` workgroups in all, shared out by rows
  int64_t want[kRowdotMulti], total = 0;
  for (int q = 0; q < n; ++q) {
    const int vw = vec ? vec[q] : 4;
    if (!rowdot_supported(a[q], vw) || a[q].ncols != a[0].ncols) return hipErrorInvalidValue;
    const int nvec = a[q].ck / vw;
    int logL = 3;
    while ((1 << logL) < nvec) ++logL;
    const int rp = kWave >> logL;
    const int64_t rows_per_block = (int64_t)rp * kDotU * (kBlock / kWave);
    want[q] = (std::min(a[q].r_out, a[q].d_rows) + rows_per_block - 1) / rows_per_block;
    total += want[q];
    RowdotArgs& r = m.a[q];
    r.D = a[q].D; r.ck = a[q].ck; r.rows = std::min(a[q].r_out, a[q].d_rows); r.colmap = a[q].colmap;
    r.X = a[q].X; r.ldx = a[q].ldx; r.col0 = a[q].col0; r.ncols = a[q].ncols;
    r.out = a[q].out; r.ldo = a[q].ldo; r.logL = logL; r.vw = vw;
  }
  const int64_t cap = 4096;   // (fewer, longer-lived workgroups with the next step's rows requested ahead measured the same)
  for (int q = 0; q < n; ++q) {
    int64_t g = total > cap ? std::max<int64_t>(1, want[q] * cap / total) : want[q];
    m.first[q + 1] = m.first[q] + (int)std::max<int64_t>(g, 1);
  }
  const int ct = a[0].ncols <= 1 ? 1 : (a[0].ncols <= 2 ? 2 : 4);
  const unsigned grid = (unsigned)m.first[n];
  if (ct == 1) lmm_rowdot_kernel<1><<<grid, kBlock, 0, st>>>(m);
  else if (ct == 2) lmm_rowdot_kernel<2><<<grid, kBlock, 0, st>>>(m);
  else lmm_rowdot_kernel<4><<<grid, kBlock, 0, st>>>(m);
  return hipGetLastError();
}

int lmm_rows_per_step(int logL) {
  int gpb = kBlock >> logL;
  int u = kBlock / gpb < kUnroll ? kBlock / gpb : kUnroll;
  return gpb * u;
}

int lmm_grid(int64_t r_out, int logL, bool fuseg) {
  int64_t rpi = lmm_rows_per_step(logL);
  int64_t g = (r_out + rpi - 1) / rpi;
  // one step per workgroup whenever possible: late workgroups then fill the slots early ones free, which
  // balances better than a resident grid whose members do one or two steps each
  int64_t cap = fuseg ? kColredBlocks : 2048;
  if (g < 1) g = 1;
  if (g > cap) {
    int64_t per = (g + cap - 1) / cap;
    g = (g + per - 1) / per;
  }
  return (int)g;
}

// True when the fused gradient variant can serve a table with these columns.
bool lmm_can_fuse_gradient(int ck, int vec, int logL) { return ck > 0 && ck / vec <= (1 << logL); }

hipError_t launch_lmm_rows(const LmmArgs& a, int vec, int mode, hipStream_t st, int* grid_out) {
  const bool fuseg = a.grad_partial != nullptr && mode != 0;
  int grid = lmm_grid(a.r_out, a.logL, fuseg);
  if (grid_out) *grid_out = grid;
  if (a.r_out <= 0) return hipSuccess;
  if (mode == 0 && !fuseg && vec == 4 && rowdot_supported(a, 4)) return launch_rowdot_multi(&a, nullptr, 1, st);
  if (lmm_lane_supported(a, vec, mode, fuseg)) return launch_lmm_lane(a, vec, mode, st, grid_out);
  if (lmm_flat_supported(a, vec, fuseg)) return launch_lmm_flat(a, mode, fuseg, st, grid_out);
  if (lmm_flat_pair_supported(a, vec, fuseg)) return launch_lmm_flat_pair(a, mode, fuseg, st, grid_out);
  switch (vec) {
    case 4: return launch_ct<4>(a, mode, fuseg, grid, st);
    case 2: return launch_ct<2>(a, mode, fuseg, grid, st);
    default: return launch_ct<1>(a, mode, fuseg, grid, st);
  }
}

}  // namespace ilargi
