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

// Plain product  P = D (M^T X)  for at most four operand columns, float4 rows of at most 64 float4: the role of the
// kernel above without gathers and epilogues, as a streaming kernel without LDS or workgroup barriers.
// L = 2^k >= ck / 4 lanes share a row (a wavefront load covers 64 / L whole rows), eight loads per lane are in
// flight, each lane keeps its operand values in registers.  The eight partial sums of a lane are reduced across
// the L lanes with a butterfly that halves the number of live values at each of its first three steps (a lane
// pair exchanges one half of the values each way), ten shuffles per operand column instead of forty-eight.
constexpr int kDotU = 8;

template <int CT>
__global__ __launch_bounds__(kBlock) void lmm_rowdot_kernel(LmmArgs a, int logL) {
  const int tid = threadIdx.x, lane = tid % kWave;
  const int L = 1 << logL;                                   // 8 <= L <= 64
  const int cg = lane & (L - 1);                             // float4 column group of this lane
  const int sub = lane >> logL;                              // row of the wavefront load
  const int rp = kWave >> logL;                              // rows per wavefront load
  const int nvec = a.ck / 4;
  float4 x[CT];
#pragma unroll
  for (int n = 0; n < CT; ++n) x[n] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  if (cg < nvec) {
    int t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = a.colmap[4 * cg + e];
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      if (n < a.ncols) {
        x[n].x = t[0] >= 0 ? a.X[(int64_t)t[0] * a.ldx + a.col0 + n] : 0.0f;
        x[n].y = t[1] >= 0 ? a.X[(int64_t)t[1] * a.ldx + a.col0 + n] : 0.0f;
        x[n].z = t[2] >= 0 ? a.X[(int64_t)t[2] * a.ldx + a.col0 + n] : 0.0f;
        x[n].w = t[3] >= 0 ? a.X[(int64_t)t[3] * a.ldx + a.col0 + n] : 0.0f;
      }
    }
  }
  const int64_t rows_per_step = (int64_t)rp * kDotU;
  const int64_t wave0 = ((int64_t)blockIdx.x * (kBlock / kWave) + tid / kWave) * rows_per_step;
  const int64_t stride = (int64_t)gridDim.x * (kBlock / kWave) * rows_per_step;
  // which of the eight rows of a step this lane reports after the reduction: bits of the lane number at the
  // three halving steps (offsets L/2, L/4, L/8)
  const int o1 = L >> 1, o2 = L >> 2, o3 = L >> 3;
  const bool h1 = (cg & o1) != 0, h2 = (cg & o2) != 0, h3 = (cg & o3) != 0;
  const int urow = (h1 ? 4 : 0) + (h2 ? 2 : 0) + (h3 ? 1 : 0);
  for (int64_t base = wave0; base < a.r_out; base += stride) {
    float4 v[kDotU];
#pragma unroll
    for (int u = 0; u < kDotU; ++u) {
      const int64_t i = base + (int64_t)u * rp + sub;
      v[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (cg < nvec && i < a.d_rows && i < a.r_out) v[u] = *reinterpret_cast<const float4*>(a.D + i * a.ck + 4 * cg);
    }
#pragma unroll
    for (int n = 0; n < CT; ++n) {
      float s8[kDotU];
#pragma unroll
      for (int u = 0; u < kDotU; ++u)
        s8[u] = fmaf(v[u].x, x[n].x, fmaf(v[u].y, x[n].y, fmaf(v[u].z, x[n].z, v[u].w * x[n].w)));
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
      if ((cg & (o3 - 1)) == 0 && n < a.ncols && i < a.r_out) a.out[i * a.ldo + a.col0 + n] = s1;
    }
  }
}

hipError_t launch_rowdot(const LmmArgs& a, hipStream_t st) {
  const int nvec = a.ck / 4;
  int logL = 3;
  while ((1 << logL) < nvec) ++logL;
  const int rp = kWave >> logL;
  const int64_t rows_per_block = (int64_t)rp * kDotU * (kBlock / kWave);
  int64_t grid = (a.r_out + rows_per_block - 1) / rows_per_block;
  if (grid > 4096) grid = 4096;
  const int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  if (ct == 1) lmm_rowdot_kernel<1><<<(int)grid, kBlock, 0, st>>>(a, logL);
  else if (ct == 2) lmm_rowdot_kernel<2><<<(int)grid, kBlock, 0, st>>>(a, logL);
  else lmm_rowdot_kernel<4><<<(int)grid, kBlock, 0, st>>>(a, logL);
  return hipGetLastError();
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
  if (mode == 0 && !fuseg && a.g.n == 0 && a.D != nullptr && vec == 4 && a.ck >= 4 && a.ck <= 256 && a.ncols <= kNarrowCT)
    return launch_rowdot(a, st);
  if (lmm_flat_supported(a, vec, fuseg)) return launch_lmm_flat(a, mode, fuseg, st, grid_out);
  if (lmm_flat_pair_supported(a, vec, fuseg)) return launch_lmm_flat_pair(a, mode, fuseg, st, grid_out);
  switch (vec) {
    case 4: return launch_ct<4>(a, mode, fuseg, grid, st);
    case 2: return launch_ct<2>(a, mode, fuseg, grid, st);
    default: return launch_ct<1>(a, mode, fuseg, grid, st);
  }
}

}  // namespace ilargi
