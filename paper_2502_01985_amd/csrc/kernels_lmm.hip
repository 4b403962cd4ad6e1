// Left multiply  T X = sum_k I_k (D_k (M_k^T X))  (paper, Sec. 2.2) for narrow operands.
//
// One kernel serves both steps of the rewrite:
//   * the per-source product  P_k = D_k X_k  with  X_k = M_k^T X  (row select through col_map, staged in LDS);
//   * the assembly  out[i,:] = D_S[i,:] X_S + sum_k P_k[row_idx_k[i], :]  where the product of the source that
//     is the identity on the target rows is fused into the pass that gathers the other sources' rows.
// In the gradient-descent modes the assembled value is turned into the residual of Alg. 1 before it is stored.
//
// Thread mapping: a row of D is read by L = 2^logL adjacent lanes, VEC floats per lane per step, so that a
// wavefront always loads one contiguous span of 64/L rows.  Lanes of a row combine with an xor butterfly.
#include "ilargi_internal.h"

namespace ilargi {

namespace {

template <int VEC> struct Vec;
template <> struct Vec<1> { using T = float; };
template <> struct Vec<2> { using T = float2; };
template <> struct Vec<4> { using T = float4; };

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

constexpr int kUnroll = 4;

// MODE 0: store the product.  MODE 1: linear residual z - y.  MODE 2: logistic residual sigmoid(z) - y.
template <int VEC, int CT, int MODE>
__global__ __launch_bounds__(kBlock) void lmm_rows_kernel(LmmArgs a) {
  extern __shared__ float Xs[];  // [ck][CT]
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
  const int gpb = kBlock >> a.logL;           // row groups per workgroup
  const int nvec = a.ck / VEC;
  const int64_t rows_per_iter = (int64_t)gpb * kUnroll;
  float loss_local[CT];
#pragma unroll
  for (int n = 0; n < CT; ++n) loss_local[n] = 0.0f;

  for (int64_t base = (int64_t)blockIdx.x * rows_per_iter; base < a.r_out;
       base += (int64_t)gridDim.x * rows_per_iter) {
    float acc[kUnroll][CT];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int n = 0; n < CT; ++n) acc[u][n] = 0.0f;

    if (a.D != nullptr) {
      if (nvec <= L) {
        // one load per lane and row: issue all of them before the arithmetic
        float v[kUnroll][VEC];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          int64_t i = base + (int64_t)u * gpb + gid;
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[u][e] = 0.0f;
          if (i < a.d_rows && lig < nvec) load_vec<VEC>(a.D + i * a.ck + lig * VEC, v[u]);
        }
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
          float v[kUnroll][VEC];
#pragma unroll
          for (int u = 0; u < kUnroll; ++u) {
            int64_t i = base + (int64_t)u * gpb + gid;
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[u][e] = 0.0f;
            if (i < a.d_rows) load_vec<VEC>(a.D + i * a.ck + t * VEC, v[u]);
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
    }

    // gathered rows of the other sources' products: lane s of the row group fetches source s
    if (a.g.n > 0) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        int64_t i = base + (int64_t)u * gpb + gid;
        if (i < a.r_out) {
          for (int s = lig; s < a.g.n; s += L) {
            int64_t j;
            if (a.g.idx[s] != nullptr) j = a.g.idx[s][i];
            else j = (i < a.g.rows[s]) ? i : -1;
            if (j >= 0) {
              const float* p = a.g.P[s] + j * a.g.ldp + a.col0;
#pragma unroll
              for (int n = 0; n < CT; ++n)
                if (n < a.ncols) acc[u][n] += p[n];
            }
          }
        }
      }
    }

    for (int m = L >> 1; m >= 1; m >>= 1) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
#pragma unroll
        for (int n = 0; n < CT; ++n) acc[u][n] += __shfl_xor(acc[u][n], m);
    }

    if (lig == 0) {
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        int64_t i = base + (int64_t)u * gpb + gid;
        if (i < a.r_out) {
          float yi = 0.0f;
          if constexpr (MODE != 0) yi = a.y[i];
#pragma unroll
          for (int n = 0; n < CT; ++n) {
            if (n < a.ncols) {
              float z = acc[u][n];
              float r = z;
              if constexpr (MODE == 1) {
                r = z - yi;
                loss_local[n] = fmaf(r, r, loss_local[n]);
              } else if constexpr (MODE == 2) {
                r = sigmoidf_stable(z) - yi;
                loss_local[n] += softplusf_stable(z) - yi * z;
              }
              a.out[i * a.ldo + a.col0 + n] = r;
            }
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
}

template <int VEC, int CT>
hipError_t launch_mode(const LmmArgs& a, int mode, int grid, size_t lds, hipStream_t st) {
  switch (mode) {
    case 0: lmm_rows_kernel<VEC, CT, 0><<<grid, kBlock, lds, st>>>(a); break;
    case 1: lmm_rows_kernel<VEC, CT, 1><<<grid, kBlock, lds, st>>>(a); break;
    default: lmm_rows_kernel<VEC, CT, 2><<<grid, kBlock, lds, st>>>(a); break;
  }
  return hipGetLastError();
}

template <int VEC>
hipError_t launch_ct(const LmmArgs& a, int mode, int grid, hipStream_t st) {
  int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
  size_t lds = (size_t)a.ck * ct * sizeof(float);
  switch (ct) {
    case 1: return launch_mode<VEC, 1>(a, mode, grid, lds, st);
    case 2: return launch_mode<VEC, 2>(a, mode, grid, lds, st);
    default: return launch_mode<VEC, 4>(a, mode, grid, lds, st);
  }
}

}  // namespace

int lmm_grid(int64_t r_out, int logL) {
  int64_t rows_per_iter = (int64_t)(kBlock >> logL) * kUnroll;
  int64_t g = (r_out + rows_per_iter - 1) / rows_per_iter;
  if (g < 1) g = 1;
  if (g > 2048) g = 2048;
  return (int)g;
}

hipError_t launch_lmm_rows(const LmmArgs& a, int vec, int mode, hipStream_t st, int* grid_out) {
  int grid = lmm_grid(a.r_out, a.logL);
  if (grid_out) *grid_out = grid;
  if (a.r_out <= 0) return hipSuccess;
  switch (vec) {
    case 4: return launch_ct<4>(a, mode, grid, st);
    case 2: return launch_ct<2>(a, mode, grid, st);
    default: return launch_ct<1>(a, mode, grid, st);
  }
}

}  // namespace ilargi
