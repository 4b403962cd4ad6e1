// Device body of the flat column reduce (see kernels_colred_flat.hip), shared by the two launches that run it.
#pragma once
#include <cstdint>

#include "ilargi_internal.h"

namespace ilargi {

constexpr int colred_flat_lds_floats(int cmax) { return kWave * (4 * cmax + 1); }

// CMAX: compile-time bound of the operand columns (8 or 16).  YV4: operand rows are whole, aligned float4s.
// The body serves the kernel of its own and the launch it shares with the join-order pass of a joined source:
// `bid` of `nblocks` workgroups, `tile_lds` = colred_flat_lds_floats(CMAX) floats of LDS.
template <int CMAX, bool YV4>
__device__ __forceinline__ void colred_flat_body(const ColredFlatArgs& a, float* tile_lds, int bid, int nblocks) {
  float (*tile)[4 * CMAX + 1] = reinterpret_cast<float (*)[4 * CMAX + 1]>(tile_lds);
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int nvec = a.nvec;
  const int rpi = kWave / nvec;                                 // rows per wavefront step
  const bool active = lane < rpi * nvec;
  const int r = lane / nvec;
  float acc[4][CMAX];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int n = 0; n < CMAX; ++n) acc[e][n] = 0.0f;
  const int64_t nsteps = (a.rows + rpi - 1) / rpi;
  const int64_t stride = (int64_t)nblocks * (kBlock / kWave);
  const float4* S4 = reinterpret_cast<const float4*>(a.S);
  auto load = [&](int64_t step, float4& s, float (&y)[CMAX]) {
    const int64_t row = step * rpi + r;
    const bool live = active && step < nsteps && row < a.rows;
    s = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
    for (int n = 0; n < CMAX; ++n) y[n] = 0.0f;
    if (live) {
      s = S4[step * rpi * nvec + lane];                         // = float4 number  row * nvec + part
      const float* yr = a.Y + row * a.ldy;
      if constexpr (YV4) {
#pragma unroll
        for (int j = 0; j < CMAX / 4; ++j) {
          if (4 * j < a.c) {
            const float4 v = *reinterpret_cast<const float4*>(yr + 4 * j);
            y[4 * j] = v.x; y[4 * j + 1] = v.y; y[4 * j + 2] = v.z; y[4 * j + 3] = v.w;
          }
        }
      } else {
#pragma unroll
        for (int n = 0; n < CMAX; ++n)
          if (n < a.c) y[n] = yr[n];
      }
    }
  };
  auto fma_row = [&](const float4& s, const float (&y)[CMAX]) {
#pragma unroll
    for (int n = 0; n < CMAX; ++n) {
      acc[0][n] = fmaf(s.x, y[n], acc[0][n]);
      acc[1][n] = fmaf(s.y, y[n], acc[1][n]);
      acc[2][n] = fmaf(s.z, y[n], acc[2][n]);
      acc[3][n] = fmaf(s.w, y[n], acc[3][n]);
    }
  };
  for (int64_t step = (int64_t)bid * (kBlock / kWave) + wave; step < nsteps; step += 2 * stride) {
    float4 s0, s1;
    float y0[CMAX], y1[CMAX];
    load(step, s0, y0);                                         // two steps in flight
    load(step + stride, s1, y1);
    fma_row(s0, y0);
    fma_row(s1, y1);
  }
  // lanes with the same part, in row order; then the wavefronts in order
  const int outs = nvec * 4 * CMAX;                             // (part, component, operand column), at most 1024
  float tot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int w = 0; w < kBlock / kWave; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int n = 0; n < CMAX; ++n) tile[lane][e * CMAX + n] = acc[e][n];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int o = tid + k * kBlock;
      if (o < outs) {
        const int p = o / (4 * CMAX), en = o - p * (4 * CMAX);
        float sum = 0.0f;
        for (int rr = 0; rr < rpi; ++rr) sum += tile[rr * nvec + p][en];
        tot[k] += sum;
      }
    }
  }
  float* gp = a.partial + (int64_t)bid * (4 * nvec) * a.c;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int o = tid + k * kBlock;
    if (o < outs) {
      const int p = o / (4 * CMAX), en = o - p * (4 * CMAX);
      const int e = en / CMAX, n = en - e * CMAX;
      if (n < a.c) gp[(4 * p + e) * a.c + n] = tot[k];
    }
  }
}


}  // namespace ilargi
