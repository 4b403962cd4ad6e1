// Scalar operators of Tab. 2 in factorized form:  T (/) x  and  f(T)  touch the source tables only (cost
// sum_k m_k instead of m_T), and so does colSum(T) = sum_k M_k (D_k^T cnt_k) with cnt_k the fan-out of the
// rows of source k (the column sums of I_k); rowSum(T) = T 1 is the left multiply by a vector of ones.
// This file holds the streaming element-wise kernel and the small fills the two sums need.
#include <algorithm>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

template <int OP>
__device__ __forceinline__ float apply_op(float a, float x) {
  if constexpr (OP == 0) return a * x;
  else if constexpr (OP == 1) return a / x;
  else if constexpr (OP == 2) return a + x;
  else if constexpr (OP == 3) return a - x;
  else if constexpr (OP == 4) return powf(a, x);
  else if constexpr (OP == 5) return expf(a);
  else if constexpr (OP == 6) return logf(a);
  else if constexpr (OP == 7) return sqrtf(a);
  else if constexpr (OP == 8) return fabsf(a);
  else return a * a;
}

// out[e] = op(in[e], x); float4 body when both pointers allow it, scalar tail.
template <int OP>
__global__ __launch_bounds__(kBlock) void elementwise_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                             int64_t n, float x, int vec4) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t nthreads = (int64_t)gridDim.x * blockDim.x;
  int64_t done = 0;
  if (vec4) {
    const int64_t n4 = n / 4;
    const float4* in4 = reinterpret_cast<const float4*>(in);
    float4* out4 = reinterpret_cast<float4*>(out);
    for (int64_t e = tid; e < n4; e += nthreads) {
      float4 v = in4[e];
      v.x = apply_op<OP>(v.x, x); v.y = apply_op<OP>(v.y, x); v.z = apply_op<OP>(v.z, x); v.w = apply_op<OP>(v.w, x);
      out4[e] = v;
    }
    done = n4 * 4;
  }
  for (int64_t e = done + tid; e < n; e += nthreads) out[e] = apply_op<OP>(in[e], x);
}

__global__ __launch_bounds__(kBlock) void fill_kernel(float* __restrict__ p, int64_t n, float v) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) p[e] = v;
}

// cnt[j] = number of target rows that take row j of the source (rowptr of the inverse index).
__global__ __launch_bounds__(kBlock) void fanout_kernel(const int32_t* __restrict__ rowptr, int64_t rows,
                                                        float* __restrict__ cnt) {
  for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < rows; j += (int64_t)gridDim.x * blockDim.x)
    cnt[j] = (float)(rowptr[j + 1] - rowptr[j]);
}

// out (cols x rows) = in (rows x cols)^T through 32 x 33 LDS tiles: reads and writes are both coalesced.
__global__ __launch_bounds__(kBlock) void transpose_kernel(const float* __restrict__ in, int64_t rows, int64_t cols,
                                                           float* __restrict__ out) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;   // 32 x 8 threads
  const int64_t tiles_c = (cols + 31) / 32, tiles_r = (rows + 31) / 32;
  for (int64_t t = blockIdx.x; t < tiles_r * tiles_c; t += gridDim.x) {
    const int64_t r0 = (t / tiles_c) * 32, c0 = (t % tiles_c) * 32;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t r = r0 + ty + 8 * k, c = c0 + tx;
      tile[ty + 8 * k][tx] = (r < rows && c < cols) ? in[r * cols + c] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t c = c0 + ty + 8 * k, r = r0 + tx;
      if (c < cols && r < rows) out[c * rows + r] = tile[tx][ty + 8 * k];
    }
  }
}

// E (rows x w, row-major) = columns [j0, j0 + w) of the rows x rows identity.
__global__ __launch_bounds__(kBlock) void eye_block_kernel(float* E, int64_t rows, int w, int64_t j0) {
  const int64_t n = rows * w;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < n; e += (int64_t)gridDim.x * kBlock) {
    const int64_t i = e / w;
    E[e] = (i - j0 == e - i * w) ? 1.0f : 0.0f;
  }
}

// G (n x n): every cell below the diagonal takes the value of its mirror cell above it.
__global__ __launch_bounds__(kBlock) void mirror_upper_kernel(float* G, int64_t n) {
  const int64_t cells = n * n;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < cells; e += (int64_t)gridDim.x * kBlock) {
    const int64_t i = e / n, j = e - i * n;
    if (j < i) G[e] = G[j * n + i];
  }
}

int grid_for(int64_t n) {
  int64_t g = (n + kBlock - 1) / kBlock;
  return (int)(g < 1 ? 1 : (g > 8192 ? 8192 : g));
}

// Streaming kernels that mostly write: one element per thread, workgroups in address order.  On the MI355X a
// grid-stride loop over a few thousand resident workgroups writes at about 4.4 TB/s, a launch of one short
// workgroup per 4 KiB, dispatched in order, at 6 to 6.9 TB/s (reads do not care).
int grid_for_stream(int64_t n) {
  int64_t g = (n + kBlock - 1) / kBlock;
  return (int)(g < 1 ? 1 : (g > (1 << 22) ? (1 << 22) : g));
}

}  // namespace

hipError_t launch_elementwise(int op, const float* in, float* out, int64_t n, float x, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int vec4 = reinterpret_cast<uintptr_t>(in) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0;
  const int grid = grid_for_stream(vec4 ? n / 4 + 1 : n);
  switch (op) {
    case 0: elementwise_kernel<0><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 1: elementwise_kernel<1><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 2: elementwise_kernel<2><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 3: elementwise_kernel<3><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 4: elementwise_kernel<4><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 5: elementwise_kernel<5><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 6: elementwise_kernel<6><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 7: elementwise_kernel<7><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 8: elementwise_kernel<8><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    case 9: elementwise_kernel<9><<<grid, kBlock, 0, st>>>(in, out, n, x, vec4); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_transpose(const float* in, int64_t rows, int64_t cols, float* out, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const int64_t tiles = ((rows + 31) / 32) * ((cols + 31) / 32);
  transpose_kernel<<<(int)std::min<int64_t>(tiles, 16384), kBlock, 0, st>>>(in, rows, cols, out);
  return hipGetLastError();
}

hipError_t launch_fill(float* p, int64_t n, float v, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  fill_kernel<<<grid_for_stream(n), kBlock, 0, st>>>(p, n, v);
  return hipGetLastError();
}

hipError_t launch_eye_block(float* E, int64_t rows, int w, int64_t j0, hipStream_t st) {
  if (rows <= 0 || w <= 0) return hipSuccess;
  eye_block_kernel<<<grid_for(rows * w), kBlock, 0, st>>>(E, rows, w, j0);
  return hipGetLastError();
}

hipError_t launch_mirror_upper(float* G, int64_t n, hipStream_t st) {
  if (n <= 1) return hipSuccess;
  mirror_upper_kernel<<<grid_for(n * n), kBlock, 0, st>>>(G, n);
  return hipGetLastError();
}

hipError_t launch_fanout(const int32_t* rowptr, int64_t rows, float* cnt, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  fanout_kernel<<<grid_for(rows), kBlock, 0, st>>>(rowptr, rows, cnt);
  return hipGetLastError();
}

}  // namespace ilargi
