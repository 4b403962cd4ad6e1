// Gram blocks of tables with 36..64 columns (crossprod, the rewrite of Sec. 2.2 applied to both factors), on the
// matrix cores, as streaming kernels without LDS staging or barriers in the loop:
//   diagonal block   C = sum_t w_t d_t^T d_t          (D_k^T diag(fan-out) D_k; w = 1 for an identity source)
//   pair block       C = sum_p a_{ia[p]}^T b_{ib[p]}  (D_k^T (I_k^T I_l) D_l over a list of (row of D_k, row of D_l)
//                                                      pairs that share a target row, built with the plan)
// A table row of at most 64 columns is at most 256 bytes.  Lane (s, q) of a wavefront loads the float4 at columns
// 4 s .. 4 s + 3 of row q of a quad of four rows: for the diagonal block four consecutive rows, i.e. one kilobyte of
// contiguous memory per load instruction.  Component c of that float4 is the operand of the 16 x 16 x 4 product for
// the INTERLEAVED column tile c = {c, 4 + c, 8 + c, ...} (M or N index s stands for column 4 s + c, K slot q for row
// q of the quad), so one 128-bit load feeds every tile: 10 products per quad for the diagonal block (tiles c <= c';
// the others follow by symmetry), 16 for a pair block.  The rows of a wavefront's next run of quads are in flight
// while the products of the current run are issued.  Every wavefront
// keeps all tiles in registers; the four wavefronts of a workgroup are added in order in LDS at the end, and the
// per-workgroup partial blocks are added in workgroup order by the caller.  No floating-point atomics.
#include <algorithm>
#include <cstdint>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kGnUDiag = 8;          // quads of rows in a wavefront's run (diagonal block)
constexpr int kGnUPairs = 4;         // ... pair block (two tables, sixteen tiles: twice the registers per quad)
constexpr int kGnWaves = kBlock / kWave;

// PAIRS: rows through the index vectors ia / ib (both valid for every entry); else row t of A with weight w_t.
template <bool PAIRS, bool WEIGHTED>
__global__ __launch_bounds__(kBlock) void gram_narrow_kernel(TredArgs a) {
  __shared__ float red[64 * 64];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int s = lane % 16, q = lane / 16;
  constexpr int NT = PAIRS ? 16 : 10;
  constexpr int kGnU = PAIRS ? kGnUPairs : kGnUDiag;
  v4f acc[NT];
#pragma unroll
  for (int u = 0; u < NT; ++u) acc[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  const int64_t t_hi = a.n_rows;
  const int cola = min(4 * s, a.ca - 4), colb = min(4 * s, a.cb - 4);     // clamped: lanes beyond the table are zeroed
  const bool ina = 4 * s < a.ca, inb = 4 * s < a.cb;
  // A wavefront takes runs of kGnU consecutive quads (4 kGnU rows: for the diagonal block 8 KiB of contiguous memory),
  // the four wavefronts of the workgroup neighbouring runs.  The rows of its next run are requested before the
  // products of the current one are issued (for a pair block the list entries of the run after that, too).
  // Workgroups walk the rows with a grid stride: at any time the device reads one moving window of the table.
  constexpr int RUN = 4 * kGnU;
  const int64_t stride = (int64_t)RUN * kGnWaves * gridDim.x;
  v4f va[kGnU], vb[PAIRS ? kGnU : 1];
  int wd = 0;                                                   // lane l: fan-out of row l of the run
  int ra[PAIRS ? kGnU : 1], rb[PAIRS ? kGnU : 1];
  auto request_idx = [&](int64_t base) {
    if constexpr (PAIRS) {
#pragma unroll
      for (int u = 0; u < kGnU; ++u) {
        const int64_t t = min(base + 4 * u + q, a.n_rows - 1);
        ra[u] = a.ia[t];
        rb[u] = a.ib[t];
      }
    }
  };
  auto request_rows = [&](int64_t base) {
#pragma unroll
    for (int u = 0; u < kGnU; ++u) {
      if constexpr (PAIRS) {
        va[u] = *reinterpret_cast<const v4f*>(a.A + (int64_t)ra[u] * a.lda + cola);
        vb[u] = *reinterpret_cast<const v4f*>(a.B + (int64_t)rb[u] * a.ldb + a.bcol0 + colb);
      } else {
        const int64_t t = min(base + 4 * u + q, a.n_rows - 1);
        va[u] = *reinterpret_cast<const v4f*>(a.A + t * a.lda + cola);
      }
    }
    if constexpr (WEIGHTED) {
      const int64_t t = min(base + min(lane, RUN - 1), a.n_rows - 1);
      wd = a.wptr[t + 1] - a.wptr[t];
    }
  };
  int64_t base = (int64_t)RUN * (kGnWaves * blockIdx.x + wave);
  request_idx(base);
  request_rows(base);
  request_idx(base + stride);
  for (; base < t_hi; base += stride) {
    v4f xa[kGnU], xb[PAIRS ? kGnU : 1];
    float wv[kGnU];
#pragma unroll
    for (int u = 0; u < kGnU; ++u) {
      const bool live = base + 4 * u + q < t_hi;
      xa[u] = (live && ina) ? va[u] : (v4f){0.0f, 0.0f, 0.0f, 0.0f};
      if constexpr (PAIRS) xb[u] = (live && inb) ? vb[u] : (v4f){0.0f, 0.0f, 0.0f, 0.0f};
      if constexpr (WEIGHTED) wv[u] = (float)__shfl(wd, 4 * u + q);
      else wv[u] = 1.0f;
    }
    request_rows(base + stride);                               // (addresses are clamped: a run beyond the end reads the last row)
    request_idx(base + 2 * stride);
#pragma unroll
    for (int u = 0; u < kGnU; ++u) {
      if constexpr (PAIRS) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int d = 0; d < 4; ++d) acc[4 * c + d] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[u][c], xb[u][d], acc[4 * c + d], 0, 0, 0);
      } else {
        v4f xw = xa[u];
        if constexpr (WEIGHTED) xw = xa[u] * wv[u];
        int k = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int d = c; d < 4; ++d) { acc[k] = __builtin_amdgcn_mfma_f32_16x16x4f32(xw[c], xa[u][d], acc[k], 0, 0, 0); ++k; }
      }
    }
  }

  // tile (c, d), register r of lane (s, q) = C[4 (4 q + r) + c][4 s + d]; the wavefronts in order
  for (int w = 0; w < kGnWaves; ++w) {
    __syncthreads();
    if (wave == w) {
      int k = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int d = PAIRS ? 0 : c; d < 4; ++d) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float* p = red + (4 * (4 * q + r) + c) * 64 + 4 * s + d;
            if (w == 0) *p = acc[k][r];
            else *p += acc[k][r];
          }
          ++k;
        }
    }
  }
  __syncthreads();
  float* out = a.partial + (int64_t)blockIdx.x * a.ca * a.cb;
  for (int e = tid; e < a.ca * a.cb; e += kBlock) {
    const int i = e / a.cb, j = e - i * a.cb;
    // diagonal block: element (i, j) with i % 4 > j % 4 was not formed; it equals element (j, i)
    const bool direct = PAIRS || (i % 4) <= (j % 4);
    out[e] = direct ? red[i * 64 + j] : red[j * 64 + i];
  }
}

// Pair list of two sources: the target rows both of them feed, in target-row order.  flag[i] = 1 for such a row
// (a source without row index feeds its first `rows` target rows); after the exclusive scan of the flags the second
// kernel writes the pair (row of the first source, row of the second) of target row i to position scan[i].
__global__ __launch_bounds__(kBlock) void pair_flag_kernel(const int32_t* __restrict__ idx_a, int64_t rows_a,
                                                           const int32_t* __restrict__ idx_b, int64_t rows_b, int64_t r_T,
                                                           int32_t* __restrict__ flag) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= r_T; i += (int64_t)gridDim.x * blockDim.x) {
    int f = 0;
    if (i < r_T) {
      const int64_t ra = idx_a ? idx_a[i] : (i < rows_a ? i : -1);
      const int64_t rb = idx_b ? idx_b[i] : (i < rows_b ? i : -1);
      f = ra >= 0 && rb >= 0;
    }
    flag[i] = f;
  }
}

__global__ __launch_bounds__(kBlock) void pair_write_kernel(const int32_t* __restrict__ idx_a, int64_t rows_a,
                                                            const int32_t* __restrict__ idx_b, int64_t rows_b, int64_t r_T,
                                                            const int32_t* __restrict__ scan, int32_t* __restrict__ list_a,
                                                            int32_t* __restrict__ list_b) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < r_T; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t ra = idx_a ? idx_a[i] : (i < rows_a ? i : -1);
    const int64_t rb = idx_b ? idx_b[i] : (i < rows_b ? i : -1);
    if (ra >= 0 && rb >= 0) {
      const int32_t p = scan[i];
      list_a[p] = (int32_t)ra;
      list_b[p] = (int32_t)rb;
    }
  }
}

}  // namespace

// scan: r_T + 1 integers of scratch (scan[r_T] receives the number of pairs), totals: ceil((r_T + 1) / 1024) more;
// list_a / list_b: room for r_T entries each.  Row indices must already be validated.
hipError_t launch_pair_list(const int32_t* idx_a, int64_t rows_a, const int32_t* idx_b, int64_t rows_b, int64_t r_T,
                            int32_t* scan, int32_t* totals, int32_t* list_a, int32_t* list_b, hipStream_t st) {
  if (r_T <= 0) return hipSuccess;
  const int grid = (int)std::min<int64_t>((r_T + kBlock) / kBlock, 8192);
  pair_flag_kernel<<<grid, kBlock, 0, st>>>(idx_a, rows_a, idx_b, rows_b, r_T, scan);
  launch_exclusive_scan(scan, r_T + 1, totals, st);
  pair_write_kernel<<<grid, kBlock, 0, st>>>(idx_a, rows_a, idx_b, rows_b, r_T, scan, list_a, list_b);
  return hipGetLastError();
}

// Diagonal block: A == B without index vectors, 36..64 columns in whole aligned float4s.
bool gram_narrow_supported(const TredArgs& a) {
  return a.upper_only && a.A == a.B && a.ia == nullptr && a.ib == nullptr && a.ca == a.cb && a.lda == a.ldb && a.bcol0 == 0 &&
         a.ca > 32 && a.ca <= 64 && a.ca % 4 == 0 && a.lda % 4 == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0 &&
         a.n_rows >= 1 && a.a_rows >= a.n_rows;
}

// Pair block: n_rows pairs (ia[p], ib[p]), every index valid; both tables with 4..64 columns in whole aligned float4s.
bool gram_pairs_supported(const TredArgs& a) {
  return !a.upper_only && a.ia != nullptr && a.ib != nullptr && a.wptr == nullptr && a.n_rows >= 1 &&
         a.ca >= 4 && a.ca <= 64 && a.ca % 4 == 0 && a.lda % 4 == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0 &&
         a.cb >= 4 && a.cb <= 64 && a.cb % 4 == 0 && a.ldb % 4 == 0 && a.bcol0 % 4 == 0 && reinterpret_cast<uintptr_t>(a.B) % 16 == 0;
}

// At most four workgroups per compute unit and as many as partial_floats holds; *nch_out partial blocks of ca x cb
// floats are left in `partial`.
hipError_t launch_gram_narrow(TredArgs& a, float* partial, int64_t partial_floats, hipStream_t st, int* nch_out) {
  *nch_out = 0;
  const bool pairs = a.ia != nullptr;
  if (!(pairs ? gram_pairs_supported(a) : gram_narrow_supported(a))) return hipErrorInvalidValue;
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      return (int)prop.multiProcessorCount;
    return 256;
  }();
  const int64_t elems = (int64_t)a.ca * a.cb;
  int64_t nch = std::min<int64_t>(4 * cus, partial_floats / elems);
  const int step_rows = 4 * kGnWaves * (pairs ? kGnUPairs : kGnUDiag);
  nch = std::min<int64_t>(nch, (a.n_rows + step_rows - 1) / step_rows);
  if (nch < 1) return hipErrorInvalidValue;
  a.partial = partial;
  if (pairs) gram_narrow_kernel<true, false><<<(unsigned)nch, kBlock, 0, st>>>(a);
  else if (a.wptr != nullptr) gram_narrow_kernel<false, true><<<(unsigned)nch, kBlock, 0, st>>>(a);
  else gram_narrow_kernel<false, false><<<(unsigned)nch, kBlock, 0, st>>>(a);
  *nch_out = (int)nch;
  return hipGetLastError();
}

}  // namespace ilargi
