// Plan-time kernels: range check of the compressed indicator vector (Def. 2) and the inverse index
// of I_k in compressed-row form, built with a stable least-significant-digit radix sort so that the
// target rows of one source row come out in ascending order.  Integer work only.
#include "ilargi_internal.h"

namespace ilargi {

// flags[0] |= 1 if an entry is outside [-1, r_k); flags[1] |= 1 if the vector is not the identity on
// its first r_k entries followed by -1.
__global__ __launch_bounds__(kBlock) void check_idx_kernel(const int32_t* __restrict__ idx, int64_t r_T,
                                                           int64_t r_k, int32_t* __restrict__ flags) {
  int bad = 0, notid = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < r_T;
       i += (int64_t)gridDim.x * blockDim.x) {
    int32_t v = idx[i];
    if (v < -1 || v >= r_k) bad = 1;
    int32_t want = (i < r_k) ? (int32_t)i : -1;
    if (v != want) notid = 1;
  }
  if (__any(bad) && (threadIdx.x % kWave) == 0) atomicOr(&flags[0], 1);
  if (__any(notid) && (threadIdx.x % kWave) == 0) atomicOr(&flags[1], 1);
}

hipError_t launch_check_idx(const int32_t* idx, int64_t r_T, int64_t r_k, int32_t* flags, hipStream_t st) {
  if (r_T == 0) return hipSuccess;
  int grid = (int)((r_T + kBlock - 1) / kBlock);
  if (grid > 2048) grid = 2048;
  check_idx_kernel<<<grid, kBlock, 0, st>>>(idx, r_T, r_k, flags);
  return hipGetLastError();
}

__device__ __forceinline__ uint32_t sort_key(int32_t v, uint32_t r_k) { return v < 0 ? r_k : (uint32_t)v; }

// Digit histogram of one chunk of keys.  hist is digit-major: hist[d * nchunks + chunk].
template <bool FIRST>
__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const int32_t* __restrict__ keys, int64_t n,
                                                            uint32_t r_k, int shift, int nchunks,
                                                            int32_t* __restrict__ hist) {
  __shared__ int32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  int64_t lo = (int64_t)blockIdx.x * kSortChunk;
  int64_t hi = lo + kSortChunk < n ? lo + kSortChunk : n;
  for (int64_t i = lo + threadIdx.x; i < hi; i += kBlock) {
    uint32_t k = FIRST ? sort_key(keys[i], r_k) : (uint32_t)keys[i];
    atomicAdd(&h[(k >> shift) & 255], 1);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nchunks + blockIdx.x] = h[threadIdx.x];
}

// In-place exclusive prefix sum of n integers by one workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void exclusive_scan_kernel(int32_t* __restrict__ a, int64_t n) {
  __shared__ int32_t wsum[16];
  __shared__ int32_t carry;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024) {
    int64_t i = base + threadIdx.x;
    int32_t v = i < n ? a[i] : 0;
    int32_t inc = v;
    for (int d = 1; d < kWave; d <<= 1) {
      int32_t t = __shfl_up(inc, d);
      if (lane >= d) inc += t;
    }
    if (lane == kWave - 1) wsum[wave] = inc;
    __syncthreads();
    int32_t woff = 0;
    for (int w = 0; w < wave; ++w) woff += wsum[w];
    int32_t c = carry;
    if (i < n) a[i] = c + woff + inc - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry = c + woff + inc;
    __syncthreads();
  }
}

// Two-level form for long arrays: every workgroup scans its own 1024 integers in place and leaves their sum;
// the sums are scanned by the single-workgroup kernel above and added back.
__global__ __launch_bounds__(1024) void scan_blocks_kernel(int32_t* __restrict__ a, int64_t n,
                                                           int32_t* __restrict__ totals) {
  __shared__ int32_t wsum[16];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
  const int32_t v = i < n ? a[i] : 0;
  int32_t inc = v;
  for (int d = 1; d < kWave; d <<= 1) {
    int32_t t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  if (lane == kWave - 1) wsum[wave] = inc;
  __syncthreads();
  int32_t woff = 0;
  for (int w = 0; w < wave; ++w) woff += wsum[w];
  if (i < n) a[i] = woff + inc - v;
  if (threadIdx.x == 1023) totals[blockIdx.x] = woff + inc;
}

__global__ __launch_bounds__(1024) void scan_add_kernel(int32_t* __restrict__ a, int64_t n,
                                                        const int32_t* __restrict__ totals) {
  const int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
  if (i < n) a[i] += totals[blockIdx.x];
}

// In-place exclusive prefix sum of n integers; `totals` holds ceil(n / 1024) integers of scratch.
void launch_exclusive_scan(int32_t* a, int64_t n, int32_t* totals, hipStream_t st) {
  if (n <= 4096) {
    exclusive_scan_kernel<<<1, 1024, 0, st>>>(a, n);
    return;
  }
  const int nb = (int)((n + 1023) / 1024);
  scan_blocks_kernel<<<nb, 1024, 0, st>>>(a, n, totals);
  exclusive_scan_kernel<<<1, 1024, 0, st>>>(totals, nb);
  scan_add_kernel<<<nb, 1024, 0, st>>>(a, n, totals);
}

// Stable scatter of one chunk: a single wavefront walks its keys 64 at a time; the rank of a key among
// the equal digits of the same step comes from a ballot match, the running per-digit offsets sit in LDS.
template <bool FIRST>
__global__ __launch_bounds__(kWave) void radix_scatter_kernel(const int32_t* __restrict__ keys_in,
                                                              const int32_t* __restrict__ vals_in, int64_t n,
                                                              uint32_t r_k, int shift, int nchunks,
                                                              const int32_t* __restrict__ hist,
                                                              int32_t* __restrict__ keys_out,
                                                              int32_t* __restrict__ vals_out) {
  __shared__ int32_t off[256];
  const int lane = threadIdx.x;
  for (int d = lane; d < 256; d += kWave) off[d] = hist[(int64_t)d * nchunks + blockIdx.x];
  __syncthreads();
  int64_t lo = (int64_t)blockIdx.x * kSortChunk;
  int64_t hi = lo + kSortChunk < n ? lo + kSortChunk : n;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  for (int64_t base = lo; base < hi; base += kWave) {
    int64_t i = base + lane;
    bool live = i < hi;
    uint32_t k = 0;
    int32_t v = 0;
    if (live) {
      k = FIRST ? sort_key(keys_in[i], r_k) : (uint32_t)keys_in[i];
      v = FIRST ? (int32_t)i : vals_in[i];
    }
    uint32_t d = (k >> shift) & 255;
    uint64_t match = __ballot(live);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      uint64_t vote = __ballot(live && ((d >> b) & 1));
      match &= ((d >> b) & 1) ? vote : ~vote;
    }
    int rank = __popcll(match & lt_mask);
    int32_t dst = 0;
    if (live) dst = off[d] + rank;
    __syncthreads();
    if (live && (match >> lane) <= 1ull) off[d] += __popcll(match);  // highest lane of its digit group
    __syncthreads();
    if (live) {
      keys_out[dst] = (int32_t)k;
      vals_out[dst] = v;
    }
  }
}

// rowptr[j] = first position in the sorted keys whose key is >= j  (keys of absent rows equal r_k).
__global__ __launch_bounds__(kBlock) void rowptr_kernel(const int32_t* __restrict__ sorted, int64_t n,
                                                        int64_t r_k, int32_t* __restrict__ rowptr) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p <= n;
       p += (int64_t)gridDim.x * blockDim.x) {
    int64_t cur = p < n ? (int64_t)sorted[p] : r_k;
    int64_t prev = p > 0 ? (int64_t)sorted[p - 1] : -1;
    for (int64_t j = prev + 1; j <= cur; ++j) rowptr[j] = (int32_t)p;
  }
}

__global__ __launch_bounds__(kBlock) void copy_i32_kernel(const int32_t* __restrict__ src, int64_t n,
                                                          int32_t* __restrict__ dst) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

size_t sort_hist_ints(int64_t r_T) {
  int64_t nchunks = (r_T + kSortChunk - 1) / kSortChunk;
  const int64_t h = 256 * (nchunks > 0 ? nchunks : 1);
  return (size_t)(h + (h + 1023) / 1024 + 1);     // digit-major histogram, then the block sums of its two-level scan
}

// Sorts (key = source row or r_k for "none", value = target row) by key, stably, and derives rowptr.
// perm receives all r_T values; its first rowptr[r_k] entries are the inverse index.
hipError_t launch_sort_by_source_row(const int32_t* idx, int64_t r_T, int64_t r_k, int32_t* keys_a,
                                     int32_t* vals_a, int32_t* keys_b, int32_t* vals_b, int32_t* hist,
                                     int32_t* rowptr, int32_t* perm, hipStream_t st) {
  int rgrid = (int)((r_T + 1 + kBlock - 1) / kBlock);
  if (rgrid > 2048) rgrid = 2048;
  if (r_T == 0) {
    rowptr_kernel<<<1, kBlock, 0, st>>>(nullptr, 0, r_k, rowptr);
    return hipGetLastError();
  }
  int nchunks = (int)((r_T + kSortChunk - 1) / kSortChunk);
  int bits = ilog2_ceil(r_k + 1);
  if (bits < 1) bits = 1;
  int npass = (bits + 7) / 8;
  const int32_t* kin = idx;
  const int32_t* vin = nullptr;
  int32_t* kout = keys_a;
  int32_t* vout = vals_a;
  for (int p = 0; p < npass; ++p) {
    int shift = 8 * p;
    if (p == 0) {
      radix_hist_kernel<true><<<nchunks, kBlock, 0, st>>>(kin, r_T, (uint32_t)r_k, shift, nchunks, hist);
    } else {
      radix_hist_kernel<false><<<nchunks, kBlock, 0, st>>>(kin, r_T, (uint32_t)r_k, shift, nchunks, hist);
    }
    launch_exclusive_scan(hist, (int64_t)256 * nchunks, hist + (int64_t)256 * nchunks, st);
    if (p == 0) {
      radix_scatter_kernel<true><<<nchunks, kWave, 0, st>>>(kin, vin, r_T, (uint32_t)r_k, shift, nchunks, hist,
                                                           kout, vout);
    } else {
      radix_scatter_kernel<false><<<nchunks, kWave, 0, st>>>(kin, vin, r_T, (uint32_t)r_k, shift, nchunks, hist,
                                                            kout, vout);
    }
    kin = kout;
    vin = vout;
    kout = (kout == keys_a) ? keys_b : keys_a;
    vout = (vout == vals_a) ? vals_b : vals_a;
  }
  rowptr_kernel<<<rgrid, kBlock, 0, st>>>(kin, r_T, r_k, rowptr);
  int cgrid = (int)((r_T + kBlock - 1) / kBlock);
  if (cgrid > 2048) cgrid = 2048;
  copy_i32_kernel<<<cgrid, kBlock, 0, st>>>(vin, r_T, perm);
  return hipGetLastError();
}

__global__ __launch_bounds__(kBlock) void fill_zero_kernel(float* __restrict__ p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = 0.0f;
}

hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int grid = (int)((n + kBlock - 1) / kBlock);
  if (grid > 4096) grid = 4096;
  fill_zero_kernel<<<grid, kBlock, 0, st>>>(p, n);
  return hipGetLastError();
}

}  // namespace ilargi

// Plain streaming kernels used to calibrate what the memory system delivers (benchmarks and counter
// scaling): copy, read-only (sum into one value per workgroup) and write-only.
namespace ilargi {

__global__ __launch_bounds__(kBlock) void probe_copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src,
                                                            int64_t n4) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

__global__ __launch_bounds__(kBlock) void probe_read_kernel(const float4* __restrict__ src, int64_t n4,
                                                            float* __restrict__ sink) {
  float acc = 0.0f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) {
    float4 v = src[i];
    acc += (v.x + v.y) + (v.z + v.w);
  }
  for (int m = kWave / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (threadIdx.x == 0) sink[blockIdx.x] = acc;
}

// read-only, every workgroup walking a contiguous chunk of its own (kind 5), and with eight loads in flight per
// thread in a grid-stride walk (kind 6)
__global__ __launch_bounds__(kBlock) void probe_read_chunked_kernel(const float4* __restrict__ src, int64_t n4,
                                                                    float* __restrict__ sink) {
  const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
  const int64_t b0 = (int64_t)blockIdx.x * per, b1 = min(b0 + per, n4);
  float acc = 0.0f;
  for (int64_t i = b0 + threadIdx.x; i < b1; i += blockDim.x) {
    float4 v = src[i];
    acc += (v.x + v.y) + (v.z + v.w);
  }
  for (int m = kWave / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (threadIdx.x == 0) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(kBlock) void probe_read_deep_kernel(const float4* __restrict__ src, int64_t n4,
                                                                 float* __restrict__ sink) {
  float acc = 0.0f;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < n4; i += 8 * stride) {
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += (v[u].x + v[u].y) + (v[u].z + v[u].w);
  }
  for (; i < n4; i += stride) {
    float4 v = src[i];
    acc += (v.x + v.y) + (v.z + v.w);
  }
  for (int m = kWave / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m);
  if (threadIdx.x == 0) sink[blockIdx.x] = acc;
}

__global__ __launch_bounds__(kBlock) void probe_write_kernel(float4* __restrict__ dst, int64_t n4) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = make_float4(1.0f, 2.0f, 3.0f, 4.0f);
}

typedef float nt4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kBlock) void probe_copy_nt_kernel(nt4* __restrict__ dst, const nt4* __restrict__ src,
                                                               int64_t n4) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
    __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}
__global__ __launch_bounds__(kBlock) void probe_write_nt_kernel(nt4* __restrict__ dst, int64_t n4) {
  nt4 v = {1.0f, 2.0f, 3.0f, 4.0f};
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x)
    __builtin_nontemporal_store(v, &dst[i]);
}

hipError_t launch_probe(int kind, float* dst, const float* src, int64_t n_floats, int blocks, hipStream_t st) {
  int64_t n4 = n_floats / 4;
  if (n4 <= 0) return hipSuccess;
  if (kind == 3) { probe_copy_nt_kernel<<<blocks, kBlock, 0, st>>>((nt4*)dst, (const nt4*)src, n4); return hipGetLastError(); }
  if (kind == 4) { probe_write_nt_kernel<<<blocks, kBlock, 0, st>>>((nt4*)dst, n4); return hipGetLastError(); }
  if (kind == 5) { probe_read_chunked_kernel<<<blocks, kBlock, 0, st>>>((const float4*)src, n4, dst); return hipGetLastError(); }
  if (kind == 6) { probe_read_deep_kernel<<<blocks, kBlock, 0, st>>>((const float4*)src, n4, dst); return hipGetLastError(); }
  if (kind == 0) probe_copy_kernel<<<blocks, kBlock, 0, st>>>((float4*)dst, (const float4*)src, n4);
  else if (kind == 1) probe_read_kernel<<<blocks, kBlock, 0, st>>>((const float4*)src, n4, dst);
  else probe_write_kernel<<<blocks, kBlock, 0, st>>>((float4*)dst, n4);
  return hipGetLastError();
}

}  // namespace ilargi
