// Transposed multiply  T^T Y = sum_k M_k (D_k^T (I_k^T Y))  for narrow operands, in three steps:
//   segment sum   Z_k = I_k^T Y        over the inverse index (rowptr, perm) -- no floating-point atomics;
//   column reduce G_k = D_k^T Z_k      per-workgroup partial sums over contiguous row chunks;
//   finalize      out[col_map_k[j], :] += G_k[j, :]   partials added in a fixed order, sources in order.
// The finalize step also performs the weight update of Alg. 1 when called from the gradient-descent step.
#include <algorithm>
#include <cstring>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

// Row of Y addressed by entry p of the inverse index (or -1 to skip).
__device__ __forceinline__ int64_t seg_row(const SegArgs& a, int64_t p) {
  int64_t i = a.perm[p];
  if (a.gidx != nullptr) return a.gidx[i];
  if (a.g_rows >= 0 && i >= a.g_rows) return -1;
  return i;
}

// Narrow form: G = 2^logG lanes share one segment and stride over its entries; CT columns per lane.
// Work items [0, r_k) are whole segments (skipped when longer than kLongSeg), items [r_k, r_k + n_chunks)
// are chunks of long segments whose sums go to chunk_partial.
// (bx of gx: this workgroup's place among the workgroups that share the work)
template <int CT>
__device__ __forceinline__ void segsum_narrow_body(const SegArgs& a, int bx, int gx) {
  const int G = 1 << a.logG;
  const int lig = threadIdx.x & (G - 1);
  const int64_t n_items = a.r_k + a.n_chunks;
  const int64_t gpb = kBlock >> a.logG;
  for (int64_t item = (int64_t)bx * gpb + (threadIdx.x >> a.logG); item < n_items + gpb;
       item += (int64_t)gx * gpb) {
    // keep whole wavefronts in the loop so that the butterfly below is convergent
    bool live = item < n_items;
    int64_t beg = 0, end = 0;
    float* dst = nullptr;
    if (live) {
      if (item < a.r_k) {
        beg = a.rowptr[item];
        end = a.rowptr[item + 1];
        dst = a.Z + item * a.ldz + a.zcol0;
        if (end - beg > kLongSeg) { live = false; }
      } else {
        int c = (int)(item - a.r_k);
        beg = a.chunk_beg[c];
        end = a.chunk_end[c];
        dst = a.chunk_partial + (int64_t)c * a.ncols;
      }
    }
    float acc[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) acc[n] = 0.0f;
    if (live) {
      for (int64_t p = beg + lig; p < end; p += G) {
        int64_t r = seg_row(a, p);
        if (r >= 0) {
          const float* y = a.Y + r * a.ldy + a.col0;
#pragma unroll
          for (int n = 0; n < CT; ++n)
            if (n < a.ncols) acc[n] += y[n];
        }
      }
    }
    for (int m = G >> 1; m >= 1; m >>= 1) {
#pragma unroll
      for (int n = 0; n < CT; ++n) acc[n] += __shfl_xor(acc[n], m);
    }
    if (live && lig == 0) {
#pragma unroll
      for (int n = 0; n < CT; ++n)
        if (n < a.ncols) dst[n] = acc[n];
    }
    if (item >= n_items) break;
  }
}

template <int CT>
__global__ __launch_bounds__(kBlock) void segsum_narrow_kernel(SegArgs a) {
  segsum_narrow_body<CT>(a, blockIdx.x, gridDim.x);
}

// Wide form: W lanes of a segment each own columns lane, lane + W, ...  The lanes first load W different
// entries of the inverse index (one coalesced load), pass the row numbers around with shuffles, and then issue
// the loads of up to 16 rows of Y together; rows are added in entry order.
template <int W>
__global__ __launch_bounds__(kBlock) void segsum_wide_kernel(SegArgs a) {
  const int lig = threadIdx.x & (W - 1);
  const int64_t n_items = a.r_k + a.n_chunks;
  constexpr int64_t gpb = kBlock / W;
  for (int64_t item = (int64_t)blockIdx.x * gpb + threadIdx.x / W; item < n_items;
       item += (int64_t)gridDim.x * gpb) {
    int64_t beg, end;
    float* dst;
    if (item < a.r_k) {
      beg = a.rowptr[item];
      end = a.rowptr[item + 1];
      dst = a.Z + item * a.ldz + a.zcol0;
      if (end - beg > kLongSeg) continue;
    } else {
      int c = (int)(item - a.r_k);
      beg = a.chunk_beg[c];
      end = a.chunk_end[c];
      dst = a.chunk_partial + (int64_t)c * a.ncols;
    }
    for (int nb = 0; nb < a.ncols; nb += W) {
      const int n0 = nb + lig;
      const bool nlive = n0 < a.ncols;
      float acc = 0.0f;
      for (int64_t pb = beg; pb < end; pb += W) {
        int myrow = (pb + lig < end) ? (int)seg_row(a, pb + lig) : -1;
        const int cnt = (int)min((int64_t)W, end - pb);
#pragma unroll
        for (int e0 = 0; e0 < W; e0 += 16) {
          if (e0 >= cnt) break;
          float v[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            int r = __shfl(myrow, e0 + e, W);
            v[e] = (nlive && r >= 0) ? a.Y[(int64_t)r * a.ldy + a.col0 + n0] : 0.0f;
          }
#pragma unroll
          for (int e = 0; e < 16; ++e) acc += v[e];
        }
      }
      if (nlive) dst[n0] = acc;
    }
  }
}

// Chunks of a run of `len` entries (more than kSlLong): about kSlChunk entries each, at most eight, so that the
// thread that adds a run's chunk sums has a short chain.
__host__ __device__ __forceinline__ int sliced_chunks(int len) {
  const int n = (len + kSlChunk - 1) / kSlChunk;
  return n > 8 ? 8 : n;
}

// Plan time, step 1: the entries of a segment are in ascending order of target row, so those that fall into slice
// x of the target rows (rows [x * slice_rows, (x + 1) * slice_rows)) are a contiguous run of it; its bounds come
// from a binary search per (source row, slice).  Writes the run's length to len[x r_k + j] (slice-major) and its
// first position in perm to src_beg.
__global__ __launch_bounds__(kBlock) void slice_runs_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ perm,
                                                            int64_t r_k, int64_t slice_rows, int32_t* __restrict__ len,
                                                            int32_t* __restrict__ src_beg) {
  for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < r_k; j += (int64_t)gridDim.x * blockDim.x) {
    const int32_t e = rowptr[j + 1];
    int32_t prev = rowptr[j];
    for (int x = 0; x < kSegSlices; ++x) {
      const int64_t bound = (int64_t)(x + 1) * slice_rows;       // first entry whose target row is >= bound
      int32_t lo = prev, hi = e;
      while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if ((int64_t)perm[mid] < bound) lo = mid + 1; else hi = mid;
      }
      if (x == kSegSlices - 1) lo = e;
      len[(int64_t)x * r_k + j] = lo - prev;
      src_beg[(int64_t)x * r_k + j] = prev;
      prev = lo;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) len[(int64_t)kSegSlices * r_k] = 0;
}

// Step 3 (after the exclusive scan of the lengths): entry q of the sliced copy belongs to the run `it` with
// sl_rowptr[it] <= q < sl_rowptr[it + 1] (binary search) and is entry src_beg[it] + q - sl_rowptr[it] of perm.
__global__ __launch_bounds__(kBlock) void slice_copy_kernel(const int32_t* __restrict__ perm, const int32_t* __restrict__ sl_rowptr,
                                                            const int32_t* __restrict__ src_beg, int64_t nitems, int64_t nnz,
                                                            int32_t* __restrict__ sl_perm) {
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nnz; q += (int64_t)gridDim.x * blockDim.x) {
    int64_t lo = 0, hi = nitems;                                 // last run that starts at or before q
    while (hi - lo > 1) {
      const int64_t mid = (lo + hi) / 2;
      if ((int64_t)sl_rowptr[mid] <= q) lo = mid; else hi = mid;
    }
    sl_perm[q] = perm[(int64_t)src_beg[lo] + q - sl_rowptr[lo]];
  }
}

// Step 4: a run of more than kSlLong entries is cut into chunks, listed per slice (the list is filled through an
// integer atomic counter: the order of the runs in it does not matter, the chunks of one run are consecutive and
// every sum has a fixed order).
__global__ __launch_bounds__(kBlock) void slice_chunks_kernel(const int32_t* __restrict__ sl_rowptr, int64_t r_k,
                                                              int32_t* __restrict__ sl_chunk0, int32_t* __restrict__ ch_beg,
                                                              int32_t* __restrict__ ch_end, int32_t* __restrict__ sl_nchunk, int cap) {
  const int64_t nitems = (int64_t)kSegSlices * r_k;
  for (int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; it < nitems; it += (int64_t)gridDim.x * blockDim.x) {
    const int x = (int)(it / r_k);
    const int32_t b = sl_rowptr[it], e = sl_rowptr[it + 1];
    int32_t c0 = -1;
    if (e - b > kSlLong) {
      const int n = sliced_chunks(e - b);
      const int clen = (e - b + n - 1) / n;
      c0 = atomicAdd(&sl_nchunk[x], n);
      for (int c = 0; c < n && c0 + c < cap; ++c) {
        ch_beg[(int64_t)x * cap + c0 + c] = min(e, b + c * clen);
        ch_end[(int64_t)x * cap + c0 + c] = min(e, b + (c + 1) * clen);
      }
    }
    sl_chunk0[it] = c0;
  }
}

// Segment sums over the sliced index for narrow operands.  Workgroup b serves slice b % kSegSlices: workgroups
// are dealt to the XCDs in turn, so the operand rows a slice gathers (r_T / 8 rows: 2.5 MB of a 5-million-row
// residual) stay in the L2 of one XCD instead of crossing the fabric once per index entry.  Lane groups of
// 2^sl_logG lanes take the (slice, source row) runs of at most kSlLong entries; the chunks of the longer runs are
// summed by whole workgroups (thread t adds the entries t, t + 256, ..., then a fixed tree over the threads).
// (bid of nblocks workgroups, nblocks a multiple of kSegSlices: several sources may share a launch.)
template <int CT>
__device__ __forceinline__ void segsum_sliced_body(const SegArgs& a, float (*red)[kBlock], int bid, int nblocks) {
  const int x = bid % kSegSlices, bi = bid / kSegSlices, nb = nblocks / kSegSlices;
  const int G = 1 << a.sl_logG;
  const int lig = threadIdx.x & (G - 1);
  const int64_t gpb = kBlock >> a.sl_logG;
  const int32_t* rp_x = a.sl_rowptr + (int64_t)x * a.r_k;
  float* Zx = a.Zs + (int64_t)x * a.r_k * CT;
  for (int64_t base = (int64_t)bi * gpb; base < a.r_k; base += (int64_t)nb * gpb) {   // same trip count for all threads
    const int64_t j = base + (threadIdx.x >> a.sl_logG);
    bool live = j < a.r_k;
    int32_t beg = 0, end = 0;
    if (live) {
      beg = rp_x[j]; end = rp_x[j + 1];
      if (end - beg > kSlLong) live = false;
    }
    float acc[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) acc[n] = 0.0f;
    if (live) {
      // four entries of the lane in flight: first their target rows, then the operand rows
      for (int64_t p = beg + lig; p < end; p += 4 * G) {
        int64_t r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) r[u] = p + u * G < end ? (int64_t)a.sl_perm[p + u * G] : -1;
        float y[4][CT];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int n = 0; n < CT; ++n) y[u][n] = (r[u] >= 0 && n < a.ncols) ? a.Y[r[u] * a.ldy + a.col0 + n] : 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int n = 0; n < CT; ++n) acc[n] += y[u][n];
      }
    }
    for (int m = G >> 1; m >= 1; m >>= 1) {
#pragma unroll
      for (int n = 0; n < CT; ++n) acc[n] += __shfl_xor(acc[n], m);
    }
    if (live && lig == 0) {
#pragma unroll
      for (int n = 0; n < CT; ++n) Zx[j * CT + n] = acc[n];
    }
  }
  // chunks of the long runs of this slice
  const int nchunk = min(a.sl_nchunk[x], a.sl_cap);
  for (int q = bi; q < nchunk; q += nb) {
    const int32_t beg = a.sl_ch_beg[(int64_t)x * a.sl_cap + q], end = a.sl_ch_end[(int64_t)x * a.sl_cap + q];
    float acc[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) acc[n] = 0.0f;
    for (int64_t p = beg + threadIdx.x; p < end; p += 4 * kBlock) {
      int64_t r[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) r[u] = p + u * kBlock < end ? (int64_t)a.sl_perm[p + u * kBlock] : -1;
      float y[4][CT];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int n = 0; n < CT; ++n) y[u][n] = (r[u] >= 0 && n < a.ncols) ? a.Y[r[u] * a.ldy + a.col0 + n] : 0.0f;
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int n = 0; n < CT; ++n) acc[n] += y[u][n];
    }
    __syncthreads();
#pragma unroll
    for (int n = 0; n < CT; ++n) red[n][threadIdx.x] = acc[n];
    __syncthreads();
    for (int w = kBlock / 2; w >= 1; w >>= 1) {
      if ((int)threadIdx.x < w) {
#pragma unroll
        for (int n = 0; n < CT; ++n) red[n][threadIdx.x] += red[n][threadIdx.x + w];
      }
      __syncthreads();
    }
    if ((int)threadIdx.x < CT) a.sl_ch_partial[((int64_t)x * a.sl_cap + q) * CT + threadIdx.x] = red[threadIdx.x][0];
  }
}

// The sliced segment sums of up to kSegMulti sources in one launch: workgroups [first[q], first[q + 1]) serve source
// q; every first[q] is a multiple of kSegSlices, so workgroup b still gathers from slice b % kSegSlices and the
// sources that run side by side on an XCD share its slice of the operand in L2.
template <int CT>
__global__ __launch_bounds__(kBlock) void segsum_sliced_kernel(SegMulti m) {
  __shared__ float red[CT][kBlock];
  int q = 0;
  while (q + 1 < m.n && (int)blockIdx.x >= m.first[q + 1]) ++q;
  segsum_sliced_body<CT>(m.s[q], red, (int)blockIdx.x - m.first[q], m.first[q + 1] - m.first[q]);
}

// Z[j, :] = the per-slice sums of source row j added in slice order; a long run's sum is its chunks added in order.
template <int CT>
__device__ __forceinline__ void segsum_sliced_combine_body(const SegArgs& a, int bid, int nblocks) {
  for (int64_t j = (int64_t)bid * blockDim.x + threadIdx.x; j < a.r_k; j += (int64_t)nblocks * blockDim.x) {
    int c0[kSegSlices];
    float v[kSegSlices][CT];
#pragma unroll
    for (int x = 0; x < kSegSlices; ++x) {                       // all slices requested together
      const int64_t it = (int64_t)x * a.r_k + j;
      c0[x] = a.sl_chunk0[it];
#pragma unroll
      for (int n = 0; n < CT; ++n) v[x][n] = a.Zs[it * CT + n];
    }
    float z[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) z[n] = 0.0f;
#pragma unroll
    for (int x = 0; x < kSegSlices; ++x) {
      if (c0[x] >= 0) {
        const int64_t it = (int64_t)x * a.r_k + j;
        const int nch = sliced_chunks(a.sl_rowptr[it + 1] - a.sl_rowptr[it]);
        float cp[8][CT];
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
          for (int n = 0; n < CT; ++n)
            cp[c][n] = c < nch ? a.sl_ch_partial[((int64_t)x * a.sl_cap + c0[x] + c) * CT + n] : 0.0f;
#pragma unroll
        for (int n = 0; n < CT; ++n) {
          float s = 0.0f;
#pragma unroll
          for (int c = 0; c < 8; ++c) s += cp[c][n];
          v[x][n] = s;
        }
      }
#pragma unroll
      for (int n = 0; n < CT; ++n) z[n] += v[x][n];
    }
#pragma unroll
    for (int n = 0; n < CT; ++n)
      if (n < a.ncols) a.Z[j * a.ldz + a.zcol0 + n] = z[n];
  }
}

template <int CT>
__global__ __launch_bounds__(kBlock) void segsum_sliced_combine_kernel(SegMulti m) {
  int q = 0;
  while (q + 1 < m.n && (int)blockIdx.x >= m.cfirst[q + 1]) ++q;
  segsum_sliced_combine_body<CT>(m.s[q], (int)blockIdx.x - m.cfirst[q], m.cfirst[q + 1] - m.cfirst[q]);
}

// Long segments: add the chunk sums in chunk order.
__global__ __launch_bounds__(kBlock) void segsum_combine_kernel(SegArgs a) {
  int64_t total = (int64_t)a.n_long * a.ncols;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
       e += (int64_t)gridDim.x * blockDim.x) {
    int s = (int)(e / a.ncols), n = (int)(e % a.ncols);
    float acc = 0.0f;
    for (int c = a.long_first[s]; c < a.long_first[s + 1]; ++c) acc += a.chunk_partial[(int64_t)c * a.ncols + n];
    a.Z[(int64_t)a.long_seg[s] * a.ldz + a.zcol0 + n] = acc;
  }
}

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

constexpr int kUnroll = 8;   // rows (float4 loads) a lane has in flight

// Partial of D^T Z over the rows [b0, b1) of one workgroup, added to the per-thread sums g.  `by` selects a slab
// of 64*VEC columns of D; inside a slab lane -> (row offset, column group), so a wavefront reads whole contiguous
// rows.  ZLDS: the operand rows come from an LDS tile (row r at zl[(r - zl_row0) * CT]) instead of a.Z.
template <int VEC, int CT, bool ZLDS>
__device__ __forceinline__ void colred_rows(const ColredArgs& a, int by, int64_t b0, int64_t b1, const float* zl,
                                            int64_t zl_row0, float (&g)[VEC][CT]) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int slab0 = by * kWave * VEC;                               // first column of the slab
  const int wck = min(a.ck - slab0, kWave * VEC);                   // its width
  const int nvec = wck / VEC;                                       // column groups (<= 64)
  const int rp = kWave / nvec;                                      // rows per wavefront step
  const int rsub = lane / nvec, cg = lane - rsub * nvec;
  if (rsub >= rp) return;
  const int64_t step = (int64_t)rp * kUnroll;                       // rows per wavefront iteration
  for (int64_t r0 = b0 + (int64_t)wave * step; r0 < b1; r0 += (int64_t)(kBlock / kWave) * step) {
    float v[kUnroll][VEC], z[kUnroll][CT];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      int64_t r = r0 + (int64_t)u * rp + rsub;
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[u][e] = 0.0f;
#pragma unroll
      for (int n = 0; n < CT; ++n) z[u][n] = 0.0f;
      if (r < b1) {
        load_vec<VEC>(a.D + r * a.ck + slab0 + cg * VEC, v[u]);
        if constexpr (ZLDS) {
          const float* zp = zl + (r - zl_row0) * CT;
#pragma unroll
          for (int n = 0; n < CT; ++n) z[u][n] = zp[n];
        } else {
          const float* zp = a.Z + r * a.ldz + a.col0;
#pragma unroll
          for (int n = 0; n < CT; ++n)
            if (n < a.ncols) z[u][n] = zp[n];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
#pragma unroll
      for (int e = 0; e < VEC; ++e)
#pragma unroll
        for (int n = 0; n < CT; ++n) g[e][n] = fmaf(v[u][e], z[u][n], g[e][n]);
  }
}

// The workgroup's per-thread sums added in a fixed order (wavefronts, then row offsets) and stored as its partial.
template <int VEC, int CT>
__device__ __forceinline__ void colred_store(const ColredArgs& a, int bx, int by, const float (&g)[VEC][CT],
                                             float (*red)[kBlock]) {
  const int tid = threadIdx.x;
  const int slab0 = by * kWave * VEC;
  const int wck = min(a.ck - slab0, kWave * VEC);
  const int nvec = wck / VEC;
  const int rp = kWave / nvec;
#pragma unroll
  for (int e = 0; e < VEC; ++e)
#pragma unroll
    for (int n = 0; n < CT; ++n) red[e * CT + n][tid] = g[e][n];
  __syncthreads();
  // column j of the slab, operand column n
  for (int o = tid; o < wck * CT; o += kBlock) {
    int j = o / CT, n = o - j * CT;
    int jcg = j / VEC, e = j - jcg * VEC;
    float s = 0.0f;
    for (int w = 0; w < kBlock / kWave; ++w)
      for (int q = 0; q < rp; ++q) s += red[e * CT + n][w * kWave + q * nvec + jcg];
    a.partial[((int64_t)bx * a.ck + slab0 + j) * kNarrowCT + n] = s;
  }
}

template <int VEC, int CT>
__device__ __forceinline__ void colred_body(const ColredArgs& a, int bx, int by) {
  __shared__ float red[VEC * CT][kBlock];
  const int64_t b0 = (int64_t)bx * a.rows_per_block;
  const int64_t b1 = min(b0 + a.rows_per_block, a.rows);
  float g[VEC][CT];
#pragma unroll
  for (int e = 0; e < VEC; ++e)
#pragma unroll
    for (int n = 0; n < CT; ++n) g[e][n] = 0.0f;
  colred_rows<VEC, CT, false>(a, by, b0, b1, nullptr, 0, g);
  colred_store<VEC, CT>(a, bx, by, g, red);
}

constexpr int kJoinRows = kBlock;    // rows of a joined table whose segment sums a workgroup forms at a time (one per thread)
constexpr int kJoinTileFloats = 2048;  // LDS floats for the gathered operand rows of one tile of index entries

// Join-order form for a joined source: the segment sums Z = I_k^T Y of up to kJoinRows rows are formed in LDS and
// multiplied right away; Z is never written to memory and the table is the only stream.  The operand rows of a
// tile of consecutive index entries are gathered with all their loads in flight (entry -> target row -> operand
// row: two dependent round trips per tile, whatever the number of rows), then the thread of each table row adds
// its entries in index order.  Needs a table without long segments (s.n_long == 0) and a single column slab.
template <int VEC, int CT>
__device__ __forceinline__ void colred_join_body(const ColredArgs& a, const SegArgs& s, int bx) {
  constexpr int kTile = kJoinTileFloats / CT;          // index entries per tile
  constexpr int kPer = kTile / kBlock;                 // ... per thread
  __shared__ float red[VEC * CT][kBlock];
  __shared__ float zs[kJoinRows * CT];
  __shared__ float ys[kTile * CT];
  __shared__ int rps[kJoinRows + 1];
  const int tid = threadIdx.x;
  const int64_t b0 = s.block_first[bx], b1 = s.block_first[bx + 1];   // balanced by table bytes + index entries
  float g[VEC][CT];
#pragma unroll
  for (int e = 0; e < VEC; ++e)
#pragma unroll
    for (int n = 0; n < CT; ++n) g[e][n] = 0.0f;
  for (int64_t s0 = b0; s0 < b1; s0 += kJoinRows) {
    const int64_t s1 = min(s0 + kJoinRows, b1);
    const int nrows = (int)(s1 - s0);
    for (int j = tid; j <= nrows; j += kBlock) rps[j] = s.rowptr[s0 + j];
    __syncthreads();
    const int pb = rps[0], pe = rps[nrows];
    const int my_beg = tid < nrows ? rps[tid] : 0, my_end = tid < nrows ? rps[tid + 1] : 0;
    float acc[CT];
#pragma unroll
    for (int n = 0; n < CT; ++n) acc[n] = 0.0f;
    for (int t0 = pb; t0 < pe; t0 += kTile) {
      const int t1 = min(t0 + kTile, pe);
      int64_t rr[kPer];
#pragma unroll
      for (int u = 0; u < kPer; ++u) {
        const int p = t0 + tid + u * kBlock;
        rr[u] = p < t1 ? seg_row(s, p) : -1;
      }
      float yv[kPer][CT];
#pragma unroll
      for (int u = 0; u < kPer; ++u)
#pragma unroll
        for (int n = 0; n < CT; ++n)
          yv[u][n] = (rr[u] >= 0 && n < s.ncols) ? s.Y[rr[u] * s.ldy + s.col0 + n] : 0.0f;
#pragma unroll
      for (int u = 0; u < kPer; ++u)
#pragma unroll
        for (int n = 0; n < CT; ++n) ys[(tid + u * kBlock) * CT + n] = yv[u][n];
      __syncthreads();
      const int lo = max(my_beg, t0), hi = min(my_end, t1);
      for (int p = lo; p < hi; ++p) {
#pragma unroll
        for (int n = 0; n < CT; ++n) acc[n] += ys[(p - t0) * CT + n];
      }
      __syncthreads();
    }
    if (tid < nrows) {
#pragma unroll
      for (int n = 0; n < CT; ++n) zs[tid * CT + n] = acc[n];
    }
    __syncthreads();
    colred_rows<VEC, CT, true>(a, 0, s0, s1, zs, s0, g);
    __syncthreads();                                              // zs and rps are rewritten by the next round
  }
  colred_store<VEC, CT>(a, bx, 0, g, red);
}

template <int VEC, int CT>
__global__ __launch_bounds__(kBlock) void colred_kernel(ColredArgs a) {
  colred_body<VEC, CT>(a, blockIdx.x, blockIdx.y);
}

// Every share of a narrow transposed multiply in one launch: up to kTmmParts sources, each either a column
// reduce that takes its operand rows from memory (an identity source: Z = Y) or the join-order form above.  The
// shares are independent; consecutive workgroup ranges serve consecutive parts.
template <int CT>
__global__ __launch_bounds__(kBlock) void tmm_parts_kernel(TmmParts t) {
  int part = 0;
#pragma unroll
  for (int q = 1; q < kTmmParts; ++q) part += (q < t.n && (int)blockIdx.x >= t.first[q]) ? 1 : 0;
  const int bx = (int)blockIdx.x - t.first[part];
  if (t.join[part]) colred_join_body<4, CT>(t.c[part], t.s[part], bx);
  else colred_body<4, CT>(t.c[part], bx, 0);
}

// Sum of float4 records rec[b * stride4] over b < count by a whole workgroup: threads stride the records
// (four independent loads in flight each), xor butterfly inside the wavefronts, wavefronts added in order.
__device__ __forceinline__ float4 block_sum4(const float4* __restrict__ rec, int64_t stride4, int count,
                                             float (*scratch)[4]) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0, s2 = s0, s3 = s0;
  int b = tid;
  for (; b + 3 * kBlock < count; b += 4 * kBlock) {
    float4 v0 = rec[(int64_t)b * stride4], v1 = rec[(int64_t)(b + kBlock) * stride4];
    float4 v2 = rec[(int64_t)(b + 2 * kBlock) * stride4], v3 = rec[(int64_t)(b + 3 * kBlock) * stride4];
    s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
    s1.x += v1.x; s1.y += v1.y; s1.z += v1.z; s1.w += v1.w;
    s2.x += v2.x; s2.y += v2.y; s2.z += v2.z; s2.w += v2.w;
    s3.x += v3.x; s3.y += v3.y; s3.z += v3.z; s3.w += v3.w;
  }
  for (; b < count; b += kBlock) {
    float4 v0 = rec[(int64_t)b * stride4];
    s0.x += v0.x; s0.y += v0.y; s0.z += v0.z; s0.w += v0.w;
  }
  float r[4] = {(s0.x + s1.x) + (s2.x + s3.x), (s0.y + s1.y) + (s2.y + s3.y), (s0.z + s1.z) + (s2.z + s3.z),
                (s0.w + s1.w) + (s2.w + s3.w)};
#pragma unroll
  for (int n = 0; n < 4; ++n)
    for (int m = kWave / 2; m >= 1; m >>= 1) r[n] += __shfl_xor(r[n], m);
  __syncthreads();   // scratch may still be read from a previous call
  if (lane == 0) {
#pragma unroll
    for (int n = 0; n < 4; ++n) scratch[wave][n] = r[n];
  }
  __syncthreads();
  float4 out;
  out.x = ((scratch[0][0] + scratch[1][0]) + scratch[2][0]) + scratch[3][0];
  out.y = ((scratch[0][1] + scratch[1][1]) + scratch[2][1]) + scratch[3][1];
  out.z = ((scratch[0][2] + scratch[1][2]) + scratch[2][2]) + scratch[3][2];
  out.w = ((scratch[0][3] + scratch[1][3]) + scratch[2][3]) + scratch[3][3];
  return out;
}

// One workgroup per target column: sum each contributing source's per-workgroup partials (records of
// kNarrowCT floats), add the sources in order.  MODE 0 stores, MODE 1 applies  W -= lr * G / r_T  and, in
// one extra workgroup, reduces the loss partials (Alg. 1).
template <int MODE>
__global__ __launch_bounds__(kBlock) void finalize_kernel(FinArgs a, int c_T) {
  static_assert(kNarrowCT == 4, "records are float4");
  __shared__ float scratch[kBlock / kWave][4];
  const int t = blockIdx.x;
  if (t == c_T) {
    if constexpr (MODE == 1) {
      float4 s = block_sum4(reinterpret_cast<const float4*>(a.loss_partial), 1, a.n_loss_partial, scratch);
      float sv[4] = {s.x, s.y, s.z, s.w};
      if ((int)threadIdx.x < a.ncols) a.loss[a.col0 + threadIdx.x] = sv[threadIdx.x] * a.loss_scale;
    }
    return;
  }
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int k = 0; k < a.n; ++k) {
    int j = a.s[k].tcol2src[t];
    if (j < 0) continue;
    float4 s = block_sum4(reinterpret_cast<const float4*>(a.s[k].partial) + j, a.s[k].ck, a.s[k].nblocks, scratch);
    acc[0] += s.x; acc[1] += s.y; acc[2] += s.z; acc[3] += s.w;
  }
  if ((int)threadIdx.x < a.ncols) {
    const int n = threadIdx.x;
    float* o = a.out + (int64_t)t * a.ldo + a.col0 + n;
    if constexpr (MODE == 0) *o = acc[n];
    else *o = *o - a.lr[a.col0 + n] * (acc[n] * a.inv_rT);
  }
}

}  // namespace

hipError_t launch_segsum(const SegArgs& a, hipStream_t st) {
  int64_t n_items = a.r_k + a.n_chunks;
  if (n_items <= 0 || a.ncols <= 0) return hipSuccess;
  if (a.ncols <= kNarrowCT) {
    int64_t gpb = kBlock >> a.logG;
    int64_t grid = (n_items + gpb - 1) / gpb;
    if (grid > 65536) grid = 65536;
    if (a.ncols == 1) segsum_narrow_kernel<1><<<(int)grid, kBlock, 0, st>>>(a);
    else if (a.ncols == 2) segsum_narrow_kernel<2><<<(int)grid, kBlock, 0, st>>>(a);
    else segsum_narrow_kernel<4><<<(int)grid, kBlock, 0, st>>>(a);
  } else {
    int W = a.ncols <= 16 ? 16 : (a.ncols <= 32 ? 32 : 64);
    int64_t gpb = kBlock / W;
    int64_t grid = (n_items + gpb - 1) / gpb;
    if (grid > 65536) grid = 65536;
    if (W == 16) segsum_wide_kernel<16><<<(int)grid, kBlock, 0, st>>>(a);
    else if (W == 32) segsum_wide_kernel<32><<<(int)grid, kBlock, 0, st>>>(a);
    else segsum_wide_kernel<64><<<(int)grid, kBlock, 0, st>>>(a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.n_long > 0) {
    int64_t total = (int64_t)a.n_long * a.ncols;
    int grid = (int)((total + kBlock - 1) / kBlock);
    if (grid > 1024) grid = 1024;
    segsum_combine_kernel<<<grid, kBlock, 0, st>>>(a);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_build_sliced_index(const int32_t* rowptr, const int32_t* perm, int64_t r_k, int64_t nnz, int64_t slice_rows,
                                     int32_t* sl_rowptr, int32_t* sl_perm, int32_t* sl_chunk0, int32_t* ch_beg, int32_t* ch_end,
                                     int32_t* sl_nchunk, int cap, int32_t* src_beg, int32_t* scan_scratch, hipStream_t st) {
  if (r_k <= 0) return hipSuccess;
  const int64_t nitems = (int64_t)kSegSlices * r_k;
  int grid = (int)std::min<int64_t>((r_k + kBlock - 1) / kBlock, 4096);
  slice_runs_kernel<<<grid, kBlock, 0, st>>>(rowptr, perm, r_k, slice_rows, sl_rowptr, src_beg);
  launch_exclusive_scan(sl_rowptr, nitems + 1, scan_scratch, st);
  if (nnz > 0) {
    grid = (int)std::min<int64_t>((nnz + kBlock - 1) / kBlock, 8192);
    slice_copy_kernel<<<grid, kBlock, 0, st>>>(perm, sl_rowptr, src_beg, nitems, nnz, sl_perm);
  }
  grid = (int)std::min<int64_t>((nitems + kBlock - 1) / kBlock, 4096);
  slice_chunks_kernel<<<grid, kBlock, 0, st>>>(sl_rowptr, r_k, sl_chunk0, ch_beg, ch_end, sl_nchunk, cap);
  return hipGetLastError();
}

// Chunk records a slice needs at most for an index of nnz entries.
int64_t segsum_sliced_chunk_cap(int64_t nnz) { return nnz / kSlLong + 1; }

hipError_t launch_segsum_sliced(const SegArgs* a, int n, hipStream_t st) {
  if (n < 1 || n > kSegMulti) return hipErrorInvalidValue;
  SegMulti m;
  memset(&m, 0, sizeof(m));
  m.n = n;
  for (int q = 0; q < n; ++q) {
    if (a[q].sl_perm == nullptr || a[q].ncols < 1 || a[q].ncols > kNarrowCT || a[q].ncols != a[0].ncols || a[q].r_k <= 0)
      return hipErrorInvalidValue;
    const int64_t gpb = kBlock >> a[q].sl_logG;
    int64_t nb = (a[q].r_k + gpb - 1) / gpb;               // workgroups per slice
    nb = std::min<int64_t>(std::max<int64_t>(nb, 64), 2048);
    int cgrid = (int)((a[q].r_k + kBlock - 1) / kBlock);
    if (cgrid > 2048) cgrid = 2048;
    m.s[q] = a[q];
    m.first[q + 1] = m.first[q] + (int)(nb * kSegSlices);
    m.cfirst[q + 1] = m.cfirst[q] + cgrid;
  }
  const unsigned grid = (unsigned)m.first[n], cgrid = (unsigned)m.cfirst[n];
  if (a[0].ncols == 1) {
    segsum_sliced_kernel<1><<<grid, kBlock, 0, st>>>(m);
    segsum_sliced_combine_kernel<1><<<cgrid, kBlock, 0, st>>>(m);
  } else if (a[0].ncols == 2) {
    segsum_sliced_kernel<2><<<grid, kBlock, 0, st>>>(m);
    segsum_sliced_combine_kernel<2><<<cgrid, kBlock, 0, st>>>(m);
  } else {
    segsum_sliced_kernel<4><<<grid, kBlock, 0, st>>>(m);
    segsum_sliced_combine_kernel<4><<<cgrid, kBlock, 0, st>>>(m);
  }
  return hipGetLastError();
}

hipError_t launch_colred(const ColredArgs& a, int nblocks, hipStream_t st) {
  if (a.ck <= 0 || nblocks <= 0) return hipSuccess;
  int slabw = kWave * a.vec;
  dim3 grid(nblocks, (a.ck + slabw - 1) / slabw);
  int ct = a.ncols <= 1 ? 1 : (a.ncols <= 2 ? 2 : 4);
#define ILARGI_COLRED(V, C) colred_kernel<V, C><<<grid, kBlock, 0, st>>>(a)
  if (a.vec == 4) { if (ct == 1) ILARGI_COLRED(4, 1); else if (ct == 2) ILARGI_COLRED(4, 2); else ILARGI_COLRED(4, 4); }
  else if (a.vec == 2) { if (ct == 1) ILARGI_COLRED(2, 1); else if (ct == 2) ILARGI_COLRED(2, 2); else ILARGI_COLRED(2, 4); }
  else { if (ct == 1) ILARGI_COLRED(1, 1); else if (ct == 2) ILARGI_COLRED(1, 2); else ILARGI_COLRED(1, 4); }
#undef ILARGI_COLRED
  return hipGetLastError();
}

hipError_t launch_finalize(const FinArgs& a, int c_T, int mode, hipStream_t st) {
  if (c_T <= 0 || a.ncols <= 0) return hipSuccess;
  if (mode == 0) finalize_kernel<0><<<c_T, kBlock, 0, st>>>(a, c_T);
  else finalize_kernel<1><<<c_T + (a.loss != nullptr ? 1 : 0), kBlock, 0, st>>>(a, c_T);
  return hipGetLastError();
}

// Rows one workgroup iteration of the column reduce covers for a table with ck columns read in groups of vec.
int colred_step_rows(int ck, int vec) {
  const int wck = std::min(ck, kWave * vec);
  const int nvec = std::max(1, wck / vec);
  return std::max(1, kWave / nvec) * kUnroll * (kBlock / kWave);
}

// A part of the merged launch: float4 rows, one column slab, and for the join-order form no long segments.
bool tmm_part_supported(const ColredArgs& c, const SegArgs* s) {
  if (c.vec != 4 || c.ck <= 0 || c.ck > kWave * 4 || c.ncols < 1 || c.ncols > kNarrowCT || c.rows <= 0) return false;
  if (s != nullptr && (s->n_long != 0 || s->ncols != c.ncols || s->r_k != c.rows || s->block_first == nullptr)) return false;
  return true;
}

hipError_t launch_tmm_parts(const TmmParts& t, hipStream_t st) {
  if (t.n < 1 || t.n > kTmmParts) return hipErrorInvalidValue;
  const int grid = t.first[t.n];
  if (grid <= 0) return hipSuccess;
  const int nc = t.c[0].ncols;
  if (nc <= 1) tmm_parts_kernel<1><<<grid, kBlock, 0, st>>>(t);
  else if (nc == 2) tmm_parts_kernel<2><<<grid, kBlock, 0, st>>>(t);
  else tmm_parts_kernel<4><<<grid, kBlock, 0, st>>>(t);
  return hipGetLastError();
}

}  // namespace ilargi
