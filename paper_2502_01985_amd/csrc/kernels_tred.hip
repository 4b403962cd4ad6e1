// Transposed reduction on the matrix cores:  C = sum_t w_t a_t^T b_t  where a_t, b_t are rows of two
// row-major float32 matrices (optionally addressed through index vectors) and t runs over a long row range.
// This one contraction serves
//   * the column reduce  G_k = D_k^T Z_k  of the transposed multiply when the operand has >= 8 columns
//     (a = D_k, b = Z_k), including the batched gradient of Alg. 1 for many models, and
//   * every block of the Gram matrix T^T T (a, b = tables or summed tables, w = fan-out counts).
//
// MFMA 16x16x4 (float32): the 16 "M" rows are table columns, the 16 "N" columns operand columns, the 4 "K"
// slots are rows t.  Lane l = 16 q + s loads the float4  a[t0 + q][j0 + 4 s .. 4 s + 3]  (a wavefront load covers
// 4 whole rows x 64 contiguous columns, fully coalesced) and feeds its four components to four MFMAs whose
// M index s stands for table column  j0 + 4 s + e.  The B operand of lane l is  b[t0 + q][n0 + s].
//
// Each wavefront owns a share of the rows and the full output tile; wavefronts and workgroups are combined
// afterwards in a fixed order, so results are reproducible.
#include <algorithm>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kU = 4;  // row quads in flight per wavefront

// Row chunk bx and output tile by of this workgroup.  The launch is one-dimensional and workgroup ids go round-robin
// over the 8 XCDs (each with an L2 of its own): the gy tiles of one row chunk get ids that are 8 apart, so they run
// on the same XCD at about the same time and the chunk's rows of both matrices come from memory once instead of
// once per tile.
__device__ __forceinline__ bool tred_block_ids(const TredArgs& a, int& bx, int& by) {
  const int64_t grp = blockIdx.x / (8 * a.gy);
  const int within = (int)(blockIdx.x - grp * (8 * a.gy));
  bx = (int)(grp * 8 + within % 8);
  by = within / 8;
  return bx < a.gx;
}

// JT: 64-column tiles of A per workgroup tile, NT: 16-column tiles of B.  JT * NT <= 4.
template <int JT, int NT, bool VEC4>
__global__ __launch_bounds__(kBlock) void tred_kernel(TredArgs a) {
  __shared__ float red[JT * 64 * NT * 16];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int s = lane % 16, q = lane / 16;
  const int nb_slabs = (a.cb + NT * 16 - 1) / (NT * 16);
  int bx, by;
  if (!tred_block_ids(a, bx, by)) return;
  const int a_slab = by / nb_slabs, b_slab = by - a_slab * nb_slabs;
  const int j0 = a_slab * JT * 64, n0 = b_slab * NT * 16;
  const int64_t t_lo = (int64_t)bx * a.rows_per_block;
  const int64_t t_hi = min(t_lo + a.rows_per_block, a.n_rows);
  // symmetric result: tiles entirely below the diagonal are never read by the caller
  if (a.upper_only && j0 >= n0 + NT * 16) return;

  v4f acc[JT][4][NT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt)
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[jt][e][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  // which of this lane's column groups / operand columns exist
  bool jok[JT], nok[NT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) jok[jt] = j0 + jt * 64 + 4 * s < a.ca;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) nok[nt] = n0 + nt * 16 + s < a.cb;

  for (int64_t base = t_lo + (int64_t)wave * (4 * kU); base < t_hi; base += (int64_t)(kBlock / kWave) * (4 * kU)) {
    float av[kU][JT][4];
    float bv[kU][NT];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      int64_t t = base + u * 4 + q;
      int64_t ra = -1, rb = -1;
      float w = 1.0f;
      if (t < t_hi) {
        ra = a.ia ? (int64_t)a.ia[t] : (t < a.a_rows ? t : -1);
        rb = a.ib ? (int64_t)a.ib[t] : (t < a.b_rows ? t : -1);
        if (a.wptr) w = (float)(a.wptr[t + 1] - a.wptr[t]);
      }
      const bool live = ra >= 0 && rb >= 0;
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) av[u][jt][e] = 0.0f;
        if (live && jok[jt]) {
          const float* p = a.A + ra * a.lda + j0 + jt * 64 + 4 * s;
          if constexpr (VEC4) {
            float4 v = *reinterpret_cast<const float4*>(p);
            av[u][jt][0] = v.x; av[u][jt][1] = v.y; av[u][jt][2] = v.z; av[u][jt][3] = v.w;
          } else {
            const int left = a.ca - (j0 + jt * 64 + 4 * s);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (e < left) av[u][jt][e] = p[e];
          }
          if (a.wptr) {
#pragma unroll
            for (int e = 0; e < 4; ++e) av[u][jt][e] *= w;
          }
        }
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bv[u][nt] = (live && nok[nt]) ? a.B[rb * a.ldb + a.bcol0 + n0 + nt * 16 + s] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
      for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[jt][e][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][jt][e], bv[u][nt], acc[jt][e][nt], 0, 0, 0);
  }

  // combine the four wavefronts in order; red is [JT*64][NT*16]
  for (int w = 0; w < kBlock / kWave; ++w) {
    if (wave == w) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              int j = jt * 64 + 4 * (4 * q + r) + e;
              int n = nt * 16 + s;
              float v = acc[jt][e][nt][r];
              if (w == 0) red[j * (NT * 16) + n] = v;
              else red[j * (NT * 16) + n] += v;
            }
    }
    __syncthreads();
  }
  float* out = a.partial + (int64_t)bx * a.ca * a.cb;
  for (int o = tid; o < JT * 64 * NT * 16; o += kBlock) {
    int j = o / (NT * 16), n = o - j * (NT * 16);
    if (j0 + j < a.ca && n0 + n < a.cb) out[(int64_t)(j0 + j) * a.cb + n0 + n] = red[o];
  }
}

// bfloat16-input form (MFMA 16x16x32, float32 sums): both factors are rounded to bfloat16, nearest even, as
// they enter the MFMA.  Lane 16 q + s loads the float4  a[t0 + 8 q + u][j0 + 4 s ..]  for u = 0..7; component e
// of the eight loads forms the A operand of MFMA e (K slots = rows t0 + 8 q + u).  One 64-column tile of A.
template <int NT, bool VEC4>
__global__ __launch_bounds__(kBlock) void tred_bf16_kernel(TredArgs a) {
  __shared__ float red[64 * NT * 16];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int s = lane % 16, q = lane / 16;
  const int nb_slabs = (a.cb + NT * 16 - 1) / (NT * 16);
  int bx, by;
  if (!tred_block_ids(a, bx, by)) return;
  const int a_slab = by / nb_slabs, b_slab = by - a_slab * nb_slabs;
  const int j0 = a_slab * 64, n0 = b_slab * NT * 16;
  const int64_t t_lo = (int64_t)bx * a.rows_per_block;
  const int64_t t_hi = min(t_lo + a.rows_per_block, a.n_rows);
  v4f acc[4][NT];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[e][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
  const bool jok = j0 + 4 * s < a.ca;
  bool nok[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) nok[nt] = n0 + nt * 16 + s < a.cb;

  for (int64_t base = t_lo + (int64_t)wave * 32; base < t_hi; base += (int64_t)(kBlock / kWave) * 32) {
    float av[8][4], bv[8][NT];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      int64_t t = base + 8 * q + u;
      int64_t ra = -1, rb = -1;
      float w = 1.0f;
      if (t < t_hi) {
        ra = a.ia ? (int64_t)a.ia[t] : (t < a.a_rows ? t : -1);
        rb = a.ib ? (int64_t)a.ib[t] : (t < a.b_rows ? t : -1);
        if (a.wptr) w = (float)(a.wptr[t + 1] - a.wptr[t]);
      }
      const bool live = ra >= 0 && rb >= 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) av[u][e] = 0.0f;
      if (live && jok) {
        const float* p = a.A + ra * a.lda + j0 + 4 * s;
        if constexpr (VEC4) {
          float4 v = *reinterpret_cast<const float4*>(p);
          av[u][0] = v.x; av[u][1] = v.y; av[u][2] = v.z; av[u][3] = v.w;
        } else {
          const int left = a.ca - (j0 + 4 * s);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (e < left) av[u][e] = p[e];
        }
        if (a.wptr) {
#pragma unroll
          for (int e = 0; e < 4; ++e) av[u][e] *= w;
        }
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bv[u][nt] = (live && nok[nt]) ? a.B[rb * a.ldb + a.bcol0 + n0 + nt * 16 + s] : 0.0f;
    }
    bf16x8 bp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int u = 0; u < 8; ++u) bp[nt][u] = (__bf16)bv[u][nt];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      bf16x8 ap;
#pragma unroll
      for (int u = 0; u < 8; ++u) ap[u] = (__bf16)av[u][e];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[e][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, bp[nt], acc[e][nt], 0, 0, 0);
    }
  }
  for (int w = 0; w < kBlock / kWave; ++w) {
    if (wave == w) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            int j = 4 * (4 * q + r) + e, n = nt * 16 + s;
            float v = acc[e][nt][r];
            if (w == 0) red[j * (NT * 16) + n] = v;
            else red[j * (NT * 16) + n] += v;
          }
    }
    __syncthreads();
  }
  float* out = a.partial + (int64_t)bx * a.ca * a.cb;
  for (int o = tid; o < 64 * NT * 16; o += kBlock) {
    int j = o / (NT * 16), n = o - j * (NT * 16);
    if (j0 + j < a.ca && n0 + n < a.cb) out[(int64_t)(j0 + j) * a.cb + n0 + n] = red[o];
  }
}

// Form for a wide A against at most 32 columns of B, both addressed directly: the four wavefronts of a workgroup
// take four neighbouring 64-column slabs of A over ALL rows of the chunk (B's few columns are read by each of
// them), so nothing has to be combined through LDS and a chunk leaves one partial result instead of four shares.
template <int NT>
__global__ __launch_bounds__(kBlock) void tred_cs_kernel(TredArgs a) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int s = lane % 16, q = lane / 16;
  int bx, by;
  if (!tred_block_ids(a, bx, by)) return;
  const int j0 = (by * (kBlock / kWave) + wave) * 64;
  if (j0 >= a.ca) return;                                       // (no workgroup barrier below)
  const int64_t t_lo = (int64_t)bx * a.rows_per_block;
  const int64_t t_hi = min(min(t_lo + a.rows_per_block, a.n_rows), min(a.a_rows, a.b_rows));
  v4f acc[4][NT];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[e][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
  const bool jok = j0 + 4 * s < a.ca;
  bool nok[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) nok[nt] = nt * 16 + s < a.cb;
  for (int64_t base = t_lo; base < t_hi; base += 4 * kU) {
    float4 av[kU];
    float bv[kU][NT];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int64_t t = base + u * 4 + q;
      const bool live = t < t_hi;
      av[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (live && jok) av[u] = *reinterpret_cast<const float4*>(a.A + t * a.lda + j0 + 4 * s);
      if (a.wptr != nullptr && live) {
        const float w = (float)(a.wptr[t + 1] - a.wptr[t]);
        av[u].x *= w; av[u].y *= w; av[u].z *= w; av[u].w *= w;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bv[u][nt] = (live && nok[nt]) ? a.B[t * a.ldb + a.bcol0 + nt * 16 + s] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kU; ++u)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        acc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u].x, bv[u][nt], acc[0][nt], 0, 0, 0);
        acc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u].y, bv[u][nt], acc[1][nt], 0, 0, 0);
        acc[2][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u].z, bv[u][nt], acc[2][nt], 0, 0, 0);
        acc[3][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u].w, bv[u][nt], acc[3][nt], 0, 0, 0);
      }
  }
  // register r of lane (s, q), component e, tile nt: column j0 + 4 (4 q + r) + e of A, column 16 nt + s of B
  float* out = a.partial + (int64_t)bx * a.ca * a.cb;
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = j0 + 4 * (4 * q + r) + e, n = nt * 16 + s;
        if (j < a.ca && n < a.cb) out[(int64_t)j * a.cb + n] = acc[e][nt][r];
      }
}

// Form for tables with at most 48 columns: 16-column tiles of A read one float per lane, one MFMA per tile,
// so that short rows do not leave three quarters of the MFMA rows empty.  JT <= 3, NT in {1, 2, 4}.
template <int JT, int NT>
__global__ __launch_bounds__(kBlock) void tred_dw_kernel(TredArgs a) {
  constexpr int kUD = 8;
  __shared__ float red[JT * 16 * NT * 16];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int s = lane % 16, q = lane / 16;
  int bx, by;
  if (!tred_block_ids(a, bx, by)) return;
  const int n0 = by * NT * 16;
  const int64_t t_lo = (int64_t)bx * a.rows_per_block;
  const int64_t t_hi = min(t_lo + a.rows_per_block, a.n_rows);
  if (a.upper_only && 0 >= n0 + NT * 16) return;
  v4f acc[JT][NT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[jt][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
  bool jok[JT], nok[NT];
#pragma unroll
  for (int jt = 0; jt < JT; ++jt) jok[jt] = jt * 16 + s < a.ca;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) nok[nt] = n0 + nt * 16 + s < a.cb;

  for (int64_t base = t_lo + (int64_t)wave * (4 * kUD); base < t_hi; base += (int64_t)(kBlock / kWave) * (4 * kUD)) {
    float av[kUD][JT], bv[kUD][NT];
#pragma unroll
    for (int u = 0; u < kUD; ++u) {
      int64_t t = base + u * 4 + q;
      int64_t ra = -1, rb = -1;
      float w = 1.0f;
      if (t < t_hi) {
        ra = a.ia ? (int64_t)a.ia[t] : (t < a.a_rows ? t : -1);
        rb = a.ib ? (int64_t)a.ib[t] : (t < a.b_rows ? t : -1);
        if (a.wptr) w = (float)(a.wptr[t + 1] - a.wptr[t]);
      }
      const bool live = ra >= 0 && rb >= 0;
#pragma unroll
      for (int jt = 0; jt < JT; ++jt) {
        av[u][jt] = (live && jok[jt]) ? a.A[ra * a.lda + jt * 16 + s] : 0.0f;
        if (a.wptr) av[u][jt] *= w;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        bv[u][nt] = (live && nok[nt]) ? a.B[rb * a.ldb + a.bcol0 + n0 + nt * 16 + s] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kUD; ++u)
#pragma unroll
      for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][jt], bv[u][nt], acc[jt][nt], 0, 0, 0);
  }
  for (int w = 0; w < kBlock / kWave; ++w) {
    if (wave == w) {
#pragma unroll
      for (int jt = 0; jt < JT; ++jt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            int j = jt * 16 + 4 * q + r, n = nt * 16 + s;
            float v = acc[jt][nt][r];
            if (w == 0) red[j * (NT * 16) + n] = v;
            else red[j * (NT * 16) + n] += v;
          }
    }
    __syncthreads();
  }
  float* out = a.partial + (int64_t)bx * a.ca * a.cb;
  for (int o = tid; o < JT * 16 * NT * 16; o += kBlock) {
    int j = o / (NT * 16), n = o - j * (NT * 16);
    if (j < a.ca && n0 + n < a.cb) out[(int64_t)j * a.cb + n0 + n] = red[o];
  }
}

// block[e] = sum over chunks.  A workgroup owns 16 consecutive elements; its 16 thread groups stride the chunks
// with eight loads in flight each, then the groups are added in order.
// tcols > 0: the partials are a (elems / tcols) x tcols matrix and block receives its transpose.
__global__ __launch_bounds__(kBlock) void tred_reduce_kernel(const float* __restrict__ partial, int nchunks,
                                                             int64_t elems, float* __restrict__ block, int tcols) {
  __shared__ float red[16][16];
  const int el = threadIdx.x % 16, cg = threadIdx.x / 16;
  const int64_t e = (int64_t)blockIdx.x * 16 + el;
  float s[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) s[u] = 0.0f;
  if (e < elems) {
    int c = cg;
    for (; c + 7 * 16 < nchunks; c += 8 * 16) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(c + u * 16) * elems + e];
#pragma unroll
      for (int u = 0; u < 8; ++u) s[u] += v[u];
    }
    for (; c < nchunks; c += 16) s[0] += partial[(int64_t)c * elems + e];
  }
  red[cg][el] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  if (threadIdx.x < 16 && e < elems) {
    float t = 0.0f;
#pragma unroll
    for (int g = 0; g < 16; ++g) t += red[g][el];
    if (tcols > 0) {
      const int64_t i = e / tcols, j = e - i * tcols;
      block[j * (elems / tcols) + i] = t;
    } else {
      block[e] = t;
    }
  }
}

// out[t, n] = sum over sources, in order, of G_k[tcol2src_k[t], n]; MODE 1 applies the update of Alg. 1.
template <int MODE>
__global__ __launch_bounds__(kBlock) void colasm_kernel(ColAsmArgs a) {
  int64_t total = (int64_t)a.c_T * a.cx;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
       e += (int64_t)gridDim.x * blockDim.x) {
    int t = (int)(e / a.cx), n = (int)(e - (int64_t)t * a.cx);
    float acc = 0.0f;
    for (int k = 0; k < a.n; ++k) {
      int j = a.tcol2src[k][t];
      if (j >= 0) acc += a.G[k][(int64_t)j * a.cx + n];
    }
    if constexpr (MODE == 0) a.out[e] = acc;
    else a.out[e] = a.out[e] - a.lr[n] * (acc * a.inv_rT);
  }
  if constexpr (MODE == 1) {
    // loss[n] = scale * sum of the per-workgroup partials: wavefront w of the grid owns columns w, w + W, ...;
    // its lanes stride the partials, fixed butterfly
    if (a.loss != nullptr) {
      const int lane = threadIdx.x % kWave;
      const int gw = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave, nw = gridDim.x * (kBlock / kWave);
      for (int n = gw; n < a.cx; n += nw) {
        float s = 0.0f;
        for (int b = lane; b < a.n_loss_partial; b += kWave) s += a.loss_partial[(int64_t)b * a.cx + n];
        for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
        if (lane == 0) a.loss[n] = s * a.loss_scale;
      }
    }
  }
}

// The same with sources that still hold per-workgroup partial blocks (nparts[k] blocks of c_k x cx): one workgroup
// per target column; thread (n, slice) adds the blocks slice, slice + S, ... of operand column n, the slices are
// added in order through LDS, the sources in source order.  For operands of at most 64 columns.
template <int MODE>
__global__ __launch_bounds__(kBlock) void colasm_parts_kernel(ColAsmArgs a, int nw) {
  __shared__ float part[kBlock];
  const int t = blockIdx.x;
  if (t >= a.c_T) {
    if constexpr (MODE == 1) {
      // one extra workgroup: loss[n] = scale * sum of the per-workgroup partials, wavefront per column
      if (a.loss != nullptr) {
        const int lane = threadIdx.x % kWave;
        for (int n = threadIdx.x / kWave; n < a.cx; n += kBlock / kWave) {
          float s = 0.0f;
          for (int b = lane; b < a.n_loss_partial; b += kWave) s += a.loss_partial[(int64_t)b * a.cx + n];
          for (int m = kWave / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m);
          if (lane == 0) a.loss[n] = s * a.loss_scale;
        }
      }
    }
    return;
  }
  const int n = threadIdx.x % nw, sl = threadIdx.x / nw, ns = kBlock / nw;
  float acc = 0.0f;
  for (int k = 0; k < a.n; ++k) {
    const int j = a.tcol2src[k][t];
    const int np = a.nparts[k] > 0 ? a.nparts[k] : 1;
    float s = 0.0f;
    if (j >= 0 && n < a.cx) {
      const float* g = a.G[k] + (int64_t)j * a.cx + n;
      const int64_t stride = (int64_t)a.ck[k] * a.cx;
      float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
      int b = sl;
      for (; b + 3 * ns < np; b += 4 * ns) {
        s0 += g[(int64_t)b * stride]; s1 += g[(int64_t)(b + ns) * stride];
        s2 += g[(int64_t)(b + 2 * ns) * stride]; s3 += g[(int64_t)(b + 3 * ns) * stride];
      }
      for (; b < np; b += ns) s0 += g[(int64_t)b * stride];
      s = (s0 + s1) + (s2 + s3);
    }
    __syncthreads();                                   // the previous source's sums are consumed
    part[threadIdx.x] = s;
    __syncthreads();
    if (sl == 0) {
      float v = 0.0f;
      for (int q = 0; q < ns; ++q) v += part[q * nw + n];
      acc += v;
    }
  }
  if (sl == 0 && n < a.cx) {
    float* o = a.out + (int64_t)t * a.cx + n;
    if constexpr (MODE == 0) *o = acc;
    else *o = *o - a.lr[n] * (acc * a.inv_rT);
  }
}

}  // namespace

namespace {

using TredFn = void (*)(TredArgs);

struct TredChoice {
  TredFn fn;
  int tiles;        // workgroups per row chunk (tiles that are actually computed)
};

// Kernel variant and tile count for these shapes.
TredChoice tred_select(const TredArgs& a, bool bf16) {
  const bool vec4 = a.lda % 4 == 0 && a.ca % 4 == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0;
  const int nt = a.cb <= 16 ? 1 : (a.cb <= 32 ? 2 : 4);
  const int b_slabs = (a.cb + nt * 16 - 1) / (nt * 16);
  TredChoice c{nullptr, 1};
  if (bf16) {
    c.tiles = ((a.ca + 63) / 64) * b_slabs;
    if (nt == 1) c.fn = vec4 ? tred_bf16_kernel<1, true> : tred_bf16_kernel<1, false>;
    else if (nt == 2) c.fn = vec4 ? tred_bf16_kernel<2, true> : tred_bf16_kernel<2, false>;
    else c.fn = vec4 ? tred_bf16_kernel<4, true> : tred_bf16_kernel<4, false>;
    return c;
  }
  // wide A against at most 32 columns of B, direct addressing: the column-split kernel
  if (a.ca >= 64 && a.cb <= 32 && vec4 && a.ia == nullptr && a.ib == nullptr && !a.upper_only) {
    c.tiles = (a.ca + 255) / 256;                       // four 64-column slabs per workgroup
    c.fn = nt == 1 ? tred_cs_kernel<1> : tred_cs_kernel<2>;
    return c;
  }
  if (a.ca <= 48) {
    const int jtd = (a.ca + 15) / 16;
    c.tiles = b_slabs;
    static const TredFn table[3][3] = {
        {tred_dw_kernel<1, 1>, tred_dw_kernel<1, 2>, tred_dw_kernel<1, 4>},
        {tred_dw_kernel<2, 1>, tred_dw_kernel<2, 2>, tred_dw_kernel<2, 4>},
        {tred_dw_kernel<3, 1>, tred_dw_kernel<3, 2>, tred_dw_kernel<3, 4>}};
    c.fn = table[jtd - 1][nt == 1 ? 0 : (nt == 2 ? 1 : 2)];
    return c;
  }
  int jt = std::min(4 / nt, (a.ca + 63) / 64);
  if (jt == 3) jt = 4;
  const int a_slabs = (a.ca + jt * 64 - 1) / (jt * 64);
  c.tiles = a_slabs * b_slabs;
#define ILARGI_PICK(J, N) (vec4 ? tred_kernel<J, N, true> : tred_kernel<J, N, false>)
  if (jt == 4) c.fn = ILARGI_PICK(4, 1);
  else if (jt == 2 && nt == 2) c.fn = ILARGI_PICK(2, 2);
  else if (jt == 2) c.fn = ILARGI_PICK(2, 1);
  else if (nt == 4) c.fn = ILARGI_PICK(1, 4);
  else if (nt == 2) c.fn = ILARGI_PICK(1, 2);
  else c.fn = ILARGI_PICK(1, 1);
#undef ILARGI_PICK
  return c;
}

}  // namespace

// Workgroup slots of the device for the variant these shapes select, and how many tiles each row chunk has
// (tiles the kernel skips for a symmetric result are not counted).  The caller sizes the row chunks so that
// the launch fills the slots in whole rounds.
void tred_occupancy(const TredArgs& a, bool bf16, int* slots, int* tiles) {
  static std::mutex cache_mutex;   // the cache below is shared by every plan of the process
  std::lock_guard<std::mutex> lock(cache_mutex);
  TredChoice c = tred_select(a, bf16);
  // both queries are cached: they cost far more than a launch
  static int cus = 0;
  static TredFn seen_fn[64];
  static int seen_occ[64];
  static int n_seen = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    cus = 256;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      cus = prop.multiProcessorCount;
  }
  int per_cu = 0;
  for (int i = 0; i < n_seen; ++i)
    if (seen_fn[i] == c.fn) per_cu = seen_occ[i];
  if (per_cu == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(c.fn), kBlock, 0) != hipSuccess || per_cu < 1)
      per_cu = 2;
    if (n_seen < 64) { seen_fn[n_seen] = c.fn; seen_occ[n_seen] = per_cu; ++n_seen; }
  }
  *slots = per_cu * cus;
  int t = c.tiles;
  if (a.upper_only && !bf16 && a.ca > 48) {
    // 64 x 64 tiles on and above the diagonal
    int n = (a.ca + 63) / 64;
    t = n * (n + 1) / 2;
  }
  *tiles = t;
}

hipError_t launch_tred(const TredArgs& a, int nchunks, bool bf16, hipStream_t st) {
  if (a.ca <= 0 || a.cb <= 0 || nchunks <= 0) return hipSuccess;
  TredChoice c = tred_select(a, bf16);
  TredArgs b = a;
  b.gx = nchunks;
  b.gy = c.tiles;
  const int64_t total = ((int64_t)nchunks + 7) / 8 * 8 * c.tiles;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(c.fn, dim3((unsigned)total), dim3(kBlock), 0, st, b);
  return hipGetLastError();
}

hipError_t launch_tred_reduce(const float* partial, int nchunks, int64_t elems, float* block, hipStream_t st, int tcols) {
  if (elems <= 0) return hipSuccess;
  int64_t grid = (elems + 15) / 16;
  tred_reduce_kernel<<<(unsigned)grid, kBlock, 0, st>>>(partial, nchunks, elems, block, tcols);
  return hipGetLastError();
}

hipError_t launch_colasm(const ColAsmArgs& a, int mode, hipStream_t st) {
  int64_t total = (int64_t)a.c_T * a.cx;
  if (total <= 0) return hipSuccess;
  bool parts = false;
  for (int k = 0; k < a.n; ++k) parts = parts || a.nparts[k] > 1;
  if (parts && a.cx <= 64) {
    const int nw = a.cx <= 16 ? 16 : (a.cx <= 32 ? 32 : 64);
    const int grid = a.c_T + ((mode == 1 && a.loss != nullptr) ? 1 : 0);
    if (mode == 0) colasm_parts_kernel<0><<<grid, kBlock, 0, st>>>(a, nw);
    else colasm_parts_kernel<1><<<grid, kBlock, 0, st>>>(a, nw);
    return hipGetLastError();
  }
  int grid = (int)((total + kBlock - 1) / kBlock);
  if (grid > 1024) grid = 1024;
  if (mode == 0) colasm_kernel<0><<<grid, kBlock, 0, st>>>(a);
  else colasm_kernel<1><<<grid, kBlock, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace ilargi
