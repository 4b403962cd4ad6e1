// Streaming kernels of the wide batch.  With bfloat16 inputs and float32 accumulation (values are rounded to
// bfloat16, nearest even, where they enter a product; products of two bfloat16 values are exact in float32):
//   lmm_prod_bf16_kernel     P = D (M^T X)            per-source product of the left multiply (Sec. 2.2)
//   tred_stream_bf16_kernel  C = A^T B  over all rows  column reduce of the transposed multiply (Sec. 2.2)
// A bfloat16 MFMA does sixteen times the work of a float32 one per cycle, so neither kernel is bound by the matrix
// cores: both are laid out around their memory streams (the tables stay float32 in memory and are converted on the
// way in) and around LDS traffic.
#include <algorithm>
#include <cstdint>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWbThreads = 512;              // one workgroup per compute unit: the operand slab takes most of its LDS
constexpr int kWbWaves = kWbThreads / kWave;
constexpr int kWbSlab = 256;                 // operand columns per workgroup (sixteen 16-column tiles)

__device__ __forceinline__ bf16x8 wb_pack(const float4& lo, const float4& hi) {
  bf16x8 v;
  v[0] = (__bf16)lo.x; v[1] = (__bf16)lo.y; v[2] = (__bf16)lo.z; v[3] = (__bf16)lo.w;
  v[4] = (__bf16)hi.x; v[5] = (__bf16)hi.y; v[6] = (__bf16)hi.z; v[7] = (__bf16)hi.w;
  return v;
}

// The operand of the product as bfloat16 in the layout the product kernel keeps in LDS: for every slab of 256
// operand columns, [K / 8][256 columns][8 consecutive K] (zero for unmapped table columns, beyond K and beyond
// the operand).  One thread per (K octet, column): eight values down a column of X, branch-free.
__global__ __launch_bounds__(kBlock) void lmm_pack_bf16_kernel(LmmArgs a, int nst, bf16x8* __restrict__ packed) {
  const int items = 4 * nst * kWbSlab;
  const int it = blockIdx.x * kBlock + threadIdx.x;
  if (it >= items) return;
  const int n0 = blockIdx.y * kWbSlab;
  const int nw = min(kWbSlab, a.ncols - n0);
  const int n = it % kWbSlab, o = it / kWbSlab;
  const float* Xc = a.X + a.col0 + n0;
  const int ns = min(n, nw - 1);
  int t[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) t[c] = 8 * o + c < a.ck ? a.colmap[8 * o + c] : -1;
  float x[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) x[c] = Xc[(int64_t)max(t[c], 0) * a.ldx + ns];
  bf16x8 v;
#pragma unroll
  for (int c = 0; c < 8; ++c) v[c] = (__bf16)((t[c] >= 0 && n < nw) ? x[c] : 0.0f);
  packed[(size_t)blockIdx.y * items + it] = v;
}

// P = D X_D for a slab of up to 256 operand columns.  The whole operand slab sits in LDS as bfloat16,
// [K / 8][256 columns][8 consecutive K]: one 128-bit read is the B operand of a 16x16x32 MFMA.  A wavefront owns
// 16 table rows at a time and streams them from memory straight into A operands (lane (row li, q) loads the 32
// bytes at columns 32 s + 8 q of its row for every step s, next tile prefetched), then walks the sixteen column
// tiles.  NST: compile-time bound of the 32-column steps of a table row.
template <int NST>
__global__ __launch_bounds__(kWbThreads) void lmm_prod_bf16_kernel(LmmArgs a, int nst, const bf16x8* __restrict__ packed) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  bf16x8* Bs = reinterpret_cast<bf16x8*>(lds_raw);            // [4 nst][kWbSlab]
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  const int ck = a.ck;
  const int n0 = blockIdx.y * kWbSlab;
  const int nw = min(kWbSlab, a.ncols - n0);                  // live columns of this slab
  const int ntc = (nw + 15) / 16;                             // live 16-column tiles
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int64_t tstride = (int64_t)gridDim.x * kWbWaves;
  int64_t tile = (int64_t)blockIdx.x * kWbWaves + wave;

  float4 av[NST][2];
  unsigned live = 0;                                          // bit 2 s + h: piece h of step s lies inside the table
  // Branch-free: a piece beyond the table reads the table's first bytes and is replaced by zero when the tile is
  // converted, not here, so that nothing waits for a load before all of them are issued.
  auto fetch = [&](int64_t t) {
    const int64_t row = t * 16 + li;
    const bool in = t < ntiles && row < a.d_rows;
    const float* rp = a.D + (in ? row * ck + 8 * q : 0);
    live = 0;
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      const int c = 32 * s + 8 * q;
      const bool ok0 = s < nst && in && c < ck, ok1 = s < nst && in && c + 4 < ck;
      av[s][0] = *reinterpret_cast<const float4*>(ok0 ? rp + 32 * s : a.D);
      av[s][1] = *reinterpret_cast<const float4*>(ok1 ? rp + 32 * s + 4 : a.D);
      live |= (ok0 ? 1u : 0u) << (2 * s) | (ok1 ? 2u : 0u) << (2 * s);
    }
  };
  fetch(tile);
  // the operand slab, packed beforehand (lmm_pack_bf16_kernel): a straight copy, every load of a thread in flight
  {
    const bf16x8* src = packed + (size_t)blockIdx.y * 4 * nst * kWbSlab;
    bf16x8 t[2 * NST];
#pragma unroll
    for (int u = 0; u < 2 * NST; ++u) t[u] = src[min(u, 2 * nst - 1) * kWbThreads + tid];
#pragma unroll
    for (int u = 0; u < 2 * NST; ++u)
      if (u < 2 * nst) Bs[u * kWbThreads + tid] = t[u];
  }
  __syncthreads();

  for (; tile < ntiles; tile += tstride) {
    bf16x8 ab[NST];
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      const float4 z = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      ab[s] = wb_pack((live >> (2 * s) & 1u) ? av[s][0] : z, (live >> (2 * s) & 2u) ? av[s][1] : z);
    }
    fetch(tile + tstride);
    const int64_t row0 = tile * 16;
#pragma unroll
    for (int nt = 0; nt < kWbSlab / 16; ++nt) {
      if (nt < ntc) {
        v4f acc = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < NST; ++s)
          if (s < nst) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab[s], Bs[(size_t)(4 * s + q) * kWbSlab + 16 * nt + li], acc, 0, 0, 0);
        // register r of lane (li, q) = P[row 4 q + r][column 16 nt + li]
        const int n = 16 * nt + li;
        if (n < nw) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int64_t row = row0 + 4 * q + r;
            if (row < a.r_out) {
              float* op = a.out + row * a.ldo + a.col0 + n0 + n;
              if (a.nt_out) __builtin_nontemporal_store(acc[r], op);
              else *op = acc[r];
            }
          }
        }
      }
    }
  }
}


// C = A^T B over all rows (A n x ca, B n x cb, both float32 in memory, plain rows): the column reduce of the
// transposed multiply for a wide operand.  The contraction runs over table ROWS, so both operands have to reach the
// matrix cores transposed: eight consecutive rows of one column are the 16 bytes a lane hands to a 16x16x32 MFMA.
// One workgroup of eight wavefronts per compute unit walks a contiguous range of rows in steps of 32.  A thread
// loads an 8-row x 4-column block of A or of B (eight float4, adjacent threads adjacent columns: whole rows per
// instruction), converts, and writes four 16-byte column pieces to LDS, laid out [row octet][column]; the next
// step's loads are issued before the current step is multiplied, LDS is double-buffered, one barrier per step.
// Wavefront w owns the column tiles 2 w and 2 w + 1 of B against every column tile of A (up to 32 accumulators),
// so the whole ca x cb result of the workgroup's rows stays in registers until the end.  Per-workgroup results are
// added afterwards in workgroup order.
constexpr int kTsMt = 16;                    // 16-column tiles of A at most (ca <= 256)
constexpr int kTsStepRows = 32;

__global__ __launch_bounds__(kWbThreads) void tred_stream_bf16_kernel(TredArgs a, int mtc, int ntc) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int cap = 16 * mtc;                                   // padded columns of A
  bf16x8* buf = reinterpret_cast<bf16x8*>(lds_raw);           // two buffers of [4][cap] (A) then [4][kWbSlab] (B)
  const int buf_units = 4 * cap + 4 * kWbSlab;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  // zero once: the padding columns are never written again
  for (int e = tid; e < 2 * buf_units; e += kWbThreads) {
    bf16x8 z;
#pragma unroll
    for (int c = 0; c < 8; ++c) z[c] = (__bf16)0.0f;
    buf[e] = z;
  }
  // this thread's loading task: threads 0..255 an 8 x 4 block of B, threads 256.. one of A
  const bool is_b = tid < 256;
  const int t = is_b ? tid : tid - 256;
  const int quads = is_b ? kWbSlab / 4 : a.ca / 4;            // column quads per row octet
  const int rb = t / quads, cq = t - rb * quads;              // row octet of the step, column quad
  const bool task = rb < 4 && (is_b ? 4 * cq < a.cb : true);
  const float* base = is_b ? a.B + a.bcol0 + 4 * cq : a.A + 4 * cq;
  const int ld = is_b ? a.ldb : a.lda;
  const int64_t row_begin = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t row_end = min(a.n_rows, row_begin + a.rows_per_block);

  float4 x[8];
  unsigned live = 0;
  auto fetch = [&](int64_t r0) {                              // rows r0 + 8 rb + i, branch-free
    live = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t row = r0 + 8 * rb + i;
      const bool ok = task && row < row_end;
      x[i] = *reinterpret_cast<const float4*>(ok ? base + row * ld : (is_b ? a.B : a.A));
      live |= (ok ? 1u : 0u) << i;
    }
  };
  v4f acc[kTsMt][2];
#pragma unroll
  for (int mt = 0; mt < kTsMt; ++mt)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[mt][j] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  fetch(row_begin);
  __syncthreads();                                            // the zero fill is in place
  int cur = 0;
  for (int64_t r0 = row_begin; r0 < row_end; r0 += kTsStepRows, cur ^= 1) {
    bf16x8* As = buf + (size_t)cur * buf_units;               // [4][cap]
    bf16x8* Bs = As + 4 * cap;                                // [4][kWbSlab]
    if (task) {
      float xs[8][4];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool ok = (live >> i & 1u) != 0;
        xs[i][0] = ok ? x[i].x : 0.0f; xs[i][1] = ok ? x[i].y : 0.0f;
        xs[i][2] = ok ? x[i].z : 0.0f; xs[i][3] = ok ? x[i].w : 0.0f;
      }
      bf16x8* dst = (is_b ? Bs + rb * kWbSlab : As + rb * cap) + 4 * cq;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (__bf16)xs[i][c];
        dst[c] = v;
      }
    }
    fetch(r0 + kTsStepRows);
    __syncthreads();
    bf16x8 bf[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) bf[j] = Bs[q * kWbSlab + 16 * (2 * wave + j) + li];
#pragma unroll
    for (int mt = 0; mt < kTsMt; ++mt) {
      if (mt < mtc) {
        const bf16x8 af = As[q * cap + 16 * mt + li];
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if (2 * wave + j < ntc) acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, bf[j], acc[mt][j], 0, 0, 0);
      }
    }
  }
  // register r of lane (li, q), tile (mt, j) = C[16 mt + 4 q + r][16 (2 wave + j) + li]
  float* out = a.partial + (int64_t)blockIdx.x * a.ca * a.cb;
#pragma unroll
  for (int mt = 0; mt < kTsMt; ++mt) {
    if (mt < mtc) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = 16 * (2 * wave + j) + li;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = 16 * mt + 4 * q + r;
          if (m < a.ca && n < a.cb) out[(int64_t)m * a.cb + n] = acc[mt][j][r];
        }
      }
    }
  }
}

// The same column reduce with float32 inputs (16x16x4 MFMA).  Here the matrix cores are the bound (a float32 MFMA
// does a sixteenth of the work per cycle).  The tiles are staged transposed as well, [column][32 rows]: the
// summation index of a product may be dealt to the K slots in any order as long as both operands agree, so K slot
// q of the four products of group h stands for rows 16 h + 4 q .. + 3, and one 128-bit LDS read per operand feeds
// four products on one accumulator.
constexpr int kTfLdr = kTsStepRows + 4;      // floats per staged column (rows of a step + padding)

__global__ __launch_bounds__(kWbThreads) void tred_stream_f32_kernel(TredArgs a, int mtc, int ntc) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int cap = 16 * mtc;
  float* buf = reinterpret_cast<float*>(lds_raw);             // two buffers of [cap][kTfLdr] (A) then [kWbSlab][kTfLdr] (B)
  const int buf_floats = (cap + kWbSlab) * kTfLdr;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  for (int e = tid; e < 2 * buf_floats; e += kWbThreads) buf[e] = 0.0f;   // padding columns stay zero
  // this thread's loading task: threads 0..255 an 8 x 4 block of B, threads 256.. one of A
  const bool is_b = tid < 256;
  const int t = is_b ? tid : tid - 256;
  const int quads = is_b ? kWbSlab / 4 : a.ca / 4;
  const int rb = t / quads, cq = t - rb * quads;              // row octet of the step, column quad
  const bool task = rb < 4 && (is_b ? 4 * cq < a.cb : true);
  const float* base = is_b ? a.B + a.bcol0 + 4 * cq : a.A + 4 * cq;
  const int ld = is_b ? a.ldb : a.lda;
  const int64_t row_begin = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t row_end = min(a.n_rows, row_begin + a.rows_per_block);

  float4 x[8];
  unsigned live = 0;
  auto fetch = [&](int64_t r0) {                              // rows r0 + 8 rb + i, branch-free
    live = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t row = r0 + 8 * rb + i;
      const bool ok = task && row < row_end;
      x[i] = *reinterpret_cast<const float4*>(ok ? base + row * ld : (is_b ? a.B : a.A));
      live |= (ok ? 1u : 0u) << i;
    }
  };
  v4f acc[kTsMt][2];
#pragma unroll
  for (int mt = 0; mt < kTsMt; ++mt)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[mt][j] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  fetch(row_begin);
  __syncthreads();
  int cur = 0;
  for (int64_t r0 = row_begin; r0 < row_end; r0 += kTsStepRows, cur ^= 1) {
    float* As = buf + (size_t)cur * buf_floats;               // [cap][kTfLdr]
    float* Bs = As + cap * kTfLdr;                            // [kWbSlab][kTfLdr]
    if (task) {
      float xs[8][4];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool ok = (live >> i & 1u) != 0;
        xs[i][0] = ok ? x[i].x : 0.0f; xs[i][1] = ok ? x[i].y : 0.0f;
        xs[i][2] = ok ? x[i].z : 0.0f; xs[i][3] = ok ? x[i].w : 0.0f;
      }
      float* dst = (is_b ? Bs : As) + (size_t)(4 * cq) * kTfLdr + 8 * rb;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        *reinterpret_cast<float4*>(dst + c * kTfLdr) = make_float4(xs[0][c], xs[1][c], xs[2][c], xs[3][c]);
        *reinterpret_cast<float4*>(dst + c * kTfLdr + 4) = make_float4(xs[4][c], xs[5][c], xs[6][c], xs[7][c]);
      }
    }
    fetch(r0 + kTsStepRows);
    __syncthreads();
#pragma unroll
    for (int h = 0; h < kTsStepRows / 16; ++h) {
      float4 bf[2];
#pragma unroll
      for (int j = 0; j < 2; ++j)
        bf[j] = *reinterpret_cast<const float4*>(Bs + (size_t)(16 * (2 * wave + j) + li) * kTfLdr + 16 * h + 4 * q);
#pragma unroll
      for (int mt = 0; mt < kTsMt; ++mt) {
        if (mt < mtc) {
          const float4 af = *reinterpret_cast<const float4*>(As + (size_t)(16 * mt + li) * kTfLdr + 16 * h + 4 * q);
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            if (2 * wave + j < ntc) {
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf[j].x, acc[mt][j], 0, 0, 0);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf[j].y, acc[mt][j], 0, 0, 0);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf[j].z, acc[mt][j], 0, 0, 0);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf[j].w, acc[mt][j], 0, 0, 0);
            }
          }
        }
      }
    }
  }
  float* out = a.partial + (int64_t)blockIdx.x * a.ca * a.cb;
#pragma unroll
  for (int mt = 0; mt < kTsMt; ++mt) {
    if (mt < mtc) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = 16 * (2 * wave + j) + li;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = 16 * mt + 4 * q + r;
          if (m < a.ca && n < a.cb) out[(int64_t)m * a.cb + n] = acc[mt][j][r];
        }
      }
    }
  }
}

// The float32 product for a wide operand, same plan: the operand slab (here 128 columns, [K / 4][128][4 consecutive
// K] floats, packed beforehand) in LDS, table rows streamed from memory straight into A operands.  Lane (row li, q)
// loads the float4 at columns 16 s + 4 q of its row; its four values and one 128-bit LDS read are four 16x16x4
// products on one accumulator (K slot q of product e stands for column 16 s + 4 q + e).  The matrix cores are the
// bound here: 52 products per column tile and 16 table rows.
constexpr int kFsSlab = 128;

__global__ __launch_bounds__(kBlock) void lmm_pack_f32_kernel(LmmArgs a, int nst, float4* __restrict__ packed) {
  const int items = 4 * nst * kFsSlab;
  const int it = blockIdx.x * kBlock + threadIdx.x;
  if (it >= items) return;
  const int n0 = blockIdx.y * kFsSlab;
  const int nw = min(kFsSlab, a.ncols - n0);
  const int n = it % kFsSlab, o = it / kFsSlab;
  const float* Xc = a.X + a.col0 + n0;
  const int ns = min(n, nw - 1);
  int t[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) t[c] = 4 * o + c < a.ck ? a.colmap[4 * o + c] : -1;
  float x[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) x[c] = Xc[(int64_t)max(t[c], 0) * a.ldx + ns];
#pragma unroll
  for (int c = 0; c < 4; ++c) x[c] = (t[c] >= 0 && n < nw) ? x[c] : 0.0f;
  packed[(size_t)blockIdx.y * items + it] = make_float4(x[0], x[1], x[2], x[3]);
}

// NST: compile-time bound of the 16-column steps of a table row.
template <int NST>
__global__ __launch_bounds__(kWbThreads) void lmm_prod_f32_wide_kernel(LmmArgs a, int nst, const float4* __restrict__ packed) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  float4* Bs = reinterpret_cast<float4*>(lds_raw);            // [4 nst][kFsSlab]
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  const int ck = a.ck;
  const int n0 = blockIdx.y * kFsSlab;
  const int nw = min(kFsSlab, a.ncols - n0);
  const int ntc = (nw + 15) / 16;
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int64_t tstride = (int64_t)gridDim.x * kWbWaves;
  int64_t tile = (int64_t)blockIdx.x * kWbWaves + wave;

  float4 av[NST];
  unsigned live = 0;
  auto fetch = [&](int64_t t) {                               // branch-free, see lmm_prod_bf16_kernel
    const int64_t row = t * 16 + li;
    const bool in = t < ntiles && row < a.d_rows;
    const float* rp = a.D + (in ? row * ck + 4 * q : 0);
    live = 0;
#pragma unroll
    for (int s = 0; s < NST; ++s) {
      const bool ok = s < nst && in && 16 * s + 4 * q < ck;
      av[s] = *reinterpret_cast<const float4*>(ok ? rp + 16 * s : a.D);
      live |= (ok ? 1u : 0u) << s;
    }
  };
  fetch(tile);
  {
    const float4* src = packed + (size_t)blockIdx.y * 4 * nst * kFsSlab;
    float4 t[NST];
#pragma unroll
    for (int u = 0; u < NST; ++u) t[u] = src[min(u, nst - 1) * kWbThreads + tid];
#pragma unroll
    for (int u = 0; u < NST; ++u)
      if (u < nst) Bs[u * kWbThreads + tid] = t[u];
  }
  __syncthreads();

  for (; tile < ntiles; tile += tstride) {
    float4 ac[NST];
#pragma unroll
    for (int s = 0; s < NST; ++s) ac[s] = (live >> s & 1u) ? av[s] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    fetch(tile + tstride);
    const int64_t row0 = tile * 16;
    // The operand values are read half a column tile ahead of the products that use them (a product chain that
    // waits for its own LDS reads leaves the matrix cores idle half of the time): units of H steps, the next
    // unit's values requested before the current unit's products are issued.
    constexpr int H = (NST + 1) / 2;
    float4 bn[H];
    auto read_unit = [&](int nt, int half) {
#pragma unroll
      for (int e = 0; e < H; ++e) bn[e] = Bs[(size_t)(4 * min(half * H + e, nst - 1) + q) * kFsSlab + 16 * nt + li];
    };
    read_unit(0, 0);
#pragma unroll
    for (int nt = 0; nt < kFsSlab / 16; ++nt) {
      if (nt < ntc) {
        v4f acc = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          float4 bv[H];
#pragma unroll
          for (int e = 0; e < H; ++e) bv[e] = bn[e];
          if (half == 0) read_unit(nt, 1);
          else read_unit(min(nt + 1, kFsSlab / 16 - 1), 0);
#pragma unroll
          for (int e = 0; e < H; ++e) {
            const int sidx = half * H + e;
            if (sidx < NST && sidx < nst) {
              acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[sidx].x, bv[e].x, acc, 0, 0, 0);
              acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[sidx].y, bv[e].y, acc, 0, 0, 0);
              acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[sidx].z, bv[e].z, acc, 0, 0, 0);
              acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ac[sidx].w, bv[e].w, acc, 0, 0, 0);
            }
          }
        }
        const int n = 16 * nt + li;
        if (n < nw) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int64_t row = row0 + 4 * q + r;
            if (row < a.r_out) {
              float* op = a.out + row * a.ldo + a.col0 + n0 + n;
              if (a.nt_out) __builtin_nontemporal_store(acc[r], op);
              else *op = acc[r];
            }
          }
        }
      }
    }
  }
}

typedef void (*PfFn)(LmmArgs, int, const float4*);

typedef void (*PbFn)(LmmArgs, int, const bf16x8*);

int wb_cus() {
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      return (int)prop.multiProcessorCount;
    return 256;
  }();
  return cus;
}

}  // namespace

// A dense table with 16-byte aligned rows of at most 256 columns, any number of operand columns, no gathers and no
// epilogue, and scratch for the packed operand (16 KiB per 32 table columns and slab of 256 operand columns).
bool lmm_prod_bf16_supported(const LmmArgs& a, int vec, int mode) {
  if (mode != 0 || a.D == nullptr || vec != 4 || a.ck < 4 || a.ck % 4 != 0 || a.ck > 256) return false;
  if (a.g.n != 0 || a.grad_partial != nullptr || a.ncols < 1) return false;
  if (reinterpret_cast<uintptr_t>(a.D) % 16 != 0 || a.d_rows < a.r_out) return false;
  const int64_t nst = (a.ck + 31) / 32, slabs = (a.ncols + kWbSlab - 1) / kWbSlab;
  if (a.scratch == nullptr || reinterpret_cast<uintptr_t>(a.scratch) % 16 != 0 || a.scratch_floats < slabs * 4 * nst * kWbSlab * 4) return false;
  return true;
}

hipError_t launch_lmm_prod_bf16(const LmmArgs& a, hipStream_t st) {
  if (!lmm_prod_bf16_supported(a, 4, 0)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nst = (a.ck + 31) / 32;
  PbFn fn = nst <= 1 ? lmm_prod_bf16_kernel<1>
          : nst <= 2 ? lmm_prod_bf16_kernel<2>
          : nst <= 4 ? lmm_prod_bf16_kernel<4>
          : nst <= 7 ? lmm_prod_bf16_kernel<7> : lmm_prod_bf16_kernel<8>;
  const size_t lds_bytes = (size_t)4 * nst * kWbSlab * 16;
  if (lds_bytes > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int slabs = (a.ncols + kWbSlab - 1) / kWbSlab;
  const int per_cu = lds_bytes <= 48 * 1024 ? 2 : 1;          // workgroups of 512 threads a compute unit holds
  int64_t grid = (ntiles + kWbWaves - 1) / kWbWaves;
  grid = std::min<int64_t>(grid, std::max(1, per_cu * wb_cus() / slabs));   // one round of resident workgroups
  bf16x8* packed = reinterpret_cast<bf16x8*>(a.scratch);
  const int items = 4 * nst * kWbSlab;
  hipLaunchKernelGGL(lmm_pack_bf16_kernel, dim3((unsigned)((items + kBlock - 1) / kBlock), (unsigned)slabs), dim3(kBlock), 0, st, a, nst, packed);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid, (unsigned)slabs), dim3(kWbThreads), lds_bytes, st, a, nst, packed);
  return hipGetLastError();
}

// The float32 counterpart (same conditions; scratch of 8 KiB per 16 table columns and slab of 128 operand columns).
bool lmm_prod_f32_wide_supported(const LmmArgs& a, int vec, int mode) {
  if (mode != 0 || a.D == nullptr || vec != 4 || a.ck < 4 || a.ck % 4 != 0 || a.ck > 256) return false;
  if (a.g.n != 0 || a.grad_partial != nullptr || a.ncols < 1) return false;
  if (reinterpret_cast<uintptr_t>(a.D) % 16 != 0 || a.d_rows < a.r_out) return false;
  const int64_t nst = (a.ck + 15) / 16, slabs = (a.ncols + kFsSlab - 1) / kFsSlab;
  if (a.scratch == nullptr || reinterpret_cast<uintptr_t>(a.scratch) % 16 != 0 || a.scratch_floats < slabs * 4 * nst * kFsSlab * 4) return false;
  return true;
}

hipError_t launch_lmm_prod_f32_wide(const LmmArgs& a, hipStream_t st) {
  if (!lmm_prod_f32_wide_supported(a, 4, 0)) return hipErrorInvalidValue;
  if (a.r_out <= 0) return hipSuccess;
  const int nst = (a.ck + 15) / 16;
  PfFn fn = nst <= 2 ? lmm_prod_f32_wide_kernel<2>
          : nst <= 4 ? lmm_prod_f32_wide_kernel<4>
          : nst <= 8 ? lmm_prod_f32_wide_kernel<8>
          : nst <= 13 ? lmm_prod_f32_wide_kernel<13> : lmm_prod_f32_wide_kernel<16>;
  const size_t lds_bytes = (size_t)4 * nst * kFsSlab * 16;
  if (lds_bytes > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  const int64_t ntiles = (a.r_out + 15) / 16;
  const int slabs = (a.ncols + kFsSlab - 1) / kFsSlab;
  const int per_cu = lds_bytes <= 48 * 1024 ? 2 : 1;
  int64_t grid = (ntiles + kWbWaves - 1) / kWbWaves;
  grid = std::min<int64_t>(grid, std::max(1, per_cu * wb_cus() / slabs));
  float4* packed = reinterpret_cast<float4*>(a.scratch);
  const int items = 4 * nst * kFsSlab;
  hipLaunchKernelGGL(lmm_pack_f32_kernel, dim3((unsigned)((items + kBlock - 1) / kBlock), (unsigned)slabs), dim3(kBlock), 0, st, a, nst, packed);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, dim3((unsigned)grid, (unsigned)slabs), dim3(kWbThreads), lds_bytes, st, a, nst, packed);
  return hipGetLastError();
}

// Plain rows of both operands (no row gathers, no weights), whole aligned float4s, at most 256 columns each.
bool tred_stream_supported(const TredArgs& a) {
  if (a.ia != nullptr || a.ib != nullptr || a.wptr != nullptr || a.upper_only) return false;
  if (a.ca < 4 || a.ca > 256 || a.ca % 4 != 0 || a.lda % 4 != 0 || reinterpret_cast<uintptr_t>(a.A) % 16 != 0) return false;
  if (a.cb < 4 || a.cb > kWbSlab || a.cb % 4 != 0 || a.ldb % 4 != 0 || a.bcol0 % 4 != 0 || reinterpret_cast<uintptr_t>(a.B) % 16 != 0) return false;
  if (a.n_rows < 1 || a.a_rows < a.n_rows || a.b_rows < a.n_rows) return false;
  return true;
}

// Workgroups (= partial blocks of ca x cb floats) the launch will use within partial_floats; 0: does not fit.
int tred_stream_grid(const TredArgs& a, int64_t partial_floats) {
  const int64_t elems = (int64_t)a.ca * a.cb;
  int64_t grid = std::min<int64_t>(wb_cus(), (a.n_rows + kTsStepRows - 1) / kTsStepRows);
  grid = std::min<int64_t>(grid, partial_floats / elems);
  return (int)std::max<int64_t>(grid, 0);
}

hipError_t launch_tred_stream(TredArgs& a, int grid, bool bf16, hipStream_t st) {
  if (!tred_stream_supported(a) || grid < 1 || a.partial == nullptr) return hipErrorInvalidValue;
  a.rows_per_block = ((a.n_rows + grid - 1) / grid + kTsStepRows - 1) / kTsStepRows * kTsStepRows;
  const int used = (int)((a.n_rows + a.rows_per_block - 1) / a.rows_per_block);
  a.gx = used;
  const int mtc = (a.ca + 15) / 16, ntc = (a.cb + 15) / 16;
  if (!bf16) {
    const size_t lds_f32 = (size_t)2 * (16 * mtc + kWbSlab) * kTfLdr * sizeof(float);
    if (lds_f32 > 64 * 1024)
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tred_stream_f32_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_f32);
    hipLaunchKernelGGL(tred_stream_f32_kernel, dim3((unsigned)used), dim3(kWbThreads), lds_f32, st, a, mtc, ntc);
    return hipGetLastError();
  }
  const size_t lds_bytes = (size_t)2 * (4 * 16 * mtc + 4 * kWbSlab) * 16;
  if (lds_bytes > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tred_stream_bf16_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  hipLaunchKernelGGL(tred_stream_bf16_kernel, dim3((unsigned)used), dim3(kWbThreads), lds_bytes, st, a, mtc, ntc);
  return hipGetLastError();
}

}  // namespace ilargi
