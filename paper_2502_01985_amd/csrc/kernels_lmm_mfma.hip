// Left multiply on the matrix cores for operands with >= 8 columns:  P_k = D_k (M_k^T X)  and the assembly
// out[i,:] = D_S[i,:] X_S + sum_k P_k[row_idx_k[i], :]  (paper, Sec. 2.2), with the residual of Alg. 1 as an
// optional epilogue.
//
// A workgroup stages a block of whole table rows in LDS with fully coalesced float4 loads (the rows of a
// row-major table are one contiguous span) together with the selected operand rows X_k, then every wavefront
// multiplies 16-row tiles with MFMA 16x16x4 (float32).  Lane l = 16 q + i reads the four table values
// D[row i][16 step + 4 q + e], e = 0..3, as one 128-bit LDS read and uses them in four MFMAs whose K slot q
// stands for column 16 step + 4 q + e; the B operand comes from an LDS copy of X_k stored as [k / 4][n][k % 4]
// so that the matching four values are again one 128-bit read.
#include <algorithm>
#include <mutex>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float sigmoidf_stable(float z) {
  if (z >= 0.0f) return 1.0f / (1.0f + __expf(-z));
  float e = __expf(z);
  return e / (1.0f + e);
}

__device__ __forceinline__ float softplusf_stable(float z) {
  return fmaxf(z, 0.0f) + log1pf(__expf(-fabsf(z)));
}

// NT: 16-column tiles of the operand slab handled by one workgroup.  MODE as in the narrow kernel.
// BF16: table and operand values are rounded to bfloat16 (nearest even) when they enter the MFMA
// (16x16x32, eight K values per lane: lane 16 q + i holds columns 32 step + 8 q .. + 7), sums stay float32.
// SB: global loads a thread keeps in flight while it stages a tile (8, or 16 for tiles of more than 8 float4 per thread).
// JG > 0 (gradient-descent modes, one K chunk of at most 16 JG columns): the staged rows of D are used
// a second time while they sit in LDS, for this workgroup's share of  D^T E  (the fused source's block of
// T^T E, Alg. 1), written to grad_partial[blockIdx.x][ck][ld_grad].  The residual tile a lane has just formed
// (rows 4 q + r, operand column li) is exactly the B operand of an MFMA whose K slot q stands for row 4 q + r,
// so the four r values take four MFMAs per 16 table columns and the residuals never leave the registers.
// With BF16 both factors of this product are rounded to bfloat16 first, which the float32 MFMA then multiplies
// exactly, as the bfloat16 MFMA would.
template <int NT, int MODE, bool VEC4, bool BF16, int SB, int JG>
__global__ __launch_bounds__(kBlock) void lmm_mfma_kernel(LmmArgs a, MfmaShape sh) {
  extern __shared__ float lds[];
  float* As = lds;                                   // [rb][lda]
  float* Xs = lds + (size_t)sh.rb * sh.lda;          // [kc / 4][NT * 16][4]
  constexpr int N = NT * 16;
  float* Gs = Xs + (size_t)sh.kc * N;                // [rb][N] sums of the gathered product rows (if any)
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  const int n0 = a.col0 + blockIdx.y * N;
  const int nw = min(N, a.col0 + a.ncols - n0);       // live operand columns of this slab
  const int nchunks = (sh.kp + sh.kc - 1) / sh.kc;
  const int64_t nblocks = (a.r_out + sh.rb - 1) / sh.rb;
  float loss_local[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) loss_local[nt] = 0.0f;
  v4f gacc[JG > 0 ? JG : 1][NT];
  if constexpr (JG > 0) {
#pragma unroll
    for (int jt = 0; jt < JG; ++jt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) gacc[jt][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
  }

  auto store_x = [&](int k, int n, float x) {
    if constexpr (BF16) reinterpret_cast<__bf16*>(Xs)[((k >> 3) * N + n) * 8 + (k & 7)] = (__bf16)x;
    else Xs[((k >> 2) * N + n) * 4 + (k & 3)] = x;
  };
  const bool x_vec = (a.ldx % 4 == 0) && (n0 % 4 == 0) && (reinterpret_cast<uintptr_t>(a.X) % 16 == 0);
  auto load_x = [&](int k0, int kw) {
    // Xs <- X[colmap[k0 + k], n0 + n]  (zero beyond the table's columns / the slab).  An item is four
    // consecutive operand columns of one k; eight items per thread at a time: all col_map loads, then all
    // operand loads, then the LDS stores.
    constexpr int NQ = N / 4;
    const int items = kw * NQ;
    for (int e0 = tid; e0 < items; e0 += 8 * kBlock) {
      int tcol[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int e = e0 + u * kBlock;
        int k = e / NQ;
        tcol[u] = (e < items && k0 + k < a.ck) ? a.colmap[k0 + k] : -1;
      }
      float4 xv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int e = e0 + u * kBlock;
        int nq = e % NQ;
        xv[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (tcol[u] >= 0 && 4 * nq < nw) {
          const float* p = a.X + (int64_t)tcol[u] * a.ldx + n0 + 4 * nq;
          if (x_vec && 4 * nq + 3 < nw) {
            xv[u] = *reinterpret_cast<const float4*>(p);
          } else {
            xv[u].x = p[0];
            if (4 * nq + 1 < nw) xv[u].y = p[1];
            if (4 * nq + 2 < nw) xv[u].z = p[2];
            if (4 * nq + 3 < nw) xv[u].w = p[3];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int e = e0 + u * kBlock;
        if (e < items) {
          int k = e / NQ, n = 4 * (e - k * NQ);
          store_x(k, n, xv[u].x); store_x(k, n + 1, xv[u].y); store_x(k, n + 2, xv[u].z); store_x(k, n + 3, xv[u].w);
        }
      }
    }
  };

  if (nchunks == 1) load_x(0, sh.kp);

  for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const int64_t row0 = blk * sh.rb;
    v4f acc[NT];
    for (int c = 0; c < nchunks; ++c) {
      const int k0 = c * sh.kc;
      const int kw = min(sh.kc, sh.kp - k0);            // multiple of 16
      __syncthreads();                                   // previous tile fully consumed
      if (nchunks > 1) load_x(k0, kw);
      if (a.D != nullptr) {
        // rows [row0, row0 + rb) x columns [k0, k0 + kw) of D -> As, zero outside the table
        const int cols_here = max(0, min(kw, a.ck - k0));
        if constexpr (VEC4) {
          const int tpr = kw / 4;                        // float4 slots per row
          const int live4 = cols_here / 4;               // ck % 4 == 0 in this variant
          int r = tid / tpr, g = tid - r * tpr;
          const int dr = kBlock / tpr, dg = kBlock - dr * tpr;
          while (r < sh.rb) {
            // SB loads in flight per thread, then the LDS stores
            float4 v[SB];
            int rr[SB], gg[SB];
#pragma unroll
            for (int u = 0; u < SB; ++u) {
              rr[u] = r; gg[u] = g;
              v[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
              int64_t row = row0 + r;
              if (r < sh.rb && g < live4 && row < a.d_rows)
                v[u] = *reinterpret_cast<const float4*>(a.D + row * a.ck + k0 + 4 * g);
              r += dr; g += dg;
              if (g >= tpr) { g -= tpr; ++r; }
            }
#pragma unroll
            for (int u = 0; u < SB; ++u)
              if (rr[u] < sh.rb) *reinterpret_cast<float4*>(As + (size_t)rr[u] * sh.lda + 4 * gg[u]) = v[u];
          }
        } else {
          int r = tid / kw, g = tid - r * kw;
          const int dr = kBlock / kw, dg = kBlock - dr * kw;
          while (r < sh.rb) {
            float v[8];
            int rr[8], gg[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              rr[u] = r; gg[u] = g;
              v[u] = 0.0f;
              int64_t row = row0 + r;
              if (r < sh.rb && g < cols_here && row < a.d_rows) v[u] = a.D[row * a.ck + k0 + g];
              r += dr; g += dg;
              if (g >= kw) { g -= kw; ++r; }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (rr[u] < sh.rb) As[(size_t)rr[u] * sh.lda + gg[u]] = v[u];
          }
        }
      }
      if (a.g.n > 0 && c + 1 == nchunks) {
        // gathered rows of the other sources' products, summed into Gs: N/4 threads per target row, all
        // row-index loads of a batch first, then all product-row loads
        constexpr int QN = N / 4;                         // float4 slots per row
        constexpr int RPP = kBlock / QN;                  // rows per pass
        const int qn = tid % QN, r0 = tid / QN;
        const bool col_ok = 4 * qn < nw;
        const bool vec_ok = (a.g.ldp % 4 == 0) && (n0 % 4 == 0) && (4 * qn + 3 < nw);
        for (int rbase = 0; rbase < sh.rb; rbase += 4 * RPP) {
          float4 gsum[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) gsum[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
          for (int s = 0; s < a.g.n; ++s) {
            int64_t j[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              int r = rbase + u * RPP + r0;
              int64_t row = row0 + r;
              j[u] = -1;
              if (r < sh.rb && row < a.r_out && col_ok) {
                if (a.g.idx[s] != nullptr) j[u] = a.g.idx[s][row];
                else j[u] = (row < a.g.rows[s]) ? row : -1;
              }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (j[u] >= 0) {
                const float* p = a.g.P[s] + j[u] * a.g.ldp + n0 + 4 * qn;
                if (vec_ok) {
                  float4 t = *reinterpret_cast<const float4*>(p);
                  gsum[u].x += t.x; gsum[u].y += t.y; gsum[u].z += t.z; gsum[u].w += t.w;
                } else {
                  gsum[u].x += p[0];
                  if (4 * qn + 1 < nw) gsum[u].y += p[1];
                  if (4 * qn + 2 < nw) gsum[u].z += p[2];
                  if (4 * qn + 3 < nw) gsum[u].w += p[3];
                }
              }
            }
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            int r = rbase + u * RPP + r0;
            if (r < sh.rb) *reinterpret_cast<float4*>(Gs + (size_t)r * N + 4 * qn) = gsum[u];
          }
        }
      }
      __syncthreads();
      // each wavefront walks its 16-row tiles of the block
      const int tiles = sh.rb / 16;
      for (int mt = wave; mt < tiles; mt += kBlock / kWave) {
        if (c == 0) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) acc[nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        }
        if constexpr (BF16) {
          if (a.D != nullptr) {
            const float* arow = As + (size_t)(mt * 16 + li) * sh.lda + 8 * q;
            for (int step = 0; step < kw / 32; ++step) {
              float4 a0 = *reinterpret_cast<const float4*>(arow + 32 * step);
              float4 a1 = *reinterpret_cast<const float4*>(arow + 32 * step + 4);
              bf16x8 av;
              av[0] = (__bf16)a0.x; av[1] = (__bf16)a0.y; av[2] = (__bf16)a0.z; av[3] = (__bf16)a0.w;
              av[4] = (__bf16)a1.x; av[5] = (__bf16)a1.y; av[6] = (__bf16)a1.z; av[7] = (__bf16)a1.w;
              const bf16x8* xb = reinterpret_cast<const bf16x8*>(Xs) + (size_t)(4 * step + q) * N + li;
#pragma unroll
              for (int nt = 0; nt < NT; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, xb[nt * 16], acc[nt], 0, 0, 0);
            }
          }
        } else if (a.D != nullptr) {
          const float* arow = As + (size_t)(mt * 16 + li) * sh.lda + 4 * q;
          for (int step = 0; step < kw / 16; ++step) {
            float4 av = *reinterpret_cast<const float4*>(arow + 16 * step);
            const float* xb = Xs + ((size_t)(4 * step + q) * N + li) * 4;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              float4 bv = *reinterpret_cast<const float4*>(xb + nt * 64);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, acc[nt], 0, 0, 0);
            }
          }
        }
        if (c + 1 < nchunks) continue;                   // (multi-chunk blocks have one tile per wavefront)
        // epilogue: rows 4 q + r of the tile, operand column li of each 16-column tile
        float ov[NT][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int64_t row = row0 + mt * 16 + 4 * q + r;
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) ov[nt][r] = 0.0f;
          if (row >= a.r_out) continue;
          float g[NT];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            g[nt] = a.g.n > 0 ? Gs[(size_t)(mt * 16 + 4 * q + r) * N + nt * 16 + li] : 0.0f;
          float yi = 0.0f;
          if constexpr (MODE != 0) yi = a.y[row];
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (nt * 16 + li < nw) {
              float z = acc[nt][r] + g[nt];
              float o = z;
              if constexpr (MODE == 1) {
                o = z - yi;
                loss_local[nt] = fmaf(o, o, loss_local[nt]);
              } else if constexpr (MODE == 2) {
                o = sigmoidf_stable(z) - yi;
                loss_local[nt] += softplusf_stable(z) - yi * z;
              }
              if constexpr (BF16 && JG > 0) ov[nt][r] = (float)(__bf16)o;
              else ov[nt][r] = o;
              float* op = a.out + row * a.ldo + n0 + nt * 16 + li;
              if (a.nt_out) __builtin_nontemporal_store(o, op);
              else *op = o;
            }
          }
        }
        if constexpr (JG > 0) {
          // D^T E of the tile: A operand = table column 16 jt + li of row 4 q + r (zero beyond the table: the
          // staging zero-fills), B operand = the residual just formed (zero for rows and columns outside)
          const float* acol = As + (size_t)(mt * 16 + 4 * q) * sh.lda + li;
#pragma unroll
          for (int jt = 0; jt < JG; ++jt) {
            if (jt * 16 < sh.kp) {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                float av = acol[(size_t)r * sh.lda + jt * 16];
                if constexpr (BF16) av = (float)(__bf16)av;   // products of two bfloat16 values are exact in float32
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                  gacc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, ov[nt][r], gacc[jt][nt], 0, 0, 0);
              }
            }
          }
        }
      }
    }
  }

  if constexpr (JG > 0) {
    // the four wavefronts' shares, added in wavefront order in LDS (over the staging area, now idle)
    float* red = lds;
    for (int w = 0; w < kBlock / kWave; ++w) {
      __syncthreads();
      if (wave == w) {
#pragma unroll
        for (int jt = 0; jt < JG; ++jt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              float* p = red + (size_t)(jt * 16 + 4 * q + r) * N + nt * 16 + li;
              if (w == 0) *p = gacc[jt][nt][r];
              else *p += gacc[jt][nt][r];
            }
      }
    }
    __syncthreads();
    for (int e = tid; e < a.ck * N; e += kBlock) {
      const int j = e / N, n = e - j * N;
      if (n < nw) a.grad_partial[((int64_t)blockIdx.x * a.ck + j) * a.ld_grad + n0 + n] = red[e];
    }
    __syncthreads();
  }

  if constexpr (MODE != 0) {
    // per-column loss of this workgroup: the four row groups of a wavefront, then the wavefronts in order
    __shared__ float lsum[kBlock / kWave][N];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float s = loss_local[nt];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (q == 0) lsum[wave][nt * 16 + li] = s;
    }
    __syncthreads();
    if (tid < nw) {
      float s = 0.0f;
      for (int w = 0; w < kBlock / kWave; ++w) s += lsum[w][tid];
      a.loss_partial[(int64_t)blockIdx.x * a.ld_loss + n0 + tid] = s;
    }
  }
}

// Plain product  P = D (M^T X)  for wide operands (slabs of 64 columns), float32: a workgroup forms a 128 x 64 block
// of P, a wavefront 32 x 64 of it (eight 16 x 16 accumulators).  The table and the operand pass through LDS in K
// chunks of 32 columns, double-buffered: the next chunk is on its way from memory into registers while the matrix
// cores work on the current one, and one workgroup barrier per chunk separates them.  Both operands are stored so
// that one 128-bit LDS read feeds four MFMAs: lane (li, q) reads columns 4 q .. 4 q + 3 of its row (MFMA c takes
// component c, K slot q = column 4 q + c of the 16-column group), and the operand chunk is kept as
// [group][q][column][c].  With 26 KiB per buffer three workgroups share a compute unit, where the general kernel
// above keeps the whole 208 x 64 operand slab in LDS and runs alone.
constexpr int kGemmBM = 128, kGemmBN = 64, kGemmKC = 32;
constexpr int kGemmLda = kGemmKC + 4;                          // 36: rows 16 bytes aligned, 128-bit reads conflict-free
constexpr int kGemmStage = kGemmBM * kGemmLda + kGemmKC * kGemmBN;   // floats per buffer

__global__ __launch_bounds__(kBlock) void lmm_gemm_kernel(LmmArgs a, MfmaShape sh) {
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  // Workgroup ids go round-robin over the 8 XCDs, each with an L2 of its own: the column slabs of one block of
  // rows get ids that are 8 apart, so they run on the same XCD at about the same time and the block of rows comes
  // from memory once.  sh.rb = number of column slabs, sh.kp = number of row blocks.
  const int gy = sh.rb;
  const int64_t grp = blockIdx.x / (8 * gy);
  const int within = (int)(blockIdx.x - grp * (8 * gy));
  const int64_t rblock = grp * 8 + within % 8;
  if (rblock >= sh.kp) return;
  const int64_t row0 = rblock * kGemmBM;
  const int n0 = (within / 8) * kGemmBN;
  const int nw = min(kGemmBN, a.ncols - n0);
  const int nch = (a.ck + kGemmKC - 1) / kGemmKC;
  const bool x_vec = (a.ldx % 4 == 0) && ((a.col0 + n0) % 4 == 0) && (reinterpret_cast<uintptr_t>(a.X) % 16 == 0);

  // staging slots of this thread: table (row ar + 32 u, float4 ac of the chunk), operand (k row bk + 16 u, float4 bn)
  const int ar = tid / 8, ac = tid % 8;                        // 32 rows x 8 float4 per pass, 4 passes
  const int bk = tid / 16, bn = tid % 16;                      // 16 k rows x 16 float4 per pass, 2 passes
  float4 va[4], vb[2];
  unsigned dead = 0;                                           // values of the chunk in flight that must read as zero
  // branch-free in the common case (whole slab, float4 operand rows): values nobody needs are read from the
  // start of the buffer and replaced by zero, so that all six loads of a chunk are in flight together
  const bool fastb = x_vec && nw == kGemmBN;
  auto fetch = [&](int ch) {
    const int k0 = ch * kGemmKC;
    dead = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t row = row0 + ar + 32 * u;
      const int col = k0 + 4 * ac;
      const bool ok = row < a.d_rows && col < a.ck;
      va[u] = *reinterpret_cast<const float4*>(ok ? a.D + row * a.ck + col : a.D);
      if (!ok) dead |= 1u << u;
    }
    if (fastb) {
      int t[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) t[u] = a.colmap[min(k0 + bk + 16 * u, a.ck - 1)];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bool ok = k0 + bk + 16 * u < a.ck && t[u] >= 0;
        vb[u] = *reinterpret_cast<const float4*>(ok ? a.X + (int64_t)t[u] * a.ldx + a.col0 + n0 + 4 * bn : a.X);
        if (!ok) dead |= 16u << u;
      }
    } else {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int k = k0 + bk + 16 * u;
        vb[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        const int t = k < a.ck ? a.colmap[k] : -1;
        if (t >= 0 && 4 * bn < nw) {
          const float* p = a.X + (int64_t)t * a.ldx + a.col0 + n0 + 4 * bn;
          vb[u].x = p[0];
          if (4 * bn + 1 < nw) vb[u].y = p[1];
          if (4 * bn + 2 < nw) vb[u].z = p[2];
          if (4 * bn + 3 < nw) vb[u].w = p[3];
        }
      }
    }
  };
  auto stash = [&](int buf) {
    float* As = lds + (size_t)buf * kGemmStage;
    float* Bs = As + kGemmBM * kGemmLda;
#pragma unroll
    for (int u = 0; u < 4; ++u)
      *reinterpret_cast<float4*>(As + (ar + 32 * u) * kGemmLda + 4 * ac) = (dead >> u & 1u) ? make_float4(0.0f, 0.0f, 0.0f, 0.0f) : va[u];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int kk = bk + 16 * u;                              // k within the chunk: group kk / 16, slot (kk % 16) / 4, c kk % 4
      float* b = Bs + ((kk / 16) * 4 + (kk % 16) / 4) * (kGemmBN * 4) + (kk % 4);
      const float4 bz = (dead >> (4 + u) & 1u) ? make_float4(0.0f, 0.0f, 0.0f, 0.0f) : vb[u];
      const float x4[4] = {bz.x, bz.y, bz.z, bz.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) b[(4 * bn + c) * 4] = x4[c];
    }
  };

  v4f acc[2][4];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[t][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  auto compute = [&](int ch) {
    const int buf = ch & 1;
    const float* As = lds + (size_t)buf * kGemmStage;
    const float4* Bs4 = reinterpret_cast<const float4*>(As + kGemmBM * kGemmLda);
    const int groups = min(2, (a.ck - ch * kGemmKC + 15) / 16);  // 16-column groups of this chunk that hold columns
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      if (g < groups) {
        float4 av[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
          av[t] = *reinterpret_cast<const float4*>(As + (32 * wave + 16 * t + li) * kGemmLda + 16 * g + 4 * q);
        float4 b[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) b[nt] = Bs4[(g * 4 + q) * kGemmBN + 16 * nt + li];
        // eight independent accumulators between two MFMAs on the same one
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
              const float ax = c == 0 ? av[t].x : (c == 1 ? av[t].y : (c == 2 ? av[t].z : av[t].w));
              const float bx = c == 0 ? b[nt].x : (c == 1 ? b[nt].y : (c == 2 ? b[nt].z : b[nt].w));
              acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(ax, bx, acc[t][nt], 0, 0, 0);
            }
      }
    }
  };
  // chunk ch in LDS; chunk ch + 1 is requested before the MFMAs of chunk ch and stored after them
  fetch(0);
  stash(0);
  __syncthreads();
  for (int ch = 0; ch < nch; ++ch) {
    if (ch + 1 < nch) fetch(ch + 1);
    compute(ch);
    if (ch + 1 < nch) stash((ch + 1) & 1);
    __syncthreads();
  }
  // the wavefront's 32 x 64 block through LDS (its own 8 KiB of the idle buffers), so that rows leave as float4
  float* Cs = lds + (size_t)wave * (32 * kGemmBN);
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) Cs[(16 * t + 4 * q + r) * kGemmBN + 16 * nt + li] = acc[t][nt][r];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  const bool o_vec = (a.ldo % 4 == 0) && ((a.col0 + n0) % 4 == 0) && (reinterpret_cast<uintptr_t>(a.out) % 16 == 0);
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int r = 4 * it + q;                                  // 4 rows per pass, 16 lanes x float4 = one 256-byte row
    const int64_t orow = row0 + 32 * wave + r;
    if (orow < a.r_out && 4 * li < nw) {
      const float4 v = *reinterpret_cast<const float4*>(Cs + r * kGemmBN + 4 * li);
      float* p = a.out + orow * a.ldo + a.col0 + n0 + 4 * li;
      if (o_vec && 4 * li + 3 < nw) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 o = {v.x, v.y, v.z, v.w};
        if (a.nt_out) __builtin_nontemporal_store(o, reinterpret_cast<f4*>(p));
        else *reinterpret_cast<f4*>(p) = o;
      } else {
        p[0] = v.x;
        if (4 * li + 1 < nw) p[1] = v.y;
        if (4 * li + 2 < nw) p[2] = v.z;
        if (4 * li + 3 < nw) p[3] = v.w;
      }
    }
  }
}

}  // namespace

// Shape decisions shared with the caller: K padding, K chunking, rows per block, LDS bytes.
MfmaShape lmm_mfma_shape(int ck, int nt, bool gathers, bool bf16) {
  MfmaShape sh;
  const int kq = bf16 ? 32 : 16;                      // K values one MFMA step consumes
  sh.kp = ck > 0 ? (ck + kq - 1) / kq * kq : kq;
  sh.kc = sh.kp <= 256 ? sh.kp : 256;
  sh.lda = sh.kc + 4;
  const int n = nt * 16;
  const size_t x_floats = (size_t)sh.kc * n;
  int rm = 1;
  if (sh.kp == sh.kc) {
    // several 16-row tiles per wavefront when rows are short, so that a block moves tens of KiB per barrier
    while (rm < 8 && (size_t)(2 * rm) * 64 * (sh.lda + (gathers ? n : 0)) * 4 + x_floats * 4 <= 48 * 1024) rm *= 2;
  }
  sh.rb = 64 * rm;
  sh.lds_bytes = ((size_t)sh.rb * sh.lda + x_floats + (gathers ? (size_t)sh.rb * n : 0)) * sizeof(float);
  return sh;
}

namespace {

typedef void (*MfmaFn)(LmmArgs, MfmaShape);

template <int NT, int MODE>
MfmaFn pick_plain(bool vec4, bool bf16, bool sb16) {
  if (vec4 && bf16) return sb16 ? lmm_mfma_kernel<NT, MODE, true, true, 16, 0> : lmm_mfma_kernel<NT, MODE, true, true, 8, 0>;
  if (vec4) return sb16 ? lmm_mfma_kernel<NT, MODE, true, false, 16, 0> : lmm_mfma_kernel<NT, MODE, true, false, 8, 0>;
  if (bf16) return sb16 ? lmm_mfma_kernel<NT, MODE, false, true, 16, 0> : lmm_mfma_kernel<NT, MODE, false, true, 8, 0>;
  return sb16 ? lmm_mfma_kernel<NT, MODE, false, false, 16, 0> : lmm_mfma_kernel<NT, MODE, false, false, 8, 0>;
}

template <int NT>
MfmaFn pick_mode(int mode, bool vec4, bool bf16, bool sb16) {
  if (mode == 0) return pick_plain<NT, 0>(vec4, bf16, sb16);
  if (mode == 1) return pick_plain<NT, 1>(vec4, bf16, sb16);
  return pick_plain<NT, 2>(vec4, bf16, sb16);
}

// fused gradient: 64-column slabs, tables of at most 64 columns (a tile of at most 8 float4 per thread)
template <int MODE, bool B>
MfmaFn pick_fused(bool vec4, int jg) {
  if (vec4) return jg == 2 ? lmm_mfma_kernel<4, MODE, true, B, 8, 2> : lmm_mfma_kernel<4, MODE, true, B, 8, 4>;
  return jg == 2 ? lmm_mfma_kernel<4, MODE, false, B, 8, 2> : lmm_mfma_kernel<4, MODE, false, B, 8, 4>;
}

// Workgroups of this kernel and LDS size the device holds at once (cached: the query costs more than a launch).
int resident_workgroups(MfmaFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;   // the cache below is shared by every plan of the process
  std::lock_guard<std::mutex> lock(cache_mutex);
  static int cus = 0;
  static MfmaFn seen_fn[128];
  static size_t seen_lds[128];
  static int seen_occ[128];
  static int n_seen = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    cus = 256;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      cus = prop.multiProcessorCount;
  }
  for (int i = 0; i < n_seen; ++i)
    if (seen_fn[i] == fn && seen_lds[i] == lds_bytes) return seen_occ[i] * cus;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, lds_bytes) != hipSuccess || per_cu < 1)
    per_cu = 1;
  if (n_seen < 128) { seen_fn[n_seen] = fn; seen_lds[n_seen] = lds_bytes; seen_occ[n_seen] = per_cu; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// The fused D^T E needs a 64-column slab shape and a table of at most 64 columns (one K chunk).
bool lmm_mfma_can_fuse_gradient(int ck, int ncols, bool bf16) {
  (void)bf16;
  return ncols > 32 && ck > 0 && ck <= 64;
}

hipError_t launch_lmm_mfma(const LmmArgs& a, int vec, int mode, bool bf16, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (a.r_out <= 0 || a.ncols <= 0) return hipSuccess;
  const int nt = a.ncols <= 16 ? 1 : (a.ncols <= 32 ? 2 : 4);
  MfmaShape sh = lmm_mfma_shape(a.ck, nt, a.g.n > 0, bf16);
  const bool vec4 = vec == 4;
  const bool sb16 = vec4 && (int64_t)sh.rb * (sh.kc / 4) > 8 * kBlock;
  MfmaFn fn;
  // plain product with bfloat16 inputs and a wide operand: the whole operand slab in LDS, table rows streamed
  if (bf16 && a.ncols >= 64 && lmm_prod_bf16_supported(a, vec, mode)) return launch_lmm_prod_bf16(a, st);
  // the same in float32 (slabs of 128 columns)
  if (!bf16 && a.ncols >= 64 && lmm_prod_f32_wide_supported(a, vec, mode)) return launch_lmm_prod_f32_wide(a, st);
  // plain product with at most 16 result columns (no gathers, no epilogue): the streaming kernel
  if (!bf16 && nt == 1 && lmm_prod_stream_supported(a, vec, mode)) return launch_lmm_prod_stream(a, st);
  // wide plain product (no gathers, no epilogue): the chunked, double-buffered kernel
  if (mode == 0 && !bf16 && a.g.n == 0 && a.D != nullptr && a.grad_partial == nullptr && nt == 4 && vec4) {
    const size_t lds_bytes = (size_t)2 * kGemmStage * sizeof(float);
    const int64_t gxm = (a.r_out + kGemmBM - 1) / kGemmBM;
    const int gyn = (a.ncols + kGemmBN - 1) / kGemmBN;
    const int64_t total = (gxm + 7) / 8 * 8 * gyn;
    if (gxm <= 0x7fffffff && total <= 0x7fffffff) {
      sh.kp = (int)gxm;
      sh.rb = gyn;
      if (grid_out) *grid_out = (int)gxm;
      hipLaunchKernelGGL(lmm_gemm_kernel, dim3((unsigned)total), dim3(kBlock), lds_bytes, st, a, sh);
      return hipGetLastError();
    }
  }
  if (a.grad_partial != nullptr) {
    if (mode == 0 || a.D == nullptr || !lmm_mfma_can_fuse_gradient(a.ck, a.ncols, bf16)) return hipErrorInvalidValue;
    const int jg = sh.kp <= 32 ? 2 : 4;
    sh.lds_bytes = std::max(sh.lds_bytes, (size_t)jg * 16 * 64 * sizeof(float));   // the wavefronts' sum
    if (bf16) fn = mode == 1 ? pick_fused<1, true>(vec4, jg) : pick_fused<2, true>(vec4, jg);
    else fn = mode == 1 ? pick_fused<1, false>(vec4, jg) : pick_fused<2, false>(vec4, jg);
  } else if (nt == 1) {
    fn = pick_mode<1>(mode, vec4, bf16, sb16);
  } else if (nt == 2) {
    fn = pick_mode<2>(mode, vec4, bf16, sb16);
  } else {
    fn = pick_mode<4>(mode, vec4, bf16, sb16);
  }
  if (sh.lds_bytes > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh.lds_bytes);
  const int64_t nblocks = (a.r_out + sh.rb - 1) / sh.rb;
  const int gy = (a.ncols + nt * 16 - 1) / (nt * 16);
  // wide slabs stage tens of KiB of operand per workgroup: give each workgroup several row blocks; every
  // workgroup does the same work, so the launch is kept within one round of the device's workgroup slots
  int64_t gx = std::min<int64_t>(nblocks, nt == 4 ? 256 : 1024);
  const int64_t slots = resident_workgroups(fn, sh.lds_bytes);
  if (gx * gy > slots) gx = std::max<int64_t>(1, slots / gy);
  if (grid_out) *grid_out = (int)gx;
  hipLaunchKernelGGL(fn, dim3((unsigned)gx, (unsigned)gy), dim3(kBlock), sh.lds_bytes, st, a, sh);
  return hipGetLastError();
}

}  // namespace ilargi
