// One gradient-descent pass (Alg. 1) over a two-table star join  T = [S | I_R R]  for a batch of more than 32
// models, without ever writing the r_T x m residual:
//
//   for every target row i:   e_i = f(S[i,:] W_S + P[fk(i),:]) - y_i          (P = R W_R, formed beforehand)
//   G_S  = S^T E              (per-workgroup partials)
//   Z[j] = sum of e_i over the rows i that join row j of R                    (the segment sums  I_R^T E)
//
// The pass walks the target rows in the order of the inverse index (grouped by the row of R they join), so a
// wavefront owns 16 consecutive rows of R at a time together with all target rows that join them: their rows
// of P are one contiguous 16-row tile (read once, kept in LDS), and the segment sums stay in registers until
// the tile is finished.  All three products run on the matrix cores (MFMA 16x16x4 float32, or 16x16x32
// bfloat16 for S W_S); the residual tile a lane has just formed is, as it stands, the B operand of
//   S^T E :  A = the staged table values of rows 4 q + r,
//   Z     :  A = 1 where row 4 q + r joins row li of the tile of R, else 0  (so each sum is exact in float32).
// Z overwrites P in place: a wavefront reads its P tile before it writes the same rows and columns of Z.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "ilargi_internal.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float star_sigmoid(float z) {
  if (z >= 0.0f) return 1.0f / (1.0f + __expf(-z));
  float e = __expf(z);
  return e / (1.0f + e);
}

__device__ __forceinline__ float star_softplus(float z) {
  return fmaxf(z, 0.0f) + log1pf(__expf(-fabsf(z)));
}

// LDS writes of some lanes of a wavefront become visible to the others (one wavefront executes its LDS
// instructions in order; the fences only keep the compiler from moving accesses across this point).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kN = 64;        // model columns per workgroup (four 16-column tiles)
constexpr int kNT = 4;
constexpr int kWaves = kBlock / kWave;

// MODE 1: linear, 2: logistic.  VEC4: rows of S are read as float4.  BF16: values of S, W and E are rounded
// to bfloat16 (nearest even) where they enter a product.  JG: 16-column tiles of S (kp / 16 rounded to 2 or 4).
// ST: target rows a wavefront stages at a time (32 or 64).
template <int MODE, bool VEC4, bool BF16, int JG, int ST>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(VEC4 ? (JG == 2 && !BF16 ? 3 : 2) : (JG == 2 ? 2 : 1)))) void gd_star_kernel(StarArgs a, int kp, int lda, int rtiles, int fold) {
  extern __shared__ float lds[];
  float* Xs = lds;                                            // [kp / 4][64][4]  (bf16: [kp / 8][64][8])
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  float* wbase = lds + (size_t)kp * kN + (size_t)wave * ((size_t)ST * lda + 16 * kN + 3 * ST);
  float* As = wbase;                                          // [ST][lda] staged rows of S
  float* Ps = As + (size_t)ST * lda;                          // [16][64] tile of P, later of Z
  int* iS = reinterpret_cast<int*>(Ps + 16 * kN);             // [ST] target row of each staged row
  int* jS = iS + ST;                                          // [ST] row of the R tile it joins (-1: none)
  float* yS = reinterpret_cast<float*>(jS + ST);              // [ST] label
  const int n0 = blockIdx.y * kN;
  const int nw = min(kN, a.m - n0);
  // fold: the table has 1..4 columns beyond whole groups of 16.  A tile of R then has 12 rows, and rows 12..15
  // of the segment-sum MFMA (whose A operand is the 0/1 indicator) carry those columns of S instead, so the
  // same MFMA forms their share of S^T E; they are collected in the last gacc slot by the lanes q == 3.
  const int tr = fold ? 12 : 16;                              // rows of R per tile
  const int full = a.cs / 16;
  const int njt = fold ? full : kp / 16;                      // 16-column groups of S that take their own MFMAs

  // W rows of S's columns -> Xs (shared by the workgroup)
  {
    const bool x_vec = (a.ldw % 4 == 0) && (reinterpret_cast<uintptr_t>(a.W) % 16 == 0);
    constexpr int NQ = kN / 4;
    for (int e = tid; e < kp * NQ; e += kBlock) {
      const int k = e / NQ, nq = e - k * NQ;
      float4 xv = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (k < a.cs && 4 * nq < nw) {
        const float* p = a.W + (int64_t)a.s_colmap[k] * a.ldw + n0 + 4 * nq;
        if (x_vec && 4 * nq + 3 < nw) {
          xv = *reinterpret_cast<const float4*>(p);
        } else {
          xv.x = p[0];
          if (4 * nq + 1 < nw) xv.y = p[1];
          if (4 * nq + 2 < nw) xv.z = p[2];
          if (4 * nq + 3 < nw) xv.w = p[3];
        }
      }
      const float x4[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int n = 4 * nq + c;
        if constexpr (BF16) reinterpret_cast<__bf16*>(Xs)[((k >> 3) * kN + n) * 8 + (k & 7)] = (__bf16)x4[c];
        else Xs[((k >> 2) * kN + n) * 4 + (k & 3)] = x4[c];
      }
    }
  }
  __syncthreads();

  float loss_local[kNT];
  v4f gacc[JG][kNT];
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) loss_local[nt] = 0.0f;
#pragma unroll
  for (int jt = 0; jt < JG; ++jt)
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) gacc[jt][nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  // staging slots of this lane: (row of the batch, float4 or scalar column slot), the same for every batch
  typedef typename std::conditional<VEC4, float4, float>::type SVal;
  constexpr int NV = VEC4 ? ST * JG / 16 : ST * JG / 4;
  const int gslots = VEC4 ? kp / 4 : kp;                      // slots per staged row
  const int glive = VEC4 ? a.cs / 4 : a.cs;                   // slots inside the table (cs % 4 == 0 with VEC4)
  int rr[NV], gg[NV];
  {
    int r = lane / gslots, g = lane - r * gslots;
    const int dr = kWave / gslots, dg = kWave - dr * gslots;
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      rr[u] = r; gg[u] = g;
      r += dr; g += dg;
      if (g >= gslots) { g -= gslots; ++r; }
    }
  }

  const float* Sb = a.Sp != nullptr ? a.Sp : a.S;
  const bool p_vec = (a.ldp % 4 == 0) && (reinterpret_cast<uintptr_t>(a.PZ) % 16 == 0);
  const int pr = lane / 16, pq = lane % 16;                   // (row mod 4, float4 slot) of the P / Z tile this lane moves

  for (int rt = blockIdx.x * kWaves + wave; rt < rtiles; rt += gridDim.x * kWaves) {
    const int64_t jb = (int64_t)rt * tr;
    const int p_begin = a.rowptr[jb];
    const int p_end = a.rowptr[min(jb + tr, a.r_R)];
    wave_sync();                                              // the previous tile's Z has left Ps
    // P tile -> Ps (zero beyond the table and the slab)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = pr + 4 * u;
      float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (r < tr && jb + r < a.r_R && 4 * pq < nw) {
        const float* p = a.PZ + (jb + r) * a.ldp + n0 + 4 * pq;
        if (p_vec && 4 * pq + 3 < nw) {
          v = *reinterpret_cast<const float4*>(p);
        } else {
          v.x = p[0];
          if (4 * pq + 1 < nw) v.y = p[1];
          if (4 * pq + 2 < nw) v.z = p[2];
          if (4 * pq + 3 < nw) v.w = p[3];
        }
      }
      *reinterpret_cast<float4*>(Ps + r * kN + 4 * pq) = v;
    }
    v4f zacc[kNT];
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt) zacc[nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

    // Batches of ST target rows, one ahead: while the matrix cores work on a batch, the next batch's rows of
    // S (registers), its row numbers / labels and the row list of the batch after that are already on their way.
    // the row of the table entry p of the inverse index stands for, its key and its label: through the target row,
    // or straight from the join-ordered copy of the table (and of the labels) when the plan keeps one
    auto row_at = [&](int p) { return a.Sp != nullptr ? p : a.perm[p]; };
    auto key_at = [&](int r) { return a.Sp != nullptr ? a.keys[r] : a.idx[r]; };
    auto label_at = [&](int r) { return a.Sp == nullptr ? a.y[r] : (a.yp != nullptr ? a.yp[r] : a.y[a.perm[r]]); };
    int pi = (lane < ST && p_begin + lane < p_end) ? row_at(p_begin + lane) : -1;
    int pi_next = (lane < ST && p_begin + ST + lane < p_end) ? row_at(p_begin + ST + lane) : -1;
    int jl = -1;
    float yv = 0.0f;
    if (pi >= 0) {
      jl = key_at(pi) - (int)jb;
      yv = label_at(pi);
    }
    wave_sync();                                              // the previous tile's batches are consumed
    if (lane < ST) iS[lane] = pi;
    wave_sync();
    SVal sv[NV];
    auto load_rows = [&](int cnt_rows) {
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        if constexpr (VEC4) sv[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        else sv[u] = 0.0f;
        if (rr[u] < cnt_rows && gg[u] < glive) {
          const int64_t row = iS[rr[u]];
          if constexpr (VEC4) sv[u] = *reinterpret_cast<const float4*>(Sb + row * a.cs + 4 * gg[u]);
          else sv[u] = Sb[row * a.cs + gg[u]];
        }
      }
    };
    load_rows(min(ST, p_end - p_begin));
    for (int p0 = p_begin; p0 < p_end; p0 += ST) {
      const int cnt = min(ST, p_end - p0);
      const int cnt_next = max(0, min(ST, p_end - p0 - ST));
      wave_sync();                                            // the previous batch is consumed
      if (lane < ST) { jS[lane] = jl; yS[lane] = yv; iS[lane] = pi_next; }
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        if (rr[u] < ST) {
          if constexpr (VEC4) *reinterpret_cast<float4*>(As + (size_t)rr[u] * lda + 4 * gg[u]) = sv[u];
          else As[(size_t)rr[u] * lda + gg[u]] = sv[u];
        }
      }
      wave_sync();
      // next batch: row numbers and labels, rows of S; the row list of the batch after it
      pi = pi_next;
      pi_next = (lane < ST && p0 + 2 * ST + lane < p_end) ? row_at(p0 + 2 * ST + lane) : -1;
      jl = -1;
      yv = 0.0f;
      if (pi >= 0) {
        jl = key_at(pi) - (int)jb;
        yv = label_at(pi);
      }
      load_rows(cnt_next);

      // residual tile t of the batch: ov[nt][r] = residual of row 4 q + r, model column li of tile nt (rounded to
      // bfloat16 with BF16), ind[r] = the indicator (or folded table) value of that row for row li of the tile of R
      auto residual_tile = [&](int t, float (&ov)[kNT][4], float (&ind)[4]) {
        // z tile = S rows x W_S
        v4f acc[kNT];
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt) acc[nt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (BF16) {
          const float* arow = As + (size_t)(t * 16 + li) * lda + 8 * q;
          for (int step = 0; step < kp / 32; ++step) {
            float4 a0 = *reinterpret_cast<const float4*>(arow + 32 * step);
            float4 a1 = *reinterpret_cast<const float4*>(arow + 32 * step + 4);
            bf16x8 av;
            av[0] = (__bf16)a0.x; av[1] = (__bf16)a0.y; av[2] = (__bf16)a0.z; av[3] = (__bf16)a0.w;
            av[4] = (__bf16)a1.x; av[5] = (__bf16)a1.y; av[6] = (__bf16)a1.z; av[7] = (__bf16)a1.w;
            const bf16x8* xb = reinterpret_cast<const bf16x8*>(Xs) + (size_t)(4 * step + q) * kN + li;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, xb[nt * 16], acc[nt], 0, 0, 0);
          }
        } else {
          // whole groups of 16 table columns: one 128-bit read feeds four MFMAs; the remaining columns in
          // groups of four (K slot q = column kb + q), so that 20 columns cost 20 MFMAs per tile, not 32
          const float* arow = As + (size_t)(t * 16 + li) * lda + 4 * q;
          for (int kb = 16 * full; kb < a.cs; kb += 4) {
            const float av = As[(size_t)(t * 16 + li) * lda + kb + q];
            const float* xb = Xs + ((size_t)(kb >> 2) * kN + li) * 4 + q;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, xb[nt * 64], acc[nt], 0, 0, 0);
          }
          for (int step = 0; step < full; ++step) {
            float4 av = *reinterpret_cast<const float4*>(arow + 16 * step);
            const float* xb = Xs + ((size_t)(4 * step + q) * kN + li) * 4;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt) {
              float4 bv = *reinterpret_cast<const float4*>(xb + nt * 64);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.x, bv.x, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.y, bv.y, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.z, bv.z, acc[nt], 0, 0, 0);
              acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av.w, bv.w, acc[nt], 0, 0, 0);
            }
          }
        }
        // residual of rows 4 q + r, model column li of each 16-column tile
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = t * 16 + 4 * q + r;
          const int j = jS[row];                              // -1 beyond the batch
          const float yi = yS[row];
          ind[r] = j == li ? 1.0f : 0.0f;
          if (fold && li >= 12) {
            ind[r] = As[(size_t)row * lda + 16 * full + (li - 12)];
            if constexpr (BF16) ind[r] = (float)(__bf16)ind[r];
          }
          // branch-free: rows beyond the batch (j < 0) read row 0 of the tile and are zeroed by a select; model
          // columns beyond the slab carry finite values (their W and P are zero) that no store lets out
          const bool live = j >= 0;
          const float* prow = Ps + max(j, 0) * kN + li;
#pragma unroll
          for (int nt = 0; nt < kNT; ++nt) {
            const float z = acc[nt][r] + prow[nt * 16];
            if constexpr (MODE == 1) {
              const float o = live ? z - yi : 0.0f;
              ov[nt][r] = o;
              loss_local[nt] = fmaf(o, o, loss_local[nt]);
            } else {
              ov[nt][r] = live ? star_sigmoid(z) - yi : 0.0f;
              loss_local[nt] += live ? star_softplus(z) - yi * z : 0.0f;
            }
          }
        }
        // With BF16 the residual is rounded once as it enters the two products below
        if constexpr (BF16) {
#pragma unroll
          for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt) ov[nt][r] = (float)(__bf16)ov[nt][r];
        }
      };
      if constexpr (!BF16) {
        for (int t = 0; 16 * t < cnt; ++t) {
          float ov[kNT][4];
          float ind[4];
          residual_tile(t, ov, ind);
          // segment sums (the product with the 0/1 indicator matrix), then S^T E
#pragma unroll
          for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
              zacc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(ind[r], ov[nt][r], zacc[nt], 0, 0, 0);
          const float* acol = As + (size_t)(t * 16 + 4 * q) * lda + li;
#pragma unroll
          for (int jt = 0; jt < JG; ++jt) {
            if (jt < njt) {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float av = acol[(size_t)r * lda + jt * 16];
#pragma unroll
                for (int nt = 0; nt < kNT; ++nt)
                  gacc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, ov[nt][r], gacc[jt][nt], 0, 0, 0);
              }
            }
          }
        }
      } else {
        // Two tiles (32 rows) at a time: their residuals, as they sit in the lanes, are the B operand of one
        // 16x16x32 bfloat16 MFMA whose K octet q stands for the rows 4 q .. 4 q + 3 of the first tile followed by
        // those of the second; the indicator (segment sums) and the staged table values (S^T E) are packed in the
        // same order.  Every value is a bfloat16 value already, every product exact, the sums float32.
        for (int t = 0; 16 * t < cnt; t += 2) {
          bf16x8 ia, eb[kNT];
          {
            float ov[kNT][4];
            float ind[4];
            residual_tile(t, ov, ind);                        // packed at once: one tile of float residuals alive at a time
#pragma unroll
            for (int r = 0; r < 4; ++r) ia[r] = (__bf16)ind[r];
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
              for (int r = 0; r < 4; ++r) eb[nt][r] = (__bf16)ov[nt][r];
          }
          if (16 * (t + 1) < cnt) {
            float ov[kNT][4];
            float ind[4];
            residual_tile(t + 1, ov, ind);
#pragma unroll
            for (int r = 0; r < 4; ++r) ia[4 + r] = (__bf16)ind[r];
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
              for (int r = 0; r < 4; ++r) eb[nt][4 + r] = (__bf16)ov[nt][r];
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) ia[4 + r] = (__bf16)0.0f;
#pragma unroll
            for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
              for (int r = 0; r < 4; ++r) eb[nt][4 + r] = (__bf16)0.0f;
          }
#pragma unroll
          for (int nt = 0; nt < kNT; ++nt)
            zacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ia, eb[nt], zacc[nt], 0, 0, 0);
          const float* acol = As + (size_t)(t * 16 + 4 * q) * lda + li;
#pragma unroll
          for (int jt = 0; jt < JG; ++jt) {
            if (jt < njt) {
              bf16x8 sa;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                sa[r] = (__bf16)acol[(size_t)r * lda + jt * 16];
                sa[4 + r] = (__bf16)acol[(size_t)(16 + r) * lda + jt * 16];
              }
#pragma unroll
              for (int nt = 0; nt < kNT; ++nt)
                gacc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sa, eb[nt], gacc[jt][nt], 0, 0, 0);
            }
          }
        }
      }
    }
    if (fold && q == 3) {
#pragma unroll
      for (int nt = 0; nt < kNT; ++nt) gacc[JG - 1][nt] += zacc[nt];
    }
    // Z tile: through Ps so that rows leave as float4
    wave_sync();
#pragma unroll
    for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) Ps[(4 * q + r) * kN + nt * 16 + li] = zacc[nt][r];
    wave_sync();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int r = pr + 4 * u;
      if (r < tr && jb + r < a.r_R && 4 * pq < nw) {
        const float4 v = *reinterpret_cast<const float4*>(Ps + r * kN + 4 * pq);
        float* p = a.PZ + (jb + r) * a.ldp + n0 + 4 * pq;
        if (p_vec && 4 * pq + 3 < nw) {
          *reinterpret_cast<float4*>(p) = v;
        } else {
          p[0] = v.x;
          if (4 * pq + 1 < nw) p[1] = v.y;
          if (4 * pq + 2 < nw) p[2] = v.z;
          if (4 * pq + 3 < nw) p[3] = v.w;
        }
      }
    }
  }

  // the four wavefronts' shares of S^T E, added in wavefront order in LDS (over the staging area, now idle)
  float* red = lds;
  for (int w = 0; w < kWaves; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int jt = 0; jt < JG; ++jt) {
        const bool tail_slot = fold && jt == JG - 1;          // rows 16 full + r, held by the lanes q == 3
        if ((jt >= njt && !tail_slot) || (tail_slot && q != 3)) continue;
#pragma unroll
        for (int nt = 0; nt < kNT; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = tail_slot ? 16 * full + r : jt * 16 + 4 * q + r;
            float* p = red + (size_t)row * kN + nt * 16 + li;
            if (w == 0) *p = gacc[jt][nt][r];
            else *p += gacc[jt][nt][r];
          }
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < a.cs * kN; e += kBlock) {
    const int j = e / kN, n = e - j * kN;
    if (n < nw) a.grad_partial[((int64_t)blockIdx.x * a.cs + j) * a.ld_grad + n0 + n] = red[e];
  }

  // per-column loss of this workgroup: the four row groups of a wavefront, then the wavefronts in order
  __shared__ float lsum[kWaves][kN];
#pragma unroll
  for (int nt = 0; nt < kNT; ++nt) {
    float s = loss_local[nt];
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    if (q == 0) lsum[wave][nt * 16 + li] = s;
  }
  __syncthreads();
  if (tid < nw) {
    float s = 0.0f;
    for (int w = 0; w < kWaves; ++w) s += lsum[w][tid];
    a.loss_partial[(int64_t)blockIdx.x * a.ld_loss + n0 + tid] = s;
  }
}

typedef void (*StarFn)(StarArgs, int, int, int, int);

template <int MODE, bool B>
StarFn pick_star(bool vec4, int jg) {
  if (vec4) return jg == 2 ? gd_star_kernel<MODE, true, B, 2, 32> : gd_star_kernel<MODE, true, B, 4, 32>;
  return jg == 2 ? gd_star_kernel<MODE, false, B, 2, 32> : gd_star_kernel<MODE, false, B, 4, 32>;
}

constexpr int kStarST = 32;

int star_slots(StarFn fn, size_t lds_bytes) {
  static std::mutex cache_mutex;   // the cache below is shared by every plan of the process
  std::lock_guard<std::mutex> lock(cache_mutex);
  static int cus = 0;
  static StarFn seen_fn[32];
  static size_t seen_lds[32];
  static int seen_occ[32];
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
  if (n_seen < 32) { seen_fn[n_seen] = fn; seen_lds[n_seen] = lds_bytes; seen_occ[n_seen] = per_cu; ++n_seen; }
  return per_cu * cus;
}

}  // namespace

// Tables of at most 64 columns and batches of more than 32 models.
bool gd_star_supported(int cs, int m) { return cs > 0 && cs <= 64 && m > 32; }

// max_grid: the caller's bound on workgroups per model slab (sizes of the partial buffers).
hipError_t launch_gd_star(const StarArgs& a, int vec, int mode, bool bf16, int max_grid, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!gd_star_supported(a.cs, a.m) || (mode != 1 && mode != 2) || a.r_R <= 0 || max_grid < 1) return hipErrorInvalidValue;
  const int kq = bf16 ? 32 : 16;
  const int kp = (a.cs + kq - 1) / kq * kq;
  const int jg = kp <= 32 ? 2 : 4;
  const int lda = kp + 4;
  const int tail = a.cs % 16;
  const int fold = (tail >= 1 && tail <= 4) ? 1 : 0;   // see the kernel: 12-row tiles of R
  const int tr = fold ? 12 : 16;
  const int rtiles = (int)((a.r_R + tr - 1) / tr);
  const bool vec4 = vec == 4;
  StarFn fn;
  if (bf16) fn = mode == 1 ? pick_star<1, true>(vec4, jg) : pick_star<2, true>(vec4, jg);
  else fn = mode == 1 ? pick_star<1, false>(vec4, jg) : pick_star<2, false>(vec4, jg);
  size_t lds_floats = (size_t)kp * kN + (size_t)kWaves * ((size_t)kStarST * lda + 16 * kN + 3 * kStarST);
  lds_floats = std::max(lds_floats, (size_t)jg * 16 * kN);     // the wavefronts' sum of S^T E
  const size_t lds_bytes = lds_floats * sizeof(float);
  if (lds_bytes > 64 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  const int gy = (a.m + kN - 1) / kN;
  int64_t gx = (rtiles + kWaves - 1) / kWaves;
  const int64_t slots = star_slots(fn, lds_bytes);
  // every wavefront walks its share of the tiles: one round of resident workgroups
  if (gx * gy > slots) gx = std::max<int64_t>(1, slots / gy);
  gx = std::min<int64_t>(gx, max_grid);
  if (grid_out) *grid_out = (int)gx;
  hipLaunchKernelGGL(fn, dim3((unsigned)gx, (unsigned)gy), dim3(kBlock), lds_bytes, st, a, kp, lda, rtiles, fold);
  return hipGetLastError();
}

}  // namespace ilargi
