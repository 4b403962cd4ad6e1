// Transposed multiply, share of a joined source for operands of 8..16 columns (Sec. 2.2):
//   G_k = D_k^T (I_k^T Y)
// in ONE pass in join order instead of a segmented sum (Z = I_k^T Y written out) followed by a reduction that
// reads D_k and Z again.  A wavefront owns 16 rows of D_k and, through the inverse index, every target row that
// joins them.  It gathers those rows of Y 64 at a time (next batch prefetched into registers) and adds them up
// per row of D_k with an indicator MFMA (A = 1 where staged row 4 q + r joins row li of the tile: exact sums).
// The summed tile then sits in the MFMA result layout, register r of lane (li, q) = Z[row 4 q + r][column li],
// which is exactly the B operand of a 16x16x4 MFMA whose K slot q stands for row 4 q + r; with
// A = D_k[row 4 q + r][16 ci + li] that MFMA adds the tile's share to columns 16 ci .. of G_k.  Z never leaves the
// registers.  The wavefront's 16 rows of D_k are requested at the start of the tile and arrive while the rows
// of Y are gathered.  Per-workgroup partial blocks are added afterwards in workgroup order.
#include <algorithm>
#include <cstdint>
#include <mutex>
#include <type_traits>

#include "ilargi_internal.h"
#include "colred_flat_body.h"

namespace ilargi {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void tj_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int kTjST = 64;            // target rows a wavefront stages at a time
constexpr int kTjLdy = 20;           // LDS row stride of the staged rows of Y
constexpr int kTjWavesPerBlock = kBlock / kWave;
constexpr int kTjWaveFloats = kTjST * kTjLdy + 2 * kTjST + 64;

// NTR: 16-column tiles of D_k (compile-time bound of the accumulators); VEC4: rows of Y as float4.
// DV4 (NTR a multiple of 4, table rows whole aligned float4s): the tiles of a group of 64 columns are interleaved,
// tile 4 g + t holding the columns 64 g + 4 li + t, so that the values a lane needs of one table row for the four
// tiles of a group are one float4 (16 lanes read 256 contiguous bytes) instead of four separate floats.
template <int NTR, bool VEC4, bool DV4>
__device__ __forceinline__ void tmm_join_body(const TmmJoinArgs& a, int rtiles, float* lds, int bid, int nblocks) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int li = lane % 16, q = lane / 16;
  float* wbase = lds + (size_t)wave * kTjWaveFloats;
  float* Ys = wbase;                                          // [ST][ldy] staged rows of Y (zero beyond c)
  int* iS = reinterpret_cast<int*>(Ys + kTjST * kTjLdy);      // [ST] target row of each staged row
  int* jS = iS + kTjST;                                       // [ST] row of the tile it joins (-1: none)
  int* rpS = jS + kTjST;                                      // [17] row pointers of the tile
  int* rpN = rpS + 32;                                        // [17] ... of the wavefront's next tile

  v4f gacc[NTR];                                              // G_k tiles: columns 16 ci .. of D_k x operand columns
#pragma unroll
  for (int ci = 0; ci < NTR; ++ci) gacc[ci] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};

  typedef typename std::conditional<VEC4, float4, float>::type SVal;
  constexpr int NV = VEC4 ? kTjST * 4 / kWave : kTjST * 16 / kWave;   // staging slots of a lane (16 columns per row)
  constexpr int gslots = VEC4 ? 4 : 16;
  const int glive = VEC4 ? a.c / 4 : a.c;
  const int ntr = (a.ck + 15) / 16;

  // A wavefront walks its tiles with the memory chain of the next tile already under way: the row pointers of a
  // tile are requested two tiles ahead, the target rows of its first two batches one tile ahead, and the rows of Y
  // of its first batch while the last batch of the tile before it is on the matrix cores.
  const int tstride = nblocks * kTjWavesPerBlock;
  int rt = bid * kTjWavesPerBlock + wave;
  // lane l <= 16 holds row pointer l of a tile (0 for a tile beyond the table: an empty range)
  auto load_rp = [&](int t) -> int {
    return (t < rtiles && lane <= 16) ? a.rowptr[min((int64_t)t * 16 + lane, a.r_k)] : 0;
  };
  int rp_cur = load_rp(rt), rp_n1 = load_rp(rt + tstride);
  int pb = __builtin_amdgcn_readlane(rp_cur, 0), pe = __builtin_amdgcn_readlane(rp_cur, 16);
  int pi = (lane < kTjST && pb + lane < pe) ? a.perm[pb + lane] : -1;
  int pi_next = (lane < kTjST && pb + kTjST + lane < pe) ? a.perm[pb + kTjST + lane] : -1;
  int jl = -1;
  bool have_sv = false;                                       // the first batch of the tile is already in sv / jl
  SVal sv[NV];
  auto load_rows = [&](int cnt_rows) {
#pragma unroll
    for (int u = 0; u < NV; ++u) {
      const int e = lane + u * kWave;
      const int r = e / gslots, g = e - r * gslots;
      if constexpr (VEC4) sv[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      else sv[u] = 0.0f;
      if (r < cnt_rows && g < glive) {
        const int64_t row = iS[r];
        if constexpr (VEC4) sv[u] = *reinterpret_cast<const float4*>(a.Y + row * a.ldy + a.col0 + 4 * g);
        else sv[u] = a.Y[row * a.ldy + a.col0 + g];
      }
    }
  };
  // row of the tile an entry joins, from the tile's 17 row pointers in LDS (the entries of a row are consecutive)
  auto joined = [&](const int* rp, int p) {
    int j = 0;
#pragma unroll
    for (int k = 1; k < 16; ++k) j += p >= rp[k] ? 1 : 0;
    return j;
  };
  for (; rt < rtiles; rt += tstride) {
    const int64_t jb = (int64_t)rt * 16;
    const int p_begin = pb, p_end = pe;
    // the tile after this one: its range and the target rows of its first two batches; row pointers of the one after
    const int rp_n2 = load_rp(rt + 2 * tstride);
    const int nb = __builtin_amdgcn_readlane(rp_n1, 0), ne = __builtin_amdgcn_readlane(rp_n1, 16);
    const int npi = (lane < kTjST && nb + lane < ne) ? a.perm[nb + lane] : -1;
    const int npi_next = (lane < kTjST && nb + kTjST + lane < ne) ? a.perm[nb + kTjST + lane] : -1;
    // this tile of D_k in the A layout of the second product: value r of tile ci is D[jb + 4 q + r][16 ci + li]
    float dv[NTR][4];
    if constexpr (DV4) {
#pragma unroll
      for (int g = 0; g < NTR / 4; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int64_t row = jb + 4 * q + r;
          const int col = 64 * g + 4 * li;
          float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
          if (row < a.r_k && col < a.ck) t = *reinterpret_cast<const float4*>(a.D + row * a.ck + col);
          dv[4 * g][r] = t.x; dv[4 * g + 1][r] = t.y; dv[4 * g + 2][r] = t.z; dv[4 * g + 3][r] = t.w;
        }
    } else {
#pragma unroll
      for (int ci = 0; ci < NTR; ++ci)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int64_t row = jb + 4 * q + r;
          const int col = 16 * ci + li;
          dv[ci][r] = (ci < ntr && row < a.r_k && col < a.ck) ? a.D[row * a.ck + col] : 0.0f;
        }
    }
    v4f zacc = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
    tj_wave_sync();                                           // the previous tile's batches are consumed
    if (lane <= 16) { rpS[lane] = rp_cur; rpN[lane] = rp_n1; }
    if (!have_sv && lane < kTjST) iS[lane] = pi;
    tj_wave_sync();
    if (!have_sv) {
      jl = pi >= 0 ? joined(rpS, p_begin + lane) : -1;
      load_rows(min(kTjST, p_end - p_begin));
    }
    for (int p0 = p_begin; p0 < p_end; p0 += kTjST) {
      const int cnt = min(kTjST, p_end - p0);
      const bool last = p0 + kTjST >= p_end;                  // then the next tile's first batch follows
      const int cnt_next = last ? min(kTjST, ne - nb) : min(kTjST, p_end - p0 - kTjST);
      tj_wave_sync();                                         // the previous batch is consumed
      if (lane < kTjST) { jS[lane] = jl; iS[lane] = last ? npi : pi_next; }
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int e = lane + u * kWave;
        const int r = e / gslots, g = e - r * gslots;
        if constexpr (VEC4) *reinterpret_cast<float4*>(Ys + r * kTjLdy + 4 * g) = sv[u];
        else Ys[r * kTjLdy + g] = sv[u];
      }
      tj_wave_sync();
      if (!last) {
        pi = pi_next;
        pi_next = (lane < kTjST && p0 + 2 * kTjST + lane < p_end) ? a.perm[p0 + 2 * kTjST + lane] : -1;
        jl = pi >= 0 ? joined(rpS, p0 + kTjST + lane) : -1;
      } else {
        pi = npi;
        pi_next = npi_next;
        jl = pi >= 0 ? joined(rpN, nb + lane) : -1;
      }
      load_rows(cnt_next);
      for (int t = 0; 16 * t < cnt; ++t) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = t * 16 + 4 * q + r;                 // rows beyond the batch hold zeros and join nothing
          const float yv = Ys[row * kTjLdy + li];
          const float ind = jS[row] == li ? 1.0f : 0.0f;
          zacc = __builtin_amdgcn_mfma_f32_16x16x4f32(ind, yv, zacc, 0, 0, 0);
        }
      }
    }
    if (p_end > p_begin) {
      have_sv = true;                                         // the last batch fetched the next tile's first one
    } else {
      have_sv = false;
      pi = npi;
      pi_next = npi_next;
    }
    rp_cur = rp_n1; rp_n1 = rp_n2; pb = nb; pe = ne;
    // G_k += D_tile^T Z_tile
#pragma unroll
    for (int ci = 0; ci < NTR; ++ci)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        gacc[ci] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv[ci][r], zacc[r], gacc[ci], 0, 0, 0);
  }

  // the four wavefronts' shares added in wavefront order in LDS; tile ci, register r of lane (li, q) is
  // G[16 ci + 4 q + r][li] (with interleaved tiles: G[64 (ci / 4) + 4 (4 q + r) + ci % 4][li])
  float* red = lds;                                           // [NTR * 16][16]
  for (int w = 0; w < kTjWavesPerBlock; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int ci = 0; ci < NTR; ++ci)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int col = DV4 ? 64 * (ci / 4) + 4 * (4 * q + r) + ci % 4 : 16 * ci + 4 * q + r;
          float* p = red + col * 16 + li;
          if (w == 0) *p = gacc[ci][r];
          else *p += gacc[ci][r];
        }
    }
  }
  __syncthreads();
  float* gp = a.partial + (int64_t)bid * a.ck * a.c;
  for (int e = tid; e < a.ck * a.c; e += kBlock) {
    const int j = e / a.c, n = e - j * a.c;
    gp[e] = red[j * 16 + n];
  }
}

template <int NTR, bool VEC4, bool DV4>
__global__ __launch_bounds__(kBlock) void tmm_join_kernel(TmmJoinArgs a, int rtiles) {
  extern __shared__ float lds[];
  tmm_join_body<NTR, VEC4, DV4>(a, rtiles, lds, (int)blockIdx.x, (int)gridDim.x);
}

// The join-order pass of a joined source and the flat column reduce of an identity source in ONE launch: the two
// are independent parts of the same transposed multiply, the first bound by the latency of its gathers, the second
// a plain stream.  Workgroups are dealt to the eight XCDs in turn, so roles are given to groups of eight consecutive
// workgroups: every XCD then runs the same mix.  Of the (n_f + n_j) / 8 groups, n_f / 8 are dealt evenly among the
// others and run the column reduce (group g is the a(g)-th of them when a(g + 1) > a(g), a(g) = floor(g n_f / (n_f + n_j))).
// n_f and n_j are multiples of 8.
template <int NTR, bool DV4, int CMAX>
__global__ __launch_bounds__(kBlock) void tmm_pair_kernel(TmmJoinArgs j, int rtiles, ColredFlatArgs f, int n_f, int n_j) {
  extern __shared__ float lds[];
  const int64_t g = blockIdx.x / 8, nt = (int64_t)n_f + n_j;
  const int x = blockIdx.x % 8;
  const int a0 = (int)(g * n_f / nt), a1 = (int)((g + 1) * n_f / nt);
  if (a1 > a0) colred_flat_body<CMAX, true>(f, lds, 8 * a0 + x, n_f);
  else tmm_join_body<NTR, true, DV4>(j, rtiles, lds, (int)(8 * (g - a0) + x), n_j);
}

typedef void (*TjFn)(TmmJoinArgs, int);
typedef void (*TpFn)(TmmJoinArgs, int, ColredFlatArgs, int, int);

template <int NTR, bool DV4>
TjFn pick_tj(bool vec4) { return vec4 ? tmm_join_kernel<NTR, true, DV4> : tmm_join_kernel<NTR, false, DV4>; }

}  // namespace

bool tmm_join_supported(int ck, int c) { return ck >= 1 && ck <= 208 && c >= 1 && c <= 16; }

// partial: partial_floats long, one ck x c block per workgroup; *grid_out workgroups were launched.
hipError_t launch_tmm_join(const TmmJoinArgs& a, int64_t partial_floats, hipStream_t st, int* grid_out) {
  if (grid_out) *grid_out = 0;
  if (!tmm_join_supported(a.ck, a.c) || a.r_k <= 0) return hipErrorInvalidValue;
  const int rtiles = (int)((a.r_k + 15) / 16);
  const int ntr = (a.ck + 15) / 16;
  const bool vec4 = a.c % 4 == 0 && a.ldy % 4 == 0 && a.col0 % 4 == 0 && reinterpret_cast<uintptr_t>(a.Y) % 16 == 0;
  const bool dv4 = a.ck % 4 == 0 && reinterpret_cast<uintptr_t>(a.D) % 16 == 0;
  TjFn fn;
  int ntr_c;
  if (dv4) {
    fn = ntr <= 4 ? pick_tj<4, true>(vec4) : (ntr <= 8 ? pick_tj<8, true>(vec4) : pick_tj<16, true>(vec4));
    ntr_c = ntr <= 4 ? 4 : (ntr <= 8 ? 8 : 16);
  } else {
    fn = ntr <= 4 ? pick_tj<4, false>(vec4) : (ntr <= 8 ? pick_tj<8, false>(vec4) : pick_tj<13, false>(vec4));
    ntr_c = ntr <= 4 ? 4 : (ntr <= 8 ? 8 : 13);
  }
  size_t lds_floats = std::max<size_t>((size_t)kTjWavesPerBlock * kTjWaveFloats, (size_t)ntr_c * 256);
  const size_t lds_bytes = lds_floats * sizeof(float);
  static std::mutex cache_mutex;
  static TjFn seen_fn[16];
  static int seen_slots[16];
  static int n_seen = 0;
  int slots = 0;
  {
    std::lock_guard<std::mutex> lock(cache_mutex);
    for (int i = 0; i < n_seen; ++i)
      if (seen_fn[i] == fn) slots = seen_slots[i];
    if (slots == 0) {
      int dev = 0, cus = 256, per_cu = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, lds_bytes) != hipSuccess ||
          per_cu < 1)
        per_cu = 1;
      slots = per_cu * cus;
      if (n_seen < 16) { seen_fn[n_seen] = fn; seen_slots[n_seen] = slots; ++n_seen; }
    }
  }
  int64_t gx = (rtiles + kTjWavesPerBlock - 1) / kTjWavesPerBlock;
  gx = std::min<int64_t>(gx, slots);                                  // one round of resident workgroups
  gx = std::min<int64_t>(gx, partial_floats / ((int64_t)a.ck * a.c));
  if (gx < 1) return hipErrorInvalidValue;
  if (grid_out) *grid_out = (int)gx;
  hipLaunchKernelGGL(fn, dim3((unsigned)gx), dim3(kBlock), lds_bytes, st, a, rtiles);
  return hipGetLastError();
}

// Both parts in one launch (operands of 8, 12 or 16 columns whose rows are whole aligned float4s).  The split of
// the resident workgroups follows the bytes each part has to move (measured on a star join of 10^6 x 20 and
// 10^5 x 200: within 4 % of the best split for 8, 12 and 16 operand columns).
bool tmm_pair_supported(const ColredFlatArgs& f, const TmmJoinArgs& j) {
  if (!tmm_join_supported(j.ck, j.c) || !colred_flat_supported(f.S, 4 * (int64_t)f.nvec, f.c)) return false;
  if (f.c != j.c || f.c % 4 != 0 || j.col0 != 0 || j.ldy % 4 != 0 || f.ldy % 4 != 0) return false;
  if (reinterpret_cast<uintptr_t>(j.Y) % 16 != 0 || reinterpret_cast<uintptr_t>(f.Y) % 16 != 0) return false;
  if (j.ck % 4 != 0 || reinterpret_cast<uintptr_t>(j.D) % 16 != 0) return false;
  // at least eight workgroups' worth of work on either side (roles go to groups of eight workgroups)
  const int64_t fsteps = (f.rows + kWave / f.nvec - 1) / (kWave / f.nvec);
  return (j.r_k + 15) / 16 >= 8 * kTjWavesPerBlock && fsteps >= 16 * kTjWavesPerBlock;
}

hipError_t launch_tmm_pair(const ColredFlatArgs& f, const TmmJoinArgs& j, int64_t nnz_j, int64_t room_f, int64_t room_j,
                           hipStream_t st, int* grid_f, int* grid_j) {
  *grid_f = *grid_j = 0;
  if (!tmm_pair_supported(f, j)) return hipErrorInvalidValue;
  const int rtiles = (int)((j.r_k + 15) / 16);
  const int ntr = (j.ck + 15) / 16;
  const int ntr_c = ntr <= 4 ? 4 : (ntr <= 8 ? 8 : 16);
  const int cmax = f.c <= 8 ? 8 : 16;
  TpFn fn;
  if (cmax == 8) fn = ntr_c == 4 ? tmm_pair_kernel<4, true, 8> : (ntr_c == 8 ? tmm_pair_kernel<8, true, 8> : tmm_pair_kernel<16, true, 8>);
  else fn = ntr_c == 4 ? tmm_pair_kernel<4, true, 16> : (ntr_c == 8 ? tmm_pair_kernel<8, true, 16> : tmm_pair_kernel<16, true, 16>);
  size_t lds_floats = std::max<size_t>((size_t)kTjWavesPerBlock * kTjWaveFloats, (size_t)ntr_c * 256);
  lds_floats = std::max<size_t>(lds_floats, (size_t)colred_flat_lds_floats(cmax));
  const size_t lds_bytes = lds_floats * sizeof(float);
  static std::mutex cache_mutex;
  static TpFn seen_fn[8];
  static int seen_slots[8];
  static int n_seen = 0;
  int slots = 0;
  {
    std::lock_guard<std::mutex> lock(cache_mutex);
    for (int i = 0; i < n_seen; ++i)
      if (seen_fn[i] == fn) slots = seen_slots[i];
    if (slots == 0) {
      int dev = 0, cus = 256, per_cu = 0;
      hipDeviceProp_t prop;
      if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(fn), kBlock, lds_bytes) != hipSuccess ||
          per_cu < 1)
        per_cu = 1;
      slots = per_cu * cus;
      if (n_seen < 8) { seen_fn[n_seen] = fn; seen_slots[n_seen] = slots; ++n_seen; }
    }
  }
  const double bytes_f = 4.0 * (double)f.rows * (4 * f.nvec + f.c);
  const double bytes_j = 4.0 * (double)j.r_k * j.ck + (double)nnz_j * (4.0 + 4.0 * j.c);
  const double share = bytes_f / (bytes_f + bytes_j);
  int n_f = (int)(slots * share + 0.5);
  n_f = std::max(1, std::min(n_f, slots - 1));
  int n_j = slots - n_f;
  n_j = (int)std::min<int64_t>(n_j, (rtiles + kTjWavesPerBlock - 1) / kTjWavesPerBlock);
  const int64_t fsteps = (f.rows + kWave / f.nvec - 1) / (kWave / f.nvec);
  n_f = (int)std::min<int64_t>(n_f, (fsteps + 2 * kTjWavesPerBlock - 1) / (2 * kTjWavesPerBlock));
  n_f = (int)std::min<int64_t>(n_f, room_f / ((int64_t)4 * f.nvec * f.c));
  n_j = (int)std::min<int64_t>(n_j, room_j / ((int64_t)j.ck * j.c));
  n_f = n_f / 8 * 8; n_j = n_j / 8 * 8;
  if (n_f < 8 || n_j < 8) return hipErrorInvalidValue;
  *grid_f = n_f; *grid_j = n_j;
  hipLaunchKernelGGL(fn, dim3((unsigned)(n_f + n_j)), dim3(kBlock), lds_bytes, st, j, rtiles, f, n_f, n_j);
  return hipGetLastError();
}

}  // namespace ilargi
