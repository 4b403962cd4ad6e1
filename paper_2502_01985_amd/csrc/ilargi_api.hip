// C ABI of libilargi: argument validation, the plan (workspace layout, inverse indices, column tables)
// and the sequencing of kernels for each operator.  See include/ilargi.h for the contract of every call.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "ilargi_internal.h"

using namespace ilargi;

namespace {

thread_local char g_err[512] = "";

ilargi_status_t fail(ilargi_status_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(ILARGI_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct SourcePlan {
  const float* D = nullptr;
  int64_t rows = 0, cols = 0;
  const int32_t* idx = nullptr;   // caller's row_idx (device) or NULL
  bool has_idx = false;           // row_idx was given
  bool ident = false;             // identity on the first `rows` target rows, nothing beyond
  bool empty = false;             // contributes nothing (no rows or no columns)
  bool sparse = false;            // given in compressed sparse rows (D is NULL)
  const int32_t* csr_rowptr = nullptr;
  const int32_t* csr_col = nullptr;
  const float* csr_val = nullptr;
  int64_t entries = 0;            // stored entries of a sparse source
  size_t o_csc_row = 0, o_csc_val = 0, o_colptr = 0, o_tchunk_beg = 0, o_tchunk_end = 0, o_col_first = 0, o_tpartial = 0,
         o_row_block = 0;
  int64_t row_block_max = 0;
  int n_row_blocks = 0;
  int64_t tchunk_max = 0;
  int n_tchunks = 0;
  int vec = 1;
  std::vector<int32_t> colmap_h;
  // offsets into the workspace
  size_t o_colmap = 0, o_tcol = 0, o_rowptr = 0, o_perm = 0, o_chunk_seg = 0, o_chunk_beg = 0, o_chunk_end = 0,
         o_long_seg = 0, o_long_first = 0, o_chunk_partial = 0, o_pz = 0, o_partial = 0, o_g = 0, o_cnt = 0;
  int64_t nch_max = 0, nl_max = 0;
  int n_chunks = 0, n_long = 0;
  size_t o_join_first = 0;        // join-order column reduce: first source row of every workgroup
  int n_join_blocks = 0;
  bool sliced = false;            // the inverse index is also split by slice of target rows (large target tables)
  size_t o_sl_rowptr = 0, o_sl_perm = 0, o_sl_chunk0 = 0, o_sl_ch_beg = 0, o_sl_ch_end = 0, o_sl_nchunk = 0,
         o_sl_ch_partial = 0, o_zslice = 0;
  int sl_cap = 0, sl_logG = 0;
  int64_t nnz = 0;
  int logG = 0;
};

struct Layout {
  size_t o_gslot = 0, o_gj0 = 0, o_ct_slot = 0, o_ct_j = 0, o_ones = 0, o_tmp_a = 0, o_tmp_b = 0, o_rmm = 0;
  size_t o_eye = 0;                          // sparse crossprod: a block of identity columns, c_T x min(max_cx, 16)
  size_t o_cn = 0, o_counts = 0, o_rr = 0;   // KMeans / NMF: centroid norms, cluster sizes, two small square matrices
  int64_t max_entries = 0;       // most stored entries of a sparse source (0: every source is dense)
  size_t o_flags = 0, o_tcol_table = 0, o_pairs = 0, o_E = 0, o_loss = 0, o_sort = 0, o_hist = 0, o_zc = 0,
         o_gpartial = 0, o_blocks = 0;
  int64_t zc_floats = 0, gpartial_floats = 0, blocks_floats = 0;
  // crossprod "via pairs": lists of (row of source k, row of source l) for the target rows both feed
  int n_pairlists = 0;
  int pairlist_k[kMaxPairLists] = {}, pairlist_l[kMaxPairLists] = {};
  size_t o_pairlist[kMaxPairLists] = {};     // 2 r_T integers each: rows of k, then rows of l
  size_t total = 0;
};

}  // namespace

// Scratch of ilargi_plan_create_static: one array per GPU, part of the library's code object, so a caller that
// cannot allocate device memory still gets a plan.  The array's name is only a host-side handle of the symbol;
// the device address is looked up once per device with hipGetSymbolAddress and used from then on.
constexpr size_t kStaticScratchBytes = 128ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
struct StaticSlot {
  void* ptr = nullptr;            // device address of `scratch` on this device
  ilargi_plan* owner = nullptr;   // the live plan that occupies it (at most one per device)
};
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mutex;
}  // namespace

ilargi_status_t ilargi::set_error(ilargi_status_t code, const char* msg) { return fail(code, "%s", msg); }

struct ilargi_plan {
  int n = 0;
  int64_t r_T = 0, c_T = 0, max_cx = 0;
  char* ws = nullptr;
  size_t ws_bytes = 0;
  std::vector<SourcePlan> src;
  Layout lay;
  int fused = -1;   // identity source whose product is fused into the assembly pass
  bool any_sparse = false;  // some source is given in compressed sparse rows: narrow kernels only
  int star_k = -1;  // two-table star join: the dimension table every target row joins (else -1)
  bool cover_disjoint = false;  // no target column is fed by two sources
  bool cover_full = false;      // every target column is fed and every source reaches every target row
  bool mat_vec4 = false;  // the grouped column tables of the vectorized join-gather are valid
  bool mat_flat = false;  // ... and every group is an aligned float4 of its source
  bool mat_cols = false;  // the per-column feeder tables (at most two feeders per column) are valid
  int npairs = 0;
  int64_t pairlist_n[kMaxPairLists] = {};   // entries of the pair lists of the layout
  bool small_gd = false;  // the schema is small enough for the single-workgroup gradient-descent iteration
  int small_ident = -1, small_joined = -1;   // ... its entity table and its joined table (or -1)
  bool rowjoin_gd = false;  // fetching every source's row per target row moves fewer bytes than the factorized sequence
  int static_dev = -1;   // >= 0: the workspace is the library's static scratch array of that device
  // two-table star join: the entity table with its rows in join order and the row of the dimension table each joins,
  // in a buffer the caller gave to ilargi_plan_cluster (NULL: not clustered)
  const float* cluster_sp = nullptr;
  const int32_t* cluster_keys = nullptr;
  int cluster_k = -1;   // the joined source
  const float* cluster_y_src = nullptr;   // the label vector whose join-ordered copy cluster_yp holds (NULL: none)
  const float* cluster_yp = nullptr;
  std::vector<size_t> block_off;  // offset (floats) of Gram block (k,l), k <= l, index k * n + l
  // optional timing of one kernel family: event pairs recorded around every launch whose tag matches
  std::string trace_tag;            // "*" traces every kernel family
  std::string trace_label;          // caller's label for the operator in flight
  std::vector<hipEvent_t> trace_events;
  std::vector<std::string> trace_names;
  int trace_n = 0;
  // a second stream for independent blocks of one call (crossprod); NULL: everything runs on the caller's stream
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool side_tried = false;   // creating a stream takes milliseconds: done at the first call that wants it
  template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
  ~ilargi_plan() {
    for (hipEvent_t e : trace_events) (void)hipEventDestroy(e);
    if (ev_fork) (void)hipEventDestroy(ev_fork);
    if (ev_join) (void)hipEventDestroy(ev_join);
    if (side) (void)hipStreamDestroy(side);
  }
};

namespace {

// Records an event pair around the launches in its scope when the plan traces this tag.
struct TraceScope {
  ilargi_plan* pl;
  hipStream_t st;
  bool on;
  TraceScope(ilargi_plan* p, const char* tag, int k, hipStream_t s) : pl(p), st(s), on(false) {
    if (p->trace_events.empty() || p->trace_n + 2 > (int)p->trace_events.size()) return;
    char full[64];
    if (k >= 0) snprintf(full, sizeof(full), "%s:%d", tag, k);
    else snprintf(full, sizeof(full), "%s", tag);
    std::string name = p->trace_label.empty() ? std::string(full) : p->trace_label + "/" + full;
    if (p->trace_tag != "*" && p->trace_tag != full && p->trace_tag != name) return;
    on = hipEventRecord(p->trace_events[p->trace_n], st) == hipSuccess;
    if (on) p->trace_names.push_back(name);
  }
  ~TraceScope() {
    if (!on) return;
    if (hipEventRecord(pl->trace_events[pl->trace_n + 1], st) == hipSuccess) pl->trace_n += 2;
    else pl->trace_names.pop_back();
  }
};

// The plan's second stream, created at the first call that can use it (never for a plan on the static scratch array,
// whose callers must not allocate, and never while `st` is being captured into a graph).  NULL: run on one stream.
hipStream_t side_stream(ilargi_plan* pl, hipStream_t st) {
  if (pl->side != nullptr || pl->side_tried || pl->static_dev >= 0) return pl->side;
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return nullptr;                                           // not now; a later eager call may create it
  }
  pl->side_tried = true;
  if (hipStreamCreateWithFlags(&pl->side, hipStreamNonBlocking) != hipSuccess) pl->side = nullptr;
  if (pl->side != nullptr &&
      (hipEventCreateWithFlags(&pl->ev_fork, hipEventDisableTiming) != hipSuccess ||
       hipEventCreateWithFlags(&pl->ev_join, hipEventDisableTiming) != hipSuccess)) {
    if (pl->ev_fork) (void)hipEventDestroy(pl->ev_fork);
    pl->ev_fork = nullptr;
    (void)hipStreamDestroy(pl->side);
    pl->side = nullptr;
  }
  (void)hipGetLastError();
  return pl->side;
}

// Rows per workgroup of the narrow column reduce: about kColredTarget chunks, each a whole number of workgroup
// iterations (so that no iteration runs half empty), never more than kColredBlocks chunks.
int64_t colred_rows_per_block(int64_t rows, int64_t cols, int vec) {
  const int64_t step = colred_step_rows((int)std::max<int64_t>(cols, 1), vec);
  int64_t rpb = (rows + kColredTarget - 1) / kColredTarget;
  rpb = (rpb + step - 1) / step * step;
  const int64_t floor_rpb = (rows + kColredBlocks - 1) / kColredBlocks;
  return std::max<int64_t>(std::max(rpb, floor_rpb), 1);
}
int colred_nblocks(int64_t rows, int64_t cols, int vec) {
  int64_t rpb = colred_rows_per_block(rows, cols, vec);
  return (int)((rows + rpb - 1) / rpb);
}

// Shape-only part of a plan: fills the offsets of every workspace region.
ilargi_status_t make_layout(int n, const ilargi_source_t* s, int64_t r_T, int64_t c_T, int64_t max_cx,
                            std::vector<SourcePlan>& src, Layout& lay) {
  if (s == nullptr) return fail(ILARGI_ERR_NULL, "sources is NULL");
  if (n < 1 || n > kMaxSources) return fail(ILARGI_ERR_SHAPE, "n = %d outside [1, %d]", n, kMaxSources);
  if (r_T < 0 || r_T > 2147483646ll) return fail(ILARGI_ERR_SHAPE, "r_T = %lld out of range", (long long)r_T);
  if (c_T < 1 || c_T > (1 << 20)) return fail(ILARGI_ERR_SHAPE, "c_T = %lld outside [1, 2^20]", (long long)c_T);
  if (max_cx < 1 || max_cx > 65536) return fail(ILARGI_ERR_SHAPE, "max_cx = %lld outside [1, 65536]", (long long)max_cx);
  src.assign(n, SourcePlan());
  int64_t cmax = 1;
  for (int k = 0; k < n; ++k) {
    if (s[k].rows < 0 || s[k].cols < 0 || s[k].rows > 2147483646ll)
      return fail(ILARGI_ERR_SHAPE, "source %d: rows = %lld, cols = %lld", k, (long long)s[k].rows, (long long)s[k].cols);
    if (s[k].cols > kMaxLdsFloats && s[k].csr_rowptr == nullptr)
      return fail(ILARGI_ERR_UNSUPPORTED, "source %d: more than %d columns (wider tables must be given in sparse rows)", k,
                  kMaxLdsFloats);
    if (s[k].cols > (1 << 20)) return fail(ILARGI_ERR_SHAPE, "source %d: cols = %lld above 2^20", k, (long long)s[k].cols);
    if (s[k].row_idx == nullptr && s[k].rows != r_T)
      return fail(ILARGI_ERR_SHAPE, "source %d: NULL row_idx (identity) needs rows == r_T", k);
    src[k].rows = s[k].rows;
    src[k].cols = s[k].cols;
    src[k].has_idx = s[k].row_idx != nullptr;
    src[k].empty = s[k].rows == 0 || s[k].cols == 0;
    src[k].sparse = s[k].csr_rowptr != nullptr && !src[k].empty;
    if (src[k].sparse) {
      if (s[k].nnz < 0 || s[k].nnz > 2147483646ll || s[k].nnz > s[k].rows * s[k].cols)
        return fail(ILARGI_ERR_SHAPE, "source %d: nnz = %lld", k, (long long)s[k].nnz);
      src[k].entries = s[k].nnz;
      lay.max_entries = std::max(lay.max_entries, std::max<int64_t>(s[k].nnz, 1));
    }
    cmax = std::max<int64_t>(cmax, s[k].cols);
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  lay.o_flags = take(sizeof(int32_t) * 3 * n);
  lay.o_tcol_table = take(sizeof(void*) * n);
  lay.o_pairs = take(sizeof(GramAsmPair) * n * (n + 1) / 2);
  lay.o_gslot = take(sizeof(int32_t) * c_T);
  lay.o_gj0 = take(sizeof(int32_t) * c_T);
  lay.o_ct_slot = take(sizeof(int32_t) * 2 * c_T);
  lay.o_ct_j = take(sizeof(int32_t) * 2 * c_T);
  lay.o_ones = take(sizeof(float) * c_T);
  lay.o_rmm = take(sizeof(float) * c_T * max_cx);
  lay.o_cn = take(sizeof(float) * max_cx);
  lay.o_counts = take(sizeof(int32_t) * max_cx);
  lay.o_rr = take(sizeof(float) * 2 * kGnmfMaxRank * kGnmfMaxRank);
  const int64_t wmax = std::max<int64_t>(max_cx, cmax);
  for (int k = 0; k < n; ++k) {
    SourcePlan& p = src[k];
    p.o_colmap = take(sizeof(int32_t) * std::max<int64_t>(p.cols, 1));
    p.o_tcol = take(sizeof(int32_t) * c_T);
    if (p.has_idx) {
      p.o_rowptr = take(sizeof(int32_t) * (p.rows + 1));
      p.o_perm = take(sizeof(int32_t) * std::max<int64_t>(r_T, 1));
      p.nl_max = r_T / kLongSeg + 1;
      p.nch_max = r_T / kSegChunk + p.nl_max + 1;
      p.o_chunk_seg = take(sizeof(int32_t) * p.nch_max);
      p.o_chunk_beg = take(sizeof(int32_t) * p.nch_max);
      p.o_chunk_end = take(sizeof(int32_t) * p.nch_max);
      p.o_long_seg = take(sizeof(int32_t) * p.nl_max);
      p.o_long_first = take(sizeof(int32_t) * (p.nl_max + 1));
      p.o_chunk_partial = take(sizeof(float) * p.nch_max * wmax);
      p.o_join_first = take(sizeof(int32_t) * (kColredBlocks + 1));
      // a residual of 6 MB or more does not stay in an XCD's 4 MB of L2: segments are then also split by slice
      // of target rows (worth it when a source row still has entries in most slices)
      p.sliced = r_T >= 1500000 && p.rows > 0 && p.rows * kSegSlices <= r_T && s[k].csr_rowptr == nullptr;
      if (p.sliced) {
        p.sl_cap = (int)segsum_sliced_chunk_cap(r_T);
        p.o_sl_rowptr = take(sizeof(int32_t) * (kSegSlices * p.rows + 1));
        p.o_sl_perm = take(sizeof(int32_t) * std::max<int64_t>(r_T, 1));
        p.o_sl_chunk0 = take(sizeof(int32_t) * kSegSlices * p.rows);
        p.o_sl_ch_beg = take(sizeof(int32_t) * kSegSlices * p.sl_cap);
        p.o_sl_ch_end = take(sizeof(int32_t) * kSegSlices * p.sl_cap);
        p.o_sl_nchunk = take(sizeof(int32_t) * kSegSlices);
        p.o_sl_ch_partial = take(sizeof(float) * kSegSlices * p.sl_cap * kNarrowCT);
        p.o_zslice = take(sizeof(float) * kSegSlices * p.rows * kNarrowCT);
      }
    }
    p.o_pz = take(sizeof(float) * std::max<int64_t>(p.rows, 1) * max_cx);
    // (a sparse source's transposed product leaves a single block of partials)
    p.o_partial = take(sizeof(float) * (p.sparse ? 1 : kColredBlocks) * std::max<int64_t>(p.cols, 1) * kNarrowCT);
    p.o_g = take(sizeof(float) * std::max<int64_t>(p.cols, 1) * max_cx);
    p.o_cnt = take(sizeof(float) * std::max<int64_t>(p.rows, 1));
    if (p.sparse) {
      const int64_t e = std::max<int64_t>(p.entries, 1);
      p.o_csc_row = take(sizeof(int32_t) * e);
      p.o_csc_val = take(sizeof(float) * e);
      p.o_colptr = take(sizeof(int32_t) * (p.cols + 1));
      p.tchunk_max = p.entries / kSparseChunk + p.cols + 1;
      p.o_tchunk_beg = take(sizeof(int32_t) * p.tchunk_max);
      p.o_tchunk_end = take(sizeof(int32_t) * p.tchunk_max);
      p.o_col_first = take(sizeof(int32_t) * (p.cols + 1));
      p.o_tpartial = take(sizeof(float) * p.tchunk_max * kNarrowCT);
      // runs of whole rows with at most cap entries: a run ends when the next row would overflow it, so two
      // neighbouring runs together hold more than cap entries (or one of them is a single row)
      p.row_block_max = 2 * (p.entries / sparse_row_block_cap((int)p.cols) + 1) + p.rows / kSparseBlockRows + 2;
      p.o_row_block = take(sizeof(int32_t) * (p.row_block_max + 1));
    }
  }
  if (lay.max_entries > 0) {
    lay.o_tmp_a = take(sizeof(int32_t) * lay.max_entries);
    lay.o_tmp_b = take(sizeof(int32_t) * lay.max_entries);
  }
  lay.o_E = take(sizeof(float) * std::max<int64_t>(r_T, 1) * max_cx);
  lay.o_eye = take(sizeof(float) * (lay.max_entries > 0 && c_T <= kSparseGramMaxCols ? c_T * std::min<int64_t>(max_cx, kSparseGramWidth) : 1));
  lay.o_loss = take(sizeof(float) * std::max<int64_t>(32768 * kNarrowCT, 1024 * max_cx));
  const int64_t sort_n = std::max<int64_t>(std::max<int64_t>(r_T, 1), lay.max_entries);
  lay.o_sort = take(sizeof(int32_t) * 4 * sort_n);
  lay.o_hist = take(sizeof(int32_t) * sort_hist_ints(sort_n));
  // Gram scratch: summed rows for the "via sums" route, chunk partials, the (k,l) blocks
  lay.zc_floats = 1;
  lay.gpartial_floats = kGramPartialFloats;
  lay.blocks_floats = 0;
  for (int k = 0; k < n && lay.max_entries == 0; ++k)    // (plans with sparse sources have no Gram matrix)
    for (int l = k; l < n; ++l) {
      int64_t cc = src[k].cols * src[l].cols;
      lay.blocks_floats += cc;
      lay.gpartial_floats = std::max(lay.gpartial_floats, cc);
      lay.gpartial_floats = std::max(lay.gpartial_floats, src[k].cols * max_cx);
      if (l > k) {
        const bool via_l = src[l].has_idx && src[l].rows * 2 <= r_T, via_k = src[k].has_idx && src[k].rows * 2 <= r_T;
        if (via_l) lay.zc_floats = std::max(lay.zc_floats, src[l].rows * src[k].cols);
        if (via_k) lay.zc_floats = std::max(lay.zc_floats, src[k].rows * src[l].cols);
        if (!via_l && !via_k && lay.n_pairlists < kMaxPairLists && src[k].cols >= 4 && src[k].cols <= 64 && src[l].cols >= 4 &&
            src[l].cols <= 64 && src[k].rows > 0 && src[l].rows > 0 && r_T > 0) {
          lay.pairlist_k[lay.n_pairlists] = k;
          lay.pairlist_l[lay.n_pairlists] = l;
          ++lay.n_pairlists;
        }
      }
    }
  for (int i = 0; i < lay.n_pairlists; ++i) lay.o_pairlist[i] = take(sizeof(int32_t) * 2 * r_T);
  lay.o_zc = take(sizeof(float) * lay.zc_floats);
  lay.o_gpartial = take(sizeof(float) * lay.gpartial_floats);
  lay.o_blocks = take(sizeof(float) * std::max<int64_t>(lay.blocks_floats, 1));
  lay.total = off;
  return ILARGI_OK;
}

int pick_vec(const float* D, int64_t cols) {
  uintptr_t a = reinterpret_cast<uintptr_t>(D);
  if (cols % 4 == 0 && a % 16 == 0) return 4;
  if (cols % 2 == 0 && a % 8 == 0) return 2;
  return 1;
}

int pick_logL(int64_t cols, int vec) {
  int64_t nvec = cols > 0 ? cols / vec : 1;
  int l = ilog2_ceil(nvec);
  return l > 6 ? 6 : l;
}

// Splits the segments longer than kLongSeg into chunks (host side, once per plan).
void build_long_tables(const std::vector<int32_t>& rowptr, std::vector<int32_t>& chunk_seg,
                       std::vector<int32_t>& chunk_beg, std::vector<int32_t>& chunk_end,
                       std::vector<int32_t>& long_seg, std::vector<int32_t>& long_first) {
  long_first.push_back(0);
  for (size_t j = 0; j + 1 < rowptr.size(); ++j) {
    int32_t b = rowptr[j], e = rowptr[j + 1];
    if (e - b <= kLongSeg) continue;
    long_seg.push_back((int32_t)j);
    for (int32_t c = b; c < e; c += kSegChunk) {
      chunk_seg.push_back((int32_t)j);
      chunk_beg.push_back(c);
      chunk_end.push_back(std::min(e, c + kSegChunk));
    }
    long_first.push_back((int32_t)chunk_seg.size());
  }
}

SegArgs seg_args(const ilargi_plan* pl, int k) {
  const SourcePlan& p = pl->src[k];
  SegArgs a;
  memset(&a, 0, sizeof(a));
  a.rowptr = pl->at<int32_t>(p.o_rowptr);
  a.perm = pl->at<int32_t>(p.o_perm);
  a.chunk_seg = pl->at<int32_t>(p.o_chunk_seg);
  a.chunk_beg = pl->at<int32_t>(p.o_chunk_beg);
  a.chunk_end = pl->at<int32_t>(p.o_chunk_end);
  a.long_seg = pl->at<int32_t>(p.o_long_seg);
  a.long_first = pl->at<int32_t>(p.o_long_first);
  a.n_chunks = p.n_chunks;
  a.n_long = p.n_long;
  a.r_k = p.rows;
  a.gidx = nullptr;
  a.g_rows = -1;
  a.chunk_partial = pl->at<float>(p.o_chunk_partial);
  a.logG = p.logG;
  a.block_first = p.n_join_blocks > 0 ? pl->at<int32_t>(p.o_join_first) : nullptr;
  if (p.sliced && !p.ident) {
    a.sl_rowptr = pl->at<int32_t>(p.o_sl_rowptr); a.sl_perm = pl->at<int32_t>(p.o_sl_perm);
    a.sl_chunk0 = pl->at<int32_t>(p.o_sl_chunk0);
    a.sl_ch_beg = pl->at<int32_t>(p.o_sl_ch_beg); a.sl_ch_end = pl->at<int32_t>(p.o_sl_ch_end);
    a.sl_nchunk = pl->at<int32_t>(p.o_sl_nchunk); a.sl_ch_partial = pl->at<float>(p.o_sl_ch_partial);
    a.sl_cap = p.sl_cap; a.sl_logG = p.sl_logG;
    a.Zs = pl->at<float>(p.o_zslice);
  }
  return a;
}

SparseArgs sparse_args(const ilargi_plan* pl, int k) {
  const SourcePlan& p = pl->src[k];
  SparseArgs a;
  memset(&a, 0, sizeof(a));
  a.rowptr = p.csr_rowptr; a.col = p.csr_col; a.val = p.csr_val;
  a.rows = p.rows; a.nnz = p.entries; a.cols = (int)p.cols;
  a.colmap = pl->at<int32_t>(p.o_colmap);
  a.row_block = pl->at<int32_t>(p.o_row_block);
  a.n_row_blocks = p.n_row_blocks;
  a.csc_row = pl->at<int32_t>(p.o_csc_row);
  a.csc_val = pl->at<float>(p.o_csc_val);
  a.chunk_beg = pl->at<int32_t>(p.o_tchunk_beg);
  a.chunk_end = pl->at<int32_t>(p.o_tchunk_end);
  a.col_first_chunk = pl->at<int32_t>(p.o_col_first);
  a.n_chunks = p.n_tchunks;
  return a;
}

// Widest operand slice one narrow pass can stage in LDS for every source of the plan.
int pass_width(const ilargi_plan* pl) {
  int64_t cmax = 1;
  for (const SourcePlan& p : pl->src)
    if (p.cols <= kMaxLdsFloats) cmax = std::max(cmax, p.cols);   // wider (sparse) tables do not stage the operand
  int w = (int)std::min<int64_t>(kNarrowCT, kMaxLdsFloats / cmax);
  return w >= 4 ? 4 : (w >= 2 ? 2 : 1);
}

// out (or the residual E) for operand columns [col0, col0 + ncols):  per-source products, then the assembly.
ilargi_status_t lmm_pass(ilargi_plan* pl, const float* X, int ldx, int col0, int ncols, float* out, int ldo,
                         int mode, const float* y, int* loss_grid, bool wide, hipStream_t st,
                         bool* fused_gradient = nullptr, bool bf16 = false) {
  if (fused_gradient) *fused_gradient = false;
  GatherArgs g;
  memset(&g, 0, sizeof(g));
  g.ldp = ldx;
  auto product_args = [&](int k) {
    const SourcePlan& p = pl->src[k];
    LmmArgs a;
    memset(&a, 0, sizeof(a));
    a.D = p.D; a.d_rows = p.rows; a.ck = (int)p.cols; a.colmap = pl->at<int32_t>(p.o_colmap);
    a.X = X; a.ldx = ldx; a.col0 = col0; a.ncols = ncols;
    a.out = pl->at<float>(p.o_pz); a.ldo = ldx; a.r_out = p.rows;
    a.logL = pick_logL(p.cols, p.vec);
    a.scratch = pl->at<float>(pl->lay.o_gpartial); a.scratch_floats = pl->lay.gpartial_floats;   // free until the assembly
    return a;
  };
  // Narrow operands: when two or more dense sources can take the streaming product kernel, their products share
  // one launch (a plan with several dimension tables otherwise pays a launch per table for a few microseconds of work).
  bool product_done[kMaxSources] = {};
  if (!wide) {
    int ks[kMaxSources], nk = 0;
    for (int k = 0; k < pl->n; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty || k == pl->fused || p.sparse) continue;
      if (rowdot_supported(product_args(k), p.vec)) ks[nk++] = k;
    }
    for (int i0 = 0; nk >= 2 && i0 < nk; i0 += kRowdotMulti) {
      LmmArgs multi[kRowdotMulti];
      int vecs[kRowdotMulti];
      const int cnt = std::min(kRowdotMulti, nk - i0);
      for (int i = 0; i < cnt; ++i) {
        multi[i] = product_args(ks[i0 + i]);
        vecs[i] = pl->src[ks[i0 + i]].vec;
        product_done[ks[i0 + i]] = true;
      }
      TraceScope ts(pl, "lmm_rows", ks[i0], st);
      HIP_TRY(launch_rowdot_multi(multi, vecs, cnt, st));
    }
  }
  for (int k = 0; k < pl->n; ++k) {
    SourcePlan& p = pl->src[k];
    if (p.empty || k == pl->fused) continue;
    if (!product_done[k]) {
      const LmmArgs a = product_args(k);
      TraceScope ts(pl, "lmm_rows", k, st);
      if (p.sparse) HIP_TRY(launch_spmm_rows(sparse_args(pl, k), X, ldx, col0, ncols, pl->at<float>(p.o_pz), ldx, st));
      else if (wide) HIP_TRY(launch_lmm_mfma(a, p.vec, 0, bf16, st, nullptr));
      else HIP_TRY(launch_lmm_rows(a, p.vec, 0, st, nullptr));
    }
    g.idx[g.n] = p.ident ? nullptr : p.idx;
    g.P[g.n] = pl->at<float>(p.o_pz);
    g.rows[g.n] = p.rows;
    ++g.n;
  }
  LmmArgs a;
  memset(&a, 0, sizeof(a));
  int vec = 1;
  if (pl->fused >= 0) {
    SourcePlan& f = pl->src[pl->fused];
    a.D = f.D; a.d_rows = f.rows; a.ck = (int)f.cols; a.colmap = pl->at<int32_t>(f.o_colmap);
    vec = f.vec;
    a.logL = pick_logL(f.cols, f.vec);
  }
  a.X = X; a.ldx = ldx; a.col0 = col0; a.ncols = ncols;
  a.out = out; a.ldo = ldo; a.r_out = pl->r_T;
  // results (and residuals) larger than the caches are streamed out past them
  a.nt_out = (int64_t)pl->r_T * ldo * (int64_t)sizeof(float) >= (64ll << 20);
  a.g = g;
  a.y = y;
  a.loss_partial = pl->at<float>(pl->lay.o_loss);
  a.ld_loss = ldx;
  if (!wide && mode != 0 && fused_gradient != nullptr && pl->fused >= 0 &&
      lmm_can_fuse_gradient(a.ck, vec, a.logL)) {
    // the fused source's share of the gradient comes out of the same pass over its rows
    a.grad_partial = pl->at<float>(pl->src[pl->fused].o_partial);
    *fused_gradient = true;
  }
  const bool wide_fuse = wide && mode != 0 && fused_gradient != nullptr && pl->fused >= 0 && col0 == 0 &&
                         lmm_mfma_can_fuse_gradient(a.ck, ncols, bf16) &&
                         (int64_t)256 * a.ck * ldx <= pl->lay.gpartial_floats;   // at most 256 workgroups per slab
  if (wide_fuse) {
    a.grad_partial = pl->at<float>(pl->lay.o_gpartial);
    a.ld_grad = ldx;
    *fused_gradient = true;
  }
  int grid = 0;
  {
    TraceScope ts(pl, "lmm_assemble", -1, st);
    if (wide && !bf16 && lmm_flat_wide_supported(a, vec, mode)) HIP_TRY(launch_lmm_flat_wide(a, st, &grid));
    else if (wide) HIP_TRY(launch_lmm_mfma(a, vec, mode, bf16, st, &grid));
    else HIP_TRY(launch_lmm_rows(a, vec, mode, st, &grid));
  }
  if (loss_grid) *loss_grid = grid;
  if (wide_fuse)   // the workgroups' shares of D^T E, added in workgroup order
    HIP_TRY(launch_tred_reduce(a.grad_partial, grid, (int64_t)a.ck * ldx, pl->at<float>(pl->src[pl->fused].o_g), st));
  return ILARGI_OK;
}

// T^T Y for operand columns [col0, col0 + ncols); mode 1 turns the finalize step into the update of Alg. 1.
ilargi_status_t tmm_pass(ilargi_plan* pl, const float* Y, int ldy, int col0, int ncols, float* out, int ldo,
                         int mode, const float* lr, float* loss, int n_loss_partial, float loss_scale,
                         hipStream_t st, int done_k = -1, int done_blocks = 0) {
  FinArgs f;
  memset(&f, 0, sizeof(f));
  auto colred_args = [&](int k, const float* Z, int ldz, int zcol0) {
    const SourcePlan& p = pl->src[k];
    ColredArgs c;
    memset(&c, 0, sizeof(c));
    c.D = p.D; c.rows = p.rows; c.ck = (int)p.cols; c.vec = p.vec;
    c.Z = Z; c.ldz = ldz; c.col0 = zcol0; c.ncols = ncols;
    c.partial = pl->at<float>(p.o_partial);
    c.rows_per_block = colred_rows_per_block(p.rows, p.cols, p.vec);
    return c;
  };
  auto segsum_args = [&](int k) {
    const SourcePlan& p = pl->src[k];
    SegArgs s = seg_args(pl, k);
    s.Y = Y; s.ldy = ldy; s.col0 = col0; s.ncols = ncols;
    s.Z = pl->at<float>(p.o_pz); s.ldz = ldy; s.zcol0 = col0;
    return s;
  };
  // Every dense source with float4 rows of at most 256 columns takes part in a merged launch: an identity source
  // (and every source of colSum, whose operand is the fan-out vector) as a plain column reduce, a joined source in
  // join-order form (segment sums in LDS, Z_k never written).  The other sources go through segment sum and
  // column reduce as separate launches.
  TmmParts parts;
  memset(&parts, 0, sizeof(parts));
  int parts_first_k = -1, parts_joins = 0;
  auto flush_parts = [&]() -> ilargi_status_t {
    if (parts.n == 0) return ILARGI_OK;
    const char* tag = parts.n > 1 ? (parts_joins > 0 ? "colred+join" : "colred") : (parts_joins > 0 ? "tmm_join" : "colred");
    {
      TraceScope ts(pl, tag, parts_first_k, st);
      HIP_TRY(launch_tmm_parts(parts, st));
    }
    memset(&parts, 0, sizeof(parts));
    parts_first_k = -1; parts_joins = 0;
    return ILARGI_OK;
  };
  // Large target table: the per-slice sums over the sliced indices of all such sources run as one launch (and the
  // sums over the slices as another); the sources then take part in the column reduce with Z_k as a plain operand.
  bool z_ready[kMaxSources] = {};
  {
    SegArgs multi[kSegMulti];
    int nm = 0, first_k = -1;
    auto flush_multi = [&]() -> ilargi_status_t {
      if (nm == 0) return ILARGI_OK;
      TraceScope ts(pl, "segsum", first_k, st);
      HIP_TRY(launch_segsum_sliced(multi, nm, st));
      nm = 0; first_k = -1;
      return ILARGI_OK;
    };
    for (int k = 0; k < pl->n && Y != nullptr; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty || k == done_k || p.ident || !p.sliced) continue;
      if (!p.sparse) {
        SegArgs sg = segsum_args(k);
        if (tmm_part_supported(colred_args(k, nullptr, 0, 0), &sg)) continue;      // join-order form: no Z_k
      }
      if (nm == kSegMulti) {
        ilargi_status_t rc = flush_multi();
        if (rc != ILARGI_OK) return rc;
      }
      if (nm == 0) first_k = k;
      multi[nm++] = segsum_args(k);
      z_ready[k] = true;
    }
    ilargi_status_t rc = flush_multi();
    if (rc != ILARGI_OK) return rc;
  }
  for (int k = 0; k < pl->n; ++k) {
    SourcePlan& p = pl->src[k];
    if (p.empty) continue;
    if (k == done_k) {
      // partials of this source were produced by the residual pass
      f.s[f.n].tcol2src = pl->at<int32_t>(p.o_tcol);
      f.s[f.n].partial = pl->at<float>(p.o_partial);
      f.s[f.n].nblocks = done_blocks;
      f.s[f.n].ck = (int)p.cols;
      ++f.n;
      continue;
    }
    int nb = colred_nblocks(p.rows, p.cols, p.vec);
    ColredArgs c;
    bool merged = false;
    if (!p.sparse) {
      const bool direct = Y == nullptr || p.ident || z_ready[k];
      c = direct ? (Y == nullptr ? colred_args(k, pl->at<float>(p.o_cnt), 1, 0)
                                 : (z_ready[k] ? colred_args(k, pl->at<float>(p.o_pz), ldy, col0) : colred_args(k, Y, ldy, col0)))
                 : colred_args(k, nullptr, 0, 0);
      SegArgs sg;
      memset(&sg, 0, sizeof(sg));
      if (!direct) sg = segsum_args(k);
      if (tmm_part_supported(c, direct ? nullptr : &sg)) {
        if (parts.n == kTmmParts) {
          ilargi_status_t rc = flush_parts();
          if (rc != ILARGI_OK) return rc;
        }
        const int q = parts.n++;
        if (q == 0) { parts.first[0] = 0; parts_first_k = k; }
        parts.join[q] = direct ? 0 : 1;
        parts_joins += direct ? 0 : 1;
        if (!direct) nb = p.n_join_blocks;
        parts.c[q] = c;
        parts.s[q] = sg;
        parts.first[q + 1] = parts.first[q] + nb;
        merged = true;
      }
    }
    if (!merged) {
      if (Y == nullptr) {
        // colSum: I_k^T 1 is the fan-out vector kept with the plan
        c = colred_args(k, pl->at<float>(p.o_cnt), 1, 0);
      } else if (p.ident) {
        c = colred_args(k, Y, ldy, col0);
      } else if (z_ready[k]) {
        c = colred_args(k, pl->at<float>(p.o_pz), ldy, col0);
      } else {
        {
          TraceScope ts(pl, "segsum", k, st);
          HIP_TRY(launch_segsum(segsum_args(k), st));
        }
        c = colred_args(k, pl->at<float>(p.o_pz), ldy, col0);
      }
      if (p.sparse) {
        // D_k^T Z_k over the column-sorted view; the result takes the place of a single block of partials
        TraceScope ts(pl, "colred", k, st);
        HIP_TRY(launch_spmm_t(sparse_args(pl, k), c.Z, c.ldz, c.col0, ncols, pl->at<float>(p.o_tpartial), c.partial, st));
        nb = 1;
      } else {
        TraceScope ts(pl, "colred", k, st);
        HIP_TRY(launch_colred(c, nb, st));
      }
    }
    f.s[f.n].tcol2src = pl->at<int32_t>(p.o_tcol);
    f.s[f.n].partial = c.partial;
    f.s[f.n].nblocks = nb;
    f.s[f.n].ck = (int)p.cols;
    ++f.n;
  }
  {
    ilargi_status_t rc = flush_parts();
    if (rc != ILARGI_OK) return rc;
  }
  f.out = out; f.ldo = ldo; f.col0 = col0; f.ncols = ncols;
  f.lr = lr;
  f.inv_rT = pl->r_T > 0 ? 1.0f / (float)pl->r_T : 0.0f;
  f.loss_partial = pl->at<float>(pl->lay.o_loss);
  f.n_loss_partial = n_loss_partial;
  f.loss = loss;
  f.loss_scale = loss_scale;
  {
    TraceScope ts(pl, "finalize", -1, st);
    HIP_TRY(launch_finalize(f, (int)pl->c_T, mode, st));
  }
  return ILARGI_OK;
}

// Runs the matrix-core transposed reduction in row chunks and adds the chunk results in order.
// transposed: block receives the cb x ca transpose of the product.
// part / part_floats: the partial-block space of this call (default: all of the plan's).
ilargi_status_t run_tred(ilargi_plan* pl, TredArgs& g, float* block, const char* tag, int tag_k, bool bf16,
                         hipStream_t st, bool transposed = false, float* part = nullptr, int64_t part_floats = 0) {
  int64_t elems = (int64_t)g.ca * g.cb;
  if (elems <= 0) return ILARGI_OK;
  if (part == nullptr) { part = pl->at<float>(pl->lay.o_gpartial); part_floats = pl->lay.gpartial_floats; }
  if (!bf16 && gram_narrow_supported(g) && elems <= part_floats) {
    // diagonal Gram block of a table with 36..64 columns: streaming kernel over interleaved column tiles
    int nch = 0;
    {
      TraceScope ts(pl, tag, tag_k, st);
      HIP_TRY(launch_gram_narrow(g, part, part_floats, st, &nch));
    }
    HIP_TRY(launch_tred_reduce(part, nch, elems, block, st, 0));
    return ILARGI_OK;
  }
  if (!bf16 && gram_sym_supported(g) && elems <= part_floats) {
    // diagonal Gram block of a table with 65..208 columns: upper-triangle tiles only
    TraceScope ts(pl, tag, tag_k, st);
    HIP_TRY(launch_gram_sym(g, part, part_floats, block, st));
    return ILARGI_OK;
  }
  if (!transposed && tred_stream_supported(g) && (bf16 || (elems >= 64 * 64 && g.n_rows >= 1024))) {
    // plain rows of both operands: one workgroup per compute unit keeps its whole ca x cb block in registers
    const int grid = tred_stream_grid(g, part_floats);
    if (grid >= 1) {
      g.partial = part;
      {
        TraceScope ts(pl, tag, tag_k, st);
        HIP_TRY(launch_tred_stream(g, grid, bf16, st));
      }
      HIP_TRY(launch_tred_reduce(g.partial, g.gx, elems, block, st, 0));
      return ILARGI_OK;
    }
  }
  // row chunks: whole rounds of the device's workgroup slots (every workgroup does the same work, so a
  // partly filled last round would idle most compute units), within the partial buffer, >= 64 rows each
  int slots = 512, tiles = 1;
  tred_occupancy(g, bf16, &slots, &tiles);
  int64_t cap = std::max<int64_t>(1, part_floats / elems);
  cap = std::min<int64_t>(cap, std::max<int64_t>(1, g.n_rows / 64));
  cap = std::min<int64_t>(cap, 4096);
  int64_t nch = std::max<int64_t>(1, slots / tiles);
  while (nch * 2 <= cap && g.n_rows / (nch * 2) >= 512) nch *= 2;   // more rounds only while chunks stay long
  nch = std::min(nch, cap);
  g.rows_per_block = (g.n_rows + nch - 1) / nch;
  g.rows_per_block = std::max<int64_t>(16, (g.rows_per_block + 15) / 16 * 16);
  nch = std::max<int64_t>(1, (g.n_rows + g.rows_per_block - 1) / g.rows_per_block);
  g.partial = part;
  {
    TraceScope ts(pl, tag, tag_k, st);
    HIP_TRY(launch_tred(g, (int)nch, bf16, st));
  }
  HIP_TRY(launch_tred_reduce(g.partial, (int)nch, elems, block, st, transposed ? g.cb : 0));
  return ILARGI_OK;
}

// T^T Y for an operand with many columns: segment sums, matrix-core column reduce, column assembly.
// done_k: a source whose block of the result is already in its o_g buffer (formed by the assembly pass).
ilargi_status_t tmm_wide(ilargi_plan* pl, const float* Y, int cx, float* out, int mode, const float* lr,
                         float* loss, int n_loss_partial, float loss_scale, bool bf16, hipStream_t st,
                         int done_k = -1) {
  ColAsmArgs c;
  memset(&c, 0, sizeof(c));
  // which kernel serves a source: 1 join-order pass, 2 flat column reduce, 0 segment sums + matrix-core reduce
  auto route = [&](const SourcePlan& p) {
    if (!p.ident && !bf16 && p.n_long == 0 && cx % 4 == 0 && tmm_join_supported((int)p.cols, cx) &&
        p.cols * cx <= pl->lay.gpartial_floats)
      return 1;
    if (p.ident && !bf16 && cx % 4 == 0 && reinterpret_cast<uintptr_t>(Y) % 16 == 0 && colred_flat_supported(p.D, p.cols, cx) &&
        p.cols * cx <= pl->lay.gpartial_floats)
      return 2;
    return 0;
  };
  // When every source leaves per-workgroup partial blocks (routes 1 and 2), the blocks stay side by side in the
  // partial buffer and the column assembly adds them itself: one launch instead of a reduction per source.
  bool defer = cx <= 64;
  int64_t worst = 0;                                     // floats of all blocks if every launch took 1024 workgroups
  for (int k = 0; k < pl->n && defer; ++k) {
    if (pl->src[k].empty || k == done_k) continue;
    if (route(pl->src[k]) == 0) defer = false;
    worst += 1024 * pl->src[k].cols * cx;
  }
  if (worst > pl->lay.gpartial_floats) defer = false;
  auto join_args = [&](const SourcePlan& p, float* part) {
    TmmJoinArgs j;
    memset(&j, 0, sizeof(j));
    j.D = p.D; j.ck = (int)p.cols; j.r_k = p.rows;
    j.rowptr = pl->at<int32_t>(p.o_rowptr); j.perm = pl->at<int32_t>(p.o_perm);
    j.Y = Y; j.ldy = cx; j.col0 = 0; j.c = cx;
    j.partial = part;
    return j;
  };
  auto flat_args = [&](const SourcePlan& p, float* part) {
    ColredFlatArgs f;
    memset(&f, 0, sizeof(f));
    f.S = p.D; f.rows = p.rows; f.nvec = (int)(p.cols / 4);
    f.Y = Y; f.ldy = cx; f.c = cx;
    f.partial = part;
    return f;
  };
  // The first identity source that takes the flat column reduce and the first joined source that takes the
  // join-order pass share a launch (the streaming part fills the gaps the gathers of the other leave).
  int pair_f = -1, pair_j = -1;
  float* pair_part[2] = {nullptr, nullptr};
  int pair_grid[2] = {0, 0};
  if (defer) {
    for (int k = 0; k < pl->n; ++k) {
      if (pl->src[k].empty || k == done_k) continue;
      const int rt = route(pl->src[k]);
      if (rt == 2 && pair_f < 0) pair_f = k;
      if (rt == 1 && pair_j < 0) pair_j = k;
    }
    if (pair_f < 0 || pair_j < 0 ||
        !tmm_pair_supported(flat_args(pl->src[pair_f], nullptr), join_args(pl->src[pair_j], nullptr)))
      pair_f = pair_j = -1;
  }
  int64_t part_off = 0;
  for (int k = 0; k < pl->n; ++k) {
    SourcePlan& p = pl->src[k];
    if (p.empty) continue;
    if (pair_f >= 0 && (k == pair_f || k == pair_j)) {
      if (pair_part[0] == nullptr) {
        const SourcePlan& pf = pl->src[pair_f];
        const SourcePlan& pj = pl->src[pair_j];
        const int64_t room_f = 1024 * pf.cols * cx, room_j = 1024 * pj.cols * cx;     // within `worst`
        pair_part[0] = pl->at<float>(pl->lay.o_gpartial) + part_off;
        pair_part[1] = pair_part[0] + room_f;
        part_off += room_f + room_j;
        TraceScope ts(pl, "colred+join", pair_f, st);
        HIP_TRY(launch_tmm_pair(flat_args(pf, pair_part[0]), join_args(pj, pair_part[1]), pj.nnz, room_f, room_j, st,
                                &pair_grid[0], &pair_grid[1]));
      }
      const int w = k == pair_f ? 0 : 1;
      c.tcol2src[c.n] = pl->at<int32_t>(p.o_tcol);
      c.ck[c.n] = (int)p.cols;
      c.G[c.n] = pair_part[w];
      c.nparts[c.n] = pair_grid[w];
      ++c.n;
      continue;
    }
    if (k == done_k) {
      c.tcol2src[c.n] = pl->at<int32_t>(p.o_tcol);
      c.G[c.n] = pl->at<float>(p.o_g);
      c.ck[c.n] = (int)p.cols;
      ++c.n;
      continue;
    }
    TredArgs g;
    memset(&g, 0, sizeof(g));
    g.A = p.D; g.lda = (int)p.cols; g.ca = (int)p.cols; g.a_rows = p.rows;
    g.ldb = cx; g.cb = cx; g.bcol0 = 0; g.b_rows = p.rows;
    g.n_rows = p.rows;
    const int rt = route(p);
    if (rt != 0) {
      float* part = pl->at<float>(pl->lay.o_gpartial) + part_off;
      const int64_t room = pl->lay.gpartial_floats - part_off;
      int grid = 0;
      if (rt == 1) {
        // segment sums and D_k^T Z_k in one pass in join order: Z_k is never written (operands whose rows are
        // whole float4s; for the others the two-step form measures the same or better)
        const TmmJoinArgs j = join_args(p, part);
        TraceScope ts(pl, "tmm_join", k, st);
        HIP_TRY(launch_tmm_join(j, room, st, &grid));
      } else {
        // short rows of an identity source, operand rows of whole float4s: flat float4 stream with plain FMAs
        // instead of padded matrix-core tiles (with element-wise operand loads the matrix-core form measures faster)
        const ColredFlatArgs f = flat_args(p, part);
        TraceScope ts(pl, "colred", k, st);
        HIP_TRY(launch_colred_flat(f, room, st, &grid));
      }
      c.tcol2src[c.n] = pl->at<int32_t>(p.o_tcol);
      c.ck[c.n] = (int)p.cols;
      if (defer) {
        c.G[c.n] = part;
        c.nparts[c.n] = grid;
        part_off += (int64_t)grid * p.cols * cx;
      } else {
        HIP_TRY(launch_tred_reduce(part, grid, p.cols * cx, pl->at<float>(p.o_g), st));
        c.G[c.n] = pl->at<float>(p.o_g);
      }
      ++c.n;
      continue;
    }
    if (p.ident) {
      g.B = Y;
    } else {
      SegArgs s = seg_args(pl, k);
      s.Y = Y; s.ldy = cx; s.col0 = 0; s.ncols = cx;
      s.Z = pl->at<float>(p.o_pz); s.ldz = cx; s.zcol0 = 0;
      {
        TraceScope ts(pl, "segsum", k, st);
        HIP_TRY(launch_segsum(s, st));
      }
      g.B = pl->at<float>(p.o_pz);
    }
    ilargi_status_t rc = run_tred(pl, g, pl->at<float>(p.o_g), "colred", k, bf16, st);
    if (rc != ILARGI_OK) return rc;
    c.tcol2src[c.n] = pl->at<int32_t>(p.o_tcol);
    c.G[c.n] = pl->at<float>(p.o_g);
    c.ck[c.n] = (int)p.cols;
    ++c.n;
  }
  c.c_T = (int)pl->c_T; c.cx = cx; c.out = out;
  c.lr = lr; c.inv_rT = pl->r_T > 0 ? 1.0f / (float)pl->r_T : 0.0f;
  c.loss_partial = pl->at<float>(pl->lay.o_loss); c.n_loss_partial = n_loss_partial;
  c.loss = loss; c.loss_scale = loss_scale;
  {
    TraceScope ts(pl, "finalize", -1, st);
    HIP_TRY(launch_colasm(c, mode, st));
  }
  return ILARGI_OK;
}

// Alg. 1 for a wide batch on a two-table star join: P = R W_R, the join-order pass (residual, S^T E, segment
// sums), R^T Z, update.  The r_T x m residual is never stored.
ilargi_status_t gd_star_step(ilargi_plan* pl, int mode, float* W, int m, const float* y, const float* lr,
                             float* loss, float loss_scale, bool bf16, hipStream_t st) {
  SourcePlan& f = pl->src[pl->fused];
  SourcePlan& d = pl->src[pl->star_k];
  {
    LmmArgs a;
    memset(&a, 0, sizeof(a));
    a.D = d.D; a.d_rows = d.rows; a.ck = (int)d.cols; a.colmap = pl->at<int32_t>(d.o_colmap);
    a.X = W; a.ldx = m; a.col0 = 0; a.ncols = m;
    a.out = pl->at<float>(d.o_pz); a.ldo = m; a.r_out = d.rows;
    a.logL = pick_logL(d.cols, d.vec);
    a.scratch = pl->at<float>(pl->lay.o_gpartial); a.scratch_floats = pl->lay.gpartial_floats;   // free until the star pass
    TraceScope ts(pl, "lmm_rows", pl->star_k, st);
    HIP_TRY(launch_lmm_mfma(a, d.vec, 0, bf16, st, nullptr));
  }
  StarArgs s;
  memset(&s, 0, sizeof(s));
  s.S = f.D; s.cs = (int)f.cols; s.s_colmap = pl->at<int32_t>(f.o_colmap);
  s.W = W; s.ldw = m; s.m = m;
  s.PZ = pl->at<float>(d.o_pz); s.ldp = m; s.r_R = d.rows;
  s.rowptr = pl->at<int32_t>(d.o_rowptr); s.perm = pl->at<int32_t>(d.o_perm); s.idx = d.idx;
  s.y = y;
  if (pl->cluster_sp != nullptr && pl->cluster_k == pl->star_k) {
    // the join-ordered copy of S (same rows in the same order): a stream instead of gathered rows
    s.Sp = pl->cluster_sp; s.keys = pl->cluster_keys;
    s.yp = y == pl->cluster_y_src ? pl->cluster_yp : nullptr;
  }
  s.loss_partial = pl->at<float>(pl->lay.o_loss); s.ld_loss = m;
  s.grad_partial = pl->at<float>(pl->lay.o_gpartial); s.ld_grad = m;
  const int64_t max_grid = std::min<int64_t>(1024, pl->lay.gpartial_floats / ((int64_t)s.cs * m));
  int grid = 0;
  {
    TraceScope ts(pl, "star_pass", -1, st);
    HIP_TRY(launch_gd_star(s, f.vec, mode, bf16, (int)max_grid, st, &grid));
  }
  HIP_TRY(launch_tred_reduce(s.grad_partial, grid, (int64_t)s.cs * m, pl->at<float>(f.o_g), st));
  TredArgs g;
  memset(&g, 0, sizeof(g));
  g.A = d.D; g.lda = (int)d.cols; g.ca = (int)d.cols; g.a_rows = d.rows;
  g.B = pl->at<float>(d.o_pz); g.ldb = m; g.cb = m; g.bcol0 = 0; g.b_rows = d.rows;
  g.n_rows = d.rows;
  ilargi_status_t rc = run_tred(pl, g, pl->at<float>(d.o_g), "colred", pl->star_k, bf16, st);
  if (rc != ILARGI_OK) return rc;
  ColAsmArgs c;
  memset(&c, 0, sizeof(c));
  for (int k : {std::min(pl->fused, pl->star_k), std::max(pl->fused, pl->star_k)}) {   // source order, as in the general path
    c.tcol2src[c.n] = pl->at<int32_t>(pl->src[k].o_tcol);
    c.G[c.n] = pl->at<float>(pl->src[k].o_g);
    ++c.n;
  }
  c.c_T = (int)pl->c_T; c.cx = m; c.out = W;
  c.lr = lr; c.inv_rT = 1.0f / (float)pl->r_T;
  c.loss_partial = pl->at<float>(pl->lay.o_loss); c.n_loss_partial = grid;
  c.loss = loss; c.loss_scale = loss_scale;
  {
    TraceScope ts(pl, "finalize", -1, st);
    HIP_TRY(launch_colasm(c, 1, st));
  }
  return ILARGI_OK;
}

constexpr int kWideMin = 8;   // operands with at least this many columns take the matrix-core kernels

// a: the c_T-row operand (never empty); b: the r_T-row one, which may be NULL when the target table has no rows.
ilargi_status_t check_call(const ilargi_plan* pl, const void* a, const void* b, int64_t cx, const char* what) {
  if (pl == nullptr) return fail(ILARGI_ERR_NULL, "%s: plan is NULL", what);
  if (a == nullptr || (b == nullptr && pl->r_T > 0)) return fail(ILARGI_ERR_NULL, "%s: operand pointer is NULL", what);
  if (cx < 1) return fail(ILARGI_ERR_SHAPE, "%s: %lld operand columns", what, (long long)cx);
  if (cx > pl->max_cx)
    return fail(ILARGI_ERR_WORKSPACE, "%s: %lld operand columns but the plan was sized for %lld", what,
                (long long)cx, (long long)pl->max_cx);
  return ILARGI_OK;
}

}  // namespace

extern "C" {

const char* ilargi_last_error(void) { return g_err; }
const char* ilargi_version(void) { return "0.1"; }

ilargi_status_t ilargi_plan_workspace_bytes(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                            int64_t max_cx, size_t* bytes) {
  if (bytes == nullptr) return fail(ILARGI_ERR_NULL, "bytes is NULL");
  std::vector<SourcePlan> src;
  Layout lay;
  ilargi_status_t st = make_layout(n, sources, r_T, c_T, max_cx, src, lay);
  if (st != ILARGI_OK) return st;
  *bytes = lay.total;
  return ILARGI_OK;
}

}  // extern "C"

namespace {

// Both ways of creating a plan: static_dev < 0 takes the caller's workspace, static_dev >= 0 the library's
// scratch array of that device (its address in `workspace`).
ilargi_status_t plan_create_impl(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                 int64_t max_cx, void* workspace, size_t workspace_bytes, void* stream,
                                 ilargi_plan_t** plan, int static_dev) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "plan is NULL");
  std::vector<SourcePlan> src;
  Layout lay;
  ilargi_status_t rc = make_layout(n, sources, r_T, c_T, max_cx, src, lay);
  if (rc != ILARGI_OK) return rc;
  // column maps (Def. 1): entries in [-1, c_T), no target column hit twice by one source
  std::vector<std::vector<int32_t>> tcol(n, std::vector<int32_t>((size_t)c_T, -1));
  for (int k = 0; k < n; ++k) {
    if (sources[k].cols > 0 && sources[k].col_map == nullptr) return fail(ILARGI_ERR_NULL, "source %d: col_map is NULL", k);
    if (src[k].sparse) {
      if (sources[k].D != nullptr) return fail(ILARGI_ERR_SHAPE, "source %d: both a dense table and sparse rows are given", k);
      if (sources[k].nnz > 0 && (sources[k].csr_col == nullptr || sources[k].csr_val == nullptr))
        return fail(ILARGI_ERR_NULL, "source %d: csr_col or csr_val is NULL", k);
      src[k].csr_rowptr = sources[k].csr_rowptr;
      src[k].csr_col = sources[k].csr_col;
      src[k].csr_val = sources[k].csr_val;
    } else if (sources[k].rows > 0 && sources[k].cols > 0 && sources[k].D == nullptr) {
      return fail(ILARGI_ERR_NULL, "source %d: D is NULL", k);
    }
    src[k].colmap_h.assign(sources[k].col_map, sources[k].col_map + sources[k].cols);
    for (int64_t j = 0; j < sources[k].cols; ++j) {
      int32_t t = sources[k].col_map[j];
      if (t < -1 || t >= c_T) return fail(ILARGI_ERR_COLMAP, "source %d: col_map[%lld] = %d outside [-1, %lld)", k, (long long)j, t, (long long)c_T);
      if (t < 0) continue;
      if (tcol[k][t] >= 0) return fail(ILARGI_ERR_COLMAP, "source %d: columns %d and %lld both map to target column %d", k, tcol[k][t], (long long)j, t);
      tcol[k][t] = (int32_t)j;
    }
    src[k].D = sources[k].D;
    src[k].idx = sources[k].row_idx;
    src[k].vec = pick_vec(sources[k].D, sources[k].cols);
  }
  if (workspace == nullptr) return fail(ILARGI_ERR_NULL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return fail(ILARGI_ERR_WORKSPACE, "workspace is not %zu-byte aligned", kAlign);
  if (workspace_bytes < lay.total)
    return static_dev >= 0
               ? fail(ILARGI_ERR_WORKSPACE, "plan needs %zu bytes of workspace, the static scratch array holds %zu: "
                      "use ilargi_plan_create with a workspace of the caller", lay.total, workspace_bytes)
               : fail(ILARGI_ERR_WORKSPACE, "workspace has %zu bytes, plan needs %zu", workspace_bytes, lay.total);

  ilargi_plan* pl = new (std::nothrow) ilargi_plan();
  if (pl == nullptr) return fail(ILARGI_ERR_DEVICE, "out of host memory");
  struct Guard { ilargi_plan* p; ~Guard() { delete p; } } guard{pl};
  pl->n = n; pl->r_T = r_T; pl->c_T = c_T; pl->max_cx = max_cx;
  pl->ws = static_cast<char*>(workspace); pl->ws_bytes = workspace_bytes;
  pl->src = std::move(src); pl->lay = lay;
  hipStream_t st = static_cast<hipStream_t>(stream);

  HIP_TRY(hipMemsetAsync(pl->at<int32_t>(lay.o_flags), 0, sizeof(int32_t) * 3 * n, st));
  std::vector<const int32_t*> tcol_ptrs(n);
  for (int k = 0; k < n; ++k) {
    SourcePlan& p = pl->src[k];
    if (p.cols > 0) HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_colmap), p.colmap_h.data(), sizeof(int32_t) * p.cols, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_tcol), tcol[k].data(), sizeof(int32_t) * c_T, hipMemcpyHostToDevice, st));
    tcol_ptrs[k] = pl->at<int32_t>(p.o_tcol);
    if (p.has_idx) HIP_TRY(launch_check_idx(p.idx, r_T, p.rows, pl->at<int32_t>(lay.o_flags) + 2 * k, st));
    if (p.sparse) {
      pl->any_sparse = true;
      SparseArgs sa;
      memset(&sa, 0, sizeof(sa));
      sa.rowptr = p.csr_rowptr; sa.col = p.csr_col; sa.rows = p.rows; sa.cols = (int)p.cols; sa.nnz = p.entries;
      HIP_TRY(launch_csr_check(sa, pl->at<int32_t>(lay.o_flags) + 2 * n + k, st));
    }
  }
  HIP_TRY(hipMemcpyAsync(pl->at<void*>(lay.o_tcol_table), tcol_ptrs.data(), sizeof(void*) * n, hipMemcpyHostToDevice, st));
  std::vector<int32_t> flags(3 * n, 0);
  HIP_TRY(hipMemcpyAsync(flags.data(), pl->at<int32_t>(lay.o_flags), sizeof(int32_t) * 3 * n, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  for (int k = 0; k < n; ++k)
    if (flags[2 * n + k] != 0)
      return fail(ILARGI_ERR_INDEX_RANGE, "source %d: sparse rows are not valid (row pointers must rise from 0 to nnz, "
                  "column indices must lie in [0, cols) and ascend strictly within a row)", k);
  for (int k = 0; k < n; ++k) {
    SourcePlan& p = pl->src[k];
    if (!p.has_idx) { p.ident = true; p.nnz = p.rows; continue; }
    if (flags[2 * k] != 0) return fail(ILARGI_ERR_INDEX_RANGE, "source %d: row_idx has an entry outside [-1, %lld)", k, (long long)p.rows);
    p.ident = flags[2 * k + 1] == 0 && p.rows <= r_T;
    if (p.ident) p.nnz = p.rows;
  }
  // inverse index of every non-identity source (Def. 2, transposed): stable sort by source row
  for (int k = 0; k < n; ++k) {
    SourcePlan& p = pl->src[k];
    if (p.ident) continue;
    int32_t* sortbuf = pl->at<int32_t>(lay.o_sort);
    int64_t rr = std::max<int64_t>(r_T, 1);
    HIP_TRY(launch_sort_by_source_row(p.idx, r_T, p.rows, sortbuf, sortbuf + rr, sortbuf + 2 * rr, sortbuf + 3 * rr,
                                      pl->at<int32_t>(lay.o_hist), pl->at<int32_t>(p.o_rowptr),
                                      pl->at<int32_t>(p.o_perm), st));
    std::vector<int32_t> rowptr((size_t)p.rows + 1);
    HIP_TRY(hipMemcpyAsync(rowptr.data(), pl->at<int32_t>(p.o_rowptr), sizeof(int32_t) * (p.rows + 1), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    p.nnz = rowptr[(size_t)p.rows];
    std::vector<int32_t> cs, cb, ce, ls, lf;
    build_long_tables(rowptr, cs, cb, ce, ls, lf);
    p.n_chunks = (int)cs.size();
    p.n_long = (int)ls.size();
    if (p.n_chunks > p.nch_max || p.n_long > p.nl_max) return fail(ILARGI_ERR_WORKSPACE, "internal: long-segment tables overflow");
    if (p.n_chunks > 0) {
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_chunk_seg), cs.data(), sizeof(int32_t) * cs.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_chunk_beg), cb.data(), sizeof(int32_t) * cb.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_chunk_end), ce.data(), sizeof(int32_t) * ce.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_long_seg), ls.data(), sizeof(int32_t) * ls.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_long_first), lf.data(), sizeof(int32_t) * lf.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipStreamSynchronize(st));
    }
    int64_t avg = p.rows > 0 ? (p.nnz + p.rows - 1) / p.rows : 1;
    p.logG = std::min(6, ilog2_ceil(std::max<int64_t>(avg, 1)));
    if (p.sliced) {
      int64_t slice_rows = (r_T + kSegSlices - 1) / kSegSlices;
      slice_rows = (slice_rows + 63) / 64 * 64;
      HIP_TRY(hipMemsetAsync(pl->at<int32_t>(p.o_sl_nchunk), 0, sizeof(int32_t) * kSegSlices, st));
      // (the sort's buffers are free again: scratch for the runs' positions and for the scan)
      HIP_TRY(launch_build_sliced_index(pl->at<int32_t>(p.o_rowptr), pl->at<int32_t>(p.o_perm), p.rows, p.nnz, slice_rows,
                                        pl->at<int32_t>(p.o_sl_rowptr), pl->at<int32_t>(p.o_sl_perm),
                                        pl->at<int32_t>(p.o_sl_chunk0), pl->at<int32_t>(p.o_sl_ch_beg),
                                        pl->at<int32_t>(p.o_sl_ch_end), pl->at<int32_t>(p.o_sl_nchunk), p.sl_cap,
                                        pl->at<int32_t>(lay.o_sort), pl->at<int32_t>(lay.o_hist), st));
      int32_t nch[kSegSlices];
      HIP_TRY(hipMemcpyAsync(nch, pl->at<int32_t>(p.o_sl_nchunk), sizeof(nch), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      for (int x = 0; x < kSegSlices; ++x)
        if (nch[x] > p.sl_cap) return fail(ILARGI_ERR_WORKSPACE, "internal: chunk table of the sliced index overflows");
      // lanes per (slice, source row) run: about four entries per lane, which it keeps in flight together
      p.sl_logG = std::min(6, ilog2_ceil(std::max<int64_t>((avg + 4 * kSegSlices - 1) / (4 * kSegSlices), 1)));
    }
    if (p.n_long == 0 && p.rows > 0 && !p.sparse && p.nnz <= 32 * p.rows && p.nnz >= 4 * p.rows) {
      // (with more index entries per row the gathers dominate and the segment-sum kernel, which spreads a
      // segment over a group of lanes, serves them better; with about one entry per row the gathers of a round
      // are too few to hide behind the other workgroups' streaming, and segment sums followed by a plain
      // column reduce measure faster: 92 against 109 microseconds on a 2,000,000 x 64 table joined one to one)
      // row ranges of the join-order column reduce, balanced by what a row costs: its table bytes plus a gathered
      // operand row per index entry (priced at 32 bytes); about kColredTarget ranges, none below 64 KiB of cost
      std::vector<int32_t> first;
      const int64_t row_bytes = std::max<int64_t>(p.cols, 1) * 4, entry_bytes = 32;
      const int64_t total = p.rows * row_bytes + p.nnz * entry_bytes;
      const int64_t target = std::max<int64_t>((total + kColredTarget - 1) / kColredTarget, 64 << 10);
      int64_t acc = 0;
      first.push_back(0);
      for (int64_t r = 0; r < p.rows; ++r) {
        acc += row_bytes + (int64_t)(rowptr[(size_t)r + 1] - rowptr[(size_t)r]) * entry_bytes;
        if (acc >= target && r + 1 < p.rows) { first.push_back((int32_t)(r + 1)); acc = 0; }
      }
      first.push_back((int32_t)p.rows);
      if ((int)first.size() - 1 <= kColredBlocks) {
        p.n_join_blocks = (int)first.size() - 1;
        HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_join_first), first.data(), sizeof(int32_t) * first.size(), hipMemcpyHostToDevice, st));
        HIP_TRY(hipStreamSynchronize(st));
      }
    }
  }
  // column-sorted view of every sparse source: the same stable sort, keyed by column index
  for (int k = 0; k < n; ++k) {
    SourcePlan& p = pl->src[k];
    if (!p.sparse) continue;
    int32_t* sortbuf = pl->at<int32_t>(lay.o_sort);
    const int64_t nn = std::max<int64_t>(std::max<int64_t>(r_T, 1), lay.max_entries);
    int32_t* entry_row = pl->at<int32_t>(lay.o_tmp_a);
    int32_t* cperm = pl->at<int32_t>(lay.o_tmp_b);
    SparseArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.rowptr = p.csr_rowptr; sa.col = p.csr_col; sa.val = p.csr_val; sa.rows = p.rows; sa.cols = (int)p.cols; sa.nnz = p.entries;
    {
      // row blocks of the row-wise product (host side, once)
      std::vector<int32_t> rp((size_t)p.rows + 1);
      HIP_TRY(hipMemcpyAsync(rp.data(), p.csr_rowptr, sizeof(int32_t) * (p.rows + 1), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      const int cap = sparse_row_block_cap((int)p.cols);
      if (p.cols > kMaxLdsFloats)
        for (int64_t r = 0; r < p.rows; ++r)
          if (rp[(size_t)r + 1] - rp[(size_t)r] > cap)
            return fail(ILARGI_ERR_UNSUPPORTED, "source %d: a row of a table wider than %d columns holds more than %d entries", k,
                        kMaxLdsFloats, cap);
      std::vector<int32_t> rb;
      rb.push_back(0);
      int64_t r = 0;
      while (r < p.rows) {
        int64_t r2 = r + 1;
        while (r2 < p.rows && r2 - r < kSparseBlockRows && rp[(size_t)r2 + 1] - rp[(size_t)r] <= cap) ++r2;
        rb.push_back((int32_t)r2);
        r = r2;
      }
      p.n_row_blocks = (int)rb.size() - 1;
      if (p.n_row_blocks > p.row_block_max) return fail(ILARGI_ERR_WORKSPACE, "internal: row block table overflow");
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_row_block), rb.data(), sizeof(int32_t) * rb.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipStreamSynchronize(st));
    }
    HIP_TRY(launch_csr_entry_rows(sa, entry_row, st));
    HIP_TRY(launch_sort_by_source_row(p.csr_col, p.entries, p.cols, sortbuf, sortbuf + nn, sortbuf + 2 * nn, sortbuf + 3 * nn,
                                      pl->at<int32_t>(lay.o_hist), pl->at<int32_t>(p.o_colptr), cperm, st));
    HIP_TRY(launch_csr_gather_rows(entry_row, p.csr_val, cperm, p.entries, pl->at<int32_t>(p.o_csc_row),
                                   pl->at<float>(p.o_csc_val), st));
    std::vector<int32_t> colptr((size_t)p.cols + 1);
    HIP_TRY(hipMemcpyAsync(colptr.data(), pl->at<int32_t>(p.o_colptr), sizeof(int32_t) * (p.cols + 1), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (colptr[(size_t)p.cols] != p.entries) return fail(ILARGI_ERR_DEVICE, "internal: column view of source %d lost entries", k);
    std::vector<int32_t> cb, ce, first((size_t)p.cols + 1, 0);
    for (int64_t j = 0; j < p.cols; ++j) {
      first[(size_t)j] = (int32_t)cb.size();
      for (int32_t b = colptr[(size_t)j]; b < colptr[(size_t)j + 1]; b += kSparseChunk) {
        cb.push_back(b);
        ce.push_back(std::min(colptr[(size_t)j + 1], b + kSparseChunk));
      }
    }
    first[(size_t)p.cols] = (int32_t)cb.size();
    p.n_tchunks = (int)cb.size();
    if (p.n_tchunks > p.tchunk_max) return fail(ILARGI_ERR_WORKSPACE, "internal: column chunk table overflow");
    if (p.n_tchunks > 0) {
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_tchunk_beg), cb.data(), sizeof(int32_t) * cb.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_tchunk_end), ce.data(), sizeof(int32_t) * ce.size(), hipMemcpyHostToDevice, st));
    }
    HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(p.o_col_first), first.data(), sizeof(int32_t) * first.size(), hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
  }
  // the dense identity source with the most cells has its product fused into the assembly pass
  int64_t best = -1;
  for (int k = 0; k < n; ++k) {
    const SourcePlan& p = pl->src[k];
    if (p.ident && !p.empty && !p.sparse && p.rows * p.cols > best) { best = p.rows * p.cols; pl->fused = k; }
  }
  // scalar operators: which element-wise operators may act on the sources alone, the vector of ones of
  // rowSum and the fan-out vectors of colSum
  {
    pl->cover_disjoint = true;
    pl->cover_full = true;
    for (int64_t t = 0; t < c_T; ++t) {
      int feeders = 0;
      for (int k = 0; k < n; ++k) feeders += (!pl->src[k].empty && tcol[k][(size_t)t] >= 0) ? 1 : 0;
      if (feeders > 1) pl->cover_disjoint = false;
      if (feeders == 0) pl->cover_full = false;
    }
    for (int k = 0; k < n; ++k)
      if (!pl->src[k].empty && pl->src[k].nnz != r_T) pl->cover_full = false;
    HIP_TRY(launch_fill(pl->at<float>(lay.o_ones), c_T, 1.0f, st));
    for (int k = 0; k < n; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty) continue;
      if (p.ident) HIP_TRY(launch_fill(pl->at<float>(p.o_cnt), p.rows, 1.0f, st));
      else HIP_TRY(launch_fanout(pl->at<int32_t>(p.o_rowptr), p.rows, pl->at<float>(p.o_cnt), st));
    }
  }
  // two-table star join: a full-height identity source plus one table that every target row joins, without
  // very long segments; wide batches of models then run their gradient pass in join order
  {
    int live = 0, dim = -1;
    for (int k = 0; k < n; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty) continue;
      ++live;
      if (k != pl->fused) dim = k;
    }
    if (live == 2 && pl->fused >= 0 && dim >= 0 && !pl->any_sparse) {
      const SourcePlan& f = pl->src[pl->fused];
      const SourcePlan& d = pl->src[dim];
      if (f.rows == r_T && d.has_idx && !d.ident && d.nnz == r_T && d.n_long == 0) pl->star_k = dim;
    }
  }
  // a small two-table star join (or a small single table): one gradient-descent iteration then runs as a
  // single workgroup with the tables in registers, which replaces five dependent launches by one
  {
    int live = 0, ki = -1, kj = -1;
    for (int k = 0; k < n; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty) continue;
      ++live;
      if (p.ident && ki < 0) ki = k; else kj = k;
    }
    bool ok = !pl->any_sparse && ki >= 0 && live <= 2 && c_T <= 1024 && r_T >= 1;
    if (ok) {
      const SourcePlan& f = pl->src[ki];
      ok = f.rows == r_T && f.vec == 4 && f.cols <= 16 && r_T <= small_star_max_rows((int)f.cols / 4);
    }
    if (ok && live == 2) {
      const SourcePlan& d = pl->src[kj];
      ok = !d.ident && d.vec == 4 && d.cols <= 16 && d.rows <= 1024 && d.n_long == 0 && d.nnz <= 16384;
    }
    if (ok) {
      SmallStarArgs probe;
      memset(&probe, 0, sizeof(probe));
      probe.r_T = (int)r_T; probe.nnz = live == 2 ? (int)pl->src[kj].nnz : 0;
      probe.cs = (int)pl->src[ki].cols;
      if (live == 2) { probe.R = pl->src[kj].D; probe.cr = (int)pl->src[kj].cols; }
      ok = small_star_lds_bytes(probe) <= kSmallGdMaxLds;
    }
    pl->small_gd = ok;
    pl->small_ident = ki; pl->small_joined = live == 2 ? kj : -1;
  }
  // sources whose rows feed fewer than two target rows on average (union-style integration): a gradient-descent
  // iteration of one model joins the rows on the fly, reading every table once, when that moves clearly fewer
  // bytes than the factorized sequence (fused source once, every other source for its product and its column reduce)
  {
    int live = 0;
    bool ok = !pl->any_sparse;
    double bytes_join = 0.0, bytes_fact = 0.0;
    for (int k = 0; k < n && ok; ++k) {
      const SourcePlan& p = pl->src[k];
      if (p.empty) continue;
      ++live;
      ok = live <= kRowJoinSources && p.vec == 4 && p.cols % 4 == 0 && p.cols <= 64 &&
           reinterpret_cast<uintptr_t>(p.D) % 16 == 0;
      bytes_join += 4.0 * (double)p.nnz * (double)p.cols;
      bytes_fact += (k == pl->fused ? 4.0 : 8.0) * (double)p.rows * (double)p.cols + (p.ident ? 0.0 : 24.0 * (double)r_T);
    }
    pl->rowjoin_gd = ok && live >= 2 && r_T >= 1 && bytes_join <= 0.85 * bytes_fact;
  }
  // join-gather tables: groups of four target columns fed by four consecutive columns of one source
  if (c_T % 4 == 0) {
    std::vector<int32_t> gslot((size_t)c_T / 4, -1), gj0((size_t)c_T / 4, 0);
    bool regular = true, flat = true;
    for (int64_t g = 0; g < c_T / 4 && regular; ++g) {
      int slot = 0;
      for (int k = 0; k < n && regular; ++k) {
        if (pl->src[k].empty) continue;
        int hits = 0;
        for (int e = 0; e < 4; ++e) hits += tcol[k][4 * g + e] >= 0;
        if (hits == 4 && gslot[g] < 0 && tcol[k][4 * g + 1] == tcol[k][4 * g] + 1 &&
            tcol[k][4 * g + 2] == tcol[k][4 * g] + 2 && tcol[k][4 * g + 3] == tcol[k][4 * g] + 3) {
          gslot[g] = slot;
          gj0[g] = tcol[k][4 * g];
          if (gj0[g] % 4 != 0 || pl->src[k].cols % 4 != 0 || reinterpret_cast<uintptr_t>(pl->src[k].D) % 16 != 0) flat = false;
        } else if (hits != 0) {
          regular = false;
        }
        ++slot;
      }
    }
    pl->mat_vec4 = regular;
    pl->mat_flat = regular && flat;
    if (regular) {
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(lay.o_gslot), gslot.data(), sizeof(int32_t) * gslot.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(lay.o_gj0), gj0.data(), sizeof(int32_t) * gj0.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipStreamSynchronize(st));
    }
  }
  // join-gather tables, general form: the first two feeders of every target column, in source order
  {
    std::vector<int32_t> cs((size_t)2 * c_T, -1), cj((size_t)2 * c_T, 0);
    bool ok = true;
    for (int64_t t = 0; t < c_T && ok; ++t) {
      int found = 0, slot = 0;
      for (int k = 0; k < n; ++k) {
        if (pl->src[k].empty) continue;
        if (tcol[k][t] >= 0) {
          if (found == 2) { ok = false; break; }
          cs[2 * t + found] = slot;
          cj[2 * t + found] = tcol[k][t];
          ++found;
        }
        ++slot;
      }
    }
    pl->mat_cols = ok;
    if (ok) {
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(lay.o_ct_slot), cs.data(), sizeof(int32_t) * cs.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(pl->at<int32_t>(lay.o_ct_j), cj.data(), sizeof(int32_t) * cj.size(), hipMemcpyHostToDevice, st));
      HIP_TRY(hipStreamSynchronize(st));
    }
  }
  // Gram blocks (k <= l) and the table the assembly kernel walks
  pl->block_off.assign((size_t)n * n, 0);
  std::vector<GramAsmPair> pairs;
  size_t boff = 0;
  for (int k = 0; k < n; ++k)
    for (int l = k; l < n; ++l) {
      pl->block_off[(size_t)k * n + l] = boff;
      if (!pl->src[k].empty && !pl->src[l].empty) {
        GramAsmPair pr;
        pr.block = pl->at<float>(lay.o_blocks) + boff;
        pr.k = k; pr.l = l; pr.cb = (int)pl->src[l].cols;
        pairs.push_back(pr);
      }
      boff += (size_t)(pl->src[k].cols * pl->src[l].cols);
    }
  // pair lists of the source pairs whose Gram block is formed over the rows both feed
  for (int i = 0; i < lay.n_pairlists; ++i) {
    const SourcePlan& a = pl->src[lay.pairlist_k[i]];
    const SourcePlan& b = pl->src[lay.pairlist_l[i]];
    int32_t* scan = pl->at<int32_t>(lay.o_sort);                 // free again: r_T + 1 integers
    int32_t* list = pl->at<int32_t>(lay.o_pairlist[i]);
    HIP_TRY(launch_pair_list(a.ident ? nullptr : a.idx, a.rows, b.ident ? nullptr : b.idx, b.rows, r_T, scan,
                             pl->at<int32_t>(lay.o_hist), list, list + r_T, st));
    int32_t cnt = 0;
    HIP_TRY(hipMemcpyAsync(&cnt, scan + r_T, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    pl->pairlist_n[i] = cnt;
  }
  pl->npairs = (int)pairs.size();
  if (!pairs.empty())
    HIP_TRY(hipMemcpyAsync(pl->at<GramAsmPair>(lay.o_pairs), pairs.data(), sizeof(GramAsmPair) * pairs.size(), hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));
  pl->static_dev = static_dev;
  guard.p = nullptr;
  *plan = pl;
  return ILARGI_OK;
}

}  // namespace

extern "C" {

ilargi_status_t ilargi_plan_create(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                   int64_t max_cx, void* workspace, size_t workspace_bytes, void* stream,
                                   ilargi_plan_t** plan) {
  return plan_create_impl(n, sources, r_T, c_T, max_cx, workspace, workspace_bytes, stream, plan, -1);
}

ilargi_status_t ilargi_plan_create_static(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                          int64_t max_cx, void* stream, ilargi_plan_t** plan) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "plan is NULL");
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(ILARGI_ERR_DEVICE, "device %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticSlot& slot = g_static[dev];
  if (slot.ptr == nullptr) {
    // once per device, with that device current: every GPU holds its own copy of the array at its own address
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr || reinterpret_cast<uintptr_t>(p) % kAlign != 0)
      return fail(ILARGI_ERR_DEVICE, "the static scratch array has no usable device address");
    slot.ptr = p;
  }
  if (slot.owner != nullptr)
    return fail(ILARGI_ERR_WORKSPACE, "the static scratch array of device %d is held by a live plan: destroy it first", dev);
  ilargi_plan_t* pl = nullptr;
  ilargi_status_t rc = plan_create_impl(n, sources, r_T, c_T, max_cx, slot.ptr, kStaticScratchBytes, stream, &pl, dev);
  if (rc != ILARGI_OK) return rc;
  slot.owner = pl;
  *plan = pl;
  return ILARGI_OK;
}

size_t ilargi_static_scratch_bytes(void) { return kStaticScratchBytes; }

namespace {
// A two-table star join (full-height identity source, one other source that every target row joins, segments of any
// length) whose tables the one-pass kernel takes: the joined source, or -1.
int cluster_dim(const ilargi_plan* pl) {
  if (pl->fused < 0 || pl->any_sparse || pl->r_T < 1) return -1;
  int live = 0, dim = -1;
  for (int k = 0; k < pl->n; ++k) {
    if (pl->src[k].empty) continue;
    ++live;
    if (k != pl->fused) dim = k;
  }
  if (live != 2 || dim < 0) return -1;
  const SourcePlan& f = pl->src[pl->fused];
  const SourcePlan& d = pl->src[dim];
  const bool ok = gd_cluster_supported((int)f.cols, (int)d.cols) && f.rows == pl->r_T && d.has_idx && !d.ident &&
                  d.nnz == pl->r_T && d.rows >= 1 && reinterpret_cast<uintptr_t>(f.D) % 16 == 0 &&
                  reinterpret_cast<uintptr_t>(d.D) % 16 == 0;
  return ok ? dim : -1;
}
}  // namespace

ilargi_status_t ilargi_plan_cluster_bytes(const ilargi_plan_t* plan, size_t* bytes) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "plan_cluster_bytes: plan is NULL");
  if (bytes == nullptr) return fail(ILARGI_ERR_NULL, "plan_cluster_bytes: bytes is NULL");
  if (cluster_dim(plan) < 0)
    return fail(ILARGI_ERR_UNSUPPORTED, "plan_cluster: needs a two-table star join (entity table of 4..32 columns, dimension "
                                        "table of 4..256 columns, whole aligned float4 rows, every target row joined)");
  const SourcePlan& f = plan->src[plan->fused];
  *bytes = align_up(sizeof(float) * (size_t)plan->r_T * (size_t)f.cols) + 2 * align_up(sizeof(int32_t) * (size_t)plan->r_T);
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_cluster(ilargi_plan_t* plan, void* buffer, size_t buffer_bytes, const float* y, void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "plan_cluster: plan is NULL");
  if (buffer == nullptr) {
    plan->cluster_sp = nullptr;
    plan->cluster_keys = nullptr;
    plan->cluster_y_src = plan->cluster_yp = nullptr;
    return ILARGI_OK;
  }
  size_t need = 0;
  ilargi_status_t rc = ilargi_plan_cluster_bytes(plan, &need);
  if (rc != ILARGI_OK) return rc;
  if (reinterpret_cast<uintptr_t>(buffer) % kAlign != 0) return fail(ILARGI_ERR_WORKSPACE, "plan_cluster: buffer is not 256-byte aligned");
  if (buffer_bytes < need)
    return fail(ILARGI_ERR_WORKSPACE, "plan_cluster: buffer of %zu bytes, %zu needed", buffer_bytes, need);
  const int dim = cluster_dim(plan);
  const SourcePlan& f = plan->src[plan->fused];
  const SourcePlan& d = plan->src[dim];
  float* sp = static_cast<float*>(buffer);
  int32_t* keys = reinterpret_cast<int32_t*>(static_cast<char*>(buffer) + align_up(sizeof(float) * (size_t)plan->r_T * (size_t)f.cols));
  float* yp = reinterpret_cast<float*>(reinterpret_cast<char*>(keys) + align_up(sizeof(int32_t) * (size_t)plan->r_T));
  plan->cluster_sp = nullptr;
  plan->cluster_keys = nullptr;
  plan->cluster_y_src = plan->cluster_yp = nullptr;
  HIP_TRY(launch_cluster_rows(f.D, (int)f.cols, plan->at<int32_t>(d.o_perm), d.idx, plan->r_T, sp, keys, y, yp,
                              static_cast<hipStream_t>(stream)));
  plan->cluster_sp = sp;
  plan->cluster_keys = keys;
  plan->cluster_k = dim;
  if (y != nullptr) { plan->cluster_y_src = y; plan->cluster_yp = yp; }
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_destroy(ilargi_plan_t* plan) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "plan is NULL");
  if (plan->static_dev >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static[plan->static_dev].owner == plan) g_static[plan->static_dev].owner = nullptr;
  }
  delete plan;
  return ILARGI_OK;
}

ilargi_status_t ilargi_stream_probe(int kind, float* dst, const float* src, int64_t n_floats, int blocks, void* stream) {
  if (kind < 0 || kind > 6) return fail(ILARGI_ERR_UNSUPPORTED, "stream_probe: kind %d", kind);
  if (dst == nullptr || (kind != 2 && kind != 4 && src == nullptr)) return fail(ILARGI_ERR_NULL, "stream_probe: NULL buffer");
  if (n_floats < 0 || n_floats % 4 != 0 || blocks < 1 || blocks > (1 << 22)) return fail(ILARGI_ERR_SHAPE, "stream_probe: bad size");
  HIP_TRY(launch_probe(kind, dst, src, n_floats, blocks, static_cast<hipStream_t>(stream)));
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_trace_begin(ilargi_plan_t* plan, const char* tag, int max_launches) {
  if (plan == nullptr || tag == nullptr) return fail(ILARGI_ERR_NULL, "trace_begin: NULL argument");
  if (max_launches < 1 || max_launches > (1 << 20)) return fail(ILARGI_ERR_SHAPE, "trace_begin: max_launches = %d", max_launches);
  for (hipEvent_t e : plan->trace_events) (void)hipEventDestroy(e);
  plan->trace_events.clear();
  plan->trace_names.clear();
  plan->trace_n = 0;
  plan->trace_tag = tag;
  for (int i = 0; i < 2 * max_launches; ++i) {
    hipEvent_t e;
    HIP_TRY(hipEventCreate(&e));
    plan->trace_events.push_back(e);
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_trace_label(ilargi_plan_t* plan, const char* label) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "trace_label: plan is NULL");
  plan->trace_label = label ? label : "";
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_trace_name(const ilargi_plan_t* plan, int i, char* buf, int buf_len) {
  if (plan == nullptr || buf == nullptr) return fail(ILARGI_ERR_NULL, "trace_name: NULL argument");
  if (i < 0 || i >= (int)plan->trace_names.size() || buf_len < 1) return fail(ILARGI_ERR_SHAPE, "trace_name: index %d", i);
  snprintf(buf, (size_t)buf_len, "%s", plan->trace_names[(size_t)i].c_str());
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_trace_end(ilargi_plan_t* plan, float* ms, int capacity, int* count) {
  if (plan == nullptr || count == nullptr) return fail(ILARGI_ERR_NULL, "trace_end: NULL argument");
  int n = plan->trace_n / 2;
  *count = n;
  for (int i = 0; i < n && i < capacity && ms != nullptr; ++i) {
    HIP_TRY(hipEventSynchronize(plan->trace_events[2 * i + 1]));
    HIP_TRY(hipEventElapsedTime(&ms[i], plan->trace_events[2 * i], plan->trace_events[2 * i + 1]));
  }
  for (hipEvent_t e : plan->trace_events) (void)hipEventDestroy(e);
  plan->trace_events.clear();
  plan->trace_n = 0;
  plan->trace_tag.clear();
  plan->trace_label.clear();
  return ILARGI_OK;
}

ilargi_status_t ilargi_plan_inverse_index(const ilargi_plan_t* plan, int k, const int32_t** rowptr,
                                          const int32_t** perm, int64_t* nnz) {
  if (plan == nullptr || rowptr == nullptr || perm == nullptr || nnz == nullptr) return fail(ILARGI_ERR_NULL, "inverse_index: NULL argument");
  if (k < 0 || k >= plan->n) return fail(ILARGI_ERR_SHAPE, "inverse_index: source %d of %d", k, plan->n);
  const SourcePlan& p = plan->src[k];
  if (p.ident) { *rowptr = nullptr; *perm = nullptr; *nnz = p.rows; return ILARGI_OK; }
  *rowptr = plan->at<int32_t>(p.o_rowptr);
  *perm = plan->at<int32_t>(p.o_perm);
  *nnz = p.nnz;
  return ILARGI_OK;
}

ilargi_status_t ilargi_lmm(ilargi_plan_t* plan, const float* X, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream) {
  ilargi_status_t rc = check_call(plan, X, out, cx, "lmm");
  if (rc != ILARGI_OK) return rc;
  const bool bf16 = precision == ILARGI_BF16_IN_F32_ACC;
  if (precision != ILARGI_F32 && !bf16) return fail(ILARGI_ERR_UNSUPPORTED, "lmm: unknown precision %d", (int)precision);
  if (bf16 && cx < kWideMin) return fail(ILARGI_ERR_UNSUPPORTED, "lmm: bf16 inputs need an operand with at least %d columns", kWideMin);
  if (bf16 && plan->any_sparse) return fail(ILARGI_ERR_UNSUPPORTED, "lmm: bf16 inputs need dense source tables");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (cx >= kWideMin && !plan->any_sparse) return lmm_pass(plan, X, (int)cx, 0, (int)cx, out, (int)cx, 0, nullptr, nullptr, true, st, nullptr, bf16);
  const int w = pass_width(plan);
  for (int64_t col0 = 0; col0 < cx; col0 += w) {
    int ncols = (int)std::min<int64_t>(w, cx - col0);
    rc = lmm_pass(plan, X, (int)cx, (int)col0, ncols, out, (int)cx, 0, nullptr, nullptr, false, st);
    if (rc != ILARGI_OK) return rc;
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_tmm(ilargi_plan_t* plan, const float* Y, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream) {
  ilargi_status_t rc = check_call(plan, out, Y, cx, "tmm");
  if (rc != ILARGI_OK) return rc;
  const bool bf16 = precision == ILARGI_BF16_IN_F32_ACC;
  if (precision != ILARGI_F32 && !bf16) return fail(ILARGI_ERR_UNSUPPORTED, "tmm: unknown precision %d", (int)precision);
  if (bf16 && cx < kWideMin) return fail(ILARGI_ERR_UNSUPPORTED, "tmm: bf16 inputs need an operand with at least %d columns", kWideMin);
  if (bf16 && plan->any_sparse) return fail(ILARGI_ERR_UNSUPPORTED, "tmm: bf16 inputs need dense source tables");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (cx >= kWideMin && !plan->any_sparse) return tmm_wide(plan, Y, (int)cx, out, 0, nullptr, nullptr, 0, 0.0f, bf16, st);
  for (int64_t col0 = 0; col0 < cx; col0 += kNarrowCT) {
    int ncols = (int)std::min<int64_t>(kNarrowCT, cx - col0);
    rc = tmm_pass(plan, Y, (int)cx, (int)col0, ncols, out, (int)cx, 0, nullptr, nullptr, 0, 0.0f, st);
    if (rc != ILARGI_OK) return rc;
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_rmm(ilargi_plan_t* plan, const float* X, int64_t cx, float* out,
                           ilargi_precision_t precision, void* stream) {
  // X T = (T^T X^T)^T: a one-row operand is its own transpose; otherwise transpose in, multiply, transpose out
  if (cx == 1) return ilargi_tmm(plan, X, 1, out, precision, stream);
  ilargi_status_t rc = check_call(plan, out, X, cx, "rmm");
  if (rc != ILARGI_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* Xt = plan->at<float>(plan->lay.o_E);          // r_T x cx
  float* Gt = plan->at<float>(plan->lay.o_rmm);        // c_T x cx
  HIP_TRY(launch_transpose(X, cx, plan->r_T, Xt, st));
  rc = ilargi_tmm(plan, Xt, cx, Gt, precision, stream);
  if (rc != ILARGI_OK) return rc;
  HIP_TRY(launch_transpose(Gt, plan->c_T, cx, out, st));
  return ILARGI_OK;
}

ilargi_status_t ilargi_gd_step(ilargi_plan_t* plan, ilargi_model_t model, float* W, int64_t m, const float* y,
                               const float* lr, float* loss, ilargi_precision_t precision, void* stream) {
  ilargi_status_t rc = check_call(plan, W, y, m, "gd_step");
  if (rc != ILARGI_OK) return rc;
  if (lr == nullptr) return fail(ILARGI_ERR_NULL, "gd_step: lr is NULL");
  if (model != ILARGI_LINEAR && model != ILARGI_LOGISTIC) return fail(ILARGI_ERR_UNSUPPORTED, "gd_step: unknown model %d", (int)model);
  if (plan->r_T < 1) return fail(ILARGI_ERR_SHAPE, "gd_step: the target table has no rows");
  const bool bf16 = precision == ILARGI_BF16_IN_F32_ACC;
  if (precision != ILARGI_F32 && !bf16) return fail(ILARGI_ERR_UNSUPPORTED, "gd_step: unknown precision %d", (int)precision);
  if (bf16 && m < kWideMin) return fail(ILARGI_ERR_UNSUPPORTED, "gd_step: bf16 inputs need at least %d models", kWideMin);
  if (bf16 && plan->any_sparse) return fail(ILARGI_ERR_UNSUPPORTED, "gd_step: bf16 inputs need dense source tables");
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* E = plan->at<float>(plan->lay.o_E);
  const int w = pass_width(plan);
  const float loss_scale = (model == ILARGI_LINEAR ? 0.5f : 1.0f) / (float)plan->r_T;
  if (plan->small_gd && !bf16 && m <= kNarrowCT) {
    // small schema: the whole iteration of a model in one launch of one workgroup
    SmallStarArgs a;
    memset(&a, 0, sizeof(a));
    const SourcePlan& f = plan->src[plan->small_ident];
    a.S = f.D; a.cs = (int)f.cols; a.tcol_s = plan->at<int32_t>(f.o_tcol);
    for (int j = 0; j < 16; ++j) {
      a.colmap[0][j] = j < f.cols ? (int16_t)f.colmap_h[(size_t)j] : (int16_t)-1;
      a.colmap[1][j] = -1;
    }
    a.s_first = 1;
    if (plan->small_joined >= 0) {
      const SourcePlan& d = plan->src[plan->small_joined];
      a.R = d.D; a.cr = (int)d.cols; a.r_R = (int)d.rows; a.idx = d.idx;
      a.rowptr = plan->at<int32_t>(d.o_rowptr); a.perm = plan->at<int32_t>(d.o_perm); a.nnz = (int)d.nnz;
      a.tcol_r = plan->at<int32_t>(d.o_tcol);
      for (int j = 0; j < d.cols; ++j) a.colmap[1][j] = (int16_t)d.colmap_h[(size_t)j];
      a.s_first = plan->small_ident < plan->small_joined ? 1 : 0;
    }
    a.W = W; a.ldw = (int)m; a.y = y; a.lr = lr; a.loss = loss;
    a.r_T = (int)plan->r_T; a.c_T = (int)plan->c_T;
    a.inv_rT = 1.0f / (float)plan->r_T; a.loss_scale = loss_scale;
    for (int col = 0; col < (int)m; ++col) {
      a.col = col;
      TraceScope ts(plan, "small_gd", -1, st);
      HIP_TRY(launch_small_star(a, model == ILARGI_LINEAR ? 1 : 2, st));
    }
    return ILARGI_OK;
  }
  // Every row of the dimension table costs the one-pass iteration two reductions over a wavefront, however few target
  // rows it serves: the pass pays from a fan-out of about four on (level at four, measured), or when the dimension
  // table is the larger of the two (then reading it once instead of twice outweighs that arithmetic).  Measured on the
  // benchmark's tuple-ratio x feature-ratio grid; below that the usual sequence is faster and is kept.
  const bool cluster_pays = plan->cluster_sp != nullptr &&
                            (plan->r_T >= 4 * plan->src[plan->cluster_k].rows ||
                             plan->src[plan->cluster_k].rows * plan->src[plan->cluster_k].cols >=
                                 plan->src[plan->fused].rows * plan->src[plan->fused].cols);
  if (cluster_pays && !bf16 && m == 1) {
    // clustered entity table: both tables are streams, every table read once, nothing but partial sums written
    const SourcePlan& fs = plan->src[plan->fused];
    const SourcePlan& d = plan->src[plan->cluster_k];
    ClusterArgs a;
    memset(&a, 0, sizeof(a));
    a.Sp = plan->cluster_sp; a.cs = (int)fs.cols;
    a.keys = plan->cluster_keys; a.perm = plan->at<int32_t>(d.o_perm);
    a.R = d.D; a.cr = (int)d.cols; a.r_R = d.rows;
    a.s_colmap = plan->at<int32_t>(fs.o_colmap); a.r_colmap = plan->at<int32_t>(d.o_colmap);
    a.W = W; a.ldw = (int)m; a.col = 0; a.y = y; a.r_T = plan->r_T;
    a.yp = y == plan->cluster_y_src ? plan->cluster_yp : nullptr;   // the labels the copy was made with
    a.loss_partial = plan->at<float>(plan->lay.o_loss);
    a.grad_partial_s = plan->at<float>(fs.o_partial);
    a.grad_partial_r = plan->at<float>(d.o_partial);
    int grid = 0;
    {
      TraceScope ts(plan, "gd_cluster", -1, st);
      HIP_TRY(launch_gd_cluster(a, model == ILARGI_LINEAR ? 1 : 2, kColredBlocks, st, &grid));
    }
    FinArgs f;
    memset(&f, 0, sizeof(f));
    for (int k = 0; k < plan->n; ++k) {
      const SourcePlan& p = plan->src[k];
      if (p.empty) continue;
      const int s = f.n++;
      f.s[s].tcol2src = plan->at<int32_t>(p.o_tcol);
      f.s[s].partial = plan->at<float>(p.o_partial);
      f.s[s].ck = (int)p.cols;
      f.s[s].nblocks = grid;
    }
    f.out = W; f.ldo = 1; f.col0 = 0; f.ncols = 1;
    f.lr = lr; f.inv_rT = 1.0f / (float)plan->r_T;
    f.loss_partial = a.loss_partial; f.n_loss_partial = grid; f.loss = loss; f.loss_scale = loss_scale;
    TraceScope ts(plan, "finalize", -1, st);
    HIP_TRY(launch_finalize(f, (int)plan->c_T, 1, st));
    return ILARGI_OK;
  }
  if (plan->rowjoin_gd && !bf16 && m == 1) {
    // every table read once: product, residual and every source's block of the gradient in one pass
    RowJoinArgs a;
    memset(&a, 0, sizeof(a));
    FinArgs f;
    memset(&f, 0, sizeof(f));
    for (int k = 0; k < plan->n; ++k) {
      const SourcePlan& p = plan->src[k];
      if (p.empty) continue;
      const int s = a.n++;
      a.D[s] = p.D; a.ck[s] = (int)p.cols; a.rows[s] = p.rows;
      a.idx[s] = p.ident ? nullptr : p.idx;
      a.colmap[s] = plan->at<int32_t>(p.o_colmap);
      a.grad_partial[s] = plan->at<float>(p.o_partial);
      f.s[s].tcol2src = plan->at<int32_t>(p.o_tcol);
      f.s[s].partial = plan->at<float>(p.o_partial);
      f.s[s].ck = (int)p.cols;
    }
    a.W = W; a.ldw = (int)m; a.col = 0; a.y = y; a.r_T = plan->r_T;
    a.loss_partial = plan->at<float>(plan->lay.o_loss);
    int grid = 0;
    {
      TraceScope ts(plan, "gd_rowjoin", -1, st);
      HIP_TRY(launch_gd_rowjoin(a, model == ILARGI_LINEAR ? 1 : 2, kColredBlocks, st, &grid));
    }
    f.n = a.n;
    for (int s = 0; s < f.n; ++s) f.s[s].nblocks = grid;
    f.out = W; f.ldo = 1; f.col0 = 0; f.ncols = 1;
    f.lr = lr; f.inv_rT = 1.0f / (float)plan->r_T;
    f.loss_partial = a.loss_partial; f.n_loss_partial = grid; f.loss = loss; f.loss_scale = loss_scale;
    TraceScope ts(plan, "finalize", -1, st);
    HIP_TRY(launch_finalize(f, (int)plan->c_T, 1, st));
    return ILARGI_OK;
  }
  if (plan->star_k >= 0 && gd_star_supported((int)plan->src[plan->fused].cols, (int)m) &&
      (int64_t)plan->src[plan->fused].cols * m <= plan->lay.gpartial_floats)
    return gd_star_step(plan, model == ILARGI_LINEAR ? 1 : 2, W, (int)m, y, lr, loss, loss_scale, bf16, st);
  if (m >= kWideMin && !plan->any_sparse) {
    int loss_grid = 0;
    bool fusedg = false;
    rc = lmm_pass(plan, W, (int)m, 0, (int)m, E, (int)m, model == ILARGI_LINEAR ? 1 : 2, y, &loss_grid, true, st,
                  &fusedg, bf16);
    if (rc != ILARGI_OK) return rc;
    return tmm_wide(plan, E, (int)m, W, 1, lr, loss, loss_grid, loss_scale, bf16, st, fusedg ? plan->fused : -1);
  }
  for (int64_t col0 = 0; col0 < m; col0 += w) {
    int ncols = (int)std::min<int64_t>(w, m - col0);
    int loss_grid = 0;
    bool fusedg = false;
    rc = lmm_pass(plan, W, (int)m, (int)col0, ncols, E, (int)m, model == ILARGI_LINEAR ? 1 : 2, y, &loss_grid, false, st,
                  &fusedg);
    if (rc != ILARGI_OK) return rc;
    rc = tmm_pass(plan, E, (int)m, (int)col0, ncols, W, (int)m, 1, lr, loss, loss_grid, loss_scale, st,
                  fusedg ? plan->fused : -1, loss_grid);
    if (rc != ILARGI_OK) return rc;
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_kmeans_step(ilargi_plan_t* plan, float* C, int64_t k, int32_t* assign, int32_t* counts,
                                   void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "kmeans_step: plan is NULL");
  if (C == nullptr) return fail(ILARGI_ERR_NULL, "kmeans_step: C is NULL");
  if (k < 1) return fail(ILARGI_ERR_SHAPE, "kmeans_step: %lld centroids", (long long)k);
  if (k > plan->max_cx)
    return fail(ILARGI_ERR_WORKSPACE, "kmeans_step: %lld centroids but the plan was sized for %lld operand columns",
                (long long)k, (long long)plan->max_cx);
  if (k > kKmeansMaxK) return fail(ILARGI_ERR_UNSUPPORTED, "kmeans_step: more than %d centroids", kKmeansMaxK);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* P = plan->at<float>(plan->lay.o_E);            // r_T x k: T C, then the assignment matrix
  float* G = plan->at<float>(plan->lay.o_rmm);          // c_T x k: per-cluster sums
  float* cn = plan->at<float>(plan->lay.o_cn);
  int32_t* cnt = plan->at<int32_t>(plan->lay.o_counts);
  HIP_TRY(launch_fill_zero(reinterpret_cast<float*>(cnt), k, st));   // all-zero bits are the integer 0
  if (plan->r_T > 0) {
    {
      TraceScope ts(plan, "centroid_norm", -1, st);
      HIP_TRY(launch_centroid_norm(C, plan->c_T, (int)k, cn, st));
    }
    ilargi_status_t rc = ilargi_lmm(plan, C, k, P, ILARGI_F32, stream);
    if (rc != ILARGI_OK) return rc;
    {
      TraceScope ts(plan, "kmeans_assign", -1, st);
      HIP_TRY(launch_kmeans_assign(P, cn, plan->r_T, (int)k, assign, plan->at<int32_t>(plan->lay.o_loss),
                                   std::max<int64_t>(32768 * kNarrowCT, 1024 * plan->max_cx), cnt, st));
    }
    rc = ilargi_tmm(plan, P, k, G, ILARGI_F32, stream);
    if (rc != ILARGI_OK) return rc;
  }
  TraceScope ts(plan, "kmeans_update", -1, st);
  HIP_TRY(launch_kmeans_update(C, G, cnt, plan->c_T, (int)k, counts, st));
  return ILARGI_OK;
}

ilargi_status_t ilargi_gnmf_step(ilargi_plan_t* plan, float* W, float* Ht, int64_t r, void* stream) {
  ilargi_status_t rc = check_call(plan, Ht, W, r, "gnmf_step");
  if (rc != ILARGI_OK) return rc;
  if (r > kGnmfMaxRank) return fail(ILARGI_ERR_UNSUPPORTED, "gnmf_step: rank above %d", kGnmfMaxRank);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* P = plan->at<float>(plan->lay.o_E);            // r_T x r: T H^T
  float* G = plan->at<float>(plan->lay.o_rmm);          // c_T x r: T^T W
  float* HHt = plan->at<float>(plan->lay.o_rr);
  float* WtW = HHt + kGnmfMaxRank * kGnmfMaxRank;
  const float tiny = 1e-30f;
  auto small_gram = [&](const float* A, int64_t rows, float* out, const char* tag) -> ilargi_status_t {
    // out (r x r) = A^T A for a rows x r matrix, chunk sums added in order
    if (rows <= 0) { HIP_TRY(launch_fill_zero(out, r * r, st)); return ILARGI_OK; }
    TredArgs g;
    memset(&g, 0, sizeof(g));
    g.A = A; g.lda = (int)r; g.ca = (int)r; g.a_rows = rows;
    g.B = A; g.ldb = (int)r; g.cb = (int)r; g.b_rows = rows;
    g.n_rows = rows;
    return run_tred(plan, g, out, tag, -1, false, st);
  };
  rc = small_gram(Ht, plan->c_T, HHt, "gnmf_hht");
  if (rc != ILARGI_OK) return rc;
  if (plan->r_T > 0) {
    rc = ilargi_lmm(plan, Ht, r, P, ILARGI_F32, stream);
    if (rc != ILARGI_OK) return rc;
    // the update also leaves each workgroup's share of W_new^T W_new, added here in workgroup order
    float* part = plan->at<float>(plan->lay.o_gpartial);
    int nparts = 0;
    {
      TraceScope ts(plan, "gnmf_update", 0, st);
      HIP_TRY(launch_gnmf_update(W, P, HHt, plan->r_T, (int)r, tiny, part, plan->lay.gpartial_floats, &nparts, st));
    }
    HIP_TRY(launch_tred_reduce(part, nparts, r * r, WtW, st));
  } else {
    HIP_TRY(launch_fill_zero(WtW, r * r, st));
  }
  if (plan->r_T > 0) {
    rc = ilargi_tmm(plan, W, r, G, ILARGI_F32, stream);
    if (rc != ILARGI_OK) return rc;
  } else {
    HIP_TRY(launch_fill_zero(G, plan->c_T * r, st));
  }
  TraceScope ts(plan, "gnmf_update", 1, st);
  HIP_TRY(launch_gnmf_update(Ht, G, WtW, plan->c_T, (int)r, tiny, nullptr, 0, nullptr, st));
  return ILARGI_OK;
}

ilargi_status_t ilargi_elementwise(ilargi_plan_t* plan, ilargi_elementwise_t op, float x, float* const* D_out,
                                   void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "elementwise: plan is NULL");
  if (D_out == nullptr) return fail(ILARGI_ERR_NULL, "elementwise: D_out is NULL");
  const int o = (int)op;
  if (o < 0 || o > (int)ILARGI_OP_SQUARE) return fail(ILARGI_ERR_UNSUPPORTED, "elementwise: unknown operator %d", o);
  // which cover of the target cells the factorized form needs (Tab. 2 states the cost, not the condition)
  const bool linear = op == ILARGI_OP_MUL || op == ILARGI_OP_DIV;
  const bool keeps_zero = op == ILARGI_OP_SQRT || op == ILARGI_OP_ABS || op == ILARGI_OP_SQUARE ||
                          (op == ILARGI_OP_POW && x > 0.0f);
  if (!linear && !plan->cover_disjoint)
    return fail(ILARGI_ERR_UNSUPPORTED, "elementwise: operator %d needs target columns fed by one source each", o);
  if (!linear && !keeps_zero && !plan->cover_full)
    return fail(ILARGI_ERR_UNSUPPORTED, "elementwise: operator %d needs every target cell fed by a source cell", o);
  if (plan->any_sparse && !linear && !keeps_zero)
    return fail(ILARGI_ERR_UNSUPPORTED, "elementwise: operator %d does not keep the zeros a sparse table leaves out", o);
  for (int k = 0; k < plan->n; ++k) {
    const SourcePlan& p = plan->src[k];
    if (!p.empty && !(p.sparse && p.entries == 0) && D_out[k] == nullptr)
      return fail(ILARGI_ERR_NULL, "elementwise: D_out[%d] is NULL", k);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  // an entity table rewritten in place no longer matches its join-ordered copy: the plan forgets the copy
  if (plan->cluster_sp != nullptr && D_out[plan->fused] == plan->src[plan->fused].D) {
    plan->cluster_sp = nullptr;
    plan->cluster_keys = nullptr;
    plan->cluster_y_src = plan->cluster_yp = nullptr;
  }
  for (int k = 0; k < plan->n; ++k) {
    const SourcePlan& p = plan->src[k];
    if (p.empty) continue;
    TraceScope ts(plan, "elementwise", k, st);
    if (p.sparse) {
      // the stored entries; updated in place, the plan's column-sorted copy of the values follows
      HIP_TRY(launch_elementwise(o, p.csr_val, D_out[k], p.entries, x, st));
      if (D_out[k] == p.csr_val)
        HIP_TRY(launch_elementwise(o, plan->at<float>(p.o_csc_val), plan->at<float>(p.o_csc_val), p.entries, x, st));
    } else {
      HIP_TRY(launch_elementwise(o, p.D, D_out[k], p.rows * p.cols, x, st));
    }
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_row_sum(ilargi_plan_t* plan, float* out, void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "row_sum: plan is NULL");
  if (plan->r_T == 0) return ILARGI_OK;
  if (out == nullptr) return fail(ILARGI_ERR_NULL, "row_sum: out is NULL");
  return lmm_pass(plan, plan->at<float>(plan->lay.o_ones), 1, 0, 1, out, 1, 0, nullptr, nullptr, false,
                  static_cast<hipStream_t>(stream));
}

ilargi_status_t ilargi_col_sum(ilargi_plan_t* plan, float* out, void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "col_sum: plan is NULL");
  if (out == nullptr) return fail(ILARGI_ERR_NULL, "col_sum: out is NULL");
  return tmm_pass(plan, nullptr, 1, 0, 1, out, 1, 0, nullptr, nullptr, 0, 0.0f, static_cast<hipStream_t>(stream));
}

ilargi_status_t ilargi_segment_sum(ilargi_plan_t* plan, int k, const float* Y, int64_t cx, float* Z, void* stream) {
  ilargi_status_t rc = check_call(plan, Z, Y, cx, "segment_sum");
  if (rc != ILARGI_OK) return rc;
  if (k < 0 || k >= plan->n) return fail(ILARGI_ERR_SHAPE, "segment_sum: source %d of %d", k, plan->n);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const SourcePlan& p = plan->src[k];
  if (p.rows == 0) return ILARGI_OK;
  if (p.ident) {
    HIP_TRY(hipMemcpyAsync(Z, Y, sizeof(float) * p.rows * cx, hipMemcpyDeviceToDevice, st));
    return ILARGI_OK;
  }
  SegArgs s = seg_args(plan, k);
  s.Y = Y; s.ldy = (int)cx; s.col0 = 0; s.ncols = (int)cx;
  s.Z = Z; s.ldz = (int)cx; s.zcol0 = 0;
  HIP_TRY(launch_segsum(s, st));
  return ILARGI_OK;
}

ilargi_status_t ilargi_materialize(ilargi_plan_t* plan, float* T, void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "materialize: plan is NULL");
  if (plan->r_T == 0) return ILARGI_OK;
  if (T == nullptr) return fail(ILARGI_ERR_NULL, "materialize: T is NULL");
  if (plan->any_sparse) {
    // zero, then one pass per source in source order: every cell receives its terms in the order of the sum
    hipStream_t st = static_cast<hipStream_t>(stream);
    TraceScope ts(plan, "materialize", -1, st);
    HIP_TRY(launch_fill_zero(T, plan->r_T * plan->c_T, st));
    for (int k = 0; k < plan->n; ++k) {
      const SourcePlan& p = plan->src[k];
      if (p.empty) continue;
      const int32_t* idx = p.ident ? nullptr : p.idx;
      if (p.sparse) {
        SparseArgs sa = sparse_args(plan, k);
        HIP_TRY(launch_mat_scatter(&sa, nullptr, p.rows, (int)p.cols, sa.colmap, idx, p.rows, T, plan->r_T, (int)plan->c_T, st));
      } else {
        HIP_TRY(launch_mat_scatter(nullptr, p.D, p.rows, (int)p.cols, plan->at<int32_t>(p.o_colmap), idx, p.rows, T,
                                   plan->r_T, (int)plan->c_T, st));
      }
    }
    return ILARGI_OK;
  }
  MatArgs a;
  memset(&a, 0, sizeof(a));
  for (int k = 0; k < plan->n; ++k) {
    const SourcePlan& p = plan->src[k];
    if (p.empty) continue;
    a.D[a.n] = p.D;
    a.idx[a.n] = p.ident ? nullptr : p.idx;
    a.tcol2src[a.n] = plan->at<int32_t>(p.o_tcol);
    a.rows[a.n] = p.rows;
    a.ck[a.n] = (int)p.cols;
    ++a.n;
  }
  a.T = T; a.r_T = plan->r_T; a.c_T = (int)plan->c_T;
  a.gslot = plan->mat_vec4 ? plan->at<int32_t>(plan->lay.o_gslot) : nullptr;
  a.gj0 = plan->mat_vec4 ? plan->at<int32_t>(plan->lay.o_gj0) : nullptr;
  a.flat_ok = plan->mat_flat ? 1 : 0;
  a.ct_slot = plan->mat_cols ? plan->at<int32_t>(plan->lay.o_ct_slot) : nullptr;
  a.ct_j = plan->mat_cols ? plan->at<int32_t>(plan->lay.o_ct_j) : nullptr;
  {
    TraceScope ts(plan, "materialize", -1, static_cast<hipStream_t>(stream));
    HIP_TRY(launch_materialize(a, static_cast<hipStream_t>(stream)));
  }
  return ILARGI_OK;
}

ilargi_status_t ilargi_crossprod(ilargi_plan_t* plan, float* out, void* stream) {
  if (plan == nullptr) return fail(ILARGI_ERR_NULL, "crossprod: plan is NULL");
  if (out == nullptr) return fail(ILARGI_ERR_NULL, "crossprod: out is NULL");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (plan->any_sparse) {
    // T^T T = T^T (T I): the identity goes through the two multiplies a block of columns at a time, which only
    // needs the products the sparse kernels have.  Block j gives columns j0.. of the result, written as its rows
    // j0.. (the result is symmetric); the cells below the diagonal are then copied from above it, so that the
    // result is symmetric to the bit like the dense route's.
    const int64_t c_T = plan->c_T;
    if (c_T > kSparseGramMaxCols)
      return fail(ILARGI_ERR_UNSUPPORTED, "crossprod: more than %lld target columns over sparse source tables", (long long)kSparseGramMaxCols);
    const int w = (int)std::min<int64_t>(plan->max_cx, kSparseGramWidth);
    float* E = plan->at<float>(plan->lay.o_eye);
    float* P = plan->at<float>(plan->lay.o_E);
    float* G = plan->at<float>(plan->lay.o_rmm);
    for (int64_t j0 = 0; j0 < c_T; j0 += w) {
      const int cw = (int)std::min<int64_t>(w, c_T - j0);
      HIP_TRY(launch_eye_block(E, c_T, cw, j0, st));
      ilargi_status_t rc = ilargi_lmm(plan, E, cw, P, ILARGI_F32, stream);
      if (rc != ILARGI_OK) return rc;
      rc = ilargi_tmm(plan, P, cw, G, ILARGI_F32, stream);
      if (rc != ILARGI_OK) return rc;
      HIP_TRY(launch_transpose(G, c_T, cw, out + j0 * c_T, st));
    }
    HIP_TRY(launch_mirror_upper(out, c_T, st));
    return ILARGI_OK;
  }
  const int n = plan->n;
  float* blocks = plan->at<float>(plan->lay.o_blocks);
  float* zc = plan->at<float>(plan->lay.o_zc);
  // The diagonal block of the dimension table of a two-table star join does not depend on the pass over the
  // entity table: with a second stream it runs beside it, each with its own half of the partial-block space.
  float* gpart = plan->at<float>(plan->lay.o_gpartial);
  const int64_t gfloats = plan->lay.gpartial_floats;
  bool forked = false;
  float* part_main = gpart;
  int64_t part_main_floats = gfloats;
  auto run_gram = [&](TredArgs& g, float* block, int pair) -> ilargi_status_t {
    return run_tred(plan, g, block, "gram", pair, false, st, false, part_main, part_main_floats);   // traced as gram:<k * n + l>
  };
  // two-table star join with a narrow entity table listed first: S^T S and the rows of S summed per row of R
  // (which the off-diagonal block needs) come from one pass over S in join order
  bool star_done = false;
  if (plan->star_k >= 0 && plan->fused < plan->star_k) {
    const SourcePlan& f = plan->src[plan->fused];
    const SourcePlan& d = plan->src[plan->star_k];
    const int64_t max_grid = std::min<int64_t>(1024, gfloats / 2 / std::max<int64_t>(f.cols * f.cols, 1));
    if (gram_star_supported((int)f.cols) && d.rows * 2 <= plan->r_T && d.rows * f.cols <= plan->lay.zc_floats && max_grid >= 1) {
      const bool fork = d.cols * d.cols <= gfloats / 2 && side_stream(plan, st) != nullptr;
      if (fork) {
        HIP_TRY(hipEventRecord(plan->ev_fork, st));
        part_main_floats = gfloats / 2;
      }
      GramStarArgs ga;
      memset(&ga, 0, sizeof(ga));
      ga.S = f.D; ga.cs = (int)f.cols; ga.r_R = d.rows;
      ga.rowptr = plan->at<int32_t>(d.o_rowptr); ga.perm = plan->at<int32_t>(d.o_perm); ga.idx = d.idx;
      // (a join-ordered copy of S kept with the plan turns the gathered rows into a stream; same sums, same order)
      ga.Sp = (plan->cluster_sp != nullptr && plan->cluster_k == plan->star_k) ? plan->cluster_sp : nullptr;
      ga.ss_partial = gpart;
      ga.zc = zc;
      int grid = 0;
      {
        TraceScope ts(plan, "gram_star", -1, st);
        HIP_TRY(launch_gram_star(ga, f.vec, (int)max_grid, st, &grid));
      }
      if (fork) {
        // R^T diag(cnt) R on the second stream, upper half of the partial space (enqueued after the pass over S, which
        // is bound by memory latency and leaves the matrix cores to it)
        HIP_TRY(hipStreamWaitEvent(plan->side, plan->ev_fork, 0));
        TredArgs g;
        memset(&g, 0, sizeof(g));
        g.A = d.D; g.lda = (int)d.cols; g.ca = (int)d.cols; g.a_rows = d.rows;
        g.B = d.D; g.ldb = (int)d.cols; g.cb = (int)d.cols; g.b_rows = d.rows;
        g.wptr = plan->at<int32_t>(d.o_rowptr);
        g.n_rows = d.rows;
        g.upper_only = 1;
        ilargi_status_t rc = run_tred(plan, g, blocks + plan->block_off[(size_t)plan->star_k * n + plan->star_k], "gram",
                                      plan->star_k * n + plan->star_k, false, plan->side, false, gpart + gfloats / 2, gfloats / 2);
        if (rc != ILARGI_OK) return rc;
        HIP_TRY(hipEventRecord(plan->ev_join, plan->side));
        forked = true;
      }
      HIP_TRY(launch_tred_reduce(ga.ss_partial, grid, f.cols * f.cols,
                                 blocks + plan->block_off[(size_t)plan->fused * n + plan->fused], st));
      star_done = true;
    }
  }
  for (int k = 0; k < n; ++k) {
    const SourcePlan& a = plan->src[k];
    if (a.empty) continue;
    for (int l = k; l < n; ++l) {
      const SourcePlan& b = plan->src[l];
      if (b.empty) continue;
      if (star_done && k == plan->fused && l == k) continue;   // S^T S is done
      if (forked && k == plan->star_k && l == k) continue;     // this block is on the second stream
      float* block = blocks + plan->block_off[(size_t)k * n + l];
      TredArgs g;
      memset(&g, 0, sizeof(g));
      ilargi_status_t rc;
      if (l == k) {
        g.A = a.D; g.lda = (int)a.cols; g.ca = (int)a.cols; g.a_rows = a.rows;
        g.B = a.D; g.ldb = (int)a.cols; g.cb = (int)a.cols; g.b_rows = a.rows;
        g.wptr = a.ident ? nullptr : plan->at<int32_t>(a.o_rowptr);
        g.n_rows = a.rows;
        g.upper_only = 1;
        rc = run_gram(g, block, k * n + l);
      } else {
        bool via_l = !b.ident && b.rows * 2 <= plan->r_T;
        bool via_k = !a.ident && a.rows * 2 <= plan->r_T;
        if (via_l && via_k) { if (a.rows < b.rows) via_l = false; else via_k = false; }
        if (via_l) {
          // Zc = I_l^T (I_k D_k):  rows of D_k summed per source row of l, then  Zc^T D_l
          SegArgs s = seg_args(plan, l);
          s.Y = a.D; s.ldy = (int)a.cols; s.col0 = 0; s.ncols = (int)a.cols;
          s.gidx = a.ident ? nullptr : a.idx; s.g_rows = a.ident ? a.rows : -1;
          s.Z = zc; s.ldz = (int)a.cols; s.zcol0 = 0;
          if (!(star_done && k == plan->fused && l == plan->star_k)) HIP_TRY(launch_segsum(s, st));   // else zc is ready
          g.A = zc; g.lda = (int)a.cols; g.ca = (int)a.cols; g.a_rows = b.rows;
          g.B = b.D; g.ldb = (int)b.cols; g.cb = (int)b.cols; g.b_rows = b.rows;
          g.n_rows = b.rows;
          if (a.cols <= 32 && b.cols >= 64) {
            // few summed columns against a wide table: the wide table takes the A role (whole rows as float4,
            // 128 columns per workgroup) and the block is written transposed, D_l^T Zc = (Zc^T D_l)^T
            std::swap(g.A, g.B); std::swap(g.lda, g.ldb); std::swap(g.ca, g.cb); std::swap(g.a_rows, g.b_rows);
            rc = run_tred(plan, g, block, "gram", k * n + l, false, st, true, part_main, part_main_floats);
            if (rc != ILARGI_OK) return rc;
            continue;
          }
        } else if (via_k) {
          SegArgs s = seg_args(plan, k);
          s.Y = b.D; s.ldy = (int)b.cols; s.col0 = 0; s.ncols = (int)b.cols;
          s.gidx = b.ident ? nullptr : b.idx; s.g_rows = b.ident ? b.rows : -1;
          s.Z = zc; s.ldz = (int)b.cols; s.zcol0 = 0;
          HIP_TRY(launch_segsum(s, st));
          g.A = a.D; g.lda = (int)a.cols; g.ca = (int)a.cols; g.a_rows = a.rows;
          g.B = zc; g.ldb = (int)b.cols; g.cb = (int)b.cols; g.b_rows = a.rows;
          g.n_rows = a.rows;
        } else {
          g.A = a.D; g.lda = (int)a.cols; g.ca = (int)a.cols; g.a_rows = a.rows;
          g.B = b.D; g.ldb = (int)b.cols; g.cb = (int)b.cols; g.b_rows = b.rows;
          int li = -1;
          for (int i = 0; i < plan->lay.n_pairlists; ++i)
            if (plan->lay.pairlist_k[i] == k && plan->lay.pairlist_l[i] == l) li = i;
          if (li >= 0) {
            // the rows both sources feed were listed with the plan: a streaming kernel over the pairs
            const int32_t* list = plan->at<int32_t>(plan->lay.o_pairlist[li]);
            g.ia = list; g.ib = list + plan->r_T; g.n_rows = plan->pairlist_n[li];
            if (g.n_rows == 0) {
              HIP_TRY(launch_fill_zero(block, (int64_t)g.ca * g.cb, st));
              continue;
            }
            if (gram_pairs_supported(g) && (int64_t)g.ca * g.cb <= part_main_floats) {
              int nch = 0;
              {
                TraceScope ts(plan, "gram", k * n + l, st);
                HIP_TRY(launch_gram_narrow(g, part_main, part_main_floats, st, &nch));
              }
              HIP_TRY(launch_tred_reduce(part_main, nch, (int64_t)g.ca * g.cb, block, st, 0));
              continue;
            }
          }
          g.ia = a.ident ? nullptr : a.idx;
          g.ib = b.ident ? nullptr : b.idx;
          g.n_rows = plan->r_T;
        }
        rc = run_gram(g, block, k * n + l);
      }
      if (rc != ILARGI_OK) return rc;
    }
  }
  if (forked) HIP_TRY(hipStreamWaitEvent(st, plan->ev_join, 0));   // join
  HIP_TRY(launch_gram_assemble(plan->at<GramAsmPair>(plan->lay.o_pairs), plan->npairs,
                               plan->at<const int32_t*>(plan->lay.o_tcol_table), (int)plan->c_T, out, st));
  return ILARGI_OK;
}

}  // extern "C"
