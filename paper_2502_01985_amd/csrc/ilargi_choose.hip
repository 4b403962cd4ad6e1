// Factorize or materialize?  (Sec. 3: complexity ratio of Eq. (1), the tuple-ratio / feature-ratio rule the
// paper compares with, and the estimator input of Sec. 3.3 that prices memory traffic against the
// memory bandwidth, turned into a prediction.)  Host code only: reads shapes, touches no device.
//
// The byte model prices one gradient-descent iteration of this library, operator by operator:
//   factorized   tables: the largest identity source once (its product, residual and gradient share a pass),
//                every other source twice (product, column reduce); per gathered source the row index and the
//                inverse index (4 r_T each) and its product / segment-sum vectors; residual and labels;
//   materialized the same formulas for the single identity source T;
//   join         written table + one source row fetched per target row and gathered source (rows of a table
//                larger than the caches are fetched again for every target row that uses them) + indices.
// Two properties of the kernels enter: the shared pass over an identity source exists for tables of at most
// 256 columns (wider ones are read twice), and a gathered row narrower than 32 bytes still costs a 32-byte
// fetch (the 4-byte gathers of a one-model pass are priced at 32 bytes each).
// Launches are priced separately: a dependent launch costs a few microseconds whatever it moves, which decides
// small schemas.
// Stacked tables (an identity source that ends before the target table does: union-style integration) are the
// one case where the shapes say how many target rows a gathered source reaches: at most its own row count.  If
// fetching those rows once per target row is clearly cheaper than the factorized sequence, an iteration of one
// model joins the rows on the fly and reads every table once; the same rule as in the plan decides.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "ilargi_internal.h"

namespace {
constexpr double kFusedMaxCols = 256.0;   // widest table whose product, residual and gradient share one pass
constexpr double kMinFetch = 32.0;        // bytes a gathered row costs at least
}  // namespace

extern "C" ilargi_status_t ilargi_choose(int n, const ilargi_source_t* sources, int64_t r_T, int64_t c_T,
                                         const ilargi_workload_t* workload, ilargi_choice_t* out) {
  if (sources == nullptr || out == nullptr) return ilargi::set_error(ILARGI_ERR_NULL, "choose: sources or out is NULL");
  if (n < 1 || n > 16 || r_T < 0 || c_T < 1) return ilargi::set_error(ILARGI_ERR_SHAPE, "choose: n outside [1, 16], r_T < 0 or c_T < 1");
  for (int k = 0; k < n; ++k)
    if (sources[k].rows < 0 || sources[k].cols < 0) return ilargi::set_error(ILARGI_ERR_SHAPE, "choose: a source has negative rows or cols");
  ilargi_workload_t w = {200, 1, 0.0, 0.0};
  if (workload != nullptr) w = *workload;
  if (w.iterations < 1 || w.models < 1) return ilargi::set_error(ILARGI_ERR_SHAPE, "choose: iterations and models must be at least 1");
  const double bw = w.bytes_per_second > 0.0 ? w.bytes_per_second : 5.0e12;
  const double launch = w.launch_seconds > 0.0 ? w.launch_seconds : 2.5e-6;

  const double rT = (double)r_T, cT = (double)c_T, mT = rT * cT;
  // Eq. (1) for linear regression with dense operands: w is c_T x 1 (m_w = c_T), X = T w is r_T x 1 (m_X = r_T)
  double o_fact = 0.0;
  for (int k = 0; k < n; ++k) {
    const double rk = (double)sources[k].rows, ck = (double)sources[k].cols;
    const double mk = sources[k].csr_rowptr != nullptr ? (double)sources[k].nnz : rk * ck;   // non-zero elements
    o_fact += (mk + rk * cT) + (mk + ck * rT);
  }
  const double o_mat = (mT + rT * cT) + (mT + cT * rT);
  out->complexity_ratio = o_fact > 0.0 ? o_mat / o_fact : 1.0;

  // tuple ratio and feature ratio: target rows per row of the joined tables, joined columns per base column
  double base_cols = 0.0, joined_rows = 0.0, joined_cols = 0.0;
  int fused = -1;
  double fused_cells = -1.0;
  for (int k = 0; k < n; ++k) {
    const double rk = (double)sources[k].rows, ck = (double)sources[k].cols;
    if (sources[k].row_idx == nullptr) {
      base_cols += ck;
      if (sources[k].csr_rowptr == nullptr && rk * ck > fused_cells) { fused_cells = rk * ck; fused = k; }
    } else {
      joined_rows += rk;
      joined_cols += ck;
    }
  }
  out->tuple_ratio = joined_rows > 0.0 ? rT / joined_rows : 0.0;
  out->feature_ratio = base_cols > 0.0 ? joined_cols / base_cols : 0.0;
  out->morpheus_rule = (joined_rows > 0.0 && out->tuple_ratio >= 5.0 && out->feature_ratio >= 1.0) ? 1 : 0;

  // bytes and launches of one iteration, for one pass of up to four models
  const double pass_models = (double)std::min<int64_t>(w.models, 4);
  const double passes = std::ceil((double)w.models / 4.0);
  const double vec = 4.0 * pass_models;                    // bytes of one row of an operand slice
  double b_fact = 0.0, join_fetch = 0.0;
  int launches_fact = 2;                                   // assembly pass, update
  for (int k = 0; k < n; ++k) {
    const double rk = (double)sources[k].rows, ck = (double)sources[k].cols;
    const bool sparse = sources[k].csr_rowptr != nullptr;
    // a stored entry of a sparse table is a value and a column index (a row index in the column-sorted view)
    const double cells = sparse ? 8.0 * (double)sources[k].nnz + 4.0 * rk : 4.0 * rk * ck;
    if (rk == 0.0 || ck == 0.0) continue;
    if (k == fused && !sparse) {
      const bool one_pass = ck <= kFusedMaxCols;
      b_fact += one_pass ? cells : 2.0 * cells;
      launches_fact += one_pass ? 0 : 1;
      join_fetch += cells;
      continue;
    }
    b_fact += 2.0 * cells;                                 // product, column reduce
    launches_fact += 2;
    if (sources[k].row_idx != nullptr) {
      b_fact += 8.0 * rT + 4.0 * vec * rk;                 // row index, inverse index; P_k written and gathered, Z_k written and read
      b_fact += 2.0 * std::max(vec, kMinFetch) * rT;       // gathered product rows, residual rows read by the segment sum
      launches_fact += 1;
      join_fetch += (sparse && rk > 0.0 ? cells / rk : 4.0 * ck) * rT + 4.0 * rT;   // one source row per target row, row index
    } else {
      b_fact += 2.0 * vec * rk + vec * rT;
      join_fetch += cells;
    }
  }
  b_fact += (vec + 4.0) * rT + 2.0 * vec * cT;             // residual written, labels, weights in and out
  // a small two-table star join (or a small table alone) runs an iteration of one model as a single launch
  const auto small_star = [&](int ns, const ilargi_source_t* s, int64_t rows_T) {
    int live = 0, ident = -1, joined = -1;
    for (int k = 0; k < ns; ++k) {
      if (s[k].rows == 0 || s[k].cols == 0) continue;
      ++live;
      if (s[k].csr_rowptr != nullptr) return false;
      if (s[k].row_idx == nullptr && ident < 0) ident = k; else joined = k;
    }
    if (ident < 0 || live > 2 || c_T > 1024 || rows_T < 1 || w.models > 4) return false;
    const int64_t ci = s[ident].cols;
    if (s[ident].rows != rows_T || ci > 16 || ci % 4 != 0 || rows_T > 1024 * (16 / (ci / 4))) return false;
    if (live == 2) {
      const ilargi_source_t& d = s[joined];
      if (d.row_idx == nullptr || d.cols > 16 || d.cols % 4 != 0 || d.rows > 1024 || rows_T > 16384) return false;
    }
    return true;
  };
  if (small_star(n, sources, r_T)) launches_fact = 1;
  {
    bool stacked = false, ok = w.models == 1;
    for (int k = 0; k < n; ++k)
      if (sources[k].row_idx == nullptr && sources[k].rows > 0 && sources[k].cols > 0 && sources[k].rows < r_T) stacked = true;
    int live = 0, gathered = 0;
    double fetch = 0.0, seq = 0.0;
    for (int k = 0; k < n && ok; ++k) {
      const double rk = (double)sources[k].rows, ck = (double)sources[k].cols;
      if (rk == 0.0 || ck == 0.0) continue;
      ++live;
      ok = sources[k].csr_rowptr == nullptr && sources[k].cols <= 64 && sources[k].cols % 4 == 0 && live <= ilargi::kRowJoinSources;
      const bool ident = sources[k].row_idx == nullptr;
      gathered += ident ? 0 : 1;
      fetch += 4.0 * (ident ? rk : std::min(rT, rk)) * ck;
      seq += (k == fused ? 4.0 : 8.0) * rk * ck + (ident ? 0.0 : 24.0 * rT);
    }
    if (ok && stacked && live >= 2 && launches_fact != 1 && fetch <= 0.85 * seq) {
      b_fact = fetch + 4.0 * rT * (double)gathered + 4.0 * rT + 2.0 * vec * cT;
      launches_fact = 2;
    }
  }
  const bool mat_one_pass = cT <= kFusedMaxCols;
  const double b_mat = (mat_one_pass ? 4.0 : 8.0) * mT + (vec + 4.0) * rT + 2.0 * vec * cT;
  ilargi_source_t joined_table;
  memset(&joined_table, 0, sizeof(joined_table));
  joined_table.rows = r_T; joined_table.cols = c_T;
  const double launches_mat = small_star(1, &joined_table, r_T) ? 1.0 : (mat_one_pass ? 2.0 : 3.0);
  const double b_join = 4.0 * mT + join_fetch;
  out->bytes_factorized = b_fact * passes;
  out->bytes_materialized = b_mat * passes;
  out->bytes_join = b_join;
  const double it = (double)w.iterations;
  // (the single-launch iteration serves one model per launch)
  const double fact_launches = launches_fact == 1 ? (double)w.models / passes : (double)launches_fact;
  out->seconds_factorized = it * passes * (b_fact / bw + fact_launches * launch);
  out->seconds_materialized = b_join / bw + launch + it * passes * (b_mat / bw + launches_mat * launch);
  out->factorize = out->seconds_factorized <= out->seconds_materialized ? 1 : 0;
  return ILARGI_OK;
}
