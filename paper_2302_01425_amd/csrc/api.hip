// C ABI of the library: argument validation and dispatch.  See include/sparse_topk.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/sparse_topk.h"
#include "launch.hpp"

namespace {

using topk::Reg;
using topk::RowInfo;
using topk::RowSel;
using topk::SortBuffers;

struct Workspace {
  void* ptr = nullptr;
  size_t bytes = 0;
};
Workspace g_ws;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// 0: p = 2, 1: p = 4/3, -1: anything else
int p_code(double p) {
  if (std::fabs(p - 2.0) < 1e-9) return topk::kP2;
  if (std::fabs(p - 4.0 / 3.0) < 1e-6) return topk::kP43;
  return -1;
}

Reg make_reg(double lambda) {
  Reg R;
  R.lambda = lambda;
  R.inv_lambda = 1.0 / lambda;
  R.lam3 = lambda * lambda * lambda;
  R.inv_lam3 = 1.0 / R.lam3;
  R.one_p_lambda = 1.0 + lambda;
  R.inv_1pl = 1.0 / (1.0 + lambda);
  return R;
}

bool is_long(int64_t n) { return n > TOPK_SHORT_ROW_MAX; }

// How rows above TOPK_SHORT_ROW_MAX are handled.  Default: one fused launch up to
// topk::kMediumRowMax elements, candidate selection + sort of the candidates above.  Through
// topk_set_route the multi-launch selection path can be chosen for every such row, or a complete
// sort of the rows (same results; for tests and comparisons).
enum LongMode { kAuto = TOPK_LONG_ROWS_AUTO, kSelect = TOPK_LONG_ROWS_SELECT,
                kFullSort = TOPK_LONG_ROWS_SORT, kWide = TOPK_LONG_ROWS_WIDE,
                kOneLaunchIndexed = TOPK_LONG_ROWS_ONE_LAUNCH_INDEXED };
LongMode long_mode() { return static_cast<LongMode>(topk::routes().long_rows); }

// Rows of 1025..2048 elements still fit one wavefront's registers as values: the values-only
// kernel takes them in one launch without scratch (it is not built for top-k in magnitude with
// p = 4/3; a route forced through topk_set_route uses the long-row kernels and their scratch).
bool value_wide(bool mag, int pc, int64_t n) {
  return is_long(n) && n <= 2048 && long_mode() == kAuto &&
         topk::routes().short_kernel == TOPK_SHORT_ROW_KERNEL_AUTO &&
         (pc == topk::kP2 || (pc == topk::kP43 && !mag));
}

struct Layout {
  size_t keys_a, keys_b, idx_a, idx_b, hist, dtot, info, hpart, bins, bins2, tcnt, tabove, toff, taboff, sel, total;
};

Layout layout_for(int64_t rows, int64_t n) {
  Layout L;
  const size_t elems = size_t(rows) * size_t(n);
  const size_t tiles = size_t(topk::radix_tiles(n));
  size_t off = 0;
  L.keys_a = off; off += align_up(elems * 4);
  L.keys_b = off; off += align_up(elems * 4);
  L.idx_a = off; off += align_up(elems * 4);
  L.idx_b = off; off += align_up(elems * 4);
  L.hist = off; off += align_up(size_t(rows) * 256 * tiles * 4);
  L.dtot = off; off += align_up(size_t(rows) * 256 * 4);
  L.info = off; off += align_up(size_t(rows) * sizeof(RowInfo));
  L.hpart = off; off += align_up(size_t(rows) * topk::sel_parts(rows, n) * topk::kSelBins * 4);
  L.bins = off; off += align_up(size_t(rows) * topk::kSelSlices * topk::kSelBins * 4);
  L.bins2 = off; off += align_up(size_t(rows) * topk::kSelSlices * 2 * topk::kSel2Bins * 4);
  L.tcnt = off; off += align_up(size_t(rows) * tiles * 4);
  L.tabove = off; off += align_up(size_t(rows) * tiles * 4);
  L.toff = off; off += align_up(size_t(rows) * tiles * 4);
  L.taboff = off; off += align_up(size_t(rows) * tiles * 4);
  L.sel = off; off += align_up(size_t(rows) * sizeof(RowSel));
  L.total = off;
  return L;
}

// `skip`: bytes at the start of the workspace that the caller keeps for itself
int carve(int64_t rows, int64_t n, SortBuffers* B, size_t skip = 0, const Workspace& ws = g_ws) {
  const Layout L = layout_for(rows, n);
  if (ws.ptr == nullptr || ws.bytes < skip + L.total) return TOPK_ERR_WORKSPACE;
  char* base = static_cast<char*>(ws.ptr) + skip;
  B->keys_a = reinterpret_cast<uint32_t*>(base + L.keys_a);
  B->keys_b = reinterpret_cast<uint32_t*>(base + L.keys_b);
  B->idx_a = reinterpret_cast<uint32_t*>(base + L.idx_a);
  B->idx_b = reinterpret_cast<uint32_t*>(base + L.idx_b);
  B->hist = reinterpret_cast<uint32_t*>(base + L.hist);
  B->dtot = reinterpret_cast<uint32_t*>(base + L.dtot);
  B->info = reinterpret_cast<RowInfo*>(base + L.info);
  B->hpart = reinterpret_cast<uint32_t*>(base + L.hpart);
  B->bins = reinterpret_cast<uint32_t*>(base + L.bins);
  B->bins2 = reinterpret_cast<uint32_t*>(base + L.bins2);
  B->tcnt = reinterpret_cast<uint32_t*>(base + L.tcnt);
  B->tabove = reinterpret_cast<uint32_t*>(base + L.tabove);
  B->toff = reinterpret_cast<uint32_t*>(base + L.toff);
  B->taboff = reinterpret_cast<uint32_t*>(base + L.taboff);
  B->sel = reinterpret_cast<RowSel*>(base + L.sel);
  return TOPK_OK;
}

int check_shape(int64_t rows, int64_t n, int64_t k, double lambda) {
  if (rows < 0 || rows >= (int64_t(1) << 31) || n < 1 || n >= (int64_t(1) << 30) || k < 0 || k > n)
    return TOPK_ERR_INVALID;
  if (!(lambda > 0.0) || !std::isfinite(lambda)) return TOPK_ERR_INVALID;
  return TOPK_OK;
}

// Launch errors are read from the runtime's last-error slot: begin() empties it after the
// arguments have been validated and before the first launch (an error left there by an earlier,
// unrelated call would otherwise be reported as this call's), finish() reads it after the last.
void begin() { (void)hipGetLastError(); }
int finish() { return hipGetLastError() == hipSuccess ? TOPK_OK : TOPK_ERR_LAUNCH; }

// shared body of the four operator entry points
int run_operator(bool mag, const float* x, const float* tangent, int64_t rows, int64_t n,
                 int64_t k, double p, double lambda, float* out, float* jvp, bool need_out,
                 bool need_jvp, void* stream, size_t ws_skip = 0, const Workspace& ws = g_ws) {
  int rc = check_shape(rows, n, k, lambda);
  if (rc != TOPK_OK) return rc;
  const int pc = p_code(p);
  if (pc < 0) return TOPK_ERR_UNSUPPORTED_P;
  if (rows == 0) return TOPK_OK;          // nothing to do; pointers of empty arrays may be NULL
  if (x == nullptr) return TOPK_ERR_NULL;
  if (need_out && out == nullptr) return TOPK_ERR_NULL;
  if (need_jvp && (jvp == nullptr || tangent == nullptr)) return TOPK_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Reg R = make_reg(lambda);
  SortBuffers B;
  const bool by_value = value_wide(mag, pc, n);
  if (is_long(n) && !by_value) {
    rc = carve(rows, n, &B, ws_skip, ws);
    if (rc != TOPK_OK) return rc;
  }
  begin();
  if (!is_long(n)) {
    if (topk::launch_short_rows(mag, pc, x, need_jvp ? tangent : nullptr, out,
                                need_jvp ? jvp : nullptr, rows, int(n), int(k), R, st) != 0)
      return TOPK_ERR_INVALID;
    return finish();
  }
  const LongMode mode = long_mode();
  if (by_value) {
    const bool vec = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(tangent) |
                                       reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(jvp)) & 15u) == 0;
    const int vrc = topk::launch_short_rows_value_wide(2048, vec, mag, pc, x, need_jvp ? tangent : nullptr,
                                                       out, need_jvp ? jvp : nullptr, rows, int(n),
                                                       int(k), R, st);
    return vrc == 0 ? finish() : TOPK_ERR_INVALID;
  }
  // k = 0 and k = n pool nothing and read no sorted value: no sort at all
  const bool trivial = (k == 0 || k == n);
  // Rows above 32768 elements: the streaming steps of a row are spread over many workgroups
  // (separate launches) and only the sort + solve of its candidates is left to one.
  if (!trivial && (mode == kWide || (mode == kAuto && n > 32768))) {
    const bool refine = n > (int64_t(1) << 18);
    if (topk::launch_wide_select(mag, pc, refine, x, need_jvp ? tangent : nullptr, rows, n, k, R, B,
                                 st) != 0)
      return TOPK_ERR_INVALID;
    if (topk::launch_wide_finish(mag, pc, B, need_jvp, refine, rows, n, k, R, st) != 0)
      return TOPK_ERR_INVALID;
    if (topk::launch_wide_dense(mag, pc, B, x, need_jvp ? tangent : nullptr, out,
                                need_jvp ? jvp : nullptr, rows, n, R, st) != 0)
      return TOPK_ERR_INVALID;
    return finish();
  }
  if ((mode == kAuto || mode == kOneLaunchIndexed) && n <= topk::kMediumRowMax) {
    // one launch, one workgroup per row; above 8192 elements the kernel that orders values only
    const bool by_value = mode == kAuto && n > 8192 && n <= 32768;
    const int lrc = by_value ? topk::launch_medium_rows2(mag, pc, B, x, need_jvp ? tangent : nullptr,
                                                         out, need_jvp ? jvp : nullptr, rows, n, k,
                                                         R, st)
                             : topk::launch_medium_rows(mag, pc, B, x, need_jvp ? tangent : nullptr,
                                                        out, need_jvp ? jvp : nullptr, rows, n, k,
                                                        R, st);
    if (lrc != 0) return TOPK_ERR_INVALID;
    return finish();
  }
  const bool selected = !trivial && mode != kFullSort;
  if (selected) {
    if (topk::launch_candidate_lists(mag, pc, x, rows, n, k, R, B, st) != 0) return TOPK_ERR_INVALID;
    if (topk::launch_finish(mag, pc, B, need_jvp ? tangent : nullptr, rows, n, k, R, st) != 0)
      return TOPK_ERR_INVALID;
    if (topk::launch_long_list_sort(mag, rows, n, B, st) != 0) return TOPK_ERR_INVALID;
  } else if (!trivial) {
    if (topk::launch_segmented_sort(mag, x, rows, n, B, st) != 0) return TOPK_ERR_INVALID;
  }
  if (topk::launch_long_tail(mag, pc, selected, B, x, need_jvp ? tangent : nullptr, out,
                             need_jvp ? jvp : nullptr, rows, n, k, R, st) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

// The operators on |x|: |x| and sign(x) t go to the first two arrays of the workspace, the mask
// kernels run on them into (out, jvp), an element-wise pass turns those into the results.
size_t abs_scratch_bytes(int64_t rows, int64_t n) { return 2 * align_up(size_t(rows) * size_t(n) * 4); }

// Rows of 3..2048 elements: these operators run inside the short-row kernel and need no scratch
// (unless another short-row kernel was asked for with topk_set_route).
bool abs_fused(int64_t n) {
  return n >= 3 && n <= 2048 && topk::routes().short_kernel == TOPK_SHORT_ROW_KERNEL_AUTO;
}

int run_abs_operator(bool signed_mask, const float* x, const float* tangent, int64_t rows,
                     int64_t n, int64_t k, double p, double lambda, float* out, float* jvp,
                     bool need_jvp, void* stream) {
  int rc = check_shape(rows, n, k, lambda);
  if (rc != TOPK_OK) return rc;
  const int pc = p_code(p);
  if (pc < 0) return TOPK_ERR_UNSUPPORTED_P;
  if (rows == 0) return TOPK_OK;
  if (x == nullptr || out == nullptr) return TOPK_ERR_NULL;
  if (need_jvp && (jvp == nullptr || tangent == nullptr)) return TOPK_ERR_NULL;
  // rows of up to 2048 elements: one fused kernel, no scratch
  if (abs_fused(n)) {
    begin();
    const int frc = topk::launch_short_rows_fused_variant(
        signed_mask ? 1 : 2, pc, x, need_jvp ? tangent : nullptr, out, need_jvp ? jvp : nullptr,
        nullptr, 0.0, rows, int(n), int(k), make_reg(lambda), static_cast<hipStream_t>(stream));
    if (frc == 0) return finish();
    if (frc != -2) return TOPK_ERR_INVALID;
  }
  // the whole workspace is checked before the first launch: two arrays here, then the mask's own
  const size_t skip = abs_scratch_bytes(rows, n);
  const size_t need = skip + (is_long(n) ? layout_for(rows, n).total : 0);
  if (g_ws.ptr == nullptr || g_ws.bytes < need) return TOPK_ERR_WORKSPACE;
  begin();
  float* ax = static_cast<float*>(g_ws.ptr);
  float* st = reinterpret_cast<float*>(static_cast<char*>(g_ws.ptr) + skip / 2);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t count = rows * n;
  if (topk::launch_abs_prepare(x, need_jvp ? tangent : nullptr, ax, st, count, s) != 0)
    return TOPK_ERR_INVALID;
  if (hipGetLastError() != hipSuccess) return TOPK_ERR_LAUNCH;
  rc = run_operator(false, ax, need_jvp ? st : nullptr, rows, n, k, p, lambda, out,
                    need_jvp ? jvp : nullptr, true, need_jvp, stream, skip);
  if (rc != TOPK_OK) return rc;
  if (topk::launch_abs_finish(signed_mask, pc, x, tangent, out, need_jvp ? jvp : nullptr, count,
                              make_reg(lambda), s) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

// ---- the library's own scratch, for the one entry point that must not allocate ------------------
// One copy of this array lives on every GPU the library is loaded on, for the life of the process.
// In host code its name is only a handle for hipGetSymbolAddress: the device address is looked up
// once per device (with that device current) and kept; kernels and carve() only ever see that
// address.
__device__ __align__(256) unsigned char scratch[TOPK_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int static_scratch(Workspace* ws) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return TOPK_ERR_LAUNCH;
  if (dev < 0 || dev >= kMaxDevices) return TOPK_ERR_INVALID;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return TOPK_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = ptr;
  }
  ws->ptr = g_scratch_ptr[dev];
  ws->bytes = TOPK_STATIC_SCRATCH_BYTES;
  return TOPK_OK;
}

}  // namespace

namespace topk {
Routes& routes() {
  static Routes r;
  return r;
}
}  // namespace topk

extern "C" {

int topk_set_route(int which, int value) {
  topk::Routes& r = topk::routes();
  switch (which) {
    case TOPK_ROUTE_LONG_ROWS:
      if (value < TOPK_LONG_ROWS_AUTO || value > TOPK_LONG_ROWS_ONE_LAUNCH_INDEXED)
        return TOPK_ERR_INVALID;
      r.long_rows = value;
      return TOPK_OK;
    case TOPK_ROUTE_SHORT_ROW_LANES:
      if (value < 0 || value > 64 || (value & (value - 1)) != 0) return TOPK_ERR_INVALID;
      r.short_lanes = value;
      return TOPK_OK;
    case TOPK_ROUTE_SHORT_ROW_KERNEL:
      if (value < TOPK_SHORT_ROW_KERNEL_AUTO || value > TOPK_SHORT_ROW_KERNEL_GENERAL)
        return TOPK_ERR_INVALID;
      r.short_kernel = value;
      return TOPK_OK;
    case TOPK_ROUTE_GENERAL_ROUNDS:
      if (value < 0 || value > 4096) return TOPK_ERR_INVALID;
      r.general_rounds = value;
      return TOPK_OK;
    default:
      return TOPK_ERR_INVALID;
  }
}

static int run_general(int phi, const float* x, const float* w, int64_t w_stride,
                       const float* tangent, int64_t rows, int64_t n, double p, double lambda,
                       float* out, float* jvp, bool need_jvp, void* stream) {
  const int rc = check_shape(rows, n, 0, lambda);
  if (rc != TOPK_OK) return rc;
  if (n > TOPK_GENERAL_ROW_MAX || (w_stride != 0 && w_stride != n)) return TOPK_ERR_INVALID;
  if (phi != TOPK_PHI_IDENTITY && phi != TOPK_PHI_HALF_SQUARE) return TOPK_ERR_INVALID;
  const int pc = p_code(p);
  if (pc < 0) return TOPK_ERR_UNSUPPORTED_P;
  if (rows == 0) return TOPK_OK;
  if (x == nullptr || w == nullptr) return TOPK_ERR_NULL;
  if (!need_jvp && out == nullptr) return TOPK_ERR_NULL;
  if (need_jvp && (jvp == nullptr || tangent == nullptr)) return TOPK_ERR_NULL;
  const bool mag = phi == TOPK_PHI_HALF_SQUARE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!is_long(n)) {
    begin();
    if (topk::launch_general_rows(mag, pc, x, w, w_stride, need_jvp ? tangent : nullptr, out,
                                  need_jvp ? jvp : nullptr, rows, int(n), make_reg(lambda), st) != 0)
      return TOPK_ERR_INVALID;
    return finish();
  }
  // long rows: a complete sort of every row, then one workgroup per row; the solver's float64
  // arrays come first in the workspace, the sort's arrays after them
  const size_t skip = topk::general_long_bytes(rows, n, pc);
  SortBuffers B;
  const int crc = carve(rows, n, &B, skip);
  if (crc != TOPK_OK) return crc;
  const topk::GeneralBuffers gb = topk::general_long_carve(g_ws.ptr, rows, n, pc);
  begin();
  if (topk::launch_segmented_sort(mag, x, rows, n, B, st) != 0) return TOPK_ERR_INVALID;
  if (topk::launch_general_long(mag, pc, B, gb, x, w, w_stride, need_jvp ? tangent : nullptr, out,
                                need_jvp ? jvp : nullptr, rows, n, make_reg(lambda), st) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

int topk_general_fwd(const float* x, const float* w, int64_t w_stride, int64_t rows, int64_t n,
                     int phi, double p, double lambda, float* out, void* stream) {
  return run_general(phi, x, w, w_stride, nullptr, rows, n, p, lambda, out, nullptr, false, stream);
}

int topk_general_jvp(const float* x, const float* w, int64_t w_stride, const float* tangent,
                     int64_t rows, int64_t n, int phi, double p, double lambda, float* out,
                     float* jvp_out, void* stream) {
  return run_general(phi, x, w, w_stride, tangent, rows, n, p, lambda, out, jvp_out, true, stream);
}

int topk_mask_sparse_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double p,
                         double lambda, int64_t max_nnz, int32_t* idx_out, float* val_out,
                         int32_t* nnz_out, void* stream) {
  const int rc = check_shape(rows, n, k, lambda);
  if (rc != TOPK_OK) return rc;
  if (max_nnz < 1 || max_nnz > n || max_nnz > 0x7fffffffLL) return TOPK_ERR_INVALID;
  const int pc = p_code(p);
  if (pc < 0) return TOPK_ERR_UNSUPPORTED_P;
  if (rows == 0) return TOPK_OK;
  if (theta == nullptr || idx_out == nullptr || val_out == nullptr || nnz_out == nullptr)
    return TOPK_ERR_NULL;
  const topk::SparseOut sp{idx_out, val_out, nnz_out, int(max_nnz)};
  if (n > topk::kMediumRowMax) {
    // rows spread over many workgroups: the selection route with (key, index) lists, then the
    // lists' leading positions
    SortBuffers B;
    const int wrc = carve(rows, n, &B);
    if (wrc != TOPK_OK) return wrc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Reg R = make_reg(lambda);
    begin();
    if (k >= 1 && k < n) {
      if (topk::launch_candidate_lists(false, pc, theta, rows, n, k, R, B, st) != 0 ||
          topk::launch_finish(false, pc, B, nullptr, rows, n, k, R, st) != 0 ||
          topk::launch_long_list_sort(false, rows, n, B, st) != 0 ||
          topk::launch_long_solve(false, pc, true, B, nullptr, rows, n, k, R, st) != 0)
        return TOPK_ERR_INVALID;
    }
    if (topk::launch_long_sparse(pc, B, theta, rows, n, k, R, sp, st) != 0) return TOPK_ERR_INVALID;
    return finish();
  }
  if (is_long(n)) {
    SortBuffers B;
    const int wrc = carve(rows, n, &B);
    if (wrc != TOPK_OK) return wrc;
    begin();
    if (topk::launch_medium_rows_sparse(pc, B, theta, rows, n, k, make_reg(lambda), sp,
                                        static_cast<hipStream_t>(stream)) != 0)
      return TOPK_ERR_INVALID;
    return finish();
  }
  begin();
  if (topk::launch_short_rows_sparse(pc, theta, rows, int(n), int(k), make_reg(lambda), sp,
                                     static_cast<hipStream_t>(stream)) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

int topk_mask_dykstra_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double lambda,
                          int iters, float* out, void* stream) {
  const int rc = check_shape(rows, n, k, lambda);
  if (rc != TOPK_OK) return rc;
  if (iters < 0 || n > TOPK_SHORT_ROW_MAX) return TOPK_ERR_INVALID;
  if (rows == 0) return TOPK_OK;
  if (theta == nullptr || out == nullptr) return TOPK_ERR_NULL;
  begin();
  if (topk::launch_short_dykstra(theta, out, rows, int(n), int(k), lambda, iters,
                                 static_cast<hipStream_t>(stream)) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

int topk_signed_mask_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p,
                         double lambda, float* out, void* stream) {
  return run_abs_operator(true, x, nullptr, rows, n, k, p, lambda, out, nullptr, false, stream);
}

int topk_signed_mask_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                         double p, double lambda, float* out, float* jvp_out, void* stream) {
  return run_abs_operator(true, x, tangent, rows, n, k, p, lambda, out, jvp_out, true, stream);
}

int topk_masked_value_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p,
                          double lambda, float* out, void* stream) {
  return run_abs_operator(false, x, nullptr, rows, n, k, p, lambda, out, nullptr, false, stream);
}

int topk_masked_value_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                          double p, double lambda, float* out, float* jvp_out, void* stream) {
  return run_abs_operator(false, x, tangent, rows, n, k, p, lambda, out, jvp_out, true, stream);
}

int topk_mask_fwd(const float* theta, int64_t rows, int64_t n, int64_t k, double p, double lambda,
                  float* out, void* stream) {
  return run_operator(false, theta, nullptr, rows, n, k, p, lambda, out, nullptr, true, false,
                      stream);
}

int topk_mask_jvp(const float* theta, const float* tangent, int64_t rows, int64_t n, int64_t k,
                  double p, double lambda, float* out, float* jvp_out, void* stream) {
  return run_operator(false, theta, tangent, rows, n, k, p, lambda, out, jvp_out, false, true,
                      stream);
}

int topk_mask_jvp_static(const float* theta, const float* tangent, int64_t rows, int64_t n,
                         int64_t k, double p, double lambda, float* out, float* jvp_out,
                         void* stream) {
  // shapes whose scratch does not fit the static array are refused before anything else happens
  const int rc = check_shape(rows, n, k, lambda);
  if (rc != TOPK_OK) return rc;
  const bool scratch = is_long(n) && !value_wide(false, p_code(p), n);
  if (scratch && layout_for(rows, n).total > size_t(TOPK_STATIC_SCRATCH_BYTES))
    return TOPK_ERR_STATIC_SCRATCH;
  Workspace ws;
  if (scratch) {
    const int src = static_scratch(&ws);
    if (src != TOPK_OK) return src;
  }
  return run_operator(false, theta, tangent, rows, n, k, p, lambda, out, jvp_out, false, true,
                      stream, 0, ws);
}

int topkmag_fwd(const float* x, int64_t rows, int64_t n, int64_t k, double p, double lambda,
                float* out, void* stream) {
  return run_operator(true, x, nullptr, rows, n, k, p, lambda, out, nullptr, true, false, stream);
}

int topkmag_jvp(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                double p, double lambda, float* out, float* jvp_out, void* stream) {
  return run_operator(true, x, tangent, rows, n, k, p, lambda, out, jvp_out, false, true, stream);
}

int topk_mask_loss(const float* theta, const float* target, int64_t rows, int64_t n, int64_t k,
                   double p, double lambda, float* loss_out, float* grad_out, void* stream) {
  if (rows > 0 && (target == nullptr || loss_out == nullptr)) {
    const int rc = check_shape(rows, n, k, lambda);
    return rc != TOPK_OK ? rc : (p_code(p) < 0 ? TOPK_ERR_UNSUPPORTED_P : TOPK_ERR_NULL);
  }
  if (rows > 0 && n <= 2048 && grad_out != nullptr && theta != nullptr &&
      check_shape(rows, n, k, lambda) == TOPK_OK && p_code(p) >= 0) {
    // rows of up to 2048 elements: mask, loss and gradient in one kernel
    const double p_ex = p_code(p) == topk::kP2 ? 2.0 : 4.0 / 3.0;
    begin();
    const int frc = topk::launch_short_rows_fused_variant(
        3, p_code(p), theta, target, grad_out, nullptr, loss_out, lambda / p_ex, rows, int(n),
        int(k), make_reg(lambda), static_cast<hipStream_t>(stream));
    if (frc == 0) return finish();
    if (frc != -2) return TOPK_ERR_INVALID;
  }
  // the mask goes to grad_out, the reduction turns it into y - target
  const int rc = run_operator(false, theta, nullptr, rows, n, k, p, lambda, grad_out, nullptr, true,
                              false, stream);
  if (rc != TOPK_OK || rows == 0) return rc;
  const double p_exact = p_code(p) == topk::kP2 ? 2.0 : 4.0 / 3.0;
  if (topk::launch_mask_loss(p_code(p), theta, target, grad_out, loss_out, rows, n, k, lambda,
                             p_exact, static_cast<hipStream_t>(stream)) != 0)
    return TOPK_ERR_INVALID;
  return finish();
}

// The Jacobians are symmetric (see the header): the VJP is the JVP of the cotangent.
int topk_mask_vjp(const float* theta, const float* cotangent, int64_t rows, int64_t n, int64_t k,
                  double p, double lambda, float* out, float* vjp_out, void* stream) {
  return topk_mask_jvp(theta, cotangent, rows, n, k, p, lambda, out, vjp_out, stream);
}

int topkmag_vjp(const float* x, const float* cotangent, int64_t rows, int64_t n, int64_t k,
                double p, double lambda, float* out, float* vjp_out, void* stream) {
  return topkmag_jvp(x, cotangent, rows, n, k, p, lambda, out, vjp_out, stream);
}

int topk_argsort_desc(const float* theta, int64_t rows, int64_t n, int32_t* perm_out,
                      void* stream) {
  if (rows < 0 || n < 1 || n >= (int64_t(1) << 30)) return TOPK_ERR_INVALID;
  if (rows == 0) return TOPK_OK;
  if (theta == nullptr || perm_out == nullptr) return TOPK_ERR_NULL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (!is_long(n)) {
    begin();
    if (topk::launch_short_argsort(theta, perm_out, rows, int(n), st) != 0) return TOPK_ERR_INVALID;
    return finish();
  }
  SortBuffers B;
  int rc = carve(rows, n, &B);
  if (rc != TOPK_OK) return rc;
  begin();
  if (topk::launch_segmented_sort(false, theta, rows, n, B, st) != 0) return TOPK_ERR_INVALID;
  if (hipMemcpyAsync(perm_out, B.idx_a, size_t(rows) * size_t(n) * 4, hipMemcpyDeviceToDevice,
                     st) != hipSuccess)
    return TOPK_ERR_LAUNCH;
  return finish();
}

size_t topk_workspace_bytes(int op, int64_t rows, int64_t n, int64_t k, double p) {
  (void)k;
  if (op < TOPK_OP_MASK_FWD || op > TOPK_OP_MASK_SPARSE) return 0;
  if (rows <= 0 || n < 1 || n >= (int64_t(1) << 30)) return 0;
  if (op == TOPK_OP_GENERAL) {
    if (!is_long(n) || n > TOPK_GENERAL_ROW_MAX) return 0;
    return topk::general_long_bytes(rows, n, p_code(p) == topk::kP2 ? topk::kP2 : topk::kP43) +
           layout_for(rows, n).total;
  }
  const bool abs_op = op == TOPK_OP_SIGNED_MASK || op == TOPK_OP_MASKED_VALUE;
  if (abs_op && abs_fused(n)) return 0;
  const size_t own = abs_op ? abs_scratch_bytes(rows, n) : 0;
  if (!is_long(n)) return own;
  if (op <= TOPK_OP_MAG_JVP && value_wide(op >= TOPK_OP_MAG_FWD, p_code(p), n)) return 0;
  return own + layout_for(rows, n).total;
}

int topk_set_workspace(void* dev_ptr, size_t bytes) {
  if (dev_ptr == nullptr) {
    if (bytes != 0) return TOPK_ERR_INVALID;
    g_ws = Workspace{};
    return TOPK_OK;
  }
  if (reinterpret_cast<uintptr_t>(dev_ptr) % kAlign != 0) return TOPK_ERR_INVALID;
  g_ws.ptr = dev_ptr;
  g_ws.bytes = bytes;
  return TOPK_OK;
}

const char* topk_strerror(int code) {
  switch (code) {
    case TOPK_OK: return "ok";
    case TOPK_ERR_INVALID: return "invalid argument (rows, n, k, lambda or alignment out of range)";
    case TOPK_ERR_NULL: return "a required pointer is NULL";
    case TOPK_ERR_UNSUPPORTED_P: return "unsupported p (only 2 and 4/3)";
    case TOPK_ERR_WORKSPACE: return "workspace missing or too small (see topk_workspace_bytes)";
    case TOPK_ERR_LAUNCH: return "HIP launch failed";
    case TOPK_ERR_STATIC_SCRATCH:
      return "shape needs more scratch than the library's static buffer of "
             "TOPK_STATIC_SCRATCH_BYTES (use topk_mask_jvp with a registered workspace)";
    default: return "unknown error code";
  }
}

}  // extern "C"
