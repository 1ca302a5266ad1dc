// Host-side launchers of the kernels (one translation unit per kernel family).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pooling.hpp"

namespace topk {

// Choice among equivalent code paths (identical results), set through topk_set_route: for tests
// that compare the routes and for tuning runs.  Values as in sparse_topk.h.
struct Routes {
  int long_rows = 0;      // TOPK_LONG_ROWS_*
  int short_lanes = 0;    // lanes per row of the short-row kernels, 0 = chosen from the shape
  int short_kernel = 0;   // TOPK_SHORT_ROW_KERNEL_*
  int general_rounds = 0; // general weights: merging rounds before the sequential fallback, 0 = default
};
Routes& routes();

// Per-row result of the long-row solve: the pooled block [a, b] (1-based, inclusive; a = k+1,
// b = k when nothing pools), its pooled value (relative to `center`), and d gamma of the JVP.
// [wa, wb] is the block widened over values tied with its two end values: every sorted position
// whose value lies in [lo_incl, hi_incl] is inside it.  Values above hi_incl are before the block,
// values below lo_incl after it.  When nothing pools, hi_incl < lo_incl and the window is empty.
struct RowInfo {
  int64_t a, b;
  int64_t wa, wb;
  double gamma, center, dgamma;
  float hi_incl, lo_incl;
  int32_t src;      // which pair of scratch arrays holds the sorted list: 0 = "a", 1 = "b"
  int32_t pad;
};

// Per-row result of the candidate selection of the long-row path.  Only the elements whose
// descending-order key lies in [klo, khi] (a value window around s_k and s_{k+1} that contains
// every position able to pool) are sorted: cn of them, and `above` elements of the row have a
// smaller key (a larger value), so sorted position q (1-based) of the candidate list is sorted
// position above + q of the row.
struct RowSel {
  uint32_t klo, khi;
  uint32_t cn;
  uint32_t pad;
  int64_t above;
  // first selection level: histogram bins of sorted positions k and k+1, and the 1-based ranks
  // of those positions inside their bins
  uint32_t bin_k, bin_k1;
  uint32_t rank_k, rank_k1;
};

constexpr int kSelBits = 12;              // leading key bits of the first selection histogram
constexpr int kSelBins = 1 << kSelBits;
constexpr int kSel2Bits = 8;              // further key bits of the second one
constexpr int kSel2Bins = 1 << kSel2Bits;
constexpr int kSelSlices = 16;            // partial sums a histogram is left in (see radix_sort.hip)

// Device scratch of the long-row path (all carved out of the caller's workspace).
struct SortBuffers {
  uint32_t* keys_a;   // [rows*n] sorted keys end here
  uint32_t* keys_b;   // [rows*n]
  uint32_t* idx_a;    // [rows*n] sorted index payload ends here
  uint32_t* idx_b;    // [rows*n]
  uint32_t* hist;     // [rows][256][tiles]
  uint32_t* dtot;     // [rows][256]
  RowInfo* info;      // [rows]
  uint32_t* hpart;    // [rows][parts][kSelBins] partial histograms of the leading key bits
  uint32_t* bins;     // [rows][slices][kSelBins] the same, summed down to <= kSelSlices slices
  uint32_t* bins2;    // [rows][kSelSlices][2][kSel2Bins] the next key bits inside the bins of k, k+1:
                      // partial histograms, tile t of a row adds to slice t % kSelSlices
  uint32_t* tcnt;     // [rows][tiles] candidates per tile
  uint32_t* tabove;   // [rows][tiles] elements above the candidate window per tile
  uint32_t* toff;     // [rows][tiles] start of the tile's candidates in the row's dense list
  uint32_t* taboff;   // [rows][tiles] elements above the candidate window in the tiles before
  RowSel* sel;        // [rows]
};

// Rows of up to 1024 elements, one row per (part of a) wavefront.  tangent/jvp may be null
// (forward only), out may be null (JVP only).  Returns 0, or -1 if no kernel fits.
int launch_short_rows(bool mag, int pc, const float* x, const float* tangent, float* out,
                      float* jvp, int64_t rows, int n, int k, const Reg& R, hipStream_t st);
int launch_short_argsort(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st);

// Compact output of the relaxed top-k mask: per row the non-zeros, idx / val [rows][max_nnz]
// (unused slots -1 / 0), nnz [rows] = their number (may exceed max_nnz: the list is then cut off).
struct SparseOut {
  int32_t* idx;
  float* val;
  int32_t* nnz;
  int max_nnz;
};

// Fast variants for padded row lengths np <= 128 with 2^lg lanes per row; return -2 when the
// (np, lg) shape is not instantiated (the caller then uses the general kernels above).
int launch_short_rows_fast(int np, int lg, bool vec, bool mag, int pc, const float* x,
                           const float* tangent, float* out, float* jvp, int64_t rows, int n,
                           int k, const Reg& R, hipStream_t st);
// Dense outputs of the same shapes without building the permutation (short_rows_select.hip).
int launch_short_rows_value(int np, int lg, bool vec, bool mag, int pc, const float* x,
                            const float* tangent, float* out, float* jvp, int64_t rows, int n,
                            int k, const Reg& R, hipStream_t st);
// the same kernel for rows of 129 .. 2048 elements (np = 256 .. 2048); -2 when there is none
int launch_short_rows_value_wide(int np, bool vec, bool mag, int pc, const float* x,
                                 const float* tangent, float* out, float* jvp, int64_t rows, int n,
                                 int k, const Reg& R, hipStream_t st);
int launch_short_rows_variant_wide(int np, bool vec, int var, int pc, const float* x,
                                   const float* tangent, float* out, float* jvp, float* loss,
                                   double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                                   hipStream_t st);
int launch_short_rows_variant(int np, int lg, bool vec, int var, int pc, const float* x,
                              const float* tangent, float* out, float* jvp, float* loss,
                              double lam_over_p, int64_t rows, int n, int k, const Reg& R,
                              hipStream_t st);
// Operators built on the mask (var: 1 signed mask, 2 x o mask(|x|), 3 Fenchel-Young loss), fused
// into the short-row kernel when a shape fits (-2 otherwise).
int launch_short_rows_fused_variant(int var, int pc, const float* x, const float* tangent, float* out,
                                    float* jvp, float* loss, double lam_over_p, int64_t rows, int n,
                                    int k, const Reg& R, hipStream_t st);
int launch_short_argsort_fast(int np, int lg, bool vec, const float* x, int32_t* perm,
                              int64_t rows, int n, hipStream_t st);
int launch_short_rows_fast_sparse(int np, int lg, bool vec, int pc, const float* x, int64_t rows,
                                  int n, int k, const Reg& R, const SparseOut& sp, hipStream_t st);

// Long rows: segmented radix sort (result in B.keys_a / B.idx_a), then solve + scatter.
int radix_tiles(int64_t n);
// workgroups per row of the first selection histogram, and the elements each of them covers
int sel_parts(int64_t rows, int64_t n);
int64_t sel_span(int64_t rows, int64_t n);
int launch_segmented_sort(bool mag, const float* x, int64_t rows, int64_t n, const SortBuffers& B,
                          hipStream_t st);
// Candidate lists of up to kFinishMax elements are sorted and solved by one workgroup
// (launch_finish); longer ones by the passes of launch_long_list_sort and the solve of
// launch_long_tail.  Every kernel of either route skips the rows of the other.
constexpr int64_t kFinishMax = 32768;

// selected: B.sel describes candidate lists (see RowSel), and rows whose list is at most
// kFinishMax long already have their RowInfo; otherwise the "a" arrays hold fully sorted rows.
// only the solve of launch_long_tail: B.info[row] of every row not solved yet
int launch_long_solve(bool mag, int pc, bool selected, const SortBuffers& B, const float* tangent,
                      int64_t rows, int64_t n, int64_t k, const Reg& R, hipStream_t st);
// Compact output of the mask for rows above kMediumRowMax elements, after the candidate lists
// have been sorted and solved (launch_candidate_lists .. launch_long_solve): the elements above
// the candidate window in index order, then sorted list positions 1..b.
int launch_long_sparse(int pc, const SortBuffers& B, const float* x, int64_t rows, int64_t n,
                       int64_t k, const Reg& R, const SparseOut& sp, hipStream_t st);
int launch_long_tail(bool mag, int pc, bool selected, const SortBuffers& B, const float* x,
                     const float* tangent, float* out, float* jvp, int64_t rows, int64_t n,
                     int64_t k, const Reg& R, hipStream_t st);

// Rows of up to kMediumRowMax elements: the whole operator in one launch, one workgroup per row
// (selection of the candidates, their sort, the solve and the outputs); scratch in B.keys_* and
// B.idx_* (row stride n).  Any 0 <= k <= n.
constexpr int64_t kMediumRowMax = 131072;
int launch_medium_rows(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                       float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                       hipStream_t st);

// The same for rows of 8193 .. kMediumRowMax elements with dense outputs computed from values:
// keys-only sort and block growth in LDS, no permutation (medium_rows2.hip).
int launch_medium_rows2(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                        float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                        hipStream_t st);

// Long rows without a full sort (0 < k < n): two histogram levels of the leading key bits -> key
// window around positions k, k+1 that holds every element able to pool -> those candidates, in
// index order, as a dense list per row in the "a" arrays; B.sel[row] = {window, length, above}.
int launch_candidate_lists(bool mag, int pc, const float* x, int64_t rows, int64_t n, int64_t k,
                           const Reg& R, const SortBuffers& B, hipStream_t st);
// Wide route (rows that several workgroups share; 0 < k < n): the same candidate selection with
// the candidates left in the tiles' slots of the "b" arrays (B.tcnt, B.tabove); one workgroup per
// row then collects them, sorts their keys, grows the block and adds up the tangent over it
// (B.info[row]: gamma, d gamma and the block's value window); one dense pass computes every
// output from its element's value.  refine: second histogram level (worth it for very long rows).
// tangent (may be null): the candidates carry their tangent as payload instead of their index.
int launch_wide_select(bool mag, int pc, bool refine, const float* x, const float* tangent,
                       int64_t rows, int64_t n, int64_t k, const Reg& R, const SortBuffers& B,
                       hipStream_t st);
int launch_wide_finish(bool mag, int pc, const SortBuffers& B, bool want_jvp, bool dense,
                       int64_t rows, int64_t n, int64_t k, const Reg& R, hipStream_t st);
int launch_wide_dense(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                      float* out, float* jvp, int64_t rows, int64_t n, const Reg& R,
                      hipStream_t st);
// Lists of up to kFinishMax candidates: sort + solve by one workgroup per row -> B.info[row].
int launch_finish(bool mag, int pc, const SortBuffers& B, const float* tangent, int64_t rows,
                  int64_t n, int64_t k, const Reg& R, hipStream_t st);
// Longer lists: four radix passes, sorted lists end in the "a" arrays.
int launch_long_list_sort(bool mag, int64_t rows, int64_t n, const SortBuffers& B, hipStream_t st);

// Fenchel-Young top-k loss from the mask: grad holds y on entry, y - target on exit; loss[rows].
int launch_mask_loss(int pc, const float* x, const float* target, float* grad, float* loss,
                     int64_t rows, int64_t n, int64_t k, double lambda, double p, hipStream_t st);

// Compact output of the relaxed top-k mask of short rows (n <= 1024): per row the non-zeros in
// descending order of theta, idx / val [rows][max_nnz] (unused slots -1 / 0), nnz [rows] = their
// number (may exceed max_nnz: the list is then cut off).
int launch_short_rows_sparse(int pc, const float* x, int64_t rows, int n, int k, const Reg& R,
                             const SparseOut& sp, hipStream_t st);
// the same for rows of 1025 .. kMediumRowMax elements (one-launch kernel; needs the workspace);
// there the entries above the key window (value 1) come first, in ascending index order
int launch_medium_rows_sparse(int pc, const SortBuffers& B, const float* x, int64_t rows, int64_t n,
                              int64_t k, const Reg& R, const SparseOut& sp, hipStream_t st);

// Relaxed operator for general non-increasing weights w ([n] with w_stride = 0, or one row of
// weights per row with w_stride = n), n <= 1024; tangent / jvp / out may be null.
int launch_general_rows(bool mag, int pc, const float* x, const float* w, int64_t w_stride,
                        const float* tangent, float* out, float* jvp, int64_t rows, int n,
                        const Reg& R, hipStream_t st);

// The same for rows of 1025 .. kGeneralLongMax elements, sorted completely beforehand
// (launch_segmented_sort): one workgroup per row, float64 prefix sums and per-block values in
// global scratch.
constexpr int64_t kGeneralLongMax = 131072;
struct DD {          // an unevaluated sum h + l of two float64 (general_long.hip)
  double h, l;
};
struct GeneralBuffers {
  DD* p1;            // [rows][n + 1] each: prefix sums of s and of w,
  DD* pw;
  double* g;         // pooled values and d gamma by block start
  double* dg;
  DD* p2;            // p = 4/3 only: prefix sums of s^2, s^3
  DD* p3;
  uint32_t* hi_of;   // [rows][n]
  float* ltau;       // [rows][n]
};
size_t general_long_bytes(int64_t rows, int64_t n, int pc);
GeneralBuffers general_long_carve(void* ptr, int64_t rows, int64_t n, int pc);
int launch_general_long(bool mag, int pc, const SortBuffers& B, const GeneralBuffers& gb,
                        const float* x, const float* w, int64_t w_stride, const float* tangent,
                        float* out, float* jvp, int64_t rows, int64_t n, const Reg& R,
                        hipStream_t st);

// Relaxed top-k mask, p = 2, by `iters` iterations of Dykstra's alternating projections (Alg. 1)
// on the sorted row instead of the exact block search; n <= 1024.
int launch_short_dykstra(const float* x, float* out, int64_t rows, int n, int k, double lambda,
                         int iters, hipStream_t st);

// Element-wise passes of the operators built on the mask of |x| (signed mask, x o mask):
// ax = |x| and st = sign(x) t before the mask kernels; afterwards, in place, out (holding the
// mask) and jvp (holding its JVP) become the operator's outputs.  t / st / jvp may be null.
int launch_abs_prepare(const float* x, const float* t, float* ax, float* st, int64_t count,
                       hipStream_t stream);
int launch_abs_finish(bool signed_mask, int pc, const float* x, const float* t, float* out,
                      float* jvp, int64_t count, const Reg& R, hipStream_t stream);

}  // namespace topk
