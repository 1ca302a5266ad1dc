// Host-side launchers of the kernels (one translation unit per kernel family).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pooling.hpp"

namespace topk {

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
};

// Device scratch of the long-row path (all carved out of the caller's workspace).
struct SortBuffers {
  uint32_t* keys_a;   // [rows*n] sorted keys end here
  uint32_t* keys_b;   // [rows*n]
  uint32_t* idx_a;    // [rows*n] sorted index payload ends here
  uint32_t* idx_b;    // [rows*n]
  uint32_t* hist;     // [rows][256][tiles]
  uint32_t* dtot;     // [rows][256]
  RowInfo* info;      // [rows]
};

// Rows of up to 1024 elements, one row per (part of a) wavefront.  tangent/jvp may be null
// (forward only), out may be null (JVP only).  Returns 0, or -1 if no kernel fits.
int launch_short_rows(bool mag, int pc, const float* x, const float* tangent, float* out,
                      float* jvp, int64_t rows, int n, int k, const Reg& R, hipStream_t st);
int launch_short_argsort(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st);

// Fast variants for padded row lengths np <= 128 with 2^lg lanes per row; return -2 when the
// (np, lg) shape is not instantiated (the caller then uses the general kernels above).
int launch_short_rows_fast(int np, int lg, bool vec, bool mag, int pc, const float* x,
                           const float* tangent, float* out, float* jvp, int64_t rows, int n,
                           int k, const Reg& R, hipStream_t st);
int launch_short_argsort_fast(int np, int lg, bool vec, const float* x, int32_t* perm,
                              int64_t rows, int n, hipStream_t st);

// Long rows: segmented radix sort (result in B.keys_a / B.idx_a), then solve + scatter.
int radix_tiles(int64_t n);
int launch_segmented_sort(bool mag, const float* x, int64_t rows, int64_t n, const SortBuffers& B,
                          hipStream_t st);
int launch_long_tail(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                     float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                     hipStream_t st);

}  // namespace topk
