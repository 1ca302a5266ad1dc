// Compact output of the relaxed top-k mask (Sec. 6, dispatch of a sparse mixture of experts) for
// rows above kMediumRowMax elements.  The multi-launch selection route has already built, per row,
// the sorted (key, index) list of the candidates (the elements inside the value window that holds
// everything able to pool) and solved it: RowInfo gives the block [a, b] in list positions, RowSel
// the number of elements above the window.  The row's non-zeros are
//   * the elements above the window (value exactly 1), written here in ascending index order: every
//     4096-element tile compacts its own with ballot prefix counts and starts at the number of
//     such elements in the tiles before it (taboff, from the selection's offsets kernel);
//   * list positions 1 .. b in sorted order (descending theta, ties by ascending index): 1 before
//     the block, the pooled formula inside it.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "radix.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kTile = 4096;                    // the selection's tile (radix_sort.hip)
constexpr int kItems = kTile / kThreads;

// slots beyond a row's non-zeros: index -1, value 0 (everything is filled first)
__global__ __launch_bounds__(kThreads) void sparse_fill_kernel(SparseOut sp, int64_t total) {
  const int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (i < total) {
    sp.idx[i] = -1;
    sp.val[i] = 0.0f;
  }
}

// k = n: every element is 1, in index order (k = 0: the fill is all there is)
__global__ __launch_bounds__(kThreads) void sparse_all_ones_kernel(SparseOut sp, int64_t rows,
                                                                   int64_t n) {
  const int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (i < rows * sp.max_nnz) {
    sp.idx[i] = int32_t(i % sp.max_nnz);
    sp.val[i] = 1.0f;
  }
  if (i < rows) sp.nnz[i] = int32_t(n);
}

__global__ __launch_bounds__(kThreads) void sparse_zero_count_kernel(SparseOut sp, int64_t rows) {
  const int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (i < rows) sp.nnz[i] = 0;
}

// one workgroup per tile: the tile's elements above the candidate window, in index order
__global__ __launch_bounds__(kThreads) void sparse_above_kernel(
    const float* __restrict__ x, const RowSel* __restrict__ sel, const uint32_t* __restrict__ taboff,
    SparseOut sp, int64_t n, int tiles) {
  __shared__ uint32_t wave_cnt[kWaves];
  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const uint32_t klo = sel[row].klo;
  const int64_t tile_first = int64_t(tile) * kTile;
  const int chunk = w * (kTile / kWaves);
  float val[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = tile_first + chunk + i * kWave + lane;
    val[i] = e < n ? x[row * n + e] : 0.0f;
  }
  uint32_t pos[kItems], cnt = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = tile_first + chunk + i * kWave + lane;
    const bool above = e < n && first_key<false>(val[i]) < klo;
    const unsigned long long bm = __ballot(above);
    pos[i] = above ? cnt + __popcll(bm & lanemask_lt()) : 0xffffffffu;
    cnt += __popcll(bm);
  }
  if (lane == 0) wave_cnt[w] = cnt;
  __syncthreads();
  uint32_t before = taboff[row * tiles + tile];
#pragma unroll
  for (int q = 0; q < kWaves; ++q)
    if (q < w) before += wave_cnt[q];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (pos[i] == 0xffffffffu) continue;
    const int64_t slot = int64_t(before) + pos[i];
    if (slot < sp.max_nnz) {
      sp.idx[row * sp.max_nnz + slot] = int32_t(tile_first + chunk + i * kWave + lane);
      sp.val[row * sp.max_nnz + slot] = 1.0f;
    }
  }
}

// sorted list positions 1 .. b of every row, after the elements above the window
template <int PC>
__global__ __launch_bounds__(kThreads) void sparse_list_kernel(
    const uint32_t* __restrict__ keys_a, const uint32_t* __restrict__ idx_a,
    const uint32_t* __restrict__ keys_b, const uint32_t* __restrict__ idx_b,
    const RowInfo* __restrict__ info, const RowSel* __restrict__ sel, SparseOut sp, int64_t n,
    int parts, Reg R) {
  using P = Pool<false, PC>;
  const int64_t row = blockIdx.x / parts;
  const int part = blockIdx.x % parts;
  const RowInfo ri = info[row];
  const int64_t above = sel[row].above;
  const uint32_t* skeys = (ri.src == 0 ? keys_a : keys_b) + row * n;
  const uint32_t* sidx = (ri.src == 0 ? idx_a : idx_b) + row * n;
  if (part == 0 && threadIdx.x == 0) sp.nnz[row] = int32_t(above + ri.b);
  for (int64_t q = int64_t(part) * kThreads + threadIdx.x + 1; q <= ri.b;
       q += int64_t(parts) * kThreads) {
    const int64_t slot = above + q - 1;
    if (slot >= sp.max_nnz) break;
    float y = 1.0f;
    if (q >= ri.a)
      y = float(P::y_in_block(double(key_to_float(skeys[q - 1])) - ri.center, ri.gamma, R));
    sp.idx[row * sp.max_nnz + slot] = int32_t(sidx[q - 1]);
    sp.val[row * sp.max_nnz + slot] = y;
  }
}

}  // namespace

int launch_long_sparse(int pc, const SortBuffers& B, const float* x, int64_t rows, int64_t n,
                       int64_t k, const Reg& R, const SparseOut& sp, hipStream_t st) {
  const int64_t total = rows * int64_t(sp.max_nnz);
  const int64_t tiles = (n + kTile - 1) / kTile;
  if ((total + kThreads - 1) / kThreads > 0x7fffffffLL || rows * tiles > 0x7fffffffLL) return -1;
  const unsigned fill_blocks = unsigned((total + kThreads - 1) / kThreads);
  if (k == n) {
    hipLaunchKernelGGL(sparse_all_ones_kernel, dim3(fill_blocks), dim3(kThreads), 0, st, sp, rows, n);
    return 0;
  }
  hipLaunchKernelGGL(sparse_fill_kernel, dim3(fill_blocks), dim3(kThreads), 0, st, sp, total);
  if (k == 0) {
    hipLaunchKernelGGL(sparse_zero_count_kernel, dim3(unsigned((rows + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, sp, rows);
    return 0;
  }
  hipLaunchKernelGGL(sparse_above_kernel, dim3(unsigned(rows * tiles)), dim3(kThreads), 0, st, x,
                     B.sel, B.taboff, sp, n, int(tiles));
  const int parts = int(tiles < 64 ? tiles : 64);
  if (pc == kP2)
    hipLaunchKernelGGL((sparse_list_kernel<kP2>), dim3(unsigned(rows * parts)), dim3(kThreads), 0, st,
                       B.keys_a, B.idx_a, B.keys_b, B.idx_b, B.info, B.sel, sp, n, parts, R);
  else if (pc == kP43)
    hipLaunchKernelGGL((sparse_list_kernel<kP43>), dim3(unsigned(rows * parts)), dim3(kThreads), 0,
                       st, B.keys_a, B.idx_a, B.keys_b, B.idx_b, B.info, B.sel, sp, n, parts, R);
  else return -1;
  return 0;
}

}  // namespace topk
