// Long rows: segmented, stable, least-significant-digit radix sort of (key, index) pairs through
// HBM, several workgroups per row.  Four passes of 8 bits; each pass is
//   digit histogram per tile  ->  exclusive scan per (row, digit) over tiles  ->  stable scatter.
// Keys are the descending-order keys of common.hpp, so ascending stable order of the keys is
// "value descending, original index ascending" (paper Sec. 3 sorts in descending order).
//
// Within a tile every wavefront owns a contiguous quarter; item i of lane l is element
// i*64 + l of that quarter, so loads are coalesced and the order (wave, item, lane) is the
// element order.  Equal digits inside a wavefront are found with ballots (no LDS atomics).
//
// The operators do not need the whole permutation: only elements in a value window around
// s_k and s_{k+1} can pool (pooling.hpp).  The second half of this file selects those candidates
// (histogram of the leading key bits, key window, ordered compaction per tile) and sorts only
// them with the same passes; topk_argsort_desc and rows with k = 0 or k = n use the full sort.
#include "common.hpp"
#include "launch.hpp"
#include "radix.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;
constexpr int kTile = kThreads * kItems;          // 4096 elements per workgroup and pass

// exclusive scan of one value per thread over the 256 threads of the block; also returns total
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot /*[kWaves]*/,
                                                         uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    uint32_t o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  __syncthreads();                                   // wave_tot may still be read from a previous use
  if (lane == kWave - 1) wave_tot[w] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    const uint32_t t = wave_tot[q];
    if (q < w) before += t;
    all += t;
  }
  if (total) *total = all;
  return before + inc - v;
}

// Number of valid elements at the start of tile `tile` of row `row` (the rest of the tile is
// padding).  Three layouts of the arrays a pass reads, all with row stride n:
//   dense, n per row            (tcnt == nullptr, sel == nullptr)
//   per-tile slots              (tcnt != nullptr): tile t holds tcnt[row][t] elements at its start
//   dense, sel[row].cn per row  (sel != nullptr)
__device__ __forceinline__ int tile_valid_count(int64_t row, int tile, int64_t n, int tiles,
                                                const uint32_t* __restrict__ tcnt,
                                                const RowSel* __restrict__ sel) {
  if (tcnt != nullptr) return int(tcnt[row * tiles + tile]);
  const int64_t len = (sel != nullptr) ? int64_t(sel[row].cn) : n;
  const int64_t left = len - int64_t(tile) * kTile;
  return int(left < 0 ? 0 : (left > kTile ? kTile : left));
}

// ---- 1. per-tile digit histogram ------------------------------------------------------------
// hist layout: [row][digit][tile]
template <bool FIRST, bool MAG>
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const float* __restrict__ x,
                                                              const uint32_t* __restrict__ keys,
                                                              uint32_t* __restrict__ hist,
                                                              const RowSel* __restrict__ sel,
                                                              int64_t n, int tiles, int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];
  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int nvalid = tile_valid_count(row, tile, n, tiles, nullptr, sel);
  if (nvalid == 0) return;                 // tiles past the end of a candidate list are not scanned
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const int64_t tile_base = row * n + int64_t(tile) * kTile;
  const int chunk = w * (kTile / kWaves);
#pragma unroll 4
  for (int i = 0; i < kItems; ++i) {
    const int e = chunk + i * kWave + lane;
    const bool valid = e < nvalid;
    uint32_t key = 0;
    if (valid) key = FIRST ? first_key<MAG>(x[tile_base + e]) : keys[tile_base + e];
    count_digit(cnt[w], (key >> shift) & (kRadix - 1), valid, lane);
  }
  __syncthreads();
  const int d = threadIdx.x;
  uint32_t tot = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) tot += cnt[q][d];
  hist[(row * kRadix + d) * tiles + tile] = tot;
}

// ---- 2. exclusive scan over tiles, per (row, digit) -------------------------------------------
// wide: one workgroup per (row, digit); narrow: one workgroup per row, thread = digit.
// `tiles` is the stride of the histogram; with `sel` only the tiles of the row's candidate list
// are scanned.
__device__ __forceinline__ int used_tiles(int64_t row, int tiles, const RowSel* __restrict__ sel) {
  if (sel == nullptr) return tiles;
  return int((int64_t(sel[row].cn) + kTile - 1) / kTile);
}

// Totals of the per-tile candidate counts of one row (first pass of a candidate sort).
__device__ __forceinline__ void total_candidates(int64_t row, int tiles,
                                                 const uint32_t* __restrict__ tcnt,
                                                 const uint32_t* __restrict__ tabove,
                                                 RowSel* __restrict__ sel_out, uint32_t* wave_tot) {
  uint32_t c = 0, a = 0;
  for (int t = threadIdx.x; t < tiles; t += kThreads) {
    c += tcnt[row * tiles + t];
    a += tabove[row * tiles + t];
  }
  uint32_t cn, above;
  block_exclusive_scan(c, wave_tot, &cn);
  block_exclusive_scan(a, wave_tot, &above);
  if (threadIdx.x == 0) {
    sel_out[row].cn = cn;
    sel_out[row].above = int64_t(above);
  }
}

__global__ __launch_bounds__(kThreads) void radix_scan_wide_kernel(
    uint32_t* __restrict__ hist, uint32_t* __restrict__ dtot, const RowSel* __restrict__ sel,
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove,
    RowSel* __restrict__ sel_out, int tiles) {
  __shared__ uint32_t wave_tot[kWaves];
  uint32_t* h = hist + int64_t(blockIdx.x) * tiles;
  if (sel_out != nullptr && blockIdx.x % kRadix == 0)
    total_candidates(blockIdx.x / kRadix, tiles, tcnt, tabove, sel_out, wave_tot);
  const int used = used_tiles(blockIdx.x / kRadix, tiles, sel);
  uint32_t carry = 0;
  for (int c = 0; c < used; c += kThreads) {
    const int t = c + threadIdx.x;
    const uint32_t v = (t < used) ? h[t] : 0u;
    uint32_t total;
    const uint32_t ex = block_exclusive_scan(v, wave_tot, &total);
    if (t < used) h[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) dtot[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kThreads) void radix_scan_narrow_kernel(
    uint32_t* __restrict__ hist, uint32_t* __restrict__ dtot, const RowSel* __restrict__ sel,
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove,
    RowSel* __restrict__ sel_out, int tiles) {
  __shared__ uint32_t wave_tot[kWaves];
  if (sel_out != nullptr) total_candidates(blockIdx.x, tiles, tcnt, tabove, sel_out, wave_tot);
  const int64_t rd = int64_t(blockIdx.x) * kRadix + threadIdx.x;
  uint32_t* h = hist + rd * tiles;
  const int used = used_tiles(blockIdx.x, tiles, sel);
  uint32_t carry = 0;
  for (int t = 0; t < used; ++t) {
    const uint32_t v = h[t];
    h[t] = carry;
    carry += v;
  }
  dtot[rd] = carry;
}

// ---- 3. stable scatter ----------------------------------------------------------------------------
// Index payload of the first pass: position in the row (mask) or 2*position + signbit (magnitude).
template <bool FIRST, bool MAG>
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(
    const float* __restrict__ x, const uint32_t* __restrict__ keys_in,
    const uint32_t* __restrict__ idx_in, uint32_t* __restrict__ keys_out,
    uint32_t* __restrict__ idx_out, const uint32_t* __restrict__ hist,
    const uint32_t* __restrict__ dtot, const uint32_t* __restrict__ tcnt,
    const RowSel* __restrict__ sel, int64_t n, int tiles, int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];       // per-wave digit counts, then per-wave offsets
  __shared__ uint32_t gdelta[kRadix];            // global destination minus position in the tile
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t kbuf[kTile];
  __shared__ uint32_t ibuf[kTile];

  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int nvalid = tile_valid_count(row, tile, n, tiles, tcnt, sel);
  if (nvalid == 0) return;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();

  const int64_t row_base = row * n;
  const int64_t tile_first = int64_t(tile) * kTile;
  const int chunk = w * (kTile / kWaves);
  uint32_t key[kItems], idx[kItems], rank[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int el = chunk + i * kWave + lane;              // element of the tile
    const int64_t e = tile_first + el;                    // element of the row
    const bool valid = el < nvalid;
    key[i] = 0xffffffffu;
    idx[i] = 0;
    if (valid) {
      if (FIRST) {
        const float v = x[row_base + e];
        key[i] = first_key<MAG>(v);
        idx[i] = MAG ? ((uint32_t(e) << 1) | (__float_as_uint(v) >> 31)) : uint32_t(e);
      } else {
        key[i] = keys_in[row_base + e];
        idx[i] = idx_in[row_base + e];
      }
    }
    const uint32_t d = (key[i] >> shift) & (kRadix - 1);
    const unsigned long long vm = __ballot(valid);
    const unsigned long long peers = match_digit(d, vm);
    const unsigned long long lower = peers & lanemask_lt();
    uint32_t pre = 0;
    if (valid) {
      pre = cnt[w][d];
      if (lower == 0) cnt[w][d] = pre + __popcll(peers);
    }
    rank[i] = pre + __popcll(lower);
  }
  __syncthreads();

  // digit d (= this thread): counts per wave -> offsets inside the tile, and the global base
  {
    const int d = threadIdx.x;
    uint32_t c[kWaves], tot = 0;
#pragma unroll
    for (int q = 0; q < kWaves; ++q) { c[q] = cnt[q][d]; tot += c[q]; }
    const uint32_t tile_ex = block_exclusive_scan(tot, wave_tot, nullptr);
    const uint32_t dt = dtot[row * kRadix + d];
    const uint32_t digit_base = block_exclusive_scan(dt, wave_tot, nullptr);
    uint32_t run = tile_ex;
#pragma unroll
    for (int q = 0; q < kWaves; ++q) { cnt[q][d] = run; run += c[q]; }
    gdelta[d] = digit_base + hist[(row * kRadix + d) * tiles + tile] - tile_ex;
  }
  __syncthreads();

  // place the pairs at their position in the sorted tile
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int el = chunk + i * kWave + lane;
    if (el < nvalid) {
      const uint32_t d = (key[i] >> shift) & (kRadix - 1);
      const uint32_t lp = cnt[w][d] + rank[i];
      kbuf[lp] = key[i];
      ibuf[lp] = idx[i];
    }
  }
  __syncthreads();

  for (int j = threadIdx.x; j < nvalid; j += kThreads) {
    const uint32_t kk = kbuf[j];
    const uint32_t d = (kk >> shift) & (kRadix - 1);
    const int64_t dst = row_base + int64_t(gdelta[d] + uint32_t(j));
    keys_out[dst] = kk;
    idx_out[dst] = ibuf[j];
  }
}

// ---- candidate selection ---------------------------------------------------------------------
// Histogram of the leading kSelBits key bits of every row (global counters, zeroed before).
constexpr int kSelItems = 32;
constexpr int kSelTile = kThreads * kSelItems;
constexpr int kSelShift = 32 - kSelBits;

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(uint32_t* __restrict__ p, int64_t count) {
  const int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (i < count) p[i] = 0u;
}

template <bool MAG>
__global__ __launch_bounds__(kThreads) void select_hist_kernel(const float* __restrict__ x,
                                                               uint32_t* __restrict__ bins,
                                                               int64_t n, int sel_tiles) {
  __shared__ uint32_t h[kSelBins];
  const int64_t row = blockIdx.x / sel_tiles;
  const int64_t first = int64_t(blockIdx.x % sel_tiles) * kSelTile;
  for (int i = threadIdx.x; i < kSelBins; i += kThreads) h[i] = 0;
  __syncthreads();
  const float* xr = x + row * n;
#pragma unroll 8
  for (int i = 0; i < kSelItems; ++i) {
    const int64_t e = first + int64_t(i) * kThreads + threadIdx.x;
    if (e < n) atomicAdd(&h[first_key<MAG>(xr[e]) >> kSelShift], 1u);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kSelBins; i += kThreads) {
    const uint32_t c = h[i];
    if (c != 0) atomicAdd(&bins[row * kSelBins + i], c);
  }
}

// One workgroup per row: the histogram bins that hold sorted positions k and k+1 bound s_k from
// below and s_{k+1} from above; the key window [klo, khi] holds both bins and every element that
// passes the necessary conditions for joining the block (pooling.hpp: left_candidate,
// right_candidate) for ANY s_k, s_{k+1} inside those bins.  Requires 1 <= k < n.
template <bool MAG>
__global__ __launch_bounds__(kThreads) void select_window_kernel(const uint32_t* __restrict__ bins,
                                                                 RowSel* __restrict__ sel,
                                                                 int64_t k, Reg R) {
  constexpr int kPerThread = kSelBins / kThreads;
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t found[2];
  const int64_t row = blockIdx.x;
  const uint32_t* b = bins + row * kSelBins;
  uint32_t c[kPerThread], mine = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    c[i] = b[threadIdx.x * kPerThread + i];
    mine += c[i];
  }
  uint32_t run = block_exclusive_scan(mine, wave_tot, nullptr);
  // position q (1-based) lies in the first bin whose inclusive count reaches q
  const uint32_t q0 = uint32_t(k), q1 = uint32_t(k + 1);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t next = run + c[i];
    if (run < q0 && q0 <= next) found[0] = threadIdx.x * kPerThread + i;
    if (run < q1 && q1 <= next) found[1] = threadIdx.x * kPerThread + i;
    run = next;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t klo, khi;
    key_window<MAG>(found[0], found[1], R, &klo, &khi);
    sel[row].klo = klo;
    sel[row].khi = khi;
  }
}

// Ordered compaction of the candidates of every tile to the start of the tile's own slot of the
// output arrays (row stride n, tile stride kTile), with their count, the number of elements of
// the tile above the window, and the digit histogram of the first sorting pass.
template <bool MAG>
__global__ __launch_bounds__(kThreads) void select_compact_kernel(
    const float* __restrict__ x, const RowSel* __restrict__ sel, uint32_t* __restrict__ keys_out,
    uint32_t* __restrict__ idx_out, uint32_t* __restrict__ tcnt, uint32_t* __restrict__ tabove,
    uint32_t* __restrict__ hist, int64_t n, int tiles) {
  __shared__ uint32_t cnt[kWaves][kRadix];
  __shared__ uint32_t wave_cand[kWaves], wave_above[kWaves];
  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const uint32_t klo = sel[row].klo, khi = sel[row].khi;
  const int64_t row_base = row * n;
  const int64_t tile_first = int64_t(tile) * kTile;
  const int chunk = w * (kTile / kWaves);
  uint32_t key[kItems], idx[kItems], pos[kItems];
  uint32_t ncand = 0, nabove = 0;                    // wavefront totals (uniform)
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = tile_first + chunk + i * kWave + lane;
    const bool valid = e < n;
    key[i] = 0xffffffffu;
    idx[i] = 0;
    if (valid) {
      const float v = x[row_base + e];
      key[i] = first_key<MAG>(v);
      idx[i] = MAG ? ((uint32_t(e) << 1) | (__float_as_uint(v) >> 31)) : uint32_t(e);
    }
    const bool cand = valid && key[i] >= klo && key[i] <= khi;
    const unsigned long long cm = __ballot(cand);
    nabove += __popcll(__ballot(valid && key[i] < klo));
    pos[i] = cand ? ncand + __popcll(cm & lanemask_lt()) : 0xffffffffu;
    ncand += __popcll(cm);
    count_digit(cnt[w], key[i] & (kRadix - 1), cand, lane);
  }
  if (lane == 0) {
    wave_cand[w] = ncand;
    wave_above[w] = nabove;
  }
  __syncthreads();
  uint32_t before = 0, total = 0, above = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) {
    if (q < w) before += wave_cand[q];
    total += wave_cand[q];
    above += wave_above[q];
  }
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (pos[i] != 0xffffffffu) {
      const int64_t dst = row_base + tile_first + before + pos[i];
      keys_out[dst] = key[i];
      idx_out[dst] = idx[i];
    }
  }
  if (threadIdx.x == 0) {
    tcnt[row * tiles + tile] = total;
    tabove[row * tiles + tile] = above;
  }
  const int d = threadIdx.x;
  uint32_t tot = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) tot += cnt[q][d];
  hist[(row * kRadix + d) * tiles + tile] = tot;
}

// ---- pass drivers ------------------------------------------------------------------------------
void launch_scan(int64_t rows, int tiles, const SortBuffers& B, const RowSel* sel,
                 RowSel* sel_out, hipStream_t st) {
  if (tiles <= 32)
    hipLaunchKernelGGL(radix_scan_narrow_kernel, dim3(unsigned(rows)), dim3(kThreads), 0, st,
                       B.hist, B.dtot, sel, B.tcnt, B.tabove, sel_out, tiles);
  else
    hipLaunchKernelGGL(radix_scan_wide_kernel, dim3(unsigned(rows * kRadix)), dim3(kThreads), 0,
                       st, B.hist, B.dtot, sel, B.tcnt, B.tabove, sel_out, tiles);
}

template <bool MAG>
void sort_passes(const float* x, int64_t rows, int64_t n, const SortBuffers& B, hipStream_t st) {
  const int tiles = int((n + kTile - 1) / kTile);
  const unsigned blocks = unsigned(rows * tiles);
  uint32_t* kin = nullptr;
  uint32_t* iin = nullptr;
  uint32_t* kout = B.keys_b;
  uint32_t* iout = B.idx_b;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 8 * pass;
    if (pass == 0)
      hipLaunchKernelGGL((radix_hist_kernel<true, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, B.hist, nullptr, n, tiles, shift);
    else
      hipLaunchKernelGGL((radix_hist_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, B.hist, nullptr, n, tiles, shift);
    launch_scan(rows, tiles, B, nullptr, nullptr, st);
    if (pass == 0)
      hipLaunchKernelGGL((radix_scatter_kernel<true, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, iin, kout, iout, B.hist, B.dtot, nullptr, nullptr, n, tiles, shift);
    else
      hipLaunchKernelGGL((radix_scatter_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st,
                         x, kin, iin, kout, iout, B.hist, B.dtot, nullptr, nullptr, n, tiles,
                         shift);
    // ping-pong: pass 0 writes b, pass 1 writes a, pass 2 writes b, pass 3 writes a
    kin = kout;
    iin = iout;
    kout = (kout == B.keys_b) ? B.keys_a : B.keys_b;
    iout = (iout == B.idx_b) ? B.idx_a : B.idx_b;
  }
}

template <bool MAG>
void candidate_passes(const float* x, int64_t rows, int64_t n, int64_t k, const Reg& R,
                      const SortBuffers& B, hipStream_t st) {
  const int tiles = int((n + kTile - 1) / kTile);
  const unsigned blocks = unsigned(rows * tiles);
  const int sel_tiles = int((n + kSelTile - 1) / kSelTile);
  const int64_t nbins = rows * kSelBins;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(unsigned((nbins + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, st, B.bins, nbins);
  hipLaunchKernelGGL((select_hist_kernel<MAG>), dim3(unsigned(rows * sel_tiles)), dim3(kThreads), 0,
                     st, x, B.bins, n, sel_tiles);
  hipLaunchKernelGGL((select_window_kernel<MAG>), dim3(unsigned(rows)), dim3(kThreads), 0, st,
                     B.bins, B.sel, k, R);
  // candidates into the per-tile slots of the "a" arrays, with the histogram of pass 0
  hipLaunchKernelGGL((select_compact_kernel<MAG>), dim3(blocks), dim3(kThreads), 0, st, x, B.sel,
                     B.keys_a, B.idx_a, B.tcnt, B.tabove, B.hist, n, tiles);
  launch_scan(rows, tiles, B, nullptr, B.sel, st);
  hipLaunchKernelGGL((radix_scatter_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                     B.keys_a, B.idx_a, B.keys_b, B.idx_b, B.hist, B.dtot, B.tcnt, nullptr, n,
                     tiles, 0);
  // passes 1..3 on the dense candidate lists: b -> a -> b -> a
  uint32_t* kin = B.keys_b;
  uint32_t* iin = B.idx_b;
  uint32_t* kout = B.keys_a;
  uint32_t* iout = B.idx_a;
  for (int pass = 1; pass < 4; ++pass) {
    const int shift = 8 * pass;
    hipLaunchKernelGGL((radix_hist_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x, kin,
                       B.hist, B.sel, n, tiles, shift);
    launch_scan(rows, tiles, B, B.sel, nullptr, st);
    hipLaunchKernelGGL((radix_scatter_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                       kin, iin, kout, iout, B.hist, B.dtot, nullptr, B.sel, n, tiles, shift);
    uint32_t* t = kin; kin = kout; kout = t;
    t = iin; iin = iout; iout = t;
  }
}

}  // namespace

int radix_tiles(int64_t n) { return int((n + kTile - 1) / kTile); }

// Sorted keys end in B.keys_a, their index payload in B.idx_a.
int launch_segmented_sort(bool mag, const float* x, int64_t rows, int64_t n, const SortBuffers& B,
                          hipStream_t st) {
  const int64_t tiles = radix_tiles(n);
  if (rows * tiles > 0x7fffffffLL || rows * kRadix > 0x7fffffffLL) return -1;
  if (mag) sort_passes<true>(x, rows, n, B, st);
  else sort_passes<false>(x, rows, n, B, st);
  return 0;
}

// Candidate lists sorted in B.keys_a / B.idx_a (row stride n), B.sel[row] = {window, count, above}.
int launch_candidate_sort(bool mag, const float* x, int64_t rows, int64_t n, int64_t k,
                          const Reg& R, const SortBuffers& B, hipStream_t st) {
  const int64_t tiles = radix_tiles(n);
  if (k < 1 || k >= n) return -1;
  if (rows * tiles > 0x7fffffffLL || rows * kRadix > 0x7fffffffLL) return -1;
  if (mag) candidate_passes<true>(x, rows, n, k, R, B, st);
  else candidate_passes<false>(x, rows, n, k, R, B, st);
  return 0;
}

}  // namespace topk
