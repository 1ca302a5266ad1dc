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
// in two histogram levels (12 + 8 leading key bits) and gathers them, in index order, into a
// dense list per row.  Short lists are then sorted and solved by one workgroup
// (medium_rows.hip); only rows whose list is longer go through the passes of this file.
// topk_argsort_desc sorts whole rows with them.
#include "common.hpp"
#include "launch.hpp"
#include "radix.hpp"
#include "wave.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;
constexpr int kTile = kThreads * kItems;          // 4096 elements per workgroup and pass

// exclusive scan of one value per thread over the NW wavefronts of the block; also returns total
template <int NW = kWaves>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot /*[NW]*/,
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
  for (int q = 0; q < NW; ++q) {
    const uint32_t t = wave_tot[q];
    if (q < w) before += t;
    all += t;
  }
  if (total) *total = all;
  return before + inc - v;
}

// Length of the list a pass sorts in row `row`: the whole row, or (sel != nullptr) the row's
// candidate list -- and then only if it is too long for the single-workgroup finish, which has
// dealt with the shorter ones.
__device__ __forceinline__ int64_t pass_length(int64_t row, int64_t n, const RowSel* __restrict__ sel) {
  if (sel == nullptr) return n;
  const int64_t cn = int64_t(sel[row].cn);
  return cn > kFinishMax ? cn : 0;
}

// ---- 1. per-tile digit histogram ------------------------------------------------------------
// hist layout: [row][digit][tile] with `tiles` tiles per row; a workgroup handles tiles
// (its index in the row) + j * grid_tiles.
template <bool FIRST, bool MAG>
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const float* __restrict__ x,
                                                              const uint32_t* __restrict__ keys,
                                                              uint32_t* __restrict__ hist,
                                                              const RowSel* __restrict__ sel,
                                                              int64_t n, int tiles, int grid_tiles,
                                                              int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];
  const int64_t row = blockIdx.x / grid_tiles;
  const int64_t len = pass_length(row, n, sel);
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int tile = blockIdx.x % grid_tiles; int64_t(tile) * kTile < len; tile += grid_tiles) {
    const int64_t left = len - int64_t(tile) * kTile;
    const int nvalid = int(left > kTile ? kTile : left);
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
    __syncthreads();
  }
}

// ---- 2. exclusive scan over tiles, per (row, digit) -------------------------------------------
// wide: one workgroup per (row, digit); narrow: one workgroup per row, thread = digit.
// `tiles` is the stride of the histogram; only the tiles of the list are scanned.
__device__ __forceinline__ int used_tiles(int64_t row, int64_t n, const RowSel* __restrict__ sel) {
  return int((pass_length(row, n, sel) + kTile - 1) / kTile);
}

__global__ __launch_bounds__(kThreads) void radix_scan_wide_kernel(uint32_t* __restrict__ hist,
                                                                   uint32_t* __restrict__ dtot,
                                                                   const RowSel* __restrict__ sel,
                                                                   int64_t n, int tiles) {
  __shared__ uint32_t wave_tot[kWaves];
  uint32_t* h = hist + int64_t(blockIdx.x) * tiles;
  const int used = used_tiles(blockIdx.x / kRadix, n, sel);
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

__global__ __launch_bounds__(kThreads) void radix_scan_narrow_kernel(uint32_t* __restrict__ hist,
                                                                     uint32_t* __restrict__ dtot,
                                                                     const RowSel* __restrict__ sel,
                                                                     int64_t n, int tiles) {
  const int64_t rd = int64_t(blockIdx.x) * kRadix + threadIdx.x;
  uint32_t* h = hist + rd * tiles;
  const int used = used_tiles(blockIdx.x, n, sel);
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
    const uint32_t* __restrict__ dtot, const RowSel* __restrict__ sel, int64_t n, int tiles,
    int grid_tiles, int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];       // per-wave digit counts, then per-wave offsets
  __shared__ uint32_t gdelta[kRadix];            // global destination minus position in the tile
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t kbuf[kTile];
  __shared__ uint32_t ibuf[kTile];

  const int64_t row = blockIdx.x / grid_tiles;
  const int64_t len = pass_length(row, n, sel);
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t row_base = row * n;
  for (int tile = blockIdx.x % grid_tiles; int64_t(tile) * kTile < len; tile += grid_tiles) {
    const int64_t tile_first = int64_t(tile) * kTile;
    const int64_t left = len - tile_first;
    const int nvalid = int(left > kTile ? kTile : left);
    for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();

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
    __syncthreads();
  }
}

// ---- candidate selection ---------------------------------------------------------------------
constexpr int kSelShift = 32 - kSelBits;

// Device-scope atomics are slow on this multi-die part (10-25 G/s), so no histogram here uses
// them: every workgroup writes its own partial histogram, and reduce_partials_kernel adds them up
// in two stages (the second stage is the loop over `slices` in the kernels that read the result).

// Every workgroup histograms a contiguous span of its row (a multiple of kSelChunk elements) in
// LDS (bin = LDS word: neighbouring bins, the ones a wavefront hits together, lie in different
// banks) and writes the whole histogram to its own slot: partial[row][part][kSelBins].
constexpr int kSelThreads = 1024;
constexpr int kSelChunk = kSelThreads * 16;

// kHistCopies copies of the histogram, chosen by the lane: lanes that hit the same bin in one
// instruction (frequent: a handful of bins hold most of a row) then mostly go to different words,
// and the copies start 8 banks apart, so that those words also lie in different banks.
constexpr int kHistCopies = 4;
constexpr int kHistStride = kSelBins + 8;

template <bool MAG>
__global__ __launch_bounds__(kSelThreads) void select_hist_kernel(const float* __restrict__ x,
                                                                  uint32_t* __restrict__ partial,
                                                                  int64_t n, int64_t span,
                                                                  int parts) {
  __shared__ uint32_t h[kHistCopies * kHistStride];
  const int64_t row = blockIdx.x / parts;
  const int part = blockIdx.x % parts;
  const int64_t first = int64_t(part) * span;
  const int64_t last = (first + span < n) ? first + span : n;
  for (int i = threadIdx.x; i < kHistCopies * kHistStride; i += kSelThreads) h[i] = 0;
  __syncthreads();
  uint32_t* mine = h + (threadIdx.x & (kHistCopies - 1)) * kHistStride;
  const float* xr = x + row * n;
  // rows whose start is 16-byte aligned: sixteen 16-byte loads in flight per thread (the kernel
  // waits on memory, not on the LDS: the more bytes in flight the better)
  const bool vec = ((reinterpret_cast<uintptr_t>(xr) | uintptr_t(first * 4)) & 15u) == 0;
  int64_t c0 = first;
  if (vec) {
    for (; c0 + 4 * kSelChunk <= last; c0 += 4 * kSelChunk) {
      float4 v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i)
        v[i] = load4_stream(xr + c0 + (int64_t(i) * kSelThreads + threadIdx.x) * 4);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        atomicAdd(&mine[first_key<MAG>(v[i].x) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].y) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].z) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].w) >> kSelShift], 1u);
      }
    }
  }
  if (vec) {                                   // what is left in whole chunks: four 16-byte loads
    for (; c0 + kSelChunk <= last; c0 += kSelChunk) {
      float4 v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        v[i] = load4_stream(xr + c0 + (int64_t(i) * kSelThreads + threadIdx.x) * 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        atomicAdd(&mine[first_key<MAG>(v[i].x) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].y) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].z) >> kSelShift], 1u);
        atomicAdd(&mine[first_key<MAG>(v[i].w) >> kSelShift], 1u);
      }
    }
  }
  for (; c0 < last; c0 += kSelChunk) {
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t e = c0 + int64_t(i) * kSelThreads + threadIdx.x;
      v[i] = e < last ? load_stream(xr + e) : 0.0f;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t e = c0 + int64_t(i) * kSelThreads + threadIdx.x;
      if (e < last) atomicAdd(&mine[first_key<MAG>(v[i]) >> kSelShift], 1u);
    }
  }
  __syncthreads();
  uint32_t* dst = partial + (row * parts + part) * kSelBins;
  for (int i = threadIdx.x; i < kSelBins; i += kSelThreads) {
    uint32_t c = 0;
#pragma unroll
    for (int q = 0; q < kHistCopies; ++q) c += h[q * kHistStride + i];
    dst[i] = c;
  }
}

// First stage of the sum of partial histograms: src[row][parts][counters] ->
// dst[row][slices][counters]; slice s adds the parts s, s + slices, ...  One workgroup per
// (row, slice, 128 counters): threads 0..127 and 128..255 take alternate parts.
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const uint32_t* __restrict__ src,
                                                                   uint32_t* __restrict__ dst,
                                                                   int parts, int slices,
                                                                   int counters) {
  __shared__ uint32_t other[128];
  const int groups = counters / 128;
  const int g = blockIdx.x % groups;
  const int slice = (blockIdx.x / groups) % slices;
  const int64_t row = blockIdx.x / (groups * slices);
  const int c = g * 128 + (threadIdx.x & 127);
  const int half = threadIdx.x >> 7;
  const uint32_t* s = src + row * int64_t(parts) * counters + c;
  uint32_t acc = 0;
  int p = slice + half * slices;
  for (; p + 14 * slices < parts; p += 16 * slices) {    // eight loads in flight
    uint32_t a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = s[int64_t(p + 2 * j * slices) * counters];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += a[j];
  }
  for (; p < parts; p += 2 * slices) acc += s[int64_t(p) * counters];
  if (half == 1) other[threadIdx.x & 127] = acc;
  __syncthreads();
  if (half == 0) dst[(row * slices + slice) * counters + c] = acc + other[threadIdx.x];
}

// One workgroup per row: the histogram bins that hold sorted positions k and k+1 bound s_k from
// below and s_{k+1} from above; the key window [klo, khi] holds both bins and every element that
// passes the necessary conditions for joining the block (pooling.hpp: left_candidate,
// right_candidate) for ANY s_k, s_{k+1} inside those bins.  Requires 1 <= k < n.
// bins2 (may be null): the row's partial histograms of the second level, cleared here because the
// compaction pass adds to them.
constexpr int kWinThreads = 1024;              // four bins per thread: every slice's load in flight
template <bool MAG>
__global__ __launch_bounds__(kWinThreads) void select_window_kernel(const uint32_t* __restrict__ bins,
                                                                    RowSel* __restrict__ sel,
                                                                    int64_t k, int gcopies, Reg R,
                                                                    bool cubic,
                                                                    uint32_t* __restrict__ bins2) {
  constexpr int kPerThread = kSelBins / kWinThreads;
  static_assert(kPerThread == 4, "a thread reads its bins of one slice as one uint4");
  __shared__ uint32_t wave_tot[kWinThreads / kWave];
  __shared__ uint32_t found[2];
  const int64_t row = blockIdx.x;
  if (bins2 != nullptr)
    for (int i = threadIdx.x; i < kSelSlices * 2 * kSel2Bins; i += kWinThreads)
      bins2[row * (kSelSlices * 2 * kSel2Bins) + i] = 0u;
  const uint32_t* b = bins + row * gcopies * kSelBins;
  uint32_t c[kPerThread] = {0u, 0u, 0u, 0u}, mine = 0;
  for (int g0 = 0; g0 < gcopies; g0 += kSelSlices) {
    uint4 v[kSelSlices];
#pragma unroll
    for (int q = 0; q < kSelSlices; ++q) {
      v[q] = make_uint4(0u, 0u, 0u, 0u);
      if (g0 + q < gcopies)
        v[q] = reinterpret_cast<const uint4*>(b + int64_t(g0 + q) * kSelBins)[threadIdx.x];
    }
#pragma unroll
    for (int q = 0; q < kSelSlices; ++q) {
      c[0] += v[q].x; c[1] += v[q].y; c[2] += v[q].z; c[3] += v[q].w;
    }
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) mine += c[i];
  uint32_t run = block_exclusive_scan<kWinThreads / kWave>(mine, wave_tot, nullptr);
  // position q (1-based) lies in the first bin whose inclusive count reaches q
  const uint32_t q0 = uint32_t(k), q1 = uint32_t(k + 1);
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t next = run + c[i];
    if (run < q0 && q0 <= next) {
      found[0] = threadIdx.x * kPerThread + i;
      sel[row].bin_k = threadIdx.x * kPerThread + i;
      sel[row].rank_k = q0 - run;
    }
    if (run < q1 && q1 <= next) {
      found[1] = threadIdx.x * kPerThread + i;
      sel[row].bin_k1 = threadIdx.x * kPerThread + i;
      sel[row].rank_k1 = q1 - run;
    }
    run = next;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t klo, khi;
    key_window<MAG>(found[0], found[1], R, cubic, &klo, &khi);
    sel[row].klo = klo;
    sel[row].khi = khi;
  }
}

// Second level: the next kSel2Bits key bits of the elements inside the bins of positions k and
// k+1 (counted by the compaction pass: bins2[row][slices][2][kSel2Bins]) narrow s_k and s_{k+1}
// down to kSelBits + kSel2Bits leading bits; the window is recomputed from those.  One sub-bin
// per thread.
template <bool MAG>
__global__ __launch_bounds__(kThreads) void select_refine_kernel(const uint32_t* __restrict__ bins2,
                                                                 RowSel* __restrict__ sel,
                                                                 int slices, Reg R, bool cubic) {
  static_assert(kSel2Bins == kThreads, "one sub-bin per thread");
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t found[2];
  const int64_t row = blockIdx.x;
  if (threadIdx.x < 2) found[threadIdx.x] = 0;       // (stays 0 only for rows with NaNs)
  const uint32_t rank[2] = {sel[row].rank_k, sel[row].rank_k1};
  uint32_t cs[2] = {0u, 0u};
  {
    const uint32_t* src = bins2 + row * slices * 2 * kSel2Bins + threadIdx.x;
    int sl = 0;
    for (; sl + 7 < slices; sl += 8) {                   // sixteen loads in flight
      uint32_t a[8][2];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        a[q][0] = src[((sl + q) * 2 + 0) * kSel2Bins];
        a[q][1] = src[((sl + q) * 2 + 1) * kSel2Bins];
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) { cs[0] += a[q][0]; cs[1] += a[q][1]; }
    }
    for (; sl < slices; ++sl) {
      cs[0] += src[(sl * 2 + 0) * kSel2Bins];
      cs[1] += src[(sl * 2 + 1) * kSel2Bins];
    }
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t c = cs[h];
    const uint32_t run = block_exclusive_scan(c, wave_tot, nullptr);
    if (run < rank[h] && rank[h] <= run + c) found[h] = threadIdx.x;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t klo, khi;
    key_window<MAG, kSelBits + kSel2Bits>((sel[row].bin_k << kSel2Bits) | found[0],
                                          (sel[row].bin_k1 << kSel2Bits) | found[1], R, cubic,
                                          &klo, &khi);
    sel[row].klo = klo;
    sel[row].khi = khi;
  }
}

// Ordered compaction of the candidates of every tile to the start of the tile's own slot of the
// output arrays (row stride n, tile stride kTile), with their count and the number of elements of
// the tile above the window.  The candidates are staged in LDS in order, so that the slot is
// written with full wavefronts; candidates inside the histogram bins of positions k and k+1 are
// also counted by their next kSel2Bits key bits (second selection level: added to the row's
// partial histograms bins2[row][tile % kSelSlices], which the window kernel has cleared).
// TAU: the payload of a candidate is not its index but the bits of its tangent in sorted-value
// coordinates (t, or sign(x) t for the magnitude operator; 0 without a tangent): what the wide
// route needs, whose outputs are computed from values.
template <bool MAG, bool HIST2 = true, bool TAU = false>
__global__ __launch_bounds__(kThreads) void select_compact_kernel(
    const float* __restrict__ x, const RowSel* __restrict__ sel, uint32_t* __restrict__ keys_out,
    uint32_t* __restrict__ idx_out, uint32_t* __restrict__ tcnt, uint32_t* __restrict__ tabove,
    uint32_t* __restrict__ bins2, int64_t n, int tiles,
    const float* __restrict__ tangent = nullptr) {
  __shared__ uint32_t wave_cand[kWaves], wave_above[kWaves];
  __shared__ uint32_t kbuf[kTile];
  __shared__ uint32_t ibuf[kTile];
  __shared__ uint32_t h2[HIST2 ? 2 * kSel2Bins : 1];
  if (HIST2)
    for (int i = threadIdx.x; i < 2 * kSel2Bins; i += kThreads) h2[i] = 0;
  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  // the window in value space: key order is reversed value order, and -0 == +0 either way
  // (bound_value clamps the keys beyond the infinities, which would decode to NaN)
  const float v_top = float(bound_value(sel[row].klo)), v_bot = float(bound_value(sel[row].khi));
  const uint32_t bin_k = sel[row].bin_k, bin_k1 = sel[row].bin_k1;
  const int64_t row_base = row * n;
  const int64_t tile_first = int64_t(tile) * kTile;
  const int chunk = w * (kTile / kWaves);
  float val[kItems];
  uint32_t pos[kItems];
  uint32_t ncand = 0, nabove = 0;                    // wavefront totals (uniform)
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = tile_first + chunk + i * kWave + lane;
    val[i] = e < n ? x[row_base + e] : 0.0f;
  }
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = tile_first + chunk + i * kWave + lane;
    const bool valid = e < n;
    const float v = MAG ? fabsf(val[i]) : val[i];
    const bool cand = valid && v <= v_top && v >= v_bot;
    const unsigned long long cm = __ballot(cand);
    nabove += __popcll(__ballot(valid && v > v_top));
    pos[i] = cand ? ncand + __popcll(cm & lanemask_lt()) : 0xffffffffu;
    ncand += __popcll(cm);
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
  float tq[TAU ? kItems : 1];              // the candidates' tangents: all loads in flight at once
  if (TAU) {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int64_t e = tile_first + chunk + i * kWave + lane;
      tq[i] = (tangent != nullptr && pos[i] != 0xffffffffu) ? tangent[row_base + e] : 0.0f;
    }
  }
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (pos[i] != 0xffffffffu) {
      const int64_t e = tile_first + chunk + i * kWave + lane;
      kbuf[before + pos[i]] = first_key<MAG>(val[i]);
      if (TAU) {
        float t = tq[TAU ? i : 0];
        if (MAG) t = val[i] == 0.0f ? 0.0f : (val[i] < 0.0f ? -t : t);
        ibuf[before + pos[i]] = __float_as_uint(t);
      } else {
        ibuf[before + pos[i]] = MAG ? ((uint32_t(e) << 1) | (__float_as_uint(val[i]) >> 31)) : uint32_t(e);
      }
    }
  }
  __syncthreads();
  for (uint32_t j = threadIdx.x; j < total; j += kThreads) {
    const uint32_t key = kbuf[j];
    keys_out[row_base + tile_first + j] = key;
    idx_out[row_base + tile_first + j] = ibuf[j];
    if (HIST2) {
      const uint32_t top = key >> kSelShift;
      const uint32_t sub = (key >> (kSelShift - kSel2Bits)) & (kSel2Bins - 1);
      if (top == bin_k) atomicAdd(&h2[sub], 1u);
      if (top == bin_k1) atomicAdd(&h2[kSel2Bins + sub], 1u);
    }
  }
  if (threadIdx.x == 0) {
    tcnt[row * tiles + tile] = total;
    tabove[row * tiles + tile] = above;
  }
  if (HIST2) {
    // the tile's few non-empty counters are added to one of the row's kSelSlices partial histograms
    __syncthreads();
    uint32_t* dst = bins2 + (row * kSelSlices + tile % kSelSlices) * (2 * kSel2Bins);
    for (int i = threadIdx.x; i < 2 * kSel2Bins; i += kThreads)
      if (h2[i] != 0u) atomicAdd(&dst[i], h2[i]);
  }
}

// Second compaction, in place, of every tile's slot to the refined window; adds the elements
// that fall above it to the tile's count of elements above.
// TAU: the surviving candidates' index payloads are replaced by tangent bits (see
// select_compact_kernel); MAG says how the payload encodes the index.
// A workgroup takes kWaves consecutive tiles of a row, one wavefront per tile: a slot of the first
// level holds a few dozen entries, and with one tile per workgroup the kernel was a chain of
// dependent latencies per tile.  Slots of more than kWaveSlot entries (a window that holds a
// quarter of the row) are left to the whole workgroup, one after the other.
constexpr int kWaveSlot = kItems * kWave;         // 1024 entries: kItems per lane

template <bool TAU, bool MAG>
__device__ __forceinline__ uint32_t recompact_payload(uint32_t key, uint32_t id, int64_t row_base,
                                                      const float* __restrict__ tangent) {
  if (!TAU) return id;
  float t = 0.0f;
  if (tangent != nullptr) {
    t = tangent[row_base + (MAG ? (id >> 1) : id)];
    // the key of |x| = 0 is that of +0.0: sign(0) = 0
    if (MAG) t = key == 0x7fffffffu ? 0.0f : ((id & 1u) ? -t : t);
  }
  return __float_as_uint(t);
}

// one wavefront, a slot of at most kWaveSlot entries
template <bool TAU, bool MAG>
__device__ __forceinline__ void recompact_tile_wave(uint32_t klo, uint32_t khi, uint32_t* keys,
                                                    uint32_t* idx, uint32_t* tcnt_p,
                                                    uint32_t* tabove_p, int64_t slot,
                                                    int64_t row_base, int nvalid,
                                                    const float* __restrict__ tangent) {
  const int lane = threadIdx.x & (kWave - 1);
  uint32_t key[kItems], id[kItems], pos[kItems];
  uint32_t ncand = 0, nabove = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    key[i] = id[i] = 0u;
    pos[i] = 0xffffffffu;
    if (i * kWave >= nvalid) continue;            // (uniform)
    const int el = i * kWave + lane;
    const bool valid = el < nvalid;
    if (valid) {
      key[i] = keys[slot + el];
      id[i] = idx[slot + el];
    }
  }
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (i * kWave >= nvalid) continue;
    const bool valid = i * kWave + lane < nvalid;
    const bool cand = valid && key[i] >= klo && key[i] <= khi;
    const unsigned long long cm = __ballot(cand);
    nabove += __popcll(__ballot(valid && key[i] < klo));
    pos[i] = cand ? ncand + __popcll(cm & lanemask_lt()) : 0xffffffffu;
    ncand += __popcll(cm);
  }
  // (every entry of the slot is in registers: the ballots have used them)
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (i * kWave >= nvalid) continue;
    if (pos[i] != 0xffffffffu) {
      keys[slot + pos[i]] = key[i];
      idx[slot + pos[i]] = recompact_payload<TAU, MAG>(key[i], id[i], row_base, tangent);
    }
  }
  if (lane == 0) {
    *tcnt_p = ncand;
    *tabove_p += nabove;
  }
}

// the whole workgroup, any slot
template <bool TAU, bool MAG>
__device__ __forceinline__ void recompact_tile_block(uint32_t klo, uint32_t khi, uint32_t* keys,
                                                     uint32_t* idx, uint32_t* tcnt_p,
                                                     uint32_t* tabove_p, int64_t slot,
                                                     int64_t row_base, int nvalid,
                                                     const float* __restrict__ tangent,
                                                     uint32_t* wave_cand, uint32_t* wave_above) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int chunk = w * (kTile / kWaves);
  uint32_t key[kItems], id[kItems], pos[kItems];
  uint32_t ncand = 0, nabove = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int el = chunk + i * kWave + lane;
    const bool valid = el < nvalid;
    key[i] = valid ? keys[slot + el] : 0u;
    id[i] = valid ? idx[slot + el] : 0u;
    const bool cand = valid && key[i] >= klo && key[i] <= khi;
    const unsigned long long cm = __ballot(cand);
    nabove += __popcll(__ballot(valid && key[i] < klo));
    pos[i] = cand ? ncand + __popcll(cm & lanemask_lt()) : 0xffffffffu;
    ncand += __popcll(cm);
  }
  if (lane == 0) {
    wave_cand[w] = ncand;
    wave_above[w] = nabove;
  }
  __syncthreads();                         // every element of the slot is in registers by now
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
      keys[slot + before + pos[i]] = key[i];
      idx[slot + before + pos[i]] = recompact_payload<TAU, MAG>(key[i], id[i], row_base, tangent);
    }
  }
  if (threadIdx.x == 0) {
    *tcnt_p = total;
    *tabove_p += above;
  }
  __syncthreads();                         // (wave_cand, wave_above are used again for the next tile)
}

template <bool TAU = false, bool MAG = false>
__global__ __launch_bounds__(kThreads) void select_recompact_kernel(
    const RowSel* __restrict__ sel, uint32_t* __restrict__ keys, uint32_t* __restrict__ idx,
    uint32_t* __restrict__ tcnt, uint32_t* __restrict__ tabove, int64_t n, int tiles, int groups,
    const float* __restrict__ tangent = nullptr) {
  __shared__ uint32_t wave_cand[kWaves], wave_above[kWaves];
  const int64_t row = blockIdx.x / groups;
  const int tile0 = (blockIdx.x % groups) * kWaves;
  const int w = threadIdx.x / kWave;
  const uint32_t klo = sel[row].klo, khi = sel[row].khi;
  const int64_t row_base = row * n;
  const int mine = tile0 + w;
  const int nv = mine < tiles ? int(tcnt[row * tiles + mine]) : 0;
  if (!__syncthreads_or(nv > kWaveSlot)) {
    if (nv > 0)
      recompact_tile_wave<TAU, MAG>(klo, khi, keys, idx, tcnt + row * tiles + mine,
                                    tabove + row * tiles + mine, row_base + int64_t(mine) * kTile,
                                    row_base, nv, tangent);
    return;
  }
  for (int q = 0; q < kWaves && tile0 + q < tiles; ++q) {
    const int tile = tile0 + q;
    const int nvalid = int(tcnt[row * tiles + tile]);
    if (nvalid == 0) continue;
    recompact_tile_block<TAU, MAG>(klo, khi, keys, idx, tcnt + row * tiles + tile,
                                   tabove + row * tiles + tile, row_base + int64_t(tile) * kTile,
                                   row_base, nvalid, tangent, wave_cand, wave_above);
  }
}

// One workgroup per row: exclusive prefix of the tiles' candidate counts (where each tile's
// candidates go in the row's dense list), the length of the list and the number of elements
// above the window.  1024 threads, four consecutive tiles each, one scan for both counts
// (candidates in the low half of a 64-bit word, elements above in the high half).
constexpr int kOffThreads = 1024;
__global__ __launch_bounds__(kOffThreads) void select_offsets_kernel(
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove,
    uint32_t* __restrict__ toff, uint32_t* __restrict__ taboff, RowSel* __restrict__ sel, int tiles) {
  constexpr int kOffWaves = kOffThreads / kWave;
  __shared__ uint64_t wave_tot[kOffWaves];
  const int64_t row = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint64_t carry = 0;
  for (int c = 0; c < tiles; c += kOffThreads * 4) {
    const int t0 = c + threadIdx.x * 4;
    uint32_t v[4], ab[4];
    uint64_t mine = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = (t0 + i < tiles) ? tcnt[row * tiles + t0 + i] : 0u;
      ab[i] = (t0 + i < tiles) ? tabove[row * tiles + t0 + i] : 0u;
      mine += uint64_t(v[i]) | (uint64_t(ab[i]) << 32);
    }
    uint64_t inc = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint64_t o = __shfl_up(inc, off, kWave);
      if (lane >= off) inc += o;
    }
    __syncthreads();                               // wave_tot may still be read from the round before
    if (lane == kWave - 1) wave_tot[w] = inc;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int q = 0; q < kOffWaves; ++q) {
      const uint64_t t = wave_tot[q];
      if (q < w) before += t;
      all += t;
    }
    uint64_t run = carry + before + inc - mine;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (t0 + i < tiles) {
        toff[row * tiles + t0 + i] = uint32_t(run);
        taboff[row * tiles + t0 + i] = uint32_t(run >> 32);   // elements above the window in earlier tiles
      }
      run += uint64_t(v[i]) | (uint64_t(ab[i]) << 32);
    }
    carry += all;
  }
  if (threadIdx.x == 0) {
    sel[row].cn = uint32_t(carry);
    sel[row].above = int64_t(carry >> 32);
  }
}

// Every tile's slot (in the "b" arrays) to its place in the row's dense list (in the "a" arrays):
// one wavefront per tile, kWaves consecutive tiles of a row per workgroup (a slot usually holds
// a handful of entries).
__global__ __launch_bounds__(kThreads) void select_gather_kernel(
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ toff,
    const uint32_t* __restrict__ slot_keys, const uint32_t* __restrict__ slot_idx,
    uint32_t* __restrict__ keys_a, uint32_t* __restrict__ idx_a, int64_t n, int tiles, int groups) {
  const int64_t row = blockIdx.x / groups;
  const int tile = (blockIdx.x % groups) * kWaves + threadIdx.x / kWave;
  if (tile >= tiles) return;
  const int lane = threadIdx.x & (kWave - 1);
  const uint32_t count = tcnt[row * tiles + tile];
  if (count == 0) return;
  uint32_t* kd = keys_a + row * n + toff[row * tiles + tile];
  uint32_t* id = idx_a + row * n + toff[row * tiles + tile];
  const int64_t slot = row * n + int64_t(tile) * kTile;
  for (uint32_t j0 = lane; j0 < count; j0 += 4 * kWave) {
    uint32_t kk[4], ii[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t j = j0 + q * kWave;
      kk[q] = j < count ? slot_keys[slot + j] : 0u;
      ii[q] = j < count ? slot_idx[slot + j] : 0u;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t j = j0 + q * kWave;
      if (j < count) {
        kd[j] = kk[q];
        id[j] = ii[q];
      }
    }
  }
}

// ---- pass drivers ------------------------------------------------------------------------------
void launch_scan(int64_t rows, int64_t n, int tiles, const SortBuffers& B, const RowSel* sel,
                 hipStream_t st) {
  if (tiles <= 32)
    hipLaunchKernelGGL(radix_scan_narrow_kernel, dim3(unsigned(rows)), dim3(kThreads), 0, st,
                       B.hist, B.dtot, sel, n, tiles);
  else
    hipLaunchKernelGGL(radix_scan_wide_kernel, dim3(unsigned(rows * kRadix)), dim3(kThreads), 0,
                       st, B.hist, B.dtot, sel, n, tiles);
}

// Four passes a -> b -> a -> b -> a over lists that are already in the "a" arrays (sel != nullptr:
// the candidate lists longer than kFinishMax), or x -> b -> a -> b -> a over whole rows.
template <bool MAG>
void sort_passes(const float* x, int64_t rows, int64_t n, const SortBuffers& B, const RowSel* sel,
                 hipStream_t st) {
  const int tiles = int((n + kTile - 1) / kTile);
  // candidate lists: a capped grid, workgroups loop over the tiles a list really has
  int grid_tiles = tiles;
  if (sel != nullptr) {
    const int64_t cap = 2048 / rows;
    grid_tiles = int(cap < 1 ? 1 : (cap < tiles ? cap : tiles));
  }
  const unsigned blocks = unsigned(rows * grid_tiles);
  const bool from_x = (sel == nullptr);
  uint32_t* kin = from_x ? nullptr : B.keys_a;
  uint32_t* iin = from_x ? nullptr : B.idx_a;
  uint32_t* kout = B.keys_b;
  uint32_t* iout = B.idx_b;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 8 * pass;
    if (pass == 0 && from_x)
      hipLaunchKernelGGL((radix_hist_kernel<true, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, B.hist, sel, n, tiles, grid_tiles, shift);
    else
      hipLaunchKernelGGL((radix_hist_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, B.hist, sel, n, tiles, grid_tiles, shift);
    launch_scan(rows, n, tiles, B, sel, st);
    if (pass == 0 && from_x)
      hipLaunchKernelGGL((radix_scatter_kernel<true, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, iin, kout, iout, B.hist, B.dtot, sel, n, tiles, grid_tiles, shift);
    else
      hipLaunchKernelGGL((radix_scatter_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st,
                         x, kin, iin, kout, iout, B.hist, B.dtot, sel, n, tiles, grid_tiles, shift);
    if (pass == 0 && from_x) {
      kin = B.keys_b; iin = B.idx_b; kout = B.keys_a; iout = B.idx_a;
    } else {
      uint32_t* t = kin; kin = kout; kout = t;
      t = iin; iin = iout; iout = t;
    }
  }
}

template <bool MAG>
void candidate_lists(const float* x, int64_t rows, int64_t n, int64_t k, const Reg& R, bool cubic,
                     const SortBuffers& B, hipStream_t st) {
  const int tiles = int((n + kTile - 1) / kTile);
  const unsigned blocks = unsigned(rows * tiles);
  const int parts = sel_parts(rows, n);
  const int64_t span = sel_span(rows, n);
  const int slices = parts < kSelSlices ? parts : kSelSlices;
  hipLaunchKernelGGL((select_hist_kernel<MAG>), dim3(unsigned(rows * parts)), dim3(kSelThreads), 0,
                     st, x, B.hpart, n, span, parts);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(unsigned(rows * slices * (kSelBins / 128))),
                     dim3(kThreads), 0, st, B.hpart, B.bins, parts, slices, kSelBins);
  hipLaunchKernelGGL((select_window_kernel<MAG>), dim3(unsigned(rows)), dim3(kWinThreads), 0, st,
                     B.bins, B.sel, k, slices, R, cubic, B.bins2);
  // first-level candidates into the per-tile slots of the "b" arrays; second level; slots
  // narrowed in place; dense lists
  hipLaunchKernelGGL((select_compact_kernel<MAG>), dim3(blocks), dim3(kThreads), 0, st, x, B.sel,
                     B.keys_b, B.idx_b, B.tcnt, B.tabove, B.bins2, n, tiles);
  hipLaunchKernelGGL((select_refine_kernel<MAG>), dim3(unsigned(rows)), dim3(kThreads), 0, st,
                     B.bins2, B.sel, kSelSlices, R, cubic);
  const int groups = (tiles + kWaves - 1) / kWaves;
  hipLaunchKernelGGL((select_recompact_kernel<false, false>), dim3(unsigned(rows * groups)),
                     dim3(kThreads), 0, st, B.sel, B.keys_b, B.idx_b, B.tcnt, B.tabove, n, tiles,
                     groups, nullptr);
  hipLaunchKernelGGL(select_offsets_kernel, dim3(unsigned(rows)), dim3(kOffThreads), 0, st, B.tcnt,
                     B.tabove, B.toff, B.taboff, B.sel, tiles);
  hipLaunchKernelGGL(select_gather_kernel, dim3(unsigned(rows * groups)), dim3(kThreads), 0, st,
                     B.tcnt, B.toff, B.keys_b, B.idx_b, B.keys_a, B.idx_a, n, tiles, groups);
}

// The candidate selection of the wide route: the same levels, but the candidates stay in the
// per-tile slots of the "b" arrays (B.tcnt / B.tabove per tile); the workgroup that sorts and
// solves a row collects them itself.  The sum of the first level's partial histograms is only
// launched when there are more partials than the window kernel adds up itself; `refine`: second
// histogram level (its partial histograms are added up by the compaction pass).
template <bool MAG>
void wide_select(const float* x, const float* tangent, int64_t rows, int64_t n, int64_t k,
                 const Reg& R, bool cubic, bool refine, const SortBuffers& B, hipStream_t st) {
  const int tiles = int((n + kTile - 1) / kTile);
  const unsigned blocks = unsigned(rows * tiles);
  const int parts = sel_parts(rows, n);
  const int64_t span = sel_span(rows, n);
  hipLaunchKernelGGL((select_hist_kernel<MAG>), dim3(unsigned(rows * parts)), dim3(kSelThreads), 0,
                     st, x, B.hpart, n, span, parts);
  if (parts > kSelSlices) {
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(unsigned(rows * kSelSlices * (kSelBins / 128))),
                       dim3(kThreads), 0, st, B.hpart, B.bins, parts, kSelSlices, kSelBins);
    hipLaunchKernelGGL((select_window_kernel<MAG>), dim3(unsigned(rows)), dim3(kWinThreads), 0, st,
                       B.bins, B.sel, k, kSelSlices, R, cubic, refine ? B.bins2 : nullptr);
  } else {
    hipLaunchKernelGGL((select_window_kernel<MAG>), dim3(unsigned(rows)), dim3(kWinThreads), 0, st,
                       B.hpart, B.sel, k, parts, R, cubic, refine ? B.bins2 : nullptr);
  }
  if (!refine) {
    hipLaunchKernelGGL((select_compact_kernel<MAG, false, true>), dim3(blocks), dim3(kThreads), 0,
                       st, x, B.sel, B.keys_b, B.idx_b, B.tcnt, B.tabove, B.bins2, n, tiles,
                       tangent);
    return;
  }
  hipLaunchKernelGGL((select_compact_kernel<MAG, true, false>), dim3(blocks), dim3(kThreads), 0, st,
                     x, B.sel, B.keys_b, B.idx_b, B.tcnt, B.tabove, B.bins2, n, tiles, nullptr);
  hipLaunchKernelGGL((select_refine_kernel<MAG>), dim3(unsigned(rows)), dim3(kThreads), 0, st,
                     B.bins2, B.sel, kSelSlices, R, cubic);
  const int groups = (tiles + kWaves - 1) / kWaves;
  hipLaunchKernelGGL((select_recompact_kernel<true, MAG>), dim3(unsigned(rows * groups)),
                     dim3(kThreads), 0, st, B.sel, B.keys_b, B.idx_b, B.tcnt, B.tabove, n, tiles,
                     groups, tangent);
  // thousands of tiles with a few candidates each: the row's dense (key, tangent) list is put
  // together here, by all compute units, and not by the one workgroup that solves the row
  hipLaunchKernelGGL(select_offsets_kernel, dim3(unsigned(rows)), dim3(kOffThreads), 0, st, B.tcnt,
                     B.tabove, B.toff, B.taboff, B.sel, tiles);
  hipLaunchKernelGGL(select_gather_kernel, dim3(unsigned(rows * groups)), dim3(kThreads), 0, st,
                     B.tcnt, B.toff, B.keys_b, B.idx_b, B.keys_a, B.idx_a, n, tiles, groups);
}

}  // namespace

int launch_wide_select(bool mag, int pc, bool refine, const float* x, const float* tangent,
                       int64_t rows, int64_t n, int64_t k, const Reg& R, const SortBuffers& B,
                       hipStream_t st) {
  const int64_t tiles = radix_tiles(n);
  if (k < 1 || k >= n) return -1;
  if (rows * tiles > 0x7fffffffLL || rows * kRadix > 0x7fffffffLL) return -1;
  if (mag) wide_select<true>(x, tangent, rows, n, k, R, pc == kP43, refine, B, st);
  else wide_select<false>(x, tangent, rows, n, k, R, pc == kP43, refine, B, st);
  return 0;
}

int radix_tiles(int64_t n) { return int((n + kTile - 1) / kTile); }

// The first histogram level: about 256 workgroups of 1024 threads in all (one per compute unit),
// each with a span of at least one chunk of its row.
int64_t sel_span(int64_t rows, int64_t n) {
  int64_t span = (n * rows + 255) / 256;
  return (span + kSelChunk - 1) / kSelChunk * kSelChunk;
}
int sel_parts(int64_t rows, int64_t n) {
  const int64_t span = sel_span(rows, n);
  return int((n + span - 1) / span);
}

// Sorted keys end in B.keys_a, their index payload in B.idx_a.
int launch_segmented_sort(bool mag, const float* x, int64_t rows, int64_t n, const SortBuffers& B,
                          hipStream_t st) {
  const int64_t tiles = radix_tiles(n);
  if (rows * tiles > 0x7fffffffLL || rows * kRadix > 0x7fffffffLL) return -1;
  if (mag) sort_passes<true>(x, rows, n, B, nullptr, st);
  else sort_passes<false>(x, rows, n, B, nullptr, st);
  return 0;
}

int launch_candidate_lists(bool mag, int pc, const float* x, int64_t rows, int64_t n, int64_t k,
                           const Reg& R, const SortBuffers& B, hipStream_t st) {
  const int64_t tiles = radix_tiles(n);
  if (k < 1 || k >= n) return -1;
  if (rows * tiles > 0x7fffffffLL || rows * kRadix > 0x7fffffffLL) return -1;
  if (mag) candidate_lists<true>(x, rows, n, k, R, pc == kP43, B, st);
  else candidate_lists<false>(x, rows, n, k, R, pc == kP43, B, st);
  return 0;
}

int launch_long_list_sort(bool mag, int64_t rows, int64_t n, const SortBuffers& B, hipStream_t st) {
  if (mag) sort_passes<true>(nullptr, rows, n, B, B.sel, st);
  else sort_passes<false>(nullptr, rows, n, B, B.sel, st);
  return 0;
}

}  // namespace topk
