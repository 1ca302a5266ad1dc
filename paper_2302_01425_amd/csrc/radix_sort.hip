// Long rows: segmented, stable, least-significant-digit radix sort of (key, index) pairs through
// HBM, several workgroups per row.  Four passes of 8 bits; each pass is
//   digit histogram per tile  ->  exclusive scan per (row, digit) over tiles  ->  stable scatter.
// Keys are the descending-order keys of common.hpp, so ascending stable order of the keys is
// "value descending, original index ascending" (paper Sec. 3 sorts in descending order).
//
// Within a tile every wavefront owns a contiguous quarter; item i of lane l is element
// i*64 + l of that quarter, so loads are coalesced and the order (wave, item, lane) is the
// element order.  Equal digits inside a wavefront are found with ballots (no LDS atomics).
#include "common.hpp"
#include "launch.hpp"

namespace topk {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;
constexpr int kTile = kThreads * kItems;          // 4096 elements per workgroup and pass
constexpr int kRadix = 256;

// lanes (among `valid`) that hold the same 8-bit digit as this lane
__device__ __forceinline__ unsigned long long match_digit(uint32_t d, unsigned long long valid) {
  unsigned long long peers = valid;
#pragma unroll
  for (int bit = 0; bit < 8; ++bit) {
    const bool one = (d >> bit) & 1u;
    const unsigned long long bal = __ballot(one);
    peers &= one ? bal : ~bal;
  }
  return peers;
}

__device__ __forceinline__ unsigned long long lanemask_lt() {
  const int lane = threadIdx.x & (kWave - 1);
  return (1ull << lane) - 1ull;
}

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

// Key of element e of a row in the first pass (from the float input), later passes read keys.
template <bool MAG>
__device__ __forceinline__ uint32_t first_key(float v) {
  return desc_key(MAG ? fabsf(v) : v);
}

// ---- 1. per-tile digit histogram ------------------------------------------------------------
// hist layout: [row][digit][tile]
template <bool FIRST, bool MAG>
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const float* __restrict__ x,
                                                              const uint32_t* __restrict__ keys,
                                                              uint32_t* __restrict__ hist,
                                                              int64_t n, int tiles, int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];
  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();
  const int64_t row_base = row * n;
  const int64_t chunk = int64_t(tile) * kTile + int64_t(w) * (kTile / kWaves);
#pragma unroll 4
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = chunk + i * kWave + lane;
    const bool valid = e < n;
    uint32_t key = 0;
    if (valid) key = FIRST ? first_key<MAG>(x[row_base + e]) : keys[row_base + e];
    const uint32_t d = (key >> shift) & (kRadix - 1);
    const unsigned long long vm = __ballot(valid);
    if (vm == 0) continue;
    // The digit of the first valid lane is counted once for all lanes that share it (this keeps
    // skewed digits, e.g. the exponent byte, from serialising); the other lanes add 1 each to
    // this wavefront's private counters.
    const int first = __ffsll((long long)vm) - 1;
    const uint32_t d0 = uint32_t(__builtin_amdgcn_readlane(int(d), first));
    const bool same = valid && d == d0;
    const unsigned long long m0 = __ballot(same);
    if (lane == first) cnt[w][d0] += __popcll(m0);
    if (valid && !same) atomicAdd(&cnt[w][d], 1u);
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
__global__ __launch_bounds__(kThreads) void radix_scan_wide_kernel(uint32_t* __restrict__ hist,
                                                                   uint32_t* __restrict__ dtot,
                                                                   int tiles) {
  __shared__ uint32_t wave_tot[kWaves];
  uint32_t* h = hist + int64_t(blockIdx.x) * tiles;
  uint32_t carry = 0;
  for (int c = 0; c < tiles; c += kThreads) {
    const int t = c + threadIdx.x;
    const uint32_t v = (t < tiles) ? h[t] : 0u;
    uint32_t total;
    const uint32_t ex = block_exclusive_scan(v, wave_tot, &total);
    if (t < tiles) h[t] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) dtot[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kThreads) void radix_scan_narrow_kernel(uint32_t* __restrict__ hist,
                                                                     uint32_t* __restrict__ dtot,
                                                                     int tiles) {
  const int64_t rd = int64_t(blockIdx.x) * kRadix + threadIdx.x;
  uint32_t* h = hist + rd * tiles;
  uint32_t carry = 0;
  for (int t = 0; t < tiles; ++t) {
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
    const uint32_t* __restrict__ dtot, int64_t n, int tiles, int shift) {
  __shared__ uint32_t cnt[kWaves][kRadix];       // per-wave digit counts, then per-wave offsets
  __shared__ uint32_t gdelta[kRadix];            // global destination minus position in the tile
  __shared__ uint32_t wave_tot[kWaves];
  __shared__ uint32_t kbuf[kTile];
  __shared__ uint32_t ibuf[kTile];

  const int64_t row = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  for (int i = threadIdx.x; i < kWaves * kRadix; i += kThreads) (&cnt[0][0])[i] = 0;
  __syncthreads();

  const int64_t row_base = row * n;
  const int64_t chunk = int64_t(tile) * kTile + int64_t(w) * (kTile / kWaves);
  uint32_t key[kItems], idx[kItems], rank[kItems];
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const int64_t e = chunk + i * kWave + lane;
    const bool valid = e < n;
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
    const int64_t e = chunk + i * kWave + lane;
    if (e < n) {
      const uint32_t d = (key[i] >> shift) & (kRadix - 1);
      const uint32_t lp = cnt[w][d] + rank[i];
      kbuf[lp] = key[i];
      ibuf[lp] = idx[i];
    }
  }
  __syncthreads();

  const int64_t tile_first = int64_t(tile) * kTile;
  const int valid_count = int(min<int64_t>(kTile, n - tile_first));
  for (int j = threadIdx.x; j < valid_count; j += kThreads) {
    const uint32_t kk = kbuf[j];
    const uint32_t d = (kk >> shift) & (kRadix - 1);
    const int64_t dst = row_base + int64_t(gdelta[d] + uint32_t(j));
    keys_out[dst] = kk;
    idx_out[dst] = ibuf[j];
  }
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
                         kin, B.hist, n, tiles, shift);
    else
      hipLaunchKernelGGL((radix_hist_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, B.hist, n, tiles, shift);
    if (tiles <= 32)
      hipLaunchKernelGGL(radix_scan_narrow_kernel, dim3(unsigned(rows)), dim3(kThreads), 0, st,
                         B.hist, B.dtot, tiles);
    else
      hipLaunchKernelGGL(radix_scan_wide_kernel, dim3(unsigned(rows * kRadix)), dim3(kThreads), 0,
                         st, B.hist, B.dtot, tiles);
    if (pass == 0)
      hipLaunchKernelGGL((radix_scatter_kernel<true, MAG>), dim3(blocks), dim3(kThreads), 0, st, x,
                         kin, iin, kout, iout, B.hist, B.dtot, n, tiles, shift);
    else
      hipLaunchKernelGGL((radix_scatter_kernel<false, MAG>), dim3(blocks), dim3(kThreads), 0, st,
                         x, kin, iin, kout, iout, B.hist, B.dtot, n, tiles, shift);
    // ping-pong: pass 0 writes b, pass 1 writes a, pass 2 writes b, pass 3 writes a
    kin = kout;
    iin = iout;
    kout = (kout == B.keys_b) ? B.keys_a : B.keys_b;
    iout = (iout == B.idx_b) ? B.idx_a : B.idx_b;
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

}  // namespace topk
