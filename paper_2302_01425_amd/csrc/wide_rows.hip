// Wide route, middle step: one workgroup per row collects, sorts and solves the row's candidates.
//
// The candidates of a row (the elements inside the key window [klo, khi] that holds everything
// able to pool, pooling.hpp) lie in the per-tile slots of the "b" arrays: tcnt[tile] of them at
// the start of each slot, in index order; tabove[tile] elements of the tile are above the window.
// This kernel
//   1. scans the tiles' counts: where each tile's candidates start in the row's list, the length
//      cn of the list, the number of elements above the window;
//   2. copies the candidates into the row's dense list in the "a" arrays (key, index payload) and
//      their keys into LDS (list position -> tile by bisection over the offsets);
//   3. sorts the KEYS.  The outputs are computed from values, so no permutation is needed and
//      equal keys may come in any order.  Lists of up to kWideLdsCap keys: one bucket pass in LDS
//      (bucket = leading bits of key - klo, about two keys per bucket; LDS atomics hand out the
//      places inside a bucket, a count of the smaller keys of the bucket orders them); lists
//      whose keys crowd into few buckets, and longer lists, take LSD radix passes (in LDS, resp.
//      through the "b" arrays, which are free by then);
//   4. grows the block on the sorted keys (long_solve.hpp);
//   5. adds up the tangent over the block's elements, found by value in the unsorted list
//      (Prop. 7), and writes the row's RowInfo: gamma, d gamma and the block's value window.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "launch.hpp"
#include "long_solve.hpp"
#include "pooling.hpp"
#include "radix.hpp"

namespace topk {
namespace {

constexpr int kWT = 1024;                      // threads
constexpr int kWW = kWT / kWave;               // wavefronts
constexpr int kWideLdsCap = 16384;             // keys of a list sorted in LDS
constexpr int kWideBuckets = 8192;             // buckets of the one-pass sort
constexpr int kBucketMax = 32;                 // longest bucket the one-pass sort orders by counting
constexpr int kSlotTile = 4096;                // slot stride of the compaction (radix_sort.hip)

struct WideShared {
  uint32_t keys_a[kWideLdsCap];                // the list's keys; the sorted keys end here
  uint32_t keys_b[kWideLdsCap];                // tile offsets during the gather, then sort buffer
  union {
    uint32_t bucket[kWideBuckets / 2];         // two 16-bit counters / offsets per word
    uint32_t cnt[kWW][kRadix];                 // radix passes: per-wave digit counts / offsets
  } u;
  uint32_t base[kRadix];
  uint32_t gofs[kRadix];
  SolveShared<kWT> solve;
  uint32_t wave_tot[kWW];
  uint32_t max_bucket;
};

// exclusive scan of one value per thread over the workgroup; *total gets the sum
__device__ __forceinline__ uint32_t wide_exclusive_scan(uint32_t v, uint32_t* wave_tot,
                                                        uint32_t* total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  __syncthreads();
  if (lane == kWave - 1) wave_tot[w] = inc;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int q = 0; q < kWW; ++q) {
    const uint32_t t = wave_tot[q];
    if (q < w) before += t;
    all += t;
  }
  if (total) *total = all;
  return before + inc - v;
}

// one keys-only LSD pass: kin -> kout (LDS or global), stable, by the 8-bit digit of (key - klo)
// at `shift`; tiles of ni * 1024 keys, wave w owns keys w * ni * 64 .. of a tile
template <int ITEMS>
__device__ __forceinline__ void wide_radix_pass(const uint32_t* kin, uint32_t* kout, uint32_t cn,
                                                uint32_t klo, int shift, int ni, WideShared& sm) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const uint32_t tile_elems = uint32_t(ni) * kWT;
  const uint32_t wave_elems = uint32_t(ni) * kWave;
  const bool single = cn <= tile_elems;
  if (!single) {
    for (int i = threadIdx.x; i < kWW * kRadix; i += kWT) (&sm.u.cnt[0][0])[i] = 0;
    __syncthreads();
    for (uint32_t tile_first = 0; tile_first < cn; tile_first += tile_elems) {
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        if (i < ni) {
          const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
          const bool valid = e < cn;
          const uint32_t key = valid ? kin[e] : 0u;
          count_digit(sm.u.cnt[w], ((key - klo) >> shift) & (kRadix - 1), valid, lane);
        }
      }
    }
    __syncthreads();
    uint32_t tot = 0;
    if (threadIdx.x < kRadix) {
#pragma unroll
      for (int q = 0; q < kWW; ++q) tot += sm.u.cnt[q][threadIdx.x];
    }
    const uint32_t ex = wide_exclusive_scan(tot, sm.wave_tot, nullptr);
    if (threadIdx.x < kRadix) sm.base[threadIdx.x] = ex;
  }
  for (uint32_t tile_first = 0; tile_first < cn; tile_first += tile_elems) {
    __syncthreads();
    for (int i = threadIdx.x; i < kWW * kRadix; i += kWT) (&sm.u.cnt[0][0])[i] = 0;
    __syncthreads();
    uint32_t key[ITEMS], rank[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i < ni) {
        const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
        const bool valid = e < cn;
        key[i] = valid ? kin[e] : 0u;
        const uint32_t d = ((key[i] - klo) >> shift) & (kRadix - 1);
        const unsigned long long peers = match_digit(d, __ballot(valid));
        const unsigned long long lower = peers & lanemask_lt();
        uint32_t pre = 0;
        if (valid) {
          pre = sm.u.cnt[w][d];
          if (lower == 0) sm.u.cnt[w][d] = pre + __popcll(peers);
        }
        rank[i] = pre + __popcll(lower);
      }
    }
    __syncthreads();
    uint32_t run = 0;
    if (threadIdx.x < kRadix) {
#pragma unroll
      for (int q = 0; q < kWW; ++q) {
        const uint32_t c = sm.u.cnt[q][threadIdx.x];
        sm.u.cnt[q][threadIdx.x] = run;
        run += c;
      }
    }
    if (single) {
      const uint32_t ex = wide_exclusive_scan(run, sm.wave_tot, nullptr);
      if (threadIdx.x < kRadix) sm.gofs[threadIdx.x] = ex;
    } else if (threadIdx.x < kRadix) {
      const uint32_t b = sm.base[threadIdx.x];
      sm.gofs[threadIdx.x] = b;
      sm.base[threadIdx.x] = b + run;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i < ni) {
        const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
        if (e < cn) {
          const uint32_t d = ((key[i] - klo) >> shift) & (kRadix - 1);
          kout[sm.gofs[d] + sm.u.cnt[w][d] + rank[i]] = key[i];
        }
      }
    }
  }
  __syncthreads();
}

// LSD passes over as many bits as the window spans: src -> b0 -> b1 -> b0 ...; returns the buffer
// that holds the sorted keys (src itself when the window is a single key)
__device__ __forceinline__ const uint32_t* wide_radix_sort(const uint32_t* src, uint32_t* b0,
                                                           uint32_t* b1, uint32_t cn, uint32_t klo,
                                                           int nbits, WideShared& sm) {
  int ni = int((cn + kWT - 1) / kWT);
  ni = ni > 16 ? 16 : ni;
  const uint32_t* cur = src;
  bool even = true;
  for (int shift = 0; shift < nbits; shift += 8) {
    uint32_t* kout = even ? b0 : b1;
    wide_radix_pass<16>(cur, kout, cn, klo, shift, ni, sm);
    cur = kout;
    even = !even;
  }
  return cur;
}

// bucket of a key of the list (keys lie in [klo, khi], so the index is below kWideBuckets; the
// clamp only keeps a key that does not from writing outside the counters)
__device__ __forceinline__ uint32_t bucket_of(uint32_t key, uint32_t klo, int shift) {
  const uint32_t b = (key - klo) >> shift;
  return b < uint32_t(kWideBuckets) ? b : uint32_t(kWideBuckets - 1);
}

__device__ __forceinline__ uint32_t half_of(uint32_t word, uint32_t b) {
  return (word >> (16u * (b & 1u))) & 0xffffu;
}

// One bucket pass over the cn <= kWideLdsCap keys in sm.keys_a; the sorted keys end in
// sm.keys_a.  Returns false (keys_a untouched) when some bucket is too long to be ordered by
// counting.
__device__ __forceinline__ bool wide_bucket_sort(uint32_t cn, uint32_t klo, int nbits,
                                                 WideShared& sm) {
  constexpr int kBucketBits = 13;
  static_assert((1 << kBucketBits) == kWideBuckets, "bucket index = leading bits of key - klo");
  const int shift = nbits > kBucketBits ? nbits - kBucketBits : 0;
  for (int i = threadIdx.x; i < kWideBuckets / 2; i += kWT) sm.u.bucket[i] = 0;
  if (threadIdx.x == 0) sm.max_bucket = 0;
  __syncthreads();
  for (uint32_t j = threadIdx.x; j < cn; j += kWT) {
    const uint32_t b = bucket_of(sm.keys_a[j], klo, shift);
    atomicAdd(&sm.u.bucket[b >> 1], 1u << (16u * (b & 1u)));
  }
  __syncthreads();
  // counts -> exclusive starts; every thread owns 4 words = 8 buckets
  constexpr int kWordsPer = kWideBuckets / 2 / kWT;
  uint32_t c[2 * kWordsPer], mine = 0, longest = 0;
#pragma unroll
  for (int i = 0; i < kWordsPer; ++i) {
    const uint32_t wd = sm.u.bucket[threadIdx.x * kWordsPer + i];
    c[2 * i] = wd & 0xffffu;
    c[2 * i + 1] = wd >> 16;
    mine += c[2 * i] + c[2 * i + 1];
    longest = max(longest, max(c[2 * i], c[2 * i + 1]));
  }
  if (longest > uint32_t(kBucketMax)) atomicMax(&sm.max_bucket, longest);
  uint32_t run = wide_exclusive_scan(mine, sm.wave_tot, nullptr);
  if (sm.max_bucket > uint32_t(kBucketMax)) return false;      // uniform: read after the barriers
#pragma unroll
  for (int i = 0; i < kWordsPer; ++i) {
    const uint32_t lo = run;
    run += c[2 * i];
    const uint32_t hi = run;
    run += c[2 * i + 1];
    sm.u.bucket[threadIdx.x * kWordsPer + i] = lo | (hi << 16);
  }
  __syncthreads();
  // places inside the buckets in arrival order (any order will do), then order each bucket
  for (uint32_t j = threadIdx.x; j < cn; j += kWT) {
    const uint32_t key = sm.keys_a[j];
    const uint32_t b = bucket_of(key, klo, shift);
    const uint32_t old = atomicAdd(&sm.u.bucket[b >> 1], 1u << (16u * (b & 1u)));
    sm.keys_b[half_of(old, b)] = key;
  }
  __syncthreads();
  // every counter now holds the end of its bucket = the start of the next one
  for (uint32_t q = threadIdx.x; q < cn; q += kWT) {
    const uint32_t key = sm.keys_b[q];
    const uint32_t b = bucket_of(key, klo, shift);
    const uint32_t end = half_of(sm.u.bucket[b >> 1], b);
    const uint32_t start = b == 0 ? 0u : half_of(sm.u.bucket[(b - 1) >> 1], b - 1);
    uint32_t rank = start;
    for (uint32_t i = start; i < end; ++i) {
      const uint32_t other = sm.keys_b[i];
      rank += (other < key || (other == key && i < q)) ? 1u : 0u;
    }
    sm.keys_a[rank] = key;
  }
  __syncthreads();
  return true;
}

template <bool MAG, int PC>
__global__ __launch_bounds__(kWT) void wide_finish_kernel(
    uint32_t* keys_a, uint32_t* idx_a, uint32_t* keys_b, uint32_t* idx_b,
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove, uint32_t* toff,
    const float* __restrict__ tangent_all, const RowSel* __restrict__ sel,
    RowInfo* __restrict__ info, int64_t n, int tiles, int64_t k_row, Reg R) {
  using P = Pool<MAG, PC>;
  __shared__ WideShared sm;
  const int64_t row = blockIdx.x;
  const int64_t base = row * n;
  const uint32_t klo = sel[row].klo, khi = sel[row].khi;
  uint32_t* ka = keys_a + base;
  uint32_t* ia = idx_a + base;
  uint32_t* kb = keys_b + base;                // slots; later a sorting buffer of long lists
  uint32_t* ib = idx_b + base;
  const uint32_t* tc = tcnt + row * tiles;
  const uint32_t* ta = tabove + row * tiles;
  // the tiles' offsets: in LDS when they fit (keys_b is free until the sort), else in global memory
  const bool offsets_in_lds = tiles <= kWideLdsCap;
  uint32_t* tf = offsets_in_lds ? sm.keys_b : toff + row * tiles;

  // ---- 1. offsets of the tiles' candidates, list length, elements above the window -------------
  uint32_t carry = 0, above = 0;
  for (int c0 = 0; c0 < tiles; c0 += kWT * 4) {
    const int t0 = c0 + threadIdx.x * 4;
    uint32_t v[4], mine = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = (t0 + i < tiles) ? tc[t0 + i] : 0u;
      above += (t0 + i < tiles) ? ta[t0 + i] : 0u;
      mine += v[i];
    }
    uint32_t total;
    uint32_t run = carry + wide_exclusive_scan(mine, sm.wave_tot, &total);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (t0 + i < tiles) tf[t0 + i] = run;
      run += v[i];
    }
    carry += total;
  }
  uint32_t above_all;
  wide_exclusive_scan(above, sm.wave_tot, &above_all);
  const uint32_t cn = carry;
  const int64_t k = k_row - int64_t(above_all);
  __syncthreads();                             // the offsets are visible to the whole workgroup

  // ---- 2. the row's dense list: element j belongs to the last tile whose offset is <= j --------
  const bool in_lds = cn <= uint32_t(kWideLdsCap);
  for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 4 * kWT) {
    int64_t src[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t j = j0 + uint32_t(i) * kWT;
      int lo = 0, hi = tiles - 1;              // invariant: tf[lo] <= j
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (tf[mid] <= j) lo = mid; else hi = mid - 1;
      }
      src[i] = int64_t(lo) * kSlotTile + int64_t(j - tf[lo]);
    }
    uint32_t key[4], id[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = j0 + uint32_t(i) * kWT < cn;
      key[i] = ok ? kb[src[i]] : 0u;
      id[i] = ok ? ib[src[i]] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t j = j0 + uint32_t(i) * kWT;
      if (j < cn) {
        ka[j] = key[i];
        ia[j] = id[i];
        if (in_lds) sm.keys_a[j] = key[i];
      }
    }
  }
  __syncthreads();

  // ---- 3. sort the keys ---------------------------------------------------------------------------
  const uint32_t span = khi - klo;
  const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
  const uint32_t* skeys;
  if (in_lds) {
    skeys = sm.keys_a;
    if (nbits > 0 && !wide_bucket_sort(cn, klo, nbits, sm))
      skeys = wide_radix_sort(sm.keys_a, sm.keys_b, sm.keys_a, cn, klo, nbits, sm);
  } else {
    skeys = wide_radix_sort(ka, kb, ib, cn, klo, nbits, sm);
  }

  // ---- 4. the block ---------------------------------------------------------------------------------
  RowInfo ri = RowSolver<kWT>::template solve<MAG, PC, true>(skeys, nullptr, nullptr, int64_t(cn), k,
                                                             R, sm.solve);

  // ---- 5. d gamma: the block's elements are those of the list with lo_incl <= value <= hi_incl --
  if (ri.a <= ri.b && tangent_all != nullptr) {
    const float* tangent = tangent_all + base;
    Acc acc{0.0, 0.0, 0.0, 0};
    for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 4 * kWT) {
      uint32_t id[4];
      float sv[4], tv[4];
      bool in[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t j = j0 + uint32_t(i) * kWT;
        sv[i] = j < cn ? key_to_float(ka[j]) : 0.0f;
        in[i] = j < cn && sv[i] >= ri.lo_incl && sv[i] <= ri.hi_incl;
        id[i] = in[i] ? ia[j] : 0u;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) tv[i] = in[i] ? tangent[MAG ? (id[i] >> 1) : id[i]] : 0.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (!in[i]) continue;
        double t = double(tv[i]);
        if (MAG) {
          if (id[i] & 1u) t = -t;
          if (sv[i] == 0.0f) t = 0.0;
        }
        const double w = P::jac_weight(double(sv[i]) - ri.center, ri.gamma);
        acc.s1 += w * t;
        acc.s2 += w;
      }
    }
    const Acc got = RowSolver<kWT>::sum_acc(acc, sm.solve.acc);
    ri.dgamma = got.s1 / P::jac_denominator(got.s2, double(k - ri.a + 1), R);
  }
  if (threadIdx.x == 0) info[row] = ri;
}

}  // namespace

int launch_wide_finish(bool mag, int pc, const SortBuffers& B, const float* tangent, int64_t rows,
                       int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  if (rows > 0x7fffffffLL) return -1;
  const dim3 grid{unsigned(rows)}, block{kWT};
  const int tiles = radix_tiles(n);
#define TOPK_WIDE_FINISH(M, P)                                                                    \
  hipLaunchKernelGGL((wide_finish_kernel<M, P>), grid, block, 0, st, B.keys_a, B.idx_a, B.keys_b, \
                     B.idx_b, B.tcnt, B.tabove, B.toff, tangent, B.sel, B.info, n, tiles, k, R)
  if (!mag && pc == kP2) TOPK_WIDE_FINISH(false, kP2);
  else if (!mag && pc == kP43) TOPK_WIDE_FINISH(false, kP43);
  else if (mag && pc == kP2) TOPK_WIDE_FINISH(true, kP2);
  else if (mag && pc == kP43) TOPK_WIDE_FINISH(true, kP43);
  else return -1;
#undef TOPK_WIDE_FINISH
  return 0;
}

}  // namespace topk
