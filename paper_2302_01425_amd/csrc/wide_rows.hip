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
  uint64_t wave_tot64[kWW];
  uint32_t max_bucket;
  // block growth on prefix sums (wide_solve)
  Sums wave_sums[kWW];
  int fail_r[kWW], fail_l[kWW];
  struct {
    int a, b;
    Sums pa1, pb;                              // prefix sums up to positions a - 1 and b
  } grow;
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

__device__ __forceinline__ uint64_t wide_exclusive_scan64(uint64_t v, uint64_t* wave_tot,
                                                          uint64_t* total) {
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  uint64_t inc = v;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint64_t o = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += o;
  }
  __syncthreads();
  if (lane == kWave - 1) wave_tot[w] = inc;
  __syncthreads();
  uint64_t before = 0, all = 0;
#pragma unroll
  for (int q = 0; q < kWW; ++q) {
    const uint64_t t = wave_tot[q];
    if (q < w) before += t;
    all += t;
  }
  *total = all;
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
template <int ITEMS>
__device__ __forceinline__ const uint32_t* wide_radix_sort(const uint32_t* src, uint32_t* b0,
                                                           uint32_t* b1, uint32_t cn, uint32_t klo,
                                                           int nbits, WideShared& sm) {
  int ni = int((cn + kWT - 1) / kWT);
  ni = ni > ITEMS ? ITEMS : ni;
  const uint32_t* cur = src;
  bool even = true;
  for (int shift = 0; shift < nbits; shift += 8) {
    uint32_t* kout = even ? b0 : b1;
    wide_radix_pass<ITEMS>(cur, kout, cn, klo, shift, ni, sm);
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


// ---- block growth on prefix sums of the sorted list (lists sorted in LDS) -------------------------
// Thread t owns the sorted positions 16 t + 1 .. 16 t + 16 (1-based): it keeps the power sums of
// all positions before its segment (one workgroup scan, once; also stored in LDS for all
// segments) and the values of its first and last position.  With the block [a, b] and the prefix
// sums up to a - 1 and b published in LDS, a round is
//   A. every thread right of the block tests the FIRST position of its segment as if everything
//      between the block and it had joined (sums = its own prefix minus the prefix up to a - 1),
//      every thread left of the block the LAST position of its segment: the strict tests of the
//      PAV loop (pooling.hpp), which are monotone along each side, so the first failing segment
//      bounds the run of positions that join;
//   B. the segment that holds the end of each run is settled by 16 lanes of the first wavefront,
//      one position each (prefix sums inside the segment by a DPP scan), which publish the new
//      end of the block with its prefix sum.
// Both sides advance in the same round (additions on one side only make the other side's tests
// more true); the growth ends with a round that changes nothing.
constexpr int kSegment = kWideLdsCap / kWT;    // 16

__device__ __forceinline__ Sums sums_sub(const Sums& x, const Sums& y) {
  return Sums{x.s1 - y.s1, x.s2 - y.s2, x.s3 - y.s3};
}
__device__ __forceinline__ Sums sums_add(const Sums& x, const Sums& y) {
  return Sums{x.s1 + y.s1, x.s2 + y.s2, x.s3 + y.s3};
}

// inclusive scan over the 16 lanes of a DPP row (vacated lanes read 0)
__device__ __forceinline__ double row16_inclusive_scan_f64(double v) {
  v += row_shr_f64<1>(v);
  v += row_shr_f64<2>(v);
  v += row_shr_f64<4>(v);
  v += row_shr_f64<8>(v);
  return v;
}

// One position per lane of the segment `seg` (16 lanes of one DPP row): its 1-based position p,
// centred value d (0 beyond the list) and the prefix sums up to p - 1 and up to p.
template <bool CUBIC>
__device__ __forceinline__ void segment_lanes(const uint32_t* keys, const Sums* seg_pre, int seg,
                                              int cn, double center, int i16, int* p_out,
                                              double* d_out, Sums* excl, Sums* incl) {
  const int p = kSegment * seg + 1 + i16;
  const bool valid = seg < kWT && p <= cn;
  const double d = valid ? double(key_to_float(keys[valid ? p - 1 : 0])) - center : 0.0;
  Sums in{row16_inclusive_scan_f64(d), 0.0, 0.0};
  if (CUBIC) {
    in.s2 = row16_inclusive_scan_f64(d * d);
    in.s3 = row16_inclusive_scan_f64(d * d * d);
  }
  Sums ex{row_shr_f64<1>(in.s1), CUBIC ? row_shr_f64<1>(in.s2) : 0.0,
          CUBIC ? row_shr_f64<1>(in.s3) : 0.0};
  const Sums base = seg < kWT ? seg_pre[seg] : Sums{0.0, 0.0, 0.0};
  *p_out = p;
  *d_out = d;
  *excl = sums_add(base, ex);
  *incl = sums_add(base, in);
}

template <bool MAG, int PC>
__device__ RowInfo wide_solve(const uint32_t* keys, uint32_t cn_u, int64_t k64, const Reg& R,
                              WideShared& sm) {
  using P = Pool<MAG, PC>;
  constexpr bool CUBIC = (PC == kP43);
  const int cn = int(cn_u), k = int(k64);
  const int t = threadIdx.x, lane = t & (kWave - 1), w = t / kWave;
  RowInfo ri;
  ri.src = 0;
  ri.pad = 0;
  ri.a = k64 + 1;
  ri.b = k64;
  ri.wa = ri.a;
  ri.wb = ri.b;
  ri.gamma = ri.center = ri.dgamma = 0.0;
  if (!(k >= 1 && k < cn)) {                    // k == 0: everything is below; k == cn: above
    ri.hi_incl = (k <= 0) ? __uint_as_float(0x7f800000u) : __uint_as_float(0xff800000u);
    ri.lo_incl = ri.hi_incl;
    return ri;
  }
  const float fk = key_to_float(keys[k - 1]), fk1 = key_to_float(keys[k]);
  const double center = P::kCentered ? double(fk) : 0.0;
  ri.center = center;
  if (!P::seed_violates(double(fk) - center, double(fk1) - center, R, center)) {
    ri.hi_incl = fk1;                           // s_{k+1} < s_k: "above hi" = the top k
    ri.lo_incl = fk;
    return ri;
  }
  // ---- own segment: totals, first and last value; prefix sums of all segments -----------------
  Sums* seg_pre = reinterpret_cast<Sums*>(sm.keys_b);      // [kWT], the sort is over
  const int q0 = kSegment * t + 1;              // first position of the segment
  const int e = q0 + kSegment - 1;              // last position of the segment
  double d_first = 0.0, d_last = 0.0;
  Sums tot{0.0, 0.0, 0.0};
#pragma unroll
  for (int i = 0; i < kSegment; ++i) {
    const int p = q0 + i;
    const double d = p <= cn ? double(key_to_float(keys[p <= cn ? p - 1 : 0])) - center : 0.0;
    if (i == 0) d_first = d;
    if (i == kSegment - 1) d_last = d;
    tot.s1 += d;
    if (CUBIC) {
      tot.s2 += d * d;
      tot.s3 += d * d * d;
    }
  }
  Sums inc{wave_inclusive_scan_f64(tot.s1), 0.0, 0.0};
  if (CUBIC) {
    inc.s2 = wave_inclusive_scan_f64(tot.s2);
    inc.s3 = wave_inclusive_scan_f64(tot.s3);
  }
  if (lane == kWave - 1) sm.wave_sums[w] = inc;
  __syncthreads();
#pragma unroll
  for (int qw = 0; qw < kWW; ++qw) {
    if (qw < w) {
      const Sums o = sm.wave_sums[qw];
      inc.s1 += o.s1;
      if (CUBIC) { inc.s2 += o.s2; inc.s3 += o.s3; }
    }
  }
  const Sums pre = sums_sub(inc, tot);           // sums of the positions before q0
  seg_pre[t] = pre;
  __syncthreads();
  // ---- the seed block (k, k+1): prefix sums up to k + 1 (row 0) and k - 1 (row 1) -------------
  const int i16 = lane & 15, rowid = lane >> 4;
  if (w == 0 && rowid < 2) {
    const int target = rowid == 0 ? k + 1 : k - 1;
    int p;
    double d;
    Sums ex, in;
    segment_lanes<CUBIC>(keys, seg_pre, target >= 1 ? (target - 1) / kSegment : 0, cn, center, i16,
                         &p, &d, &ex, &in);
    if (rowid == 0 && p == target) sm.grow.pb = in;
    if (rowid == 1 && target >= 1 && p == target) sm.grow.pa1 = in;
    if (rowid == 1 && target == 0 && i16 == 0) sm.grow.pa1 = Sums{0.0, 0.0, 0.0};
    if (lane == 0) { sm.grow.a = k; sm.grow.b = k + 1; }
  }
  __syncthreads();
  int a = k, b = k + 1;
  Sums pa1 = sm.grow.pa1, pb = sm.grow.pb;
  for (int round = 0; round <= cn; ++round) {
    const double m = double(k - a + 1);
    // ---- A: segment tests --------------------------------------------------------------------------
    // right: first position of the segment, block [a, q0 - 1]; segments beyond the list fail
    const bool right_of = q0 > b;
    bool fail_r = right_of;
    if (right_of && q0 <= cn)
      fail_r = !P::right_violates(d_first, double(q0 - a), m, sums_sub(pre, pa1), R, center);
    // left: last position e of the segment, block [e + 1, b]
    bool fail_l = false;
    if (e < a)
      fail_l = !P::left_violates(d_last, double(b - e), double(k - e), sums_sub(pb, inc), R, center);
    const unsigned long long br = __ballot(fail_r), bl = __ballot(fail_l);
    if (lane == 0) {
      sm.fail_r[w] = br ? w * kWave + (__ffsll((long long)br) - 1) : kWT;
      sm.fail_l[w] = bl ? w * kWave + (63 - __clzll((long long)bl)) : -1;
    }
    __syncthreads();
    // ---- B: the two segments that hold the ends of the runs, one position per lane -------------
    if (w == 0 && rowid < 2) {
      int first_fail_r = kWT, last_fail_l = -1;
#pragma unroll
      for (int qw = 0; qw < kWW; ++qw) {
        first_fail_r = min(first_fail_r, sm.fail_r[qw]);
        last_fail_l = max(last_fail_l, sm.fail_l[qw]);
      }
      const int seg = rowid == 0 ? first_fail_r - 1 : last_fail_l + 1;
      int p;
      double d;
      Sums ex, in;
      segment_lanes<CUBIC>(keys, seg_pre, seg, cn, center, i16, &p, &d, &ex, &in);
      // right (row 0): position p joins the block [a, p - 1]; positions up to b are in already
      const bool pass_r = p <= b || (p <= cn && P::right_violates(d, double(p - a), m,
                                                                  sums_sub(ex, pa1), R, center));
      // left (row 1): position p joins the block [p + 1, b]; positions from a on are in already
      const bool pass_l = p >= a || P::left_violates(d, double(b - p), double(k - p),
                                                     sums_sub(pb, in), R, center);
      const unsigned long long ball_r = __ballot(pass_r), ball_l = __ballot(pass_l);
      if (rowid == 0) {
        const uint32_t fails = ~uint32_t(ball_r) & 0xffffu;            // row 0 = lanes 0..15
        const int f = fails ? __ffs(int(fails)) - 1 : kSegment;        // first failing lane
        // the run ends at lane f - 1 (f = 0: at the end of the segment before)
        if (f >= 1 && i16 == f - 1) { sm.grow.b = p; sm.grow.pb = in; }
        if (f == 0 && i16 == 0) { sm.grow.b = p - 1; sm.grow.pb = ex; }
      } else {
        const uint32_t fails = ~uint32_t(ball_l >> 16) & 0xffffu;      // row 1 = lanes 16..31
        const int f = fails ? 31 - __clz(int(fails)) : -1;             // last failing lane
        // the run (downwards) ends at lane f + 1 (f = 15: at the start of the segment after)
        if (f >= 0 && i16 == f) { sm.grow.a = p + 1; sm.grow.pa1 = in; }
        if (f < 0 && i16 == 0) { sm.grow.a = p; sm.grow.pa1 = ex; }
      }
    }
    __syncthreads();
    const int na = sm.grow.a, nb = sm.grow.b;
    pa1 = sm.grow.pa1;
    pb = sm.grow.pb;
    const bool same = (na == a) && (nb == b);
    a = na;
    b = nb;
    __syncthreads();                            // everyone has read the state before it changes again
    if (same) break;
  }
  const Sums S = sums_sub(pb, pa1);
  const float fa = key_to_float(keys[a - 1]), fb = key_to_float(keys[b - 1]);
  const double da = double(fa) - center, db = double(fb) - center;
  ri.a = a;
  ri.b = b;
  ri.wa = a;
  ri.wb = b;
  ri.gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, MAG ? -center : da - R.lambda,
                       MAG ? da : db, center);
  ri.hi_incl = fa;
  ri.lo_incl = fb;
  return ri;
}

// block-wide sum of two doubles (every thread gets the totals)
__device__ __forceinline__ void wide_sum2(double& x, double& y, WideShared& sm) {
#pragma unroll
  for (int off = kWave >> 1; off >= 1; off >>= 1) {
    x += __shfl_xor(x, off, kWave);
    y += __shfl_xor(y, off, kWave);
  }
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) sm.wave_sums[threadIdx.x / kWave] = Sums{x, y, 0.0};
  __syncthreads();
  x = y = 0.0;
#pragma unroll
  for (int q = 0; q < kWW; ++q) {
    x += sm.wave_sums[q].s1;
    y += sm.wave_sums[q].s2;
  }
}

// keys_a / tau_a: the row's dense list (key, tangent of the element in sorted-value coordinates:
// sign(x) t for the magnitude operator); keys_b / pay_b: the tiles' slots with the same payload.
template <bool MAG, int PC>
__global__ __launch_bounds__(kWT) void wide_finish_kernel(
    uint32_t* keys_a, uint32_t* tau_a, uint32_t* keys_b, uint32_t* pay_b,
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove, uint32_t* toff,
    const RowSel* __restrict__ sel, RowInfo* __restrict__ info, int64_t n, int tiles,
    int64_t k_row, Reg R, bool want_jvp) {
  using P = Pool<MAG, PC>;
  __shared__ WideShared sm;
  const int64_t row = blockIdx.x;
  const int64_t base = row * n;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const uint32_t klo = sel[row].klo, khi = sel[row].khi;
  uint32_t* ka = keys_a + base;
  uint32_t* pa = tau_a + base;
  uint32_t* kb = keys_b + base;                // slots; later a sorting buffer of long lists
  uint32_t* pb = pay_b + base;
  const uint32_t* tc = tcnt + row * tiles;
  const uint32_t* ta = tabove + row * tiles;
  // the tiles' offsets: in LDS when they fit (the counters of the sort are free until then)
  constexpr int kLdsTiles = kWideBuckets / 2;
  const bool lds_offsets = tiles <= kLdsTiles;
  uint32_t* gtf = toff + row * tiles;
  uint32_t* tf = lds_offsets ? sm.u.bucket : gtf;      // (generic pointer: for the stores)
  auto off_at = [&](int tl) -> uint32_t { return lds_offsets ? sm.u.bucket[tl] : gtf[tl]; };

  // ---- 1. offsets of the tiles' candidates, list length, elements above the window -------------
  // (one scan for both: candidates in the low half of a 64-bit word, elements above in the high)
  uint64_t carry2 = 0;
  for (int c0 = 0; c0 < tiles; c0 += kWT * 4) {
    const int t0 = c0 + threadIdx.x * 4;
    uint32_t v[4];
    uint64_t mine = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = (t0 + i < tiles) ? tc[t0 + i] : 0u;
      const uint32_t ab = (t0 + i < tiles) ? ta[t0 + i] : 0u;
      mine += uint64_t(v[i]) | (uint64_t(ab) << 32);
    }
    uint64_t total;
    const uint64_t ex = wide_exclusive_scan64(mine, sm.wave_tot64, &total);
    uint32_t run = uint32_t(carry2) + uint32_t(ex);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (t0 + i < tiles) tf[t0 + i] = run;
      run += v[i];
    }
    carry2 += total;
  }
  const uint32_t carry = uint32_t(carry2), above_all = uint32_t(carry2 >> 32);
  const uint32_t cn = carry;
  const int64_t k = k_row - int64_t(above_all);
  const bool in_lds = cn <= uint32_t(kWideLdsCap);
  __syncthreads();                             // the offsets are visible to the whole workgroup

  RowInfo ri;
  if (in_lds) {
    // ---- 2. the row's dense list.  owner[j] = tile of list position j: every non-empty tile
    // marks the start of its candidates, a running maximum fills the rest ------------------------
    uint32_t* owner = sm.keys_b;
    for (uint32_t j = threadIdx.x; j < cn; j += kWT) owner[j] = 0;
    __syncthreads();
    for (int tl = threadIdx.x; tl < tiles; tl += kWT) {
      const uint32_t o = off_at(tl);
      const uint32_t nxt = tl + 1 < tiles ? off_at(tl + 1) : cn;
      if (nxt > o) owner[o] = uint32_t(tl);
    }
    __syncthreads();
    {
      const uint32_t j0 = uint32_t(threadIdx.x) * kSegment;
      uint32_t own[kSegment], mx = 0;
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        own[i] = j0 + i < cn ? owner[j0 + i] : 0u;
        mx = max(mx, own[i]);
      }
      uint32_t inc = mx;                       // inclusive running maximum over the threads
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t o = __shfl_up(inc, off, kWave);
        if (lane >= off) inc = max(inc, o);
      }
      if (lane == kWave - 1) sm.wave_tot[w] = inc;
      __syncthreads();
      uint32_t before = 0;
#pragma unroll
      for (int q = 0; q < kWW; ++q)
        if (q < w) before = max(before, sm.wave_tot[q]);
      const uint32_t up = __shfl_up(inc, 1, kWave);
      uint32_t run = max(before, lane >= 1 ? up : 0u);
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        run = max(run, own[i]);
        if (j0 + i < cn) owner[j0 + i] = run;
      }
    }
    __syncthreads();
    // copy: wave w takes list positions w * 1024 + i * 64 + lane, so that a wavefront reads
    // neighbouring slot entries together.  The (key, tangent) pairs stay in registers for step 5.
    uint32_t key[kSegment], pay[kSegment];
    {
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        const uint32_t j = uint32_t(w) * (kSegment * kWave) + uint32_t(i) * kWave + lane;
        key[i] = pay[i] = 0u;
        if (j < cn) {
          const uint32_t tl = owner[j];
          const int64_t src = int64_t(tl) * kSlotTile + int64_t(j - off_at(int(tl)));
          key[i] = kb[src];
          if (want_jvp) pay[i] = pb[src];
        }
      }
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        const uint32_t j = uint32_t(w) * (kSegment * kWave) + uint32_t(i) * kWave + lane;
        if (j < cn) sm.keys_a[j] = key[i];
      }
    }
    __syncthreads();

    // ---- 3. sort the keys ------------------------------------------------------------------------
    const uint32_t span = khi - klo;
    const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
    const uint32_t* skeys = sm.keys_a;
    if (nbits > 0 && !wide_bucket_sort(cn, klo, nbits, sm)) {
      skeys = wide_radix_sort<8>(sm.keys_a, sm.keys_b, sm.keys_a, cn, klo, nbits, sm);
      if (skeys != sm.keys_a) {                // the solve uses keys_b for its own tables
        for (uint32_t j = threadIdx.x; j < cn; j += kWT) sm.keys_a[j] = sm.keys_b[j];
        __syncthreads();
        skeys = sm.keys_a;
      }
    }

    // ---- 4. the block ----------------------------------------------------------------------------
    ri = wide_solve<MAG, PC>(skeys, cn, k, R, sm);

    // ---- 5. d gamma (Prop. 7): the block's elements are those of the list whose value lies in
    // [lo_incl, hi_incl] -------------------------------------------------------------------------
    if (ri.a <= ri.b && want_jvp) {
      double num = 0.0, den = 0.0;
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        const uint32_t j = uint32_t(w) * (kSegment * kWave) + uint32_t(i) * kWave + lane;
        const float sv = key_to_float(key[i]);
        if (j < cn && sv >= ri.lo_incl && sv <= ri.hi_incl) {
          const double wgt = P::jac_weight(double(sv) - ri.center, ri.gamma);
          num += wgt * double(__uint_as_float(pay[i]));
          den += wgt;
        }
      }
      wide_sum2(num, den, sm);
      ri.dgamma = num / P::jac_denominator(den, double(k - ri.a + 1), R);
    }
  } else {
    // ---- lists too long for LDS (rare: the window holds more than kWideLdsCap elements): the
    // same steps through global memory -----------------------------------------------------------
    int top_step = 1;                          // largest power of two below the number of tiles
    while (2 * top_step < tiles) top_step *= 2;
    if (tiles <= 1) top_step = 0;
    for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 4 * kWT) {
      int64_t src[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t j = j0 + uint32_t(i) * kWT;
        int lo = 0;                            // invariant: tf[lo] <= j
        for (int step = top_step; step > 0; step >>= 1) {
          const int mid = lo + step;
          const uint32_t o = tf[mid < tiles ? mid : 0];
          lo = (mid < tiles && o <= j) ? mid : lo;
        }
        src[i] = int64_t(lo) * kSlotTile + int64_t(j - tf[lo]);
      }
      uint32_t key[4], pay[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = j0 + uint32_t(i) * kWT < cn;
        key[i] = ok ? kb[src[i]] : 0u;
        pay[i] = (ok && want_jvp) ? pb[src[i]] : 0u;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t j = j0 + uint32_t(i) * kWT;
        if (j < cn) {
          ka[j] = key[i];
          if (want_jvp) pa[j] = pay[i];
        }
      }
    }
    __syncthreads();
    const uint32_t span = khi - klo;
    const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
    const uint32_t* skeys = wide_radix_sort<16>(ka, kb, pb, cn, klo, nbits, sm);
    ri = RowSolver<kWT>::template solve<MAG, PC, true>(skeys, nullptr, nullptr, int64_t(cn), k, R,
                                                       sm.solve);
    if (ri.a <= ri.b && want_jvp) {
      double num = 0.0, den = 0.0;
      for (uint32_t j = threadIdx.x; j < cn; j += kWT) {
        const float sv = key_to_float(ka[j]);
        if (sv >= ri.lo_incl && sv <= ri.hi_incl) {
          const double wgt = P::jac_weight(double(sv) - ri.center, ri.gamma);
          num += wgt * double(__uint_as_float(pa[j]));
          den += wgt;
        }
      }
      wide_sum2(num, den, sm);
      ri.dgamma = num / P::jac_denominator(den, double(k - ri.a + 1), R);
    }
  }
  if (threadIdx.x == 0) info[row] = ri;
}

}  // namespace

int launch_wide_finish(bool mag, int pc, const SortBuffers& B, bool want_jvp, int64_t rows,
                       int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  if (rows > 0x7fffffffLL) return -1;
  const dim3 grid{unsigned(rows)}, block{kWT};
  const int tiles = radix_tiles(n);
#define TOPK_WIDE_FINISH(M, P)                                                                    \
  hipLaunchKernelGGL((wide_finish_kernel<M, P>), grid, block, 0, st, B.keys_a, B.idx_a, B.keys_b, \
                     B.idx_b, B.tcnt, B.tabove, B.toff, B.sel, B.info, n, tiles, k, R, want_jvp)
  if (!mag && pc == kP2) TOPK_WIDE_FINISH(false, kP2);
  else if (!mag && pc == kP43) TOPK_WIDE_FINISH(false, kP43);
  else if (mag && pc == kP2) TOPK_WIDE_FINISH(true, kP2);
  else if (mag && pc == kP43) TOPK_WIDE_FINISH(true, kP43);
  else return -1;
#undef TOPK_WIDE_FINISH
  return 0;
}

}  // namespace topk
