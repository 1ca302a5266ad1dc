// Sort and solve of one row's candidate list by one workgroup of 1024 threads, shared by the wide
// route (wide_rows.hip) and the one-launch kernel of medium rows.
//
//   * keys-only sort of a list in LDS: one bucket pass (bucket = leading bits of key - klo, about
//     two keys per bucket; LDS atomics hand out the places inside a bucket, a count of the smaller
//     keys of the bucket orders them); LSD radix passes (in LDS or through global buffers) for
//     lists whose keys crowd into few buckets and for lists that do not fit;
//   * block growth on prefix sums of the sorted list (see wide_solve).
// The outputs are computed from values (thresholds), so no permutation is needed and equal keys
// may come in any order.
#pragma once

#include <hip/hip_runtime.h>

#include "common.hpp"
#include "launch.hpp"
#include "long_solve.hpp"
#include "pooling.hpp"
#include "radix.hpp"

namespace topk {

constexpr int kWT = 1024;                      // threads
constexpr int kWW = kWT / kWave;               // wavefronts
constexpr int kWideBuckets = 8192;             // buckets of the one-pass sort
constexpr int kBucketMax = 32;                 // longest bucket the one-pass sort orders by counting

// CAP: keys of a list that is sorted and solved in LDS (a multiple of 16 * 1024 / 2).
template <int CAP>
struct ListShared {
  static constexpr int kCap = CAP;
  uint32_t keys_a[CAP];                // the list's keys; the sorted keys end here
  uint32_t keys_b[CAP];                // tile offsets during the gather, then sort buffer
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
  // solve of an unsorted list (solve_unsorted_list)
  uint32_t red[4][kWW];
  struct {
    uint32_t bin, below;
  } pick;
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
template <int ITEMS, int CAP>
__device__ __forceinline__ void wide_radix_pass(const uint32_t* kin, uint32_t* kout, uint32_t cn,
                                                uint32_t klo, int shift, int ni, ListShared<CAP>& sm) {
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
template <int ITEMS, int CAP>
__device__ __forceinline__ const uint32_t* wide_radix_sort(const uint32_t* src, uint32_t* b0,
                                                           uint32_t* b1, uint32_t cn, uint32_t klo,
                                                           int nbits, ListShared<CAP>& sm) {
  int ni = int((cn + kWT - 1) / kWT);
  ni = ni > ITEMS ? ITEMS : ni;
  const uint32_t* cur = src;
  bool even = true;
  for (int shift = 0; shift < nbits; shift += 8) {
    uint32_t* kout = even ? b0 : b1;
    wide_radix_pass<ITEMS, CAP>(cur, kout, cn, klo, shift, ni, sm);
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

// One bucket pass over the cn <= CAP keys in sm.keys_a; the sorted keys end in
// sm.keys_a.  Returns false (keys_a untouched) when some bucket is too long to be ordered by
// counting.
template <int CAP>
__device__ __forceinline__ bool wide_bucket_sort(uint32_t cn, uint32_t klo, int nbits,
                                                 ListShared<CAP>& sm) {
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
// The sorted positions are cut into segments of kSegment = CAP / 1024 positions (8 or 16).  All
// threads first compute, once, the power sums of everything before each segment (one workgroup
// scan; kept in LDS).  The growth itself is left to the first wavefront, which needs no barriers:
// with the block [a, b] and the prefix sums up to a - 1 and b in registers, a round is
//   A. lane l tests, for its segments l, l + 64, ..., the FIRST position of a segment right of
//      the block as if everything between the block and it had joined (sums = the segment's prefix
//      minus the prefix up to a - 1), and the LAST position of a segment left of the block: the
//      strict tests of the PAV loop (pooling.hpp), which are monotone along each side, so the
//      first failing segment bounds the run of positions that join;
//   B. the segment that holds the end of each run is settled by 16 lanes, one position each
//      (prefix sums inside the segment by a DPP scan); the new end of the block and its prefix
//      sum are broadcast from the lane that holds them.
// Both sides advance in the same round (additions on one side only make the other side's tests
// more true); the growth ends with a round that changes nothing.
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

template <bool CUBIC>
__device__ __forceinline__ Sums readlane_sums(const Sums& v, int src_lane) {
  return Sums{readlane_f64(v.s1, src_lane), CUBIC ? readlane_f64(v.s2, src_lane) : 0.0,
              CUBIC ? readlane_f64(v.s3, src_lane) : 0.0};
}

// One position per lane of 16 consecutive positions starting with segment `seg` (the 16 lanes of
// one DPP row): its 1-based position p, centred value d (0 beyond the list) and the prefix sums
// up to p - 1 and up to p.
template <bool CUBIC, int kSegment>
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

template <bool MAG, int PC, int CAP>
__device__ RowInfo wide_solve(const uint32_t* keys, uint32_t cn_u, int64_t k64, const Reg& R,
                              ListShared<CAP>& sm) {
  using P = Pool<MAG, PC>;
  constexpr bool CUBIC = (PC == kP43);
  constexpr int kSegment = CAP / kWT;          // positions per segment: 8 or 16
  static_assert(kSegment == 8 || kSegment == 16, "a segment fits one DPP row");
  static_assert(sizeof(Sums) * (kWT + 1) <= sizeof(uint32_t) * CAP, "segment prefixes fit keys_b");
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
  // ---- prefix sums of all segments: seg_pre[s] = sums of the positions before segment s --------
  Sums* seg_pre = reinterpret_cast<Sums*>(sm.keys_b);      // [kWT + 1], the sort is over
  {
    const int q0 = kSegment * t + 1;
    Sums tot{0.0, 0.0, 0.0};
    if (q0 <= cn) {                             // (wavefronts beyond the list skip this)
#pragma unroll
      for (int i = 0; i < kSegment; ++i) {
        const int p = q0 + i;
        const double d = p <= cn ? double(key_to_float(keys[p <= cn ? p - 1 : 0])) - center : 0.0;
        tot.s1 += d;
        if (CUBIC) {
          tot.s2 += d * d;
          tot.s3 += d * d * d;
        }
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
    seg_pre[t] = sums_sub(inc, tot);
    if (t == kWT - 1) seg_pre[kWT] = inc;
  }
  __syncthreads();

  // ---- the growth, by the first wavefront -----------------------------------------------------------
  if (w == 0) {
    const int nseg = (cn + kSegment - 1) / kSegment;       // segments that hold positions
    const int i16 = lane & 15, rowid = lane >> 4;
    int a = k, b = k + 1;
    Sums pa1, pb;
    {
      // the seed block (k, k+1): prefix sums up to k + 1 (row 0) and k - 1 (row 1)
      const int target = rowid == 0 ? k + 1 : k - 1;
      int p;
      double d;
      Sums ex, in;
      segment_lanes<CUBIC, kSegment>(keys, seg_pre, target >= 1 ? (target - 1) / kSegment : 0, cn,
                                     center, i16, &p, &d, &ex, &in);
      // position k + 1 sits in lane (k % kSegment) of row 0, position k - 1 (k >= 2) in lane
      // 16 + (k - 2) % kSegment of row 1
      pb = readlane_sums<CUBIC>(in, k % kSegment);
      pa1 = readlane_sums<CUBIC>(in, 16 + (k >= 2 ? (k - 2) % kSegment : 0));
      if (k == 1) pa1 = Sums{0.0, 0.0, 0.0};
    }
    for (int round = 0; round <= cn; ++round) {
      const double m = double(k - a + 1);
      // ---- A: segment tests ------------------------------------------------------------------------
      // right: first segment starting beyond b whose first position does not join (or lies beyond
      // the list); the segments are visited 64 at a time, away from the block
      int first_fail_r = nseg;
      for (int s0 = b / kSegment; s0 < nseg; s0 += kWave) {   // segment of position b + 1 is b / kSegment
        const int sg = s0 + lane;
        const int q0 = kSegment * sg + 1;
        bool fail = false;
        if (q0 > b) {
          fail = true;
          if (sg < nseg) {
            const double d0 = double(key_to_float(keys[q0 - 1])) - center;
            fail = !P::right_violates(d0, double(q0 - a), m, sums_sub(seg_pre[sg], pa1), R, center);
          }
        }
        const unsigned long long bal = __ballot(fail);
        if (bal != 0ull) {
          first_fail_r = s0 + (__ffsll((long long)bal) - 1);
          break;
        }
      }
      // left: last segment ending before a whose last position does not join; visited 64 at a
      // time, away from the block
      int last_fail_l = -1;
      for (int s1 = (a - 2) / kSegment; s1 >= 0 && a >= 2; s1 -= kWave) {   // segment of position a - 1
        const int sg = s1 - lane;
        const int e = kSegment * sg + kSegment;              // last position of the segment
        bool fail = false;
        if (sg >= 0 && e < a) {
          const double de = double(key_to_float(keys[e - 1])) - center;
          fail = !P::left_violates(de, double(b - e), double(k - e), sums_sub(pb, seg_pre[sg + 1]), R,
                                   center);
        }
        const unsigned long long bal = __ballot(fail);
        if (bal != 0ull) {
          last_fail_l = s1 - (__ffsll((long long)bal) - 1);  // lowest lane = highest segment
          break;
        }
      }
      // ---- B: the two segments that hold the ends of the runs, one position per lane -----------
      const int seg = rowid == 0 ? first_fail_r - 1 : last_fail_l + 1;
      int p;
      double d;
      Sums ex, in;
      segment_lanes<CUBIC, kSegment>(keys, seg_pre, seg, cn, center, i16, &p, &d, &ex, &in);
      // right (row 0): position p joins the block [a, p - 1]; positions up to b are in already
      const bool pass_r = p <= b || (p <= cn && P::right_violates(d, double(p - a), m,
                                                                  sums_sub(ex, pa1), R, center));
      // left (row 1): position p joins the block [p + 1, b]; positions from a on are in already
      const bool pass_l = p >= a || P::left_violates(d, double(b - p), double(k - p),
                                                     sums_sub(pb, in), R, center);
      const unsigned long long ball_r = __ballot(pass_r), ball_l = __ballot(pass_l);
      int na, nb;
      Sums npa1, npb;
      {
        const uint32_t fails = ~uint32_t(ball_r) & 0xffffu;              // row 0 = lanes 0..15
        const int f = fails ? __ffs(int(fails)) - 1 : 16;                // first failing lane
        // the run ends at lane f - 1 (f = 0: at the end of the segment before)
        const int src = f >= 1 ? f - 1 : 0;
        nb = __builtin_amdgcn_readlane(p, src) - (f >= 1 ? 0 : 1);
        npb = f >= 1 ? readlane_sums<CUBIC>(in, src) : readlane_sums<CUBIC>(ex, src);
      }
      {
        const uint32_t fails = ~uint32_t(ball_l >> 16) & 0xffffu;        // row 1 = lanes 16..31
        const int f = fails ? 31 - __clz(int(fails)) : -1;               // last failing lane
        // the run (downwards) ends at lane f + 1 (f = 15: at the start of the segment after)
        const int src = 16 + (f >= 0 ? f : 0);
        na = __builtin_amdgcn_readlane(p, src) + (f >= 0 ? 1 : 0);
        npa1 = f >= 0 ? readlane_sums<CUBIC>(in, src) : readlane_sums<CUBIC>(ex, src);
      }
      const bool same = (na == a) && (nb == b);
      a = na;
      b = nb;
      pa1 = npa1;
      pb = npb;
      if (same) break;
    }
    if (lane == 0) {
      sm.grow.a = a;
      sm.grow.b = b;
      sm.grow.pa1 = pa1;
      sm.grow.pb = pb;
    }
  }
  __syncthreads();
  const int a = sm.grow.a, b = sm.grow.b;
  const Sums S = sums_sub(sm.grow.pb, sm.grow.pa1);
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
template <int CAP>
__device__ __forceinline__ void wide_sum2(double& x, double& y, ListShared<CAP>& sm) {
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



// d gamma (Prop. 7) from the row's unsorted list in global memory (keys, tangent bits): the
// block's elements are those whose value lies in [lo_incl, hi_incl].
template <bool MAG, int PC, int CAP>
__device__ __forceinline__ double list_dgamma(const uint32_t* ka, const uint32_t* pa, uint32_t cn,
                                              const RowInfo& ri, int64_t k, const Reg& R,
                                              ListShared<CAP>& sm) {
  using P = Pool<MAG, PC>;
  double num = 0.0, den = 0.0;
  for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 4 * kWT) {
    uint32_t key[4], pay[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t j = j0 + uint32_t(i) * kWT;
      key[i] = j < cn ? ka[j] : 0u;
      pay[i] = j < cn ? pa[j] : 0u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float sv = key_to_float(key[i]);
      if (j0 + uint32_t(i) * kWT < cn && sv >= ri.lo_incl && sv <= ri.hi_incl) {
        const double wgt = P::jac_weight(double(sv) - ri.center, ri.gamma);
        num += wgt * double(__uint_as_float(pay[i]));
        den += wgt;
      }
    }
  }
  wide_sum2(num, den, sm);
  return num / P::jac_denominator(den, double(k - ri.a + 1), R);
}

// ---- lists that do not fit the LDS buffers: solved WITHOUT sorting them ---------------------------
// The block is a set of values: with gamma its pooled value, a candidate above s_k belongs to it
// iff its singleton minimiser lies below gamma, one below s_{k+1} iff its value lies above gamma
// (the tests of the growth, which hold for every member of the final block and fail for every
// non-member, all values being compared with the same gamma), and everything from s_{k+1} to s_k
// belongs to it.  gamma is therefore the root of the non-increasing function
//     Psi(g) = #above(g) + sum over the set at g of grad r*(s - g) - k,
// found by solving one piece after the other: classify the list at g (one pass: counts, sums and
// extreme values of the set), take the pooled value g' of that set - the root of the piece of Psi
// that g lies on - and classify again at g'; when the set does not change, g' is the root.  A
// bracket [lo, hi] from the signs seen so far (g' > g means Psi(g) > 0) guards the iteration.
// s_k and s_{k+1} come from a radix selection on the keys (11 bits per pass).

// key of rank r (1-based) in ascending key order among list[0, cn); also the number of keys
// below it and the number equal to it
template <int CAP>
__device__ uint32_t list_select(const uint32_t* list, uint32_t cn, uint32_t klo, int nbits,
                                uint32_t rank, uint32_t* below_out, uint32_t* equal_out,
                                ListShared<CAP>& sm) {
  uint32_t prefix = 0, pmask = 0, r = rank - 1, equal = cn;   // r: 0-based rank among the matches
  for (int top = nbits; top > 0;) {
    const int width = top < 11 ? top : 11;
    const int shift = top - width;
    const uint32_t bins = 1u << width;
    uint32_t* hist = sm.u.bucket;
    for (uint32_t i = threadIdx.x; i < bins; i += kWT) hist[i] = 0;
    __syncthreads();
    for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 8 * kWT) {     // eight loads in flight
      uint32_t key[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) key[i] = j0 + uint32_t(i) * kWT < cn ? list[j0 + uint32_t(i) * kWT] : 0u;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t u = key[i] - klo;
        if (j0 + uint32_t(i) * kWT < cn && (u & pmask) == prefix)
          atomicAdd(&hist[(u >> shift) & (bins - 1u)], 1u);
      }
    }
    __syncthreads();
    const uint32_t b0 = 2u * threadIdx.x, b1 = b0 + 1u;       // two bins per thread (2048 at most)
    const uint32_t c0 = b0 < bins ? hist[b0] : 0u, c1 = b1 < bins ? hist[b1] : 0u;
    const uint32_t ex = wide_exclusive_scan(c0 + c1, sm.wave_tot, nullptr);
    if (r >= ex && r < ex + c0) sm.pick = {b0, ex};
    else if (r >= ex + c0 && r < ex + c0 + c1) sm.pick = {b1, ex + c0};
    __syncthreads();
    const uint32_t bin = sm.pick.bin;
    r -= sm.pick.below;
    equal = hist[bin];
    prefix |= bin << shift;
    pmask |= (bins - 1u) << shift;
    top = shift;
    __syncthreads();
  }
  *below_out = rank - 1 - r;
  *equal_out = equal;
  return klo + prefix;
}

struct SetStats {
  uint32_t above, cnt;       // candidates above the set, members of the set
  uint32_t kmin, kmax;       // smallest / largest key of the set (its largest / smallest value)
  Sums S;                    // power sums of the members' centred values
};

// smallest key whose value is strictly below T / largest key whose value is strictly above T
// (keys run against values; key + 1 is the next smaller value)
__device__ __forceinline__ uint32_t first_key_below(double T) {
  const float f = __double2float_rn(T);
  return desc_key(f) + (double(f) >= T ? 1u : 0u);
}
__device__ __forceinline__ uint32_t last_key_above(double T) {
  const float f = __double2float_rn(T);
  return desc_key(f) - (double(f) <= T ? 1u : 0u);
}

// One pass over the list: the set at the pooled value g (centred).  Membership is a value
// interval: a candidate above s_k is in iff its singleton minimiser lies below g, i.e. its value
// below T_hi(g) = g + lambda (mask), g (1 + lambda) (magnitude, p = 2), g + lambda g^(1/3)
// (magnitude, p = 4/3: where the one-element cubic at g changes sign); one below s_{k+1} iff its
// value lies above g; the values from s_{k+1} to s_k (keys kk .. kk1) always.
template <bool MAG, int PC, int CAP>
__device__ SetStats list_classify(const uint32_t* list, uint32_t cn, uint32_t kk, uint32_t kk1,
                                  double g, double center, const Reg& R, ListShared<CAP>& sm) {
  constexpr bool CUBIC = (PC == kP43);
  const double g_abs = g + center;
  double t_hi;
  if (MAG && CUBIC) t_hi = g_abs + R.lambda * cbrt(fmax(g_abs, 0.0));
  else if (MAG) t_hi = g_abs * R.one_p_lambda;
  else t_hi = g_abs + R.lambda;
  const uint32_t k_first = min(first_key_below(t_hi), kk);      // members: k_first <= key <= k_last
  const uint32_t k_last = max(last_key_above(g_abs), kk1);
  uint32_t above = 0, cnt = 0, kmin = 0xffffffffu, kmax = 0u;
  Sums S{0.0, 0.0, 0.0};
  for (uint32_t j0 = threadIdx.x; j0 < cn; j0 += 8 * kWT) {     // eight loads in flight
    uint32_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      key[i] = j0 + uint32_t(i) * kWT < cn ? list[j0 + uint32_t(i) * kWT] : 0xffffffffu;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bool real = j0 + uint32_t(i) * kWT < cn;
      const bool in = real && key[i] >= k_first && key[i] <= k_last;
      above += (real && key[i] < k_first) ? 1u : 0u;
      if (in) {
        ++cnt;
        kmin = min(kmin, key[i]);
        kmax = max(kmax, key[i]);
        const double d = double(key_to_float(key[i])) - center;
        S.s1 += d;
        if (CUBIC) { S.s2 += d * d; S.s3 += d * d * d; }
      }
    }
  }
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
#pragma unroll
  for (int off = kWave >> 1; off >= 1; off >>= 1) {
    above += __shfl_xor(above, off, kWave);
    cnt += __shfl_xor(cnt, off, kWave);
    kmin = min(kmin, uint32_t(__shfl_xor(kmin, off, kWave)));
    kmax = max(kmax, uint32_t(__shfl_xor(kmax, off, kWave)));
    S.s1 += __shfl_xor(S.s1, off, kWave);
    if (CUBIC) { S.s2 += __shfl_xor(S.s2, off, kWave); S.s3 += __shfl_xor(S.s3, off, kWave); }
  }
  __syncthreads();
  if (lane == 0) {
    sm.red[0][w] = above;
    sm.red[1][w] = cnt;
    sm.red[2][w] = kmin;
    sm.red[3][w] = kmax;
    sm.wave_sums[w] = S;
  }
  __syncthreads();
  SetStats st{0u, 0u, 0xffffffffu, 0u, Sums{0.0, 0.0, 0.0}};
#pragma unroll
  for (int q = 0; q < kWW; ++q) {
    st.above += sm.red[0][q];
    st.cnt += sm.red[1][q];
    st.kmin = min(st.kmin, sm.red[2][q]);
    st.kmax = max(st.kmax, sm.red[3][q]);
    st.S.s1 += sm.wave_sums[q].s1;
    if (CUBIC) { st.S.s2 += sm.wave_sums[q].s2; st.S.s3 += sm.wave_sums[q].s3; }
  }
  return st;
}

// The row's unsorted candidate list (keys ka, tangent payload pa) -> RowInfo in list coordinates.
template <bool MAG, int PC, int CAP>
__device__ RowInfo solve_unsorted_list(const uint32_t* ka, const uint32_t* pa, uint32_t cn,
                                       int64_t k64, uint32_t klo, uint32_t khi, const Reg& R,
                                       bool want_jvp, ListShared<CAP>& sm) {
  using P = Pool<MAG, PC>;
  const int64_t k = k64;
  RowInfo ri;
  ri.src = 0;
  ri.pad = 0;
  ri.a = k64 + 1;
  ri.b = k64;
  ri.wa = ri.a;
  ri.wb = ri.b;
  ri.gamma = ri.center = ri.dgamma = 0.0;
  if (!(k >= 1 && k < int64_t(cn))) {           // k == 0: everything is below; k == cn: above
    ri.hi_incl = (k <= 0) ? __uint_as_float(0x7f800000u) : __uint_as_float(0xff800000u);
    ri.lo_incl = ri.hi_incl;
    return ri;
  }
  const uint32_t span = khi - klo;
  const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
  // s_k and s_{k+1}: the keys of ranks k and k + 1
  uint32_t below, equal;
  const uint32_t kk = list_select<CAP>(ka, cn, klo, nbits, uint32_t(k), &below, &equal, sm);
  uint32_t kk1 = kk;
  if (uint32_t(k) + 1u > below + equal) {       // rank k + 1 is the next larger key
    uint32_t nk = 0xffffffffu;
    for (uint32_t j = threadIdx.x; j < cn; j += kWT) {
      const uint32_t key = ka[j];
      if (key > kk) nk = min(nk, key);
    }
#pragma unroll
    for (int off = kWave >> 1; off >= 1; off >>= 1) nk = min(nk, uint32_t(__shfl_xor(nk, off, kWave)));
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) sm.red[0][threadIdx.x / kWave] = nk;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kWW; ++q) nk = min(nk, sm.red[0][q]);
    kk1 = nk;
  }
  const float fk = key_to_float(kk), fk1 = key_to_float(kk1);
  const double center = P::kCentered ? double(fk) : 0.0;
  ri.center = center;
  if (!P::seed_violates(double(fk) - center, double(fk1) - center, R, center)) {
    ri.hi_incl = fk1;                           // s_{k+1} < s_k: "above hi" = the top k
    ri.lo_incl = fk;
    return ri;
  }
  auto pooled_of = [&](const SetStats& st) {
    const double da = double(key_to_float(st.kmin)) - center, db = double(key_to_float(st.kmax)) - center;
    // bracket of the cubic's root, valid for any set: at its largest value every term is >= 0;
    // one lambda below its smallest value the sum is <= lambda^3 (m - cnt) <= 0 (magnitude: at 0)
    return P::pooled(double(st.cnt), double(k - int64_t(st.above)), st.S, R,
                     MAG ? -center : db - R.lambda, da, center);
  };
  // start: the pooled value of the pair (s_k, s_{k+1}) alone
  const double dk = double(fk) - center, dk1 = double(fk1) - center;
  Sums S2{dk + dk1, dk * dk + dk1 * dk1, dk * dk * dk + dk1 * dk1 * dk1};
  double g = P::pooled(2.0, 1.0, S2, R, MAG ? -center : dk1 - R.lambda, dk, center);
  SetStats st{0xffffffffu, 0xffffffffu, 0u, 0u, Sums{0.0, 0.0, 0.0}};
  double lo = -1e300, hi = 1e300;
  bool from_piece = false;                      // g is the root of the piece classified last
  for (int it = 0; it < 200; ++it) {
    const SetStats nx = list_classify<MAG, PC, CAP>(ka, cn, kk, kk1, g, center, R, sm);
    const bool same = nx.above == st.above && nx.cnt == st.cnt;
    st = nx;
    if (same && from_piece) break;              // the set at its own pooled value: done
    const double g2 = pooled_of(st);
    if (g2 == g) break;                         // g is the root of the piece it lies on
    if (g2 > g) lo = g; else hi = g;
    from_piece = g2 > lo && g2 < hi;
    g = from_piece ? g2 : 0.5 * (lo + hi);
  }
  ri.a = int64_t(st.above) + 1;
  ri.b = int64_t(st.above) + int64_t(st.cnt);
  ri.wa = ri.a;
  ri.wb = ri.b;
  ri.gamma = g;
  ri.hi_incl = key_to_float(st.kmin);
  ri.lo_incl = key_to_float(st.kmax);
  if (want_jvp) ri.dgamma = list_dgamma<MAG, PC, CAP>(ka, pa, cn, ri, k, R, sm);
  return ri;
}

// A list of cn <= CAP keys in sm.keys_a: sort and block growth in LDS (d gamma is the caller's).
template <bool MAG, int PC, int CAP>
__device__ RowInfo solve_lds_list(uint32_t cn, int64_t k, uint32_t klo, uint32_t khi, const Reg& R,
                                  ListShared<CAP>& sm) {
  const uint32_t span = khi - klo;
  const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
  const uint32_t* skeys = sm.keys_a;
  if (nbits > 0 && !wide_bucket_sort<CAP>(cn, klo, nbits, sm)) {
    skeys = wide_radix_sort<8, CAP>(sm.keys_a, sm.keys_b, sm.keys_a, cn, klo, nbits, sm);
    if (skeys != sm.keys_a) {                  // the solve uses keys_b for its own tables
      for (uint32_t j = threadIdx.x; j < cn; j += kWT) sm.keys_a[j] = sm.keys_b[j];
      __syncthreads();
      skeys = sm.keys_a;
    }
  }
  return wide_solve<MAG, PC, CAP>(skeys, cn, k, R, sm);
}

}  // namespace topk
