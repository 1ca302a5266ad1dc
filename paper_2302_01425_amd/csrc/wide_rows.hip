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
//      whose keys crowd into few buckets take LSD radix passes in LDS.  Longer lists are not
//      sorted at all: their block is found as a set of values (sort_solve.hpp);
//   4. grows the block on the sorted keys (long_solve.hpp);
//   5. adds up the tangent over the block's elements, found by value in the unsorted list
//      (Prop. 7), and writes the row's RowInfo: gamma, d gamma and the block's value window.
#include <hip/hip_runtime.h>

#include "sort_solve.hpp"

namespace topk {
namespace {

constexpr int kWideLdsCap = 16384;             // keys of a list sorted in LDS
constexpr int kSegment = kWideLdsCap / kWT;    // list positions per thread
constexpr int kSlotTile = 4096;                // slot stride of the compaction (radix_sort.hip)

// keys_a / tau_a: the row's dense list (key, tangent of the element in sorted-value coordinates:
// sign(x) t for the magnitude operator); keys_b / pay_b: the tiles' slots with the same payload.
template <bool MAG, int PC>
__global__ __launch_bounds__(kWT) void wide_finish_kernel(
    uint32_t* keys_a, uint32_t* tau_a, uint32_t* keys_b, uint32_t* pay_b,
    const uint32_t* __restrict__ tcnt, const uint32_t* __restrict__ tabove, uint32_t* toff,
    const RowSel* __restrict__ sel, RowInfo* __restrict__ info, int64_t n, int tiles,
    int64_t k_row, Reg R, bool want_jvp, bool dense) {
  using P = Pool<MAG, PC>;
  __shared__ ListShared<kWideLdsCap> sm;
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
  // dense: launches before this one have put the list together in the "a" arrays
  uint64_t carry2 = dense ? (uint64_t(sel[row].cn) | (uint64_t(sel[row].above) << 32)) : 0;
  for (int c0 = 0; c0 < tiles && !dense; c0 += kWT * 4) {
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
  if (in_lds && dense) {
    // ---- 2. the list is there: keys into LDS, the (key, tangent) pairs into registers ------------
    uint32_t key[kSegment], pay[kSegment];
#pragma unroll
    for (int i = 0; i < kSegment; ++i) {
      const uint32_t j = uint32_t(w) * (kSegment * kWave) + uint32_t(i) * kWave + lane;
      key[i] = j < cn ? ka[j] : 0u;
      pay[i] = (j < cn && want_jvp) ? pa[j] : 0u;
    }
#pragma unroll
    for (int i = 0; i < kSegment; ++i) {
      const uint32_t j = uint32_t(w) * (kSegment * kWave) + uint32_t(i) * kWave + lane;
      if (j < cn) sm.keys_a[j] = key[i];
    }
    __syncthreads();
    ri = solve_lds_list<MAG, PC, kWideLdsCap>(cn, k, klo, khi, R, sm);
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
  } else if (in_lds) {
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

    // ---- 3., 4. sort the keys, grow the block -------------------------------------------------------
    ri = solve_lds_list<MAG, PC, kWideLdsCap>(cn, k, klo, khi, R, sm);

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
    // ---- lists too long for LDS (the window holds more than kWideLdsCap elements: a long pooled
    // block).  A wavefront copies sixteen tiles at a time into the row's dense list (their loads in
    // flight together); the list is then solved as it is, without sorting it (sort_solve.hpp) ----
    for (int t0 = w * 16; t0 < tiles && !dense; t0 += kWW * 16) {
      const int tl_l = t0 + (lane & 15);
      const uint32_t c_l = tl_l < tiles ? tc[tl_l] : 0u, o_l = tl_l < tiles ? tf[tl_l] : 0u;
      uint32_t cmax = c_l;
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) cmax = max(cmax, uint32_t(__shfl_xor(cmax, off, kWave)));
      for (uint32_t ch = 0; ch < cmax; ch += kWave) {
        const uint32_t e = ch + lane;
        uint32_t key[16], pay[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const uint32_t c = __shfl(c_l, q, kWave);
          const int64_t src = int64_t(t0 + q) * kSlotTile + e;
          key[q] = e < c ? kb[src] : 0u;
          pay[q] = (e < c && want_jvp) ? pb[src] : 0u;
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const uint32_t c = __shfl(c_l, q, kWave), o = __shfl(o_l, q, kWave);
          if (e < c) {
            ka[o + e] = key[q];
            if (want_jvp) pa[o + e] = pay[q];
          }
        }
      }
    }
    __syncthreads();
    ri = solve_unsorted_list<MAG, PC, kWideLdsCap>(ka, pa, cn, k, klo, khi, R, want_jvp, sm);
  }
  if (threadIdx.x == 0) info[row] = ri;
}

}  // namespace

// dense: the selection has also gathered the rows' lists (second level: launch_wide_select with
// refine)
int launch_wide_finish(bool mag, int pc, const SortBuffers& B, bool want_jvp, bool dense,
                       int64_t rows, int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  if (rows > 0x7fffffffLL) return -1;
  const dim3 grid{unsigned(rows)}, block{kWT};
  const int tiles = radix_tiles(n);
#define TOPK_WIDE_FINISH(M, P)                                                                    \
  hipLaunchKernelGGL((wide_finish_kernel<M, P>), grid, block, 0, st, B.keys_a, B.idx_a, B.keys_b, \
                     B.idx_b, B.tcnt, B.tabove, B.toff, B.sel, B.info, n, tiles, k, R, want_jvp,   \
                     dense)
  if (!mag && pc == kP2) TOPK_WIDE_FINISH(false, kP2);
  else if (!mag && pc == kP43) TOPK_WIDE_FINISH(false, kP43);
  else if (mag && pc == kP2) TOPK_WIDE_FINISH(true, kP2);
  else if (mag && pc == kP43) TOPK_WIDE_FINISH(true, kP43);
  else return -1;
#undef TOPK_WIDE_FINISH
  return 0;
}

}  // namespace topk
