// Medium rows (1024 < n <= 131072): the whole operator for one row in ONE workgroup of 1024
// threads, one launch.
//
//   1. histogram of the leading key bits of the row (LDS atomics; bin = LDS word, so that
//      neighbouring bins, the ones a wavefront hits together, lie in different banks)
//   2. the bins of sorted positions k and k+1 give the key window that holds every element able
//      to pool (radix.hpp: key_window)
//   3. ordered compaction of those candidates (key, index payload) into the row's scratch
//   4. stable LSD radix sort of the candidates on (key - klo), 8 bits per pass, only as many
//      passes as the window has significant bits; the candidates come in index order, so equal
//      values keep ascending index
//   5. isotonic solve on the sorted candidates (long_solve.hpp)
//   6. dense pass over the row for everything outside the block's value window, and the window's
//      positions through sigma
//
// Steps 3..5 go through global scratch that only this workgroup touches (L2-resident at these
// sizes); the row itself is read three times, the second and third time from L2.
#include <hip/hip_runtime.h>

#include "common.hpp"
#include "launch.hpp"
#include "long_solve.hpp"
#include "pooling.hpp"
#include "radix.hpp"

namespace topk {
namespace {

// Workgroups of NT = 1024 threads for long rows; of 256 threads for rows up to kSmallRowMax
// elements, where the per-row latency is what counts and four times as many rows are in flight.
constexpr int kSmallRowMax = 8192;
constexpr int kMItems = 8;                 // elements per thread and tile of a sorting pass
constexpr int kCItems = 16;                // elements per thread and tile of the compaction
constexpr int kSelShift = 32 - kSelBits;

template <int NT>
struct MedCfg {
  static constexpr int kMW = NT / kWave;                     // wavefronts
  static constexpr int kCTile = NT * kCItems;
  static constexpr int kLdsCap = NT >= 1024 ? 2048 : 1024;   // lists up to this length are sorted in LDS
  // words of the union below: the selection histogram, later the sorted keys of a list for the solve
  static constexpr int kLdsKeys = NT >= 1024 ? 16384 : kSelBins;
};

template <int NT>
struct MedShared {
  using C = MedCfg<NT>;
  union {
    uint32_t hist[C::kLdsKeys];            // steps 1-2: kSelBins counters; later sorted keys
    struct {
      uint32_t cnt[C::kMW][kRadix];        // per-wave digit counts, then per-wave offsets
      uint32_t base[kRadix];               // running start of every digit in the output
      uint32_t gofs[kRadix];               // start of the current tile's items of every digit
      uint32_t lk[2][C::kLdsCap];          // short candidate lists: keys, ping-pong
      uint32_t li[2][C::kLdsCap];          //                        index payloads
    } sort;                                // steps 3-6
  } u;
  SolveShared<NT> solve;
  uint32_t wave_a[C::kMW], wave_b[C::kMW];
  uint32_t found[2];
};

// exclusive scan of one value per thread over the workgroup; *total gets the sum
template <int NT>
__device__ __forceinline__ uint32_t med_exclusive_scan(uint32_t v, uint32_t* wave_tot,
                                                       uint32_t* total) {
  constexpr int kMW = NT / kWave;
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
  for (int q = 0; q < kMW; ++q) {
    const uint32_t t = wave_tot[q];
    if (q < w) before += t;
    all += t;
  }
  if (total) *total = all;
  return before + inc - v;
}

// One LSD pass over the cn candidates: (kin, iin) -> (kout, iout), stable, by the 8-bit digit of
// (key - klo) at `shift`.  Tiles of ni*1024 elements; wave w owns elements w*ni*64 .. of a tile.
template <int NT, int ITEMS>
__device__ __forceinline__ void med_sort_pass(const uint32_t* kin, const uint32_t* iin, uint32_t* kout,
                              uint32_t* iout, uint32_t cn, uint32_t klo, int shift, int ni,
                              MedShared<NT>& sm) {
  constexpr int kMT = NT, kMW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const uint32_t tile_elems = uint32_t(ni) * kMT;
  const uint32_t wave_elems = uint32_t(ni) * kWave;
  // several tiles: digit totals of the whole list first -> start of every digit (a single tile
  // gets them from its own ranking below)
  const bool single = cn <= tile_elems;
  if (!single) {
    for (int i = threadIdx.x; i < kMW * kRadix; i += kMT) (&sm.u.sort.cnt[0][0])[i] = 0;
    __syncthreads();
    for (uint32_t tile_first = 0; tile_first < cn; tile_first += tile_elems) {
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        if (i < ni) {
          const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
          const bool valid = e < cn;
          const uint32_t key = valid ? kin[e] : 0u;
          count_digit(sm.u.sort.cnt[w], ((key - klo) >> shift) & (kRadix - 1), valid, lane);
        }
      }
    }
    __syncthreads();
    uint32_t tot = 0;
    if (threadIdx.x < kRadix) {
#pragma unroll
      for (int q = 0; q < kMW; ++q) tot += sm.u.sort.cnt[q][threadIdx.x];
    }
    const uint32_t ex = med_exclusive_scan<NT>(tot, sm.wave_a, nullptr);
    if (threadIdx.x < kRadix) sm.u.sort.base[threadIdx.x] = ex;
  }
  // tile by tile: rank inside the wavefront, offsets of the wavefronts, scatter
  for (uint32_t tile_first = 0; tile_first < cn; tile_first += tile_elems) {
    __syncthreads();                       // previous users of cnt / gofs are done
    for (int i = threadIdx.x; i < kMW * kRadix; i += kMT) (&sm.u.sort.cnt[0][0])[i] = 0;
    __syncthreads();
    uint32_t key[ITEMS], idx[ITEMS], rank[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i < ni) {
        const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
        const bool valid = e < cn;
        key[i] = valid ? kin[e] : 0u;
        idx[i] = valid ? iin[e] : 0u;
        const uint32_t d = ((key[i] - klo) >> shift) & (kRadix - 1);
        const unsigned long long peers = match_digit(d, __ballot(valid));
        const unsigned long long lower = peers & lanemask_lt();
        uint32_t pre = 0;
        if (valid) {
          pre = sm.u.sort.cnt[w][d];
          if (lower == 0) sm.u.sort.cnt[w][d] = pre + __popcll(peers);
        }
        rank[i] = pre + __popcll(lower);
      }
    }
    __syncthreads();
    uint32_t run = 0;
    if (threadIdx.x < kRadix) {
#pragma unroll
      for (int q = 0; q < kMW; ++q) {
        const uint32_t c = sm.u.sort.cnt[q][threadIdx.x];
        sm.u.sort.cnt[q][threadIdx.x] = run;
        run += c;
      }
    }
    if (single) {
      const uint32_t ex = med_exclusive_scan<NT>(run, sm.wave_a, nullptr);
      if (threadIdx.x < kRadix) sm.u.sort.gofs[threadIdx.x] = ex;
    } else if (threadIdx.x < kRadix) {
      const uint32_t b = sm.u.sort.base[threadIdx.x];
      sm.u.sort.gofs[threadIdx.x] = b;
      sm.u.sort.base[threadIdx.x] = b + run;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i < ni) {
        const uint32_t e = tile_first + w * wave_elems + i * kWave + lane;
        if (e < cn) {
          const uint32_t d = ((key[i] - klo) >> shift) & (kRadix - 1);
          const uint32_t dst = sm.u.sort.gofs[d] + sm.u.sort.cnt[w][d] + rank[i];
          kout[dst] = key[i];
          iout[dst] = idx[i];
        }
      }
    }
  }
  __syncthreads();          // workgroup-scope release/acquire: the next pass reads what this one wrote
}

// Where sort_candidates left the sorted list.
struct SortedList {
  const uint32_t* keys;   // LDS or global
  const uint32_t* idx;    // LDS or global
  int global_src;         // global copy of (keys, idx): 0 = (ka, ia), 1 = (kb, ib), -1 = none yet
  bool keys_in_lds;
};

// Stable LSD sort of the cn candidates in (ka, ia) on key - klo, one pass per 8 significant bits
// of khi - klo.  The passes alternate between two buffers: in LDS for short lists, else (kb, ib)
// and (ka, ia).
template <int NT, int ITEMS>
__device__ __forceinline__ SortedList sort_candidates(uint32_t* ka, uint32_t* ia, uint32_t* kb, uint32_t* ib,
                                      uint32_t cn, uint32_t klo, uint32_t khi, MedShared<NT>& sm) {
  constexpr int kMT = NT, kLdsCap = MedCfg<NT>::kLdsCap;
  const uint32_t span = khi - klo;
  const int nbits = span == 0 ? 0 : 32 - __clz(int(span));
  int ni = int((cn + kMT - 1) / kMT);
  ni = ni > ITEMS ? ITEMS : ni;
  if (nbits == 0) return SortedList{ka, ia, 0, false};
  const bool in_lds = cn <= uint32_t(kLdsCap);
  uint32_t* k0 = in_lds ? sm.u.sort.lk[0] : kb;
  uint32_t* i0 = in_lds ? sm.u.sort.li[0] : ib;
  uint32_t* k1 = in_lds ? sm.u.sort.lk[1] : ka;
  uint32_t* i1 = in_lds ? sm.u.sort.li[1] : ia;
  const uint32_t* kin = ka;
  const uint32_t* iin = ia;
  bool even = true;
  for (int shift = 0; shift < nbits; shift += 8) {
    uint32_t* kout = even ? k0 : k1;
    uint32_t* iout = even ? i0 : i1;
    med_sort_pass<NT, ITEMS>(kin, iin, kout, iout, cn, klo, shift, ni, sm);
    kin = kout;
    iin = iout;
    even = !even;
  }
  if (in_lds) return SortedList{kin, iin, -1, true};
  return SortedList{kin, iin, even ? 0 : 1, false};    // even: an even number of passes was made
}

// SPARSE (mask only): instead of the dense outputs the row's non-zeros are written as (index,
// value) lists: first the elements above the key window (value exactly 1) in ascending index
// order, then the candidates' non-zeros in descending order of theta.
template <bool MAG, int PC, int NT, bool SPARSE = false>
__global__ __launch_bounds__(NT) void medium_rows_kernel(
    const float* __restrict__ x_all, const float* __restrict__ tangent_all,
    float* __restrict__ out_all, float* __restrict__ jvp_all, uint32_t* keys_a, uint32_t* idx_a,
    uint32_t* keys_b, uint32_t* idx_b, int n, int k_row, Reg R, SparseOut sp) {
  constexpr int kMT = NT, kMW = NT / kWave, kCTile = MedCfg<NT>::kCTile;
  __shared__ MedShared<NT> sm;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int64_t base = int64_t(blockIdx.x) * n;
  const float* x = x_all + base;
  const float* tangent = tangent_all != nullptr ? tangent_all + base : nullptr;
  float* out = out_all != nullptr ? out_all + base : nullptr;
  float* jvp = jvp_all != nullptr ? jvp_all + base : nullptr;
  uint32_t* ka = keys_a + base;
  uint32_t* ia = idx_a + base;
  uint32_t* kb = keys_b + base;
  uint32_t* ib = idx_b + base;

  uint32_t cn = 0;
  uint32_t above_total = 0;              // elements of the row above the key window
  int k = k_row;
  const uint32_t* skeys = ka;
  const uint32_t* sidx = ia;
  if (k_row >= 1 && k_row < n) {
    // ---- 1. histogram of the leading key bits ---------------------------------------------------
    for (int i = threadIdx.x; i < kSelBins; i += kMT) sm.u.hist[i] = 0;
    __syncthreads();
    for (int e0 = threadIdx.x; e0 < n; e0 += 16 * kMT) {
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = (e0 + i * kMT < n) ? x[e0 + i * kMT] : 0.0f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const uint32_t bin = first_key<MAG>(v[i]) >> kSelShift;
        if (e0 + i * kMT < n) atomicAdd(&sm.u.hist[bin], 1u);
      }
    }
    __syncthreads();
    // ---- 2. bins of positions k and k+1, key window ---------------------------------------------
    constexpr int kPerThread = kSelBins / kMT;
    uint32_t c[kPerThread], mine = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      c[i] = sm.u.hist[threadIdx.x * kPerThread + i];
      mine += c[i];
    }
    uint32_t run = med_exclusive_scan<NT>(mine, sm.wave_a, nullptr);
    const uint32_t q0 = uint32_t(k_row), q1 = uint32_t(k_row) + 1u;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const uint32_t next = run + c[i];
      if (run < q0 && q0 <= next) sm.found[0] = threadIdx.x * kPerThread + i;
      if (run < q1 && q1 <= next) sm.found[1] = threadIdx.x * kPerThread + i;
      run = next;
    }
    __syncthreads();
    uint32_t klo, khi;
    key_window<MAG>(sm.found[0], sm.found[1], R, PC == kP43, &klo, &khi);
    __syncthreads();                       // the histogram's memory is reused below

    // ---- 3. ordered compaction of the candidates into (ka, ia) ----------------------------------
    // the window in value space (key order is reversed value order, -0 == +0 either way; keys
    // beyond the infinities are clamped, they would decode to NaN)
    const float v_top = float(bound_value(klo)), v_bot = float(bound_value(khi));
    uint32_t above = 0;                    // per wavefront, summed at the end
    uint32_t above_done = 0;               // SPARSE: elements above the window in earlier tiles
    int32_t* sp_idx = SPARSE ? sp.idx + int64_t(blockIdx.x) * sp.max_nnz : nullptr;
    float* sp_val = SPARSE ? sp.val + int64_t(blockIdx.x) * sp.max_nnz : nullptr;
    for (int tile_first = 0; tile_first < n; tile_first += kCTile) {
      uint32_t pos[kCItems];
      float xv[kCItems];
      uint32_t ncand = 0;
      uint32_t apos[SPARSE ? kCItems : 1];
      uint32_t nabove = 0;                 // SPARSE: this wavefront's above-elements of the tile
#pragma unroll
      for (int i = 0; i < kCItems; ++i) {
        const int e = tile_first + w * (kCItems * kWave) + i * kWave + lane;
        xv[i] = e < n ? x[e] : 0.0f;
      }
#pragma unroll
      for (int i = 0; i < kCItems; ++i) {
        const int e = tile_first + w * (kCItems * kWave) + i * kWave + lane;
        const bool valid = e < n;
        const float v = MAG ? fabsf(xv[i]) : xv[i];
        const bool cand = valid && v <= v_top && v >= v_bot;
        const unsigned long long cm = __ballot(cand);
        const unsigned long long am = __ballot(valid && v > v_top);
        above += __popcll(am);
        if (SPARSE) {
          apos[i] = (valid && v > v_top) ? nabove + __popcll(am & lanemask_lt()) : 0xffffffffu;
          nabove += __popcll(am);
        }
        pos[i] = cand ? ncand + __popcll(cm & lanemask_lt()) : 0xffffffffu;
        ncand += __popcll(cm);
      }
      __syncthreads();                     // wave_a of the previous tile has been read
      if (lane == 0) {
        sm.wave_a[w] = ncand;
        if (SPARSE) sm.wave_b[w] = nabove;
      }
      __syncthreads();
      uint32_t before = 0, total = 0;
#pragma unroll
      for (int q = 0; q < kMW; ++q) {
        const uint32_t t = sm.wave_a[q];
        if (q < w) before += t;
        total += t;
      }
      if (SPARSE) {
        uint32_t abefore = 0, atotal = 0;
#pragma unroll
        for (int q = 0; q < kMW; ++q) {
          const uint32_t t = sm.wave_b[q];
          if (q < w) abefore += t;
          atotal += t;
        }
#pragma unroll
        for (int i = 0; i < kCItems; ++i) {
          const uint32_t o = above_done + abefore + apos[i];
          if (apos[i] != 0xffffffffu && o < uint32_t(sp.max_nnz)) {
            sp_idx[o] = tile_first + w * (kCItems * kWave) + i * kWave + lane;
            sp_val[o] = 1.0f;
          }
        }
        above_done += atotal;
      }
#pragma unroll
      for (int i = 0; i < kCItems; ++i) {
        if (pos[i] != 0xffffffffu) {
          const int e = tile_first + w * (kCItems * kWave) + i * kWave + lane;
          ka[cn + before + pos[i]] = first_key<MAG>(xv[i]);
          ia[cn + before + pos[i]] =
              MAG ? ((uint32_t(e) << 1) | (__float_as_uint(xv[i]) >> 31)) : uint32_t(e);
        }
      }
      cn += total;
    }
    if (SPARSE) __syncthreads();           // the last tile's wave_b has been read
    if (lane == 0) sm.wave_b[w] = above;
    __syncthreads();
    uint32_t above_all = 0;
#pragma unroll
    for (int q = 0; q < kMW; ++q) above_all += sm.wave_b[q];
    k = k_row - int(above_all);
    above_total = above_all;

    // ---- 4. sort the candidates -------------------------------------------------------------------
    const SortedList sorted = sort_candidates<NT, kMItems>(ka, ia, kb, ib, cn, klo, khi, sm);
    skeys = sorted.keys;
    sidx = sorted.idx;
  }

  // ---- 5. solve ---------------------------------------------------------------------------------------
  const int64_t n_sorted = (k_row >= 1 && k_row < n) ? int64_t(cn) : int64_t(n);
  const RowInfo ri = RowSolver<NT>::template solve<MAG, PC>(skeys, sidx, tangent, n_sorted, int64_t(k), R,
                                                    sm.solve);

  // ---- 6. outputs ----------------------------------------------------------------------------------
  if constexpr (SPARSE) {
    int32_t* sp_idx = sp.idx + int64_t(blockIdx.x) * sp.max_nnz;
    float* sp_val = sp.val + int64_t(blockIdx.x) * sp.max_nnz;
    int64_t nnz;
    if (k_row >= 1 && k_row < n) {
      // the candidates' sorted positions 1 .. b follow the elements above the window
      nnz = int64_t(above_total) + ri.b;
      for (int64_t pos1 = 1 + threadIdx.x; pos1 <= ri.b; pos1 += kMT) {
        const int64_t o = int64_t(above_total) + pos1 - 1;
        if (o >= sp.max_nnz) break;
        const double v = double(key_to_float(skeys[pos1 - 1])) - ri.center;
        const double y = pos1 < ri.a ? 1.0 : Pool<false, PC>::y_in_block(v, ri.gamma, R);
        sp_idx[o] = int32_t(sidx[pos1 - 1]);
        sp_val[o] = float(y);
      }
    } else {
      nnz = k_row == 0 ? 0 : n;            // k = n: every entry is 1
      for (int64_t o = threadIdx.x; o < nnz && o < sp.max_nnz; o += kMT) {
        sp_idx[o] = int32_t(o);
        sp_val[o] = 1.0f;
      }
    }
    for (int64_t o = nnz + threadIdx.x; o < sp.max_nnz; o += kMT) {
      sp_idx[o] = -1;
      sp_val[o] = 0.0f;
    }
    if (threadIdx.x == 0) sp.nnz[blockIdx.x] = int32_t(nnz);
    return;
  }
  for (int e0 = threadIdx.x; e0 < n; e0 += 8 * kMT) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (e0 + i * kMT < n) ? load_stream(x + e0 + i * kMT) : 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (e0 + i * kMT < n)
        emit_dense_element<MAG, PC>(ri, v[i], int64_t(e0 + i * kMT), tangent, out, jvp, R);
  }
  for (int64_t pos1 = ri.wa + threadIdx.x; pos1 <= ri.wb; pos1 += kMT)
    emit_window_position<MAG, PC>(ri, pos1, key_to_float(skeys[pos1 - 1]), sidx[pos1 - 1], tangent,
                                  out, jvp, R);
}

// Long rows: sort and solve of a candidate list of up to kFinishMax elements (the dense list in
// the "a" arrays, described by sel[row]) by one workgroup; writes the row's RowInfo.  Longer
// lists are left to the multi-workgroup passes.
constexpr int kFinishThreads = 1024;

template <bool MAG, int PC>
__global__ __launch_bounds__(kFinishThreads) void finish_kernel(uint32_t* keys_a, uint32_t* idx_a,
                                                     uint32_t* keys_b, uint32_t* idx_b,
                                                     const float* __restrict__ tangent_all,
                                                     const RowSel* __restrict__ sel,
                                                     RowInfo* __restrict__ info, int64_t n,
                                                     int64_t k_row, Reg R) {
  constexpr int kMT = kFinishThreads, kLdsKeys = MedCfg<kFinishThreads>::kLdsKeys;
  __shared__ MedShared<kFinishThreads> sm;
  const int64_t row = blockIdx.x;
  const RowSel rs = sel[row];
  if (int64_t(rs.cn) > kFinishMax) return;
  const int64_t base = row * n;
  uint32_t* ka = keys_a + base;
  uint32_t* ia = idx_a + base;
  uint32_t* kb = keys_b + base;
  uint32_t* ib = idx_b + base;
  const SortedList sorted = sort_candidates<kFinishThreads, 16>(ka, ia, kb, ib, rs.cn, rs.klo, rs.khi, sm);
  const uint32_t* skeys = sorted.keys;
  const uint32_t* sidx = sorted.idx;
  int src = sorted.global_src;
  if (src < 0) {
    // sorted in LDS only; the window pass reads the list from global memory
    for (uint32_t j = threadIdx.x; j < rs.cn; j += kMT) {
      ka[j] = skeys[j];
      ia[j] = sidx[j];
    }
    src = 0;
  } else if (rs.cn <= uint32_t(kLdsKeys)) {
    // the solve reads the sorted keys many times: from LDS when they fit (the sort is over and
    // its LDS is free)
    uint32_t* lds_keys = sm.u.hist;
    for (uint32_t j = threadIdx.x; j < rs.cn; j += kMT) lds_keys[j] = skeys[j];
    skeys = lds_keys;
    __syncthreads();
  }
  RowInfo ri = RowSolver<kMT>::solve<MAG, PC>(
      skeys, sidx, tangent_all != nullptr ? tangent_all + base : nullptr, int64_t(rs.cn),
      k_row - rs.above, R, sm.solve);
  ri.src = src;
  if (threadIdx.x == 0) info[row] = ri;
}


template <bool MAG, int PC>
void launch(const SortBuffers& B, const float* x, const float* tangent, float* out, float* jvp,
            int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  const SparseOut none{nullptr, nullptr, nullptr, 0};
  if (n <= kSmallRowMax)
    hipLaunchKernelGGL((medium_rows_kernel<MAG, PC, 256>), dim3(unsigned(rows)), dim3(256), 0, st, x,
                       tangent, out, jvp, B.keys_a, B.idx_a, B.keys_b, B.idx_b, n, k, R, none);
  else
    hipLaunchKernelGGL((medium_rows_kernel<MAG, PC, 1024>), dim3(unsigned(rows)), dim3(1024), 0, st,
                       x, tangent, out, jvp, B.keys_a, B.idx_a, B.keys_b, B.idx_b, n, k, R, none);
}

template <int PC>
void launch_sparse(const SortBuffers& B, const float* x, int64_t rows, int n, int k, const Reg& R,
                   const SparseOut& sp, hipStream_t st) {
  if (n <= kSmallRowMax)
    hipLaunchKernelGGL((medium_rows_kernel<false, PC, 256, true>), dim3(unsigned(rows)), dim3(256), 0,
                       st, x, nullptr, nullptr, nullptr, B.keys_a, B.idx_a, B.keys_b, B.idx_b, n, k,
                       R, sp);
  else
    hipLaunchKernelGGL((medium_rows_kernel<false, PC, 1024, true>), dim3(unsigned(rows)), dim3(1024),
                       0, st, x, nullptr, nullptr, nullptr, B.keys_a, B.idx_a, B.keys_b, B.idx_b, n,
                       k, R, sp);
}

}  // namespace

int launch_medium_rows(bool mag, int pc, const SortBuffers& B, const float* x, const float* tangent,
                       float* out, float* jvp, int64_t rows, int64_t n, int64_t k, const Reg& R,
                       hipStream_t st) {
  if (n > kMediumRowMax || rows > 0x7fffffffLL) return -1;
  if (!mag && pc == kP2) launch<false, kP2>(B, x, tangent, out, jvp, rows, int(n), int(k), R, st);
  else if (!mag && pc == kP43) launch<false, kP43>(B, x, tangent, out, jvp, rows, int(n), int(k), R, st);
  else if (mag && pc == kP2) launch<true, kP2>(B, x, tangent, out, jvp, rows, int(n), int(k), R, st);
  else if (mag && pc == kP43) launch<true, kP43>(B, x, tangent, out, jvp, rows, int(n), int(k), R, st);
  else return -1;
  return 0;
}

int launch_medium_rows_sparse(int pc, const SortBuffers& B, const float* x, int64_t rows, int64_t n,
                              int64_t k, const Reg& R, const SparseOut& sp, hipStream_t st) {
  if (n > kMediumRowMax || rows > 0x7fffffffLL) return -1;
  if (pc == kP2) launch_sparse<kP2>(B, x, rows, int(n), int(k), R, sp, st);
  else if (pc == kP43) launch_sparse<kP43>(B, x, rows, int(n), int(k), R, sp, st);
  else return -1;
  return 0;
}

int launch_finish(bool mag, int pc, const SortBuffers& B, const float* tangent, int64_t rows,
                  int64_t n, int64_t k, const Reg& R, hipStream_t st) {
  if (rows > 0x7fffffffLL) return -1;
  const dim3 grid{unsigned(rows)}, block{kFinishThreads};
  if (!mag && pc == kP2)
    hipLaunchKernelGGL((finish_kernel<false, kP2>), grid, block, 0, st, B.keys_a, B.idx_a, B.keys_b,
                       B.idx_b, tangent, B.sel, B.info, n, k, R);
  else if (!mag && pc == kP43)
    hipLaunchKernelGGL((finish_kernel<false, kP43>), grid, block, 0, st, B.keys_a, B.idx_a,
                       B.keys_b, B.idx_b, tangent, B.sel, B.info, n, k, R);
  else if (mag && pc == kP2)
    hipLaunchKernelGGL((finish_kernel<true, kP2>), grid, block, 0, st, B.keys_a, B.idx_a, B.keys_b,
                       B.idx_b, tangent, B.sel, B.info, n, k, R);
  else if (mag && pc == kP43)
    hipLaunchKernelGGL((finish_kernel<true, kP43>), grid, block, 0, st, B.keys_a, B.idx_a,
                       B.keys_b, B.idx_b, tangent, B.sel, B.info, n, k, R);
  else return -1;
  return 0;
}

}  // namespace topk
