// Short rows of up to 128 elements: the fast variant of the fused kernel.
//
// Differences to short_rows.hip (which stays the general kernel up to 1024 elements):
//
//  * the sort runs on ONE 32-bit word per element, (descending-order key with its low log2(NP)
//    bits replaced by the element index).  A compare-exchange across lanes is then a DPP compare
//    plus a DPP select, and v_min_u32 / v_max_u32 inside a lane.  Two values whose keys agree
//    in all but the dropped low bits can come out in the wrong order; such neighbours are
//    detected after the network (equal truncated keys, different values) and put right by
//    odd-even transposition passes on the full (value, index) order, so the permutation is
//    exactly the stable descending argsort.
//  * nothing is unpacked per element after the sort: the sorted words and the original rows sit
//    in LDS, the block growth reads the few positions it needs through them, and the epilogue
//    only visits the sorted positions 1..b that can be non-zero (one element per lane and pass);
//    everything else is the zero fill of the staging buffers.
//
// LDS per row (NP floats + 4 of padding each): lx (x in original order, later the sorted index
// words), lt (tangent), ls (sorted values), ly (y, zero-filled), ld (dy, zero-filled).
#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "wave.hpp"

namespace topk {
namespace {

__device__ __forceinline__ uint32_t median3_u32(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// ---- 32-bit sorting network (same mirror-bitonic schedule as the float64 one) ----------------
template <int GL, int E, int M>
__device__ __forceinline__ void sort_stage32(uint32_t (&K)[E], int lr) {
  constexpr int RM = M & (E - 1);
  constexpr int LM = M / E;
  if constexpr (LM == 0) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int r2 = r ^ RM;
      if (r < r2) {
        const uint32_t lo = min(K[r], K[r2]);
        const uint32_t hi = max(K[r], K[r2]);
        K[r] = lo;
        K[r2] = hi;
      }
    }
  } else {
    // the lower lane keeps the minimum, the upper one the maximum: both are the median of
    // (own, other, bound) with bound = 0 resp. 0xffffffff, one instruction instead of min, max
    // and a select
    const uint32_t bound = (lr & top_bit(LM)) == 0 ? 0u : 0xffffffffu;
    uint32_t O[E];
#pragma unroll
    for (int r = 0; r < E; ++r) O[r] = lane_xor<LM>(K[r ^ RM]);
#pragma unroll
    for (int r = 0; r < E; ++r) K[r] = median3_u32(K[r], O[r], bound);
  }
}

template <int GL, int E, int STRIDE>
struct HalfCleaners32 {
  static __device__ __forceinline__ void run(uint32_t (&K)[E], int lr) {
    sort_stage32<GL, E, STRIDE>(K, lr);
    HalfCleaners32<GL, E, STRIDE / 2>::run(K, lr);
  }
};
template <int GL, int E>
struct HalfCleaners32<GL, E, 0> {
  static __device__ __forceinline__ void run(uint32_t (&)[E], int) {}
};
template <int GL, int E, int SIZE>
struct SortRuns32 {
  static __device__ __forceinline__ void run(uint32_t (&K)[E], int lr) {
    SortRuns32<GL, E, SIZE / 2>::run(K, lr);
    sort_stage32<GL, E, SIZE - 1>(K, lr);
    HalfCleaners32<GL, E, SIZE / 4>::run(K, lr);
  }
};
template <int GL, int E>
struct SortRuns32<GL, E, 1> {
  static __device__ __forceinline__ void run(uint32_t (&)[E], int) {}
};

template <int GL, int E>
struct FastCfg {
  static constexpr int NP = GL * E;
  static constexpr int RPW = kWave / GL;
  static constexpr int RS = NP + 4;                        // row stride in LDS, floats
  static constexpr int Arrays = 5;
  static constexpr int WaveBytes = Arrays * RPW * RS * 4;
  // wavefronts per workgroup: single-wavefront workgroups measured 7 % faster on 32768 x 128
  // (16 lanes per row) and the same on 16384 x 64 (8 lanes per row)
  static constexpr int WPB = GL >= 16 ? 1 : ((4 * WaveBytes <= 64 * 1024) ? 4 : ((2 * WaveBytes <= 64 * 1024) ? 2 : 1));
  static constexpr uint32_t IM = NP - 1;                   // index mask inside a sorted word
};

// Sort the row's words and repair the order of neighbours that only differ in dropped key bits.
// On return c[] holds the words and s[] the values (|x| for the magnitude operator) of the sorted
// positions lr*E .. lr*E+E-1.  lx: the row in LDS.
template <int GL, int E, bool MAG>
__device__ __forceinline__ void sort_words(uint32_t (&c)[E], float (&s)[E], int lr, const float* lx) {
  using C = FastCfg<GL, E>;
  constexpr uint32_t IM = C::IM;
  SortRuns32<GL, E, C::NP>::run(c, lr);
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const float v = lx[c[r] & IM];
    s[r] = MAG ? fabsf(v) : v;
  }
  // After the network the values are non-increasing unless two neighbours with equal truncated
  // keys came out in the wrong order (different truncated keys imply a strict value order).
  // `wrong` is the full test used by the repair passes: equal truncated keys and
  // (value, index) out of order.  No short-circuit operators: these run as straight-line code.
  auto wrong = [&](uint32_t cp, float sp, uint32_t cq, float sq) -> bool {
    const bool same = (cp ^ cq) <= IM;
    const bool lt = sp < sq;
    const bool tie = (sp == sq) & ((cp & IM) > (cq & IM));
    return same & (lt | tie);
  };
  bool dirty = false;
#pragma unroll
  for (int r = 0; r + 1 < E; ++r) dirty |= (s[r] < s[r + 1]);
  if constexpr (GL > 1) {
    const float s_up = __uint_as_float(dpp_mov<0x101>(__float_as_uint(s[0])));   // row_shl:1: lane + 1
    dirty |= (lr < GL - 1) & (s[E - 1] < s_up);
  }
  // odd-even transposition passes until every neighbour pair is in order (rare)
  while (__any(dirty)) {
    dirty = false;
#pragma unroll
    for (int par = 0; par < 2; ++par) {
#pragma unroll
      for (int r = par; r + 1 < E; r += 2) {
        const bool sw = wrong(c[r], s[r], c[r + 1], s[r + 1]);
        const uint32_t c0 = c[r], c1 = c[r + 1];
        const float s0 = s[r], s1 = s[r + 1];
        c[r] = sw ? c1 : c0; c[r + 1] = sw ? c0 : c1;
        s[r] = sw ? s1 : s0; s[r + 1] = sw ? s0 : s1;
        dirty |= sw;
      }
    }
    // the odd pair across lanes: (last of lane l, first of lane l+1); E >= 4, so slots 0 and E-1
    // are distinct registers
    if constexpr (GL > 1) {
      const uint32_t c_up = dpp_mov<0x101>(c[0]);
      const float s_up = __uint_as_float(dpp_mov<0x101>(__float_as_uint(s[0])));
      const uint32_t c_dn = dpp_mov<0x111>(c[E - 1]);                  // row_shr:1: lane - 1
      const float s_dn = __uint_as_float(dpp_mov<0x111>(__float_as_uint(s[E - 1])));
      const bool sw_hi = (lr < GL - 1) & wrong(c[E - 1], s[E - 1], c_up, s_up);
      const bool sw_lo = (lr > 0) & wrong(c_dn, s_dn, c[0], s[0]);
      c[E - 1] = sw_hi ? c_up : c[E - 1];
      s[E - 1] = sw_hi ? s_up : s[E - 1];
      c[0] = sw_lo ? c_dn : c[0];
      s[0] = sw_lo ? s_dn : s[0];
      dirty |= sw_hi | sw_lo;
    }
  }
}

template <int E, bool MAG>
__device__ __forceinline__ void make_words(const float (&v)[E], int e0, int n, uint32_t im,
                                           uint32_t (&c)[E]) {
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = e0 + r;
    const uint32_t key = desc_key(MAG ? fabsf(v[r]) : v[r]);
    c[r] = (e < n) ? ((key & ~im) | uint32_t(e)) : 0xffffffffu;
  }
}

template <int E>
__device__ __forceinline__ void lds_zero(float* p) {
#pragma unroll
  for (int q = 0; q < E / 4; ++q) *reinterpret_cast<float4*>(p + 4 * q) = make_float4(0.f, 0.f, 0.f, 0.f);
}

// ---- argsort only ------------------------------------------------------------------------------
template <int GL, int E, bool VEC>
__global__ __launch_bounds__((FastCfg<GL, E>::WPB * kWave)) void fast_argsort_kernel(
    const float* __restrict__ x, int32_t* __restrict__ perm, int64_t rows, int n) {
  using C = FastCfg<GL, E>;
  __shared__ __attribute__((aligned(16))) float lds[C::WPB][C::RPW * C::RS];
  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  int64_t row = (int64_t(blockIdx.x) * C::WPB + wv) * C::RPW + lane / GL;
  const bool valid = row < rows;
  if (!valid) row = rows - 1;
  const int e0 = lr * E;
  float* lx = &lds[wv][(lane / GL) * C::RS];
  float xin[E];
  load_elems<E, VEC>(x, row * n, e0, n, xin);
  uint32_t c[E];
  make_words<E, false>(xin, e0, n, C::IM, c);
#pragma unroll
  for (int r = 0; r < E; ++r) xin[r] = (e0 + r < n) ? xin[r] : __uint_as_float(0x7fc00000u);
  lds_store<E>(lx + e0, xin);
  __builtin_amdgcn_wave_barrier();
  float sv[E];
  sort_words<GL, E, false>(c, sv, lr, lx);
  if (!valid) return;
#pragma unroll
  for (int r = 0; r < E; ++r)
    if (e0 + r < n) perm[row * n + e0 + r] = int32_t(c[r] & C::IM);
}

// ---- the fused operator -------------------------------------------------------------------------
// inclusive prefix sum over groups of H consecutive lanes (H <= 8, inside one DPP row); t = lane
// index inside the group
template <int H>
__device__ __forceinline__ void half_scan(double& v, int t) {
  if constexpr (H >= 2) { const double o = row_shr_f64<1>(v); v = (t >= 1) ? v + o : v; }
  if constexpr (H >= 4) { const double o = row_shr_f64<2>(v); v = (t >= 2) ? v + o : v; }
  if constexpr (H >= 8) { const double o = row_shr_f64<4>(v); v = (t >= 4) ? v + o : v; }
}

// Element offset of the q-th float4 of a lane in a full row: the lanes of a row take consecutive
// float4s, so every load / store instruction of a row group covers one contiguous span of the row
// (which elements a lane holds is immaterial to the sort: the index travels in the word).
#define TOPK_FULL_OFF(q) ((((q) * GL) + lr) * 4)

// VEC: rows are 16-byte aligned and n % 4 == 0 (float4 loads and stores).
// FULL: additionally n == NP, so there is no padding and no bounds test anywhere.
// MODE: 0 forward only, 1 JVP only, 2 forward + JVP, 3 forward only in compact form (compile-time,
// so no output is tested for at run time).
template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE>
__global__ __launch_bounds__((FastCfg<GL, E>::WPB * kWave)) void short_rows_fast_kernel(
    const float* __restrict__ x, const float* __restrict__ tangent, float* __restrict__ out,
    float* __restrict__ jvp, int64_t rows, int n, int k, Reg R, float inv_lambda32,
    float inv_1pl32, SparseOut sp) {
  using P = Pool<MAG, PC>;
  using C = FastCfg<GL, E>;
  constexpr int NP = C::NP, RS = C::RS;
  constexpr uint32_t IM = C::IM;
  constexpr bool CUBIC = (PC == kP43);
  constexpr bool CHUNKED = GL >= 4;      // rows with at least 4 lanes also grow the block in chunks
  __shared__ __attribute__((aligned(16))) float lds[C::WPB][C::Arrays][C::RPW * RS];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int64_t row_raw = (int64_t(blockIdx.x) * C::WPB + wv) * C::RPW + lane / GL;
  const bool valid = row_raw < rows;
  const int64_t row = valid ? row_raw : rows - 1;   // lanes stay alive for the exchanges; no stores
  const int64_t base = row * n;
  const int e0 = lr * E;
  const int roff = (lane / GL) * RS;
  float* lx = &lds[wv][0][roff];         // x in original order; later the sorted index words
  float* lt = &lds[wv][1][roff];         // tangent, original order
  float* ls = &lds[wv][2][roff];         // sorted values
  float* ly = &lds[wv][3][roff];         // y, original order, zero-filled
  float* ld = &lds[wv][4][roff];         // dy, original order, zero-filled
  const int nn = FULL ? NP : n;
  constexpr bool kSparse = (MODE == 3);  // forward only, the non-zeros as (index, value) lists
  constexpr bool want_out = (MODE == 0 || MODE == 2), want_jvp = (MODE == 1 || MODE == 2);

  // ---- load, stage, sort ---------------------------------------------------------------------
  float xin[E], tin[E];
  if (FULL) {
#pragma unroll
    for (int q = 0; q < E / 4; ++q) {
      const float4 v = load4_stream(x + base + TOPK_FULL_OFF(q));
      xin[4 * q] = v.x; xin[4 * q + 1] = v.y; xin[4 * q + 2] = v.z; xin[4 * q + 3] = v.w;
    }
    if (want_jvp) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q) {
        const float4 v = load4_stream(tangent + base + TOPK_FULL_OFF(q));
        tin[4 * q] = v.x; tin[4 * q + 1] = v.y; tin[4 * q + 2] = v.z; tin[4 * q + 3] = v.w;
      }
    }
  } else {
    load_elems<E, VEC>(x, base, e0, n, xin);
    if (want_jvp) load_elems<E, VEC>(tangent, base, e0, n, tin);
  }
  uint32_t c[E];
  if (FULL) {
#pragma unroll
    for (int r = 0; r < E; ++r)
      c[r] = (desc_key(MAG ? fabsf(xin[r]) : xin[r]) & ~IM) | uint32_t(TOPK_FULL_OFF(r / 4) + (r & 3));
  } else {
    make_words<E, MAG>(xin, e0, n, IM, c);
    // padding reads as NaN so that it never looks out of order next to a real value
#pragma unroll
    for (int r = 0; r < E; ++r) xin[r] = (e0 + r < n) ? xin[r] : __uint_as_float(0x7fc00000u);
  }
  if (FULL) {
#pragma unroll
    for (int q = 0; q < E / 4; ++q)
      *reinterpret_cast<float4*>(lx + TOPK_FULL_OFF(q)) =
          make_float4(xin[4 * q], xin[4 * q + 1], xin[4 * q + 2], xin[4 * q + 3]);
  } else {
    lds_store<E>(lx + e0, xin);
  }
  if (want_out) lds_zero<E>(ly + e0);
  if (want_jvp) lds_zero<E>(ld + e0);
  __builtin_amdgcn_wave_barrier();
  float s[E];
  sort_words<GL, E, MAG>(c, s, lr, lx);
  if (want_jvp) {                               // staged after the sort: the sort need not wait for it
    if (FULL) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q)
        *reinterpret_cast<float4*>(lt + TOPK_FULL_OFF(q)) =
            make_float4(tin[4 * q], tin[4 * q + 1], tin[4 * q + 2], tin[4 * q + 3]);
    } else {
      lds_store<E>(lt + e0, tin);
    }
  }
  lds_store<E>(ls + e0, s);
  __builtin_amdgcn_wave_barrier();

  // ---- isotonic solve: grow the one pooled block outwards from (k, k+1) ----------------------
  // All lanes of a row carry the same (a, b, sums).  A step tests the two neighbours of the block
  // with the strict violation tests of the PAV loop and takes in whichever violates; both may
  // join in one step (the right one raises the pooled value, the left one lowers it, so each
  // still violates after the other has joined).  Straight-line selects, one branch per step.
  int a = k + 1, b = k;                  // 1-based inclusive block [a, b]; empty when a > b
  double center = 0.0, gamma = 0.0, cnt = 0.0, m = 0.0;
  float c32 = 0.0f;                      // s_k: the epilogue works on values relative to it
  if (k >= 1 && k < nn) {                // uniform
    c32 = ls[k - 1];
    const float fk1 = ls[k];
    float nl = ls[k >= 2 ? k - 2 : 0];       // value left of the block (position a-1)
    float nr = ls[k + 1 < nn ? k + 1 : k];   // value right of the block (position b+1)
    const double sk = double(c32), sk1 = double(fk1);
    if (!MAG) center = sk;
    const double dk = sk - center, dk1 = sk1 - center;
    const bool grew = P::seed_violates(dk, dk1, R);
    if (__any(grew)) {
      Sums S{dk + dk1, 0.0, 0.0};
      if (CUBIC) {
        S.s2 = dk * dk + dk1 * dk1;
        S.s3 = dk * dk * dk + dk1 * dk1 * dk1;
      }
      a = grew ? k : a;
      b = grew ? k + 1 : b;
      cnt = 2.0;
      m = 1.0;
      // (1) a few single-neighbour steps: the usual p = 2 block has 2-5 positions
      constexpr int kSingleSteps = CUBIC ? 0 : 3;
      bool pending = true;               // some row of the wavefront may still grow
      for (int step = 0; step < kSingleSteps || !CHUNKED; ++step) {
        const double dj = double(nr) - center, di = double(nl) - center;
        const bool add_r = grew & (b < nn) & P::right_violates(dj, cnt, m, S, R);
        const bool add_l = grew & (a > 1) & P::left_violates(di, cnt, m, S, R);
        if (!__any(add_r | add_l)) { pending = false; break; }
        b += add_r ? 1 : 0;
        a -= add_l ? 1 : 0;
        nr = ls[b < nn ? b : nn - 1];
        nl = ls[a >= 2 ? a - 2 : 0];
        const double ar = add_r ? dj : 0.0, al = add_l ? di : 0.0;
        S.s1 += ar + al;
        if (CUBIC) {
          S.s2 += ar * ar + al * al;
          S.s3 += ar * ar * ar + al * al * al;
        }
        cnt = double(b - a + 1);
        m = double(k - a + 1);
      }
      // (2) larger blocks: every step tests GL/2 positions on each side at once.  The lower half
      // of the row's lanes takes the positions b+1, b+2, .. and the upper half a-1, a-2, ..; an
      // exclusive scan of the power sums inside each half gives every lane the block it would
      // join (all candidates before it included), and the violation tests hold on a prefix of
      // each half, whose length is read off a ballot.
      if constexpr (CHUNKED) {
        constexpr int H = GL / 2;
        const int t = lr & (H - 1);
        const bool left = lr >= H;
        bool first_chunk = true;
        while (pending) {
          if (!first_chunk) {
            // the tests are monotone along each side: if neither immediate neighbour of the block
            // violates now, no position does, and the growth is over (this replaces a whole
            // chunk step that would find nothing)
            const double dj = double(ls[b < nn ? b : nn - 1]) - center;
            const double di = double(ls[a >= 2 ? a - 2 : 0]) - center;
            const bool add_r = grew & (b < nn) & P::right_violates(dj, cnt, m, S, R);
            const bool add_l = grew & (a > 1) & P::left_violates(di, cnt, m, S, R);
            if (!__any(add_r | add_l)) break;
          }
          first_chunk = false;
          const int q = left ? a - 2 - t : b + t;            // 0-based sorted position
          const bool ok = grew & (left ? q >= 0 : q < nn);
          const float v = ls[ok ? q : 0];
          const double d = ok ? double(v) - center : 0.0;
          Sums own{d, CUBIC ? d * d : 0.0, CUBIC ? d * d * d : 0.0};
          Sums pre = own;                                    // inclusive scan over the half
          half_scan<H>(pre.s1, t);
          if (CUBIC) { half_scan<H>(pre.s2, t); half_scan<H>(pre.s3, t); }
          Sums blk{S.s1 + (pre.s1 - own.s1), S.s2 + (pre.s2 - own.s2), S.s3 + (pre.s3 - own.s3)};
          const double cnt_t = cnt + double(t), m_t = m + (left ? double(t) : 0.0);
          const bool viol = left ? P::left_violates(d, cnt_t, m_t, blk, R)
                                 : P::right_violates(d, cnt_t, m_t, blk, R);
          const unsigned long long bal = __ballot(ok & viol);
          const uint32_t rowbits = uint32_t(bal >> (lane & ~(GL - 1))) & ((1u << GL) - 1u);
          // number of leading candidates that join, per side (the tests are monotone)
          const int n_r = __builtin_ctz(~(rowbits & ((1u << H) - 1u)) | (1u << H));
          const int n_l = __builtin_ctz(~(rowbits >> H) | (1u << H));
          if (!__any((n_r | n_l) != 0)) break;
          const bool take = t < (left ? n_l : n_r);
          Sums add{take ? own.s1 : 0.0, take ? own.s2 : 0.0, take ? own.s3 : 0.0};
          S.s1 += group_sum_f64<GL>(add.s1);
          if (CUBIC) {
            S.s2 += group_sum_f64<GL>(add.s2);
            S.s3 += group_sum_f64<GL>(add.s3);
          }
          b += n_r;
          a -= n_l;
          cnt = double(b - a + 1);
          m = double(k - a + 1);
        }
      }
      const double da = double(ls[a - 1]) - center, db = double(ls[b - 1]) - center;
      if (MAG) gamma = S.s1 * recip(cnt + R.lambda * m);
      else if (!CUBIC) gamma = (S.s1 - R.lambda * m) * recip(cnt);
      else if (grew) gamma = P::pooled(cnt, m, S, R, da - R.lambda, db);   // (rows without a
      // block skip the Newton solve: their sums may hold the -inf of an unlisted s_{k+1})
      gamma = grew ? gamma : 0.0;
    }
  }

  // ---- epilogue over the sorted positions 1..b (everything else stays zero) --------------------
  // pass j handles sorted position j*GL + lr + 1 of every row of the wavefront.  The original
  // index of a sorted position comes from its word; the words replace x in LDS (x is no longer
  // needed except for its sign, which rides in bit 31 of the word for the magnitude operator).
  {
    float cf[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
      uint32_t w = c[r] & IM;
      if (MAG) w |= (__float_as_uint(lx[w]) & 0x80000000u);
      cf[r] = __uint_as_float(w);
    }
    __builtin_amdgcn_wave_barrier();
    lds_store<E>(lx + e0, cf);
    __builtin_amdgcn_wave_barrier();
  }
  const float g32 = float(MAG ? gamma - double(c32) : gamma);   // pooled value relative to s_k
  const bool more = __any(b > GL);       // some row has non-zeros beyond the first pass
  // first pass: position lr (always inside the row's padded length)
  const uint32_t w0 = __float_as_uint(lx[lr]);
  const float s0 = ls[lr];
  float t0 = 0.0f;
  if (want_jvp) {
    t0 = lt[w0 & IM];
    if (MAG) {
      t0 = (w0 >> 31) ? -t0 : t0;
      t0 = (s0 == 0.0f) ? 0.0f : t0;     // sign(0) = 0
    }
  }
  const bool have0 = lr < b;
  const bool blk0 = have0 & (lr + 1 >= a);
  double dgamma = 0.0;
  if (want_jvp && __any(a <= b)) {
    // Prop. 7: d gamma = sum_B c_j tau_j / (sum_B c_j [+ lambda m])
    double num, wsum = 0.0;
    if (CUBIC) {
      const double w = blk0 ? P::jac_weight(double(s0) - center, gamma) : 0.0;
      num = w * double(t0);
      wsum = w;
    } else {
      num = blk0 ? double(t0) : 0.0;
    }
    if (more) {
      for (int q = lr + GL; __any(q < b); q += GL) {
        const bool in = (q < b) & (q + 1 >= a);
        const int qq = q < NP ? q : 0;
        const uint32_t w = __float_as_uint(lx[qq]);
        const float sv = ls[qq];
        float tv = lt[w & IM];
        if (MAG) {
          tv = (w >> 31) ? -tv : tv;
          tv = (sv == 0.0f) ? 0.0f : tv;
        }
        if (CUBIC) {
          const double wt = in ? P::jac_weight(double(sv) - center, gamma) : 0.0;
          num += wt * double(tv);
          wsum += wt;
        } else {
          num += in ? double(tv) : 0.0;
        }
      }
    }
    num = group_sum_f64<GL>(num);
    if (CUBIC) wsum = group_sum_f64<GL>(wsum);
    else wsum = cnt;
    const double den = P::jac_denominator(wsum, m, R);
    dgamma = (a <= b) ? num * recip(den) : 0.0;
  }
  // outputs of one sorted position; rows that have nothing there write to the padding slot
  auto emit = [&](int q, bool have, bool in_block, uint32_t w, float sv, float tv) {
    const uint32_t e = have ? (w & IM) : uint32_t(NP);
    const bool neg = MAG && (w >> 31);
    const float t = ((sv - c32) - g32) * inv_lambda32;       // (s - gamma) / lambda
    if (want_out || kSparse) {
      float y;
      if (MAG) {
        const double yd = in_block ? P::y_in_block(double(sv), gamma, R) : double(sv) * R.inv_1pl;
        y = float(yd);
        y = (y == 0.0f) ? 0.0f : (neg ? -y : y);
      } else {
        y = in_block ? (CUBIC ? t * t * t : t) : 1.0f;
      }
      if (want_out) ly[e] = y;
      // compact form: sorted position q of the row is entry q of its list
      if (kSparse && valid && q < sp.max_nnz) {
        const int64_t o = row * sp.max_nnz + q;
        sp.idx[o] = have ? int32_t(w & IM) : -1;
        sp.val[o] = have ? y : 0.0f;
      }
    }
    if (want_jvp) {
      const double diff = double(tv) - dgamma;
      float dyb;
      if (CUBIC) dyb = 3.0f * t * t * inv_lambda32 * float(diff);
      else dyb = float(diff * R.inv_lambda);
      float dy = in_block ? dyb : (MAG ? tv * inv_1pl32 : 0.0f);
      if (MAG) dy = (dy == 0.0f || sv == 0.0f) ? 0.0f : (neg ? -dy : dy);
      ld[e] = dy;
    }
  };
  emit(lr, have0, blk0, w0, s0, t0);
  if (more) {
    for (int q = lr + GL; __any(q < b); q += GL) {
      const bool have = q < b;
      const int qq = q < NP ? q : 0;
      const uint32_t w = __float_as_uint(lx[qq]);
      const float sv = ls[qq];
      float tv = 0.0f;
      if (want_jvp) {
        tv = lt[w & IM];
        if (MAG) {
          tv = (w >> 31) ? -tv : tv;
          tv = (sv == 0.0f) ? 0.0f : tv;
        }
      }
      emit(q, have, have & (q + 1 >= a), w, sv, tv);
    }
  }
  if (kSparse && valid) {
    // slots after the non-zeros that no pass reached, and the count
    for (int q = lr + GL; q < sp.max_nnz; q += GL) {
      if (q >= b) {
        sp.idx[row * sp.max_nnz + q] = -1;
        sp.val[row * sp.max_nnz + q] = 0.0f;
      }
    }
    if (lr == 0) sp.nnz[row] = b;
  }
  __builtin_amdgcn_wave_barrier();
  if (!valid) return;

  // ---- coalesced stores of the un-sorted rows ---------------------------------------------------
  if (want_out) {
    float yv[E];
    if (FULL) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q)
        store4_stream(out + base + TOPK_FULL_OFF(q), *reinterpret_cast<const float4*>(ly + TOPK_FULL_OFF(q)));
    } else {
      lds_load<E>(ly + e0, yv);
      store_elems<E, VEC>(out, base, e0, n, yv);
    }
  }
  if (want_jvp) {
    float jv[E];
    if (FULL) {
#pragma unroll
      for (int q = 0; q < E / 4; ++q)
        store4_stream(jvp + base + TOPK_FULL_OFF(q), *reinterpret_cast<const float4*>(ld + TOPK_FULL_OFF(q)));
    } else {
      lds_load<E>(ld + e0, jv);
      store_elems<E, VEC>(jvp, base, e0, n, jv);
    }
  }
}

template <int GL, int E, bool MAG, int PC, bool VEC, bool FULL, int MODE>
int launch_fast_mode(const float* x, const float* t, float* out, float* jvp, int64_t rows, int n,
                     int k, const Reg& R, hipStream_t st,
                     const SparseOut& sp = SparseOut{nullptr, nullptr, nullptr, 0}) {
  using C = FastCfg<GL, E>;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + C::WPB - 1) / C::WPB;
  if (blocks > 0x7fffffffLL) return -1;
  dim3 grid((unsigned)blocks), block(C::WPB * kWave);
  const float il = float(R.inv_lambda), i1 = float(R.inv_1pl);
  hipLaunchKernelGGL((short_rows_fast_kernel<GL, E, MAG, PC, VEC, FULL, MODE>), grid, block, 0, st,
                     x, t, out, jvp, rows, n, k, R, il, i1, sp);
  return 0;
}

// mask: p = 2 and p = 4/3; magnitude: p = 2
template <int GL, int E, bool VEC, bool FULL>
int launch_fast_shape2(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                       int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  const int mode = (jvp == nullptr) ? 0 : (out == nullptr ? 1 : 2);
#define TOPK_MODE_CALL(MAGV, PCV, M) \
  return launch_fast_mode<GL, E, MAGV, PCV, VEC, FULL, M>(x, t, out, jvp, rows, n, k, R, st)
  if (!mag && pc == kP2) {
    if (mode == 0) TOPK_MODE_CALL(false, kP2, 0);
    if (mode == 1) TOPK_MODE_CALL(false, kP2, 1);
    TOPK_MODE_CALL(false, kP2, 2);
  }
  if (!mag && pc == kP43) {
    if (mode == 0) TOPK_MODE_CALL(false, kP43, 0);
    if (mode == 1) TOPK_MODE_CALL(false, kP43, 1);
    TOPK_MODE_CALL(false, kP43, 2);
  }
  if (mag && pc == kP2) {
    if (mode == 0) TOPK_MODE_CALL(true, kP2, 0);
    if (mode == 1) TOPK_MODE_CALL(true, kP2, 1);
    TOPK_MODE_CALL(true, kP2, 2);
  }
#undef TOPK_MODE_CALL
  return -2;
}

template <int GL, int E, bool VEC>
int launch_fast_shape(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                      int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  if (VEC && n == GL * E)
    return launch_fast_shape2<GL, E, true, true>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
  return launch_fast_shape2<GL, E, VEC, false>(mag, pc, x, t, out, jvp, rows, n, k, R, st);
}

template <int GL, int E, bool VEC>
int launch_fast_argsort_shape(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st) {
  using C = FastCfg<GL, E>;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + C::WPB - 1) / C::WPB;
  if (blocks > 0x7fffffffLL) return -1;
  hipLaunchKernelGGL((fast_argsort_kernel<GL, E, VEC>), dim3((unsigned)blocks),
                     dim3(C::WPB * kWave), 0, st, x, perm, rows, n);
  return 0;
}

}  // namespace

// Shapes of the fast kernels: rows of 4..128 padded elements, at most 16 lanes per row (one DPP
// row), 4 or 8 elements per lane.  Returns -2 when (np, lg) is not one of them.
#define TOPK_FAST_SHAPE(GL, E) \
  if (np == (GL) * (E) && lg == ilog2(GL)) return vec ? CALL(GL, E, true) : CALL(GL, E, false);
#define TOPK_FAST_TABLE                                                                      \
  TOPK_FAST_SHAPE(1, 4) TOPK_FAST_SHAPE(1, 8) TOPK_FAST_SHAPE(2, 4) TOPK_FAST_SHAPE(2, 8)    \
  TOPK_FAST_SHAPE(4, 4) TOPK_FAST_SHAPE(4, 8) TOPK_FAST_SHAPE(8, 4) TOPK_FAST_SHAPE(8, 8)    \
  TOPK_FAST_SHAPE(16, 4) TOPK_FAST_SHAPE(16, 8)

int launch_short_rows_fast(int np, int lg, bool vec, bool mag, int pc, const float* x,
                           const float* tangent, float* out, float* jvp, int64_t rows, int n,
                           int k, const Reg& R, hipStream_t st) {
#define CALL(GL, E, V) launch_fast_shape<GL, E, V>(mag, pc, x, tangent, out, jvp, rows, n, k, R, st)
  TOPK_FAST_TABLE
#undef CALL
  return -2;
}

// compact output of the mask (mode 3)
template <int GL, int E, bool VEC>
int launch_fast_sparse_shape(int pc, const float* x, int64_t rows, int n, int k, const Reg& R,
                             const SparseOut& sp, hipStream_t st) {
  if (VEC && n == GL * E) {
    if (pc == kP2) return launch_fast_mode<GL, E, false, kP2, true, true, 3>(x, nullptr, nullptr, nullptr, rows, n, k, R, st, sp);
    return launch_fast_mode<GL, E, false, kP43, true, true, 3>(x, nullptr, nullptr, nullptr, rows, n, k, R, st, sp);
  }
  if (pc == kP2) return launch_fast_mode<GL, E, false, kP2, VEC, false, 3>(x, nullptr, nullptr, nullptr, rows, n, k, R, st, sp);
  return launch_fast_mode<GL, E, false, kP43, VEC, false, 3>(x, nullptr, nullptr, nullptr, rows, n, k, R, st, sp);
}

int launch_short_rows_fast_sparse(int np, int lg, bool vec, int pc, const float* x, int64_t rows,
                                  int n, int k, const Reg& R, const SparseOut& sp, hipStream_t st) {
  if (pc != kP2 && pc != kP43) return -2;
#define CALL(GL, E, V) launch_fast_sparse_shape<GL, E, V>(pc, x, rows, n, k, R, sp, st)
  TOPK_FAST_TABLE
#undef CALL
  return -2;
}

int launch_short_argsort_fast(int np, int lg, bool vec, const float* x, int32_t* perm,
                              int64_t rows, int n, hipStream_t st) {
#define CALL(GL, E, V) launch_fast_argsort_shape<GL, E, V>(x, perm, rows, n, st)
  TOPK_FAST_TABLE
#undef CALL
  return -2;
}

}  // namespace topk
