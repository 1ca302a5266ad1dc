// Short rows (n <= 1024): one row per group of GL lanes of a wavefront, E elements per lane,
// 64/GL rows per wavefront; everything between the load and the store stays in registers, plus
// one small per-wavefront LDS buffer for the un-sort scatter and the tangent gather.
//
//   load -> pack (key, index) into one float64 -> bitonic network (v_min/v_max_f64 in a lane,
//   DPP exchanges across lanes) -> float64 windowed prefix sums -> block growth -> pooled value
//   -> y and dy in sorted order -> scatter through LDS -> coalesced store
//
// Layout: lane l of a row group holds elements l*E .. l*E+E-1 of its row (a contiguous,
// vectorisable load) and, after the sort, the sorted positions l*E .. l*E+E-1.
//
// The composite sort key is (descending-order key : 32 bits | index field) stored as the integer
// part of a float64 in [2^52, 2^53): all such doubles are positive normals whose order is the
// order of the integers, so v_min_f64 / v_max_f64 are exact compare-exchanges and ties in the
// value fall back to the index (ascending), which is the tie rule of the library.
#include <cstdlib>

#include "common.hpp"
#include "pooling.hpp"
#include "launch.hpp"
#include "wave.hpp"
#include "sort_network.hpp"


namespace topk {
namespace {

// rows are read once and written once: streaming accesses (each instruction of a row group
// covers a contiguous span, see load_row)
constexpr bool kStreamRows = true;


// E consecutive floats of a row starting at element e0; VEC: rows are 16-byte aligned and n % 4 == 0
// ---- argsort only ------------------------------------------------------------------------------
template <int GL, int E, bool VEC>
__global__ __launch_bounds__(256) void short_argsort_kernel(const float* __restrict__ x,
                                                            int32_t* __restrict__ perm,
                                                            int64_t rows, int n) {
  constexpr int NP = GL * E, RPW = kWave / GL, IDXB = ilog2(NP) + 1;
  const int lr = lane_in_group<GL>();
  const int64_t wave = int64_t(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
  int64_t row = wave * RPW + ((threadIdx.x & (kWave - 1)) / GL);
  const bool valid = row < rows;
  if (!valid) row = rows - 1;
  float v[E];
  load_row<GL, E, VEC, kStreamRows>(x, row * n, lr, n, v);
  double K[E];
  make_keys_row<GL, E, VEC, false, IDXB>(v, lr, n, K);
  SortRuns<GL, E, NP>::run(K, lr);
  if (!valid) return;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int pos = lr * E + r;
    uint32_t key, field;
    unpack<IDXB>(K[r], key, field);
    if (pos < n) perm[row * n + pos] = int32_t(field);
  }
}

// ---- the fused operator -------------------------------------------------------------------------
// LDS per wavefront: three arrays of 64/GL rows, each row NP floats plus 4 floats of padding (so
// that the same position of different rows falls into different banks):
//   ls : the sorted values (read by the block growth, one broadcast read per row and step)
//   lt : the tangent in original order (gathered through sigma), later dy in original order
//   ly : y in original order
template <int GL, int E>
struct ShortCfg {
  static constexpr int NP = GL * E;
  static constexpr int RPW = kWave / GL;
  static constexpr int RS = NP + 4;                       // row stride in floats
  static constexpr int WaveFloats = 3 * RPW * RS;
  static constexpr int WPB = (WaveFloats * 4 * 4 <= 64 * 1024) ? 4 : 1;   // wavefronts per block
  static constexpr int IDXB = ilog2(NP) + 1;              // index (+ sign bit for magnitude)
};

template <int GL, int E, bool MAG, int PC, bool VEC>
__global__ __launch_bounds__((ShortCfg<GL, E>::WPB * kWave)) void short_rows_kernel(
    const float* __restrict__ x, const float* __restrict__ tangent, float* __restrict__ out,
    float* __restrict__ jvp, int64_t rows, int n, int k, Reg R, SparseOut sp) {
  using P = Pool<MAG, PC>;
  using C = ShortCfg<GL, E>;
  constexpr int NP = C::NP, RPW = C::RPW, RS = C::RS, IDXB = C::IDXB;
  constexpr bool CUBIC = (PC == kP43);
  __shared__ __attribute__((aligned(16))) float lds[C::WPB][3][RPW * RS];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int64_t wave = int64_t(blockIdx.x) * C::WPB + wv;
  int64_t row = wave * RPW + lane / GL;
  const bool valid = row < rows;
  if (!valid) row = rows - 1;            // keep the lanes alive for the exchanges; no stores
  const int64_t base = row * n;
  const int e0 = lr * E;
  float* ls = &lds[wv][0][(lane / GL) * RS];
  float* lt = &lds[wv][1][(lane / GL) * RS];
  float* ly = &lds[wv][2][(lane / GL) * RS];

  // ---- load, sort ----------------------------------------------------------------------------
  float xin[E];
  load_row<GL, E, VEC, kStreamRows>(x, base, lr, n, xin);
  if (jvp != nullptr) {
    float tin[E];
    load_row<GL, E, VEC, kStreamRows>(tangent, base, lr, n, tin);
    lds_store_row<GL, E, VEC>(lt, lr, tin);
  }
  double K[E];
  make_keys_row<GL, E, VEC, MAG, IDXB>(xin, lr, n, K);
  SortRuns<GL, E, NP>::run(K, lr);

  float s32[E];
  uint32_t field[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    uint32_t key;
    unpack<IDXB>(K[r], key, field[r]);
    s32[r] = key_to_float(key);
  }
  lds_store<E>(ls + e0, s32);
  __builtin_amdgcn_wave_barrier();

  // ---- isotonic solve: grow the one pooled block outwards from (k, k+1) ----------------------
  // All lanes of a row carry the same (a, b, sums).  A step tests the two neighbours of the block
  // with the strict violation tests of the PAV loop and takes in whichever violates; both may
  // join in one step (the right one raises the pooled value, the left one lowers it, so each
  // still violates after the other has joined).  Values are centred on s_k for the mask.
  int a = k + 1, b = k;                  // 1-based inclusive block [a, b]; empty when a > b
  double center = 0.0, gamma = 0.0;
  if (k >= 1 && k < n) {                 // uniform
    const double sk = double(ls[k - 1]), sk1 = double(ls[k]);
    if (P::kCentered) center = sk;
    const double dk = sk - center, dk1 = sk1 - center;
    bool active = P::seed_violates(dk, dk1, R, center);
    if (__any(active)) {
      Sums S{dk + dk1, 0.0, 0.0};
      if (CUBIC) {
        S.s2 = dk * dk + dk1 * dk1;
        S.s3 = dk * dk * dk + dk1 * dk1 * dk1;
      }
      if (active) { a = k; b = k + 1; }
      const bool grew = active;
      while (__any(active)) {
        const bool can_r = active && b < n, can_l = active && a > 1;
        const double dj = double(ls[can_r ? b : 0]) - center;
        const double di = double(ls[can_l ? a - 2 : 0]) - center;
        const double cnt = double(b - a + 1), m = double(k - a + 1);
        const bool add_r = can_r && P::right_violates(dj, cnt, m, S, R, center);
        const bool add_l = can_l && P::left_violates(di, cnt, m, S, R, center);
        if (add_r) {
          S.s1 += dj;
          if (CUBIC) { S.s2 += dj * dj; S.s3 += dj * dj * dj; }
          b += 1;
        }
        if (add_l) {
          S.s1 += di;
          if (CUBIC) { S.s2 += di * di; S.s3 += di * di * di; }
          a -= 1;
        }
        active = add_r || add_l;
      }
      if (grew) {
        const double da = double(ls[a - 1]) - center, db = double(ls[b - 1]) - center;
        // bracket of the pooled value: above the singleton minimiser of position a (mask:
        // s_a - lambda; magnitude: at least 0), below s_b (magnitude, p = 4/3: below s_a)
        const double lo = MAG ? -center : da - R.lambda;
        gamma = P::pooled(double(b - a + 1), double(k - a + 1), S, R, lo, MAG ? da : db, center);
      }
    }
  }

  // ---- y in sorted order, scattered to the original index (in LDS) ---------------------------
  // Positions before the block keep their singleton solution (mask: exactly 1; magnitude:
  // s/(1+lambda) for p = 2, the root of the one-element cubic for p = 4/3); positions after it
  // are exactly 0.
  if (out != nullptr || sp.idx != nullptr) {
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = e0 + r + 1;
      const double v = double(s32[r]) - center;
      const double yb = P::y_in_block(v, gamma, R);
      const double ya = P::above(v, R, center);
      double y = (pos1 < a) ? ya : yb;
      y = (pos1 > b) ? 0.0 : y;
      float yf = float(y);
      if (MAG) yf = (yf == 0.0f) ? 0.0f : ((field[r] & 1u) ? -yf : yf);
      if (out != nullptr && pos1 <= n) ly[MAG ? (field[r] >> 1) : field[r]] = yf;
      // compact output: the non-zeros are the sorted positions 1..b, in that order
      if (sp.idx != nullptr && valid && pos1 <= sp.max_nnz) {
        const bool nz = pos1 <= b;
        const int64_t o = row * sp.max_nnz + pos1 - 1;
        sp.idx[o] = nz ? int32_t(MAG ? (field[r] >> 1) : field[r]) : -1;
        sp.val[o] = nz ? yf : 0.0f;
      }
    }
    if (sp.idx != nullptr && valid && lr == 0) sp.nnz[row] = b;
  }

  // ---- JVP (Prop. 7): d gamma = weighted block average of the sorted tangent ------------------
  if (jvp != nullptr) {
    double tau[E];
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = e0 + r + 1;
      float tf = 0.0f;
      if (pos1 <= n) tf = lt[MAG ? (field[r] >> 1) : field[r]];
      if (MAG) {
        if (field[r] & 1u) tf = -tf;
        if (s32[r] == 0.0f) tf = 0.0f;         // sign(0) = 0
      }
      tau[r] = double(tf);
    }
    double dgamma = 0.0;
    if (__any(a <= b)) {
      double num = 0.0, wsum = 0.0;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const int pos1 = e0 + r + 1;
        const bool in = pos1 >= a && pos1 <= b;
        const double w = in ? P::jac_weight(double(s32[r]) - center, gamma) : 0.0;
        num += w * tau[r];
        if (CUBIC) wsum += w;
      }
      num = group_sum_f64<GL>(num);
      if (CUBIC) wsum = group_sum_f64<GL>(wsum);
      else wsum = double(b - a + 1);
      if (a <= b) dgamma = num / P::jac_denominator(wsum, double(k - a + 1), R);
    }
    __builtin_amdgcn_wave_barrier();         // every gather of the tangent is done
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const int pos1 = e0 + r + 1;
      const double hb = P::hess(double(s32[r]) - center, gamma, R) * (tau[r] - dgamma);
      const double ha = P::above_slope(double(s32[r]) - center, R, center) * tau[r];
      double dy = (pos1 < a) ? ha : hb;
      dy = (pos1 > b) ? 0.0 : dy;
      float df = float(dy);
      if (MAG) {
        if (s32[r] == 0.0f) df = 0.0f;
        df = (df == 0.0f) ? 0.0f : ((field[r] & 1u) ? -df : df);
      }
      if (pos1 <= n) lt[MAG ? (field[r] >> 1) : field[r]] = df;
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (!valid) return;

  // ---- coalesced stores of the un-sorted rows ---------------------------------------------------
  if (out != nullptr) {
    float yv[E];
    lds_load_row<GL, E, VEC>(ly, lr, yv);
    store_row<GL, E, VEC, kStreamRows>(out, base, lr, n, yv);
  }
  if (jvp != nullptr) {
    float jv[E];
    lds_load_row<GL, E, VEC>(lt, lr, jv);
    store_row<GL, E, VEC, kStreamRows>(jvp, base, lr, n, jv);
  }
}

// ---- Dykstra's alternating projections (Sec. 5, Alg. 1) as an alternative solver ----------------
// p = 2, phi = identity.  The isotonic problem is the Euclidean projection of s - lambda w onto
// the monotone cone C1 n C2 (C1: v_1 >= v_2, v_3 >= v_4, ..; C2: v_2 >= v_3, ..).  The linear term
// is applied once, to the starting point; each iteration is
//     z = v + p,  y = P_C1(z),  p = z - y,   z' = y + q,  v = P_C2(z'),  q = z' - v,
// where a projection replaces every violating pair (z_i < z_{i+1}) by its mean.  Everything stays
// in float64 registers: the C1 pairs lie inside a lane (E is even), the C2 pairs inside a lane or
// between the last position of a lane and the first of the next.  Output (s - v) / lambda.
template <int GL, int E, bool VEC>
__global__ __launch_bounds__((ShortCfg<GL, E>::WPB * kWave)) void dykstra_rows_kernel(
    const float* __restrict__ x, float* __restrict__ out, int64_t rows, int n, int k, double lambda,
    double inv_lambda, int iters) {
  using C = ShortCfg<GL, E>;
  constexpr int NP = C::NP, RPW = C::RPW, RS = C::RS, IDXB = C::IDXB;
  static_assert(E % 2 == 0, "pairs of C1 must not straddle lanes");
  __shared__ __attribute__((aligned(16))) float lds[C::WPB][RPW * RS];

  const int lane = threadIdx.x & (kWave - 1);
  const int lr = lane_in_group<GL>();
  const int wv = threadIdx.x / kWave;
  const int64_t wave = int64_t(blockIdx.x) * C::WPB + wv;
  int64_t row = wave * RPW + lane / GL;
  const bool valid = row < rows;
  if (!valid) row = rows - 1;            // keep the lanes alive for the exchanges; no stores
  const int64_t base = row * n;
  const int e0 = lr * E;
  float* ly = &lds[wv][(lane / GL) * RS];

  float xin[E];
  load_row<GL, E, VEC, kStreamRows>(x, base, lr, n, xin);
  double K[E];
  make_keys_row<GL, E, VEC, false, IDXB>(xin, lr, n, K);
  SortRuns<GL, E, NP>::run(K, lr);

  double s[E], v[E], pc[E], qc[E];
  uint32_t field[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    uint32_t key;
    unpack<IDXB>(K[r], key, field[r]);
    s[r] = double(key_to_float(key));
    v[r] = (e0 + r < k) ? s[r] - lambda : s[r];
    pc[r] = 0.0;
    qc[r] = 0.0;
  }
  // pairs (i, i+1), 0-based sorted positions, exist for i + 1 < n
  const bool pair_up = (GL > 1) && (lr < GL - 1) && (e0 + E < n);   // (last of this lane, first of the next)
  const bool pair_dn = (GL > 1) && (lr > 0) && (e0 < n);            // (last of the previous lane, first of this)
  for (int it = 0; it < iters; ++it) {
    double z[E], y[E];
#pragma unroll
    for (int r = 0; r < E; ++r) { z[r] = v[r] + pc[r]; y[r] = z[r]; }
#pragma unroll
    for (int r = 0; r + 1 < E; r += 2) {
      const bool viol = (e0 + r + 1 < n) && (z[r] < z[r + 1]);
      const double mean = 0.5 * (z[r] + z[r + 1]);
      y[r] = viol ? mean : z[r];
      y[r + 1] = viol ? mean : z[r + 1];
    }
#pragma unroll
    for (int r = 0; r < E; ++r) { pc[r] = z[r] - y[r]; z[r] = y[r] + qc[r]; v[r] = z[r]; }
#pragma unroll
    for (int r = 1; r + 1 < E; r += 2) {
      const bool viol = (e0 + r + 1 < n) && (z[r] < z[r + 1]);
      const double mean = 0.5 * (z[r] + z[r + 1]);
      v[r] = viol ? mean : z[r];
      v[r + 1] = viol ? mean : z[r + 1];
    }
    if constexpr (GL > 1) {
      const double next_first = __shfl_down(z[0], 1, GL);
      const double prev_last = __shfl_up(z[E - 1], 1, GL);
      const bool viol_up = pair_up && (z[E - 1] < next_first);
      const bool viol_dn = pair_dn && (prev_last < z[0]);
      v[E - 1] = viol_up ? 0.5 * (z[E - 1] + next_first) : v[E - 1];
      v[0] = viol_dn ? 0.5 * (prev_last + z[0]) : v[0];
    }
#pragma unroll
    for (int r = 0; r < E; ++r) qc[r] = z[r] - v[r];
  }
#pragma unroll
  for (int r = 0; r < E; ++r)
    if (e0 + r < n) ly[field[r]] = float((s[r] - v[r]) * inv_lambda);
  __builtin_amdgcn_wave_barrier();
  if (!valid) return;
  float yv[E];
  lds_load_row<GL, E, VEC>(ly, lr, yv);
  store_row<GL, E, VEC, kStreamRows>(out, base, lr, n, yv);
}

template <int GL, int E, bool VEC>
int launch_dykstra_shape(const float* x, float* out, int64_t rows, int n, int k, double lambda,
                         int iters, hipStream_t st) {
  using C = ShortCfg<GL, E>;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + C::WPB - 1) / C::WPB;
  if (blocks > 0x7fffffffLL) return -1;
  hipLaunchKernelGGL((dykstra_rows_kernel<GL, E, VEC>), dim3((unsigned)blocks),
                     dim3(C::WPB * kWave), 0, st, x, out, rows, n, k, lambda, 1.0 / lambda, iters);
  return 0;
}

// ---------------------------------------------------------------------------------------------
template <int GL, int E, bool VEC>
int launch_shape(bool mag, int pc, const float* x, const float* t, float* out, float* jvp,
                 int64_t rows, int n, int k, const Reg& R, hipStream_t st,
                 const SparseOut& sp = SparseOut{nullptr, nullptr, nullptr, 0}) {
  using C = ShortCfg<GL, E>;
  const int64_t waves = (rows + C::RPW - 1) / C::RPW;
  const int64_t blocks = (waves + C::WPB - 1) / C::WPB;
  if (blocks > 0x7fffffffLL) return -1;
  dim3 grid((unsigned)blocks), block(C::WPB * kWave);
  if (!mag && pc == kP2)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, false, kP2, VEC>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R, sp);
  else if (!mag && pc == kP43)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, false, kP43, VEC>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R, sp);
  else if (mag && pc == kP2)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, true, kP2, VEC>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R, sp);
  else if (mag && pc == kP43)
    hipLaunchKernelGGL((short_rows_kernel<GL, E, true, kP43, VEC>), grid, block, 0, st, x, t, out, jvp, rows, n, k, R, sp);
  else
    return -1;
  return 0;
}

template <int GL, int E, bool VEC>
int launch_argsort_shape(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st) {
  constexpr int RPW = kWave / GL;
  const int64_t waves = (rows + RPW - 1) / RPW;
  const int64_t blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffLL) return -1;
  hipLaunchKernelGGL((short_argsort_kernel<GL, E, VEC>), dim3((unsigned)blocks), dim3(256), 0, st,
                     x, perm, rows, n);
  return 0;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// log2 of the number of lanes that share a row, for a padded row length np (a power of two).
// Fewer lanes per row mean fewer cross-lane stages of the network and less replicated work in
// the solve, but also fewer wavefronts; with few rows the rows are spread over more lanes so
// that every SIMD of the chip (1024 of them) still gets wavefronts.
int pick_log_gl(int np, int64_t rows) {
  const int forced = routes().short_lanes;             // tuning override: lanes per row
  // smallest allowed log2(GL): at most 8 elements per lane up to 128 padded elements (measured:
  // 16 per lane lose to 8 on both router workloads), at most 16 beyond
  const int emax = np <= 128 ? 8 : 16;
  int lo = 0;
  while ((np >> lo) > emax) ++lo;
  int hi = 0;                                            // largest allowed: E >= min(4, np)
  while ((np >> (hi + 1)) >= 4 && hi < 6) ++hi;
  if (hi < lo) hi = lo;
  if (forced > 0) {
    int lg = 0;
    while ((1 << lg) < forced) ++lg;
    return lg < lo ? lo : (lg > hi ? hi : lg);
  }
  int lg = lo;
  // want at least ~2048 wavefronts when the batch allows it
  while (lg < hi && (rows << lg) / kWave < 2048) ++lg;
  return lg;
}

// A/B switches (topk_set_route): TOPK_SHORT_ROW_KERNEL_GENERAL keeps the general float64-key
// kernels for all shapes, _INDEXED the 32-bit-word kernels that build the permutation also for the
// dense outputs (by default those come from the value-ordering kernel).
bool fast_enabled() { return routes().short_kernel != 2; }
bool value_enabled() { return routes().short_kernel == 0; }

}  // namespace

// Dispatch over (lanes per row GL, elements per lane E) with GL * E = padded row length.
#define TOPK_FOR_SHAPE(GL, E)                                                      \
  if (np == (GL) * (E) && lg == topk::ilog2(GL)) return vec ? CALL(GL, E, true) : CALL(GL, E, false);

#define TOPK_SHAPE_TABLE                                                           \
  TOPK_FOR_SHAPE(1, 4) TOPK_FOR_SHAPE(1, 8) TOPK_FOR_SHAPE(2, 4) TOPK_FOR_SHAPE(1, 16)      \
  TOPK_FOR_SHAPE(2, 8) TOPK_FOR_SHAPE(4, 4) TOPK_FOR_SHAPE(2, 16) TOPK_FOR_SHAPE(4, 8)      \
  TOPK_FOR_SHAPE(8, 4) TOPK_FOR_SHAPE(4, 16) TOPK_FOR_SHAPE(8, 8) TOPK_FOR_SHAPE(16, 4)     \
  TOPK_FOR_SHAPE(8, 16) TOPK_FOR_SHAPE(16, 8) TOPK_FOR_SHAPE(32, 4) TOPK_FOR_SHAPE(16, 16)  \
  TOPK_FOR_SHAPE(32, 8) TOPK_FOR_SHAPE(64, 4) TOPK_FOR_SHAPE(32, 16) TOPK_FOR_SHAPE(64, 8)  \
  TOPK_FOR_SHAPE(64, 16)

int launch_short_rows(bool mag, int pc, const float* x, const float* tangent, float* out,
                      float* jvp, int64_t rows, int n, int k, const Reg& R, hipStream_t st) {
  const bool vec = (n % 4 == 0) && aligned16(x) && aligned16(tangent) && aligned16(out) &&
                   aligned16(jvp);
  int np = 2;
  while (np < n) np <<= 1;
#define CALL(GL, E, V) launch_shape<GL, E, V>(mag, pc, x, tangent, out, jvp, rows, n, k, R, st)
  if (np == 2) return CALL(1, 2, false);
  const int lg = pick_log_gl(np, rows);
  if (np <= 128 && value_enabled()) {
    const int rc = launch_short_rows_value(np, lg, vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    if (rc != -2) return rc;
  }
  if (np <= 128 && fast_enabled()) {
    const int rc = launch_short_rows_fast(np, lg, vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    if (rc != -2) return rc;
  }
  if (np >= 256 && value_enabled()) {
    const int rc = launch_short_rows_value_wide(np, vec, mag, pc, x, tangent, out, jvp, rows, n, k, R, st);
    if (rc != -2) return rc;
  }
  TOPK_SHAPE_TABLE
#undef CALL
  return -1;
}

// The operators built on the mask, fused into the value-ordering kernel of rows up to 2048
// elements (var: 1 signed mask, 2 x o mask(|x|), 3 Fenchel-Young loss with tangent = target and
// out = gradient).  Returns -2 when no fused kernel fits the shape: the caller then runs the
// mask kernels between element-wise passes.
int launch_short_rows_fused_variant(int var, int pc, const float* x, const float* tangent, float* out,
                                    float* jvp, float* loss, double lam_over_p, int64_t rows, int n,
                                    int k, const Reg& R, hipStream_t st) {
  if (!value_enabled()) return -2;
  const bool vec = (n % 4 == 0) && aligned16(x) && aligned16(tangent) && aligned16(out) &&
                   aligned16(jvp);
  int np = 2;
  while (np < n) np <<= 1;
  if (np >= 256 && np <= 2048)
    return launch_short_rows_variant_wide(np, vec, var, pc, x, tangent, out, jvp, loss, lam_over_p,
                                          rows, n, k, R, st);
  if (np < 4 || np > 128) return -2;
  // the kernel's shapes: 1..16 lanes per row with 4 or 8 elements each
  int lg = pick_log_gl(np, rows);
  if (lg > 4 || ((np >> lg) != 4 && (np >> lg) != 8)) lg = np >= 8 ? ilog2(np / 8) : 0;
  return launch_short_rows_variant(np, lg, vec, var, pc, x, tangent, out, jvp, loss, lam_over_p,
                                   rows, n, k, R, st);
}

int launch_short_rows_sparse(int pc, const float* x, int64_t rows, int n, int k, const Reg& R,
                             const SparseOut& sp, hipStream_t st) {
  const bool vec = (n % 4 == 0) && aligned16(x);
  int np = 2;
  while (np < n) np <<= 1;
#define CALL(GL, E, V) \
  launch_shape<GL, E, V>(false, pc, x, nullptr, nullptr, nullptr, rows, n, k, R, st, sp)
  if (np == 2) return CALL(1, 2, false);
  const int lg = pick_log_gl(np, rows);
  if (np <= 128 && fast_enabled()) {
    const int rc = launch_short_rows_fast_sparse(np, lg, vec, pc, x, rows, n, k, R, sp, st);
    if (rc != -2) return rc;
  }
  TOPK_SHAPE_TABLE
#undef CALL
  return -1;
}

int launch_short_dykstra(const float* x, float* out, int64_t rows, int n, int k, double lambda,
                         int iters, hipStream_t st) {
  const bool vec = (n % 4 == 0) && aligned16(x) && aligned16(out);
  int np = 2;
  while (np < n) np <<= 1;
#define CALL(GL, E, V) launch_dykstra_shape<GL, E, V>(x, out, rows, n, k, lambda, iters, st)
  if (np == 2) return CALL(1, 2, false);
  const int lg = pick_log_gl(np, rows);
  TOPK_SHAPE_TABLE
#undef CALL
  return -1;
}

int launch_short_argsort(const float* x, int32_t* perm, int64_t rows, int n, hipStream_t st) {
  const bool vec = (n % 4 == 0) && aligned16(x);
  int np = 2;
  while (np < n) np <<= 1;
#define CALL(GL, E, V) launch_argsort_shape<GL, E, V>(x, perm, rows, n, st)
  if (np == 2) return CALL(1, 2, false);
  const int lg = pick_log_gl(np, rows);
  if (np <= 128 && fast_enabled()) {
    const int rc = launch_short_argsort_fast(np, lg, vec, x, perm, rows, n, st);
    if (rc != -2) return rc;
  }
  TOPK_SHAPE_TABLE
#undef CALL
  return -1;
}

}  // namespace topk
