// Device helpers shared by the MARS kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mars.h"

namespace mars {

constexpr int kWave = 64;

__device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }

// ---------------------------------------------------------------- storage types
// bf16 logits are handled as raw 16-bit patterns; widening to fp32 is a shift.
using bf16_t = uint16_t;

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(bf16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }

// A 16-byte vector of EPV elements (or a single element when EPV == 1), with
// compile-time element access.
template <typename T, int EPV> struct Vec;

// The logits are read exactly once per call: the streaming loads carry the non-temporal hint so
// that they do not displace each other in the caches on their way through.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <> struct Vec<bf16_t, 8> {
  uint4 r;
  __device__ __forceinline__ void load(const bf16_t* row, unsigned int vec) {
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row) + vec);
    r = make_uint4(t.x, t.y, t.z, t.w);
  }
  __device__ __forceinline__ void fill_neg_inf() { r = make_uint4(0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u); }
  __device__ __forceinline__ float get(int e) const {
    const int w = e >> 1;
    const uint32_t word = w == 0 ? r.x : w == 1 ? r.y : w == 2 ? r.z : r.w;
    return __uint_as_float((e & 1) ? (word & 0xFFFF0000u) : (word << 16));
  }
};

template <> struct Vec<bf16_t, 1> {
  bf16_t r;
  __device__ __forceinline__ void load(const bf16_t* row, unsigned int vec) { r = __builtin_nontemporal_load(row + vec); }
  __device__ __forceinline__ void fill_neg_inf() { r = 0xFF80u; }
  __device__ __forceinline__ float get(int) const { return widen(r); }
};

template <> struct Vec<float, 4> {
  float4 r;
  __device__ __forceinline__ void load(const float* row, unsigned int vec) {
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row) + vec);
    r = make_float4(t.x, t.y, t.z, t.w);
  }
  __device__ __forceinline__ void fill_neg_inf() { r = make_float4(neg_inf(), neg_inf(), neg_inf(), neg_inf()); }
  __device__ __forceinline__ float get(int e) const { return e == 0 ? r.x : e == 1 ? r.y : e == 2 ? r.z : r.w; }
};

template <> struct Vec<float, 1> {
  float r;
  __device__ __forceinline__ void load(const float* row, unsigned int vec) { r = __builtin_nontemporal_load(row + vec); }
  __device__ __forceinline__ void fill_neg_inf() { r = neg_inf(); }
  __device__ __forceinline__ float get(int) const { return r; }
};

// ---------------------------------------------------------------- total order (value desc, index asc)
// A 64-bit key whose unsigned order is (value ascending, index descending): the
// largest key is the best candidate.  Key 0 means "no candidate".
__device__ __forceinline__ uint32_t ord_bits(float x) {
  x += 0.0f;  // -0.0 -> +0.0 so that equal values have equal keys
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unord_bits(uint32_t o) {
  return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ unsigned long long make_key(float x, int idx) {
  // ord_bits(-inf) = 0x007FFFFF > 0, so a real candidate never collides with key 0.
  return (static_cast<unsigned long long>(ord_bits(x)) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(idx));
}
__device__ __forceinline__ float key_value(unsigned long long k) { return unord_bits(static_cast<uint32_t>(k >> 32)); }
__device__ __forceinline__ int key_index(unsigned long long k) {
  return static_cast<int>(0xFFFFFFFFu - static_cast<uint32_t>(k & 0xFFFFFFFFull));
}
// Insert a key into a running (k1 >= k2) pair.  Written with selects on the values: as two
// conditional assignments the compiler merges the stores into one store through a selected
// address, which pins k1 and k2 to scratch memory.
__device__ __forceinline__ void top2_insert(unsigned long long& k1, unsigned long long& k2, unsigned long long k) {
  const bool first = k > k1, second = k > k2;
  k2 = first ? k1 : (second ? k : k2);
  k1 = first ? k : k1;
}

// ---------------------------------------------------------------- wave-level reductions (wave64)
// Butterfly inside each row of 16 lanes with DPP (no LDS traffic): xor 1 and xor 2 by quad
// permutes, then the two mirrors; the four row results are combined through readlane.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i inside each group of 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i inside each row of 16

// The value a given lane holds, the lane being the same for the whole wave (a scalar): a register read,
// not a trip through the LDS crossbar as a shuffle with a per-lane source would be.
__device__ __forceinline__ int lane_value(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<kDppXor1>(v));
  v = fmaxf(v, dpp_move<kDppXor2>(v));
  v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_move<kDppMirror>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<kDppXor1>(v);
  v += dpp_move<kDppXor2>(v);
  v += dpp_move<kDppHalfMirror>(v);
  v += dpp_move<kDppMirror>(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const long long bits = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(bits >> 32), CTRL, 0xF, 0xF, true);
  return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}
__device__ __forceinline__ double lane_value(double v, int lane) {
  const long long bits = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_readlane(static_cast<int>(bits), lane);
  const int hi = __builtin_amdgcn_readlane(static_cast<int>(bits >> 32), lane);
  return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move<kDppXor1>(v);
  v += dpp_move<kDppXor2>(v);
  v += dpp_move<kDppHalfMirror>(v);
  v += dpp_move<kDppMirror>(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}
// Inclusive prefix sum over the 64 lanes, lane 0 first: shifts by 1, 2, 4, 8 inside each row of 16 (a lane
// whose source falls outside its row receives 0), then the totals of the rows in front, through readlane.
// No LDS traffic: a tenth of the time of the same scan through cross-lane reads.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
__device__ __forceinline__ double wave_prefix_sum(double v) {
  v += dpp_move<kDppRowShr1>(v);
  v += dpp_move<kDppRowShr2>(v);
  v += dpp_move<kDppRowShr4>(v);
  v += dpp_move<kDppRowShr8>(v);
  const double t0 = lane_value(v, 15), t1 = lane_value(v, 31), t2 = lane_value(v, 47);
  const int row = (threadIdx.x % kWave) >> 4;
  const double t01 = t0 + t1;
  const double front = row == 0 ? 0.0 : (row == 1 ? t0 : (row == 2 ? t01 : t01 + t2));
  return front + v;
}
// Two largest values (with multiplicity) of the union of two pairs a1 >= a2, b1 >= b2.
__device__ __forceinline__ void top2_merge_values(float& a1, float& a2, float b1, float b2) {
  const float lo = fminf(a1, b1);
  a1 = fmaxf(a1, b1);
  a2 = fmaxf(lo, fmaxf(a2, b2));
}
// Merge value-only top-2 pairs (a1 >= a2) across the wave.
__device__ __forceinline__ void wave_top2_values(float& a1, float& a2) {
  top2_merge_values(a1, a2, dpp_move<kDppXor1>(a1), dpp_move<kDppXor1>(a2));
  top2_merge_values(a1, a2, dpp_move<kDppXor2>(a1), dpp_move<kDppXor2>(a2));
  top2_merge_values(a1, a2, dpp_move<kDppHalfMirror>(a1), dpp_move<kDppHalfMirror>(a2));
  top2_merge_values(a1, a2, dpp_move<kDppMirror>(a1), dpp_move<kDppMirror>(a2));
  float r1 = lane_value(a1, 0), r2 = lane_value(a2, 0);
  top2_merge_values(r1, r2, lane_value(a1, 16), lane_value(a2, 16));
  top2_merge_values(r1, r2, lane_value(a1, 32), lane_value(a2, 32));
  top2_merge_values(r1, r2, lane_value(a1, 48), lane_value(a2, 48));
  a1 = r1; a2 = r2;
}

// Partial result of the row reduction for the share of a row one wave streamed.  id < 0 marks
// an absent candidate (a share with fewer than two elements).  s is the partial sum of
// exp2(z * c - ref) over the split; ref is integer-valued, so that sums taken against
// different references are brought together by exact power-of-two scalings.
struct Partial {
  float   z1;
  int32_t id1;
  float   z2;
  int32_t id2;
  float   s;
  float   ref;
};

// 2^x for a double argument, to fp32 accuracy whatever the magnitude of x: the integer part is
// applied exactly, the fraction in [-1/2, 1/2] goes through one fp32 exp2.
__device__ __forceinline__ float exp2_split(double x) {
  if (!(x > -400.0)) return 0.0f;
  const double n = rint(x);
  const float frac = static_cast<float>(x - n);
  return static_cast<float>(ldexp(static_cast<double>(__builtin_amdgcn_exp2f(frac)), static_cast<int>(n)));
}

// The low-margin test on the two largest logits of a row (Sec. 3.3), strict, against the
// request's threshold.  cind = log2(e) / T' with T' the sampling temperature, or 1 in greedy mode.
//   logit ratio (Eq. 4):  z1 > 0 and z2/z1 > theta, one correctly rounded fp32 division; no
//                         relaxation outside the positive domain the paper assumes for z(1)
//   probability ratio:    P(v2)/P(v1) = exp(-(z1 - z2)/T') > theta
//   fixed margin:         Delta = z1 - z2 < theta (Delta of Eq. 5, one rounded fp32 subtraction)
struct Indicator {
  int kind;      // mars_indicator
  double cind;
};
__device__ __forceinline__ float prob_ratio(float z1, float z2, double cind) {
  return exp2_split(-static_cast<double>(__fsub_rn(z1, z2)) * cind);
}
__device__ __forceinline__ int low_margin(float z1, float z2, float theta, const Indicator& ind) {
  if (ind.kind == MARS_IND_PROB_RATIO) return prob_ratio(z1, z2, ind.cind) > theta ? 1 : 0;
  if (ind.kind == MARS_IND_LOGIT_GAP) return __fsub_rn(z1, z2) < theta ? 1 : 0;
  return (z1 > 0.0f && (z2 / z1) > theta) ? 1 : 0;
}

// Finish one row: the merged keys and the sum S (relative to the integer reference R) become
// the public statistics entry.  Moving the reference to the row maximum needs the only
// exponential of the merge, of an argument split into its integer part (exact) and a
// fraction in [-1/2, 1/2] (one fp32 exp2).
__device__ __forceinline__ mars_row_stat finish_row(unsigned long long k1, unsigned long long k2, float R, double S,
                                                    float theta, float c, const Indicator& ind) {
  const float z1 = key_value(k1), z2 = key_value(k2);
  float sum_exp = 0.0f;
  if (c > 0.0f && S > 0.0) {
    // S * 2^(R - z1*c)
    const double d = static_cast<double>(R) - static_cast<double>(z1) * static_cast<double>(c);
    const double n = rint(d);
    const float frac = static_cast<float>(d - n);
    sum_exp = static_cast<float>(ldexp(S * static_cast<double>(__builtin_amdgcn_exp2f(frac)), static_cast<int>(n)));
  }
  mars_row_stat st;
  st.z1 = z1; st.id1 = key_index(k1);
  st.z2 = z2; st.id2 = key_index(k2);
  st.sum_exp = sum_exp;
  st.relax_ok = low_margin(z1, z2, theta, ind);
  return st;
}

// Sum S (relative to reference R) absorbs a partial sum s taken against reference ref; both
// references are integers, so the scalings are exact powers of two.
__device__ __forceinline__ void absorb_sum(float& R, double& S, float ref, double s) {
  if (ref > R) {
    S *= static_cast<double>(__builtin_ldexpf(1.0f, static_cast<int>(fmaxf(R - ref, -140.0f))));
    R = ref;
  }
  S += s * static_cast<double>(__builtin_ldexpf(1.0f, static_cast<int>(fmaxf(ref - R, -140.0f))));
}

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_move(unsigned long long v) {
  const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, true);
  const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(v >> 32), CTRL, 0xF, 0xF, true);
  return (static_cast<unsigned long long>(static_cast<unsigned int>(hi)) << 32) | static_cast<unsigned int>(lo);
}

// Cooperative merge of the partial results of rows [0, nrows): sixteen consecutive lanes (one
// DPP row) take one row, each lane reads every sixteenth partial (coalesced, one round trip
// when a row has at most sixteen), and a butterfly inside the DPP row merges keys and sums.
// Every lane of the sixteen ends with the row's result; lane 0 of them hands it to `emit`.
// Must be called by all NT threads of the work-group (NT a multiple of 64).
constexpr int kMergeBatch = 4;  // partial results a lane has in flight at a time (a kernel with registers to spare: 8)
// Partial results s0, s0 + 16, ... of one row (empty ones past the end, or for a row that does not exist).
template <int BATCH>
__device__ __forceinline__ void load_partials(const Partial* __restrict__ partials, int row, int nrows, int parts,
                                              int s0, Partial (&q)[BATCH]) {
  const Partial* __restrict__ p = partials + static_cast<size_t>(row) * parts;
#pragma unroll
  for (int j = 0; j < BATCH; ++j) {
    const int s = s0 + 16 * j;
    if (row < nrows && s < parts) {
      q[j] = p[s];
    } else {
      q[j].id1 = -1; q[j].id2 = -1; q[j].s = 0.0f; q[j].z1 = 0.0f; q[j].z2 = 0.0f; q[j].ref = 0.0f;
    }
  }
}
// One butterfly step of a merge over lanes: every lane absorbs what its partner under CTRL holds.  (All
// lanes take part; the two sides hold disjoint sets of elements, so no key is inserted twice.)
template <int CTRL>
__device__ __forceinline__ void merge_step(unsigned long long& k1, unsigned long long& k2, float& R, double& S) {
  const unsigned long long o1 = dpp_move<CTRL>(k1), o2 = dpp_move<CTRL>(k2);
  const float oR = dpp_move<CTRL>(R);
  const double oS = dpp_move<CTRL>(S);
  top2_insert(k1, k2, o1);
  top2_insert(k1, k2, o2);
  if (oS > 0.0) absorb_sum(R, S, oR, oS);
}

// The first `parts` (<= COUNT) partial results of one row, empty ones behind them.
template <int COUNT>
__device__ __forceinline__ void load_partials_of_row(const Partial* __restrict__ p, int parts, Partial (&q)[COUNT]) {
#pragma unroll
  for (int j = 0; j < COUNT; ++j) {
    if (j < parts) {
      q[j] = p[j];
    } else {
      q[j].id1 = -1; q[j].id2 = -1; q[j].s = 0.0f; q[j].z1 = 0.0f; q[j].z2 = 0.0f; q[j].ref = 0.0f;
    }
  }
}
template <int BATCH>
__device__ __forceinline__ void fold_partials(const Partial (&q)[BATCH], float c, unsigned long long& k1,
                                              unsigned long long& k2, float& R, double& S) {
#pragma unroll
  for (int j = 0; j < BATCH; ++j) {
    if (q[j].id1 >= 0) top2_insert(k1, k2, make_key(q[j].z1, q[j].id1));
    if (q[j].id2 >= 0) top2_insert(k1, k2, make_key(q[j].z2, q[j].id2));
    if (c > 0.0f && q[j].s > 0.0f) absorb_sum(R, S, q[j].ref, static_cast<double>(q[j].s));
  }
}

// A row with at most kFewParts partial results, merged by one thread.
constexpr int kFewParts = 4;
__device__ __forceinline__ mars_row_stat merge_row_few(const Partial (&q)[kFewParts], float c, const Indicator& ind,
                                                       float theta) {
  unsigned long long k1 = 0, k2 = 0;
  float R = -3.0e38f;
  double S = 0.0;
  fold_partials(q, c, k1, k2, R, S);
  return finish_row(k1, k2, R, S, theta, c, ind);
}

template <int NT, int BATCH = kMergeBatch, typename ThetaAt, typename Emit>
__device__ __forceinline__ void merge_rows_coop(const Partial* __restrict__ partials, int nrows, int parts,
                                                float c, const Indicator& ind, ThetaAt theta_at, Emit emit) {
  // Few partial results per row (the row reduction leaves one per split): a thread per row, one round
  // trip to memory for all of them.
  if (parts <= kFewParts) {
    for (int row = threadIdx.x; row < nrows; row += NT) {
      Partial q[kFewParts];
      load_partials_of_row(partials + static_cast<size_t>(row) * parts, parts, q);
      emit(row, merge_row_few(q, c, ind, theta_at(row)));
    }
    return;
  }
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  constexpr int kGroups = NT / 16;
  // A lane has BATCH loads in flight at a time, and the first batch of the next pass over the
  // rows is requested before the current pass is worked on: merging N rows costs about one memory
  // round trip, not one per pass.
  Partial nxt[BATCH];
  load_partials(partials, grp, nrows, parts, sub, nxt);
  for (int row0 = 0; row0 < nrows; row0 += kGroups) {
    const int row = row0 + grp;
    const bool live = row < nrows;
    unsigned long long k1 = 0, k2 = 0;
    float R = -3.0e38f;
    double S = 0.0;
    Partial cur[BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) cur[j] = nxt[j];
    load_partials(partials, row + kGroups, nrows, parts, sub, nxt);
    fold_partials(cur, c, k1, k2, R, S);
    for (int s0 = sub + 16 * BATCH; s0 < parts; s0 += 16 * BATCH) {
      load_partials(partials, row, nrows, parts, s0, cur);
      fold_partials(cur, c, k1, k2, R, S);
    }
    // Butterfly over the sixteen lanes: at every step the two sides hold disjoint sets of
    // elements, so no key can be inserted twice.  (All lanes take part; dead rows carry nothing.)
    merge_step<kDppXor1>(k1, k2, R, S);
    merge_step<kDppXor2>(k1, k2, R, S);
    merge_step<kDppHalfMirror>(k1, k2, R, S);
    merge_step<kDppMirror>(k1, k2, R, S);
    if (live && sub == 0) emit(row, finish_row(k1, k2, R, S, theta_at(row), c, ind));
  }
}

}  // namespace mars
