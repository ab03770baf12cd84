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

template <> struct Vec<bf16_t, 8> {
  uint4 r;
  __device__ __forceinline__ void load(const bf16_t* row, unsigned int vec) {
    r = reinterpret_cast<const uint4*>(row)[vec];
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
  __device__ __forceinline__ void load(const bf16_t* row, unsigned int vec) { r = row[vec]; }
  __device__ __forceinline__ void fill_neg_inf() { r = 0xFF80u; }
  __device__ __forceinline__ float get(int) const { return widen(r); }
};

template <> struct Vec<float, 4> {
  float4 r;
  __device__ __forceinline__ void load(const float* row, unsigned int vec) {
    r = reinterpret_cast<const float4*>(row)[vec];
  }
  __device__ __forceinline__ void fill_neg_inf() { r = make_float4(neg_inf(), neg_inf(), neg_inf(), neg_inf()); }
  __device__ __forceinline__ float get(int e) const { return e == 0 ? r.x : e == 1 ? r.y : e == 2 ? r.z : r.w; }
};

template <> struct Vec<float, 1> {
  float r;
  __device__ __forceinline__ void load(const float* row, unsigned int vec) { r = row[vec]; }
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
// Insert a key into a running (k1 >= k2) pair.
__device__ __forceinline__ void top2_insert(unsigned long long& k1, unsigned long long& k2, unsigned long long k) {
  if (k > k1) { k2 = k1; k1 = k; }
  else if (k > k2) { k2 = k; }
}

// ---------------------------------------------------------------- wave-level reductions (wave64)
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
// Merge value-only top-2 pairs (a1 >= a2) across the wave: the two largest values
// of the union, with multiplicity.
__device__ __forceinline__ void wave_top2_values(float& a1, float& a2) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const float b1 = __shfl_xor(a1, m, kWave);
    const float b2 = __shfl_xor(a2, m, kWave);
    const float lo = fminf(a1, b1);
    a1 = fmaxf(a1, b1);
    a2 = fmaxf(lo, fmaxf(a2, b2));
  }
}

// Per-(row, split) partial result of the row reduction.  id < 0 marks an absent
// candidate (a split with fewer than two elements).  s is the partial sum of
// exp2((z - z1) * c) over the split, relative to the split's own z1.
struct Partial {
  float   z1;
  int32_t id1;
  float   z2;
  int32_t id2;
  float   s;
  int32_t pad;
};

// Merge the splits of one row into the public statistics entry.
// c = log2(e) / T (0 in greedy mode).
__device__ __forceinline__ void merge_row(const Partial* __restrict__ p, int splits, float theta, float c,
                                          mars_row_stat* __restrict__ out) {
  unsigned long long k1 = 0, k2 = 0;
  for (int s = 0; s < splits; ++s) {
    if (p[s].id1 >= 0) top2_insert(k1, k2, make_key(p[s].z1, p[s].id1));
    if (p[s].id2 >= 0) top2_insert(k1, k2, make_key(p[s].z2, p[s].id2));
  }
  const float z1 = key_value(k1), z2 = key_value(k2);
  double S = 0.0;
  if (c > 0.0f) {
    for (int s = 0; s < splits; ++s)
      if (p[s].s > 0.0f)
        S += static_cast<double>(p[s].s) *
             exp2((static_cast<double>(p[s].z1) - static_cast<double>(z1)) * static_cast<double>(c));
  }
  mars_row_stat st;
  st.z1 = z1; st.id1 = key_index(k1);
  st.z2 = z2; st.id2 = key_index(k2);
  st.sum_exp = static_cast<float>(S);
  // Eq. 4 and the strict test r > theta, one correctly rounded fp32 division; no
  // relaxation outside the positive domain the paper assumes for z(1).
  st.relax_ok = (z1 > 0.0f && (z2 / z1) > theta) ? 1 : 0;
  *out = st;
}

}  // namespace mars
