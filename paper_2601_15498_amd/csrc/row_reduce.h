// Row reduction: per (row, split) the two largest logits with their indices under
// (value desc, index asc) and, in sampling mode, the sum of exp2(z*c - ref).
// One streaming read of the logits; this is the HBM-bound kernel of the pass
// (paper Sec. 3.3 top-2 identification, Eq. 3 softmax normaliser).
//
// The per-element work is kept to the minimum the arithmetic units can hide behind the
// memory stream: widen, half a max3 and, when sampling, one fma + exp2 + add.  A lane only
// tracks the maxima of its batches (32 elements each): the best and second-best batch
// maximum and the batches they came from.  A lane's two largest elements are then known to
// lie in those two batches, so after the stream the few lanes that can hold a row-level
// candidate reload one or two batches and produce exact (value, index) pairs.
#pragma once

#include "common.h"

namespace mars {

#ifndef MARS_ROW_THREADS
#define MARS_ROW_THREADS 256
#endif
#ifndef MARS_ROW_UNROLL
#define MARS_ROW_UNROLL 4
#endif
constexpr int kRowThreads = MARS_ROW_THREADS;  // 4 waves per work-group
constexpr int kUnroll = MARS_ROW_UNROLL;       // 16-byte loads per lane per batch
constexpr float kRescaleLog2 = 24.0f;  // move the sum-exp reference when the max rises by 2^24

// Exact (value desc, index asc) top-2 among the elements >= cut of the lane's batches b1 and
// (when two == true) b2, merged into (k1, k2).  All loads are issued before the first use: the
// rescan sits at the very end of a work-group's life, where a dependent round trip per vector
// would be paid in full.
template <typename T, int EPV>
__device__ void scan_batches(const T* __restrict__ rowp, int v_begin, int v_end, int b1, int b2, bool two, int tid,
                             float cut, unsigned long long& k1, unsigned long long& k2) {
  Vec<T, EPV> va[kUnroll], vb[kUnroll];
#pragma unroll
  for (int j = 0; j < kUnroll; ++j) {
    const int veca = v_begin + (b1 * kUnroll + j) * kRowThreads + tid;
    if (veca < v_end) va[j].load(rowp, static_cast<unsigned int>(veca)); else va[j].fill_neg_inf();
    const int vecb = v_begin + (b2 * kUnroll + j) * kRowThreads + tid;
    if (two && vecb < v_end) vb[j].load(rowp, static_cast<unsigned int>(vecb)); else vb[j].fill_neg_inf();
  }
  // Only a vector whose maximum reaches the cut is looked at element by element (normally one
  // or two of them): the insertions are a serial chain run by a wave with one or two live lanes.
  auto scan_vec = [&](const Vec<T, EPV>& v, int vec) {
    float vm = v.get(0);
#pragma unroll
    for (int e = 1; e < EPV; ++e) vm = fmaxf(vm, v.get(e));
    if (vm >= cut) {
#pragma unroll
      for (int e = 0; e < EPV; ++e) {
        const float x = v.get(e);
        if (x >= cut) top2_insert(k1, k2, make_key(x, vec * EPV + e));
      }
    }
  };
#pragma unroll
  for (int j = 0; j < kUnroll; ++j) scan_vec(va[j], v_begin + (b1 * kUnroll + j) * kRowThreads + tid);
#pragma unroll
  for (int j = 0; j < kUnroll; ++j) scan_vec(vb[j], v_begin + (b2 * kUnroll + j) * kRowThreads + tid);
}

template <typename T, int EPV, bool SAMPLING>
__global__ __launch_bounds__(kRowThreads) void row_reduce_kernel(const T* __restrict__ logits, int V, int splits,
                                                                  int vecs_per_split, float c,
                                                                  Partial* __restrict__ partials,
                                                                  unsigned long long* __restrict__ xslots, int N, int xwords) {
  constexpr int U = kUnroll;
  constexpr int BV = kRowThreads * U;  // vectors per batch
  constexpr int NE = U * EPV;          // elements per lane per batch
  constexpr int NW = kRowThreads / kWave;
  const int item = blockIdx.x;
  const int row = item / splits;
  const int split = item - row * splits;
  const T* __restrict__ rowp = logits + static_cast<size_t>(row) * static_cast<size_t>(V);
  const int nvec = V / EPV;
  const int v_begin = min(nvec, split * vecs_per_split);
  const int v_end = min(nvec, v_begin + vecs_per_split);
  const int nv = v_end - v_begin;
  const int tid = threadIdx.x;
  const int nb = (nv + BV - 1) / BV;
  const int nfull = nv / BV;  // batches that need no bounds check

  // Exchange words of the tail kernel that follows on the stream (xwords per (request, exchange),
  // N + 2 exchanges per request): cleared here so that the call needs no separate memset.
  if (split == 0 && tid < xwords) {
    const int b = row / N, i = row - b * N;
    unsigned long long* cells = xslots + static_cast<size_t>(b) * (N + 2) * xwords;
    cells[static_cast<size_t>(i) * xwords + tid] = 0ull;
    if (i == 0) {
      cells[static_cast<size_t>(N) * xwords + tid] = 0ull;
      cells[static_cast<size_t>(N + 1) * xwords + tid] = 0ull;
    }
  }

  float m1 = neg_inf(), m2 = neg_inf();  // best and second-best batch maximum of this lane
  int b1 = -1, b2 = -1;                  // the (distinct) batches they belong to
  float s = 0.0f;                        // sum of exp2(z*c - ref_c) over the lane's elements
  float ref_c = -1.0e30f;                // wave-uniform, integer-valued reference (already times c)
  float thresh = -3.0e38f;               // rescale when a lane maximum exceeds this (wave-uniform)
  const float tau_over_c = SAMPLING ? kRescaleLog2 / c : 0.0f;

  Vec<T, EPV> bufA[U], bufB[U];

  // Unconditional loads for a full batch; bounds-checked loads (padding with -inf) for the last one.
  auto load_full = [&](Vec<T, EPV>(&buf)[U], int k) {
    const T* __restrict__ bp = rowp + static_cast<size_t>(v_begin + k * BV) * EPV;  // wave-uniform
#pragma unroll
    for (int j = 0; j < U; ++j) buf[j].load(bp, static_cast<unsigned int>(tid + j * kRowThreads));
  };
  auto load_tail = [&](Vec<T, EPV>(&buf)[U], int k) {
    const int base = v_begin + k * BV + tid;
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const int vec = base + j * kRowThreads;
      if (vec < v_end) buf[j].load(rowp, static_cast<unsigned int>(vec)); else buf[j].fill_neg_inf();
    }
  };

  auto process = [&](const Vec<T, EPV>(&buf)[U], int k) {
    float x[NE];
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
      for (int e = 0; e < EPV; ++e) x[j * EPV + e] = buf[j].get(e);
    // batch maximum: max3 over pairs, two independent chains
    float bm;
    if (NE >= 4) {
      float ma = fmaxf(x[0], x[1]), mb = fmaxf(x[2], x[3]);
#pragma unroll
      for (int i = 4; i + 3 < NE; i += 4) {
        ma = fmaxf(fmaxf(ma, x[i]), x[i + 1]);
        mb = fmaxf(fmaxf(mb, x[i + 2]), x[i + 3]);
      }
      bm = fmaxf(ma, mb);
    } else {
      bm = x[0];
#pragma unroll
      for (int i = 1; i < NE; ++i) bm = fmaxf(bm, x[i]);
    }
    // Best and second-best batch maximum, first occurrence wins ties (later batches have
    // higher vocabulary indices).  A new best demotes the old one.
    const bool gt = bm > m1;
    const bool g2 = bm > m2;
    m2 = gt ? m1 : (g2 ? bm : m2);
    b2 = gt ? b1 : (g2 ? k : b2);
    m1 = gt ? bm : m1;
    b1 = gt ? k : b1;
    if (SAMPLING) {
      if (__any(m1 > thresh)) {
        // Rare: the wave's maximum rose more than 2^kRescaleLog2 above the reference (or this is
        // the wave's first batch).  Move the reference up to the wave maximum, rounded up to an
        // integer, before any term of this batch is formed: no exponent ever exceeds
        // kRescaleLog2, and references differ by exact powers of two.
        const float wm = wave_max(m1);
        const float new_ref_c = __builtin_ceilf(wm * c);
        s *= __builtin_amdgcn_exp2f(ref_c - new_ref_c);
        ref_c = new_ref_c;
        thresh = wm + tau_over_c;
      }
      float bs[U];
#pragma unroll
      for (int j = 0; j < U; ++j) {
        bs[j] = 0.0f;
#pragma unroll
        for (int e = 0; e < EPV; ++e) bs[j] += __builtin_amdgcn_exp2f(__builtin_fmaf(x[j * EPV + e], c, -ref_c));
      }
      float t = bs[0];
#pragma unroll
      for (int j = 1; j < U; ++j) t += bs[j];
      s += t;
    }
  };

  // Double-buffered stream over the full batches: the loads of batch k+1 are in flight while
  // batch k is processed.  The ragged last batch (if any) is loaded with bounds checks.
  const bool has_tail = nb > nfull;
  int k = 0;
  if (nfull > 0) {
    load_full(bufA, 0);
    for (; k + 2 < nfull; k += 2) {
      load_full(bufB, k + 1);
      process(bufA, k);
      load_full(bufA, k + 2);
      process(bufB, k + 1);
    }
    // one or two full batches left; bufA holds batch k
    if (k + 1 < nfull) {
      load_full(bufB, k + 1);
      process(bufA, k);
      if (has_tail) load_tail(bufA, nfull);
      process(bufB, k + 1);
      if (has_tail) process(bufA, nfull);
    } else {
      if (has_tail) load_tail(bufB, nfull);
      process(bufA, k);
      if (has_tail) process(bufB, nfull);
    }
  } else if (has_tail) {
    load_tail(bufA, 0);
    process(bufA, 0);
  }

  // ------------------------------------------------------------------ work-group epilogue
  __shared__ float sh_m1[NW], sh_m2[NW], sh_ref[NW], sh_sum[NW];
  __shared__ unsigned long long sh_cand[4 * kRowThreads];
  __shared__ int sh_ncand;

  const int wave = tid / kWave, lane = tid % kWave;
  float w1 = m1, w2 = m2;
  wave_top2_values(w1, w2);
  float ws = 0.0f;
  if (SAMPLING) ws = wave_sum(s);
  if (lane == 0) {
    sh_m1[wave] = w1; sh_m2[wave] = w2;
    sh_ref[wave] = ref_c; sh_sum[wave] = ws;
  }
  if (tid == 0) sh_ncand = 0;
  __syncthreads();
  float Z1 = sh_m1[0], L2 = sh_m2[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) top2_merge_values(Z1, L2, sh_m1[w], sh_m2[w]);
  // Z1 is the split's maximum; L2, the second largest batch maximum over all lanes, is a lower
  // bound of its runner-up.  Every element >= L2 lies in batch b1 or b2 of a lane whose own
  // maxima reach L2; those lanes rescan.  -inf entries (masked tokens, padding) are never
  // searched: among them the order is the index order, known in closed form.
  // (L2 == -inf only says that a single lane saw finite values in a single batch; the runner-up
  // may still be finite inside that batch, so the scan then takes every finite element.)
  const float cut = L2 > neg_inf() ? L2 : -3.4028235e38f;
  if (Z1 > neg_inf() && m1 >= cut) {
    unsigned long long k1 = 0, k2 = 0;
    scan_batches<T, EPV>(rowp, v_begin, v_end, b1, b2, m2 >= cut, tid, cut, k1, k2);
    const int n = (k1 != 0) + (k2 != 0);
    const int slot = atomicAdd(&sh_ncand, n);
    if (k1 != 0) sh_cand[slot] = k1;
    if (k2 != 0) sh_cand[slot + 1] = k2;
  }
  __syncthreads();
  if (tid == 0) {
    unsigned long long k1 = 0, k2 = 0;
    const int n = sh_ncand;
    for (int i = 0; i < n; ++i) top2_insert(k1, k2, sh_cand[i]);
    const int first = v_begin * EPV, count = nv * EPV;
    Partial out;
    out.z1 = neg_inf(); out.id1 = -1; out.z2 = neg_inf(); out.id2 = -1; out.s = 0.0f; out.ref = 0.0f;
    if (count > 0) {
      if (k1 != 0) { out.z1 = key_value(k1); out.id1 = key_index(k1); }
      else { out.id1 = first; }  // every element is -inf
      if (k2 != 0) { out.z2 = key_value(k2); out.id2 = key_index(k2); }
      else if (count > 1) { out.id2 = (out.id1 == first) ? first + 1 : first; }  // runner-up is a -inf entry
    }
    if (SAMPLING) {
      float R = -3.0e38f;
#pragma unroll
      for (int w = 0; w < NW; ++w)
        if (sh_sum[w] > 0.0f) R = fmaxf(R, sh_ref[w]);
      float S = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w)  // exact power-of-two scalings
        if (sh_sum[w] > 0.0f) S += __builtin_ldexpf(sh_sum[w], static_cast<int>(fmaxf(sh_ref[w] - R, -300.0f)));
      out.s = S; out.ref = S > 0.0f ? R : 0.0f;
    }
    partials[item] = out;
  }
}

// One thread per row: merge the splits into the statistics table.
__global__ void merge_stats_kernel(const Partial* __restrict__ partials, int rows, int N, int splits,
                                   const float* __restrict__ theta, float c, mars_row_stat* __restrict__ stats) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < rows) merge_row(partials + static_cast<size_t>(r) * splits, splits, theta[r / N], c, &stats[r]);
}

}  // namespace mars
