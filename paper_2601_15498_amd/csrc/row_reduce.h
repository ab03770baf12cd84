// Row reduction: per (row, split) the two largest logits with their indices under
// (value desc, index asc) and, in sampling mode, the sum of exp((z - ref)/T).
// One streaming read of the logits; this is the HBM-bound kernel of the pass
// (paper Sec. 3.3 top-2 identification, Eq. 3 softmax normaliser).
//
// Per element the lane does value-only work: widen, a (max, second max) update and,
// when sampling, one fma + exp2 + add.  Indices are recovered afterwards: each lane
// remembers in which batch its two best values first appeared, and only the few
// lanes that hold a row-level candidate reload that one batch to find the position.
#pragma once

#include "common.h"

namespace mars {

constexpr int kRowThreads = 256;  // 4 waves per work-group
constexpr int kUnroll = 4;        // 16-byte loads per lane per batch
constexpr float kRescaleLog2 = 24.0f;  // rescale the sum-exp reference when the max rises by 2^24

// (m1 >= m2) <- the two largest of {m1, m2, x}: m2 = median(m1, m2, x), m1 = max(m1, x).
// Written as one two-instruction block so that the pair stays together: left to itself the
// scheduler hoists the whole max chain and keeps every intermediate maximum alive for the
// medians, which triples the register count of the loop.
__device__ __forceinline__ void top2_update(float& m1, float& m2, float x) {
  asm("v_med3_f32 %1, %0, %1, %2\n\tv_max_f32 %0, %0, %2" : "+v"(m1), "+v"(m2) : "v"(x));
}

// Position (within the lane's batch) of the first element equal to `target`, other than
// position `skip`; -1 if none.  Positions are j * EPV + e, ascending in vocabulary index.
template <typename T, int EPV>
__device__ int find_in_batch(const T* __restrict__ rowp, int v_begin, int v_end, int batch, int tid,
                             float target, int skip) {
  int found = -1;
  for (int j = kUnroll - 1; j >= 0; --j) {
    const int vec = v_begin + (batch * kUnroll + j) * kRowThreads + tid;
    if (vec < v_end) {
      Vec<T, EPV> v;
      v.load(rowp, vec);
#pragma unroll
      for (int e = EPV - 1; e >= 0; --e) {
        const int pos = j * EPV + e;
        if (v.get(e) == target && pos != skip) found = pos;
      }
    }
  }
  return found;
}

template <typename T, int EPV, bool SAMPLING>
__global__ __launch_bounds__(kRowThreads) void row_reduce_kernel(const T* __restrict__ logits, int V, int splits,
                                                                  int vecs_per_split, float c,
                                                                  Partial* __restrict__ partials) {
  constexpr int U = kUnroll;
  constexpr int BV = kRowThreads * U;  // vectors per batch
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

  float m1 = neg_inf(), m2 = neg_inf();  // the lane's two largest values so far (with multiplicity)
  int b1 = -1, b2 = -1;                  // batch in which each first appeared
  float s = 0.0f;                        // sum of exp2(z*c - ref_c) over the lane's elements
  float ref_c = -1.0e30f;                // wave-uniform reference, already multiplied by c
  float thresh = -3.0e38f;               // rescale when a lane max exceeds this (wave-uniform)
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
      if (vec < v_end) buf[j].load(rowp, vec); else buf[j].fill_neg_inf();
    }
  };

  auto process = [&](const Vec<T, EPV>(&buf)[U], int k) {
    const float o1 = m1, o2 = m2;
    float x[U * EPV];
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
      for (int e = 0; e < EPV; ++e) x[j * EPV + e] = buf[j].get(e);
#pragma unroll
    for (int i = 0; i < U * EPV; ++i) top2_update(m1, m2, x[i]);
    // Where did the lane's two best values first appear?  A new maximum demotes the old one,
    // whose first occurrence stays where it was; anything else that raises m2 is in this batch.
    const bool gt = m1 > o1;
    const bool ch2 = m2 > o2;
    const int nb2 = (gt && m2 == o1) ? b1 : k;
    b2 = ch2 ? nb2 : b2;
    b1 = gt ? k : b1;
    if (SAMPLING) {
      if (__any(m1 > thresh)) {
        // Rare: the wave's maximum rose by more than 2^kRescaleLog2 above the reference (or this
        // is the wave's first batch).  Move the reference to the wave maximum before any term of
        // this batch is formed, so that no exponent ever exceeds kRescaleLog2.
        const float wm = wave_max(m1);
        const float new_ref_c = wm * c;
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
  __shared__ float sh_m1[kRowThreads / kWave], sh_m2[kRowThreads / kWave];
  __shared__ float sh_ref[kRowThreads / kWave], sh_sum[kRowThreads / kWave];
  __shared__ unsigned long long sh_cand[2 * kRowThreads];
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
  float Z1 = sh_m1[0], Z2 = sh_m2[0];
#pragma unroll
  for (int w = 1; w < kRowThreads / kWave; ++w) {
    const float c1 = sh_m1[w], c2 = sh_m2[w];
    const float lo = fminf(Z1, c1);
    Z1 = fmaxf(Z1, c1);
    Z2 = fmaxf(lo, fmaxf(Z2, c2));
  }
  // Z1 >= Z2 are the split's two largest values.  Lanes holding a value >= Z2 recover the
  // index of that element from the batch they remembered.  -inf entries (masked tokens,
  // padding) are never searched: among them the order is the index order, known in closed form.
  const bool finite2 = Z2 > neg_inf();
  const float cut = finite2 ? Z2 : Z1;
  if (cut > neg_inf() && m1 >= cut) {
    const int p1 = find_in_batch<T, EPV>(rowp, v_begin, v_end, b1, tid, m1, -1);
    const int vec1 = v_begin + (b1 * U + p1 / EPV) * kRowThreads + tid;
    const int slot = atomicAdd(&sh_ncand, 1);
    sh_cand[slot] = make_key(m1, vec1 * EPV + p1 % EPV);
    if (finite2 && m2 >= cut) {
      const int p2 = find_in_batch<T, EPV>(rowp, v_begin, v_end, b2, tid, m2, b2 == b1 ? p1 : -1);
      const int vec2 = v_begin + (b2 * U + p2 / EPV) * kRowThreads + tid;
      const int slot2 = atomicAdd(&sh_ncand, 1);
      sh_cand[slot2] = make_key(m2, vec2 * EPV + p2 % EPV);
    }
  }
  __syncthreads();
  if (tid == 0) {
    unsigned long long k1 = 0, k2 = 0;
    const int n = sh_ncand;
    for (int i = 0; i < n; ++i) top2_insert(k1, k2, sh_cand[i]);
    const int first = v_begin * EPV, count = nv * EPV;
    Partial out;
    out.z1 = neg_inf(); out.id1 = -1; out.z2 = neg_inf(); out.id2 = -1; out.s = 0.0f; out.pad = 0;
    if (count > 0) {
      if (k1 != 0) { out.z1 = key_value(k1); out.id1 = key_index(k1); }
      else { out.id1 = first; }  // every element is -inf
      if (k2 != 0) { out.z2 = key_value(k2); out.id2 = key_index(k2); }
      else if (count > 1) { out.id2 = (out.id1 == first) ? first + 1 : first; }  // runner-up is a -inf entry
    }
    if (SAMPLING && out.z1 > neg_inf()) {
      const double z1c = static_cast<double>(out.z1) * static_cast<double>(c);
      double S = 0.0;
#pragma unroll
      for (int w = 0; w < kRowThreads / kWave; ++w)
        if (sh_sum[w] > 0.0f) S += static_cast<double>(sh_sum[w]) * exp2(static_cast<double>(sh_ref[w]) - z1c);
      out.s = static_cast<float>(S);
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
