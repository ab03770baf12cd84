// Row reduction: per (row, split) the two largest logits with their indices under
// (value desc, index asc) and, in sampling mode, the sum of exp2(z*c - ref).
// One streaming read of the logits; this is the HBM-bound kernel of the pass
// (paper Sec. 3.3 top-2 identification, Eq. 3 softmax normaliser).
//
// The per-element work is kept to the minimum the arithmetic units can hide behind the
// memory stream: widen, half a max3 and, when sampling, one fma + exp2 + add.  A lane only
// tracks the maxima of its batches (two 16-byte vectors each): the best and second-best batch
// maximum and the batches they came from, and keeps a raw copy of its best batch in LDS.
// A lane's two largest elements are then known to lie in those two batches, so after the
// stream the few lanes that can hold a candidate look through their LDS copy (and, rarely,
// reload the second batch) and produce exact (value, index) pairs.
//
// Every wave works for itself from the first load to its own result: there is no barrier and
// no cross-wave traffic while the stream runs, so a wave that has finished leaves the memory
// pipeline to the others instead of holding them at a rendezvous.  The waves meet once, at the
// very end, to fold their eight results into the work-group's one.
#pragma once

#include "common.h"

namespace mars {

constexpr int kRowThreads = 512;  // 8 waves per work-group (512 x 2 measured best of {128..1024} x {1,2,4,8})
constexpr int kUnroll = 2;        // 16-byte loads per lane per batch
constexpr float kRescaleLog2 = 24.0f;  // move the sum-exp reference when the max rises by 2^24

// Insert the elements >= cut of one vector into the running key pair (k1 >= k2).  Only a
// vector whose maximum reaches the cut is looked at element by element (normally one or two):
// the insertions are a serial chain run by a wave with one or two live lanes.
template <typename T, int EPV>
__device__ __forceinline__ void scan_vec(const Vec<T, EPV>& v, int vec, float cut, unsigned long long& k1,
                                         unsigned long long& k2) {
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
}

// Exact ranking of every element a lane owns (cold path, kept out of line).
// (Results come back by value: a local whose address is handed to an out-of-line function lives in
// scratch memory, and every later access to it becomes a memory round trip.)
struct KeyPair { unsigned long long k1, k2; };
template <typename T, int EPV>
__device__ __noinline__ KeyPair rank_all(const T* __restrict__ rowp, int v_begin, int v_end, int nb, int tid) {
  unsigned long long k1 = 0, k2 = 0;
#pragma unroll 1
  for (int kb = 0; kb < nb; ++kb) {
#pragma unroll 1
    for (int j = 0; j < kUnroll; ++j) {
      const int vec = v_begin + (kb * kUnroll + j) * kRowThreads + tid;
      if (vec < v_end) {
        Vec<T, EPV> v;
        v.load(rowp, static_cast<unsigned int>(vec));
#pragma unroll 1
        for (int e = 0; e < EPV; ++e) top2_insert(k1, k2, make_key(v.get(e), vec * EPV + e));
      }
    }
  }
  KeyPair r;
  r.k1 = k1; r.k2 = k2;
  return r;
}

__device__ __forceinline__ unsigned long long lane_value(unsigned long long v, int lane) {
  const unsigned int lo = __builtin_amdgcn_readlane(static_cast<int>(v), lane);
  const unsigned int hi = __builtin_amdgcn_readlane(static_cast<int>(v >> 32), lane);
  return (static_cast<unsigned long long>(hi) << 32) | lo;
}

// What the row reduction does on behalf of the kernel that follows it on the stream: memory it clears,
// and the gather the sampling walk starts from.
struct ClearArgs {
  unsigned long long* xslots;  // exchange words of the sampling tail: [copies*B][N+2][xwords]
  int N, B, xwords, copies;
  unsigned int* counters;      // histogram counters (nullptr / 0 = none)
  long ncounters;
  // Every acceptance test (Eq. 1) needs the logit and the draft probability of a node's token in its
  // parent's row.  Gathered by the per-request kernel that costs a chain of two trips to memory (tree and
  // tokens, then the gather) on its critical path; here, the work-group of the parent's row reads the tree
  // while its first loads are in flight and leaves the pair in `gathered`, at no cost in time.
  // par == nullptr: not wanted (greedy mode, calls without a tree).
  const int32_t* par;
  const int32_t* tok;
  const void* q;               // draft probabilities [B,N,V] or nullptr (one-hot: the pair's second half is 1)
  int q_bf16;
  float2* gathered;            // [B*N]: (logit, draft probability) of node i's token in row par[i]
};

template <typename T, int EPV, bool SAMPLING>
__global__ __launch_bounds__(kRowThreads) void row_reduce_kernel(const T* __restrict__ logits, int V, int splits,
                                                                  int vecs_per_split, float c,
                                                                  Partial* __restrict__ partials, ClearArgs clr) {
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

  // The first batch is requested before anything else is done: what follows up to the stream proper
  // (clearing memory for the kernel behind this one, the tree of the request, set-up) then runs beside
  // the first trip to memory instead of in front of it.
  Vec<T, EPV> bufA[U], bufB[U];
  // Unconditional loads for a full batch; bounds-checked loads (padding with -inf) for the last one.
  auto load_full = [&](Vec<T, EPV>(&buf)[U], int k) {
    const T* __restrict__ bp = rowp + static_cast<size_t>(v_begin + k * BV) * EPV;  // wave-uniform
#pragma unroll
    for (int j = 0; j < U; ++j) buf[j].load(bp, static_cast<unsigned int>(tid + j * kRowThreads));
    // Keep the scheduler from hoisting uses of the other buffer above these loads: that would
    // turn the wait for the previous batch into a wait before this one is even issued.
    __builtin_amdgcn_sched_barrier(0);
  };
  if (nfull > 2) load_full(bufA, 0);

  // Exchange words of the tail kernel that follows on the stream (xwords per (request, exchange),
  // N + 2 exchanges per request, `copies` sets of B requests): cleared here so that the call
  // needs no separate memset.  Likewise the counters a following kernel accumulates into.
  if (split == 0 && tid < clr.xwords) {
    const int N = clr.N;
    const int b = row / N, i = row - b * N;
    for (int k = 0; k < clr.copies; ++k) {
      unsigned long long* cells =
          clr.xslots + (static_cast<size_t>(k) * clr.B + b) * static_cast<size_t>(N + 2) * clr.xwords;
      cells[static_cast<size_t>(i) * clr.xwords + tid] = 0ull;
      if (i == 0) {
        cells[static_cast<size_t>(N) * clr.xwords + tid] = 0ull;
        cells[static_cast<size_t>(N + 1) * clr.xwords + tid] = 0ull;
      }
    }
  }
  for (long i = static_cast<long>(item) * kRowThreads + tid; i < clr.ncounters;
       i += static_cast<long>(gridDim.x) * kRowThreads)
    clr.counters[i] = 0u;

  // The children of this row's node, at most kGatherPer per thread: tree and tokens are requested now and
  // looked at behind the first loads of the stream.
  constexpr int kGatherPer = (MARS_MAX_NODES + kRowThreads - 1) / kRowThreads;
  const bool gather = clr.par != nullptr && split == 0;
  const int gnode = row % clr.N;
  const size_t greq = static_cast<size_t>(row - gnode);  // first row of the request
  int gpar[kGatherPer], gtok[kGatherPer];
  float2 gval[kGatherPer];
#pragma unroll
  for (int j = 0; j < kGatherPer; ++j) {
    const int i = tid + j * kRowThreads;
    gpar[j] = -2; gtok[j] = -1;
    if (gather && i > gnode && i < clr.N) { gpar[j] = clr.par[greq + i]; gtok[j] = clr.tok[greq + i]; }
  }
  auto gather_issue = [&]() {
#pragma unroll
    for (int j = 0; j < kGatherPer; ++j) {
      gval[j] = make_float2(0.0f, 1.0f);
      if (gpar[j] == gnode && static_cast<unsigned int>(gtok[j]) < static_cast<unsigned int>(V)) {
        gval[j].x = widen(rowp[gtok[j]]);
        if (clr.q) {
          const size_t at = static_cast<size_t>(row) * static_cast<size_t>(V) + gtok[j];
          gval[j].y = clr.q_bf16 ? widen(static_cast<const bf16_t*>(clr.q)[at]) : static_cast<const float*>(clr.q)[at];
        }
      } else {
        gpar[j] = -2;
      }
    }
  };
  auto gather_store = [&]() {
#pragma unroll
    for (int j = 0; j < kGatherPer; ++j)
      if (gpar[j] == gnode) clr.gathered[greq + tid + j * kRowThreads] = gval[j];
  };

  float m1 = neg_inf(), m2 = neg_inf();  // best and second-best batch maximum of this lane
  int b1 = -1, b2 = -1;                  // the (distinct) batches they belong to
  float s = 0.0f;                        // sum of exp2(z*c - ref_c) over the lane's elements
  float ref_c = -1.0e30f;                // wave-uniform, integer-valued reference (already times c)
  float thresh = -3.0e38f;               // rescale when a lane maximum exceeds this (wave-uniform)
  const float tau_over_c = SAMPLING ? kRescaleLog2 / c : 0.0f;

  // Raw copy of every lane's best batch (vector j of lane t at [j][t]: conflict-free 16-byte rows).
  __shared__ Vec<T, EPV> sh_best[U][kRowThreads];
  // Results of the eight waves and the number of waves that have theirs (cleared here; the only barrier
  // of the kernel stands behind every wave's first loads, where nobody has anything to wait for yet).
  __shared__ unsigned long long sh_k[NW][2];
  __shared__ float sh_s[NW], sh_ref[NW];
  __shared__ int sh_done;
  if (tid == 0) sh_done = 0;

  auto load_edge = [&](Vec<T, EPV>(&buf)[U], int kk) {
    const int base = v_begin + kk * BV + tid;
#pragma unroll
    for (int j = 0; j < U; ++j)
      buf[j].load(rowp, static_cast<unsigned int>(min(base + j * kRowThreads, v_end - 1)));
    __builtin_amdgcn_sched_barrier(0);
  };
  auto trim_edge = [&](Vec<T, EPV>(&buf)[U], int kk) {
    const int base = v_begin + kk * BV + tid;
#pragma unroll
    for (int j = 0; j < U; ++j)
      if (base + j * kRowThreads >= v_end) buf[j].fill_neg_inf();
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
    if (__any(gt)) {
      if (gt) {
#pragma unroll
        for (int j = 0; j < U; ++j) sh_best[j][tid] = buf[j];
      }
    }
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
      // The batch's terms are summed here and now.  Left to itself the compiler sinks this block behind
      // the next batch's wait, widening and maxima (the scheduling barriers order instructions, not the
      // passes that move computations towards their uses): a wave then sits out its wait with this work
      // still to do, and thirty-two widened elements are live instead of sixteen -- 76 registers instead
      // of 59, six waves per SIMD instead of eight, three work-groups per compute unit instead of four.
      asm volatile("" : "+v"(s));
    }
  };

  // Double-buffered stream over the full batches: the loads of batch k+1 are in flight while
  // batch k is processed.  The last one to three batches (the ragged one among them) run
  // through a plain loop with bounds-checked loads; keeping that part small keeps the kernel's
  // code small, which matters for the cold code every wave runs once at its end.
  int k = 0;
  if (nfull > 2) {
    __syncthreads();
    gather_issue();
    for (; k + 2 < nfull; k += 2) {
      load_full(bufB, k + 1);
      process(bufA, k);
      load_full(bufA, k + 2);
      process(bufB, k + 1);
    }
    // bufA holds batch k; at most two batches follow it (the last full one, the ragged one).  They are
    // requested ahead like the others -- every lane loads, one past the end of the share from the share's last
    // vector, and what such a lane has loaded is replaced when it arrives -- so that a wave does not end its
    // stream on one or two trips to memory with nothing else in flight.  (The requests stand under no
    // condition: where no batch follows, the last one is asked for again and not looked at.  Under a
    // condition, even one that is the same for the whole wave, the compiler no longer knows how many loads
    // are in flight and waits for all of them before batch k is processed.)
    const bool more1 = k + 1 < nb, more2 = k + 2 < nb;
    load_edge(bufB, min(k + 1, nb - 1));
    process(bufA, k);
    load_edge(bufA, min(k + 2, nb - 1));
    if (more1) { trim_edge(bufB, k + 1); process(bufB, k + 1); }
    if (more2) { trim_edge(bufA, k + 2); process(bufA, k + 2); }
    k = nb;
  } else {
    __syncthreads();
    gather_issue();
  }
#pragma unroll 1
  for (; k < nb; ++k) {
    load_tail(bufB, k);
    process(bufB, k);
  }
  gather_store();

  // ------------------------------------------------------------------ per-wave epilogue
  const int wave = tid / kWave, lane = tid % kWave;
  float w1 = m1, w2 = m2;
  wave_top2_values(w1, w2);
  // w1 is the wave's maximum; w2, the second largest batch maximum over its lanes, is a lower
  // bound of its runner-up.  Every element >= w2 lies in batch b1 or b2 of a lane whose own
  // maxima reach w2: those lanes look through their batches.
  unsigned long long k1 = 0, k2 = 0;
  if (w2 > neg_inf()) {
    const float cut = w2;
    if (m1 >= cut) {
#pragma unroll 1
      for (int j = 0; j < U; ++j) {
        const int vec = v_begin + (b1 * U + j) * kRowThreads + tid;
        if (vec < v_end) scan_vec<T, EPV>(sh_best[j][tid], vec, cut, k1, k2);
      }
      if (m2 >= cut) {  // rare: both of the lane's batches matter; the second comes from memory
#pragma unroll 1
        for (int j = 0; j < U; ++j) {
          const int vec = v_begin + (b2 * U + j) * kRowThreads + tid;
          if (vec < v_end) {
            Vec<T, EPV> v;
            v.load(rowp, static_cast<unsigned int>(vec));
            scan_vec<T, EPV>(v, vec, cut, k1, k2);
          }
        }
      }
    }
  } else {
    // The wave saw fewer than two finite batch maxima (a tiny or almost entirely masked share):
    // every element it owns, -inf entries included, is ranked exactly.
    const KeyPair r = rank_all<T, EPV>(rowp, v_begin, v_end, nb, tid);
    k1 = r.k1; k2 = r.k2;
  }
  // Wave-level top-2 of the lanes' keys: walk the (few) lanes that hold any.
  unsigned long long K1 = 0, K2 = 0;
  unsigned long long holders = __ballot(k1 != 0ull);
  while (holders != 0ull) {
    const int l = __ffsll(static_cast<long long>(holders)) - 1;
    holders &= holders - 1;
    top2_insert(K1, K2, lane_value(k1, l));
    const unsigned long long second = lane_value(k2, l);
    if (second != 0ull) top2_insert(K1, K2, second);
  }
  float ws = 0.0f;
  if (SAMPLING) ws = wave_sum(s);
  // The wave that is last to have its result folds the eight into the work-group's partial result; the
  // others leave at once.  (LDS operations of one wave are performed in order, so a wave that sees the
  // count complete sees every result behind it.)  The kernel behind this one then reads one partial
  // result per (row, split) instead of eight -- on its critical path, where this merge is not.
  int last = 0;
  if (lane == 0) {
    sh_k[wave][0] = K1; sh_k[wave][1] = K2;
    sh_s[wave] = ws; sh_ref[wave] = ref_c;
    last = __hip_atomic_fetch_add(&sh_done, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP) == NW - 1;
  }
  if (!__builtin_amdgcn_readfirstlane(last)) return;
  static_assert(NW == 8, "three butterfly steps merge eight waves");
  unsigned long long B1 = 0, B2 = 0;
  float R = -3.0e38f;
  double S = 0.0;
  if (lane < NW) {
    B1 = sh_k[lane][0]; B2 = sh_k[lane][1];
    if (SAMPLING && sh_s[lane] > 0.0f) { R = sh_ref[lane]; S = static_cast<double>(sh_s[lane]); }
  }
  merge_step<kDppXor1>(B1, B2, R, S);
  merge_step<kDppXor2>(B1, B2, R, S);
  merge_step<kDppHalfMirror>(B1, B2, R, S);
  if (lane == 0) {
    Partial out;
    out.z1 = neg_inf(); out.id1 = -1; out.z2 = neg_inf(); out.id2 = -1; out.s = 0.0f; out.ref = 0.0f;
    if (B1 != 0ull) { out.z1 = key_value(B1); out.id1 = key_index(B1); }
    if (B2 != 0ull) { out.z2 = key_value(B2); out.id2 = key_index(B2); }
    if (SAMPLING && S > 0.0) { out.s = static_cast<float>(S); out.ref = R; }
    partials[item] = out;
  }
}

// Partial results per (row, split).
constexpr int kPartsPerItem = 1;

// Merge the partial results of every row into the statistics table (16 rows per work-group).
__global__ __launch_bounds__(256) void merge_stats_kernel(const Partial* __restrict__ partials, int rows, int N,
                                                          int parts, const float* __restrict__ theta, float c,
                                                          Indicator ind, mars_row_stat* __restrict__ stats) {
  const int first = blockIdx.x * 16;
  const int n = min(16, rows - first);
  if (n <= 0) return;
  merge_rows_coop<256>(partials + static_cast<size_t>(first) * parts, n, parts, c, ind,
                       [&](int row) { return theta[(first + row) / N]; },
                       [&](int row, const mars_row_stat& st) { stats[first + row] = st; });
}

// Distributions of the top-2 statistics over the rows (appendix histogram figure of the paper:
// top-1 logit, logit ratio z2/z1, probability ratio p2/p1, share of negative top-1 logits).
// A histogram over [lo, hi) with `bins` equal cells owns bins + 2 counters: below lo, the cells,
// at or above hi.  The cell is trunc(fl(fl(x - lo) * w)), w = fl32(bins / (hi - lo)), capped.
struct HistSpec {
  float lo[3], hi[3], w[3];
  int bins[3];
};
__device__ __forceinline__ int hist_cell(float x, float lo, float hi, float w, int bins) {
  if (x < lo) return 0;
  if (!(x < hi)) return bins + 1;
  const int k = static_cast<int>(__fmul_rn(__fsub_rn(x, lo), w));
  return min(k, bins - 1) + 1;
}
// counters: [bins0+2 | bins1+2 | bins2+2 | rows, z1 < 0, z1 <= 0, low margin at theta], cleared by the
// row reduction of the same call.  Rows with z1 <= 0 have no ratio (Sec. 3.3) and skip its histogram.
__global__ __launch_bounds__(256) void margin_stats_kernel(const Partial* __restrict__ partials, int rows, int N,
                                                           int parts, const float* __restrict__ theta, double cind,
                                                           HistSpec hs, mars_margin_row* __restrict__ rows_out,
                                                           unsigned int* __restrict__ counters) {
  const int first = blockIdx.x * 16;
  const int n = min(16, rows - first);
  if (n <= 0) return;
  unsigned int* h0 = counters;
  unsigned int* h1 = h0 + hs.bins[0] + 2;
  unsigned int* h2 = h1 + hs.bins[1] + 2;
  unsigned int* summary = h2 + hs.bins[2] + 2;
  // The summary counters would take one atomic per row on a single address each: they are
  // gathered in LDS first and leave the work-group as one atomic per counter.
  __shared__ unsigned int sh_sum[4];
  if (threadIdx.x < 4) sh_sum[threadIdx.x] = 0u;
  __syncthreads();
  const Indicator ind = {MARS_IND_LOGIT_RATIO, cind};
  merge_rows_coop<256>(partials + static_cast<size_t>(first) * parts, n, parts, 0.0f, ind,
                       [&](int row) { return theta[(first + row) / N]; },
                       [&](int row, const mars_row_stat& st) {
                         mars_margin_row m;
                         m.z1 = st.z1; m.z2 = st.z2;
                         m.ratio = st.z2 / st.z1;
                         m.prob_ratio = prob_ratio(st.z1, st.z2, cind);
                         if (rows_out) rows_out[first + row] = m;
                         atomicAdd(&h0[hist_cell(m.z1, hs.lo[0], hs.hi[0], hs.w[0], hs.bins[0])], 1u);
                         if (st.z1 > 0.0f) atomicAdd(&h1[hist_cell(m.ratio, hs.lo[1], hs.hi[1], hs.w[1], hs.bins[1])], 1u);
                         atomicAdd(&h2[hist_cell(m.prob_ratio, hs.lo[2], hs.hi[2], hs.w[2], hs.bins[2])], 1u);
                         if (st.z1 < 0.0f) atomicAdd(&sh_sum[1], 1u);
                         if (!(st.z1 > 0.0f)) atomicAdd(&sh_sum[2], 1u);
                         if (st.relax_ok) atomicAdd(&sh_sum[3], 1u);
                       });
  __syncthreads();
  if (threadIdx.x == 0) sh_sum[0] = static_cast<unsigned int>(n);
  __syncthreads();
  if (threadIdx.x < 4 && sh_sum[threadIdx.x] != 0u) atomicAdd(&summary[threadIdx.x], sh_sum[threadIdx.x]);
}

}  // namespace mars
