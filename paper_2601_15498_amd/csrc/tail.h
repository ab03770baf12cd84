// Per-request tail of the verification pass: merge the row partials, take the
// per-node decisions, select the path and produce the correction / bonus token.
// One work-group per request in greedy mode; in sampling mode up to 32 work-groups share a
// request, each owning a slice of the vocabulary.
//
// Greedy mode is Algorithm 1 on a tree: local three-way test per node, reachability
// by pointer jumping, deepest reachable node (lowest index on ties), token = v(1) of
// its row.  Sampling mode is multi-round rejection sampling down the tree (Eq. 1) with
// the runner-up relaxation of Sec. 3.4 as a deterministic accept, residual
// renormalisation after every rejection (Sec. 2.3) and an inverse-CDF draw at the end.
#pragma once

#include "common.h"

namespace mars {

constexpr int kGreedyThreads = 1024;  // 64 rows merged at a time
constexpr int kSamplingThreads = 512;    // sampling tail whose slices stay in registers
constexpr int kStreamingThreads = 1024;  // sampling tail that streams its slices: more loads in flight per compute unit
constexpr int kMaxTiles = 512;  // CDF tiles kept in LDS for the final draw
constexpr int kMaxGroupsPerRequest = 32;   // work-groups that may share one request

struct TailArgs {
  const void* logits;
  const int32_t* tok;
  const int32_t* par;
  const void* dprobs;  // nullptr = one-hot draft distribution
  const float* theta;
  const float* u;
  const Partial* partials;
  const float2* gathered;   // sampling mode: (logit, draft probability) of every node's token in its parent's row
                            // (left by the row reduction; nullptr: the walk gathers them itself)
  mars_row_stat* stats;     // optional caller's table [B*N]
  mars_row_stat* stats_ws;  // [B*N] in the workspace: the table the tail itself reads
  uint8_t* mask;
  int32_t* len;
  int32_t* path;
  int32_t* bonus;
  uint8_t* dec;          // optional
  int32_t* status;       // optional
  mars_req_diag* diag;   // optional
  int B, N, V, splits;   // splits = partial results per row
  // Threshold sweep: B = K * Bd requests are verified, request b reading the inputs (logits,
  // tokens, tree, draft distribution, uniforms, row partials) of request b % Bd with its own
  // theta[b]; every output is indexed by b.  Bd == B without a sweep.
  int Bd;
  Indicator ind;         // which low-margin test (Sec. 3.3)
  int32_t* out_tok;      // optional [B,N]: committed sequence V_out (Alg. 1), -1 padded
  int32_t* out_len;      // optional [B]
  float c;               // log2(e) / T, 0 in greedy mode
  // sampling mode: G work-groups share one request and exchange partial sums
  int G;
  int spin_limit;        // polls a work-group gives a partner before it works out the partner's sum itself
  unsigned long long* xslots;  // [B][N+2][G][2] tagged exchange words, cleared by the row reduction
};

// ---------------------------------------------------------------- shared by both modes
// Outputs of a request that failed validation: nothing accepted, token = v(1) of the root row.
template <int NT>
__device__ void write_rejected_request(const TailArgs& a, int b, int status, int root_top1) {
  const int N = a.N;
  for (int i = threadIdx.x; i < N; i += NT) {
    const size_t r = static_cast<size_t>(b) * N + i;
    a.mask[r] = i == 0 ? 1 : 0;
    a.path[r] = -1;
    if (a.dec) a.dec[r] = 0;
    if (a.out_tok && i > 0) a.out_tok[r] = -1;
  }
  if (threadIdx.x == 0) {
    a.len[b] = 0;
    a.bonus[b] = root_top1;
    if (a.out_tok) { a.out_tok[static_cast<size_t>(b) * N] = root_top1; a.out_len[b] = 1; }
    if (a.status) a.status[b] = status;
    if (a.diag) { mars_req_diag d = {0.0f, 0.0f, 0, 0}; a.diag[b] = d; }
  }
}

// ---------------------------------------------------------------- greedy mode
// The kernel is a chain of latencies, so it makes one trip to memory: the tree and the tokens are
// requested ahead of the partial results, the merged rows go to the caller's table and, for the
// kernel's own use, to LDS, and everything after that -- decisions, reachability, the walk back
// along the accepted path -- reads LDS only.
__global__ __launch_bounds__(kGreedyThreads) void tail_greedy_kernel(TailArgs a) {
  constexpr int NT = kGreedyThreads;
  static_assert(MARS_MAX_NODES <= NT, "a thread holds the parent and the token of one node");
  __shared__ uint8_t sh_code[MARS_MAX_NODES];
  __shared__ uint8_t sh_ok[2][MARS_MAX_NODES];
  __shared__ int16_t sh_anc[2][MARS_MAX_NODES];
  __shared__ int16_t sh_dep[2][MARS_MAX_NODES];
  __shared__ int16_t sh_par[MARS_MAX_NODES];
  __shared__ int32_t sh_tok[MARS_MAX_NODES];
  __shared__ int32_t sh_top1[MARS_MAX_NODES];    // v(1) of the node's row
  __shared__ int32_t sh_relax[MARS_MAX_NODES];   // v(2) of the node's row where its low-margin test holds, else -1
  __shared__ unsigned int sh_best;

  const int b = blockIdx.x;
  const int N = a.N;
  const int i = threadIdx.x;
  const size_t rb = static_cast<size_t>(b) * N;
  const size_t rd = static_cast<size_t>(b % a.Bd) * N;  // where the request's inputs are
  int p = -1, t = 0;
  if (i < N) { p = a.par[rd + i]; t = a.tok[rd + i]; }
  const float theta = a.theta[b];
  // (eight loads in flight per lane: this kernel has the registers, and behind the fused LM head a
  // row has up to a few hundred partial results)
  merge_rows_coop<NT, 8>(a.partials + rd * a.splits, N, a.splits, a.c, a.ind, [&](int) { return theta; },
                         [&](int row, const mars_row_stat& st) {
                           a.stats_ws[rb + row] = st;
                           if (a.stats) a.stats[rb + row] = st;
                           sh_top1[row] = st.id1;
                           sh_relax[row] = st.relax_ok ? st.id2 : -1;
                         });
  int bad = 0;
  if (i < N) {
    if (i == 0) { if (p != -1) bad |= 1; }
    else {
      if (p < 0 || p >= i) bad |= 1;
      if (t < 0 || t >= a.V) bad |= 2;
    }
    sh_par[i] = static_cast<int16_t>(p);
    sh_tok[i] = t;
  }
  if (i == 0) sh_best = 0;
  if (__syncthreads_or(bad)) {  // (the barrier also publishes what the merge left in LDS)
    const int any_tree = __syncthreads_or(bad & 1);
    write_rejected_request<NT>(a, b, any_tree ? MARS_REQ_BAD_TREE : MARS_REQ_BAD_TOKEN, sh_top1[0]);
    return;
  }

  // Local decision of every node against its parent's row (Alg. 1 if-chain).
  if (i < N) {
    int code = 0, anc = 0, dep = 0;
    if (i > 0) {
      if (t == sh_top1[p]) code = MARS_DEC_EXACT;
      else if (t == sh_relax[p]) code = MARS_DEC_RELAXED;  // (t >= 0: never equal to the -1 of a failed test)
      anc = p; dep = 1;
    }
    sh_code[i] = static_cast<uint8_t>(code);
    sh_ok[0][i] = (i == 0 || code != 0) ? 1 : 0;
    sh_anc[0][i] = static_cast<int16_t>(anc);
    sh_dep[0][i] = static_cast<int16_t>(dep);
  }
  __syncthreads();
  // Pointer jumping: after round k, anc is the 2^k-th ancestor (or the root), dep the number
  // of edges to it and ok the AND of the local decisions along those edges.
  int cur = 0;
  for (int span = 1; span < N; span <<= 1) {
    const int nxt = cur ^ 1;
    if (i < N) {
      const int an = sh_anc[cur][i];
      sh_ok[nxt][i] = sh_ok[cur][i] & sh_ok[cur][an];
      sh_dep[nxt][i] = static_cast<int16_t>(sh_dep[cur][i] + sh_dep[cur][an]);
      sh_anc[nxt][i] = sh_anc[cur][an];
    }
    cur = nxt;
    __syncthreads();
  }
  // Deepest reachable node, lowest index on ties: max of (depth << 16 | (0xFFFF - i)).
  if (i < N) {
    if (sh_ok[cur][i]) atomicMax(&sh_best, (static_cast<unsigned int>(sh_dep[cur][i]) << 16) | (0xFFFFu - i));
    a.mask[rb + i] = i == 0 ? 1 : 0;
    a.path[rb + i] = -1;
    if (a.dec) a.dec[rb + i] = 0;
    if (a.out_tok) a.out_tok[rb + i] = -1;
  }
  __syncthreads();
  if (i == 0) {
    const unsigned int bk = sh_best;
    const int e = 0xFFFF - static_cast<int>(bk & 0xFFFFu);
    const int L = static_cast<int>(bk >> 16);
    int n = e;
    for (int d = L; d >= 1; --d) {
      a.mask[rb + n] = 1;
      a.path[rb + d - 1] = n;
      if (a.dec) a.dec[rb + n] = sh_code[n];
      if (a.out_tok) a.out_tok[rb + d - 1] = sh_tok[n];  // V_out: the accepted drafts ...
      n = sh_par[n];
    }
    a.len[b] = L;
    const int correction = sh_top1[e];  // correction after a rejection, bonus after a leaf
    a.bonus[b] = correction;
    if (a.out_tok) { a.out_tok[rb + L] = correction; a.out_len[b] = L + 1; }  // ... then this token
    if (a.status) a.status[b] = MARS_REQ_OK;
    if (a.diag) { mars_req_diag dg = {0.0f, 0.0f, 0, e}; a.diag[b] = dg; }
  }
}

// ---------------------------------------------------------------- sampling mode
// Eight consecutive elements of a row, widened; out-of-range positions read as `fill`.
template <typename T>
__device__ __forceinline__ void load8(const T* __restrict__ row, int g, int V, bool vec_ok, float fill, float (&x)[8]);

template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* __restrict__ row, int g, int V, bool vec_ok, float fill,
                                              float (&x)[8]) {
  if (vec_ok) {
    Vec<bf16_t, 8> v;
    v.load(row, g);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = v.get(e);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) { const int i = g * 8 + e; x[e] = i < V ? widen(row[i]) : fill; }
  }
}
template <>
__device__ __forceinline__ void load8<float>(const float* __restrict__ row, int g, int V, bool vec_ok, float fill,
                                             float (&x)[8]) {
  if (vec_ok) {
    const float4 lo = *reinterpret_cast<const float4*>(row + static_cast<size_t>(g) * 8);
    const float4 hi = *reinterpret_cast<const float4*>(row + static_cast<size_t>(g) * 8 + 4);
    x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w; x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) { const int i = g * 8 + e; x[e] = i < V ? row[i] : fill; }
  }
}

// Eight consecutive elements as they lie in memory (one aligned group): requested without being looked at,
// so that nothing waits for them until they are widened.
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
  u32x4 v;
  __device__ __forceinline__ void load(const bf16_t* __restrict__ row, int g) {
    v = *reinterpret_cast<const u32x4*>(row + static_cast<size_t>(g) * 8);
  }
  __device__ __forceinline__ void widen_to(float (&x)[8]) const {
    x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xFFFF0000u);
    x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xFFFF0000u);
    x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xFFFF0000u);
    x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
};
template <> struct Raw8<float> {
  f32x4 lo, hi;
  __device__ __forceinline__ void load(const float* __restrict__ row, int g) {
    lo = *reinterpret_cast<const f32x4*>(row + static_cast<size_t>(g) * 8);
    hi = *reinterpret_cast<const f32x4*>(row + static_cast<size_t>(g) * 8 + 4);
  }
  __device__ __forceinline__ void widen_to(float (&x)[8]) const {
    x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w; x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
  }
};

// The residual chain at the current node: rejection j replaced f by
// max(0, f - q_j) * inv_norm[j] (q_j dense, or one-hot at tok[j]).
// The first kChainRegs entries live in (wave-uniform) registers, so that the per-element
// evaluation touches no memory; longer chains continue in LDS.
constexpr int kChainRegs = 4;
struct Chain {
  const int32_t* tok;      // LDS
  const float* inv_norm;   // LDS; 0 marks "Z was 0, f left unchanged"
  int n;
  int rtok[kChainRegs];
  float rinv[kChainRegs];
};

// f(v) for the current node: softmax term, then the residual chain.
__device__ __forceinline__ float eval_f(float z, float q, int v, float z1, float c, float inv_S, bool dense,
                                        const Chain& ch) {
  float f = __builtin_amdgcn_exp2f((z - z1) * c) * inv_S;
#pragma unroll
  for (int j = 0; j < kChainRegs; ++j) {
    if (j < ch.n) {
      const float qj = dense ? q : (v == ch.rtok[j] ? 1.0f : 0.0f);
      const float g = fmaxf(f - qj, 0.0f);
      f = ch.rinv[j] > 0.0f ? g * ch.rinv[j] : f;
    }
  }
  for (int j = kChainRegs; j < ch.n; ++j) {
    const float qj = dense ? q : (v == ch.tok[j] ? 1.0f : 0.0f);
    const float g = fmaxf(f - qj, 0.0f);
    const float inv = ch.inv_norm[j];
    f = inv > 0.0f ? g * inv : f;
  }
  return f;
}

// A child tested against the plain softmax of its parent's row (no rejection at that node yet): the
// runner-up of a low-margin row is accepted outright (Alg. 1), anything else with probability
// min(1, f(x)/q(x)) (Eq. 1).  Returns the decision code (0 = rejected) and f(x).
__device__ __forceinline__ int first_try(const mars_row_stat& st, float zx, float qx, int x, float u, float c,
                                         float& fx) {
  fx = 0.0f;
  if (x == st.id2 && st.relax_ok) return MARS_DEC_RELAXED;
  fx = __builtin_amdgcn_exp2f((zx - st.z1) * c) * (1.0f / st.sum_exp);
  float acc;
  if (fx == 0.0f) acc = 0.0f;
  else if (qx <= 0.0f) acc = 1.0f;
  else acc = fminf(1.0f, fx / qx);
  return u < acc ? MARS_DEC_SAMPLED : 0;
}

// Sum over the work-group.  The caller keeps a barrier between two calls (the exchange that follows
// every call has one), so the staging array needs none in front of the write.
template <int NT>
__device__ __forceinline__ double block_sum(double v, double* sh) {
  v = wave_sum(v);
  if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) t += sh[w];
  return t;
}

// Sum of one double per work-group over the G work-groups of a request, in work-group order
// (so every work-group obtains the same bits).  Exchange number `idx` of request b has its own
// 2*G words, cleared by the row reduction of the same call.  A work-group publishes its value as
// two floats (head and tail of the double), each packed with a non-zero tag into one 64-bit
// word, so that a single store both delivers the data and signals arrival; the partners poll
// the words directly.
//
// No work-group depends on another one being there.  A partner whose words have not arrived
// after `spin_limit` polls (it may not have been given a compute unit yet: the GPU is shared with
// other kernels, other streams, other calls of this library) is not waited for any longer: the
// work-group goes over that partner's slice itself, with the partner's own assignment of elements
// to threads and order of additions, so that it obtains the very bits the partner will publish,
// and carries on.  Whatever the placement of the work-groups, every one of them finishes, and
// all agree.  The exchange therefore comes in three steps, and the caller's pass over a slice is
// written once, inside a loop over "whose slice": its own first, then those of the missing partners.
//   exchange_begin  publish `mine`, poll the partners; returns the set of those that did not arrive
//   exchange_fill   the value worked out here for a missing partner
//   exchange_end    the sum, in work-group order
__device__ __forceinline__ unsigned long long pack_tagged(float v) {
  return (1ull << 32) | static_cast<unsigned long long>(__float_as_uint(v));
}
template <int NT>
__device__ __forceinline__ unsigned int exchange_begin(const TailArgs& a, int b, int g, int idx, double mine,
                                                       double* sh_part, unsigned int* sh_missing) {
  const int G = a.G;
  if (G == 1) { sh_part[0] = mine; return 0u; }
  static_assert(2 * kMaxGroupsPerRequest <= kWave, "one wave polls every word of an exchange");
  unsigned long long* cell = a.xslots + (static_cast<size_t>(b) * (a.N + 2) + idx) * (2 * G);
  if (threadIdx.x == 0) {
    const float hi = static_cast<float>(mine);
    const float lo = static_cast<float>(mine - static_cast<double>(hi));
    __hip_atomic_store(&cell[2 * g], pack_tagged(hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&cell[2 * g + 1], pack_tagged(lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *sh_missing = 0u;
  }
  if (threadIdx.x < 2 * G) {
    // One wave polls all 2*G words at once: lane 2i the head of work-group i's value, lane 2i+1 its tail.
    unsigned long long w = 0;
    int spins = 0;
    for (;;) {
      w = __hip_atomic_load(&cell[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((w >> 32) != 0ull) break;
      if (++spins > a.spin_limit) { atomicOr(sh_missing, 1u << (threadIdx.x >> 1)); break; }
      __builtin_amdgcn_s_sleep(1);
    }
    double v = static_cast<double>(__uint_as_float(static_cast<unsigned int>(w)));
    v += __shfl_down(v, 1, kWave);  // even lanes: head + tail
    if ((threadIdx.x & 1) == 0) sh_part[threadIdx.x >> 1] = v;
  }
  __syncthreads();
  // (written again only behind the caller's next barrier; the same in every lane, and said so: what
  // is derived from it -- whose slice comes next, its bounds -- then lives in scalar registers)
  return static_cast<unsigned int>(__builtin_amdgcn_readfirstlane(static_cast<int>(*sh_missing)));
}
// (a value worked out here goes through the same two floats as one that travelled)
__device__ __forceinline__ void exchange_fill(double* sh_part, int i, double v) {
  if (threadIdx.x == 0) {
    const float hi = static_cast<float>(v);
    const float lo = static_cast<float>(v - static_cast<double>(hi));
    sh_part[i] = static_cast<double>(hi) + static_cast<double>(lo);
  }
}
// (Behind the barrier that ends exchange_begin, or the one the caller keeps behind its last exchange_fill.
// Lane i holds work-group i's value; the same tree of additions in every wave of every work-group.  The
// caller keeps a barrier between this and the next exchange_begin, which writes sh_part again.)
__device__ __forceinline__ double exchange_end(const TailArgs& a, const double* sh_part) {
  if (a.G == 1) return sh_part[0];
  const int lane = threadIdx.x % kWave;
  return wave_sum(lane < a.G ? sh_part[lane] : 0.0);
}

// Everything a pass over a row needs to evaluate the current distribution f.
template <typename T, typename TQ>
struct RowView {
  const T* zrow;
  const TQ* qrow;   // nullptr = one-hot draft distribution
  bool use_q;       // false: this pass does not look at q (no rejection at this node so far), skip its loads
  int V;
  bool vec_ok;
  float z1, c, inv_S;
  Chain ch;
  __device__ __forceinline__ void load(int gi, float (&z)[8], float (&q)[8]) const {
    load8<T>(zrow, gi, V, vec_ok, neg_inf(), z);
    if (qrow && use_q) {
      load8<TQ>(qrow, gi, V, vec_ok, 0.0f, q);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) q[e] = 0.0f;
    }
  }
  __device__ __forceinline__ float f(const float (&z)[8], const float (&q)[8], int gi, int e) const {
    return eval_f(z[e], qrow ? q[e] : 0.0f, gi * 8 + e, z1, c, inv_S, qrow != nullptr, ch);
  }
};

// Groups whose loads a thread issues before it starts computing.  (The streamed form runs 1024 threads, so 128
// registers each; with four groups in flight the kernel needs about 160 and spills, which on the B = 128 chain
// workload costs 25 us of 105; with two it needs 106 and the sixteen waves keep the memory pipeline as full.)
constexpr int kPassBatch = 2;

// This work-group's share of Z = sum_v max(0, f(v) - q_k(v)) over groups [g_begin, g_end):
// q_k dense, or one-hot at token x.  The loads of kPassBatch groups are issued together so
// that a pass costs about one memory round trip per batch, not one per group.
template <typename T, typename TQ, int NT>
__device__ __forceinline__ double residual_mass_slice(const RowView<T, TQ>& rv, int g_begin, int g_end, int x) {
  double part = 0.0;
  for (int base = g_begin + static_cast<int>(threadIdx.x); base < g_end; base += kPassBatch * NT) {
    float z[kPassBatch][8], q[kPassBatch][8];
#pragma unroll
    for (int i = 0; i < kPassBatch; ++i) {  // (no load under a per-lane condition: see the final draw)
      const int gi = base + i * NT;
      rv.load(gi < g_end ? gi : g_end - 1, z[i], q[i]);
    }
#pragma unroll
    for (int i = 0; i < kPassBatch; ++i) {
      const int gi = base + i * NT;
      if (gi < g_end) {
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float qk = rv.qrow ? q[i][e] : (gi * 8 + e == x ? 1.0f : 0.0f);
          acc += fmaxf(rv.f(z[i], q[i], gi, e) - qk, 0.0f);
        }
        part += static_cast<double>(acc);
      }
    }
  }
  return part;
}

// Prefix sums over the n <= kMaxTiles tile sums in LDS, by one wave: lane l owns the contiguous
// run of `per` tiles starting at l*per; the runs are summed in index order and scanned across the
// lanes.  Every lane ends with the same answers, and the total and the search use the same
// additions (any wave of the work-group may call these and obtains the same bits).
struct TilePrefix {
  double mine;  // sum of the lane's run
  double incl;  // sum of the runs of lanes 0..l
};
__device__ __forceinline__ TilePrefix tile_prefix(const double* sh_tile, int n, int per, int lane) {
  TilePrefix p;
  p.mine = 0.0;
  for (int i = 0; i < per; ++i) {
    const int t = lane * per + i;
    if (t < n) p.mine += sh_tile[t];
  }
  p.incl = wave_prefix_sum(p.mine);
  return p;
}
__device__ __forceinline__ double tile_total(const double* sh_tile, int n, int lane) {
  const int per = (n + kWave - 1) / kWave;
  return lane_value(tile_prefix(sh_tile, n, per, lane).incl, kWave - 1);
}
// The first tile whose inclusive prefix (on top of `before`) exceeds target, and the prefix in
// front of it; when rounding leaves none, the last tile with mass (tile 0 if there is none).
__device__ __forceinline__ void tile_find(const double* sh_tile, int n, int lane, double before, double target,
                                          int& tile, double& cum) {
  const int per = (n + kWave - 1) / kWave;
  const TilePrefix p = tile_prefix(sh_tile, n, per, lane);
  const double excl = before + (p.incl - p.mine);
  int my_last = -1;
  for (int i = 0; i < per; ++i) {
    const int t = lane * per + i;
    if (t < n && sh_tile[t] > 0.0) my_last = t;
  }
  const unsigned long long has = __ballot(my_last >= 0);
  const int last_tile = has != 0ull ? lane_value(my_last, 63 - __clzll(static_cast<long long>(has))) : 0;
  const unsigned long long hit = __ballot(before + p.incl > target);
  int found = -1;
  double front = 0.0;
  if (hit != 0ull) {
    const int hl = __ffsll(static_cast<long long>(hit)) - 1;
    if (lane == hl) {
      double run = excl;
      for (int i = 0; i < per && found < 0; ++i) {
        const int t = lane * per + i;
        if (t < n) {
          if (run + sh_tile[t] > target) { found = t; front = run; } else run += sh_tile[t];
        }
      }
    }
    found = lane_value(found, hl);
    front = lane_value(front, hl);
  }
  if (found < 0) {  // rounding: the last tile with mass, with the prefix in front of it
    found = last_tile;
    const int ol = found / per;
    double run = excl;
    for (int i = 0; i < per; ++i) {
      const int t = lane * per + i;
      if (t < found) run += sh_tile[t];
    }
    front = lane_value(run, ol);
  }
  tile = found;
  cum = front;
}

// A slice that is resident in a partner's registers, gone over from memory here because the partner has
// not arrived (see exchange_begin).  A rarely taken path: one group of eight at a time, so that it adds next
// to nothing to the registers of the walk around it; groups go to threads, and sums are formed, as in the
// owner's resident form.  (The streamed form of the tail needs no such twin: its own pass reads memory.)
template <typename T, typename TQ, int NT>
__device__ __forceinline__ double resident_mass_from_memory(const RowView<T, TQ>& rv, int gb, int ge, int x) {
  double part = 0.0;
#pragma unroll 1
  for (int gi = gb + static_cast<int>(threadIdx.x); gi < ge; gi += NT) {
    float z[8], q[8];
    rv.load(gi, z, q);
    float acc = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float qk = rv.qrow ? q[e] : (gi * 8 + e == x ? 1.0f : 0.0f);
      acc += fmaxf(rv.f(z, q, gi, e) - qk, 0.0f);
    }
    part += static_cast<double>(acc);
  }
  return part;
}
// Tile sums (a tile = a step of 64 groups, the steps dealt out to the waves in turn); returns their number.
template <typename T, typename TQ, int NT, int kRes>
__device__ __forceinline__ int resident_tiles_from_memory(const RowView<T, TQ>& rv, int gb, int ge, double* out) {
  constexpr int NW = NT / kWave;
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int nst = (ge - gb + kWave - 1) / kWave;
#pragma unroll 1
  for (int i = 0; i < kRes; ++i) {
    const int s = i * NW + wave;
    if (s < nst) {  // wave-uniform
      const int gi = gb + i * NT + tid;
      float gs = 0.0f;
      if (gi < ge) {
        float z[8], q[8], f[8];
        rv.load(gi, z, q);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = rv.f(z, q, gi, e);
        gs = ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
      }
      const double t = wave_sum(static_cast<double>(gs));
      if (lane == 0) out[s] = t;
    }
  }
  return nst;
}

constexpr float kClosedFormMinNorm = 0.1f; // one-hot residual: Z = 1 - f(x) is used when at least this
constexpr int kResident = 3;               // groups of eight elements a thread can keep in registers

// RESIDENT: every slice is at most kResident groups per thread (decided by the host from G and V).
// VEC: every group of eight elements is one aligned 16-byte (or 32-byte) load -- the host checks V % 8 and
// the alignment of the arrays.  The form that checks every element against the end of the row costs some
// eighty comparisons and as many scalar registers before the walk starts, on the critical path of every call.
template <typename T, typename TQ, bool RESIDENT, bool VEC>
__device__ __forceinline__ void tail_sampling_body(const TailArgs& a) {
  constexpr int NT = RESIDENT ? kSamplingThreads : kStreamingThreads;
  constexpr int NW = NT / kWave;
  __shared__ int16_t sh_par[MARS_MAX_NODES];     // parent of every node
  __shared__ int32_t sh_tok[MARS_MAX_NODES];     // draft token of every node
  __shared__ float sh_zx[MARS_MAX_NODES];        // logit of the node's token in its parent's row
  __shared__ float sh_qx[MARS_MAX_NODES];        // draft probability of the node's token (1 if one-hot)
  __shared__ int32_t sh_ctok[MARS_MAX_NODES];    // residual chain: rejected tokens
  __shared__ float sh_cinv[MARS_MAX_NODES];      // residual chain: 1/Z
  __shared__ mars_row_stat sh_st[MARS_MAX_NODES];  // merged row statistics of the request
  __shared__ double sh_red[NW];
  __shared__ double sh_part[kMaxGroupsPerRequest];
  __shared__ double sh_tile[kMaxTiles];
  __shared__ float sh_u[MARS_MAX_NODES + 1];     // the request's uniforms
  __shared__ double sh_tile2[kMaxTiles];         // tile sums of a partner's slice, when they have to be worked out here
  __shared__ unsigned int sh_missing;            // partners of the current exchange that have not arrived
  __shared__ int sh_bad;                         // validation bits of the request
  __shared__ int32_t sh_first[MARS_MAX_NODES];   // lowest-numbered child of every node (kNoChild: a leaf)
  __shared__ uint8_t sh_code0[MARS_MAX_NODES];   // decision of every node if it is the first child tested
  constexpr int32_t kNoChild = 0x7FFFFFFF;

  const int G = a.G;
  const int b = blockIdx.x / G, g = blockIdx.x - b * G;
  const int N = a.N, V = a.V;
  const size_t rb = static_cast<size_t>(b) * N;
  const int bd = b % a.Bd;  // the request whose inputs this (possibly swept) request reads
  const size_t rd = static_cast<size_t>(bd) * N;
  const int tid = threadIdx.x;
  const int wave = tid / kWave, lane = tid % kWave;
  if (tid == 0) sh_bad = 0;
  for (int i = tid; i < a.N; i += NT) sh_first[i] = kNoChild;
  __syncthreads();

  const T* __restrict__ zall = static_cast<const T*>(a.logits) + rd * static_cast<size_t>(V);
  const TQ* __restrict__ qall = a.dprobs ? static_cast<const TQ*>(a.dprobs) + rd * static_cast<size_t>(V) : nullptr;
  const bool dense = qall != nullptr;

  // Prologue, one node per thread.  It is one trip to memory: tree, tokens, the row's partial results,
  // uniforms, and the logit and draft probability of every node's token in its parent's row (which every
  // acceptance test needs, and which the row reduction of this call has gathered) all go out together.
  // Every work-group of the request does this for itself; they produce identical bits, and only the first
  // writes the caller's outputs.
  const int nwords = (N + kWave - 1) / kWave;
  {
    constexpr int kPerThread = (MARS_MAX_NODES + NT - 1) / NT;
    const float theta = a.theta[b];
    const bool few = a.splits <= kFewParts;  // one thread merges a row (else sixteen lanes do)
    const float* __restrict__ ureq = a.u + static_cast<size_t>(bd) * (N + 1);
    int pr[kPerThread], tk[kPerThread];
    float zx[kPerThread], qx[kPerThread], uv[kPerThread];  // (zx, qx: gathered by the row reduction of this call)
    Partial pq[kPerThread][kFewParts];
#pragma unroll
    for (int t = 0; t < kPerThread; ++t) {
      const int i = tid + t * NT;
      pr[t] = -1; tk[t] = 0; uv[t] = 0.0f; zx[t] = 0.0f; qx[t] = 1.0f;
      if (i < N) {
        pr[t] = a.par[rd + i];
        tk[t] = a.tok[rd + i];
        // (the streamed form is short of registers here: its partial results are requested further down)
        if (RESIDENT && few) load_partials_of_row(a.partials + (rd + i) * a.splits, a.splits, pq[t]);
        uv[t] = ureq[i];
        if (a.gathered) {
          const float2 zq = a.gathered[rd + i];
          zx[t] = zq.x; qx[t] = zq.y;
        }
      }
    }
    const float u_draw = tid == 0 ? ureq[N] : 0.0f;  // the uniform of the final draw
#pragma unroll
    for (int t = 0; t < kPerThread; ++t) {
      const int i = tid + t * NT;
      if (i < N) {
        const size_t r = rb + i;
        const int p = pr[t];
        const int x = tk[t];
        int bad = 0;
        if (i == 0) { if (p != -1) bad = 1; }
        else {
          if (p < 0 || p >= i) bad |= 1;
          if (x < 0 || x >= V) bad |= 2;
        }
        if (i == 0 || bad != 0) {  // (nothing was gathered for these)
          zx[t] = 0.0f; qx[t] = 1.0f;
        } else if (!a.gathered) {  // behind the fused LM head nobody has gathered: a second trip to memory
          const size_t at = static_cast<size_t>(p) * V + x;
          zx[t] = widen(zall[at]);
          if (dense) qx[t] = widen(qall[at]);
        }
        sh_par[i] = static_cast<int16_t>(p);
        sh_tok[i] = x;
        if (bad) atomicOr(&sh_bad, bad);
        else if (i > 0) atomicMin(&sh_first[p], i);
        if (g == 0) {
          a.mask[r] = i == 0 ? 1 : 0;
          a.path[r] = -1;
          if (a.dec) a.dec[r] = 0;
        }
      }
    }
    auto emit = [&](int row, const mars_row_stat& st) {
      sh_st[row] = st;
      if (g == 0) {
        a.stats_ws[rb + row] = st;
        if (a.stats) a.stats[rb + row] = st;
      }
    };
    if (few) {
#pragma unroll
      for (int t = 0; t < kPerThread; ++t) {
        const int i = tid + t * NT;
        if (i < N) {
          if (!RESIDENT) load_partials_of_row(a.partials + (rd + i) * a.splits, a.splits, pq[t]);
          const mars_row_stat st = merge_row_few(pq[t], a.c, a.ind, theta);
          sh_st[i] = st;
          if (g == 0) {
            a.stats_ws[rb + i] = st;
            if (a.stats) a.stats[rb + i] = st;
          }
        }
      }
    } else {
      merge_rows_coop<NT, 2>(a.partials + rd * a.splits, N, a.splits, a.c, a.ind, [&](int) { return theta; }, emit);
    }
#pragma unroll
    for (int t = 0; t < kPerThread; ++t) {
      const int i = tid + t * NT;
      if (i < N) { sh_zx[i] = zx[t]; sh_qx[i] = qx[t]; sh_u[i] = uv[t]; }
    }
    if (tid == 0) sh_u[N] = u_draw;
    __syncthreads();
    if (sh_bad != 0) {
      if (g == 0) write_rejected_request<NT>(a, b, (sh_bad & 1) ? MARS_REQ_BAD_TREE : MARS_REQ_BAD_TOKEN, sh_st[0].id1);
      return;
    }
    // What the walk decides at a node it reaches is, for the node's first child, a function of the inputs
    // alone: taken here for all nodes at once, so that the walk follows accepted first children at the
    // price of two LDS reads each.
#pragma unroll
    for (int t = 0; t < kPerThread; ++t) {
      const int i = tid + t * NT;
      if (i < N) {
        int code0 = 0;
        if (i > 0) {
          float fx;
          code0 = first_try(sh_st[pr[t]], zx[t], qx[t], tk[t], uv[t], a.c, fx);
        }
        sh_code0[i] = static_cast<uint8_t>(code0);
      }
    }
    __syncthreads();
  }

  constexpr bool vec_ok = VEC;
  const int ngroups = (V + 7) / 8;
  // This work-group's slice of the vocabulary, in groups of eight elements (a multiple of 64
  // groups, so that the slices are made of whole wave steps).
  const int slice = ((ngroups + G - 1) / G + kWave - 1) / kWave * kWave;
  const int g_begin = min(ngroups, g * slice), g_end = min(ngroups, g_begin + slice);
  // A slice of at most kResident groups per thread stays in registers between the passes over
  // one node: f is then loaded and exponentiated once per visited node, every further
  // rejection at that node only updates it in place, and the final draw reads it where it is.
  // Thread t holds groups g_begin + i*NT + t; "step" s = i*NW + wave is 64 consecutive groups.
  constexpr bool resident = RESIDENT;
  const int nsteps = (g_end - g_begin + kWave - 1) / kWave;
  const float c = a.c;
  const float* u = sh_u;

  int cnode = 0, plen = 0, passes = 0, nexch = 0;
  float last_norm = 0.0f;
  bool pending_norm = false;  // the last rejection's normaliser is still to come out of the final pass
  RowView<T, TQ> rv;
  rv.V = V; rv.vec_ok = vec_ok; rv.c = c;
  rv.ch.tok = sh_ctok; rv.ch.inv_norm = sh_cinv; rv.ch.n = 0;
  float fc[kResident][8], qv[kResident][8];  // resident slice: current f and the draft probabilities
  bool have = false;                          // fc holds the current f of this node's slice
  bool raw = false;                           // fc / qv hold the node's raw slice (logits, draft probabilities)
  int applied = 0;                            // chain entries already worked into fc

  // The loads of the resident slice, issued when a pass first needs it.  (Issuing them on arrival at every
  // node, in case a rejection follows, was tried: the next node's loads then have to wait for the registers
  // of the previous node's, and every accepted draft costs a trip to memory -- 86 instead of 80 us per pass.)
  // (With whole groups the loads are kept as they come until the slice is needed -- `widen_resident` -- so that
  // a request made ahead of time is not waited for where it is made.)
  Raw8<T> rz[kResident];
  Raw8<TQ> rq[kResident];
  bool rq_loaded = false;
  auto load_resident = [&]() {
    rq_loaded = rv.qrow && rv.use_q;
    if (VEC) {
      // No load stands under a condition, per lane or per call: a lane past the end of its slice reads the
      // row's last group and throws it away, and when the draft probabilities are not wanted every lane reads
      // the first 32 bytes of the logits in their place.  With a branch between two loads the compiler can no
      // longer count what is in flight and makes each wait for the one before (three trips to memory instead
      // of one); with a branch around them it copies what they return into the registers of the other path
      // right away, and waits for it there.
      const TQ* __restrict__ qsrc = rq_loaded ? rv.qrow : reinterpret_cast<const TQ*>(zall);
#pragma unroll
      for (int i = 0; i < kResident; ++i) {
        const int gi = min(g_begin + i * NT + tid, ngroups - 1);
        rz[i].load(rv.zrow, gi);
        rq[i].load(qsrc, rq_loaded ? gi : 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < kResident; ++i) {
        const int gi = g_begin + i * NT + tid;
        if (gi < g_end) rv.load(gi, fc[i], qv[i]);
      }
    }
    raw = true;
    have = false;
  };
  auto widen_resident = [&]() {
#pragma unroll
    for (int i = 0; i < kResident; ++i) {
      const int gi = g_begin + i * NT + tid;
      if (gi < g_end) {
        if (VEC) {
          rz[i].widen_to(fc[i]);
          if (rq_loaded) rq[i].widen_to(qv[i]);
        }
      } else {  // nothing there: f = 0 and q = 0 contribute nothing
#pragma unroll
        for (int e = 0; e < 8; ++e) { fc[i][e] = neg_inf(); qv[i][e] = 0.0f; }
      }
      if (!dense || (VEC && !rq_loaded)) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[i][e] = 0.0f;
      }
    }
  };
  // Bring the resident slice up to date with the chain (turning the raw slice into f on first use).
  auto refresh_resident = [&]() {
    if (!have) {
      if (!raw) load_resident();
      widen_resident();
#pragma unroll
      for (int i = 0; i < kResident; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e)
          fc[i][e] = __builtin_amdgcn_exp2f((fc[i][e] - rv.z1) * c) * rv.inv_S;  // softmax term (Eq. 3)
      raw = false;
      have = true;
      applied = 0;
    }
    for (int j = applied; j < rv.ch.n; ++j) {
      int tj = sh_ctok[j];
      float inv = sh_cinv[j];
#pragma unroll
      for (int r = 0; r < kChainRegs; ++r)
        if (r == j) { tj = rv.ch.rtok[r]; inv = rv.ch.rinv[r]; }
      if (inv > 0.0f) {
#pragma unroll
        for (int i = 0; i < kResident; ++i) {
          const int gi = g_begin + i * NT + tid;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float qj = dense ? qv[i][e] : (gi * 8 + e == tj ? 1.0f : 0.0f);
            fc[i][e] = fmaxf(fc[i][e] - qj, 0.0f) * inv;
          }
        }
      }
    }
    applied = rv.ch.n;
  };

  for (;;) {
    const int k1 = __builtin_amdgcn_readfirstlane(sh_first[cnode]);
    const bool leaf = k1 >= N;
    {
      const int code0 = !leaf ? __builtin_amdgcn_readfirstlane(static_cast<int>(sh_code0[k1])) : 0;
      if (code0 != 0) {  // the first child is accepted: nothing else at this node matters
        if (tid == 0 && g == 0) {
          a.mask[rb + k1] = 1;
          a.path[rb + plen] = k1;
          if (a.dec) a.dec[rb + k1] = static_cast<uint8_t>(code0);
          if (a.out_tok) a.out_tok[rb + plen] = sh_tok[k1];
        }
        cnode = k1;
        plen += 1;
        continue;
      }
    }
    const mars_row_stat st = sh_st[cnode];
    rv.zrow = zall + static_cast<size_t>(cnode) * V;
    rv.qrow = dense ? qall + static_cast<size_t>(cnode) * V : nullptr;
    rv.z1 = st.z1; rv.inv_S = 1.0f / st.sum_exp;
    rv.use_q = dense && !leaf;  // a rejection pass subtracts q; nothing is rejected at a leaf
    rv.ch.n = 0;
    pending_norm = false;
    have = false;
    raw = false;
    applied = 0;
    // The walk stops here or rejects here: at a leaf the final draw reads this row, and a node whose first
    // child is rejected sees a pass over it either now (further children) or in the final draw, unless a later
    // child is accepted off a closed-form normaliser (one-hot draft: the request is then wasted, nothing
    // waits for it).  The row's slice is requested at once, so that its trip to memory runs beside the tests
    // below instead of behind them.  (Only here: a node that is merely passed through never asks for its row.)
    if (RESIDENT) load_resident();
    // The children of cnode as bit masks over the nodes (increasing node index = increasing bit), 64
    // nodes to a word.  Every wave forms the words for itself from the parents in LDS: no wave waits for
    // another one on the way down the tree.
    auto kids_word = [&](int wd) {
      const int i = wd * kWave + lane;
      return __ballot(i < N && i > cnode && sh_par[i] == cnode);
    };
    int accepted = -1;
    int wd = cnode / kWave;              // children have larger indices than their parent
    unsigned long long bits = kids_word(wd);
    for (;;) {
      while (bits == 0ull && wd + 1 < nwords) bits = kids_word(++wd);
      if (bits == 0ull) break;
      const int k = wd * kWave + __ffsll(static_cast<long long>(bits)) - 1;
      bits &= bits - 1;
      bool more = bits != 0ull;          // does cnode have further children after k?
      for (int w2 = wd + 1; w2 < nwords && !more; ++w2) more = kids_word(w2) != 0ull;
      const int x = sh_tok[k];
      // Every thread takes the decision for itself from the same LDS-resident inputs (same
      // instructions, same bits): no broadcast and no barrier per tested child.
      int code = 0;
      float fx = 0.0f;
      if (rv.ch.n == 0) {
        code = first_try(st, sh_zx[k], sh_qx[k], x, u[k], c, fx);
      } else if (x == st.id2 && st.relax_ok) {
        code = MARS_DEC_RELAXED;  // runner-up in a low-margin row: accepted outright
      } else {
        const float qx = sh_qx[k];
        fx = eval_f(sh_zx[k], qx, x, st.z1, c, rv.inv_S, dense, rv.ch);
        // Eq. 1: accept with probability min(1, f(x)/q(x))
        float acc;
        if (fx == 0.0f) acc = 0.0f;
        else if (qx <= 0.0f) acc = 1.0f;
        else acc = fminf(1.0f, fx / qx);
        if (u[k] < acc) code = MARS_DEC_SAMPLED;
      }
      if (code) {
        if (tid == 0 && g == 0) {
          a.mask[rb + k] = 1;
          a.path[rb + plen] = k;
          if (a.dec) a.dec[rb + k] = static_cast<uint8_t>(code);
          if (a.out_tok) a.out_tok[rb + plen] = x;
        }
        accepted = k;
        break;
      }
      // Rejected: f <- max(0, f - q_k) / Z with Z = sum_v max(0, f(v) - q_k(v)).
      //  * With a one-hot q_k only the entry x changes and Z = 1 - f(x); that form is used while
      //    it is well conditioned.
      //  * After the node's last child nothing is tested against f any more: the division is
      //    left out (factor 1) and Z comes out of the final pass as the total of what is left.
      //  * Otherwise Z is summed over the row, every work-group of the request taking a slice.
      float inv;
      if (!dense && 1.0f - fx >= kClosedFormMinNorm) {
        last_norm = 1.0f - fx;
        inv = 1.0f / last_norm;
      } else if (!more) {
        pending_norm = true;
        inv = 1.0f;
      } else {
        // This work-group's slice first, then (rarely) those of partners that have not arrived.  The
        // streamed form reads memory either way and runs one loop over "whose slice"; the resident form has
        // its own slice in registers and a lean pass over memory for the others, kept out of the way
        // behind the exchange (both forms are short of registers in different places).
        if (resident) {
          refresh_resident();
          double part = 0.0;
#pragma unroll
          for (int i = 0; i < kResident; ++i) {
            const int gi = g_begin + i * NT + tid;
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const float qk = dense ? qv[i][e] : (gi * 8 + e == x ? 1.0f : 0.0f);
              acc += fmaxf(fc[i][e] - qk, 0.0f);
            }
            part += static_cast<double>(acc);
          }
          part = block_sum<NT>(part, sh_red);
          unsigned int missing = exchange_begin<NT>(a, b, g, nexch++, part, sh_part, &sh_missing);
          while (missing != 0u) {
            const int who = __ffs(static_cast<int>(missing)) - 1;
            missing &= missing - 1u;
            const int gb = min(ngroups, who * slice), ge = min(ngroups, gb + slice);
            const double theirs = block_sum<NT>(resident_mass_from_memory<T, TQ, NT>(rv, gb, ge, x), sh_red);
            exchange_fill(sh_part, who, theirs);
            __syncthreads();  // (sh_red is free again)
          }
        } else {
          int who = g;
          unsigned int missing = 0u;
          for (;;) {
            const int gb = min(ngroups, who * slice), ge = min(ngroups, gb + slice);
            const double part = block_sum<NT>(residual_mass_slice<T, TQ, NT>(rv, gb, ge, x), sh_red);
            if (who == g) {
              missing = exchange_begin<NT>(a, b, g, nexch++, part, sh_part, &sh_missing);
            } else {
              exchange_fill(sh_part, who, part);
              __syncthreads();  // (sh_red is free again)
            }
            if (missing == 0u) break;
            who = __ffs(static_cast<int>(missing)) - 1;
            missing &= missing - 1u;
          }
        }
        const double Z = exchange_end(a, sh_part);
        last_norm = static_cast<float>(Z);
        inv = Z > 0.0 ? static_cast<float>(1.0 / Z) : 0.0f;  // 0: f is left as it is
      }
      if (tid == 0) { sh_ctok[rv.ch.n] = x; sh_cinv[rv.ch.n] = inv; }
#pragma unroll
      for (int j = 0; j < kChainRegs; ++j)
        if (j == rv.ch.n) { rv.ch.rtok[j] = x; rv.ch.rinv[j] = inv; }
      rv.ch.n += 1;
      passes += 1;
      __syncthreads();
    }
    if (accepted < 0) break;
    cnode = accepted;
    plen += 1;
  }

  // ---------------------------------------------------------------- inverse-CDF draw from f at cnode
  const mars_row_stat st = sh_st[cnode];
  // Without a rejection at this node f is the plain softmax: the draft distribution is not read.
  // (A resident slice that was loaded for a rejection already holds it.)
  rv.use_q = dense && rv.ch.n > 0;
  // Tiles of the slice, in vocabulary order.  Resident slice: a tile is one step (64 groups).
  // Otherwise wave w owns a contiguous run of steps and a tile is `rep` consecutive steps of it.
  const int steps_per_wave = (nsteps + NW - 1) / NW;
  const int rep = max(1, (steps_per_wave * NW + kMaxTiles - 1) / kMaxTiles);
  const int tiles_per_wave = (steps_per_wave + rep - 1) / rep;
  const int ntiles = resident ? nsteps : tiles_per_wave * NW;

  auto step_group = [&](int w, int sw) {  // streamed slice: group of this lane in step sw of wave w, -1 = none
    const int gi = g_begin + (w * steps_per_wave + sw) * kWave + lane;
    return (sw < steps_per_wave && gi < g_end) ? gi : -1;
  };
  auto group_sum = [&](const float (&z)[8], const float (&q)[8], int gi, float (&f)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = rv.f(z, q, gi, e);
    return ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
  };

  double total = 0.0, before = 0.0;
  int owner = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
    // This work-group's slice first (tile sums into sh_tile, which the search below reads), then (rarely)
    // those of partners that have not arrived (into sh_tile2); the two forms as above.
    if (resident) {
      refresh_resident();
#pragma unroll
      for (int i = 0; i < kResident; ++i) {
        const int s = i * NW + wave;
        if (s < nsteps) {  // wave-uniform
          const float gs = ((fc[i][0] + fc[i][1]) + (fc[i][2] + fc[i][3])) +
                           ((fc[i][4] + fc[i][5]) + (fc[i][6] + fc[i][7]));
          const double t = wave_sum(static_cast<double>(gs));
          if (lane == 0) sh_tile[s] = t;
        }
      }
      __syncthreads();
      // slice total = sum of its tiles, taken by the same prefix scheme the search below uses
      unsigned int missing = exchange_begin<NT>(a, b, g, N + attempt, tile_total(sh_tile, nsteps, lane), sh_part, &sh_missing);
      while (missing != 0u) {
        const int who = __ffs(static_cast<int>(missing)) - 1;
        missing &= missing - 1u;
        const int gb = min(ngroups, who * slice), ge = min(ngroups, gb + slice);
        const int nt = resident_tiles_from_memory<T, TQ, NT, kResident>(rv, gb, ge, sh_tile2);
        __syncthreads();
        exchange_fill(sh_part, who, tile_total(sh_tile2, nt, lane));
        __syncthreads();  // (sh_tile2 may be filled again)
      }
    } else {
      int who = g;
      unsigned int missing = 0u;
      for (;;) {
        const int gb = min(ngroups, who * slice), ge = min(ngroups, gb + slice);
        double* tiles = who == g ? sh_tile : sh_tile2;
        // tile sums of a streamed slice, kPassBatch steps of loads in flight at a time
        const int spw = (((ge - gb + kWave - 1) / kWave) + NW - 1) / NW;  // steps per wave of this slice
        const int rp = max(1, (spw * NW + kMaxTiles - 1) / kMaxTiles);
        const int tpw = (spw + rp - 1) / rp;
        auto group_at = [&](int sw) {  // group of this lane in step sw of its wave, -1 = none
          const int gi = gb + (wave * spw + sw) * kWave + lane;
          return (sw < spw && gi < ge) ? gi : -1;
        };
        double acc = 0.0;
        for (int s0 = 0; s0 < spw; s0 += kPassBatch) {
          float z[kPassBatch][8], q[kPassBatch][8];
#pragma unroll
          for (int i = 0; i < kPassBatch; ++i) {  // (no load under a per-lane condition: a lane without a group
            const int gi = group_at(s0 + i);      // reads the row's last one and ignores it, and the loads of a
            rv.load(gi >= 0 ? gi : ngroups - 1, z[i], q[i]);  // batch go out together instead of one by one)
          }
#pragma unroll
          for (int i = 0; i < kPassBatch; ++i) {
            const int sw = s0 + i;
            if (sw < spw) {
              const int gi = group_at(sw);
              if (gi >= 0) { float f[8]; acc += static_cast<double>(group_sum(z[i], q[i], gi, f)); }
              if ((sw + 1) % rp == 0 || sw + 1 == spw) {
                const double t = wave_sum(acc);
                if (lane == 0) tiles[wave * tpw + sw / rp] = t;
                acc = 0.0;
              }
            }
          }
        }
        __syncthreads();
        const double slice_total = tile_total(tiles, tpw * NW, lane);
        if (who == g) {
          missing = exchange_begin<NT>(a, b, g, N + attempt, slice_total, sh_part, &sh_missing);
        } else {
          exchange_fill(sh_part, who, slice_total);
          __syncthreads();  // (sh_tile2 may be filled again)
        }
        if (missing == 0u) break;
        who = __ffs(static_cast<int>(missing)) - 1;
        missing &= missing - 1u;
      }
    }
    // Which work-group's slice holds the target?  The last one with mass if rounding leaves none.  Lane i
    // holds the total of work-group i and the prefix up to it; the grand total is the last prefix.
    {
      const double pg = lane < G ? sh_part[lane] : 0.0;
      const double pincl = wave_prefix_sum(pg);
      total = lane_value(pincl, kWave - 1);
      const double target = static_cast<double>(u[N]) * total;
      const unsigned long long hit = __ballot(lane < G && pincl > target);
      const unsigned long long mass = __ballot(lane < G && pg > 0.0);
      if (hit != 0ull) owner = __ffsll(static_cast<long long>(hit)) - 1;
      else owner = mass != 0ull ? 63 - __clzll(static_cast<long long>(mass)) : 0;
      before = lane_value(pincl - pg, owner);
    }
    __syncthreads();
    if (!(pending_norm && total <= 0.0)) break;
    // The postponed normaliser turned out to be 0: that rejection leaves f as it was
    // (cannot happen in exact arithmetic).  Drop it from the chain and draw again.
    if (tid == 0) sh_cinv[rv.ch.n - 1] = 0.0f;
#pragma unroll
    for (int j = 0; j < kChainRegs; ++j)
      if (j == rv.ch.n - 1) rv.ch.rinv[j] = 0.0f;
    pending_norm = false;
    last_norm = 0.0f;
    have = false;
    raw = false;
    applied = 0;
    __syncthreads();
  }
  if (pending_norm) last_norm = static_cast<float>(total);
  const double target = static_cast<double>(u[N]) * total;
  if (g == 0 && tid == 0) a.len[b] = plen;
  // (The request's status was set to MARS_REQ_OK by the row reduction of this call.)
  // V_out (Alg. 1): the accepted drafts were written as they were accepted; the first work-group
  // pads behind the slot of the final token, which the work-group that draws it fills in.  (No
  // address is written by two work-groups.)
  if (g == 0 && a.out_tok) {
    for (int j = plen + 1 + tid; j < N; j += NT) a.out_tok[rb + j] = -1;
    if (tid == 0) a.out_len[b] = plen + 1;
  }
  if (g != owner) return;

  // The owning work-group locates the tile (every wave does, from the same LDS values).
  int tile = -1;
  double cum = before;
  if (total > 0.0) tile_find(sh_tile, ntiles, lane, before, target, tile, cum);
  // One wave finishes: the one holding the tile in registers, or wave 0 re-reading it.
  const int finder = (resident && tile >= 0) ? tile % NW : 0;
  if (wave != finder) return;

  int pick = -1;
  float pick_f = 0.0f;
  if (total > 0.0) {
    const int tw = resident ? 0 : tile / tiles_per_wave, ts = resident ? 0 : (tile % tiles_per_wave) * rep;
    const int nrep = resident ? 1 : rep;
    int last_pos_v = -1;
    float last_pos_f = 0.0f;
    for (int r = 0; r < nrep && pick < 0; ++r) {
      int gi;
      float f[8];
      float gs = 0.0f;
      if (resident) {
        const int ii = tile / NW;
        gi = g_begin + ii * NT + tid;
        if (gi >= g_end) gi = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = 0.0f;
#pragma unroll
        for (int i = 0; i < kResident; ++i)
          if (i == ii) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = fc[i][e];
          }
        gs = ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
      } else {
        gi = step_group(tw, ts + r);
        if (gi >= 0) {
          float z[8], q[8];
          rv.load(gi, z, q);
          gs = group_sum(z, q, gi, f);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] = 0.0f;
        }
      }
      const double gincl = wave_prefix_sum(static_cast<double>(gs));
      const unsigned long long hit = __ballot(cum + gincl > target);
      // remember the last element with mass, in case rounding leaves no step above the target
      int my_last = -1;
#pragma unroll
      for (int e = 0; e < 8; ++e) if (f[e] > 0.0f) my_last = e;
      const unsigned long long has = __ballot(my_last >= 0);
      if (has != 0ull) {
        const int hl = 63 - __clzll(static_cast<long long>(has));
        const int le = lane_value(my_last, hl);
        float fv = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) if (e == my_last) fv = f[e];
        last_pos_f = lane_value(fv, hl);
        last_pos_v = lane_value(gi, hl) * 8 + le;
      }
      if (hit != 0ull) {
        const int hl = __ffsll(static_cast<long long>(hit)) - 1;
        double run = cum + lane_value(gincl - static_cast<double>(gs), hl);
        int pe = -1;
        float pf = 0.0f;
        if (lane == hl) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (pe < 0) {
              run += static_cast<double>(f[e]);
              if (run > target) { pe = e; pf = f[e]; }
            }
          }
        }
        pe = lane_value(pe, hl);
        if (pe >= 0) {
          pick_f = lane_value(pf, hl);
          pick = lane_value(gi, hl) * 8 + pe;
        } else {  // rounding left no step above the target inside the lane: last element with mass
          pick = last_pos_v; pick_f = last_pos_f;
          break;
        }
      } else {
        cum += lane_value(gincl, kWave - 1);
      }
    }
    if (pick < 0) { pick = last_pos_v; pick_f = last_pos_f; }
  }
  if (pick < 0) { pick = st.id1; pick_f = 0.0f; }  // degenerate: no mass anywhere
  if (lane == 0) {
    a.bonus[b] = pick;
    if (a.out_tok) a.out_tok[rb + plen] = pick;
    if (a.diag) {
      mars_req_diag dg;
      dg.bonus_prob = total > 0.0 ? static_cast<float>(static_cast<double>(pick_f) / total) : 0.0f;
      dg.last_residual_norm = last_norm;
      dg.residual_passes = passes;
      dg.last_node = cnode;
      a.diag[b] = dg;
    }
  }
}

template <typename T, typename TQ, bool VEC>
__global__ __launch_bounds__(kSamplingThreads) void tail_sampling_resident_kernel(TailArgs a) {
  tail_sampling_body<T, TQ, true, VEC>(a);
}
template <typename T, typename TQ, bool VEC>
__global__ __launch_bounds__(kStreamingThreads) void tail_sampling_streamed_kernel(TailArgs a) {
  tail_sampling_body<T, TQ, false, VEC>(a);
}

// ---------------------------------------------------------------- cache rows that stay
// After the walk: the rows of the root and of the accepted nodes of every request, as flat row
// numbers bd*N + node, request by request in path order ("standard rollback" of Sec. 3.4 keeps
// exactly these), with the exclusive prefix sums of their counts.  One work-group per set of Bd
// requests (per threshold of a sweep); unused entries of keep_rows are -1.
constexpr int kKeepThreads = 256;
__global__ __launch_bounds__(kKeepThreads) void compact_keep_kernel(const int32_t* __restrict__ out_len,
                                                                    const int32_t* __restrict__ path, int Bd, int N,
                                                                    int32_t* __restrict__ keep_rows,
                                                                    int32_t* __restrict__ keep_offsets) {
  constexpr int NT = kKeepThreads;
  __shared__ int sh_wave[NT / kWave];
  __shared__ int sh_carry;
  const int k = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int32_t* len = out_len + static_cast<size_t>(k) * Bd;
  const int32_t* pth = path + static_cast<size_t>(k) * Bd * N;
  int32_t* rows = keep_rows + static_cast<size_t>(k) * Bd * N;
  int32_t* offs = keep_offsets + static_cast<size_t>(k) * (Bd + 1);
  if (tid == 0) sh_carry = 0;
  __syncthreads();
  for (int b0 = 0; b0 < Bd; b0 += NT) {
    const int b = b0 + tid;
    const int mine = b < Bd ? len[b] : 0;
    // inclusive scan inside the wave, then across the waves of the work-group
    int incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int o = __shfl_up(incl, d, kWave);
      if (lane >= d) incl += o;
    }
    if (lane == kWave - 1) sh_wave[wave] = incl;
    __syncthreads();
    int before = sh_carry;
    for (int w = 0; w < wave; ++w) before += sh_wave[w];
    const int start = before + incl - mine;
    if (b < Bd) {
      offs[b] = start;
      rows[start] = b * N;  // the root's row
      for (int j = 1; j < mine; ++j) rows[start + j] = b * N + pth[static_cast<size_t>(b) * N + j - 1];
    }
    __syncthreads();
    if (tid == NT - 1) sh_carry = before + incl;
    __syncthreads();
  }
  const int total = sh_carry;
  if (tid == 0) offs[Bd] = total;
  for (int i = total + tid; i < Bd * N; i += NT) rows[i] = -1;
}

}  // namespace mars
