// Per-request tail of the verification pass: merge the row partials, take the
// per-node decisions, select the path and produce the correction / bonus token.
// One work-group per request.
//
// Greedy mode is Algorithm 1 on a tree: local three-way test per node, reachability
// by pointer jumping, deepest reachable node (lowest index on ties), token = v(1) of
// its row.  Sampling mode is multi-round rejection sampling down the tree (Eq. 1) with
// the runner-up relaxation of Sec. 3.4 as a deterministic accept, residual
// renormalisation after every rejection (Sec. 2.3) and an inverse-CDF draw at the end.
#pragma once

#include "common.h"

namespace mars {

constexpr int kGreedyThreads = 256;
constexpr int kSamplingThreads = 1024;
constexpr int kMaxTiles = 512;  // CDF tiles kept in LDS for the final draw

struct TailArgs {
  const void* logits;
  const int32_t* tok;
  const int32_t* par;
  const void* dprobs;  // nullptr = one-hot draft distribution
  const float* theta;
  const float* u;
  const Partial* partials;
  mars_row_stat* stats;  // [B*N], written here (caller's table or workspace)
  uint8_t* mask;
  int32_t* len;
  int32_t* path;
  int32_t* bonus;
  uint8_t* dec;          // optional
  int32_t* status;       // optional
  mars_req_diag* diag;   // optional
  int B, N, V, splits;
  float c;               // log2(e) / T, 0 in greedy mode
};

// ---------------------------------------------------------------- steps shared by both modes
// Merge this request's rows, validate tree and tokens.  Returns the request status
// (uniform over the work-group).  Ends with a barrier: stats of the request are visible.
template <int NT>
__device__ int merge_and_validate(const TailArgs& a, int b) {
  const int N = a.N;
  const float theta = a.theta[b];
  int bad = 0;
  for (int i = threadIdx.x; i < N; i += NT) {
    const size_t r = static_cast<size_t>(b) * N + i;
    merge_row(a.partials + r * a.splits, a.splits, theta, a.c, &a.stats[r]);
    const int p = a.par[r];
    const int t = a.tok[r];
    if (i == 0) { if (p != -1) bad |= 1; }
    else {
      if (p < 0 || p >= i) bad |= 1;
      if (t < 0 || t >= a.V) bad |= 2;
    }
  }
  const int any_tree = __syncthreads_or(bad & 1);
  const int any_tok = __syncthreads_or(bad & 2);
  return any_tree ? MARS_REQ_BAD_TREE : (any_tok ? MARS_REQ_BAD_TOKEN : MARS_REQ_OK);
}

// Outputs of a request that failed validation: nothing accepted, token = v(1) of the root row.
template <int NT>
__device__ void write_rejected_request(const TailArgs& a, int b, int status) {
  const int N = a.N;
  for (int i = threadIdx.x; i < N; i += NT) {
    const size_t r = static_cast<size_t>(b) * N + i;
    a.mask[r] = i == 0 ? 1 : 0;
    a.path[r] = -1;
    if (a.dec) a.dec[r] = 0;
  }
  if (threadIdx.x == 0) {
    a.len[b] = 0;
    a.bonus[b] = a.stats[static_cast<size_t>(b) * N].id1;
    if (a.status) a.status[b] = status;
    if (a.diag) { mars_req_diag d = {0.0f, 0.0f, 0, 0}; a.diag[b] = d; }
  }
}

// ---------------------------------------------------------------- greedy mode
__global__ __launch_bounds__(kGreedyThreads) void tail_greedy_kernel(TailArgs a) {
  constexpr int NT = kGreedyThreads;
  __shared__ uint8_t sh_code[MARS_MAX_NODES];
  __shared__ uint8_t sh_ok[2][MARS_MAX_NODES];
  __shared__ int16_t sh_anc[2][MARS_MAX_NODES];
  __shared__ int16_t sh_dep[2][MARS_MAX_NODES];
  __shared__ unsigned int sh_best;

  const int b = blockIdx.x;
  const int N = a.N;
  const size_t rb = static_cast<size_t>(b) * N;
  const int status = merge_and_validate<NT>(a, b);
  if (status != MARS_REQ_OK) { write_rejected_request<NT>(a, b, status); return; }

  // Local decision of every node against its parent's row (Alg. 1 if-chain).
  for (int i = threadIdx.x; i < N; i += NT) {
    int code = 0, anc = 0, dep = 0;
    if (i > 0) {
      const int p = a.par[rb + i];
      const int t = a.tok[rb + i];
      const mars_row_stat st = a.stats[rb + p];
      if (t == st.id1) code = MARS_DEC_EXACT;
      else if (t == st.id2 && st.relax_ok) code = MARS_DEC_RELAXED;
      anc = p; dep = 1;
    }
    sh_code[i] = static_cast<uint8_t>(code);
    sh_ok[0][i] = (i == 0 || code != 0) ? 1 : 0;
    sh_anc[0][i] = static_cast<int16_t>(anc);
    sh_dep[0][i] = static_cast<int16_t>(dep);
  }
  if (threadIdx.x == 0) sh_best = 0;
  __syncthreads();
  // Pointer jumping: after round k, anc is the 2^k-th ancestor (or the root), dep the number
  // of edges to it and ok the AND of the local decisions along those edges.
  int cur = 0;
  for (int span = 1; span < N; span <<= 1) {
    const int nxt = cur ^ 1;
    for (int i = threadIdx.x; i < N; i += NT) {
      const int an = sh_anc[cur][i];
      sh_ok[nxt][i] = sh_ok[cur][i] & sh_ok[cur][an];
      sh_dep[nxt][i] = static_cast<int16_t>(sh_dep[cur][i] + sh_dep[cur][an]);
      sh_anc[nxt][i] = sh_anc[cur][an];
    }
    cur = nxt;
    __syncthreads();
  }
  // Deepest reachable node, lowest index on ties: max of (depth << 16 | (0xFFFF - i)).
  unsigned int best = 0;
  for (int i = threadIdx.x; i < N; i += NT)
    if (sh_ok[cur][i]) best = max(best, (static_cast<unsigned int>(sh_dep[cur][i]) << 16) | (0xFFFFu - i));
  atomicMax(&sh_best, best);
  for (int i = threadIdx.x; i < N; i += NT) {
    a.mask[rb + i] = i == 0 ? 1 : 0;
    a.path[rb + i] = -1;
    if (a.dec) a.dec[rb + i] = 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int bk = sh_best;
    const int e = 0xFFFF - static_cast<int>(bk & 0xFFFFu);
    const int L = static_cast<int>(bk >> 16);
    int n = e;
    for (int d = L; d >= 1; --d) {
      a.mask[rb + n] = 1;
      a.path[rb + d - 1] = n;
      if (a.dec) a.dec[rb + n] = sh_code[n];
      n = a.par[rb + n];
    }
    a.len[b] = L;
    a.bonus[b] = a.stats[rb + e].id1;  // correction after a rejection, bonus after a leaf
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

// The residual chain at the current node: rejection j replaced f by
// max(0, f - q_j) * inv_norm[j] (q_j dense, or one-hot at tok[j]).
struct Chain {
  const int32_t* tok;      // LDS
  const float* inv_norm;   // LDS; 0 marks "Z was 0, f left unchanged"
  int n;
};

// f(v) for the current node: softmax term, then the residual chain.
__device__ __forceinline__ float eval_f(float z, float q, int v, float z1, float c, float inv_S, bool dense,
                                        const Chain& ch) {
  float f = __builtin_amdgcn_exp2f((z - z1) * c) * inv_S;
  for (int j = 0; j < ch.n; ++j) {
    const float qj = dense ? q : (v == ch.tok[j] ? 1.0f : 0.0f);
    const float g = fmaxf(f - qj, 0.0f);
    const float inv = ch.inv_norm[j];
    f = inv > 0.0f ? g * inv : f;
  }
  return f;
}

template <int NT>
__device__ __forceinline__ double block_sum(double v, double* sh) {
  v = wave_sum(v);
  __syncthreads();
  if (threadIdx.x % kWave == 0) sh[threadIdx.x / kWave] = v;
  __syncthreads();
  double t = 0.0;
#pragma unroll
  for (int w = 0; w < NT / kWave; ++w) t += sh[w];
  return t;
}

template <typename T, typename TQ>
__global__ __launch_bounds__(kSamplingThreads) void tail_sampling_kernel(TailArgs a) {
  constexpr int NT = kSamplingThreads;
  constexpr int NW = NT / kWave;
  __shared__ int16_t sh_first[MARS_MAX_NODES];   // first child (-1 none)
  __shared__ int16_t sh_next[MARS_MAX_NODES];    // next sibling (-1 none)
  __shared__ int32_t sh_ctok[MARS_MAX_NODES];    // residual chain: rejected tokens
  __shared__ float sh_cinv[MARS_MAX_NODES];      // residual chain: 1/Z
  __shared__ double sh_red[NW];
  __shared__ double sh_tile[kMaxTiles];
  __shared__ int sh_accept;                      // decision code of the child under test

  const int b = blockIdx.x;
  const int N = a.N, V = a.V;
  const size_t rb = static_cast<size_t>(b) * N;
  const int tid = threadIdx.x;
  const int status = merge_and_validate<NT>(a, b);
  if (status != MARS_REQ_OK) { write_rejected_request<NT>(a, b, status); return; }

  // Child lists in increasing node index.
  for (int i = tid; i < N; i += NT) {
    int fc = -1, ns = -1;
    for (int j = i + 1; j < N; ++j)
      if (a.par[rb + j] == i) { fc = j; break; }
    if (i > 0) {
      const int p = a.par[rb + i];
      for (int j = i + 1; j < N; ++j)
        if (a.par[rb + j] == p) { ns = j; break; }
    }
    sh_first[i] = static_cast<int16_t>(fc);
    sh_next[i] = static_cast<int16_t>(ns);
    a.mask[rb + i] = i == 0 ? 1 : 0;
    a.path[rb + i] = -1;
    if (a.dec) a.dec[rb + i] = 0;
  }
  __syncthreads();

  const T* __restrict__ zall = static_cast<const T*>(a.logits) + rb * static_cast<size_t>(V);
  const TQ* __restrict__ qall = a.dprobs ? static_cast<const TQ*>(a.dprobs) + rb * static_cast<size_t>(V) : nullptr;
  const bool dense = qall != nullptr;
  const bool vec_ok = (V % 8 == 0) && (reinterpret_cast<uintptr_t>(zall) % 16 == 0) &&
                      (!dense || reinterpret_cast<uintptr_t>(qall) % 16 == 0);
  const int ngroups = (V + 7) / 8;
  const float c = a.c;
  const float* __restrict__ u = a.u + static_cast<size_t>(b) * (N + 1);

  int cnode = 0, plen = 0, passes = 0;
  float last_norm = 0.0f;
  Chain ch = {sh_ctok, sh_cinv, 0};
  for (;;) {
    const mars_row_stat st = a.stats[rb + cnode];
    const float inv_S = 1.0f / st.sum_exp;
    const T* __restrict__ zrow = zall + static_cast<size_t>(cnode) * V;
    const TQ* __restrict__ qrow = dense ? qall + static_cast<size_t>(cnode) * V : nullptr;
    ch.n = 0;
    int k = sh_first[cnode];
    int accepted = -1;
    while (k >= 0) {
      const int x = a.tok[rb + k];
      if (tid == 0) {
        int code = 0;
        if (x == st.id2 && st.relax_ok) {
          code = MARS_DEC_RELAXED;  // runner-up in a low-margin row: accepted outright
        } else {
          const float qx = dense ? widen(qrow[x]) : 1.0f;
          const float fx = eval_f(widen(zrow[x]), qx, x, st.z1, c, inv_S, dense, ch);
          // Eq. 1: accept with probability min(1, f(x)/q(x))
          float acc;
          if (fx == 0.0f) acc = 0.0f;
          else if (qx <= 0.0f) acc = 1.0f;
          else acc = fminf(1.0f, fx / qx);
          if (u[k] < acc) code = MARS_DEC_SAMPLED;
        }
        sh_accept = code;
      }
      __syncthreads();
      const int code = sh_accept;
      __syncthreads();  // everyone has read the decision before thread 0 may overwrite it
      if (code) {
        if (tid == 0) {
          a.mask[rb + k] = 1;
          a.path[rb + plen] = k;
          if (a.dec) a.dec[rb + k] = static_cast<uint8_t>(code);
        }
        accepted = k;
        break;
      }
      // Rejected: Z = sum_v max(0, f(v) - q_k(v)) over the whole row, f the current distribution.
      double part = 0.0;
      for (int g = tid; g < ngroups; g += NT) {
        float z[8], q[8];
        load8<T>(zrow, g, V, vec_ok, neg_inf(), z);
        if (dense) load8<TQ>(qrow, g, V, vec_ok, 0.0f, q);
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int v = g * 8 + e;
          const float f = eval_f(z[e], dense ? q[e] : 0.0f, v, st.z1, c, inv_S, dense, ch);
          const float qk = dense ? q[e] : (v == x ? 1.0f : 0.0f);
          acc += fmaxf(f - qk, 0.0f);
        }
        part += static_cast<double>(acc);
      }
      const double Z = block_sum<NT>(part, sh_red);
      if (tid == 0) {
        sh_ctok[ch.n] = x;
        sh_cinv[ch.n] = Z > 0.0 ? static_cast<float>(1.0 / Z) : 0.0f;
      }
      ch.n += 1;
      passes += 1;
      last_norm = static_cast<float>(Z);
      __syncthreads();
      k = sh_next[k];
    }
    if (accepted < 0) break;
    cnode = accepted;
    plen += 1;
  }

  // ---------------------------------------------------------------- inverse-CDF draw from f at cnode
  const mars_row_stat st = a.stats[rb + cnode];
  const float inv_S = 1.0f / st.sum_exp;
  const T* __restrict__ zrow = zall + static_cast<size_t>(cnode) * V;
  const TQ* __restrict__ qrow = dense ? qall + static_cast<size_t>(cnode) * V : nullptr;
  // Wave w owns a contiguous run of groups; a tile is `rep` consecutive 64-group steps of a wave.
  const int steps_total = (ngroups + kWave - 1) / kWave;
  const int steps_per_wave = (steps_total + NW - 1) / NW;
  const int rep = (steps_per_wave * NW + kMaxTiles - 1) / kMaxTiles;
  const int tiles_per_wave = (steps_per_wave + rep - 1) / rep;
  const int ntiles = tiles_per_wave * NW;
  const int wave = tid / kWave, lane = tid % kWave;

  auto group_values = [&](int g, float (&f)[8]) {
    float z[8], q[8];
    load8<T>(zrow, g, V, vec_ok, neg_inf(), z);
    if (dense) load8<TQ>(qrow, g, V, vec_ok, 0.0f, q);
#pragma unroll
    for (int e = 0; e < 8; ++e)
      f[e] = eval_f(z[e], dense ? q[e] : 0.0f, g * 8 + e, st.z1, c, inv_S, dense, ch);
  };
  auto tile_step_group = [&](int tile, int r) {  // group handled by this lane in step r of a tile
    const int w = tile / tiles_per_wave, t = tile % tiles_per_wave;
    const int step = w * steps_per_wave + t * rep + r;
    const bool in_wave = (t * rep + r) < steps_per_wave;
    return in_wave ? step * kWave + lane : ngroups;  // ngroups = out of range
  };

  for (int t = 0; t < tiles_per_wave; ++t) {
    const int tile = wave * tiles_per_wave + t;
    double acc = 0.0;
    for (int r = 0; r < rep; ++r) {
      const int g = tile_step_group(tile, r);
      if (g < ngroups) {
        float f[8];
        group_values(g, f);
        acc += static_cast<double>(((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7])));
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) sh_tile[tile] = acc;
  }
  __syncthreads();
  // Wave 0: prefix over the tiles in index order, locate the tile, then the element.
  if (wave == 0) {
    const int per_lane = (ntiles + kWave - 1) / kWave;
    double mine = 0.0;
    for (int i = 0; i < per_lane; ++i) {
      const int t = lane * per_lane + i;
      if (t < ntiles) mine += sh_tile[t];
    }
    double incl = mine;  // inclusive scan over lanes
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const double o = __shfl_up(incl, d, kWave);
      if (lane >= d) incl += o;
    }
    const double total = __shfl(incl, kWave - 1, kWave);
    const double target = static_cast<double>(u[N]) * total;
    // first lane whose inclusive prefix exceeds the target
    const unsigned long long over = __ballot(incl > target);
    int pick = -1;
    float pick_f = 0.0f;
    if (total > 0.0 && over != 0ull) {
      const int L = __ffsll(static_cast<long long>(over)) - 1;
      const double before_lane = __shfl(incl - mine, L, kWave);
      // tiles of lane L in order
      double cum = before_lane;
      int tile = -1;
      for (int i = 0; i < per_lane; ++i) {
        const int t = L * per_lane + i;
        if (t >= ntiles) break;
        const double nxt = cum + sh_tile[t];
        if (nxt > target) { tile = t; break; }
        cum = nxt;
      }
      if (tile < 0) tile = min(ntiles - 1, L * per_lane + per_lane - 1);
      // walk the tile step by step; cum is the mass before the current step
      int last_pos_v = -1;
      float last_pos_f = 0.0f;
      for (int r = 0; r < rep && pick < 0; ++r) {
        const int g = tile_step_group(tile, r);
        float f[8];
        float gs = 0.0f;
        if (g < ngroups) {
          group_values(g, f);
          gs = ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] = 0.0f;
        }
        double gincl = static_cast<double>(gs);
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
          const double o = __shfl_up(gincl, d, kWave);
          if (lane >= d) gincl += o;
        }
        const unsigned long long hit = __ballot(cum + gincl > target);
        // remember the last element with mass, in case rounding leaves no step above the target
        int my_last = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) if (f[e] > 0.0f) my_last = e;
        const unsigned long long has = __ballot(my_last >= 0);
        if (has != 0ull) {
          const int hl = 63 - __clzll(static_cast<long long>(has));
          const int le = __shfl(my_last, hl, kWave);
          float fv = 0.0f;
#pragma unroll
          for (int e = 0; e < 8; ++e) if (e == my_last) fv = f[e];
          last_pos_f = __shfl(fv, hl, kWave);
          last_pos_v = __shfl(g, hl, kWave) * 8 + le;
        }
        if (hit != 0ull) {
          const int hl = __ffsll(static_cast<long long>(hit)) - 1;
          double run = cum + __shfl(gincl - static_cast<double>(gs), hl, kWave);
          // lane hl scans its eight elements
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
          pe = __shfl(pe, hl, kWave);
          if (pe >= 0) {
            pick_f = __shfl(pf, hl, kWave);
            pick = __shfl(g, hl, kWave) * 8 + pe;
          } else {  // rounding left no step above the target inside the lane: last element with mass
            pick = last_pos_v; pick_f = last_pos_f;
            break;
          }
        } else {
          cum += __shfl(gincl, kWave - 1, kWave);
        }
      }
      if (pick < 0) { pick = last_pos_v; pick_f = last_pos_f; }
    }
    if (pick < 0) { pick = st.id1; pick_f = 0.0f; }  // degenerate: no mass anywhere
    if (lane == 0) {
      a.len[b] = plen;
      a.bonus[b] = pick;
      if (a.status) a.status[b] = MARS_REQ_OK;
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
}

}  // namespace mars
