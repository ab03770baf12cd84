// LM head fused with the row reduction (paper Eq. 2, z = W h, followed by the top-2
// identification of Sec. 3.3): the logits of a tile are formed on the matrix cores, rounded to
// bf16 in registers, reduced to each row's two largest (value desc, index asc) and dropped --
// they are never written to memory.  Output: partial results in the format of the streaming row
// reduction, so that the per-request kernels behind it are the same.
//
// A work-group owns a slab of BM hidden-state rows and a contiguous run of vocabulary tiles
// (256 entries each).  Per tile it walks the hidden dimension in slabs of 64: both operands are
// staged through LDS (double-buffered, one barrier per slab), four waves in a 2 x 2 arrangement
// each accumulate (BM/2) x 128 logits with v_mfma_f32_32x32x16_bf16.  The weight rows are the
// first MFMA operand and the hidden states the second, so that a lane ends up holding, for one
// hidden-state row, 16 vocabulary entries per accumulator block: the row's top-2 over the wave's
// 128 entries is taken inside the lane, a running pair per row is carried across the tiles of the
// run, and the two halves of a wave and the two waves that share a row meet once at the very end:
// one partial result per (row, run).
#pragma once

#include "common.h"

namespace mars {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kLmThreads = 256;           // 4 waves: 2 (hidden rows) x 2 (vocabulary)
constexpr int kLmBN = 256;                // vocabulary entries per tile
constexpr int kLmBK = 64;                 // hidden-state elements per staged slab
constexpr int kLmStride = kLmBK + 8;      // LDS row stride in elements: 144 bytes, conflict-free 16-byte reads
constexpr int kLmChunks = kLmBK / 8;      // 16-byte chunks per staged row
constexpr int kLmDepth = 2;               // steps between the request of an operand slab and its use
constexpr int kLmMaxBM = 192;             // tallest slab of hidden-state rows (256 no longer fits the register file)

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// The bits of a float as a signed integer with the same order (an involution: negative values
// have their magnitude bits flipped).
__device__ __forceinline__ int lm_ordered(int t) { return t ^ static_cast<int>(static_cast<uint32_t>(t >> 31) >> 1); }
// The bf16 value in the upper half of a key, widened.
__device__ __forceinline__ float lm_key_value(int key) {
  return __int_as_float(static_cast<int>(static_cast<uint32_t>(lm_ordered(key & static_cast<int>(0xFFFF0000u))) & 0xFFFF0000u));
}

// Staging of one operand slab: n 16-byte chunks per thread, rows 32 apart.
template <int n>
__device__ __forceinline__ void lm_load_global(u32x4 (&g)[n], const bf16_t* __restrict__ base,
                                               const unsigned int (&off)[n], int k) {
#pragma unroll
  for (int i = 0; i < n; ++i) g[i] = *reinterpret_cast<const u32x4*>(base + off[i] + k);
}
template <int n>
__device__ __forceinline__ void lm_store_lds(const u32x4 (&g)[n], bf16_t* first) {
#pragma unroll
  for (int i = 0; i < n; ++i) *reinterpret_cast<u32x4*>(first + i * 32 * kLmStride) = g[i];
}

// n operand fragments (16 bytes per lane each) of rows 32 apart.
template <int n>
__device__ __forceinline__ void lm_load_frags(u32x4 (&f)[n], const bf16_t* first) {
#pragma unroll
  for (int i = 0; i < n; ++i) f[i] = *reinterpret_cast<const u32x4*>(first + i * 32 * kLmStride);
}

// SAMPLING (Eq. 2 followed by Eq. 3): the rounded logits are also written out, once, from the registers
// they are formed in (the residual passes of the sampling walk read rows of them again), and each row's
// sum of exp2(z*c - ref) is taken on the way, against an integer-valued reference per row that moves up with
// the row's running maximum -- the same (reference, sum) pairs the streaming row reduction leaves.
template <int BM, bool SAMPLING>
__global__ __launch_bounds__(kLmThreads) void lmhead_reduce_kernel(const bf16_t* __restrict__ hidden,
                                                                   const bf16_t* __restrict__ weight, int M, int V,
                                                                   int H, int slabs, int tiles_n, int tiles_per_run,
                                                                   int runs, Partial* __restrict__ partials,
                                                                   bf16_t* __restrict__ logits_out, float c) {
  constexpr int WM = BM / 2;      // hidden-state rows per wave
  constexpr int IB = WM / 32;     // 32-row blocks per wave
  constexpr int JB = 4;           // 32-entry vocabulary blocks per wave (128 entries)
  constexpr int A_LOADS = BM * kLmChunks / kLmThreads;      // 16-byte loads per thread and slab, hidden states
  constexpr int W_LOADS = kLmBN * kLmChunks / kLmThreads;   // ... weight rows
  static_assert(BM % 64 == 0 && BM >= 64 && BM <= kLmMaxBM, "slab height");

  __shared__ __attribute__((aligned(16))) bf16_t sh_a[2][BM][kLmStride];
  __shared__ __attribute__((aligned(16))) bf16_t sh_w[2][kLmBN][kLmStride];

  // (run, slab) pairs are dealt out die by die (block index mod 8 is the die): the slabs of a run
  // sit next to each other on one die and read the same weight tiles at the same time.
  const int per_die = gridDim.x >> 3;
  const int pair = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
  if (pair >= runs * slabs) return;
  const int run = pair / slabs, slab = pair - run * slabs;
  const int m0 = slab * BM;
  const int tile_begin = run * tiles_per_run, tile_end = min(tiles_n, tile_begin + tiles_per_run);

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wn = wave & 1, wm = wave >> 1;
  const int l32 = lane & 31, half = lane >> 5;
  const int KT = H / kLmBK;

  // What this thread stages per slab of 64: 16-byte chunk tid%8 of rows tid/8, tid/8 + 32, ...
  // of the tile (rows past the end are clamped to the last valid row; their values are never
  // used).  Tile base pointers are uniform, the offsets inside a tile fit 32 bits.
  const int srow = tid / kLmChunks, schunk = (tid % kLmChunks) * 8;
  const bf16_t* __restrict__ a_tile = hidden + static_cast<size_t>(m0) * H;
  unsigned int a_off[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i)
    a_off[i] = static_cast<unsigned int>(min(M - 1 - m0, srow + i * 32)) * H + schunk;

  unsigned long long best1[IB], best2[IB];
  float sref[IB], ssum[IB];  // SAMPLING: reference (already times c) and sum of this lane's share of its rows
#pragma unroll
  for (int ib = 0; ib < IB; ++ib) { best1[ib] = 0ull; best2[ib] = 0ull; sref[ib] = -1.0e30f; ssum[ib] = 0.0f; }

  // The run is one sequence of steps (tile, slab of 64) whose operand requests do not stop at
  // tile boundaries.  A step's operands are requested kLmDepth steps ahead into one of kLmDepth
  // register sets -- a weight line comes from HBM, microseconds away under load, while a step's
  // multiplications take well under one -- and pass through LDS one step ahead of their use.
  // (KT is a multiple of kLmDepth, so every tile starts with register set 0.)
  constexpr int D = kLmDepth;
  u32x4 ga[D][A_LOADS], gw[D][W_LOADS];
  int l_kt = 0, l_tile = tile_begin;  // the step the next request is for
  // With a single slab of at most 128 rows (the kernel then streams the weight at the memory rate)
  // every run walks the hidden dimension from a starting slab of its own and wraps round -- a sum
  // in another order.  The rows of a tile lie a whole multiple of 128 bytes apart, so work-groups
  // in step would otherwise ask for the same address bits 7..12 all over the chip at the same
  // time; staggered, the weight streams 7 % faster (3 % at 120 rows).  From 180 rows on nothing
  // is gained, and with several slabs it costs 2-5 %: the work-groups of a die would no longer
  // read the same columns of the hidden states at the same time.
  int l_kp = M <= 128 ? (run * 37) % KT : 0;  // the slab of 64 the next request reads
  const bf16_t* __restrict__ w_tile = weight + static_cast<size_t>(l_tile) * kLmBN * H;
  unsigned int w_off[W_LOADS];
#pragma unroll
  for (int i = 0; i < W_LOADS; ++i)
    w_off[i] = static_cast<unsigned int>(min(V - 1 - l_tile * kLmBN, srow + i * 32)) * H + schunk;

  // (Requests are unconditional on purpose: with a request under a branch the compiler has to
  // place its s_waitcnt for the case that nothing was issued, which makes every step wait for the
  // loads it has just sent.  Past the end of the run the last slab is simply requested again.
  // The bookkeeping with its branch is kept apart from the loads, which the steps below issue one
  // by one between their matrix instructions.)
#define MARS_LM_REQUEST(SET)                                                                        \
  {                                                                                                 \
    lm_load_global<A_LOADS>(ga[SET], a_tile, a_off, l_kp * kLmBK);                                  \
    lm_load_global<W_LOADS>(gw[SET], w_tile, w_off, l_kp * kLmBK);                                  \
  }
#define MARS_LM_ADVANCE()                                                                           \
  if (++l_kp == KT) l_kp = 0;                                                                       \
  if (++l_kt == KT) {                                                                               \
    l_kt = 0;                                                                                       \
    l_tile = min(l_tile + 1, tile_end - 1);                                                         \
    w_tile = weight + static_cast<size_t>(l_tile) * kLmBN * H;                                      \
    _Pragma("unroll") for (int i = 0; i < W_LOADS; ++i)                                             \
      w_off[i] = static_cast<unsigned int>(min(V - 1 - l_tile * kLmBN, srow + i * 32)) * H + schunk; \
  }

#pragma unroll
  for (int u = 0; u < D; ++u) {
    MARS_LM_REQUEST(u)
    MARS_LM_ADVANCE()
  }
  lm_store_lds<A_LOADS>(ga[0], &sh_a[0][srow][schunk]);
  lm_store_lds<W_LOADS>(gw[0], &sh_w[0][srow][schunk]);
  __syncthreads();
  // operand fragments of the current and the next quarter (lane l: row l%32 of its block,
  // elements 8*(l/32) .. +7 of the 16-deep quarter)
  u32x4 wf[2][JB], hf[2][IB];
  lm_load_frags<JB>(wf[0], &sh_w[0][wn * 128 + l32][half * 8]);
  lm_load_frags<IB>(hf[0], &sh_a[0][wm * WM + l32][half * 8]);

  int step = 0;  // the step being multiplied
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    f32x16_t acc[JB][IB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[jb][ib][r] = 0.0f;

    for (int kt = 0; kt < KT; kt += D) {
#pragma unroll
      for (int u = 0; u < D; ++u, ++step) {
        const int cur = step & 1;
        // Four 16-deep multiplication quarters of twelve MFMAs.  A wave is alone on its SIMD, so
        // nothing hides a memory instruction's issue time or an LDS round trip but its own matrix
        // instructions: every memory instruction of the step is slotted between two MFMAs (the
        // code is written in that order and a scheduling barrier behind every MFMA keeps the
        // compiler from regrouping it).  Quarters 0..2: the fragments of the next quarter
        // (7 LDS reads), the step's operand request for two steps ahead (set u held this step's
        // operands, which are in LDS by now: 14 global loads) and the operands of the next step
        // (set u+1, requested a step ago: 14 LDS writes into the other stage).  The step's only
        // barrier follows quarter 2 -- by then this stage has been read for the last time (quarter
        // 3's fragments are in registers) and the other one is complete -- so that quarter 3 can
        // already fetch the next step's first fragments.
        constexpr int kRounds = kLmBK / 16;
        constexpr int kMfma = JB * IB;  // MFMAs per quarter
        const bf16_t* __restrict__ a_src = a_tile + l_kp * kLmBK;
        const bf16_t* __restrict__ w_src = w_tile + l_kp * kLmBK;
#pragma unroll
        for (int ks = 0; ks < kRounds; ++ks) {
          const bool last = ks + 1 == kRounds;
          // where the fragments of the next quarter come from: this stage, or (quarter 3) the next step's
          const bf16_t* wsrc = last ? &sh_w[cur ^ 1][wn * 128 + l32][half * 8]
                                    : &sh_w[cur][wn * 128 + l32][(ks + 1) * 16 + half * 8];
          const bf16_t* hsrc = last ? &sh_a[cur ^ 1][wm * WM + l32][half * 8]
                                    : &sh_a[cur][wm * WM + l32][(ks + 1) * 16 + half * 8];
          // this quarter's share of the request (set u) and of the LDS writes (set u+1): rows ks,
          // ks+3, ... of either operand; none in quarter 3 (behind the barrier)
          const int nA = (last || ks >= A_LOADS) ? 0 : (A_LOADS - ks + kRounds - 2) / (kRounds - 1);
          const int nW = (last || ks >= W_LOADS) ? 0 : (W_LOADS - ks + kRounds - 2) / (kRounds - 1);
          const int nmoves = nA + nW;
#pragma unroll
          for (int i = 0; i < kMfma; ++i) {
            const int jb = i / IB, ib = i % IB;
            acc[jb][ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wf[ks & 1][jb]),
                                                                  __builtin_bit_cast(bf16x8_t, hf[ks & 1][ib]),
                                                                  acc[jb][ib], 0, 0, 0);
            // one fragment of the next quarter behind each of the first MFMAs
#pragma unroll
            for (int r = 0; r < JB + IB; ++r)
              if (min(r, kMfma - 1) == i) {
                if (r < JB) wf[(ks + 1) & 1][r] = *reinterpret_cast<const u32x4*>(wsrc + r * 32 * kLmStride);
                else hf[(ks + 1) & 1][r - JB] = *reinterpret_cast<const u32x4*>(hsrc + (r - JB) * 32 * kLmStride);
              }
            // a global load and an LDS write behind some of them, none behind the last two (the
            // barrier after quarter 2 should not have to wait for an LDS instruction just issued)
#pragma unroll
            for (int m = 0; m < nmoves; ++m)
              if (1 + m * (kMfma - 3) / nmoves == i) {  // slots 1 .. kMfma - 3
                if (m < nA) {
                  const int j = ks + m * (kRounds - 1);
                  ga[u][j] = *reinterpret_cast<const u32x4*>(a_src + a_off[j]);
                  *reinterpret_cast<u32x4*>(&sh_a[cur ^ 1][srow + j * 32][schunk]) = ga[(u + 1) % D][j];
                } else {
                  const int j = ks + (m - nA) * (kRounds - 1);
                  gw[u][j] = *reinterpret_cast<const u32x4*>(w_src + w_off[j]);
                  *reinterpret_cast<u32x4*>(&sh_w[cur ^ 1][srow + j * 32][schunk]) = gw[(u + 1) % D][j];
                }
              }
            __builtin_amdgcn_sched_barrier(0);  // keep this order
          }
          if (ks + 2 == kRounds) __syncthreads();
        }
        MARS_LM_ADVANCE()
      }
    }

    // The tile's logits, in this lane: hidden-state row m0 + wm*WM + ib*32 + l32, vocabulary
    // entries n0 + wn*128 + jb*32 + 8*(r/4) + 4*half + r%4.  Round to bf16 (two at a time, the
    // hardware conversion: nearest even), take the top-2 of the 16*JB entries per row block with
    // signed 32-bit keys: the bf16 pattern made order-preserving in the upper half, 127 - entry
    // below it (larger value first, then the lower entry; `half` is the same for all of a
    // lane's entries and is added afterwards).  INT_MIN = no candidate.
    const int n0 = tile * kLmBN;
    const int nbase = n0 + wn * 128 + 4 * half;
    const bool ragged = n0 + kLmBN > V;
    constexpr int kNone = -2147483647 - 1;
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
      int k1 = kNone, k2 = kNone;
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) {
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const f32x2_t pair = {acc[jb][ib][r], acc[jb][ib][r + 1]};
          const uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int e = jb * 32 + 8 * (r / 4) + (r % 4) + h;
            // widened again; + 0 turns -0 into +0, so that equal values have equal keys
            const int t = __float_as_int(__uint_as_float(h ? (w & 0xFFFF0000u) : (w << 16)) + 0.0f);
            int key = static_cast<int>((static_cast<uint32_t>(lm_ordered(t)) & 0xFFFF0000u) | static_cast<uint32_t>(127 - e));
            if (ragged && nbase + e >= V) key = kNone;
            const int lo = min(k1, key);
            k1 = max(k1, key);
            k2 = max(k2, lo);
          }
        }
        // one accumulator block at a time: the operand sets in flight stay in their registers
        __builtin_amdgcn_sched_barrier(0);
      }
      if (k1 != kNone)
        top2_insert(best1[ib], best2[ib], make_key(lm_key_value(k1), nbase + 127 - (k1 & 0x7F)));
      if (k2 != kNone)
        top2_insert(best1[ib], best2[ib], make_key(lm_key_value(k2), nbase + 127 - (k2 & 0x7F)));
      if (SAMPLING && k1 != kNone) {
        // Second pass over the block row, now that its maximum is known: move the reference if the maximum
        // has risen above it (references are integers, so sums against different ones combine by exact
        // powers of two), store the rounded logits -- four consecutive entries, 8 bytes, at a time; lane
        // l + 32 holds the next four -- and add their exponentials.
        const float nref = __builtin_ceilf(lm_key_value(k1) * c);
        if (nref > sref[ib]) {
          ssum[ib] *= __builtin_amdgcn_exp2f(sref[ib] - nref);
          sref[ib] = nref;
        }
        const int row = m0 + wm * WM + ib * 32 + l32;
        bf16_t* __restrict__ orow = logits_out + static_cast<size_t>(min(row, M - 1)) * static_cast<size_t>(V);
        float add = 0.0f;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const f32x2_t p0 = {acc[jb][ib][4 * q4], acc[jb][ib][4 * q4 + 1]};
            const f32x2_t p1 = {acc[jb][ib][4 * q4 + 2], acc[jb][ib][4 * q4 + 3]};
            const uint32_t w0 = __builtin_bit_cast(uint32_t, __builtin_convertvector(p0, bf16x2_t));
            const uint32_t w1 = __builtin_bit_cast(uint32_t, __builtin_convertvector(p1, bf16x2_t));
            const int e = jb * 32 + 8 * q4;  // first of the four entries, relative to nbase
            if (!ragged || nbase + e + 3 < V) {
              if (row < M) *reinterpret_cast<uint2*>(orow + nbase + e) = make_uint2(w0, w1);
              const float x0 = __uint_as_float(w0 << 16), x1 = __uint_as_float(w0 & 0xFFFF0000u);
              const float x2 = __uint_as_float(w1 << 16), x3 = __uint_as_float(w1 & 0xFFFF0000u);
              add += (__builtin_amdgcn_exp2f(__builtin_fmaf(x0, c, -sref[ib])) +
                      __builtin_amdgcn_exp2f(__builtin_fmaf(x1, c, -sref[ib]))) +
                     (__builtin_amdgcn_exp2f(__builtin_fmaf(x2, c, -sref[ib])) +
                      __builtin_amdgcn_exp2f(__builtin_fmaf(x3, c, -sref[ib])));
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        ssum[ib] += add;
      }
    }
  }
#undef MARS_LM_REQUEST
#undef MARS_LM_ADVANCE

  // Lanes l and l + 32 hold the same rows (different vocabulary entries), and so do the two waves
  // side by side (wn = 0, 1): the half-waves combine through a lane exchange, the waves through LDS
  // (the operand stages are free by now), and wave column 0 writes the one partial result of
  // (row, run).
  __syncthreads();  // every wave is done with the operand stages
  unsigned long long* xch = reinterpret_cast<unsigned long long*>(&sh_a[0][0][0]);  // [wm][ib][32 rows][2 keys]
  float* xsum = reinterpret_cast<float*>(xch + 2 * IB * 32 * 2);                   // [wm][ib][32 rows][ref, sum]
  unsigned long long r1[IB], r2[IB];
  float rR[IB];
  double rS[IB];
#pragma unroll
  for (int ib = 0; ib < IB; ++ib) {
    const unsigned long long o1 = __shfl_xor(best1[ib], 32, kWave), o2 = __shfl_xor(best2[ib], 32, kWave);
    r1[ib] = best1[ib]; r2[ib] = best2[ib];
    top2_insert(r1[ib], r2[ib], o1);
    top2_insert(r1[ib], r2[ib], o2);
    rR[ib] = -3.0e38f; rS[ib] = 0.0;
    if (SAMPLING) {
      const float oR = __shfl_xor(sref[ib], 32, kWave), oS = __shfl_xor(ssum[ib], 32, kWave);
      // (both halves add in the order lower half, upper half: the same bits in either lane)
      const float aR = half == 0 ? sref[ib] : oR, aS = half == 0 ? ssum[ib] : oS;
      const float bR = half == 0 ? oR : sref[ib], bS = half == 0 ? oS : ssum[ib];
      if (aS > 0.0f) absorb_sum(rR[ib], rS[ib], aR, static_cast<double>(aS));
      if (bS > 0.0f) absorb_sum(rR[ib], rS[ib], bR, static_cast<double>(bS));
    }
    if (wn == 1 && half == 0) {
      xch[((wm * IB + ib) * 32 + l32) * 2 + 0] = r1[ib];
      xch[((wm * IB + ib) * 32 + l32) * 2 + 1] = r2[ib];
      if (SAMPLING) {
        xsum[((wm * IB + ib) * 32 + l32) * 2 + 0] = rR[ib];
        xsum[((wm * IB + ib) * 32 + l32) * 2 + 1] = static_cast<float>(rS[ib]);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int ib = 0; ib < IB; ++ib) {
    const int row = m0 + wm * WM + ib * 32 + l32;
    if (wn == 0 && half == 0 && row < M) {
      unsigned long long k1 = r1[ib], k2 = r2[ib];
      top2_insert(k1, k2, xch[((wm * IB + ib) * 32 + l32) * 2 + 0]);
      top2_insert(k1, k2, xch[((wm * IB + ib) * 32 + l32) * 2 + 1]);
      Partial out;
      out.z1 = neg_inf(); out.id1 = -1; out.z2 = neg_inf(); out.id2 = -1; out.s = 0.0f; out.ref = 0.0f;
      if (k1 != 0ull) { out.z1 = key_value(k1); out.id1 = key_index(k1); }
      if (k2 != 0ull) { out.z2 = key_value(k2); out.id2 = key_index(k2); }
      if (SAMPLING) {
        float R = rR[ib];
        double S = rS[ib];
        const float oS = xsum[((wm * IB + ib) * 32 + l32) * 2 + 1];
        if (oS > 0.0f) absorb_sum(R, S, xsum[((wm * IB + ib) * 32 + l32) * 2 + 0], static_cast<double>(oS));
        if (S > 0.0) { out.s = static_cast<float>(S); out.ref = R; }
      }
      partials[static_cast<size_t>(row) * runs + run] = out;
    }
  }
}

}  // namespace mars
