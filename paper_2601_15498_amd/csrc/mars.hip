// C ABI of the MARS verification pass (see include/mars.h): argument checks,
// workspace carving and kernel launches.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

#include "../../include/mars.h"
#include "common.h"
#include "row_reduce.h"
#include "tail.h"
#include "lmhead.h"

namespace mars {

constexpr int kMaxTargetItems = 768;    // work-groups the row reduction aims for on a large input: three per compute unit
                                        // (four fit; 960 rows of 151 936 run faster as 960 work-groups than as 1 920)
constexpr int kMinTargetItems = 128;    // ... and on a small one
constexpr int kItemElemsLog2 = 16;      // in between: about one work-group per 65 536 elements
constexpr int kMinSplitElems = 8192;    // no split shorter than this
constexpr size_t kAlign = 256;
constexpr int kDefaultSpinLimit = 256;  // polls before a work-group stops waiting for a partner's sum

static size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Splits per row: a function of (rows, V) only, so that the workspace size does not depend on
// the element type.  A large input needs several work-groups per compute unit to keep the memory
// pipeline full.  A small one (a single request) is bound by latency, not by bandwidth: the row
// reduction takes about as long with a few hundred work-groups as with a thousand, while every
// split adds partial results that the per-request kernel behind it has to merge.
static int choose_splits(long rows, int V) {
  long target = (rows * static_cast<long>(V)) >> kItemElemsLog2;
  if (target < kMinTargetItems) target = kMinTargetItems;
  if (target > kMaxTargetItems) target = kMaxTargetItems;
  long want = (target + rows - 1) / rows;
  long cap = V / kMinSplitElems;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return static_cast<int>(want);
}

struct Layout {
  int splits, G;
  size_t partials_off, stats_off, xslots_off, gathered_off, total;
};

// Work-groups per request in the sampling tail: enough to spread a request's row passes over
// the chip when there are few requests, not more than one work-group per compute unit in
// total (they exchange sums, and that is quick only while all of them are resident), and every
// slice at least 4096 vocabulary entries long.  The workspace is laid out for the compute units
// of an MI355X; a GPU with fewer gets fewer work-groups per request at launch (below).
constexpr int kComputeUnits = 256;
static int compute_units() {  // of the current GPU, asked once
  static int cached = 0;
  if (cached <= 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      return kComputeUnits;
    cached = n;
  }
  return cached;
}
static int choose_groups(int B, int V) {
  int G = kComputeUnits / B;
  const int cap = V / 4096;
  if (G > cap) G = cap;
  if (G > kMaxGroupsPerRequest) G = kMaxGroupsPerRequest;
  if (G < 1) G = 1;
  return G;
}

// K = thresholds per request: the row reduction works on the B*N rows once, the per-request
// part on K*B requests (statistics table and exchange words per (threshold, request)).
static Layout layout(int B, int N, int V, int K = 1) {
  Layout L;
  const long rows = static_cast<long>(B) * N;
  L.splits = choose_splits(rows, V);
  L.partials_off = 0;
  L.stats_off = align_up(static_cast<size_t>(rows) * L.splits * kPartsPerItem * sizeof(Partial));
  L.G = choose_groups(K * B, V);
  L.xslots_off = L.stats_off + align_up(static_cast<size_t>(K) * rows * sizeof(mars_row_stat));
  L.gathered_off = L.xslots_off +
                   align_up(static_cast<size_t>(K) * B * (N + 2) * 2 * L.G * sizeof(unsigned long long));
  L.total = L.gathered_off + align_up(static_cast<size_t>(rows) * sizeof(float2));
  return L;
}

static bool sizes_ok(int B, int N, int V, int K = 1) {
  if (B < 1 || N < 1 || N > MARS_MAX_NODES || V < MARS_MIN_VOCAB || K < 1 || K > MARS_MAX_THETAS) return false;
  const long rows = static_cast<long>(B) * N * K;
  return rows <= 0x7FFFFFFFL / 64;  // rows * splits must fit the grid and int arithmetic
}

template <typename T, int EPV>
static hipError_t launch_row_reduce_t(const void* logits, long rows, int V, int splits, bool sampling, float c,
                                      Partial* partials, const ClearArgs& clr, hipStream_t stream) {
  const int nvec = V / EPV;
  const int vps = (nvec + splits - 1) / splits;
  const dim3 grid(static_cast<unsigned int>(rows * splits)), block(kRowThreads);
  if (sampling)
    hipLaunchKernelGGL((row_reduce_kernel<T, EPV, true>), grid, block, 0, stream, static_cast<const T*>(logits), V,
                       splits, vps, c, partials, clr);
  else
    hipLaunchKernelGGL((row_reduce_kernel<T, EPV, false>), grid, block, 0, stream, static_cast<const T*>(logits), V,
                       splits, vps, c, partials, clr);
  return hipGetLastError();
}

// 16-byte loads need every row to start on a 16-byte boundary; otherwise the same kernel runs
// with one element per load.
static hipError_t launch_row_reduce(const void* logits, int dtype, long rows, int V, int splits, bool sampling,
                                    float c, Partial* partials, const ClearArgs& clr, hipStream_t stream) {
  const size_t elt = dtype == MARS_BF16 ? 2 : 4;
  const bool wide = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((static_cast<size_t>(V) * elt) % 16 == 0);
  if (dtype == MARS_BF16)
    return wide ? launch_row_reduce_t<bf16_t, 8>(logits, rows, V, splits, sampling, c, partials, clr, stream)
                : launch_row_reduce_t<bf16_t, 1>(logits, rows, V, splits, sampling, c, partials, clr, stream);
  return wide ? launch_row_reduce_t<float, 4>(logits, rows, V, splits, sampling, c, partials, clr, stream)
              : launch_row_reduce_t<float, 1>(logits, rows, V, splits, sampling, c, partials, clr, stream);
}

static float log2e_over_t(float temperature) {
  return temperature > 0.0f ? static_cast<float>(1.4426950408889634 / static_cast<double>(temperature)) : 0.0f;
}

// log2(e) / T' for the probability-ratio indicator: T' is the sampling temperature, 1 in greedy mode.
static double indicator_scale(float temperature) {
  return 1.4426950408889634 / (temperature > 0.0f ? static_cast<double>(temperature) : 1.0);
}

static ClearArgs clear_args(char* ws, const Layout& L, int B, int N, int K) {
  ClearArgs clr;
  clr.xslots = reinterpret_cast<unsigned long long*>(ws + L.xslots_off);
  clr.N = N; clr.B = B; clr.xwords = 2 * L.G; clr.copies = K;
  clr.counters = nullptr; clr.ncounters = 0;
  clr.par = nullptr; clr.tok = nullptr; clr.q = nullptr; clr.q_bf16 = 0; clr.gathered = nullptr;
  return clr;
}

// ---------------------------------------------------------------- LM head fused with the row reduction
// Slab height: the one that costs least for the padded row count (below).  Runs of vocabulary tiles: about one work-group per compute unit in all, so that
// the whole grid is resident at once with the same amount of work for every work-group.  The
// hardware hands work-group i to die i mod 8 and a work-group fills a compute unit, so the
// (run, slab) pairs are dealt out die by die, an equal share to each: the slabs of a run then sit on one die
// (at most two) and find the weight tiles they share in its L2, and no die is given more
// work-groups than it has compute units (its last ones would start when the others have
// finished: twice the time).
struct LmPlan {
  int bm, slabs, tiles_n, tiles_per_run, runs, parts;
};
constexpr int kDies = 8;
static LmPlan lm_plan(long rows, int V) {
  LmPlan p;
  // (time ~ padded rows x cost per row of the slab height: a taller slab reuses a weight tile more,
  // measured 1.2 PFLOP/s with 192 rows against 1.07 with 128; 64 only pays for a single small slab)
  double best = -1.0;
  p.bm = 64;
  for (int bm = 64; bm <= kLmMaxBM; bm += 64) {
    const long padded = (rows + bm - 1) / bm * bm;
    const double cost = static_cast<double>(padded) * (bm == 192 ? 1.0 : bm == 128 ? 1.12 : 1.6);
    if (best < 0.0 || cost <= best) { best = cost; p.bm = bm; }
  }
  p.slabs = static_cast<int>((rows + p.bm - 1) / p.bm);
  p.tiles_n = (V + kLmBN - 1) / kLmBN;
  int want = kComputeUnits / p.slabs;
  if (want < 1) want = 1;
  if (want > p.tiles_n) want = p.tiles_n;
  p.tiles_per_run = (p.tiles_n + want - 1) / want;
  p.runs = (p.tiles_n + p.tiles_per_run - 1) / p.tiles_per_run;
  p.parts = p.runs;  // one partial result per (row, run)
  return p;
}

struct LmLayout {
  LmPlan plan;
  int G;  // work-groups per request of the sampling walk
  size_t partials_off, stats_off, xslots_off, total;
};
static LmLayout lm_layout(int B, int N, int V, int K) {
  LmLayout L;
  const long rows = static_cast<long>(B) * N;
  L.plan = lm_plan(rows, V);
  L.partials_off = 0;
  L.stats_off = align_up(static_cast<size_t>(rows) * L.plan.parts * sizeof(Partial));
  L.G = choose_groups(K * B, V);
  L.xslots_off = L.stats_off + align_up(static_cast<size_t>(K) * rows * sizeof(mars_row_stat));
  L.total = L.xslots_off + align_up(static_cast<size_t>(K) * B * (N + 2) * 2 * L.G * sizeof(unsigned long long));
  return L;
}

// Scratch of mars_verify_static: one copy per GPU, held from the moment the library is loaded on it
// until the process ends.  In host code the array's name is only a handle for the symbol lookup
// below; kernels are given the device address the lookup returns.
static __device__ __align__(256) unsigned char scratch[MARS_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on every GPU seen so far
static std::mutex g_scratch_lock;

// Device address of the current GPU's copy of `scratch` (looked up once per GPU), nullptr on failure.
static void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

// The sampling walk: G work-groups per request (a.G), a.B requests.  draft_dtype < 0: one-hot.
static hipError_t launch_sampling_tail(const TailArgs& a, int logits_dtype, int draft_dtype, hipStream_t stream) {
  const int V = a.V;
  const bool dense = draft_dtype >= 0;
  // Slices of at most kResident groups of eight per thread stay in registers between passes.
  const int ngroups8 = (V + 7) / 8;
  const int slice8 = ((ngroups8 + a.G - 1) / a.G + kWave - 1) / kWave * kWave;
  const bool resident = slice8 <= kResident * kSamplingThreads;
  const bool qbf = dense && draft_dtype == MARS_BF16;
  const void* kernel;
  // groups of eight elements as single aligned loads: whole rows of groups, arrays on 16-byte boundaries
  const bool vec = (V % 8 == 0) && (reinterpret_cast<uintptr_t>(a.logits) % 16 == 0) &&
                   (!dense || reinterpret_cast<uintptr_t>(a.dprobs) % 16 == 0);
#define MARS_PICK2(TT, QQ, VV) (resident ? reinterpret_cast<const void*>(&tail_sampling_resident_kernel<TT, QQ, VV>) \
                                         : reinterpret_cast<const void*>(&tail_sampling_streamed_kernel<TT, QQ, VV>))
#define MARS_PICK(TT, QQ) (vec ? MARS_PICK2(TT, QQ, true) : MARS_PICK2(TT, QQ, false))
  if (logits_dtype == MARS_BF16) kernel = qbf ? MARS_PICK(bf16_t, bf16_t) : MARS_PICK(bf16_t, float);
  else kernel = qbf ? MARS_PICK(float, bf16_t) : MARS_PICK(float, float);
#undef MARS_PICK
#undef MARS_PICK2
  TailArgs copy = a;
  void* params[] = {&copy};
  // With G > 1 the work-groups of a request exchange sums.  The grid never exceeds one work-group
  // per compute unit, so on a GPU that is free to run it all of them are resident together and the
  // exchanges take a couple of microseconds; when other work keeps some of them waiting for a
  // compute unit, those that run work out the missing sums themselves (tail.h: exchange_begin) --
  // slower, same bits, and no work-group ever depends on another one being there.
  return hipLaunchKernel(kernel, dim3(static_cast<unsigned int>(a.B) * a.G),
                         dim3(resident ? kSamplingThreads : kStreamingThreads), params, 0, stream);
}

// Work-groups per request at launch: what the workspace was laid out for, fewer on a GPU with fewer compute units.
static int launch_groups(int G, int KB) {
  if (static_cast<long>(KB) * G > compute_units()) {
    G = compute_units() / KB;
    if (G < 1) G = 1;
  }
  return G;
}

// Zeroes words (the exchange words of the sampling walk, request status words) where no row reduction
// runs in front of the walk to do it.
__global__ __launch_bounds__(256) void clear_words_kernel(unsigned long long* words, long nwords, int32_t* status,
                                                          int nstatus) {
  const long i = static_cast<long>(blockIdx.x) * 256 + threadIdx.x;
  if (i < nwords) words[i] = 0ull;
  if (status && i < nstatus) status[i] = 0;
}

static bool lm_sizes_ok(int B, int N, int V, int H, int K) {
  return sizes_ok(B, N, V, K) && H >= kLmBK * kLmDepth && H % (kLmBK * kLmDepth) == 0 && static_cast<long>(B) * N <= (1L << 22);
}

}  // namespace mars

extern "C" {

int mars_version(void) { return 200; }  // 0.2.0: mars_lmhead_verify

const char* mars_status_string(int status) {
  switch (status) {
    case MARS_OK: return "ok";
    case MARS_ERR_ARG: return "invalid argument";
    case MARS_ERR_DTYPE: return "unknown element type";
    case MARS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MARS_ERR_HIP: return "HIP call failed";
    case MARS_ERR_SCRATCH: return "sizes need more scratch memory than mars_verify_static holds";
    default: return "unknown status";
  }
}

size_t mars_workspace_bytes(int B, int N, int V) {
  if (!mars::sizes_ok(B, N, V)) return 0;
  return mars::layout(B, N, V).total;
}

int mars_row_reduce(const void* logits, int logits_dtype, float temperature, int B, int N, int V, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  using namespace mars;
  if (!logits) return MARS_ERR_ARG;
  if (!sizes_ok(B, N, V)) return MARS_ERR_ARG;
  if (!(temperature >= 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  if (logits_dtype != MARS_F32 && logits_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const Layout L = layout(B, N, V);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  Partial* partials = reinterpret_cast<Partial*>(static_cast<char*>(workspace) + L.partials_off);
  const hipError_t e = launch_row_reduce(logits, logits_dtype, static_cast<long>(B) * N, V, L.splits,
                                         temperature > 0.0f, log2e_over_t(temperature), partials,
                                         clear_args(static_cast<char*>(workspace), L, B, N, 1),
                                         static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

int mars_row_stats(const void* logits, int logits_dtype, const float* theta, float temperature, int B, int N, int V,
                   mars_row_stat* stats, void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace mars;
  if (!logits || !theta || !stats) return MARS_ERR_ARG;
  if (!sizes_ok(B, N, V)) return MARS_ERR_ARG;
  if (!(temperature >= 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  if (logits_dtype != MARS_F32 && logits_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const Layout L = layout(B, N, V);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const long rows = static_cast<long>(B) * N;
  Partial* partials = reinterpret_cast<Partial*>(static_cast<char*>(workspace) + L.partials_off);
  const float c = log2e_over_t(temperature);
  if (launch_row_reduce(logits, logits_dtype, rows, V, L.splits, temperature > 0.0f, c, partials,
                        clear_args(static_cast<char*>(workspace), L, B, N, 1), stream) != hipSuccess)
    return MARS_ERR_HIP;
  const int threads = 256, rows_per_group = 16;
  const Indicator ind = {MARS_IND_LOGIT_RATIO, indicator_scale(temperature)};
  hipLaunchKernelGGL(merge_stats_kernel, dim3(static_cast<unsigned int>((rows + rows_per_group - 1) / rows_per_group)),
                     dim3(threads), 0, stream, partials, static_cast<int>(rows), N, L.splits * kPartsPerItem, theta, c,
                     ind, stats);
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

size_t mars_workspace_bytes_ex(int B, int N, int V, int n_theta) {
  if (!mars::sizes_ok(B, N, V, n_theta)) return 0;
  return mars::layout(B, N, V, n_theta).total;
}

int mars_verify(const void* logits, int logits_dtype, const int32_t* draft_tokens, const int32_t* tree_parent,
                const void* draft_probs, int draft_dtype, const float* theta, float temperature,
                const float* uniforms, int B, int N, int V, uint8_t* accept_mask, int32_t* accept_len,
                int32_t* path_idx, int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                mars_row_stat* stats, mars_req_diag* diag, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  return mars_verify_ex(logits, logits_dtype, draft_tokens, tree_parent, draft_probs, draft_dtype, theta, temperature,
                        uniforms, B, N, V, accept_mask, accept_len, path_idx, bonus_token, decision, request_status,
                        stats, diag, workspace, workspace_bytes, hip_stream, nullptr);
}

int mars_verify_ex(const void* logits, int logits_dtype, const int32_t* draft_tokens, const int32_t* tree_parent,
                   const void* draft_probs, int draft_dtype, const float* theta, float temperature,
                   const float* uniforms, int B, int N, int V, uint8_t* accept_mask, int32_t* accept_len,
                   int32_t* path_idx, int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                   mars_row_stat* stats, mars_req_diag* diag, void* workspace, size_t workspace_bytes,
                   void* hip_stream, const mars_verify_options* options) {
  using namespace mars;
  if (!logits || !draft_tokens || !tree_parent || !theta || !accept_mask || !accept_len || !path_idx || !bonus_token)
    return MARS_ERR_ARG;
  int K = 1, indicator = MARS_IND_LOGIT_RATIO, spin_limit = 0, stages = MARS_STAGE_ROWS | MARS_STAGE_REQUESTS;
  int32_t *out_tokens = nullptr, *out_len = nullptr, *keep_rows = nullptr, *keep_offsets = nullptr;
  if (options) {
    K = options->n_theta == 0 ? 1 : options->n_theta;
    indicator = options->indicator;
    spin_limit = options->spin_limit;
    if (spin_limit < 0 || options->stages < 0 || options->stages > 3) return MARS_ERR_ARG;
    if (options->stages != 0) stages = options->stages;
    out_tokens = options->out_tokens; out_len = options->out_len;
    keep_rows = options->keep_rows; keep_offsets = options->keep_offsets;
  }
  if (indicator != MARS_IND_LOGIT_RATIO && indicator != MARS_IND_PROB_RATIO && indicator != MARS_IND_LOGIT_GAP)
    return MARS_ERR_ARG;
  const int given = (out_tokens != nullptr) + (out_len != nullptr) + (keep_rows != nullptr) + (keep_offsets != nullptr);
  if (given != 0 && given != 4) return MARS_ERR_ARG;
  if (!sizes_ok(B, N, V, K)) return MARS_ERR_ARG;
  if (!(temperature >= 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  const bool sampling = temperature > 0.0f;
  if (sampling && !uniforms) return MARS_ERR_ARG;
  if (logits_dtype != MARS_F32 && logits_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const bool dense = sampling && draft_probs != nullptr;
  if (dense && draft_dtype != MARS_F32 && draft_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const Layout L = layout(B, N, V, K);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const long rows = static_cast<long>(B) * N;
  char* ws = static_cast<char*>(workspace);
  Partial* partials = reinterpret_cast<Partial*>(ws + L.partials_off);
  const float c = log2e_over_t(temperature);

  ClearArgs clr = clear_args(ws, L, B, N, K);
  if (sampling) {  // the sampling walk starts from what the row reduction gathers for it
    clr.par = tree_parent; clr.tok = draft_tokens;
    clr.q = dense ? draft_probs : nullptr;
    clr.q_bf16 = draft_dtype == MARS_BF16 ? 1 : 0;
    clr.gathered = reinterpret_cast<float2*>(ws + L.gathered_off);
  }
  if (sampling && request_status) {  // the sampling tail only raises a request's status
    clr.counters = reinterpret_cast<unsigned int*>(request_status);
    clr.ncounters = static_cast<long>(K) * B;
  }
  if ((stages & MARS_STAGE_ROWS) &&
      launch_row_reduce(logits, logits_dtype, rows, V, L.splits, sampling, c, partials, clr, stream) != hipSuccess)
    return MARS_ERR_HIP;
  if (!(stages & MARS_STAGE_REQUESTS)) return MARS_OK;

  TailArgs a;
  a.logits = logits; a.tok = draft_tokens; a.par = tree_parent;
  a.dprobs = dense ? draft_probs : nullptr;
  a.theta = theta; a.u = uniforms; a.partials = partials;
  a.stats = stats;
  a.stats_ws = reinterpret_cast<mars_row_stat*>(ws + L.stats_off);
  a.gathered = reinterpret_cast<const float2*>(ws + L.gathered_off);
  a.G = sampling ? launch_groups(L.G, K * B) : 1;
  // polls (about a microsecond each) a work-group gives a partner before it works out the partner's sum itself
  a.spin_limit = spin_limit > 0 ? spin_limit : kDefaultSpinLimit;
  a.xslots = clr.xslots;
  a.mask = accept_mask; a.len = accept_len; a.path = path_idx; a.bonus = bonus_token;
  a.dec = decision; a.status = request_status; a.diag = diag;
  a.B = K * B; a.Bd = B; a.N = N; a.V = V; a.splits = L.splits * kPartsPerItem; a.c = c;
  a.ind.kind = indicator; a.ind.cind = indicator_scale(temperature);
  a.out_tok = out_tokens; a.out_len = out_len;

  // The cache rows that stay: a small kernel behind the walk (one work-group per threshold).
  auto finish = [&]() -> int {
    if (hipGetLastError() != hipSuccess) return MARS_ERR_HIP;
    if (!keep_rows) return MARS_OK;
    hipLaunchKernelGGL(compact_keep_kernel, dim3(static_cast<unsigned int>(K)), dim3(kKeepThreads), 0, stream,
                       out_len, path_idx, B, N, keep_rows, keep_offsets);
    return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
  };

  if (!sampling) {
    hipLaunchKernelGGL(tail_greedy_kernel, dim3(static_cast<unsigned int>(K * B)), dim3(kGreedyThreads), 0, stream, a);
    return finish();
  }
  if (launch_sampling_tail(a, logits_dtype, dense ? draft_dtype : -1, stream) != hipSuccess) return MARS_ERR_HIP;
  return finish();
}

int mars_verify_static(const void* logits, int logits_dtype, const int32_t* draft_tokens, const int32_t* tree_parent,
                       const void* draft_probs, int draft_dtype, const float* theta, float temperature,
                       const float* uniforms, int B, int N, int V, uint8_t* accept_mask, int32_t* accept_len,
                       int32_t* path_idx, int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                       mars_row_stat* stats, mars_req_diag* diag, void* hip_stream,
                       const mars_verify_options* options) {
  using namespace mars;
  const int K = options && options->n_theta != 0 ? options->n_theta : 1;
  if (!sizes_ok(B, N, V, K)) return MARS_ERR_ARG;
  if (layout(B, N, V, K).total > static_cast<size_t>(MARS_STATIC_SCRATCH_BYTES)) return MARS_ERR_SCRATCH;
  void* ws = static_scratch();
  if (!ws) return MARS_ERR_HIP;
  return mars_verify_ex(logits, logits_dtype, draft_tokens, tree_parent, draft_probs, draft_dtype, theta, temperature,
                        uniforms, B, N, V, accept_mask, accept_len, path_idx, bonus_token, decision, request_status,
                        stats, diag, ws, MARS_STATIC_SCRATCH_BYTES, hip_stream, options);
}

int mars_margin_stats(const void* logits, int logits_dtype, const float* theta, float temperature, int B, int N, int V,
                      const float* range, const int32_t* bins, mars_margin_row* rows_out, uint32_t* counts,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace mars;
  if (!logits || !theta || !range || !bins || !counts) return MARS_ERR_ARG;
  if (!sizes_ok(B, N, V)) return MARS_ERR_ARG;
  if (!(temperature >= 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  if (logits_dtype != MARS_F32 && logits_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  HistSpec hs;
  long ncounters = 4;
  for (int h = 0; h < 3; ++h) {
    const float lo = range[2 * h], hi = range[2 * h + 1];
    if (!(lo < hi) || std::isinf(lo) || std::isinf(hi) || bins[h] < 1 || bins[h] > (1 << 20)) return MARS_ERR_ARG;
    hs.lo[h] = lo; hs.hi[h] = hi; hs.bins[h] = bins[h];
    hs.w[h] = static_cast<float>(static_cast<double>(bins[h]) / (static_cast<double>(hi) - static_cast<double>(lo)));
    ncounters += bins[h] + 2;
  }
  if (ncounters > (1 << 20)) return MARS_ERR_ARG;
  const Layout L = layout(B, N, V);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const long rows = static_cast<long>(B) * N;
  char* ws = static_cast<char*>(workspace);
  Partial* partials = reinterpret_cast<Partial*>(ws + L.partials_off);
  // The top-2 alone: the greedy form of the row reduction (no sum-exp); it also clears the counters.
  ClearArgs clr = clear_args(ws, L, B, N, 1);
  clr.counters = counts; clr.ncounters = ncounters;
  if (launch_row_reduce(logits, logits_dtype, rows, V, L.splits, false, 0.0f, partials, clr, stream) != hipSuccess)
    return MARS_ERR_HIP;
  hipLaunchKernelGGL(margin_stats_kernel, dim3(static_cast<unsigned int>((rows + 15) / 16)), dim3(256), 0, stream,
                     partials, static_cast<int>(rows), N, L.splits * kPartsPerItem, theta, indicator_scale(temperature),
                     hs, rows_out, counts);
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

size_t mars_lmhead_workspace_bytes(int B, int N, int V, int H, int n_theta) {
  const int K = n_theta == 0 ? 1 : n_theta;
  if (!mars::lm_sizes_ok(B, N, V, H, K)) return 0;
  return mars::lm_layout(B, N, V, K).total;
}

int mars_lmhead_verify(const void* hidden, const void* weight, int H, const int32_t* draft_tokens,
                       const int32_t* tree_parent, const float* theta, int B, int N, int V, uint8_t* accept_mask,
                       int32_t* accept_len, int32_t* path_idx, int32_t* bonus_token, uint8_t* decision,
                       int32_t* request_status, mars_row_stat* stats, void* workspace, size_t workspace_bytes,
                       void* hip_stream, const mars_verify_options* options) {
  using namespace mars;
  if (!hidden || !weight || !draft_tokens || !tree_parent || !theta || !accept_mask || !accept_len || !path_idx ||
      !bonus_token)
    return MARS_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(hidden) % 16 != 0 || reinterpret_cast<uintptr_t>(weight) % 16 != 0)
    return MARS_ERR_ARG;
  int K = 1, indicator = MARS_IND_LOGIT_RATIO, lm_stages = MARS_STAGE_ROWS | MARS_STAGE_REQUESTS;
  int32_t *out_tokens = nullptr, *out_len = nullptr, *keep_rows = nullptr, *keep_offsets = nullptr;
  if (options) {
    K = options->n_theta == 0 ? 1 : options->n_theta;
    indicator = options->indicator;
    if (options->spin_limit < 0 || options->stages < 0 || options->stages > 3) return MARS_ERR_ARG;
    if (options->stages != 0) lm_stages = options->stages;
    out_tokens = options->out_tokens; out_len = options->out_len;
    keep_rows = options->keep_rows; keep_offsets = options->keep_offsets;
  }
  if (indicator != MARS_IND_LOGIT_RATIO && indicator != MARS_IND_PROB_RATIO && indicator != MARS_IND_LOGIT_GAP)
    return MARS_ERR_ARG;
  const int given = (out_tokens != nullptr) + (out_len != nullptr) + (keep_rows != nullptr) + (keep_offsets != nullptr);
  if (given != 0 && given != 4) return MARS_ERR_ARG;
  if (!lm_sizes_ok(B, N, V, H, K)) return MARS_ERR_ARG;
  const LmLayout L = lm_layout(B, N, V, K);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int rows = B * N;
  char* ws = static_cast<char*>(workspace);
  Partial* partials = reinterpret_cast<Partial*>(ws + L.partials_off);
  const LmPlan& p = L.plan;

  const int pairs = p.runs * p.slabs, per_die = (pairs + kDies - 1) / kDies;
  const dim3 grid(static_cast<unsigned int>(kDies * per_die)), block(kLmThreads);
  const bf16_t* hp = static_cast<const bf16_t*>(hidden);
  const bf16_t* wp = static_cast<const bf16_t*>(weight);
#define MARS_LM_LAUNCH(BM)                                                                                      \
  hipLaunchKernelGGL((lmhead_reduce_kernel<BM, false>), grid, block, 0, stream, hp, wp, rows, V, H, p.slabs, p.tiles_n, \
                     p.tiles_per_run, p.runs, partials, static_cast<bf16_t*>(nullptr), 0.0f)
  if (lm_stages & MARS_STAGE_ROWS) {
    switch (p.bm) {
      case 64: MARS_LM_LAUNCH(64); break;
      case 128: MARS_LM_LAUNCH(128); break;
      default: MARS_LM_LAUNCH(192); break;
    }
    if (hipGetLastError() != hipSuccess) return MARS_ERR_HIP;
  }
#undef MARS_LM_LAUNCH
  if (!(lm_stages & MARS_STAGE_REQUESTS)) return MARS_OK;

  TailArgs a;
  a.logits = nullptr; a.tok = draft_tokens; a.par = tree_parent; a.dprobs = nullptr;
  a.theta = theta; a.u = nullptr; a.partials = partials;
  a.stats = stats;
  a.stats_ws = reinterpret_cast<mars_row_stat*>(ws + L.stats_off);
  a.G = 1; a.spin_limit = 0; a.xslots = nullptr; a.gathered = nullptr;
  a.mask = accept_mask; a.len = accept_len; a.path = path_idx; a.bonus = bonus_token;
  a.dec = decision; a.status = request_status; a.diag = nullptr;
  a.B = K * B; a.Bd = B; a.N = N; a.V = V; a.splits = p.parts; a.c = 0.0f;
  a.ind.kind = indicator; a.ind.cind = indicator_scale(0.0f);
  a.out_tok = out_tokens; a.out_len = out_len;
  hipLaunchKernelGGL(tail_greedy_kernel, dim3(static_cast<unsigned int>(K * B)), dim3(kGreedyThreads), 0, stream, a);
  if (hipGetLastError() != hipSuccess) return MARS_ERR_HIP;
  if (!keep_rows) return MARS_OK;
  hipLaunchKernelGGL(compact_keep_kernel, dim3(static_cast<unsigned int>(K)), dim3(kKeepThreads), 0, stream, out_len,
                     path_idx, B, N, keep_rows, keep_offsets);
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

int mars_lmhead_verify_sampling(const void* hidden, const void* weight, int H, const int32_t* draft_tokens,
                                const int32_t* tree_parent, const void* draft_probs, int draft_dtype,
                                const float* theta, float temperature, const float* uniforms, int B, int N, int V,
                                void* logits_out, uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                                int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                                mars_row_stat* stats, mars_req_diag* diag, void* workspace, size_t workspace_bytes,
                                void* hip_stream, const mars_verify_options* options) {
  using namespace mars;
  if (!hidden || !weight || !draft_tokens || !tree_parent || !theta || !uniforms || !logits_out || !accept_mask ||
      !accept_len || !path_idx || !bonus_token)
    return MARS_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(hidden) % 16 != 0 || reinterpret_cast<uintptr_t>(weight) % 16 != 0 ||
      reinterpret_cast<uintptr_t>(logits_out) % 16 != 0 || V % 8 != 0)
    return MARS_ERR_ARG;
  if (!(temperature > 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  const bool dense = draft_probs != nullptr;
  if (dense && draft_dtype != MARS_F32 && draft_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  int K = 1, indicator = MARS_IND_LOGIT_RATIO, spin_limit = 0, lm_stages = MARS_STAGE_ROWS | MARS_STAGE_REQUESTS;
  int32_t *out_tokens = nullptr, *out_len = nullptr, *keep_rows = nullptr, *keep_offsets = nullptr;
  if (options) {
    K = options->n_theta == 0 ? 1 : options->n_theta;
    indicator = options->indicator;
    spin_limit = options->spin_limit;
    if (spin_limit < 0 || options->stages < 0 || options->stages > 3) return MARS_ERR_ARG;
    if (options->stages != 0) lm_stages = options->stages;
    out_tokens = options->out_tokens; out_len = options->out_len;
    keep_rows = options->keep_rows; keep_offsets = options->keep_offsets;
  }
  if (indicator != MARS_IND_LOGIT_RATIO && indicator != MARS_IND_PROB_RATIO && indicator != MARS_IND_LOGIT_GAP)
    return MARS_ERR_ARG;
  const int given = (out_tokens != nullptr) + (out_len != nullptr) + (keep_rows != nullptr) + (keep_offsets != nullptr);
  if (given != 0 && given != 4) return MARS_ERR_ARG;
  if (!lm_sizes_ok(B, N, V, H, K)) return MARS_ERR_ARG;
  const LmLayout L = lm_layout(B, N, V, K);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const int rows = B * N;
  char* ws = static_cast<char*>(workspace);
  Partial* partials = reinterpret_cast<Partial*>(ws + L.partials_off);
  unsigned long long* xslots = reinterpret_cast<unsigned long long*>(ws + L.xslots_off);
  const LmPlan& p = L.plan;
  const float c = log2e_over_t(temperature);

  if (lm_stages & MARS_STAGE_ROWS) {
    // What the streaming row reduction clears for the walk behind it, the fused kernel does not.
    const long nwords = static_cast<long>(K) * B * (N + 2) * 2 * L.G;
    const long nclear = nwords > static_cast<long>(K) * B ? nwords : static_cast<long>(K) * B;
    hipLaunchKernelGGL(clear_words_kernel, dim3(static_cast<unsigned int>((nclear + 255) / 256)), dim3(256), 0, stream,
                       xslots, nwords, request_status, K * B);
    const int pairs = p.runs * p.slabs, per_die = (pairs + kDies - 1) / kDies;
    const dim3 grid(static_cast<unsigned int>(kDies * per_die)), block(kLmThreads);
    const bf16_t* hp = static_cast<const bf16_t*>(hidden);
    const bf16_t* wp = static_cast<const bf16_t*>(weight);
    bf16_t* lo = static_cast<bf16_t*>(logits_out);
#define MARS_LM_LAUNCH(BM)                                                                                            \
  hipLaunchKernelGGL((lmhead_reduce_kernel<BM, true>), grid, block, 0, stream, hp, wp, rows, V, H, p.slabs, p.tiles_n, \
                     p.tiles_per_run, p.runs, partials, lo, c)
    switch (p.bm) {
      case 64: MARS_LM_LAUNCH(64); break;
      case 128: MARS_LM_LAUNCH(128); break;
      default: MARS_LM_LAUNCH(192); break;
    }
#undef MARS_LM_LAUNCH
    if (hipGetLastError() != hipSuccess) return MARS_ERR_HIP;
  }
  if (!(lm_stages & MARS_STAGE_REQUESTS)) return MARS_OK;

  TailArgs a;
  a.logits = logits_out; a.tok = draft_tokens; a.par = tree_parent;
  a.dprobs = dense ? draft_probs : nullptr;
  a.theta = theta; a.u = uniforms; a.partials = partials;
  a.gathered = nullptr;  // the walk gathers for itself: no streaming row reduction has run
  a.stats = stats;
  a.stats_ws = reinterpret_cast<mars_row_stat*>(ws + L.stats_off);
  a.G = launch_groups(L.G, K * B);
  a.spin_limit = spin_limit > 0 ? spin_limit : kDefaultSpinLimit;
  a.xslots = xslots;
  a.mask = accept_mask; a.len = accept_len; a.path = path_idx; a.bonus = bonus_token;
  a.dec = decision; a.status = request_status; a.diag = diag;
  a.B = K * B; a.Bd = B; a.N = N; a.V = V; a.splits = p.parts; a.c = c;
  a.ind.kind = indicator; a.ind.cind = indicator_scale(temperature);
  a.out_tok = out_tokens; a.out_len = out_len;
  if (launch_sampling_tail(a, MARS_BF16, dense ? draft_dtype : -1, stream) != hipSuccess) return MARS_ERR_HIP;
  if (hipGetLastError() != hipSuccess) return MARS_ERR_HIP;
  if (!keep_rows) return MARS_OK;
  hipLaunchKernelGGL(compact_keep_kernel, dim3(static_cast<unsigned int>(K)), dim3(kKeepThreads), 0, stream, out_len,
                     path_idx, B, N, keep_rows, keep_offsets);
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

}  // extern "C"
