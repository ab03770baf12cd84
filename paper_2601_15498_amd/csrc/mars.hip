// C ABI of the MARS verification pass (see include/mars.h): argument checks,
// workspace carving and kernel launches.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "../../include/mars.h"
#include "common.h"
#include "row_reduce.h"
#include "tail.h"

namespace mars {

constexpr int kTargetItems = 1024;      // aim for at least this many work-groups in the row reduction
constexpr int kMinSplitElems = 8192;    // but keep every split at least this long
constexpr size_t kAlign = 256;

static size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Splits per row: a function of (rows, V) only, so that the workspace size does not depend on
// the element type.
static int choose_splits(long rows, int V) {
  long want = (kTargetItems + rows - 1) / rows;
  long cap = V / kMinSplitElems;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  return static_cast<int>(want);
}

struct Layout {
  int splits;
  size_t partials_off, stats_off, total;
};

static Layout layout(int B, int N, int V) {
  Layout L;
  const long rows = static_cast<long>(B) * N;
  L.splits = choose_splits(rows, V);
  L.partials_off = 0;
  L.stats_off = align_up(static_cast<size_t>(rows) * L.splits * sizeof(Partial));
  L.total = L.stats_off + align_up(static_cast<size_t>(rows) * sizeof(mars_row_stat));
  return L;
}

static bool sizes_ok(int B, int N, int V) {
  if (B < 1 || N < 1 || N > MARS_MAX_NODES || V < MARS_MIN_VOCAB) return false;
  const long rows = static_cast<long>(B) * N;
  return rows <= 0x7FFFFFFFL / 64;  // rows * splits must fit the grid and int arithmetic
}

template <typename T, int EPV>
static hipError_t launch_row_reduce_t(const void* logits, long rows, int V, int splits, bool sampling, float c,
                                      Partial* partials, hipStream_t stream) {
  const int nvec = V / EPV;
  const int vps = (nvec + splits - 1) / splits;
  const dim3 grid(static_cast<unsigned int>(rows * splits)), block(kRowThreads);
  if (sampling)
    hipLaunchKernelGGL((row_reduce_kernel<T, EPV, true>), grid, block, 0, stream, static_cast<const T*>(logits), V,
                       splits, vps, c, partials);
  else
    hipLaunchKernelGGL((row_reduce_kernel<T, EPV, false>), grid, block, 0, stream, static_cast<const T*>(logits), V,
                       splits, vps, c, partials);
  return hipGetLastError();
}

// 16-byte loads need every row to start on a 16-byte boundary; otherwise the same kernel runs
// with one element per load.
static hipError_t launch_row_reduce(const void* logits, int dtype, long rows, int V, int splits, bool sampling,
                                    float c, Partial* partials, hipStream_t stream) {
  const size_t elt = dtype == MARS_BF16 ? 2 : 4;
  const bool wide = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((static_cast<size_t>(V) * elt) % 16 == 0);
  if (dtype == MARS_BF16)
    return wide ? launch_row_reduce_t<bf16_t, 8>(logits, rows, V, splits, sampling, c, partials, stream)
                : launch_row_reduce_t<bf16_t, 1>(logits, rows, V, splits, sampling, c, partials, stream);
  return wide ? launch_row_reduce_t<float, 4>(logits, rows, V, splits, sampling, c, partials, stream)
              : launch_row_reduce_t<float, 1>(logits, rows, V, splits, sampling, c, partials, stream);
}

static float log2e_over_t(float temperature) {
  return temperature > 0.0f ? static_cast<float>(1.4426950408889634 / static_cast<double>(temperature)) : 0.0f;
}

}  // namespace mars

extern "C" {

int mars_version(void) { return 100; }

const char* mars_status_string(int status) {
  switch (status) {
    case MARS_OK: return "ok";
    case MARS_ERR_ARG: return "invalid argument";
    case MARS_ERR_DTYPE: return "unknown element type";
    case MARS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MARS_ERR_HIP: return "HIP call failed";
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
  if (launch_row_reduce(logits, logits_dtype, rows, V, L.splits, temperature > 0.0f, c, partials, stream) !=
      hipSuccess)
    return MARS_ERR_HIP;
  const int threads = 256;
  hipLaunchKernelGGL(merge_stats_kernel, dim3(static_cast<unsigned int>((rows + threads - 1) / threads)),
                     dim3(threads), 0, stream, partials, static_cast<int>(rows), N, L.splits, theta, c, stats);
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

int mars_verify(const void* logits, int logits_dtype, const int32_t* draft_tokens, const int32_t* tree_parent,
                const void* draft_probs, int draft_dtype, const float* theta, float temperature,
                const float* uniforms, int B, int N, int V, uint8_t* accept_mask, int32_t* accept_len,
                int32_t* path_idx, int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                mars_row_stat* stats, mars_req_diag* diag, void* workspace, size_t workspace_bytes,
                void* hip_stream) {
  using namespace mars;
  if (!logits || !draft_tokens || !tree_parent || !theta || !accept_mask || !accept_len || !path_idx || !bonus_token)
    return MARS_ERR_ARG;
  if (!sizes_ok(B, N, V)) return MARS_ERR_ARG;
  if (!(temperature >= 0.0f) || std::isinf(temperature)) return MARS_ERR_ARG;
  const bool sampling = temperature > 0.0f;
  if (sampling && !uniforms) return MARS_ERR_ARG;
  if (logits_dtype != MARS_F32 && logits_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const bool dense = sampling && draft_probs != nullptr;
  if (dense && draft_dtype != MARS_F32 && draft_dtype != MARS_BF16) return MARS_ERR_DTYPE;
  const Layout L = layout(B, N, V);
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 || workspace_bytes < L.total)
    return MARS_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const long rows = static_cast<long>(B) * N;
  char* ws = static_cast<char*>(workspace);
  Partial* partials = reinterpret_cast<Partial*>(ws + L.partials_off);
  const float c = log2e_over_t(temperature);

  if (launch_row_reduce(logits, logits_dtype, rows, V, L.splits, sampling, c, partials, stream) != hipSuccess)
    return MARS_ERR_HIP;

  TailArgs a;
  a.logits = logits; a.tok = draft_tokens; a.par = tree_parent;
  a.dprobs = dense ? draft_probs : nullptr;
  a.theta = theta; a.u = uniforms; a.partials = partials;
  a.stats = stats ? stats : reinterpret_cast<mars_row_stat*>(ws + L.stats_off);
  a.mask = accept_mask; a.len = accept_len; a.path = path_idx; a.bonus = bonus_token;
  a.dec = decision; a.status = request_status; a.diag = diag;
  a.B = B; a.N = N; a.V = V; a.splits = L.splits; a.c = c;

  const dim3 grid(static_cast<unsigned int>(B));
  if (!sampling) {
    hipLaunchKernelGGL(tail_greedy_kernel, grid, dim3(kGreedyThreads), 0, stream, a);
  } else if (logits_dtype == MARS_BF16) {
    if (dense && draft_dtype == MARS_BF16)
      hipLaunchKernelGGL((tail_sampling_kernel<bf16_t, bf16_t>), grid, dim3(kSamplingThreads), 0, stream, a);
    else
      hipLaunchKernelGGL((tail_sampling_kernel<bf16_t, float>), grid, dim3(kSamplingThreads), 0, stream, a);
  } else {
    if (dense && draft_dtype == MARS_BF16)
      hipLaunchKernelGGL((tail_sampling_kernel<float, bf16_t>), grid, dim3(kSamplingThreads), 0, stream, a);
    else
      hipLaunchKernelGGL((tail_sampling_kernel<float, float>), grid, dim3(kSamplingThreads), 0, stream, a);
  }
  return hipGetLastError() == hipSuccess ? MARS_OK : MARS_ERR_HIP;
}

}  // extern "C"
