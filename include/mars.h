/*
 * mars.h -- C ABI of the MARS verification pass for AMD MI355X (gfx950).
 *
 * MARS (margin-aware speculative verification) changes only the accept/reject
 * rule of speculative decoding (paper Sec. 2.3 last paragraph, Sec. 3.4,
 * Algorithm 1).  This library is the verification pass over the target model's
 * logits for every node of a drafted chain or token tree:
 *
 *   - per-row top-1 / top-2 over the vocabulary (Sec. 3.3: v(1), v(2),
 *     z(1) >= z(2)) and, when sampling, max / sum-exp of the softmax (Eq. 3);
 *   - the logit ratio r = z(2)/z(1) (Eq. 4, "ratio_def") and the margin test
 *     r > theta (Sec. 3.4 "Adaptive Relaxation");
 *   - per-node acceptance: exact match / relaxed runner-up / reject (Alg. 1)
 *     in greedy mode, the rejection-sampling test min(1, P_t/P_s) (Eq. 1)
 *     plus the relaxed runner-up in sampling mode;
 *   - residual-distribution resampling after a rejection (Sec. 2.3);
 *   - longest accepted path over the chain or tree (Sec. 2.3 tree paragraph)
 *     and the correction / bonus token (Alg. 1 "Correction"; Table 1 caption:
 *     tau <= K+1).
 *
 * Conventions
 *   B requests, N nodes per request INCLUDING the root (node 0 = the last
 *   committed token), V vocabulary entries.  logits[b,i,:] is the target's
 *   next-token row after node i; node i >= 1 is verified against the row of
 *   parent(i); the correction / bonus token comes from the row of the last
 *   accepted node.  A chain of K drafts is N = K+1 with parent(i) = i-1.
 *
 *   Ties are ordered (value descending, index ascending): id1 is the lowest
 *   index holding the maximum, id2 the lowest index, other than id1, holding
 *   the maximum of the rest.
 *
 *   Relaxation needs z(1) > 0 (the paper's positive-domain assumption,
 *   Sec. 3.3) and the strict inequality fl32(z(2)/z(1)) > theta[b], evaluated
 *   with one correctly rounded fp32 division.
 *
 * All pointers are DEVICE pointers unless stated.  The library never frees or
 * keeps caller memory.  Calls only enqueue work on the given HIP stream;
 * outputs are valid once that stream has been synchronised.  No exceptions
 * and no C++ types cross this boundary.
 */
#ifndef MARS_H_
#define MARS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of logits / draft_probs. */
enum { MARS_F32 = 0, MARS_BF16 = 1 };

/* Return codes (argument, type and workspace errors are detected on the host and enqueue nothing). */
enum {
  MARS_OK            = 0,
  MARS_ERR_ARG       = -1, /* null required pointer, B/N/V out of range, T < 0 or NaN */
  MARS_ERR_DTYPE     = -2, /* unknown element type */
  MARS_ERR_WORKSPACE = -3, /* workspace missing, misaligned or too small */
  MARS_ERR_HIP       = -4, /* a kernel launch failed; kernels of the same call launched before it stay enqueued */
  MARS_ERR_SCRATCH   = -5  /* mars_verify_static: these sizes need more than MARS_STATIC_SCRATCH_BYTES */
};

/* Per-request status written by the device (data-dependent problems). */
enum {
  MARS_REQ_OK        = 0,
  MARS_REQ_BAD_TREE  = 1, /* parent[0] != -1, or parent[i] not in [0, i) for i >= 1 */
  MARS_REQ_BAD_TOKEN = 2, /* draft token of a node i >= 1 outside [0, V) */
  MARS_REQ_TIMEOUT   = 3  /* not produced any more (a work-group no longer gives up on its partners: it works
                             out their share itself); the value is kept so that old callers still compile */
};

/* decision[b,i] codes (Sec. 3.4 bullets; code 3 is Eq. 1's stochastic accept). */
enum {
  MARS_DEC_NONE    = 0, /* not on the selected path */
  MARS_DEC_EXACT   = 1, /* draft token == v(1) (greedy mode) */
  MARS_DEC_RELAXED = 2, /* draft token == v(2) and r > theta */
  MARS_DEC_SAMPLED = 3  /* accepted by u < min(1, f(x)/q(x)) (sampling mode) */
};

/* Largest N (nodes per request, root included) and smallest V accepted. */
#define MARS_MAX_NODES 1024
#define MARS_MIN_VOCAB 2

/* Which quantity of the two largest logits decides that a row has a low margin (Sec. 3.3).
 * All three compare against theta[b], strictly:
 *   MARS_IND_LOGIT_RATIO  z1 > 0 and fl32(z2/z1) > theta           (Eq. 4; the paper's choice)
 *   MARS_IND_PROB_RATIO   P(v2)/P(v1) = exp(-(z1 - z2)/T') > theta  with T' = temperature, or 1 in greedy
 *                         mode (softmax of the raw logits); evaluated in fp32 (about 1 ulp)
 *   MARS_IND_LOGIT_GAP    fl32(z1 - z2) < theta                     (a fixed margin on Delta of Eq. 5)
 * Only the logit ratio needs the positive-domain condition. */
enum { MARS_IND_LOGIT_RATIO = 0, MARS_IND_PROB_RATIO = 1, MARS_IND_LOGIT_GAP = 2 };

/* Parts of the pass (mars_verify_options.stages). */
enum { MARS_STAGE_ROWS = 1, MARS_STAGE_REQUESTS = 2 };

/* Most thresholds per request one call of mars_verify_ex sweeps. */
#define MARS_MAX_THETAS 64

/* Per-row statistics table, one entry per (b, i) row, 24 bytes.
 * z1/z2 are the logit values widened exactly to fp32.  sum_exp is
 * S = sum_v exp((z_v - z1)/T) (Eq. 3 with the max subtracted); 0 in greedy mode. */
typedef struct mars_row_stat {
  float   z1;
  int32_t id1;
  float   z2;
  int32_t id2;
  float   sum_exp;
  int32_t relax_ok; /* 1 iff the low-margin test holds: z1 > 0 and fl32(z2/z1) > theta[b] (Eq. 4), or the
                       test of the indicator chosen in mars_verify_ex */
} mars_row_stat;

/* Optional per-request diagnostics of the sampling-mode walk (floats the
 * parity tests compare against the oracle). */
typedef struct mars_req_diag {
  float   bonus_prob;      /* f(bonus_token) / sum_v f(v) for the final distribution f the token is drawn from */
  float   last_residual_norm; /* Z = sum_v max(0, f - q) of the last rejection (0 if none) */
  int32_t residual_passes; /* number of rejections, i.e. residual renormalisations performed */
  int32_t last_node;       /* node whose row produced the bonus token */
} mars_req_diag;

/* Library version: major*10000 + minor*100 + patch. */
int mars_version(void);

/* Static string for a return code (host memory, never freed). */
const char* mars_status_string(int status);

/*
 * Bytes of device workspace mars_verify / mars_row_stats need for these sizes
 * (0 if an argument is out of range).  The workspace must be 256-byte aligned.
 * Its contents are scratch: undefined before and after a call.
 */
size_t mars_workspace_bytes(int B, int N, int V);

/*
 * First stage only: the streaming row reduction (Sec. 3.3 top-2 identification, Eq. 3
 * max / sum-exp) into per-(row, split) partial results inside the workspace.  This is the
 * HBM-bound kernel of the pass; the entry point exists so that it can be timed by itself.
 * Arguments as for mars_row_stats.  Returns MARS_OK or a negative code.
 */
int mars_row_reduce(const void* logits, int logits_dtype, float temperature, int B, int N, int V,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Row reduction and merge (Sec. 3.3 top-2, Eq. 3 sum-exp, Eq. 4 ratio test):
 * fills stats[B*N].  temperature == 0 skips the sum-exp (sum_exp = 0).
 *
 *   logits       device, [B,N,V] row-major, element type logits_dtype, rows contiguous
 *                (row stride V elements).  No NaN / +inf; -inf = masked token.
 *   theta        device, [B] fp32 per-request threshold.
 *   stats        device out, [B*N].
 *   workspace    device, >= mars_workspace_bytes(B,N,V), 256-byte aligned.
 *   hip_stream   hipStream_t (NULL = default stream).
 * Returns MARS_OK or a negative code; on error nothing is enqueued.
 */
int mars_row_stats(const void* logits, int logits_dtype, const float* theta,
                   float temperature, int B, int N, int V, mars_row_stat* stats,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The whole verification pass.
 *
 *   logits        device, [B,N,V] as above.
 *   draft_tokens  device, [B,N] int32; [b,0] is the root token (never read).
 *   tree_parent   device, [B,N] int32; [b,0] = -1; 0 <= parent[b,i] < i for i >= 1.
 *   draft_probs   device, [B,N,V] (element type draft_dtype): the draft model's
 *                 distribution AFTER node i, i.e. the one the children of i were
 *                 drawn from (Eq. 1's P_Ms).  Non-negative; used as given.
 *                 NULL = deterministic draft: q is one-hot at each child's token.
 *                 Ignored in greedy mode.
 *   theta         device, [B] fp32 thresholds (Sec. 3.4; the paper uses 0.9).
 *   temperature   host scalar.  0 selects greedy verification (Alg. 1 on a tree,
 *                 correction = v(1)).  > 0 selects sampling verification with
 *                 p = softmax(z / T): relaxed runner-up accept, else Eq. 1,
 *                 residual resampling on rejection.
 *   uniforms      device, [B,N+1] fp32 in [0,1): [b,i] tests node i (i >= 1),
 *                 [b,N] draws the correction / bonus token.  May be NULL when
 *                 temperature == 0.
 *   accept_mask   device out, [B,N] uint8: 1 iff node on the selected path (root always 1).
 *   accept_len    device out, [B] int32: accepted draft tokens (root and bonus
 *                 excluded); tau = accept_len + 1.
 *   path_idx      device out, [B,N] int32: node at depth 1..accept_len, then -1.
 *   bonus_token   device out, [B] int32.
 *   decision      device out, optional (NULL ok), [B,N] uint8 MARS_DEC_* codes.
 *   request_status device out, optional (NULL ok), [B] int32 MARS_REQ_* codes.  A
 *                 request with a non-zero status (malformed tree, token out of range) gets
 *                 accept_len = 0, an empty path and bonus_token = v(1) of its root row.
 *   stats         device out, optional (NULL ok), [B*N] row statistics.
 *   diag          device out, optional (NULL ok), [B]; in greedy mode only last_node is set.
 *   workspace     device, >= mars_workspace_bytes(B,N,V), 256-byte aligned.
 *   hip_stream    hipStream_t (NULL = default stream).
 *
 * Sampling-mode walk: starting at the root, the children of the current node
 * are tried in increasing node index against the current distribution f
 * (initially the node's softmax); the first accepted child becomes the current
 * node with a fresh f; every rejected child replaces f by norm(max(0, f - q)).
 * When no child is accepted the token is drawn from f by inverse CDF in index
 * order with uniforms[b,N].
 *
 * Returns MARS_OK or a negative code; on error nothing is enqueued.
 * Calls that share a workspace must not overlap.  Calls with workspaces (and outputs) of their
 * own may run side by side on any number of streams: the library keeps no state, the
 * latency-bound per-request kernel of one call then runs beside the bandwidth-bound row
 * reduction of another, and no work-group of a call waits for another one to be resident.
 */
int mars_verify(const void* logits, int logits_dtype,
                const int32_t* draft_tokens, const int32_t* tree_parent,
                const void* draft_probs, int draft_dtype,
                const float* theta, float temperature, const float* uniforms,
                int B, int N, int V,
                uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                mars_row_stat* stats, mars_req_diag* diag,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Options of mars_verify_ex (a HOST struct; the pointers in it are device pointers).
 *
 *   indicator     MARS_IND_*: the low-margin test used for the relaxation (Sec. 3.3 discusses the
 *                 three; theta[b] is the threshold of whichever is chosen).
 *   n_theta       K >= 1 (0 is read as 1): thresholds per request.  With K > 1 the call is the
 *                 threshold ablation of Sec. 4 in one pass over the logits: theta is [K,B], the row
 *                 reduction runs once, and the per-request part runs for every (k, b) on the same
 *                 inputs; EVERY output of mars_verify gains a leading axis of length K
 *                 (accept_mask [K,B,N], accept_len [K,B], ..., stats [K,B*N], diag [K,B]).
 *   spin_limit    sampling mode: the work-groups that share a request exchange partial sums.  This is
 *                 the number of polls (about a microsecond each) a work-group gives a partner before it
 *                 stops waiting and works out the partner's sum itself -- same bits, so the outputs
 *                 do not depend on it; no work-group ever depends on another one being resident.
 *                 0 = the default (256).  Only of interest to callers that share the GPU with other
 *                 work, and to tests of that path (1 = never wait).
 *   stages        which part of the pass the call enqueues: 0 or MARS_STAGE_ROWS | MARS_STAGE_REQUESTS = all of
 *                 it; MARS_STAGE_ROWS = the row reduction only (it also clears what the second part
 *                 accumulates into and, in sampling mode, gathers the logit and draft probability of
 *                 every node's token for it); MARS_STAGE_REQUESTS = the per-request part only, on a
 *                 workspace that the first part of a mars_verify_ex call with the same arguments has
 *                 filled (mars_row_reduce does not: it knows no tree).  Splitting a pass lets a caller
 *                 that overlaps passes on several streams put its own events between the parts: the
 *                 per-request part of a sampling-mode pass holds up to one work-group per compute unit
 *                 and is quickest when all of them are resident together, so the per-request parts of
 *                 overlapping passes are best run one after the other while row reductions run beside
 *                 them freely.
 *   out_tokens    device out, optional, [K,B,N] int32: the committed sequence V_out of Alg. 1 -- the
 *                 tokens of the accepted nodes in path order, then the correction / bonus token,
 *                 then -1.
 *   out_len       device out, [K,B] int32: accept_len + 1.
 *   keep_rows     device out, [K,B*N] int32: the cache rows that stay after rollback (Sec. 3.4) -- the
 *                 row b*N + node of the root and of every accepted node, request by request in path
 *                 order, compacted; then -1.
 *   keep_offsets  device out, [K,B+1] int32: request b's rows are keep_rows[offsets[b] .. offsets[b+1]).
 *                 The four are given together or not at all.
 */
typedef struct mars_verify_options {
  int32_t  indicator;
  int32_t  n_theta;
  int32_t  spin_limit;
  int32_t  stages;
  int32_t* out_tokens;
  int32_t* out_len;
  int32_t* keep_rows;
  int32_t* keep_offsets;
} mars_verify_options;

/* Workspace of mars_verify_ex for a sweep over n_theta thresholds (n_theta = 1: same as
 * mars_workspace_bytes).  0 if an argument is out of range. */
size_t mars_workspace_bytes_ex(int B, int N, int V, int n_theta);

/*
 * mars_verify with options: another low-margin indicator (Sec. 3.3), several thresholds per
 * request from one read of the logits (the ablation over theta of Sec. 4), and the committed
 * sequence with the cache rows to keep (Alg. 1, V_out).  Arguments as for mars_verify, with the
 * shapes stated above when n_theta > 1 and workspace >= mars_workspace_bytes_ex(B,N,V,n_theta);
 * options == NULL is mars_verify.  n_theta * B requests are verified side by side, which in
 * sampling mode leaves fewer work-groups per request.  Errors as for mars_verify, plus
 * MARS_ERR_ARG for an unknown indicator, n_theta outside [0, MARS_MAX_THETAS], a negative
 * spin_limit, stages outside [0, 3], or some but not all of the four commit outputs.
 */
int mars_verify_ex(const void* logits, int logits_dtype,
                   const int32_t* draft_tokens, const int32_t* tree_parent,
                   const void* draft_probs, int draft_dtype,
                   const float* theta, float temperature, const float* uniforms,
                   int B, int N, int V,
                   uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                   int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                   mars_row_stat* stats, mars_req_diag* diag,
                   void* workspace, size_t workspace_bytes, void* hip_stream,
                   const mars_verify_options* options);

/*
 * mars_verify_ex for callers that cannot allocate or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The partial results of the row
 * reduction, the merged statistics and the exchange words of the sampling-mode walk live in a
 * device array of MARS_STATIC_SCRATCH_BYTES that is part of the library's code object: every GPU the
 * library runs on holds its own copy from load until the process ends.  The call allocates
 * nothing, frees nothing and calls no routine that does; on its first use on a GPU it looks up the
 * array's device address (once per GPU, with that GPU current) and keeps it.
 *
 * Arguments, outputs and errors as for mars_verify_ex (options may be NULL), without workspace and
 * workspace_bytes.  Sizes whose mars_workspace_bytes_ex(B,N,V,n_theta) exceeds
 * MARS_STATIC_SCRATCH_BYTES are rejected with MARS_ERR_SCRATCH and nothing is enqueued (the
 * headline shape, 16 requests of 60 nodes over 151 936 entries, needs 0.7 MB; 256 requests of 26
 * nodes 1.4 MB).  The kernels are launched on hip_stream, which must belong to the current GPU.
 * All calls on one GPU share that GPU's array: it keeps the previous call's contents (whatever has
 * to start at zero is cleared by the call's own first kernel), and calls that overlap on one GPU --
 * on different streams, or a graph replay beside an eager call -- race on it and give undefined
 * results.  Calls on one stream, one after the other, are safe.
 */
#define MARS_STATIC_SCRATCH_BYTES (8u << 20)
int mars_verify_static(const void* logits, int logits_dtype,
                       const int32_t* draft_tokens, const int32_t* tree_parent,
                       const void* draft_probs, int draft_dtype,
                       const float* theta, float temperature, const float* uniforms,
                       int B, int N, int V,
                       uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                       int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                       mars_row_stat* stats, mars_req_diag* diag,
                       void* hip_stream, const mars_verify_options* options);

/* One row of mars_margin_stats: the two largest logits, their ratio fl32(z2/z1) (IEEE result also
 * when z1 <= 0) and the probability ratio P(v2)/P(v1) = exp(-(z1 - z2)/T'), T' as above. */
typedef struct mars_margin_row {
  float z1;
  float z2;
  float ratio;
  float prob_ratio;
} mars_margin_row;

/*
 * Distributions of the top-2 statistics over all B*N rows, from one pass over the logits: what
 * the paper's appendix plots to justify theta and the positive-domain assumption (histograms of
 * the top-1 logit, of z2/z1 and of p2/p1, share of negative top-1 logits), and the share of rows
 * inside the relaxation zone (Sec. 3.3, scatter figure).
 *
 *   theta     device, [B]: threshold of the logit-ratio test counted in the summary.
 *   range     HOST, 6 floats: lo, hi of the histogram of z1, of z2/z1, of p2/p1 (lo < hi).
 *   bins      HOST, 3 ints >= 1: cells of each histogram.
 *   rows_out  device out, optional (NULL ok), [B*N].
 *   counts    device out, uint32, (bins[0]+2) + (bins[1]+2) + (bins[2]+2) + 4 entries: the three
 *             histograms one after the other, each as [x < lo | cell 0 .. cell bins-1 | x >= hi],
 *             then the summary: rows, rows with z1 < 0, rows with z1 <= 0, rows that pass the
 *             logit-ratio test at theta[b].  The cell of x is trunc(fl32(fl32(x - lo) * w)) with
 *             w = fl32(bins / (hi - lo)) (the quotient taken in double), capped at bins - 1; x is
 *             the fp32 value stored in rows_out.  Rows with z1 <= 0 have no ratio and are left out
 *             of the ratio histogram.
 *   workspace device, >= mars_workspace_bytes(B,N,V).
 * Returns MARS_OK or a negative code (MARS_ERR_ARG also for bins < 1, lo >= hi, or more than 2^20
 * counters); on error nothing is enqueued.
 */
int mars_margin_stats(const void* logits, int logits_dtype, const float* theta, float temperature,
                      int B, int N, int V, const float* range, const int32_t* bins,
                      mars_margin_row* rows_out, uint32_t* counts,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Greedy verification straight from the target model's last hidden states (Eq. 2: the logits of a
 * row are z = W h): the LM-head product and the top-2 identification of Sec. 3.3 run in one
 * kernel on the matrix cores, and the logits are never written to memory.  The logits are
 * defined as the fp32-accumulated products rounded once to bf16 (what a bf16 LM head hands to the
 * verifier); everything behind them -- low-margin test, Alg. 1 on a chain or tree, committed
 * sequence, sweep over thresholds -- is mars_verify_ex in greedy mode.
 * The order in which a row's products are added is the kernel's own and depends on the launch
 * plan (so on B*N and V): a logit whose exact value lies within the fp32 accumulation error of a
 * bf16 rounding boundary may come out one bf16 step apart between two batch shapes; for one shape
 * the result is reproducible bit for bit.
 *
 *   hidden   device, [B,N,H] bf16, 16-byte aligned: last hidden state of every node.
 *   weight   device, [V,H] bf16, 16-byte aligned: the LM head, one row per vocabulary entry.
 *   H        hidden size, a multiple of 128.
 *   theta, draft_tokens, tree_parent, outputs, options: as for mars_verify_ex with temperature 0
 *            (request_status, decision, stats optional; options may be NULL).
 *   workspace device, 256-byte aligned, >= mars_lmhead_workspace_bytes(B,N,V,H,n_theta).
 *            options->stages works as for mars_verify_ex: MARS_STAGE_ROWS is the fused LM-head kernel.
 * Returns MARS_OK or a negative code; MARS_ERR_ARG also for H not a multiple of 128 or misaligned
 * hidden / weight.  On MARS_ERR_HIP kernels launched before the failing one stay enqueued;
 * otherwise an error enqueues nothing.  Calls with workspaces of their own may overlap.
 */
size_t mars_lmhead_workspace_bytes(int B, int N, int V, int H, int n_theta);
int mars_lmhead_verify(const void* hidden, const void* weight, int H,
                       const int32_t* draft_tokens, const int32_t* tree_parent, const float* theta,
                       int B, int N, int V,
                       uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                       int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                       mars_row_stat* stats,
                       void* workspace, size_t workspace_bytes, void* hip_stream,
                       const mars_verify_options* options);

/*
 * Sampling-mode verification straight from the last hidden states: Eq. 2 followed by Eq. 3 in one kernel.
 * The LM-head product runs on the matrix cores as in mars_lmhead_verify; the logits (fp32-accumulated
 * products rounded once to bf16) are written to `logits_out` once, from the registers they are formed in
 * -- under sampling the residual passes of the walk read rows of them again (Sec. 2.3), so they have to
 * exist -- and each row's top-2 and sum of exponentials are taken on the way: the logits are not read
 * back for the statistics.  Everything behind that is the sampling walk of mars_verify_ex on `logits_out`.
 *
 *   hidden, weight, H   as for mars_lmhead_verify.
 *   draft_probs, draft_dtype, temperature (> 0), uniforms   as for mars_verify.
 *   V                   a multiple of 8.
 *   logits_out          device out, [B,N,V] bf16, 16-byte aligned, caller-owned.
 *   outputs, options    as for mars_verify_ex (request_status, decision, stats, diag optional).
 *   workspace           device, 256-byte aligned, >= mars_lmhead_workspace_bytes(B,N,V,H,n_theta).
 * Returns MARS_OK or a negative code (MARS_ERR_ARG also for temperature <= 0: use mars_lmhead_verify).
 * Error behaviour and overlap of calls as for mars_lmhead_verify.
 */
int mars_lmhead_verify_sampling(const void* hidden, const void* weight, int H,
                                const int32_t* draft_tokens, const int32_t* tree_parent,
                                const void* draft_probs, int draft_dtype,
                                const float* theta, float temperature, const float* uniforms,
                                int B, int N, int V, void* logits_out,
                                uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                                int32_t* bonus_token, uint8_t* decision, int32_t* request_status,
                                mars_row_stat* stats, mars_req_diag* diag,
                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                const mars_verify_options* options);

#ifdef __cplusplus
}
#endif
#endif /* MARS_H_ */
