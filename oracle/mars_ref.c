/*
 * mars_ref.c -- CPU oracle for the MARS verification pass.
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, fp64 implementation written
 * straight from the paper; it shares no code, header, table or helper with the
 * HIP library and the product path never calls it.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may load it.
 *
 * What it follows, in the paper's notation:
 *   - top-2 identification v(1), v(2), z(1) >= z(2)            (Sec. 3.3; Alg. 1 "Identify top-2")
 *   - logit ratio r = z(2)/z(1)                                  (Eq. 4 "ratio_def"; Alg. 1 "Compute ratio")
 *   - exact match / adaptive relaxation (r > theta) / rejection  (Sec. 3.4 bullets; Alg. 1 if-chain)
 *   - softmax P(v) = exp(z_v) / sum_u exp(z_u)                   (Eq. 3), on z/T
 *   - rejection-sampling acceptance min(1, P_t / P_s)            (Eq. 1 "rejection_sampling")
 *   - residual distribution after a rejection                    (Sec. 2.3: norm(max(0, P_t - P_s)),
 *                                                                 the form of the cited speculative-sampling rule)
 *   - token trees verified in one pass                           (Sec. 2.3, tree paragraph)
 *   - bonus token when every draft is accepted, tau <= K+1       (Table 1 caption)
 *   - the committed sequence V_out: accepted drafts, then the    (Alg. 1, V_out; Sec. 3.4 "standard rollback")
 *     correction / bonus token; the nodes whose cache rows stay
 *   - other indicators of a low margin on the same two logits:   (Sec. 3.3: probability ratio P(v2)/P(v1),
 *     probability ratio, fixed logit margin                       logit margin Delta = z(1) - z(2), Eq. 5-6)
 *   - distributions of z(1), z(2)/z(1), p2/p1 over rows          (Appendix "Additional Analysis", histogram figure;
 *                                                                 Sec. 3.3 scatter figure)
 *
 * Readings where the paper is silent (kept identical on purpose in the
 * library's header so both sides state them):
 *   - node 0 is the root; row i is the target's distribution after node i;
 *     node i >= 1 is tested against row parent(i);
 *   - ties: (value descending, index ascending);
 *   - no relaxation unless z(1) > 0 (positive-domain assumption, Sec. 3.3);
 *   - the decision r > theta is taken in fp32 (one correctly rounded division
 *     of the two fp32-exact logits), the precision the GPU path computes in;
 *     the fp64 ratio is reported beside it so tests can check that both agree
 *     outside the guard band;
 *   - sampling mode: the runner-up relaxation is a deterministic accept, every
 *     other token (the top-1 included) goes through Eq. 1 unchanged; siblings
 *     are tried in node order, multi-round, with the residual renormalised
 *     after each rejection;
 *   - draft_probs == NULL: q is one-hot at the child's token;
 *   - greedy tree: the deepest fully accepted node wins, ties to the lowest
 *     node index; the emitted token is v(1) of that node's row;
 *   - indicators other than the logit ratio reuse theta[b] as their threshold:
 *     probability ratio exp(-(z1 - z2)/T') > theta with T' = T, or 1 in greedy
 *     mode (softmax of the raw logits); fixed margin z1 - z2 < theta.  Neither
 *     needs the positive-domain condition.  The margin is one rounded fp32
 *     subtraction on both sides; the probability ratio is evaluated in fp32
 *     here and the fp64 decision reported beside it (inputs keep a guard band);
 *   - the cache rows that stay are the root's and the accepted nodes', listed
 *     request by request in path order as flat row numbers b*N + node.
 *
 * Parity pins: every exported function is pinned by tests/test_oracle_*.py
 * (hand-worked examples, the paper's Fig. 2 ratios, theta > 1 invariants
 * against independent numpy routines, brute force on tiny vocabularies, a
 * chi-square test of the strict sampling path).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_F32 = 0, REF_BF16 = 1 };

typedef struct mars_ref_row {
  double  z1, z2;     /* top-2 logit values, widened exactly */
  double  ratio;      /* z2 / z1 in fp64 (NaN if z1 == 0) */
  double  sum_exp;    /* S = sum_v exp((z_v - z1)/T); 0 when T == 0 */
  double  prob_ratio; /* P(v2)/P(v1) = exp(-(z1 - z2)/T'), T' = T or 1 when T == 0 */
  double  gap;        /* Delta = z1 - z2 */
  int32_t id1, id2;
  int32_t relax_ok;   /* the low-margin test of the chosen indicator, decided in fp32 */
  int32_t relax_ok64; /* same test decided in fp64 against (double)theta */
} mars_ref_row;

enum { IND_LOGIT_RATIO = 0, IND_PROB_RATIO = 1, IND_LOGIT_GAP = 2 };

typedef struct mars_ref_diag {
  double  bonus_prob;         /* f(bonus) / sum f for the final distribution */
  double  last_residual_norm; /* Z of the last rejection, 0 if none */
  double  min_accept_margin;  /* min |u - f(x)/q(x)| over the Eq. 1 tests taken (inf if none) */
  double  min_cdf_margin;     /* distance of u*sum(f) to the nearest CDF step of the draw, / sum(f) */
  double  min_norm;           /* smallest residual normaliser Z met (inf if none) */
  int32_t residual_passes;
  int32_t last_node;
  int32_t small_norm_plen;    /* drafts accepted so far when the first normaliser below the floor (see
                                 mars_ref_set_norm_floor) was met, -1 if none: what the walk decided up to
                                 there does not depend on that normaliser */
  int32_t small_norm_node;    /* the node whose children were being tried then, -1 if none */
} mars_ref_diag;

static int g_threads = 1;
/* A residual normaliser below this is reported in small_norm_plen / small_norm_node.  It changes no
   result: it only tells a test from where on an fp32 implementation may legitimately differ (Z is a
   difference of probability masses of order 1, so its relative error grows like 1/Z). */
static double g_norm_floor = 2e-2;

void mars_ref_set_norm_floor(double z) { g_norm_floor = z; }

double mars_ref_get_norm_floor(void) { return g_norm_floor; }

void mars_ref_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int mars_ref_get_threads(void) { return g_threads; }

int mars_ref_has_openmp(void) {
#ifdef _OPENMP
  return 1;
#else
  return 0;
#endif
}

static double load_elem(const void* base, int dtype, size_t idx) {
  if (dtype == REF_F32) return (double)((const float*)base)[idx];
  uint16_t h = ((const uint16_t*)base)[idx];
  uint32_t w = (uint32_t)h << 16; /* bf16 is the upper half of an fp32 */
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

/* Sec. 3.3 / Eq. 4 / Eq. 3 for one row. */
static void row_stats(const void* logits, int dtype, size_t base, int V, float T32,
                      float theta, int indicator, mars_ref_row* st) {
  const double T = (double)T32;
  int id1 = 0;
  double z1 = load_elem(logits, dtype, base);
  for (int v = 1; v < V; ++v) {
    double z = load_elem(logits, dtype, base + (size_t)v);
    if (z > z1) { z1 = z; id1 = v; }
  }
  int id2 = -1;
  double z2 = 0.0;
  for (int v = 0; v < V; ++v) {
    if (v == id1) continue;
    double z = load_elem(logits, dtype, base + (size_t)v);
    if (id2 < 0 || z > z2) { z2 = z; id2 = v; }
  }
  st->z1 = z1; st->id1 = id1; st->z2 = z2; st->id2 = id2;
  st->ratio = z2 / z1;
  const double Tind = T > 0.0 ? T : 1.0;
  st->gap = z1 - z2;
  st->prob_ratio = exp(-(z1 - z2) / Tind);
  const float z1f = (float)z1, z2f = (float)z2; /* exact: the logits are fp32 or bf16 */
  if (indicator == IND_LOGIT_RATIO) {        /* Eq. 4 */
    float r32 = z2f / z1f;
    st->relax_ok = (z1 > 0.0 && r32 > theta) ? 1 : 0;
    st->relax_ok64 = (z1 > 0.0 && st->ratio > (double)theta) ? 1 : 0;
  } else if (indicator == IND_PROB_RATIO) {  /* Sec. 3.3: ratio of the two softmax probabilities */
    volatile float d32 = z1f - z2f;
    volatile float x32 = d32 / (T32 > 0.0f ? T32 : 1.0f);
    float p32 = expf(-x32);
    st->relax_ok = p32 > theta ? 1 : 0;
    st->relax_ok64 = st->prob_ratio > (double)theta ? 1 : 0;
  } else {                                   /* fixed margin on Delta of Eq. 5 */
    volatile float d32 = z1f - z2f;
    st->relax_ok = d32 < theta ? 1 : 0;
    st->relax_ok64 = st->gap < (double)theta ? 1 : 0;
  }
  double S = 0.0;
  if (T > 0.0) {
    for (int v = 0; v < V; ++v)
      S += exp((load_elem(logits, dtype, base + (size_t)v) - z1) / T);
  }
  st->sum_exp = S;
}

int mars_ref_row_stats_ex(const void* logits, int logits_dtype, const float* theta,
                          float temperature, int indicator, int B, int N, int V,
                          mars_ref_row* out) {
  if (!logits || !theta || !out || B < 1 || N < 1 || V < 2) return -1;
  if (logits_dtype != REF_F32 && logits_dtype != REF_BF16) return -2;
  if (!(temperature >= 0.0f)) return -1;
  if (indicator < IND_LOGIT_RATIO || indicator > IND_LOGIT_GAP) return -1;
  long rows = (long)B * N;
#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
  for (long r = 0; r < rows; ++r)
    row_stats(logits, logits_dtype, (size_t)r * (size_t)V, V, temperature,
              theta[r / N], indicator, &out[r]);
  return 0;
}

int mars_ref_row_stats(const void* logits, int logits_dtype, const float* theta,
                       float temperature, int B, int N, int V, mars_ref_row* out) {
  return mars_ref_row_stats_ex(logits, logits_dtype, theta, temperature, IND_LOGIT_RATIO, B, N, V, out);
}

/* Tree / token validation shared by both modes. */
static int request_status(const int32_t* tok, const int32_t* par, int N, int V) {
  if (par[0] != -1) return 1;
  for (int i = 1; i < N; ++i)
    if (par[i] < 0 || par[i] >= i) return 1;
  for (int i = 1; i < N; ++i)
    if (tok[i] < 0 || tok[i] >= V) return 2;
  return 0;
}

/* Alg. 1 on a tree: local codes, reachability, deepest reachable node. */
static void verify_greedy(const mars_ref_row* st, const int32_t* tok, const int32_t* par, int N,
                          uint8_t* mask, int32_t* len, int32_t* path, int32_t* bonus,
                          uint8_t* decision, mars_ref_diag* dg) {
  uint8_t* code = (uint8_t*)calloc((size_t)N, 1);
  uint8_t* reach = (uint8_t*)calloc((size_t)N, 1);
  int32_t* depth = (int32_t*)calloc((size_t)N, sizeof(int32_t));
  reach[0] = 1;
  int best = 0;
  for (int i = 1; i < N; ++i) {
    int p = par[i];
    depth[i] = depth[p] + 1;
    if (tok[i] == st[p].id1) code[i] = 1;                         /* exact match */
    else if (tok[i] == st[p].id2 && st[p].relax_ok) code[i] = 2;  /* adaptive relaxation */
    else code[i] = 0;                                             /* rejection */
    reach[i] = (uint8_t)(code[i] != 0 && reach[p]);
    if (reach[i] && depth[i] > depth[best]) best = i; /* strict: ties keep the lower index */
  }
  *len = depth[best];
  for (int i = 0; i < N; ++i) { mask[i] = 0; path[i] = -1; if (decision) decision[i] = 0; }
  mask[0] = 1;
  for (int n = best; n != 0; n = par[n]) {
    mask[n] = 1;
    path[depth[n] - 1] = n;
    if (decision) decision[n] = code[n];
  }
  *bonus = st[best].id1; /* correction after a rejection, bonus after a leaf */
  if (dg) dg->last_node = best;
  free(code); free(reach); free(depth);
}

/* Multi-round rejection sampling down the tree with the MARS relaxation. */
static void verify_sampling(const void* logits, int ldt, size_t req_base, int V, double T,
                            const void* dprobs, int ddt, const mars_ref_row* st,
                            const int32_t* tok, const int32_t* par, const float* u, int N,
                            uint8_t* mask, int32_t* len, int32_t* path, int32_t* bonus,
                            uint8_t* decision, mars_ref_diag* dg) {
  double* f = (double*)malloc((size_t)V * sizeof(double));
  for (int i = 0; i < N; ++i) { mask[i] = 0; path[i] = -1; if (decision) decision[i] = 0; }
  mask[0] = 1;
  int c = 0, plen = 0;
  double min_acc = INFINITY, min_norm = INFINITY, lastZ = 0.0;
  int passes = 0, small_plen = -1, small_node = -1;
  for (;;) {
    /* f = softmax(z_c / T), Eq. 3 */
    size_t rb = req_base + (size_t)c * (size_t)V;
    for (int v = 0; v < V; ++v)
      f[v] = exp((load_elem(logits, ldt, rb + (size_t)v) - st[c].z1) / T) / st[c].sum_exp;
    int next = -1;
    for (int k = c + 1; k < N; ++k) {
      if (par[k] != c) continue;
      int x = tok[k];
      int code = 0;
      if (x == st[c].id2 && st[c].relax_ok) {
        code = 2; /* adaptive relaxation: deterministic accept */
      } else {
        double qx = dprobs ? load_elem(dprobs, ddt, rb + (size_t)x) : 1.0;
        double fx = f[x];
        double a, rho;
        if (fx == 0.0) { a = 0.0; rho = 0.0; }
        else if (qx <= 0.0) { a = 1.0; rho = INFINITY; }
        else { rho = fx / qx; a = rho < 1.0 ? rho : 1.0; }   /* Eq. 1 */
        double m = fabs((double)u[k] - rho);
        if (m < min_acc) min_acc = m;
        if ((double)u[k] < a) code = 3;
      }
      if (code) {
        next = k;
        mask[k] = 1; path[plen++] = k;
        if (decision) decision[k] = (uint8_t)code;
        break;
      }
      /* rejected: f <- norm(max(0, f - q_k)) */
      double Z = 0.0;
      for (int v = 0; v < V; ++v) {
        double q = dprobs ? load_elem(dprobs, ddt, rb + (size_t)v) : (v == x ? 1.0 : 0.0);
        double g = f[v] - q;
        Z += g > 0.0 ? g : 0.0;
      }
      ++passes; lastZ = Z;
      if (Z < min_norm) min_norm = Z;
      if (Z < g_norm_floor && small_plen < 0) { small_plen = plen; small_node = c; }
      /* Z == 0 cannot follow a rejection in exact arithmetic (it needs f <= q everywhere,
         hence f == q and acceptance probability 1); f is left as it is then. */
      if (Z > 0.0)
        for (int v = 0; v < V; ++v) {
          double q = dprobs ? load_elem(dprobs, ddt, rb + (size_t)v) : (v == x ? 1.0 : 0.0);
          double g = f[v] - q;
          f[v] = (g > 0.0 ? g : 0.0) / Z;
        }
    }
    if (next < 0) break;
    c = next;
  }
  /* inverse CDF in index order with u[N] */
  double total = 0.0;
  for (int v = 0; v < V; ++v) total += f[v];
  double target = (double)u[N] * total, cum = 0.0;
  int pick = -1;
  double cdf_margin = INFINITY;
  for (int v = 0; v < V; ++v) {
    double prev = cum;
    cum += f[v];
    if (cum > target) {
      pick = v;
      double lo = (target - prev) / total, hi = (cum - target) / total;
      cdf_margin = lo < hi ? lo : hi;
      break;
    }
  }
  if (pick < 0) { /* rounding left no step above the target: last token with mass */
    for (int v = V - 1; v >= 0; --v) if (f[v] > 0.0) { pick = v; break; }
    if (pick < 0) pick = st[c].id1; /* all-zero f: degenerate input */
    cdf_margin = 0.0;
  }
  *bonus = pick; *len = plen;
  if (dg) {
    dg->bonus_prob = total > 0.0 ? f[pick] / total : 0.0;
    dg->last_residual_norm = lastZ;
    dg->min_accept_margin = min_acc;
    dg->min_cdf_margin = cdf_margin;
    dg->min_norm = min_norm;
    dg->residual_passes = passes;
    dg->last_node = c;
    dg->small_norm_plen = small_plen;
    dg->small_norm_node = small_node;
  }
  free(f);
}

int mars_ref_verify_ex(const void* logits, int logits_dtype,
                       const int32_t* draft_tokens, const int32_t* tree_parent,
                       const void* draft_probs, int draft_dtype,
                       const float* theta, float temperature, const float* uniforms,
                       int B, int N, int V, int indicator,
                       uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                       int32_t* bonus_token, uint8_t* decision, int32_t* req_status,
                       mars_ref_row* stats, mars_ref_diag* diag) {
  if (!logits || !draft_tokens || !tree_parent || !theta || !accept_mask || !accept_len ||
      !path_idx || !bonus_token)
    return -1;
  if (B < 1 || N < 1 || V < 2) return -1;
  if (!(temperature >= 0.0f)) return -1;
  if (temperature > 0.0f && !uniforms) return -1;
  if (logits_dtype != REF_F32 && logits_dtype != REF_BF16) return -2;
  if (draft_probs && draft_dtype != REF_F32 && draft_dtype != REF_BF16) return -2;

  mars_ref_row* st_all = stats;
  if (!st_all) st_all = (mars_ref_row*)malloc((size_t)B * N * sizeof(mars_ref_row));
  int rc = mars_ref_row_stats_ex(logits, logits_dtype, theta, temperature, indicator, B, N, V, st_all);
  if (rc) { if (!stats) free(st_all); return rc; }

#pragma omp parallel for schedule(dynamic, 1) num_threads(g_threads)
  for (int b = 0; b < B; ++b) {
    const mars_ref_row* st = st_all + (size_t)b * N;
    const int32_t* tok = draft_tokens + (size_t)b * N;
    const int32_t* par = tree_parent + (size_t)b * N;
    uint8_t* mask = accept_mask + (size_t)b * N;
    int32_t* path = path_idx + (size_t)b * N;
    uint8_t* dec = decision ? decision + (size_t)b * N : NULL;
    mars_ref_diag* dg = diag ? diag + b : NULL;
    if (dg) {
      memset(dg, 0, sizeof *dg);
      dg->min_accept_margin = INFINITY; dg->min_cdf_margin = INFINITY; dg->min_norm = INFINITY;
      dg->small_norm_plen = -1; dg->small_norm_node = -1;
    }
    int s = request_status(tok, par, N, V);
    if (req_status) req_status[b] = s;
    if (s) {
      for (int i = 0; i < N; ++i) { mask[i] = 0; path[i] = -1; if (dec) dec[i] = 0; }
      mask[0] = 1; accept_len[b] = 0; bonus_token[b] = st[0].id1;
      continue;
    }
    if (temperature == 0.0f)
      verify_greedy(st, tok, par, N, mask, &accept_len[b], path, &bonus_token[b], dec, dg);
    else
      verify_sampling(logits, logits_dtype, (size_t)b * N * (size_t)V, V, (double)temperature,
                      draft_probs, draft_dtype, st, tok, par, uniforms + (size_t)b * (N + 1), N,
                      mask, &accept_len[b], path, &bonus_token[b], dec, dg);
  }
  if (!stats) free(st_all);
  return 0;
}

int mars_ref_verify(const void* logits, int logits_dtype,
                    const int32_t* draft_tokens, const int32_t* tree_parent,
                    const void* draft_probs, int draft_dtype,
                    const float* theta, float temperature, const float* uniforms,
                    int B, int N, int V,
                    uint8_t* accept_mask, int32_t* accept_len, int32_t* path_idx,
                    int32_t* bonus_token, uint8_t* decision, int32_t* req_status,
                    mars_ref_row* stats, mars_ref_diag* diag) {
  return mars_ref_verify_ex(logits, logits_dtype, draft_tokens, tree_parent, draft_probs, draft_dtype,
                            theta, temperature, uniforms, B, N, V, IND_LOGIT_RATIO, accept_mask,
                            accept_len, path_idx, bonus_token, decision, req_status, stats, diag);
}

/* Alg. 1's V_out and the cache rows that survive (Sec. 3.4, "standard rollback"): per request the
 * tokens of the accepted nodes in path order followed by the correction / bonus token, and, over
 * the whole batch, the flat row numbers b*N + node of the root and the accepted nodes. */
int mars_ref_commit(const int32_t* draft_tokens, const int32_t* accept_len, const int32_t* path_idx,
                    const int32_t* bonus_token, int B, int N,
                    int32_t* out_tokens, int32_t* out_len, int32_t* keep_rows, int32_t* keep_offsets) {
  if (!draft_tokens || !accept_len || !path_idx || !bonus_token || !out_tokens || !out_len ||
      !keep_rows || !keep_offsets || B < 1 || N < 1)
    return -1;
  int total = 0;
  for (int b = 0; b < B; ++b) {
    const int32_t* tok = draft_tokens + (size_t)b * N;
    const int32_t* path = path_idx + (size_t)b * N;
    int32_t* out = out_tokens + (size_t)b * N;
    int L = accept_len[b];
    if (L < 0 || L > N - 1) return -1;
    keep_offsets[b] = total;
    keep_rows[total++] = b * N; /* the root's row */
    for (int j = 0; j < L; ++j) {
      out[j] = tok[path[j]];
      keep_rows[total++] = b * N + path[j];
    }
    out[L] = bonus_token[b];
    for (int j = L + 1; j < N; ++j) out[j] = -1;
    out_len[b] = L + 1;
  }
  keep_offsets[B] = total;
  for (int j = total; j < B * N; ++j) keep_rows[j] = -1;
  return 0;
}

/* Distributions of the top-2 statistics over rows (appendix histogram figure: top-1 logit, logit
 * ratio z2/z1, probability ratio p2/p1; share of negative top-1 logits).
 *
 * A histogram over [lo, hi) with `bins` equal cells has bins + 2 counters: [0] counts x < lo,
 * [bins + 1] counts x >= hi, cell k (0-based) is counter k + 1.  The cell of x is decided in fp32:
 * trunc(fl(fl(x - lo) * w)), w = fl32(bins / (hi - lo)) from a double division, capped at bins - 1;
 * x itself is the fp32 value: z1 exactly, fl32(z2 / z1), and the fp32 rounding of the fp64 p2/p1.
 * Rows with z1 <= 0 have no ratio (Sec. 3.3) and are left out of the ratio histogram.
 * edge_dist[r] (optional) is the distance, in cells, of row r's p2/p1 from the nearest cell
 * boundary: p2/p1 goes through an exponential, so a caller comparing against another
 * implementation can set aside the rows that sit on a boundary. */
typedef struct mars_ref_margin_row { double z1, z2, ratio, prob_ratio; } mars_ref_margin_row;

static int hist_cell(float x, float lo, float hi, int bins) {
  if (x < lo) return 0;
  if (!(x < hi)) return bins + 1;
  float w = (float)((double)bins / ((double)hi - (double)lo));
  volatile float d = x - lo;
  volatile float t = d * w;
  int k = (int)t;
  if (k > bins - 1) k = bins - 1;
  return k + 1;
}

int mars_ref_margin_stats(const void* logits, int logits_dtype, const float* theta, float temperature,
                          int B, int N, int V,
                          const float* range /* 6: lo,hi of z1, ratio, p2/p1 */, const int32_t* bins /* 3 */,
                          mars_ref_margin_row* rows_out, uint32_t* hist_z1, uint32_t* hist_ratio,
                          uint32_t* hist_prob, uint32_t* summary /* 4 */, double* edge_dist) {
  if (!logits || !theta || !range || !bins || !hist_z1 || !hist_ratio || !hist_prob || !summary) return -1;
  if (B < 1 || N < 1 || V < 2 || !(temperature >= 0.0f)) return -1;
  for (int h = 0; h < 3; ++h)
    if (bins[h] < 1 || !(range[2 * h] < range[2 * h + 1])) return -1;
  long rows = (long)B * N;
  mars_ref_row* st = (mars_ref_row*)malloc((size_t)rows * sizeof(mars_ref_row));
  int rc = mars_ref_row_stats(logits, logits_dtype, theta, temperature, B, N, V, st);
  if (rc) { free(st); return rc; }
  memset(hist_z1, 0, (size_t)(bins[0] + 2) * sizeof(uint32_t));
  memset(hist_ratio, 0, (size_t)(bins[1] + 2) * sizeof(uint32_t));
  memset(hist_prob, 0, (size_t)(bins[2] + 2) * sizeof(uint32_t));
  uint32_t negative = 0, nonpositive = 0, low_margin = 0;
  for (long r = 0; r < rows; ++r) {
    if (rows_out) {
      rows_out[r].z1 = st[r].z1; rows_out[r].z2 = st[r].z2;
      rows_out[r].ratio = st[r].ratio; rows_out[r].prob_ratio = st[r].prob_ratio;
    }
    float z1f = (float)st[r].z1, z2f = (float)st[r].z2;
    ++hist_z1[hist_cell(z1f, range[0], range[1], bins[0])];
    if (st[r].z1 < 0.0) ++negative;
    if (st[r].z1 <= 0.0) ++nonpositive;
    else ++hist_ratio[hist_cell(z2f / z1f, range[2], range[3], bins[1])];
    float pf = (float)st[r].prob_ratio;
    ++hist_prob[hist_cell(pf, range[4], range[5], bins[2])];
    if (st[r].relax_ok) ++low_margin;
    if (edge_dist) {
      double t = (st[r].prob_ratio - (double)range[4]) * (double)bins[2] / ((double)range[5] - (double)range[4]);
      edge_dist[r] = fabs(t - nearbyint(t));
    }
  }
  summary[0] = (uint32_t)rows; summary[1] = negative; summary[2] = nonpositive; summary[3] = low_margin;
  free(st);
  return 0;
}

/* Struct sizes, so the Python wrapper can check its mirror of the layouts. */
int mars_ref_sizeof_row(void) { return (int)sizeof(mars_ref_row); }
int mars_ref_sizeof_diag(void) { return (int)sizeof(mars_ref_diag); }
