/* Driver for the sanitizer build of the CPU oracle (tests/test_sanitizers.py compiles this file together
 * with oracle/mars_ref.c under -fsanitize=address,undefined and runs it): seeded inputs of several shapes
 * -- chains and trees, greedy and sampling, one-hot and dense draft distributions, bf16 and fp32, every
 * indicator, a malformed request -- through every exported function.  The sanitizers abort on the first
 * out-of-bounds access, use of uninitialised stack, signed overflow or misaligned access; the driver itself
 * only checks the structural bounds every output must meet.  Test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/mars_ref.c"

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* splitmix64 -> [0,1) */
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (double)(z >> 11) / 9007199254740992.0;
}
static double gauss(void) { return sqrt(-2.0 * log(rnd() + 1e-300)) * cos(6.283185307179586 * rnd()); }
static uint16_t to_bf16(float x) { uint32_t u; memcpy(&u, &x, 4); return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16); }

static int run_case(int B, int N, int V, int bf16, float T, int dense, int tree, int indicator, int break_one) {
  const size_t rows = (size_t)B * N;
  void* logits = malloc(rows * V * (bf16 ? 2 : 4));
  float* q = dense ? (float*)malloc(rows * V * sizeof(float)) : NULL;
  int32_t* tok = (int32_t*)malloc(rows * sizeof(int32_t));
  int32_t* par = (int32_t*)malloc(rows * sizeof(int32_t));
  float* theta = (float*)malloc(B * sizeof(float));
  float* u = (float*)malloc((size_t)B * (N + 1) * sizeof(float));
  for (size_t i = 0; i < rows * V; ++i) {
    const float z = (float)(3.0 * gauss());
    if (bf16) ((uint16_t*)logits)[i] = to_bf16(z); else ((float*)logits)[i] = z;
  }
  if (dense)
    for (size_t r = 0; r < rows; ++r) {
      double s = 0.0;
      for (int v = 0; v < V; ++v) { q[r * V + v] = (float)exp(gauss()); s += q[r * V + v]; }
      for (int v = 0; v < V; ++v) q[r * V + v] = (float)(q[r * V + v] / s);
    }
  for (int b = 0; b < B; ++b) {
    theta[b] = indicator == 2 ? 1.25f : (indicator == 1 ? 0.35f : 0.9f);
    for (int i = 0; i < N; ++i) {
      par[b * N + i] = i == 0 ? -1 : (tree ? (int32_t)(rnd() * i) : i - 1);
      tok[b * N + i] = (int32_t)(rnd() * V);
    }
    for (int i = 0; i <= N; ++i) u[b * (N + 1) + i] = (float)rnd();
  }
  if (break_one && N > 2) { par[2] = 5000; tok[N + 1 < (int)rows ? N + 1 : 1] = V + 3; }
  uint8_t* mask = (uint8_t*)malloc(rows);
  uint8_t* dec = (uint8_t*)malloc(rows);
  int32_t* alen = (int32_t*)malloc(B * sizeof(int32_t));
  int32_t* path = (int32_t*)malloc(rows * sizeof(int32_t));
  int32_t* bonus = (int32_t*)malloc(B * sizeof(int32_t));
  int32_t* status = (int32_t*)malloc(B * sizeof(int32_t));
  mars_ref_row* st = (mars_ref_row*)malloc(rows * sizeof(mars_ref_row));
  mars_ref_diag* dg = (mars_ref_diag*)malloc(B * sizeof(mars_ref_diag));
  int rc = mars_ref_verify_ex(logits, bf16, tok, par, q, 0, theta, T, u, B, N, V, indicator, mask, alen, path, bonus,
                              dec, status, st, dg);
  int bad = rc != 0;
  for (int b = 0; b < B && !bad; ++b) {
    if (alen[b] < 0 || alen[b] >= N || bonus[b] < 0 || bonus[b] >= V || mask[b * N] != 1) bad = 1;
    for (int d = 0; d < alen[b] && !bad; ++d)
      if (path[b * N + d] < 1 || path[b * N + d] >= N) bad = 1;
  }
  /* the committed sequence and the kept rows, the margin statistics */
  int32_t* out_tok = (int32_t*)malloc(rows * sizeof(int32_t));
  int32_t* out_len = (int32_t*)malloc(B * sizeof(int32_t));
  int32_t* keep = (int32_t*)malloc(rows * sizeof(int32_t));
  int32_t* offs = (int32_t*)malloc((B + 1) * sizeof(int32_t));
  if (!bad && mars_ref_commit(tok, alen, path, bonus, B, N, out_tok, out_len, keep, offs) != 0) bad = 1;
  if (!bad && (offs[B] < B || offs[B] > (int)rows)) bad = 1;
  free(logits); free(q); free(tok); free(par); free(theta); free(u); free(mask); free(dec); free(alen); free(path);
  free(bonus); free(status); free(st); free(dg); free(out_tok); free(out_len); free(keep); free(offs);
  return bad;
}

int main(void) {
  int bad = 0, n = 0;
  const int shapes[][3] = {{1, 1, 2}, {2, 9, 64}, {3, 17, 1000}, {1, 60, 4099}, {5, 8, 7}};
  for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s)
    for (int bf16 = 0; bf16 < 2; ++bf16)
      for (int mode = 0; mode < 3; ++mode)          /* greedy, sampling one-hot, sampling dense */
        for (int tree = 0; tree < 2; ++tree)
          for (int ind = 0; ind < 3; ++ind) {
            const float T = mode == 0 ? 0.0f : (mode == 1 ? 1.0f : 0.7f);
            bad += run_case(shapes[s][0], shapes[s][1], shapes[s][2], bf16, T, mode == 2, tree, ind, (n % 7) == 3);
            ++n;
          }
  printf("sanitize_oracle: %d cases, %d failed\n", n, bad);
  return bad != 0;
}
