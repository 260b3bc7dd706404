/*
 * Drives the CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.
 *
 * Built by tests/test_oracle_sanitizers.py together with oracle/espo_oracle.c (gcc,
 * -fsanitize=address,undefined, no recovery) and run as a plain host program: any
 * out-of-bounds access, use of uninitialised stack beyond its frame, signed overflow or
 * misaligned access in the oracle ends the run with a non-zero status.  The inputs are the
 * hand examples of tests/golden/ (typed here as numbers: the regret on three-token rows,
 * the three advantage cases) plus the shapes where indexing mistakes would hide: a
 * vocabulary that is not a multiple of the 64-index draw block, in both input types, with
 * and without a filter on the draw; trajectories stored back to back with clipped, empty
 * and reversed extents; lengths outside [0, T].  Every buffer is allocated at its exact
 * size, so that the sanitizer sees the first byte beyond it.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  float mu_g, var_g, delta, clip_c, alpha_s, beta, eps;
  int32_t stop_enabled, eos_id, stop_mode;
  float stop_threshold;
  int32_t simulate;
  float top_p;
  int32_t top_k;
} oracle_params;

int oracle_step(const void* logits, int dtype, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const oracle_params* p, float* z, uint8_t* alive,
                int32_t* stop_step, int32_t* tokens, float* regret, float* logprob, const int32_t* forced_tokens,
                double* best_score, double* second_score, int32_t* second_token, double* sum_exp, float* row_max,
                float* entropy, int64_t* kept);
int oracle_state_update(int64_t B, const float* g, const int32_t* tokens, const float* values, const oracle_params* p,
                        uint64_t seed, int32_t step, float* z, uint8_t* alive, int32_t* stop_step);
int oracle_advantages(const float* rewards, const float* values, const int32_t* lengths, const uint8_t* stopped,
                      int64_t B, int64_t T, float r_fail, float gamma, float lambda, double* td, double* adv,
                      double* scale);
int oracle_gae_bruteforce(const float* rewards, const float* values, const int32_t* lengths, const uint8_t* stopped,
                          int64_t B, int64_t T, float r_fail, float gamma, float lambda, double* adv);
int oracle_advantages_terminal(const float* values, const int32_t* lengths, const uint8_t* stopped,
                               const float* terminal_reward, int64_t B, int64_t T, float r_fail, float gamma,
                               float lambda, double* td, double* adv, double* ret);
int oracle_advantages_packed(const float* rewards, const float* terminal_reward, const float* values, const int64_t* cu,
                             const uint8_t* stopped, int64_t B, int64_t N, float r_fail, float gamma, float lambda,
                             double* td, double* adv, double* ret, double* scale);
int oracle_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean, int ddof,
                  double* out, double* stats);
int oracle_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                       float mu_g, float var_g, float beta, float alpha_ema, float eta_beta, float target_rate,
                       float beta_min, float beta_max, double* out);
void oracle_set_threads(int n);

static int failures = 0;
#define CHECK(cond, ...)                                   \
  do {                                                     \
    if (!(cond)) {                                         \
      fprintf(stderr, "FAILED %s:%d: ", __FILE__, __LINE__); \
      fprintf(stderr, __VA_ARGS__);                        \
      fprintf(stderr, "\n");                               \
      ++failures;                                          \
    }                                                      \
  } while (0)

static void* exact(size_t bytes) {  /* an allocation of exactly this size (at least one byte) */
  void* p = malloc(bytes ? bytes : 1);
  if (!p) abort();
  memset(p, 0x7e, bytes ? bytes : 1);
  return p;
}

static uint32_t lcg_state = 12345u;
static float lcg_unit(void) {  /* in [0, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)(lcg_state >> 8) * (1.0f / 16777216.0f);
}

static oracle_params default_params(void) {
  oracle_params p;
  memset(&p, 0, sizeof p);
  p.mu_g = 1.0f; p.var_g = 2.0f; p.delta = 1e-8f; p.clip_c = 10.0f; p.alpha_s = 0.9f; p.beta = 7.0f; p.eps = 0.2f;
  p.stop_enabled = 1; p.eos_id = -1;
  return p;
}

/* the regret on three-token rows, forced tokens (tests/golden/regret_three_token.txt) */
static void regret_hand_values(void) {
  static const float rows[12][6] = {
      {2, 1, 0, 1.0f, 0, 0},      {2, 1, 0, 1.0f, 1, 1},      {2, 1, 0, 1.0f, 2, 2},       {2, 1, 0, 0.5f, 0, 0},
      {2, 1, 0, 0.5f, 1, 2},      {2, 1, 0, 0.5f, 2, 4},      {-1, 3, 3, 1.0f, 0, 4},      {-1, 3, 3, 1.0f, 1, 0},
      {-1, 3, 3, 1.0f, 2, 0},     {0.5f, -0.25f, 1.75f, 0.25f, 0, 5}, {0.5f, -0.25f, 1.75f, 0.25f, 1, 8},
      {0.5f, -0.25f, 1.75f, 0.25f, 2, 0}};
  for (int i = 0; i < 12; ++i) {
    float* x = exact(3 * sizeof(float));
    memcpy(x, rows[i], 3 * sizeof(float));
    float* values = exact(4); values[0] = 0.5f;
    float* z = exact(4); z[0] = 0.0f;
    uint8_t* alive = exact(1); alive[0] = 1;
    int32_t* ss = exact(4); ss[0] = -1;
    int32_t* tok = exact(4);
    float* g = exact(4);
    float* lp = exact(4);
    int32_t* forced = exact(4); forced[0] = (int32_t)rows[i][4];
    oracle_params p = default_params();
    int rc = oracle_step(x, 0, 1, 3, 3, rows[i][3], 9, 0, values, &p, z, alive, ss, tok, g, lp, forced, NULL, NULL, NULL,
                         NULL, NULL, NULL, NULL);
    CHECK(rc == 0, "oracle_step rc %d", rc);
    CHECK(tok[0] == forced[0] && g[0] == rows[i][5], "regret case %d: token %d g %g", i, tok[0], g[0]);
    free(x); free(values); free(z); free(alive); free(ss); free(tok); free(g); free(lp); free(forced);
  }
}

/* vocabularies that end inside a draw block, both input types, every optional output, filters */
static void ragged_steps(void) {
  static const int64_t Vs[] = {1, 3, 63, 64, 65, 130, 1000};
  for (unsigned vi = 0; vi < sizeof Vs / sizeof Vs[0]; ++vi) {
    for (int dtype = 0; dtype < 2; ++dtype) {
      for (int filter = 0; filter < 3; ++filter) {
        const int64_t B = 3, V = Vs[vi], stride = V;  /* no slack behind a row */
        const size_t esz = dtype == 0 ? 4 : 2;
        void* x = exact((size_t)(B * stride) * esz);
        for (int64_t i = 0; i < B * stride; ++i) {
          const float f = (lcg_unit() - 0.5f) * 8.0f;
          if (dtype == 0) {
            ((float*)x)[i] = f;
          } else {  /* bf16: the upper half of the float */
            uint32_t bits;
            memcpy(&bits, &f, 4);
            ((uint16_t*)x)[i] = (uint16_t)(bits >> 16);
          }
        }
        if (V > 2 && dtype == 0) ((float*)x)[1] = -INFINITY;  /* a masked entry */
        float* values = exact(B * 4);
        float* z = exact(B * 4);
        uint8_t* alive = exact(B);
        int32_t* ss = exact(B * 4);
        for (int b = 0; b < B; ++b) { values[b] = 0.3f * b; z[b] = 0.1f * b; alive[b] = b != 1; ss[b] = -1; }
        int32_t* tok = exact(B * 4);
        float* g = exact(B * 4);
        float* lp = exact(B * 4);
        double* s1 = exact(B * 8);
        double* s2 = exact(B * 8);
        int32_t* t2 = exact(B * 4);
        double* se = exact(B * 8);
        float* rm = exact(B * 4);
        float* ent = exact(B * 4);
        int64_t* kept = exact(B * 8);
        oracle_params p = default_params();
        if (filter == 1) p.top_p = 0.7f;
        if (filter == 2) p.top_k = 5;
        for (int step = 0; step < 3; ++step) {
          int rc = oracle_step(x, dtype, B, V, stride, 0.6f, 77, step, values, &p, z, alive, ss, tok, g, lp, NULL, s1, s2,
                               t2, se, rm, ent, kept);
          CHECK(rc == 0, "oracle_step rc %d", rc);
          for (int b = 0; b < B; ++b) {
            if (b == 1) { CHECK(tok[b] == -1 && g[b] == 0.0f, "dead row touched"); continue; }
            if (!alive[b] && ss[b] != step) continue;
            CHECK(tok[b] >= 0 && tok[b] < V, "V=%lld token %d", (long long)V, tok[b]);
            CHECK(g[b] >= 0.0f && lp[b] <= 0.0f && ent[b] >= 0.0f, "V=%lld g %g lp %g H %g", (long long)V, g[b], lp[b], ent[b]);
          }
        }
        free(x); free(values); free(z); free(alive); free(ss); free(tok); free(g); free(lp); free(s1); free(s2);
        free(t2); free(se); free(rm); free(ent); free(kept);
      }
    }
  }
}

/* the three hand examples of tests/golden/gae_hand_example.txt, in the padded and the packed layout */
static void advantage_hand_examples(void) {
  const int64_t B = 2, T = 3;
  float* values = exact(B * T * 4);
  float* rewards = exact(B * T * 4);
  const float v[6] = {0.5f, 0.2f, -0.1f, 0.5f, 0.2f, -0.1f}, r[6] = {0, 0, 1, 0, 5, 0};
  memcpy(values, v, sizeof v);
  memcpy(rewards, r, sizeof r);
  int32_t* lengths = exact(B * 4); lengths[0] = 3; lengths[1] = 2;
  uint8_t* stopped = exact(B); stopped[0] = 0; stopped[1] = 1;
  double* td = exact(B * T * 8);
  double* adv = exact(B * T * 8);
  double* scale = exact(B * T * 8);
  double* brute = exact(B * T * 8);
  CHECK(oracle_advantages(rewards, values, lengths, stopped, B, T, -1.0f, 1.0f, 0.95f, td, adv, scale) == 0, "rc");
  CHECK(oracle_gae_bruteforce(rewards, values, lengths, stopped, B, T, -1.0f, 1.0f, 0.95f, brute) == 0, "rc");
  const double want_td[6] = {-0.3, -0.3, 1.1, -0.3, -1.2, 0}, want_adv[6] = {0.40775, 0.745, 1.1, -1.44, -1.2, 0};
  for (int i = 0; i < 6; ++i) {
    CHECK(fabs(td[i] - want_td[i]) < 1e-6 && fabs(adv[i] - want_adv[i]) < 1e-6, "hand example %d: %g %g", i, td[i], adv[i]);
    CHECK(fabs(brute[i] - adv[i]) < 1e-12, "brute force %d", i);
  }
  /* case C: gamma = lambda = 0.5 */
  const float vc[3] = {1, 2, 4}, rc3[3] = {0, 0, 2};
  memcpy(values, vc, sizeof vc);
  memcpy(rewards, rc3, sizeof rc3);
  lengths[0] = 3; stopped[0] = 0;
  CHECK(oracle_advantages(rewards, values, lengths, stopped, 1, T, -1.0f, 0.5f, 0.5f, td, adv, scale) == 0, "rc");
  CHECK(td[2] == -2 && adv[1] == -0.5 && adv[0] == -0.125, "case C");
  /* lengths outside [0, T] are clamped */
  lengths[0] = -4; lengths[1] = 99;
  CHECK(oracle_advantages(rewards, values, lengths, stopped, B, T, -1.0f, 1.0f, 0.95f, td, adv, scale) == 0, "rc");
  CHECK(adv[0] == 0 && adv[2] == 0, "negative length");
  /* the terminal form and the value targets */
  float* term = exact(B * 4); term[0] = 1.0f; term[1] = 0.0f;
  double* ret = exact(B * T * 8);
  memcpy(values, v, sizeof v);
  lengths[0] = 3; lengths[1] = 2; stopped[0] = 0; stopped[1] = 1;
  CHECK(oracle_advantages_terminal(values, lengths, stopped, term, B, T, -1.0f, 1.0f, 0.95f, td, adv, ret) == 0, "rc");
  for (int i = 0; i < 6; ++i) CHECK(fabs(adv[i] - want_adv[i]) < 1e-6, "terminal form %d", i);
  CHECK(fabs(ret[0] - (0.40775 + 0.5)) < 1e-6, "value target");
  free(values); free(rewards); free(lengths); free(stopped); free(td); free(adv); free(scale); free(brute); free(term); free(ret);
}

/* trajectories stored back to back: extents that are clipped, empty, reversed, and a gap nobody owns */
static void packed_extents(void) {
  const int64_t N = 11, B = 5;
  float* values = exact(N * 4);
  float* rewards = exact(N * 4);
  for (int i = 0; i < N; ++i) { values[i] = lcg_unit() - 0.5f; rewards[i] = lcg_unit(); }
  int64_t* cu = exact((B + 1) * 8);
  const int64_t offs[6] = {-3, 4, 4, 2, 7, 40};  /* [-3,4) clipped to [0,4); [4,4) empty; [4,2) reversed; [2,7) overlaps; [7,40) clipped */
  memcpy(cu, offs, sizeof offs);
  uint8_t* stopped = exact(B);
  for (int b = 0; b < B; ++b) stopped[b] = (uint8_t)(b & 1);
  float* term = exact(B * 4);
  for (int b = 0; b < B; ++b) term[b] = 1.0f;
  double* td = exact(N * 8);
  double* adv = exact(N * 8);
  double* ret = exact(N * 8);
  double* scale = exact(N * 8);
  for (int form = 0; form < 2; ++form) {
    for (int i = 0; i < N; ++i) td[i] = adv[i] = ret[i] = scale[i] = NAN;
    int rc = oracle_advantages_packed(form == 0 ? rewards : NULL, form == 0 ? NULL : term, values, cu, stopped, B, N, -1.0f,
                                      1.0f, 0.95f, td, adv, ret, scale);
    CHECK(rc == 0, "packed rc %d", rc);
    for (int i = 0; i < N; ++i) CHECK(isfinite(adv[i]) && isfinite(td[i]), "packed form %d position %d not written", form, i);
  }
  /* a gap: positions 4..6 belong to nobody */
  const int64_t gap[3] = {0, 4, 0};
  int64_t* cu2 = exact(3 * 8);
  memcpy(cu2, gap, sizeof gap);
  cu2[2] = 4;
  for (int i = 0; i < N; ++i) td[i] = adv[i] = NAN;
  CHECK(oracle_advantages_packed(rewards, NULL, values, cu2, stopped, 2, N, -1.0f, 1.0f, 0.95f, td, adv, NULL, NULL) == 0, "rc");
  CHECK(isfinite(adv[3]) && isnan(adv[4]) && isnan(adv[10]), "unowned positions were written");
  free(values); free(rewards); free(cu); free(cu2); free(stopped); free(term); free(td); free(adv); free(ret); free(scale);
}

static void whitening_and_batch_statistics(void) {
  const int64_t B = 3, T = 7;
  float* a = exact(B * T * 4);
  for (int i = 0; i < B * T; ++i) a[i] = lcg_unit() * 4.0f;
  int32_t* lengths = exact(B * 4); lengths[0] = 7; lengths[1] = 0; lengths[2] = 12;  /* the last one is clamped */
  uint8_t* stopped = exact(B); stopped[0] = 1; stopped[1] = 0; stopped[2] = 0;
  double* out = exact(B * T * 8);
  double* stats = exact(3 * 8);
  CHECK(oracle_whiten(a, lengths, B, T, 1e-8f, 1, 0, out, stats) == 0, "rc");
  CHECK(stats[2] == 14.0, "whiten n %g", stats[2]);
  double m = 0;
  for (int t = 0; t < 7; ++t) m += out[t] + out[2 * T + t];
  CHECK(fabs(m) < 1e-9, "whitened mean %g", m);
  CHECK(oracle_whiten(a, lengths, B, T, 0.0f, 0, 1, out, NULL) == 0, "rc");
  /* the hand example: 1, 2, 3, 4 has mean 5/2 and variance 5/4 */
  const float h[4] = {1, 2, 3, 4};
  memcpy(a, h, sizeof h);
  lengths[0] = 4;
  CHECK(oracle_whiten(a, lengths, 1, T, 0.0f, 1, 0, out, stats) == 0, "rc");
  CHECK(stats[0] == 2.5 && stats[1] == 1.25, "whiten hand example %g %g", stats[0], stats[1]);
  double* res = exact(7 * 8);
  lengths[0] = 4; lengths[1] = -1; lengths[2] = 2;
  CHECK(oracle_batch_stats(a, lengths, stopped, B, T, 1.0f, 2.0f, 7.0f, 0.99f, 0.1f, 0.25f, 0.0f, 7.0f, res) == 0, "rc");
  CHECK(res[6] == 6.0, "batch tokens %g", res[6]);
  CHECK(oracle_batch_stats(NULL, NULL, NULL, 0, 0, 1.0f, 2.0f, 7.0f, 0.99f, 0.1f, 0.25f, 0.0f, 7.0f, res) == 0, "rc");
  free(a); free(lengths); free(stopped); free(out); free(stats); free(res);
}

static void scalar_chain_replay(void) {
  const int64_t B = 4;
  float* g = exact(B * 4);
  int32_t* tok = exact(B * 4);
  float* values = exact(B * 4);
  float* z = exact(B * 4);
  uint8_t* alive = exact(B);
  int32_t* ss = exact(B * 4);
  for (int b = 0; b < B; ++b) { g[b] = 3.0f * b; tok[b] = b; values[b] = 0.1f; z[b] = 0; alive[b] = 1; ss[b] = -1; }
  oracle_params p = default_params();
  for (int mode = 0; mode < 4; ++mode) {
    p.stop_mode = mode;
    p.stop_threshold = 0.5f;
    for (int step = 0; step < 20; ++step)
      CHECK(oracle_state_update(B, g, tok, values, &p, 5, step, z, alive, ss) == 0, "rc");
  }
  CHECK(alive[0] == 1 || ss[0] >= 0, "state");
  free(g); free(tok); free(values); free(z); free(alive); free(ss);
}

int main(void) {
  oracle_set_threads(2);
  regret_hand_values();
  ragged_steps();
  advantage_hand_examples();
  packed_extents();
  whitening_and_batch_statistics();
  scalar_chain_replay();
  if (failures) {
    fprintf(stderr, "%d check(s) failed\n", failures);
    return 1;
  }
  printf("oracle ran clean under the sanitizers\n");
  return 0;
}
