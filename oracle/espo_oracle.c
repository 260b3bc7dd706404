/*
 * espo_oracle.c -- plain CPU oracle for the ESPO per-step hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
 * what the GPU kernels must compute.  It is used by the test-suite, by the smoke
 * check and by the "cpu_baseline" leg of the benchmark, and by nothing else; the
 * GPU library neither links nor imports it, and it shares no source, header, table
 * or helper with the GPU code.
 *
 * What follows the paper, and where:
 *   oracle_step        Algorithm 1 (body of the while loop), Eq. step_gap,
 *                      Eq. normalized_gap, Eq. smoothed_score, Eq. stop_rule,
 *                      Eq. failure_reward.  The paper only says "sample a_t from pi";
 *                      the draw is realised as Gumbel-max, a = argmax_v (y_v + G_v) with
 *                      iid standard Gumbel G_v, over a Philox4x32-10 stream (Salmon et
 *                      al., "Parallel random numbers: as easy as 1, 2, 3", SC'11); the
 *                      stream definition below is the one the GPU path implements too.
 *                      Optional output: the entropy of that distribution (the quantity
 *                      tracked in the section on policy entropy and diversity, Fig. 2b),
 *                      by its definition.
 *                      Optional filters on the draw: top-p (nucleus) as in the evaluation
 *                      set-up of Section 5, and top-k; the kept set by its definition over a
 *                      library sort, the draw over the kept set with the same stream.
 *   oracle_advantages  Section 3 (TD error, Eq. gae) on the truncated trajectory of
 *                      Section 4.4 (failure reward at the stop step, no bootstrap).
 *   oracle_gae_bruteforce  Eq. gae written as the explicit double sum, O(L^2).
 *   oracle_advantages_packed  both forms for trajectories stored back to back
 *   oracle_advantages_terminal  the same for the reward structure of Algorithm 1 (zero
 *                      until the last step), plus the value targets A_t + V(s_t).
 *   oracle_whiten      advantage whitening over the valid tokens (standard PPO practice),
 *                      two-pass definitions.
 *   oracle_batch_stats Section 4.2 (EMA of the batch mean and variance of the regret) and
 *                      Eq. beta_update, plain two-pass definitions.
 *   stop_decision      Eq. stop_rule and the replacement tests of the ablations (Section 6,
 *                      variants D, E, F); the simulate mode of Section 7 ("ESPO/Original").
 *
 * Pins (tests marked "not gpu"): hand values of the regret on 3-token rows, closed
 * forms of the smoothed state, stop rule never/always firing, softmax frequencies of
 * the sampler on tiny vocabularies, moments of the Gumbel variates, closed forms of the
 * entropy (uniform, two-token, masked rows) and a library routine on random rows, the kept
 * set of top-p / top-k against its O(V^2) definition and a sorted cumulative sum, frequencies of
 * filtered draws against the renormalised distribution, GAE against the
 * explicit double sum and against telescoping identities.
 * The paper fixes no random stream, so the identity of the sampled token on a large
 * vocabulary rests on this file's own definition of the stream: the generator is pinned
 * to the published Philox4x32-10 by its authors' three known-answer inputs (zeros, ones,
 * digits of pi), the construction of the variates by the distribution tests.
 *
 * Precision: scores, the softmax sum and the advantages are in double.  The scalar
 * chain g -> g~ -> z -> test is in fp32, one rounding per operation in the order
 * written below, because the stop decision is an integer decided by floating point
 * and must be taken in the precision the kernel uses.  Build with -ffp-contract=off.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  float mu_g, var_g, delta, clip_c, alpha_s, beta, eps;
  int32_t stop_enabled;
  int32_t eos_id;
  int32_t stop_mode;      /* 0 full rule; 1 value only; 2 regret only; 3 random (Section 6, variants D, E, F) */
  float stop_threshold;   /* the fixed threshold of variants D and E; the per-step stop probability of F      */
  int32_t simulate;       /* record the first stop step but keep decoding ("ESPO/Original", Section 7)        */
  float top_p;            /* nucleus sampling, as in the evaluation set-up of Section 5 (p = 0.7 there); 0 or >= 1: off */
  int32_t top_k;          /* keep the k largest logits; <= 0: off (the paper's evaluation leaves it off)       */
} oracle_params;

/* ------------------------------------------------------------------ Philox4x32-10 */
/* Salmon et al. 2011: four 32-bit counter words, two key words, ten rounds.  One
 * round multiplies words 0 and 2 by fixed odd constants, keeps the low halves and
 * folds the high halves into the other two words together with the round key; the
 * key advances by a Weyl sequence between rounds. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Random stream of the draw.  The Gumbel variates G_v (v = 0..V-1) of one row and step
 * are iid standard Gumbel, generated top-down in blocks of 64 consecutive vocabulary
 * indices (the joint law of n iid Gumbels factorises into: their maximum M, which is
 * Gumbel shifted by ln n; the position of the maximum, uniform; and the others, iid
 * Gumbel truncated to (-inf, M) -- Maddison, Tarlow & Minka, "A* sampling", 2014):
 *   block q = v / 64 holds indices [64 q, min(64 q + 64, V)), n_q of them;
 *   w     = word (q & 3) of Philox(counter = (q >> 2, step, row, TAG_BLOCK), key = seed);
 *   M_q   = ln n_q - ln(-ln u(w))            maximum of the block's variates
 *   pos_q = (w >> 3) & 63                     which index of the block attains it (n_q = 64;
 *           the ragged last block takes (w' * n_q) >> 32 with w' = word 0 of
 *           Philox(counter = (q, step, row, TAG_RAGGED), key = seed) instead)
 *   w_v   = word (v & 3) of Philox(counter = (v >> 2, step, row, TAG_ELEM), key = seed)
 *   G_v   = M_q                               if v = 64 q + pos_q
 *         = -ln(exp(-M_q) - ln u(w_v))        otherwise (inverse cdf of the truncation)
 * with u(w) = (2 (w >> 9) + 1) / 2^24 in (0, 1).
 */
#define ORACLE_TAG_BLOCK 0x4553504Fu
#define ORACLE_TAG_ELEM 0x6573706Fu
#define ORACLE_TAG_RAGGED 0x52414747u
#define ORACLE_BLOCK 64

/* u in (0,1): the top 23 bits r of the word give u = (2r+1)/2^24. */
double oracle_uniform(uint32_t word) {
  uint32_t r = word >> 9;
  return (double)(2u * r + 1u) / 16777216.0;
}

/* Standard Gumbel variate G = -ln(-ln u). */
double oracle_gumbel(uint32_t word) { return -log(-log(oracle_uniform(word))); }

/* The 32-bit word that belongs to vocabulary index v of row `row` at `step`. */
uint32_t oracle_stream_word(uint64_t seed, int64_t row, int32_t step, int64_t v) {
  uint32_t ctr[4] = {(uint32_t)(v >> 2), (uint32_t)step, (uint32_t)row, ORACLE_TAG_ELEM};
  uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  return out[v & 3];
}

/* Maximum M_q of block q (which holds n indices) and the offset pos_q that attains it. */
void oracle_block_draw(uint64_t seed, int64_t row, int32_t step, int64_t q, int64_t n,
                       double* M, int64_t* pos) {
  uint32_t ctr[4] = {(uint32_t)(q >> 2), (uint32_t)step, (uint32_t)row, ORACLE_TAG_BLOCK};
  uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  uint32_t out[4];
  oracle_philox4x32_10(ctr, key, out);
  const uint32_t w = out[q & 3];
  *M = log((double)n) + oracle_gumbel(w);               /* top 23 bits of w */
  if (n == ORACLE_BLOCK) {
    *pos = (int64_t)((w >> 3) & 63u);                    /* six of the bits u(w) does not use */
  } else {                                               /* the ragged last block: own draw */
    uint32_t ctr2[4] = {(uint32_t)q, (uint32_t)step, (uint32_t)row, ORACLE_TAG_RAGGED};
    oracle_philox4x32_10(ctr2, key, out);
    *pos = (int64_t)(((uint64_t)out[0] * (uint64_t)n) >> 32);
  }
}

/* G_v for an index v of the block that starts at `first` and drew (M, pos). */
static double gumbel_in_block(uint64_t seed, int64_t row, int32_t step, int64_t v,
                              int64_t first, double M, int64_t pos) {
  if (v == first + pos) return M;
  const double u = oracle_uniform(oracle_stream_word(seed, row, step, v));
  return -log(exp(-M) - log(u));
}

/* The Gumbel variate of vocabulary index v in a row of V entries. */
double oracle_gumbel_at(uint64_t seed, int64_t row, int32_t step, int64_t v, int64_t V) {
  const int64_t q = v / ORACLE_BLOCK;
  const int64_t first = q * ORACLE_BLOCK;
  const int64_t n = (V - first < ORACLE_BLOCK) ? V - first : ORACLE_BLOCK;
  double M;
  int64_t pos;
  oracle_block_draw(seed, row, step, q, n, &M, &pos);
  return gumbel_in_block(seed, row, step, v, first, M, pos);
}

/*
 * The stop decision of one live row at one step, after its state z has been advanced.
 *   mode 0  Eq. stop_rule: z > beta * max(V, eps), strict, in fp32.
 *   mode 1  the value alone: V < threshold (ablation D).
 *   mode 2  the smoothed regret alone: z > threshold (ablation E).
 *   mode 3  a coin: u < threshold with u = u(word 0 of Philox(counter (0, step, row,
 *           0x53544F50), key)), independent of logits and values (ablation F).
 * All are gated by stop_enabled.
 */
static int stop_decision(const oracle_params* p, float zn, float value, uint64_t seed, int64_t row, int32_t step) {
  if (!p->stop_enabled) return 0;
  switch (p->stop_mode) {
    case 1: return value < p->stop_threshold;
    case 2: return zn > p->stop_threshold;
    case 3: {
      const uint32_t ctr[4] = {0u, (uint32_t)step, (uint32_t)row, 0x53544F50u};
      const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
      uint32_t w[4];
      oracle_philox4x32_10(ctr, key, w);
      return oracle_uniform(w[0]) < (double)p->stop_threshold;
    }
    default: {
      const float thr = p->beta * fmaxf(value, p->eps);
      return zn > thr;                                   /* Eq. stop_rule, strict     */
    }
  }
}

/* What a stop (or the end-of-sequence token) does to the row's state. */
static void apply_end(const oracle_params* p, int eos, int stop, int32_t step, uint8_t* alive, int32_t* stop_step) {
  if (eos) {
    *alive = 0;                                          /* natural end, not a failure */
  } else if (stop) {
    if (p->simulate) {
      if (*stop_step < 0) *stop_step = step;             /* first stop only; decoding goes on */
    } else {
      *alive = 0;                                        /* absorbing failure          */
      *stop_step = step;
    }
  }
}

static inline float load_logit(const void* base, int dtype, int64_t idx) {
  if (dtype == 0) return ((const float*)base)[idx];
  uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16; /* bf16 -> fp32, exact */
  float f;
  memcpy(&f, &bits, 4);
  return f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * The kept set of filtered sampling, as the smallest logit it contains.
 *   top-p: the tokens of largest probability whose mass reaches p; tokens of equal logit stay
 *          together, so v is kept iff the mass of all tokens with a strictly larger logit is
 *          below p (the most probable token is always kept);
 *   top-k: v is kept iff fewer than k tokens have a strictly larger logit.
 * `ys` are the row's V tempered logits, `S` the softmax sum relative to y_max.  Returns the
 * smallest kept y and the number of kept tokens.
 */
static int cmp_desc(const void* a, const void* b) {
  const double x = *(const double*)a, y = *(const double*)b;
  return (x < y) - (x > y);
}

static double kept_threshold(const double* ys, int64_t V, double y_max, double S, double top_p, int64_t top_k,
                             int64_t* kept) {
  double* sorted = (double*)malloc((size_t)V * sizeof(double));
  memcpy(sorted, ys, (size_t)V * sizeof(double));
  qsort(sorted, (size_t)V, sizeof(double), cmp_desc);      /* library sort, descending */
  double mass_above = 0.0, thr = sorted[0];
  int64_t count_above = 0, n = 0, i = 0;
  while (i < V) {                                          /* groups of equal logit, largest first */
    int64_t j = i;
    double group = 0.0;
    while (j < V && sorted[j] == sorted[i]) { group += exp(sorted[j] - y_max); ++j; }
    const int keep = top_k > 0 ? (count_above < top_k) : (mass_above < top_p * S);
    if (!keep) break;
    thr = sorted[i];
    n = j;
    mass_above += group;
    count_above = j;
    i = j;
  }
  free(sorted);
  *kept = n;
  return thr;
}

/*
 * One decode step for B rows.  Arrays are host memory with the same meaning and
 * layout as the GPU entry point's.  Extra, optional (NULL-able) arguments:
 *   forced_tokens[b] >= 0  use that token instead of the draw (near-tie protocol);
 *   best_score / second_score / second_token  the two largest perturbed scores of
 *                          the draw and the index of the runner-up;
 *   sum_exp                S = sum_v exp(y_v - y_max);
 *   row_max                the row maximum m;
 *   kept                   number of tokens the top-p / top-k filter keeps (V without filter);
 *   entropy                H = -sum_v pi_v ln pi_v of the distribution the token is drawn
 *                          from, pi_v = exp(y_v - y_max) / S (the policy entropy tracked in
 *                          the section on policy entropy and diversity, Fig. 2b); indices
 *                          with pi_v = 0 contribute nothing.
 * Returns 0, or -1 on invalid arguments.
 */
int oracle_step(const void* logits, int dtype, int64_t B, int64_t V, int64_t row_stride,
                float temperature, uint64_t seed, int32_t step,
                const float* values, const oracle_params* p,
                float* z, uint8_t* alive, int32_t* stop_step,
                int32_t* tokens, float* regret, float* logprob,
                const int32_t* forced_tokens,
                double* best_score, double* second_score, int32_t* second_token,
                double* sum_exp, float* row_max, float* entropy, int64_t* kept) {
  if (!logits || !values || !p || !z || !alive || !stop_step || !tokens || !regret) return -1;
  if (B < 0 || V < 1 || row_stride < V || !(temperature > 0.0f) || !isfinite(temperature)) return -1;
  if (dtype != 0 && dtype != 1) return -1;
  if (!(p->top_p >= 0.0f && p->top_p <= 1.0f) || p->top_k < 0) return -1;
  if (p->top_p > 0.0f && p->top_p < 1.0f && p->top_k > 0) return -1;   /* one filter at a time */

  const float inv_tau = 1.0f / temperature;              /* one fp32 division        */
  const float rsd = 1.0f / sqrtf(p->var_g + p->delta);   /* 1/sqrt(sigma_g^2+delta)  */
  const float oma = 1.0f - p->alpha_s;

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t b = 0; b < B; ++b) {
    if (!alive[b]) {                                     /* done rows are not decoded */
      tokens[b] = -1;
      regret[b] = 0.0f;
      if (logprob) logprob[b] = 0.0f;
      if (best_score) best_score[b] = 0.0;
      if (second_score) second_score[b] = 0.0;
      if (second_token) second_token[b] = -1;
      if (sum_exp) sum_exp[b] = 0.0;
      if (row_max) row_max[b] = 0.0f;
      if (entropy) entropy[b] = 0.0f;
      if (kept) kept[b] = 0;
      continue;
    }
    const int64_t base = b * row_stride;

    /* row maximum (exact) */
    float m = -INFINITY;
    for (int64_t v = 0; v < V; ++v) {
      float x = load_logit(logits, dtype, base + v);
      if (x > m) m = x;
    }
    const double y_max = (double)m * (double)inv_tau;

    /* filtered sampling (the evaluation set-up's top-p; top-k): the kept set is {v : y_v >= y_keep} */
    const int filter_p = p->top_p > 0.0f && p->top_p < 1.0f, filter_k = p->top_k > 0;
    double y_keep = -INFINITY;
    int64_t n_kept = V;
    if ((filter_p || filter_k) && m > -INFINITY) {
      double* ys = (double*)malloc((size_t)V * sizeof(double));
      double S0 = 0.0;
      for (int64_t v = 0; v < V; ++v) {
        ys[v] = (double)load_logit(logits, dtype, base + v) * (double)inv_tau;
        S0 += exp(ys[v] - y_max);
      }
      y_keep = kept_threshold(ys, V, y_max, S0, (double)p->top_p, filter_k ? p->top_k : 0, &n_kept);
      free(ys);
    }

    /* softmax normaliser and Gumbel-max draw, in index order */
    double S = 0.0;
    double s1 = -INFINITY, s2 = -INFINITY;
    int64_t a1 = -1, a2 = -1;
    double M_q = 0.0;
    int64_t pos_q = 0, first_q = 0;
    for (int64_t v = 0; v < V; ++v) {
      if (v % ORACLE_BLOCK == 0) {                       /* a new block: draw its maximum */
        first_q = v;
        const int64_t n_q = (V - v < ORACLE_BLOCK) ? V - v : ORACLE_BLOCK;
        oracle_block_draw(seed, b, step, v / ORACLE_BLOCK, n_q, &M_q, &pos_q);
      }
      float x = load_logit(logits, dtype, base + v);
      double y = (double)x * (double)inv_tau;            /* tempered logit           */
      S += exp(y - y_max);
      double s = y + gumbel_in_block(seed, b, step, v, first_q, M_q, pos_q);
      if (y < y_keep) continue;                          /* filtered out: cannot be drawn */
      if (s > s1) {                                      /* strict: lowest index wins */
        s2 = s1; a2 = a1;
        s1 = s; a1 = v;
      } else if (s > s2) {
        s2 = s; a2 = v;
      }
    }
    int64_t a = a1;
    if (forced_tokens && forced_tokens[b] >= 0) a = forced_tokens[b];
    if (a < 0) a = 0;                                    /* row of -inf only: unspecified */
    const float x_a = load_logit(logits, dtype, base + a);

    /* scalar chain, fp32, one rounding per operation */
    const float d = m - x_a;
    const float g = d * inv_tau;                         /* Eq. step_gap              */
    const float n = (g - p->mu_g) * rsd;
    const float gt = fminf(fmaxf(n, -p->clip_c), p->clip_c);   /* Eq. normalized_gap  */
    const float t = oma * gt;
    const float zn = fmaf(p->alpha_s, z[b], t);          /* Eq. smoothed_score        */
    const int stop = stop_decision(p, zn, values[b], seed, b, step);

    tokens[b] = (int32_t)a;
    regret[b] = g;
    z[b] = zn;
    if (logprob) logprob[b] = (float)(-(double)g - log(S));
    apply_end(p, p->eos_id >= 0 && a == (int64_t)p->eos_id, stop, step, &alive[b], &stop_step[b]);
    if (best_score) best_score[b] = s1;
    if (second_score) second_score[b] = s2;
    if (second_token) second_token[b] = (int32_t)a2;
    if (sum_exp) sum_exp[b] = S;
    if (row_max) row_max[b] = m;
    if (kept) kept[b] = n_kept;
    if (entropy) {                                       /* the definition, term by term */
      double H = 0.0;
      for (int64_t v = 0; v < V; ++v) {
        const double y = (double)load_logit(logits, dtype, base + v) * (double)inv_tau;
        const double pi = exp(y - y_max) / S;
        if (pi > 0.0) H -= pi * log(pi);
      }
      entropy[b] = (float)H;
    }
  }
  return 0;
}

/*
 * The scalar chain alone: given the regret g of a live row, advance (z, alive,
 * stop_step) exactly as oracle_step does.  Lets a test replay the state of every
 * row of a large batch from a recorded regret/token stream.
 */
int oracle_state_update(int64_t B, const float* g, const int32_t* tokens, const float* values,
                        const oracle_params* p, uint64_t seed, int32_t step,
                        float* z, uint8_t* alive, int32_t* stop_step) {
  if (!g || !tokens || !values || !p || !z || !alive || !stop_step || B < 0) return -1;
  const float rsd = 1.0f / sqrtf(p->var_g + p->delta);
  const float oma = 1.0f - p->alpha_s;
  for (int64_t b = 0; b < B; ++b) {
    if (!alive[b]) continue;
    const float n = (g[b] - p->mu_g) * rsd;
    const float gt = fminf(fmaxf(n, -p->clip_c), p->clip_c);
    const float t = oma * gt;
    const float zn = fmaf(p->alpha_s, z[b], t);
    const int stop = stop_decision(p, zn, values[b], seed, b, step);
    z[b] = zn;
    apply_end(p, p->eos_id >= 0 && tokens[b] == p->eos_id, stop, step, &alive[b], &stop_step[b]);
  }
  return 0;
}

/*
 * TD errors and GAE on truncated trajectories, by the backward recursion
 * A_t = delta_t + gamma*lambda*A_{t+1} that Eq. gae unrolls to.  Outputs in double.
 * `scale` (optional) receives sum_l |gamma*lambda|^l (|r| + |gamma V'| + |V|)_{t+l}, the
 * magnitude of the terms that enter the sum: an fp32 evaluation rounds each delta to a
 * relative 2^-24 of its largest term (not of delta itself, which may cancel) and each
 * partial sum likewise, so errors are judged against this magnitude.
 */
int oracle_advantages(const float* rewards, const float* values,
                      const int32_t* lengths, const uint8_t* stopped,
                      int64_t B, int64_t T, float r_fail, float gamma, float lambda,
                      double* td, double* adv, double* scale) {
  if (B < 0 || T < 0) return -1;
  if (B == 0 || T == 0) return 0;
  if (!rewards || !values || !lengths || !stopped || !td || !adv) return -1;
  const double gam = (double)gamma;
  const double c = (double)gamma * (double)lambda;

#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    const float* r = rewards + b * T;
    const float* val = values + b * T;
    double* d = td + b * T;
    double* A = adv + b * T;
    double* sc = scale ? scale + b * T : NULL;
    for (int64_t t = L; t < T; ++t) {
      d[t] = 0.0;
      A[t] = 0.0;
      if (sc) sc[t] = 0.0;
    }
    double a_next = 0.0;      /* advantage beyond the last token is zero            */
    double s_next = 0.0;
    for (int64_t t = L - 1; t >= 0; --t) {
      double r_t = (double)r[t];
      if (t == L - 1 && stopped[b]) r_t = (double)r_fail;       /* Eq. failure_reward */
      const double v_next = (t + 1 < L) ? (double)val[t + 1] : 0.0;  /* no bootstrap  */
      const double delta = r_t + gam * v_next - (double)val[t];
      a_next = delta + c * a_next;
      s_next = (fabs(r_t) + fabs(gam * v_next) + fabs((double)val[t])) + fabs(c) * s_next;
      d[t] = delta;
      A[t] = a_next;
      if (sc) sc[t] = s_next;
    }
  }
  return 0;
}

/*
 * Eq. gae as printed: A_t = sum_{l=0}^{L-t-1} (gamma*lambda)^l delta_{t+l}, every
 * power and every delta formed from scratch.  O(L^2); for small T only.
 */
int oracle_gae_bruteforce(const float* rewards, const float* values,
                          const int32_t* lengths, const uint8_t* stopped,
                          int64_t B, int64_t T, float r_fail, float gamma, float lambda,
                          double* adv) {
  if (B < 0 || T < 0) return -1;
  if (B == 0 || T == 0) return 0;
  if (!rewards || !values || !lengths || !stopped || !adv) return -1;
  const double c = (double)gamma * (double)lambda;
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < T; ++t) {
      double acc = 0.0;
      for (int64_t l = 0; t + l < L; ++l) {
        const int64_t u = t + l;
        double r_u = (double)rewards[b * T + u];
        if (u == L - 1 && stopped[b]) r_u = (double)r_fail;
        const double v_u = (double)values[b * T + u];
        const double v_un = (u + 1 < L) ? (double)values[b * T + u + 1] : 0.0;
        const double delta = r_u + (double)gamma * v_un - v_u;
        acc += pow(c, (double)l) * delta;
      }
      adv[b * T + t] = (t < L) ? acc : 0.0;
    }
  }
  return 0;
}

/*
 * The trajectory that Algorithm 1 returns has r_t = 0 at every step that goes on and one
 * reward at its last step: r_fail if the stop rule ended it (Eq. failure_reward), else the
 * task's terminal reward.  This is TD error and GAE (Section 3) for that reward structure,
 * given per row only the terminal reward, and also the critic's regression target
 * R_t = A_t + V(s_t) (the lambda-return that PPO's value loss uses; the paper keeps "the
 * standard PPO formulation").  Same recursion as above, written for this case on its own.
 * Outputs in double; td, adv, ret (ret may be NULL) are zero at t >= L.
 */
int oracle_advantages_terminal(const float* values, const int32_t* lengths, const uint8_t* stopped,
                               const float* terminal_reward, int64_t B, int64_t T,
                               float r_fail, float gamma, float lambda,
                               double* td, double* adv, double* ret) {
  if (B < 0 || T < 0) return -1;
  if (B == 0 || T == 0) return 0;
  if (!values || !lengths || !stopped || !terminal_reward || !td || !adv) return -1;
  const double gam = (double)gamma;
  const double c = (double)gamma * (double)lambda;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    const float* val = values + b * T;
    for (int64_t t = L; t < T; ++t) {
      td[b * T + t] = 0.0;
      adv[b * T + t] = 0.0;
      if (ret) ret[b * T + t] = 0.0;
    }
    double A = 0.0;
    for (int64_t t = L - 1; t >= 0; --t) {
      double delta;
      if (t == L - 1) {                                   /* last step: its reward, no bootstrap */
        const double r_end = stopped[b] ? (double)r_fail : (double)terminal_reward[b];
        delta = r_end - (double)val[t];
      } else {                                            /* a step that went on: r_t = 0        */
        delta = gam * (double)val[t + 1] - (double)val[t];
      }
      A = delta + c * A;
      td[b * T + t] = delta;
      adv[b * T + t] = A;
      if (ret) ret[b * T + t] = A + (double)val[t];
    }
  }
  return 0;
}

/*
 * The same quantities for trajectories stored back to back: trajectory b occupies positions
 * cu[b] .. cu[b+1]-1 of arrays of N tokens, so a truncated trajectory takes no padding.
 * Section 3 and Eq. failure_reward on each slice, written out once more for this layout:
 * rewards == NULL means the reward structure of Algorithm 1 (zero at every step that goes on,
 * terminal_reward[b] at the last); with a stop the last reward is r_fail in both forms.
 * An extent is clipped to [0, N] and an empty or reversed one holds no token.  Outputs in
 * double, written only at the positions some trajectory owns; ret (optional) is A_t + V(s_t),
 * scale (optional) the magnitude described at oracle_advantages.
 */
int oracle_advantages_packed(const float* rewards, const float* terminal_reward, const float* values,
                             const int64_t* cu, const uint8_t* stopped, int64_t B, int64_t N,
                             float r_fail, float gamma, float lambda,
                             double* td, double* adv, double* ret, double* scale) {
  if (B < 0 || N < 0) return -1;
  if (B == 0 || N == 0) return 0;
  if (!values || !cu || !stopped || !td || !adv) return -1;
  if (!rewards && !terminal_reward) return -1;
  const double gam = (double)gamma;
  const double c = (double)gamma * (double)lambda;
  for (int64_t b = 0; b < B; ++b) {
    int64_t first = cu[b], end = cu[b + 1];
    if (first < 0) first = 0;
    if (first > N) first = N;
    if (end > N) end = N;
    double A = 0.0, S = 0.0;                     /* nothing follows the last token */
    for (int64_t i = end - 1; i >= first; --i) {
      const int is_last = (i == end - 1);
      double r_i = rewards ? (double)rewards[i] : 0.0;
      if (is_last && !rewards) r_i = (double)terminal_reward[b];
      if (is_last && stopped[b]) r_i = (double)r_fail;
      const double v_next = is_last ? 0.0 : (double)values[i + 1];   /* no bootstrap past the end */
      const double delta = r_i + gam * v_next - (double)values[i];
      A = delta + c * A;
      S = (fabs(r_i) + fabs(gam * v_next) + fabs((double)values[i])) + fabs(c) * S;
      td[i] = delta;
      adv[i] = A;
      if (ret) ret[i] = A + (double)values[i];
      if (scale) scale[i] = S;
    }
  }
  return 0;
}

/*
 * Advantage whitening over the valid tokens of a batch, the normalisation that PPO
 * implementations apply to the GAE output before the clipped objective (the paper keeps the
 * standard PPO update, Section 3, and does not spell this step out): with n = sum_b L_b,
 *   mean = sum A / n,   var = sum (A - mean)^2 / (n - ddof),
 *   out[b,t] = (A[b,t] - (shift_mean ? mean : 0)) / sqrt(var + eps)        for t < L_b.
 * Plain two-pass definitions in double.  Positions at t >= L_b are neither read nor written.
 * With n - ddof <= 0 the variance is taken as 0, and with var + eps = 0 (a constant batch
 * and eps = 0) every output is 0 rather than 0/0.  stats (optional): mean, var, n.
 */
int oracle_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps,
                  int shift_mean, int ddof, double* out, double* stats) {
  if (B < 0 || T < 0 || ddof < 0 || ddof > 1) return -1;
  if (stats) stats[0] = stats[1] = stats[2] = 0.0;
  if (B == 0 || T == 0) return 0;
  if (!adv || !lengths || !out) return -1;
  double n = 0.0, sum = 0.0;
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < L; ++t) sum += (double)adv[b * T + t];
    n += (double)L;
  }
  if (n == 0.0) return 0;
  const double mean = sum / n;
  double ss = 0.0;
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < L; ++t) {
      const double d = (double)adv[b * T + t] - mean;
      ss += d * d;
    }
  }
  const double var = (n - (double)ddof > 0.0) ? ss / (n - (double)ddof) : 0.0;
  const double sd = sqrt(var + (double)eps);
  const double inv = sd > 0.0 ? 1.0 / sd : 0.0;   /* constant batch and eps = 0: nothing to scale by */
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < L; ++t)
      out[b * T + t] = inv > 0.0 ? ((double)adv[b * T + t] - (shift_mean ? mean : 0.0)) / sd : 0.0;
  }
  if (stats) {
    stats[0] = mean;
    stats[1] = var;
    stats[2] = n;
  }
  return 0;
}

/*
 * Batch-boundary update of the frozen statistics and of the threshold multiplier
 * (Section 4.2: EMA of the batch mean and variance of the regret; Eq. beta_update).
 *
 * The batch B is every valid token of every trajectory: regret[b,t] for t < L_b
 * (L_b clamped to [0,T]); entries at t >= L_b are never read.  Mean and variance are the
 * plain two-pass definitions in double, the variance with divisor n (the paper writes
 * Var(g_B) without a correction).  The stop rate is the fraction of trajectories that the
 * stop rule ended.  The three updated parameters are formed in double and rounded to
 * float once, since they are float fields of the rollout parameters.
 *   out[0] batch mean, out[1] batch variance, out[2] stop rate,
 *   out[3] mu_g', out[4] var_g', out[5] beta' (each exactly a float), out[6] token count n.
 * With n = 0 the two statistics are left as they are; with B = 0 beta as well.
 */
int oracle_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped,
                       int64_t B, int64_t T, float mu_g, float var_g, float beta,
                       float alpha_ema, float eta_beta, float target_rate, float beta_min, float beta_max,
                       double* out) {
  if (B < 0 || T < 0 || !out) return -1;
  if (B > 0 && (!lengths || !stopped || (T > 0 && !regret))) return -1;
  double n = 0.0, sum = 0.0;
  int64_t nstop = 0;
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < L; ++t) sum += (double)regret[b * T + t];
    n += (double)L;
    if (stopped[b]) ++nstop;
  }
  const double mean = n > 0.0 ? sum / n : 0.0;
  double ss = 0.0;
  for (int64_t b = 0; b < B; ++b) {
    int64_t L = lengths[b];
    if (L < 0) L = 0;
    if (L > T) L = T;
    for (int64_t t = 0; t < L; ++t) {
      const double d = (double)regret[b * T + t] - mean;
      ss += d * d;
    }
  }
  const double var = n > 0.0 ? ss / n : 0.0;
  const double rate = B > 0 ? (double)nstop / (double)B : 0.0;
  const double a = (double)alpha_ema;
  float mu_new = mu_g, var_new = var_g, beta_new = beta;
  if (n > 0.0) {
    mu_new = (float)(a * (double)mu_g + (1.0 - a) * mean);
    var_new = (float)(a * (double)var_g + (1.0 - a) * var);
  }
  if (B > 0) {
    double bt = (double)beta + (double)eta_beta * (rate - (double)target_rate);   /* Eq. beta_update */
    if (bt < (double)beta_min) bt = (double)beta_min;
    if (bt > (double)beta_max) bt = (double)beta_max;
    beta_new = (float)bt;
  }
  out[0] = mean; out[1] = var; out[2] = rate;
  out[3] = (double)mu_new; out[4] = (double)var_new; out[5] = (double)beta_new; out[6] = n;
  return 0;
}
