/*
 * espo.h -- C ABI of the ESPO per-generation-step hot path for AMD MI355X (gfx950).
 *
 * ESPO (Early-Stopping Proximal Policy Optimization) changes how rollouts are
 * collected: at every decode step it derives a regret signal from the policy
 * logits, smooths it per trajectory, and ends the trajectory as an absorbing
 * failure once the smoothed regret exceeds a value-dependent threshold
 * (Section 4, Algorithm 1).  GAE is then run on the truncated trajectories with
 * the failure reward placed at the stop step (Section 4.4, Eq. failure_reward,
 * Eq. gae).
 *
 * Four operations are exported, the advantage pass in three layouts:
 *   espo_step         one decode step for a batch of trajectories (Algorithm 1 body)
 *   espo_advantages   TD errors + GAE over the truncated trajectories (Section 3, 4.4)
 *   espo_advantages_terminal  the same for the rewards Algorithm 1 produces (zero until
 *                     the last step), optionally with the critic's value targets
 *   espo_advantages_packed    both for trajectories stored back to back, without padding
 *   espo_batch_stats  update of the frozen statistics and of beta between batches (Section 4.2, 4.3)
 *   espo_whiten       whitening of the advantages over the valid tokens (standard PPO step)
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     never allocates, frees or keeps them.  "host" pointers are ordinary host
 *     memory read during the call only.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  Calls never synchronise; outputs are valid once the
 *     stream has reached the point of the call.
 *   - Return value: ESPO_OK (0) or a negative espo_status.  On any error nothing
 *     has been enqueued.
 *   - No global mutable state: calls from several host threads on different streams
 *     are safe as long as they do not share output or workspace buffers.  (The one
 *     exception is espo_batch_stats_static, which says so.)
 *   - A call consists of kernel launches only (no allocation, no copy, no memset,
 *     no synchronisation), so it may be recorded while its stream is being captured
 *     into a HIP graph; scalar arguments (seed, step, parameters) are then fixed in
 *     the recorded nodes.
 */
#ifndef ESPO_H_
#define ESPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ESPO_OK = 0,
  ESPO_EINVAL = -1,     /* null pointer, negative size, bad temperature / parameter */
  ESPO_EALIGN = -2,     /* logits base or row pitch not 16-byte aligned              */
  ESPO_EWORKSPACE = -3, /* workspace missing or smaller than required                */
  ESPO_EHIP = -4,       /* the HIP runtime refused the launch                        */
  ESPO_ERANGE = -5      /* a size exceeds what the kernels index (see each call)     */
} espo_status;

typedef enum { ESPO_F32 = 0, ESPO_BF16 = 1 } espo_dtype;

/*
 * Parameters that stay frozen for a whole rollout batch (Section 4.2: the batch
 * statistics are only updated at the batch boundary; Algorithm 1 "Require").
 */
typedef struct {
  float mu_g;           /* EMA batch mean of the regret, Eq. normalized_gap           */
  float var_g;          /* EMA batch variance of the regret (sigma_g^2)               */
  float delta;          /* numerical stabiliser under the square root, > 0            */
  float clip_c;         /* clipping bound c >= 0 of the normalised regret             */
  float alpha_s;        /* smoothing factor of Eq. smoothed_score, in [0,1]           */
  float beta;           /* threshold multiplier of Eq. stop_rule, >= 0                */
  float eps;            /* floor on the value in Eq. stop_rule                        */
  int32_t stop_enabled; /* "warmup complete" gate of Algorithm 1; 0 = never stop      */
  int32_t eos_id;       /* token id that ends a trajectory naturally; -1 = none       */
  int32_t stop_mode;    /* which stop test, see espo_stop_mode; 0 = Eq. stop_rule      */
  float stop_threshold; /* the fixed threshold / probability of modes 1-3             */
  int32_t simulate;     /* non-zero: record the first stop step but keep decoding     */
  float top_p;          /* nucleus filter on the draw, active for 0 < top_p < 1       */
  int32_t top_k;        /* top-k filter on the draw, active for top_k > 0             */
} espo_params;

/*
 * Filtered draws.  Rollouts for training draw from the whole vocabulary (both fields 0).  The
 * evaluation set-up of Section 5 draws with a nucleus of 0.7 at temperature 1 and top-k off;
 * for that, step 2 of espo_step below draws from a kept subset of the vocabulary instead:
 *   top_p  v is kept iff the tokens with a strictly larger logit hold less than top_p of the
 *          probability mass: the most probable tokens whose mass reaches top_p, with tokens
 *          of equal logit kept or dropped together (the most probable token is always kept);
 *   top_k  v is kept iff fewer than top_k tokens have a strictly larger logit (ties at the
 *          k-th value are all kept).
 * The token is argmax (y_v + G_v) over the kept set, with the same G_v as without a filter, so
 * it is distributed as the renormalised distribution on the kept set.  regret, logprob, entropy
 * and the state update are as without a filter (logprob and entropy refer to the unfiltered
 * distribution; the regret of a kept token does not depend on the renormalisation).  At most
 * one of the two may be active (ESPO_EINVAL otherwise).  A filtered step reads the row more than
 * once (the later passes mostly from the caches) and runs as its own kernel instantiation.
 */

/*
 * Stop tests.  ESPO_STOP_RULE is the method (Eq. stop_rule); the others are the replacements
 * studied in the ablations (Section 6, variants D, E and F).  All are gated by stop_enabled
 * and all leave the update of z untouched.
 *   ESPO_STOP_VALUE_ONLY   stop iff values[b] < stop_threshold
 *   ESPO_STOP_REGRET_ONLY  stop iff z[b] > stop_threshold (after this step's update)
 *   ESPO_STOP_RANDOM       stop iff u < stop_threshold with u = u(word 0 of
 *                          Philox(counter (0, step, b, 0x53544F50), key)): a coin per row and
 *                          step that looks at neither logits nor values
 * With `simulate` set (the "ESPO/Original" bookkeeping of Section 7) a stop only writes
 * stop_step[b] = step if stop_step[b] is still negative; alive[b] stays 1 and later steps
 * keep decoding the row and updating z.  The end-of-sequence token ends the row either way.
 */
typedef enum {
  ESPO_STOP_RULE = 0,
  ESPO_STOP_VALUE_ONLY = 1,
  ESPO_STOP_REGRET_ONLY = 2,
  ESPO_STOP_RANDOM = 3
} espo_stop_mode;

/*
 * espo_step -- one decode step of Algorithm 1 for B trajectories.
 *
 * For every row b with alive[b] != 0, in one pass over logits[b, 0:V]:
 *   1. pi = softmax(x / temperature) (the distribution actually sampled);
 *      row maximum m and S = sum_v exp((x_v - m)/temperature).
 *   2. token a = argmax_v (x_v/temperature + G_v) with iid standard Gumbel G_v
 *      (Gumbel-max draw from pi; the paper only asks for a_t ~ pi).  Equal scores:
 *      lowest v wins.  Scores of contenders are formed in double precision.
 *      The variates come from Philox4x32-10 keyed by the seed and are generated
 *      top-down in blocks of 64 consecutive vocabulary indices, which has the same
 *      joint law as drawing each G_v on its own but lets a block be ruled out from
 *      one random number.  With u(w) = (2 (w >> 9) + 1) / 2^24 and
 *      key = (seed & 0xffffffff, seed >> 32):
 *        block q = v / 64 holds n_q = min(64, V - 64 q) indices;
 *        w     = word (q & 3) of Philox(counter = (q >> 2, step, b, 0x4553504F), key);
 *        M_q   = ln n_q - ln(-ln u(w))        the largest variate of the block,
 *        pos_q = (w >> 3) & 63                the index (within the block) that gets it
 *                (bits that u(w) does not use); a ragged last block (n_q < 64) takes
 *                pos_q = (w' * n_q) >> 32 with w' = word 0 of
 *                Philox(counter = (q, step, b, 0x52414747), key) instead;
 *        w_v   = word (v & 3) of Philox(counter = (v >> 2, step, b, 0x6573706F), key);
 *        G_v   = M_q                           if v = 64 q + pos_q,
 *              = -ln(exp(-M_q) - ln u(w_v))    otherwise.
 *   3. regret g = max_a log pi(a) - log pi(a_t) = (m - x_a)/temperature
 *      (Eq. step_gap), evaluated in fp32 as (m - x_a) * (1.0f/temperature).
 *   4. g~ = clip((g - mu_g) * (1.0f/sqrtf(var_g + delta)), -c, c)   (Eq. normalized_gap)
 *   5. z[b] <- fmaf(alpha_s, z[b], (1.0f - alpha_s) * g~)            (Eq. smoothed_score;
 *      the state before the first step is 0 and step 0 already updates it, as
 *      Algorithm 1 does).
 *   6. stop = stop_enabled && z[b] > beta * fmaxf(values[b], eps)   (Eq. stop_rule,
 *      strict; stop_mode selects the tests of the ablations instead, see
 *      espo_stop_mode).
 *      If stop: alive[b] = 0 and stop_step[b] = step (the trajectory keeps the token
 *      of this step and has length step + 1; Eq. failure_reward).
 *      If eos_id >= 0 and a == eos_id the row ends naturally instead: alive[b] = 0
 *      and stop_step[b] is left alone.
 *   Outputs: tokens[b] = a, regret[b] = g, logprob[b] = -g - ln S, and on request
 *   entropy[b] = -sum_v pi_v ln pi_v = ln S - sum_v pi_v (y_v - y_max), the entropy of
 *   pi(.|s_t) that the section on policy entropy and diversity tracks (Fig. 2b), taken
 *   here for the distribution the token is drawn from (temperature included); masked
 *   entries contribute 0.  It comes out of the same single pass over the row.
 * Steps 3-6 are single correctly rounded fp32 operations in exactly the order
 * written, so a host re-computation reproduces z, the mask and the stop step bit
 * for bit.
 * For rows with alive[b] == 0 the logits are not read; tokens[b] = -1,
 * regret[b] = 0, logprob[b] = 0, entropy[b] = 0, and z, alive, stop_step are left
 * untouched.
 *
 * Arguments
 *   logits      device, [B, row_stride] elements of `dt` (row-major, row b starts
 *               at element b*row_stride); only the first V of each row are read.
 *               Base address and row pitch in bytes must be multiples of 16.
 *               -inf entries are allowed (masked vocabulary); NaN and +inf are not
 *               supported (results for that row are unspecified, no fault).
 *   dt          ESPO_F32 or ESPO_BF16.
 *   B, V        rows and vocabulary size; B >= 0 (0 is a no-op), 1 <= V <= 400000
 *               (ESPO_ERANGE beyond: without a workspace the per-block bounds of a row live
 *               in the LDS of one workgroup; a filtered draw keeps one more table there and
 *               stops at about 350000 for fp32 logits).
 *   row_stride  elements between rows, >= V.
 *   temperature > 0 and finite.
 *   seed, step  key and counter word of the random stream; step >= 0.
 *   values      device, [B] fp32 critic values V_phi(s_t) of this step.
 *   params      host, read during the call.
 *   z           device, [B] fp32 in/out.
 *   alive       device, [B] uint8 in/out (1 = live).
 *   stop_step   device, [B] int32 in/out (caller initialises to -1).
 *   tokens      device, [B] int32 out.
 *   regret      device, [B] fp32 out.
 *   logprob     device, [B] fp32 out, may be NULL.  With logprob and entropy both NULL and
 *               no filter on the draw the softmax sum is not needed by anything that is
 *               left (token, regret and state take the row maximum only) and is not formed:
 *               a leaner instantiation of the kernel runs (about 8 % faster at B = 512).
 *               logprob and entropy are fp32 sums whose order of summation follows the
 *               launch layout (how many wavefronts stream a row), which the library picks
 *               from B and from whether the draw is filtered: the same row can differ in
 *               the last bits between a batch below 256 rows and a larger one, and
 *               between a filtered and a plain draw.  Tokens, regret, z, alive and
 *               stop_step do not depend on the layout.
 *   entropy     device, [B] fp32 out, may be NULL (then nothing is spent on it: the
 *               pass with the entropy does two more vector operations per logit).
 *   workspace   device scratch of at least espo_step_workspace_bytes(B, V, dt) bytes, 16-byte
 *               aligned, or NULL if that size is 0, as it is for every shape in this version:
 *               one workgroup handles a whole row and needs no scratch in device memory.
 *               (Splitting a row over several workgroups that combine through a workspace is
 *               implemented and reachable through espo_debug_step in espo_debug.h; on an
 *               MI355X it measured slower for every shape tried, so espo_step does not do it.)
 *               A workspace that is given but smaller than that size or misaligned is
 *               ESPO_EWORKSPACE.
 *   stream      hipStream_t as void*.
 */
int espo_step(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride,
              float temperature, uint64_t seed, int32_t step,
              const float* values, const espo_params* params,
              float* z, uint8_t* alive, int32_t* stop_step,
              int32_t* tokens, float* regret, float* logprob, float* entropy,
              void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace espo_step needs for this shape (0 in this version). */
size_t espo_step_workspace_bytes(int64_t B, int64_t V, espo_dtype dt);

/*
 * espo_advantages -- TD errors and GAE on truncated trajectories
 * (Section 3: delta_t and Eq. gae; Section 4.4: Eq. failure_reward, no bootstrap
 * beyond the absorbing state).
 *
 * For row b let L = min(max(lengths[b], 0), T).  With
 *   r_t = rewards[b,t] for t < L-1,
 *   r_{L-1} = stopped[b] ? r_fail : rewards[b,L-1]     (the failure reward replaces
 *                                                       whatever was stored there),
 *   V_L = 0                                             (no bootstrap past the end),
 *   td[b,t]  = r_t + gamma * values[b,t+1] - values[b,t]            for t < L,
 *   adv[b,t] = sum_{l=0}^{L-1-t} (gamma*lambda)^l td[b,t+l]          for t < L,
 * and td[b,t] = adv[b,t] = 0 for L <= t < T.  rewards and values are never read at
 * t >= L.  (The ablation without the terminal failure penalty, Section 6 variant C, is this
 * call with all `stopped` flags zero: the truncated trajectory then keeps its stored last
 * reward.)  Rows are independent and may come in any order: in a batch of more than 512 rows
 * the library itself scans the rows from the 513th on longest first (the workgroups look their
 * rows up by length; no result depends on it).
 *
 * Arguments
 *   rewards, values  device, [B, T] fp32 row-major, 16-byte aligned base; T*4 need
 *                    not be a multiple of 16.
 *   lengths          device, [B] int32 (clamped to [0, T] on the device).
 *   stopped          device, [B] uint8, non-zero = ended by the stop rule.
 *   B, T             B >= 0, T >= 0 (either 0 is a no-op); T < 2^31, B < 2^30 (ESPO_ERANGE).
 *   r_fail, gamma, lambda   scalars; gamma, lambda finite.
 *   td, adv          device, [B, T] fp32 out, 16-byte aligned base.
 *   stream           hipStream_t as void*.
 */
int espo_advantages(const float* rewards, const float* values,
                    const int32_t* lengths, const uint8_t* stopped,
                    int64_t B, int64_t T, float r_fail, float gamma, float lambda,
                    float* td, float* adv, void* stream);

/*
 * espo_advantages_terminal -- the same pass for the reward structure of Algorithm 1:
 * r_t = 0 at every step that goes on and one reward at the last step,
 *   r_{L-1} = stopped[b] ? r_fail : terminal_reward[b]       (Eq. failure_reward),
 * so no [B, T] reward array is read (4 bytes per token instead of 8).  td and adv are
 * as in espo_advantages with these rewards.  Two options for the training step that
 * follows:
 *   returns       if not NULL, returns[b,t] = adv[b,t] + values[b,t] for t < L: the
 *                 lambda-return that the critic of the (standard) PPO update regresses on.
 *   zero_padding  non-zero: td, adv (and returns) are 0 for L <= t < T, as in
 *                 espo_advantages.  Zero: positions at t >= L are not part of the result;
 *                 each is either left as it was or set to 0 (a caller that masks by
 *                 `lengths` saves the 8 to 12 bytes per padded token of the zero fill).
 * Other arguments, alignment rules and errors as for espo_advantages; terminal_reward is
 * device, [B] fp32 (read only for rows with stopped[b] == 0 and L > 0); returns, if given,
 * device [B, T] fp32 with a 16-byte aligned base.
 */
int espo_advantages_terminal(const float* values, const int32_t* lengths, const uint8_t* stopped,
                             const float* terminal_reward, int64_t B, int64_t T,
                             float r_fail, float gamma, float lambda, int32_t zero_padding,
                             float* td, float* adv, float* returns, void* stream);

/*
 * espo_advantages_packed -- the same pass for trajectories stored back to back.  Early
 * stopping makes trajectories end long before the horizon (Section 4.4: nothing is decoded
 * after T_stop), so a [B, T] layout is mostly padding; here trajectory b owns positions
 * cu_seqlens[b] .. cu_seqlens[b+1]-1 of arrays of N tokens and only those are read and
 * written: delta_t, A_t (Section 3, Eq. gae) and optionally A_t + V(s_t) over each
 * trajectory on its own, V := 0 after its last token, r_fail at the last token of a stopped
 * one (Eq. failure_reward).
 *
 * Exactly one of rewards / terminal_reward is given (ESPO_EINVAL otherwise):
 *   rewards          device, [N] fp32 in the same layout: the dense form of espo_advantages;
 *   terminal_reward  device, [B] fp32: the form of espo_advantages_terminal (zero reward
 *                    before the last token).
 * Other arguments
 *   values       device, [N] fp32.
 *   cu_seqlens   device, [B + 1] int64, non-decreasing offsets.  Each extent is clipped to
 *                [0, N] on the device and an empty or reversed one holds no token, so no
 *                content of this array leads to an access outside the arrays; extents that
 *                overlap give unspecified results in the overlap.
 *   stopped      device, [B] uint8.
 *   B, N         B >= 0, N >= 0 (either 0 is a no-op); B < 2^31 (ESPO_ERANGE), N any int64.
 *   td, adv      device, [N] fp32 out; returns device [N] fp32 out or NULL.  Positions
 *                that no trajectory owns are left as they are.
 *   All [N] arrays need 16-byte aligned bases (ESPO_EALIGN); offsets need no alignment.
 *   stream       hipStream_t as void*.
 */
int espo_advantages_packed(const float* rewards, const float* terminal_reward, const float* values,
                           const int64_t* cu_seqlens, const uint8_t* stopped, int64_t B, int64_t N,
                           float r_fail, float gamma, float lambda,
                           float* td, float* adv, float* returns, void* stream);

/*
 * espo_batch_stats -- the update at the boundary of a rollout batch: exponential moving
 * averages of the batch mean and variance of the regret (Section 4.2) and the proportional
 * controller of the threshold multiplier (Eq. beta_update).  The statistics stay frozen
 * during a rollout; this call produces the values for the next one.
 *
 * The batch is every valid token of every trajectory, regret[b, t] for
 * t < L_b = min(max(lengths[b], 0), T); entries at t >= L_b are never read.  With n = sum L_b:
 *   mean = sum g / n,   var = sum (g - mean)^2 / n     (divisor n, accumulated in double)
 *   rate = (number of rows with stopped[b] != 0) / B
 *   mu_g'  = alpha_ema * mu_g  + (1 - alpha_ema) * mean
 *   var_g' = alpha_ema * var_g + (1 - alpha_ema) * var
 *   beta'  = min(max(beta + eta_beta * (rate - target_rate), beta_min), beta_max)
 * each formed in double and rounded to float once.  With n = 0 mu_g and var_g are returned
 * unchanged; with B = 0 beta as well.  The result does not depend on scheduling (fixed
 * reduction order).
 *
 * Arguments
 *   regret      device, [B, T] fp32 row-major (the per-step `regret` outputs of espo_step laid
 *               out by trajectory), 16-byte aligned base.
 *   lengths     device, [B] int32;  stopped  device, [B] uint8.
 *   B, T        B >= 0, T >= 0.
 *   mu_g, var_g, beta   the values the finished rollout used.
 *   ctrl        host, read during the call.  alpha_ema in [0,1]; beta_min <= beta_max.
 *   out         device, one espo_batch_result, written once the stream reaches the call.
 *   workspace   device scratch of at least espo_batch_stats_workspace_bytes(B, T) bytes,
 *               8-byte aligned; contents before and after the call are irrelevant.
 *   stream      hipStream_t as void*.
 */
typedef struct {
  float alpha_ema;   /* paper: 0.99 */
  float eta_beta;    /* adjustment rate of beta, paper: 0.1 */
  float target_rate; /* target termination rate, paper: 0.25 */
  float beta_min;    /* paper: 0.0 */
  float beta_max;    /* upper clip; the paper gives no value (its initial beta is 7.0) */
} espo_batch_ctrl;

typedef struct {
  double mean_g;      /* batch mean of the regret over the valid tokens */
  double var_g_batch; /* batch variance, divisor n */
  double stop_rate;   /* fraction of trajectories ended by the stop rule */
  int64_t tokens;     /* n */
  float mu_g;         /* updated parameters for the next rollout */
  float var_g;
  float beta;
  int32_t stopped;    /* number of trajectories ended by the stop rule */
} espo_batch_result;

int espo_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped,
                     int64_t B, int64_t T, float mu_g, float var_g, float beta,
                     const espo_batch_ctrl* ctrl, espo_batch_result* out,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace espo_batch_stats needs (at most 32 KiB). */
size_t espo_batch_stats_workspace_bytes(int64_t B, int64_t T);

/*
 * espo_batch_stats_static -- espo_batch_stats for callers that cannot allocate device memory
 * (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same result, bit for bit, but the partial sums go to a 32 KiB array that
 * the library holds on every GPU it is loaded on, instead of a caller's workspace.  The call
 * allocates and frees nothing.  Every B fits that array (a launch never has more than 1024
 * partial sums of 32 bytes); the size is checked all the same and a batch that would not fit
 * returns ESPO_ERANGE with nothing enqueued, as do B or T of 2^31 or more.  ESPO_EHIP if the
 * runtime cannot give the array's address on the current device (the device that is current
 * at the call must be the one `stream` belongs to).  All calls on one GPU share the array:
 * two calls that can overlap there (different streams, or different host threads without
 * ordering between their streams) race on it; calls on one stream are ordered and safe.
 * Arguments, alignment rules and other errors as for espo_batch_stats.
 */
int espo_batch_stats_static(const float* regret, const int32_t* lengths, const uint8_t* stopped,
                            int64_t B, int64_t T, float mu_g, float var_g, float beta,
                            const espo_batch_ctrl* ctrl, espo_batch_result* out, void* stream);

/*
 * espo_whiten -- advantage whitening over the valid tokens of a batch: the normalisation
 * that PPO implementations apply to the GAE output before the clipped objective.  (The paper
 * keeps the standard PPO update, Section 3, and does not spell this step out; it belongs
 * to the training step that consumes espo_advantages' output.)  With n = sum_b L_b,
 * L_b = min(max(lengths[b], 0), T):
 *   mean = sum A / n,    var = sum (A - mean)^2 / (n - (unbiased ? 1 : 0))   (0 if that divisor is <= 0)
 *   out[b,t] = (A[b,t] - (shift_mean ? mean : 0)) / sqrt(var + eps)           for t < L_b,
 * sums in double, each element normalised in double and rounded to float once.  Positions
 * at t >= L_b are neither read nor written.  The result does not depend on scheduling
 * (fixed reduction order).  With n = 0 nothing is written to out; with var + eps = 0 (a
 * constant batch and eps = 0) every valid position of out is 0.
 *
 * Arguments
 *   adv        device, [B, T] fp32 row-major, 16-byte aligned base.  Trajectories stored
 *              back to back (espo_advantages_packed) are the case B = 1, T = N, lengths = {N}.
 *   lengths    device, [B] int32.
 *   B, T       B >= 0, T >= 0 (either 0 is a no-op); B, T and B * ceil(T / 4096) below 2^31
 *              (ESPO_ERANGE).
 *   eps        >= 0, finite (common choice: 1e-8).
 *   shift_mean, unbiased   flags as above.
 *   out        device, [B, T] fp32, 16-byte aligned base; may be the same array as adv.
 *   stats      device, 3 doubles (mean, var, n) written by the call, or NULL; 8-byte aligned.
 *   workspace  device scratch of at least espo_whiten_workspace_bytes(B, T) bytes, 8-byte
 *              aligned; contents before and after the call are irrelevant.
 *   stream     hipStream_t as void*.
 */
int espo_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps,
                int32_t shift_mean, int32_t unbiased, float* out, double* stats,
                void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace espo_whiten needs (at most 16 KiB). */
size_t espo_whiten_workspace_bytes(int64_t B, int64_t T);

/*
 * espo_advantages_ws, espo_advantages_terminal_ws, espo_whiten_from_ws, espo_length_order --
 * espo_advantages (or espo_advantages_terminal) followed by espo_whiten with less work between them (Section 3, Eq. gae; Section 4.4, Eq. failure_reward;
 * the whitening as described at espo_whiten).
 *
 * espo_advantages_ws computes exactly what espo_advantages computes (same td and adv, bit for
 * bit) and does two more things.  Every row leaves the count, sum and sum of squares of its
 * advantages in the workspace, in double about a shift of the row's own.  And the rows are
 * scanned in an order that suits their lengths instead of 0, 1, 2, ...: with the long rows
 * first, a batch of more than 512 rows of mixed lengths takes about an eighth less time, and
 * no row has to be moved for it.  If `order` is given, that is the order.  If it is NULL and
 * the batch has more than 512 rows (what the chip works on at once), the launch's first
 * workgroup sorts the rows from the 513th on by length while the first 512 are scanned in index
 * order, which gains as much as a full order does.
 *
 * espo_length_order writes such an order: the rows 0 .. B-1 by length (clamped to [0, T]) in
 * 256 classes, longest first, rows of one class in no particular order.  It is one small
 * launch, about as long as what the order then saves if it runs right before the pass; a caller
 * that knows the lengths earlier (they are final when the rollout ends) runs it then.
 *
 * espo_whiten_from_ws is espo_whiten for an `adv` that one of the two has just written,
 * with the same B, T, lengths and workspace: mean and variance are merged from the rows' sums
 * (pairwise, in a fixed order, in double) instead of by a first pass over adv, so only the
 * rewrite remains.  The two ways of summing differ by rounding: mean and variance agree with
 * espo_whiten's to about 1e-14 relative, `out` to the last bit or one unit of it.
 *
 * Arguments as for espo_advantages and espo_whiten, and
 *   order      device, [B] int32, every row once, or NULL (the launch then sorts its later rows
 *              itself, as described above).  An entry
 *              outside [0, B) is skipped; a row that is missing from the order is not computed,
 *              one that is named twice is computed twice.
 *   workspace  device, at least espo_advantages_ws_bytes(B) bytes (256, plus 32 per row, plus 4
 *              per row beyond the 512th), 16-byte aligned.  Its first 256 bytes must be zero
 *              before the first call that uses it (two words in there are how the sorting
 *              workgroup tells the others that it is done and how the last of them knows that
 *              it is the last; every call leaves them zero again); the rest may hold anything.
 *              Written by espo_advantages_ws, read by espo_whiten_from_ws.  Missing, misaligned
 *              or too small: ESPO_EWORKSPACE.  Two calls that overlap in time need a workspace each.
 * Calls on one stream are ordered; a caller that puts them on different streams orders them
 * itself.
 */
int espo_advantages_ws(const float* rewards, const float* values,
                       const int32_t* lengths, const uint8_t* stopped,
                       int64_t B, int64_t T, float r_fail, float gamma, float lambda,
                       float* td, float* adv, const int32_t* order,
                       void* workspace, size_t workspace_bytes, void* stream);

/* espo_advantages_terminal with the same two additions (same td, adv and returns, bit for bit); arguments as there and as above. */
int espo_advantages_terminal_ws(const float* values, const int32_t* lengths, const uint8_t* stopped,
                                const float* terminal_reward, int64_t B, int64_t T,
                                float r_fail, float gamma, float lambda, int32_t zero_padding,
                                float* td, float* adv, float* returns, const int32_t* order,
                                void* workspace, size_t workspace_bytes, void* stream);

int espo_whiten_from_ws(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps,
                        int32_t shift_mean, int32_t unbiased, float* out, double* stats,
                        const void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace for espo_advantages_ws and espo_whiten_from_ws (0 for B <= 0). */
size_t espo_advantages_ws_bytes(int64_t B);

/* lengths: device [B] int32; order: device [B] int32 out.  B, T >= 0 (B = 0 is a no-op), T < 2^31, B < 2^30. */
int espo_length_order(const int32_t* lengths, int64_t B, int64_t T, int32_t* order, void* stream);

/* Static, human-readable text for a status code (never NULL). */
const char* espo_strerror(int code);

/* Library version as major*10000 + minor*100 + patch. */
int espo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ESPO_H_ */
