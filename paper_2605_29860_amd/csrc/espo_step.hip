// espo_step: one decode step of ESPO rollout collection (Algorithm 1 body) on gfx950.
//
// One workgroup of 16 wavefronts owns one row.  The row is streamed exactly once
// through 16-byte nontemporal loads; a wave iteration covers one block of 512
// consecutive vocabulary indices (8 per lane), which is also the block of the random
// stream, so everything a block contributes is wave-uniform:
//   phase 1 (streaming, HBM bound): per block the maximum logit, the running softmax
//     sum against a lazily advanced reference, and an fp32 upper bound
//     ub_q >= max_v (y_v + G_v) built from the block's largest Gumbel variate M_q;
//   phase 2 (a handful of blocks): the block with the largest bound is evaluated
//     exactly in double, its best score L rules out every block with ub_q < L, the
//     few survivors are evaluated the same way, and one lane runs the scalar chain
//     regret -> normalise/clip -> smoothed state -> stop test (Eq. step_gap,
//     Eq. normalized_gap, Eq. smoothed_score, Eq. stop_rule).
// Pruning only ever discards indices that provably cannot attain the maximum, so the
// token equals the exhaustive argmax with lowest-index tie-break.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

namespace espo {
namespace {

constexpr int kStepThreads = 1024;
constexpr int kStepWaves = kStepThreads / kWave;
constexpr int kRing = 4;            // 16-byte loads kept in flight per lane
constexpr float kRescaleAt = 64.0f; // advance the softmax reference when a block tops it by 2^64

struct StepArgs {
  const void* logits;
  int64_t V, row_stride;
  int nblocks;
  float inv_tau, k2;   // 1/temperature (fp32 division) and inv_tau * log2(e)
  uint32_t key0, key1;
  int32_t step;
  const float* values;
  float mu_g, rsd, clip_c, alpha_s, oma, beta, eps;
  int32_t stop_enabled, eos_id;
  float* z;
  uint8_t* alive;
  int32_t* stop_step;
  int32_t* tokens;
  float* regret;
  float* logprob;
};

// ---------------------------------------------------------------- row access
// The raw words of a lane's 8 elements.  Kept as scalars on purpose: the ring of loads in
// flight is carried around the streaming loop, and per-word values keep that rotation in
// plain 32-bit registers.
template <int DT>
struct Raw {
  static constexpr int kWords = DT == ESPO_BF16 ? 4 : 8;
  uint32_t w[kWords];
};

constexpr uint32_t kBf16NegInfPair = 0xFF80FF80u;
constexpr uint32_t kF32NegInf = 0xFF800000u;

// Lane's 8 consecutive elements starting at e0 (a multiple of 8) of a row; elements of a
// 16-byte group that starts at or beyond V read as -inf.
template <int DT>
__device__ __forceinline__ Raw<DT> load_raw(const void* row, int64_t e0, int64_t V) {
  Raw<DT> r;
  if constexpr (DT == ESPO_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) r.w[i] = kBf16NegInfPair;
    if (e0 < V) {
      const u32x4 t = __builtin_nontemporal_load((const u32x4*)((const uint16_t*)row + e0));
      r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) r.w[i] = kF32NegInf;
    if (e0 < V) {
      const u32x4 t = __builtin_nontemporal_load((const u32x4*)((const float*)row + e0));
      r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    }
    if (e0 + 4 < V) {
      const u32x4 t = __builtin_nontemporal_load((const u32x4*)((const float*)row + e0 + 4));
      r.w[4] = t.x; r.w[5] = t.y; r.w[6] = t.z; r.w[7] = t.w;
    }
  }
  return r;
}

template <int DT>
__device__ __forceinline__ void unpack(const Raw<DT>& r, float x[8]) {
  if constexpr (DT == ESPO_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __builtin_bit_cast(float, r.w[i] << 16);
      x[2 * i + 1] = __builtin_bit_cast(float, r.w[i] & 0xFFFF0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = __builtin_bit_cast(float, r.w[i]);
  }
}

template <int DT>
__device__ __forceinline__ float load_one(const void* row, int64_t v) {
  if constexpr (DT == ESPO_BF16)
    return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)row)[v] << 16);
  else
    return ((const float*)row)[v];
}

// ---------------------------------------------------------------- exact evaluation
struct Best {
  double s;   // perturbed score y + G
  int32_t v;  // vocabulary index, -1 = none yet
  float x;    // its logit
};

__device__ __forceinline__ bool better(double s, int32_t v, const Best& b) {
  return s > b.s || (s == b.s && (uint32_t)v < (uint32_t)b.v);
}

__device__ __forceinline__ Best wave_best(Best b) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Best o;
    o.s = __shfl_xor(b.s, off);
    o.v = __shfl_xor(b.v, off);
    o.x = __shfl_xor(b.x, off);
    if (better(o.s, o.v, b)) b = o;
  }
  return b;
}

struct BlockDraw {
  double M, emM;  // largest Gumbel variate of the block and exp(-M)
  int64_t vpos;   // vocabulary index that receives it
};

__device__ __forceinline__ BlockDraw block_draw(const StepArgs& a, int row, int q) {
  const int64_t first = (int64_t)q * kDrawBlock;
  const int64_t n = (a.V - first < kDrawBlock) ? a.V - first : kDrawBlock;
  const Philox4 p = philox4x32_10((uint32_t)q, (uint32_t)a.step, (uint32_t)row, kTagBlock, a.key0, a.key1);
  BlockDraw d;
  d.M = log((double)n) - log(-log(uniform_f64(p.w[0])));
  d.emM = exp(-d.M);
  d.vpos = first + (int64_t)(((uint64_t)p.w[1] * (uint64_t)n) >> 32);
  return d;
}

// G_v of the stream definition, in double.
__device__ __forceinline__ double gumbel_at(const StepArgs& a, int row, int64_t v, const BlockDraw& d) {
  if (v == d.vpos) return d.M;
  const Philox4 p = philox4x32_10((uint32_t)(v >> 2), (uint32_t)a.step, (uint32_t)row, kTagElem, a.key0, a.key1);
  const uint32_t w = (v & 3) == 0 ? p.w[0] : (v & 3) == 1 ? p.w[1] : (v & 3) == 2 ? p.w[2] : p.w[3];
  return -log(d.emM - log(uniform_f64(w)));
}

// Exact evaluation of block q by one wave.  Only indices with y_v + M_q >= bound can beat
// a score `bound` that some index is already known to attain (G_v <= M_q), so the rest are
// skipped.  `best` is this lane's running best; the lane's bound rises as scores are found.
// Pass 0 scores each lane's largest logit (64 exact scores at once give a tight bound for
// the block), passes 1..7 take the lane's other indices in order.  One evaluation site and
// no unrolling: this code runs a few times per row and should stay small.
template <int DT>
__device__ __forceinline__ void visit_block(const StepArgs& a, const void* rowp, int row, int q, double bound, Best& best) {
  const int lane = threadIdx.x & (kWave - 1);
  const BlockDraw d = block_draw(a, row, q);
  const int64_t v0 = (int64_t)q * kDrawBlock + lane * 8;
  const double itau = (double)a.inv_tau;
  float x[8];
  unpack<DT>(load_raw<DT>(rowp, v0, a.V), x);
  float xt = kNegInf;
  int jt = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (v0 + j >= a.V) x[j] = kNegInf;
    if (x[j] > xt) { xt = x[j]; jt = j; }
  }
#pragma unroll 1
  for (int pass = 0; pass < 8; ++pass) {
    const int j = pass == 0 ? jt : (pass <= jt ? pass - 1 : pass);
    float xj = x[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) xj = (j == k) ? x[k] : xj;
    const int64_t v = v0 + j;
    const double y = (double)xj * itau;
    if (v < a.V && y + d.M >= bound) {
      const double s = y + gumbel_at(a, row, v, d);
      if (better(s, (int32_t)v, best)) best = Best{s, (int32_t)v, xj};
      bound = fmax(bound, s);
    }
    if (pass == 0) {  // share the best of the 64 lane maxima before looking at the rest
      double top = bound;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) top = fmax(top, __shfl_xor(top, off));
      bound = top;
    }
  }
}

// The scalar chain regret -> normalised, clipped regret -> smoothed state -> stop test.
// Every operation is a single correctly rounded fp32 operation in the order written
// (contraction off), so a host re-computation reproduces z and the stop decision bit for bit.
struct ChainOut {
  float g, z;
  bool stop;
};

__device__ __forceinline__ ChainOut scalar_chain(const StepArgs& a, float m, float x_a, float z_prev, float value) {
#pragma clang fp contract(off)
  const float d = m - x_a;
  const float g = d * a.inv_tau;                                    // Eq. step_gap
  const float n = (g - a.mu_g) * a.rsd;
  const float gt = fminf(fmaxf(n, -a.clip_c), a.clip_c);            // Eq. normalized_gap
  const float t = a.oma * gt;
  const float zn = __builtin_fmaf(a.alpha_s, z_prev, t);            // Eq. smoothed_score
  const float thr = a.beta * fmaxf(value, a.eps);
  return ChainOut{g, zn, a.stop_enabled && (zn > thr)};             // Eq. stop_rule (strict)
}

// ---------------------------------------------------------------- the kernel
template <int DT>
__global__ __launch_bounds__(kStepThreads) void espo_step_kernel(StepArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  if (a.alive[row] == 0) {  // done rows are not decoded (Algorithm 1, loop condition)
    if (tid == 0) {
      a.tokens[row] = -1;
      a.regret[row] = 0.0f;
      if (a.logprob) a.logprob[row] = 0.0f;
    }
    return;
  }
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nblocks = a.nblocks;

  // LDS: ub[nblocks] | surv[nblocks] | per-wave partials | scalars
  float* s_ub = (float*)smem_raw;
  int* s_surv = (int*)(s_ub + nblocks);
  double* s_best_s = (double*)(smem_raw + (((size_t)nblocks * 8 + 15) & ~(size_t)15));
  int* s_best_v = (int*)(s_best_s + kStepWaves);
  float* s_best_x = (float*)(s_best_v + kStepWaves);
  float* s_m = s_best_x + kStepWaves;
  float* s_ref = s_m + kStepWaves;
  float* s_sum = s_ref + kStepWaves;
  float* s_bound = s_sum + kStepWaves;  // [0] = score bound after the first visit
  int* s_nsurv = (int*)(s_bound + 1);

  const void* rowp = DT == ESPO_BF16 ? (const void*)((const uint16_t*)a.logits + (int64_t)row * a.row_stride)
                                     : (const void*)((const float*)a.logits + (int64_t)row * a.row_stride);

  // ------------------------------------------------------------ phase 1: stream the row
  const int nit = (nblocks + kStepWaves - 1) / kStepWaves;  // wave iteration `it` handles block it*16 + wave
  Raw<DT> ring[kRing];
#pragma unroll
  for (int d = 0; d < kRing; ++d) {
    const int q = d * kStepWaves + wave;
    ring[d] = load_raw<DT>(rowp, (d < nit && q < nblocks) ? (int64_t)q * kDrawBlock + lane * 8 : a.V, a.V);
  }
  if (tid == 0) *s_nsurv = 0;

  // Softmax sum against a lazily advanced, wave-uniform reference: the lane accumulates
  // sum_v 2^(x_v k2 + nrk) with nrk = -(reference logit) * k2; the final combine multiplies
  // by 2^-(m k2 + nrk), so the rounding of nrk itself cancels.
  float nrk = 1e30f;
  float sum = 0.0f;            // lane's share of sum_v 2^(x_v k2 + nrk)
  float m_w = kNegInf;         // wave's running maximum logit
  float gub = 0.0f;            // lane i: Gumbel bound of the block of iteration (chunk + i)

  for (int it0 = 0; it0 < nit; it0 += kRing) {
#pragma unroll
    for (int d = 0; d < kRing; ++d) {
      const int it = it0 + d;
      if (it >= nit) break;
      if ((it & (kWave - 1)) == 0) {  // bounds for the next 64 iterations, one block per lane
        const int ql = (it + lane) * kStepWaves + wave;
        if (ql < nblocks) {
          const Philox4 p = philox4x32_10((uint32_t)ql, (uint32_t)a.step, (uint32_t)row, kTagBlock, a.key0, a.key1);
          gub = gumbel_upper_f32(p.w[0]);
        }
      }
      const int q = it * kStepWaves + wave;
      float x[8];
      unpack<DT>(ring[d], x);
      {  // refill this ring slot
        const int qn = q + kRing * kStepWaves;
        ring[d] = load_raw<DT>(rowp, (it + kRing < nit && qn < nblocks) ? (int64_t)qn * kDrawBlock + lane * 8 : a.V, a.V);
      }
      if (q >= nblocks) continue;  // wave-uniform
      const int64_t first = (int64_t)q * kDrawBlock;
      const int64_t nq = (a.V - first < kDrawBlock) ? a.V - first : kDrawBlock;
      if (nq < kDrawBlock) {  // ragged last block: indices at or beyond V do not exist
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (lane * 8 + j >= nq) x[j] = kNegInf;
      }
      const float gm = fmaxf(fmaxf(__builtin_fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                             fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      const float bm = wave_max(gm);  // block maximum, wave-uniform
      m_w = fmaxf(m_w, bm);
      if (fmaf(bm, a.k2, nrk) > kRescaleAt) {  // wave-uniform: move the reference up to bm
        const float nrk_new = -bm * a.k2;
        sum *= __builtin_amdgcn_exp2f(nrk_new - nrk);
        nrk = nrk_new;
      }
      float acc0 = 0.0f, acc1 = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        acc0 += __builtin_amdgcn_exp2f(fmaf(x[j], a.k2, nrk));
        acc1 += __builtin_amdgcn_exp2f(fmaf(x[j + 1], a.k2, nrk));
      }
      sum += acc0 + acc1;
      // upper bound of every perturbed score in the block: y_max + M_q, rounded up
      const float g_q = uniform_f32(gub, it & (kWave - 1));
      const float lnn = __builtin_amdgcn_logf((float)nq) * kLn2 + 2e-6f;
      const float ym = bm * a.inv_tau;
      const float ub = ym + (lnn + g_q) + (1e-5f + 4e-7f * (fabsf(ym) + fabsf(g_q) + lnn));
      if (lane == 0) s_ub[q] = ub;
    }
  }
  {
    const float tot = wave_sum(sum);
    if (lane == 0) {
      s_m[wave] = m_w;
      s_ref[wave] = nrk;
      s_sum[wave] = tot;
    }
  }
  __syncthreads();

  // ------------------------------------------------------------ phase 2: exact argmax
  // block with the largest bound (lowest index among equals); every wave finds it alone
  float ubx = kNegInf;
  int qx = 0x7fffffff;
  for (int q = lane; q < nblocks; q += kWave) {
    const float u = s_ub[q];
    if (u > ubx) { ubx = u; qx = q; }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float ou = __shfl_xor(ubx, off);
    const int oq = __shfl_xor(qx, off);
    if (ou > ubx || (ou == ubx && oq < qx)) { ubx = ou; qx = oq; }
  }
  const int qstar = qx;

  // Round 0: wave 0 evaluates the block with the largest bound; its best score rules out
  // every block whose bound is lower.  Round 1: the survivors, dealt round-robin to the waves.
  Best best{-__builtin_huge_val(), -1, 0.0f};
  double bound = -__builtin_huge_val();
#pragma unroll 1
  for (int round = 0; round < 2; ++round) {
    const int count = round == 0 ? 1 : *s_nsurv;
    const int stride = round == 0 ? 1 : kStepWaves;
#pragma unroll 1
    for (int k = (round == 0 && wave != 0) ? 1 : (round == 0 ? 0 : wave); k < count; k += stride) {
      visit_block<DT>(a, rowp, row, round == 0 ? qstar : s_surv[k], bound, best);
      double top = best.s;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) top = fmax(top, __shfl_xor(top, off));
      bound = fmax(bound, top);
    }
    if (round == 0) {
      if (tid == 0) {
        float lf = (float)bound;  // round the shared bound down so that it never overshoots
        if ((double)lf > bound) lf = __builtin_bit_cast(float, __builtin_bit_cast(int32_t, lf) + (lf > 0.0f ? -1 : 1));
        if (lf == 0.0f && bound < 0.0) lf = -1e-37f;
        s_bound[0] = lf;
      }
      __syncthreads();
      const float bound_f = s_bound[0];
      for (int q = tid; q < nblocks; q += kStepThreads)
        if (q != qstar && s_ub[q] >= bound_f) s_surv[atomicAdd(s_nsurv, 1)] = q;
      __syncthreads();
      bound = fmax(bound, (double)bound_f);
    }
  }
  best = wave_best(best);
  if (lane == 0) {
    s_best_s[wave] = best.s;
    s_best_v[wave] = best.v;
    s_best_x[wave] = best.x;
  }
  __syncthreads();

  // ------------------------------------------------------------ finalize: one lane
  if (tid == 0) {
    Best win{s_best_s[0], s_best_v[0], s_best_x[0]};
    float m = s_m[0];
    for (int w = 1; w < kStepWaves; ++w) {
      if (s_best_v[w] >= 0 && better(s_best_s[w], s_best_v[w], win)) win = Best{s_best_s[w], s_best_v[w], s_best_x[w]};
      m = fmaxf(m, s_m[w]);
    }
    float S = 0.0f;  // sum_v exp((x_v - m)/tau), waves combined in a fixed order
    for (int w = 0; w < kStepWaves; ++w)
      if (s_sum[w] > 0.0f) S += s_sum[w] * __builtin_amdgcn_exp2f(-fmaf(m, a.k2, s_ref[w]));
    int32_t tok = win.v;
    float x_a = win.x;
    if (tok < 0) { tok = 0; x_a = load_one<DT>(rowp, 0); }  // row of -inf only: unspecified, stay in range

    const ChainOut c = scalar_chain(a, m, x_a, a.z[row], a.values[row]);
    const float g = c.g, zn = c.z;
    const bool stop = c.stop;
    a.tokens[row] = tok;
    a.regret[row] = g;
    a.z[row] = zn;
    if (a.logprob) a.logprob[row] = -g - logf(S);
    if (a.eos_id >= 0 && tok == a.eos_id) {
      a.alive[row] = 0;  // natural end
    } else if (stop) {
      a.alive[row] = 0;  // absorbing failure (Eq. failure_reward): the trajectory ends here
      a.stop_step[row] = a.step;
    }
  }
}

size_t step_lds_bytes(int nblocks) { return (((size_t)nblocks * 8 + 15) & ~(size_t)15) + kStepWaves * 32 + 16; }

}  // namespace

int launch_step(const void* logits, int dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const espo_params& p, float* z,
                uint8_t* alive, int32_t* stop_step, int32_t* tokens, float* regret, float* logprob,
                hipStream_t stream) {
  StepArgs a;
  a.logits = logits;
  a.V = V;
  a.row_stride = row_stride;
  a.nblocks = (int)((V + kDrawBlock - 1) / kDrawBlock);
  a.inv_tau = 1.0f / temperature;
  a.k2 = a.inv_tau * kLog2e;
  a.key0 = (uint32_t)(seed & 0xffffffffu);
  a.key1 = (uint32_t)(seed >> 32);
  a.step = step;
  a.values = values;
  a.mu_g = p.mu_g;
  a.rsd = 1.0f / sqrtf(p.var_g + p.delta);
  a.clip_c = p.clip_c;
  a.alpha_s = p.alpha_s;
  a.oma = 1.0f - p.alpha_s;
  a.beta = p.beta;
  a.eps = p.eps;
  a.stop_enabled = p.stop_enabled;
  a.eos_id = p.eos_id;
  a.z = z;
  a.alive = alive;
  a.stop_step = stop_step;
  a.tokens = tokens;
  a.regret = regret;
  a.logprob = logprob;
  const size_t lds = step_lds_bytes(a.nblocks);
  if (lds > kMaxStepLds) return ESPO_ERANGE;
  const dim3 grid((unsigned)B), block(kStepThreads);
  if (dt == ESPO_BF16)
    hipLaunchKernelGGL(espo_step_kernel<ESPO_BF16>, grid, block, lds, stream, a);
  else
    hipLaunchKernelGGL(espo_step_kernel<ESPO_F32>, grid, block, lds, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
