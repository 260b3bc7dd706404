// espo_step: one decode step of ESPO rollout collection (Algorithm 1 body) on gfx950.
//
// One workgroup of 16 wavefronts owns one row.  The row is streamed exactly once through
// 16-byte nontemporal loads; a wave iteration covers a tile of 512 consecutive vocabulary
// indices, 8 per lane, so that each aligned group of 8 lanes holds exactly one 64-index
// block of the random stream.
//   phase 1 (streaming, HBM bound): per lane the running maximum and the softmax sum
//     against a lazily advanced per-lane reference; per block the maximum logit (three
//     DPP steps) and an fp32 upper bound ub_q >= max_v (y_v + G_v) built from the block's
//     largest Gumbel variate M_q, kept in LDS.
//   phase 2 (a handful of blocks): the blocks with the largest bounds are evaluated
//     exactly in double, their best score L rules out every block with ub_q < L, the few
//     survivors are evaluated the same way, and one lane runs the scalar chain regret ->
//     normalise/clip -> smoothed state -> stop test (Eq. step_gap, Eq. normalized_gap,
//     Eq. smoothed_score, Eq. stop_rule).
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
constexpr int kTile = 512;                        // indices per wave iteration
constexpr int kGroups = kTile / kDrawBlock;       // draw blocks per tile = lane groups per wave
constexpr int kRing = 4;                          // 16-byte loads kept in flight per lane
constexpr float kRescaleAt = 64.0f;               // advance a lane's softmax reference when topped by 2^64

struct StepArgs {
  const void* logits;
  int64_t V, row_stride;
  int ntiles, nblocks;
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

// Exact evaluation of up to 8 blocks by one wave: lane group g (8 lanes x 8 indices) takes
// block q (q < 0: the group idles).  Only indices with y_v + M_q >= bound can beat a score
// `bound` that some index is already known to attain (G_v <= M_q), so the rest are skipped.
// `best` is the lane's running best; the lane's bound rises as scores are found.  Pass 0
// scores each lane's largest logit and shares the best of the group's 8 scores, passes 1..7
// take the lane's other indices in order.  One evaluation site and no unrolling: this code
// runs a few times per row and should stay small.
template <int DT>
__device__ __forceinline__ void visit_blocks(const StepArgs& a, const void* rowp, int row, int q, double bound, Best& best) {
  const int lane = threadIdx.x & (kWave - 1);
  const bool active = q >= 0;
  const BlockDraw d = block_draw(a, row, active ? q : 0);
  const int64_t v0 = active ? (int64_t)q * kDrawBlock + (lane & 7) * 8 : a.V;
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
    if (xj > kNegInf && y + d.M >= bound) {   // masked (-inf) entries never win
      const double s = y + gumbel_at(a, row, v, d);
      if (better(s, (int32_t)v, best)) best = Best{s, (int32_t)v, xj};
      bound = fmax(bound, s);
    }
    if (pass == 0) {  // share the best of the group's 8 lane maxima before looking at the rest
      double top = bound;
#pragma unroll
      for (int off = 4; off >= 1; off >>= 1) top = fmax(top, __shfl_xor(top, off));
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
  const int grp = lane >> 3;
  const int ntiles = a.ntiles;
  const int nslots = ntiles * kGroups;  // block slots incl. the non-existent ones of the last tile

  // LDS: ub[nslots] | surv[nslots] | per-wave partials | scalars
  float* s_ub = (float*)smem_raw;
  int* s_surv = (int*)(s_ub + nslots);
  double* s_best_s = (double*)(smem_raw + (((size_t)nslots * 8 + 15) & ~(size_t)15));
  int* s_best_v = (int*)(s_best_s + kStepWaves);
  float* s_best_x = (float*)(s_best_v + kStepWaves);
  float* s_m = s_best_x + kStepWaves;
  float* s_sum = s_m + kStepWaves;
  float* s_top_ub = s_sum + kStepWaves;            // [16 waves][8 groups]: largest bound seen
  int* s_top_q = (int*)(s_top_ub + kStepWaves * kGroups);
  float* s_bound = (float*)(s_top_q + kStepWaves * kGroups);
  int* s_nsurv = (int*)(s_bound + 1);

  const void* rowp = DT == ESPO_BF16 ? (const void*)((const uint16_t*)a.logits + (int64_t)row * a.row_stride)
                                     : (const void*)((const float*)a.logits + (int64_t)row * a.row_stride);

  // ------------------------------------------------------------ phase 1: stream the row
  const int nit = (ntiles + kStepWaves - 1) / kStepWaves;  // wave iteration `it` handles tile it*16 + wave
  Raw<DT> ring[kRing];
#pragma unroll
  for (int d = 0; d < kRing; ++d) {
    const int t = d * kStepWaves + wave;
    ring[d] = load_raw<DT>(rowp, (d < nit && t < ntiles) ? (int64_t)t * kTile + lane * 8 : a.V, a.V);
  }
  // While the first loads are in flight: M_q bounds of all blocks, one Philox call each.
  for (int b = tid; b < nslots; b += kStepThreads) {
    float mub = kNegInf;
    if (b < a.nblocks) {
      const int64_t n = a.V - (int64_t)b * kDrawBlock < kDrawBlock ? a.V - (int64_t)b * kDrawBlock : kDrawBlock;
      const Philox4 p = philox4x32_10((uint32_t)b, (uint32_t)a.step, (uint32_t)row, kTagBlock, a.key0, a.key1);
      mub = (__builtin_amdgcn_logf((float)n) * kLn2 + 2e-6f) + gumbel_upper_f32(p.w[0]);
    }
    s_ub[b] = mub;
  }
  if (tid == 0) *s_nsurv = 0;
  __syncthreads();

  // Softmax sum against a lazily advanced per-lane reference: the lane accumulates
  // sum_v 2^(x_v k2 + nrk) with nrk = -(reference logit) * k2; the final combine multiplies
  // by 2^-(m k2 + nrk), so the rounding of nrk itself cancels.
  float nrk = 1e30f;
  float sum = 0.0f;
  float m_l = kNegInf;       // lane's running maximum logit
  float top_ub = kNegInf;    // largest block bound this lane group has produced, and its block
  int top_q = -1;

  for (int it0 = 0; it0 < nit; it0 += kRing) {
#pragma unroll
    for (int d = 0; d < kRing; ++d) {
      const int it = it0 + d;
      if (it >= nit) break;
      const int t = it * kStepWaves + wave;
      float x[8];
      unpack<DT>(ring[d], x);
      {  // refill this ring slot
        const int tn = t + kRing * kStepWaves;
        ring[d] = load_raw<DT>(rowp, (it + kRing < nit && tn < ntiles) ? (int64_t)tn * kTile + lane * 8 : a.V, a.V);
      }
      if (t >= ntiles) continue;  // wave-uniform
      const int64_t e0 = (int64_t)t * kTile + lane * 8;
      if ((int64_t)(t + 1) * kTile > a.V) {  // ragged last tile: indices at or beyond V do not exist
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (e0 + j >= a.V) x[j] = kNegInf;
      }
      const float gm = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      m_l = fmaxf(m_l, gm);
      if (fmaf(gm, a.k2, nrk) > kRescaleAt) {  // rare: move this lane's reference up to gm
        const float nrk_new = -gm * a.k2;
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
      // upper bound of every perturbed score in the lane group's block: y_max + M_q, rounded up
      const float bm = group8_max(gm);
      const int q = t * kGroups + grp;
      const float mub = s_ub[q];
      const float ym = bm * a.inv_tau;
      const float ub = ym + mub + (1e-5f + 4e-7f * (fminf(fabsf(ym), 1e30f) + fabsf(mub)));
      s_ub[q] = ub;  // the 8 lanes of the group store the same value
      if (ub > top_ub) { top_ub = ub; top_q = q; }
    }
  }
  {
    const float m_w = wave_max(m_l);
    if (lane == 0) s_m[wave] = m_w;
    if ((lane & 7) == 0) {
      s_top_ub[wave * kGroups + grp] = top_ub;
      s_top_q[wave * kGroups + grp] = top_q;
    }
  }
  __syncthreads();
  float m = s_m[0];  // row maximum
#pragma unroll
  for (int w = 1; w < kStepWaves; ++w) m = fmaxf(m, s_m[w]);
  {
    const float part = sum > 0.0f ? sum * __builtin_amdgcn_exp2f(-fmaf(m, a.k2, nrk)) : 0.0f;
    const float tot = wave_sum(part);
    if (lane == 0) s_sum[wave] = tot;
  }

  // ------------------------------------------------------------ phase 2: exact argmax
  // Round 0: wave 0 evaluates eight strong blocks at once (lane group g takes the best block
  // that any wave's group g has seen; the block with the largest bound overall is among
  // them).  Their best score rules out every block whose bound is lower.  Round 1: the
  // survivors, eight per wave visit.
  Best best{-__builtin_huge_val(), -1, 0.0f};
  double bound = -__builtin_huge_val();
  if (wave == 0) {
    const int j = lane & 7;
    float u0 = s_top_ub[j * kGroups + grp], u1 = s_top_ub[(j + 8) * kGroups + grp];
    int q0 = s_top_q[j * kGroups + grp], q1 = s_top_q[(j + 8) * kGroups + grp];
    if (u1 > u0 || (u1 == u0 && (uint32_t)q1 < (uint32_t)q0)) { u0 = u1; q0 = q1; }
#pragma unroll
    for (int off = 4; off >= 1; off >>= 1) {
      const float ou = __shfl_xor(u0, off);
      const int oq = __shfl_xor(q0, off);
      if (ou > u0 || (ou == u0 && (uint32_t)oq < (uint32_t)q0)) { u0 = ou; q0 = oq; }
    }
    visit_blocks<DT>(a, rowp, row, q0, bound, best);
    double top = best.s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) top = fmax(top, __shfl_xor(top, off));
    bound = top;
    if (q0 >= 0 && j == 0) s_ub[q0] = kNegInf;  // visited: keep it off the survivor list
    if (lane == 0) {
      float lf = (float)bound;  // round the shared bound down so that it never overshoots
      if ((double)lf > bound) lf = __builtin_bit_cast(float, __builtin_bit_cast(int32_t, lf) + (lf > 0.0f ? -1 : 1));
      if (lf == 0.0f && bound < 0.0) lf = -1e-37f;
      s_bound[0] = lf;
    }
  }
  __syncthreads();
  const float bound_f = s_bound[0];
  for (int q = tid; q < nslots; q += kStepThreads) {
    const float u = s_ub[q];
    if (u > kNegInf && u >= bound_f) s_surv[atomicAdd(s_nsurv, 1)] = q;
  }
  __syncthreads();
  const int nsurv = *s_nsurv;
  bound = fmax(bound, (double)bound_f);
#pragma unroll 1
  for (int k0 = wave * kGroups; k0 < nsurv; k0 += kStepWaves * kGroups) {
    visit_blocks<DT>(a, rowp, row, (k0 + grp < nsurv) ? s_surv[k0 + grp] : -1, bound, best);
    double top = best.s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) top = fmax(top, __shfl_xor(top, off));
    bound = fmax(bound, top);
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
    for (int w = 1; w < kStepWaves; ++w)
      if (s_best_v[w] >= 0 && better(s_best_s[w], s_best_v[w], win)) win = Best{s_best_s[w], s_best_v[w], s_best_x[w]};
    float S = 0.0f;  // sum_v exp((x_v - m)/tau), waves combined in a fixed order
    for (int w = 0; w < kStepWaves; ++w) S += s_sum[w];
    int32_t tok = win.v;
    float x_a = win.x;
    if (tok < 0) { tok = 0; x_a = load_one<DT>(rowp, 0); }  // row of -inf only: unspecified, stay in range

    const ChainOut c = scalar_chain(a, m, x_a, a.z[row], a.values[row]);
    a.tokens[row] = tok;
    a.regret[row] = c.g;
    a.z[row] = c.z;
    if (a.logprob) a.logprob[row] = -c.g - logf(S);
    if (a.eos_id >= 0 && tok == a.eos_id) {
      a.alive[row] = 0;  // natural end
    } else if (c.stop) {
      a.alive[row] = 0;  // absorbing failure (Eq. failure_reward): the trajectory ends here
      a.stop_step[row] = a.step;
    }
  }
}

size_t step_lds_bytes(int ntiles) {
  return (((size_t)ntiles * kGroups * 8 + 15) & ~(size_t)15) + kStepWaves * (8 + 4 + 4 + 4 + 4) + kStepWaves * kGroups * 8 + 16;
}

}  // namespace

int launch_step(const void* logits, int dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const espo_params& p, float* z,
                uint8_t* alive, int32_t* stop_step, int32_t* tokens, float* regret, float* logprob,
                hipStream_t stream) {
  StepArgs a;
  a.logits = logits;
  a.V = V;
  a.row_stride = row_stride;
  a.ntiles = (int)((V + kTile - 1) / kTile);
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
  const size_t lds = step_lds_bytes(a.ntiles);
  if (lds > kMaxStepLds) return ESPO_ERANGE;
  const dim3 grid((unsigned)B), block(kStepThreads);
  if (dt == ESPO_BF16)
    hipLaunchKernelGGL(espo_step_kernel<ESPO_BF16>, grid, block, lds, stream, a);
  else
    hipLaunchKernelGGL(espo_step_kernel<ESPO_F32>, grid, block, lds, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
