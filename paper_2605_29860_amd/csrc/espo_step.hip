// espo_step: one decode step of ESPO rollout collection (Algorithm 1 body) on gfx950.
//
// One workgroup of 16 wavefronts owns one row.  The row is streamed exactly once through
// 16-byte nontemporal loads; a wave iteration covers a tile of 512 consecutive vocabulary
// indices, 8 per lane, so that each aligned group of 8 lanes holds exactly one 64-index
// block of the random stream.
//   phase 1 (streaming, HBM bound): per lane the running maximum and the softmax sum
//     against a lazily advanced per-lane reference; per block the maximum logit (three
//     DPP steps) and an fp32 upper bound ub_q >= max_v (y_v + G_v) built from the block's
//     largest Gumbel variate M_q, kept in LDS.  Each lane group also keeps the raw data of
//     the block with the largest bound it has seen, so that phase 2 seldom re-reads memory.
//   phase 2 (a handful of blocks, lanes = the 64 indices of a block): every wave scores the
//     block with the largest bound it has streamed, the best score found rules out every
//     block with a lower bound, the few survivors are scored by the waves in parallel (a long
//     list is first reduced to the indices whose own bound y_v + M_q still reaches the score
//     attained, and those are scored one per thread).  Scores are first formed in fp32 with a
//     proven error margin; if the best two cannot be told apart within that margin, the
//     indices that reach the fp32 winner's lower end are scored again in double, which
//     decides exactly.
//   One lane then runs the scalar chain regret -> normalise/clip -> smoothed state -> stop
//   test (Eq. step_gap, Eq. normalized_gap, Eq. smoothed_score, Eq. stop_rule).
// Pruning only ever discards indices that provably cannot attain the maximum, so the
// token equals the exhaustive double-precision argmax with lowest-index tie-break.
//
// Two optional features are template parameters, so that the plain step pays nothing for them:
// the entropy of the sampling distribution (one more accumulator in phase 1) and filtered
// draws (top-p / top-k: a table of block maxima in phase 1, and after phase 2 the search for
// the edge of the kept set, see the comment at `if constexpr (Filter)`).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

namespace espo {
namespace {

// A workgroup has W wavefronts (a template parameter of everything below that depends on it): 16 when
// one workgroup owns a whole row, 4 when a row is split into chunks that several workgroups stream.
constexpr int kTile = 512;                        // indices per wave iteration
constexpr int kGroups = kTile / kDrawBlock;       // draw blocks per tile = lane groups per wave
constexpr int kMaxChunks = 64;                    // a row is split over at most this many workgroups (one lane each in the combine)
constexpr int kRing = 4;                          // 16-byte loads kept in flight per lane
constexpr int kCandCap = 1024;                    // candidate indices kept for a row with a long survivor list
constexpr float kRescaleAt = 64.0f;               // advance a lane's softmax reference when topped by 2^64

// What the workgroup of one chunk hands to the combine: the chunk's largest logit, its softmax
// sums relative to that logit, and its exact local winner (score known to within +-e).
struct __attribute__((aligned(16))) ChunkResult {
  float m, sum, sumw, s;
  float e, x;
  int32_t v;
  int32_t pad;
};

struct StepArgs {
  const void* logits;
  int64_t row_stride;
  int32_t V, ntiles, nblocks;
  float inv_tau, k2;   // 1/temperature (fp32 division) and inv_tau * log2(e)
  float ref_lead;      // a lane's softmax reference is advanced once a logit tops it by this much (2^64 in the sum)
  float margin_scale;  // scales the fp32 score margin (1 in production)
  uint32_t key0, key1;
  int32_t step;
  const float* values;
  float mu_g, rsd, clip_c, alpha_s, oma, beta, eps;
  int32_t stop_enabled, eos_id, stop_mode, simulate;
  float stop_threshold;
  float top_p;    // nucleus filter on the draw, active for 0 < top_p < 1
  int32_t top_k;  // top-k filter on the draw, active for top_k > 0
  float* z;
  uint8_t* alive;
  int32_t* stop_step;
  int32_t* tokens;
  float* regret;
  float* logprob;
  float* entropy;
  // a row split over `nch` workgroups: workgroup row * nch + c streams tiles [c ntiles / nch, (c + 1) ntiles / nch)
  int32_t nch;
  ChunkResult* partials;         // [B * nch] what each chunk found, combined by the last one of a row to arrive
  uint32_t* tickets;             // [B] arrivals per row; zero before the launch and again after it
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

template <int DT>
constexpr int elem_bytes() { return DT == ESPO_BF16 ? 2 : 4; }

// The lane's 8 consecutive elements starting at element e0 (a multiple of 8, e0 < V).  The row
// pitch is a multiple of 4 floats only, so the second half of an fp32 group is read from the
// row's last group of four if it would start at or beyond V (those elements are masked later).
template <int DT>
__device__ __forceinline__ Raw<DT> load_raw(const void* row, uint32_t e0, uint32_t V) {
  Raw<DT> r;
  const char* p = (const char*)row + (size_t)(e0 * (uint32_t)elem_bytes<DT>());
  const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
  r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
  if constexpr (DT == ESPO_F32) {
    const uint32_t last4 = (V - 1u) & ~3u;
    const uint32_t e1 = e0 + 4u < last4 ? e0 + 4u : last4;
    const u32x4 u = __builtin_nontemporal_load((const u32x4*)((const char*)row + (size_t)(e1 * 4u)));
    r.w[4] = u.x; r.w[5] = u.y; r.w[6] = u.z; r.w[7] = u.w;
  }
  return r;
}

// The same for a tile that lies wholly inside the row: `tile` is the tile's first element
// (wave-uniform, so the address stays a scalar base plus a constant lane offset).
template <int DT>
__device__ __forceinline__ Raw<DT> load_raw_inner(const void* tile, uint32_t lane_bytes) {
  Raw<DT> r;
  const char* p = (const char*)tile + lane_bytes;
  const u32x4 t = __builtin_nontemporal_load((const u32x4*)p);
  r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
  if constexpr (DT == ESPO_F32) {
    const u32x4 u = __builtin_nontemporal_load((const u32x4*)(p + 16));
    r.w[4] = u.x; r.w[5] = u.y; r.w[6] = u.z; r.w[7] = u.w;
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
__device__ __forceinline__ float elem_at(const void* base, int64_t idx) {
  if constexpr (DT == ESPO_BF16)
    return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)base)[idx] << 16);
  else
    return ((const float*)base)[idx];
}

// ---------------------------------------------------------------- scores
// A candidate for the argmax: score s = y + G known to within +-e, its index and logit.
template <typename F>
struct Cand {
  F s;
  float e;
  int32_t v;
  float x;
};

// Running state of the search: the best candidate and `hi2`, the largest upper end s + e
// among all other scored indices.  The winner is certain iff best.s - best.e > hi2.
template <typename F>
struct Search {
  Cand<F> best;
  F hi2;
  __device__ __forceinline__ void init() {
    best = Cand<F>{(F)-__builtin_huge_val(), 0.0f, -1, 0.0f};
    hi2 = (F)-__builtin_huge_val();
  }
  __device__ __forceinline__ void offer(const Cand<F>& c) {
    if (c.v < 0 || c.v == best.v) return;  // nothing, or the element that already leads
    if (c.s > best.s || (c.s == best.s && (uint32_t)c.v < (uint32_t)best.v)) {
      if (best.v >= 0) hi2 = hi2 > best.s + (F)best.e ? hi2 : best.s + (F)best.e;
      best = c;
    } else {
      hi2 = hi2 > c.s + (F)c.e ? hi2 : c.s + (F)c.e;
    }
  }
  __device__ __forceinline__ void merge(const Search& o) {
    hi2 = hi2 > o.hi2 ? hi2 : o.hi2;
    offer(o.best);
  }
  __device__ __forceinline__ F lower() const { return best.v >= 0 ? best.s - (F)best.e : (F)-__builtin_huge_val(); }
};

template <typename F>
__device__ __forceinline__ Search<F> wave_merge(Search<F> s) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    Search<F> o;
    o.best.s = __shfl_xor(s.best.s, off);
    o.best.e = __shfl_xor(s.best.e, off);
    o.best.v = __shfl_xor(s.best.v, off);
    o.best.x = __shfl_xor(s.best.x, off);
    o.hi2 = __shfl_xor(s.hi2, off);
    s.merge(o);
  }
  return s;
}

// -ln u(word) in the working precision.  fp32: |ln u| >= ln 2 for u < 1/2, and log1p keeps
// full relative accuracy for u >= 1/2 (1 - u is exact in fp32).
template <typename F>
__device__ __forceinline__ F neg_log_uniform(uint32_t word);
template <>
__device__ __forceinline__ double neg_log_uniform<double>(uint32_t word) { return -log(uniform_f64(word)); }
template <>
__device__ __forceinline__ float neg_log_uniform<float>(uint32_t word) {
  return -__builtin_amdgcn_logf((float)(2u * (word >> 9) + 1u) * (1.0f / 16777216.0f)) * kLn2;
}
// fp32 ln and exp from the hardware log2 / exp2.  Measured over all inputs that occur here
// (every positive float in [2^-26, 64) for ln, every u(w); [-40, 8] for exp): relative error
// below 1.7e-7 for ln, also next to 1, and below 2e-6 for exp; a GPU test re-measures this.
__device__ __forceinline__ float flog(float x) { return __builtin_amdgcn_logf(x) * kLn2; }
__device__ __forceinline__ double flog(double x) { return log(x); }
__device__ __forceinline__ float fexp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ double fexp(double x) { return exp(x); }

// Error margin of an fp32 score y + G.  With ln accurate to 1.7e-7 and exp to 2e-6 (relative):
// -ln u carries 1.7e-7, M_q = ln n - ln(-ln u) at most 5e-6 for |M_q| <= 25, exp(-M_q) at most
// 7e-6 relative (4e-7 where it is formed as (-ln u)/n), G = -ln(exp(-M_q) - ln u) at most
// 1.1e-5, and the product and sum forming y + G add 2^-23 (|y| + |G|).  The margin below is
// more than three times that.
__device__ __forceinline__ float score_margin(const StepArgs& a, float y) {
  return a.margin_scale * (4e-5f + 2.5e-7f * fabsf(y));
}

// The block-level part of the draw for block q: its largest variate M_q, exp(-M_q), and the
// index that receives M_q.
template <typename F>
struct BlockDraw {
  F M, emM;
  int32_t vpos;
};

template <typename F>
__device__ __forceinline__ BlockDraw<F> block_draw(const StepArgs& a, int row, int q) {
  const int32_t first = q * kDrawBlock;
  const int32_t n = a.V - first < kDrawBlock ? a.V - first : kDrawBlock;
  const Philox4 pb = philox4x32_10((uint32_t)(q >> 2), (uint32_t)a.step, (uint32_t)row, kTagBlock, a.key0, a.key1);
  const uint32_t wb = (q & 3) == 0 ? pb.w[0] : (q & 3) == 1 ? pb.w[1] : (q & 3) == 2 ? pb.w[2] : pb.w[3];
  BlockDraw<F> d;
  d.M = flog((F)n) - flog(neg_log_uniform<F>(wb));
  d.emM = fexp(-d.M);
  d.vpos = first + (int32_t)((wb >> 3) & 63u);
  if (n < kDrawBlock) {  // ragged last block: own position draw
    const Philox4 pr = philox4x32_10((uint32_t)q, (uint32_t)a.step, (uint32_t)row, kTagRagged, a.key0, a.key1);
    d.vpos = first + (int32_t)(((uint64_t)pr.w[0] * (uint64_t)n) >> 32);
  }
  return d;
}

// Scores index v (logit x) of a block with draw d and offers it to the search, unless its
// upper bound y + M_q (+ margins) cannot reach `bound`, a score already known to be attained,
// or its logit is not above `floor` (-inf: only masked entries are left out).
template <typename F>
__device__ __forceinline__ void score_index(const StepArgs& a, int row, int32_t v, float x, const BlockDraw<F>& d,
                                            F bound, float floor, Search<F>& st) {
  const F y = (F)x * (F)a.inv_tau;
  const float e = sizeof(F) == 4 ? score_margin(a, (float)y) : 0.0f;
  if (x > floor && (y + d.M) + (F)(2.0f * e) >= bound) {   // masked (-inf) and filtered entries never win
    F G = d.M;
    if (v != d.vpos) {
      const Philox4 p = philox4x32_10((uint32_t)(v >> 2), (uint32_t)a.step, (uint32_t)row, kTagElem, a.key0, a.key1);
      const uint32_t w = (v & 3) == 0 ? p.w[0] : (v & 3) == 1 ? p.w[1] : (v & 3) == 2 ? p.w[2] : p.w[3];
      G = -flog(d.emM + neg_log_uniform<F>(w));
    }
    st.offer(Cand<F>{y + G, e, v, x});
  }
}

// Scores the 64 indices of block q, one per lane.  `data` points at the block's 64 elements
// (LDS copy or the row itself).
template <int DT, typename F>
__device__ __forceinline__ void visit_block(const StepArgs& a, int row, int q, const void* data, F bound, float floor,
                                            Search<F>& st) {
  const int lane = threadIdx.x & (kWave - 1);
  const BlockDraw<F> d = block_draw<F>(a, row, q);
  const int32_t v = q * kDrawBlock + lane;
  if (v < a.V) score_index<F>(a, row, v, elem_at<DT>(data, lane), d, bound, floor, st);
}

// The scalar chain regret -> normalised, clipped regret -> smoothed state -> stop test.
// Every operation is a single correctly rounded fp32 operation in the order written
// (contraction off), so a host re-computation reproduces z and the stop decision bit for bit.
struct ChainOut {
  float g, z;
  bool stop;
};

constexpr uint32_t kTagStop = 0x53544F50u;  // counter word 3 of the coin of the random stop mode

__device__ __forceinline__ ChainOut scalar_chain(const StepArgs& a, int row, float m, float x_a, float z_prev, float value) {
#pragma clang fp contract(off)
  const float d = m - x_a;
  const float g = d * a.inv_tau;                                    // Eq. step_gap
  const float n = (g - a.mu_g) * a.rsd;
  const float gt = fminf(fmaxf(n, -a.clip_c), a.clip_c);            // Eq. normalized_gap
  const float t = a.oma * gt;
  const float zn = __builtin_fmaf(a.alpha_s, z_prev, t);            // Eq. smoothed_score
  bool stop;
  if (a.stop_mode == ESPO_STOP_VALUE_ONLY) {
    stop = value < a.stop_threshold;
  } else if (a.stop_mode == ESPO_STOP_REGRET_ONLY) {
    stop = zn > a.stop_threshold;
  } else if (a.stop_mode == ESPO_STOP_RANDOM) {
    const Philox4 p = philox4x32_10(0u, (uint32_t)a.step, (uint32_t)row, kTagStop, a.key0, a.key1);
    stop = (float)(2u * (p.w[0] >> 9) + 1u) * (1.0f / 16777216.0f) < a.stop_threshold;  // u(w) is exact in fp32
  } else {
    const float thr = a.beta * fmaxf(value, a.eps);
    stop = zn > thr;                                                // Eq. stop_rule (strict)
  }
  return ChainOut{g, zn, a.stop_enabled && stop};
}

// ---------------------------------------------------------------- shared memory
// Blocks are named by their index q in the row everywhere (survivor lists, top_q, visq); the
// per-block tables only cover the workgroup's chunk and are reached through the accessors, which
// subtract q0, the chunk's first block (a multiple of 8).
struct StepShared {
  float* mu;        // [nslots][2] per block slot (tile * 8 + group): upper bound of M_q (phase 1 only; phase 2
                    //   keeps its survivor list there), and the bound of the block's best score
  uint32_t* wq;     // [nslots] the block's word of the random stream
  int q0;           // first block of the chunk
  __device__ __forceinline__ float& mub(int q) const { return mu[2 * (q - q0)]; }
  __device__ __forceinline__ float& ub(int q) const { return mu[2 * (q - q0) + 1]; }
  __device__ __forceinline__ uint32_t& word(int q) const { return wq[q - q0]; }
  __device__ __forceinline__ float& blockmax(int q) const { return bmx[q - q0]; }
  __device__ __forceinline__ int& surv(int k) const { return ((int*)mu)[2 * k]; }
  void* top_raw;    // [8 W][64 elements] data of each lane group's best block
  int* top_q;       // [8 W] which block each lane group kept
  float* m;         // [W] wave maxima
  float* sum;       // [W] wave softmax sums (relative to the chunk maximum)
  float* sumw;      // [W] wave sums of 2^t t, t = (y_v - y_max) log2 e (entropy output only)
  double* res_s;    // [W] per-wave search results
  double* res_hi2;
  float* res_e;
  int* res_v;
  float* res_x;
  float* lo;        // [W] score each wave knows to be attained
  int* visq;        // [2][W] blocks each wave scored before the first barrier, or -1
  float* fres;      // [5][W] per-wave results of the fp32 search: s, e, x, hi2, v
  int32_t* cand_v;  // [kCandCap] long survivor lists: indices that can still win ...
  float* cand_x;    // [kCandCap] ... and their logits
  int* ncand;       // [1]
  int* nsurv;       // [1]
  int* bkey;        // [1] best attained score published during long survivor lists (order-preserving key)
  float floor;      // only logits above this take part in the search (-inf unless the draw is filtered)
  float* bmx;       // [nslots] largest logit of every block (filtered draws only, else null)
};

template <int DT, bool Filter, int W>
__device__ __forceinline__ StepShared carve(unsigned char* base, int nslots, int q0) {
  constexpr int kStepWaves = W, kSlots = W * kGroups;
  StepShared s;
  s.floor = kNegInf;
  s.q0 = q0;
  size_t off = 0;
  auto take = [&](size_t bytes) { void* p = base + off; off += (bytes + 15) & ~(size_t)15; return p; };
  s.res_s = (double*)take(kStepWaves * 8);
  s.res_hi2 = (double*)take(kStepWaves * 8);
  s.top_raw = take((size_t)kSlots * kDrawBlock * elem_bytes<DT>());
  s.top_q = (int*)take(kSlots * 4);
  s.m = (float*)take(kStepWaves * 4);
  s.sum = (float*)take(kStepWaves * 4);
  s.sumw = (float*)take(kStepWaves * 4);
  s.res_e = (float*)take(kStepWaves * 4);
  s.res_v = (int*)take(kStepWaves * 4);
  s.res_x = (float*)take(kStepWaves * 4);
  s.lo = (float*)take(kStepWaves * 4);
  s.visq = (int*)take(2 * kStepWaves * 4);
  s.fres = (float*)take(5 * kStepWaves * 4);
  s.cand_v = (int32_t*)take(kCandCap * 4);
  s.cand_x = (float*)take(kCandCap * 4);
  s.nsurv = (int*)take(16);
  s.bkey = s.nsurv + 1;
  s.ncand = s.nsurv + 2;
  s.mu = (float*)take((size_t)nslots * 8);
  s.wq = (uint32_t*)take((size_t)nslots * 4);
  s.bmx = Filter ? (float*)take((size_t)nslots * 4) : nullptr;
  return s;
}

// Dynamic LDS of a workgroup of `waves` wavefronts whose chunk has `ntiles` tiles (what carve() lays out).
size_t step_lds_bytes(int dt, int ntiles, bool filter, int waves) {
  const size_t esz = dt == ESPO_BF16 ? 2 : 4;
  const size_t nslots = (size_t)ntiles * kGroups, slots = (size_t)waves * kGroups;
  return 2 * (size_t)waves * 8 + slots * kDrawBlock * esz + slots * 4 + 14 * (size_t)waves * 4 + 16 + 2 * kCandCap * 4 +
         ((nslots * 8 + 15) & ~(size_t)15) + (filter ? 2 : 1) * ((nslots * 4 + 15) & ~(size_t)15);
}

// The streaming loop stores a block's bound as the plain fma(y_max, 1/tau, bound of M_q); what
// that fma may have rounded away (2^-24 relative) is added back where bounds are compared.
__device__ __forceinline__ float ub_rounded_up(float u) { return fmaf(fabsf(u), 2e-7f, u); }

// Whether block b can hold a logit that takes part in the search: always, unless the draw is
// filtered; then only if its largest logit is above the floor.
__device__ __forceinline__ bool holds_eligible(const StepShared& sh, int q) { return sh.bmx == nullptr || sh.blockmax(q) > sh.floor; }

// Wave that streamed block q in phase 1, and the slot (wave, group) of that block.
template <int W>
__device__ __forceinline__ int wave_of(const StepShared& sh, int q) { return ((q - sh.q0) >> 3) & (W - 1); }
template <int W>
__device__ __forceinline__ int slot_of(const StepShared& sh, int q) { return wave_of<W>(sh, q) * kGroups + (q & (kGroups - 1)); }

// ---------------------------------------------------------------- phase 2
__device__ __forceinline__ int float_key(float f) {  // order-preserving map to signed int
  const int b = __builtin_bit_cast(int, f);
  return b >= 0 ? b : b ^ 0x7fffffff;
}

template <typename F>
__device__ __forceinline__ float round_down_f32(F v) {
  float f = (float)v;
  if ((F)f > v) f = __builtin_bit_cast(float, __builtin_bit_cast(int32_t, f) + (f > 0.0f ? -1 : 1));
  if (f == 0.0f && v < (F)0) f = -1e-37f;
  return f;
}

// Merges the lanes' and then the waves' search states in a fixed order; returns the same
// result in every thread.  All threads of the workgroup must call it.
template <typename F, int W>
__device__ __forceinline__ Search<F> combine_search(const StepShared& sh, Search<F> st) {
  constexpr int kStepWaves = W;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  st = wave_merge(st);
  if (lane == 0) {
    sh.res_s[wave] = (double)st.best.s;
    sh.res_hi2[wave] = (double)st.hi2;
    sh.res_e[wave] = st.best.e;
    sh.res_v[wave] = st.best.v;
    sh.res_x[wave] = st.best.x;
  }
  __syncthreads();
  Search<F> all;
  all.init();
#pragma unroll 1
  for (int w = 0; w < kStepWaves; ++w) {  // fixed order: deterministic
    Search<F> o;
    o.best = Cand<F>{(F)sh.res_s[w], sh.res_e[w], sh.res_v[w], sh.res_x[w]};
    o.hi2 = (F)sh.res_hi2[w];
    all.merge(o);
  }
  return all;
}

// Finds the argmax over the row in precision F.  `bound0` is a score that is known to be
// attained or exceeded (prunes from the start); `q_own` is the block this wave scores
// first, without waiting for the others (or -1).  Every block whose bound reaches the best
// score found that way is then scored, one block per wave visit.  `between` runs right
// after the first barrier.  Returns the winner, the same in every thread; all threads of
// the workgroup must call it.
template <int DT, typename F, int W, typename Between>
__device__ __forceinline__ Search<F> find_argmax(const StepArgs& a, const StepShared& sh, const void* rowp, int row,
                                                 int nslots, int q_own, F bound0, Between between) {
  constexpr int kStepWaves = W, kStepThreads = W * kWave;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  auto data_of = [&](int q) -> const void* {  // LDS copy if a lane group kept this block, else the row
    const int slot = slot_of<W>(sh, q);
    if (sh.top_q[slot] == q) return (const char*)sh.top_raw + (size_t)slot * kDrawBlock * elem_bytes<DT>();
    return (const char*)rowp + (size_t)q * kDrawBlock * elem_bytes<DT>();
  };
  Search<F> st;
  st.init();
  F bound = bound0;
  int q = q_own, k = wave, nsurv = 0;
  bool first = true;
#pragma unroll 1
  while (true) {  // one visit site for the wave's own block and for the survivors
    if (q >= 0) {
      visit_block<DT, F>(a, row, q, data_of(q), bound, sh.floor, st);
      const float lo = wave_max(round_down_f32(st.lower()));  // best score this wave has seen, rounded down
      bound = bound > (F)lo ? bound : (F)lo;
    }
    if (first) {
      first = false;
      if (lane == 0) {
        sh.lo[wave] = round_down_f32(bound);  // rounded down: a shared bound must never overshoot
        sh.visq[wave] = q_own;
      }
      if (tid == 0) *sh.nsurv = 0;
      __syncthreads();
      between();
      float bound_f = sh.lo[0];
#pragma unroll
      for (int w = 1; w < kStepWaves; ++w) bound_f = fmaxf(bound_f, sh.lo[w]);
      // blocks whose bound reaches the best score found so far
      for (int b = sh.q0 + tid; b < sh.q0 + nslots; b += kStepThreads) {
        const float u = sh.ub(b);
        if (u > -1e30f && ub_rounded_up(u) >= bound_f && sh.visq[wave_of<W>(sh, b)] != b && holds_eligible(sh, b))
          sh.surv(atomicAdd(sh.nsurv, 1)) = b;
      }
      __syncthreads();
      nsurv = *sh.nsurv;
      bound = bound > (F)bound_f ? bound : (F)bound_f;
    } else {
      k += kStepWaves;
    }
    if (k >= nsurv) break;
    q = sh.surv(k);
  }
  return combine_search<F, W>(sh, st);
}

// ---------------------------------------------------------------- phase 2 in fp32
// State of the fp32 search, per lane while blocks are visited and wave-uniform once reduced:
// the best index scored (score s known to within +-e, logit x) and hi2, the largest upper
// end s + e among all other scored indices.  The winner is certain iff s - e > hi2.
struct Best {
  float s, e, x, hi2;
  int32_t v;
};

__device__ __forceinline__ Best no_best() { return Best{kNegInf, 0.0f, 0.0f, kNegInf, -1}; }

// Scores index v (logit x) in fp32 and offers it to the lane's state.  An index is scored at
// most once in this search, so a lane never meets the same index twice.
__device__ __forceinline__ void score_element(const StepArgs& a, const StepShared& sh, int row, int32_t v, float x,
                                              bool valid, Best& st) {
  const int32_t q = v >> 6;
  const int32_t first = q * kDrawBlock;
  const int32_t n = a.V - first < kDrawBlock ? a.V - first : kDrawBlock;
  // the index's own word depends on nothing else here: its ten rounds overlap the loads
  const Philox4 p = philox4x32_10((uint32_t)(v >> 2), (uint32_t)a.step, (uint32_t)row, kTagElem, a.key0, a.key1);
  const uint32_t w = (v & 3) == 0 ? p.w[0] : (v & 3) == 1 ? p.w[1] : (v & 3) == 2 ? p.w[2] : p.w[3];
  const uint32_t wb = sh.word(q);
  const float nlb = neg_log_uniform<float>(wb);
  const float M = flog((float)n) - flog(nlb);                 // M_q = ln n - ln(-ln u)
  const float emM = nlb * __builtin_amdgcn_rcpf((float)n);    // exp(-M_q) = (-ln u) / n
  int32_t vpos = first + (int32_t)((wb >> 3) & 63u);
  if (n < kDrawBlock) {  // ragged last block: own position draw
    const Philox4 pr = philox4x32_10((uint32_t)q, (uint32_t)a.step, (uint32_t)row, kTagRagged, a.key0, a.key1);
    vpos = first + (int32_t)(((uint64_t)pr.w[0] * (uint64_t)n) >> 32);
  }
  const float G = v == vpos ? M : -flog(emM + neg_log_uniform<float>(w));
  const float y = x * a.inv_tau;
  const float sc = y + G;
  const float e = score_margin(a, y);
  if (valid && x > sh.floor) {  // masked (-inf) and filtered entries never win
    if (sc > st.s) {
      st.hi2 = fmaxf(st.hi2, st.s + st.e);
      st.s = sc; st.e = e; st.x = x; st.v = v;
    } else {
      st.hi2 = fmaxf(st.hi2, sc + e);
    }
  }
}

// This lane's element of block q: from LDS if a lane group kept the block, else from the row.
template <int DT, int W>
__device__ __forceinline__ float block_elem(const StepArgs& a, const StepShared& sh, const void* rowp, int q) {
  const int lane = threadIdx.x & (kWave - 1);
  const int32_t first = q * kDrawBlock;
  const int32_t n = a.V - first < kDrawBlock ? a.V - first : kDrawBlock;
  const int slot = slot_of<W>(sh, q);
  const int idx = lane < n ? lane : n - 1;  // stay inside the row in a ragged last block
  if (sh.top_q[slot] == q) return elem_at<DT>((const char*)sh.top_raw + (size_t)slot * kDrawBlock * elem_bytes<DT>(), idx);
  return elem_at<DT>((const char*)rowp + (size_t)first * elem_bytes<DT>(), idx);
}

// Scores the 64 indices of block q, one per lane.
template <int DT, int W>
__device__ __forceinline__ void fast_visit(const StepArgs& a, const StepShared& sh, const void* rowp, int row, int q,
                                           Best& st) {
  const int lane = threadIdx.x & (kWave - 1);
  const int32_t n = a.V - q * kDrawBlock < kDrawBlock ? a.V - q * kDrawBlock : kDrawBlock;
  score_element(a, sh, row, q * kDrawBlock + lane, block_elem<DT, W>(a, sh, rowp, q), lane < n, st);
}

// For a row with a long survivor list: instead of scoring every index of every surviving
// block, the blocks' logits are only compared with the bound (index v can win only if
// y_v + M_q reaches it); the few indices that pass are collected and then scored by all threads
// at once.  The blocks are read again from the row, laid out as in phase 1: a lane group of 8
// lanes per block, 16 bytes per lane, so one load of a wave covers 8 blocks; with four loads in
// flight the workgroup covers 512 blocks per trip to memory (a flat row at temperature 1 has a
// hundred survivors and more; one block per load took a trip per 64 of them).
template <int DT, int W>
__device__ __forceinline__ void collect_candidates(const StepArgs& a, const StepShared& sh, const void* rowp, int nsurv,
                                                   float bound) {
  constexpr int kStepWaves = W, kLoads = 4;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int grp = lane >> 3;
  const uint32_t sub = (uint32_t)(lane & 7) * 8u;  // the lane's 8 elements within its block
  const uint32_t last_group = (uint32_t)(a.V - 1) & ~7u;
#pragma unroll 1
  for (int base = wave * kGroups; base < nsurv; base += kLoads * kStepWaves * kGroups) {
    int qs[kLoads];
    Raw<DT> raw[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int k = base + j * kStepWaves * kGroups + grp;
      qs[j] = k < nsurv ? sh.surv(k) : -1;
      // a group without a block reads block 0 and drops it; a ragged last block is masked below
      const uint32_t e0 = (uint32_t)(qs[j] < 0 ? 0 : qs[j]) * kDrawBlock + sub;
      raw[j] = load_raw<DT>(rowp, e0 < last_group ? e0 : last_group, (uint32_t)a.V);
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      if (qs[j] < 0) continue;
      float x[8];
      unpack<DT>(raw[j], x);
      const int32_t first = qs[j] * kDrawBlock;
      const int32_t n = a.V - first < kDrawBlock ? a.V - first : kDrawBlock;
      const float M = flog((float)n) - flog(neg_log_uniform<float>(sh.word(qs[j])));
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int32_t v = first + (int32_t)sub + u;
        const float y = x[u] * a.inv_tau;
        if (v < a.V && x[u] > sh.floor && (y + M) + 2.0f * score_margin(a, y) >= bound) {
          const int i = atomicAdd(sh.ncand, 1);
          if (i < kCandCap) {
            sh.cand_v[i] = v;
            sh.cand_x[i] = x[u];
          }
        }
      }
    }
  }
}

// The exact decision for a row whose best fp32 scores overlap: `lower` is a score known to be
// attained (the fp32 winner's lower end), so only indices with y_v + M_q at or above it can
// be the maximum.  They are collected as above, usually two or three, and scored in double
// by one thread each.  Returns false if they do not fit the candidate buffer (then the
// caller searches block by block); all threads of the workgroup must call it.
template <int DT, int W>
__device__ __forceinline__ bool exact_among_candidates(const StepArgs& a, const StepShared& sh, const void* rowp, int row,
                                                       int nslots, float lower, Search<double>& out) {
  constexpr int kStepThreads = W * kWave;
  const int tid = threadIdx.x;
  if (tid == 0) {
    *sh.nsurv = 0;
    *sh.ncand = 0;
  }
  __syncthreads();
  for (int b = sh.q0 + tid; b < sh.q0 + nslots; b += kStepThreads) {
    const float u = sh.ub(b);
    if (u > -1e30f && ub_rounded_up(u) >= lower && holds_eligible(sh, b)) sh.surv(atomicAdd(sh.nsurv, 1)) = b;
  }
  __syncthreads();
  collect_candidates<DT, W>(a, sh, rowp, *sh.nsurv, lower);
  __syncthreads();
  const int ncand = *sh.ncand;
  if (ncand > kCandCap) return false;
  Search<double> st;
  st.init();
  for (int i = tid; i < ncand; i += kStepThreads) {
    const int32_t v = sh.cand_v[i];
    const BlockDraw<double> d = block_draw<double>(a, row, v >> 6);
    score_index<double>(a, row, v, sh.cand_x[i], d, -__builtin_huge_val(), sh.floor, st);
  }
  out = combine_search<double, W>(sh, st);
  return true;
}

// Combines the lanes' states into the wave's: highest score, lowest index among equals.
__device__ __forceinline__ Best wave_best(const Best& st) {
  const float smax = wave_max(st.s);
  const bool cand = st.v >= 0 && st.s == smax;
  const uint32_t vmin = wave_min_u32(cand ? (uint32_t)st.v : 0xffffffffu);
  if (vmin == 0xffffffffu) return no_best();
  const bool win = cand && (uint32_t)st.v == vmin;
  const int src = (int)__builtin_ctzll(__builtin_amdgcn_ballot_w64(win));
  Best r;
  r.s = smax;
  r.v = (int32_t)vmin;
  r.e = uniform_f32(st.e, src);
  r.x = uniform_f32(st.x, src);
  r.hi2 = wave_max(win ? st.hi2 : fmaxf(st.hi2, st.s + st.e));
  return r;
}

__device__ __forceinline__ float key_float(int k) { return __builtin_bit_cast(float, k >= 0 ? k : k ^ 0x7fffffff); }

// The fp32 search over the row.  Every wave first scores `q_own`, the block with the largest
// bound it has streamed, and `q_own2`, its second (or -1: a workgroup of 16 waves scores one each,
// one of 8 waves two each: with fewer first blocks the bound is poorer and flat rows keep many more
// survivors; measured at temperature 1.0, B = 512: 58 us per launch with 8 first blocks, 38 with 16);
// the best lower end s - e found that way is a score known to be
// attained, and every other block whose bound reaches it is then scored, one block per wave
// visit.  `between` runs right after the first barrier.  Returns the wave-uniform result,
// the same in every wave; all threads of the workgroup must call it.
template <int DT, int W, typename Between>
__device__ __forceinline__ Best fast_argmax(const StepArgs& a, const StepShared& sh, const void* rowp, int row, int nslots,
                                            int q_own, int q_own2, Between between) {
  constexpr int kStepWaves = W, kStepThreads = W * kWave;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  Best st = no_best();
  int q = q_own, k = wave, nsurv = 0;
  bool first = true, second = q_own2 >= 0;
#pragma unroll 1
  while (true) {  // one visit site for the wave's own blocks and for the survivors
    if (q >= 0) fast_visit<DT, W>(a, sh, rowp, row, q, st);
    if (first && second) {  // (wave-uniform)
      second = false;
      q = q_own2;
      continue;
    }
    if (first) {
      first = false;
      const float lo = wave_max(st.s - st.e);
      if (lane == 0) {
        sh.lo[wave] = lo;
        sh.visq[wave] = q_own;
        sh.visq[kStepWaves + wave] = q_own2;
      }
      if (tid == 0) {
        *sh.nsurv = 0;
        *sh.ncand = 0;
      }
      __syncthreads();
      between();
      const float bound = wave_max(lane < kStepWaves ? sh.lo[lane] : kNegInf);
      for (int b = sh.q0 + tid; b < sh.q0 + nslots; b += kStepThreads) {  // blocks whose bound reaches the best score found so far
        const float u = sh.ub(b);
        const int w_b = wave_of<W>(sh, b);
        if (u > -1e30f && ub_rounded_up(u) >= bound && sh.visq[w_b] != b && sh.visq[kStepWaves + w_b] != b && holds_eligible(sh, b))
          sh.surv(atomicAdd(sh.nsurv, 1)) = b;
      }
      if (tid == 0) *sh.bkey = float_key(bound);
      __syncthreads();
      nsurv = *sh.nsurv;
      if (nsurv > kStepWaves) {  // long list
        collect_candidates<DT, W>(a, sh, rowp, nsurv, bound);
        __syncthreads();
        const int ncand = *sh.ncand;
        if (ncand <= kCandCap) {  // else (tie-heavy rows): block by block below
          for (int i = tid; i < ncand; i += kStepThreads) score_element(a, sh, row, sh.cand_v[i], sh.cand_x[i], true, st);
          k = nsurv;
        }
      }
    } else {
      if (nsurv > kStepWaves) {  // long list: publish what this wave has attained, later visits may then be skipped
        const float lo = wave_max(st.s - st.e);
        if (lane == 0) atomicMax(sh.bkey, float_key(lo));
      }
      k += kStepWaves;
    }
    q = -1;
    while (k < nsurv) {  // this wave's next survivor that can still matter
      const int c = sh.surv(k);
      if (nsurv <= kStepWaves || ub_rounded_up(sh.ub(c)) >= key_float(*sh.bkey)) { q = c; break; }
      k += kStepWaves;
    }
    if (q < 0) break;
  }
  const Best mine = wave_best(st);
  if (lane == 0) {
    sh.fres[0 * kStepWaves + wave] = mine.s;
    sh.fres[1 * kStepWaves + wave] = mine.e;
    sh.fres[2 * kStepWaves + wave] = mine.x;
    sh.fres[3 * kStepWaves + wave] = mine.hi2;
    sh.fres[4 * kStepWaves + wave] = __builtin_bit_cast(float, mine.v);
  }
  __syncthreads();
  Best t = no_best();
  if (lane < kStepWaves) {
    t.s = sh.fres[0 * kStepWaves + lane];
    t.e = sh.fres[1 * kStepWaves + lane];
    t.x = sh.fres[2 * kStepWaves + lane];
    t.hi2 = sh.fres[3 * kStepWaves + lane];
    t.v = __builtin_bit_cast(int32_t, sh.fres[4 * kStepWaves + lane]);
  }
  return wave_best(t);
}

// ---------------------------------------------------------------- the kernel
// alive[row] == 0, read through the scalar data path: the aligned 32-bit word that holds the flag (it
// lies in the same page as the flag, so the read cannot fault wherever the array ends).  A workgroup
// whose row is done holds its place in the dispatcher's queue until it knows; the scalar path tells
// it sooner than a vector load.  The kernel writes the flag later with a vector store, after this
// read, and never reads it again.
__device__ __forceinline__ bool row_is_done(const uint8_t* alive, int row) {
  const uintptr_t addr = (uintptr_t)(alive + row);
  const uint32_t* word = (const uint32_t*)(addr & ~(uintptr_t)3);
  uint32_t bits;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(bits) : "s"(word) : "memory");
  return ((bits >> (8u * (uint32_t)(addr & 3))) & 0xffu) == 0u;
}

template <int DT, bool Entropy, bool Filter, bool Sum, int W>
// Registers: 64 per lane for 16 waves (two workgroups on a compute unit); workgroups of 8 waves get up
// to 80 (three of them fit, in registers and in LDS) and use 75 without spilling; a filtered draw gets 128.
__global__ __launch_bounds__(W * kWave, Filter ? 4 : W == 8 ? 6 : 8) void espo_step_kernel(StepArgs a) {
  static_assert(Sum || (!Entropy && !Filter), "entropy and filtered draws need the softmax sum");
  static_assert(!Filter || W == 8, "a filtered draw looks at the whole row: one workgroup of 8 waves per row");
  constexpr int kStepWaves = W, kStepThreads = W * kWave, kSlots = W * kGroups;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int tid = threadIdx.x;
  // workgroup row * nch + c owns chunk c of the row: tiles [tile0, tile1)
  const unsigned unit = blockIdx.x;
  const int nch = Filter ? 1 : a.nch;
  const int row = nch == 1 ? (int)unit : (int)(unit / (unsigned)nch);
  const int chunk = (int)unit - row * nch;
  if (row_is_done(a.alive, row)) {  // done rows are not decoded (Algorithm 1, loop condition)
    if (tid == 0 && chunk == 0) {
      a.tokens[row] = -1;
      a.regret[row] = 0.0f;
      if (a.logprob) a.logprob[row] = 0.0f;
      if (Entropy) a.entropy[row] = 0.0f;
    }
    return;
  }
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = lane >> 3;
  const int ntiles = a.ntiles;  // of the row
  const int tile0 = nch == 1 ? 0 : (int)(((int64_t)chunk * ntiles) / nch);
  const int tile1 = nch == 1 ? ntiles : (int)(((int64_t)(chunk + 1) * ntiles) / nch);
  const int ctiles = tile1 - tile0;
  const int nslots = ctiles * kGroups;  // block slots of the chunk incl. the non-existent ones of the row's last tile
  const StepShared sh = carve<DT, Filter, W>(smem_raw, nslots, tile0 * kGroups);
  const void* rowp = (const char*)a.logits + (size_t)row * (size_t)a.row_stride * elem_bytes<DT>();

  // ------------------------------------------------------------ phase 1: stream the chunk
  // Wave iteration i handles tile tile0 + i*W + wave.  Lanes whose 16-byte group starts at or beyond
  // V (the row's last tile only) read the last valid group instead and are masked below.
  const int my_tiles = wave < ctiles ? (ctiles - wave + kStepWaves - 1) / kStepWaves : 0;
  const uint32_t last_group = (uint32_t)(a.V - 1) & ~7u;
  // the last 16-byte group of the chunk: where the first ring's loads of a wave with fewer tiles go
  const uint32_t chunk_last = tile1 == ntiles ? last_group : (uint32_t)tile1 * kTile - 8u;
  const uint32_t lane_off = (uint32_t)lane * 8u;
  const uint32_t lane_bytes = lane_off * (uint32_t)elem_bytes<DT>();
  auto load_tile = [&](int t) {  // t is wave-uniform
    if (t != ntiles - 1) return load_raw_inner<DT>((const char*)rowp + (size_t)t * kTile * elem_bytes<DT>(), lane_bytes);
    const uint32_t e0 = (uint32_t)t * kTile + lane_off;  // last tile: may be ragged
    return load_raw<DT>(rowp, e0 < last_group ? e0 : last_group, (uint32_t)a.V);
  };
  // The first ring of loads is issued by every wave, whether it has that many tiles or not
  // (addresses beyond the chunk fall back on its last group): with a fixed number of loads in
  // flight the compiler can wait for exactly the one a ring slot needs.
  Raw<DT> ring[kRing];
#pragma unroll
  for (int d = 0; d < kRing; ++d) {
    const uint32_t e0 = (uint32_t)(tile0 + d * kStepWaves + wave) * kTile + lane_off;
    ring[d] = load_raw<DT>(rowp, e0 < chunk_last ? e0 : chunk_last, (uint32_t)a.V);
  }
  // While the first loads are in flight: M_q bounds of the chunk's blocks, four per Philox call
  // (the chunk starts at a multiple of 8 blocks, so the calls' groups of four line up).
  for (int c = tid; c * 4 < nslots; c += kStepThreads) {
    const int b0 = sh.q0 + c * 4;
    const Philox4 p = philox4x32_10((uint32_t)(b0 >> 2), (uint32_t)a.step, (uint32_t)row, kTagBlock, a.key0, a.key1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int b = b0 + j;
      float mub = kNegInf;
      if (b < a.nblocks) {
        const int32_t n = a.V - b * kDrawBlock < kDrawBlock ? a.V - b * kDrawBlock : kDrawBlock;
        mub = (__builtin_amdgcn_logf((float)n) * kLn2 + 2e-6f) + gumbel_upper_f32(p.w[j]);
        mub += 1e-5f + 4e-7f * fabsf(mub);  // room for the rounding of y_max + M_q below
      }
      if (c * 4 + j < nslots) {
        sh.mub(b) = mub;
        sh.word(b) = p.w[j];
      }
    }
  }
  __syncthreads();

  // Softmax sum against a lazily advanced per-lane reference: the lane accumulates
  // sum_v 2^(x_v k2 + nrk) with nrk = -(reference logit) * k2; the final combine multiplies
  // by 2^-(m k2 + nrk), so the rounding of nrk itself cancels.  `lead` is the logit beyond
  // which the reference has to move up (the sum would grow past 2^64 per term otherwise).
  float nrk = 1e30f;
  float lead = kNegInf;
  float sum = 0.0f;
  float sumw = 0.0f;         // entropy output: sum_v 2^t_v t_v with t_v = x_v k2 + nrk (see below)
  float mx = kNegInf;        // largest logit this lane group has seen
  float mx_odd = kNegInf;    // filtered draws keep it apart for the odd tiles: twice as many values to choose a floor from
  float top_ub = kNegInf;    // largest block bound this lane group has seen, and its block
  int top_q = -1;
  char* const my_raw = (char*)sh.top_raw + ((size_t)(wave * kGroups + grp) * kDrawBlock + (lane & 7) * 8) * elem_bytes<DT>();
  float* const bmx_lane = Filter ? sh.bmx + (wave * kGroups + grp) : nullptr;
  float* const mu_lane = sh.mu + 2 * (wave * kGroups + grp);  // this lane group's entry of tile `wave`; 256 floats per iteration

  // One wave iteration over ring slot d, tile index i of this wave.  `Steady` iterations are
  // those that need no checks: the tile is whole, not the row's last, and its ring slot is
  // refilled with a tile that is not the last either.
  auto iteration = [&](auto steady, int d, int i) {
    constexpr bool Steady = decltype(steady)::value;
    const int t = tile0 + i * kStepWaves + wave;
    float x[8];
    unpack<DT>(ring[d], x);
    if (!Steady && (t + 1) * kTile > a.V) {  // ragged last tile: indices at or beyond V do not exist
      const int32_t e0 = t * kTile + (int32_t)lane_off;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (e0 + j >= a.V) x[j] = kNegInf;
    }
    const float gm = fmaxf(fmaxf(fmaxf(fmaxf(fmaxf(x[0], x[1]), x[2]), fmaxf(fmaxf(x[3], x[4]), x[5])), x[6]), x[7]);
    if constexpr (Sum) {
      if (__builtin_amdgcn_ballot_w64(gm > lead) != 0) {  // rare after the first tile
        asm volatile("" ::: "memory");  // keep this rare path out of the straight-line code
        if (gm > lead) {  // move this lane's reference up to gm
          const float nrk_new = -gm * a.k2;
          const float shift = nrk_new - nrk;  // every t_v moves by this much
          const float f = __builtin_amdgcn_exp2f(shift);
          if (Entropy) sumw = f * fmaf(shift, sum, sumw);
          sum *= f;
          nrk = nrk_new;
          lead = gm + a.ref_lead;
        }
      }
    }
    if constexpr (!Sum) {
      // nobody asked for the log-probability, the entropy or a filtered draw: token, regret and
      // state need the row maximum only, and the eight fma / exp2 / add per lane are left out
    } else if constexpr (!Entropy) {
      float acc0 = __builtin_amdgcn_exp2f(fmaf(x[0], a.k2, nrk));
      float acc1 = __builtin_amdgcn_exp2f(fmaf(x[1], a.k2, nrk));
#pragma unroll
      for (int j = 2; j < 8; j += 2) {
        acc0 += __builtin_amdgcn_exp2f(fmaf(x[j], a.k2, nrk));
        acc1 += __builtin_amdgcn_exp2f(fmaf(x[j + 1], a.k2, nrk));
      }
      sum += acc0 + acc1;
    } else {
      // The entropy needs sum_v pi_v ln pi_v = (ln 2 / S) sum_v 2^t_v t_v - ln S.  t_v is kept
      // above -200: 2^t_v is 0 in fp32 from far above that, so the sum is unchanged and a
      // masked logit (-inf) contributes 0 * -200 instead of 0 * -inf.
      float acc0 = 0.0f, acc1 = 0.0f, w0 = 0.0f, w1 = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; j += 2) {
        const float t0 = fmaxf(fmaf(x[j], a.k2, nrk), -200.0f), t1 = fmaxf(fmaf(x[j + 1], a.k2, nrk), -200.0f);
        const float e0 = __builtin_amdgcn_exp2f(t0), e1 = __builtin_amdgcn_exp2f(t1);
        acc0 += e0;
        acc1 += e1;
        w0 = fmaf(e0, t0, w0);
        w1 = fmaf(e1, t1, w1);
      }
      sum += acc0 + acc1;
      sumw += w0 + w1;
    }
    // upper bound of every perturbed score in the lane group's block: y_max + M_q
    const float bm = group8_max(gm);
    float* const mu = mu_lane + (size_t)i * (2 * kStepWaves * kGroups);
    const float ub = fmaf(bm, a.inv_tau, mu[0]);
    mu[1] = ub;  // the 8 lanes of the group store the same value
    if constexpr (Filter) bmx_lane[(size_t)i * (kStepWaves * kGroups)] = bm;
    if (Filter && (i & 1)) mx_odd = fmaxf(mx_odd, bm);
    else mx = fmaxf(mx, bm);
    if (ub > top_ub) {  // keep the data of the block with the group's largest bound
      top_ub = ub;
      top_q = t * kGroups + grp;
      *(u32x4*)my_raw = u32x4{ring[d].w[0], ring[d].w[1], ring[d].w[2], ring[d].w[3]};
      if constexpr (DT == ESPO_F32) *(u32x4*)(my_raw + 16) = u32x4{ring[d].w[4], ring[d].w[5], ring[d].w[6], ring[d].w[7]};
    }
    if (Steady)  // refill this ring slot
      ring[d] = load_raw_inner<DT>((const char*)rowp + (size_t)(t + kRing * kStepWaves) * kTile * elem_bytes<DT>(), lane_bytes);
    else if (i + kRing < my_tiles)
      ring[d] = load_tile(t + kRing * kStepWaves);
  };
  // Steady passes: all kRing tiles and their refills lie before this wave's last tile.
  const int steady_end = my_tiles > 2 * kRing ? ((my_tiles - kRing - 1) / kRing) * kRing : 0;
  int i0 = 0;
#pragma unroll 1
  for (; i0 < steady_end; i0 += kRing) {
#pragma unroll
    for (int d = 0; d < kRing; ++d) iteration(std::true_type{}, d, i0 + d);
  }
#pragma unroll 1
  for (; i0 < my_tiles; i0 += kRing) {
#pragma unroll
    for (int d = 0; d < kRing; ++d)
      if (i0 + d < my_tiles) iteration(std::false_type{}, d, i0 + d);  // wave-uniform
  }
  // The wave's largest logit, and the block with its largest bound (lowest block among equals).
  const float mx_even = mx;
  if constexpr (Filter) mx = fmaxf(mx, mx_odd);
  const float mw = wave_max(mx);
  const float ubw = wave_max(top_ub);
  const int q_own = (int)wave_min_u32(top_q >= 0 && top_ub == ubw ? (uint32_t)top_q : 0xffffffffu);  // -1 if none
  int q_own2 = -1;  // with fewer than 16 waves, also the best block of the wave's other lane groups
  if constexpr (W < 16) {
    const bool other = top_q >= 0 && top_q != q_own;
    const float ubw2 = wave_max(other ? top_ub : kNegInf);
    q_own2 = (int)wave_min_u32(other && top_ub == ubw2 ? (uint32_t)top_q : 0xffffffffu);
  }
  if (lane == 0) sh.m[wave] = mw;
  if ((lane & 7) == 0) sh.top_q[wave * kGroups + grp] = top_q;
  float z_prev = 0.0f, value = 0.0f;  // wanted at the very end: fetched now, off the critical path
  if (tid == 0 && nch == 1) {
    z_prev = a.z[row];
    value = a.values[row];
  }

  // ------------------------------------------------------------ phase 2: argmax of y + G
  float m = kNegInf;
  auto softmax_sum = [&]() {  // after the first barrier: row maximum, then the wave's share of the sum
    m = wave_max(lane < kStepWaves ? sh.m[lane] : kNegInf);
    if constexpr (!Sum) return;
    const float shift = -fmaf(m, a.k2, nrk);  // from this lane's reference to the row maximum
    const float f = __builtin_amdgcn_exp2f(shift);
    const float part = sum > 0.0f ? sum * f : 0.0f;
    const float tot = wave_sum(part);
    if (lane == 0) sh.sum[wave] = tot;
    if constexpr (Entropy) {
      const float totw = wave_sum(sum > 0.0f ? f * fmaf(shift, sum, sumw) : 0.0f);
      if (lane == 0) sh.sumw[wave] = totw;
    }
  };
  int32_t tok;
  float x_a;
  float s_a = kNegInf, e_a = 0.0f;  // the winner's score as a float known to within +-e_a (what the combine of a split row compares)
  // the argmax over the indices whose logit is above shx.floor: fp32 search, decided in double where needed
  auto search = [&](const StepShared& shx, auto between) {
    const Best fast = fast_argmax<DT, W>(a, shx, rowp, row, nslots, q_own, q_own2, between);
    tok = fast.v;
    x_a = fast.x;
    s_a = fast.s;
    e_a = fast.e;
    if (fast.v >= 0 && !(fast.s - fast.e > fast.hi2)) {
      // the two best fp32 scores overlap within their margins: decide in double (rare)
      __syncthreads();  // everyone has read the fp32 results
      Search<double> exact;
      if (!exact_among_candidates<DT, W>(a, shx, rowp, row, nslots, fast.s - fast.e, exact)) {
        __syncthreads();
        exact = find_argmax<DT, double, W>(a, shx, rowp, row, nslots, q_own, (double)fast.s - (double)fast.e, [] {});
      }
      tok = exact.best.v;
      x_a = exact.best.x;
      s_a = (float)exact.best.s;                 // rounded to float: within 2^-24 relative of the double score
      e_a = fmaf(fabsf(s_a), 1.2e-7f, 1e-30f);
    }
  };
  // the largest float below x (x finite or +inf): a floor that lets x itself through
  const auto next_below = [](float x) {
    const int32_t bits = __builtin_bit_cast(int32_t, x);
    return x == 0.0f ? -1.401298464e-45f : __builtin_bit_cast(float, bits + (x > 0.0f ? -1 : 1));
  };
  if constexpr (!Filter) {
    search(sh, softmax_sum);
  } else {
    __syncthreads();  // the waves' maxima are in place
    softmax_sum();    // m, and the waves' shares of S
    __syncthreads();
    tok = -1;         // a row without a finite logit keeps this
    x_a = 0.0f;
  }

  if constexpr (Filter) {
    // Filtered draw (top-p as in the evaluation set-up of Section 5, or top-k).  The kept set is
    // {v : the mass (the number) of strictly larger logits is below p (k)}, an upper set in the
    // logit, so the filtered draw is the argmax of y + G over it.  What is needed is the mass
    // (number) of the logits above a given floor, and those logits themselves when they are few.
    // A table of the blocks' largest logits, filled while streaming, names the blocks that hold
    // any; up to two thirds of the row's blocks are read again block by block, more of them by one
    // more pass over the row.  First a floor that leaves about 64 blocks above it is tried: on rows
    // like a language model's the kept set lies above it.  If it does not (a flat row, some hundred
    // kept logits), a floor that leaves several hundred blocks is tried.  The smallest kept logit is
    // then read off the collected logits (the smallest whose strictly larger ones hold less than p,
    // number fewer than k) and one search above that edge gives the token; the unfiltered winner is
    // not needed then and is not searched for.  Sums within 1e-5 of p times the softmax sum are not
    // trusted in fp32: the search then runs above the smallest logit that may be kept, and its winner
    // stands if it is kept for sure.  Otherwise (still flatter rows, or a winner in doubt) the winner
    // is tested by measuring the mass above it, in double over the whole row and in the oracle's
    // arithmetic where fp32 cannot tell, and while it is not kept the search is repeated above it;
    // that floor rises strictly, so the loop ends.
    // A workgroup of 8 waves with 128 registers per lane runs this instantiation, two of them on a
    // compute unit: with 64 registers the stages below spill, and every reload is a trip to a memory
    // system whose queues are full of the other rows' streaming (measured: 53 us per launch with 16
    // waves and 64 registers, 46 us this way, B = 512, V = 152064, top-p 0.7 at temperature 0.6).
    const auto nothing = [] {};
    const bool by_count = a.top_k > 0;
    const float nrk_row = -m * a.k2;
    const float total = wave_sum(lane < kStepWaves ? sh.sum[lane] : 0.0f);  // S, as the last step forms it
    const float want = a.top_p * total;
    // The collected logits use both candidate areas as one array; their 2^t are formed again where needed.
    constexpr int kKeptCap = 2 * kCandCap;
    float* const kept_x = (float*)sh.cand_v;
    static_assert(kCandCap % 4 == 0, "cand_x follows cand_v without a gap");
    float mass = 0.0f, count = 0.0f;
    int ncand = 0;

    // mass and number of the logits above floor_x; the logits themselves in kept_x if they fit
    auto measure = [&](float floor_x) {
      __syncthreads();  // whatever used the scratch before is over in every wave
      if (tid == 0) {
        *sh.nsurv = 0;
        *sh.ncand = 0;
      }
      __syncthreads();
      for (int b = tid; b < nslots; b += kStepThreads)  // blocks that hold a logit above the floor
        if (sh.bmx[b] > floor_x) sh.surv(atomicAdd(sh.nsurv, 1)) = b;
      __syncthreads();
      const int nabove = *sh.nsurv;
      float acc_m = 0.0f, acc_n = 0.0f;
      constexpr int kVisit = 8, kLoads = 4, kGroupRead = 1536;  // beyond that many blocks (two thirds of this row's) the whole row is streamed
      if (nabove <= 16 * kStepWaves) {
        // The usual case: one block per wave visit, one index per lane, eight loads in flight.  Most of
        // these blocks are their lane group's best, which phase 1 kept in LDS: no trip to memory, whose
        // queues are full of the other rows' streaming.
#pragma unroll 1
        for (int base = wave; base < nabove; base += kVisit * kStepWaves) {
          float xs[kVisit];
          int32_t ns[kVisit];
#pragma unroll
          for (int u = 0; u < kVisit; ++u) {
            const int k = base + u * kStepWaves;
            xs[u] = kNegInf;
            ns[u] = 0;
            if (k < nabove) {
              const int q = __builtin_amdgcn_readfirstlane(sh.surv(k));
              ns[u] = a.V - q * kDrawBlock < kDrawBlock ? a.V - q * kDrawBlock : kDrawBlock;
              xs[u] = block_elem<DT, W>(a, sh, rowp, q);
            }
          }
#pragma unroll
          for (int u = 0; u < kVisit; ++u) {
            if (lane < ns[u] && xs[u] > floor_x) {
              acc_m += __builtin_amdgcn_exp2f(fmaf(xs[u], a.k2, nrk_row));
              acc_n += 1.0f;  // counts stay exact in fp32: V < 2^24
              const int c = atomicAdd(sh.ncand, 1);
              if (c < kKeptCap) kept_x[c] = xs[u];
            }
          }
        }
      } else if (nabove <= kGroupRead) {
        // The listed blocks only, laid out as in phase 1: a lane group of 8 lanes per block, 16 bytes
        // per lane, so one load of a wave covers 8 blocks and the workgroup 256 per trip to memory (eight
        // loads in flight instead of four: 8 us slower on every row, with spills).
        const uint32_t sub = (uint32_t)(lane & 7) * 8u;
#pragma unroll 1
        for (int base = wave * kGroups; base < nabove; base += kLoads * kStepWaves * kGroups) {
          int qs[kLoads];
          Raw<DT> raw[kLoads];
#pragma unroll
          for (int j = 0; j < kLoads; ++j) {
            const int k = base + j * kStepWaves * kGroups + grp;
            qs[j] = k < nabove ? sh.surv(k) : -1;
            // a group without a block reads block 0 and drops it; a ragged last block is masked below
            const uint32_t e0 = (uint32_t)(qs[j] < 0 ? 0 : qs[j]) * kDrawBlock + sub;
            raw[j] = load_raw<DT>(rowp, e0 < last_group ? e0 : last_group, (uint32_t)a.V);
          }
          uint64_t mine = 0;  // which of this lane's elements are above the floor
#pragma unroll
          for (int j = 0; j < kLoads; ++j) {
            float x[8];
            unpack<DT>(raw[j], x);
            const int32_t v0 = qs[j] * kDrawBlock + (int32_t)sub;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const bool above = qs[j] >= 0 && v0 + u < a.V && x[u] > floor_x;
              const float e = __builtin_amdgcn_exp2f(fmaf(x[u], a.k2, nrk_row));
              acc_m += above ? e : 0.0f;
              acc_n += above ? 1.0f : 0.0f;  // counts stay exact in fp32: V < 2^24
              mine |= above ? 1ull << (j * 8 + u) : 0ull;
            }
          }
          // one counter update per lane that has any; its logits take consecutive entries
          int c = mine != 0 ? atomicAdd(sh.ncand, (int)__builtin_popcountll(mine)) : 0;
#pragma unroll
          for (int j = 0; j < kLoads; ++j) {
            if (((mine >> (j * 8)) & 0xffull) == 0) continue;
            float x[8];
            unpack<DT>(raw[j], x);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              if ((mine >> (j * 8 + u)) & 1ull) {
                if (c < kKeptCap) kept_x[c] = x[u];
                ++c;
              }
            }
          }
        }
      } else {  // many blocks: stream the row once more, six loads in flight per lane
        constexpr int kDeep = 6;
#pragma unroll 1
        for (int i0 = 0; i0 < my_tiles; i0 += kDeep) {
          Raw<DT> raw[kDeep];
#pragma unroll
          for (int d = 0; d < kDeep; ++d)
            if (i0 + d < my_tiles) raw[d] = load_tile((i0 + d) * kStepWaves + wave);
#pragma unroll
          for (int d = 0; d < kDeep; ++d) {
            if (i0 + d < my_tiles) {
              float x[8];
              unpack<DT>(raw[d], x);
              const int32_t e0 = ((i0 + d) * kStepWaves + wave) * kTile + (int32_t)lane_off;
              const bool room = *sh.ncand <= kKeptCap;  // once the buffer has overflowed nothing more is kept
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                const bool above = e0 + u < a.V && x[u] > floor_x;
                const float e = __builtin_amdgcn_exp2f(fmaf(x[u], a.k2, nrk_row));
                acc_m += above ? e : 0.0f;
                acc_n += above ? 1.0f : 0.0f;
                const uint64_t who = __builtin_amdgcn_ballot_w64(above);
                if (who != 0 && room) {  // one counter update per wave, the lanes take consecutive entries
                  int base = 0;
                  if (lane == (int)__builtin_ctzll(who)) base = atomicAdd(sh.ncand, (int)__builtin_popcountll(who));
                  base = __builtin_amdgcn_readlane(base, (int)__builtin_ctzll(who));
                  const int c = base + (int)__builtin_popcountll(who & ((1ull << lane) - 1ull));
                  if (above && c < kKeptCap) kept_x[c] = x[u];
                }
              }
            }
          }
        }
      }
      acc_m = wave_sum(acc_m);
      acc_n = wave_sum(acc_n);
      if (lane == 0) {
        sh.res_s[wave] = (double)acc_m;
        sh.fres[wave] = acc_n;
      }
      __syncthreads();
      mass = 0.0f;
      count = 0.0f;
      for (int w = 0; w < kStepWaves; ++w) {  // fixed order, the same in every thread
        mass += (float)sh.res_s[w];
        count += sh.fres[w];
      }
      ncand = *sh.ncand;
    };

    // The smallest kept logit among the collected ones (all logits above floor_x, which lies below the
    // kept set): the smallest candidate whose strictly larger candidates hold less than p (number
    // fewer than k).  False if a sum is too close to p to tell in fp32, or if the method at hand
    // does not fit.  A few hundred candidates are compared all with all.  More of them are first
    // binned by their distance from the row's largest logit (256 bins of equal width down to the
    // floor): the bins' weights, summed from the top, name the one bin in which
    // the edge lies, and only that bin's candidates are compared with each other.  Weights are
    // integers there (2^t in units of 2^-31 of the measured mass, or 1 for top-k), so the sums do
    // not depend on the order in which the candidates arrive.
    constexpr int kPairwise = 256, kBins = 256, kMembers = 256;
    auto kept_edge = [&](float floor_x, float& edge_sure, float& edge_maybe) {
      // this thread's candidate if it is kept for sure / if it may be kept, else +inf
      float mine_sure = __builtin_huge_valf(), mine_maybe = __builtin_huge_valf();
      const float slack = by_count ? 0.0f : 1e-5f * total;  // what an fp32 sum may be off by
      const bool binned = ncand > kPairwise && nslots >= kBins + 2 * kMembers && (by_count || mass > 0.0f) && floor_x > kNegInf;
      if (!binned) {
        if (ncand > kCandCap) return false;
        float* const cand_e = kept_x + kCandCap;  // the candidates' 2^t, in the half that their logits leave free
        for (int c = tid; c < ncand; c += kStepThreads) cand_e[c] = __builtin_amdgcn_exp2f(fmaf(kept_x[c], a.k2, nrk_row));
        __syncthreads();
        for (int c = tid; c < ncand; c += kStepThreads) {  // at most one per thread
          const float xc = kept_x[c];
          float m_above = 0.0f, n_above = 0.0f;
          // every thread reads the same entries (LDS broadcasts), four at a time and several
          // reads in flight: one entry per dependent read would cost a microsecond per ten candidates
          const int whole = ncand & ~3;
#pragma unroll 4
          for (int o = 0; o < whole; o += 4) {
            const f32x4 xo = *(const f32x4*)(kept_x + o), eo = *(const f32x4*)(cand_e + o);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const bool larger = xo[u] > xc;
              m_above += larger ? eo[u] : 0.0f;
              n_above += larger ? 1.0f : 0.0f;
            }
          }
          for (int o = whole; o < ncand; ++o) {
            const bool larger = kept_x[o] > xc;
            m_above += larger ? cand_e[o] : 0.0f;
            n_above += larger ? 1.0f : 0.0f;
          }
          if (by_count ? n_above < (float)a.top_k : m_above < want - slack) mine_sure = xc;
          if (by_count ? n_above < (float)a.top_k : m_above < want + slack) mine_maybe = xc;
        }
      } else {
        // the survivor list of the measurement is over: its words hold the bins and the edge bin's members
        uint32_t* const words = (uint32_t*)sh.mu;
        auto bin_w = [&](int b) -> uint32_t& { return words[2 * b]; };
        auto mem_x = [&](int i) -> float& { return ((float*)words)[2 * (kBins + i)]; };
        auto mem_w = [&](int i) -> uint32_t& { return words[2 * (kBins + kMembers + i)]; };
        const float per_logit = (float)kBins / (m - floor_x);  // bins of equal width between the floor and the row's largest logit
        const float scale = by_count ? 1.0f : 2147483648.0f / (mass * 1.001f);
        // what may be kept has less than `limit` above it, what is kept for sure less than `limit_sure`
        const float limit_f = by_count ? (float)a.top_k : (want + slack) * scale;
        const float limit_sure_f = by_count ? (float)a.top_k : (want - slack) * scale;
        const uint32_t limit = limit_f < 1.0f ? 1u : limit_f < 4.0e9f ? (uint32_t)limit_f : 4000000000u;
        const uint32_t limit_sure = limit_sure_f < 1.0f ? 1u : limit_sure_f < 4.0e9f ? (uint32_t)limit_sure_f : 4000000000u;
        if (tid < kBins) bin_w(tid) = 0;
        if (tid == 0) *sh.nsurv = 0;
        __syncthreads();
        float cx[kKeptCap / kStepThreads];
        uint32_t cw[kKeptCap / kStepThreads];
        int cb[kKeptCap / kStepThreads];
#pragma unroll
        for (int i = 0; i < kKeptCap / kStepThreads; ++i) {
          const int c = tid + i * kStepThreads;
          cb[i] = -1;
          if (c < ncand) {
            cx[i] = kept_x[c];
            cw[i] = by_count ? 1u : (uint32_t)(__builtin_amdgcn_exp2f(fmaf(cx[i], a.k2, nrk_row)) * scale + 0.5f);
            const int b = (int)((m - cx[i]) * per_logit);  // rounding is monotone: a larger logit never lands in a later bin
            cb[i] = b < kBins ? b : kBins - 1;
            atomicAdd(&bin_w(cb[i]), cw[i]);
          }
        }
        __syncthreads();
        // every wave for itself: the weight above each bin, and the last bins that have candidates and less
        // than the two limits above them: the two edges lie in these bins or between them (nearly always one bin)
        static_assert(kBins == 4 * kWave, "four bins per lane");
        uint32_t h[4], above[4];
        uint32_t lane_total = 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          h[u] = bin_w(4 * lane + u);
          lane_total += h[u];
        }
        uint32_t incl = lane_total;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
          const uint32_t up = __shfl_up(incl, d);
          if (lane >= d) incl += up;
        }
        above[0] = incl - lane_total;
#pragma unroll
        for (int u = 1; u < 4; ++u) above[u] = above[u - 1] + h[u - 1];
        float best = -1.0f, best_sure = -1.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (h[u] != 0 && above[u] < limit) best = (float)(4 * lane + u);
          if (h[u] != 0 && above[u] < limit_sure) best_sure = (float)(4 * lane + u);
        }
        const int last_bin = (int)wave_max(best);        // the bin of the largest candidate at least: nothing is above it
        const int edge_bin = (int)wave_max(best_sure);   // not after last_bin: its limit is the smaller one
        const int u_sel = edge_bin & 3;
        const uint32_t above_sel = u_sel == 0 ? above[0] : u_sel == 1 ? above[1] : u_sel == 2 ? above[2] : above[3];
        const uint32_t above_edge_bin = __shfl(above_sel, edge_bin >> 2);
#pragma unroll
        for (int i = 0; i < kKeptCap / kStepThreads; ++i) {
          if (cb[i] >= edge_bin && cb[i] <= last_bin) {
            const int k = atomicAdd(sh.nsurv, 1);
            if (k < kMembers) {
              mem_x(k) = cx[i];
              mem_w(k) = cw[i];
            }
          }
        }
        __syncthreads();
        const int members = *sh.nsurv;
        if (members > kMembers) return false;  // (uniform) a bin of ties, or of many close logits
        // (the largest candidate of the next bin after last_bin that has any has the limit at least above
        // it: it is not kept, nor is anything after it; everything before edge_bin is kept for sure)
        if (tid < members) {
          const float xc = mem_x(tid);
          uint32_t w_above = above_edge_bin;
#pragma unroll 4
          for (int o = 0; o < members; ++o) w_above += mem_x(o) > xc ? mem_w(o) : 0u;
          const float m_above = (float)w_above / scale;
          if (by_count ? w_above < (uint32_t)a.top_k : m_above < want - slack) mine_sure = xc;
          if (by_count ? w_above < (uint32_t)a.top_k : m_above < want + slack) mine_maybe = xc;
        }
      }
      const float wave_sure = -wave_max(-mine_sure), wave_maybe = -wave_max(-mine_maybe);  // the wave's smallest ones
      __syncthreads();  // the sums of the measurement have been read by everyone
      if (lane == 0) {
        sh.fres[wave] = wave_sure;
        sh.fres[kStepWaves + wave] = wave_maybe;
      }
      __syncthreads();
      edge_sure = __builtin_huge_valf();
      edge_maybe = __builtin_huge_valf();
      for (int w = 0; w < kStepWaves; ++w) {
        edge_sure = fminf(edge_sure, sh.fres[w]);
        edge_maybe = fminf(edge_maybe, sh.fres[kStepWaves + w]);
      }
      return edge_maybe < __builtin_huge_valf();
    };

    // The winner among everything that may be kept (the floor is the next float below that edge).  If
    // its logit is kept for sure it is the token: leaving out the logits in doubt would not change the
    // winner.  Else (seldom: the winner is one of the few logits whose sums are too close to p to
    // tell in fp32) false, and the loop below tests that winner in double.
    auto winner_above = [&](float edge_sure, float edge_maybe) {
      StepShared kept_only = sh;
      kept_only.floor = next_below(edge_maybe);
      search(kept_only, nothing);
      return tok < 0 || x_a >= edge_sure;
    };

    bool done = !(m > kNegInf);
    float edge_known = kNegInf, edge_open = kNegInf;  // the edge of the kept set for sure, and the smallest logit that may be kept
    bool have_edge = false;
    if (!done && a.top_k == 1) {  // greedy decoding up to ties: the kept set is the row's largest logit
      edge_known = edge_open = m;
      have_edge = true;
    } else if (!done) {
      // a floor with about 64 blocks above it, the 64th largest of the 128 lane groups' largest logits
      // (for top-k the (32 + k)-th: k logits have to lie above it).  Measured, 32 is 2 us faster on rows
      // whose nucleus is a few dozen tokens and 10 to 30 us slower where it is a few hundred.  If the
      // kept set turns out to reach below that floor (a flat row), the smallest of the 128 is tried:
      // several hundred blocks lie above it, and a nucleus of some hundred tokens still does.
      __syncthreads();
      constexpr int kVals = 2 * kSlots;  // two values per lane group: its even and its odd tiles
      if ((lane & 7) == 0) {
        sh.cand_x[2 * (wave * kGroups + grp)] = mx_even;
        sh.cand_x[2 * (wave * kGroups + grp) + 1] = mx_odd;
      }
      if (tid < kVals) sh.cand_v[tid] = 0;  // the ranks, summed from partial counts
      __syncthreads();
      const int trial_rank = by_count ? (a.top_k < kVals - 32 ? 31 + a.top_k : kVals - 1) : kVals / 2 - 1;
      {
        constexpr int kParts = kStepThreads / kVals, kOthers = kVals / kParts;  // threads per value, values each of them compares with
        static_assert(kStepThreads % kVals == 0 && kVals % kParts == 0 && kOthers % 4 == 0, "the values are shared out evenly, four at a time");
        const int j = tid & (kVals - 1), part = tid / kVals;
        const float mine = sh.cand_x[j];
        int r = 0;
#pragma unroll
        for (int q = 0; q < kOthers / 4; ++q) {
          const f32x4 o4 = ((const f32x4*)sh.cand_x)[part * (kOthers / 4) + q];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int o = part * kOthers + q * 4 + u;
            r += (o4[u] > mine || (o4[u] == mine && o < j)) ? 1 : 0;
          }
        }
        atomicAdd(&sh.cand_v[j], r);
      }
      __syncthreads();
      if (tid < kVals) {  // -inf if fewer lane groups than that saw a finite logit
        if (sh.cand_v[tid] == trial_rank) sh.fres[2 * kStepWaves] = sh.cand_x[tid];
        if (sh.cand_v[tid] == kVals - 1) sh.fres[2 * kStepWaves + 1] = sh.cand_x[tid];
      }
      __syncthreads();
      const float trials[2] = {sh.fres[2 * kStepWaves], sh.fres[2 * kStepWaves + 1]};
#pragma unroll 1
      for (int attempt = 0; attempt < 2; ++attempt) {
        if (attempt == 1 && !(trials[1] < trials[0])) break;
        const float trial = attempt == 0 ? trials[0] : trials[1];
        measure(trial);
        const bool below_edge = by_count ? count >= (float)a.top_k : mass - want > 1e-5f * total;
        if (below_edge) {  // every kept logit has been seen; a lower floor could only add to them
          if (ncand <= kKeptCap) have_edge = kept_edge(trial, edge_known, edge_open);
          break;
        }
      }
    }
    if (have_edge) {  // the kept set is everything at or above the edge
      done = winner_above(edge_known, edge_open);
    } else if (!done) {
      search(sh, nothing);  // the unfiltered winner, for the loop below
    }
    while (!done && tok >= 0) {
      const float floor_x = x_a;
      measure(floor_x);
      bool kept;
      if (by_count) {
        kept = count < (float)a.top_k;
      } else if (fabsf(mass - want) > 1e-5f * total) {
        kept = mass < want;
      } else {  // too close for fp32: the same two sums in double, y and y_max formed as the oracle forms them
        const double inv = (double)a.inv_tau, y_max = (double)m * inv;
        double dm = 0.0, ds = 0.0;
#pragma unroll 1
        for (int i = 0; i < my_tiles; ++i) {
          const int t = i * kStepWaves + wave;
          const Raw<DT> raw = load_tile(t);
          float x[8];
          unpack<DT>(raw, x);
          const int32_t e0 = t * kTile + (int32_t)lane_off;
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (e0 + u < a.V && x[u] > kNegInf) {
              const double e = exp((double)x[u] * inv - y_max);
              ds += e;
              if (x[u] > floor_x) dm += e;
            }
          }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
          dm += __shfl_xor(dm, off);
          ds += __shfl_xor(ds, off);
        }
        __syncthreads();
        if (lane == 0) {
          sh.res_s[wave] = dm;
          sh.res_hi2[wave] = ds;
        }
        __syncthreads();
        double dmass = 0.0, dtotal = 0.0;
        for (int w = 0; w < kStepWaves; ++w) {
          dmass += sh.res_s[w];
          dtotal += sh.res_hi2[w];
        }
        kept = dmass < (double)a.top_p * dtotal;
      }
      if (kept) break;
      if (ncand <= kKeptCap) {  // every logit above the winner's is at hand
        float edge, open_edge;
        if (kept_edge(floor_x, edge, open_edge)) {
          if (winner_above(edge, open_edge)) break;  // that winner is kept by construction
          continue;                                  // or it is in doubt: tested next
        }
      }
      StepShared above = sh;  // the bulk case, or a sum too close to tell: the next winner above the floor
      above.floor = floor_x;
      search(above, nothing);
    }
  }

  // ------------------------------------------------------------ finalize: one lane
  if (wave != 0) return;
  float S = wave_sum(lane < kStepWaves ? sh.sum[lane] : 0.0f);  // sum_v exp((x_v - m)/tau) over the chunk, fixed order
  float Sw = 0.0f;
  if constexpr (Entropy) Sw = wave_sum(lane < kStepWaves ? sh.sumw[lane] : 0.0f);
  if constexpr (!Filter) {
    if (nch > 1) {
      // A row split over nch workgroups: each leaves its chunk's result in the workspace and takes a
      // ticket; the one that takes the row's last ticket finishes the row.  Results, tickets and the
      // reads of the results all go through device-scope atomic accesses, which bypass the caches that
      // are private to a part of the chip, and a workgroup takes its ticket only once its stores have
      // been acknowledged, so whoever sees the last ticket also sees every result.  (A device-scope
      // fence would do too, but writes back and invalidates a whole L2 per workgroup: measured, 50 ns
      // of serialised work per workgroup, 100 us per launch.)  atomicInc wraps to zero at nch - 1, so
      // the ticket is ready for the next launch without anyone clearing it.
      uint32_t arrived = 0;
      if (lane == 0) {
        uint32_t* const dst = (uint32_t*)(a.partials + (size_t)unit);
        const uint32_t w[7] = {__builtin_bit_cast(uint32_t, m),   __builtin_bit_cast(uint32_t, S),   __builtin_bit_cast(uint32_t, Sw),
                               __builtin_bit_cast(uint32_t, s_a), __builtin_bit_cast(uint32_t, e_a), __builtin_bit_cast(uint32_t, x_a),
                               (uint32_t)tok};
#pragma unroll
        for (int j = 0; j < 7; ++j) __hip_atomic_store(dst + j, w[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stores are done before the ticket is taken
        arrived = atomicInc(a.tickets + row, (uint32_t)(nch - 1));
      }
      arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)arrived);
      if (arrived != (uint32_t)(nch - 1)) return;
      if (lane == 0) {
        z_prev = a.z[row];
        value = a.values[row];
      }
      // lane c holds chunk c (nch <= 64); the other lanes hold a chunk without any finite logit
      float m_c = kNegInf, S_c = 0.0f, Sw_c = 0.0f;
      Best win = no_best();
      if (lane < nch) {
        const uint32_t* src = (const uint32_t*)(a.partials + (size_t)row * nch + lane);
        uint32_t w[7];
#pragma unroll
        for (int j = 0; j < 7; ++j) w[j] = __hip_atomic_load(src + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // hand the workspace back as it came: all zero (the tickets clear themselves), so that a later call of
        // another shape, whose tickets may lie where these results were, can use the same buffer
        u32x4* const back = (u32x4*)(a.partials + (size_t)row * nch + lane);
        back[0] = u32x4{0u, 0u, 0u, 0u};
        back[1] = u32x4{0u, 0u, 0u, 0u};
        m_c = __builtin_bit_cast(float, w[0]);
        S_c = __builtin_bit_cast(float, w[1]);
        Sw_c = __builtin_bit_cast(float, w[2]);
        win.s = __builtin_bit_cast(float, w[3]);
        win.e = __builtin_bit_cast(float, w[4]);
        win.x = __builtin_bit_cast(float, w[5]);
        win.v = (int32_t)w[6];
        if (win.v < 0) win = no_best();
      }
      m = wave_max(m_c);
      // the chunks' sums are relative to their own maxima: moved to the row maximum like a lane's in phase 1
      const float shift = (m_c - m) * a.k2;
      const float f = __builtin_amdgcn_exp2f(shift);
      S = wave_sum(S_c > 0.0f ? S_c * f : 0.0f);
      if constexpr (Entropy) Sw = wave_sum(S_c > 0.0f ? f * fmaf(shift, S_c, Sw_c) : 0.0f);
      // every chunk's winner is its exact argmax, so the row's is the best of them: decided in fp32
      // where the margins allow, else by scoring those few indices in double
      const Best top = wave_best(win);
      tok = top.v;
      x_a = top.x;
      if (top.v >= 0 && !(top.s - top.e > top.hi2)) {
        Search<double> st;
        st.init();
        if (win.v >= 0) {
          const BlockDraw<double> d = block_draw<double>(a, row, win.v >> 6);
          score_index<double>(a, row, win.v, win.x, d, -__builtin_huge_val(), kNegInf, st);
        }
        st = wave_merge(st);
        tok = st.best.v;
        x_a = st.best.x;
      }
    }
  }
  if (lane == 0) {
    if (tok < 0) { tok = 0; x_a = elem_at<DT>(rowp, 0); }  // row of -inf only: unspecified, stay in range
    const ChainOut c = scalar_chain(a, row, m, x_a, z_prev, value);
    a.tokens[row] = tok;
    a.regret[row] = c.g;
    a.z[row] = c.z;
    if (Sum && a.logprob) a.logprob[row] = -c.g - flog(S);
    if constexpr (Entropy)  // H = ln S - E_pi[y - y_max] >= 0; rounding can leave S a few ulp below 1
      a.entropy[row] = fmaxf(flog(S) - kLn2 * Sw / S, 0.0f);
    if (a.eos_id >= 0 && tok == a.eos_id) {
      a.alive[row] = 0;  // natural end
    } else if (c.stop) {
      if (a.simulate) {  // bookkeeping only: the first stop step is recorded, decoding goes on
        if (a.stop_step[row] < 0) a.stop_step[row] = a.step;
      } else {
        a.alive[row] = 0;  // absorbing failure (Eq. failure_reward): the trajectory ends here
        a.stop_step[row] = a.step;
      }
    }
  }
}

// Measures what score_margin assumes about the hardware transcendentals: the largest relative
// error of flog over every u(w) and over positive floats from 2^-26 to 64, and of fexp over
// [-40, 8], against the double-precision library functions.  out[0..2] hold the maxima as
// float bit patterns (non-negative floats order like unsigned integers).
__global__ void math_error_kernel(uint32_t* out) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;  // 2^23 threads
  float e_u = 0.0f, e_ln = 0.0f, e_exp = 0.0f;
  {
    const float u = (float)(2u * i + 1u) * (1.0f / 16777216.0f);  // every value u(w) takes
    const double ref = log((double)u);
    e_u = (float)fabs(((double)flog(u) - ref) / ref);
  }
  {
    // exponents -26..5 (32 of them), 2^18 mantissas each, spread over the 2^23 mantissa values
    const uint32_t bits = ((101u + (i >> 18)) << 23) | ((i & 0x3ffffu) * 32u + (i >> 18));
    const float x = __builtin_bit_cast(float, bits);
    const double ref = log((double)x);
    if (x != 1.0f) e_ln = (float)fabs(((double)flog(x) - ref) / ref);
  }
  {
    const float x = -40.0f + 48.0f * ((float)i * (1.0f / 8388608.0f));
    const double ref = exp((double)x);
    e_exp = (float)fabs(((double)fexp(x) - ref) / ref);
  }
  e_u = wave_max(e_u);
  e_ln = wave_max(e_ln);
  e_exp = wave_max(e_exp);
  if ((threadIdx.x & (kWave - 1)) == 0) {
    atomicMax(out + 0, __builtin_bit_cast(uint32_t, e_u));
    atomicMax(out + 1, __builtin_bit_cast(uint32_t, e_ln));
    atomicMax(out + 2, __builtin_bit_cast(uint32_t, e_exp));
  }
}

}  // namespace

int launch_math_errors(float* out, hipStream_t stream) {
  hipLaunchKernelGGL(math_error_kernel, dim3(1u << 15), dim3(256), 0, stream, (uint32_t*)out);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

// ---------------------------------------------------------------- launch configuration
// How a call is laid out on the GPU.  One workgroup streams a whole row: 8 waves, three workgroups to a
// compute unit, from 256 rows on; 16 waves, two to a compute unit, for smaller batches, where a
// compute unit has one row at most and more waves stream it faster (B = 128: 17.0 against 18.5 us).
// With every row live the two are within 1 us of each other from B = 256 to 4096; with rows that are
// done in the batch the smaller workgroups are 2 to 5 us faster (B = 1024 with 431 live rows: 36.8
// against 41.7 us; B = 512 with 446: 30.6 against 32.9): workgroups are dispatched in order, and with
// only 512 slots live rows further back in the batch wait for one (timestamps: a tenth of them start
// more than 8 us late); with 768 slots all have started within 4 us.  A filtered draw always runs 8 waves, with
// twice the registers each.  The diagnostics
// entry point can force fewer waves per workgroup and a split of every row into `chunks` runs of
// tiles, each streamed by a workgroup of its own and combined by the last one to arrive.  Measured on
// an MI355X (B = 512, V = 152064 bf16, all rows live): 34.7 us unsplit, 41 us in 2 chunks of 16 waves,
// 39.6 us in 2 chunks of 8 waves, 53 us in 8 chunks of 4 waves: every chunk pays for a search of its
// own and the row for one more round trip through memory (ticket, then the partial results), which is
// more than the finer grain gains, so the library itself never splits.  (Also measured and left out:
// 512 resident workgroups that claim rows from a counter in the workspace instead of one workgroup
// per row, meant to make rows that are done cost a claim instead of a workgroup: 512 device-scope
// atomics on one address take 50 ns each, and a launch of B = 1024 live rows went from 56 to 82 us.)

// tickets first (256-byte aligned size), then the chunk results
size_t step_workspace_layout(int64_t B, int chunks, size_t* partials_offset) {
  const size_t tickets = (((size_t)B * sizeof(uint32_t)) + 255) & ~(size_t)255;
  if (partials_offset) *partials_offset = tickets;
  return tickets + (size_t)B * (size_t)chunks * sizeof(ChunkResult);
}

constexpr int64_t kEightWavesFrom = 256;

StepPlan plan_step(int dt, int64_t B, int64_t V, bool filter, int waves, int chunks) {
  StepPlan p;
  const int ntiles = (int)((V + kTile - 1) / kTile);
  p.waves = waves > 0 ? waves : filter || B >= kEightWavesFrom ? 8 : 16;
  int nch = filter || chunks <= 0 ? 1 : chunks;
  if (nch > ntiles) nch = ntiles;
  if (nch > kMaxChunks) nch = kMaxChunks;
  p.chunks = nch;
  p.grid = B * nch;
  const int ctiles = (ntiles + nch - 1) / nch;
  p.lds = step_lds_bytes(dt, ctiles, filter, p.waves);
  p.workspace = nch > 1 ? step_workspace_layout(B, nch, nullptr) : 0;
  return p;
}

template <int DT, int W>
void (*pick_kernel(bool sum, bool filter, bool entropy))(StepArgs) {
  if constexpr (W == 8) {
    if (filter) return entropy ? espo_step_kernel<DT, true, true, true, 8> : espo_step_kernel<DT, false, true, true, 8>;
  }
  if (!sum) return espo_step_kernel<DT, false, false, false, W>;
  return entropy ? espo_step_kernel<DT, true, false, true, W> : espo_step_kernel<DT, false, false, true, W>;
}

int launch_step(const void* logits, int dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const espo_params& p, float margin_scale,
                float* z, uint8_t* alive, int32_t* stop_step, int32_t* tokens, float* regret, float* logprob,
                float* entropy, void* workspace, const StepPlan& plan, hipStream_t stream) {
  StepArgs a;
  a.logits = logits;
  a.V = (int32_t)V;
  a.row_stride = row_stride;
  a.ntiles = (int)((V + kTile - 1) / kTile);
  a.nblocks = (int)((V + kDrawBlock - 1) / kDrawBlock);
  a.inv_tau = 1.0f / temperature;
  a.k2 = a.inv_tau * kLog2e;
  a.ref_lead = kRescaleAt / a.k2;
  a.margin_scale = margin_scale;
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
  a.stop_mode = p.stop_mode;
  a.simulate = p.simulate;
  a.stop_threshold = p.stop_threshold;
  a.top_p = p.top_p;
  a.top_k = p.top_k;
  a.z = z;
  a.alive = alive;
  a.stop_step = stop_step;
  a.tokens = tokens;
  a.regret = regret;
  a.logprob = logprob;
  a.entropy = entropy;
  a.nch = plan.chunks;
  a.partials = nullptr;
  a.tickets = nullptr;
  if (plan.chunks > 1) {
    size_t off = 0;
    step_workspace_layout(B, plan.chunks, &off);
    a.tickets = (uint32_t*)workspace;
    a.partials = (ChunkResult*)((char*)workspace + off);
  }

  // the entropy output costs two more vector operations per logit: its own instantiation
  // and so does a filtered draw (more passes over the row)
  const bool filter = (p.top_p > 0.0f && p.top_p < 1.0f) || p.top_k > 0;
  if (plan.lds > kMaxStepLds) return ESPO_ERANGE;
  if (filter && (plan.waves != 8 || plan.chunks != 1)) return ESPO_EINVAL;
  if (plan.chunks > a.ntiles || plan.chunks > kMaxChunks || (int64_t)B * plan.chunks > 0x7fffffff) return ESPO_ERANGE;
  // and a step that is asked for neither log-probabilities nor either of these needs no softmax sum at all
  const bool sum = logprob != nullptr || entropy != nullptr || filter;
  void (*kernel)(StepArgs) = nullptr;
  const bool ent = entropy != nullptr;
  if (dt == ESPO_BF16)
    kernel = plan.waves == 16 ? pick_kernel<ESPO_BF16, 16>(sum, filter, ent)
             : plan.waves == 8 ? pick_kernel<ESPO_BF16, 8>(sum, filter, ent)
             : plan.waves == 4 ? pick_kernel<ESPO_BF16, 4>(sum, filter, ent) : nullptr;
  else
    kernel = plan.waves == 16 ? pick_kernel<ESPO_F32, 16>(sum, filter, ent)
             : plan.waves == 8 ? pick_kernel<ESPO_F32, 8>(sum, filter, ent)
             : plan.waves == 4 ? pick_kernel<ESPO_F32, 4>(sum, filter, ent) : nullptr;
  if (!kernel) return ESPO_EINVAL;
  if (plan.lds > 64 * 1024) {  // beyond the default limit the kernel has to be told (very large vocabularies)
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxStepLds) != hipSuccess)
      return ESPO_EHIP;
  }
  const dim3 grid((unsigned)plan.grid), block((unsigned)(plan.waves * kWave));
  hipLaunchKernelGGL(kernel, grid, block, plan.lds, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
