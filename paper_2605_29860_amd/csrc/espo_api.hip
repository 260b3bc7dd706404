// C ABI of the library: argument validation and dispatch.  Every entry point is declared
// and documented in include/espo.h.
#include <hip/hip_runtime.h>
#include <math.h>

#include "../../include/espo.h"
#include "../../include/espo_debug.h"
#include "espo_host.h"

namespace {

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Plain streaming copy, 16 bytes per lane: reads n16*16 bytes once and writes them once.
typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_kernel(copy_u32x4* __restrict__ dst, const copy_u32x4* __restrict__ src, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

// Bare streaming read: every lane keeps eight nontemporal 16-byte loads in flight over a span of
// 32 KB per workgroup and folds what arrives into one word, which is stored only if it takes a value
// that the fold cannot produce for the caller's data in practice (so nothing is written, yet the
// loads cannot be dropped).
constexpr int kReadLoads = 8;
__global__ __launch_bounds__(256) void read_kernel(const copy_u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * (256 * kReadLoads) + threadIdx.x;
  copy_u32x4 v[kReadLoads];
#pragma unroll
  for (int j = 0; j < kReadLoads; ++j) {
    const size_t i = base + (size_t)j * 256;
    v[j] = i < n16 ? __builtin_nontemporal_load(src + i) : copy_u32x4{0u, 0u, 0u, 0u};
  }
  unsigned acc = 0;
#pragma unroll
  for (int j = 0; j < kReadLoads; ++j) acc |= (v[j].x ^ v[j].y) + (v[j].z ^ v[j].w);
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

// Flat sweep with a given read / write mix and no dependency between elements: lane i reads the i-th
// 16 bytes of src (while there are any) and writes the i-th 16 bytes of dst (while there are any),
// nontemporal both ways.
__global__ __launch_bounds__(256) void sweep_kernel(const copy_u32x4* __restrict__ src, size_t nr, copy_u32x4* __restrict__ dst, size_t nw) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  copy_u32x4 v = copy_u32x4{(unsigned)i, 1u, 2u, 3u};
  if (i < nr) v = __builtin_nontemporal_load(src + i);
  if (i < nw) __builtin_nontemporal_store(v, dst + i);
}

// The same traffic as espo_advantages in its own layout, with no dependency between elements: four [B, T]
// arrays, inputs read below each row's length, both outputs written everywhere.  The grid covers the batch
// twice: its first half writes the zeros beyond the lengths, its second half does the rest (a phase of pure
// writes before the phase of reads and writes measured faster than the two mixed: 37.5 against 40 us on
// the B = 1024, T = 16384 batch).  T is a multiple of 1024.
__global__ __launch_bounds__(256) void sweep_padded_kernel(const float* __restrict__ r, const float* __restrict__ v,
                                                           const int32_t* __restrict__ lengths, float* __restrict__ td,
                                                           float* __restrict__ adv, int64_t B, int64_t T) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int64_t per_row = T / 1024, half = B * per_row;
  const bool fill = (int64_t)blockIdx.x < half;
  const int64_t id = fill ? (int64_t)blockIdx.x : (int64_t)blockIdx.x - half;
  const int64_t row = id / per_row, t = (id - row * per_row) * 1024 + threadIdx.x * 4;
  int64_t L = lengths[row];
  L = L < 0 ? 0 : (L > T ? T : L);
  const int64_t off = row * T + t;
  if (fill) {
    if (t + 4 > L) {
      __builtin_nontemporal_store(f4{0, 0, 0, 0}, (f4*)(td + off));
      __builtin_nontemporal_store(f4{0, 0, 0, 0}, (f4*)(adv + off));
    }
  } else if (t + 4 <= L) {
    const f4 x = __builtin_nontemporal_load((const f4*)(r + off));
    const f4 y = __builtin_nontemporal_load((const f4*)(v + off));
    __builtin_nontemporal_store(x + y, (f4*)(td + off));
    __builtin_nontemporal_store(x - y, (f4*)(adv + off));
  }
}

bool filtered(const espo_params* p) { return (p->top_p > 0.0f && p->top_p < 1.0f) || p->top_k > 0; }

// Argument checks of espo_step and of its diagnostics twin; ESPO_OK means "go on", B == 0 is reported
// through *empty.  `waves`, `chunks`: 0 for the library's choice (see espo_debug_step).
int step_checked(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                 uint64_t seed, int32_t step, const float* values, const espo_params* params, float* z, uint8_t* alive,
                 int32_t* stop_step, int32_t* tokens, float* regret, float* logprob, float* entropy, void* workspace,
                 size_t workspace_bytes, float margin_scale, int waves, int chunks, void* stream) {
  if (dt != ESPO_F32 && dt != ESPO_BF16) return ESPO_EINVAL;
  if (B < 0 || V < 1 || row_stride < V || step < 0) return ESPO_EINVAL;
  if (!params) return ESPO_EINVAL;
  if (!(temperature > 0.0f) || !isfinite(temperature)) return ESPO_EINVAL;
  if (!(params->alpha_s >= 0.0f && params->alpha_s <= 1.0f)) return ESPO_EINVAL;
  if (!(params->var_g + params->delta > 0.0f) || !isfinite(params->var_g + params->delta)) return ESPO_EINVAL;
  if (!(params->clip_c >= 0.0f) || !(params->beta >= 0.0f) || isnan(params->eps) || isnan(params->mu_g)) return ESPO_EINVAL;
  if (params->stop_mode < ESPO_STOP_RULE || params->stop_mode > ESPO_STOP_RANDOM) return ESPO_EINVAL;
  if (params->stop_mode != ESPO_STOP_RULE && isnan(params->stop_threshold)) return ESPO_EINVAL;
  if (!(params->top_p >= 0.0f && params->top_p <= 1.0f) || params->top_k < 0) return ESPO_EINVAL;
  if (params->top_p > 0.0f && params->top_p < 1.0f && params->top_k > 0) return ESPO_EINVAL;  // one filter at a time
  if (!(margin_scale >= 1.0f)) return ESPO_EINVAL;  // below 1 the fp32 search would no longer be exact
  if (waves != 0 && waves != 4 && waves != 8 && waves != 16) return ESPO_EINVAL;
  if (chunks < 0) return ESPO_EINVAL;
  if (B == 0) return ESPO_OK;
  if (!logits || !values || !z || !alive || !stop_step || !tokens || !regret) return ESPO_EINVAL;
  if (V > espo::kMaxVocab || B > 0x7fffffff) return ESPO_ERANGE;
  const size_t esize = dt == ESPO_BF16 ? 2 : 4;
  if (!aligned16(logits) || ((size_t)row_stride * esize) % 16 != 0) return ESPO_EALIGN;
  const bool filter = filtered(params);
  if (filter && ((waves != 0 && waves != 8) || chunks > 1)) return ESPO_EINVAL;  // a filtered draw has one layout
  const espo::StepPlan plan = espo::plan_step(dt, B, V, filter, waves, chunks);
  if (plan.lds > espo::kMaxStepLds) return ESPO_ERANGE;
  if (plan.workspace > 0 && (!workspace || workspace_bytes < plan.workspace || !aligned16(workspace))) return ESPO_EWORKSPACE;
  return espo::launch_step(logits, dt, B, V, row_stride, temperature, seed, step, values, *params, margin_scale, z, alive,
                           stop_step, tokens, regret, logprob, entropy, workspace, plan, (hipStream_t)stream);
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int espo_version(void) { return 310; }

int espo_debug_step(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                    uint64_t seed, int32_t step, const float* values, const espo_params* params, float* z, uint8_t* alive,
                    int32_t* stop_step, int32_t* tokens, float* regret, float* logprob, float* entropy, void* workspace,
                    size_t workspace_bytes, void* stream, float score_margin_scale, int32_t waves, int32_t chunks) {
  return step_checked(logits, dt, B, V, row_stride, temperature, seed, step, values, params, z, alive, stop_step, tokens,
                      regret, logprob, entropy, workspace, workspace_bytes, score_margin_scale, waves, chunks, stream);
}

size_t espo_debug_step_workspace_bytes(int64_t B, int32_t chunks) {
  if (B <= 0 || chunks <= 1) return 0;
  return espo::step_workspace_layout(B, chunks, nullptr);
}

int espo_debug_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes % 16 != 0 || !aligned16(src)) return ESPO_EINVAL;
  if (bytes == 0) return ESPO_OK;
  const size_t n16 = bytes / 16, groups = (n16 + 256 * kReadLoads - 1) / (256 * kReadLoads);
  if (groups > 0x7fffffffu) return ESPO_ERANGE;
  hipLaunchKernelGGL(read_kernel, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream, (const copy_u32x4*)src, n16,
                     (unsigned*)sink);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

int espo_debug_sweep_padded(const float* rewards, const float* values, const int32_t* lengths, int64_t B, int64_t T,
                            float* td, float* adv, void* stream) {
  if (!rewards || !values || !lengths || !td || !adv || B < 0 || T < 0 || T % 1024 != 0) return ESPO_EINVAL;
  if (!aligned16(rewards) || !aligned16(values) || !aligned16(td) || !aligned16(adv)) return ESPO_EALIGN;
  if (B == 0 || T == 0) return ESPO_OK;
  if (2 * B * (T / 1024) > 0x7fffffff) return ESPO_ERANGE;
  hipLaunchKernelGGL(sweep_padded_kernel, dim3((unsigned)(2 * B * (T / 1024))), dim3(256), 0, (hipStream_t)stream, rewards, values,
                     lengths, td, adv, B, T);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

int espo_debug_sweep(const void* src, size_t read_bytes, void* dst, size_t write_bytes, void* stream) {
  if (!src || !dst || read_bytes % 16 != 0 || write_bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return ESPO_EINVAL;
  if (read_bytes == 0 && write_bytes == 0) return ESPO_OK;
  const size_t nr = read_bytes / 16, nw = write_bytes / 16, n = nr > nw ? nr : nw;
  if ((n + 255) / 256 > 0x7fffffffu) return ESPO_ERANGE;
  hipLaunchKernelGGL(sweep_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     (const copy_u32x4*)src, nr, (copy_u32x4*)dst, nw);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

int espo_debug_math_errors(float* out, void* stream) {
  if (!out) return ESPO_EINVAL;
  return espo::launch_math_errors(out, (hipStream_t)stream);
}

size_t espo_batch_stats_workspace_bytes(int64_t B, int64_t T) {
  (void)T;
  return espo::batch_stats_workspace(B);
}

int espo_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                     float mu_g, float var_g, float beta, const espo_batch_ctrl* ctrl, espo_batch_result* out,
                     void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || T < 0 || !ctrl || !out) return ESPO_EINVAL;
  if (!(ctrl->alpha_ema >= 0.0f && ctrl->alpha_ema <= 1.0f) || !(ctrl->beta_min <= ctrl->beta_max)) return ESPO_EINVAL;
  if (!isfinite(ctrl->eta_beta) || !isfinite(ctrl->target_rate) || !isfinite(mu_g) || !isfinite(var_g) || !isfinite(beta))
    return ESPO_EINVAL;
  if (B > 0 && (!lengths || !stopped || (T > 0 && !regret))) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x7fffffff) return ESPO_ERANGE;
  if (regret && !aligned16(regret)) return ESPO_EALIGN;
  if (((uintptr_t)out & 7u) != 0) return ESPO_EALIGN;
  if (B > 0 && (!workspace || workspace_bytes < espo::batch_stats_workspace(B) || ((uintptr_t)workspace & 7u) != 0))
    return ESPO_EWORKSPACE;
  return espo::launch_batch_stats(regret, lengths, stopped, B, T, mu_g, var_g, beta, *ctrl, out, workspace,
                                  (hipStream_t)stream);
}

int espo_batch_stats_static(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                            float mu_g, float var_g, float beta, const espo_batch_ctrl* ctrl, espo_batch_result* out,
                            void* stream) {
  if (B < 0 || T < 0 || !ctrl || !out) return ESPO_EINVAL;
  if (!(ctrl->alpha_ema >= 0.0f && ctrl->alpha_ema <= 1.0f) || !(ctrl->beta_min <= ctrl->beta_max)) return ESPO_EINVAL;
  if (!isfinite(ctrl->eta_beta) || !isfinite(ctrl->target_rate) || !isfinite(mu_g) || !isfinite(var_g) || !isfinite(beta))
    return ESPO_EINVAL;
  if (B > 0 && (!lengths || !stopped || (T > 0 && !regret))) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x7fffffff) return ESPO_ERANGE;
  if (regret && !aligned16(regret)) return ESPO_EALIGN;
  if (((uintptr_t)out & 7u) != 0) return ESPO_EALIGN;
  // the partial sums of this batch must fit the library's own scratch
  if (B > 0 && espo::batch_stats_workspace(B) > espo::batch_stats_static_capacity()) return ESPO_ERANGE;
  void* scratch_ptr = espo::batch_stats_static_scratch();
  if (!scratch_ptr) return ESPO_EHIP;
  return espo::launch_batch_stats(regret, lengths, stopped, B, T, mu_g, var_g, beta, *ctrl, out, scratch_ptr,
                                  (hipStream_t)stream);
}

size_t espo_whiten_workspace_bytes(int64_t B, int64_t T) {
  if (B <= 0 || T <= 0) return 0;
  return espo::whiten_workspace(B, T);
}

int espo_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int32_t shift_mean,
                int32_t unbiased, float* out, double* stats, void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || T < 0 || !(eps >= 0.0f) || !isfinite(eps)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!adv || !lengths || !out) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x7fffffff || B * ((T + 4095) / 4096) > 0x7fffffff) return ESPO_ERANGE;  // 2^31 items of 4096 tokens
  if (!aligned16(adv) || !aligned16(out) || ((uintptr_t)stats & 7u) != 0) return ESPO_EALIGN;
  if (!workspace || workspace_bytes < espo::whiten_workspace(B, T) || ((uintptr_t)workspace & 7u) != 0)
    return ESPO_EWORKSPACE;
  return espo::launch_whiten(adv, lengths, B, T, eps, shift_mean != 0, unbiased != 0, out, stats, workspace,
                             (hipStream_t)stream);
}

int espo_debug_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) return ESPO_EINVAL;
  if (bytes == 0) return ESPO_OK;
  const size_t n16 = bytes / 16;
  if ((n16 + 255) / 256 > 0x7fffffffu) return ESPO_ERANGE;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     (copy_u32x4*)dst, (const copy_u32x4*)src, n16);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

const char* espo_strerror(int code) {
  switch (code) {
    case ESPO_OK: return "success";
    case ESPO_EINVAL: return "invalid argument (null pointer, negative size, or parameter out of range)";
    case ESPO_EALIGN: return "logits/rewards/values base address or row pitch is not 16-byte aligned";
    case ESPO_EWORKSPACE: return "workspace missing, misaligned or too small";
    case ESPO_EHIP: return "the HIP runtime rejected the kernel launch";
    case ESPO_ERANGE: return "size exceeds what the kernels index";
    default: return "unknown espo status";
  }
}

size_t espo_step_workspace_bytes(int64_t B, int64_t V, espo_dtype dt) {
  if (B <= 0 || V < 1 || V > espo::kMaxVocab || (dt != ESPO_F32 && dt != ESPO_BF16)) return 0;
  return espo::plan_step(dt, B, V, false, 0, 0).workspace;
}

int espo_step(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride,
              float temperature, uint64_t seed, int32_t step, const float* values,
              const espo_params* params, float* z, uint8_t* alive, int32_t* stop_step,
              int32_t* tokens, float* regret, float* logprob, float* entropy, void* workspace,
              size_t workspace_bytes, void* stream) {
  return step_checked(logits, dt, B, V, row_stride, temperature, seed, step, values, params, z, alive, stop_step, tokens,
                      regret, logprob, entropy, workspace, workspace_bytes, 1.0f, 0, 0, stream);
}

int espo_advantages(const float* rewards, const float* values, const int32_t* lengths,
                    const uint8_t* stopped, int64_t B, int64_t T, float r_fail, float gamma, float lambda,
                    float* td, float* adv, void* stream) {
  if (B < 0 || T < 0) return ESPO_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda) || isnan(r_fail)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!rewards || !values || !lengths || !stopped || !td || !adv) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x3fffffff) return ESPO_ERANGE;  // the grid has 2 B workgroups
  if (!aligned16(rewards) || !aligned16(values) || !aligned16(td) || !aligned16(adv)) return ESPO_EALIGN;
  return espo::launch_advantages(rewards, nullptr, values, lengths, nullptr, 0, stopped, B, T, r_fail, gamma, lambda, 1, td, adv,
                                 nullptr, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

size_t espo_advantages_ws_bytes(int64_t B) {
  if (B <= 0) return 0;
  return espo::advantages_workspace_layout(B, nullptr, nullptr);
}

int espo_length_order(const int32_t* lengths, int64_t B, int64_t T, int32_t* order, void* stream) {
  if (B < 0 || T < 0) return ESPO_EINVAL;
  if (B == 0) return ESPO_OK;
  if (!lengths || !order) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x3fffffff) return ESPO_ERANGE;
  return espo::launch_length_order(lengths, B, T, order, (hipStream_t)stream);
}

int espo_advantages_ws(const float* rewards, const float* values, const int32_t* lengths, const uint8_t* stopped,
                       int64_t B, int64_t T, float r_fail, float gamma, float lambda, float* td, float* adv,
                       const int32_t* order, void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || T < 0) return ESPO_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda) || isnan(r_fail)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!rewards || !values || !lengths || !stopped || !td || !adv) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x3fffffff) return ESPO_ERANGE;  // the grid has 2 B workgroups
  if (!aligned16(rewards) || !aligned16(values) || !aligned16(td) || !aligned16(adv)) return ESPO_EALIGN;
  size_t stats_off = 0, sorted_off = 0;
  const size_t need = espo::advantages_workspace_layout(B, &stats_off, &sorted_off);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u) != 0) return ESPO_EWORKSPACE;
  return espo::launch_advantages(rewards, nullptr, values, lengths, nullptr, 0, stopped, B, T, r_fail, gamma, lambda, 1, td, adv,
                                 nullptr, order, (espo::AdvRowStats*)((char*)workspace + stats_off),
                                 (int32_t*)((char*)workspace + sorted_off), (uint32_t*)workspace, (hipStream_t)stream);
}

int espo_whiten_from_ws(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int32_t shift_mean,
                        int32_t unbiased, float* out, double* stats, const void* workspace, size_t workspace_bytes,
                        void* stream) {
  if (B < 0 || T < 0 || !(eps >= 0.0f) || !isfinite(eps)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!adv || !lengths || !out) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x7fffffff || B * ((T + 4095) / 4096) > 0x7fffffff) return ESPO_ERANGE;  // 2^31 items of 4096 tokens
  if (!aligned16(adv) || !aligned16(out) || ((uintptr_t)stats & 7u) != 0) return ESPO_EALIGN;
  size_t stats_off = 0;
  if (!workspace || workspace_bytes < espo::advantages_workspace_layout(B, &stats_off, nullptr) || ((uintptr_t)workspace & 15u) != 0)
    return ESPO_EWORKSPACE;
  return espo::launch_whiten_rows(adv, lengths, B, T, eps, shift_mean != 0, unbiased != 0, out, stats,
                                  (const espo::AdvRowStats*)((const char*)workspace + stats_off), (hipStream_t)stream);
}

int espo_advantages_terminal(const float* values, const int32_t* lengths, const uint8_t* stopped,
                             const float* terminal_reward, int64_t B, int64_t T, float r_fail, float gamma,
                             float lambda, int32_t zero_padding, float* td, float* adv, float* returns,
                             void* stream) {
  if (B < 0 || T < 0) return ESPO_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda) || isnan(r_fail)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!values || !lengths || !stopped || !terminal_reward || !td || !adv) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x3fffffff) return ESPO_ERANGE;  // with zero padding the grid has 2 B workgroups
  if (!aligned16(values) || !aligned16(td) || !aligned16(adv) || !aligned16(returns)) return ESPO_EALIGN;
  return espo::launch_advantages(nullptr, terminal_reward, values, lengths, nullptr, 0, stopped, B, T, r_fail, gamma, lambda,
                                 zero_padding != 0, td, adv, returns, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

int espo_advantages_terminal_ws(const float* values, const int32_t* lengths, const uint8_t* stopped,
                                const float* terminal_reward, int64_t B, int64_t T, float r_fail, float gamma,
                                float lambda, int32_t zero_padding, float* td, float* adv, float* returns,
                                const int32_t* order, void* workspace, size_t workspace_bytes, void* stream) {
  if (B < 0 || T < 0) return ESPO_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda) || isnan(r_fail)) return ESPO_EINVAL;
  if (B == 0 || T == 0) return ESPO_OK;
  if (!values || !lengths || !stopped || !terminal_reward || !td || !adv) return ESPO_EINVAL;
  if (T > 0x7fffffff || B > 0x3fffffff) return ESPO_ERANGE;  // with zero padding the grid has 2 B + 1 workgroups
  if (!aligned16(values) || !aligned16(td) || !aligned16(adv) || !aligned16(returns)) return ESPO_EALIGN;
  size_t stats_off = 0, sorted_off = 0;
  const size_t need = espo::advantages_workspace_layout(B, &stats_off, &sorted_off);
  if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15u) != 0) return ESPO_EWORKSPACE;
  return espo::launch_advantages(nullptr, terminal_reward, values, lengths, nullptr, 0, stopped, B, T, r_fail, gamma, lambda,
                                 zero_padding != 0, td, adv, returns, order, (espo::AdvRowStats*)((char*)workspace + stats_off),
                                 (int32_t*)((char*)workspace + sorted_off), (uint32_t*)workspace, (hipStream_t)stream);
}

int espo_advantages_packed(const float* rewards, const float* terminal_reward, const float* values,
                           const int64_t* cu_seqlens, const uint8_t* stopped, int64_t B, int64_t N, float r_fail,
                           float gamma, float lambda, float* td, float* adv, float* returns, void* stream) {
  if (B < 0 || N < 0) return ESPO_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda) || isnan(r_fail)) return ESPO_EINVAL;
  if (B == 0 || N == 0) return ESPO_OK;
  if ((rewards != nullptr) == (terminal_reward != nullptr)) return ESPO_EINVAL;  // exactly one form
  if (!values || !cu_seqlens || !stopped || !td || !adv) return ESPO_EINVAL;
  if (B > 0x7fffffff) return ESPO_ERANGE;
  if (!aligned16(rewards) || !aligned16(values) || !aligned16(td) || !aligned16(adv) || !aligned16(returns))
    return ESPO_EALIGN;
  return espo::launch_advantages(rewards, terminal_reward, values, nullptr, cu_seqlens, N, stopped, B, 0, r_fail, gamma,
                                 lambda, 0, td, adv, returns, nullptr, nullptr, nullptr, nullptr, (hipStream_t)stream);
}

}  // extern "C"
#pragma GCC visibility pop
