// C ABI of the library: argument validation and dispatch.  Every entry point is declared
// and documented in include/espo.h.
#include <hip/hip_runtime.h>
#include <math.h>

#include "../../include/espo.h"
#include "espo_host.h"

#include <atomic>

namespace {

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// Plain streaming copy, 16 bytes per lane: reads n16*16 bytes once and writes them once.
typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_kernel(copy_u32x4* __restrict__ dst, const copy_u32x4* __restrict__ src, size_t n16) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

std::atomic<float> g_margin_scale{1.0f};

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int espo_version(void) { return 200; }

int espo_debug_set_score_margin_scale(float scale) {
  if (!(scale >= 1.0f)) return ESPO_EINVAL;  // below 1 the fast path would no longer be exact
  g_margin_scale.store(scale);
  return ESPO_OK;
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
  (void)B; (void)V; (void)dt;
  return 0;  // a row is handled by a single workgroup: no inter-workgroup scratch
}

int espo_step(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride,
              float temperature, uint64_t seed, int32_t step, const float* values,
              const espo_params* params, float* z, uint8_t* alive, int32_t* stop_step,
              int32_t* tokens, float* regret, float* logprob, float* entropy, void* workspace,
              size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
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
  if (B == 0) return ESPO_OK;
  if (!logits || !values || !z || !alive || !stop_step || !tokens || !regret) return ESPO_EINVAL;
  if (V > espo::kMaxVocab || B > 0x7fffffff || espo::step_shared_bytes(dt, V, (params->top_p > 0.0f && params->top_p < 1.0f) || params->top_k > 0) > espo::kMaxStepLds)
    return ESPO_ERANGE;
  const size_t esize = dt == ESPO_BF16 ? 2 : 4;
  if (!aligned16(logits) || ((size_t)row_stride * esize) % 16 != 0) return ESPO_EALIGN;
  return espo::launch_step(logits, dt, B, V, row_stride, temperature, seed, step, values, *params,
                           g_margin_scale.load(), z, alive, stop_step, tokens, regret, logprob, entropy,
                           (hipStream_t)stream);
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
                                 nullptr, (hipStream_t)stream);
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
                                 zero_padding != 0, td, adv, returns, (hipStream_t)stream);
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
                                 lambda, 0, td, adv, returns, (hipStream_t)stream);
}

}  // extern "C"
#pragma GCC visibility pop
