// Host-side declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/espo.h"

namespace espo {

constexpr size_t kMaxStepLds = 128 * 1024;         // dynamic LDS a step workgroup may ask for (160 KB per CU)
constexpr int64_t kMaxVocab = 400000;               // 96 bytes of LDS per 512-index tile plus 26-42 KB fixed

// Bytes of dynamic LDS a step workgroup needs for this dtype and vocabulary.
size_t step_shared_bytes(int dt, int64_t V, bool filter);  // filter: a top-p / top-k draw (one more table per row)

int launch_step(const void* logits, int dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const espo_params& p, float margin_scale,
                float* z, uint8_t* alive, int32_t* stop_step, int32_t* tokens, float* regret, float* logprob,
                float* entropy, hipStream_t stream);

size_t batch_stats_workspace(int64_t B);

int launch_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                       float mu_g, float var_g, float beta, const espo_batch_ctrl& c, espo_batch_result* out,
                       void* workspace, hipStream_t stream);

// The library's own scratch for espo_batch_stats_static: its size, and its device address on the
// current GPU (nullptr if the runtime cannot provide it).
size_t batch_stats_static_capacity();
void* batch_stats_static_scratch();

size_t whiten_workspace(int64_t B, int64_t T);
int launch_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean,
                  int unbiased, float* out, double* stats, void* workspace, hipStream_t stream);

int launch_math_errors(float* out, hipStream_t stream);

// rewards != nullptr: dense form; else the terminal form with terminal_reward[B].
// cu != nullptr: trajectories stored back to back in arrays of N tokens (lengths, T, zero_padding unused).
int launch_advantages(const float* rewards, const float* terminal_reward, const float* values, const int32_t* lengths,
                      const int64_t* cu, int64_t N, const uint8_t* stopped, int64_t B, int64_t T, float r_fail, float gamma,
                      float lambda, int zero_padding, float* td, float* adv, float* returns, hipStream_t stream);

}  // namespace espo
