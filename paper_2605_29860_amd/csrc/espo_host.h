// Host-side declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/espo.h"

namespace espo {

constexpr size_t kMaxStepLds = 128 * 1024;         // dynamic LDS a step workgroup may ask for (160 KB per CU)
constexpr int64_t kMaxVocab = 400000;               // one workgroup per row: 96 bytes of LDS per 512-index tile plus 26-42 KB fixed

// How one espo_step call is laid out: wavefronts per workgroup (16, 8 or 4), workgroups per row,
// workgroups in the launch, dynamic LDS per workgroup, and the bytes of workspace a split needs.
struct StepPlan {
  int waves, chunks;
  int64_t grid;
  size_t lds, workspace;
};

// The plan for this shape.  `filter`: a top-p / top-k draw (one more table in LDS, never split).
// waves / chunks > 0 force those values (the diagnostics entry point); 0 is the library's choice
// (16 waves, no split).
StepPlan plan_step(int dt, int64_t B, int64_t V, bool filter, int waves, int chunks);

// Bytes of workspace for B rows split `chunks` ways; the offset of the chunk results behind the tickets.
size_t step_workspace_layout(int64_t B, int chunks, size_t* partials_offset);

int launch_step(const void* logits, int dt, int64_t B, int64_t V, int64_t row_stride, float temperature,
                uint64_t seed, int32_t step, const float* values, const espo_params& p, float margin_scale,
                float* z, uint8_t* alive, int32_t* stop_step, int32_t* tokens, float* regret, float* logprob,
                float* entropy, void* workspace, const StepPlan& plan, hipStream_t stream);

size_t batch_stats_workspace(int64_t B);

int launch_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                       float mu_g, float var_g, float beta, const espo_batch_ctrl& c, espo_batch_result* out,
                       void* workspace, hipStream_t stream);

// The library's own scratch for espo_batch_stats_static: its size, and its device address on the
// current GPU (nullptr if the runtime cannot provide it).
size_t batch_stats_static_capacity();
void* batch_stats_static_scratch();

// Sums of one row's advantages over its valid tokens, about a shift of the row's own (its last
// token's advantage): n, sum (A - shift), sum (A - shift)^2.  The advantage pass can leave one per
// row; the batch's mean and variance are combined from them without another pass over the batch.
struct AdvRowStats {
  double s1, s2, shift;
  long long n;
};

size_t whiten_workspace(int64_t B, int64_t T);
// The second half of the whitening alone: mean and variance from the rows' sums, then the rewrite.
int launch_whiten_rows(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean,
                       int unbiased, float* out, double* stats, const AdvRowStats* rows, hipStream_t stream);
int launch_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean,
                  int unbiased, float* out, double* stats, void* workspace, hipStream_t stream);

int launch_math_errors(float* out, hipStream_t stream);

// rewards != nullptr: dense form; else the terminal form with terminal_reward[B].
// cu != nullptr: trajectories stored back to back in arrays of N tokens (lengths, T, zero_padding unused).
// order != nullptr (padded forms only): the scanning workgroups take their rows in that order.
// row_stats != nullptr (padded forms only): every row's sums of its advantages are left there.
// sorted, sync != nullptr, no order and more rows than the chip holds workgroups (padded forms only): the
// launch's first workgroup sorts the later rows by length into `sorted`, and `sync` (words 0 and 32, zero between
// launches) tells the others when it is done.
int launch_advantages(const float* rewards, const float* terminal_reward, const float* values, const int32_t* lengths,
                      const int64_t* cu, int64_t N, const uint8_t* stopped, int64_t B, int64_t T, float r_fail, float gamma,
                      float lambda, int zero_padding, float* td, float* adv, float* returns, const int32_t* order,
                      AdvRowStats* row_stats, int32_t* sorted, uint32_t* sync, hipStream_t stream);

// Workspace of espo_advantages_ws: the two words of `sync` (in 256 bytes of their own), B AdvRowStats, the sorted later rows.
size_t advantages_workspace_layout(int64_t B, size_t* stats_offset, size_t* sorted_offset);

// The rows 0 .. B-1 ordered by clipped length, longest first (256 classes of length; one workgroup).
int launch_length_order(const int32_t* lengths, int64_t B, int64_t T, int32_t* order, hipStream_t stream);

}  // namespace espo
