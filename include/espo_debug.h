/*
 * espo_debug.h -- diagnostics of the ESPO library for the callers that test and profile it.
 * Nothing here is part of the method (Algorithm 1 and Section 3 are in espo.h); nothing here
 * keeps state between calls.  Conventions (device pointers, streams, status codes) as in espo.h.
 */
#ifndef ESPO_DEBUG_H_
#define ESPO_DEBUG_H_

#include "espo.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * espo_step with its internal choices exposed, for this call only:
 *   score_margin_scale  espo_step scores contenders in fp32 first and repeats the decision in
 *                       double only when the two best scores overlap within the fp32 error
 *                       margin.  A scale >= 1 multiplies that margin (1 = what espo_step uses; a
 *                       huge value sends every row through the double-precision search).  The
 *                       sampled token does not depend on it.  ESPO_EINVAL below 1 or for NaN.
 *   waves               wavefronts per workgroup: 4, 8 or 16, or 0 for the library's choice (16; 8 for a
 *                       filtered draw).
 *   chunks              workgroups a row is split over, or 0 for the library's choice (1).  With
 *                       more than one, every workgroup streams a run of 512-index tiles of its row,
 *                       finds the exact winner of that run and leaves it in the workspace with the
 *                       run's maximum and softmax sum; the last workgroup of a row to arrive
 *                       combines them (tokens, regret, state and masks are the same bits as without
 *                       a split; logprob and entropy may differ in the last bits, their sums being
 *                       added in another order).  Needs a zeroed workspace of
 *                       espo_debug_step_workspace_bytes(B, chunks) bytes (ESPO_EWORKSPACE
 *                       otherwise), which comes back zero; the value is lowered to the number of
 *                       tiles of a row and to 64 if it exceeds them.  espo_step itself never splits
 *                       rows: on an MI355X every split measured slower than one workgroup per row.
 * A filtered draw (top_p / top_k) has one layout: waves 0 or 8, chunks 0 or 1.
 * Everything else is espo_step.
 */
int espo_debug_step(const void* logits, espo_dtype dt, int64_t B, int64_t V, int64_t row_stride,
                    float temperature, uint64_t seed, int32_t step,
                    const float* values, const espo_params* params,
                    float* z, uint8_t* alive, int32_t* stop_step,
                    int32_t* tokens, float* regret, float* logprob, float* entropy,
                    void* workspace, size_t workspace_bytes, void* stream,
                    float score_margin_scale, int32_t waves, int32_t chunks);

/* Bytes of workspace espo_debug_step needs to split B rows `chunks` ways (0 for chunks <= 1). */
size_t espo_debug_step_workspace_bytes(int64_t B, int32_t chunks);

/*
 * Measures on the device the accuracy of the hardware logarithm and exponential that the fp32
 * scores of espo_step are built from, against the double-precision functions.  `out` is device
 * memory, 3 floats that the caller has set to zero; once the stream has reached the call they
 * hold the largest relative error of
 *   out[0]  ln u over every value u(w) = (2r+1)/2^24, r = 0 .. 2^23-1, the stream can produce,
 *   out[1]  ln x over 2^23 positive floats spread over [2^-26, 64),
 *   out[2]  exp x over 2^23 points of [-40, 8].
 * The margin of the fp32 scores assumes at most 1.7e-7, 1.7e-7 and 2e-6.
 */
int espo_debug_math_errors(float* out, void* stream);

/*
 * Four kernels of known memory traffic, to calibrate hardware counters and to measure what this
 * GPU's memory system delivers to the simplest possible kernels of the same shape as the two hot
 * kernels.  Device pointers, 16-byte aligned; byte counts multiples of 16 (ESPO_EINVAL otherwise).
 *   espo_debug_copy   reads `bytes` once and writes them once.
 *   espo_debug_read   reads `bytes` once with nontemporal 16-byte loads, eight in flight per lane,
 *                     and writes nothing (`sink`, 4 bytes, is only written if the data folds to one
 *                     particular word): the ceiling for espo_step's one read of the logits.
 *   espo_debug_sweep  lane i reads the i-th 16 bytes of src (read_bytes of them) and writes the i-th
 *                     16 bytes of dst (write_bytes of them), no dependency between elements: the
 *                     ceiling for a pass with the read / write mix of espo_advantages on contiguous
 *                     buffers.
 *   espo_debug_sweep_padded  the traffic of espo_advantages in its own layout, no dependency between
 *                     elements: rewards and values [B, T] are read below lengths[b], td and adv [B, T]
 *                     are written everywhere (not the method's numbers).  T a multiple of 1024.  The
 *                     ceiling for espo_advantages itself: what the four-array padded layout allows.
 */
int espo_debug_copy(void* dst, const void* src, size_t bytes, void* stream);
int espo_debug_read(const void* src, size_t bytes, void* sink, void* stream);
int espo_debug_sweep(const void* src, size_t read_bytes, void* dst, size_t write_bytes, void* stream);
int espo_debug_sweep_padded(const float* rewards, const float* values, const int32_t* lengths, int64_t B, int64_t T,
                            float* td, float* adv, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ESPO_DEBUG_H_ */
