// espo_whiten: advantage whitening over the valid tokens of a batch, the normalisation that
// PPO applies to the GAE output before the clipped objective (the paper keeps the standard PPO
// update, Section 3):  out = (A - mean) / sqrt(var + eps), mean and var over all A[b, t < L_b].
//
// Two launches over the same decomposition.  The batch is cut into items of 4096 consecutive
// tokens of one row; workgroup w takes items w, w + G, ... and every lane moves 16 bytes per
// item.  The first launch reduces each workgroup's items to (n, sum d, sum d^2) in double, with
// d = A - shift and shift the first valid token the workgroup sees: a shift that is itself a
// data value keeps the one-pass variance free of cancellation however far the mean is from
// zero.  The second launch starts by combining the at most 1024 partials (re-based to the
// first non-empty partial's shift, added in a fixed tree, so every workgroup gets the same
// bits whatever the scheduling), then rewrites its items.  Each element is normalised in
// double and rounded to float once.  Positions at t >= L_b are neither read nor written.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

namespace espo {
namespace {

constexpr int kWhThreads = 1024;
constexpr int kWhWaves = kWhThreads / kWave;
constexpr int kWhItem = kWhThreads * 4;  // tokens per item
constexpr int kWhMaxGroups = 1024;

struct WhPartial {
  double s1, s2, shift;
  long long n;
};

struct WhArgs {
  const float* adv;
  const int32_t* lengths;
  int64_t B, T, nch;  // nch: items per row
  int64_t items;      // B * nch
  int groups;
  float eps;
  int shift_mean, ddof;
  float* out;
  double* stats;  // optional [3]: mean, var, n
  WhPartial* part;
};

__device__ __forceinline__ double shfl_down_f64(double v, int d) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_down(lo, d);
  hi = __shfl_down(hi, d);
  return __hiloint2double(hi, lo);
}

// Sum over the workgroup in a fixed tree, returned to every thread.
__device__ __forceinline__ double block_sum_all(double v, double* lds) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += shfl_down_f64(v, d);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  __syncthreads();  // lds may still be read from the call before
  if (lane == 0) lds[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < kWhWaves; ++w) t += lds[w];
  return t;
}

__device__ __forceinline__ int64_t clamped_length(const WhArgs& a, int64_t row) {
  const int64_t L = a.lengths[row];
  return L < 0 ? 0 : (L > a.T ? a.T : L);
}

template <bool VEC>
__global__ __launch_bounds__(kWhThreads) void whiten_partial_kernel(WhArgs a) {
  __shared__ double lds[kWhWaves];
  const int tid = threadIdx.x;
  // the shift: the first valid token of this workgroup's items (the same address in every lane)
  double shift = 0.0;
  for (int64_t it = blockIdx.x; it < a.items; it += a.groups) {
    const int64_t row = it / a.nch, t0 = (it % a.nch) * kWhItem;
    if (t0 < clamped_length(a, row)) {
      shift = (double)a.adv[row * a.T + t0];
      break;
    }
  }
  double s1 = 0.0, s2 = 0.0;
  long long n = 0;
  for (int64_t it = blockIdx.x; it < a.items; it += a.groups) {
    const int64_t row = it / a.nch, t0 = (it % a.nch) * kWhItem;
    const int64_t L = clamped_length(a, row);
    if (t0 >= L) continue;
    const float* p = a.adv + row * a.T;
    if (VEC) {  // T % 4 == 0: every row is 16-byte aligned
      const int64_t t = t0 + (int64_t)tid * 4;
      if (t + 4 <= L) {
        const f32x4 g = __builtin_nontemporal_load((const f32x4*)(p + t));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = (double)g[j] - shift;
          s1 += d;
          s2 += d * d;
        }
      } else {
        for (int j = 0; j < 4 && t + j < L; ++j) {
          const double d = (double)p[t + j] - shift;
          s1 += d;
          s2 += d * d;
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t t = t0 + tid + (int64_t)j * kWhThreads;
        if (t < L) {
          const double d = (double)p[t] - shift;
          s1 += d;
          s2 += d * d;
        }
      }
    }
    if (tid == 0) n += (L - t0 < kWhItem ? L - t0 : kWhItem);
  }
  const double t1 = block_sum_all(s1, lds);
  const double t2 = block_sum_all(s2, lds);
  if (tid == 0) a.part[blockIdx.x] = WhPartial{t1, t2, shift, n};
}

template <bool VEC>
__global__ __launch_bounds__(kWhThreads) void whiten_apply_kernel(WhArgs a) {
  __shared__ double lds[kWhWaves];
  __shared__ int s_first[kWhWaves];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid >> 6;
  // combine the partials: thread i holds partial i
  WhPartial mine{0.0, 0.0, 0.0, 0};
  if (tid < a.groups) mine = a.part[tid];
  const uint32_t first_w = wave_min_u32(mine.n > 0 ? (uint32_t)tid : 0xffffffffu);
  if (lane == 0) s_first[wave] = (int)first_w;
  __syncthreads();
  uint32_t first = 0xffffffffu;
  for (int w = 0; w < kWhWaves; ++w) first = min(first, (uint32_t)s_first[w]);
  if (first == 0xffffffffu) {  // no valid token in the batch: nothing to write
    if (a.stats && blockIdx.x == 0 && tid < 3) a.stats[tid] = 0.0;
    return;
  }
  const double shift = a.part[first].shift;
  const double off = mine.shift - shift;  // re-base this partial: d' = d + off
  const double nn = (double)mine.n;       // below 2^53: exact
  const double n = block_sum_all(nn, lds);
  const double s1 = block_sum_all(mine.n > 0 ? mine.s1 + nn * off : 0.0, lds);
  const double s2 = block_sum_all(mine.n > 0 ? mine.s2 + 2.0 * off * mine.s1 + nn * off * off : 0.0, lds);
  const double md = s1 / n;
  const double mean = shift + md;
  double ss = s2 - n * md * md;  // sum of squared deviations from the mean
  if (ss < 0.0) ss = 0.0;
  const double denom = n - (double)a.ddof;
  const double var = denom > 0.0 ? ss / denom : 0.0;
  const double rstd = 1.0 / sqrt(var + (double)a.eps);
  const double sub = a.shift_mean ? mean : 0.0;
  if (a.stats && blockIdx.x == 0 && tid == 0) {
    a.stats[0] = mean;
    a.stats[1] = var;
    a.stats[2] = n;
  }

  for (int64_t it = blockIdx.x; it < a.items; it += a.groups) {
    const int64_t row = it / a.nch, t0 = (it % a.nch) * kWhItem;
    const int64_t L = clamped_length(a, row);
    if (t0 >= L) continue;
    const float* p = a.adv + row * a.T;
    float* q = a.out + row * a.T;
    if (VEC) {
      const int64_t t = t0 + (int64_t)tid * 4;
      if (t + 4 <= L) {
        const f32x4 g = __builtin_nontemporal_load((const f32x4*)(p + t));
        f32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (float)(((double)g[j] - sub) * rstd);
        __builtin_nontemporal_store(o, (f32x4*)(q + t));
      } else {
        for (int j = 0; j < 4 && t + j < L; ++j) q[t + j] = (float)(((double)p[t + j] - sub) * rstd);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int64_t t = t0 + tid + (int64_t)j * kWhThreads;
        if (t < L) q[t] = (float)(((double)p[t] - sub) * rstd);
      }
    }
  }
}

int whiten_groups(int64_t B, int64_t T) {
  const int64_t nch = (T + kWhItem - 1) / kWhItem;
  const int64_t items = B * nch;
  return (int)(items < 1 ? 1 : (items > kWhMaxGroups ? kWhMaxGroups : items));
}

}  // namespace

size_t whiten_workspace(int64_t B, int64_t T) { return (size_t)whiten_groups(B, T) * sizeof(WhPartial); }

int launch_whiten(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean,
                  int unbiased, float* out, double* stats, void* workspace, hipStream_t stream) {
  WhArgs a;
  a.adv = adv;
  a.lengths = lengths;
  a.B = B;
  a.T = T;
  a.nch = (T + kWhItem - 1) / kWhItem;
  a.items = B * a.nch;
  a.groups = whiten_groups(B, T);
  a.eps = eps;
  a.shift_mean = shift_mean;
  a.ddof = unbiased ? 1 : 0;
  a.out = out;
  a.stats = stats;
  a.part = (WhPartial*)workspace;
  const bool vec = (T % 4 == 0);
  hipLaunchKernelGGL(vec ? whiten_partial_kernel<true> : whiten_partial_kernel<false>, dim3(a.groups), dim3(kWhThreads), 0,
                     stream, a);
  if (hipGetLastError() != hipSuccess) return ESPO_EHIP;
  hipLaunchKernelGGL(vec ? whiten_apply_kernel<true> : whiten_apply_kernel<false>, dim3(a.groups), dim3(kWhThreads), 0,
                     stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
