// espo_whiten: advantage whitening over the valid tokens of a batch, the normalisation that
// PPO applies to the GAE output before the clipped objective (the paper keeps the standard PPO
// update, Section 3):  out = (A - mean) / sqrt(var + eps), mean and var over all A[b, t < L_b].
//
// Two launches over the same decomposition.  The batch is cut into items of 4096 consecutive
// tokens of one row, numbered chunk position first so that a workgroup, which takes items
// w, w + G, ..., sees every chunk position; every lane moves 16 bytes per item.  The first launch reduces each workgroup's items to (n, sum d, sum d^2) in double, with
// d = A - shift and shift the first valid token of the batch: a shift that is itself a data
// value keeps the one-pass variance free of cancellation however far the mean is from zero.
// The second launch starts by adding the at most 512 partials in a fixed tree (every workgroup
// gets the same bits whatever the scheduling), then rewrites its items.  Each element is normalised in
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
constexpr int kWhMaxGroups = 512;  // one workgroup per slot of the chip

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

// One pass of a workgroup over its items, four at a time with their loads issued together.
// An item is (row, first token); `whole(g, t)` gets the four tokens of a lane that lies wholly
// inside the trajectory, `single(x, t)` a token of a lane that the trajectory's end cuts.
constexpr int kWhUnroll = 4;  // eight spill: three 64-bit offsets per item in flight
template <bool VEC, typename Whole, typename Single, typename Count>
__device__ __forceinline__ void for_items(const WhArgs& a, Whole&& whole, Single&& single, Count&& count) {
  const int tid = threadIdx.x;
  for (uint32_t it0 = blockIdx.x; it0 < (uint32_t)a.items; it0 += kWhUnroll * (uint32_t)a.groups) {
    int64_t base[kWhUnroll], t[kWhUnroll], L[kWhUnroll];
#pragma unroll
    for (int u = 0; u < kWhUnroll; ++u) {
      const uint32_t it = it0 + (uint32_t)u * (uint32_t)a.groups;
      L[u] = 0;
      base[u] = 0;
      t[u] = 0;
      if (it < (uint32_t)a.items) {
        const uint32_t ch = it / (uint32_t)a.B, row = it - ch * (uint32_t)a.B;  // chunk-major: a workgroup sees every chunk position
        const int64_t len = a.lengths[row];
        L[u] = len < 0 ? 0 : (len > a.T ? a.T : len);
        base[u] = (int64_t)row * a.T;
        t[u] = (int64_t)ch * kWhItem + (VEC ? tid * 4 : tid);
        const int64_t left = L[u] - (int64_t)ch * kWhItem;
        count(left < 0 ? 0 : (left < kWhItem ? left : kWhItem));  // valid tokens of the item
      }
    }
    if (VEC) {  // T % 4 == 0: every row is 16-byte aligned
      f32x4 g[kWhUnroll];
#pragma unroll
      for (int u = 0; u < kWhUnroll; ++u)
        if (t[u] + 4 <= L[u]) g[u] = __builtin_nontemporal_load((const f32x4*)(a.adv + base[u] + t[u]));
#pragma unroll
      for (int u = 0; u < kWhUnroll; ++u) {
        if (t[u] + 4 <= L[u]) {
          whole(g[u], base[u] + t[u]);
        } else {
          for (int j = 0; j < 4 && t[u] + j < L[u]; ++j) single(a.adv[base[u] + t[u] + j], base[u] + t[u] + j);
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < kWhUnroll; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t tt = t[u] + (int64_t)j * kWhThreads;
          if (tt < L[u]) single(a.adv[base[u] + tt], base[u] + tt);
        }
    }
  }
}

// From the batch's count, mean and sum of squared deviations to the rewrite of this workgroup's items.
template <bool VEC>
__device__ __forceinline__ void normalise_items(const WhArgs& a, double n, double mean, double ss) {
  const int tid = threadIdx.x;
  if (n == 0.0) {  // no valid token in the batch: nothing to write
    if (a.stats && blockIdx.x == 0 && tid < 3) a.stats[tid] = 0.0;
    return;
  }
  if (ss < 0.0) ss = 0.0;
  const double denom = n - (double)a.ddof;
  const double var = denom > 0.0 ? ss / denom : 0.0;
  const double sd = sqrt(var + (double)a.eps);
  const double rstd = sd > 0.0 ? 1.0 / sd : 0.0;  // a constant batch with eps = 0: every output is 0
  const double sub = a.shift_mean ? mean : 0.0;
  if (a.stats && blockIdx.x == 0 && tid == 0) {
    a.stats[0] = mean;
    a.stats[1] = var;
    a.stats[2] = n;
  }
  for_items<VEC>(
      a,
      [&](const f32x4& g, int64_t at) {
        f32x4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = rstd > 0.0 ? (float)(((double)g[j] - sub) * rstd) : 0.0f;
        __builtin_nontemporal_store(o, (f32x4*)(a.out + at));
      },
      [&](float x, int64_t at) { a.out[at] = rstd > 0.0 ? (float)(((double)x - sub) * rstd) : 0.0f; }, [](int64_t) {});
}

template <bool VEC>
__global__ __launch_bounds__(kWhThreads) void whiten_partial_kernel(WhArgs a) {
  __shared__ double lds[kWhWaves];
  const int tid = threadIdx.x;
  // the shift: the first valid token of the batch (the same in every workgroup)
  double shift = 0.0;
  for (int64_t b = 0; b < a.B; ++b)
    if (a.lengths[b] > 0) {
      shift = (double)a.adv[b * a.T];
      break;
    }
  long long n = 0;
  double s1 = 0.0, s2 = 0.0;
  for_items<VEC>(
      a,
      [&](const f32x4& g, int64_t) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = (double)g[j] - shift;
          s1 += d;
          s2 += d * d;
        }
      },
      [&](float x, int64_t) {
        const double d = (double)x - shift;
        s1 += d;
        s2 += d * d;
      },
      [&](int64_t valid) { n += valid; });
  const double t1 = block_sum_all(s1, lds);
  const double t2 = block_sum_all(s2, lds);
  if (tid == 0) a.part[blockIdx.x] = WhPartial{t1, t2, shift, n};
}

template <bool VEC>
__global__ __launch_bounds__(kWhThreads) void whiten_apply_kernel(WhArgs a) {
  __shared__ double lds[3 * kWhWaves];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid >> 6;
  // combine the partials (all about the same shift): thread i holds partial i
  WhPartial mine{0.0, 0.0, 0.0, 0};
  if (tid < a.groups) mine = a.part[tid];
  double v0 = (double)mine.n, v1 = mine.s1, v2 = mine.s2;  // counts are below 2^53: exact
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    v0 += shfl_down_f64(v0, d);
    v1 += shfl_down_f64(v1, d);
    v2 += shfl_down_f64(v2, d);
  }
  if (lane == 0) {
    lds[wave] = v0;
    lds[kWhWaves + wave] = v1;
    lds[2 * kWhWaves + wave] = v2;
  }
  __syncthreads();
  double n = 0.0, s1 = 0.0, s2 = 0.0;
  for (int w = 0; w < kWhWaves; ++w) {  // fixed order: the same bits in every workgroup
    n += lds[w];
    s1 += lds[kWhWaves + w];
    s2 += lds[2 * kWhWaves + w];
  }
  const double shift = a.part[0].shift;
  const double md = n > 0.0 ? s1 / n : 0.0;
  normalise_items<VEC>(a, n, shift + md, s2 - n * md * md);  // s2 - n md^2: the sum of squared deviations from the mean
}

// The same rewrite with the mean and variance combined from sums that the advantage pass left per row,
// each about a shift of that row's own: every row gives (n, mean, sum of squared deviations), and two
// such triples merge exactly (the pairwise update of Chan, Golub and LeVeque).  Thread i merges rows
// i, i + 1024, ...; lanes and waves follow in a fixed tree, so every workgroup gets the same bits.
struct Moments {
  double n, mean, m2;
};

__device__ __forceinline__ double shfl_lane0_f64(double v) {
  return __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v)), __builtin_amdgcn_readfirstlane(__double2loint(v)));
}

__device__ __forceinline__ Moments merge(const Moments& x, const Moments& y) {
  const double n = x.n + y.n;
  if (n == 0.0) return Moments{0.0, 0.0, 0.0};
  const double delta = y.mean - x.mean;
  return Moments{n, x.mean + delta * (y.n / n), x.m2 + y.m2 + delta * delta * (x.n * (y.n / n))};
}

template <bool VEC>
__global__ __launch_bounds__(kWhThreads) void whiten_apply_rows_kernel(WhArgs a, const AdvRowStats* __restrict__ rows) {
  __shared__ double lds[3 * kWhWaves];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid >> 6;
  Moments mine{0.0, 0.0, 0.0};
  for (int64_t b = tid; b < a.B; b += kWhThreads) {
    const AdvRowStats r = rows[b];
    if (r.n > 0) {
      const double n = (double)r.n, md = r.s1 / n;
      const double m2 = r.s2 - n * md * md;
      mine = merge(mine, Moments{n, r.shift + md, m2 > 0.0 ? m2 : 0.0});
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const Moments other{shfl_down_f64(mine.n, d), shfl_down_f64(mine.mean, d), shfl_down_f64(mine.m2, d)};
    if (lane + d < kWave) mine = merge(mine, other);
  }
  if (lane == 0) {
    lds[wave] = mine.n;
    lds[kWhWaves + wave] = mine.mean;
    lds[2 * kWhWaves + wave] = mine.m2;
  }
  __syncthreads();
  // the sixteen wave results, merged by the same tree in every wave
  Moments all{0.0, 0.0, 0.0};
  if (lane < kWhWaves) all = Moments{lds[lane], lds[kWhWaves + lane], lds[2 * kWhWaves + lane]};
#pragma unroll
  for (int d = kWhWaves / 2; d >= 1; d >>= 1) {
    const Moments other{shfl_down_f64(all.n, d), shfl_down_f64(all.mean, d), shfl_down_f64(all.m2, d)};
    if (lane + d < kWhWaves) all = merge(all, other);
  }
  all = Moments{shfl_lane0_f64(all.n), shfl_lane0_f64(all.mean), shfl_lane0_f64(all.m2)};
  normalise_items<VEC>(a, all.n, all.mean, all.m2);
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

int launch_whiten_rows(const float* adv, const int32_t* lengths, int64_t B, int64_t T, float eps, int shift_mean,
                       int unbiased, float* out, double* stats, const AdvRowStats* rows, hipStream_t stream) {
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
  a.part = nullptr;
  const bool vec = (T % 4 == 0);
  hipLaunchKernelGGL(vec ? whiten_apply_rows_kernel<true> : whiten_apply_rows_kernel<false>, dim3(a.groups),
                     dim3(kWhThreads), 0, stream, a, rows);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
