// espo_batch_stats: the update at the boundary of a rollout batch (Section 4.2: exponential
// moving averages of the batch mean and variance of the regret; Eq. beta_update: proportional
// controller of the threshold multiplier).
//
// Two small kernels.  The first reduces the valid tokens regret[b, t < L_b] to per-workgroup
// partial sums of d = g - mu_g and d^2 in double (shifting by the current mean estimate keeps
// the one-pass variance free of cancellation), plus token and stop counts; workgroup w takes
// rows w, w + G, ...  The second adds the partials in a fixed order and forms the outputs.
// Every reduction tree is fixed, so the result does not depend on scheduling.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

// Scratch of espo_batch_stats_static: room for the partial sums of the largest launch (1024
// workgroups, 32 bytes each).  One copy per GPU, held from the moment the library is loaded.
// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[32768];

namespace espo {
namespace {

constexpr int kStatThreads = 256;
constexpr int kStatWaves = kStatThreads / kWave;
constexpr int kMaxStatGroups = 1024;

struct Partial {
  double s1, s2;
  long long n, nstop;
};

__device__ __forceinline__ double shfl_down_f64(double v, int d) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_down(lo, d);
  hi = __shfl_down(hi, d);
  return __hiloint2double(hi, lo);
}

// Sum over the workgroup in a fixed tree; the result is valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double* lds) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += shfl_down_f64(v, d);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  __syncthreads();  // lds may still be read from the call before
  if (lane == 0) lds[wave] = v;
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0)
    for (int w = 0; w < kStatWaves; ++w) t += lds[w];
  return t;
}

template <bool VEC>
__global__ __launch_bounds__(kStatThreads) void batch_partial_kernel(const float* __restrict__ regret,
                                                                     const int32_t* __restrict__ lengths,
                                                                     const uint8_t* __restrict__ stopped, int64_t B,
                                                                     int64_t T, float mu_g, Partial* __restrict__ part) {
  __shared__ double lds[kStatWaves];
  const double shift = (double)mu_g;
  double s1 = 0.0, s2 = 0.0;
  long long n = 0, nstop = 0;
  for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
    int64_t L = lengths[b];
    L = L < 0 ? 0 : (L > T ? T : L);
    const float* row = regret + b * T;
    if (VEC) {  // T % 4 == 0: rows are 16-byte aligned
      const int64_t full = L & ~(int64_t)3;
      for (int64_t t = (int64_t)threadIdx.x * 4; t < full; t += kStatThreads * 4) {
        const f32x4 g = __builtin_nontemporal_load((const f32x4*)(row + t));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const double d = (double)g[j] - shift;
          s1 += d;
          s2 += d * d;
        }
      }
      if (threadIdx.x < (unsigned)(L - full)) {  // the last one to three tokens
        const double d = (double)row[full + threadIdx.x] - shift;
        s1 += d;
        s2 += d * d;
      }
    } else {
      for (int64_t t = threadIdx.x; t < L; t += kStatThreads) {
        const double d = (double)row[t] - shift;
        s1 += d;
        s2 += d * d;
      }
    }
    if (threadIdx.x == 0) {
      n += L;
      nstop += stopped[b] != 0;
    }
  }
  const double t1 = block_sum(s1, lds);
  const double t2 = block_sum(s2, lds);
  if (threadIdx.x == 0) part[blockIdx.x] = Partial{t1, t2, n, nstop};
}

struct FinalArgs {
  const Partial* part;
  int groups;
  int64_t B;
  float mu_g, var_g, beta, alpha_ema, eta_beta, target_rate, beta_min, beta_max;
  espo_batch_result* out;
};

__global__ __launch_bounds__(kStatThreads) void batch_final_kernel(FinalArgs a) {
  __shared__ double lds[kStatWaves];
  double s1 = 0.0, s2 = 0.0, n = 0.0, ns = 0.0;  // counts are below 2^53: exact in double
  for (int i = threadIdx.x; i < a.groups; i += kStatThreads) {
    const Partial p = a.part[i];
    s1 += p.s1;
    s2 += p.s2;
    n += (double)p.n;
    ns += (double)p.nstop;
  }
  s1 = block_sum(s1, lds);
  s2 = block_sum(s2, lds);
  n = block_sum(n, lds);
  ns = block_sum(ns, lds);
  if (threadIdx.x != 0) return;
  espo_batch_result r;
  const double md = n > 0.0 ? s1 / n : 0.0;                        // mean of g - mu_g
  const double mean = n > 0.0 ? (double)a.mu_g + md : 0.0;
  double var = n > 0.0 ? s2 / n - md * md : 0.0;
  if (var < 0.0) var = 0.0;
  const double rate = a.B > 0 ? ns / (double)a.B : 0.0;
  const double al = (double)a.alpha_ema;
  r.mean_g = mean;
  r.var_g_batch = var;
  r.stop_rate = rate;
  r.tokens = (int64_t)n;
  r.stopped = (int32_t)ns;
  r.mu_g = a.mu_g;
  r.var_g = a.var_g;
  r.beta = a.beta;
  if (n > 0.0) {
    r.mu_g = (float)(al * (double)a.mu_g + (1.0 - al) * mean);
    r.var_g = (float)(al * (double)a.var_g + (1.0 - al) * var);
  }
  if (a.B > 0) {
    double bt = (double)a.beta + (double)a.eta_beta * (rate - (double)a.target_rate);  // Eq. beta_update
    bt = bt < (double)a.beta_min ? (double)a.beta_min : bt;
    bt = bt > (double)a.beta_max ? (double)a.beta_max : bt;
    r.beta = (float)bt;
  }
  *a.out = r;
}

int stat_groups(int64_t B) { return (int)(B < 1 ? 1 : (B > kMaxStatGroups ? kMaxStatGroups : B)); }

// Device address of `scratch` on the current GPU: looked up once per device, with that device
// current, and kept.  Returns nullptr if the runtime cannot name the device or the symbol.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices];

void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

size_t batch_stats_static_capacity() { return sizeof(scratch); }
void* batch_stats_static_scratch() { return static_scratch(); }

size_t batch_stats_workspace(int64_t B) { return (size_t)stat_groups(B) * sizeof(Partial); }

int launch_batch_stats(const float* regret, const int32_t* lengths, const uint8_t* stopped, int64_t B, int64_t T,
                       float mu_g, float var_g, float beta, const espo_batch_ctrl& c, espo_batch_result* out,
                       void* workspace, hipStream_t stream) {
  const int groups = B > 0 ? stat_groups(B) : 0;
  if (groups > 0) {
    if (T % 4 == 0)
      hipLaunchKernelGGL(batch_partial_kernel<true>, dim3(groups), dim3(kStatThreads), 0, stream, regret, lengths,
                         stopped, B, T, mu_g, (Partial*)workspace);
    else
      hipLaunchKernelGGL(batch_partial_kernel<false>, dim3(groups), dim3(kStatThreads), 0, stream, regret, lengths,
                         stopped, B, T, mu_g, (Partial*)workspace);
    if (hipGetLastError() != hipSuccess) return ESPO_EHIP;
  }
  FinalArgs a;
  a.part = (const Partial*)workspace;
  a.groups = groups;
  a.B = B;
  a.mu_g = mu_g; a.var_g = var_g; a.beta = beta;
  a.alpha_ema = c.alpha_ema; a.eta_beta = c.eta_beta; a.target_rate = c.target_rate;
  a.beta_min = c.beta_min; a.beta_max = c.beta_max;
  a.out = out;
  hipLaunchKernelGGL(batch_final_kernel, dim3(1), dim3(kStatThreads), 0, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
