// espo_advantages: TD errors and GAE on truncated trajectories (Section 3: delta_t and
// Eq. gae; Section 4.4: failure reward at the stop step, no bootstrap past the end).
//
// A_t = delta_t + c A_{t+1} (c = gamma*lambda) is a first-order linear recurrence that
// runs backwards over each row's valid prefix [0, L).  One workgroup owns one row and
// walks it in tiles of 2048 tokens from the tile that holds L-1 down to tile 0; tiles at
// or beyond L are only zero-filled.  Inside a tile every lane holds 8 consecutive tokens
// (two 16-byte loads per input array), runs the recurrence serially over them, the 64
// lane results are combined by a suffix scan with the weights c^8, c^16, ... inside the
// wave, the four wave results through LDS, and one scalar carries A at the tile boundary
// into the next (earlier) tile.  The next tile's loads are issued before the scan so that
// HBM latency overlaps the arithmetic.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

namespace espo {
namespace {

constexpr int kAdvThreads = 256;
constexpr int kAdvWaves = kAdvThreads / kWave;
constexpr int kPerLane = 8;
constexpr int kTile = kAdvThreads * kPerLane;  // 2048 tokens

struct AdvArgs {
  const float* rewards;
  const float* values;
  const int32_t* lengths;
  const uint8_t* stopped;
  int64_t T;
  float r_fail, gamma, c;
  float cj[kPerLane + 1];  // c^0 .. c^8
  float cscan[6];          // c^(8*2^k), k = 0..5: weights of the in-wave suffix scan
  float cwave;             // c^512: weight between consecutive waves
  float* td;
  float* adv;
};

struct TileIn {
  float r[kPerLane], v[kPerLane];
};

// Loads the lane's 8 tokens starting at t0; tokens at or beyond L are never read.
template <bool VEC>
__device__ __forceinline__ TileIn load_tile(const float* __restrict__ rrow, const float* __restrict__ vrow,
                                            int64_t t0, int64_t L) {
  TileIn in;
#pragma unroll
  for (int j = 0; j < kPerLane; ++j) { in.r[j] = 0.0f; in.v[j] = 0.0f; }
  if constexpr (VEC) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t t = t0 + 4 * h;
      if (t + 4 <= L) {
        const f32x4 a = __builtin_nontemporal_load((const f32x4*)(rrow + t));
        const f32x4 b = __builtin_nontemporal_load((const f32x4*)(vrow + t));
#pragma unroll
        for (int j = 0; j < 4; ++j) { in.r[4 * h + j] = a[j]; in.v[4 * h + j] = b[j]; }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (t + j < L) { in.r[4 * h + j] = rrow[t + j]; in.v[4 * h + j] = vrow[t + j]; }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < kPerLane; ++j)
      if (t0 + j < L) { in.r[j] = rrow[t0 + j]; in.v[j] = vrow[t0 + j]; }
  }
  return in;
}

template <bool VEC>
__device__ __forceinline__ void store8(float* __restrict__ row, int64_t t0, int64_t T, const float x[kPerLane]) {
  if constexpr (VEC) {
    if (t0 + kPerLane <= T) {
      __builtin_nontemporal_store(f32x4{x[0], x[1], x[2], x[3]}, (f32x4*)(row + t0));
      __builtin_nontemporal_store(f32x4{x[4], x[5], x[6], x[7]}, (f32x4*)(row + t0 + 4));
      return;
    }
  }
#pragma unroll
  for (int j = 0; j < kPerLane; ++j)
    if (t0 + j < T) row[t0 + j] = x[j];
}

template <bool VEC>
__global__ __launch_bounds__(kAdvThreads) void espo_advantages_kernel(AdvArgs a) {
  __shared__ float s_wave[kAdvWaves];   // per-wave scan result at its first token
  __shared__ float s_vfirst[kAdvWaves + 1];  // first value of each wave's span (for the V_{t+1} of the lane before)
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid >> 6;
  const int64_t T = a.T;
  int64_t L = a.lengths[row];
  L = L < 0 ? 0 : (L > T ? T : L);
  const bool stopped = a.stopped[row] != 0;
  const float* rrow = a.rewards + (int64_t)row * T;
  const float* vrow = a.values + (int64_t)row * T;
  float* drow = a.td + (int64_t)row * T;
  float* arow = a.adv + (int64_t)row * T;

  const int64_t ntiles = (T + kTile - 1) / kTile;
  const int64_t nvalid = (L + kTile - 1) / kTile;  // tiles that hold at least one valid token

  // tiles wholly beyond the trajectory: outputs are exactly zero
  const float zero[kPerLane] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int64_t k = ntiles - 1; k >= nvalid; --k) {
    const int64_t t0 = k * kTile + (int64_t)tid * kPerLane;
    store8<VEC>(drow, t0, T, zero);
    store8<VEC>(arow, t0, T, zero);
  }
  if (nvalid == 0) return;

  float carry = 0.0f;  // A at the first token of the tile processed before (the later one)
  TileIn cur = load_tile<VEC>(rrow, vrow, (nvalid - 1) * kTile + (int64_t)tid * kPerLane, L);
  for (int64_t k = nvalid - 1; k >= 0; --k) {
    const int64_t t0 = k * kTile + (int64_t)tid * kPerLane;
    TileIn nxt;
    if (k > 0) nxt = load_tile<VEC>(rrow, vrow, t0 - kTile, L);  // prefetch the earlier tile

    // V_{t+1} of the lane's last token: first value of the next lane / wave / tile
    if (lane == 0) s_vfirst[wave] = cur.v[0];
    float vnext = __shfl_down(cur.v[0], 1);
    __syncthreads();
    if (lane == kWave - 1) {
      if (wave + 1 < kAdvWaves) vnext = s_vfirst[wave + 1];
      else vnext = (t0 + kPerLane < L) ? vrow[t0 + kPerLane] : 0.0f;
    }

    // delta_t and the serial recurrence over the lane's 8 tokens (later tokens first)
    float d[kPerLane], loc[kPerLane];
    float acc = 0.0f;
#pragma unroll
    for (int j = kPerLane - 1; j >= 0; --j) {
      const int64_t t = t0 + j;
      float vn = (j == kPerLane - 1) ? vnext : cur.v[j + 1];
      if (t + 1 >= L) vn = 0.0f;                           // no bootstrap beyond the last token
      float r = cur.r[j];
      if (stopped && t == L - 1) r = a.r_fail;              // Eq. failure_reward
      float dj = (r + a.gamma * vn) - cur.v[j];
      if (t >= L) dj = 0.0f;
      d[j] = dj;
      acc = dj + a.c * acc;
      loc[j] = acc;
    }

    // suffix scan over the lanes of the wave: s_i = sum_{i' >= i} c^(8 (i'-i)) loc_i'[0]
    float s = acc;
#pragma unroll
    for (int kk = 0; kk < 6; ++kk) {
      const int dist = 1 << kk;
      const float o = __shfl_down(s, dist);
      if (lane + dist < kWave) s = fmaf(a.cscan[kk], o, s);
    }
    if (lane == 0) s_wave[wave] = s;
    __syncthreads();
    // value of A at the first token after this wave's span, then after this lane's span
    float after_wave = carry;
    for (int w = kAdvWaves - 1; w > wave; --w) after_wave = fmaf(a.cwave, after_wave, s_wave[w]);
    const float tile_first = [&] {  // A at the tile's first token = new carry
      float x = carry;
      for (int w = kAdvWaves - 1; w >= 0; --w) x = fmaf(a.cwave, x, s_wave[w]);
      return x;
    }();
    // A at the next lane's first token: its in-wave suffix plus the decayed tail
    float s_next = __shfl_down(s, 1);
    // c^(8 (63 - lane)) * after_wave, built from the scan weights (binary expansion)
    float tail_w = after_wave;
    {
      const int e = kWave - 1 - lane;
#pragma unroll
      for (int kk = 0; kk < 6; ++kk)
        if (e & (1 << kk)) tail_w *= a.cscan[kk];
    }
    const float a_next = (lane == kWave - 1) ? after_wave : (s_next + tail_w);

    float outA[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
      const int64_t t = t0 + j;
      outA[j] = (t < L) ? fmaf(a.cj[kPerLane - j], a_next, loc[j]) : 0.0f;
    }
    store8<VEC>(drow, t0, T, d);
    store8<VEC>(arow, t0, T, outA);

    carry = tile_first;
    if (k > 0) cur = nxt;
    __syncthreads();  // s_wave / s_vfirst are rewritten by the next tile
  }
}

}  // namespace

int launch_advantages(const float* rewards, const float* values, const int32_t* lengths,
                      const uint8_t* stopped, int64_t B, int64_t T, float r_fail, float gamma,
                      float lambda, float* td, float* adv, hipStream_t stream) {
  AdvArgs a;
  a.rewards = rewards;
  a.values = values;
  a.lengths = lengths;
  a.stopped = stopped;
  a.T = T;
  a.r_fail = r_fail;
  a.gamma = gamma;
  const double c = (double)gamma * (double)lambda;
  a.c = (float)c;
  for (int j = 0; j <= kPerLane; ++j) a.cj[j] = (float)pow(c, (double)j);
  for (int k = 0; k < 6; ++k) a.cscan[k] = (float)pow(c, (double)(kPerLane << k));
  a.cwave = (float)pow(c, (double)(kPerLane * kWave));
  a.td = td;
  a.adv = adv;
  const bool vec = (T % 4 == 0);
  const dim3 grid((unsigned)B), block(kAdvThreads);
  if (vec)
    hipLaunchKernelGGL(espo_advantages_kernel<true>, grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL(espo_advantages_kernel<false>, grid, block, 0, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
