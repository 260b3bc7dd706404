// espo_advantages: TD errors and GAE on truncated trajectories (Section 3: delta_t and
// Eq. gae; Section 4.4: failure reward at the stop step, no bootstrap past the end).
//
// A_t = delta_t + c A_{t+1} (c = gamma*lambda) is a first-order linear recurrence that
// runs backwards over each row's valid prefix [0, L).  One workgroup of 16 wavefronts owns
// one row and walks it in tiles of 4096 tokens from the tile that holds L-1 down to tile 0;
// tiles at or beyond L are only zero-filled.  Inside a tile every lane holds 4 consecutive
// tokens (one 16-byte load per input array, one 16-byte store per output array), and the
// lanes are laid out backwards: thread 0 holds the tile's last four tokens.  That turns the
// suffix sums of the recurrence into prefix sums over the lanes, which the DPP row shifts
// and row broadcasts of gfx9 compute in six steps without touching LDS; the sixteen wave
// totals are combined the same way after one trip through LDS, and a single scalar carries A
// across the tile boundary.  Only that scalar depends on the previous tile, so the next
// tile's loads are issued before the current one is reduced.
//
// The same kernel serves the terminal-reward form (the rewards of Algorithm 1: zero at every
// step that goes on, one reward at the last): no reward array is read, the last token takes
// r_fail or the row's terminal reward, and on request the value targets A_t + V(s_t) are
// stored and the padding beyond the lengths is left alone.
//
// It also serves trajectories stored back to back (extents from cu_seqlens): the workgroup
// then works on the span that starts at the 16-byte boundary at or before the trajectory's
// first token, so every lane still moves 16 aligned bytes; the up to three tokens before the
// first one belong to the neighbour, come last in the backward scan (nothing valid depends on
// them) and are not stored, and neither is anything at or after the trajectory's end.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/espo.h"
#include "espo_device.h"
#include "espo_host.h"

namespace espo {
namespace {

constexpr int kAdvThreads = 1024;
constexpr int kAdvWaves = kAdvThreads / kWave;
constexpr int kPerLane = 4;
constexpr int kAdvTile = kAdvThreads * kPerLane;  // 4096 tokens
constexpr int kDppWaveShr1 = 0x138;               // lane i takes lane i-1 across the whole wave

struct AdvArgs {
  const float* rewards;          // dense form: [B, T]
  const float* terminal_reward;  // terminal form: [B]
  float* returns;                // optional [B, T]: A_t + V(s_t)
  int32_t zero_padding;          // write zeros at t >= L (else those positions are not written by whole lanes)
  const float* values;
  const int64_t* cu;             // packed form: [B + 1] extents into arrays of N tokens
  int64_t N;
  const int32_t* lengths;
  const uint8_t* stopped;
  int64_t T;
  int32_t B;  // rows; with zero padding the grid has 2 B workgroups, the second B only fill
  float r_fail, gamma, c;
  float cj[kPerLane + 1];  // c^0 .. c^4
  float clane[6];          // c^(4*2^k), k = 0..5: a distance of 2^k lanes
  float cwave[5];          // c^(256*2^k), k = 0..4: a distance of 2^k waves; cwave[4] spans a tile
  float* td;
  float* adv;
  const int32_t* order;    // optional [B]: the rows, longest first (padded forms)
  AdvRowStats* row_stats;  // optional [B]: sums of every row's advantages (padded forms)
  int32_t* sorted;         // optional [B - kAdvFirstRows]: the rows from kAdvFirstRows on, longest first, written by
                           //   workgroup 0 of this launch (padded forms, no `order` given)
  uint32_t* sync;          // with `sorted`: [0] set once `sorted` is complete, [32] readers so far; both 0 between launches
};

// Workgroups that the chip holds at once (256 CUs x 2 of 1024 threads): the rows that are scanned first whatever
// their lengths.  Only the order of the rows that follow decides how ragged the launch's end is (measured: rows
// 512.. of 1024 longest first gives what a full order gives, 39.9 us against 45.3 in index order; rows 768.. 43.3).
constexpr int kAdvFirstRows = 512;
// The word that says "sorted" and the count of its readers lie in different 128-byte lines: loads of the one and
// read-modify-writes of the other on the same line cost the readers 15 us per launch between them.
constexpr int kAdvSyncStride = 32;       // words
constexpr size_t kAdvSyncBytes = 256;
constexpr int kOrderClasses = 256;

// Writes the rows first .. B-1 to order[0 .. B-first), longest first: a counting sort of the clipped lengths into
// 256 classes by one workgroup (rows of one class in no particular order; no result depends on it).  The entries
// are written past the caches that other parts of the chip do not see, and are complete when the call returns.
__device__ __forceinline__ void sort_rows_by_length(const int32_t* __restrict__ lengths, int32_t first, int32_t B, int64_t T,
                                                    int32_t* __restrict__ order) {
  __shared__ int count[kOrderClasses];
  __shared__ int wave_total[kOrderClasses / kWave];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  auto class_of = [&](int32_t i) {
    int64_t L = lengths[i];
    L = L < 0 ? 0 : (L > T ? T : L);
    return kOrderClasses - 1 - (int)((L * kOrderClasses) / (T + 1));
  };
  if (tid < kOrderClasses) count[tid] = 0;
  __syncthreads();
  for (int32_t i = first + tid; i < B; i += kAdvThreads) atomicAdd(&count[class_of(i)], 1);
  __syncthreads();
  int mine = 0, incl = 0;
  if (tid < kOrderClasses) {  // inclusive prefix over the classes: inside each wave, then over the four waves
    mine = count[tid];
    incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) wave_total[tid >> 6] = incl;
  }
  __syncthreads();
  if (tid < kOrderClasses) {
    int before = 0;
    for (int w = 0; w < (tid >> 6); ++w) before += wave_total[w];
    count[tid] = before + incl - mine;  // where the class starts
  }
  __syncthreads();
  for (int32_t i = first + tid; i < B; i += kAdvThreads)
    __hip_atomic_store(order + atomicAdd(&count[class_of(i)], 1), i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// The k-th row of that same order (rows first .. B-1 by class of length, longest first; inside a class by
// index), found by the calling workgroup for itself: every workgroup that asks gets the same permutation, so
// no memory and no waiting is needed.  All threads must call it; the result is uniform.
__device__ __forceinline__ int32_t kth_row_by_length(const int32_t* __restrict__ lengths, int32_t first, int32_t B, int64_t T,
                                                     int32_t k) {
  __shared__ int count[kOrderClasses];
  __shared__ int wave_total[kAdvWaves];
  __shared__ int s_class, s_rank, s_found;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
  auto class_of = [&](int32_t i) {
    int64_t L = lengths[i];
    L = L < 0 ? 0 : (L > T ? T : L);
    return kOrderClasses - 1 - (int)((L * kOrderClasses) / (T + 1));
  };
  if (tid < kOrderClasses) count[tid] = 0;
  if (tid == 0) s_found = -1;
  __syncthreads();
  for (int32_t i = first + tid; i < B; i += kAdvThreads) atomicAdd(&count[class_of(i)], 1);
  __syncthreads();
  int mine = 0, incl = 0;
  if (tid < kOrderClasses) {  // inclusive prefix over the classes: inside each wave, then over the four waves
    mine = count[tid];
    incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) wave_total[wave] = incl;
  }
  __syncthreads();
  if (tid < kOrderClasses) {
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_total[w];
    const int start = before + incl - mine;  // where the class starts
    if (k >= start && k < start + mine) {
      s_class = tid;
      s_rank = k - start;
    }
  }
  __syncthreads();
  const int want_class = s_class, want_rank = s_rank;
  int seen = 0;  // rows of the class before this chunk (uniform)
  for (int32_t chunk = first; chunk < B; chunk += kAdvThreads) {
    const int32_t i = chunk + tid;
    const bool in = i < B && class_of(i) == want_class;
    const uint64_t who = __builtin_amdgcn_ballot_w64(in);
    if (lane == 0) wave_total[wave] = (int)__builtin_popcountll(who);
    __syncthreads();
    int before = seen, all = 0;
    for (int w = 0; w < kAdvWaves; ++w) {
      const int n = wave_total[w];
      before += w < wave ? n : 0;
      all += n;
    }
    if (in && before + (int)__builtin_popcountll(who & ((1ull << lane) - 1ull)) == want_rank) s_found = i;
    seen += all;
    __syncthreads();
    if (seen > want_rank) break;  // (uniform) found in this chunk
  }
  return s_found;
}

struct TileIn {
  float r[kPerLane], v[kPerLane];
  float halo;  // value of the token after the wave's span (lane 0 only)
};

// c^(unit * e) for 0 <= e < 2^Bits from the table of c^(unit * 2^k).
template <int Bits>
__device__ __forceinline__ float pow_from_table(const float* tab, int e) {
  float w = 1.0f;
#pragma unroll
  for (int k = 0; k < Bits; ++k)
    if (e & (1 << k)) w *= tab[k];
  return w;
}

// Loads the lane's 4 tokens starting at t0 and, in lane 0, the value at t0 + 4; tokens at or
// beyond L are never read.
template <bool VEC, bool Dense>
__device__ __forceinline__ TileIn load_tile(const float* __restrict__ rrow, const float* __restrict__ vrow, int64_t t0,
                                            int64_t L, bool want_halo) {
  TileIn in;
#pragma unroll
  for (int j = 0; j < kPerLane; ++j) { in.r[j] = 0.0f; in.v[j] = 0.0f; }
  in.halo = 0.0f;
  if (VEC && t0 + kPerLane <= L) {
    if constexpr (Dense) {
      const f32x4 a = __builtin_nontemporal_load((const f32x4*)(rrow + t0));
#pragma unroll
      for (int j = 0; j < kPerLane; ++j) in.r[j] = a[j];
    }
    const f32x4 b = __builtin_nontemporal_load((const f32x4*)(vrow + t0));
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) in.v[j] = b[j];
  } else {
#pragma unroll
    for (int j = 0; j < kPerLane; ++j)
      if (t0 + j < L) {
        if constexpr (Dense) in.r[j] = rrow[t0 + j];
        in.v[j] = vrow[t0 + j];
      }
  }
  if (want_halo && t0 + kPerLane < L) in.halo = vrow[t0 + kPerLane];
  return in;
}

template <bool VEC>
__device__ __forceinline__ void store4(float* __restrict__ row, int64_t t0, int64_t T, const float x[kPerLane]) {
  if (VEC) {
    if (t0 < T) __builtin_nontemporal_store(f32x4{x[0], x[1], x[2], x[3]}, (f32x4*)(row + t0));  // T % 4 == 0 here
    return;
  }
#pragma unroll
  for (int j = 0; j < kPerLane; ++j)
    if (t0 + j < T) row[t0 + j] = x[j];
}

// Stores x[j] at t0 + j for lo <= t0 + j < hi (t0 a multiple of 4, the row 16-byte aligned).
__device__ __forceinline__ void store_span(float* __restrict__ row, int64_t t0, int64_t lo, int64_t hi, const float x[kPerLane]) {
  if (t0 >= lo && t0 + kPerLane <= hi) {
    __builtin_nontemporal_store(f32x4{x[0], x[1], x[2], x[3]}, (f32x4*)(row + t0));
    return;
  }
#pragma unroll
  for (int j = 0; j < kPerLane; ++j)
    if (t0 + j >= lo && t0 + j < hi) row[t0 + j] = x[j];
}

// One step of a weighted inclusive prefix sum over lanes: s += w * (s of the lane the DPP control names).
template <int Ctrl, int RowMask>
__device__ __forceinline__ float scan_step(float s, float w) {
  return fmaf(w, dpp_f32<Ctrl, RowMask>(0.0f, s), s);
}

template <bool VEC, bool Dense, bool Packed>
__global__ __launch_bounds__(kAdvThreads, 8) void espo_advantages_kernel(AdvArgs a) {
  __shared__ float s_tot[2][kAdvWaves];  // wave totals, double-buffered by tile parity
  // With zero padding, the tiles wholly beyond a trajectory are filled by a workgroup of their
  // own (the second half of the grid): the two kinds of work of a row are then dispatched
  // separately, which evens out the rows (a row costs 16 bytes per valid and 8 per padded token):
  // 2 to 3 us on the B = 1024, T = 16384 batches when their rows come in order of length, nothing
  // when they come in random order.  (Ranking the rows by length inside every workgroup, 8 or 64
  // classes, cost 3 to 5 us per launch, as much as the order gains; only the order of the rows that do
  // not fit the chip at once matters, and only their scans look their row up: see below.)
  int unit = (int)blockIdx.x;
  if (!Packed && a.sorted) {
    // No order was given and the batch has more rows than the chip holds workgroups: workgroup 0 of this launch
    // sorts the later rows while the first kAdvFirstRows are being scanned, and tells the others when it is done.
    // It waits for nobody and is dispatched before every workgroup that waits for it.
    if (unit == 0) {
      sort_rows_by_length(a.lengths, kAdvFirstRows, a.B, a.T, a.sorted);
      if (threadIdx.x == 0) __hip_atomic_store(a.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
    unit -= 1;
  }
  const bool fill_only = !Packed && unit >= a.B;
  int row = fill_only ? unit - a.B : unit;
  // Rows in order of length: the long scans start first and the short ones fill the launch's end (the
  // workgroups that only fill take the rows the other way round: the shortest row has the most padding).
  // An entry that names no row makes its workgroup do nothing.
  if (!Packed && a.order) {
    row = a.order[fill_only ? a.B - 1 - row : row];
    if ((unsigned)row >= (unsigned)a.B) return;
  } else if (!Packed && a.sorted && !fill_only && row >= kAdvFirstRows) {
    // one of the later scans: its row comes from the sorted list.  The last reader clears the two words, so the
    // next launch finds them as this one did.
    __shared__ int s_row;
    if (threadIdx.x == 0) {
      while (__hip_atomic_load(a.sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) __builtin_amdgcn_s_sleep(8);
      s_row = __hip_atomic_load(a.sorted + (row - kAdvFirstRows), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const uint32_t readers = (uint32_t)(a.B - kAdvFirstRows);
      if (atomicInc(a.sync + kAdvSyncStride, readers - 1u) == readers - 1u)
        __hip_atomic_store(a.sync, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    row = s_row;
    if ((unsigned)row >= (unsigned)a.B) return;
  } else if (!Packed && !fill_only && row >= kAdvFirstRows) {
    // No order and nowhere to keep one: each of the later scans finds its row for itself, the
    // (row - kAdvFirstRows)-th longest of the later rows (five barriers and a few hundred LDS operations
    // before its first load, while the other workgroups of the compute unit stream).  Measured on the
    // B = 1024, T = 16384 batches: 40.6 against 43.7 us per launch.
    row = kth_row_by_length(a.lengths, kAdvFirstRows, a.B, a.T, row - kAdvFirstRows);
    if ((unsigned)row >= (unsigned)a.B) return;
  }
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int64_t T = a.T;
  int64_t L, base = (int64_t)row * T, head = 0;
  if constexpr (Packed) {
    // extent clipped to the arrays; the span starts at the 16-byte boundary at or before it
    int64_t first = a.cu[row], end = a.cu[row + 1];
    first = first < 0 ? 0 : (first > a.N ? a.N : first);
    end = end > a.N ? a.N : end;
    if (end <= first) return;
    base = first & ~(int64_t)(kPerLane - 1);
    head = first - base;
    L = end - base;
    T = L;
  } else {
    L = a.lengths[row];
    L = L < 0 ? 0 : (L > T ? T : L);
  }
  const bool stopped = a.stopped[row] != 0;
  // reward of the last token where it does not come from the reward array: r_fail after a stop
  // (Eq. failure_reward), the row's terminal reward in the terminal form
  const bool last_given = stopped || !Dense;
  float r_last = a.r_fail;
  if (!Dense && !stopped) r_last = a.terminal_reward[row];
  const float* rrow = Dense ? a.rewards + base : nullptr;
  const float* vrow = a.values + base;
  float* drow = a.td + base;
  float* arow = a.adv + base;
  float* trow = a.returns ? a.returns + base : nullptr;

  const int64_t ntiles = (T + kAdvTile - 1) / kAdvTile;
  const int64_t nvalid = (L + kAdvTile - 1) / kAdvTile;  // tiles that hold at least one valid token
  const int64_t lane_off = (int64_t)(kAdvThreads - 1 - tid) * kPerLane;  // backwards: thread 0 holds the last tokens

  // tiles wholly beyond the trajectory: outputs are exactly zero
  const float zero[kPerLane] = {0, 0, 0, 0};
  if (fill_only) {
    for (int64_t k = ntiles - 1; k >= nvalid; --k) {
      store4<VEC>(drow, k * kAdvTile + lane_off, T, zero);
      store4<VEC>(arow, k * kAdvTile + lane_off, T, zero);
      if (trow) store4<VEC>(trow, k * kAdvTile + lane_off, T, zero);
    }
    return;
  }
  if (nvalid == 0) {
    if (!Packed && a.row_stats && tid == 0) a.row_stats[row] = AdvRowStats{0.0, 0.0, 0.0, 0};
    return;
  }
  // Sums of the row's advantages for the batch statistics, in double about the advantage of the row's
  // last token (r - V there: nothing is bootstrapped beyond the end), which every thread can form.
  const bool want_stats = !Packed && a.row_stats != nullptr;
  double st_shift = 0.0, st_s1 = 0.0, st_s2 = 0.0;
  if (want_stats) st_shift = (double)((last_given ? r_last : rrow[L - 1]) - vrow[L - 1]);

  // per-lane weights of the cross-row scan steps and of the carry into this lane and this wave
  const float w_b15 = pow_from_table<5>(a.clane, (lane & 15) + 1);  // from lane 15 of the row before
  const float w_b31 = pow_from_table<6>(a.clane, (lane & 31) + 1);  // from lane 31
  const float w_lane = pow_from_table<6>(a.clane, lane);            // c^(4 lane): the wave's carry-in seen from this lane
  const float w_wave = pow_from_table<4>(a.cwave, wave);            // c^(256 wave): the tile's carry-in seen from this wave

  float carry = 0.0f;  // A at the first token of the tile processed before (the later one)
  TileIn cur = load_tile<VEC, Dense>(rrow, vrow, (nvalid - 1) * kAdvTile + lane_off, L, lane == 0);
  for (int64_t k = nvalid - 1; k >= 0; --k) {
    const int64_t t0 = k * kAdvTile + lane_off;
    TileIn nxt;
    if (k > 0) nxt = load_tile<VEC, Dense>(rrow, vrow, t0 - kAdvTile, L, lane == 0);  // the earlier tile, in flight during the scan

    // V_{t+1} of the lane's last token: first value of the lane that holds the following tokens
    float vnext = dpp_f32<kDppWaveShr1, 0xf>(0.0f, cur.v[0]);
    if (lane == 0) vnext = cur.halo;

    // delta_t and the recurrence over the lane's 4 tokens, later tokens first
    const int64_t rem = L - t0;  // valid tokens from t0 on (may be <= 0 or large)
    float d[kPerLane], loc[kPerLane];
    float acc = 0.0f;
    if (__builtin_amdgcn_ballot_w64(rem <= kPerLane) == 0) {  // whole wave strictly inside the trajectory
#pragma unroll
      for (int j = kPerLane - 1; j >= 0; --j) {
        const float vn = (j == kPerLane - 1) ? vnext : cur.v[j + 1];
        d[j] = (cur.r[j] + a.gamma * vn) - cur.v[j];
        acc = d[j] + a.c * acc;
        loc[j] = acc;
      }
    } else {
#pragma unroll
      for (int j = kPerLane - 1; j >= 0; --j) {
        float vn = (j == kPerLane - 1) ? vnext : cur.v[j + 1];
        if (j + 1 >= rem) vn = 0.0f;                        // no bootstrap beyond the last token
        float r = cur.r[j];
        if (last_given && j + 1 == rem) r = r_last;
        float dj = (r + a.gamma * vn) - cur.v[j];
        if (j >= rem) dj = 0.0f;
        d[j] = dj;
        acc = dj + a.c * acc;
        loc[j] = acc;
      }
    }

    // inclusive prefix over the lanes: s_i = sum_{i' <= i} c^(4 (i - i')) acc_i'
    float s = acc;
    s = scan_step<kDppRowShr1, 0xf>(s, a.clane[0]);
    s = scan_step<kDppRowShr2, 0xf>(s, a.clane[1]);
    s = scan_step<kDppRowShr4, 0xf>(s, a.clane[2]);
    s = scan_step<kDppRowShr8, 0xf>(s, a.clane[3]);
    s = scan_step<kDppBcast15, 0xa>(s, w_b15);
    s = scan_step<kDppBcast31, 0xc>(s, w_b31);
    const int par = (int)(k & 1);
    if (lane == kWave - 1) s_tot[par][wave] = s;
    __syncthreads();
    // the same scan over the sixteen wave totals, one per lane of the first row
    float p = lane < kAdvWaves ? s_tot[par][lane] : 0.0f;
    p = scan_step<kDppRowShr1, 0xf>(p, a.cwave[0]);
    p = scan_step<kDppRowShr2, 0xf>(p, a.cwave[1]);
    p = scan_step<kDppRowShr4, 0xf>(p, a.cwave[2]);
    p = scan_step<kDppRowShr8, 0xf>(p, a.cwave[3]);
    // A at the first token after this wave's span
    const float before = wave > 0 ? uniform_f32(p, wave - 1) : 0.0f;
    const float wave_in = fmaf(w_wave, carry, before);
    carry = fmaf(a.cwave[4], carry, uniform_f32(p, kAdvWaves - 1));  // A at the tile's first token
    // A at the first token after this lane's span
    const float s_prev = dpp_f32<kDppWaveShr1, 0xf>(0.0f, s);
    const float a_next = fmaf(w_lane, wave_in, s_prev);

    float outA[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) outA[j] = (j < rem) ? fmaf(a.cj[kPerLane - j], a_next, loc[j]) : 0.0f;
    float outR[kPerLane] = {0, 0, 0, 0};  // value targets: the lambda-return A_t + V(s_t)
    if (trow) {
#pragma unroll
      for (int j = 0; j < kPerLane; ++j) outR[j] = (j < rem) ? outA[j] + cur.v[j] : 0.0f;
    }
    if constexpr (Packed) {  // only what the trajectory owns
      if (rem > 0 && t0 + kPerLane > head) {
        store_span(drow, t0, head, L, d);
        store_span(arow, t0, head, L, outA);
        if (trow) store_span(trow, t0, head, L, outR);
      }
    } else if (a.zero_padding || rem > 0) {  // lanes wholly beyond L only ever hold zeros
      store4<VEC>(drow, t0, T, d);
      store4<VEC>(arow, t0, T, outA);
      if (trow) store4<VEC>(trow, t0, T, outR);
    }
    if (want_stats) {
#pragma unroll
      for (int j = 0; j < kPerLane; ++j)
        if (j < rem) {
          const double dd = (double)outA[j] - st_shift;
          st_s1 += dd;
          st_s2 += dd * dd;
        }
    }
    if (k > 0) cur = nxt;
  }
  if (want_stats) {  // lanes, then waves, in a fixed order
    __shared__ double s_stats[2][kAdvWaves];
    st_s1 = wave_sum_f64(st_s1);
    st_s2 = wave_sum_f64(st_s2);
    if (lane == 0) {
      s_stats[0][wave] = st_s1;
      s_stats[1][wave] = st_s2;
    }
    __syncthreads();
    if (tid == 0) {
      double t1 = 0.0, t2 = 0.0;
      for (int w = 0; w < kAdvWaves; ++w) {
        t1 += s_stats[0][w];
        t2 += s_stats[1][w];
      }
      a.row_stats[row] = AdvRowStats{t1, t2, st_shift, (long long)L};
    }
  }
}

__global__ __launch_bounds__(kAdvThreads) void length_order_kernel(const int32_t* __restrict__ lengths, int32_t B, int64_t T,
                                                                  int32_t* __restrict__ order) {
  sort_rows_by_length(lengths, 0, B, T, order);
}

}  // namespace

int launch_advantages(const float* rewards, const float* terminal_reward, const float* values, const int32_t* lengths,
                      const int64_t* cu, int64_t N, const uint8_t* stopped, int64_t B, int64_t T, float r_fail, float gamma,
                      float lambda, int zero_padding, float* td, float* adv, float* returns, const int32_t* order,
                      AdvRowStats* row_stats, int32_t* sorted, uint32_t* sync, hipStream_t stream) {
  AdvArgs a;
  a.order = order;
  a.row_stats = row_stats;
  const bool sort_here = cu == nullptr && order == nullptr && sorted != nullptr && sync != nullptr && B > kAdvFirstRows;
  a.sorted = sort_here ? sorted : nullptr;
  a.sync = sort_here ? sync : nullptr;
  a.rewards = rewards;
  a.terminal_reward = terminal_reward;
  a.returns = returns;
  a.zero_padding = zero_padding;
  a.values = values;
  a.lengths = lengths;
  a.cu = cu;
  a.N = N;
  a.stopped = stopped;
  a.T = T;
  a.B = (int32_t)B;
  a.r_fail = r_fail;
  a.gamma = gamma;
  const double c = (double)gamma * (double)lambda;
  a.c = (float)c;
  for (int j = 0; j <= kPerLane; ++j) a.cj[j] = (float)pow(c, (double)j);
  for (int k = 0; k < 6; ++k) a.clane[k] = (float)pow(c, (double)(kPerLane << k));
  for (int k = 0; k < 5; ++k) a.cwave[k] = (float)pow(c, (double)((kPerLane * kWave) << k));
  a.td = td;
  a.adv = adv;
  const bool vec = (T % 4 == 0);
  const dim3 grid((unsigned)((cu == nullptr && zero_padding ? 2 * B : B) + (sort_here ? 1 : 0))), block(kAdvThreads);
  void (*kernel)(AdvArgs);
  if (cu)
    kernel = rewards ? espo_advantages_kernel<true, true, true> : espo_advantages_kernel<true, false, true>;
  else
    kernel = rewards ? (vec ? espo_advantages_kernel<true, true, false> : espo_advantages_kernel<false, true, false>)
                     : (vec ? espo_advantages_kernel<true, false, false> : espo_advantages_kernel<false, false, false>);
  hipLaunchKernelGGL(kernel, grid, block, 0, stream, a);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

size_t advantages_workspace_layout(int64_t B, size_t* stats_offset, size_t* sorted_offset) {
  // the two words of `sync` come first, so that they are where they were whatever B a call has
  const size_t stats = (size_t)B * sizeof(AdvRowStats);
  const size_t later = B > kAdvFirstRows ? (size_t)(B - kAdvFirstRows) : 0;
  if (stats_offset) *stats_offset = kAdvSyncBytes;
  if (sorted_offset) *sorted_offset = kAdvSyncBytes + stats;
  return kAdvSyncBytes + stats + ((later * sizeof(int32_t) + 15) & ~(size_t)15);
}

int launch_length_order(const int32_t* lengths, int64_t B, int64_t T, int32_t* order, hipStream_t stream) {
  hipLaunchKernelGGL(length_order_kernel, dim3(1), dim3(kAdvThreads), 0, stream, lengths, (int32_t)B, T, order);
  return hipGetLastError() == hipSuccess ? ESPO_OK : ESPO_EHIP;
}

}  // namespace espo
