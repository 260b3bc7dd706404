// Device-side helpers shared by the ESPO kernels: wave64 reductions for gfx950,
// Philox4x32-10, and the uniform / Gumbel transforms of the sampling stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace espo {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kLn2 = 0.693147180559945309417f;
constexpr float kLog2e = 1.44269504088896340736f;

// ---------------------------------------------------------------- wave64 reductions
// DPP controls of the GFX9 family: row_shr:n shifts within a 16-lane row, row_bcast:15 /
// row_bcast:31 carry the last lane of a row / of the lower half into the following rows.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;

template <int Ctrl, int RowMask>
__device__ __forceinline__ float dpp_f32(float identity, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity),
                                                               __builtin_bit_cast(int, v), Ctrl, RowMask, 0xf, false));
}

// Maximum over the 64 lanes, returned to every lane as a wave-uniform value.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<kDppRowShr1, 0xf>(kNegInf, v));
  v = fmaxf(v, dpp_f32<kDppRowShr2, 0xf>(kNegInf, v));
  v = fmaxf(v, dpp_f32<kDppRowShr4, 0xf>(kNegInf, v));
  v = fmaxf(v, dpp_f32<kDppRowShr8, 0xf>(kNegInf, v));
  v = fmaxf(v, dpp_f32<kDppBcast15, 0xa>(kNegInf, v));
  v = fmaxf(v, dpp_f32<kDppBcast31, 0xc>(kNegInf, v));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Minimum of unsigned values over the 64 lanes, wave-uniform.
template <int Ctrl, int RowMask>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, Ctrl, RowMask, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, dpp_u32<kDppRowShr1, 0xf>(0xffffffffu, v));
  v = min(v, dpp_u32<kDppRowShr2, 0xf>(0xffffffffu, v));
  v = min(v, dpp_u32<kDppRowShr4, 0xf>(0xffffffffu, v));
  v = min(v, dpp_u32<kDppRowShr8, 0xf>(0xffffffffu, v));
  v = min(v, dpp_u32<kDppBcast15, 0xa>(0xffffffffu, v));
  v = min(v, dpp_u32<kDppBcast31, 0xc>(0xffffffffu, v));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Sum over the 64 lanes in a fixed order (deterministic), wave-uniform result.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppRowShr1, 0xf>(0.0f, v);
  v += dpp_f32<kDppRowShr2, 0xf>(0.0f, v);
  v += dpp_f32<kDppRowShr4, 0xf>(0.0f, v);
  v += dpp_f32<kDppRowShr8, 0xf>(0.0f, v);
  v += dpp_f32<kDppBcast15, 0xa>(0.0f, v);
  v += dpp_f32<kDppBcast31, 0xc>(0.0f, v);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// The same for doubles: the two halves travel separately.
template <int Ctrl, int RowMask>
__device__ __forceinline__ double dpp_f64(double v) {  // 0.0 where the control names no source lane
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), Ctrl, RowMask, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), Ctrl, RowMask, 0xf, false);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum_f64(double v) {
  v += dpp_f64<kDppRowShr1, 0xf>(v);
  v += dpp_f64<kDppRowShr2, 0xf>(v);
  v += dpp_f64<kDppRowShr4, 0xf>(v);
  v += dpp_f64<kDppRowShr8, 0xf>(v);
  v += dpp_f64<kDppBcast15, 0xa>(v);
  v += dpp_f64<kDppBcast31, 0xc>(v);
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// Maximum over each aligned group of 8 lanes, returned to all 8 (xor-butterfly: swap within
// pairs, swap pairs within quads, mirror the two quads of the group).
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E, kDppHalfMirror = 0x141;
template <int Ctrl>
__device__ __forceinline__ float dpp_all_lanes(float v) {  // every lane has a source: no fill value needed
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), Ctrl, 0xf, 0xf, true));
}
__device__ __forceinline__ float group8_max(float v) {
  v = fmaxf(v, dpp_all_lanes<kDppQuadXor1>(v));
  v = fmaxf(v, dpp_all_lanes<kDppQuadXor2>(v));
  v = fmaxf(v, dpp_all_lanes<kDppHalfMirror>(v));
  return v;
}

__device__ __forceinline__ float uniform_f32(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// A double from `d` lanes further on in the wave (the lane's own where there is none).
__device__ __forceinline__ double shfl_down_f64(double v, int d) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_down(lo, d);
  hi = __shfl_down(hi, d);
  return __hiloint2double(hi, lo);
}

// ---------------------------------------------------------------- Philox4x32-10
// Salmon et al., SC'11: ten rounds; each round multiplies words 0 and 2 by fixed odd
// constants, keeps the low halves and folds the high halves with the other words and
// the round key, which advances by a Weyl sequence.
struct Philox4 {
  uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    // both halves of each product from one 64-bit multiply: one v_mad_u64_u32 instead of a high and a low
    // multiply, a quarter off the time of a call (the multiplies are what a call costs)
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{{c0, c1, c2, c3}};
}

constexpr uint32_t kTagBlock = 0x4553504Fu;  // counter word 3 of the per-block draw
constexpr uint32_t kTagElem = 0x6573706Fu;   // counter word 3 of the per-index draw
constexpr uint32_t kTagRagged = 0x52414747u; // counter word 3 of the position draw of a ragged last block
constexpr int kDrawBlock = 64;               // vocabulary indices per block of the draw

// u = (2r+1)/2^24 with r the top 23 bits of the word: never 0 or 1, exact in fp32.
__device__ __forceinline__ double uniform_f64(uint32_t word) {
  return (double)(2u * (word >> 9) + 1u) * (1.0 / 16777216.0);
}

// fp32 upper bound of the standard Gumbel variate -ln(-ln u(word)).  Used only to rule
// blocks out, so it may be loose but must never fall below the exact value.  The hardware
// log2 times ln 2 is accurate to 1.7e-7 relative over every u(word), also next to 1, and
// over the range of -ln u (a device test measures both); the inner value is lowered by
// 1e-6 relative and the result raised by more than the outer logarithm's error.
__device__ __forceinline__ float gumbel_upper_f32(uint32_t word) {
  const float u = (float)(2u * (word >> 9) + 1u) * (1.0f / 16777216.0f);
  const float e_lb = -__builtin_amdgcn_logf(u) * kLn2 * (1.0f - 1e-6f);
  const float g = -__builtin_amdgcn_logf(e_lb) * kLn2;
  return g + (2e-5f + 4e-6f * fabsf(g));
}

}  // namespace espo
