// Sum over the 64 lanes of a wavefront, result in every lane.
//
// The paper's starter reduces with a cascade of 32-lane shuffles (kernel table,
// row rmsnorm); the CDNA4 counterpart is the data-parallel
// primitive (DPP) operand modifier, which lets a v_add_f32 read a neighbouring
// lane directly, with no LDS traffic.  The order of additions is fixed, and
// because a + b == b + a bit for bit, both partners of every exchange hold the
// same value, so all 64 lanes end with one identical total and the result is
// reproducible from run to run.
//
// Must be called with all 64 lanes active.
#pragma once

#include <hip/hip_runtime.h>

namespace rms {

template <int CTRL>
__device__ __forceinline__ float add_dpp(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                0xF, 0xF, false);
  return v + __builtin_bit_cast(float, moved);
}

__device__ __forceinline__ float read_lane(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

__device__ __forceinline__ float wave_sum(float v) {
  v = add_dpp<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
  v = add_dpp<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2      -> sum of each quad
  v = add_dpp<0x141>(v);  // row_half_mirror: lane i <-> 7 - i  -> sum of each 8
  v = add_dpp<0x140>(v);  // row_mirror: lane i <-> 15 - i      -> sum of each 16-lane row
  const float r0 = read_lane(v, 0);
  const float r1 = read_lane(v, 16);
  const float r2 = read_lane(v, 32);
  const float r3 = read_lane(v, 48);
  return (r0 + r1) + (r2 + r3);
}

// Maximum over the 64 lanes, result in every lane; same exchanges as wave_sum.
// fmaxf returns the other operand when one is NaN, so NaNs do not take part.
template <int CTRL>
__device__ __forceinline__ float max_dpp(float v) {
  const int moved = __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v),
                                                __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false);
  return __builtin_fmaxf(v, __builtin_bit_cast(float, moved));
}

__device__ __forceinline__ float wave_max(float v) {
  v = max_dpp<0xB1>(v);
  v = max_dpp<0x4E>(v);
  v = max_dpp<0x141>(v);
  v = max_dpp<0x140>(v);
  const float r0 = read_lane(v, 0);
  const float r1 = read_lane(v, 16);
  const float r2 = read_lane(v, 32);
  const float r3 = read_lane(v, 48);
  return __builtin_fmaxf(__builtin_fmaxf(r0, r1), __builtin_fmaxf(r2, r3));
}

// ---------------------------------------------------------------------------
// Per-wavefront partials parked in LDS and combined by every thread after a barrier.
// The partials are read with 128-bit LDS loads, all issued before the first is used: a loop
// that reads them one by one waits for each read in turn, which at 8 wavefronts costs a few
// tenths of a microsecond on every row's critical path.
//
// Compile-time workgroup size: sum_waves / max_waves over exactly WAVES slots (the array
// must be 16-byte aligned).  Run-time workgroup size: 16 slots; park_partial fills the slots
// past `waves` with the identity before the barrier, and sum16 / max16 take all 16.
// ---------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int WAVES>
__device__ __forceinline__ void read_partials(const float* part, float (&p)[WAVES]) {
  if constexpr (WAVES % 4 == 0) {
#pragma unroll
    for (int q = 0; q < WAVES / 4; ++q) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(part + 4 * q);
      p[4 * q] = v.x; p[4 * q + 1] = v.y; p[4 * q + 2] = v.z; p[4 * q + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int k = 0; k < WAVES; ++k) p[k] = part[k];
  }
}

template <int WAVES>
__device__ __forceinline__ float sum_waves(const float* part) {      // in wave order
  float p[WAVES];
  read_partials<WAVES>(part, p);
  float s = p[0];
#pragma unroll
  for (int k = 1; k < WAVES; ++k) s += p[k];
  return s;
}

template <int WAVES>
__device__ __forceinline__ float max_waves(const float* part) {
  float p[WAVES];
  read_partials<WAVES>(part, p);
  float m = p[0];
#pragma unroll
  for (int k = 1; k < WAVES; ++k) m = __builtin_fmaxf(m, p[k]);
  return m;
}

constexpr int kMaxPartials = 16;

// Lane 0 of every wavefront parks its value; lanes waves .. 15 of wavefront 0 fill the unused
// slots with `identity` (0 for a sum, -inf for a maximum).  Call before the barrier.
__device__ __forceinline__ void park_partial(float* part, int lane, int wave, int waves, float v,
                                             float identity) {
  if (lane == 0) part[wave] = v;
  else if (wave == 0 && lane >= waves && lane < kMaxPartials) part[lane] = identity;
}

__device__ __forceinline__ float sum16(const float* part) {          // in wave order
  return sum_waves<kMaxPartials>(part);
}

__device__ __forceinline__ float max16(const float* part) { return max_waves<kMaxPartials>(part); }

template <int L>
__device__ __forceinline__ float subwave_max(float v) {
  static_assert(L == 8 || L == 16 || L == 32, "group size");
  v = max_dpp<0xB1>(v);
  v = max_dpp<0x4E>(v);
  v = max_dpp<0x141>(v);
  if constexpr (L >= 16) v = max_dpp<0x140>(v);
  if constexpr (L == 32) {
    const int other = __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F);
    v = __builtin_fmaxf(v, __builtin_bit_cast(float, other));
  }
  return v;
}

// Sum over aligned groups of L = 8, 16 or 32 lanes, result in every lane of the
// group: the first three or four DPP steps of wave_sum, then for L = 32 one
// ds_swizzle that swaps neighbouring 16-lane rows (a cross-lane move in the LDS
// crossbar; no memory is touched).  Must be called with all 64 lanes active.
template <int L>
__device__ __forceinline__ float subwave_sum(float v) {
  static_assert(L == 8 || L == 16 || L == 32, "group size");
  v = add_dpp<0xB1>(v);
  v = add_dpp<0x4E>(v);
  v = add_dpp<0x141>(v);
  if constexpr (L >= 16) v = add_dpp<0x140>(v);
  if constexpr (L == 32) {
    // BitMode swizzle: and_mask 0x1F, or_mask 0, xor_mask 0x10 -> lane ^ 16
    const int other = __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F);
    v = v + __builtin_bit_cast(float, other);
  }
  return v;
}

}  // namespace rms
