// Row LayerNorm forward kernels for gfx950 (MI355X).
//
//   y[i, j] = (x[i, j] - mean_i) * rsqrt(var_i + eps) * w[j] + b[j]
//   mean_i = (1/N) sum_j x[i, j],  var_i = (1/N) sum_j (x[i, j] - mean_i)^2
//
// The paper lists the kernel next to RMSNorm in its "Supported kernel types"
// table (regime Memory, metric GB/s, "Welford single-pass, float4 loads").  Its
// starter needs Welford's recurrence because it streams the row; here the row is
// read from HBM once with 16-byte non-temporal loads and then sits in registers,
// so the two moments are taken in two passes over registers, which is both
// simpler and more accurate than any one-pass formula:
//
//   1. every value is shifted by the row's first element K (a broadcast load), so
//      that the sum for the mean runs over numbers of the size of the spread, not
//      of the size of the mean: a row with mean 1000 and spread 0.01 keeps its
//      digits;
//   2. the mean of the shifted values is subtracted and the squares of the
//      centred values are summed; the centred values stay in registers for the
//      scale pass.
//
// Same variants as the other row kernels: 8/16/32 lanes per row for rows up to
// 1 KiB, one wavefront per row, one workgroup of 256..1024 threads per row (two
// LDS reductions, two barriers per row), and an element-wise three-pass
// fallback.  Fixed reduction order, no atomics: bit-identical from run to run.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"

namespace rms {

constexpr int kLnWave = 64;

__device__ __forceinline__ float ln_rstd(float spread, float n, float eps) {
  return 1.0f / __builtin_sqrtf(spread / n + eps);
}

// y chunk = round(c * rstd * w + b); b_ptr may be null (no bias).
template <int DT>
__device__ __forceinline__ u32x4 ln_scale(const float (&c)[Storage<DT>::kVec], u32x4 wv, u32x4 bv,
                                          bool has_bias, float rstd) {
  constexpr int VEC = Storage<DT>::kVec;
  float wf[VEC], bf[VEC], yf[VEC];
  Storage<DT>::unpack(wv, wf);
  Storage<DT>::unpack(bv, bf);
#pragma unroll
  for (int k = 0; k < VEC; ++k) {
    const float t = (c[k] * rstd) * wf[k];
    yf[k] = has_bias ? t + bf[k] : t;
  }
  return Storage<DT>::pack(yf);
}

// At least four wavefronts per SIMD (128 VGPRs): without the bound the compiler hoists every
// weight and bias load above the reductions and long rows drop to two wavefronts per SIMD.
template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G) __attribute__((amdgpu_waves_per_eu(4)))
layernorm_row_kernel(const u32x4* x, const u32x4* __restrict__ w, const u32x4* __restrict__ b,
                     u32x4* y, int64_t M, int nvec, float n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  __shared__ float part_a[2][WAVES];
  __shared__ float part_b[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  const bool has_bias = b != nullptr;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * G + t);
    v[CHUNKS - 1] = zero;
    if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);
    const float shift = S::load_one(xr, 0);           // K: the row's first element

    // Weight and bias: with up to four chunks per thread they are fetched now, together with
    // the row (32 more registers at most); longer rows fetch them after the reductions.
    constexpr bool EARLY = CHUNKS <= 4;
    u32x4 we[EARLY ? CHUNKS : 1], be[EARLY ? CHUNKS : 1];
    if constexpr (EARLY) {
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        const int idx = c * G + t;
        const bool live = c < CHUNKS - 1 || last_ok;
        we[c] = live ? w[idx] : zero;
        be[c] = (live && has_bias) ? b[idx] : zero;
      }
    }

    float f[CHUNKS][VEC];
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      S::unpack(v[c], f[c]);
      const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = live ? f[c][k] - shift : 0.f;
        acc[k & 3] += f[c][k];
      }
    }
    float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_a[slot][wave] = s1;
      __syncthreads();
      s1 = part_a[slot][0];
#pragma unroll
      for (int k = 1; k < WAVES; ++k) s1 += part_a[slot][k];
    }
    const float mean_shifted = s1 / n;

    float sq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = live ? f[c][k] - mean_shifted : 0.f;
        sq[k & 3] = __builtin_fmaf(f[c][k], f[c][k], sq[k & 3]);
      }
    }
    float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_b[slot][wave] = s2;
      __syncthreads();
      s2 = part_b[slot][0];
#pragma unroll
      for (int k = 1; k < WAVES; ++k) s2 += part_b[slot][k];
      slot ^= 1;
    }
    const float rstd = ln_rstd(s2, n, eps);

    // The weight and bias are fetched only now (L2 hits): the empty asm keeps the compiler
    // from hoisting sixteen more vectors above the reductions, where the centred row already
    // fills the register budget.
    const u32x4* wp = w;
    const u32x4* bp = b;
    asm volatile("" : "+s"(wp), "+s"(bp));
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * G + t;
      if (c < CHUNKS - 1 || last_ok) {
        const u32x4 wv = EARLY ? we[EARLY ? c : 0] : wp[idx];
        const u32x4 bv = EARLY ? be[EARLY ? c : 0] : (has_bias ? bp[idx] : zero);
        store_vec<NT>(yr + idx, ln_scale<DT>(f[c], wv, bv, has_bias, rstd));
      }
    }
  }
}

// L = 8, 16 or 32 lanes per row, 64 / L consecutive rows per wavefront.
template <int DT, int CHUNKS, int L, bool NT>
__global__ void __launch_bounds__(kLnWave)
layernorm_subwave_kernel(const u32x4* x, const u32x4* __restrict__ w, const u32x4* __restrict__ b,
                         u32x4* y, int64_t M, int nvec, float n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int ROWS = kLnWave / L;
  const int lane = threadIdx.x;
  const int sub = lane % L;
  const int r = lane / L;
  const bool has_bias = b != nullptr;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + (row_ok ? row : 0) * nvec;     // rows past M read row 0 and store nothing
    u32x4* yr = y + row * nvec;
    const float shift = S::load_one(xr, 0);

    float f[CHUNKS][VEC];
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
      const bool live = idx < nvec;
      S::unpack(live ? load_vec<NT>(xr + idx) : zero, f[c]);
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = live ? f[c][k] - shift : 0.f;
        acc += f[c][k];
      }
    }
    const float mean_shifted = subwave_sum<L>(acc) / n;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const bool live = c * L + sub < nvec;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = live ? f[c][k] - mean_shifted : 0.f;
        sq = __builtin_fmaf(f[c][k], f[c][k], sq);
      }
    }
    const float rstd = ln_rstd(subwave_sum<L>(sq), n, eps);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
      if (row_ok && idx < nvec) {
        const u32x4 wv = w[idx];
        const u32x4 bv = has_bias ? b[idx] : zero;
        store_vec<NT>(yr + idx, ln_scale<DT>(f[c], wv, bv, has_bias, rstd));
      }
    }
  }
}

// Element-wise fallback: any alignment, any N; three passes (shifted sum, centred
// squares, write).  In-place safe for the same reason as the other fallbacks.
template <int DT, int T>
__global__ void __launch_bounds__(T)
layernorm_generic_kernel(const void* x, const void* __restrict__ w, const void* __restrict__ b,
                         void* y, int64_t M, int64_t N, float n, float eps) {
  using S = Storage<DT>;
  constexpr int WAVES = T / kLnWave;
  __shared__ float part_a[2][WAVES];
  __shared__ float part_b[2][WAVES];
  const int tid = threadIdx.x;
  const int lane = tid & (kLnWave - 1);
  const int wave = tid / kLnWave;
  const bool has_bias = b != nullptr;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const int64_t base = row * N;
    const float shift = S::load_one(x, base);
    float acc = 0.f;
    for (int64_t j = tid; j < N; j += T) acc += S::load_one(x, base + j) - shift;
    float s1 = wave_sum(acc);
    if (lane == 0) part_a[slot][wave] = s1;
    __syncthreads();
    s1 = part_a[slot][0];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) s1 += part_a[slot][k];
    const float mean_shifted = s1 / n;

    float sq = 0.f;
    for (int64_t j = tid; j < N; j += T) {
      const float c = (S::load_one(x, base + j) - shift) - mean_shifted;
      sq = __builtin_fmaf(c, c, sq);
    }
    float s2 = wave_sum(sq);
    if (lane == 0) part_b[slot][wave] = s2;
    __syncthreads();
    s2 = part_b[slot][0];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) s2 += part_b[slot][k];
    slot ^= 1;
    const float rstd = ln_rstd(s2, n, eps);

    for (int64_t j = tid; j < N; j += T) {
      const float c = (S::load_one(x, base + j) - shift) - mean_shifted;
      const float tq = (c * rstd) * S::load_one(w, j);
      S::store_one(y, base + j, has_bias ? tq + S::load_one(b, j) : tq);
    }
  }
}

}  // namespace rms
