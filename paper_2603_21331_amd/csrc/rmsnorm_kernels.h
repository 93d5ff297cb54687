// RMSNorm forward kernels for gfx950 (MI355X).
//
//   y[i, j] = x[i, j] * rsqrt(mean_j x[i, :]^2 + eps) * w[j]
//
// The kernel is memory-bound (the paper's kernel table lists it under regime
// "Memory", metric GB/s), so each design decision below serves one aim: move
// every byte of x and y across HBM exactly once, in 16-byte accesses, with as
// many of them in flight as possible.  The paper credits its own gain to a
// single fused pass and to folding the weight multiply into the epilogue
// (Section 7.1 key findings, Section 7.3 tier 3); both hold here, and the row
// additionally stays in registers between the reduce and the scale, so the
// second pass costs no memory traffic at all.
//
//  * rmsnorm_wave_kernel  : one 64-lane wavefront per row.  No LDS, no barrier.
//  * rmsnorm_block_kernel : one workgroup per row, per-wave partial sums
//                           combined through LDS in wave order.
//  * rmsnorm_generic_kernel: element-wise two-pass fallback for rows that are
//                           not 16-byte aligned or too long for registers.
//
// All sums are fp32, in an order fixed by (kernel, shape) alone: no atomics,
// so repeated runs give identical bits.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"

namespace rms {

constexpr int kWave = 64;

// Per-lane sum of squares of CHUNKS vectors, four independent fp32 chains.
template <int DT, int CHUNKS>
__device__ __forceinline__ float lane_sum_sq(const u32x4 (&v)[CHUNKS]) {
  constexpr int VEC = Storage<DT>::kVec;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    float f[VEC];
    Storage<DT>::unpack(v[c], f);
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k & 3] = __builtin_fmaf(f[k], f[k], acc[k & 3]);
  }
  return (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// rstd = 1 / sqrt(sum / n + eps), with correctly rounded divide and root: it
// runs once per row, so the "fast rsqrt" of the paper's starter would buy
// nothing here and would cost accuracy on subnormal sums.
__device__ __forceinline__ float row_rstd(float sum_sq, float n, float eps) {
  return 1.0f / __builtin_sqrtf(sum_sq / n + eps);
}

// y = round((x * rstd) * w) for one vector.
template <int DT>
__device__ __forceinline__ u32x4 scale_vec(u32x4 xv, u32x4 wv, float rstd) {
  constexpr int VEC = Storage<DT>::kVec;
  float xf[VEC], wf[VEC], yf[VEC];
  Storage<DT>::unpack(xv, xf);
  Storage<DT>::unpack(wv, wf);
#pragma unroll
  for (int k = 0; k < VEC; ++k) yf[k] = (xf[k] * rstd) * wf[k];
  return Storage<DT>::pack(yf);
}

// ---------------------------------------------------------------------------
// One wavefront per row.  Vector c * 64 + lane of the row goes to lane `lane`,
// chunk c, so each load instruction covers 1 KiB of contiguous memory.
// CHUNKS = ceil(nvec / 64): only the last chunk can be ragged.  All CHUNKS
// loads are issued before the first use.  The grid may be smaller than the
// number of rows; each wavefront then strides over rows.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int WAVES_PER_BLOCK, bool NT>
__global__ void __launch_bounds__(WAVES_PER_BLOCK* kWave)
rmsnorm_wave_kernel(const u32x4* x, const u32x4* __restrict__ w, u32x4* y,
                    int64_t M, int nvec, float n, float eps) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t row_stride = (int64_t)gridDim.x * WAVES_PER_BLOCK;
  const int last = (CHUNKS - 1) * kWave + lane;
  const bool last_ok = last < nvec;

  for (int64_t row = (int64_t)blockIdx.x * WAVES_PER_BLOCK + wave; row < M; row += row_stride) {
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * kWave + lane);
    {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      v[CHUNKS - 1] = zero;
      if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);
    }

    const float total = wave_sum(lane_sum_sq<DT, CHUNKS>(v));
    const float rstd = row_rstd(total, n, eps);

#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) {
      const int idx = c * kWave + lane;
      store_vec<NT>(yr + idx, scale_vec<DT>(v[c], w[idx], rstd));
    }
    if (last_ok) store_vec<NT>(yr + last, scale_vec<DT>(v[CHUNKS - 1], w[last], rstd));
  }
}

// ---------------------------------------------------------------------------
// One workgroup of T threads per row, for rows too long for one wavefront's
// registers.  Vector c * T + tid goes to thread tid, chunk c.  Each wavefront
// reduces its own lanes with DPP, lane 0 parks the partial in LDS, and after
// one barrier every thread adds the T/64 partials in wave order.  Two LDS
// slots alternate between consecutive rows, so one barrier per row is enough.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int T, bool NT>
__global__ void __launch_bounds__(T)
rmsnorm_block_kernel(const u32x4* x, const u32x4* __restrict__ w, u32x4* y,
                     int64_t M, int nvec, float n, float eps) {
  constexpr int WAVES = T / kWave;
  __shared__ float partial[2][WAVES];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int last = (CHUNKS - 1) * T + tid;
  const bool last_ok = last < nvec;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * T + tid);
    {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      v[CHUNKS - 1] = zero;
      if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);
    }

    const float wsum = wave_sum(lane_sum_sq<DT, CHUNKS>(v));
    if (lane == 0) partial[slot][wave] = wsum;
    __syncthreads();
    float total = partial[slot][0];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) total += partial[slot][k];
    slot ^= 1;
    const float rstd = row_rstd(total, n, eps);

#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) {
      const int idx = c * T + tid;
      store_vec<NT>(yr + idx, scale_vec<DT>(v[c], w[idx], rstd));
    }
    if (last_ok) store_vec<NT>(yr + last, scale_vec<DT>(v[CHUNKS - 1], w[last], rstd));
  }
}

// ---------------------------------------------------------------------------
// Element-wise fallback: any element alignment, any N.  One workgroup per row,
// thread tid takes elements tid, tid + T, ...; x is read a second time for the
// scale pass (from cache when the row fits).  In-place safe: the barrier in
// the reduction separates every read of pass one from every write of pass two,
// and in pass two each thread reads an element before it overwrites it.
// ---------------------------------------------------------------------------
template <int DT, int T>
__global__ void __launch_bounds__(T)
rmsnorm_generic_kernel(const void* x, const void* __restrict__ w, void* y,
                       int64_t M, int64_t N, float n, float eps) {
  constexpr int WAVES = T / kWave;
  __shared__ float partial[2][WAVES];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const int64_t base = row * N;
    float acc = 0.f;
    for (int64_t j = tid; j < N; j += T) {
      const float f = Storage<DT>::load_one(x, base + j);
      acc = __builtin_fmaf(f, f, acc);
    }
    const float wsum = wave_sum(acc);
    if (lane == 0) partial[slot][wave] = wsum;
    __syncthreads();
    float total = partial[slot][0];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) total += partial[slot][k];
    slot ^= 1;
    const float rstd = row_rstd(total, n, eps);

    for (int64_t j = tid; j < N; j += T) {
      const float f = Storage<DT>::load_one(x, base + j);
      const float g = Storage<DT>::load_one(w, j);
      Storage<DT>::store_one(y, base + j, (f * rstd) * g);
    }
  }
}

// Streaming copy with the kernels' access pattern (measurement aid).
template <int UNROLL, int T>
__global__ void __launch_bounds__(T)
calib_copy_kernel(const u32x4* src, u32x4* dst, int64_t nvec) {
  const int64_t tile = (int64_t)UNROLL * T;
  for (int64_t base = (int64_t)blockIdx.x * tile; base < nvec; base += (int64_t)gridDim.x * tile) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t i = base + (int64_t)u * T + threadIdx.x;
      if (i < nvec) v[u] = load_vec<true>(src + i);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t i = base + (int64_t)u * T + threadIdx.x;
      if (i < nvec) store_vec<true>(dst + i, v[u]);
    }
  }
}

}  // namespace rms
