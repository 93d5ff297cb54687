// Row-wise sum reduction for gfx950 (MI355X):   y[i] = sum_j x[i, j]   in fp32.
//
// The paper lists the kernel under the name reduce in its table of supported kernel types
// (memory-bound, measured in GB/s; its starter reduces level by level with lane shuffles).  It
// only reads: every element crosses HBM once
// and one float per row goes back, so the whole design is about keeping enough 16-byte loads
// in flight; the arithmetic (one widening and one add per element) hides under them.  The
// levels are, on CDNA4: a running sum per vector position in each lane, a
// fold of those, the DPP butterfly across the 64 lanes of a wavefront, and the wavefront
// partials added in wave order through LDS.  The order depends on the shape, the thread count
// and the row's alignment only (no atomics), so results are bit-identical from run to run.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"
#include "packed_rows.h"

namespace rms {

constexpr int kRsWave = 64;
constexpr int kRsMaxWaves = kMaxPartials;

// Adds the elements of one vector to the running sums, position by position.
template <int DT>
__device__ __forceinline__ void rs_add(u32x4 v, float (&acc)[Storage<DT>::kVec]) {
  constexpr int VEC = Storage<DT>::kVec;
  float g[VEC];
  Storage<DT>::unpack(v, g);
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] += g[k];
}

// Pairwise fold of the per-position sums.
template <int VEC>
__device__ __forceinline__ float rs_fold(const float (&acc)[VEC]) {
  if constexpr (VEC == 8) return ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  else return (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// Vectors (k0 + u) * G + t, u < COUNT, of the aligned body of a row: each load instruction
// of a wavefront covers one contiguous kilobyte.  All COUNT loads are issued before the first
// add.  Indices past the body (only possible in a thread's last vector) are clamped to the
// body's last vector so that no load sits inside a lane-dependent branch, and the lanes
// concerned add zeros instead of what the clamped load brought.  Needs nfull >= 1.
template <int DT, int COUNT, bool NT>
__device__ __forceinline__ void rs_batch(const u32x4* body, int k0, int G, int t, int nfull,
                                         float (&acc)[Storage<DT>::kVec]) {
  u32x4 v[COUNT];
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    const int idx = (k0 + u) * G + t;
    v[u] = load_vec<NT>(body + (idx < nfull ? idx : nfull - 1));
  }
  const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    if ((k0 + u) * G + t >= nfull) v[u] = zero;
    rs_add<DT>(v[u], acc);
  }
}

// One row per workgroup of G = blockDim.x threads, G any multiple of 64 up to 1024; any N
// and any element-aligned base pointer.  A row is cut into a head of single elements up to
// the next 16-byte boundary, a body of aligned 16-byte vectors and a tail of single elements,
// so the body moves with aligned 128-bit loads whatever N is.
template <int DT, int U, bool NT>
__global__ void __launch_bounds__(kRsMaxWaves * kRsWave)
rowsum_row_kernel(const void* x, float* __restrict__ y, int64_t M, int64_t N) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  static_assert(U == 4 || U == 8, "the remainder code below covers up to U - 1 vectors");
  __shared__ __attribute__((aligned(16))) float part[2][kRsMaxWaves];
  const int G = blockDim.x;
  const int waves = G / kRsWave;
  const int t = threadIdx.x;
  const int lane = t & (kRsWave - 1);
  const int wave = t / kRsWave;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    const int64_t to_boundary = (int64_t)((16u - (unsigned)((uintptr_t)xr & 15u)) & 15u) / S::kBytes;
    const int head = (int)(to_boundary < N ? to_boundary : N);
    const int nfull = (int)((N - head) / VEC);
    const int rem = (int)(N - head - (int64_t)nfull * VEC);
    const u32x4* body = reinterpret_cast<const u32x4*>(xr + head * S::kBytes);
    const int per_thread = (nfull + G - 1) / G;          // vectors k * G + t, k < per_thread

    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    int k = 0;
    for (; k + U <= per_thread; k += U) rs_batch<DT, U, NT>(body, k, G, t, nfull, acc);
    int left = per_thread - k;                           // the same for every thread of the grid
    if constexpr (U == 8) {
      if (left >= 4) { rs_batch<DT, 4, NT>(body, k, G, t, nfull, acc); k += 4; left -= 4; }
    }
    switch (left) {
      case 1: rs_batch<DT, 1, NT>(body, k, G, t, nfull, acc); break;
      case 2: rs_batch<DT, 2, NT>(body, k, G, t, nfull, acc); break;
      case 3: rs_batch<DT, 3, NT>(body, k, G, t, nfull, acc); break;
      default: break;
    }
    if (t < head + rem) {                     // at most 2 * (VEC - 1) single elements per row
      const int64_t j = t < head ? t : (int64_t)head + (int64_t)nfull * VEC + (t - head);
      acc[0] += S::load_one(x, row * N + j);
    }

    float total = wave_sum(rs_fold<VEC>(acc));
    if (waves > 1) {
      park_partial(part[slot], lane, wave, waves, total, 0.0f);
      __syncthreads();
      total = sum16(part[slot]);
      slot ^= 1;
    }
    if (t == 0) y[row] = total;
  }
}

// Short rows (16-byte aligned, at most 8 * L vectors): L = 8, 16 or 32 lanes share a row and
// a wavefront takes 64 / L consecutive rows, so a row of 256 bytes does not leave three
// quarters of a wavefront idle.  The reduction stays inside the lane group (DPP, plus one
// swizzle for L = 32).  Lanes whose row lies past M add zeros, so the cross-lane steps
// always see 64 active lanes.
template <int DT, int L, bool NT>
__global__ void __launch_bounds__(kRsWave)
rowsum_subwave_kernel(const u32x4* x, float* __restrict__ y, int64_t M, int nvec) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int ROWS = kRsWave / L;
  const int lane = threadIdx.x;
  const int s = lane % L;
  const int r = lane / L;
  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + (row_ok ? row : M - 1) * nvec;   // every load stays inside x
    const u32x4 zero = {0u, 0u, 0u, 0u};
    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    const int chunks = (nvec + L - 1) / L;                 // at most 8; the same for every lane
#pragma unroll 2
    for (int c = 0; c < chunks; ++c) {
      const int idx = c * L + s;
      u32x4 v = load_vec<NT>(xr + (idx < nvec ? idx : nvec - 1));
      if (!row_ok || idx >= nvec) v = zero;
      rs_add<DT>(v, acc);
    }
    const float total = subwave_sum<L>(rs_fold<VEC>(acc));
    if (row_ok && s == 0) y[row] = total;
  }
}

// Rows of up to 512 elements that are not whole aligned vectors (100 elements in fp16, a base
// pointer off a boundary): runs of whole rows, up to 16 KiB, are copied into LDS with aligned
// 128-bit loads that are contiguous across the workgroup (see packed_rows.h), and lane groups
// of L lanes add one row each out of LDS, E elements per lane ((E - 1) * L < N <= E * L) in index order, then the
// DPP butterfly inside the group.  Only one float per row is written, so any alignment of x
// will do.
template <int DT, int L, int E, bool NT>
__global__ void __launch_bounds__(kPackThreads)
rowsum_packed_kernel(const void* x, float* __restrict__ y, int64_t M, int N, int tile_rows) {
  using S = Storage<DT>;
  constexpr int GROUPS = kPackThreads / L;
  __shared__ u32x4 tile[kPackLdsVecs];
  const int t = threadIdx.x;
  const int sub = t % L;
  const int group = t / L;

  for (int64_t r0 = (int64_t)blockIdx.x * tile_rows; r0 < M; r0 += (int64_t)gridDim.x * tile_rows) {
    const int rows = (int)(M - r0 < tile_rows ? M - r0 : tile_rows);
    const char* src = static_cast<const char*>(x) + r0 * N * S::kBytes;
    const TileCut cut = tile_cut(src, rows * N * S::kBytes);
    const int origin = cut.skew / S::kBytes;               // tile element of the run's first element
    tile_fill<DT, NT>(src, tile, cut, t);
    __syncthreads();
    for (int first = 0; first < rows; first += GROUPS) {   // the same trip count for every thread
      const int r = first + group;
      const int at = origin + (r < rows ? r : rows - 1) * N;
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        const float value = tile_get<DT>(tile, (i < E - 1 || j < N) ? at + j : at);   // only the last step can pass N
        acc += (i == E - 1 && j >= N) ? 0.f : value;
      }
      const float total = group_sum<L>(acc);
      if (r < rows && sub == 0) y[r0 + r] = total;
    }
    __syncthreads();                                       // the next step refills the tile
  }
}

}  // namespace rms
