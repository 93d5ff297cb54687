// Row cross-entropy forward (log-sum-exp fused with the target pick) for gfx950 (MI355X).
//
//   loss[i] = log( sum_j exp(x[i, j] - m_i) ) - (x[i, t_i] - m_i),   m_i = max_j x[i, :]
//
// The paper lists the kernel in its table of supported kernel types (memory-bound, measured in
// GB/s; its starter keeps a running log-sum-exp and picks the target's logit in the same pass).
// It only reads: every logit crosses HBM once and one
// float per row goes back, so nothing has to stay in registers and rows of any length stream
// through.  Each thread keeps a running maximum and a running sum of exponentials relative to
// it (that running log-sum-exp), in batches: a batch of up to 4 16-byte vectors
// is loaded at once, its maximum taken first, the running sum rescaled at most once per batch,
// and a subtract, a multiply and one v_exp_f32 spent per element.  The per-thread pairs are
// combined in a fixed order (DPP maximum, rescale, DPP sum, LDS across wavefronts), so results
// are bit-identical from run to run.
//
// Any class count and any element-aligned base pointer run through the same code: each row
// is cut at its own 16-byte boundaries (odd counts such as 50257 shift them from row to row)
// and only the few logits outside the aligned body are read one by one.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"
#include "packed_rows.h"

namespace rms {

constexpr int kCeWave = 64;
constexpr float kCeNegInf = -__builtin_inff();
constexpr float kCeLog2e = 1.44269502162933349609375f;

// 2^((a - b) log2 e) for a <= b, with the convention that equal arguments (including two
// infinities of the same sign) give exactly 1.
__device__ __forceinline__ float ce_rescale(float a, float b) {
  return a == b ? 1.0f : __builtin_amdgcn_exp2f((a - b) * kCeLog2e);
}

// ln(s) for the kernels that take one logarithm per short row, where it would otherwise be a
// sixth of all instructions: the hardware base-2 logarithm (1 ulp) times ln 2.  The sum s lies in
// [1, N] (the maximum contributes exp(0)), so the result's absolute error stays below 1e-6,
// a tenth of the comparison's absolute allowance; NaN and infinity pass through.
__device__ __forceinline__ float ce_log_fast(float s) {
  return __builtin_amdgcn_logf(s) * 0.693147182464599609375f;
}

// Folds COUNT values into the running (m, s) pair.  Each term is 2^((f - m) log2 e): the
// difference is formed first (exact for the 16-bit types when the exponents are close,
// correctly rounded otherwise), so the error of a term grows with its distance from the
// maximum, where the term is small, and not with the size of the logits; rows of large
// identical values (the paper's stability probe for softmax-like kernels, Section 4 stage 3)
// give exactly COUNT.
template <int COUNT>
__device__ __forceinline__ void ce_fold(const float (&f)[COUNT], float& m, float& s) {
  float bm = m;
#pragma unroll
  for (int k = 0; k < COUNT; ++k) bm = __builtin_fmaxf(bm, f[k]);
  s *= ce_rescale(m, bm);
  m = bm;
  // only -inf so far: every term is exp(-inf) = 0; subtracting 0 keeps -inf - (-inf) from NaN
  const float ref = bm == kCeNegInf ? 0.0f : bm;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < COUNT; ++k) acc[k & 3] += __builtin_amdgcn_exp2f((f[k] - ref) * kCeLog2e);
  s += (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// 16 bytes of -inf in the storage type: what a thread folds where the row has no vector left.
template <int DT>
__device__ __forceinline__ u32x4 ce_neg_inf_vec() {
  constexpr uint32_t p = DT == kFp32 ? 0xFF800000u : DT == kFp16 ? 0xFC00FC00u : 0xFF80FF80u;
  u32x4 v = {p, p, p, p};
  return v;
}

// Vectors (k0 + u) * G + t, u < COUNT, of the aligned body of a row: each load instruction
// of a wavefront covers one contiguous kilobyte.  Indices past the body (only possible in a
// thread's last vector) are clamped to the body's last vector, so that every load is
// unconditional (a load inside a lane-dependent branch makes the compiler wait for the loads
// before it, and the loads of a batch would go out one after the other); the lanes concerned
// then fold -inf instead of what the clamped load brought.  Needs nfull >= 1.
template <int DT, int COUNT, bool NT>
__device__ __forceinline__ void ce_batch(const u32x4* body, int k0, int G, int t, int nfull,
                                         float& m, float& s) {
  constexpr int VEC = Storage<DT>::kVec;
  u32x4 v[COUNT];
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    const int idx = (k0 + u) * G + t;
    v[u] = load_vec<NT>(body + (idx < nfull ? idx : nfull - 1));
  }
  float f[COUNT * VEC];
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    if ((k0 + u) * G + t >= nfull) v[u] = ce_neg_inf_vec<DT>();
    float g[VEC];
    Storage<DT>::unpack(v[u], g);
#pragma unroll
    for (int k = 0; k < VEC; ++k) f[u * VEC + k] = g[k];
  }
  ce_fold<COUNT * VEC>(f, m, s);
}

constexpr int kCeMaxWaves = kMaxPartials;

// One row per workgroup of G = blockDim.x threads, G any multiple of 64 up to 1024 (the host
// picks it so that the vectors of a row divide evenly among the threads).
template <int DT, int U, bool NT>
__global__ void __launch_bounds__(kCeMaxWaves * kCeWave)
crossentropy_row_kernel(const void* x, const int64_t* __restrict__ target, float* __restrict__ loss,
                        float* __restrict__ lse_out, int64_t M, int64_t N) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  static_assert(U == 4, "the remainder switch below covers 1..3 vectors");
  __shared__ __attribute__((aligned(16))) float part_m[2][kCeMaxWaves];
  __shared__ __attribute__((aligned(16))) float part_s[2][kCeMaxWaves];
  const int G = blockDim.x;
  const int waves = G / kCeWave;
  const int t = threadIdx.x;
  const int lane = t & (kCeWave - 1);
  const int wave = t / kCeWave;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    // A row is cut into a head of single logits up to the next 16-byte boundary, a body of
    // aligned 16-byte vectors, and a tail of single logits: whatever N and the base pointer
    // are, the body moves with aligned 128-bit loads.
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    const int64_t to_boundary = (int64_t)((16u - (unsigned)((uintptr_t)xr & 15u)) & 15u) / S::kBytes;
    const int head = (int)(to_boundary < N ? to_boundary : N);
    const int nfull = (int)((N - head) / VEC);
    const int rem = (int)(N - head - (int64_t)nfull * VEC);
    const u32x4* body = reinterpret_cast<const u32x4*>(xr + head * S::kBytes);
    const int per_thread = (nfull + G - 1) / G;          // vectors k * G + t, k < per_thread
    float m = kCeNegInf, s = 0.f;

    // Batches of U vectors per thread, one batch at a time (requesting the next batch before
    // folding the current one was measured and is slower: more bytes in flight per compute
    // unit, not fewer stalls), then the 1..3 vectors left over, so no load is wasted.
    int k = 0;
    for (; k + U <= per_thread; k += U) ce_batch<DT, U, NT>(body, k, G, t, nfull, m, s);
    switch (per_thread - k) {                            // the same for every thread of the grid
      case 1: ce_batch<DT, 1, NT>(body, k, G, t, nfull, m, s); break;
      case 2: ce_batch<DT, 2, NT>(body, k, G, t, nfull, m, s); break;
      case 3: ce_batch<DT, 3, NT>(body, k, G, t, nfull, m, s); break;
      default: break;
    }
    if (t < head + rem) {                     // at most 2 * (VEC - 1) single logits per row
      const int64_t j = t < head ? t : (int64_t)head + (int64_t)nfull * VEC + (t - head);
      const float single[1] = {S::load_one(x, row * N + j)};
      ce_fold<1>(single, m, s);
    }

    // combine the per-thread pairs: row maximum, rescale, row sum
    float row_m = wave_max(m);
    if (waves > 1) {
      park_partial(part_m[slot], lane, wave, waves, row_m, kCeNegInf);
      __syncthreads();
      row_m = max16(part_m[slot]);
    }
    float row_s = wave_sum(s * ce_rescale(m, row_m));
    if (waves > 1) {
      park_partial(part_s[slot], lane, wave, waves, row_s, 0.0f);
      __syncthreads();
      row_s = sum16(part_s[slot]);
      slot ^= 1;
    }

    if (t == 0) {
      // a row of -inf only has no maximum to subtract: NaN, as the formula gives
      const float log_s = row_m == kCeNegInf ? __builtin_nanf("") : __builtin_logf(row_s);
      if (lse_out) lse_out[row] = row_m + log_s;
      const int64_t cls = target[row];
      float out = 0.0f;                                   // target outside [0, N): ignored row
      if (cls >= 0 && cls < N) out = log_s - (S::load_one(x, row * N + cls) - row_m);
      loss[row] = out;
    }
  }
}

// Few classes (16-byte aligned rows of at most 8 * L vectors: a 1000-way classifier, a
// 128-way head): one workgroup per row would leave most of a wavefront idle and pay a launch
// slot per kilobyte, so L = 8, 16 or 32 lanes share a row and a wavefront takes 64 / L
// consecutive rows.  Same batches, same online pair per lane; the combination stays inside
// the lane group (DPP, one swizzle for L = 32), so there is no LDS and no barrier.  Lanes
// whose row lies past M work on the last row and store nothing, so the cross-lane steps
// always see 64 active lanes and every load stays inside x.
template <int DT, int L, int U, bool NT>
__global__ void __launch_bounds__(kCeWave)
crossentropy_subwave_kernel(const u32x4* x, const int64_t* __restrict__ target,
                            float* __restrict__ loss, float* __restrict__ lse_out, int64_t M,
                            int64_t N, int nvec) {
  using S = Storage<DT>;
  static_assert(U == 4, "the remainder switch below covers 1..3 vectors");
  constexpr int ROWS = kCeWave / L;
  const int lane = threadIdx.x;
  const int sub = lane % L;
  const int r = lane / L;
  const int per_lane = (nvec + L - 1) / L;                // at most 8; the same for every lane
  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + (row_ok ? row : M - 1) * nvec;
    float m = kCeNegInf, s = 0.f;
    int k = 0;
    for (; k + U <= per_lane; k += U) ce_batch<DT, U, NT>(xr, k, L, sub, nvec, m, s);
    switch (per_lane - k) {
      case 1: ce_batch<DT, 1, NT>(xr, k, L, sub, nvec, m, s); break;
      case 2: ce_batch<DT, 2, NT>(xr, k, L, sub, nvec, m, s); break;
      case 3: ce_batch<DT, 3, NT>(xr, k, L, sub, nvec, m, s); break;
      default: break;
    }
    const float row_m = subwave_max<L>(m);
    const float row_s = subwave_sum<L>(s * ce_rescale(m, row_m));
    if (row_ok && sub == 0) {
      const float log_s = row_m == kCeNegInf ? __builtin_nanf("") : ce_log_fast(row_s);
      if (lse_out) lse_out[row] = row_m + log_s;
      const int64_t cls = target[row];
      float out = 0.0f;                                   // target outside [0, N): ignored row
      if (cls >= 0 && cls < N) out = log_s - (S::load_one(x, row * N + cls) - row_m);
      loss[row] = out;
    }
  }
}

// Up to 512 classes in rows that are not 16-byte aligned (100 classes in fp16, 1000 / 3 of
// anything): runs of whole rows, up to 16 KiB, are copied into LDS with aligned 128-bit loads
// that are contiguous across the workgroup (see packed_rows.h), and lane groups of L lanes take
// one row each out of LDS, E logits per lane with (E - 1) * L < N <= E * L, with the same online pair and the same
// DPP-only combination as the lane-group kernel above.  Nothing is written but one float per
// row (two with the log-sum-exp), so any alignment of x will do.
template <int DT, int L, int E, bool NT>
__global__ void __launch_bounds__(kPackThreads)
crossentropy_packed_kernel(const void* x, const int64_t* __restrict__ target, float* __restrict__ loss,
                           float* __restrict__ lse_out, int64_t M, int N, int tile_rows) {
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
      float f[E];
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        f[i] = tile_get<DT>(tile, (i < E - 1 || j < N) ? at + j : at);   // only the last step can pass N
        if (i == E - 1 && j >= N) f[i] = kCeNegInf;
      }
      float m = kCeNegInf, s = 0.f;
      ce_fold<E>(f, m, s);
      const float row_m = group_max<L>(m);
      const float row_s = group_sum<L>(s * ce_rescale(m, row_m));
      if (r < rows && sub == 0) {
        const int64_t row = r0 + r;
        const float log_s = row_m == kCeNegInf ? __builtin_nanf("") : ce_log_fast(row_s);
        if (lse_out) lse_out[row] = row_m + log_s;
        const int64_t cls = target[row];
        float out = 0.0f;                                  // target outside [0, N): ignored row
        if (cls >= 0 && cls < N) out = log_s - (tile_get<DT>(tile, at + (int)cls) - row_m);
        loss[row] = out;
      }
    }
    __syncthreads();                                       // the next step refills the tile
  }
}

}  // namespace rms
