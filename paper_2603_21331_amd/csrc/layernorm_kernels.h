// Row LayerNorm forward kernels for gfx950 (MI355X).
//
//   y[i, j] = (x[i, j] - mean_i) * rsqrt(var_i + eps) * w[j] + b[j]
//   mean_i = (1/N) sum_j x[i, j],  var_i = (1/N) sum_j (x[i, j] - mean_i)^2
//
// The paper lists the kernel next to RMSNorm in its table of supported kernel
// types (memory-bound, measured in GB/s; its starter takes both moments in one
// pass with Welford's recurrence over 16-byte loads).  The starter needs the
// recurrence because it streams the row; here the row is
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
// LDS reductions, two barriers per row) either launched per row or, for rows of
// at most 24 elements per thread, resident with weight and bias in registers
// (walking a fixed stride, or in large launches drawing its rows from counters:
// layernorm_queue_kernel), and an element-wise three-pass fallback.  Fixed
// reduction order within a row, and a row's result does not depend on which
// workgroup takes it: bit-identical from run to run.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"
#include "packed_rows.h"

namespace rms {

constexpr int kLnWave = 64;

__device__ __forceinline__ float ln_rstd(float spread, float n, float eps) {
  return 1.0f / __builtin_sqrtf(spread / n + eps);
}

// The same value through the hardware reciprocal square root and one Newton step (within
// 1.5 ulp of the exact value); arguments that are not normal numbers (zero or subnormal: a
// constant row with eps = 0; infinite; NaN) take the plain formula.  It sits on every
// thread's path between the arrival of the row and the first store.
__device__ __forceinline__ float ln_rstd_fast(float spread, float inv_n, float eps) {
  const float a = __builtin_fmaf(spread, inv_n, eps);
  if (__builtin_expect(!__builtin_isnormal(a) || a < 0.0f, 0)) return 1.0f / __builtin_sqrtf(a);
  const float y0 = __builtin_amdgcn_rsqf(a);
  const float e = __builtin_fmaf(-a * y0, y0, 1.0f);
  return __builtin_fmaf(0.5f * y0, e, y0);
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
//
// 1024 threads of a 16-bit type (rows of 16 k elements and more): the fp32 form of the row
// would leave room for one workgroup per compute unit, with nothing to overlap its load,
// reduce and store phases.  Those instances keep the row packed and widen, shift and centre it
// again in each of the three passes (the same operations on the same values, so the same bits):
// 64 registers, two workgroups per compute unit.
template <int DT, int G>
inline constexpr bool kLnLean = G == 1024 && DT != kFp32;

template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G) __attribute__((amdgpu_waves_per_eu(kLnLean<DT, G> ? 8 : 4)))
layernorm_row_kernel(const u32x4* x, const u32x4* __restrict__ w, const u32x4* __restrict__ b,
                     u32x4* y, int64_t M, int nvec, float n, float eps, int xcd_blocks) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  constexpr bool LEAN = kLnLean<DT, G>;
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  const bool has_bias = b != nullptr;
  const float inv_n = 1.0f / n;       // the mean and the reciprocal root as in the resident kernel
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;

  for (int64_t row = flat_first_row(blockIdx.x, xcd_blocks); row < M; row += gridDim.x) {
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * G + t);
    v[CHUNKS - 1] = zero;
    if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);
    const float shift = S::load_one(xr, 0);           // K: the row's first element

    if constexpr (LEAN) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        float g[VEC];
        S::unpack(v[c], g);
        const float sub = (c < CHUNKS - 1 || last_ok) ? shift : 0.f;   // a chunk past the end holds zeros
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k & 3] += g[k] - sub;
      }
      float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
      if (lane == 0) part_a[slot][wave] = s1;
      __syncthreads();
      s1 = sum_waves<WAVES>(part_a[slot]);
      const float mean_shifted = s1 * inv_n;
      forget_unpacked<CHUNKS>(v);
      float sq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        float g[VEC];
        S::unpack(v[c], g);
        const bool live = c < CHUNKS - 1 || last_ok;
        const float sub = live ? shift : 0.f, sub2 = live ? mean_shifted : 0.f;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
          const float d = (g[k] - sub) - sub2;
          sq[k & 3] = __builtin_fmaf(d, d, sq[k & 3]);
        }
      }
      float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
      if (lane == 0) part_b[slot][wave] = s2;
      __syncthreads();
      s2 = sum_waves<WAVES>(part_b[slot]);
      slot ^= 1;
      const float rstd = ln_rstd_fast(s2, inv_n, eps);
      forget_unpacked<CHUNKS>(v);
      const u32x4* wp = w;
      const u32x4* bp = b;
      asm volatile("" : "+s"(wp), "+s"(bp));               // keeps the loads below the reductions
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        const int idx = c * G + t;
        if (c < CHUNKS - 1 || last_ok) {
          float g[VEC];
          S::unpack(v[c], g);
#pragma unroll
          for (int k = 0; k < VEC; ++k) g[k] = (g[k] - shift) - mean_shifted;
          store_vec<NT>(yr + idx, ln_scale<DT>(g, wp[idx], has_bias ? bp[idx] : zero, has_bias, rstd));
        }
      }
      continue;
    }

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
      // a chunk past the end of the row holds zeros; subtracting zero keeps it at zero
      const float sub = (c < CHUNKS - 1 || last_ok) ? shift : 0.f;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] -= sub;
        acc[k & 3] += f[c][k];
      }
    }
    float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_a[slot][wave] = s1;
      __syncthreads();
      s1 = sum_waves<WAVES>(part_a[slot]);
    }
    const float mean_shifted = s1 * inv_n;

    float sq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const float sub = (c < CHUNKS - 1 || last_ok) ? mean_shifted : 0.f;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] -= sub;
        sq[k & 3] = __builtin_fmaf(f[c][k], f[c][k], sq[k & 3]);
      }
    }
    float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_b[slot][wave] = s2;
      __syncthreads();
      s2 = sum_waves<WAVES>(part_b[slot]);
      slot ^= 1;
    }
    const float rstd = ln_rstd_fast(s2, inv_n, eps);

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

// ---------------------------------------------------------------------------
// Resident workgroups.  Measured on MI355X, a one-row-per-workgroup LayerNorm spends 12 % of
// its time at N = 8192 re-reading weight and bias from L2 for every row (with the row itself
// that is three streams through the compute unit's vector cache and the L2 crossbar instead
// of one), and a fifth of its vector-ALU work widening them.  Here a grid of a few workgroups
// per compute unit stays for the whole launch: each workgroup widens its slices of weight
// and bias to fp32 ONCE, keeps them in registers, and walks rows blockIdx.x,
// blockIdx.x + gridDim.x, ...  Two packed register copies of a row take turns: while one is
// reduced, scaled and stored, the other is being filled with the workgroup's next row (the
// last step requests its own row again, a cache hit, so that no load hides in a branch, and
// the loop is unrolled twice so that no register is copied from one copy to the other,
// which would make the loop wait for loads it has only just issued).
//
// Same arithmetic as layernorm_row_kernel (shift by the row's first element, mean of the
// shifted values, squares of the centred values; two reductions, two barriers).  For rows of
// at most 24 elements per thread (CHUNKS * VEC), which is what fits in registers next to
// weight and bias; ragged last chunks are allowed.
// ---------------------------------------------------------------------------
// First element of a row as raw bits (no arithmetic hangs on the load), and its value.
template <int DT>
__device__ __forceinline__ uint32_t ln_first_raw(const u32x4* row) {
  if constexpr (DT == kFp32) return *reinterpret_cast<const uint32_t*>(row);
  else return *reinterpret_cast<const uint16_t*>(row);
}
template <int DT>
__device__ __forceinline__ float ln_first_value(uint32_t raw) {
  if constexpr (DT == kFp32) return as_f32(raw);
  else if constexpr (DT == kBf16) return as_f32(raw << 16);
  else return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(raw)));
}

// One row: requests row `pre` into (nxt, nxt_raw), then reduces, scales and stores the row
// held in (cur, cur_raw).
template <int DT, int CHUNKS, int G, bool NT>
__device__ __forceinline__ void ln_resident_step(
    const u32x4* x, u32x4* y, int64_t row, int64_t pre, int nvec, int t, int lane, int wave,
    bool last_ok, const u32x4 (&cur)[CHUNKS], uint32_t cur_raw, u32x4 (&nxt)[CHUNKS],
    uint32_t& nxt_raw, const float (&wf)[CHUNKS][Storage<DT>::kVec],
    const float (&bf)[CHUNKS][Storage<DT>::kVec], float inv_n, float eps,
    float (&part_a)[G / kLnWave], float (&part_b)[G / kLnWave]) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  const int last = (CHUNKS - 1) * G + t;
#pragma unroll
  for (int c = 0; c < CHUNKS - 1; ++c) nxt[c] = load_vec<NT>(x + pre * nvec + c * G + t);
  nxt[CHUNKS - 1] = load_vec<NT>(x + pre * nvec + (last_ok ? last : nvec - 1));
  nxt_raw = ln_first_raw<DT>(x + pre * nvec);

  const float shift = ln_first_value<DT>(cur_raw);
  float d[CHUNKS][VEC];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    S::unpack(cur[c], d[c]);
    const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      d[c][k] = live ? d[c][k] - shift : 0.f;
      acc[k & 3] += d[c][k];
    }
  }
  float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
  if constexpr (WAVES > 1) {
    if (lane == 0) part_a[wave] = s1;
    __syncthreads();
    s1 = sum_waves<WAVES>(part_a);
  }
  const float mean_shifted = s1 * inv_n;

  float sq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      d[c][k] = live ? d[c][k] - mean_shifted : 0.f;
      sq[k & 3] = __builtin_fmaf(d[c][k], d[c][k], sq[k & 3]);
    }
  }
  float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
  if constexpr (WAVES > 1) {
    if (lane == 0) part_b[wave] = s2;
    __syncthreads();
    s2 = sum_waves<WAVES>(part_b);
  }
  const float rstd = ln_rstd_fast(s2, inv_n, eps);

  const __amdgpu_buffer_rsrc_t yr = row_resource(y + row * nvec, nvec * 16);
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    float yf[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) yf[k] = (d[c][k] * rstd) * wf[c][k] + bf[c][k];
    if (c < CHUNKS - 1 || last_ok) store_row_vec<NT>(yr, c * G + t, S::pack(yf));
  }
}

template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G)
layernorm_row_resident_kernel(const u32x4* x, const u32x4* __restrict__ w,
                              const u32x4* __restrict__ b, u32x4* y, int64_t M, int nvec,
                              float inv_n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  const int64_t stride = gridDim.x;
  int64_t row = blockIdx.x;
  if (row >= M) return;

  u32x4 ra[CHUNKS], rb[CHUNKS];
  uint32_t raw_a, raw_b = 0;
#pragma unroll
  for (int c = 0; c < CHUNKS - 1; ++c) ra[c] = load_vec<NT>(x + row * nvec + c * G + t);
  ra[CHUNKS - 1] = load_vec<NT>(x + row * nvec + (last_ok ? last : nvec - 1));
  raw_a = ln_first_raw<DT>(x + row * nvec);

  float wf[CHUNKS][VEC], bf[CHUNKS][VEC];
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    const int idx = (c < CHUNKS - 1 || last_ok) ? c * G + t : nvec - 1;
    S::unpack(w[idx], wf[c]);
    S::unpack(b != nullptr ? b[idx] : zero, bf[c]);
  }
  while (true) {
    int64_t next = row + stride;
    ln_resident_step<DT, CHUNKS, G, NT>(x, y, row, next < M ? next : row, nvec, t, lane, wave,
                                        last_ok, ra, raw_a, rb, raw_b, wf, bf, inv_n, eps,
                                        part_a[0], part_b[0]);
    if (next >= M) break;                              // uniform over the workgroup
    row = next;
    next = row + stride;
    ln_resident_step<DT, CHUNKS, G, NT>(x, y, row, next < M ? next : row, nvec, t, lane, wave,
                                        last_ok, rb, raw_b, ra, raw_a, wf, bf, inv_n, eps,
                                        part_a[1], part_b[1]);
    if (next >= M) break;
    row = next;
  }
}

// ---------------------------------------------------------------------------
// Work-queue form of the resident kernel, for launches of a few hundred megabytes: the
// resident workgroups draw their rows from counters in device memory instead of walking a
// fixed stride, which evens out the compute units, and take them in blocks of consecutive
// rows per XCD.  Row order and counters are those of RMSNorm's work-queue kernel: workgroup b
// belongs to shard b % shards, the rows are cut into blocks of 2^block_shift rows, block k
// belongs to shard k % shards; shard s owns counters[s * kLnQueueStride] (slots handed out
// beyond the two every member takes statically) and counters[s * kLnQueueStride + 1] (members
// that have finished); both are zero between launches (the last member of a shard to finish
// puts them back), and launches that share counters must not overlap.  Nobody waits for
// anybody, so the grid drains whatever the order the hardware starts it in.
//
// Who draws.  The compiler waits for a returning atomic where it issues it, with a count that
// covers every load the wavefront has in flight; a wavefront that has its next row requested
// would stall there in every step, and the workgroup behind it at the next barrier.  So the
// workgroup has one wavefront more than the G threads that hold the row: it touches no row,
// draws one ticket per step (for the row after next), leaves it in LDS before the step's
// first barrier and takes part in both barriers.  The workers read it after that barrier.
// ---------------------------------------------------------------------------
constexpr int kLnQueueStride = 32;      // counters of neighbouring shards are 128 bytes apart
constexpr int kLnQueueMaxShards = 32;

// A thread's slices of weight and bias.  Widened to fp32 once where the registers allow it
// (up to 24 elements per thread); kept as loaded and widened again in every step beyond that
// (32 elements of a 16-bit type: the widened form would not leave room for two row copies).
template <int DT, int CHUNKS, bool PACKED>
struct LnSlices;
template <int DT, int CHUNKS>
struct LnSlices<DT, CHUNKS, false> {
  float w[CHUNKS][Storage<DT>::kVec], b[CHUNKS][Storage<DT>::kVec];
  __device__ __forceinline__ void set(int c, u32x4 wv, u32x4 bv) {
    Storage<DT>::unpack(wv, w[c]);
    Storage<DT>::unpack(bv, b[c]);
  }
  __device__ __forceinline__ void step() {}
  __device__ __forceinline__ void widen(int) {}
  __device__ __forceinline__ float scale(int c, int k, float v) const { return v * w[c][k] + b[c][k]; }
};
template <int DT, int CHUNKS>
struct LnSlices<DT, CHUNKS, true> {
  u32x4 w[CHUNKS], b[CHUNKS];
  float wf[Storage<DT>::kVec], bf[Storage<DT>::kVec];   // chunk c, between widen(c) and the next
  __device__ __forceinline__ void set(int c, u32x4 wv, u32x4 bv) {
    w[c] = wv;
    b[c] = bv;
  }
  // once per step: the compiler must not carry widened values from one step to the next
  __device__ __forceinline__ void step() {
    forget_unpacked<CHUNKS>(w);
    forget_unpacked<CHUNKS>(b);
  }
  __device__ __forceinline__ void widen(int c) {
    Storage<DT>::unpack(w[c], wf);
    Storage<DT>::unpack(b[c], bf);
  }
  __device__ __forceinline__ float scale(int, int k, float v) const { return v * wf[k] + bf[k]; }
};

// One step: requests row `pre` into (nxt, nxt_raw), then reduces, scales and stores row `row`
// held in (cur, cur_raw); the extra wavefront draws.  Returns the ticket drawn in this step.
template <int DT, int CHUNKS, int G, bool NT, bool PACKED>
__device__ __forceinline__ unsigned ln_queue_step(
    const u32x4* x, u32x4* y, int64_t row, int64_t pre, int nvec, int t, int lane, int wave,
    bool last_ok, const u32x4 (&cur)[CHUNKS], uint32_t cur_raw, u32x4 (&nxt)[CHUNKS],
    uint32_t& nxt_raw, LnSlices<DT, CHUNKS, PACKED>& wb, float inv_n, float eps, unsigned* q,
    float (&part_a)[G / kLnWave], float (&part_b)[G / kLnWave], unsigned& ticket) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  const bool worker = t < G;
  const int last = (CHUNKS - 1) * G + t;
  float d[CHUNKS][VEC];
  if (worker) {
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) nxt[c] = load_vec<NT>(x + pre * nvec + c * G + t);
    nxt[CHUNKS - 1] = load_vec<NT>(x + pre * nvec + (last_ok ? last : nvec - 1));
    nxt_raw = ln_first_raw<DT>(x + pre * nvec);

    const float shift = ln_first_value<DT>(cur_raw);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      S::unpack(cur[c], d[c]);
      const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        d[c][k] = live ? d[c][k] - shift : 0.f;
        acc[k & 3] += d[c][k];
      }
    }
    const float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if (lane == 0) part_a[wave] = s1;
  } else if (lane == 0) {
    ticket = atomicAdd(q, 1u);
  }
  __syncthreads();
  const unsigned drawn = ticket;
  if (worker) {
    const float mean_shifted = sum_waves<WAVES>(part_a) * inv_n;
    float sq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const bool live = c < CHUNKS - 1 || last_ok;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        d[c][k] = live ? d[c][k] - mean_shifted : 0.f;
        sq[k & 3] = __builtin_fmaf(d[c][k], d[c][k], sq[k & 3]);
      }
    }
    const float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
    if (lane == 0) part_b[wave] = s2;
  }
  __syncthreads();
  if (worker) {
    const float rstd = ln_rstd_fast(sum_waves<WAVES>(part_b), inv_n, eps);
    const __amdgpu_buffer_rsrc_t yr = row_resource(y + row * nvec, nvec * 16);
    wb.step();
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      float yf[VEC];
      wb.widen(c);
#pragma unroll
      for (int k = 0; k < VEC; ++k) yf[k] = wb.scale(c, k, d[c][k] * rstd);
      if (c < CHUNKS - 1 || last_ok) store_row_vec<NT>(yr, c * G + t, S::pack(yf));
    }
  }
  return drawn;
}

template <int DT, int CHUNKS, int G, bool NT, bool PACKED>
__global__ void __launch_bounds__(G + kLnWave, PACKED ? 4 : 1)   // PACKED: at most 128 registers, see LnSlices
layernorm_queue_kernel(const u32x4* x, const u32x4* __restrict__ w, const u32x4* __restrict__ b,
                       u32x4* y, int64_t M, int nvec, float inv_n, float eps, unsigned* counters,
                       int shards, int block_shift) {
  constexpr int WAVES = G / kLnWave;
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
  __shared__ unsigned ticket[2];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const bool worker = t < G;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  // this workgroup's shard, and how many row slots the shard has
  const unsigned SH = (unsigned)shards;
  const unsigned shard = blockIdx.x % SH;
  const unsigned local = blockIdx.x / SH;
  const unsigned members = (gridDim.x - shard + SH - 1) / SH;
  const int64_t block_rows = (int64_t)1 << block_shift;
  const int64_t nblocks = (M + block_rows - 1) >> block_shift;
  const int64_t mine = nblocks > shard ? (nblocks - shard + SH - 1) / SH : 0;
  // (only the last block can be short, and it is the last block of its shard)
  const int64_t slots = mine * block_rows - ((nblocks - 1) % SH == shard ? nblocks * block_rows - M : 0);
  unsigned* q = counters + shard * kLnQueueStride;
  auto row_of = [&](int64_t i) {
    return ((((i >> block_shift) * SH + shard)) << block_shift) + (i & (block_rows - 1));
  };

  int64_t i = local, inext = (int64_t)local + members;   // two static slots, then tickets
  u32x4 ra[CHUNKS], rb[CHUNKS];
  uint32_t raw_a = 0, raw_b = 0;
  LnSlices<DT, CHUNKS, PACKED> wb;
  if (worker && i < slots) {
    const int64_t row = row_of(i);
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) ra[c] = load_vec<NT>(x + row * nvec + c * G + t);
    ra[CHUNKS - 1] = load_vec<NT>(x + row * nvec + (last_ok ? last : nvec - 1));
    raw_a = ln_first_raw<DT>(x + row * nvec);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = (c < CHUNKS - 1 || last_ok) ? c * G + t : nvec - 1;
      wb.set(c, w[idx], b != nullptr ? b[idx] : zero);
    }
  }
  while (i < slots) {                                       // uniform over the workgroup
    int64_t row = row_of(i);
    unsigned drawn = ln_queue_step<DT, CHUNKS, G, NT, PACKED>(x, y, row, inext < slots ? row_of(inext) : row, nvec, t,
                                                              lane, wave, last_ok, ra, raw_a, rb, raw_b, wb, inv_n, eps,
                                                              q, part_a[0], part_b[0], ticket[0]);
    i = inext;
    inext = (int64_t)2 * members + drawn;
    if (i >= slots) break;
    row = row_of(i);
    drawn = ln_queue_step<DT, CHUNKS, G, NT, PACKED>(x, y, row, inext < slots ? row_of(inext) : row, nvec, t, lane,
                                                     wave, last_ok, rb, raw_b, ra, raw_a, wb, inv_n, eps, q, part_a[1],
                                                     part_b[1], ticket[1]);
    i = inext;
    inext = (int64_t)2 * members + drawn;
  }
  // Every member has drawn its last ticket when it gets here; the last to arrive resets.
  if (t == G) {
    const unsigned done = atomicAdd(&q[1], 1u);
    if (done == members - 1) {
      atomicExch(&q[0], 0u);
      atomicExch(&q[1], 0u);
    }
  }
}

// Short rows that are not 16-byte aligned, several per workgroup, staged through LDS (see
// packed_rows.h): L lanes per row, E elements per lane with (E - 1) * L < N <= E * L (so only a
// lane's last element can lie past the end of its row), `tile_rows` rows (at most 16 KiB) per
// step.  A lane keeps its slices of weight and bias in registers for all the tiles of its workgroup.  The same two
// passes over registers as the other kernels: shift by the row's first element, sum, centre,
// sum of squares.  Lane groups without a row repeat the last one and write nothing back.
template <int DT, int L, int E, bool NT>
__global__ void __launch_bounds__(kPackThreads)
layernorm_packed_kernel(const void* x, const void* w, const void* b, void* y, int64_t M, int N,
                        int tile_rows, float n, float eps) {
  using S = Storage<DT>;
  constexpr int GROUPS = kPackThreads / L;
  __shared__ u32x4 tile[kPackLdsVecs];
  const int t = threadIdx.x;
  const int sub = t % L;
  const int group = t / L;
  const bool has_bias = b != nullptr;
  // Short rows pay the per-row arithmetic most: the mean through 1 / N and the reciprocal
  // square root through the hardware instruction plus a Newton step, as in the resident kernel.
  const float inv_n = 1.0f / n;

  // Weight and bias go through LDS as well (see param_request).
  __shared__ u32x4 wl[param_lds_vecs<DT>()];
  __shared__ u32x4 bl[param_lds_vecs<DT>()];
  ParamRegs wregs, bregs;
  param_request<DT>(w, N, t, wregs);
  if (has_bias) param_request<DT>(b, N, t, bregs);

  // The run of a tile is requested one tile ahead (see tile_request).
  const int64_t stride = (int64_t)gridDim.x * tile_rows;
  auto run_of = [&](int64_t r0, int& rows, const char*& src) {
    rows = (int)(M - r0 < tile_rows ? M - r0 : tile_rows);
    src = static_cast<const char*>(x) + r0 * N * S::kBytes;
    return tile_cut(src, rows * N * S::kBytes);
  };
  TileRegs<DT> regs;
  int next_rows = 0;
  const char* src = nullptr;
  TileCut next_cut = {};
  int64_t r0 = (int64_t)blockIdx.x * tile_rows;
  if (r0 < M) {
    next_cut = run_of(r0, next_rows, src);
    tile_request<DT, NT>(src, next_cut, t, regs);
  }
  param_commit<DT>(wl, N, t, wregs);
  if (has_bias) param_commit<DT>(bl, N, t, bregs);
  float wf[E], bf[E];
  bool have_params = false;
  for (; r0 < M; r0 += stride) {
    const TileCut cut = next_cut;
    const int rows = next_rows;
    const int origin = cut.skew / S::kBytes;               // tile element of the run's first element
    tile_commit<DT>(tile, cut, t, regs);
    __syncthreads();
    if (r0 + stride < M) {
      next_cut = run_of(r0 + stride, next_rows, src);
      tile_request<DT, NT>(src, next_cut, t, regs);
    }
    if (!have_params) {                                    // after the first tile's barrier
      param_slice<DT, L, E>(wl, N, sub, wf);
      if (has_bias) {
        param_slice<DT, L, E>(bl, N, sub, bf);
      } else {
#pragma unroll
        for (int i = 0; i < E; ++i) bf[i] = 0.f;
      }
      have_params = true;
    }
    for (int first = 0; first < rows; first += GROUPS) {   // the same trip count for every thread
      const int r = first + group;
      const int at = origin + (r < rows ? r : rows - 1) * N;
      const float shift = tile_get<DT>(tile, at);
      float f[E];
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        f[i] = tile_get<DT>(tile, (i < E - 1 || j < N) ? at + j : at) - shift;   // only the last step can pass N
        if (i == E - 1 && j >= N) f[i] = 0.f;
        acc += f[i];
      }
      const float mean_shifted = group_sum<L>(acc) * inv_n;
      float sq = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        f[i] -= mean_shifted;
        if (i == E - 1 && j >= N) f[i] = 0.f;
        sq = __builtin_fmaf(f[i], f[i], sq);
      }
      const float rstd = ln_rstd_fast(group_sum<L>(sq), inv_n, eps);
      if (r < rows) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
          const int j = sub + i * L;
          const float scaled = (f[i] * rstd) * wf[i];
          if (i < E - 1 || j < N) tile_put<DT>(tile, at + j, has_bias ? scaled + bf[i] : scaled);
        }
      }
    }
    __syncthreads();
    tile_drain<DT, NT>(static_cast<char*>(y) + r0 * N * S::kBytes, tile, cut, t);
    __syncthreads();                                       // the next step refills the tile
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
  const float inv_n = 1.0f / n;       // short rows pay the per-row arithmetic most: see ln_rstd_fast
  const u32x4 zero = {0u, 0u, 0u, 0u};

  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + (row_ok ? row : 0) * nvec;     // rows past M read row 0 and store nothing
    u32x4* yr = y + row * nvec;
    const float shift = S::load_one(xr, 0);

    // Weight and bias are requested with the row (at most 16 more registers), so that
    // nothing is left to wait for between the second reduction and the stores.
    u32x4 v[CHUNKS], wv[CHUNKS], bv[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
      const bool live = idx < nvec;
      v[c] = live ? load_vec<NT>(xr + idx) : zero;
      wv[c] = live ? w[idx] : zero;
      bv[c] = (live && has_bias) ? b[idx] : zero;
    }
    float f[CHUNKS][VEC];
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      // lanes past the end of the row hold zeros; subtracting zero keeps them at zero
      const float off = c * L + sub < nvec ? shift : 0.f;
      S::unpack(v[c], f[c]);
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] -= off;
        acc += f[c][k];
      }
    }
    const float mean_shifted = subwave_sum<L>(acc) * inv_n;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const float off = c * L + sub < nvec ? mean_shifted : 0.f;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] -= off;
        sq = __builtin_fmaf(f[c][k], f[c][k], sq);
      }
    }
    const float rstd = ln_rstd_fast(subwave_sum<L>(sq), inv_n, eps);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
      if (row_ok && idx < nvec) store_vec<NT>(yr + idx, ln_scale<DT>(f[c], wv[c], bv[c], has_bias, rstd));
    }
  }
}

// ---------------------------------------------------------------------------
// The register-resident kernel for rows that are NOT 16-byte aligned (odd N such as the
// paper's edge dims 1023 / 4097 / 1537, or base pointers off a 16-byte boundary).  Rows,
// weight and bias are addressed in bytes, and the 16-byte slots of a row are counted from the
// 128-byte line in which it starts (RowCut in vec_io.h): thread t holds slots c * G + t, so
// every load and store instruction of a wavefront covers eight whole lines; the slots that
// the row does not cover whole hold nothing, the at most VEC - 1 elements before the first
// whole slot go to threads 0 .. head - 1 one each, those after the last to threads
// 16 .. 16 + tail - 1.  CHUNKS * G need only be the whole 16-byte pieces of a row,
// floor(N * sizeof(element) / 16): the slots a row reaches past slot CHUNKS * G - 1 (at most
// as many as it starts into its line) go to the lanes of chunk 0 that this start leaves idle.
// x is still read exactly once.  Same arithmetic as layernorm_row_kernel.
//
//  Either way the grid is a multiple of 64 workgroups and workgroup b starts with row
//  xcd_block_row(b) (vec_io.h): eight consecutive rows out of every 64 for each XCD.
//  WALK == false : one row per workgroup (striding only beyond the grid limit), the cut taken
//                  per row; weight and bias slices, at element-aligned addresses, are read in
//                  the epilogue of every row.
//  WALK == true  : the grid is a multiple of 64 workgroups that stay for the whole launch.
//                  Rows blockIdx.x + k * gridDim.x then all start at the same offset from a
//                  line, so the cut is the workgroup's, and it reads its slices of weight and
//                  bias once, into registers.
//  Where y sits at another offset from a line than x, its stores straddle the lines.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int G, bool NT, bool WALK>
__global__ void __launch_bounds__(G) __attribute__((amdgpu_waves_per_eu(4)))
layernorm_row_unaligned_kernel(const void* x, const void* __restrict__ w, const void* __restrict__ b,
                               void* y, int64_t M, int n_cols, float n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  constexpr int kGroupBytes = 16;
  constexpr int kTailThread = 16;                       // first thread that takes a trailing element
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const bool has_bias = b != nullptr;
  // the mean through 1 / N and the reciprocal root through the hardware instruction plus a
  // Newton step, as in the resident kernel: both sit between the row's arrival and its stores
  const float inv_n = 1.0f / n;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;
  const int64_t first_row = xcd_block_row(blockIdx.x);   // either way the grid is a multiple of 64
  if (first_row >= M) return;

  RowCut cut = row_cut<S::kBytes>(static_cast<const char*>(x) + first_row * n_cols * S::kBytes, n_cols);
  // Lane t holds slot c * G + t in chunk c, except that the lanes of chunk 0 before the row's
  // first whole slot take the slots past the last chunk.
  auto slot_of = [&](int c) { return (c == 0 && t < cut.first) ? CHUNKS * G + t : c * G + t; };
  auto holds = [&](int c) { return (c > 0 && c < CHUNKS - 1) || slot_of(c) < cut.end; };
  bool tail_ok = false;
  int tail_col = 0;
  const char* wl = nullptr;                             // weight / bias bytes of slot 0
  const char* bl = nullptr;
  auto place_edges = [&]() {
    tail_ok = t < cut.head || (t >= kTailThread && t - kTailThread < cut.tail);
    tail_col = t < cut.head ? t : n_cols - cut.tail + (t - kTailThread);
    wl = static_cast<const char*>(w) - cut.off;
    bl = static_cast<const char*>(b) - cut.off;
  };

  u32x4 wv[WALK ? CHUNKS : 1], bv[WALK ? CHUNKS : 1];
  float tail_w = 0.f, tail_b = 0.f;
  if constexpr (WALK) {
    place_edges();
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int64_t at = (int64_t)slot_of(c) * kGroupBytes;
      wv[c] = bv[c] = zero;
      if (holds(c)) {
        wv[c] = load_vec_unaligned<false>(wl + at);
        if (has_bias) bv[c] = load_vec_unaligned<false>(bl + at);
      }
    }
    if (tail_ok) {
      tail_w = S::load_one(w, tail_col);
      tail_b = has_bias ? S::load_one(b, tail_col) : 0.f;
    }
  }

  for (int64_t row = first_row; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * n_cols * S::kBytes;
    char* yr = static_cast<char*>(y) + row * n_cols * S::kBytes;
    if constexpr (!WALK) {
      cut = row_cut<S::kBytes>(xr, n_cols);
      place_edges();
    }
    const char* xl = xr - cut.off;                      // the line the row starts in
    char* yl = yr - cut.off;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      v[c] = zero;
      if (holds(c)) v[c] = load_vec_unaligned<NT>(xl + (int64_t)slot_of(c) * kGroupBytes);
    }
    const float shift = S::load_one(xr, 0);             // the row's first element
    float tail = 0.f;
    if (tail_ok) tail = S::load_one(xr, tail_col) - shift;

    float f[CHUNKS][VEC];
    float acc[4] = {tail, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      S::unpack(v[c], f[c]);
      const bool live = holds(c);
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
      s1 = sum_waves<WAVES>(part_a[slot]);
    }
    const float mean_shifted = s1 * inv_n;

    tail = tail_ok ? tail - mean_shifted : 0.f;
    float sq[4] = {tail * tail, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const bool live = holds(c);
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
      s2 = sum_waves<WAVES>(part_b[slot]);
      slot ^= 1;
    }
    const float rstd = ln_rstd_fast(s2, inv_n, eps);

    if constexpr (WALK) {
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c)
        if (holds(c))
          store_vec_unaligned<NT>(yl + (int64_t)slot_of(c) * kGroupBytes,
                                  ln_scale<DT>(f[c], wv[c], bv[c], has_bias, rstd));
    } else {
      // weight and bias only now (L2 hits), behind an empty asm so that they are not hoisted
      // above the reductions, where the centred row already fills the register budget
      const char* wp = wl;
      const char* bp = bl;
      asm volatile("" : "+s"(wp), "+s"(bp));
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        if (holds(c)) {
          const int64_t at = (int64_t)slot_of(c) * kGroupBytes;
          const u32x4 wc = load_vec_unaligned<false>(wp + at);
          const u32x4 bc = has_bias ? load_vec_unaligned<false>(bp + at) : zero;
          store_vec_unaligned<NT>(yl + at, ln_scale<DT>(f[c], wc, bc, has_bias, rstd));
        }
      }
      if (tail_ok) {
        tail_w = S::load_one(w, tail_col);
        tail_b = has_bias ? S::load_one(b, tail_col) : 0.f;
      }
    }
    if (tail_ok) {
      const float tq = (tail * rstd) * tail_w;
      S::store_one(yr, tail_col, has_bias ? tq + tail_b : tq);
    }
  }
}

// ---------------------------------------------------------------------------
// The walking form of the kernel above with the next row requested ahead, as the resident
// kernel for aligned rows does: two packed register copies of a row take turns, and while one
// is reduced, scaled and stored the other is being filled with the workgroup's next row
// (first + k * gridDim, all at the workgroup's offset from a line, so one cut serves them
// all).  Without it a workgroup has nothing in flight while it works on a row, and with the
// four wavefronts per SIMD that the centred row, weight and bias leave room for, that shows in
// the 16-bit types, which is where this kernel is used (fp16 16384 x 2057: 40.7 -> 34.7 us;
// bf16 4096 x 20481: 69.4 -> 61.3; fp16 8192 x 4097: 28.4 -> 27.8).  No load sits in
// a branch: a slot that the row does not cover reads the row's first whole slot instead and is
// masked afterwards, the last step requests its own row again, and the loop is unrolled twice
// so that no register is copied from one copy to the other.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ uint32_t ln_elem_raw(const void* p, int64_t i) {
  if constexpr (DT == kFp32) return static_cast<const uint32_t*>(p)[i];
  else return static_cast<const uint16_t*>(p)[i];
}

// What a thread of the walking form keeps for the whole launch.
template <int CHUNKS>
struct LnWalkLane {
  RowCut cut;
  int slot_bytes[CHUNKS];       // byte offset of the thread's slot of chunk c from the row's line
  bool holds[CHUNKS];           // whether the row covers that slot whole
  bool edge_ok;                 // whether the thread holds a single leading or trailing element
  int edge_col;                 // ... and which
};

// One row: requests row `pre` into (nxt, nxt_first, nxt_edge), then reduces, scales and stores
// the row held in (cur, cur_first, cur_edge).
template <int DT, int CHUNKS, int G, bool NT>
__device__ __forceinline__ void ln_walk_step(
    const void* x, void* y, int64_t row, int64_t pre, int n_cols, const LnWalkLane<CHUNKS>& ln,
    int lane, int wave, const u32x4 (&cur)[CHUNKS], uint32_t cur_first, uint32_t cur_edge,
    u32x4 (&nxt)[CHUNKS], uint32_t& nxt_first, uint32_t& nxt_edge, u32x4 (&wv)[CHUNKS],
    u32x4 (&bv)[CHUNKS], float edge_w, float edge_b, bool has_bias, float inv_n, float eps,
    float (&part_a)[G / kLnWave], float (&part_b)[G / kLnWave]) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kLnWave;
  const char* xp = static_cast<const char*>(x) + pre * n_cols * S::kBytes;
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) nxt[c] = load_vec_unaligned<NT>(xp - ln.cut.off + ln.slot_bytes[c]);
  nxt_first = ln_elem_raw<DT>(xp, 0);
  nxt_edge = ln_elem_raw<DT>(xp, ln.edge_col);

  const float shift = ln_first_value<DT>(cur_first);
  float tail = ln.edge_ok ? ln_first_value<DT>(cur_edge) - shift : 0.f;
  float f[CHUNKS][VEC];
  float acc[4] = {tail, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    S::unpack(cur[c], f[c]);
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      f[c][k] = ln.holds[c] ? f[c][k] - shift : 0.f;
      acc[k & 3] += f[c][k];
    }
  }
  float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
  if constexpr (WAVES > 1) {
    if (lane == 0) part_a[wave] = s1;
    __syncthreads();
    s1 = sum_waves<WAVES>(part_a);
  }
  const float mean_shifted = s1 * inv_n;

  tail = ln.edge_ok ? tail - mean_shifted : 0.f;
  float sq[4] = {tail * tail, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
      f[c][k] = ln.holds[c] ? f[c][k] - mean_shifted : 0.f;
      sq[k & 3] = __builtin_fmaf(f[c][k], f[c][k], sq[k & 3]);
    }
  }
  float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
  if constexpr (WAVES > 1) {
    if (lane == 0) part_b[wave] = s2;
    __syncthreads();
    s2 = sum_waves<WAVES>(part_b);
  }
  const float rstd = ln_rstd_fast(s2, inv_n, eps);

  // weight and bias stay packed from row to row: widened once for the whole launch they would
  // take the registers that the second copy of the row needs
  forget_unpacked<CHUNKS>(wv);
  forget_unpacked<CHUNKS>(bv);
  char* yr = static_cast<char*>(y) + row * n_cols * S::kBytes;
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c)
    if (ln.holds[c])
      store_vec_unaligned<NT>(yr - ln.cut.off + ln.slot_bytes[c], ln_scale<DT>(f[c], wv[c], bv[c], has_bias, rstd));
  if (ln.edge_ok) {
    const float tq = (tail * rstd) * edge_w;
    S::store_one(yr, ln.edge_col, has_bias ? tq + edge_b : tq);
  }
}

template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G) __attribute__((amdgpu_waves_per_eu(4)))
layernorm_walk_kernel(const void* x, const void* __restrict__ w, const void* __restrict__ b, void* y,
                      int64_t M, int n_cols, float n, float eps) {
  using S = Storage<DT>;
  constexpr int WAVES = G / kLnWave;
  constexpr int kGroupBytes = 16;
  constexpr int kTailThread = 16;                       // first thread that takes a trailing element
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const bool has_bias = b != nullptr;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  const float inv_n = 1.0f / n;
  int64_t row = xcd_block_row(blockIdx.x);               // the grid is a multiple of 64
  if (row >= M) return;
  const int64_t stride = gridDim.x;

  LnWalkLane<CHUNKS> ln;
  ln.cut = row_cut<S::kBytes>(static_cast<const char*>(x) + row * n_cols * S::kBytes, n_cols);
  // Lane t holds slot c * G + t in chunk c, except that the lanes of chunk 0 before the row's
  // first whole slot take the slots past the last chunk.
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    const int slot = (c == 0 && t < ln.cut.first) ? CHUNKS * G + t : c * G + t;
    ln.holds[c] = (c > 0 && c < CHUNKS - 1) || slot < ln.cut.end;
    ln.slot_bytes[c] = (ln.holds[c] ? slot : ln.cut.first) * kGroupBytes;
  }
  ln.edge_ok = t < ln.cut.head || (t >= kTailThread && t - kTailThread < ln.cut.tail);
  ln.edge_col = !ln.edge_ok ? 0 : t < ln.cut.head ? t : n_cols - ln.cut.tail + (t - kTailThread);

  const char* wl = static_cast<const char*>(w) - ln.cut.off;
  const char* bl = static_cast<const char*>(b) - ln.cut.off;
  u32x4 wv[CHUNKS], bv[CHUNKS];
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) {
    wv[c] = bv[c] = zero;
    if (ln.holds[c]) {
      wv[c] = load_vec_unaligned<false>(wl + ln.slot_bytes[c]);
      if (has_bias) bv[c] = load_vec_unaligned<false>(bl + ln.slot_bytes[c]);
    }
  }
  float edge_w = 0.f, edge_b = 0.f;
  if (ln.edge_ok) {
    edge_w = S::load_one(w, ln.edge_col);
    edge_b = has_bias ? S::load_one(b, ln.edge_col) : 0.f;
  }

  u32x4 ra[CHUNKS], rb[CHUNKS];
  uint32_t first_a, first_b = 0, edge_a, edge_b_raw = 0;
  {
    const char* xr = static_cast<const char*>(x) + row * n_cols * S::kBytes;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) ra[c] = load_vec_unaligned<NT>(xr - ln.cut.off + ln.slot_bytes[c]);
    first_a = ln_elem_raw<DT>(xr, 0);
    edge_a = ln_elem_raw<DT>(xr, ln.edge_col);
  }
  while (true) {
    int64_t next = row + stride;
    ln_walk_step<DT, CHUNKS, G, NT>(x, y, row, next < M ? next : row, n_cols, ln, lane, wave, ra, first_a, edge_a,
                                    rb, first_b, edge_b_raw, wv, bv, edge_w, edge_b, has_bias, inv_n, eps,
                                    part_a[0], part_b[0]);
    if (next >= M) break;                              // uniform over the workgroup
    row = next;
    next = row + stride;
    ln_walk_step<DT, CHUNKS, G, NT>(x, y, row, next < M ? next : row, n_cols, ln, lane, wave, rb, first_b, edge_b_raw,
                                    ra, first_a, edge_a, wv, bv, edge_w, edge_b, has_bias, inv_n, eps,
                                    part_a[1], part_b[1]);
    if (next >= M) break;
    row = next;
  }
}

// ---------------------------------------------------------------------------
// Rows too long for registers: three streaming passes by one workgroup per row (the shifted
// sum for the mean, the squares of the centred values, the write), four 16-byte groups
// requested at a time; passes two and three read the row from L2 or the Infinity Cache.
// All accesses are element-aligned 128-bit ones over the row's floor(N / VEC) full groups
// plus a scalar tail, so any N and any base alignment take this one path.  Same arithmetic
// as layernorm_row_kernel.  In-place safe: two barriers separate every read of passes one
// and two from every write of pass three, where a thread reads a group before it overwrites it.
// ---------------------------------------------------------------------------
constexpr int kLnStreamBatch = 4;
constexpr int kLnStreamMaxWaves = kMaxPartials;

// Calls fn(values, live) for every batch group of the row that thread t owns: VEC widened
// values and whether the group exists (clamped loads, so that every load is unconditional).
template <int DT, typename Fn>
__device__ __forceinline__ void ln_stream_groups(const char* xr, int per_thread, int G, int t, int nfull,
                                                 Fn&& fn) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int U = kLnStreamBatch;
  for (int k0 = 0; k0 < per_thread; k0 += U) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int idx = (k0 + u) * G + t;
      v[u] = load_vec_unaligned<false>(xr + (int64_t)(idx < nfull ? idx : nfull - 1) * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[VEC];
      S::unpack(v[u], f);
      fn(f, (k0 + u) * G + t);
    }
  }
}

template <int DT>
__global__ void __launch_bounds__(kLnStreamMaxWaves * kLnWave)
layernorm_stream_kernel(const void* x, const void* __restrict__ w, const void* __restrict__ b, void* y,
                        int64_t M, int64_t N, float n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  __shared__ __attribute__((aligned(16))) float part_a[2][kLnStreamMaxWaves];
  __shared__ __attribute__((aligned(16))) float part_b[2][kLnStreamMaxWaves];
  const int G = blockDim.x;
  const int waves = G / kLnWave;
  const int t = threadIdx.x;
  const int lane = t & (kLnWave - 1);
  const int wave = t / kLnWave;
  const int nfull = (int)(N / VEC);
  const int rem = (int)(N - (int64_t)nfull * VEC);
  const int per_thread = (nfull + G - 1) / G;
  const bool has_bias = b != nullptr;
  const char* wb = static_cast<const char*>(w);
  const char* bb = static_cast<const char*>(b);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    char* yr = static_cast<char*>(y) + row * N * S::kBytes;
    const float shift = S::load_one(x, row * N);      // the row's first element
    const int64_t tail_col = (int64_t)nfull * VEC + t;
    float tail = 0.f;
    if (t < rem) tail = S::load_one(x, row * N + tail_col) - shift;

    float acc[4] = {tail, 0.f, 0.f, 0.f};
    ln_stream_groups<DT>(xr, per_thread, G, t, nfull, [&](const float (&f)[VEC], int idx) {
      const bool live = idx < nfull;
#pragma unroll
      for (int k = 0; k < VEC; ++k) acc[k & 3] += live ? f[k] - shift : 0.f;
    });
    float s1 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if (waves > 1) {
      park_partial(part_a[slot], lane, wave, waves, s1, 0.0f);
      __syncthreads();
      s1 = sum16(part_a[slot]);
    }
    const float mean_shifted = s1 / n;

    tail = t < rem ? tail - mean_shifted : 0.f;
    float sq[4] = {tail * tail, 0.f, 0.f, 0.f};
    ln_stream_groups<DT>(xr, per_thread, G, t, nfull, [&](const float (&f)[VEC], int idx) {
      const bool live = idx < nfull;
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        const float c = live ? (f[k] - shift) - mean_shifted : 0.f;
        sq[k & 3] = __builtin_fmaf(c, c, sq[k & 3]);
      }
    });
    float s2 = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
    if (waves > 1) {
      park_partial(part_b[slot], lane, wave, waves, s2, 0.0f);
      __syncthreads();
      s2 = sum16(part_b[slot]);
      slot ^= 1;
    }
    const float rstd = ln_rstd(s2, n, eps);

    ln_stream_groups<DT>(xr, per_thread, G, t, nfull, [&](const float (&f)[VEC], int idx) {
      if (idx < nfull) {
        const int64_t off = (int64_t)idx * 16;
        float c[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) c[k] = (f[k] - shift) - mean_shifted;
        const u32x4 wv = load_vec_unaligned<false>(wb + off);
        const u32x4 bv = has_bias ? load_vec_unaligned<false>(bb + off) : zero;
        store_vec_unaligned<true>(yr + off, ln_scale<DT>(c, wv, bv, has_bias, rstd));
      }
    });
    if (t < rem) {
      const float tq = (tail * rstd) * S::load_one(w, tail_col);
      S::store_one(y, row * N + tail_col, has_bias ? tq + S::load_one(b, tail_col) : tq);
    }
  }
}

// ---------------------------------------------------------------------------
// Element-wise fallback: any alignment, any N; three passes (shifted sum, centred
// squares, write).  In-place safe for the same reason as the other fallbacks.
template <int DT, int T>
__global__ void __launch_bounds__(T)
layernorm_generic_kernel(const void* x, const void* __restrict__ w, const void* __restrict__ b,
                         void* y, int64_t M, int64_t N, float n, float eps) {
  using S = Storage<DT>;
  constexpr int WAVES = T / kLnWave;
  __shared__ __attribute__((aligned(16))) float part_a[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_b[2][WAVES];
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
    s1 = sum_waves<WAVES>(part_a[slot]);
    const float mean_shifted = s1 / n;

    float sq = 0.f;
    for (int64_t j = tid; j < N; j += T) {
      const float c = (S::load_one(x, base + j) - shift) - mean_shifted;
      sq = __builtin_fmaf(c, c, sq);
    }
    float s2 = wave_sum(sq);
    if (lane == 0) part_b[slot][wave] = s2;
    __syncthreads();
    s2 = sum_waves<WAVES>(part_b[slot]);
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
