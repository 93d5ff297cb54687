// Row softmax forward kernels for gfx950 (MI355X).
//
//   y[i, j] = exp(x[i, j] - max_j x[i, :]) / sum_j exp(x[i, j] - max_j x[i, :])
//
// The paper lists the kernel next to RMSNorm in its table of supported kernel
// types (memory-bound, measured in GB/s; its starter reduces with lane shuffles
// over two-element fp16 loads) and
// it has the same reduce-then-scale shape, so it reuses the RMSNorm design: each
// row is read from HBM once with 16-byte non-temporal loads, held in registers
// across both reductions, and written once.  What is held differs: after the
// maximum is known the row is kept as fp32 exponentials (8 registers per 16-byte
// chunk of a 16-bit type instead of 4), because computing exp a second time for
// the scale pass would make the kernel ALU-bound (v_exp_f32 issues at a quarter
// of the FMA rate).
//
//  * softmax_row_kernel<.., G = 64> : one wavefront per row (DPP max and sum).
//  * softmax_row_kernel<.., G > 64> : one workgroup per row, cross-wave max and
//                                     sum through LDS, two barriers per row.
//  * softmax_subwave_kernel        : 8, 16 or 32 lanes per row for rows <= 1 KiB
//                                     (attention scores over short contexts).
//  * softmax_row_unaligned_kernel  : the row kernel for rows that are not 16-byte
//                                     aligned (element-aligned 128-bit accesses
//                                     plus a scalar tail).
//  * softmax_stream_kernel         : rows too long for registers: two streaming
//                                     passes (online max/sum, then scale), any N
//                                     and alignment.
//  * softmax_generic_kernel        : element-wise three-pass kernel, kept as the
//                                     plainest implementation to test against.
//
// Reductions have a fixed order and use no atomics: results are bit-identical
// from run to run.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"
#include "packed_rows.h"

namespace rms {

constexpr int kWaveSize = 64;
constexpr float kNegInf = -__builtin_inff();

// exp(d) for d <= 0 as 2^(d * log2 e), to the accuracy each output type needs.
//  - fp32 outputs: the product d * log2 e is carried in two floats (t + lo); a
//    single rounded product would put up to 1e-5 relative error into the result
//    for |d| ~ 100.  e == 0 is returned as is so that d = -inf (lo is NaN then)
//    gives 0; a NaN d still gives NaN.
//  - bf16 outputs share the fp32 exponent range and can be subnormal, so they
//    take __builtin_exp2f, which keeps subnormal results; the single product is
//    accurate enough for 8 significand bits.
//  - fp16 outputs underflow to zero long before fp32 does: raw v_exp_f32.
template <int DT>
__device__ __forceinline__ float exp_neg(float d) {
  constexpr float kLog2eHi = 1.44269502162933349609375f;      // fp32(log2 e)
  constexpr float kLog2eLo = 1.92596299112661746704e-8f;      // log2 e - fp32(log2 e)
  constexpr float kLn2 = 0.693147182464599609375f;
  const float t = d * kLog2eHi;
  if constexpr (DT == kFp16) {
    return __builtin_amdgcn_exp2f(t);
  } else if constexpr (DT == kBf16) {
    return __builtin_exp2f(t);
  } else {
    const float lo = __builtin_fmaf(d, kLog2eHi, -t) + d * kLog2eLo;
    const float e = __builtin_exp2f(t);
    return e == 0.f ? 0.f : __builtin_fmaf(e, lo * kLn2, e);   // 2^(t+lo) = 2^t (1 + lo ln 2 + ..)
  }
}

// ---------------------------------------------------------------------------
// Register-resident row kernel: G threads share one row, one row per workgroup.
// Same data layout as the RMSNorm row kernel: vector c * G + t goes to thread t,
// chunk c; only the last chunk can be ragged, and its missing elements are
// filled with -inf so that they take no part in the maximum and add exp(-inf)
// = 0 to the sum.
//
// With 1024 threads and five chunks or more of a 16-bit type, the fp32 form of the row (8
// registers per chunk) would leave room for one workgroup per compute unit only, and with
// one workgroup nothing overlaps its load, reduce and store phases (bf16 4096 x 50304:
// 4.7 TB/s).  Those instances keep the row packed, widen it again in each of the three passes
// and take the exponentials twice: 64 registers or fewer, two workgroups per compute unit.
// The results are the same bits: every pass computes the same values from the same inputs.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ u32x4 sm_neg_inf_vec() {
  constexpr uint32_t p = DT == kFp32 ? 0xFF800000u : DT == kFp16 ? 0xFC00FC00u : 0xFF80FF80u;
  u32x4 v = {p, p, p, p};
  return v;
}

template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G)
softmax_row_kernel(const u32x4* x, u32x4* y, int64_t M, int nvec, int xcd_blocks) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kWaveSize;
  constexpr bool LEAN = G == 1024 && CHUNKS >= 5 && DT != kFp32;
  __shared__ __attribute__((aligned(16))) float part_max[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_sum[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kWaveSize - 1);
  const int wave = t / kWaveSize;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  int slot = 0;

  for (int64_t row = flat_first_row(blockIdx.x, xcd_blocks); row < M; row += gridDim.x) {
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * G + t);
    {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      v[CHUNKS - 1] = zero;
      if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);
    }

    if constexpr (LEAN) {
      // The row stays packed; every pass widens it again and the exponentials are taken twice.
      if (!last_ok) v[CHUNKS - 1] = sm_neg_inf_vec<DT>();
      float m = kNegInf;
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        float g[VEC];
        S::unpack(v[c], g);
#pragma unroll
        for (int k = 0; k < VEC; ++k) m = __builtin_fmaxf(m, g[k]);
      }
      m = wave_max(m);
      if (lane == 0) part_max[slot][wave] = m;
      __syncthreads();
      m = max_waves<WAVES>(part_max[slot]);
      forget_unpacked<CHUNKS>(v);
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        float g[VEC];
        S::unpack(v[c], g);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k & 3] += exp_neg<DT>(g[k] - m);
      }
      float s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
      if (lane == 0) part_sum[slot][wave] = s;
      __syncthreads();
      s = sum_waves<WAVES>(part_sum[slot]);
      slot ^= 1;
      const float inv = 1.0f / s;
      forget_unpacked<CHUNKS>(v);
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        float g[VEC];
        S::unpack(v[c], g);
#pragma unroll
        for (int k = 0; k < VEC; ++k) g[k] = exp_neg<DT>(g[k] - m) * inv;
        const int idx = c * G + t;
        if (c < CHUNKS - 1 || last_ok) store_vec<NT>(yr + idx, S::pack(g));
      }
      continue;
    }

    float f[CHUNKS][VEC];
    float m = kNegInf;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      S::unpack(v[c], f[c]);
      if (c == CHUNKS - 1 && !last_ok) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) f[c][k] = kNegInf;
      }
#pragma unroll
      for (int k = 0; k < VEC; ++k) m = __builtin_fmaxf(m, f[c][k]);
    }
    m = wave_max(m);
    if constexpr (WAVES > 1) {
      if (lane == 0) part_max[slot][wave] = m;
      __syncthreads();
      m = max_waves<WAVES>(part_max[slot]);
    }

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = exp_neg<DT>(f[c][k] - m);
        acc[k & 3] += f[c][k];
      }
    }
    float s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_sum[slot][wave] = s;
      __syncthreads();
      s = sum_waves<WAVES>(part_sum[slot]);
      slot ^= 1;
    }
    const float inv = 1.0f / s;

#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) f[c][k] *= inv;
      const int idx = c * G + t;
      if (c < CHUNKS - 1 || last_ok) store_vec<NT>(yr + idx, S::pack(f[c]));
    }
  }
}

// ---------------------------------------------------------------------------
// Short rows that are not 16-byte aligned (an attention row of 77, 197 or 257 scores), several
// per workgroup, staged through LDS (see packed_rows.h): L lanes per row, E elements per lane
// with (E - 1) * L < N <= E * L (so only a lane's last element can lie past the end of its row),
// `tile_rows` rows (at most 16 KiB) per step.  Lane groups without a row repeat the last one
// and write nothing back.  (Skipping the steps that hold no element of any row, a test that is the same for
// every lane, was measured and is 10 % slower: the branches keep the LDS reads apart.)
// ---------------------------------------------------------------------------
template <int DT, int L, int E, bool NT>
__global__ void __launch_bounds__(kPackThreads)
softmax_packed_kernel(const void* x, void* y, int64_t M, int N, int tile_rows) {
  using S = Storage<DT>;
  constexpr int GROUPS = kPackThreads / L;
  __shared__ u32x4 tile[kPackLdsVecs];
  const int t = threadIdx.x;
  const int sub = t % L;
  const int group = t / L;

  // The run of a tile is requested one tile ahead (see tile_request).
  const int64_t stride = (int64_t)gridDim.x * tile_rows;
  auto run_of = [&](int64_t r0, int& rows, const char*& src) {
    rows = (int)(M - r0 < tile_rows ? M - r0 : tile_rows);
    src = static_cast<const char*>(x) + r0 * N * S::kBytes;
    return tile_cut(src, rows * N * S::kBytes);
  };
  TileRegs<DT> regs;
  int rows = 0;
  const char* src = nullptr;
  TileCut cut = {};
  int64_t r0 = packed_first_tile(blockIdx.x, gridDim.x) * tile_rows;
  if (r0 < M) {
    cut = run_of(r0, rows, src);
    tile_request<DT, NT>(src, cut, t, regs);
  }
  for (; r0 < M; r0 += stride) {
    const int origin = cut.skew / S::kBytes;               // tile element of the run's first element
    tile_commit<DT>(tile, cut, t, regs);
    __syncthreads();
    const TileCut this_cut = cut;
    const int this_rows = rows;
    if (r0 + stride < M) {
      cut = run_of(r0 + stride, rows, src);
      tile_request<DT, NT>(src, cut, t, regs);
    }
    for (int first = 0; first < this_rows; first += GROUPS) {   // the same trip count for every thread
      const int r = first + group;
      const int at = origin + (r < this_rows ? r : this_rows - 1) * N;
      float f[E];
      float m = kNegInf;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        f[i] = tile_get<DT>(tile, (i < E - 1 || j < N) ? at + j : at);   // only the last step can pass N
        if (i == E - 1 && j >= N) f[i] = kNegInf;              // exp(-inf - m) adds 0 to the sum
        m = __builtin_fmaxf(m, f[i]);
      }
      m = group_max<L>(m);
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        f[i] = exp_neg<DT>(f[i] - m);
        acc += f[i];
      }
      // The sum is at least 1 (the maximum contributes exp(0)) and at most N: the hardware
      // reciprocal (1 ulp) replaces the ten-instruction correctly rounded division.
      const float inv = __builtin_amdgcn_rcpf(group_sum<L>(acc));
      if (r < this_rows) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
          const int j = sub + i * L;
          if (i < E - 1 || j < N) tile_put<DT>(tile, at + j, f[i] * inv);
        }
      }
    }
    __syncthreads();
    tile_drain<DT, NT>(static_cast<char*>(y) + r0 * N * S::kBytes, tile, this_cut, t);
    __syncthreads();                                       // the next step refills the tile
  }
}

// ---------------------------------------------------------------------------
// Short rows: L = 8, 16 or 32 lanes per row, 64 / L consecutive rows per
// wavefront; reductions stay inside the lane group.  Lanes whose row lies past
// M run on -inf so that the cross-lane steps always see 64 active lanes; their
// result (NaN) is never stored.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int L, bool NT>
__global__ void __launch_bounds__(kWaveSize)
softmax_subwave_kernel(const u32x4* x, u32x4* y, int64_t M, int nvec) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int ROWS = kWaveSize / L;
  const int lane = threadIdx.x;
  const int sub = lane % L;
  const int r = lane / L;

  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    float f[CHUNKS][VEC];
    float m = kNegInf;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
      if (row_ok && idx < nvec) {
        S::unpack(load_vec<NT>(xr + idx), f[c]);
      } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) f[c][k] = kNegInf;
      }
#pragma unroll
      for (int k = 0; k < VEC; ++k) m = __builtin_fmaxf(m, f[c][k]);
    }
    m = subwave_max<L>(m);
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = exp_neg<DT>(f[c][k] - m);
        acc += f[c][k];
      }
    }
    const float inv = 1.0f / subwave_sum<L>(acc);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + sub;
#pragma unroll
      for (int k = 0; k < VEC; ++k) f[c][k] *= inv;
      if (row_ok && idx < nvec) store_vec<NT>(yr + idx, S::pack(f[c]));
    }
  }
}

// ---------------------------------------------------------------------------
// The same register-resident kernel for rows that are NOT 16-byte aligned (odd N such as
// the paper's edge dims 1023 / 4097 / 1537, or base pointers off a 16-byte boundary).
// Rows are addressed in bytes, and the 16-byte slots of a row are counted from the 128-byte
// line in which it starts (RowCut in vec_io.h): thread t holds slots c * G + t, so every
// load and store instruction of a wavefront covers eight whole lines; the slots that the
// row does not cover whole hold -inf, the at most VEC - 1 elements before the first whole
// slot go to threads 0 .. head - 1 one each, those after the last to threads 16 .. 16 + tail
// - 1.  The cut is taken per row (no weight to keep, so no need for resident workgroups); the
// grid is a multiple of 64 workgroups and rows go to them in XCD blocks (xcd_block_row), which
// keeps the line two consecutive rows share in one L2 (fp16 8192 x 4097: 23.4 -> 22.7 us).
// CHUNKS * G need only be the whole 16-byte pieces of a row, floor(N * sizeof(element) / 16):
// the slots a row reaches past slot CHUNKS * G - 1 (at most as many as it starts into its
// line) go to the lanes of chunk 0 that this start leaves idle, so 4097 elements need no more
// chunks than 4096.  Where y sits at another offset from a line than x, its stores straddle
// the lines.  x is still read exactly once.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int G, bool NT>
__global__ void __launch_bounds__(G)
softmax_row_unaligned_kernel(const void* x, void* y, int64_t M, int n) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kWaveSize;
  constexpr int kGroupBytes = 16;
  constexpr int kTailThread = 16;                       // first thread that takes a trailing element
  __shared__ __attribute__((aligned(16))) float part_max[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_sum[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kWaveSize - 1);
  const int wave = t / kWaveSize;
  int slot = 0;

  for (int64_t row = xcd_block_row(blockIdx.x); row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * n * S::kBytes;
    char* yr = static_cast<char*>(y) + row * n * S::kBytes;
    const RowCut cut = row_cut<S::kBytes>(xr, n);
    auto slot_of = [&](int c) { return (c == 0 && t < cut.first) ? CHUNKS * G + t : c * G + t; };
    auto holds = [&](int c) { return (c > 0 && c < CHUNKS - 1) || slot_of(c) < cut.end; };
    const bool tail_ok = t < cut.head || (t >= kTailThread && t - kTailThread < cut.tail);
    const int tail_col = t < cut.head ? t : n - cut.tail + (t - kTailThread);
    const char* xl = xr - cut.off;                      // the line the row starts in
    char* yl = yr - cut.off;

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      v[c] = sm_neg_inf_vec<DT>();
      if (holds(c)) v[c] = load_vec_unaligned<NT>(xl + (int64_t)slot_of(c) * kGroupBytes);
    }
    float tail = kNegInf;
    if (tail_ok) tail = S::load_one(xr, tail_col);

    float f[CHUNKS][VEC];
    float m = tail;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      S::unpack(v[c], f[c]);
#pragma unroll
      for (int k = 0; k < VEC; ++k) m = __builtin_fmaxf(m, f[c][k]);
    }
    m = wave_max(m);
    if constexpr (WAVES > 1) {
      if (lane == 0) part_max[slot][wave] = m;
      __syncthreads();
      m = max_waves<WAVES>(part_max[slot]);
    }

    // a lane without a leftover element adds exactly 0 (its -inf gives exp(-inf) = 0, or
    // NaN when the whole row is -inf, which is what such a row must give anyway)
    tail = exp_neg<DT>(tail - m);
    float acc[4] = {tail, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) {
        f[c][k] = exp_neg<DT>(f[c][k] - m);
        acc[k & 3] += f[c][k];
      }
    }
    float s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_sum[slot][wave] = s;
      __syncthreads();
      s = sum_waves<WAVES>(part_sum[slot]);
      slot ^= 1;
    }
    const float inv = 1.0f / s;

#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
#pragma unroll
      for (int k = 0; k < VEC; ++k) f[c][k] *= inv;
      if (holds(c)) store_vec_unaligned<NT>(yl + (int64_t)slot_of(c) * kGroupBytes, S::pack(f[c]));
    }
    if (tail_ok) S::store_one(yr, tail_col, tail * inv);
  }
}

// ---------------------------------------------------------------------------
// Rows too long for registers (a softmax over a vocabulary of 100 k to 250 k entries, or
// longer): two streaming passes by one workgroup per row.  Pass one keeps, per thread, a
// running maximum and a running sum of exponentials relative to it (the online form the
// paper names for its cross-entropy kernel), folded in batches of four 16-byte groups: the
// batch maximum first, at most one rescale per batch.  Pass two reads the row again (from
// L2 or the Infinity Cache: a row of 256 k fp16 values is 512 KiB), forms exp(x - m) / s with
// the full-accuracy exponential and writes y with streaming stores.  All accesses are
// element-aligned 128-bit ones over the row's floor(N / VEC) full groups plus a scalar tail,
// so any N and any base alignment take this one path.  HBM traffic stays one read of x and
// one write of y as long as the rows in flight fit the Infinity Cache.  In-place safe: a
// barrier separates every read of pass one from every write of pass two, and in pass two a
// thread reads a group before it overwrites it.
// ---------------------------------------------------------------------------
constexpr int kStreamBatch = 4;
constexpr int kStreamMaxWaves = kMaxPartials;

// 2^((a - b) log2 e) for a <= b, with equal arguments (two -inf included) giving exactly 1.
__device__ __forceinline__ float sm_rescale(float a, float b) {
  return a == b ? 1.0f : __builtin_amdgcn_exp2f((a - b) * 1.44269502162933349609375f);
}

// Folds COUNT values into the running (m, s) pair.
template <int COUNT>
__device__ __forceinline__ void sm_fold(const float (&f)[COUNT], float& m, float& s) {
  float bm = m;
#pragma unroll
  for (int k = 0; k < COUNT; ++k) bm = __builtin_fmaxf(bm, f[k]);
  s *= sm_rescale(m, bm);
  m = bm;
  // only -inf so far: every term is exp(-inf) = 0; subtracting 0 keeps -inf - (-inf) from NaN
  const float ref = bm == kNegInf ? 0.0f : bm;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < COUNT; ++k)
    acc[k & 3] += __builtin_amdgcn_exp2f((f[k] - ref) * 1.44269502162933349609375f);
  s += (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

// Groups (k0 + u) * G + t, u < COUNT, of a row; indices past the last full group (only
// possible in a thread's last batch) are clamped to it, so that every load is unconditional,
// and the lanes concerned fold -inf instead of what the clamped load brought.  nfull >= 1.
template <int DT, int COUNT>
__device__ __forceinline__ void sm_stream_batch(const char* xr, int k0, int G, int t, int nfull,
                                                float& m, float& s) {
  constexpr int VEC = Storage<DT>::kVec;
  u32x4 v[COUNT];
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    const int idx = (k0 + u) * G + t;
    v[u] = load_vec_unaligned<false>(xr + (int64_t)(idx < nfull ? idx : nfull - 1) * 16);
  }
  float f[COUNT * VEC];
#pragma unroll
  for (int u = 0; u < COUNT; ++u) {
    float g[VEC];
    Storage<DT>::unpack(v[u], g);
    const bool live = (k0 + u) * G + t < nfull;
#pragma unroll
    for (int k = 0; k < VEC; ++k) f[u * VEC + k] = live ? g[k] : kNegInf;
  }
  sm_fold<COUNT * VEC>(f, m, s);
}

template <int DT>
__global__ void __launch_bounds__(kStreamMaxWaves * kWaveSize)
softmax_stream_kernel(const void* x, void* y, int64_t M, int64_t N) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int U = kStreamBatch;
  __shared__ __attribute__((aligned(16))) float part_max[2][kStreamMaxWaves];
  __shared__ __attribute__((aligned(16))) float part_sum[2][kStreamMaxWaves];
  const int G = blockDim.x;
  const int waves = G / kWaveSize;
  const int t = threadIdx.x;
  const int lane = t & (kWaveSize - 1);
  const int wave = t / kWaveSize;
  const int nfull = (int)(N / VEC);
  const int rem = (int)(N - (int64_t)nfull * VEC);
  const int per_thread = (nfull + G - 1) / G;             // groups k * G + t, k < per_thread
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    char* yr = static_cast<char*>(y) + row * N * S::kBytes;

    // pass one: running maximum and sum
    float m = kNegInf, s = 0.f;
    int k = 0;
    for (; k + U <= per_thread; k += U) sm_stream_batch<DT, U>(xr, k, G, t, nfull, m, s);
    switch (per_thread - k) {                             // the same for every thread
      case 1: sm_stream_batch<DT, 1>(xr, k, G, t, nfull, m, s); break;
      case 2: sm_stream_batch<DT, 2>(xr, k, G, t, nfull, m, s); break;
      case 3: sm_stream_batch<DT, 3>(xr, k, G, t, nfull, m, s); break;
      default: break;
    }
    float tail = kNegInf;
    if (t < rem) {
      tail = S::load_one(x, row * N + (int64_t)nfull * VEC + t);
      const float single[1] = {tail};
      sm_fold<1>(single, m, s);
    }
    float row_m = wave_max(m);
    if (waves > 1) {
      park_partial(part_max[slot], lane, wave, waves, row_m, kNegInf);
      __syncthreads();
      row_m = max16(part_max[slot]);
    }
    float row_s = wave_sum(s * sm_rescale(m, row_m));
    if (waves > 1) {
      park_partial(part_sum[slot], lane, wave, waves, row_s, 0.0f);
      __syncthreads();
      row_s = sum16(part_sum[slot]);
      slot ^= 1;
    }
    const float inv = 1.0f / row_s;

    // pass two: exp(x - m) / s, written once; four groups requested at a time
    for (int k2 = 0; k2 < per_thread; k2 += U) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = (k2 + u) * G + t;
        v[u] = load_vec_unaligned<false>(xr + (int64_t)(idx < nfull ? idx : nfull - 1) * 16);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = (k2 + u) * G + t;
        float f[VEC];
        S::unpack(v[u], f);
#pragma unroll
        for (int j = 0; j < VEC; ++j) f[j] = exp_neg<DT>(f[j] - row_m) * inv;
        if (idx < nfull) store_vec_unaligned<true>(yr + (int64_t)idx * 16, S::pack(f));
      }
    }
    if (t < rem)
      S::store_one(y, row * N + (int64_t)nfull * VEC + t, exp_neg<DT>(tail - row_m) * inv);
  }
}

// ---------------------------------------------------------------------------
// Element-wise fallback: any element alignment, any N; three passes over the
// row (maximum, sum of exponentials, scaled write), the second and third mostly
// from cache.  In-place safe: every read of passes one and two precedes, by a
// barrier, every write of pass three, and in pass three a thread reads an
// element before it overwrites it.
// ---------------------------------------------------------------------------
template <int DT, int T>
__global__ void __launch_bounds__(T)
softmax_generic_kernel(const void* x, void* y, int64_t M, int64_t N) {
  using S = Storage<DT>;
  constexpr int WAVES = T / kWaveSize;
  __shared__ __attribute__((aligned(16))) float part_max[2][WAVES];
  __shared__ __attribute__((aligned(16))) float part_sum[2][WAVES];
  const int tid = threadIdx.x;
  const int lane = tid & (kWaveSize - 1);
  const int wave = tid / kWaveSize;
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const int64_t base = row * N;
    float m = kNegInf;
    for (int64_t j = tid; j < N; j += T) m = __builtin_fmaxf(m, S::load_one(x, base + j));
    m = wave_max(m);
    if (lane == 0) part_max[slot][wave] = m;
    __syncthreads();
    m = max_waves<WAVES>(part_max[slot]);

    float acc = 0.f;
    for (int64_t j = tid; j < N; j += T) acc += exp_neg<DT>(S::load_one(x, base + j) - m);
    float s = wave_sum(acc);
    if (lane == 0) part_sum[slot][wave] = s;
    __syncthreads();
    s = sum_waves<WAVES>(part_sum[slot]);
    slot ^= 1;
    const float inv = 1.0f / s;

    for (int64_t j = tid; j < N; j += T)
      S::store_one(y, base + j, exp_neg<DT>(S::load_one(x, base + j) - m) * inv);
  }
}

}  // namespace rms
