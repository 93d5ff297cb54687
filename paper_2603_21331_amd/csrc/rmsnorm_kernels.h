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
//  * rmsnorm_row_kernel<.., G = 64>  : one 64-lane wavefront per row.  No LDS,
//                                      no barrier.
//  * rmsnorm_row_kernel<.., G > 64>  : one workgroup per row, per-wave partial
//                                      sums combined through LDS in wave order.
//  * rmsnorm_subwave_kernel          : 8, 16 or 32 lanes per row, several rows per
//                                      wavefront, for rows of at most 1 KiB.
//  * rmsnorm_row_unaligned_kernel    : the same, for rows that are not 16-byte
//                                      aligned (element-aligned 128-bit accesses
//                                      plus a scalar tail).
//  * rmsnorm_stream_kernel           : rows too long for registers: two streaming
//                                      passes, any N and alignment.
//  * rmsnorm_generic_kernel          : element-wise two-pass kernel, kept as the
//                                      plainest implementation to test against.
//
// All sums are fp32, in an order fixed by (kernel, shape) alone: no atomics,
// so repeated runs give identical bits.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"
#include "packed_rows.h"

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

// (forget_unpacked, from vec_io.h, sits between the sum of squares and the scale pass: without
// it the fp32 forms unpacked for the sum are kept alive, which multiplies the register
// footprint of the row by two for the 16-bit types and spills long rows.)

// rstd = 1 / sqrt(sum / n + eps).  Every thread of a row computes it between the arrival of
// the row and the first store, so its latency is paid once per row on the critical path: the
// correctly rounded divide, root and reciprocal of a plain 1 / sqrt(sum / n + eps) take about
// fifty dependent instructions there, and replacing them was worth 0.7 % of the kernel at the
// headline shape.  Here: one fused multiply-add for the mean (inv_n = 1 / n rounded to fp32),
// the hardware reciprocal square root (1 ulp; the paper's kernel table names a fast reciprocal
// square root for this kernel too) and one Newton step,
// which together stay within 1.5 ulp of the exact value.  Arguments that are not normal
// numbers (zero or subnormal: a zero row with eps = 0; infinite: a sum that overflowed; NaN)
// take the plain formula, so the IEEE corner cases are unchanged.
__device__ __forceinline__ float row_rstd(float sum_sq, float inv_n, float eps) {
  const float a = __builtin_fmaf(sum_sq, inv_n, eps);
  // one class test, and the plain formula laid out off the straight path
  if (__builtin_expect(!__builtin_isnormal(a) || a < 0.0f, 0)) return 1.0f / __builtin_sqrtf(a);
  const float y0 = __builtin_amdgcn_rsqf(a);
  const float e = __builtin_fmaf(-a * y0, y0, 1.0f);
  return __builtin_fmaf(0.5f * y0, e, y0);
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
// Register-resident row kernel: G threads (G/64 wavefronts) share one row, one
// row per workgroup.  Vector c * G + t of the row goes to thread t, chunk c, so
// every load instruction of a wavefront covers 1 KiB of contiguous memory.
// CHUNKS = ceil(nvec / G): only the last chunk can be ragged.  All loads of x
// and w are issued before the first use; x is then held in registers across
// the reduction, so the scale pass reads nothing from memory.
//
//  G == 64 : one wavefront per row.  DPP reduction only; no LDS, no barrier.
//  G  > 64 : one workgroup per row.  Each wavefront reduces its lanes with DPP,
//            lane 0 parks the partial in LDS, and after one barrier every
//            thread adds the G/64 partials in wave order.  Two LDS slots
//            alternate between consecutive rows of a striding workgroup, so
//            one barrier per row is enough.
//
// Short per-thread work wins on MI355X: at N = 8192 (bf16) four 16-byte chunks
// per thread with 256 threads per row sustain about 10 % more bandwidth than
// sixteen chunks in one wavefront, because load, reduce and store phases of
// the many small wavefronts interleave more finely.  The grid is flat (one
// workgroup per row); it only strides when M exceeds the grid limit.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int G, bool NT, bool FLAT = false>
__global__ void __launch_bounds__(G)
rmsnorm_row_kernel(const u32x4* x, const u32x4* w, u32x4* y,
                   int64_t M, int nvec, float inv_n, float eps, int xcd_blocks) {
  constexpr int WAVES = G / kWave;
  // When the weight chunks are fetched.  The weight is re-read by every row and misses the
  // compute unit's vector cache most of the time (the streaming row pushes it out), so its
  // loads cost real bandwidth between L2 and the compute unit: measured at N = 8192 bf16,
  // 3 to 5 % of the kernel.  Fetching them after the reduction, when the row's own loads
  // have landed, takes them out of the way of those loads and recovers about a third of
  // that; with a single chunk per thread there is nothing to get out of the way of and
  // the extra latency only hurts.  Long rows (more than 8 chunks per thread) fetch one
  // chunk at a time in the epilogue to stay inside the register budget (a 1024-thread
  // workgroup is capped at 128 VGPRs); one wavefront per row keeps them with the row's loads.
  constexpr int kWithRow = 0, kAfterReduce = 1, kOneByOne = 2;
  constexpr int W_WHEN = G == kWave ? (CHUNKS <= 16 ? kWithRow : kOneByOne)
                         : CHUNKS > 8 ? kOneByOne
                         : CHUNKS > 1 ? kAfterReduce : kWithRow;
  __shared__ __attribute__((aligned(16))) float partial[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kWave - 1);
  const int wave = t / kWave;
  // FLAT: the host promises nvec == CHUNKS * G (no ragged last chunk) and one row per
  // workgroup (gridDim.x == M), which removes the predicates and the loop bookkeeping from
  // both ends of a workgroup's short life; worth 1 % at the headline shape.
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = FLAT || last < nvec;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;

  for (int64_t row = flat_first_row(blockIdx.x, xcd_blocks); row < M; row += FLAT ? M : (int64_t)gridDim.x) {
    const u32x4* xr = x + row * nvec;
    const __amdgpu_buffer_rsrc_t yr = row_resource(y + row * nvec, nvec * 16);

    u32x4 v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<NT>(xr + c * G + t);
    v[CHUNKS - 1] = zero;
    if (last_ok) v[CHUNKS - 1] = load_vec<NT>(xr + last);

    u32x4 wv[W_WHEN == kOneByOne ? 1 : CHUNKS];
    if constexpr (W_WHEN == kWithRow) {
#pragma unroll
      for (int c = 0; c < CHUNKS - 1; ++c) wv[c] = w[c * G + t];
      wv[CHUNKS - 1] = zero;
      if (last_ok) wv[CHUNKS - 1] = w[last];
    }

    float total = wave_sum(lane_sum_sq<DT, CHUNKS>(v));
    forget_unpacked<CHUNKS>(v);
    // (A pointer that has been through an asm statement is no longer known to point to global
    // memory and would be read with flat loads: the address space is stated again.)
    typedef const u32x4 __attribute__((address_space(1)))* GlobalVec;
    const u32x4* wp = w;
    GlobalVec wl = (GlobalVec)wp;
    if constexpr (WAVES > 1) {
      if (lane == 0) partial[slot][wave] = total;
      __syncthreads();
      total = partial[slot][0];
      if constexpr (W_WHEN == kAfterReduce) {
        // Tied to the first value read after the barrier: the loads cannot move above it,
        // and they are in flight while the partial sums are added and rstd is formed.
        // They go through the generic pointer as it comes out of the asm statement (flat
        // loads): measured 0.5 % faster here than the same loads marked global.
        asm volatile("" : "+s"(wp) : "v"(total));
#pragma unroll
        for (int c = 0; c < CHUNKS - 1; ++c) wv[c] = wp[c * G + t];
        wv[CHUNKS - 1] = zero;
        if (last_ok) wv[CHUNKS - 1] = wp[last];
      }
      total = sum_waves<WAVES>(partial[slot]);
      slot ^= 1;
    }
    const float rstd = row_rstd(total, inv_n, eps);
    if constexpr (W_WHEN == kOneByOne) {
      // ties the pointer to the result of the reduction, so the loads cannot move above it
      asm volatile("" : "+s"(wp) : "v"(rstd));
      wl = (GlobalVec)wp;
    }

#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) {
      const int idx = c * G + t;
      const u32x4 wc = W_WHEN == kOneByOne ? wl[idx] : wv[W_WHEN == kOneByOne ? 0 : c];
      store_row_vec<NT>(yr, idx, scale_vec<DT>(v[c], wc, rstd));
    }
    if (last_ok) {
      const u32x4 wc = W_WHEN == kOneByOne ? wl[last] : wv[W_WHEN == kOneByOne ? 0 : CHUNKS - 1];
      store_row_vec<NT>(yr, last, scale_vec<DT>(v[CHUNKS - 1], wc, rstd));
    }
  }
}

// ---------------------------------------------------------------------------
// Work-queue form of the workgroup-per-row kernel, for long rows (16 KiB and more) in
// launches of a few hundred megabytes.  A grid of one or two workgroups per compute unit
// stays for the whole launch; each keeps its slices of the weight in registers (so the
// weight is read from L2 once per workgroup instead of once per row: the re-reads miss the
// compute unit's vector cache two times in three and sit on every row's path between the
// reduction and the first store) and draws rows from a counter in device memory, which
// balances the compute units the way the hardware dispatcher balances a flat grid.
//
// Row order.  The workgroups are split into `shards` groups (workgroup b belongs to shard
// b % shards; the hardware deals workgroups to the 8 XCDs in turn, so a shard of a multiple
// of 8 shards sits on one XCD).  The rows are cut into blocks of 2^block_shift consecutive
// rows (128 KiB in the tuned configurations), block k belongs to shard k % shards, and the
// members of a shard take the rows of its blocks in order: each XCD then walks contiguous
// 128 KiB pieces of x and y instead of single rows 8 rows apart.  Measured at bf16
// 16384 x 8192 the whole form is 3.5 % ahead of one workgroup per row with rows handed out one
// by one, and 1 % ahead of it with rows in XCD blocks of eight (flat_first_row), which is what
// the flat kernel now does at this row length.
//
// Counters.  Shard s owns counters[s * kQueueStride] (slots handed out beyond the two that
// every member takes statically) and counters[s * kQueueStride + 1] (members that have
// finished).  Both must be zero when the kernel starts; the last member of a shard to
// finish puts them back to zero, so the same memory serves the next launch without a
// clearing step in between.  Launches that share counters must not overlap.  Every
// workgroup leaves its loop after finitely many tickets and nobody waits for anybody, so
// the grid drains whatever the hardware's scheduling order.
//
// The row a workgroup takes next is known one row ahead, so with PREFETCH its loads are
// requested before the stores of the current row (what a single workgroup per compute unit
// needs to keep requests in flight); without it they follow the stores.  A row's sums do
// not depend on which workgroup takes it: results are bit-identical from run to run.
// ---------------------------------------------------------------------------
constexpr int kQueueStride = 32;      // counters of neighbouring shards are 128 bytes apart
constexpr int kQueueMaxShards = 32;

template <int DT, int CHUNKS, int G, bool PREFETCH>
__global__ void __launch_bounds__(G)
rmsnorm_queue_kernel(const u32x4* x, const u32x4* __restrict__ w, u32x4* y, int64_t M, int nvec,
                     float inv_n, float eps, unsigned* counters, int shards, int block_shift) {
  constexpr int WAVES = G / kWave;
  __shared__ __attribute__((aligned(16))) float partial[2][WAVES];
  __shared__ unsigned ticket[2];
  const int t = threadIdx.x;
  const int lane = t & (kWave - 1);
  const int wave = t / kWave;
  const int last = (CHUNKS - 1) * G + t;
  const bool last_ok = last < nvec;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  // this workgroup's shard, and how many row slots the shard has
  const unsigned S = (unsigned)shards;
  const unsigned shard = blockIdx.x % S;
  const unsigned local = blockIdx.x / S;
  const unsigned members = (gridDim.x - shard + S - 1) / S;
  const int64_t block_rows = (int64_t)1 << block_shift;
  const int64_t nblocks = (M + block_rows - 1) >> block_shift;
  const int64_t mine = nblocks > shard ? (nblocks - shard + S - 1) / S : 0;
  // (only the last block can be short, and it is the last block of its shard)
  const int64_t slots = mine * block_rows - ((nblocks - 1) % S == shard ? nblocks * block_rows - M : 0);
  unsigned* q = counters + shard * kQueueStride;
  auto row_of = [&](int64_t i) {
    return ((((i >> block_shift) * S + shard)) << block_shift) + (i & (block_rows - 1));
  };

  u32x4 wv[CHUNKS];
#pragma unroll
  for (int c = 0; c < CHUNKS - 1; ++c) wv[c] = w[c * G + t];
  wv[CHUNKS - 1] = zero;
  if (last_ok) wv[CHUNKS - 1] = w[last];

  auto load_row = [&](u32x4 (&v)[CHUNKS], int64_t row) {
    const u32x4* xr = x + row * nvec;
#pragma unroll
    for (int c = 0; c < CHUNKS - 1; ++c) v[c] = load_vec<true>(xr + c * G + t);
    v[CHUNKS - 1] = zero;
    if (last_ok) v[CHUNKS - 1] = load_vec<true>(xr + last);
  };

  int slot = 0;
  int64_t i = local, inext = (int64_t)local + members;   // two static slots, then tickets
  u32x4 v[CHUNKS];
  if (i < slots) load_row(v, row_of(i));
  while (i < slots) {
    const int64_t row = row_of(i);
    const bool more = inext < slots;
    if (t == 0) ticket[slot] = atomicAdd(&q[0], 1u);
    float total = wave_sum(lane_sum_sq<DT, CHUNKS>(v));
    forget_unpacked<CHUNKS>(v);
    if (lane == 0) partial[slot][wave] = total;
    __syncthreads();
    total = sum_waves<WAVES>(partial[slot]);
    const int64_t after_next = (int64_t)2 * members + ticket[slot];
    slot ^= 1;
    const float rstd = row_rstd(total, inv_n, eps);
    const __amdgpu_buffer_rsrc_t yr = row_resource(y + row * nvec, nvec * 16);
    if constexpr (PREFETCH) {
      u32x4 o[CHUNKS];
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) o[c] = scale_vec<DT>(v[c], wv[c], rstd);
      if (more) load_row(v, row_of(inext));
#pragma unroll
      for (int c = 0; c < CHUNKS - 1; ++c) store_row_vec<true>(yr, c * G + t, o[c]);
      if (last_ok) store_row_vec<true>(yr, last, o[CHUNKS - 1]);
    } else {
#pragma unroll
      for (int c = 0; c < CHUNKS - 1; ++c) store_row_vec<true>(yr, c * G + t, scale_vec<DT>(v[c], wv[c], rstd));
      if (last_ok) store_row_vec<true>(yr, last, scale_vec<DT>(v[CHUNKS - 1], wv[CHUNKS - 1], rstd));
      if (more) load_row(v, row_of(inext));
    }
    i = inext;
    inext = after_next;
  }
  // Every member has drawn its last ticket when it gets here; the last to arrive resets.
  if (t == 0) {
    const unsigned done = atomicAdd(&q[1], 1u);
    if (done == members - 1) {
      atomicExch(&q[0], 0u);
      atomicExch(&q[1], 0u);
    }
  }
}

// ---------------------------------------------------------------------------
// Short rows that are not 16-byte aligned, several per workgroup, staged through LDS (see
// packed_rows.h): L lanes per row, E elements per lane with (E - 1) * L < N <= E * L (so only
// a lane's last element can lie past the end of its row), `tile_rows` rows (at most 16 KiB) per
// step.  A lane keeps its slice of the weight in registers for all the tiles of its workgroup.
// Lane groups without a row repeat the last one and write nothing back.
// ---------------------------------------------------------------------------
template <int DT, int L, int E, bool NT>
__global__ void __launch_bounds__(kPackThreads)
rmsnorm_packed_kernel(const void* x, const void* w, void* y, int64_t M, int N, int tile_rows,
                      float inv_n, float eps) {
  using S = Storage<DT>;
  constexpr int GROUPS = kPackThreads / L;
  __shared__ u32x4 tile[kPackLdsVecs];
  const int t = threadIdx.x;
  const int sub = t % L;
  const int group = t / L;

  // The weight goes through LDS as well (see param_request).
  __shared__ u32x4 wl[param_lds_vecs<DT>()];
  ParamRegs wregs;
  param_request<DT>(w, N, t, wregs);

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
  float wf[E];
  bool have_w = false;
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
    if (!have_w) {                                         // after the first tile's barrier
      param_slice<DT, L, E>(wl, N, sub, wf);
      have_w = true;
    }
    for (int first = 0; first < rows; first += GROUPS) {   // the same trip count for every thread
      const int r = first + group;
      const int at = origin + (r < rows ? r : rows - 1) * N;
      float f[E];
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < E; ++i) {
        const int j = sub + i * L;
        f[i] = tile_get<DT>(tile, (i < E - 1 || j < N) ? at + j : at);   // only the last step can pass N
        if (i == E - 1 && j >= N) f[i] = 0.f;
        acc = __builtin_fmaf(f[i], f[i], acc);
      }
      const float rstd = row_rstd(group_sum<L>(acc), inv_n, eps);
      if (r < rows) {
#pragma unroll
        for (int i = 0; i < E; ++i) {
          const int j = sub + i * L;
          if (i < E - 1 || j < N) tile_put<DT>(tile, at + j, (f[i] * rstd) * wf[i]);
        }
      }
    }
    __syncthreads();
    tile_drain<DT, NT>(static_cast<char*>(y) + r0 * N * S::kBytes, tile, cut, t);
    __syncthreads();                                       // the next step refills the tile
  }
}

// ---------------------------------------------------------------------------
// Short rows (at most 32 * CHUNKS vectors, e.g. the 128-element rows of a
// per-head normalisation): one wavefront would leave most of its lanes idle on
// a row of 256 bytes, so L = 8, 16 or 32 lanes share a row and a wavefront
// takes 64 / L consecutive rows at once.  When the row fills its lanes exactly
// the wavefront's loads are still one contiguous kilobyte.  The reduction stays
// inside the lane group (DPP, plus one swizzle for L = 32); no LDS storage, no
// barrier.  Lanes whose row lies past M keep running with zeros so that the
// cross-lane steps see all 64 lanes active; only their loads and stores are
// predicated off.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int L, bool NT>
__global__ void __launch_bounds__(kWave)
rmsnorm_subwave_kernel(const u32x4* x, const u32x4* __restrict__ w, u32x4* y,
                       int64_t M, int nvec, float inv_n, float eps) {
  constexpr int ROWS = kWave / L;
  const int lane = threadIdx.x;
  const int s = lane % L;
  const int r = lane / L;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  for (int64_t base = (int64_t)blockIdx.x * ROWS; base < M; base += (int64_t)gridDim.x * ROWS) {
    const int64_t row = base + r;
    const bool row_ok = row < M;
    const u32x4* xr = x + row * nvec;
    u32x4* yr = y + row * nvec;

    u32x4 v[CHUNKS], wv[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + s;
      const bool ok = row_ok && idx < nvec;
      v[c] = zero;
      wv[c] = zero;
      if (ok) {
        v[c] = load_vec<NT>(xr + idx);
        wv[c] = w[idx];
      }
    }
    const float total = subwave_sum<L>(lane_sum_sq<DT, CHUNKS>(v));
    forget_unpacked<CHUNKS>(v);
    const float rstd = row_rstd(total, inv_n, eps);
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int idx = c * L + s;
      if (row_ok && idx < nvec) store_vec<NT>(yr + idx, scale_vec<DT>(v[c], wv[c], rstd));
    }
  }
}

// ---------------------------------------------------------------------------
// The same register-resident kernel for rows that are NOT 16-byte aligned (odd
// N such as 1023 or 4097, or base pointers off a 16-byte boundary).  Rows are
// addressed in bytes, and the 16-byte slots of a row are counted from the
// 128-byte line in which the row starts, not from its first element: slot j
// lies at line + 16 * j, thread t holds slots c * G + t, so the kilobyte that
// one load or store instruction of a wavefront covers is always eight whole
// lines.  (Slots counted from the row's first aligned group put every such
// kilobyte across nine lines, and both neighbours of a line then request it
// again: a plain copy with its wavefronts 16 bytes off the lines runs at 67 to
// 76 % of peak where the aligned one reaches 83.)  The slots that the row does
// not cover whole (some before its start, one at each end in part, the rest
// after its end) hold nothing; the at most VEC - 1 elements before the first
// whole slot go to threads 0 .. head - 1 one each, those after the last to
// threads 16 .. 16 + tail - 1.  x is still read exactly once.  CHUNKS * G
// need only be the whole 16-byte pieces of a row, floor(N * sizeof(element) /
// 16): a row that starts `first` slots into its line leaves the first `first`
// lanes of chunk 0 idle and can reach at most `first` slots past slot
// CHUNKS * G - 1, and those lanes take these slots (slot CHUNKS * G + t for
// lane t), so a row of 8191 or 4097 elements needs no more chunks than its
// aligned neighbour.  Only chunk 0 and the last chunk can hold nothing.
//
//  Either way the grid is a multiple of 64 workgroups and workgroup b starts
//  with row xcd_block_row(b) (vec_io.h): eight consecutive rows out of every
//  64 for each XCD.
//  WALK == false : one row per workgroup (striding only beyond the grid
//                  limit), the cut taken per row; the weight slices, which sit
//                  at element-aligned addresses, are read for every row.
//  WALK == true  : the grid is a multiple of 64 workgroups that stay for the
//                  whole launch.  Rows blockIdx.x + k * gridDim.x then all
//                  start at the same offset from a line, so the cut is the
//                  workgroup's, and it reads its slices of the weight once,
//                  into registers.  Measured, element-aligned weight loads
//                  repeated for every row cost more than the aligned row
//                  accesses gain.
//  Where y sits at another offset from a line than x, its stores are off the
//  lines whatever the cut; that costs what it costs a copy.
// ---------------------------------------------------------------------------
template <int DT, int CHUNKS, int G, bool NT, bool WALK>
__global__ void __launch_bounds__(G)
rmsnorm_row_unaligned_kernel(const void* x, const void* __restrict__ w, void* y,
                             int64_t M, int n, float inv_n, float eps) {
  using S = Storage<DT>;
  constexpr int WAVES = G / kWave;
  constexpr int kGroupBytes = 16;
  constexpr int kTailThread = 16;                       // first thread that takes a trailing element
  __shared__ __attribute__((aligned(16))) float partial[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kWave - 1);
  const int wave = t / kWave;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;
  const int64_t first_row = xcd_block_row(blockIdx.x);   // either way the grid is a multiple of 64
  if (first_row >= M) return;

  RowCut cut = row_cut<S::kBytes>(static_cast<const char*>(x) + first_row * n * S::kBytes, n);
  // Lane t holds slot c * G + t in chunk c, except that the lanes of chunk 0 before the row's
  // first whole slot take the slots past the last chunk.
  auto slot_of = [&](int c) { return (c == 0 && t < cut.first) ? CHUNKS * G + t : c * G + t; };
  auto holds = [&](int c) { return (c > 0 && c < CHUNKS - 1) || slot_of(c) < cut.end; };

  // 1024 threads with 8 and more groups each (a workgroup of that size is capped at 128
  // registers per thread): the weight is fetched group by group in the epilogue instead of
  // all at once with the row, which would spill.
  constexpr bool W_LATE = !WALK && G == 1024 && CHUNKS >= 8;
  u32x4 wv[W_LATE ? 1 : CHUNKS];
  float edge_w = 0.f;
  bool edge_ok = false;
  int edge_col = 0;
  const char* wl = nullptr;                             // weight bytes of slot 0 (element-aligned)
  auto place_edges = [&]() {
    edge_ok = t < cut.head || (t >= kTailThread && t - kTailThread < cut.tail);
    edge_col = t < cut.head ? t : n - cut.tail + (t - kTailThread);
    wl = static_cast<const char*>(w) - cut.off;
  };
  auto load_weight = [&]() {
    if constexpr (!W_LATE) {
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        wv[c] = zero;
        if (holds(c)) wv[c] = load_vec_unaligned<false>(wl + (int64_t)slot_of(c) * kGroupBytes);
      }
    }
    if (edge_ok) edge_w = S::load_one(w, edge_col);
  };
  if constexpr (WALK) {
    place_edges();
    load_weight();
  }

  for (int64_t row = first_row; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * n * S::kBytes;
    char* yr = static_cast<char*>(y) + row * n * S::kBytes;
    if constexpr (!WALK) {
      cut = row_cut<S::kBytes>(xr, n);
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
    float edge_x = 0.f;
    if (edge_ok) edge_x = S::load_one(xr, edge_col);
    if constexpr (!WALK) load_weight();

    float total = wave_sum(__builtin_fmaf(edge_x, edge_x, lane_sum_sq<DT, CHUNKS>(v)));
    forget_unpacked<CHUNKS>(v);
    if constexpr (WAVES > 1) {
      if (lane == 0) partial[slot][wave] = total;
      __syncthreads();
      total = sum_waves<WAVES>(partial[slot]);
      slot ^= 1;
    }
    const float rstd = row_rstd(total, inv_n, eps);

    const char* wp = wl;
    if constexpr (W_LATE) asm volatile("" : "+s"(wp) : "v"(rstd));   // not before the reduction
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      if (holds(c)) {
        const int64_t at = (int64_t)slot_of(c) * kGroupBytes;
        const u32x4 wc = W_LATE ? load_vec_unaligned<false>(wp + at) : wv[W_LATE ? 0 : c];
        store_vec_unaligned<NT>(yl + at, scale_vec<DT>(v[c], wc, rstd));
      }
    }
    if (edge_ok) S::store_one(yr, edge_col, (edge_x * rstd) * edge_w);
  }
}

// ---------------------------------------------------------------------------
// Rows too long for registers: two streaming passes by one workgroup per row.  Pass one adds
// the squares, four 16-byte groups requested at a time; pass two reads the row again (from
// L2 or the Infinity Cache), scales it and writes y with streaming stores.  All accesses are
// element-aligned 128-bit ones over the row's floor(N / VEC) full groups plus a scalar tail,
// so any N and any base alignment take this one path.  In-place safe: the barrier of the
// reduction separates every read of pass one from every write of pass two, and in pass two
// a thread reads a group before it overwrites it.
// ---------------------------------------------------------------------------
constexpr int kStreamBatch = 4;
constexpr int kStreamMaxWaves = kMaxPartials;

template <int DT>
__global__ void __launch_bounds__(kStreamMaxWaves * kWave)
rmsnorm_stream_kernel(const void* x, const void* __restrict__ w, void* y, int64_t M, int64_t N,
                      float inv_n, float eps) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int U = kStreamBatch;
  __shared__ __attribute__((aligned(16))) float partial[2][kStreamMaxWaves];
  const int G = blockDim.x;
  const int waves = G / kWave;
  const int t = threadIdx.x;
  const int lane = t & (kWave - 1);
  const int wave = t / kWave;
  const int nfull = (int)(N / VEC);
  const int rem = (int)(N - (int64_t)nfull * VEC);
  const int per_thread = (nfull + G - 1) / G;             // groups k * G + t, k < per_thread
  const char* wb = static_cast<const char*>(w);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    char* yr = static_cast<char*>(y) + row * N * S::kBytes;

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < per_thread; k0 += U) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {       // clamped, so that every load is unconditional
        const int idx = (k0 + u) * G + t;
        v[u] = load_vec_unaligned<false>(xr + (int64_t)(idx < nfull ? idx : nfull - 1) * 16);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if ((k0 + u) * G + t >= nfull) v[u] = zero;
        float f[VEC];
        S::unpack(v[u], f);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k & 3] = __builtin_fmaf(f[k], f[k], acc[k & 3]);
      }
    }
    float tail = 0.f;
    if (t < rem) tail = S::load_one(x, row * N + (int64_t)nfull * VEC + t);
    float total = wave_sum(__builtin_fmaf(tail, tail, (acc[0] + acc[1]) + (acc[2] + acc[3])));
    if (waves > 1) {
      park_partial(partial[slot], lane, wave, waves, total, 0.0f);
      __syncthreads();
      total = sum16(partial[slot]);
      slot ^= 1;
    }
    const float rstd = row_rstd(total, inv_n, eps);

    for (int k0 = 0; k0 < per_thread; k0 += U) {
      u32x4 v[U], wv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = (k0 + u) * G + t;
        const int64_t off = (int64_t)(idx < nfull ? idx : nfull - 1) * 16;
        v[u] = load_vec_unaligned<false>(xr + off);
        wv[u] = load_vec_unaligned<false>(wb + off);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = (k0 + u) * G + t;
        if (idx < nfull) store_vec_unaligned<true>(yr + (int64_t)idx * 16, scale_vec<DT>(v[u], wv[u], rstd));
      }
    }
    if (t < rem) {
      const int64_t col = (int64_t)nfull * VEC + t;
      S::store_one(y, row * N + col, (tail * rstd) * S::load_one(w, col));
    }
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
                       int64_t M, int64_t N, float inv_n, float eps) {
  constexpr int WAVES = T / kWave;
  __shared__ __attribute__((aligned(16))) float partial[2][WAVES];
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
    float total = sum_waves<WAVES>(partial[slot]);
    slot ^= 1;
    const float rstd = row_rstd(total, inv_n, eps);

    for (int64_t j = tid; j < N; j += T) {
      const float f = Storage<DT>::load_one(x, base + j);
      const float g = Storage<DT>::load_one(w, j);
      Storage<DT>::store_one(y, base + j, (f * rstd) * g);
    }
  }
}

}  // namespace rms
