// Short rows, several per workgroup, staged through LDS: rows that are not 16-byte aligned (odd
// lengths such as a 77- or 197-entry attention row, or a base pointer off a boundary) and rows
// too short to fill a lane group.
//
// One workgroup per row pays a launch slot and two partly used cache lines for a few hundred
// bytes, and a lane group cannot use 128-bit accesses on rows that start anywhere.  Consecutive
// rows are contiguous in memory, though: a workgroup of 256 threads takes a run of rows (a
// tile: up to 16 KiB), copies that byte range into LDS with aligned 128-bit accesses that are contiguous
// across the workgroup (the few bytes before the first and after the last 16-byte boundary of
// x go element by element), lets lane groups of L = 1, 2, 4 ... 64 lanes work on one row each out
// of LDS (element reads, up to kPackElems elements per lane, results written back in place),
// and copies the range out to y the same way.  Every byte of x and y still crosses HBM once.
// The reductions and the per-row arithmetic of a lane group cost the same however many elements
// its lanes hold, so few lanes with many elements beat many lanes with few.  The kernels are
// not bound by instruction issue (about 12 vector-ALU and 2.5 LDS instructions per element, the
// ALU busy a fraction of the time): a copy of the same bytes through LDS tiles with no
// arithmetic at all runs at 92 to 95 % of the plain copy's rate, and the row kernels at 93 to
// 96 % of that; what they lose goes to the phases of a workgroup (fill, barrier, work, barrier,
// drain), which is why tiles are kept small enough for several workgroup generations to
// overlap and why nothing but the tile's own vectors is loaded per tile.  The paper's playbook
// names the ingredients (wide coalesced accesses, staging in on-chip memory) without giving a
// kernel; the arrangement is this library's.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"

namespace rms {

constexpr int kPackThreads = 256;
constexpr int kPackTileBytes = 16384;                 // LDS per workgroup
constexpr int kPackTileVecs = kPackTileBytes / 16;
constexpr int kPackLdsVecs = kPackTileVecs + 1;          // the run keeps its skew inside the tile
constexpr int kPackVecsPerThread = kPackTileVecs / kPackThreads;   // 4
constexpr int kPackElems = 16;                        // elements a lane holds at most

// Element `i` of the tile, widened to fp32 / rounded from fp32.  `tile` points into LDS.
template <int DT>
__device__ __forceinline__ float tile_get(const u32x4* tile, int i) {
  if constexpr (DT == kFp32) return reinterpret_cast<const float*>(tile)[i];
  else if constexpr (DT == kFp16) return static_cast<float>(reinterpret_cast<const _Float16*>(tile)[i]);
  else return as_f32(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(tile)[i]) << 16);
}

template <int DT>
__device__ __forceinline__ void tile_put(u32x4* tile, int i, float f) {
  if constexpr (DT == kFp32) reinterpret_cast<float*>(tile)[i] = f;
  else if constexpr (DT == kFp16) reinterpret_cast<_Float16*>(tile)[i] = static_cast<_Float16>(f);
  else reinterpret_cast<uint16_t*>(tile)[i] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

// Where a run of `bytes` bytes that starts `skew` bytes past a 16-byte boundary of global
// memory is cut: single elements up to the next boundary, aligned 16-byte vectors, single
// elements again.  The tile keeps the skew (tile byte skew + i holds byte i of the run), so an
// aligned vector of global memory is an aligned vector of LDS; measured, 128-bit global
// accesses at addresses that are not even dword-aligned cost a quarter of the bandwidth.
struct TileCut {
  int skew;        // bytes between the boundary before the run and the run's start, 0..15
  int head;        // bytes of the run before its first aligned vector
  int nvec;        // aligned vectors
  int tail;        // bytes after the last aligned vector
};

__device__ __forceinline__ TileCut tile_cut(const void* start, int bytes) {
  TileCut c;
  c.skew = (int)(reinterpret_cast<uintptr_t>(start) & 15u);
  const int to_boundary = (16 - c.skew) & 15;
  c.head = to_boundary < bytes ? to_boundary : bytes;
  c.nvec = (bytes - c.head) >> 4;
  c.tail = bytes - c.head - 16 * c.nvec;
  return c;
}

// The aligned vectors of a run, STEPS per thread: all of a thread's loads are issued before its
// first LDS write, and indices past the end are clamped so that no load sits in a branch.
template <bool NT, int STEPS>
__device__ __forceinline__ void tile_fill_vectors(const u32x4* body, u32x4* dst, int nvec, int t) {
  u32x4 v[STEPS];
#pragma unroll
  for (int k = 0; k < STEPS; ++k) {
    const int i = k * kPackThreads + t;
    v[k] = load_vec<NT>(body + (i < nvec ? i : nvec - 1));
  }
#pragma unroll
  for (int k = 0; k < STEPS; ++k) {
    const int i = k * kPackThreads + t;
    if (i < nvec) dst[i] = v[k];
  }
}

// Copies the run at `src` (element-aligned, at most kPackTileBytes) into the tile.  A thread
// takes as many vectors as the run needs (1 to 4 steps of 256, the same for every thread: a
// short tile must not pay for the loads of a full one).  Element i of the run lands at element
// skew / sizeof(element) + i of the tile.
template <int DT, bool NT>
__device__ __forceinline__ void tile_fill(const char* src, u32x4* tile, TileCut c, int t) {
  constexpr int EB = Storage<DT>::kBytes;
  const int first = (c.skew + c.head) >> 4;             // tile vector of the first aligned vector
  const int skew_elems = c.skew / EB;
  const int done = (c.head + 16 * c.nvec) / EB;         // elements before the tail
  // The single elements are requested first and unconditionally (threads without one read
  // element 0 of the run), so that they travel with the vectors instead of after them.
  // A run that starts and ends on 16-byte boundaries (every tile of a whole number of 8 rows of
  // 16-bit elements does, if x does) has none: the test is the same for every thread.
  const bool has_head = t < c.head / EB, has_tail = t < c.tail / EB;
  float head = 0.f, tail = 0.f;
  if ((c.head | c.tail) != 0) {
    head = Storage<DT>::load_one(src, has_head ? t : 0);
    tail = Storage<DT>::load_one(src, has_tail ? done + t : 0);
  }
  if (c.nvec > 0) {                                     // the same for every thread
    const u32x4* body = reinterpret_cast<const u32x4*>(src + c.head);
    const int steps = (c.nvec + kPackThreads - 1) / kPackThreads;
    if (steps == 1) tile_fill_vectors<NT, 1>(body, tile + first, c.nvec, t);
    else if (steps == 2) tile_fill_vectors<NT, 2>(body, tile + first, c.nvec, t);
    else if (steps == 3) tile_fill_vectors<NT, 3>(body, tile + first, c.nvec, t);
    else tile_fill_vectors<NT, kPackVecsPerThread>(body, tile + first, c.nvec, t);
  }
  if (has_head) tile_put<DT>(tile, skew_elems + t, head);
  if (has_tail) tile_put<DT>(tile, skew_elems + done + t, tail);
}

// First tile of workgroup `block` where every workgroup has a tile of its own: tiles go to the
// workgroups in XCD blocks of eight (xcd_block_row, for the part of the grid that is whole runs of
// 64), so that neighbouring tiles, which share a cache line wherever a tile does not end on one,
// sit on one XCD.  Measured on softmax, 64 MiB of fp16 rows: 197 elements 23.9 -> 23.4 us, 257
// elements 24.9 -> 24.0, no change at 77, 136, 513 and 1000; RMSNorm and LayerNorm, whose
// workgroups walk several tiles, moved by less than their noise and keep tiles one by one.
__device__ __forceinline__ int64_t packed_first_tile(unsigned block, unsigned grid) {
  return block < (grid & ~63u) ? xcd_block_row(block) : (int64_t)block;
}

// The same copy in two halves, for workgroups that walk several tiles: tile_request issues the
// loads of a run into registers, tile_commit writes them into the tile.  Between the two a
// workgroup works on the tile it filled before, so the next run is on its way from HBM while
// the current one is reduced, scaled and written out (a workgroup that waits for every run
// before it touches it has nothing in flight half of the time: measured on 64 MiB of fp16 rows
// of 197 elements, filling and draining tiles with no arithmetic at all took 23.8 us against
// 21.6 for a plain copy).
template <int DT>
struct TileRegs {
  u32x4 v[kPackVecsPerThread];
  float head, tail;
};

template <int DT, bool NT>
__device__ __forceinline__ void tile_request(const char* src, TileCut c, int t, TileRegs<DT>& r) {
  constexpr int EB = Storage<DT>::kBytes;
  const int done = (c.head + 16 * c.nvec) / EB;
  r.head = r.tail = 0.f;
  if ((c.head | c.tail) != 0) {                         // the same for every thread
    r.head = Storage<DT>::load_one(src, t < c.head / EB ? t : 0);
    r.tail = Storage<DT>::load_one(src, t < c.tail / EB ? done + t : 0);
  }
  const u32x4* body = reinterpret_cast<const u32x4*>(src + c.head);
#pragma unroll
  for (int k = 0; k < kPackVecsPerThread; ++k) {
    if (k * kPackThreads >= c.nvec) break;              // the same for every thread
    const int i = k * kPackThreads + t;
    r.v[k] = load_vec<NT>(body + (i < c.nvec ? i : c.nvec - 1));
  }
}

template <int DT>
__device__ __forceinline__ void tile_commit(u32x4* tile, TileCut c, int t, const TileRegs<DT>& r) {
  constexpr int EB = Storage<DT>::kBytes;
  const int first = (c.skew + c.head) >> 4;
  const int skew_elems = c.skew / EB;
  const int done = (c.head + 16 * c.nvec) / EB;
#pragma unroll
  for (int k = 0; k < kPackVecsPerThread; ++k) {
    if (k * kPackThreads >= c.nvec) break;
    const int i = k * kPackThreads + t;
    if (i < c.nvec) tile[first + i] = r.v[k];
  }
  if (t < c.head / EB) tile_put<DT>(tile, skew_elems + t, r.head);
  if (t < c.tail / EB) tile_put<DT>(tile, skew_elems + done + t, r.tail);
}

// The reverse: the tile's run to global memory at `dst`, in the cut it was filled with.  Where
// dst sits at the same offset from a 16-byte boundary as the source (both aligned, or in
// place) the vector stores fall on the boundaries; elsewhere they are element-aligned, which
// costs a few per cent.
template <int DT, bool NT>
__device__ __forceinline__ void tile_drain(char* dst, const u32x4* tile, TileCut c, int t) {
  constexpr int EB = Storage<DT>::kBytes;
  const int first = (c.skew + c.head) >> 4;
  char* body = dst + c.head;
#pragma unroll
  for (int k = 0; k < kPackVecsPerThread; ++k) {
    if (k * kPackThreads >= c.nvec) break;              // the same for every thread
    const int i = k * kPackThreads + t;
    if (i < c.nvec) store_vec_unaligned<NT>(body + 16 * i, tile[first + i]);
  }
  const int skew_elems = c.skew / EB;
  if (t < c.head / EB) Storage<DT>::store_one(dst, t, tile_get<DT>(tile, skew_elems + t));
  const int done = (c.head + 16 * c.nvec) / EB;
  if (t < c.tail / EB) Storage<DT>::store_one(dst, done + t, tile_get<DT>(tile, skew_elems + done + t));
}

// A per-column vector (weight, bias) of N <= kPackMaxN elements, also through LDS.  A lane's
// slice of it is E elements L apart; read from global memory that is E two-byte loads per lane,
// more load instructions than the lane issues for its share of a tile, and with a workgroup
// per tile it cost more than the tile did (bf16 RMSNorm over 64 MiB of 197-element rows: 45 us;
// with workgroups that walk five tiles each to spread the cost, 26.5; with the vector through
// LDS and a workgroup per one or two tiles, 24.4).  The workgroup fetches the vector with
// consecutive threads on consecutive elements (param_request: N / 256 loads per thread, issued
// next to the first tile's), writes it into LDS in the storage type (param_commit, before the
// barrier that publishes the first tile), and every lane then picks its slice (param_slice).
constexpr int kPackMaxN = kPackElems * 64;
constexpr int kPackParamSteps = kPackMaxN / kPackThreads;   // 4

template <int DT>
constexpr int param_lds_vecs() { return kPackMaxN * Storage<DT>::kBytes / 16; }

struct ParamRegs {
  float v[kPackParamSteps];
};

template <int DT>
__device__ __forceinline__ void param_request(const void* p, int N, int t, ParamRegs& r) {
#pragma unroll
  for (int k = 0; k < kPackParamSteps; ++k) {
    if (k * kPackThreads >= N) break;                     // the same for every thread
    const int j = k * kPackThreads + t;
    r.v[k] = Storage<DT>::load_one(p, j < N ? j : N - 1);
  }
}

template <int DT>
__device__ __forceinline__ void param_commit(u32x4* lds, int N, int t, const ParamRegs& r) {
#pragma unroll
  for (int k = 0; k < kPackParamSteps; ++k) {
    if (k * kPackThreads >= N) break;
    const int j = k * kPackThreads + t;
    if (j < N) tile_put<DT>(lds, j, r.v[k]);              // exact: the value came from this type
  }
}

// Elements sub, sub + L, ... of the vector; an element past N reads as 0.
template <int DT, int L, int E>
__device__ __forceinline__ void param_slice(const u32x4* lds, int N, int sub, float (&out)[E]) {
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int j = sub + i * L;
    const bool in = i < E - 1 || j < N;                   // only the last step can pass N
    out[i] = tile_get<DT>(lds, in ? j : 0);
    if (!in) out[i] = 0.f;
  }
}

// Sum / maximum over aligned groups of L lanes (1: the lane itself; 2 and 4: the first steps of
// the butterfly inside a quad; 64: the whole wavefront), result in every lane of the group.
// All 64 lanes must be active.
template <int L>
__device__ __forceinline__ float group_sum(float v) {
  if constexpr (L == 1) return v;
  else if constexpr (L == 2) return add_dpp<0xB1>(v);
  else if constexpr (L == 4) return add_dpp<0x4E>(add_dpp<0xB1>(v));
  else if constexpr (L == 64) return wave_sum(v);
  else return subwave_sum<L>(v);
}

template <int L>
__device__ __forceinline__ float group_max(float v) {
  if constexpr (L == 1) return v;
  else if constexpr (L == 2) return max_dpp<0xB1>(v);
  else if constexpr (L == 4) return max_dpp<0x4E>(max_dpp<0xB1>(v));
  else if constexpr (L == 64) return wave_max(v);
  else return subwave_max<L>(v);
}

}  // namespace rms
