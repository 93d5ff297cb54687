// Short rows, several per workgroup, staged through LDS: rows that are not 16-byte aligned (odd
// lengths such as a 77- or 197-entry attention row, or a base pointer off a boundary) and rows
// too short to fill a lane group.
//
// One workgroup per row pays a launch slot and two partly used cache lines for a few hundred
// bytes, and a lane group cannot use 128-bit accesses on rows that start anywhere.  Consecutive
// rows are contiguous in memory, though: a workgroup of 256 threads takes a run of rows (up to
// 16 KiB), copies that byte range into LDS with aligned 128-bit accesses that are contiguous
// across the workgroup (the few bytes before the first and after the last 16-byte boundary of
// x go element by element), lets lane groups of L = 1, 2, 4 ... 64 lanes work on one row each out
// of LDS (element reads, up to kPackElems elements per lane, results written back in place),
// and copies the range out to y the same way.  Every byte of x and y still crosses HBM once.
// The kernels are bound by vector-ALU issue, and the reductions and the per-row arithmetic of a
// lane group cost the same however many elements its lanes hold, so few lanes with many
// elements beat many lanes with few.  The paper's playbook names the ingredients (vectorised,
// coalesced accesses; shared-memory staging) without giving a kernel; the arrangement is this
// library's.
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

// Copies the run at `src` (element-aligned, at most kPackTileBytes) into the tile.  All of a
// thread's vector loads are issued before its first LDS write; indices past the end are
// clamped so that no load sits in a branch.  Element i of the run lands at element
// skew / sizeof(element) + i of the tile.
template <int DT, bool NT>
__device__ __forceinline__ void tile_fill(const char* src, u32x4* tile, TileCut c, int t) {
  constexpr int EB = Storage<DT>::kBytes;
  const int first = (c.skew + c.head) >> 4;             // tile vector of the first aligned vector
  const int skew_elems = c.skew / EB;
  const int done = (c.head + 16 * c.nvec) / EB;         // elements before the tail
  // The single elements are requested first and unconditionally (threads without one read
  // element 0 of the run), so that they travel with the vectors instead of after them.
  const bool has_head = t < c.head / EB, has_tail = t < c.tail / EB;
  const float head = Storage<DT>::load_one(src, has_head ? t : 0);
  const float tail = Storage<DT>::load_one(src, has_tail ? done + t : 0);
  if (c.nvec > 0) {                                     // the same for every thread
    const u32x4* body = reinterpret_cast<const u32x4*>(src + c.head);
    u32x4 v[kPackVecsPerThread];
#pragma unroll
    for (int k = 0; k < kPackVecsPerThread; ++k) {
      const int i = k * kPackThreads + t;
      v[k] = load_vec<NT>(body + (i < c.nvec ? i : c.nvec - 1));
    }
#pragma unroll
    for (int k = 0; k < kPackVecsPerThread; ++k) {
      const int i = k * kPackThreads + t;
      if (i < c.nvec) tile[first + i] = v[k];
    }
  }
  if (has_head) tile_put<DT>(tile, skew_elems + t, head);
  if (has_tail) tile_put<DT>(tile, skew_elems + done + t, tail);
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
    const int i = k * kPackThreads + t;
    if (i < c.nvec) store_vec_unaligned<NT>(body + 16 * i, tile[first + i]);
  }
  const int skew_elems = c.skew / EB;
  if (t < c.head / EB) Storage<DT>::store_one(dst, t, tile_get<DT>(tile, skew_elems + t));
  const int done = (c.head + 16 * c.nvec) / EB;
  if (t < c.tail / EB) Storage<DT>::store_one(dst, done + t, tile_get<DT>(tile, skew_elems + done + t));
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
