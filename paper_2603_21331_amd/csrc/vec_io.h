// 128-bit global memory access and storage-type conversion for gfx950.
//
// Every row is moved as 16-byte vectors: one global_load_dwordx4 /
// global_store_dwordx4 per lane per chunk, so a 64-lane wavefront touches one
// contiguous 1 KiB span per instruction.  The paper's CUDA starters use the
// same idea at their hardware's width (Section 5 lists wide vector loads among
// the properties of its starter kernels); here the unit is the CDNA4 dwordx4
// access.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rms {

enum : int { kFp32 = 0, kFp16 = 1, kBf16 = 2 };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Streaming accesses carry the non-temporal hint: x and y are touched exactly
// once, so keeping them in L2 / Infinity Cache only evicts the weight vector.
template <bool NT>
__device__ __forceinline__ u32x4 load_vec(const u32x4* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

template <bool NT>
__device__ __forceinline__ void store_vec(u32x4* p, u32x4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// The same 16-byte access through a pointer that is only element-aligned.  The
// amdhsa ABI runs the memory pipeline in unaligned-access mode, and the compiler
// knows it: these still compile to single global_load/store_dwordx4 instructions.
typedef u32x4 u32x4_unaligned __attribute__((aligned(2)));

template <bool NT>
__device__ __forceinline__ u32x4 load_vec_unaligned(const void* p) {
  if constexpr (NT) return __builtin_nontemporal_load(static_cast<const u32x4_unaligned*>(p));
  else return *static_cast<const u32x4_unaligned*>(p);
}

template <bool NT>
__device__ __forceinline__ void store_vec_unaligned(void* p, u32x4 v) {
  if constexpr (NT) __builtin_nontemporal_store(v, static_cast<u32x4_unaligned*>(p));
  else *static_cast<u32x4_unaligned*>(p) = v;
}

// Streaming stores of an output row go through a buffer resource that covers exactly that
// row: the instruction then carries the cache-policy bits of choice (the non-temporal hint
// plus sc1, which on MI355X sends the line on without keeping it in L2 and measured about
// 1 % faster than the hint alone), and the hardware drops any access past the row's end.
// 0x00020000 is the raw 32-bit data format word of a gfx9-family resource.
constexpr int kStreamStorePolicy = 2 | 16;   // nt | sc1

__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_resource(void* row, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(row, 0, bytes, 0x00020000);
}

// Stores 16-byte vector `index` of the row behind `res`.
template <bool NT>
__device__ __forceinline__ void store_row_vec(__amdgpu_buffer_rsrc_t res, int index, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, res, index * 16, 0, NT ? kStreamStorePolicy : 0);
}

// Makes the compiler treat packed vectors as new values, so that fp32 forms unpacked from them
// earlier cannot be kept alive in registers for a later pass (widening again costs one ALU
// operation per element; keeping them costs the registers that decide the occupancy).
template <int CHUNKS>
__device__ __forceinline__ void forget_unpacked(u32x4 (&v)[CHUNKS]) {
#pragma unroll
  for (int c = 0; c < CHUNKS; ++c) asm volatile("" : "+v"(v[c]));
}

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Storage traits.  VEC = elements per 16-byte vector.  unpack widens exactly to
// fp32; pack rounds to nearest-even with the hardware converters
// (v_cvt_pk_bf16_f32 / v_cvt_pk_f16_f32 on gfx950), which also give the IEEE
// results for overflow, subnormals and NaN.
template <int DT> struct Storage;

template <> struct Storage<kFp32> {
  static constexpr int kVec = 4;
  static constexpr int kBytes = 4;
  __device__ static __forceinline__ void unpack(u32x4 v, float (&f)[4]) {
    f[0] = as_f32(v.x); f[1] = as_f32(v.y); f[2] = as_f32(v.z); f[3] = as_f32(v.w);
  }
  __device__ static __forceinline__ u32x4 pack(const float (&f)[4]) {
    u32x4 v = {as_u32(f[0]), as_u32(f[1]), as_u32(f[2]), as_u32(f[3])};
    return v;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return static_cast<const float*>(p)[i];
  }
  __device__ static __forceinline__ void store_one(void* p, int64_t i, float f) {
    static_cast<float*>(p)[i] = f;
  }
};

template <> struct Storage<kBf16> {
  static constexpr int kVec = 8;
  static constexpr int kBytes = 2;
  __device__ static __forceinline__ void unpack(u32x4 v, float (&f)[8]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t d = v[k];
      f[2 * k] = as_f32(d << 16);               // a bf16 is the top half of an fp32
      f[2 * k + 1] = as_f32(d & 0xFFFF0000u);
    }
  }
  __device__ static __forceinline__ u32x4 pack(const float (&f)[8]) {
    u32x4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f32x2 p = {f[2 * k], f[2 * k + 1]};
      v[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
    }
    return v;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return as_f32(static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
  }
  __device__ static __forceinline__ void store_one(void* p, int64_t i, float f) {
    static_cast<uint16_t*>(p)[i] = __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
  }
};

template <> struct Storage<kFp16> {
  static constexpr int kVec = 8;
  static constexpr int kBytes = 2;
  __device__ static __forceinline__ void unpack(u32x4 v, float (&f)[8]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // The element is copied to a scalar first: a bit_cast applied directly to
      // a vector-element expression reads element 0 whatever k is.
      const uint32_t d = v[k];
      f32x2 p = __builtin_convertvector(__builtin_bit_cast(f16x2, d), f32x2);
      f[2 * k] = p.x;
      f[2 * k + 1] = p.y;
    }
  }
  __device__ static __forceinline__ u32x4 pack(const float (&f)[8]) {
    u32x4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f32x2 p = {f[2 * k], f[2 * k + 1]};
      v[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, f16x2));
    }
    return v;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return static_cast<float>(static_cast<const _Float16*>(p)[i]);
  }
  __device__ static __forceinline__ void store_one(void* p, int64_t i, float f) {
    static_cast<_Float16*>(p)[i] = static_cast<_Float16>(f);
  }
};

// Rows that are not 16-byte aligned, held in registers: the 16-byte slots of a row are counted
// from the 128-byte line in which the row starts (slot j lies at line + 16 * j), so that the
// kilobyte one load or store instruction of a wavefront covers is eight whole lines wherever
// the row starts.  The cut names the slots that the row covers whole and the single elements
// before the first and after the last of them.
constexpr int kLineBytes = 128;

struct RowCut {
  int off;          // bytes from the line boundary at or before the row's first byte to that byte
  int first;        // first slot that the row covers whole
  int end;          // one past the last such slot
  int head, tail;   // elements before slot `first` and after slot `end - 1`
};

template <int EB>
__host__ __device__ __forceinline__ RowCut row_cut(const void* row, int n) {
  RowCut c;
  c.off = (int)(reinterpret_cast<uintptr_t>(row) & (kLineBytes - 1));
  c.first = (c.off + 15) >> 4;
  const int total = c.off + n * EB;
  c.end = total >> 4;
  if (c.end < c.first) c.end = c.first;                 // a row inside one slot: elements only
  c.head = (16 * c.first - c.off) / EB;
  c.head = c.head < n ? c.head : n;
  c.tail = c.end > c.first ? (total - 16 * c.end) / EB : n - c.head;
  return c;
}

// Which row workgroup `block` starts with, in grids that are a multiple of 64 workgroups (the
// flat grids of one workgroup per row, rounded up, where workgroups whose row lies past M have
// nothing to do; the resident grids of the walking forms, whose workgroups go on to rows
// first + gridDim, ...).  Workgroup b runs on XCD b mod 8.  Taking row b would hand each XCD
// every eighth row; this permutation of each run of 64 hands it eight consecutive rows out of
// every 64 instead, so an XCD's accesses run over contiguous stretches of memory, and the
// line that an unaligned row shares with the next is fetched into one L2 instead of two
// (bf16 RMSNorm 16384 x 8191 in the walking form: 88.2 -> 85.7 us).  As a permutation of the
// row classes r mod 64 it keeps every row of a resident workgroup at one offset from a line.
constexpr bool kXcdRowBlocks = true;

__host__ __device__ __forceinline__ int64_t xcd_block_row(unsigned block) {
  if constexpr (kXcdRowBlocks) return (int64_t)(block & ~63u) + ((block & 7u) << 3) + ((block >> 3) & 7u);
  else return (int64_t)block;
}

// First row of workgroup `block` in the aligned one-workgroup-per-row kernels, whose launch code
// decides per call whether the rows go out in XCD blocks (host::flat_rows in launch_util.h).
__device__ __forceinline__ int64_t flat_first_row(unsigned block, int xcd_blocks) {
  return xcd_blocks ? xcd_block_row(block) : (int64_t)block;
}

}  // namespace rms
