// The measurement aid: streaming copies of known traffic.  Contract in include/measure.h.
#include "../../include/measure.h"

#include <hip/hip_runtime.h>

#include "build_id.h"
#include "launch_util.h"
#include "vec_io.h"

RMS_DEFINE_BUILD_ID(measure_build_id);

namespace rms {

constexpr int kCopyThreads = 64;

// One 16-byte vector per thread, one wavefront per workgroup.  Of the copy shapes tried on
// MI355X (1 to 16 vectors per thread, 64 to 1024 threads, flat and resident grids) this finest
// one is the fastest, so its rate serves as the practical ceiling for a stream that is half
// reads and half writes.
__global__ void __launch_bounds__(kCopyThreads)
measure_copy_kernel(const u32x4* src, u32x4* dst, int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * kCopyThreads;
  for (int64_t i = (int64_t)blockIdx.x * kCopyThreads + threadIdx.x; i < nvec; i += stride)
    store_vec<true>(dst + i, load_vec<true>(src + i));
}

// The same bytes through LDS: 256 threads take a tile of 512 vectors (8 KiB), write it to LDS,
// meet at a barrier, read it back one wavefront over (so the round trip cannot be elided) and
// store it.  No arithmetic and no ragged edges: what is left of the copy's rate when the data is
// staged the way the short-row kernels stage it, and so the ceiling those are read against.
constexpr int kStagedThreads = 256;
constexpr int kStagedVecs = 2;

__global__ void __launch_bounds__(kStagedThreads)
measure_staged_copy_kernel(const u32x4* src, u32x4* dst, int64_t nvec) {
  __shared__ u32x4 tile[kStagedThreads * kStagedVecs];
  const int t = threadIdx.x;
  const int other = (t + 64) % kStagedThreads;
  const int64_t base = (int64_t)blockIdx.x * (kStagedThreads * kStagedVecs);
  u32x4 v[kStagedVecs];
#pragma unroll
  for (int k = 0; k < kStagedVecs; ++k) {
    const int64_t i = base + k * kStagedThreads + t;
    v[k] = load_vec<true>(src + (i < nvec ? i : nvec - 1));
  }
#pragma unroll
  for (int k = 0; k < kStagedVecs; ++k) tile[k * kStagedThreads + t] = v[k];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kStagedVecs; ++k) {
    const int64_t i = base + k * kStagedThreads + other;
    if (i < nvec) store_vec<true>(dst + i, tile[k * kStagedThreads + other]);
  }
}

}  // namespace rms

extern "C" {

int measure_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (bytes < 0 || bytes % 16 != 0) return MEASURE_ERR_INVALID_ARG;
  if (bytes == 0) return MEASURE_OK;
  if (!src || !dst) return MEASURE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return MEASURE_ERR_INVALID_ARG;
  const int64_t nvec = bytes / 16;
  int64_t blocks = (nvec + rms::kCopyThreads - 1) / rms::kCopyThreads;
  if (blocks > (int64_t)1 << 24) blocks = (int64_t)1 << 24;
  RMS_LAUNCH(rms::measure_copy_kernel, dim3((unsigned)blocks), dim3(rms::kCopyThreads), 0,
             static_cast<hipStream_t>(stream), (const rms::u32x4*)src, (rms::u32x4*)dst, nvec);
  return rms::host::launch_status() == hipSuccess ? MEASURE_OK : MEASURE_ERR_LAUNCH;
}

int measure_staged_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (bytes < 0 || bytes % 16 != 0) return MEASURE_ERR_INVALID_ARG;
  if (bytes == 0) return MEASURE_OK;
  if (!src || !dst) return MEASURE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return MEASURE_ERR_INVALID_ARG;
  const int64_t nvec = bytes / 16;
  constexpr int64_t kTile = rms::kStagedThreads * rms::kStagedVecs;
  const int64_t blocks = (nvec + kTile - 1) / kTile;
  if (blocks > (int64_t)1 << 30) return MEASURE_ERR_INVALID_ARG;       // 8 TiB: past any device
  RMS_LAUNCH(rms::measure_staged_copy_kernel, dim3((unsigned)blocks), dim3(rms::kStagedThreads), 0,
             static_cast<hipStream_t>(stream), (const rms::u32x4*)src, (rms::u32x4*)dst, nvec);
  return rms::host::launch_status() == hipSuccess ? MEASURE_OK : MEASURE_ERR_LAUNCH;
}

const char* measure_status_string(int status) {
  switch (status) {
    case MEASURE_OK: return "ok";
    case MEASURE_ERR_INVALID_ARG: return "invalid argument";
    case MEASURE_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
