// The measurement aid: a streaming copy of known traffic.  Contract in include/measure.h.
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

const char* measure_status_string(int status) {
  switch (status) {
    case MEASURE_OK: return "ok";
    case MEASURE_ERR_INVALID_ARG: return "invalid argument";
    case MEASURE_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
