// C ABI of the row-sum library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/rowsum.h.
#include "../../include/rowsum.h"

#include <hip/hip_runtime.h>

#include "build_id.h"
#include "dispatch_util.h"
#include "launch_util.h"
#include "rowsum_kernels.h"

RMS_DEFINE_BUILD_ID(rowsum_build_id);

namespace {

constexpr int kBatch = 4;                       // 16-byte vectors loaded per thread per step
constexpr int kWave = 64;
constexpr int kMaxThreads = 1024;
constexpr int kWideThreads = 768;             // largest workgroup the automatic path uses
constexpr int kSubwaveMaxChunks = 8;            // vectors a lane takes in the short-row kernel
constexpr int64_t kMaxGrid = 1 << 20;
constexpr int64_t kMaxN = (int64_t)1 << 32;     // keeps the count of 16-byte groups inside an int

int elem_bytes(int dtype) {
  switch (dtype) {
    case ROWSUM_DTYPE_FP32: return 4;
    case ROWSUM_DTYPE_FP16: return 2;
    case ROWSUM_DTYPE_BF16: return 2;
    default: return 0;
  }
}

bool block_threads_ok(int g) { return g >= kWave && g <= kMaxThreads && g % kWave == 0; }

// threads_per_row 2: not a thread count, the LDS-staged kernel (N <= 1024, lane groups of 1 to
// 64 lanes chosen from N; what the automatic path takes for every such row).
constexpr int kPackedCode = 2;
constexpr int64_t kPackedMaxN = 64 * rms::kPackElems;
constexpr int64_t kPackedMaxGrid = 8192;
bool subwave_threads_ok(int g) { return g == 8 || g == 16 || g == 32; }

bool rows_aligned(const void* x, int64_t N, int dtype) {
  return ((uintptr_t)x & 15u) == 0 && (N * elem_bytes(dtype)) % 16 == 0;
}

// Threads per row for aligned rows of `groups` 16-byte vectors, from sweeps on the GPU (fp16,
// bf16, fp32; N = 128 ... 262144).  Rows of up to two kilobytes share a wavefront, about four
// vectors per lane (since the automatic path sends every row of up to 1024 elements through LDS,
// it no longer reaches these lane groups: they remain as a forced choice); longer rows get a workgroup in which a thread takes two or three vectors
// (all of them requested at once: a read-only stream wants loads in flight, not reuse), in
// whole wavefronts, and no more than 768 threads: beyond that the barrier costs more than
// the extra loads in flight bring.
int pick_threads(int64_t groups) {
  if (groups <= 32) return 8;
  if (groups <= 64) return 16;
  if (groups <= 128) return 32;
  const int64_t want = groups * 3 / 8 / kWave * kWave;
  return (int)(want < kWave ? kWave : want > kWideThreads ? kWideThreads : want);
}

// The automatic choice, from sweeps over rows of 16 bytes to 4 KiB: the LDS-staged kernel for
// every row of up to 1024 elements, aligned or not (a handful of elements: one lane per row,
// 14.5 us per 64 MiB at fp16 N = 8; 30 % faster than lane groups at 128 bytes, level with them to
// 2 % better from 256 bytes on); lane groups or a workgroup for longer aligned rows; a workgroup
// of at least one wavefront for the rest.
int pick_auto(int64_t N, int dtype, bool aligned) {
  const int b = elem_bytes(dtype);
  if (N <= kPackedMaxN) return kPackedCode;
  const int threads = pick_threads(N / (16 / b));
  return (!aligned && threads < kWave) ? kWave : threads;
}

int check_args(const void* x, const float* y, int64_t M, int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || M < 0 || N <= 0 || N >= kMaxN) return ROWSUM_ERR_INVALID_ARG;
  if (M > INT64_MAX / N) return ROWSUM_ERR_INVALID_ARG;
  if (M == 0) return ROWSUM_OK;
  if (!x || !y) return ROWSUM_ERR_INVALID_ARG;
  if (((uintptr_t)x & (uintptr_t)(b - 1)) || ((uintptr_t)y & 3u)) return ROWSUM_ERR_INVALID_ARG;
  return ROWSUM_OK;
}

template <int DT>
int run_block(const void* x, float* y, int64_t M, int64_t N, hipStream_t stream, int threads) {
  const int64_t blocks = M < kMaxGrid ? M : kMaxGrid;
  RMS_LAUNCH((rms::rowsum_row_kernel<DT, kBatch, true>), dim3((unsigned)blocks),
                     dim3((unsigned)threads), 0, stream, x, y, M, N);
  return rms::host::launch_status() == hipSuccess ? ROWSUM_OK : ROWSUM_ERR_LAUNCH;
}

template <int DT, int L>
int run_subwave_l(const void* x, float* y, int64_t M, int nvec, hipStream_t stream) {
  constexpr int kRows = kWave / L;
  int64_t blocks = (M + kRows - 1) / kRows;
  if (blocks > kMaxGrid) blocks = kMaxGrid;
  RMS_LAUNCH((rms::rowsum_subwave_kernel<DT, L, true>), dim3((unsigned)blocks), dim3(kWave),
                     0, stream, (const rms::u32x4*)x, y, M, nvec);
  return rms::host::launch_status() == hipSuccess ? ROWSUM_OK : ROWSUM_ERR_LAUNCH;
}

template <int DT, int L, int E>
void launch_packed(const void* x, float* y, int64_t M, int64_t N, hipStream_t stream) {
  const rms::host::PackedShape shape = rms::host::packed_shape(M, N * rms::Storage<DT>::kBytes, L, rms::kPackThreads,
                                                               rms::kPackTileBytes,
                                                               rms::host::kPackedTargetReadOnly, kPackedMaxGrid);
  const int tile_rows = shape.tile_rows;
  const int64_t blocks = shape.blocks;
  RMS_LAUNCH((rms::rowsum_packed_kernel<DT, L, E, true>), dim3((unsigned)blocks),
                     dim3(rms::kPackThreads), 0, stream, x, y, M, (int)N, tile_rows);
}

template <int DT>
int run_packed(const void* x, float* y, int64_t M, int64_t N, hipStream_t stream) {
  // Lanes per row and elements per lane: see with_packed_shape.
  rms::host::with_packed_shape(N, rms::Storage<DT>::kBytes, 64, [&](auto lanes, auto elems) {
    launch_packed<DT, decltype(lanes)::value, decltype(elems)::value>(x, y, M, N, stream);
  });
  return rms::host::launch_status() == hipSuccess ? ROWSUM_OK : ROWSUM_ERR_LAUNCH;
}

template <int DT>
int run_typed(const void* x, float* y, int64_t M, int64_t N, int nvec, hipStream_t stream,
              int threads) {
  switch (threads) {
    case kPackedCode: return run_packed<DT>(x, y, M, N, stream);
    case 8: return run_subwave_l<DT, 8>(x, y, M, nvec, stream);
    case 16: return run_subwave_l<DT, 16>(x, y, M, nvec, stream);
    case 32: return run_subwave_l<DT, 32>(x, y, M, nvec, stream);
    default: return run_block<DT>(x, y, M, N, stream, threads);
  }
}

int run(const void* x, float* y, int64_t M, int64_t N, int dtype, void* stream, int threads) {
  const int rc = check_args(x, y, M, N, dtype);
  if (rc != ROWSUM_OK) return rc;
  const int64_t groups = N / (16 / elem_bytes(dtype));
  const bool aligned = rows_aligned(x, N, dtype);
  if (threads != 0) {
    if (threads == kPackedCode) {
      if (N > kPackedMaxN) return ROWSUM_ERR_INVALID_ARG;
    } else if (subwave_threads_ok(threads)) {
      if (!aligned || groups > (int64_t)threads * kSubwaveMaxChunks) return ROWSUM_ERR_INVALID_ARG;
    } else if (!block_threads_ok(threads)) {
      return ROWSUM_ERR_INVALID_ARG;
    }
  }
  if (M == 0) return ROWSUM_OK;
  if (threads == 0) threads = pick_auto(N, dtype, aligned);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nvec = (int)groups;
  switch (dtype) {
    case ROWSUM_DTYPE_FP32: return run_typed<rms::kFp32>(x, y, M, N, nvec, s, threads);
    case ROWSUM_DTYPE_FP16: return run_typed<rms::kFp16>(x, y, M, N, nvec, s, threads);
    case ROWSUM_DTYPE_BF16: return run_typed<rms::kBf16>(x, y, M, N, nvec, s, threads);
    default: return ROWSUM_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

int rowsum_fwd(const void* x, float* y, int64_t M, int64_t N, int dtype, void* stream) {
  return run(x, y, M, N, dtype, stream, 0);
}

int rowsum_fwd_tuned(const void* x, float* y, int64_t M, int64_t N, int dtype, void* stream,
                     int threads_per_row) {
  if (threads_per_row == 0) return ROWSUM_ERR_INVALID_ARG;
  return run(x, y, M, N, dtype, stream, threads_per_row);
}

int rowsum_auto_threads_per_row(int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0 || N >= kMaxN) return ROWSUM_ERR_INVALID_ARG;
  return pick_auto(N, dtype, (N * b) % 16 == 0);
}

const char* rowsum_status_string(int status) {
  switch (status) {
    case ROWSUM_OK: return "ok";
    case ROWSUM_ERR_INVALID_ARG: return "invalid argument";
    case ROWSUM_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
