// C ABI of the row cross-entropy library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/crossentropy.h.
#include "../../include/crossentropy.h"

#include <hip/hip_runtime.h>

#include "build_id.h"
#include "dispatch_util.h"
#include "launch_util.h"
#include "crossentropy_kernels.h"

RMS_DEFINE_BUILD_ID(crossentropy_build_id);

namespace {

constexpr int kBatch = 4;                       // 16-byte vectors loaded per thread per step
constexpr int kWave = 64;
constexpr int kMaxThreads = 1024;
constexpr int kWideThreads = 512;               // largest workgroup short of the full 1024
constexpr int64_t kMaxGrid = 1 << 20;
constexpr int64_t kMaxN = (int64_t)1 << 32;     // keeps the count of 16-byte groups well inside an int

int elem_bytes(int dtype) {
  switch (dtype) {
    case CROSSENTROPY_DTYPE_FP32: return 4;
    case CROSSENTROPY_DTYPE_FP16: return 2;
    case CROSSENTROPY_DTYPE_BF16: return 2;
    default: return 0;
  }
}

// threads_per_row == kPackedCode selects the LDS-staged kernel (lane-group width from N).
constexpr int kPackedCode = 2;
constexpr int64_t kPackedMaxN = 64 * rms::kPackElems;
constexpr int64_t kPackedMaxGrid = 8192;

bool threads_ok(int g) {
  return g == kPackedCode || g == 8 || g == 16 || g == 32 ||
         (g >= kWave && g <= kMaxThreads && g % kWave == 0);
}

constexpr int64_t kPackedAutoBytes = 256;    // aligned 16-bit rows up to this long also go through LDS

// Lane groups take 16-byte aligned rows of at most 8 vectors per lane.
constexpr int kSubwaveMaxChunks = 8;

bool subwave_can(const void* x, int64_t N, int dtype, int lanes) {
  const int b = elem_bytes(dtype);
  return ((uintptr_t)x & 15u) == 0 && (N * b) % 16 == 0 &&
         N * b / 16 <= (int64_t)lanes * kSubwaveMaxChunks;
}

// From sweeps on the GPU (fp16/bf16/fp32, N = 2048 ... 262144, 64 ... 1024 threads in steps
// of a wavefront).  The best thread count gives a thread about two batches of a 16-bit type
// (8 vectors) or one batch of fp32 (4 vectors): 16-bit logits cost twice the arithmetic per
// byte, and a second batch lets it overlap the loads of the other wavefronts.  Workgroups of
// more than 512 threads pay off only once every thread of 1024 still gets that much.
int pick_threads(int64_t N, int dtype, bool aligned) {
  const int b = elem_bytes(dtype);
  // From sweeps over rows of 16 bytes to 4 KiB: up to 256 bytes per row the LDS-staged kernel
  // beats the lane groups even on aligned rows (fp16 N = 128: 27 against 34 us per 128 MiB), and
  // for fp32 logits up to its limit of 1024 classes (12.2 to 14.2 against 12.8 to 18.3 us per
  // 64 MiB); a handful of classes (a 10-way classifier) take it with one lane per row.
  if (N * b <= kPackedAutoBytes || (dtype == CROSSENTROPY_DTYPE_FP32 && N <= kPackedMaxN)) return kPackedCode;
  const int64_t groups = N / (16 / b);
  // Few classes: 8, 16 or 32 lanes per row, four to eight vectors per lane.  Measured at
  // 128 MiB of fp16 logits: N = 128 64 us (one workgroup per row: 322), 256 53 (166), 512 48
  // (90), 1000 45 (58), 2048 43 (46); fp32 rows beyond 128 vectors are faster with 64 threads.
  if (aligned && groups >= 1) {
    if (groups <= 32) return 8;
    if (groups <= 64) return 16;
    if (groups <= (dtype == CROSSENTROPY_DTYPE_FP32 ? 128 : 256)) return 32;
  }
  // Rows of up to 512 classes that are not whole aligned vectors: several per workgroup
  // through LDS (fp16 N = 100: 0.55 TB/s with one workgroup per row).
  if (!aligned && N <= kPackedMaxN) return kPackedCode;
  const int64_t per_thread = dtype == CROSSENTROPY_DTYPE_FP32 ? kBatch : 2 * kBatch;
  const int64_t want = (groups + per_thread - 1) / per_thread;
  if (want >= kMaxThreads) return kMaxThreads;
  const int64_t rounded = (want + kWave - 1) / kWave * kWave;
  return (int)(rounded < kWave ? kWave : rounded > kWideThreads ? kWideThreads : rounded);
}

int check_args(const void* x, const int64_t* target, const float* loss, const float* lse,
               int64_t M, int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || M < 0 || N <= 0 || N >= kMaxN) return CROSSENTROPY_ERR_INVALID_ARG;
  if (M > INT64_MAX / N) return CROSSENTROPY_ERR_INVALID_ARG;
  if (M == 0) return CROSSENTROPY_OK;
  if (!x || !target || !loss) return CROSSENTROPY_ERR_INVALID_ARG;
  if (((uintptr_t)x & (uintptr_t)(b - 1)) || ((uintptr_t)target & 7u) || ((uintptr_t)loss & 3u) ||
      ((uintptr_t)lse & 3u))
    return CROSSENTROPY_ERR_INVALID_ARG;
  return CROSSENTROPY_OK;
}

template <int DT, int L>
void launch_subwave(const void* x, const int64_t* target, float* loss, float* lse, int64_t M,
                    int64_t N, hipStream_t stream) {
  constexpr int kRows = kWave / L;
  int64_t blocks = (M + kRows - 1) / kRows;
  if (blocks > ((int64_t)1 << 24)) blocks = (int64_t)1 << 24;
  const int nvec = (int)(N / rms::Storage<DT>::kVec);
  RMS_LAUNCH((rms::crossentropy_subwave_kernel<DT, L, kBatch, true>), dim3((unsigned)blocks),
                     dim3(kWave), 0, stream, (const rms::u32x4*)x, target, loss, lse, M, N, nvec);
}

template <int DT, int L, int E>
void launch_packed(const void* x, const int64_t* target, float* loss, float* lse, int64_t M,
                   int64_t N, hipStream_t stream) {
  const rms::host::PackedShape shape = rms::host::packed_shape(M, N * rms::Storage<DT>::kBytes, L, rms::kPackThreads,
                                                               rms::kPackTileBytes,
                                                               rms::host::kPackedTargetReadOnly, kPackedMaxGrid);
  const int tile_rows = shape.tile_rows;
  const int64_t blocks = shape.blocks;
  RMS_LAUNCH((rms::crossentropy_packed_kernel<DT, L, E, true>), dim3((unsigned)blocks),
                     dim3(rms::kPackThreads), 0, stream, x, target, loss, lse, M, (int)N, tile_rows);
}

template <int DT>
int run_typed(const void* x, const int64_t* target, float* loss, float* lse, int64_t M, int64_t N,
              hipStream_t stream, int threads) {
  if (threads == kPackedCode) {
    // Lanes per row and elements per lane: see with_packed_shape.  Rows of a multiple of 128
    // bytes get at least 8 lanes (at 64 bytes the narrow groups still win here: fewer
    // reductions).
    rms::host::with_packed_shape(N, rms::Storage<DT>::kBytes, 128, [&](auto lanes, auto elems) {
      launch_packed<DT, decltype(lanes)::value, decltype(elems)::value>(x, target, loss, lse, M, N, stream);
    });
    return rms::host::launch_status() == hipSuccess ? CROSSENTROPY_OK : CROSSENTROPY_ERR_LAUNCH;
  }
  if (threads < kWave) {
    switch (threads) {
      case 8: launch_subwave<DT, 8>(x, target, loss, lse, M, N, stream); break;
      case 16: launch_subwave<DT, 16>(x, target, loss, lse, M, N, stream); break;
      default: launch_subwave<DT, 32>(x, target, loss, lse, M, N, stream); break;
    }
    return rms::host::launch_status() == hipSuccess ? CROSSENTROPY_OK : CROSSENTROPY_ERR_LAUNCH;
  }
  const int64_t blocks = M < kMaxGrid ? M : kMaxGrid;
  RMS_LAUNCH((rms::crossentropy_row_kernel<DT, kBatch, true>), dim3((unsigned)blocks),
                     dim3((unsigned)threads), 0, stream, x, target, loss, lse, M, N);
  return rms::host::launch_status() == hipSuccess ? CROSSENTROPY_OK : CROSSENTROPY_ERR_LAUNCH;
}

int run(const void* x, const int64_t* target, float* loss, float* lse, int64_t M, int64_t N,
        int dtype, void* stream, int threads) {
  const int rc = check_args(x, target, loss, lse, M, N, dtype);
  if (rc != CROSSENTROPY_OK) return rc;
  if (threads != 0 && !threads_ok(threads)) return CROSSENTROPY_ERR_INVALID_ARG;
  if (M == 0) return CROSSENTROPY_OK;
  const int b = elem_bytes(dtype);
  if (threads == 0) {
    const bool aligned = ((uintptr_t)x & 15u) == 0 && (N * b) % 16 == 0;
    threads = pick_threads(N, dtype, aligned);
  } else if (threads == kPackedCode ? N > kPackedMaxN
                                    : (threads < kWave && !subwave_can(x, N, dtype, threads))) {
    return CROSSENTROPY_ERR_UNSUPPORTED;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (dtype) {
    case CROSSENTROPY_DTYPE_FP32: return run_typed<rms::kFp32>(x, target, loss, lse, M, N, s, threads);
    case CROSSENTROPY_DTYPE_FP16: return run_typed<rms::kFp16>(x, target, loss, lse, M, N, s, threads);
    case CROSSENTROPY_DTYPE_BF16: return run_typed<rms::kBf16>(x, target, loss, lse, M, N, s, threads);
    default: return CROSSENTROPY_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

int crossentropy_fwd(const void* x, const int64_t* target, float* loss, float* lse, int64_t M,
                     int64_t N, int dtype, void* stream) {
  return run(x, target, loss, lse, M, N, dtype, stream, 0);
}

int crossentropy_fwd_tuned(const void* x, const int64_t* target, float* loss, float* lse,
                           int64_t M, int64_t N, int dtype, void* stream, int threads_per_row) {
  if (threads_per_row == 0) return CROSSENTROPY_ERR_INVALID_ARG;
  return run(x, target, loss, lse, M, N, dtype, stream, threads_per_row);
}

int crossentropy_auto_threads_per_row(int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0 || N >= kMaxN) return CROSSENTROPY_ERR_INVALID_ARG;
  return pick_threads(N, dtype, (N * b) % 16 == 0);
}

const char* crossentropy_status_string(int status) {
  switch (status) {
    case CROSSENTROPY_OK: return "ok";
    case CROSSENTROPY_ERR_INVALID_ARG: return "invalid argument";
    case CROSSENTROPY_ERR_UNSUPPORTED: return "this thread count cannot run this shape or alignment";
    case CROSSENTROPY_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
