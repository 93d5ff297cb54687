// C ABI of the row cross-entropy library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/crossentropy.h.
#include "../../include/crossentropy.h"

#include <hip/hip_runtime.h>

#include "crossentropy_kernels.h"

namespace {

constexpr int kBatch = 4;                       // 16-byte vectors loaded per thread per step
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

bool threads_ok(int g) { return g == 64 || g == 256 || g == 512 || g == 1024; }

// One wavefront per row while a row is at most 256 groups (4 KiB); then 256 threads, and
// 1024 once a thread of 256 would loop more than 16 times (rows beyond 256 KiB).
int pick_threads(int64_t groups) {
  if (groups <= 256) return 64;
  if (groups <= 256 * kBatch * 16) return 256;
  return 1024;
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

template <int DT, int G>
void launch(const void* x, const int64_t* target, float* loss, float* lse, int64_t M, int64_t N,
            hipStream_t stream) {
  const int nfull = (int)(N / rms::Storage<DT>::kVec);
  const int64_t blocks = M < kMaxGrid ? M : kMaxGrid;
  hipLaunchKernelGGL((rms::crossentropy_row_kernel<DT, G, kBatch, true>), dim3((unsigned)blocks),
                     dim3(G), 0, stream, x, target, loss, lse, M, N, nfull);
}

template <int DT>
int run_typed(const void* x, const int64_t* target, float* loss, float* lse, int64_t M, int64_t N,
              hipStream_t stream, int threads) {
  switch (threads) {
    case 64: launch<DT, 64>(x, target, loss, lse, M, N, stream); break;
    case 256: launch<DT, 256>(x, target, loss, lse, M, N, stream); break;
    case 512: launch<DT, 512>(x, target, loss, lse, M, N, stream); break;
    case 1024: launch<DT, 1024>(x, target, loss, lse, M, N, stream); break;
    default: return CROSSENTROPY_ERR_INVALID_ARG;
  }
  return hipGetLastError() == hipSuccess ? CROSSENTROPY_OK : CROSSENTROPY_ERR_LAUNCH;
}

int run(const void* x, const int64_t* target, float* loss, float* lse, int64_t M, int64_t N,
        int dtype, void* stream, int threads) {
  const int rc = check_args(x, target, loss, lse, M, N, dtype);
  if (rc != CROSSENTROPY_OK) return rc;
  if (threads != 0 && !threads_ok(threads)) return CROSSENTROPY_ERR_INVALID_ARG;
  if (M == 0) return CROSSENTROPY_OK;
  if (threads == 0) threads = pick_threads(N / (16 / elem_bytes(dtype)));
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
  return pick_threads(N / (16 / b));
}

const char* crossentropy_status_string(int status) {
  switch (status) {
    case CROSSENTROPY_OK: return "ok";
    case CROSSENTROPY_ERR_INVALID_ARG: return "invalid argument";
    case CROSSENTROPY_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
