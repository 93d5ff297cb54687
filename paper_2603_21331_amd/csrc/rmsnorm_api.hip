// C ABI of the RMSNorm forward library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/rmsnorm.h.
#include "../../include/rmsnorm.h"

#include <hip/hip_runtime.h>

#include "rmsnorm_kernels.h"

namespace {

using rms::u32x4;

constexpr int kWaveMaxChunks16 = 16;   // 16-bit types: 16 chunks * 64 lanes * 8 = 8192 elements
constexpr int kWaveMaxChunks32 = 32;   // fp32:         32 chunks * 64 lanes * 4 = 8192 elements
constexpr int kBlockMaxChunks = 16;
constexpr int kBlockMaxThreads = 1024;
constexpr int kWavesPerBlock = 4;
constexpr int kGenericThreads = 256;
constexpr int64_t kMaxGrid = 1 << 20;  // beyond this the kernels stride over rows

int elem_bytes(int dtype) {
  switch (dtype) {
    case RMSNORM_DTYPE_FP32: return 4;
    case RMSNORM_DTYPE_FP16: return 2;
    case RMSNORM_DTYPE_BF16: return 2;
    default: return 0;
  }
}

int wave_max_chunks(int dtype) {
  return dtype == RMSNORM_DTYPE_FP32 ? kWaveMaxChunks32 : kWaveMaxChunks16;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_args(const void* x, const void* w, const void* y, int64_t M, int64_t N,
               float eps, int dtype) {
  if (elem_bytes(dtype) == 0) return RMSNORM_ERR_INVALID_ARG;
  if (M < 0 || N <= 0) return RMSNORM_ERR_INVALID_ARG;
  if (!(eps >= 0.0f)) return RMSNORM_ERR_INVALID_ARG;  // rejects negative and NaN
  if (M > 0 && (!x || !w || !y)) return RMSNORM_ERR_INVALID_ARG;
  if (M > INT64_MAX / N) return RMSNORM_ERR_INVALID_ARG;
  const uintptr_t mask = (uintptr_t)elem_bytes(dtype) - 1;
  if (M > 0 && (((uintptr_t)x | (uintptr_t)w | (uintptr_t)y) & mask)) return RMSNORM_ERR_INVALID_ARG;
  return RMSNORM_OK;
}

bool rows_vectorisable(const void* x, const void* w, const void* y, int64_t N, int dtype) {
  return aligned16(x) && aligned16(w) && aligned16(y) && (N * elem_bytes(dtype)) % 16 == 0;
}

int64_t vectors_per_row(int64_t N, int dtype) { return N * elem_bytes(dtype) / 16; }

bool wave_can(int64_t nvec, int dtype) {
  return nvec >= 1 && nvec <= (int64_t)rms::kWave * wave_max_chunks(dtype);
}

bool block_can(int64_t nvec) {
  return nvec >= 1 && nvec <= (int64_t)kBlockMaxThreads * kBlockMaxChunks;
}

int choose(const void* x, const void* w, const void* y, int64_t N, int dtype) {
  if (!rows_vectorisable(x, w, y, N, dtype)) return RMSNORM_VARIANT_GENERIC;
  const int64_t nvec = vectors_per_row(N, dtype);
  if (wave_can(nvec, dtype)) return RMSNORM_VARIANT_WAVE;
  if (block_can(nvec)) return RMSNORM_VARIANT_BLOCK;
  return RMSNORM_VARIANT_GENERIC;
}

struct Args {
  const void* x;
  const void* w;
  void* y;
  int64_t M;
  int64_t N;
  int nvec;
  float eps;
  hipStream_t stream;
};

template <int DT, int CHUNKS>
void launch_wave(const Args& a) {
  int64_t blocks = (a.M + kWavesPerBlock - 1) / kWavesPerBlock;
  if (blocks > kMaxGrid) blocks = kMaxGrid;
  hipLaunchKernelGGL((rms::rmsnorm_wave_kernel<DT, CHUNKS, kWavesPerBlock, true>),
                     dim3((unsigned)blocks), dim3(kWavesPerBlock * rms::kWave), 0, a.stream,
                     (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
                     (float)a.N, a.eps);
}

template <int DT, int CHUNKS, int T>
void launch_block(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  hipLaunchKernelGGL((rms::rmsnorm_block_kernel<DT, CHUNKS, T, true>),
                     dim3((unsigned)blocks), dim3(T), 0, a.stream,
                     (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
                     (float)a.N, a.eps);
}

template <int DT>
void launch_generic(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  hipLaunchKernelGGL((rms::rmsnorm_generic_kernel<DT, kGenericThreads>),
                     dim3((unsigned)blocks), dim3(kGenericThreads), 0, a.stream,
                     a.x, a.w, a.y, a.M, a.N, (float)a.N, a.eps);
}

#define RMS_CASE(n, call) case n: call; break;
#define RMS_CASES_1_16(M_)                                                            \
  RMS_CASE(1, M_(1)) RMS_CASE(2, M_(2)) RMS_CASE(3, M_(3)) RMS_CASE(4, M_(4))         \
  RMS_CASE(5, M_(5)) RMS_CASE(6, M_(6)) RMS_CASE(7, M_(7)) RMS_CASE(8, M_(8))         \
  RMS_CASE(9, M_(9)) RMS_CASE(10, M_(10)) RMS_CASE(11, M_(11)) RMS_CASE(12, M_(12))   \
  RMS_CASE(13, M_(13)) RMS_CASE(14, M_(14)) RMS_CASE(15, M_(15)) RMS_CASE(16, M_(16))
#define RMS_CASES_17_32(M_)                                                           \
  RMS_CASE(17, M_(17)) RMS_CASE(18, M_(18)) RMS_CASE(19, M_(19)) RMS_CASE(20, M_(20)) \
  RMS_CASE(21, M_(21)) RMS_CASE(22, M_(22)) RMS_CASE(23, M_(23)) RMS_CASE(24, M_(24)) \
  RMS_CASE(25, M_(25)) RMS_CASE(26, M_(26)) RMS_CASE(27, M_(27)) RMS_CASE(28, M_(28)) \
  RMS_CASE(29, M_(29)) RMS_CASE(30, M_(30)) RMS_CASE(31, M_(31)) RMS_CASE(32, M_(32))

template <int DT>
int dispatch_wave(const Args& a) {
  const int chunks = (a.nvec + rms::kWave - 1) / rms::kWave;
#define RMS_W(c) launch_wave<DT, c>(a)
  if constexpr (DT == rms::kFp32) {
    switch (chunks) {
      RMS_CASES_1_16(RMS_W)
      RMS_CASES_17_32(RMS_W)
      default: return RMSNORM_ERR_UNSUPPORTED;
    }
  } else {
    switch (chunks) {
      RMS_CASES_1_16(RMS_W)
      default: return RMSNORM_ERR_UNSUPPORTED;
    }
  }
#undef RMS_W
  return RMSNORM_OK;
}

// Threads per row for the block kernel: the smallest workgroup that keeps the
// row within 16 chunks per thread, so short rows do not pay for idle waves.
template <int DT>
int dispatch_block(const Args& a) {
  if (a.nvec <= 256 * kBlockMaxChunks) {
    const int chunks = (a.nvec + 255) / 256;
#define RMS_B(c) launch_block<DT, c, 256>(a)
    switch (chunks) { RMS_CASES_1_16(RMS_B) default: return RMSNORM_ERR_UNSUPPORTED; }
#undef RMS_B
  } else if (a.nvec <= 512 * kBlockMaxChunks) {
    const int chunks = (a.nvec + 511) / 512;
#define RMS_B(c) launch_block<DT, c, 512>(a)
    switch (chunks) {
      RMS_CASE(9, RMS_B(9)) RMS_CASE(10, RMS_B(10)) RMS_CASE(11, RMS_B(11)) RMS_CASE(12, RMS_B(12))
      RMS_CASE(13, RMS_B(13)) RMS_CASE(14, RMS_B(14)) RMS_CASE(15, RMS_B(15)) RMS_CASE(16, RMS_B(16))
      default: return RMSNORM_ERR_UNSUPPORTED;
    }
#undef RMS_B
  } else {
    const int chunks = (a.nvec + 1023) / 1024;
#define RMS_B(c) launch_block<DT, c, 1024>(a)
    switch (chunks) {
      RMS_CASE(9, RMS_B(9)) RMS_CASE(10, RMS_B(10)) RMS_CASE(11, RMS_B(11)) RMS_CASE(12, RMS_B(12))
      RMS_CASE(13, RMS_B(13)) RMS_CASE(14, RMS_B(14)) RMS_CASE(15, RMS_B(15)) RMS_CASE(16, RMS_B(16))
      default: return RMSNORM_ERR_UNSUPPORTED;
    }
#undef RMS_B
  }
  return RMSNORM_OK;
}

template <int DT>
int run_typed(const Args& a, int variant) {
  int rc = RMSNORM_OK;
  switch (variant) {
    case RMSNORM_VARIANT_WAVE: rc = dispatch_wave<DT>(a); break;
    case RMSNORM_VARIANT_BLOCK: rc = dispatch_block<DT>(a); break;
    case RMSNORM_VARIANT_GENERIC: launch_generic<DT>(a); break;
    default: return RMSNORM_ERR_INVALID_ARG;
  }
  if (rc != RMSNORM_OK) return rc;
  return hipGetLastError() == hipSuccess ? RMSNORM_OK : RMSNORM_ERR_LAUNCH;
}

int run(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps, int dtype,
        void* stream, int variant) {
  int rc = check_args(x, w, y, M, N, eps, dtype);
  if (rc != RMSNORM_OK) return rc;
  if (variant < RMSNORM_VARIANT_AUTO || variant > RMSNORM_VARIANT_GENERIC)
    return RMSNORM_ERR_INVALID_ARG;
  if (M == 0) return RMSNORM_OK;

  const bool vec_ok = rows_vectorisable(x, w, y, N, dtype);
  const int64_t nvec = vec_ok ? vectors_per_row(N, dtype) : 0;
  if (variant == RMSNORM_VARIANT_AUTO) variant = choose(x, w, y, N, dtype);
  if (variant == RMSNORM_VARIANT_WAVE && !(vec_ok && wave_can(nvec, dtype)))
    return RMSNORM_ERR_UNSUPPORTED;
  if (variant == RMSNORM_VARIANT_BLOCK && !(vec_ok && block_can(nvec)))
    return RMSNORM_ERR_UNSUPPORTED;

  Args a{x, w, y, M, N, (int)nvec, eps, static_cast<hipStream_t>(stream)};
  switch (dtype) {
    case RMSNORM_DTYPE_FP32: return run_typed<rms::kFp32>(a, variant);
    case RMSNORM_DTYPE_FP16: return run_typed<rms::kFp16>(a, variant);
    case RMSNORM_DTYPE_BF16: return run_typed<rms::kBf16>(a, variant);
    default: return RMSNORM_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

int rmsnorm_fwd(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                int dtype, void* stream) {
  return run(x, w, y, M, N, eps, dtype, stream, RMSNORM_VARIANT_AUTO);
}

int rmsnorm_fwd_variant(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                        int dtype, void* stream, int variant) {
  return run(x, w, y, M, N, eps, dtype, stream, variant);
}

int rmsnorm_select_variant(const void* x, const void* w, const void* y, int64_t M, int64_t N,
                           int dtype) {
  const int rc = check_args(x, w, y, M, N, 0.0f, dtype);
  if (rc != RMSNORM_OK) return rc;
  return choose(x, w, y, N, dtype);
}

int64_t rmsnorm_wave_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)rms::kWave * wave_max_chunks(dtype) * (16 / b) : 0;
}

int64_t rmsnorm_block_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)kBlockMaxThreads * kBlockMaxChunks * (16 / b) : 0;
}

int rmsnorm_calib_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (bytes < 0 || bytes % 16 != 0) return RMSNORM_ERR_INVALID_ARG;
  if (bytes == 0) return RMSNORM_OK;
  if (!src || !dst || !aligned16(src) || !aligned16(dst)) return RMSNORM_ERR_INVALID_ARG;
  constexpr int kUnroll = 8, kThreads = 256;
  const int64_t nvec = bytes / 16;
  int64_t blocks = (nvec + kUnroll * kThreads - 1) / (kUnroll * kThreads);
  if (blocks > kMaxGrid) blocks = kMaxGrid;
  hipLaunchKernelGGL((rms::calib_copy_kernel<kUnroll, kThreads>), dim3((unsigned)blocks),
                     dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     (const u32x4*)src, (u32x4*)dst, nvec);
  return hipGetLastError() == hipSuccess ? RMSNORM_OK : RMSNORM_ERR_LAUNCH;
}

const char* rmsnorm_status_string(int status) {
  switch (status) {
    case RMSNORM_OK: return "ok";
    case RMSNORM_ERR_INVALID_ARG: return "invalid argument";
    case RMSNORM_ERR_UNSUPPORTED: return "variant does not support this shape or alignment";
    case RMSNORM_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
