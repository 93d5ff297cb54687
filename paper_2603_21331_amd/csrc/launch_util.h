// Host-side helpers shared by the libraries' launch code (each library is built on its own;
// everything here is inline).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <tuple>
#include <utility>

namespace rms {
namespace host {

// Kernel launch whose status is this launch's own.  hipGetLastError() after a <<<>>> launch
// also returns, and clears, an error that an earlier and unrelated runtime call of the thread
// left behind: a healthy launch would be blamed and the caller's pending error lost.
// hipLaunchKernel returns the status of the launch itself.  The arguments are converted to
// the kernel's parameter types first, as a <<<>>> launch would convert them.
template <typename... Params, typename... Args, size_t... I>
inline hipError_t launch_impl(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes,
                              hipStream_t stream, std::index_sequence<I...>, Args&&... args) {
  std::tuple<Params...> params{static_cast<Params>(args)...};
  void* ptrs[] = {static_cast<void*>(&std::get<I>(params))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream);
}

template <typename... Params, typename... Args>
inline hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes,
                         hipStream_t stream, Args&&... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "kernel argument count");
  return launch_impl(kernel, grid, block, lds_bytes, stream, std::index_sequence_for<Params...>{},
                     std::forward<Args>(args)...);
}

// Status of the calling thread's most recent RMS_LAUNCH.
inline hipError_t& launch_status() {
  static thread_local hipError_t status = hipSuccess;
  return status;
}

#define RMS_LAUNCH(kernel, grid, block, lds_bytes, stream, ...) \
  (::rms::host::launch_status() = ::rms::host::launch(kernel, grid, block, lds_bytes, stream, __VA_ARGS__))

// x and y at the same offset from a 16-byte boundary: then so is every row of theirs.
inline bool same_skew(const void* x, const void* y) {
  return ((reinterpret_cast<uintptr_t>(x) ^ reinterpret_cast<uintptr_t>(y)) & 15u) == 0;
}

// Compute units of the current device (256 on MI355X), looked up once per device.
inline int compute_units() {
  constexpr int kMaxDevices = 64;
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// Workgroups of the grid for the walking form of the element-addressed row kernels (resident
// workgroups that take rows blockIdx, blockIdx + grid, ...), 0 if the one-row-per-workgroup
// form should run.
// Each resident workgroup has one row in flight, and the sweeps on MI355X (N = 1025 .. 40961)
// put the best grid where about `bytes_per_cu` of rows are in flight per compute unit.  Around
// that number the grid is chosen so that the rows divide evenly among the workgroups (8192 rows
// over 5 workgroups per compute unit leave a sixth of the last round idle; over 4 none), and it
// stays a multiple of the compute units (other grids load them unevenly, measured 10 to 20 %
// slower) and of 8.  With fewer than four rows per workgroup there is nothing to spread the
// weight over.
inline int64_t walk_grid(int64_t M, int64_t row_bytes, int threads, int64_t bytes_per_cu) {
  constexpr int kMaxThreadsPerCu = 2048;
  constexpr int64_t kMinRows = 4;
  const int64_t cus = compute_units();
  if (cus % 8 != 0) return 0;
  const double want = (double)bytes_per_cu / (double)row_bytes;
  int64_t most = kMaxThreadsPerCu / threads;
  if (most > M / (kMinRows * cus)) most = M / (kMinRows * cus);
  int64_t best = 0;
  double best_cost = 0.0;
  for (int64_t p = 1; p <= most; ++p) {
    if ((double)p < 0.55 * want || (double)p > 1.5 * want + 1.0) continue;
    const int64_t grid = cus * p;
    const double rounds = (double)((M + grid - 1) / grid);
    const double miss = ((double)p > want ? (double)p - want : want - (double)p) / want;
    const double cost = rounds * (double)grid / (double)M * (1.0 + 0.15 * miss);
    if (best == 0 || cost < best_cost) {
      best = p;
      best_cost = cost;
    }
  }
  return cus * best;
}

}  // namespace host
}  // namespace rms
