// Host-side helpers shared by the libraries' launch code (each library is built on its own;
// everything here is inline).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
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

// Launch shape of the LDS-staged short-row kernels (packed_rows.h): rows per tile and
// workgroups.  A workgroup of `threads` threads works on threads / lanes rows at a time (one
// pass), so a tile is a whole number of passes wherever more than one pass fits: 41 rows of 197
// fp16 elements in passes of 16 leave a sixth of the third pass idle.  Among the whole numbers
// the one nearest to `target_bytes` is taken.  Kernels that write the tile back want small
// tiles (kPackedTargetReadWrite): then a launch is several workgroup generations whose load,
// compute and store phases overlap, where two generations of 16 KiB tiles run in lockstep
// (fp16 softmax over 64 MiB: 197 elements per row 26.0 -> 24.4 us, 77 elements 27.9 -> 25.0,
// 257 elements 26.5 -> 25.1).  Kernels that only read (row sum, cross-entropy) have no store
// phase to overlap and want as many bytes in flight as the tile holds (kPackedTargetReadOnly;
// row sum over 64 MiB of fp16 rows of 100 to 1001 elements: 11.9 to 12.4 us against 13.3 to 15.0
// with the small tiles).
constexpr int64_t kPackedTargetReadWrite = 7 * 1024;
constexpr int64_t kPackedTargetReadOnly = 16 * 1024;

struct PackedShape {
  int tile_rows;
  int64_t blocks;
};

inline PackedShape packed_shape(int64_t M, int64_t row_bytes, int lanes, int threads, int tile_bytes,
                                int64_t target_bytes, int64_t max_blocks) {
  const int groups = threads / lanes;
  const int64_t fit = tile_bytes / row_bytes;              // rows the tile can hold (at least 1)
  int64_t rows = fit;
  if (fit > groups) {
    const int64_t pass_bytes = groups * row_bytes;
    int64_t passes = (target_bytes + pass_bytes / 2) / pass_bytes;
    if (passes < 1) passes = 1;
    rows = passes * groups;
    if (rows > fit) rows = fit / groups * groups;
  }
  if (rows > M) rows = M;
  if (rows < 1) rows = 1;
  PackedShape s;
  s.tile_rows = (int)rows;
  s.blocks = (M + rows - 1) / rows;
  if (s.blocks > max_blocks) {
    // A workgroup takes several tiles then: as many workgroups as share them out evenly (10646
    // tiles over 2048 workgroups are six rounds, the last of them a fifth full; over 1775 all
    // six are full).
    const int64_t rounds = (s.blocks + max_blocks - 1) / max_blocks;
    s.blocks = (s.blocks + rounds - 1) / rounds;
  }
  return s;
}

// Workgroups of a flat grid of one workgroup per row whose kernel takes its row from
// xcd_block_row (vec_io.h): M, or `max_grid` (a multiple of 64) if that is less, rounded up to a
// multiple of 64; workgroups whose row lies past M have nothing to do.
inline int64_t flat_grid(int64_t M, int64_t max_grid) {
  return ((M < max_grid ? M : max_grid) + 63) / 64 * 64;
}

// The grid of an aligned one-workgroup-per-row kernel and whether its rows go out in XCD blocks
// of eight (flat_first_row in vec_io.h).  Measured on MI355X, blocks against rows one by one:
// workgroups of 256 to 1024 threads on rows of 8 to 64 KiB gain 0 to 4 % (RMSNorm bf16
// 16384 x 8192 with 512 threads 84.7 -> 82.4 us, softmax fp16 8192 x 32000 170.3 -> 163.8,
// LayerNorm fp16 4096 x 32768 97.0 -> 94.8, rows of 8 to 16 KiB 0.1 to 1.2 %); one wavefront
// per row loses 1 to 5 % (rows of 3 and 4 KiB), rows of 100 KiB and more lose 1.5 to 2 %, and
// the read-only kernels (cross-entropy, row sum) lose 1 to 4 %, so those keep rows one by one.
struct FlatRows {
  int64_t blocks;
  int xcd_blocks;
};
inline FlatRows flat_rows(int64_t M, int64_t max_grid, int threads, int64_t row_bytes) {
  const bool in_blocks = threads >= 256 && row_bytes >= 8 * 1024 && row_bytes <= 64 * 1024;
  return FlatRows{in_blocks ? flat_grid(M, max_grid) : (M < max_grid ? M : max_grid), in_blocks ? 1 : 0};
}

// Compute units of the current device (256 on MI355X), looked up once per device.
inline int compute_units() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cached[kMaxDevices] = {};      // threads may race to fill an entry: same value
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Workgroups of the grid for the walking form of the element-addressed row kernels (resident
// workgroups that take rows blockIdx, blockIdx + grid, ...), 0 if the one-row-per-workgroup
// form should run.
// Each resident workgroup has one row in flight, and the sweeps on MI355X (N = 1025 .. 40961)
// put the best grid where about `bytes_per_cu` of rows are in flight per compute unit.  Around
// that number the grid is chosen so that the rows divide evenly among the workgroups (8192 rows
// over 5 workgroups per compute unit leave a sixth of the last round idle; over 4 none), and it
// stays a multiple of the compute units (other grids load them unevenly, measured 10 to 20 %
// slower) and of 64: rows that many apart start at the same offset from a 128-byte line
// whatever the row length, which the walking kernels rely on.  A workgroup needs at least two
// rows to spread its weight fetch over, and with fewer than four the grid must also be close to
// the best one: small batches are over before an undersized grid has paid (bf16 rows of 8191
// elements: 1024 and 1536 rows 12 and 17 % faster on 512 resident workgroups than with one
// workgroup per row, 512 and 768 rows 10 and 3 % slower on 256).
inline int64_t walk_grid(int64_t M, int64_t row_bytes, int threads, int64_t bytes_per_cu) {
  constexpr int kMaxThreadsPerCu = 2048;
  constexpr int64_t kMinRows = 2;
  constexpr int64_t kSettledRows = 4;
  const int64_t cus = compute_units();
  if (cus % 64 != 0) return 0;
  const double want = (double)bytes_per_cu / (double)row_bytes;
  int64_t most = kMaxThreadsPerCu / threads;
  if (most > M / (kMinRows * cus)) most = M / (kMinRows * cus);
  int64_t best = 0;
  double best_cost = 0.0;
  for (int64_t p = 1; p <= most; ++p) {
    if ((double)p < 0.55 * want || (double)p > 1.5 * want + 1.0) continue;
    if (M < kSettledRows * cus * p && (double)p < 0.9 * want) continue;
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
