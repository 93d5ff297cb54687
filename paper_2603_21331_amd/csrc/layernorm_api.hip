// C ABI of the row LayerNorm library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/layernorm.h.
#include "../../include/layernorm.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "build_id.h"
#include "dispatch_util.h"
#include "launch_util.h"
#include "layernorm_kernels.h"
#include "queue_slots.h"

RMS_DEFINE_BUILD_ID(layernorm_build_id);

// Counters of the work-queue kernel: one block of kQueueSlotWords words per stream slot
// (queue_slots.h), all zero between launches (the kernel leaves them zero).  128 KiB per GPU,
// held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address of each GPU's copy is looked up once per device
// (queue_base below) and only that address is ever passed to a kernel.
namespace {
constexpr int kQueueSlotWords = rms::kLnQueueMaxShards * rms::kLnQueueStride;   // 4 KiB
}  // namespace
static __device__ __align__(256) unsigned queue_counters[rms::host::kStreamSlots * kQueueSlotWords];

namespace {

using rms::host::compute_units;
using rms::host::walk_grid;

using rms::u32x4;

// Instantiated (threads per row : chunks per thread); a chunk is one 16-byte vector.
//   8, 16, 32 : 1..2     64 : 1..4     256, 512, 1024 : 1..8
constexpr int kSubwaveMaxChunks = 2;
constexpr int kWaveMaxChunks = 4;
constexpr int kBlockMaxChunks = 8;
constexpr int kMaxThreads = 1024;
constexpr int kSmallRowVectors = 256;
constexpr int kGenericThreads = 256;
constexpr int64_t kMaxGrid = 1 << 20;

int elem_bytes(int dtype) {
  switch (dtype) {
    case LAYERNORM_DTYPE_FP32: return 4;
    case LAYERNORM_DTYPE_FP16: return 2;
    case LAYERNORM_DTYPE_BF16: return 2;
    default: return 0;
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// b may be null (no bias); everything else is required when M > 0.
int check_args(const void* x, const void* w, const void* b, const void* y, int64_t M, int64_t N,
               float eps, int dtype) {
  if (elem_bytes(dtype) == 0) return LAYERNORM_ERR_INVALID_ARG;
  if (M < 0 || N <= 0) return LAYERNORM_ERR_INVALID_ARG;
  if (!(eps >= 0.0f)) return LAYERNORM_ERR_INVALID_ARG;
  if (M > 0 && (!x || !w || !y)) return LAYERNORM_ERR_INVALID_ARG;
  if (M > INT64_MAX / N) return LAYERNORM_ERR_INVALID_ARG;
  const uintptr_t mask = (uintptr_t)elem_bytes(dtype) - 1;
  if (M > 0 && (((uintptr_t)x | (uintptr_t)w | (uintptr_t)b | (uintptr_t)y) & mask))
    return LAYERNORM_ERR_INVALID_ARG;
  return LAYERNORM_OK;
}

bool rows_vectorisable(const void* x, const void* w, const void* b, const void* y, int64_t N,
                       int dtype) {
  return aligned16(x) && aligned16(w) && aligned16(b) && aligned16(y) &&
         (N * elem_bytes(dtype)) % 16 == 0;
}

int max_chunks_for(int threads) {
  switch (threads) {
    case 8: case 16: case 32: return kSubwaveMaxChunks;
    case 64: return kWaveMaxChunks;
    case 256: case 512: case 1024: return kBlockMaxChunks;
    default: return 0;
  }
}

bool threads_can(int threads, int64_t nvec) {
  const int mc = max_chunks_for(threads);
  return mc > 0 && nvec >= 1 && (nvec + threads - 1) / threads <= mc;
}

// Threads per row of the automatic path, from sweeps on the GPU: lane groups for rows up to
// 64 vectors, one wavefront up to 256 vectors; then the smallest workgroup in which a
// thread holds at most 24 elements of a 16-bit type or 16 of fp32 (three or four chunks),
// which runs the resident kernel; rows too long for that (beyond 3072 vectors of a 16-bit
// type, 4096 of fp32) take the smallest workgroup that holds them in at most 8 chunks per
// thread.  0: does not fit in registers.
constexpr int kResidentMaxElems = 24;    // elements per thread the resident kernel holds
constexpr int kResidentAutoElems32 = 16; // what the automatic path asks of it for fp32

int pick_threads(int64_t nvec, int min_threads, int dtype) {
  if (min_threads <= 8) {
    if (nvec <= 8) return 8;
    if (nvec <= 16) return 16;
    // Two chunks per lane beat twice the lanes with one chunk each (3 to 20 %, most where the
    // row does not fill the wider group).
    // In fp32 a lane holds half as many elements and the exact fits keep one chunk.
    const bool fp32 = dtype == LAYERNORM_DTYPE_FP32;
    if (nvec <= 32) return (fp32 && nvec == 32) ? 32 : 16;
    if (nvec <= 64) return (fp32 && nvec == 64) ? 64 : 32;
  }
  if (min_threads <= 64 && nvec <= kSmallRowVectors) return 64;
  const int vec = 16 / elem_bytes(dtype);
  const int limit = dtype == LAYERNORM_DTYPE_FP32 ? kResidentAutoElems32 : kResidentMaxElems;
  for (int g = 256; g <= kMaxThreads; g *= 2)
    if (g >= min_threads && (nvec + g - 1) / g * vec <= limit) return g;
  for (int g = 256; g <= kMaxThreads; g *= 2)
    if (g >= min_threads && threads_can(g, nvec)) return g;
  return 0;
}

// Threads per row for the element-addressed kernel over the whole 16-byte pieces of a row
// (whole_pieces); 0 if the row does not fit in registers.
int pick_threads_unaligned(int64_t slots) {
  if (slots <= kSmallRowVectors) return 64;
  for (int g = 256; g <= kMaxThreads; g *= 2)
    if (slots <= (int64_t)g * kBlockMaxChunks) return g;
  return 0;
}

// ---------------------------------------------------------------------------
// The work-queue form of the resident kernel: when it runs, with what grid, and where its
// counters live.
// ---------------------------------------------------------------------------
constexpr int64_t kQueueMaxRows = (int64_t)1 << 30;          // tickets are 32-bit
constexpr int kQueueWideElems = 32;    // elements of a 16-bit type per thread, weight and bias kept packed

struct QueuePlan {
  int threads;       // 256 or 512 threads hold the row; the workgroup has one wavefront more
  int grid;          // resident workgroups, a multiple of `shards`
  int shards;        // 1 .. kLnQueueMaxShards
  int block_shift;   // rows are handed to the shards in blocks of 1 << block_shift
};

// Threads that hold a row in the work-queue kernel, 0 if it cannot take the row: the smaller of
// 256 and 512 (with 1024 the workgroup has no room for the wavefront that draws) in which a
// thread holds at most 32 elements of a 16-bit type (beyond 24 with weight and bias kept packed,
// see LnSlices) or 16 of fp32; fewer than 2^30 rows.
int queue_threads(int64_t M, int64_t nvec, int dtype) {
  if (nvec < 1 || M < 1 || M >= kQueueMaxRows) return 0;
  const int vec = 16 / elem_bytes(dtype);
  const int limit = dtype == LAYERNORM_DTYPE_FP32 ? kResidentAutoElems32 : kQueueWideElems;
  for (int g = 256; g <= 512; g *= 2)
    if ((nvec + g - 1) / g * vec <= limit) return g;
  return 0;
}

// Tuned on MI355X (sustained runs over rotating buffers; the resident kernel in brackets).
// 256 threads: two workgroups per compute unit (three for rows of 6 KiB and less), 16 shards:
//   fp16 32768 x 4096 84.0 us (90.8), 32768 x 5120 103.8 (115.0), 32768 x 6144 123.0 (133.4),
//   65536 x 3072 128.0 (145.0), fp32 32768 x 4096 162.6 (179.1), 65536 x 2048 163.9 (185.7);
//   8 shards are 10 to 15 % slower than 16, 32 level; three or four workgroups per compute
//   unit 1 to 4 % slower from 8 KiB rows on.
// 512 threads: one workgroup per compute unit, 8 shards: bf16 8192 x 12288 62.2 (67.6), fp32
//   8192 x 8192 83.8 (91.4), fp32 16384 x 6144 125.4 (129.6), bf16 8192 x 16384 86.5 (95.2 with
//   1024 threads); 16 and 32 shards 0.5 to 2 % slower, two workgroups per compute unit 2 to 3 %.
// Blocks of at most 128 KiB of rows, as in RMSNorm's kernel.
QueuePlan queue_plan(int64_t nvec, int threads) {
  const int cus = compute_units();
  const int64_t row_bytes = nvec * 16;
  QueuePlan p;
  p.threads = threads;
  p.shards = threads == 256 ? 16 : 8;
  const int per_cu = threads != 256 ? 1 : nvec <= 384 ? 3 : 2;
  p.grid = cus * per_cu / p.shards * p.shards;
  if (p.grid < p.shards) p.grid = p.shards;
  int shift = 0;
  while (((int64_t)2 << shift) * row_bytes <= 128 * 1024) ++shift;   // largest block of at most 128 KiB
  p.block_shift = shift;
  return p;
}

// Whether the automatic path takes the work-queue kernel.  It wins once a launch is long enough
// for the compute units to drift apart (x of 64 to 96 MiB: level or up to 5 % behind the
// resident kernel; 128 MiB: 2 to 2.5 % ahead at 8 and 16 KiB rows in 256 threads; 192 MiB: 5 to
// 6 %; 512 MiB: 9 to 12 %).  Rows of 6 KiB and less, and the rows of 12 to 16 KiB of a 16-bit type
// that 256 threads hold with weight and bias packed, are level at 128 MiB and ahead from 192 to
// 256 MiB (bf16 16384 x 8192: 85.6 -> 82.9 us, 32768 x 8192: 171.2 -> 161.7; fp16 16384 x 7168:
// 77.4 -> 74.7).  With 512 threads, rows beyond 20 KiB are ahead from 96 MiB (24 KiB rows 5.5 %;
// bf16 rows of 32 KiB, which otherwise take 1024 threads: 2 % at 96 MiB, 9 % at 256 MiB), rows of
// up to 20 KiB only from 256 MiB (160 MiB: 0.4 to 3 % behind, 320 MiB: 2 to 3 % ahead).
bool queue_pays(int64_t M, int64_t nvec, int dtype) {
  const int g = queue_threads(M, nvec, dtype);
  if (g == 0 || nvec <= kSmallRowVectors) return false;   // (one wavefront takes rows that short)
  if ((nvec * 16) % 64 != 0 && nvec * 16 <= 32 * 1024) return false;   // (the element-addressed kernel takes those: off_line_kernel)
  const int64_t bytes = M * nvec * 16;
  const bool packed_slices = dtype != LAYERNORM_DTYPE_FP32 && nvec > 768;
  if (g == 256) return bytes >= ((int64_t)(nvec <= 384 || packed_slices ? 192 : 128) << 20);
  return bytes >= ((int64_t)(nvec <= 1280 ? 256 : 96) << 20);
}

bool plan_valid(const QueuePlan& p) {
  return (p.threads == 256 || p.threads == 512) && p.shards >= 1 && p.shards <= rms::kLnQueueMaxShards &&
         p.grid >= p.shards && p.grid % p.shards == 0 && p.grid <= (1 << 16) && p.block_shift >= 0 &&
         p.block_shift <= 16;
}

// Device address of this GPU's copy of `queue_counters`, looked up once per device with that
// device current; nullptr if the lookup fails.
unsigned* queue_base() {
  static std::mutex mu;
  static unsigned* base[rms::host::kSlotDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= rms::host::kSlotDevices) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (base[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(queue_counters)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    base[dev] = static_cast<unsigned*>(p);
  }
  return base[dev];
}

// The counter block of `stream` on the current device, nullptr if the call has to do without
// the work-queue kernel (see queue_slots.h for the streams that get none).
unsigned* queue_counters_for(hipStream_t stream) {
  static rms::host::StreamSlots slots;
  unsigned* base = queue_base();
  if (base == nullptr) return nullptr;
  const int k = slots.block_of(stream);
  return k < 0 ? nullptr : base + (size_t)k * kQueueSlotWords;
}

struct Args {
  const void* x;
  const void* w;
  const void* b;
  void* y;
  int64_t M;
  int64_t N;
  int nvec;
  float eps;
  hipStream_t stream;
  unsigned* counters;   // work-queue kernel only
  QueuePlan plan;
};

template <int DT, int CHUNKS, int G>
void launch_queue(const Args& a) {
  constexpr int kElems = CHUNKS * rms::Storage<DT>::kVec;
  if constexpr (kElems <= kQueueWideElems) {
    RMS_LAUNCH((rms::layernorm_queue_kernel<DT, CHUNKS, G, true, (kElems > kResidentMaxElems)>), dim3((unsigned)a.plan.grid),
               dim3(G + rms::kLnWave), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w, (const u32x4*)a.b,
               (u32x4*)a.y, a.M, a.nvec, 1.0f / (float)a.N, a.eps, a.counters, a.plan.shards, a.plan.block_shift);
  }
}

template <int DT, int CHUNKS, int G>
void launch_row(const Args& a) {
  // Rows of at most 24 elements per thread: resident workgroups, weight and bias in registers.
  // Each workgroup has one row requested ahead, so the workgroups on a compute unit decide
  // how many bytes it has in flight; about 24 KiB measured best on MI355X.  Rows of 10 KiB
  // and more: eight wavefronts per compute unit (sixteen for 1024 threads, which cannot be
  // fewer; twice as many are 4 to 8 % slower).  Shorter rows need more workgroups: three at
  // 8 KiB (1 % faster than two), four at 6 KiB and below (10 to 15 % faster).
  if constexpr (CHUNKS * rms::Storage<DT>::kVec <= kResidentMaxElems && G >= 256) {
    const int per_cu = G != 256 ? 1 : a.nvec <= 384 ? 4 : a.nvec <= 512 ? 3 : 2;
    int64_t grid = (int64_t)compute_units() * per_cu;
    if (grid > a.M) grid = a.M;
    RMS_LAUNCH((rms::layernorm_row_resident_kernel<DT, CHUNKS, G, true>), dim3((unsigned)grid),
                       dim3(G), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w,
                       (const u32x4*)a.b, (u32x4*)a.y, a.M, a.nvec, 1.0f / (float)a.N, a.eps);
    return;
  }
  const rms::host::FlatRows rows = rms::host::flat_rows(a.M, kMaxGrid, G, (int64_t)a.nvec * 16);
  RMS_LAUNCH((rms::layernorm_row_kernel<DT, CHUNKS, G, true>), dim3((unsigned)rows.blocks),
                     dim3(G), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w,
                     (const u32x4*)a.b, (u32x4*)a.y, a.M, a.nvec, (float)a.N, a.eps, rows.xcd_blocks);
}

template <int DT, int CHUNKS, int L>
void launch_subwave(const Args& a) {
  constexpr int kRows = rms::kLnWave / L;
  int64_t blocks = (a.M + kRows - 1) / kRows;
  if (blocks > ((int64_t)1 << 24)) blocks = (int64_t)1 << 24;
  RMS_LAUNCH((rms::layernorm_subwave_kernel<DT, CHUNKS, L, true>), dim3((unsigned)blocks),
                     dim3(rms::kLnWave), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w,
                     (const u32x4*)a.b, (u32x4*)a.y, a.M, a.nvec, (float)a.N, a.eps);
}

// The walking form of the element-addressed kernel: groups per thread that fit in registers
// next to the packed weight and bias, and where its grid is best, in bytes of rows in flight
// per compute unit (each resident workgroup has one row in flight; swept on MI355X: 6
// workgroups of 256 threads at N = 4097, 3 at N = 8191, 2 of 512 at N = 12289).
constexpr int kWalkMaxChunks = 4;
constexpr int64_t kWalkBytesPerCu = 48 * 1024;

// The grid of the walking form for this call and its threads per row, 0 for one workgroup
// per row: the smallest workgroup that holds the row's slots in kWalkMaxChunks per thread.
// Rows of up to 256 slots, which one wavefront holds, gain nothing measurable and stay as they
// are.  The rows are cut at the 128-byte lines of x; where y sits at another offset from a line
// its stores straddle the lines.  walk_grid returns multiples of 64 workgroups only, which is
// what keeps every row of a workgroup at the same offset from a line.
int64_t unaligned_walk_grid(int64_t M, int64_t N, int bytes, int* threads) {
  const int64_t slots = rms::host::whole_pieces(N, bytes);
  int g = 256;
  while (g < kMaxThreads && slots > (int64_t)g * kWalkMaxChunks) g *= 2;
  if (slots <= rms::kLnWave * kWalkMaxChunks || slots > (int64_t)g * kWalkMaxChunks) return 0;
  *threads = g;
  return walk_grid(M, N * bytes, g, kWalkBytesPerCu);
}

// walk > 0: the walking form with that many resident workgroups.
template <int DT, int CHUNKS, int G>
void launch_row_unaligned(const Args& a, int64_t walk) {
  if constexpr (CHUNKS <= kWalkMaxChunks) {
    if (walk > 0) {
      // The 16-bit types with the next row requested ahead (2 to 15 % faster: fp16 16384 x 2057
      // 40.7 -> 34.7 us, bf16 4096 x 20481 69.4 -> 61.3, fp16 16384 x 8191 99.6 -> 97.1); fp32 rows,
      // with half the elements to work on per byte, are level to 4 % slower that way.
      if constexpr (DT != rms::kFp32)
        RMS_LAUNCH((rms::layernorm_walk_kernel<DT, CHUNKS, G, true>),
                           dim3((unsigned)walk), dim3(G), 0, a.stream, a.x, a.w, a.b, a.y, a.M,
                           (int)a.N, (float)a.N, a.eps);
      else
        RMS_LAUNCH((rms::layernorm_row_unaligned_kernel<DT, CHUNKS, G, true, true>),
                           dim3((unsigned)walk), dim3(G), 0, a.stream, a.x, a.w, a.b, a.y, a.M,
                           (int)a.N, (float)a.N, a.eps);
      return;
    }
  }
  const int64_t blocks = rms::host::flat_grid(a.M, kMaxGrid);
  RMS_LAUNCH((rms::layernorm_row_unaligned_kernel<DT, CHUNKS, G, true, false>),
                     dim3((unsigned)blocks), dim3(G), 0, a.stream, a.x, a.w, a.b, a.y, a.M,
                     (int)a.N, (float)a.N, a.eps);
}

// The LDS-staged kernel for short rows that are not 16-byte aligned: the narrowest lane group
// that holds the row (16 elements per lane), whole passes of the workgroup's lane groups per
// tile, at most 4096 workgroups (beyond that a workgroup takes several tiles and pays for its
// slices of weight and bias once; 64 MiB of 77-, 197- and 257-element fp16 rows: 26.5 to 27.0 us
// at 4096 workgroups, 28.5 to 32.4 with a workgroup per tile).  Its tile mirrors the offset of
// x from a 16-byte boundary; where y sits at another, the stores are element-aligned.
constexpr int64_t kPackedMaxN = 64 * rms::kPackElems;
constexpr int64_t kPackedMaxGrid = 4096;
// Aligned rows of at most 64 bytes also take it: one to four of the eight lanes of the
// narrowest lane group would hold a vector, and the LDS-staged kernel is 1.2 to 2 times faster.
constexpr int64_t kPackedAutoVectors = 4;

// Short aligned rows that would leave more than three lanes in ten of their lane group idle (5
// vectors on 8 lanes, 9 or 10 on 16: N = 40, 72, 80 in the 16-bit types) are up to 15 % faster
// through LDS.
bool packed_beats_lanes(int64_t nvec, int lanes) {
  const int64_t slots = (nvec + lanes - 1) / lanes * lanes;
  return nvec <= 16 && nvec * 10 < slots * 7;
}

bool packed_can(int64_t N) { return N <= kPackedMaxN; }

// Rows of at least 1 KiB whose loads are all 16-byte aligned, so that only y sits off a
// boundary: the register-resident kernel with element-aligned stores beats the LDS-staged one
// there (fp16 N = 1024: 3 to 30 % over the three operations); shorter rows stay with the
// LDS-staged kernel (N = 256: 12 to 25 % the other way).
bool only_stores_unaligned(const void* x, const void* w, const void* b, int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  return aligned16(x) && aligned16(w) && aligned16(b) && row_bytes % 16 == 0 && row_bytes >= 1024;
}

template <int DT, int L, int E>
void launch_packed(const Args& a) {
  const int n = (int)a.N;
  const rms::host::PackedShape shape = rms::host::packed_shape(a.M, (int64_t)n * rms::Storage<DT>::kBytes, L,
                                                               rms::kPackThreads, rms::kPackTileBytes,
                                                               rms::host::kPackedTargetReadWrite, kPackedMaxGrid);
  const int tile_rows = shape.tile_rows;
  const int64_t blocks = shape.blocks;
  RMS_LAUNCH((rms::layernorm_packed_kernel<DT, L, E, true>), dim3((unsigned)blocks),
                     dim3(rms::kPackThreads), 0, a.stream, a.x, a.w, a.b, a.y, a.M, n, tile_rows,
                     (float)a.N, a.eps);
}

// Lanes per row and elements per lane: see with_packed_shape.
template <int DT>
void dispatch_packed(const Args& a) {
  rms::host::with_packed_shape(a.N, rms::Storage<DT>::kBytes, 64, [&](auto lanes, auto elems) {
    launch_packed<DT, decltype(lanes)::value, decltype(elems)::value>(a);
  });
}

// The three-pass streaming kernel: about one batch of four groups per thread, whole
// wavefronts, at most 1024 threads (what every row long enough to need this kernel gets).
constexpr int64_t kStreamMaxN = (int64_t)1 << 31;   // it counts groups in an int

template <int DT>
void launch_stream(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  const int64_t nfull = a.N / rms::Storage<DT>::kVec;
  int64_t threads = (nfull / rms::kLnStreamBatch + rms::kLnWave - 1) / rms::kLnWave * rms::kLnWave;
  threads = threads < rms::kLnWave ? rms::kLnWave : threads > kMaxThreads ? kMaxThreads : threads;
  RMS_LAUNCH((rms::layernorm_stream_kernel<DT>), dim3((unsigned)blocks), dim3((unsigned)threads),
                     0, a.stream, a.x, a.w, a.b, a.y, a.M, a.N, (float)a.N, a.eps);
}

template <int DT>
void launch_generic(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  RMS_LAUNCH((rms::layernorm_generic_kernel<DT, kGenericThreads>), dim3((unsigned)blocks),
                     dim3(kGenericThreads), 0, a.stream, a.x, a.w, a.b, a.y, a.M, a.N, (float)a.N,
                     a.eps);
}

template <int DT>
int dispatch(const Args& a, int threads) {
  using rms::host::with_shape;
  const int chunks = (a.nvec + threads - 1) / threads;
  auto subwave = [&](auto l, auto c) { launch_subwave<DT, decltype(c)::value, decltype(l)::value>(a); };
  auto row = [&](auto g, auto c) { launch_row<DT, decltype(c)::value, decltype(g)::value>(a); };
  const bool launched = with_shape<8, 2>(threads, chunks, subwave) || with_shape<16, 2>(threads, chunks, subwave) ||
                        with_shape<32, 2>(threads, chunks, subwave) || with_shape<64, 4>(threads, chunks, row) ||
                        with_shape<256, 8>(threads, chunks, row) || with_shape<512, 8>(threads, chunks, row) ||
                        with_shape<1024, 8>(threads, chunks, row);
  return launched ? LAYERNORM_OK : LAYERNORM_ERR_UNSUPPORTED;
}

// Launches the element-addressed row kernel.  The caller has checked that the row fits.
template <int DT>
int dispatch_unaligned(const Args& a) {
  using rms::host::with_shape;
  const int slots = (int)rms::host::whole_pieces(a.N, rms::Storage<DT>::kBytes);
  int threads = pick_threads_unaligned(slots);
  int walk_threads = 0;
  const int64_t walk = unaligned_walk_grid(a.M, a.N, rms::Storage<DT>::kBytes, &walk_threads);
  if (walk > 0) threads = walk_threads;
  int chunks = (slots + threads - 1) / threads;
  if (chunks < 1) chunks = 1;
  auto row = [&](auto g, auto c) { launch_row_unaligned<DT, decltype(c)::value, decltype(g)::value>(a, walk); };
  const bool launched = with_shape<64, 4>(threads, chunks, row) || with_shape<256, 8>(threads, chunks, row) ||
                        with_shape<512, 8>(threads, chunks, row) || with_shape<1024, 8>(threads, chunks, row);
  return launched ? LAYERNORM_OK : LAYERNORM_ERR_UNSUPPORTED;
}

// Rows that are a multiple of 16 bytes but not of the 128-byte line cost the aligned kernels 3 to
// 19 %: every second or every eighth row starts off a line, a wavefront's 1 KiB then touches nine
// lines instead of eight, and the last line of a row is shared with the next row, which another
// XCD reads.  From 1 KiB on (below, the lane-group kernels are as often ahead as behind: fp16 rows of
// 136 elements 25 % slower than through LDS, of 328 elements 6 % faster) such rows go through LDS
// up to 1.75 KiB (fp16 60000 x 520: 29.5 -> 24.5 us, fp32 65536 x 260: 29.0 -> 24.6) and to the
// element-addressed kernel beyond, which lays its slots out from the line a row starts in (fp16
// 65536 x 2040 102.1 -> 95.8 us, 32768 x 3064 91.2 -> 81.9, 8192 x 12280 76.0 -> 70.4, 4096 x 8184
// 32.2 -> 26.1, 4096 x 16376 61.3 -> 47.5, fp32 16384 x 4092 96.1 -> 87.2), up to 32 KiB: at 64 KiB
// that kernel's four slots per thread in 1024 threads lose to the aligned one (bf16 2048 x 32760:
// 60.6 against 53.3 us).  Returns -3, -1 or 0 (the rule does not apply).
constexpr int64_t kLineRuleMinBytes = 1023;
constexpr int64_t kLineRulePackedBytes = 1792;
constexpr int64_t kLineRuleMaxBytes = 32 * 1024;

int off_line_kernel(int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  if (row_bytes % rms::kLineBytes == 0 || row_bytes <= kLineRuleMinBytes || row_bytes > kLineRuleMaxBytes) return 0;
  if (row_bytes <= kLineRulePackedBytes && packed_can(N)) return -3;
  // (rows of whole half lines keep the aligned kernels beyond that: what costs those most is their
  // stores' write-through policy, which works on 64-byte pieces, and without that cost they are 10
  // to 15 % ahead of the element-addressed kernel: fp16 32768 x 4128 94.1 against 108.4 us)
  if (row_bytes % 64 != 0 && pick_threads_unaligned(rms::host::whole_pieces(N, elem_bytes(dtype))) != 0) return -1;
  return 0;
}

// The caller has checked queue_threads and that the plan is valid.
template <int DT>
int dispatch_queue(const Args& a) {
  using rms::host::with_shape;
  constexpr int kMaxChunks = (DT == rms::kFp32 ? kResidentAutoElems32 : kQueueWideElems) / rms::Storage<DT>::kVec;
  const int chunks = (a.nvec + a.plan.threads - 1) / a.plan.threads;
  auto row = [&](auto g, auto c) { launch_queue<DT, decltype(c)::value, decltype(g)::value>(a); };
  const bool launched = with_shape<256, kMaxChunks>(a.plan.threads, chunks, row) ||
                        with_shape<512, kMaxChunks>(a.plan.threads, chunks, row);
  return launched ? LAYERNORM_OK : LAYERNORM_ERR_UNSUPPORTED;
}

// threads == 0 means the element-wise kernel, -1 the element-addressed row kernel, -2 the
// three-pass streaming kernel, -3 the LDS-staged kernel, -4 the work-queue kernel.
template <int DT>
int run_typed(const Args& a, int threads) {
  int rc = LAYERNORM_OK;
  if (threads == 0) launch_generic<DT>(a);
  else if (threads == -1) rc = dispatch_unaligned<DT>(a);
  else if (threads == -2) launch_stream<DT>(a);
  else if (threads == -3) dispatch_packed<DT>(a);
  else if (threads == -4) rc = dispatch_queue<DT>(a);
  else rc = dispatch<DT>(a, threads);
  if (rc != LAYERNORM_OK) return rc;
  return rms::host::launch_status() == hipSuccess ? LAYERNORM_OK : LAYERNORM_ERR_LAUNCH;
}

// variant: a layernorm_variant, or -1 with `threads` forced by the caller.
int run(const void* x, const void* w, const void* b, void* y, int64_t M, int64_t N, float eps,
        int dtype, void* stream, int variant, int threads) {
  int rc = check_args(x, w, b, y, M, N, eps, dtype);
  if (rc != LAYERNORM_OK) return rc;
  if (variant < -1 || variant > LAYERNORM_VARIANT_QUEUE) return LAYERNORM_ERR_INVALID_ARG;
  if (variant == -1 && max_chunks_for(threads) == 0) return LAYERNORM_ERR_INVALID_ARG;
  if (M == 0) return LAYERNORM_OK;

  const bool vec_ok = rows_vectorisable(x, w, b, y, N, dtype);
  const int64_t nvec = vec_ok ? N * elem_bytes(dtype) / 16 : 0;
  const bool unaligned_fits = pick_threads_unaligned(rms::host::whole_pieces(N, elem_bytes(dtype))) != 0;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  unsigned* counters = nullptr;
  switch (variant) {
    case LAYERNORM_VARIANT_AUTO:
      threads = vec_ok ? (nvec <= kPackedAutoVectors ? -3 : pick_threads(nvec, 8, dtype))
                       : (packed_can(N) && !only_stores_unaligned(x, w, b, N, dtype)) ? -3
                       : unaligned_fits ? -1 : 0;
      if (vec_ok && threads > 0 && threads < 64 && packed_beats_lanes(nvec, threads)) threads = -3;
      if (vec_ok && off_line_kernel(N, dtype) != 0) threads = off_line_kernel(N, dtype);
      if (threads == 0 && N < kStreamMaxN) threads = -2;     // too long for registers
      // The work-queue form of the resident kernel where it pays, if this stream has counters.
      if (threads >= 256 && queue_pays(M, nvec, dtype)) {
        counters = queue_counters_for(hs);
        if (counters != nullptr) threads = -4;
      }
      break;
    case LAYERNORM_VARIANT_QUEUE:
      if (!(vec_ok && queue_threads(M, nvec, dtype) != 0)) return LAYERNORM_ERR_UNSUPPORTED;
      counters = queue_counters_for(hs);
      if (counters == nullptr) return LAYERNORM_ERR_UNSUPPORTED;   // a stream that gets no counters
      threads = -4;
      break;
    case LAYERNORM_VARIANT_PACKED:
      if (!packed_can(N)) return LAYERNORM_ERR_UNSUPPORTED;
      threads = -3;
      break;
    case LAYERNORM_VARIANT_STREAM:
      if (N >= kStreamMaxN) return LAYERNORM_ERR_UNSUPPORTED;
      threads = -2;
      break;
    case LAYERNORM_VARIANT_UNALIGNED:
      if (!unaligned_fits) return LAYERNORM_ERR_UNSUPPORTED;
      threads = -1;
      break;
    case -1:
      if (!(vec_ok && threads_can(threads, nvec))) return LAYERNORM_ERR_UNSUPPORTED;
      break;
    case LAYERNORM_VARIANT_SUBWAVE:
      threads = nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
      if (!(vec_ok && threads_can(threads, nvec))) return LAYERNORM_ERR_UNSUPPORTED;
      break;
    case LAYERNORM_VARIANT_WAVE:
      if (!(vec_ok && threads_can(64, nvec))) return LAYERNORM_ERR_UNSUPPORTED;
      threads = 64;
      break;
    case LAYERNORM_VARIANT_BLOCK:
      threads = vec_ok ? pick_threads(nvec, 256, dtype) : 0;
      if (threads == 0) return LAYERNORM_ERR_UNSUPPORTED;
      break;
    default:
      threads = 0;
      break;
  }

  Args a{x, w, b, y, M, N, (int)nvec, eps, hs, counters, QueuePlan{}};
  if (threads == -4) {
    a.plan = queue_plan(nvec, queue_threads(M, nvec, dtype));
    if (!plan_valid(a.plan)) return LAYERNORM_ERR_UNSUPPORTED;
  }
  switch (dtype) {
    case LAYERNORM_DTYPE_FP32: return run_typed<rms::kFp32>(a, threads);
    case LAYERNORM_DTYPE_FP16: return run_typed<rms::kFp16>(a, threads);
    case LAYERNORM_DTYPE_BF16: return run_typed<rms::kBf16>(a, threads);
    default: return LAYERNORM_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

int layernorm_fwd(const void* x, const void* w, const void* b, void* y, int64_t M, int64_t N,
                  float eps, int dtype, void* stream) {
  return run(x, w, b, y, M, N, eps, dtype, stream, LAYERNORM_VARIANT_AUTO, 0);
}

int layernorm_fwd_variant(const void* x, const void* w, const void* b, void* y, int64_t M,
                          int64_t N, float eps, int dtype, void* stream, int variant) {
  if (variant < LAYERNORM_VARIANT_AUTO) return LAYERNORM_ERR_INVALID_ARG;
  return run(x, w, b, y, M, N, eps, dtype, stream, variant, 0);
}

int layernorm_fwd_tuned(const void* x, const void* w, const void* b, void* y, int64_t M,
                        int64_t N, float eps, int dtype, void* stream, int threads_per_row) {
  return run(x, w, b, y, M, N, eps, dtype, stream, -1, threads_per_row);
}

int layernorm_auto_threads_per_row(int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0) return LAYERNORM_ERR_INVALID_ARG;
  if ((N * b) % 16 != 0) return 0;
  // rows off the 128-byte lines (see off_line_kernel): through LDS, or the element-addressed kernel
  const int off_line = off_line_kernel(N, dtype);
  if (off_line == -3) return 1;
  if (off_line == -1) return pick_threads_unaligned(rms::host::whole_pieces(N, b));
  const int64_t nvec = N * b / 16;
  const int g = pick_threads(nvec, 8, dtype);
  // the aligned rows that the automatic path sends through LDS instead (see run)
  if (nvec <= kPackedAutoVectors || (g > 0 && g < 64 && packed_beats_lanes(nvec, g))) return 1;
  return g;
}

int64_t layernorm_unaligned_walk_grid(const void* x, const void* w, const void* b, const void* y,
                                      int64_t M, int64_t N, int dtype) {
  if (check_args(x, w, b, y, M, N, 0.0f, dtype) != LAYERNORM_OK) return LAYERNORM_ERR_INVALID_ARG;
  if (pick_threads_unaligned(rms::host::whole_pieces(N, elem_bytes(dtype))) == 0) return 0;
  int threads = 0;
  return unaligned_walk_grid(M, N, elem_bytes(dtype), &threads);
}

int layernorm_queue_plan(int64_t M, int64_t N, int dtype, int* threads, int* grid, int* shards,
                         int* block_rows) {
  const int eb = elem_bytes(dtype);
  if (eb == 0 || N <= 0 || M < 0) return LAYERNORM_ERR_INVALID_ARG;
  if ((N * eb) % 16 != 0) return LAYERNORM_ERR_UNSUPPORTED;
  const int64_t nvec = N * eb / 16;
  const int g = queue_threads(M, nvec, dtype);
  if (g == 0) return LAYERNORM_ERR_UNSUPPORTED;
  const QueuePlan p = queue_plan(nvec, g);
  if (threads) *threads = p.threads;
  if (grid) *grid = p.grid;
  if (shards) *shards = p.shards;
  if (block_rows) *block_rows = 1 << p.block_shift;
  return queue_pays(M, nvec, dtype) ? 1 : 0;
}

int64_t layernorm_register_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)kMaxThreads * kBlockMaxChunks * (16 / b) : 0;
}

const char* layernorm_status_string(int status) {
  switch (status) {
    case LAYERNORM_OK: return "ok";
    case LAYERNORM_ERR_INVALID_ARG: return "invalid argument";
    case LAYERNORM_ERR_UNSUPPORTED: return "kernel does not support this shape or alignment";
    case LAYERNORM_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
