// C ABI of the RMSNorm forward library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/rmsnorm.h.
#include "../../include/rmsnorm.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "build_id.h"
#include "dispatch_util.h"
#include "launch_util.h"
#include "queue_slots.h"
#include "rmsnorm_kernels.h"

RMS_DEFINE_BUILD_ID(rmsnorm_build_id);

// Counters of the work-queue kernel for callers that bring no workspace: blocks of
// kQueueSlotWords words, all zero between launches (the kernel leaves them zero).  Blocks
// 0 .. kStreamSlots - 1 are handed to streams by rmsnorm_fwd; the last block belongs to
// rmsnorm_fwd_static.  132 KiB per GPU, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress: the device address of each
// GPU's copy is looked up once per device (queue_scratch below) and only that address is ever
// passed to a kernel.
namespace {
constexpr int kQueueSlotWords = rms::kQueueMaxShards * rms::kQueueStride;   // 4 KiB
using rms::host::kStreamSlots;
constexpr int kStaticSlot = kStreamSlots;
constexpr int kScratchSlots = kStreamSlots + 1;
}  // namespace
static __device__ __align__(256) unsigned scratch[kScratchSlots * kQueueSlotWords];

namespace {

using rms::host::compute_units;
using rms::host::walk_grid;

using rms::u32x4;

// Instantiated (threads per row : chunks per thread) combinations.  A chunk is
// one 16-byte vector per thread.
//   8, 16, 32 : 1..2             several rows per wavefront, rows up to 1 KiB
//   64   : 1..16 (fp32: 1..32)   one wavefront per row, N <= 8192
//   128, 256, 512 : 1..8
//   1024 : 1..16                 N <= 131072 (16-bit) / 65536 (fp32)
constexpr int kWaveMaxChunks16 = 16;
constexpr int kWaveMaxChunks32 = 32;
constexpr int kMidMaxChunks = 8;
constexpr int kBlockMaxChunks = 16;
constexpr int kBlockMaxThreads = 1024;
constexpr int kSmallRowVectors = 256;  // rows up to this many vectors: one wavefront per row
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

constexpr int kSubwaveMaxChunks = 2;

int max_chunks_for(int threads, int dtype) {
  switch (threads) {
    case 8: case 16: case 32: return kSubwaveMaxChunks;
    case 64: return wave_max_chunks(dtype);
    case 128: case 256: case 512: return kMidMaxChunks;
    case 1024: return kBlockMaxChunks;
    default: return 0;
  }
}

bool threads_can(int threads, int64_t nvec, int dtype) {
  const int mc = max_chunks_for(threads, dtype);
  return mc > 0 && nvec >= 1 && (nvec + threads - 1) / threads <= mc;
}

bool wave_can(int64_t nvec, int dtype) { return threads_can(64, nvec, dtype); }

// Threads per row for the automatic path, from timing sweeps on MI355X over
// N = 128 .. 131072 in all three dtypes, each timed in a sustained run (the
// first milliseconds after idle run in a clock transient): rows of up to 256
// vectors (4 KiB) run fastest with one wavefront per row; up to 704 vectors with
// 256 threads; up to 2048 with 512 (at 1024 vectors, the headline row, two
// chunks per thread beat four by 2 %); longer rows with 1024.  Within those
// bands the neighbouring choices are within about 2 % of each other, with one
// exception: a row of exactly 256 or 512 vectors (N = 2048 and 4096 in the
// 16-bit types) runs 2 to 3 % faster with one vector per thread, the whole row
// in one predicate-free load per wavefront, than with fewer threads.
// min_threads > 64 restricts the choice to the workgroup-per-row kernels.
// Returns 0 if the row does not fit in registers at all.
constexpr int64_t kMax256Vectors = 704;
constexpr int64_t kMax512Vectors = 2048;

int pick_threads(int64_t nvec, int min_threads, int dtype) {
  if (min_threads <= 8) {
    for (int l = 8; l <= 32; l *= 2)
      if (nvec <= l) return l;
    if (nvec <= 40) return 32;   // two chunks in 32 lanes: 4 % faster than 64 lanes, 3/8 of them idle
  }
  if ((nvec == 256 && min_threads <= 256) || (nvec == 512 && min_threads <= 512)) return (int)nvec;
  if (min_threads <= 64 && nvec <= kSmallRowVectors && threads_can(64, nvec, dtype)) return 64;
  if (nvec <= kMax256Vectors && min_threads <= 256 && threads_can(256, nvec, dtype)) return 256;
  if (nvec <= kMax512Vectors && min_threads <= 512 && threads_can(512, nvec, dtype)) return 512;
  return threads_can(kBlockMaxThreads, nvec, dtype) ? kBlockMaxThreads : 0;
}

// Threads per row for a batch of M rows.  A compute unit holds 2048 threads, so a grid of one
// workgroup of g threads per row runs in rounds of 2048 / g workgroups per compute unit, and
// the first rounds do not overlap well: every workgroup of a round loads, then every one
// stores.  A batch of one to three rounds at the usual thread count that fits into a single
// round of narrower workgroups is faster that way (bf16, one workgroup per row, in
// microseconds: 1536 x 8192 with 512 threads 10.0, with 256 8.3; 2048 x 8192 13.2 against 12.6;
// 2048 x 4096 7.3 against 5.8; 3072 x 4096 10.1 against 8.3 with 128; 4096 x 2048 with 256
// threads 6.7, with 128 5.9); from four rounds on the usual count wins again.  Narrower
// workgroups are only taken down to 128 threads and up to 4 chunks per thread, which keeps
// them at full occupancy.
constexpr int kThreadsPerCu = 2048;
constexpr int kBatchMaxRounds = 3;
constexpr int kBatchMaxChunks = 4;

int pick_threads_batch(int64_t nvec, int64_t M, int dtype) {
  const int g0 = pick_threads(nvec, 128, dtype);
  if (g0 < 256) return g0;
  const int64_t cus = compute_units();
  const int64_t round0 = cus * (kThreadsPerCu / g0);
  if (M <= round0 || M > kBatchMaxRounds * round0) return g0;
  for (int g = g0 / 2; g >= 128; g /= 2)
    if (M <= cus * (kThreadsPerCu / g) && (nvec + g - 1) / g <= kBatchMaxChunks && threads_can(g, nvec, dtype))
      return g;
  return g0;
}

// Threads per row for the element-addressed kernel, from the 16-byte slots its workgroup must
// cover (fewer instantiations: 64 threads up to 4 chunks, 256 and 512 up to 8, 1024 up to 16);
// 0 if the row does not fit in registers.
int pick_threads_unaligned(int64_t slots) {
  if (slots <= kSmallRowVectors) return 64;
  if (slots <= 256 * kMidMaxChunks) return 256;
  if (slots <= 512 * kMidMaxChunks) return 512;
  if (slots <= (int64_t)kBlockMaxThreads * kBlockMaxChunks) return 1024;
  return 0;
}

// 16-byte slots that the element-addressed kernel's workgroup must hold: the whole 16-byte
// pieces of a row, at most floor(row bytes / 16) wherever the row starts (the slots are counted
// from the 128-byte line in which the row starts, and those past the last chunk wrap onto the
// lanes that the row's offset from the line leaves idle in the first).
int64_t slots_per_row(int64_t N, int dtype) { return rms::host::whole_pieces(N, elem_bytes(dtype)); }

constexpr int64_t kStreamMaxN = (int64_t)1 << 31;   // the streaming kernel counts groups in an int

// The LDS-staged kernel takes rows of at most 16 elements per lane of a 64-lane group at any
// alignment (its tile mirrors the offset of x from a 16-byte boundary, so aligned vectors of x
// are aligned vectors of LDS, and of y when y sits at the same offset); the automatic path uses
// it for such rows when they are not 16-byte aligned, and for aligned rows of at most four
// vectors.
constexpr int64_t kPackedMaxN = 64 * rms::kPackElems;
// Workgroups at most: beyond that a workgroup takes several tiles and pays for its weight slice
// once (64 MiB of 77-, 197- and 257-element bf16 rows: 25.5 us at 1024, 24.2 to 24.8 at 8192,
// 24.5 to 26.6 with a workgroup per tile).
constexpr int64_t kPackedMaxGrid = 8192;
constexpr int64_t kPackedAutoVectors = 4;

// Short aligned rows that would leave more than three lanes in ten of their lane group idle (5
// vectors on 8 lanes, 9 or 10 on 16: N = 40, 72, 80 in the 16-bit types) are 6 to 15 % faster
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
bool only_stores_unaligned(const void* x, const void* w, int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  return aligned16(x) && aligned16(w) && row_bytes % 16 == 0 && row_bytes >= 1024;
}

// Rows that are a multiple of 16 bytes but not of the 128-byte line: every second or every
// eighth row starts off a line, the 1 KiB that a wavefront of the aligned kernels loads or
// stores then touches nine lines instead of eight, and the last line of a row is shared with the
// next row, which another XCD reads.  Measured, such rows cost the aligned kernels 15 to 40 %
// (fp16 65536 x 2040: 113 us where 65536 x 2048 takes 80).  The kernels written for rows that are
// not 16-byte aligned do not care: the element-addressed kernel lays its 16-byte slots out from
// the line a row starts in, the LDS-staged kernel moves whole tiles.  So beyond 256 bytes (below,
// packed_beats_lanes has the measured choice) such rows go through LDS up to 2 KiB (64 MiB of
// fp16 rows of 136 to 1000 elements: 23.3 to 24.4 us against 25.7 to 31.4) and to the
// element-addressed kernel beyond (fp16 65536 x 2040 113.0 -> 93.7 us, 32768 x 4088
// 107.0 -> 87.9, 16384 x 8184 105.2 -> 85.9, fp32 16384 x 4092 105.2 -> 85.4, 4096 x 8184
// 27.5 -> 23.3, bf16 2048 x 50296 87.7 -> 71.2, fp16 1024 x 65528 60.5 -> 48.2), at every length
// that kernel takes.  0: the rule does not apply.
constexpr int64_t kLineRuleMinBytes = 256;
constexpr int64_t kLineRulePackedBytes = 2048;

int off_line_variant(int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  if (row_bytes % rms::kLineBytes == 0 || row_bytes <= kLineRuleMinBytes) return 0;
  if (row_bytes <= kLineRulePackedBytes && packed_can(N)) return RMSNORM_VARIANT_PACKED;
  // (rows of whole half lines keep the aligned kernels beyond that: what costs those most is their
  // stores' write-through policy, which works on 64-byte pieces; fp16 65536 x 2080 92.4 us against
  // 96.7 in the element-addressed kernel, 32768 x 4128 92.5 against 89.2)
  if (row_bytes % 64 != 0 && pick_threads_unaligned(slots_per_row(N, dtype))) return RMSNORM_VARIANT_UNALIGNED;
  return 0;
}

int choose(const void* x, const void* w, const void* y, int64_t N, int dtype) {
  if (!rows_vectorisable(x, w, y, N, dtype)) {
    if (packed_can(N) && !only_stores_unaligned(x, w, N, dtype)) return RMSNORM_VARIANT_PACKED;
    if (pick_threads_unaligned(slots_per_row(N, dtype))) return RMSNORM_VARIANT_UNALIGNED;
    return N < kStreamMaxN ? RMSNORM_VARIANT_STREAM : RMSNORM_VARIANT_GENERIC;
  }
  if (const int v = off_line_variant(N, dtype)) return v;
  // Rows of whole lines written to a y that starts off the 64-byte pieces of the lines: it is the
  // stores that pay for straddling (x off a line alone costs nothing measurable, nor does a y 64
  // bytes off; y 16 bytes off: bf16 16384 x 8192 82.1 -> 94.6 us, 8192 x 4096 22.6 -> 26.7), and the
  // element-addressed kernel, which cuts the row at the lines of x and stores element-aligned, is
  // ahead from 2 KiB rows on (85.9 and 23.5 us; 65536 x 2048: 98.4 -> 93.9; rows of 1 KiB: 71.0
  // against 79.5 the other way).
  if ((reinterpret_cast<uintptr_t>(y) & 63u) != 0 && N * elem_bytes(dtype) >= 2048 &&
      pick_threads_unaligned(slots_per_row(N, dtype)))
    return RMSNORM_VARIANT_UNALIGNED;
  // Rows of at most 64 bytes leave most of the narrowest lane group idle (one to four of its
  // eight lanes hold a vector): the LDS-staged kernel is 1.2 to 2.9 times faster there.
  if (vectors_per_row(N, dtype) <= kPackedAutoVectors) return RMSNORM_VARIANT_PACKED;
  const int g = pick_threads(vectors_per_row(N, dtype), 8, dtype);
  if (g == 0) return N < kStreamMaxN ? RMSNORM_VARIANT_STREAM : RMSNORM_VARIANT_GENERIC;
  if (g < 64) return packed_beats_lanes(vectors_per_row(N, dtype), g) ? RMSNORM_VARIANT_PACKED
                                                                      : RMSNORM_VARIANT_SUBWAVE;
  return g == 64 ? RMSNORM_VARIANT_WAVE : RMSNORM_VARIANT_BLOCK;
}


// ---------------------------------------------------------------------------
// The work-queue kernel: when it runs, with what grid, and where its counters live.
// ---------------------------------------------------------------------------
constexpr int kQueueThreads = 512;
constexpr int kQueueMaxChunks = 8;
constexpr int64_t kQueueMaxRows = (int64_t)1 << 30;          // tickets are 32-bit

struct QueuePlan {
  int grid;          // resident workgroups, a multiple of `shards`
  int shards;        // 1 .. kQueueMaxShards
  int block_shift;   // rows are handed to the shards in blocks of 1 << block_shift
  bool prefetch;     // next row requested before the stores of the current one
};

// Rows the kernel can take at all: 16-byte aligned rows of 513 .. 4096 vectors (2 to 8 chunks in
// 512 threads), fewer than 2^30 of them.
bool queue_can(int64_t M, int64_t nvec) {
  return nvec > kQueueThreads && nvec <= (int64_t)kQueueThreads * kQueueMaxChunks && M >= 1 && M < kQueueMaxRows;
}

// Tuned on MI355X (bf16, sustained runs over rotating buffers, 256 MiB of x per launch; one
// workgroup per row, its rows in XCD blocks of eight, in brackets):
//   rows of 16 KiB: two workgroups per compute unit, 16 shards, blocks of 8 rows (128 KiB), no
//     prefetch: 81.8 us (82.5; 84.7 with rows one by one); grids of 1.75 and 2.25 per compute
//     unit are 2 to 4 us slower, blocks of 4 or 16 rows 1 to 1.5 us, 8 shards 2 us;
//   rows of 20 and 24 KiB: the same with blocks of 4 rows: 85.1 (86.5) and 84.4 (87.2);
//   rows of 32 KiB: two per compute unit, 8 shards, blocks of 4 rows: 85.1 (87.0);
//   rows of 40 to 64 KiB: one workgroup per compute unit, which then has to request its next
//     row before it stores the current one, 8 shards, blocks of 2 rows: 85.8 (85.1), 85.9
//     (86.8), 85.9 (88.1).
// Rows of 10 to 14 KiB are level or behind at that size; from x of 320 MiB on they are level
// (12 KiB) or gain 1.5 to 2.5 % (10 KiB: 107.6 -> 106.1 us at 320 MiB, 173.5 -> 169.3 at 512 MiB;
// 14 KiB: 105.1 -> 103.4 and 168.3 -> 164.9).  Rows of 8 KiB and less
// would be one chunk per thread of the 512, and lose 4 to 20 % to one workgroup per row.
QueuePlan queue_plan(int64_t row_bytes) {
  const int cus = compute_units();
  QueuePlan p;
  const bool two_per_cu = row_bytes <= 32 * 1024;
  p.shards = row_bytes <= 24 * 1024 ? 16 : 8;
  p.prefetch = !two_per_cu;
  p.grid = (two_per_cu ? 2 * cus : cus) / p.shards * p.shards;
  if (p.grid < p.shards) p.grid = p.shards;
  int shift = 0;
  while (((int64_t)2 << shift) * row_bytes <= 128 * 1024) ++shift;   // largest block of at most 128 KiB
  p.block_shift = shift;
  return p;
}

// Whether the automatic path takes the work-queue kernel: it wins once the launch moves a few
// hundred megabytes (x of 128 MiB: 0.5 to 3 % ahead of one workgroup per row at rows of 16 to
// 32 KiB, 1 to 2 % behind at 40 and 48 KiB; x of 256 MiB: 1 to 3 % ahead, level at 40 KiB; x of
// 512 MiB: 2 to 4 % ahead).
constexpr int64_t kQueueMinRowBytes = 16 * 1024;
constexpr int64_t kQueueMinBytes = (int64_t)96 << 20;        // rows up to 32 KiB
constexpr int64_t kQueueMinBytesLong = (int64_t)192 << 20;   // longer rows
constexpr int64_t kQueueMinBytesShort = (int64_t)320 << 20;  // rows below 16 KiB

bool queue_pays(int64_t M, int64_t nvec) {
  const int64_t row_bytes = nvec * 16;
  if (!queue_can(M, nvec)) return false;
  if (row_bytes % 64 != 0) return false;   // (the element-addressed kernel takes those: off_line_variant)
  if (row_bytes < kQueueMinRowBytes) return M * row_bytes >= kQueueMinBytesShort;
  return M * row_bytes >= (row_bytes <= 32 * 1024 ? kQueueMinBytes : kQueueMinBytesLong);
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device
// current; nullptr if the lookup fails.
unsigned* queue_scratch() {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static unsigned* base[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (base[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    base[dev] = static_cast<unsigned*>(p);
  }
  return base[dev];
}

// The counter block of `stream` on the current device for rmsnorm_fwd, nullptr if the call
// has to do without the work-queue kernel (see queue_slots.h for the streams that get none).
unsigned* queue_counters_for(hipStream_t stream) {
  static rms::host::StreamSlots slots;
  unsigned* base = queue_scratch();
  if (base == nullptr) return nullptr;
  const int k = slots.block_of(stream);
  return k < 0 ? nullptr : base + (size_t)k * kQueueSlotWords;
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
  unsigned* counters;   // the work-queue kernel's counters for this call (nullptr: none)
  QueuePlan plan;
};

template <int DT, int CHUNKS, int G>
void launch_row(const Args& a) {
  const rms::host::FlatRows rows = rms::host::flat_rows(a.M, kMaxGrid, G, (int64_t)a.nvec * 16);
  const int64_t blocks = rows.blocks;
  // Rows that fill their chunks exactly, one row per workgroup: the instance without
  // predicates and loop bookkeeping (256 and 512 threads, where the headline shapes fall).
  if constexpr ((G == 256 || G == 512) && CHUNKS <= 8) {
    if (a.nvec == CHUNKS * G && a.M <= kMaxGrid) {
      RMS_LAUNCH((rms::rmsnorm_row_kernel<DT, CHUNKS, G, true, true>),
                         dim3((unsigned)blocks), dim3(G), 0, a.stream,
                         (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
                         1.0f / (float)a.N, a.eps, rows.xcd_blocks);
      return;
    }
  }
  RMS_LAUNCH((rms::rmsnorm_row_kernel<DT, CHUNKS, G, true>),
                     dim3((unsigned)blocks), dim3(G), 0, a.stream,
                     (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
                     1.0f / (float)a.N, a.eps, rows.xcd_blocks);
}

template <int DT, int CHUNKS, int L>
void launch_subwave(const Args& a) {
  constexpr int kRows = rms::kWave / L;
  int64_t blocks = (a.M + kRows - 1) / kRows;
  if (blocks > ((int64_t)1 << 24)) blocks = (int64_t)1 << 24;
  RMS_LAUNCH((rms::rmsnorm_subwave_kernel<DT, CHUNKS, L, true>),
                     dim3((unsigned)blocks), dim3(rms::kWave), 0, a.stream,
                     (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
                     1.0f / (float)a.N, a.eps);
}

// The walking form of the element-addressed kernel: where its grid is best, in bytes of rows in
// flight per compute unit (each resident workgroup has one row in flight; swept over
// N = 1025 .. 40961: 12 single-wavefront workgroups per compute unit at N = 1025, 3 or 4 of
// 256 threads at N = 4097, 2 at N = 8191, 1 from N = 12289 on).
constexpr int64_t kWalkBytesPerCu = 26 * 1024;
constexpr int kWalkMaxChunks = 8;   // what fits in registers next to the packed weight

// The grid of the walking form for this call, 0 for one workgroup per row.  Its rows are cut at
// the 128-byte lines of x; where y sits at another offset from a line its stores straddle the
// lines.  walk_grid returns multiples of 64 workgroups only, which is what keeps every row of a
// workgroup at the same offset from a line.
int64_t unaligned_walk_grid(int64_t M, int64_t N, int dtype) {
  const int64_t slots = slots_per_row(N, dtype);
  const int threads = pick_threads_unaligned(slots);
  if (threads == 0) return 0;
  // (1024 threads are capped at 128 registers each: 7 groups next to their weight)
  if ((slots + threads - 1) / threads > (threads == kBlockMaxThreads ? kWalkMaxChunks - 1 : kWalkMaxChunks)) return 0;
  return walk_grid(M, N * elem_bytes(dtype), threads, kWalkBytesPerCu);
}

// walk > 0: the walking form with that many resident workgroups.
template <int DT, int CHUNKS, int G>
void launch_row_unaligned(const Args& a, int64_t walk) {
  if constexpr (CHUNKS <= (G == kBlockMaxThreads ? kWalkMaxChunks - 1 : kWalkMaxChunks)) {
    if (walk > 0) {
      RMS_LAUNCH((rms::rmsnorm_row_unaligned_kernel<DT, CHUNKS, G, true, true>),
                         dim3((unsigned)walk), dim3(G), 0, a.stream,
                         a.x, a.w, a.y, a.M, (int)a.N, 1.0f / (float)a.N, a.eps);
      return;
    }
  }
  const int64_t blocks = rms::host::flat_grid(a.M, kMaxGrid);
  RMS_LAUNCH((rms::rmsnorm_row_unaligned_kernel<DT, CHUNKS, G, true, false>),
                     dim3((unsigned)blocks), dim3(G), 0, a.stream,
                     a.x, a.w, a.y, a.M, (int)a.N, 1.0f / (float)a.N, a.eps);
}

// The two-pass streaming kernel: about one batch of four groups per thread, whole wavefronts,
// at most 1024 threads (what every row long enough to need this kernel gets).
template <int DT>
void launch_stream(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  const int64_t nfull = a.N / rms::Storage<DT>::kVec;
  int64_t threads = (nfull / rms::kStreamBatch + rms::kWave - 1) / rms::kWave * rms::kWave;
  threads = threads < rms::kWave ? rms::kWave : threads > kBlockMaxThreads ? kBlockMaxThreads : threads;
  RMS_LAUNCH((rms::rmsnorm_stream_kernel<DT>), dim3((unsigned)blocks), dim3((unsigned)threads),
                     0, a.stream, a.x, a.w, a.y, a.M, a.N, 1.0f / (float)a.N, a.eps);
}

template <int DT>
void launch_generic(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  RMS_LAUNCH((rms::rmsnorm_generic_kernel<DT, kGenericThreads>),
                     dim3((unsigned)blocks), dim3(kGenericThreads), 0, a.stream,
                     a.x, a.w, a.y, a.M, a.N, 1.0f / (float)a.N, a.eps);
}

// Launches the row kernel with `threads` threads per row.  The caller has
// checked threads_can(threads, nvec, DT).
template <int DT>
int dispatch_row(const Args& a, int threads) {
  using rms::host::with_shape;
  const int chunks = (a.nvec + threads - 1) / threads;
  auto subwave = [&](auto l, auto c) { launch_subwave<DT, decltype(c)::value, decltype(l)::value>(a); };
  auto row = [&](auto g, auto c) { launch_row<DT, decltype(c)::value, decltype(g)::value>(a); };
  constexpr int kWaveChunks = DT == rms::kFp32 ? kWaveMaxChunks32 : kWaveMaxChunks16;
  const bool launched =
      with_shape<8, kSubwaveMaxChunks>(threads, chunks, subwave) || with_shape<16, kSubwaveMaxChunks>(threads, chunks, subwave) ||
      with_shape<32, kSubwaveMaxChunks>(threads, chunks, subwave) || with_shape<64, kWaveChunks>(threads, chunks, row) ||
      with_shape<128, kMidMaxChunks>(threads, chunks, row) || with_shape<256, kMidMaxChunks>(threads, chunks, row) ||
      with_shape<512, kMidMaxChunks>(threads, chunks, row) || with_shape<kBlockMaxThreads, kBlockMaxChunks>(threads, chunks, row);
  return launched ? RMSNORM_OK : RMSNORM_ERR_UNSUPPORTED;
}

// Launches the LDS-staged kernel: the narrowest lane group that holds the row, as many whole
// rows per step as fit the tile.  The caller has checked N <= kPackedMaxN.
template <int DT, int L, int E>
void launch_packed(const Args& a) {
  const int n = (int)a.N;
  const rms::host::PackedShape shape = rms::host::packed_shape(a.M, (int64_t)n * rms::Storage<DT>::kBytes, L,
                                                               rms::kPackThreads, rms::kPackTileBytes,
                                                               rms::host::kPackedTargetReadWrite, kPackedMaxGrid);
  const int tile_rows = shape.tile_rows;
  const int64_t blocks = shape.blocks;
  RMS_LAUNCH((rms::rmsnorm_packed_kernel<DT, L, E, true>), dim3((unsigned)blocks),
                     dim3(rms::kPackThreads), 0, a.stream, a.x, a.w, a.y, a.M, n, tile_rows,
                     1.0f / (float)a.N, a.eps);
}

// Lanes per row and elements per lane: see with_packed_shape.
template <int DT>
void dispatch_packed(const Args& a) {
  rms::host::with_packed_shape(a.N, rms::Storage<DT>::kBytes, 64, [&](auto lanes, auto elems) {
    launch_packed<DT, decltype(lanes)::value, decltype(elems)::value>(a);
  });
}

// Launches the element-addressed row kernel.  The caller has checked that the row fits.
template <int DT>
int dispatch_row_unaligned(const Args& a) {
  using rms::host::with_shape;
  const int dtype = DT == rms::kFp32 ? RMSNORM_DTYPE_FP32 : RMSNORM_DTYPE_FP16;
  const int slots = (int)slots_per_row(a.N, dtype);
  const int threads = pick_threads_unaligned(slots);
  const int64_t walk = unaligned_walk_grid(a.M, a.N, dtype);
  int chunks = (slots + threads - 1) / threads;
  if (chunks < 1) chunks = 1;
  auto row = [&](auto g, auto c) { launch_row_unaligned<DT, decltype(c)::value, decltype(g)::value>(a, walk); };
  const bool launched = with_shape<64, 4>(threads, chunks, row) || with_shape<256, kMidMaxChunks>(threads, chunks, row) ||
                        with_shape<512, kMidMaxChunks>(threads, chunks, row) ||
                        with_shape<kBlockMaxThreads, kBlockMaxChunks>(threads, chunks, row);
  return launched ? RMSNORM_OK : RMSNORM_ERR_UNSUPPORTED;
}

template <int DT, int CHUNKS>
void launch_queue(const Args& a) {
  if (a.plan.prefetch)
    RMS_LAUNCH((rms::rmsnorm_queue_kernel<DT, CHUNKS, kQueueThreads, true>), dim3((unsigned)a.plan.grid),
               dim3(kQueueThreads), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
               1.0f / (float)a.N, a.eps, a.counters, a.plan.shards, a.plan.block_shift);
  else
    RMS_LAUNCH((rms::rmsnorm_queue_kernel<DT, CHUNKS, kQueueThreads, false>), dim3((unsigned)a.plan.grid),
               dim3(kQueueThreads), 0, a.stream, (const u32x4*)a.x, (const u32x4*)a.w, (u32x4*)a.y, a.M, a.nvec,
               1.0f / (float)a.N, a.eps, a.counters, a.plan.shards, a.plan.block_shift);
}

// The caller has checked queue_can and that the plan is valid.
template <int DT>
int dispatch_queue(const Args& a) {
  const int chunks = (a.nvec + kQueueThreads - 1) / kQueueThreads;
  const bool launched = rms::host::with_chunks<2, 8>(chunks, [&](auto c) { launch_queue<DT, decltype(c)::value>(a); });
  return launched ? RMSNORM_OK : RMSNORM_ERR_UNSUPPORTED;
}

// threads == 0 means the element-wise kernel, -1 the element-addressed row kernel, -2 the
// two-pass streaming kernel, -3 the LDS-staged kernel, -4 the work-queue kernel.
template <int DT>
int run_typed(const Args& a, int threads) {
  int rc = RMSNORM_OK;
  rms::host::launch_status() = hipSuccess;
  if (threads == 0) launch_generic<DT>(a);
  else if (threads == -1) rc = dispatch_row_unaligned<DT>(a);
  else if (threads == -2) launch_stream<DT>(a);
  else if (threads == -3) dispatch_packed<DT>(a);
  else if (threads == -4) rc = dispatch_queue<DT>(a);
  else rc = dispatch_row<DT>(a, threads);
  if (rc != RMSNORM_OK) return rc;
  return rms::host::launch_status() == hipSuccess ? RMSNORM_OK : RMSNORM_ERR_LAUNCH;
}

// Whether a plan is one the kernel can run: a grid that is a whole number of shards.
bool plan_valid(const QueuePlan& p) {
  return p.shards >= 1 && p.shards <= rms::kQueueMaxShards && p.grid >= p.shards && p.grid % p.shards == 0 &&
         p.grid <= (1 << 16) && p.block_shift >= 0 && p.block_shift <= 16;
}

// variant: an rmsnorm_variant, or -1 with `threads` forced by the caller.
// counters: the work-queue kernel's counters if the caller brings them; nullptr means the block
// of `stream` in the library's own array (which some streams do not get, see queue_counters_for).
// forced_plan: nullptr for the tuned plan.
int run(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps, int dtype,
        void* stream, int variant, int threads, unsigned* counters = nullptr,
        const QueuePlan* forced_plan = nullptr) {
  int rc = check_args(x, w, y, M, N, eps, dtype);
  if (rc != RMSNORM_OK) return rc;
  if (variant < -1 || variant > RMSNORM_VARIANT_QUEUE) return RMSNORM_ERR_INVALID_ARG;
  if (variant == -1 && max_chunks_for(threads, dtype) == 0) return RMSNORM_ERR_INVALID_ARG;
  if (forced_plan && !plan_valid(*forced_plan)) return RMSNORM_ERR_INVALID_ARG;
  if (M == 0) return RMSNORM_OK;

  const bool vec_ok = rows_vectorisable(x, w, y, N, dtype);
  const int64_t nvec = vec_ok ? vectors_per_row(N, dtype) : 0;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool automatic = variant == RMSNORM_VARIANT_AUTO;
  if (automatic) {
    variant = choose(x, w, y, N, dtype);
    // The work-queue kernel where it pays, if this call has counters to run it on.
    if (variant == RMSNORM_VARIANT_BLOCK && queue_pays(M, nvec)) {
      if (counters == nullptr) counters = queue_counters_for(hs);
      if (counters != nullptr) variant = RMSNORM_VARIANT_QUEUE;
    }
  }
  switch (variant) {
    case -1:
      if (!(vec_ok && threads_can(threads, nvec, dtype))) return RMSNORM_ERR_UNSUPPORTED;
      break;
    case RMSNORM_VARIANT_WAVE:
      if (!(vec_ok && wave_can(nvec, dtype))) return RMSNORM_ERR_UNSUPPORTED;
      threads = 64;
      break;
    case RMSNORM_VARIANT_SUBWAVE:
      if (!vec_ok) return RMSNORM_ERR_UNSUPPORTED;
      threads = nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
      if (!threads_can(threads, nvec, dtype)) return RMSNORM_ERR_UNSUPPORTED;
      break;
    case RMSNORM_VARIANT_BLOCK:
      threads = !vec_ok ? 0 : automatic ? pick_threads_batch(nvec, M, dtype) : pick_threads(nvec, 128, dtype);
      if (threads == 0) return RMSNORM_ERR_UNSUPPORTED;
      break;
    case RMSNORM_VARIANT_UNALIGNED:
      if (pick_threads_unaligned(slots_per_row(N, dtype)) == 0) return RMSNORM_ERR_UNSUPPORTED;
      threads = -1;
      break;
    case RMSNORM_VARIANT_STREAM:
      if (N >= kStreamMaxN) return RMSNORM_ERR_UNSUPPORTED;
      threads = -2;
      break;
    case RMSNORM_VARIANT_PACKED:
      if (!packed_can(N)) return RMSNORM_ERR_UNSUPPORTED;
      threads = -3;
      break;
    case RMSNORM_VARIANT_QUEUE:
      if (!(vec_ok && queue_can(M, nvec))) return RMSNORM_ERR_UNSUPPORTED;
      if (counters == nullptr) counters = queue_counters_for(hs);
      if (counters == nullptr) return RMSNORM_ERR_UNSUPPORTED;   // a stream that gets no counters
      threads = -4;
      break;
    default:
      threads = 0;
      break;
  }

  Args a{x, w, y, M, N, (int)nvec, eps, hs, counters, QueuePlan{}};
  if (threads == -4) a.plan = forced_plan ? *forced_plan : queue_plan(nvec * 16);
  switch (dtype) {
    case RMSNORM_DTYPE_FP32: return run_typed<rms::kFp32>(a, threads);
    case RMSNORM_DTYPE_FP16: return run_typed<rms::kFp16>(a, threads);
    case RMSNORM_DTYPE_BF16: return run_typed<rms::kBf16>(a, threads);
    default: return RMSNORM_ERR_INVALID_ARG;
  }
}

// A caller's workspace as the kernel's counters; nullptr if it does not qualify.
unsigned* workspace_counters(void* workspace, int64_t workspace_bytes) {
  if (workspace == nullptr || workspace_bytes < (int64_t)kQueueSlotWords * 4) return nullptr;
  if (reinterpret_cast<uintptr_t>(workspace) & 3u) return nullptr;
  return static_cast<unsigned*>(workspace);
}

}  // namespace

extern "C" {

int rmsnorm_fwd(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                int dtype, void* stream) {
  return run(x, w, y, M, N, eps, dtype, stream, RMSNORM_VARIANT_AUTO, 0);
}

int rmsnorm_fwd_variant(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                        int dtype, void* stream, int variant) {
  if (variant < RMSNORM_VARIANT_AUTO) return RMSNORM_ERR_INVALID_ARG;
  return run(x, w, y, M, N, eps, dtype, stream, variant, 0);
}

int rmsnorm_fwd_tuned(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                      int dtype, void* stream, int threads_per_row) {
  return run(x, w, y, M, N, eps, dtype, stream, -1, threads_per_row);
}

int64_t rmsnorm_workspace_bytes(void) { return (int64_t)kQueueSlotWords * 4; }

int rmsnorm_fwd_workspace(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                          int dtype, void* stream, void* workspace, int64_t workspace_bytes) {
  unsigned* counters = workspace_counters(workspace, workspace_bytes);
  if (counters == nullptr) return RMSNORM_ERR_INVALID_ARG;
  return run(x, w, y, M, N, eps, dtype, stream, RMSNORM_VARIANT_QUEUE, 0, counters);
}

int rmsnorm_fwd_static(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                       int dtype, void* stream) {
  int rc = check_args(x, w, y, M, N, eps, dtype);
  if (rc != RMSNORM_OK) return rc;
  // beyond what the fixed scratch and its 32-bit tickets cover
  if (M >= kQueueMaxRows || N * elem_bytes(dtype) > (int64_t)kQueueThreads * kQueueMaxChunks * 16)
    return RMSNORM_ERR_TOO_LARGE;
  if (M == 0) return RMSNORM_OK;
  unsigned* base = queue_scratch();
  if (base == nullptr) return RMSNORM_ERR_LAUNCH;
  return run(x, w, y, M, N, eps, dtype, stream, RMSNORM_VARIANT_QUEUE, 0,
             base + (size_t)kStaticSlot * kQueueSlotWords);
}

int rmsnorm_fwd_queue_tuned(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                            int dtype, void* stream, void* workspace, int64_t workspace_bytes,
                            int grid, int shards, int block_rows, int prefetch) {
  unsigned* counters = workspace_counters(workspace, workspace_bytes);
  if (counters == nullptr) return RMSNORM_ERR_INVALID_ARG;
  if (block_rows < 1 || (block_rows & (block_rows - 1)) != 0) return RMSNORM_ERR_INVALID_ARG;
  QueuePlan plan{grid, shards, 0, prefetch != 0};
  while ((1 << plan.block_shift) < block_rows) ++plan.block_shift;
  return run(x, w, y, M, N, eps, dtype, stream, RMSNORM_VARIANT_QUEUE, 0, counters, &plan);
}

int rmsnorm_queue_plan(int64_t M, int64_t N, int dtype, int* grid, int* shards, int* block_rows,
                       int* prefetch) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0 || M < 0) return RMSNORM_ERR_INVALID_ARG;
  if ((N * b) % 16 != 0 || !queue_can(M, vectors_per_row(N, dtype))) return RMSNORM_ERR_UNSUPPORTED;
  const QueuePlan p = queue_plan(N * b);
  if (grid) *grid = p.grid;
  if (shards) *shards = p.shards;
  if (block_rows) *block_rows = 1 << p.block_shift;
  if (prefetch) *prefetch = p.prefetch ? 1 : 0;
  return queue_pays(M, vectors_per_row(N, dtype)) ? 1 : 0;
}

int rmsnorm_auto_threads_for_batch(int64_t M, int64_t N, int dtype) {
  const int g = rmsnorm_auto_threads_per_row(N, dtype);
  if (g < 256 || M < 0) return M < 0 ? RMSNORM_ERR_INVALID_ARG : g;
  if (off_line_variant(N, dtype) != 0) return g;      // the element-addressed kernel: no batch rule
  return pick_threads_batch(vectors_per_row(N, dtype), M, dtype);
}

int rmsnorm_auto_threads_per_row(int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0) return RMSNORM_ERR_INVALID_ARG;
  if ((N * b) % 16 != 0) return 0;
  // rows off the 128-byte lines (see off_line_variant): through LDS, or the element-addressed kernel
  const int off_line = off_line_variant(N, dtype);
  if (off_line == RMSNORM_VARIANT_PACKED) return 1;
  if (off_line == RMSNORM_VARIANT_UNALIGNED) return pick_threads_unaligned(slots_per_row(N, dtype));
  const int64_t nvec = vectors_per_row(N, dtype);
  const int g = pick_threads(nvec, 8, dtype);
  // the aligned rows that the automatic path sends through LDS instead (see choose)
  if (nvec <= kPackedAutoVectors || (g > 0 && g < 64 && packed_beats_lanes(nvec, g))) return 1;
  return g;
}

int rmsnorm_select_variant(const void* x, const void* w, const void* y, int64_t M, int64_t N,
                           int dtype) {
  const int rc = check_args(x, w, y, M, N, 0.0f, dtype);
  if (rc != RMSNORM_OK) return rc;
  const int variant = choose(x, w, y, N, dtype);
  if (variant == RMSNORM_VARIANT_BLOCK && queue_pays(M, vectors_per_row(N, dtype))) return RMSNORM_VARIANT_QUEUE;
  return variant;
}

int64_t rmsnorm_wave_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)rms::kWave * wave_max_chunks(dtype) * (16 / b) : 0;
}

int64_t rmsnorm_block_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)kBlockMaxThreads * kBlockMaxChunks * (16 / b) : 0;
}

int64_t rmsnorm_unaligned_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)kBlockMaxThreads * kBlockMaxChunks * (16 / b) + (16 / b - 1) : 0;
}

int64_t rmsnorm_unaligned_walk_grid(const void* x, const void* w, const void* y, int64_t M,
                                    int64_t N, int dtype) {
  if (check_args(x, w, y, M, N, 0.0f, dtype) != RMSNORM_OK) return RMSNORM_ERR_INVALID_ARG;
  if (pick_threads_unaligned(slots_per_row(N, dtype)) == 0) return 0;
  return unaligned_walk_grid(M, N, dtype);
}

const char* rmsnorm_status_string(int status) {
  switch (status) {
    case RMSNORM_OK: return "ok";
    case RMSNORM_ERR_INVALID_ARG: return "invalid argument";
    case RMSNORM_ERR_UNSUPPORTED: return "variant does not support this shape or alignment";
    case RMSNORM_ERR_LAUNCH: return "kernel launch failed";
    case RMSNORM_ERR_TOO_LARGE: return "larger than the fixed scratch of this entry point covers";
    default: return "unknown status";
  }
}

}  // extern "C"
