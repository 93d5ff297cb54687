// C ABI of the row softmax library: argument checks, kernel choice, launch.
// Declarations and the full contract are in include/softmax.h.
#include "../../include/softmax.h"

#include <hip/hip_runtime.h>

#include "build_id.h"
#include "dispatch_util.h"
#include "launch_util.h"
#include "softmax_kernels.h"

RMS_DEFINE_BUILD_ID(softmax_build_id);

namespace {


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
    case SOFTMAX_DTYPE_FP32: return 4;
    case SOFTMAX_DTYPE_FP16: return 2;
    case SOFTMAX_DTYPE_BF16: return 2;
    default: return 0;
  }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_args(const void* x, const void* y, int64_t M, int64_t N, int dtype) {
  if (elem_bytes(dtype) == 0) return SOFTMAX_ERR_INVALID_ARG;
  if (M < 0 || N <= 0) return SOFTMAX_ERR_INVALID_ARG;
  if (M > 0 && (!x || !y)) return SOFTMAX_ERR_INVALID_ARG;
  if (M > INT64_MAX / N) return SOFTMAX_ERR_INVALID_ARG;
  const uintptr_t mask = (uintptr_t)elem_bytes(dtype) - 1;
  if (M > 0 && (((uintptr_t)x | (uintptr_t)y) & mask)) return SOFTMAX_ERR_INVALID_ARG;
  return SOFTMAX_OK;
}

bool rows_vectorisable(const void* x, const void* y, int64_t N, int dtype) {
  return aligned16(x) && aligned16(y) && (N * elem_bytes(dtype)) % 16 == 0;
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

// Threads per row of the automatic path, from sustained timing sweeps on MI355X: lane
// groups for rows up to 48 vectors (a lane takes two chunks where that avoids idle lanes:
// 16 lanes up to 24 vectors, 32 lanes up to 48; 5 to 11 % faster than the next wider
// group), one wavefront up to 256 vectors, then 256, 512 and 1024 threads while a thread
// holds at most 8 chunks; rows of 705 to 1024 vectors (N = 8192 in the 16-bit types) run 3 %
// faster with two chunks in each of 512 threads than with four in 256, and rows beyond 2048
// vectors (a 32000-entry vocabulary) 2 to 3 % faster with 1024 threads.  0: does not fit.
int pick_threads(int64_t nvec, int min_threads) {
  if (min_threads <= 8) {
    if (nvec <= 8) return 8;
    if (nvec <= 24) return 16;
    if (nvec <= 48) return 32;
  }
  if (min_threads <= 64 && nvec <= kSmallRowVectors) return 64;
  if (nvec > 704 && nvec <= 1024 && min_threads <= 512) return 512;
  if (nvec > 2048 && threads_can(kMaxThreads, nvec)) return kMaxThreads;   // 2 to 3 % over 512 threads
  for (int g = 256; g <= kMaxThreads; g *= 2)
    if (g >= min_threads && threads_can(g, nvec)) return g;
  return 0;
}

// Threads per row for the element-addressed kernel over the whole 16-byte pieces of a row
// (whole_pieces; the same bands); 0 if the row does not fit in registers.
int pick_threads_unaligned(int64_t slots) {
  if (slots <= kSmallRowVectors) return 64;
  for (int g = 256; g <= kMaxThreads; g *= 2)
    if (slots <= (int64_t)g * kBlockMaxChunks) return g;
  return 0;
}

struct Args {
  const void* x;
  void* y;
  int64_t M;
  int64_t N;
  int nvec;
  hipStream_t stream;
};

template <int DT, int CHUNKS, int G>
void launch_row(const Args& a) {
  const rms::host::FlatRows rows = rms::host::flat_rows(a.M, kMaxGrid, G, (int64_t)a.nvec * 16);
  RMS_LAUNCH((rms::softmax_row_kernel<DT, CHUNKS, G, true>), dim3((unsigned)rows.blocks),
                     dim3(G), 0, a.stream, (const u32x4*)a.x, (u32x4*)a.y, a.M, a.nvec, rows.xcd_blocks);
}

template <int DT, int CHUNKS, int L>
void launch_subwave(const Args& a) {
  constexpr int kRows = rms::kWaveSize / L;
  int64_t blocks = (a.M + kRows - 1) / kRows;
  if (blocks > ((int64_t)1 << 24)) blocks = (int64_t)1 << 24;
  RMS_LAUNCH((rms::softmax_subwave_kernel<DT, CHUNKS, L, true>), dim3((unsigned)blocks),
                     dim3(rms::kWaveSize), 0, a.stream, (const u32x4*)a.x, (u32x4*)a.y, a.M,
                     a.nvec);
}

template <int DT, int CHUNKS, int G>
void launch_row_unaligned(const Args& a) {
  const int64_t blocks = rms::host::flat_grid(a.M, kMaxGrid);
  RMS_LAUNCH((rms::softmax_row_unaligned_kernel<DT, CHUNKS, G, true>), dim3((unsigned)blocks),
                     dim3(G), 0, a.stream, a.x, a.y, a.M, (int)a.N);
}

// The LDS-staged kernel for short rows that are not 16-byte aligned: the narrowest lane group
// that holds the row (16 elements per lane), whole passes of the workgroup's lane groups per
// tile (about 7 KiB), a workgroup per tile up to 32768 workgroups (with nothing to carry from
// tile to tile, workgroups that walk several tiles were slower at every grid tried: 64 MiB of
// 197-element fp16 rows 25.0 to 26.7 us on 1536 to 4096 workgroups, 24.2 with one per tile).
// Its tile mirrors the offset of x from a 16-byte boundary; where y sits at another, the stores
// are element-aligned.
constexpr int64_t kPackedMaxN = 64 * rms::kPackElems;
constexpr int64_t kPackedMaxGrid = 1 << 15;
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
bool only_stores_unaligned(const void* x, int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  return aligned16(x) && row_bytes % 16 == 0 && row_bytes >= 1024;
}

template <int DT, int L, int E>
void launch_packed(const Args& a) {
  const int n = (int)a.N;
  const rms::host::PackedShape shape = rms::host::packed_shape(a.M, (int64_t)n * rms::Storage<DT>::kBytes, L,
                                                               rms::kPackThreads, rms::kPackTileBytes,
                                                               rms::host::kPackedTargetReadWrite, kPackedMaxGrid);
  const int tile_rows = shape.tile_rows;
  const int64_t blocks = shape.blocks;
  RMS_LAUNCH((rms::softmax_packed_kernel<DT, L, E, true>), dim3((unsigned)blocks),
                     dim3(rms::kPackThreads), 0, a.stream, a.x, a.y, a.M, n, tile_rows);
}

// Lanes per row and elements per lane: see with_packed_shape.
template <int DT>
void dispatch_packed(const Args& a) {
  rms::host::with_packed_shape(a.N, rms::Storage<DT>::kBytes, 64, [&](auto lanes, auto elems) {
    launch_packed<DT, decltype(lanes)::value, decltype(elems)::value>(a);
  });
}

// The two-pass streaming kernel: about one batch of four groups per thread, whole wavefronts,
// at most 1024 threads (what every row long enough to need this kernel gets).
constexpr int64_t kStreamMaxN = (int64_t)1 << 31;

template <int DT>
void launch_stream(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  const int64_t nfull = a.N / rms::Storage<DT>::kVec;
  int64_t threads = (nfull / rms::kStreamBatch + rms::kWaveSize - 1) / rms::kWaveSize * rms::kWaveSize;
  threads = threads < rms::kWaveSize ? rms::kWaveSize : threads > kMaxThreads ? kMaxThreads : threads;
  RMS_LAUNCH((rms::softmax_stream_kernel<DT>), dim3((unsigned)blocks), dim3((unsigned)threads),
                     0, a.stream, a.x, a.y, a.M, a.N);
}

template <int DT>
void launch_generic(const Args& a) {
  const int64_t blocks = a.M < kMaxGrid ? a.M : kMaxGrid;
  RMS_LAUNCH((rms::softmax_generic_kernel<DT, kGenericThreads>), dim3((unsigned)blocks),
                     dim3(kGenericThreads), 0, a.stream, a.x, a.y, a.M, a.N);
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
  return launched ? SOFTMAX_OK : SOFTMAX_ERR_UNSUPPORTED;
}

// Launches the element-addressed row kernel.  The caller has checked that the row fits.
template <int DT>
int dispatch_unaligned(const Args& a) {
  using rms::host::with_shape;
  const int slots = (int)rms::host::whole_pieces(a.N, rms::Storage<DT>::kBytes);
  const int threads = pick_threads_unaligned(slots);
  int chunks = (slots + threads - 1) / threads;
  if (chunks < 1) chunks = 1;
  auto row = [&](auto g, auto c) { launch_row_unaligned<DT, decltype(c)::value, decltype(g)::value>(a); };
  const bool launched = with_shape<64, 4>(threads, chunks, row) || with_shape<256, 8>(threads, chunks, row) ||
                        with_shape<512, 8>(threads, chunks, row) || with_shape<1024, 8>(threads, chunks, row);
  return launched ? SOFTMAX_OK : SOFTMAX_ERR_UNSUPPORTED;
}

// Rows that are a multiple of 16 bytes but not of the 128-byte line cost the aligned kernels 5 to
// 20 %: every second or every eighth row starts off a line, a wavefront's 1 KiB then touches nine
// lines instead of eight, and the last line of a row is shared with the next row, which another
// XCD reads.  Beyond 256 bytes (below, packed_beats_lanes has the measured choice) such rows go
// through LDS up to 1.5 KiB (64 MiB of fp16 rows of 136 to 520 elements: 22.9 to 23.7 us against
// 26.2 to 28.8) and to the element-addressed kernel beyond, which lays its slots out from the
// line a row starts in (fp16 65536 x 2040 101.3 -> 92.5 us, 32768 x 4088 88.1 -> 82.9, 8192 x 12280
// 70.1 -> 64.4, 131072 x 1000 93.0 -> 84.0, 4096 x 16376 47.1 -> 44.1), up to 64 KiB: beyond, the
// aligned kernel with 1024 threads is 6 to 14 % ahead again (bf16 2048 x 40952: 66.2 against 73.8
// us).  Returns -3, -1 or 0 (the rule does not apply).
constexpr int64_t kLineRuleMinBytes = 256;
constexpr int64_t kLineRulePackedBytes = 1536;
constexpr int64_t kLineRuleMaxBytes = 64 * 1024;

int off_line_kernel(int64_t N, int dtype) {
  const int64_t row_bytes = N * elem_bytes(dtype);
  if (row_bytes % rms::kLineBytes == 0 || row_bytes <= kLineRuleMinBytes || row_bytes > kLineRuleMaxBytes) return 0;
  if (row_bytes <= kLineRulePackedBytes && packed_can(N)) return -3;
  if (pick_threads_unaligned(rms::host::whole_pieces(N, elem_bytes(dtype))) != 0) return -1;
  return 0;
}

// threads == 0 means the element-wise kernel, -1 the element-addressed row kernel, -2 the
// two-pass streaming kernel, -3 the LDS-staged kernel.
template <int DT>
int run_typed(const Args& a, int threads) {
  int rc = SOFTMAX_OK;
  if (threads == 0) launch_generic<DT>(a);
  else if (threads == -1) rc = dispatch_unaligned<DT>(a);
  else if (threads == -2) launch_stream<DT>(a);
  else if (threads == -3) dispatch_packed<DT>(a);
  else rc = dispatch<DT>(a, threads);
  if (rc != SOFTMAX_OK) return rc;
  return rms::host::launch_status() == hipSuccess ? SOFTMAX_OK : SOFTMAX_ERR_LAUNCH;
}

// variant: a softmax_variant, or -1 with `threads` forced by the caller.
int run(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream, int variant,
        int threads) {
  int rc = check_args(x, y, M, N, dtype);
  if (rc != SOFTMAX_OK) return rc;
  if (variant < -1 || variant > SOFTMAX_VARIANT_PACKED) return SOFTMAX_ERR_INVALID_ARG;
  if (variant == -1 && max_chunks_for(threads) == 0) return SOFTMAX_ERR_INVALID_ARG;
  if (M == 0) return SOFTMAX_OK;

  const bool vec_ok = rows_vectorisable(x, y, N, dtype);
  const int64_t nvec = vec_ok ? N * elem_bytes(dtype) / 16 : 0;
  const bool unaligned_fits = pick_threads_unaligned(rms::host::whole_pieces(N, elem_bytes(dtype))) != 0;
  switch (variant) {
    case SOFTMAX_VARIANT_AUTO:
      threads = vec_ok ? (nvec <= kPackedAutoVectors ? -3 : pick_threads(nvec, 8))
                       : (packed_can(N) && !only_stores_unaligned(x, N, dtype)) ? -3
                       : unaligned_fits ? -1 : 0;
      if (vec_ok && threads > 0 && threads < 64 && packed_beats_lanes(nvec, threads)) threads = -3;
      if (vec_ok && off_line_kernel(N, dtype) != 0) threads = off_line_kernel(N, dtype);
      if (threads == 0 && N < kStreamMaxN) threads = -2;     // too long for registers
      break;
    case SOFTMAX_VARIANT_PACKED:
      if (!packed_can(N)) return SOFTMAX_ERR_UNSUPPORTED;
      threads = -3;
      break;
    case SOFTMAX_VARIANT_STREAM:
      if (N >= kStreamMaxN) return SOFTMAX_ERR_UNSUPPORTED;
      threads = -2;
      break;
    case SOFTMAX_VARIANT_UNALIGNED:
      if (!unaligned_fits) return SOFTMAX_ERR_UNSUPPORTED;
      threads = -1;
      break;
    case -1:
      if (!(vec_ok && threads_can(threads, nvec))) return SOFTMAX_ERR_UNSUPPORTED;
      break;
    case SOFTMAX_VARIANT_SUBWAVE:
      threads = nvec <= 8 ? 8 : nvec <= 16 ? 16 : 32;
      if (!(vec_ok && threads_can(threads, nvec))) return SOFTMAX_ERR_UNSUPPORTED;
      break;
    case SOFTMAX_VARIANT_WAVE:
      if (!(vec_ok && threads_can(64, nvec))) return SOFTMAX_ERR_UNSUPPORTED;
      threads = 64;
      break;
    case SOFTMAX_VARIANT_BLOCK:
      threads = vec_ok ? pick_threads(nvec, 256) : 0;
      if (threads == 0) return SOFTMAX_ERR_UNSUPPORTED;
      break;
    default:
      threads = 0;
      break;
  }

  Args a{x, y, M, N, (int)nvec, static_cast<hipStream_t>(stream)};
  switch (dtype) {
    case SOFTMAX_DTYPE_FP32: return run_typed<rms::kFp32>(a, threads);
    case SOFTMAX_DTYPE_FP16: return run_typed<rms::kFp16>(a, threads);
    case SOFTMAX_DTYPE_BF16: return run_typed<rms::kBf16>(a, threads);
    default: return SOFTMAX_ERR_INVALID_ARG;
  }
}

}  // namespace

extern "C" {

int softmax_fwd(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream) {
  return run(x, y, M, N, dtype, stream, SOFTMAX_VARIANT_AUTO, 0);
}

int softmax_fwd_variant(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream,
                        int variant) {
  if (variant < SOFTMAX_VARIANT_AUTO) return SOFTMAX_ERR_INVALID_ARG;
  return run(x, y, M, N, dtype, stream, variant, 0);
}

int softmax_fwd_tuned(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream,
                      int threads_per_row) {
  return run(x, y, M, N, dtype, stream, -1, threads_per_row);
}

int softmax_auto_threads_per_row(int64_t N, int dtype) {
  const int b = elem_bytes(dtype);
  if (b == 0 || N <= 0) return SOFTMAX_ERR_INVALID_ARG;
  if ((N * b) % 16 != 0) return 0;
  // rows off the 128-byte lines (see off_line_kernel): through LDS, or the element-addressed kernel
  const int off_line = off_line_kernel(N, dtype);
  if (off_line == -3) return 1;
  if (off_line == -1) return pick_threads_unaligned(rms::host::whole_pieces(N, b));
  const int64_t nvec = N * b / 16;
  const int g = pick_threads(nvec, 8);
  // the aligned rows that the automatic path sends through LDS instead (see run)
  if (nvec <= kPackedAutoVectors || (g > 0 && g < 64 && packed_beats_lanes(nvec, g))) return 1;
  return g;
}

int64_t softmax_register_max_n(int dtype) {
  const int b = elem_bytes(dtype);
  return b ? (int64_t)kMaxThreads * kBlockMaxChunks * (16 / b) : 0;
}

const char* softmax_status_string(int status) {
  switch (status) {
    case SOFTMAX_OK: return "ok";
    case SOFTMAX_ERR_INVALID_ARG: return "invalid argument";
    case SOFTMAX_ERR_UNSUPPORTED: return "kernel does not support this shape or alignment";
    case SOFTMAX_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
