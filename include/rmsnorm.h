/*
 * rmsnorm.h - C ABI of the MI355X (gfx950) row-wise RMSNorm forward library.
 *
 * The operation is the "rmsnorm" row of the paper's "Supported kernel types"
 * table (memory-bound, measured in GB/s) and the kernel of its headline result
 * in Section 7.1 "Kernel Performance": one fused pass that reads each row once,
 * normalises it by its root mean square and multiplies by the weight in the
 * epilogue (the fusion Section 7.3 credits for saving a round trip to memory):
 *
 *     y[i, j] = x[i, j] * rsqrt( mean_j( x[i, :]^2 ) + eps ) * w[j]
 *
 * Inputs are widened exactly to fp32, the sum of squares and both products are
 * carried in fp32, and the result is rounded once (nearest-even) to the
 * storage type.  Domain: finite inputs whose row sum of squares stays below
 * FLT_MAX; NaN and infinity propagate by IEEE rules.  A finite row past that
 * limit (a square or the sum overflows fp32) comes back as zeros carrying the
 * sign of x[j] * w[j] from every kernel: the sum is +inf, so the scale is 0.
 *
 * Conventions for every entry point:
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    never allocates, frees, copies or synchronises; a call enqueues work on
 *    `stream` and returns at once.  Buffers must stay alive until that work
 *    has run.  (The library holds one static device array of 132 KiB per GPU,
 *    part of its code object: the counters described under rmsnorm_fwd.)
 *  - x and y are M x N, row-major, leading dimension N (no stride argument);
 *    w has N elements.  x, w and y share one storage type `dtype`.
 *  - Pointers need only the alignment of their element type.  Rows whose
 *    start is 16-byte aligned (16-byte aligned bases and N * sizeof(dtype) a
 *    multiple of 16) take the aligned kernels; other rows of up to 1024
 *    elements go through LDS several at a time, longer ones take the
 *    register-resident kernel addressed in bytes; both read x with 128-bit
 *    loads on 16-byte boundaries (the longer rows laid out from the 128-byte
 *    line they start in, so that a wavefront's accesses cover whole lines)
 *    and write y the same way if x and y sit at the same offset from a
 *    boundary (from a line), with element-aligned 128-bit stores otherwise;
 *    rows too long for registers stream through a two-pass kernel that reads x
 *    a second time from cache.  None of these is an error.
 *  - y == x (exactly in place) is allowed; any other overlap of y with x or w
 *    is undefined.
 *  - Calls return RMSNORM_OK or a negative rmsnorm_status; nothing throws or
 *    aborts.  On RMSNORM_ERR_INVALID_ARG and RMSNORM_ERR_UNSUPPORTED nothing
 *    was launched.
 *  - Results are bit-identical from run to run for a given (shape, dtype,
 *    alignment, variant): reductions have a fixed order and no sum goes through
 *    an atomic (RMSNORM_VARIANT_QUEUE hands out rows with atomic counters; which
 *    workgroup takes a row does not change the row's arithmetic).
 */
#ifndef RMSNORM_H_
#define RMSNORM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RMSNORM_DTYPE_FP32 = 0, /* IEEE binary32 */
  RMSNORM_DTYPE_FP16 = 1, /* IEEE binary16 */
  RMSNORM_DTYPE_BF16 = 2  /* bfloat16: upper half of a binary32 */
} rmsnorm_dtype;

typedef enum {
  RMSNORM_OK = 0,
  RMSNORM_ERR_INVALID_ARG = -1, /* null pointer, M < 0, N <= 0, bad dtype, eps < 0 or NaN */
  RMSNORM_ERR_UNSUPPORTED = -2, /* the forced variant cannot run this shape or alignment */
  RMSNORM_ERR_LAUNCH = -3,      /* the HIP runtime refused the launch */
  RMSNORM_ERR_TOO_LARGE = -4    /* rmsnorm_fwd_static only: more rows, or longer rows, than its fixed
                                   scratch covers */
} rmsnorm_status;

typedef enum {
  RMSNORM_VARIANT_AUTO = 0,    /* dispatch on (dtype, N, alignment) */
  RMSNORM_VARIANT_WAVE = 1,    /* one 64-lane wavefront per row, row held in registers */
  RMSNORM_VARIANT_BLOCK = 2,   /* one workgroup of 128..1024 threads per row, row held in
                                  registers, cross-wave reduction in LDS */
  RMSNORM_VARIANT_GENERIC = 3, /* element-wise, any alignment, any N; reads x twice */
  RMSNORM_VARIANT_UNALIGNED = 4, /* row held in registers like WAVE / BLOCK, but addressed in
                                   bytes: 128-bit accesses on the 16-byte boundaries of x,
                                   laid out from the 128-byte line in which the row starts
                                   so that a wavefront's accesses cover whole lines (of y
                                   too if x and y are congruent modulo 128 bytes), single
                                   elements at both ends; with enough rows, resident
                                   workgroups that read their weight slices once (see
                                   rmsnorm_unaligned_walk_grid); any alignment, N up to
                                   rmsnorm_unaligned_max_n(dtype) */
  RMSNORM_VARIANT_SUBWAVE = 5,  /* 8, 16 or 32 lanes per row, several rows per wavefront;
                                   16-byte aligned rows of at most 1 KiB */
  RMSNORM_VARIANT_STREAM = 6,   /* two streaming passes with 128-bit accesses for rows too
                                   long for registers (the second read comes from cache);
                                   any alignment, N < 2^31 */
  RMSNORM_VARIANT_PACKED = 7,   /* runs of short rows copied through LDS with 128-bit accesses,
                                   1 to 64 lanes per row; N <= 1024, any alignment (the stores
                                   fall on 16-byte boundaries if x and y are congruent modulo 16
                                   bytes); what rows that are not 16-byte aligned take up to that
                                   length, and aligned rows that are very short or fill their
                                   lane group badly */
  RMSNORM_VARIANT_QUEUE = 8     /* BLOCK's arithmetic on a grid of one or two workgroups per compute
                                   unit that stay for the whole launch, keep their slices of the
                                   weight in registers and draw rows from counters in device
                                   memory; 16-byte aligned rows of 513 to 4096 vectors of 16 bytes
                                   (8 KiB to 64 KiB), fewer than 2^30 rows.  What AUTO takes for rows
                                   of 16 KiB and more once the launch reads 96 MiB (192 MiB beyond
                                   32 KiB rows), and for shorter ones from 320 MiB on, on streams
                                   that have counters (see rmsnorm_fwd) */
} rmsnorm_variant;

/*
 * RMSNorm forward (the "rmsnorm" kernel of the paper's kernel table; formula
 * above).
 *   x      device, M*N elements of `dtype`, read once
 *   w      device, N elements of `dtype`
 *   y      device, M*N elements of `dtype`, written once
 *   M, N   rows and row length; M == 0 is a successful no-op; N must be >= 1
 *   eps    added to the mean of squares inside the root; must be >= 0
 *   dtype  an rmsnorm_dtype
 *   stream a hipStream_t passed as void*; NULL is the default stream
 *
 * Large launches of long rows (RMSNORM_VARIANT_QUEUE) need 4 KiB of counters in device memory.
 * This entry point takes them from an array inside the library, one block per stream: launches
 * on one stream run one after the other, so a block is never used by two kernels at once, and
 * the kernel leaves its counters at zero for the next launch.  The first 32 streams seen on a
 * device get a block each and keep it; a call on any other stream, on the per-thread default
 * stream, or on a stream that is being captured into a graph (a graph can be replayed on any
 * stream) runs the one-workgroup-per-row kernel instead, with the same bits in y.  The only
 * state kept between calls is which stream owns which block.
 */
int rmsnorm_fwd(const void* x, const void* w, void* y, int64_t M, int64_t N,
                float eps, int dtype, void* stream);

/*
 * Same operation with the kernel choice forced (tests and benchmarks use this
 * to run every kernel on every shape it supports).  `variant` is an
 * rmsnorm_variant.  RMSNORM_ERR_UNSUPPORTED if that kernel cannot take the
 * shape: SUBWAVE needs 16-byte aligned rows of at most 1 KiB, WAVE needs
 * 16-byte aligned rows of at most rmsnorm_wave_max_n(dtype) elements, BLOCK
 * needs 16-byte aligned rows of at most rmsnorm_block_max_n(dtype) elements,
 * UNALIGNED takes any alignment up to rmsnorm_unaligned_max_n(dtype) elements,
 * PACKED any alignment up to 1024 elements, STREAM any
 * alignment up to N < 2^31, GENERIC takes everything.  QUEUE needs 16-byte
 * aligned rows of 513 to 4096 vectors and a stream that has counters (see
 * rmsnorm_fwd).
 */
int rmsnorm_fwd_variant(const void* x, const void* w, void* y, int64_t M, int64_t N,
                        float eps, int dtype, void* stream, int variant);

/*
 * Same operation with the number of threads that share one row forced: the
 * block-size axis that the paper's optimisation playbook sweeps first
 * (Section 3.3, tier 1; Section 7.3 reports it as the largest single gain for
 * RMSNorm).  threads_per_row is 8, 16 or 32 (several rows per wavefront), 64
 * (one wavefront per row), 128, 256, 512 or 1024 (one workgroup per row);
 * anything else is RMSNORM_ERR_INVALID_ARG.  Each thread then holds
 * ceil(N * sizeof(dtype) / 16 / threads_per_row) 16-byte chunks of the row in
 * registers; RMSNORM_ERR_UNSUPPORTED if that exceeds what is built for the
 * thread count (8, 16, 32: 2 chunks; 64: 16 chunks, 32 for fp32; 128, 256,
 * 512: 8 chunks; 1024: 16 chunks) or if the rows are not 16-byte aligned.
 * Tests use it to run every instantiation; tuning sweeps use it to check the
 * automatic choice.
 */
int rmsnorm_fwd_tuned(const void* x, const void* w, void* y, int64_t M, int64_t N,
                      float eps, int dtype, void* stream, int threads_per_row);

/*
 * The work-queue kernel (RMSNORM_VARIANT_QUEUE: the paper's single fused pass, Section 7.1,
 * with the weight multiply of Section 7.3 tier 3 fed from registers instead of from cache) on
 * counters that the caller brings.
 *   workspace        device memory, 4-byte aligned, at least rmsnorm_workspace_bytes() bytes,
 *                    owned by the caller.  It must be zero-filled before its first use; every
 *                    call leaves it zero-filled, so it can be passed again without clearing.
 *                    Two calls whose kernels may run at the same time need a workspace each.
 *   workspace_bytes  its size
 * Other arguments as for rmsnorm_fwd.  RMSNORM_ERR_INVALID_ARG for a workspace that is null,
 * misaligned or too small; RMSNORM_ERR_UNSUPPORTED for rows the kernel does not take (see
 * RMSNORM_VARIANT_QUEUE); nothing is launched in either case.  y holds the same bits as after
 * rmsnorm_fwd_tuned with 512 threads per row.
 */
int rmsnorm_fwd_workspace(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                          int dtype, void* stream, void* workspace, int64_t workspace_bytes);

/*
 * rmsnorm_fwd_workspace for callers that cannot allocate device memory at all (code under HIP
 * graph capture, tight serving loops, harnesses that forbid it) and therefore cannot bring a
 * workspace: the counters live in one fixed block of 4 KiB inside the library's static device
 * array (each GPU the library runs on holds its own copy until the process ends; its address is
 * looked up once per device, on the first call with that device current).  The call allocates
 * nothing and calls no allocating routine.  Same arguments, kernel, launch shape and result
 * bits as rmsnorm_fwd_workspace.
 *   Limits: rows of at most 4096 vectors of 16 bytes (64 KiB) and fewer than 2^30 rows, which
 *   is what the block and its 32-bit row tickets cover; beyond either, RMSNORM_ERR_TOO_LARGE
 *   and nothing is launched.  Rows the kernel does not take for other reasons (513 vectors at
 *   least, 16-byte aligned): RMSNORM_ERR_UNSUPPORTED, as for rmsnorm_fwd_workspace.
 *   Sharing: every call on a GPU uses that GPU's one block, whatever the stream.  The block
 *   keeps what the last kernel left in it, which is all zeros once that kernel has finished
 *   (every launch puts its counters back), so calls need no clearing between them; but two
 *   calls whose kernels overlap on one GPU (two streams, two host threads, a graph replayed
 *   beside an eager call) race on the counters and give wrong rows.  Callers that need
 *   overlap use rmsnorm_fwd_workspace with a workspace per stream, or rmsnorm_fwd.
 */
int rmsnorm_fwd_static(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                       int dtype, void* stream);

/* Bytes of workspace that rmsnorm_fwd_workspace and rmsnorm_fwd_queue_tuned need (4096). */
int64_t rmsnorm_workspace_bytes(void);

/*
 * rmsnorm_fwd_workspace with the launch shape forced (tests run odd shapes through it, tuning
 * sweeps check the automatic choice):
 *   grid        resident workgroups of 512 threads, a multiple of `shards`, at most 65536
 *   shards      1 .. 32 groups of workgroups, each with its own counters and its own rows
 *   block_rows  a power of two up to 65536: rows are dealt to the shards in blocks of that many
 *   prefetch    non-zero: a workgroup requests its next row before it stores the current one
 * RMSNORM_ERR_INVALID_ARG for values outside these ranges.
 */
int rmsnorm_fwd_queue_tuned(const void* x, const void* w, void* y, int64_t M, int64_t N, float eps,
                            int dtype, void* stream, void* workspace, int64_t workspace_bytes,
                            int grid, int shards, int block_rows, int prefetch);

/*
 * The launch shape RMSNORM_VARIANT_QUEUE uses for M rows of N elements on the current device
 * (any of the four output pointers may be NULL).  Returns 1 if RMSNORM_VARIANT_AUTO takes that
 * variant for such a call (given 16-byte aligned pointers and a stream with counters), 0 if the
 * variant can run it but AUTO prefers another, RMSNORM_ERR_UNSUPPORTED if it cannot run it,
 * RMSNORM_ERR_INVALID_ARG for a bad dtype, N <= 0 or M < 0.  No memory is touched.
 */
int rmsnorm_queue_plan(int64_t M, int64_t N, int dtype, int* grid, int* shards, int* block_rows,
                       int* prefetch);

/*
 * The threads_per_row that RMSNORM_VARIANT_AUTO uses for 16-byte aligned rows
 * of N elements: 0 if such rows do not fit in registers (they take the
 * streaming kernel), 1 if it sends them through LDS several rows at a time
 * (RMSNORM_VARIANT_PACKED: rows of at most 64 bytes, and short rows that would
 * fill their lane group badly), a negative rmsnorm_status for a bad dtype or
 * N <= 0.  Large launches of long rows run RMSNORM_VARIANT_QUEUE with 512
 * threads per row whatever this returns (see rmsnorm_queue_plan).
 * Rows of more than 256 bytes that are a multiple of 16 bytes but not of the
 * 128-byte cache line are dispatched like rows that are not 16-byte aligned
 * (the aligned kernels lose 15 to 40 % on them): RMSNORM_VARIANT_PACKED up to
 * 2 KiB (1), RMSNORM_VARIANT_UNALIGNED beyond (its threads per row) unless the
 * row is a multiple of 64 bytes.  So are rows of 2 KiB and more of whole lines
 * when y is not 64-byte aligned (RMSNORM_VARIANT_UNALIGNED; see
 * rmsnorm_select_variant, which looks at the pointers).
 */
int rmsnorm_auto_threads_per_row(int64_t N, int dtype);

/*
 * The same for a batch of M rows: batches of one to three rounds of resident workgroups at the
 * usual thread count run with narrower workgroups (256 or 128 threads) if the whole batch then
 * fits on the GPU at once; every other M gives what rmsnorm_auto_threads_per_row gives.  (The
 * tier-1 axis of the paper's playbook, Section 3.3, chosen per launch instead of per kernel.)
 * Uses the compute-unit count of the current device (256 if there is none).
 */
int rmsnorm_auto_threads_for_batch(int64_t M, int64_t N, int dtype);

/*
 * Which kernel RMSNORM_VARIANT_AUTO would pick for this call (an
 * rmsnorm_variant), without launching anything; a negative rmsnorm_status for
 * arguments rmsnorm_fwd would reject.  Only pointer alignment is inspected.
 */
int rmsnorm_select_variant(const void* x, const void* w, const void* y, int64_t M,
                           int64_t N, int dtype);

/*
 * How RMSNORM_VARIANT_UNALIGNED would run this call, without launching anything: the
 * number of resident workgroups of its walking form (a multiple of 64; each takes rows
 * blockIdx, blockIdx + grid, ..., all of which start at the same offset from a 128-byte
 * line, and reads its slices of the weight once), or 0 if it would run one workgroup per
 * row and read the weight slices for every row (fewer than two rows per workgroup, or
 * fewer than four on a grid well below the best one; rows of more than 8 16-byte pieces
 * per thread, 7 with 1024 threads; N beyond rmsnorm_unaligned_max_n).  A negative rmsnorm_status for arguments rmsnorm_fwd would
 * reject.  No memory is touched.
 */
int64_t rmsnorm_unaligned_walk_grid(const void* x, const void* w, const void* y, int64_t M,
                                    int64_t N, int dtype);

/* Largest N the register-resident kernels accept for `dtype`; 0 for a bad dtype. */
int64_t rmsnorm_wave_max_n(int dtype);
int64_t rmsnorm_block_max_n(int dtype);
int64_t rmsnorm_unaligned_max_n(int dtype);

/* Static, human-readable text for a status code. */
const char* rmsnorm_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char rmsnorm_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* RMSNORM_H_ */
