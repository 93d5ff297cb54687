/*
 * layernorm.h - C ABI of the MI355X (gfx950) row-wise LayerNorm forward library.
 *
 * The operation is the "layernorm" row of the paper's "Supported kernel types"
 * table (memory-bound, measured in GB/s, one pass with Welford's recurrence in the
 * starter; results in the table "Kernel performance on H100", Section 7.1):
 *
 *     mean_i = (1/N) sum_j x[i, j]
 *     var_i  = (1/N) sum_j (x[i, j] - mean_i)^2          (biased)
 *     y[i, j] = (x[i, j] - mean_i) * rsqrt(var_i + eps) * w[j] + b[j]
 *
 * Inputs are widened exactly to fp32, both moments, the products and the bias
 * add are carried in fp32, and the result is rounded once (nearest-even) to the
 * storage type.  The moments are taken in two passes over the register-resident
 * row after shifting it by its first element, so rows whose mean is large
 * against their spread keep their accuracy.  Domain: finite inputs whose row sum
 * of squared deviations stays below FLT_MAX.
 *
 * Conventions are those of rmsnorm.h: device pointers owned by the caller; the
 * library never allocates, copies or synchronises; work is enqueued on `stream`;
 * x and y are M x N row-major with leading dimension N, w and b have N elements,
 * all of one storage type; b may be NULL (no bias); pointers need only element
 * alignment (rows that are not 16-byte aligned go through LDS several at a time up to 1024
 * elements and beyond that run a register-resident kernel addressed in bytes, see
 * LAYERNORM_VARIANT_UNALIGNED; rows too long for registers, beyond
 * layernorm_register_max_n, stream through a three-pass kernel that re-reads them
 * from cache); y == x exactly is allowed, any other overlap is
 * undefined; a call returns LAYERNORM_OK or a negative layernorm_status and
 * launches nothing on INVALID_ARG / UNSUPPORTED; results are bit-identical from
 * run to run.
 */
#ifndef LAYERNORM_H_
#define LAYERNORM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LAYERNORM_DTYPE_FP32 = 0,
  LAYERNORM_DTYPE_FP16 = 1,
  LAYERNORM_DTYPE_BF16 = 2
} layernorm_dtype;

typedef enum {
  LAYERNORM_OK = 0,
  LAYERNORM_ERR_INVALID_ARG = -1, /* null x/w/y, M < 0, N <= 0, bad dtype, eps < 0 or NaN */
  LAYERNORM_ERR_UNSUPPORTED = -2, /* the forced kernel cannot run this shape or alignment */
  LAYERNORM_ERR_LAUNCH = -3       /* the HIP runtime refused the launch */
} layernorm_status;

typedef enum {
  LAYERNORM_VARIANT_AUTO = 0,    /* dispatch on (dtype, N, alignment) */
  LAYERNORM_VARIANT_WAVE = 1,    /* one wavefront per row */
  LAYERNORM_VARIANT_BLOCK = 2,   /* one workgroup of 256..1024 threads per row */
  LAYERNORM_VARIANT_GENERIC = 3, /* element-wise, three passes, any alignment, any N */
  LAYERNORM_VARIANT_SUBWAVE = 4, /* 8, 16 or 32 lanes per row; 16-byte aligned rows <= 1 KiB */
  LAYERNORM_VARIANT_UNALIGNED = 5, /* the register-resident row kernel addressed in bytes:
                                      128-bit accesses on the 16-byte boundaries of x, laid out
                                      from the 128-byte line in which the row starts so that a
                                      wavefront's accesses cover whole lines (of y too if x and
                                      y are congruent modulo 128 bytes), single elements at both
                                      ends; with enough rows, resident workgroups that read their
                                      slices of weight and bias once (see
                                      layernorm_unaligned_walk_grid): any alignment, N up to the
                                      register limit */
  LAYERNORM_VARIANT_STREAM = 6,    /* three streaming passes with 128-bit accesses for rows too
                                      long for registers (the second and third read come from
                                      cache); any alignment, N < 2^31 */
  LAYERNORM_VARIANT_PACKED = 7,    /* runs of short rows copied through LDS with 128-bit accesses,
                                      1 to 64 lanes per row: N <= 1024, any alignment (the stores
                                      fall on 16-byte boundaries if x and y are congruent modulo 16
                                      bytes); what rows that are not 16-byte aligned take up to that
                                      length, and aligned rows that are very short or fill their
                                      lane group badly */
  LAYERNORM_VARIANT_QUEUE = 8      /* resident workgroups that keep their slices of weight and
                                      bias in registers and draw their rows from counters in
                                      device memory, in blocks of consecutive rows per XCD
                                      (see layernorm_queue_plan): 16-byte aligned rows that 256
                                      or 512 threads hold with at most 32 elements of a 16-bit
                                      type or 16 of fp32 each (N up to 16384 and 8192), fewer
                                      than 2^30 rows; what the automatic path takes for such
                                      rows in launches of a few hundred megabytes.  The counters
                                      are the library's own (a static array of 128 KiB of device
                                      memory per GPU, one 4 KiB block per stream for up to 32
                                      streams per device, zero between launches); a stream that
                                      gets none (the 33rd, the per-thread default stream, a
                                      stream under graph capture) gets LAYERNORM_ERR_UNSUPPORTED
                                      when the variant is forced and the other kernels on the
                                      automatic path.  Same bits as the other kernels. */
} layernorm_variant;

/*
 * LayerNorm over the last dimension (formula above).
 *   x      device, M*N elements of `dtype`, read once
 *   w      device, N elements (scale)
 *   b      device, N elements (shift), or NULL for no bias
 *   y      device, M*N elements, written once
 *   M, N   rows and row length; M == 0 is a successful no-op; N must be >= 1
 *   eps    added to the variance inside the root; must be >= 0
 *   dtype  a layernorm_dtype
 *   stream a hipStream_t passed as void*; NULL is the default stream
 */
int layernorm_fwd(const void* x, const void* w, const void* b, void* y, int64_t M, int64_t N,
                  float eps, int dtype, void* stream);

/* Same, with the kernel family forced (a layernorm_variant); LAYERNORM_ERR_UNSUPPORTED
 * if that family cannot take the shape or alignment. */
int layernorm_fwd_variant(const void* x, const void* w, const void* b, void* y, int64_t M,
                          int64_t N, float eps, int dtype, void* stream, int variant);

/*
 * Same, with the number of threads sharing one row forced: 8, 16, 32 (several
 * rows per wavefront, up to 2 chunks per thread), 64 (up to 4 chunks), 256, 512
 * or 1024 (up to 8 chunks); a chunk is 16 bytes of the row.  Other values:
 * LAYERNORM_ERR_INVALID_ARG; a row that needs more chunks, or is not 16-byte
 * aligned: LAYERNORM_ERR_UNSUPPORTED.
 */
int layernorm_fwd_tuned(const void* x, const void* w, const void* b, void* y, int64_t M,
                        int64_t N, float eps, int dtype, void* stream, int threads_per_row);

/* threads_per_row of the automatic path for 16-byte aligned rows of N elements; 0 if
 * such rows do not fit in registers (they take the streaming kernel); 1 if it sends them
 * through LDS several rows at a time (LAYERNORM_VARIANT_PACKED: rows of at most 64 bytes, and
 * short rows that would fill their lane group badly); a negative layernorm_status for bad
 * arguments.  Rows of 1 to 32 KiB that are a multiple of 16 bytes but not of the 128-byte cache
 * line are dispatched like rows that are not 16-byte aligned (the aligned kernels lose 3 to
 * 19 % on them): LAYERNORM_VARIANT_PACKED up to 1.75 KiB (1), LAYERNORM_VARIANT_UNALIGNED beyond
 * (its threads per row; those never take LAYERNORM_VARIANT_QUEUE on the automatic path) unless
 * the row is a multiple of 64 bytes. */
int layernorm_auto_threads_per_row(int64_t N, int dtype);

/*
 * How LAYERNORM_VARIANT_UNALIGNED would run this call, without launching anything: the
 * number of resident workgroups of its walking form (a multiple of 64; each takes rows
 * blockIdx, blockIdx + grid, ..., all of which start at the same offset from a 128-byte line,
 * and reads its slices of weight and bias once), or 0 if it would run one workgroup per row
 * and read those slices for every row (fewer than two rows per workgroup, or fewer than four
 * on a grid well below the best one; rows of at most 256 or more than 4096 whole 16-byte
 * pieces: N below 2056 or above 32775 elements of a 16-bit type, below 1028 or above 16387 of
 * fp32).  A negative layernorm_status for arguments
 * layernorm_fwd would reject.  No memory is touched.
 */
int64_t layernorm_unaligned_walk_grid(const void* x, const void* w, const void* b, const void* y,
                                      int64_t M, int64_t N, int dtype);

/*
 * How LAYERNORM_VARIANT_QUEUE would run M rows of N elements, without launching anything:
 * *threads (256 or 512 threads hold a row; the workgroup has one wavefront more, which draws
 * the rows), *grid resident workgroups in *shards groups, rows dealt to the groups in blocks of
 * *block_rows consecutive rows (any of the pointers may be NULL).  Returns 1 if layernorm_fwd
 * takes this kernel for such a call (on a stream that has counters), 0 if it can run but the
 * automatic path prefers another, LAYERNORM_ERR_UNSUPPORTED if it cannot run (rows that are not
 * a multiple of 16 bytes, rows of more than 2048 16-byte vectors, 2^30 rows or more, M == 0),
 * LAYERNORM_ERR_INVALID_ARG for a bad dtype, N <= 0 or M < 0.
 */
int layernorm_queue_plan(int64_t M, int64_t N, int dtype, int* threads, int* grid, int* shards,
                         int* block_rows);

/* Largest N the register-resident kernels accept for `dtype`; 0 for a bad dtype. */
int64_t layernorm_register_max_n(int dtype);

/* Static, human-readable text for a status code. */
const char* layernorm_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char layernorm_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* LAYERNORM_H_ */
