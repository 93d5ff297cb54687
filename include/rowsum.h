/*
 * rowsum.h - C ABI of the MI355X (gfx950) row-wise sum reduction library.
 *
 * The operation is the "reduce" row of the paper's "Supported kernel types" table
 * (memory-bound, measured in GB/s, a level-by-level shuffle reduction in the starter; results
 * for 8192 x 8192 and 16384 x 4096 in the table "Kernel performance on H100", Section 7.1).
 * The paper prints
 * no formula; its two-dimensional shapes and its throughput column (one read of the input,
 * nothing of comparable size written) fit the sum over the last dimension:
 *
 *     y[i] = sum_j x[i, j]
 *
 * Elements are widened exactly to fp32 and added in fp32, in a fixed hierarchical order
 * (per-lane running sums, then the lanes of a wavefront, then the wavefronts of a
 * workgroup); y is fp32 whatever the storage type of x.  IEEE arithmetic decides the corner
 * cases: a row holding NaN, or +inf and -inf together, gives NaN; an infinity alone gives
 * that infinity.  The error against the exact sum is bounded by
 * (N / 256 + 32) * 2^-24 * sum_j |x[i, j]| (each addition rounds by at most 2^-24 of a
 * partial sum, and no element passes through more additions than that); partial sums must
 * stay below FLT_MAX.
 *
 * Conventions are those of rmsnorm.h: device pointers owned by the caller; the library
 * never allocates, copies or synchronises; work is enqueued on `stream`; x is M x N
 * row-major with leading dimension N; pointers need only element alignment and N may be odd;
 * a call returns ROWSUM_OK or a negative rowsum_status and launches nothing on INVALID_ARG;
 * results are bit-identical from run to run for the same shape and pointer alignment.
 */
#ifndef ROWSUM_H_
#define ROWSUM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ROWSUM_DTYPE_FP32 = 0,
  ROWSUM_DTYPE_FP16 = 1,
  ROWSUM_DTYPE_BF16 = 2
} rowsum_dtype;

typedef enum {
  ROWSUM_OK = 0,
  ROWSUM_ERR_INVALID_ARG = -1, /* null x/y, M < 0, N <= 0 or >= 2^32, bad dtype, misaligned
                                  pointer, threads_per_row the shape does not allow */
  ROWSUM_ERR_LAUNCH = -3       /* the HIP runtime refused the launch */
} rowsum_status;

/*
 * Row sums (formula above).
 *   x       device, M*N elements of `dtype`, read once
 *   y       device, M floats, written
 *   M, N    rows and row length; M == 0 is a successful no-op; N must be >= 1
 *   dtype   a rowsum_dtype
 *   stream  a hipStream_t passed as void*; NULL is the default stream
 */
int rowsum_fwd(const void* x, float* y, int64_t M, int64_t N, int dtype, void* stream);

/* Same, with the number of threads that share one row forced: a multiple of 64 from 64 to
 * 1024 (one workgroup per row, every shape), or 8, 16 or 32 (several rows per wavefront:
 * only for 16-byte aligned rows of at most 8 * threads_per_row 16-byte vectors), or 2 (not a
 * thread count: runs of rows copied through LDS, 1 to 64 lanes per row chosen from N; any
 * alignment, N <= 1024).  Any other value, or a shape the value does not allow, is
 * ROWSUM_ERR_INVALID_ARG. */
int rowsum_fwd_tuned(const void* x, float* y, int64_t M, int64_t N, int dtype, void* stream,
                     int threads_per_row);

/* threads_per_row of the automatic path for rows of N elements whose base is 16-byte aligned:
 * 2 for rows of at most 1024 elements, otherwise a thread count; a negative rowsum_status for
 * a bad dtype or N <= 0.  (With a base that is not 16-byte aligned every row of at most 1024 elements takes 2,
 * and longer ones the workgroup-per-row kernel with at least 64 threads.) */
int rowsum_auto_threads_per_row(int64_t N, int dtype);

/* Static, human-readable text for a status code. */
const char* rowsum_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char rowsum_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* ROWSUM_H_ */
