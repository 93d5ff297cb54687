/*
 * crossentropy.h - C ABI of the MI355X (gfx950) row-wise cross-entropy forward library.
 *
 * The operation is the "cross_ent" row of the paper's "Supported kernel types" table
 * (memory-bound, measured in GB/s, a running log-sum-exp fused with the target pick; results
 * for 4096 x 32k and 8192 x 32k in the table "Kernel performance on H100", Section 7.1).  Per
 * row i with
 * target class t_i:
 *
 *     m_i     = max_j x[i, j]
 *     loss[i] = log( sum_j exp(x[i, j] - m_i) ) - (x[i, t_i] - m_i)
 *     lse[i]  = m_i + log( sum_j exp(x[i, j] - m_i) )              (optional output)
 *
 * Logits are widened exactly to fp32 and everything is carried in fp32; loss and lse are
 * fp32 whatever the storage type of the logits.  A target outside [0, N) marks an ignored
 * row: its loss is exactly 0 (its lse is still written).  -inf logits drop out of the sum; a
 * target on a -inf logit gives +inf; a row holding NaN or +inf, or only -inf, gives NaN.
 * No reduction over rows is applied: the caller sums or averages the M losses as it needs,
 * in an order of its own choosing.
 *
 * Conventions are those of rmsnorm.h: device pointers owned by the caller; the library
 * never allocates, copies or synchronises; work is enqueued on `stream`; x is M x N
 * row-major with leading dimension N; pointers need only element alignment and N may be odd
 * (every shape runs through the same kernel); a call returns CROSSENTROPY_OK or a negative
 * crossentropy_status and launches nothing on INVALID_ARG; results are bit-identical from
 * run to run.
 */
#ifndef CROSSENTROPY_H_
#define CROSSENTROPY_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CROSSENTROPY_DTYPE_FP32 = 0,
  CROSSENTROPY_DTYPE_FP16 = 1,
  CROSSENTROPY_DTYPE_BF16 = 2
} crossentropy_dtype;

typedef enum {
  CROSSENTROPY_OK = 0,
  CROSSENTROPY_ERR_INVALID_ARG = -1, /* null x/target/loss, M < 0, N <= 0 or >= 2^32, bad dtype,
                                        misaligned pointer, bad threads_per_row */
  CROSSENTROPY_ERR_UNSUPPORTED = -2, /* a forced lane-group size (8, 16, 32) on rows that are not
                                        16-byte aligned or longer than 8 vectors per lane, or
                                        the LDS-staged kernel with N > 1024; nothing was
                                        launched */
  CROSSENTROPY_ERR_LAUNCH = -3       /* the HIP runtime refused the launch */
} crossentropy_status;

/*
 * Cross-entropy forward (formula above).
 *   x       device, M*N logits of `dtype`, read once
 *   target  device, M int64 class indices (8-byte aligned)
 *   loss    device, M floats, written
 *   lse     device, M floats, written; or NULL
 *   M, N    rows and classes; M == 0 is a successful no-op; N must be >= 1
 *   dtype   a crossentropy_dtype
 *   stream  a hipStream_t passed as void*; NULL is the default stream
 */
int crossentropy_fwd(const void* x, const int64_t* target, float* loss, float* lse, int64_t M,
                     int64_t N, int dtype, void* stream);

/* Same, with the number of threads that share one row forced: a multiple of 64 from 64 to
 * 1024 (one workgroup per row; every such count runs every shape), or 8, 16 or 32 (lane
 * groups, several rows per wavefront: x 16-byte aligned, N * sizeof(dtype) a multiple of 16 and
 * at most 128 bytes per lane, otherwise CROSSENTROPY_ERR_UNSUPPORTED), or 2 (not a thread count:
 * runs of rows copied through LDS, 1 to 64 lanes per row chosen from N; any alignment,
 * N <= 1024, otherwise CROSSENTROPY_ERR_UNSUPPORTED).  Any other value is
 * CROSSENTROPY_ERR_INVALID_ARG. */
int crossentropy_fwd_tuned(const void* x, const int64_t* target, float* loss, float* lse,
                           int64_t M, int64_t N, int dtype, void* stream, int threads_per_row);

/* threads_per_row of the automatic path for rows of N classes whose base is 16-byte aligned:
 * 2 for rows up to 256 bytes and for fp32 rows up to 1024 classes, lane groups
 * for rows of whole 16-byte vectors up to 4 KiB (2 KiB for fp32), 2 for other rows of at most
 * 1024 classes (an unaligned base makes every such row take 2, and longer ones 64 threads);
 * a negative crossentropy_status for a bad dtype or N <= 0. */
int crossentropy_auto_threads_per_row(int64_t N, int dtype);

/* Static, human-readable text for a status code. */
const char* crossentropy_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char crossentropy_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* CROSSENTROPY_H_ */
