/*
 * softmax.h - C ABI of the MI355X (gfx950) row-wise softmax forward library.
 *
 * The operation is the "softmax" row of the paper's "Supported kernel types"
 * table (memory-bound, measured in GB/s; results in the table "Kernel
 * performance on H100", Section 7.1), the sibling of RMSNorm with the same
 * reduce-then-scale structure:
 *
 *     y[i, j] = exp(x[i, j] - max_j x[i, :]) / sum_j exp(x[i, j] - max_j x[i, :])
 *
 * Inputs are widened exactly to fp32, the maximum, the exponentials, their sum
 * and the quotient are carried in fp32, and the result is rounded once
 * (nearest-even, subnormals kept) to the storage type.  An entry of -inf gives
 * an output of exactly 0; a row that contains NaN or +inf, or only -inf, comes
 * out as NaN in every position, as IEEE arithmetic on the formula gives.
 *
 * Conventions are those of rmsnorm.h: device pointers owned by the caller; the
 * library never allocates, copies or synchronises; work is enqueued on `stream`;
 * x and y are M x N row-major with leading dimension N and share one storage
 * type; pointers need only element alignment (rows that are not 16-byte aligned
 * go through LDS several at a time up to 1024 elements and beyond that run the
 * register-resident kernel addressed in bytes, SOFTMAX_VARIANT_UNALIGNED; rows too long
 * for registers, beyond softmax_register_max_n, stream through a two-pass kernel
 * that reads them a second time from cache); y == x exactly
 * is allowed, any other overlap is undefined; a call returns SOFTMAX_OK or a
 * negative softmax_status and launches nothing on INVALID_ARG / UNSUPPORTED;
 * results are bit-identical from run to run.
 */
#ifndef SOFTMAX_H_
#define SOFTMAX_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SOFTMAX_DTYPE_FP32 = 0,
  SOFTMAX_DTYPE_FP16 = 1,
  SOFTMAX_DTYPE_BF16 = 2
} softmax_dtype;

typedef enum {
  SOFTMAX_OK = 0,
  SOFTMAX_ERR_INVALID_ARG = -1, /* null pointer, M < 0, N <= 0, bad dtype, misaligned element */
  SOFTMAX_ERR_UNSUPPORTED = -2, /* the forced kernel cannot run this shape or alignment */
  SOFTMAX_ERR_LAUNCH = -3       /* the HIP runtime refused the launch */
} softmax_status;

typedef enum {
  SOFTMAX_VARIANT_AUTO = 0,    /* dispatch on (dtype, N, alignment) */
  SOFTMAX_VARIANT_WAVE = 1,    /* one wavefront per row */
  SOFTMAX_VARIANT_BLOCK = 2,   /* one workgroup of 256..1024 threads per row */
  SOFTMAX_VARIANT_GENERIC = 3, /* element-wise, three passes, any alignment, any N */
  SOFTMAX_VARIANT_SUBWAVE = 4, /* 8, 16 or 32 lanes per row; 16-byte aligned rows <= 1 KiB */
  SOFTMAX_VARIANT_UNALIGNED = 5, /* the register-resident row kernel addressed in bytes: 128-bit
                                    accesses on the 16-byte boundaries of x, laid out from the
                                    128-byte line in which the row starts so that a wavefront's
                                    accesses cover whole lines (of y too if x and y are
                                    congruent modulo 128 bytes), single elements at both ends:
                                    any alignment, N up to the register limit */
  SOFTMAX_VARIANT_STREAM = 6,    /* two streaming passes (online max and sum, then scale) for
                                    rows too long for registers: any alignment, N < 2^31 */
  SOFTMAX_VARIANT_PACKED = 7     /* runs of short rows copied through LDS with 128-bit accesses,
                                    1 to 64 lanes per row: N <= 1024, any alignment (the stores
                                    fall on 16-byte boundaries if x and y are congruent modulo 16
                                    bytes); what rows that are not 16-byte aligned take up to that
                                    length, and aligned rows that are very short or fill their
                                    lane group badly */
} softmax_variant;

/*
 * Softmax over the last dimension (formula above).
 *   x      device, M*N elements of `dtype`, read once
 *   y      device, M*N elements of `dtype`, written once
 *   M, N   rows and row length; M == 0 is a successful no-op; N must be >= 1
 *   dtype  a softmax_dtype
 *   stream a hipStream_t passed as void*; NULL is the default stream
 */
int softmax_fwd(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream);

/* Same, with the kernel family forced (a softmax_variant); SOFTMAX_ERR_UNSUPPORTED
 * if that family cannot take the shape or alignment. */
int softmax_fwd_variant(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream,
                        int variant);

/*
 * Same, with the number of threads sharing one row forced: 8, 16, 32 (several
 * rows per wavefront, up to 2 chunks per thread), 64 (one wavefront per row, up
 * to 4 chunks), 256, 512 or 1024 (one workgroup per row, up to 8 chunks); a
 * chunk is 16 bytes of the row.  Other values: SOFTMAX_ERR_INVALID_ARG; a row
 * that needs more chunks, or is not 16-byte aligned: SOFTMAX_ERR_UNSUPPORTED.
 */
int softmax_fwd_tuned(const void* x, void* y, int64_t M, int64_t N, int dtype, void* stream,
                      int threads_per_row);

/* threads_per_row of the automatic path for 16-byte aligned rows of N elements; 0 if
 * such rows do not fit in registers (they take the streaming kernel); 1 if it sends them
 * through LDS several rows at a time (SOFTMAX_VARIANT_PACKED: rows of at most 64 bytes, and
 * short rows that would fill their lane group badly); a negative softmax_status for bad
 * arguments.  Rows of more than 256 bytes and at most 64 KiB that are a multiple of 16 bytes
 * but not of the 128-byte cache line are dispatched like rows that are not 16-byte aligned (the
 * aligned kernels lose 5 to 20 % on them): SOFTMAX_VARIANT_PACKED up to 1.5 KiB (1),
 * SOFTMAX_VARIANT_UNALIGNED beyond (its threads per row). */
int softmax_auto_threads_per_row(int64_t N, int dtype);

/* Largest N the register-resident kernels accept for `dtype`; 0 for a bad dtype. */
int64_t softmax_register_max_n(int dtype);

/* Static, human-readable text for a status code. */
const char* softmax_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char softmax_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* SOFTMAX_H_ */
