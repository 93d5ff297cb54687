/*
 * measure.h - C ABI of the measurement aid that the benchmark uses beside the row kernels.
 *
 * Not part of any operation of the paper: a streaming copy whose HBM traffic is known exactly.
 * It serves two purposes in the measurement the paper's Section 5 asks for (throughput and the
 * fraction of the detected peak): the FETCH_SIZE / WRITE_SIZE hardware counters are scaled by
 * what they read for this copy, and its rate is the practical ceiling of a stream that is half
 * reads and half writes, which the roofline fraction of the row kernels is read against.
 */
#ifndef MEASURE_H_
#define MEASURE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEASURE_OK = 0,
  MEASURE_ERR_INVALID_ARG = -1, /* null or misaligned pointer, negative size, size not a multiple of 16 */
  MEASURE_ERR_LAUNCH = -3       /* the HIP runtime refused the launch */
} measure_status;

/*
 * dst <- src, `bytes` bytes (a multiple of 16; both DEVICE pointers 16-byte aligned, owned by
 * the caller, not overlapping), with 128-bit non-temporal loads and stores: one 16-byte vector
 * per thread, one 64-lane wavefront per workgroup, the fastest copy shape measured on MI355X.
 * Reads `bytes` from HBM and writes `bytes` to it.  Enqueues on `stream` (a hipStream_t as
 * void*, NULL = default stream) and returns at once; nothing is allocated or synchronised.
 * bytes == 0 is a successful no-op.
 */
int measure_copy(const void* src, void* dst, int64_t bytes, void* stream);

/*
 * The same copy through LDS, the way the kernels for short rows stage their data: workgroups of
 * 256 threads load a tile of 8 KiB, write it to LDS, meet at a barrier, read it back and store
 * it.  Same arguments, traffic and behaviour as measure_copy (a last tile that is not full is
 * handled).  Its rate is the ceiling for a kernel that stages whole tiles through LDS; what
 * such a kernel loses beyond it goes to its arithmetic and to rows that do not fill vectors.
 */
int measure_staged_copy(const void* src, void* dst, int64_t bytes, void* stream);

/* Static, human-readable text for a status code. */
const char* measure_status_string(int status);

/* "RMS_BUILD_ID:" followed by the hash of the sources this library was built from. */
extern const char measure_build_id[];

#ifdef __cplusplus
}
#endif

#endif /* MEASURE_H_ */
