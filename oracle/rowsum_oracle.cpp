// CPU oracle for the row-wise sum reduction.  TEST INFRASTRUCTURE ONLY; shares no code with
// the GPU side or with the other oracle files.
//
// The paper lists "reduce" in its "Supported kernel types" table (regime Memory, metric
// GB/s; its starter reduces level by level with lane shuffles) and reports 8192 x 8192 and 16384 x 4096 in the table
// "Kernel performance on H100" (Section 7.1); it prints no formula.  The definition used
// here is the sum over the last dimension:
//
//     y_i = round_to_fp32( sum_j X(i, j) )         (index order j = 0 .. N-1, fp64)
//
// X widened exactly to fp64; the result is fp32 whatever the storage type of X, rounded
// once.  IEEE corner cases follow from the formula: a row holding NaN, or +inf and -inf
// together, gives NaN; +inf (or -inf) alone gives that infinity.  The optional second
// output is sum_j |X(i, j)| in fp64, the scale against which a floating-point sum's
// error is measured.
//
// A reduction by levels (per-lane partial sums, then wavefront, then workgroup) is a
// way of adding the same numbers in another order; the oracle takes them in index order.
//
// Pinned by tests/test_rowsum_oracle_pins.py.
// Build: g++ -O2 -std=c++17 -shared -fPIC -pthread.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum { kF32 = 0, kF16 = 1, kBF16 = 2 };

// Element k of the input as a double (exact).
double element(const void* base, int64_t k, int dtype) {
  const unsigned char* p = static_cast<const unsigned char*>(base);
  if (dtype == kF32) {
    float f;
    std::memcpy(&f, p + 4 * k, sizeof f);
    return f;
  }
  uint16_t bits;
  std::memcpy(&bits, p + 2 * k, sizeof bits);
  if (dtype == kBF16) {
    const uint32_t as32 = static_cast<uint32_t>(bits) << 16;   // bf16 = upper half of an fp32
    float f;
    std::memcpy(&f, &as32, sizeof f);
    return f;
  }
  // binary16: sign | 5-bit exponent (bias 15) | 10-bit fraction
  const bool negative = (bits & 0x8000u) != 0;
  const int exponent = (bits >> 10) & 0x1F;
  const int fraction = bits & 0x3FF;
  double magnitude;
  if (exponent == 0x1F) magnitude = fraction != 0 ? std::nan("") : INFINITY;
  else if (exponent == 0) magnitude = std::ldexp(static_cast<double>(fraction), -24);
  else magnitude = std::ldexp(static_cast<double>(1024 + fraction), exponent - 25);
  return negative ? -magnitude : magnitude;
}

void sum_rows(const void* x, float* y, double* abs_sum, int64_t first, int64_t end, int64_t N,
              int dtype) {
  for (int64_t i = first; i < end; ++i) {
    double total = 0.0, total_abs = 0.0;
    for (int64_t j = 0; j < N; ++j) {
      const double v = element(x, i * N + j, dtype);
      total += v;
      total_abs += std::fabs(v);
    }
    if (y) y[i] = static_cast<float>(total);        // one rounding, to nearest-even
    if (abs_sum) abs_sum[i] = total_abs;
  }
}

}  // namespace

extern "C" {

// x: HOST, M x N row-major of `dtype` (0 fp32, 1 fp16, 2 bf16); y: M floats out (may be
// NULL); abs_sum: M doubles out (may be NULL).  Returns 0, or -1 on a bad argument.
int rowsum_oracle(const void* x, float* y, double* abs_sum, int64_t M, int64_t N, int dtype,
                  int nthreads) {
  if (dtype < 0 || dtype > 2 || M < 0 || N <= 0) return -1;
  if (M == 0) return 0;
  if (!x || (!y && !abs_sum)) return -1;
  int64_t workers = nthreads > 0 ? nthreads : static_cast<int64_t>(std::thread::hardware_concurrency());
  if (workers < 1) workers = 1;
  if (workers > M) workers = M;
  if (workers == 1) {
    sum_rows(x, y, abs_sum, 0, M, N, dtype);
    return 0;
  }
  std::vector<std::thread> pool;
  const int64_t share = (M + workers - 1) / workers;
  for (int64_t k = 0; k < workers; ++k) {
    const int64_t first = k * share;
    const int64_t end = first + share < M ? first + share : M;
    if (first >= end) break;
    pool.emplace_back(sum_rows, x, y, abs_sum, first, end, N, dtype);
  }
  for (auto& t : pool) t.join();
  return 0;
}

}  // extern "C"
