// CPU oracle for row-wise cross-entropy forward (log-sum-exp fused with the negative
// log-likelihood pick).  TEST INFRASTRUCTURE ONLY; shares no code with the GPU side or
// with the other oracle files.
//
// The paper lists "cross_ent" in its "Supported kernel types" table (regime Memory,
// metric GB/s; its starter keeps a running log-sum-exp and picks the target's logit in
// the same pass) and reports it in the table "Kernel
// performance on H100" (Section 7.1: 4096 x 32k and 8192 x 32k); it prints no formula.
// The definition used here is the standard one, per row i with target class t_i:
//
//     m_i    = max_j X(i,j)
//     s_i    = sum_j exp(X(i,j) - m_i)                     (index order, fp64)
//     lse_i  = m_i + log(s_i)
//     loss_i = round_to_fp32( log(s_i) - (X(i, t_i) - m_i) )      ( = lse_i - X(i, t_i) )
//
// The loss is formed from the max-subtracted pieces, not as lse - X: the two are the
// same number, but lse_i - X(i,t_i) cancels when the logits are large (a row of
// identical values 3e38 would give 0 instead of log N).
//
// X widened exactly to fp64; the loss is fp32 whatever the storage type of X, rounded
// once.  A target outside [0, N) marks an ignored row: its loss is exactly 0.  IEEE
// corner cases follow from the formula: -inf logits drop out of the sum; a target on a
// -inf logit gives +inf; a row holding NaN or +inf, or only -inf, gives NaN.
//
// A running log-sum-exp (running maximum with rescaling) is a way of computing the
// same lse in one pass; the oracle takes the two plain passes.
//
// Pinned by tests/test_crossentropy_oracle_pins.py.
// Build: g++ -O2 -std=c++17 -shared -fPIC -pthread.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum { DT_FP32 = 0, DT_FP16 = 1, DT_BF16 = 2 };

// Logit at flat index k as a double (exact).
double logit(const void* base, int64_t k, int dtype) {
  if (dtype == DT_FP32) {
    float f;
    std::memcpy(&f, static_cast<const char*>(base) + 4 * k, 4);
    return static_cast<double>(f);
  }
  uint16_t h;
  std::memcpy(&h, static_cast<const char*>(base) + 2 * k, 2);
  if (dtype == DT_BF16) {
    const uint32_t wide = static_cast<uint32_t>(h) << 16;   // a bf16 is the top half of an fp32
    float f;
    std::memcpy(&f, &wide, 4);
    return static_cast<double>(f);
  }
  // IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits
  const int sign = h >> 15, ex = (h >> 10) & 31, frac = h & 1023;
  double v;
  if (ex == 31) v = frac ? std::nan("") : INFINITY;
  else if (ex == 0) v = std::ldexp(static_cast<double>(frac), -24);
  else v = std::ldexp(static_cast<double>(frac + 1024), ex - 25);
  return sign ? -v : v;
}

void rows_range(const void* x, const int64_t* target, float* loss, double* lse_out,
                int64_t r0, int64_t r1, int64_t N, int dtype) {
  for (int64_t i = r0; i < r1; ++i) {
    double m = -INFINITY;
    for (int64_t j = 0; j < N; ++j) {
      const double v = logit(x, i * N + j, dtype);
      if (v > m) m = v;                       // NaN never wins a comparison; it shows up in the sum
    }
    double s = 0.0;
    for (int64_t j = 0; j < N; ++j) s += std::exp(logit(x, i * N + j, dtype) - m);
    const double lse = m + std::log(s);
    if (lse_out) lse_out[i] = lse;
    if (!loss) continue;
    const int64_t t = target[i];
    if (t < 0 || t >= N) {
      loss[i] = 0.0f;                         // ignored row
    } else {
      // one rounding, to nearest-even
      loss[i] = static_cast<float>(std::log(s) - (logit(x, i * N + t, dtype) - m));
    }
  }
}

}  // namespace

extern "C" {

// x: HOST, M x N row-major logits of `dtype` (0 fp32, 1 fp16, 2 bf16); target: M int64
// class indices; loss: M floats out (may be NULL if only lse is wanted); lse: optional M
// doubles out.  Returns 0, or -1 on a bad argument.
int crossentropy_oracle(const void* x, const int64_t* target, float* loss, double* lse,
                        int64_t M, int64_t N, int dtype, int nthreads) {
  if (dtype < 0 || dtype > 2 || M < 0 || N <= 0) return -1;
  if (M == 0) return 0;
  if (!x || (!loss && !lse) || (loss && !target)) return -1;
  int64_t nt = nthreads <= 0 ? static_cast<int64_t>(std::thread::hardware_concurrency()) : nthreads;
  if (nt < 1) nt = 1;
  if (nt > M) nt = M;
  if (nt == 1) {
    rows_range(x, target, loss, lse, 0, M, N, dtype);
    return 0;
  }
  std::vector<std::thread> pool;
  const int64_t per = (M + nt - 1) / nt;
  for (int64_t t = 0; t < nt; ++t) {
    const int64_t lo = t * per, hi = (lo + per < M) ? lo + per : M;
    if (lo >= hi) break;
    pool.emplace_back(rows_range, x, target, loss, lse, lo, hi, N, dtype);
  }
  for (auto& th : pool) th.join();
  return 0;
}

}  // extern "C"
