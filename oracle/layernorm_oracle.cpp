// CPU oracle for row-wise LayerNorm forward.  TEST INFRASTRUCTURE ONLY.
//
// Only the tests, the smoke entry and the benchmark's cpu_baseline leg may call
// it; the product path never does.  It shares no code with the GPU side or with
// the other oracle files.
//
// The paper lists "layernorm" in its "Supported kernel types" table (regime
// Memory, metric GB/s; its starter takes one pass with Welford's recurrence) and reports it in the
// table "Kernel performance on H100" (Section 7.1); it prints no formula.  The
// definition used here is the standard one, written as its plain two-pass form
// (Welford's recurrence is a way of computing the same two moments in one pass;
// the oracle has no reason to use it):
//
//     mu_i   = (1/N) sum_j X(i,j)
//     var_i  = (1/N) sum_j (X(i,j) - mu_i)^2            (biased, divide by N)
//     y(i,j) = round_to_dtype( (X(i,j) - mu_i) / sqrt(var_i + eps) * W(j) + B(j) )
//
// X, W, B widened exactly to fp64, sums in index order, ONE rounding at the end
// (nearest-even, overflow to infinity, subnormals kept).  B may be absent.
//
// Pinned by tests/test_layernorm_oracle_pins.py.
// Build: g++ -O2 -std=c++17 -shared -fPIC -pthread.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum { DT_FP32 = 0, DT_FP16 = 1, DT_BF16 = 2 };

struct Layout {
  int sig;     // significand bits with the hidden bit
  int e_lo;    // smallest normal exponent
  int e_hi;    // largest exponent, equal to the bias
  int e_bits;  // width of the exponent field
};

bool layout_of(int dtype, Layout* out) {
  switch (dtype) {
    case DT_FP32: *out = Layout{24, -126, 127, 8}; return true;
    case DT_FP16: *out = Layout{11, -14, 15, 5}; return true;
    case DT_BF16: *out = Layout{8, -126, 127, 8}; return true;
    default: return false;
  }
}

uint32_t get_bits(const void* base, int64_t idx, int dtype) {
  if (dtype == DT_FP32) {
    uint32_t b;
    std::memcpy(&b, static_cast<const char*>(base) + 4 * idx, 4);
    return b;
  }
  uint16_t h;
  std::memcpy(&h, static_cast<const char*>(base) + 2 * idx, 2);
  return h;
}

void put_bits(void* base, int64_t idx, int dtype, uint32_t bits) {
  if (dtype == DT_FP32) {
    std::memcpy(static_cast<char*>(base) + 4 * idx, &bits, 4);
  } else {
    const uint16_t h = static_cast<uint16_t>(bits);
    std::memcpy(static_cast<char*>(base) + 2 * idx, &h, 2);
  }
}

double to_double(uint32_t bits, const Layout& L) {
  const int frac_bits = L.sig - 1;
  const uint32_t frac = bits & ((1u << frac_bits) - 1u);
  const uint32_t ex = (bits >> frac_bits) & ((1u << L.e_bits) - 1u);
  const bool minus = (bits >> (frac_bits + L.e_bits)) & 1u;
  double v;
  if (ex == (1u << L.e_bits) - 1u) v = frac ? std::nan("") : INFINITY;
  else if (ex == 0) v = std::ldexp(static_cast<double>(frac), L.e_lo - frac_bits);
  else v = std::ldexp(static_cast<double>(frac | (1u << frac_bits)), static_cast<int>(ex) - L.e_hi - frac_bits);
  return minus ? -v : v;
}

// One round-to-nearest-even from fp64 straight to the target's bit pattern.
uint32_t from_double(double v, const Layout& L) {
  const int frac_bits = L.sig - 1;
  const uint32_t all_ones = (1u << L.e_bits) - 1u;
  const uint32_t sign = std::signbit(v) ? (1u << (frac_bits + L.e_bits)) : 0u;
  if (std::isnan(v)) return (all_ones << frac_bits) | (1u << (frac_bits - 1));
  if (std::isinf(v)) return sign | (all_ones << frac_bits);
  const double a = std::fabs(v);
  if (a == 0.0) return sign;
  int e = std::ilogb(a);
  if (e > L.e_hi) return sign | (all_ones << frac_bits);
  if (e < L.e_lo) e = L.e_lo;
  double q = std::nearbyint(std::ldexp(a, frac_bits - e));   // exact scaling, one rounding
  if (q >= std::ldexp(1.0, L.sig)) {                          // carried into the next binade
    q = std::ldexp(1.0, frac_bits);
    e += 1;
    if (e > L.e_hi) return sign | (all_ones << frac_bits);
  }
  if (q < std::ldexp(1.0, frac_bits)) return sign | static_cast<uint32_t>(q);   // subnormal
  return sign | (static_cast<uint32_t>(e + L.e_hi) << frac_bits) |
         (static_cast<uint32_t>(q) & ((1u << frac_bits) - 1u));
}

void do_rows(const void* x, const void* w, const void* b, void* y, double* mean_out,
             double* rstd_out, int64_t r0, int64_t r1, int64_t N, double eps, int dtype) {
  Layout L{24, -126, 127, 8};
  layout_of(dtype, &L);
  std::vector<double> wv(static_cast<size_t>(N)), bv(static_cast<size_t>(N), 0.0);
  for (int64_t j = 0; j < N; ++j) {
    wv[static_cast<size_t>(j)] = to_double(get_bits(w, j, dtype), L);
    if (b) bv[static_cast<size_t>(j)] = to_double(get_bits(b, j, dtype), L);
  }
  for (int64_t i = r0; i < r1; ++i) {
    double total = 0.0;
    for (int64_t j = 0; j < N; ++j) total += to_double(get_bits(x, i * N + j, dtype), L);
    const double mu = total / static_cast<double>(N);
    double spread = 0.0;
    for (int64_t j = 0; j < N; ++j) {
      const double c = to_double(get_bits(x, i * N + j, dtype), L) - mu;
      spread += c * c;
    }
    const double var = spread / static_cast<double>(N);
    const double rstd = 1.0 / std::sqrt(var + eps);
    if (mean_out) mean_out[i] = mu;
    if (rstd_out) rstd_out[i] = rstd;
    if (!y) continue;
    for (int64_t j = 0; j < N; ++j) {
      const double c = to_double(get_bits(x, i * N + j, dtype), L) - mu;
      const double out = c * rstd * wv[static_cast<size_t>(j)] + bv[static_cast<size_t>(j)];
      put_bits(y, i * N + j, dtype, from_double(out, L));
    }
  }
}

}  // namespace

extern "C" {

// x, y: HOST, M x N row-major; w: N elements; b: N elements or NULL (no bias); all of
// `dtype` (0 fp32, 1 fp16, 2 bf16).  mean / rstd: optional fp64 outputs of M entries
// (NULL to skip; y may be NULL when only the statistics are wanted).  eps is the fp64
// widening of the float the GPU call receives.  Returns 0, or -1 on a bad argument.
int layernorm_oracle(const void* x, const void* w, const void* b, void* y, double* mean,
                     double* rstd, int64_t M, int64_t N, double eps, int dtype, int nthreads) {
  Layout L{24, -126, 127, 8};
  if (!layout_of(dtype, &L) || M < 0 || N <= 0 || !(eps >= 0.0)) return -1;
  if (M == 0) return 0;
  if (!x || !w || (!y && !mean && !rstd)) return -1;
  int64_t nt = nthreads <= 0 ? static_cast<int64_t>(std::thread::hardware_concurrency()) : nthreads;
  if (nt < 1) nt = 1;
  if (nt > M) nt = M;
  if (nt == 1) {
    do_rows(x, w, b, y, mean, rstd, 0, M, N, eps, dtype);
    return 0;
  }
  std::vector<std::thread> pool;
  const int64_t per = (M + nt - 1) / nt;
  for (int64_t t = 0; t < nt; ++t) {
    const int64_t lo = t * per, hi = (lo + per < M) ? lo + per : M;
    if (lo >= hi) break;
    pool.emplace_back(do_rows, x, w, b, y, mean, rstd, lo, hi, N, eps, dtype);
  }
  for (auto& th : pool) th.join();
  return 0;
}

}  // extern "C"
