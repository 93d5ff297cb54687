// CPU oracle for row-wise RMSNorm forward.  TEST INFRASTRUCTURE ONLY.
//
// This file is the slow, plain definition that the HIP kernels are checked
// against.  Only the tests, the smoke entry and the benchmark's cpu_baseline
// leg may call it; the product path never does.  It shares no code with the
// GPU side: own decoders, own rounding, own loops.
//
// What it computes (the paper names the operation in its "Supported kernel
// types" table, row "rmsnorm", and in the Section 7.1 key findings, but prints
// no formula; the definition used here is the standard one and is spelled out
// by this project's statement of the task):
//
//     ms_i   = (1/N) * sum_j X(i,j)^2
//     r_i    = 1 / sqrt(ms_i + eps)
//     y(i,j) = round_to_dtype( X(i,j) * r_i * W(j) )
//
// with X, W the inputs widened exactly to fp64, every intermediate in fp64,
// the sum taken in index order j = 0..N-1, and exactly ONE rounding at the
// end (round-to-nearest-even, overflow to infinity, subnormals kept).
//
// Pinned by tests/test_oracle_pins.py against closed forms, exact rational
// arithmetic on small inputs, numpy's own conversions and a library 2-norm.
//
// Build: g++ -O2 -std=c++17 -shared -fPIC -pthread (no -ffast-math: the
// rounding code relies on IEEE semantics).

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum { DT_FP32 = 0, DT_FP16 = 1, DT_BF16 = 2 };

// A binary interchange format: p significand bits (hidden bit included),
// minimum normal exponent emin, exponent field width ebits.
struct Format {
  int p;
  int emin;
  int emax;
  int ebits;
};

constexpr Format kFp32{24, -126, 127, 8};
constexpr Format kFp16{11, -14, 15, 5};
constexpr Format kBf16{8, -126, 127, 8};

// Bit pattern -> value.  Every value of these formats is an fp64 number.
double decode_bits(uint32_t bits, const Format& f) {
  const int mbits = f.p - 1;
  const uint32_t mant = bits & ((1u << mbits) - 1u);
  const uint32_t expo = (bits >> mbits) & ((1u << f.ebits) - 1u);
  const bool neg = (bits >> (mbits + f.ebits)) & 1u;
  double v;
  if (expo == (1u << f.ebits) - 1u) {
    v = mant ? std::nan("") : INFINITY;
  } else if (expo == 0) {
    v = std::ldexp((double)mant, f.emin - mbits);          // subnormal or zero
  } else {
    const int bias = f.emax;
    v = std::ldexp((double)(mant | (1u << mbits)), (int)expo - bias - mbits);
  }
  return neg ? -v : v;
}

// Value -> nearest representable value of the format (ties to even), as fp64.
// One rounding only: the scaling by a power of two is exact, nearbyint rounds
// to nearest-even in the default rounding mode, and scaling back is exact.
double round_to_format(double v, const Format& f) {
  if (std::isnan(v) || std::isinf(v) || v == 0.0) return v;
  const double a = std::fabs(v);
  int e = std::ilogb(a);
  if (e < f.emin) e = f.emin;                               // subnormal spacing
  if (e > f.emax) return std::copysign(INFINITY, v);
  const double q = std::nearbyint(std::ldexp(a, f.p - 1 - e));
  const double r = std::ldexp(q, e - (f.p - 1));
  const double max_finite = std::ldexp(std::ldexp(1.0, f.p) - 1.0, f.emax - (f.p - 1));
  if (r > max_finite) return std::copysign(INFINITY, v);
  return std::copysign(r, v);
}

// Representable value -> bit pattern.
uint32_t encode_bits(double r, const Format& f) {
  const int mbits = f.p - 1;
  const uint32_t sign = std::signbit(r) ? (1u << (mbits + f.ebits)) : 0u;
  const uint32_t emask = (1u << f.ebits) - 1u;
  if (std::isnan(r)) return sign | (emask << mbits) | (1u << (mbits - 1));
  if (std::isinf(r)) return sign | (emask << mbits);
  const double a = std::fabs(r);
  if (a == 0.0) return sign;
  const int e = std::ilogb(a);
  if (e < f.emin) {
    return sign | (uint32_t)std::ldexp(a, mbits - f.emin);  // subnormal: exact integer
  }
  const uint32_t m = (uint32_t)std::ldexp(a, mbits - e);    // in [2^mbits, 2^p)
  return sign | ((uint32_t)(e + f.emax) << mbits) | (m & ((1u << mbits) - 1u));
}

const Format* format_of(int dtype) {
  switch (dtype) {
    case DT_FP32: return &kFp32;
    case DT_FP16: return &kFp16;
    case DT_BF16: return &kBf16;
    default: return nullptr;
  }
}

uint32_t load_bits(const void* base, int64_t idx, int dtype) {
  if (dtype == DT_FP32) {
    uint32_t b;
    std::memcpy(&b, (const char*)base + 4 * idx, 4);
    return b;
  }
  uint16_t h;
  std::memcpy(&h, (const char*)base + 2 * idx, 2);
  return h;
}

void store_bits(void* base, int64_t idx, int dtype, uint32_t bits) {
  if (dtype == DT_FP32) {
    std::memcpy((char*)base + 4 * idx, &bits, 4);
  } else {
    const uint16_t h = (uint16_t)bits;
    std::memcpy((char*)base + 2 * idx, &h, 2);
  }
}

void rows(const void* x, const void* w, void* y, double* rstd_out,
          int64_t row_begin, int64_t row_end, int64_t N, double eps, int dtype) {
  const Format& f = *format_of(dtype);
  std::vector<double> wd((size_t)N);
  for (int64_t j = 0; j < N; ++j) wd[(size_t)j] = decode_bits(load_bits(w, j, dtype), f);
  for (int64_t i = row_begin; i < row_end; ++i) {
    double ss = 0.0;
    for (int64_t j = 0; j < N; ++j) {
      const double xv = decode_bits(load_bits(x, i * N + j, dtype), f);
      ss += xv * xv;
    }
    const double ms = ss / (double)N;
    const double r = 1.0 / std::sqrt(ms + eps);
    if (rstd_out) rstd_out[i] = r;
    if (!y) continue;
    for (int64_t j = 0; j < N; ++j) {
      const double xv = decode_bits(load_bits(x, i * N + j, dtype), f);
      const double v = xv * r * wd[(size_t)j];
      store_bits(y, i * N + j, dtype, encode_bits(round_to_format(v, f), f));
    }
  }
}

int run(const void* x, const void* w, void* y, double* rstd_out,
        int64_t M, int64_t N, double eps, int dtype, int nthreads) {
  if (!format_of(dtype) || M < 0 || N <= 0 || !(eps >= 0.0)) return -1;
  if (M == 0) return 0;
  if (!x || !w || (!y && !rstd_out)) return -1;
  int64_t nt = nthreads <= 0 ? (int64_t)std::thread::hardware_concurrency() : nthreads;
  if (nt < 1) nt = 1;
  if (nt > M) nt = M;
  if (nt == 1) {
    rows(x, w, y, rstd_out, 0, M, N, eps, dtype);
    return 0;
  }
  // Rows are independent, so a contiguous split gives the same bits for any
  // thread count.
  std::vector<std::thread> pool;
  const int64_t per = (M + nt - 1) / nt;
  for (int64_t t = 0; t < nt; ++t) {
    const int64_t b = t * per, e = (b + per < M) ? b + per : M;
    if (b >= e) break;
    pool.emplace_back(rows, x, w, y, rstd_out, b, e, N, eps, dtype);
  }
  for (auto& th : pool) th.join();
  return 0;
}

}  // namespace

extern "C" {

// x, w, y: HOST buffers of `dtype` (0 fp32, 1 fp16, 2 bf16); x and y are M x N
// row-major with leading dimension N, w has N elements.  eps is the fp64
// widening of the float the GPU call receives.  nthreads <= 0 uses all
// hardware threads.  Returns 0, or -1 on a bad argument.
int rmsnorm_oracle(const void* x, const void* w, void* y, int64_t M, int64_t N,
                   double eps, int dtype, int nthreads) {
  if (M > 0 && !y) return -1;
  return run(x, w, y, nullptr, M, N, eps, dtype, nthreads);
}

// The per-row reciprocal RMS r_i in fp64 (an intermediate the tests pin).
int rmsnorm_oracle_rstd(const void* x, double* rstd, int64_t M, int64_t N,
                        double eps, int dtype) {
  if (M > 0 && !rstd) return -1;
  // w is unused when y is null, but run() wants a non-null pointer.
  return run(x, x, nullptr, rstd, M, N, eps, dtype, 1);
}

// Storage bits -> fp64 (exact).
int rmsnorm_oracle_decode(const void* src, double* dst, int64_t n, int dtype) {
  const Format* f = format_of(dtype);
  if (!f || n < 0 || (n > 0 && (!src || !dst))) return -1;
  for (int64_t k = 0; k < n; ++k) dst[k] = decode_bits(load_bits(src, k, dtype), *f);
  return 0;
}

// fp64 -> storage bits with a single round-to-nearest-even.
int rmsnorm_oracle_encode(const double* src, void* dst, int64_t n, int dtype) {
  const Format* f = format_of(dtype);
  if (!f || n < 0 || (n > 0 && (!src || !dst))) return -1;
  for (int64_t k = 0; k < n; ++k)
    store_bits(dst, k, dtype, encode_bits(round_to_format(src[k], *f), *f));
  return 0;
}

int rmsnorm_oracle_hardware_threads(void) {
  const unsigned n = std::thread::hardware_concurrency();
  return n ? (int)n : 1;
}

}  // extern "C"
