// CPU oracle for row-wise softmax forward.  TEST INFRASTRUCTURE ONLY.
//
// Only the tests, the smoke entry and the benchmark's cpu_baseline leg may call
// it; the product path never does.  It shares no code with the GPU side and none
// with the RMSNorm oracle either: each oracle file stands alone.
//
// The paper lists "softmax" in its "Supported kernel types" table (regime Memory,
// metric GB/s; its starter reduces with lane shuffles over two-element fp16 loads),
// reports it in the table "Kernel performance on H100" (Section 7.1) and names its
// stability probe, a row whose entries are all one large value, in Section 4 stage 3;
// it prints no formula.
// The definition used here is the standard one:
//
//     m_i    = max_j X(i,j)
//     s_i    = sum_j exp(X(i,j) - m_i)          (index order, fp64)
//     y(i,j) = round_to_dtype( exp(X(i,j) - m_i) / s_i )
//
// with X widened exactly to fp64 and ONE rounding at the end (nearest-even,
// subnormals kept).  IEEE corner cases follow from the formula: an entry of
// -inf gives 0; a row holding +inf or only -inf gives NaN (inf - inf); a NaN
// anywhere in the row makes the whole row NaN.
//
// Pinned by tests/test_softmax_oracle_pins.py (closed forms, invariants, an
// arbitrary-precision reference).  Build: g++ -O2 -std=c++17 -shared -fPIC -pthread.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum { DT_FP32 = 0, DT_FP16 = 1, DT_BF16 = 2 };

struct Format {
  int p;      // significand bits, hidden bit included
  int emin;   // minimum normal exponent
  int emax;   // maximum exponent (= bias)
  int ebits;  // exponent field width
};

constexpr Format kFp32{24, -126, 127, 8};
constexpr Format kFp16{11, -14, 15, 5};
constexpr Format kBf16{8, -126, 127, 8};

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

double widen(uint32_t bits, const Format& f) {
  const int mbits = f.p - 1;
  const uint32_t mant = bits & ((1u << mbits) - 1u);
  const uint32_t expo = (bits >> mbits) & ((1u << f.ebits) - 1u);
  const bool neg = (bits >> (mbits + f.ebits)) & 1u;
  double v;
  if (expo == (1u << f.ebits) - 1u) v = mant ? std::nan("") : INFINITY;
  else if (expo == 0) v = std::ldexp((double)mant, f.emin - mbits);
  else v = std::ldexp((double)(mant | (1u << mbits)), (int)expo - f.emax - mbits);
  return neg ? -v : v;
}

// Nearest representable value (ties to even) and its bit pattern.  Softmax
// outputs lie in [0, 1], so overflow cannot occur; NaN is kept.
uint32_t narrow(double v, const Format& f) {
  const int mbits = f.p - 1;
  const uint32_t emask = (1u << f.ebits) - 1u;
  const uint32_t sign = std::signbit(v) ? (1u << (mbits + f.ebits)) : 0u;
  if (std::isnan(v)) return (emask << mbits) | (1u << (mbits - 1));
  if (std::isinf(v)) return sign | (emask << mbits);
  const double a = std::fabs(v);
  if (a == 0.0) return sign;
  int e = std::ilogb(a);
  if (e < f.emin) e = f.emin;
  double q = std::nearbyint(std::ldexp(a, mbits - e));     // in [0, 2^p]
  if (q == std::ldexp(1.0, f.p)) {                          // carried into the next binade
    q = std::ldexp(1.0, mbits);
    e += 1;
  }
  if (e > f.emax) return sign | (emask << mbits);
  if (q < std::ldexp(1.0, mbits)) return sign | (uint32_t)q;  // subnormal (e == emin)
  return sign | ((uint32_t)(e + f.emax) << mbits) | ((uint32_t)q & ((1u << mbits) - 1u));
}

void rows(const void* x, void* y, int64_t row_begin, int64_t row_end, int64_t N, int dtype) {
  const Format& f = *format_of(dtype);
  std::vector<double> e((size_t)N);
  for (int64_t i = row_begin; i < row_end; ++i) {
    double m = -INFINITY;
    bool has_nan = false;
    for (int64_t j = 0; j < N; ++j) {
      const double v = widen(load_bits(x, i * N + j, dtype), f);
      if (std::isnan(v)) has_nan = true;
      else if (v > m) m = v;
    }
    double s = 0.0;
    for (int64_t j = 0; j < N; ++j) {
      const double v = widen(load_bits(x, i * N + j, dtype), f);
      e[(size_t)j] = std::exp(v - m);          // -inf - -inf and inf - inf give NaN, as IEEE says
      s += e[(size_t)j];
    }
    for (int64_t j = 0; j < N; ++j) {
      const double out = has_nan ? std::nan("") : e[(size_t)j] / s;
      store_bits(y, i * N + j, dtype, narrow(out, f));
    }
  }
}

}  // namespace

extern "C" {

// x, y: HOST buffers, M x N row-major, dtype 0 fp32 / 1 fp16 / 2 bf16.
// nthreads <= 0 uses all hardware threads.  Returns 0, or -1 on a bad argument.
int softmax_oracle(const void* x, void* y, int64_t M, int64_t N, int dtype, int nthreads) {
  if (!format_of(dtype) || M < 0 || N <= 0) return -1;
  if (M == 0) return 0;
  if (!x || !y) return -1;
  int64_t nt = nthreads <= 0 ? (int64_t)std::thread::hardware_concurrency() : nthreads;
  if (nt < 1) nt = 1;
  if (nt > M) nt = M;
  if (nt == 1) {
    rows(x, y, 0, M, N, dtype);
    return 0;
  }
  std::vector<std::thread> pool;
  const int64_t per = (M + nt - 1) / nt;
  for (int64_t t = 0; t < nt; ++t) {
    const int64_t b = t * per, e = (b + per < M) ? b + per : M;
    if (b >= e) break;
    pool.emplace_back(rows, x, y, b, e, N, dtype);
  }
  for (auto& th : pool) th.join();
  return 0;
}

int softmax_oracle_hardware_threads(void) {
  const unsigned n = std::thread::hardware_concurrency();
  return n ? (int)n : 1;
}

}  // extern "C"
