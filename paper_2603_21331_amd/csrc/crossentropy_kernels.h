// Row cross-entropy forward (log-sum-exp fused with the target pick) for gfx950 (MI355X).
//
//   loss[i] = log( sum_j exp(x[i, j] - m_i) ) - (x[i, t_i] - m_i),   m_i = max_j x[i, :]
//
// The paper lists the kernel in its "Supported kernel types" table (regime Memory, metric
// GB/s, "online log-sum-exp, fused NLL").  It only reads: every logit crosses HBM once and one
// float per row goes back, so nothing has to stay in registers and rows of any length stream
// through.  Each thread keeps a running maximum and a running sum of exponentials relative to
// it (the online log-sum-exp the paper names), in batches: a batch of U 16-byte vectors is
// loaded at once, its maximum taken first, the running sum rescaled at most once per batch,
// and a subtract, a multiply and one v_exp_f32 spent per element.  The per-thread pairs are
// combined in a fixed order (DPP maximum, rescale, DPP sum, LDS across wavefronts), so results
// are bit-identical from run to run.
//
// Rows are addressed in elements with element-aligned 128-bit loads (single
// global_load_dwordx4 instructions under the amdhsa unaligned-access mode), so odd class
// counts such as 50257 run through the same code; the last N mod VEC logits of a row are
// read one by one.
#pragma once

#include "vec_io.h"
#include "wave_reduce.h"

namespace rms {

constexpr int kCeWave = 64;
constexpr float kCeNegInf = -__builtin_inff();
constexpr float kCeLog2e = 1.44269502162933349609375f;

// 2^((a - b) log2 e) for a <= b, with the convention that equal arguments (including two
// infinities of the same sign) give exactly 1.
__device__ __forceinline__ float ce_rescale(float a, float b) {
  return a == b ? 1.0f : __builtin_amdgcn_exp2f((a - b) * kCeLog2e);
}

// Folds COUNT values into the running (m, s) pair.  Each term is 2^((f - m) log2 e): the
// difference is formed first (exact for the 16-bit types when the exponents are close,
// correctly rounded otherwise), so the error of a term grows with its distance from the
// maximum, where the term is small, and not with the size of the logits; rows of large
// identical values (the paper's stability probe for softmax-like kernels, Section 4 stage 3)
// give exactly COUNT.
template <int COUNT>
__device__ __forceinline__ void ce_fold(const float (&f)[COUNT], float& m, float& s) {
  float bm = m;
#pragma unroll
  for (int k = 0; k < COUNT; ++k) bm = __builtin_fmaxf(bm, f[k]);
  s *= ce_rescale(m, bm);
  m = bm;
  // only -inf so far: every term is exp(-inf) = 0; subtracting 0 keeps -inf - (-inf) from NaN
  const float ref = bm == kCeNegInf ? 0.0f : bm;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < COUNT; ++k) acc[k & 3] += __builtin_amdgcn_exp2f((f[k] - ref) * kCeLog2e);
  s += (acc[0] + acc[1]) + (acc[2] + acc[3]);
}

template <int DT, int G, int U, bool NT>
__global__ void __launch_bounds__(G)
crossentropy_row_kernel(const void* x, const int64_t* __restrict__ target, float* __restrict__ loss,
                        float* __restrict__ lse_out, int64_t M, int64_t N, int nfull) {
  using S = Storage<DT>;
  constexpr int VEC = S::kVec;
  constexpr int WAVES = G / kCeWave;
  __shared__ float part_m[2][WAVES];
  __shared__ float part_s[2][WAVES];
  const int t = threadIdx.x;
  const int lane = t & (kCeWave - 1);
  const int wave = t / kCeWave;
  const int rem = (int)(N - (int64_t)nfull * VEC);
  int slot = 0;

  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const char* xr = static_cast<const char*>(x) + row * N * S::kBytes;
    float m = kCeNegInf, s = 0.f;

    for (int base = t; base < nfull; base += G * U) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = base + u * G;
        if (idx < nfull) v[u] = load_vec_unaligned<NT>(xr + (int64_t)idx * 16);
      }
      float f[U * VEC];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float g[VEC];
        S::unpack(v[u], g);
        const bool live = base + u * G < nfull;
#pragma unroll
        for (int k = 0; k < VEC; ++k) f[u * VEC + k] = live ? g[k] : kCeNegInf;
      }
      ce_fold<U * VEC>(f, m, s);
    }
    if (t < rem) {
      const float tail[1] = {S::load_one(x, row * N + (int64_t)nfull * VEC + t)};
      ce_fold<1>(tail, m, s);
    }

    // combine the per-thread pairs: row maximum, rescale, row sum
    float row_m = wave_max(m);
    if constexpr (WAVES > 1) {
      if (lane == 0) part_m[slot][wave] = row_m;
      __syncthreads();
      row_m = part_m[slot][0];
#pragma unroll
      for (int k = 1; k < WAVES; ++k) row_m = __builtin_fmaxf(row_m, part_m[slot][k]);
    }
    float row_s = wave_sum(s * ce_rescale(m, row_m));
    if constexpr (WAVES > 1) {
      if (lane == 0) part_s[slot][wave] = row_s;
      __syncthreads();
      row_s = part_s[slot][0];
#pragma unroll
      for (int k = 1; k < WAVES; ++k) row_s += part_s[slot][k];
      slot ^= 1;
    }

    if (t == 0) {
      // a row of -inf only has no maximum to subtract: NaN, as the formula gives
      const float log_s = row_m == kCeNegInf ? __builtin_nanf("") : __builtin_logf(row_s);
      if (lse_out) lse_out[row] = row_m + log_s;
      const int64_t cls = target[row];
      float out = 0.0f;                                   // target outside [0, N): ignored row
      if (cls >= 0 && cls < N) out = log_s - (S::load_one(x, row * N + cls) - row_m);
      loss[row] = out;
    }
  }
}

}  // namespace rms
