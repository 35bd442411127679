// Order-independent sign of a SimHash projection (Sec. 2.2 / Sec. 4.3: Sign(w^T x)).
//
// The hash bit is defined as [ sum_d x_d*w_d - sum_d mu_d*w_d >= 0 ] over the stored values,
// in exact real arithmetic.  Every operand is float32-representable, so each product is
// exact in float64.  A float64 accumulation decides the sign whenever the result exceeds a
// rigorous bound on its own rounding error; the rare remainder is summed exactly in a
// fixed-point accumulator by the whole wavefront.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mp {

// 2*128 terms, unit roundoff 2^-53: |fl(sum) - sum| <= 255 * 2^-53 * sum|t| < 2^-45 sum|t|.
// 2^-43 leaves a factor of four.
constexpr double kF64Slack = 1.1368683772161603e-13;   // 2^-43

constexpr int kLimbs = 20;   // 32-bit digits held in int64 cells: covers 2^-298 .. 2^342

// Adds the exact float64 value p (a product of two float32 values, or its negation) into
// the wavefront's fixed-point accumulator in LDS.  Digit i has weight 2^(32 i - 298).
__device__ inline void limb_add(long long* limb, double p) {
  const uint64_t bits = (uint64_t)__double_as_longlong(p);
  const int E = (int)((bits >> 52) & 0x7ff);
  uint64_t M = bits & ((1ull << 52) - 1);
  if (E == 0) return;                       // zero (float64 subnormals cannot occur here)
  M |= 1ull << 52;
  int shift = E - 1075 + 298;               // p = M * 2^(E-1075); lowest possible bit is 2^-298
  if (shift < 0) { M >>= -shift; shift = 0; }   // the dropped bits are zero by construction
  const int idx = shift >> 5, off = shift & 31;
  const uint64_t lo = (M & 0xffffffffull) << off;
  const uint64_t hi = ((M >> 32) << off) + (lo >> 32);
  long long d0 = (long long)(lo & 0xffffffffull);
  long long d1 = (long long)(hi & 0xffffffffull);
  long long d2 = (long long)(hi >> 32);
  if (bits >> 63) { d0 = -d0; d1 = -d1; d2 = -d2; }
  if (d0) atomicAdd((unsigned long long*)&limb[idx], (unsigned long long)d0);
  if (d1) atomicAdd((unsigned long long*)&limb[idx + 1], (unsigned long long)d1);
  if (d2) atomicAdd((unsigned long long*)&limb[idx + 2], (unsigned long long)d2);
}

// Whole wavefront: exact [ x.w - mu.w >= 0 ] for one 128-long projection.  xv/wv/mv are
// callables d -> float64 value of element d (mv may return 0).  `limb` is this wavefront's
// kLimbs-cell LDS array, all zero on entry and on exit.  Returns the same value in all lanes.
template <class FX, class FW, class FM>
__device__ inline bool exact_sign_nonneg_wave(long long* limb, FX xv, FW wv, FM mv, bool has_mu) {
  const int lane = threadIdx.x & 63;
  for (int d = lane; d < 128; d += 64) {
    const double w = wv(d);
    limb_add(limb, xv(d) * w);
    if (has_mu) limb_add(limb, -(mv(d) * w));
  }
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  int negative = 0;
  if (lane == 0) {
    long long carry = 0;
    for (int i = 0; i < kLimbs; ++i) {
      const long long t = limb[i] + carry;
      carry = t >> 32;                      // floor division: digits stay in [0, 2^32)
      limb[i] = 0;
    }
    negative = carry < 0;                   // value = carry*2^(32*kLimbs) + (digits >= 0)
  }
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  return __shfl(negative, 0) == 0;
}

}  // namespace mp
