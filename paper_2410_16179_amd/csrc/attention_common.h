// Pieces shared by the decode kernels: inclusion probability, code-block loads.
#pragma once
#include "mp_common.h"
#include "device_utils.h"

namespace mp {

typedef const uint32_t __attribute__((address_space(4))) * const_u32_ptr;

// u = P[Binomial(L, x) >= tau], x = p^K, in float32 without cancellation: the complement
// 1 - P[< tau] when that is below one half, otherwise the positive upper-tail terms.  The
// hardware exp2/log2/rcp based intrinsics are accurate to about 1e-6 relative here, which
// moves log u by about 1e-5: two orders below the output tolerance.
__device__ inline float inclusion_probability(float cosv, int K, int L, int tau) {
  const float c = fminf(fmaxf(cosv, -1.f), 1.f);
  const float p = 1.f - acosf(c) * 0.31830988618379067f;
  float x = 1.f;
  for (int i = 0; i < K; ++i) x *= p;
  if (x >= 1.f) return L >= tau ? 1.f : 0.f;
  if (!(x > 0.f)) return 0.f;
  const float r = __fdividef(x, 1.f - x);
  float t = __expf((float)L * log1pf(-x));   // term j = 0
  float head = 0.f;
  for (int j = 0; j < tau; ++j) {
    head += t;
    t *= (float)(L - j) * __frcp_rn((float)(j + 1)) * r;
  }
  if (head < 0.5f) return 1.f - head;
  float sum = 0.f;
  for (int j = tau; j <= L; ++j) {
    sum += t;
    t *= (float)(L - j) * __frcp_rn((float)(j + 1)) * r;
    if (t < 1e-9f * sum) break;
  }
  return sum;
}

// Code words are read once per decode step: the non-temporal hint keeps them from displacing
// the rest of the working set in L2 (measured: about 7 % faster scan).
template <int NW>
__device__ inline void load_code_block(const uint32_t* blkp, int lane, uint32_t (&kw)[NW]) {
  constexpr int full = NW / 4, rem = NW % 4;
#pragma unroll
  for (int g4 = 0; g4 < full; ++g4) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(blkp + g4 * 256 + lane * 4));
    kw[4 * g4] = v.x; kw[4 * g4 + 1] = v.y; kw[4 * g4 + 2] = v.z; kw[4 * g4 + 3] = v.w;
  }
  if constexpr (rem == 1) {
    kw[4 * full] = blkp[full * 256 + lane];
  } else if constexpr (rem == 2) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(blkp + full * 256 + lane * 2));
    kw[4 * full] = v.x; kw[4 * full + 1] = v.y;
  } else if constexpr (rem == 3) {
    kw[4 * full] = blkp[full * 256 + lane * 3];
    kw[4 * full + 1] = blkp[full * 256 + lane * 3 + 1];
    kw[4 * full + 2] = blkp[full * 256 + lane * 3 + 2];
  }
}

}  // namespace mp
