// Small device helpers shared by the gfx950 kernels: row fragment loads and
// wavefront / 16-lane reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mp {

// Element types of the tensors.  The helpers below take one as template argument; a `bool FP32`
// converts to kBF16 / kFP32.  kFP8: OCP e4m3 bytes (value = the decoded byte, no scale), a storage
// type of the K / V cache only; every e4m3 value is a bf16 value.
enum : int { kBF16 = 0, kFP32 = 1, kFP8 = 2 };

typedef float mp_f32x2 __attribute__((ext_vector_type(2)));
// eight e4m3 bytes -> eight floats (v_cvt_pk_f32_fp8: two per instruction)
__device__ inline void fp8x8_to_float(uint32_t lo, uint32_t hi, float (&v)[8]) {
  const mp_f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)lo, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)lo, true);
  const mp_f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)hi, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)hi, true);
  v[0] = a.x; v[1] = a.y; v[2] = b.x; v[3] = b.y; v[4] = c.x; v[5] = c.y; v[6] = d.x; v[7] = d.y;
}
// eight e4m3 bytes -> the same eight values as bf16 (exact: e4m3 has 3 mantissa bits), packed
__device__ inline uint4 fp8x8_to_bf16x8(uint32_t lo, uint32_t hi) {
  float v[8];
  fp8x8_to_float(lo, hi, v);
  uint4 r;
  r.x = (__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xffff0000u);
  r.y = (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xffff0000u);
  r.z = (__float_as_uint(v[4]) >> 16) | (__float_as_uint(v[5]) & 0xffff0000u);
  r.w = (__float_as_uint(v[6]) >> 16) | (__float_as_uint(v[7]) & 0xffff0000u);
  return r;
}
__device__ inline float fp8_to_float(uint8_t b) {
  const mp_f32x2 v = __builtin_amdgcn_cvt_pk_f32_fp8((int)(uint32_t)b, false);
  return v.x;
}
// bytes per element
__host__ __device__ inline int elem_bytes(int et) { return et == kFP32 ? 4 : (et == kFP8 ? 1 : 2); }

// Eight consecutive elements of a 128-element row, as stored (e4m3: 8 bytes in a.x, a.y; bf16: 16
// bytes; float32: 32).
struct Frag {
  uint4 a, b;
};

// The rows of a decode step are read once: non-temporal loads.
template <int ET>
__device__ inline void frag_load(const void* base, int64_t elem, Frag& f) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  if constexpr (ET == kFP8) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 a = __builtin_nontemporal_load(
        reinterpret_cast<const u32x2*>(reinterpret_cast<const uint8_t*>(base) + elem));
    f.a.x = a.x; f.a.y = a.y;
  } else if constexpr (ET == kFP32) {
    const u32x4* p = reinterpret_cast<const u32x4*>(reinterpret_cast<const float*>(base) + elem);
    const u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 1);
    f.a = make_uint4(a.x, a.y, a.z, a.w);
    f.b = make_uint4(b.x, b.y, b.z, b.w);
  } else {
    const u32x4 a = __builtin_nontemporal_load(
        reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(base) + elem));
    f.a = make_uint4(a.x, a.y, a.z, a.w);
  }
}

template <int ET>
__device__ inline void frag_zero(Frag& f) {
  f.a = make_uint4(0, 0, 0, 0);
  if constexpr (ET == kFP32) f.b = make_uint4(0, 0, 0, 0);
}

template <int ET>
__device__ inline void frag_to_float(const Frag& f, float (&v)[8]) {
  if constexpr (ET == kFP8) {
    fp8x8_to_float(f.a.x, f.a.y, v);
  } else if constexpr (ET == kFP32) {
    v[0] = __uint_as_float(f.a.x); v[1] = __uint_as_float(f.a.y);
    v[2] = __uint_as_float(f.a.z); v[3] = __uint_as_float(f.a.w);
    v[4] = __uint_as_float(f.b.x); v[5] = __uint_as_float(f.b.y);
    v[6] = __uint_as_float(f.b.z); v[7] = __uint_as_float(f.b.w);
  } else {
    const uint32_t u[4] = {f.a.x, f.a.y, f.a.z, f.a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(u[i] << 16);
      v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
}

// Eight consecutive elements starting at element index `elem`, converted to float32.
template <int ET>
__device__ inline void load8(const void* base, int64_t elem, float (&v)[8]) {
  if constexpr (ET == kFP8) {
    const uint2 r = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint8_t*>(base) + elem);
    fp8x8_to_float(r.x, r.y, v);
  } else if constexpr (ET == kFP32) {
    const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem);
    const float4 a = p[0], b = p[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  } else {
    const uint4 r = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + elem);
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] = __uint_as_float(u[i] << 16);
      v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
}

// Sum over the 16 lanes of a DPP row (rotate-and-add); every lane of the row gets the total.
template <int N>
__device__ inline float dpp_row_ror(float v) {
  const int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf, false);
  return __builtin_bit_cast(float, r);
}
__device__ inline float row_sum16(float v) {
  v += dpp_row_ror<8>(v);
  v += dpp_row_ror<4>(v);
  v += dpp_row_ror<2>(v);
  v += dpp_row_ror<1>(v);
  return v;
}

// Inclusive prefix sums over the lanes of every row of 16 lanes (row shifts, zeros shifted in), and
// over lanes 0 .. 31 and 32 .. 63 (the total of an even row joins the row behind it).
__device__ inline int row_prefix_sum16(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);
  return v;
}
__device__ inline int half_prefix_sum32(int v) {
  v = row_prefix_sum16(v);
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // lane 15 of rows 0 and 2 to rows 1 and 3
  return v;
}

// Lane n (0 .. 15) of every row of 16 lanes, in all lanes of that row.
template <int N>
__device__ inline float dpp_row_bcast(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x150 + N, 0xf, 0xf, false));
}
__device__ inline float row_bcast16(float v, int n) {      // n: a constant after unrolling
  switch (n) {
    case 0: return dpp_row_bcast<0>(v);   case 1: return dpp_row_bcast<1>(v);   case 2: return dpp_row_bcast<2>(v);
    case 3: return dpp_row_bcast<3>(v);   case 4: return dpp_row_bcast<4>(v);   case 5: return dpp_row_bcast<5>(v);
    case 6: return dpp_row_bcast<6>(v);   case 7: return dpp_row_bcast<7>(v);   case 8: return dpp_row_bcast<8>(v);
    case 9: return dpp_row_bcast<9>(v);   case 10: return dpp_row_bcast<10>(v); case 11: return dpp_row_bcast<11>(v);
    case 12: return dpp_row_bcast<12>(v); case 13: return dpp_row_bcast<13>(v); case 14: return dpp_row_bcast<14>(v);
    default: return dpp_row_bcast<15>(v);
  }
}

template <int N>
__device__ inline float dpp_row_ror_keep(float v) {
  const int r = __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf, false);
  return __builtin_bit_cast(float, r);
}
// Wavefront-wide max / sum: DPP rotations inside each 16-lane row, then the four row results
// are read through scalar registers (no LDS crossbar round trips).
__device__ inline float wave_max(float v) {
  v = fmaxf(v, dpp_row_ror_keep<8>(v));
  v = fmaxf(v, dpp_row_ror_keep<4>(v));
  v = fmaxf(v, dpp_row_ror_keep<2>(v));
  v = fmaxf(v, dpp_row_ror_keep<1>(v));
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ inline float wave_sum(float v) {
  v = row_sum16(v);
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

}  // namespace mp
