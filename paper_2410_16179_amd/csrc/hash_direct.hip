// Direct SimHash coding with an exact fallback (Sec. 2.2; Algorithm 1 "Encode").
//
// Used for the decode queries (a few thousand projections), for float32 inputs, and as the
// reference-accurate path for bf16 keys when the matrix-core kernel cannot be used.  A
// projection is accumulated in float64 from exact products (hash_rows_kernel: in float32
// first, float64 only where the float32 error bound leaves the sign open); results inside
// the float64 error bound are re-summed exactly (exact_dot.h), so the bits do not depend on
// summation order.
#include <type_traits>
#include "mp_common.h"
#include "exact_dot.h"
#include "device_utils.h"
#include <hip/hip_bf16.h>
#include <hip/hip_ext.h>

namespace mp {

template <bool FP32>
__device__ inline double load_elem(const void* p, int64_t idx) {
  if constexpr (FP32) return (double)reinterpret_cast<const float*>(p)[idx];
  const uint32_t b = reinterpret_cast<const uint16_t*>(p)[idx];
  return (double)__uint_as_float(b << 16);
}
// element idx of the vectors X of a call: as above, or an e4m3 byte of a quantised K cache
template <bool FP32>
__device__ inline double load_x_elem(const HashDirectArgs& a, int64_t idx) {
  if constexpr (!FP32) {
    if (a.x_fp8) return (double)fp8_to_float(reinterpret_cast<const uint8_t*>(a.X)[idx]);
  }
  return load_elem<FP32>(a.X, idx);
}
template <bool FP32>
__device__ inline void load_x8(const HashDirectArgs& a, int64_t idx, float (&v)[8]) {
  if constexpr (!FP32) {
    if (a.x_fp8) { load8<kFP8>(a.X, idx, v); return; }
  }
  load8<FP32>(a.X, idx, v);
}

// One wavefront codes two vectors at a time: lanes 0..31 take tables 32w..32w+31 of the
// first, lanes 32..63 of the second; a ballot turns the 64 sign tests into two code words.
template <bool FP32>
__global__ __launch_bounds__(256) void hash_direct_kernel(HashDirectArgs a) {
  __shared__ long long limbs[4][kLimbs];
  if (a.run_flag && *a.run_flag == 0) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane < kLimbs) limbs[wave][lane] = 0;
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();

  const int half = lane >> 5, beta = lane & 31;
  // workgroups walk the groups of eight vectors (one step unless the grid was capped)
  for (int64_t grp = blockIdx.x; grp * 8 < a.total_rows; grp += gridDim.x) {
  const int64_t row0 = (grp * 4 + wave) * 2;
  if (row0 >= a.total_rows) continue;
  const int64_t row = row0 + half;
  const bool row_ok = row < a.total_rows;
  const int64_t rr = row_ok ? row : row0;
  const int64_t unit = rr / a.n_keys;
  const int64_t key = a.first_key + rr % a.n_keys;
  const int64_t xbase = (unit / a.n_kv_heads) * a.stride_b + (unit % a.n_kv_heads) * a.stride_h +
                        key * a.stride_n;
  const float* mu = a.mu ? a.mu + unit * kHeadDim : nullptr;
  const int ncol = a.K * a.L;
  const int Wd = table_words(a.L);

  // plane word x of this lane half's vector (tables 32w .. 32w+31, bit b)
  auto plane = [&](int x) -> uint32_t {
    const int w = x / a.K, b = x % a.K;
    const int t = 32 * w + beta;
    const bool col_ok = t < a.L;
    const int j = col_ok ? t * a.K + b : 0;
    double s = 0.0, mag = 0.0;
    // All 128 projector elements of the column and the whole vector are requested before any
    // is used (their addresses do not depend on data), so the dot product costs one memory
    // round trip; the vector is read as 16-byte pieces shared by the 32 lanes of its half.
    {
      float wf[kHeadDim], xf[kHeadDim];
#pragma unroll
      for (int i = 0; i < kHeadDim; ++i) {
        if constexpr (FP32) {
          wf[i] = reinterpret_cast<const float*>(a.W)[(int64_t)i * ncol + j];
        } else {
          wf[i] = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(a.W)[(int64_t)i * ncol + j] << 16);
        }
      }
#pragma unroll
      for (int i = 0; i < kHeadDim; i += 8) {
        float v[8];
        load_x8<FP32>(a, xbase + i, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) xf[i + e] = v[e];
      }
#pragma unroll
      for (int i = 0; i < kHeadDim; ++i) {
        const double wv = (double)wf[i];
        const double p = (double)xf[i] * wv;
        s += p;
        mag += fabs(p);
        if (mu) {
          const double pm = (double)mu[i] * wv;
          s -= pm;
          mag += fabs(pm);
        }
      }
    }
    bool bit = s >= 0.0;
    bool unsure = col_ok && row_ok && mag > 0.0 && fabs(s) <= kF64Slack * mag;
    uint64_t pending = __ballot(unsure);
    while (pending) {
      const int src = __ffsll((unsigned long long)pending) - 1;
      const int64_t sx = __shfl((int)(xbase >> 32), src);   // 64-bit broadcast in two halves
      const int64_t sxl = (uint32_t)__shfl((int)(xbase & 0xffffffff), src);
      const int64_t xb = (sx << 32) | sxl;
      const int sj = __shfl(j, src);
      const int64_t su = ((int64_t)__shfl((int)(unit >> 32), src) << 32) |
                         (uint32_t)__shfl((int)(unit & 0xffffffff), src);
      const float* smu = a.mu ? a.mu + su * kHeadDim : nullptr;
      const bool r = exact_sign_nonneg_wave(
          limbs[wave],
          [&](int d) { return load_x_elem<FP32>(a, xb + d); },
          [&](int d) { return load_elem<FP32>(a.W, (int64_t)d * ncol + sj); },
          [&](int d) { return smu ? (double)smu[d] : 0.0; }, smu != nullptr);
      if (lane == src) bit = r;
      pending &= pending - 1;
    }
    const uint64_t m = __ballot(bit && col_ok);
    uint32_t word = half ? (uint32_t)(m >> 32) : (uint32_t)m;
    if (a.query_layout && (w == Wd - 1) && (a.L & 31)) word |= ~0u << (a.L & 31);
    return word;
  };
  uint32_t* kdst = a.codes + (unit * a.blocks_cap + key / kBlockKeys) * (kBlockKeys * (int64_t)a.NW);
  auto store_key_word = [&](int x, uint32_t word) {
    if (beta == 0 && row_ok) kdst[slot_in_block(a.NW, x, (int)(key % kBlockKeys))] = word;
  };
  // blockIdx.y walks the items of a vector - its plane words, and for keys the densely packed
  // last table group as one item - so that the few vectors of a small call are spread over
  // the chip.
  const int xs = a.query_layout ? a.NQ : tail_begin(a.K, a.L);
  const int nitems = a.query_layout ? a.NQ : xs + 1;
  for (int it = blockIdx.y; it < nitems; it += gridDim.y) {
    if (it < xs) {
      const uint32_t word = plane(it);
      if (a.query_layout) {
        if (beta == 0 && row_ok) a.codes[row * a.NQ + it] = word;
      } else {
        store_key_word(it, word);
      }
    } else {                                             // keys: the K planes of the last group, packed
      BitString bs;
      int xo = xs;
      for (int b = 0; b < a.K; ++b) {
        uint32_t full;
        if (bs.append(plane(xs + b), tail_tables(a.L), &full)) store_key_word(xo++, full);
      }
      if (bs.nbits > 0) store_key_word(xo, (uint32_t)bs.acc);
    }
  }
  }
}

// Coding of a few vectors: the queries of a decode step (Algorithm 1 "Encode(q, W)") or the
// keys appended to the cache since the last call.  One workgroup codes two vectors against the
// 32*K projector columns of one table word (one vector when it has a centering vector).
// Thread = column, so the 128 loads of a column are coalesced across the workgroup and all in
// flight at once; the vectors are staged in LDS and read back as broadcasts.  Sign bits go
// through LDS
// to be regrouped from column order (table-major) into the bit-plane words of the code layout.
// A launch takes two sets of vectors (the first `pairs0` rows of the grid code a0's, the rest
// a1's), so that a decode step codes its queries and its new keys together.
// QUAD (the number of columns K*L is a multiple of four): a lane loads four neighbouring columns
// of a row at once, 16 lanes cover the 64 columns of the wavefront, and the four 16-lane groups
// take a quarter of the rows each (group g the rows 32 g .. 32 g + 31): a quarter of the load
// instructions for the same bytes.  The partial sums of the four groups are added at the end and
// lane (g, i) keeps column 4 i + g of the wavefront.
template <bool FP32, bool QUAD>
__global__ __launch_bounds__(512) void hash_rows_kernel(HashDirectArgs a0, HashDirectArgs a1, int pairs0) {
  __shared__ long long limbs[8][kLimbs];
  __shared__ unsigned char sbit[2][512];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  if (lane < kLimbs) limbs[wave][lane] = 0;
  const int w = blockIdx.x;
  const bool second = (int)blockIdx.y >= pairs0;
  const HashDirectArgs& a = second ? a1 : a0;
  // keys of a decode step whose context length lives in device memory: the newest n_keys keys
  const int64_t first_key = a.n_dev ? *a.n_dev - a.n_keys : a.first_key;
  if (a.n_dev && (first_key < 0 || first_key + a.n_keys > a.n_cap)) return;   // (uniform in the workgroup)
  // vectors with a centering term cost twice the arithmetic: they are taken one per workgroup
  const int per_wg = a.mu ? 1 : 2;
  const int64_t r0 = (int64_t)((int)blockIdx.y - (second ? pairs0 : 0)) * per_wg;
  const int nrow = a.total_rows - r0 >= per_wg ? per_wg : 1;
  const int ncol = a.K * a.L;
  // column of this thread inside the 32 K columns of the table word
  const int cid = QUAD ? wave * 64 + 4 * (lane & 15) + (lane >> 4) : tid;
  const int t = 32 * w + cid / a.K, b = cid % a.K;
  const bool col_ok = cid < 32 * a.K && t < a.L;
  const int j = col_ok ? t * a.K + b : 0;
  // 32-bit element offsets from the (uniform) projector base keep the 128 addresses cheap
  // wavefronts whose 64 threads all lie behind the last column (K < 16: 32 K < 512) neither load
  // nor multiply: the column loads of a workgroup are what its compute unit issues longest
  const bool wave_has_columns = wave * 64 < 32 * a.K;
  // !QUAD: wf[i] = W[i][j].  QUAD: wf[4 k + c] = W[32 g + k][j4 + c], j4 the first column of
  // the lane's four (whole quads lie inside or outside the projector: K*L is a multiple of 4)
  float wf[kHeadDim];
  const uint32_t ucol = (uint32_t)ncol, uj = (uint32_t)j;
  if (wave_has_columns) {
    if constexpr (QUAD) {
      const int g = lane >> 4;
      const int c4 = wave * 64 + 4 * (lane & 15);
      const bool quad_ok = 32 * w * a.K + c4 + 3 < ncol && c4 < 32 * a.K;
      const uint32_t j4 = quad_ok ? (uint32_t)(32 * w * a.K + c4) : 0u;
#pragma unroll
      for (uint32_t k = 0; k < 32u; ++k) {
        const uint32_t at = (32u * (uint32_t)g + k) * ucol + j4;
        if constexpr (FP32) {
          const float4 v = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.W) + at);
          wf[4 * k] = v.x; wf[4 * k + 1] = v.y; wf[4 * k + 2] = v.z; wf[4 * k + 3] = v.w;
        } else {
          const uint2 v = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.W) + at);
          wf[4 * k] = __uint_as_float(v.x << 16); wf[4 * k + 1] = __uint_as_float(v.x & 0xffff0000u);
          wf[4 * k + 2] = __uint_as_float(v.y << 16); wf[4 * k + 3] = __uint_as_float(v.y & 0xffff0000u);
        }
      }
    } else {
#pragma unroll
      for (uint32_t i = 0; i < (uint32_t)kHeadDim; ++i) {
        if constexpr (FP32) wf[i] = reinterpret_cast<const float*>(a.W)[i * ucol + uj];
        else wf[i] = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(a.W)[i * ucol + uj] << 16);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < kHeadDim; ++i) wf[i] = 0.f;
  }
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  // vector r of the call is key first_key + r % n_keys of unit r / n_keys (queries: one unit)
  int64_t unit[2], key[2], xb[2];
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const int64_t r = r0 + (rr < nrow ? rr : 0);
    unit[rr] = r / a.n_keys;
    key[rr] = first_key + r % a.n_keys;
    xb[rr] = (unit[rr] / a.n_kv_heads) * a.stride_b + (unit[rr] % a.n_kv_heads) * a.stride_h + key[rr] * a.stride_n;
  }
  // The two vectors (or the vector and its centering vector) are staged once in LDS as float32
  // and read back as broadcasts: every thread needs all 128 elements of both.
  __shared__ float4 sx[2][kHeadDim / 4];
  __shared__ float sxq[2][kHeadDim];                      // QUAD: sxq[v][4 k + g] = x_v[32 g + k]
  __shared__ float sxnorm[2];
  {
    const int rr = (tid >> 5) & 1, i4 = tid & 31;         // threads 0..63: four elements each
    if (tid < 64) {
      float4 v;
      if (a.mu && rr == 1) {                             // second "vector": minus the centering vector
        const float4 m = *reinterpret_cast<const float4*>(a.mu + unit[0] * kHeadDim + i4 * 4);
        v = make_float4(-m.x, -m.y, -m.z, -m.w);
      } else if constexpr (FP32) {
        v = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.X) + xb[rr] + i4 * 4);
      } else if (a.x_fp8) {                              // rows of an e4m3 K cache
        const uint32_t r = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(a.X) + xb[rr] + i4 * 4);
        const mp_f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)r, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)r, true);
        v = make_float4(lo.x, lo.y, hi.x, hi.y);
      } else {
        const uint2 r = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.X) + xb[rr] + i4 * 4);
        v = make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                        __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
      }
      sx[rr][i4] = v;
      if constexpr (QUAD) {
        const float ve[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int e = 4 * i4 + c;                        // element e = 32 g + k
          sxq[rr][4 * (e & 31) + (e >> 5)] = ve[c];
        }
      }
      // Euclidean norm of the staged vector (32 lanes hold one vector)
      float q2 = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, v.w * v.w)));
#pragma unroll
      for (int o = 16; o >= 1; o >>= 1) q2 += __shfl_xor(q2, o);
      if (i4 == 0) sxnorm[rr] = __builtin_sqrtf(q2);
    }
  }
  __syncthreads();
  const bool with_mu = a.mu != nullptr;                  // then there is one vector: x.w - mu.w
  // First a float32 pass: one fused multiply-add per term.  n roundings of relative size 2^-24
  // at most (n = 128 terms, 257 with a centering vector) give |sum32 - exact| <= n 2^-24 (1 +
  // small) * sum|terms| <= that factor * |x| |w| (Cauchy-Schwarz; with a centering vector
  // (|x| + |mu|) |w|), plus what underflowing products lose, far below the absolute floor.  The
  // norms are float32 sums of squares (relative error below 1e-5, inside the margin of kClose32
  // over the factor): a result beyond kClose32 |x| |w| has the exact sign.  The few columns with
  // a closer result (a few in ten thousand) are redone in float64, where every product of two
  // float32 values is exact.
  const float kClose32 = with_mu ? 1.6e-5f : 8.0e-6f;
  float s32[2] = {0.f, 0.f}, w2 = 0.f;
  if (wave_has_columns) {
    if constexpr (QUAD) {
      const int g = lane >> 4;
      float p0[4] = {0.f, 0.f, 0.f, 0.f}, p1[4] = {0.f, 0.f, 0.f, 0.f}, pw[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < 32; ++k) {
        const float xa = sxq[0][4 * k + g], xc = sxq[1][4 * k + g];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float wv = wf[4 * k + c];
          p0[c] = fmaf(xa, wv, p0[c]);
          p1[c] = fmaf(xc, wv, p1[c]);
          pw[c] = fmaf(wv, wv, pw[c]);
        }
      }
      // the four row quarters of a column sit in the lanes i, i + 16, i + 32, i + 48
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        p0[c] += __shfl_xor(p0[c], 16); p0[c] += __shfl_xor(p0[c], 32);
        p1[c] += __shfl_xor(p1[c], 16); p1[c] += __shfl_xor(p1[c], 32);
        pw[c] += __shfl_xor(pw[c], 16); pw[c] += __shfl_xor(pw[c], 32);
      }
      s32[0] = g == 0 ? p0[0] : g == 1 ? p0[1] : g == 2 ? p0[2] : p0[3];
      s32[1] = g == 0 ? p1[0] : g == 1 ? p1[1] : g == 2 ? p1[2] : p1[3];
      w2 = g == 0 ? pw[0] : g == 1 ? pw[1] : g == 2 ? pw[2] : pw[3];
    } else {
#pragma unroll
      for (int i4 = 0; i4 < kHeadDim / 4; ++i4) {
        const float4 x0 = sx[0][i4], x1 = sx[1][i4];
        const float xa[4] = {x0.x, x0.y, x0.z, x0.w}, xc[4] = {x1.x, x1.y, x1.z, x1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float wv = wf[i4 * 4 + e];
          s32[0] = fmaf(xa[e], wv, s32[0]);
          s32[1] = fmaf(xc[e], wv, s32[1]);
          w2 = fmaf(wv, wv, w2);
        }
      }
    }
  }
  const float wnorm = __builtin_sqrtf(w2);
  float m32[2] = {sxnorm[0] * wnorm, sxnorm[1] * wnorm};
  if (with_mu) {
    s32[0] += s32[1];                                    // one more rounding, inside the factor
    m32[0] += m32[1];
  }
  const bool close0 = !(fabsf(s32[0]) > kClose32 * m32[0] + 1e-30f);
  const bool close1 = !with_mu && nrow > 1 && !(fabsf(s32[1]) > kClose32 * m32[1] + 1e-30f);
  double s[2] = {(double)s32[0], (double)s32[1]}, mag[2] = {0.0, 0.0};
  // The few close columns of a wavefront are redone one at a time by the whole wavefront: the
  // owning lane hands its column over through LDS, every lane forms the exact float64 products
  // of its two (four) terms, and a butterfly adds them up: at most nine roundings of 2^-53
  // relative to the magnitude sum, far inside the slack the final test allows.
  __shared__ float4 scol[8][kHeadDim / 4];
  uint64_t redo = __ballot(col_ok && (close0 || close1));
  while (redo) {
    const int src = __ffsll((unsigned long long)redo) - 1;
    redo &= redo - 1;
    if constexpr (QUAD) {
      // the column is spread over the four lanes (g', i) of the owner's i: each writes its quarter
      const int gs = src >> 4;                           // wave-uniform: which of the four columns
      if ((lane & 15) == (src & 15)) {
        float* dst = reinterpret_cast<float*>(scol[wave]) + 32 * (lane >> 4);
        if (gs == 0) {
#pragma unroll
          for (int k = 0; k < 32; ++k) dst[k] = wf[4 * k];
        } else if (gs == 1) {
#pragma unroll
          for (int k = 0; k < 32; ++k) dst[k] = wf[4 * k + 1];
        } else if (gs == 2) {
#pragma unroll
          for (int k = 0; k < 32; ++k) dst[k] = wf[4 * k + 2];
        } else {
#pragma unroll
          for (int k = 0; k < 32; ++k) dst[k] = wf[4 * k + 3];
        }
      }
    } else if (lane == src) {
#pragma unroll
      for (int i4 = 0; i4 < kHeadDim / 4; ++i4)
        scol[wave][i4] = make_float4(wf[4 * i4], wf[4 * i4 + 1], wf[4 * i4 + 2], wf[4 * i4 + 3]);
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    const float* cf = reinterpret_cast<const float*>(scol[wave]);
    const float* xf = reinterpret_cast<const float*>(sx);
    const double w0 = (double)cf[lane], w1 = (double)cf[lane + 64];
    const double p00 = (double)xf[lane] * w0, p01 = (double)xf[lane + 64] * w1;                        // exact
    const double p10 = (double)xf[kHeadDim + lane] * w0, p11 = (double)xf[kHeadDim + lane + 64] * w1;  // exact
    double t0 = p00 + p01, g0 = fabs(p00) + fabs(p01);
    double t1 = p10 + p11, g1 = fabs(p10) + fabs(p11);
    if (with_mu) {
      t0 += t1;
      g0 += g1;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      t0 += __shfl_xor(t0, o);
      g0 += __shfl_xor(g0, o);
      t1 += __shfl_xor(t1, o);
      g1 += __shfl_xor(g1, o);
    }
    if (lane == src) {
      s[0] = t0; mag[0] = g0;
      s[1] = t1; mag[1] = g1;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
  }
  for (int rr = 0; rr < nrow; ++rr) {
    bool bit = s[rr] >= 0.0;
    const bool unsure = col_ok && mag[rr] > 0.0 && fabs(s[rr]) <= kF64Slack * mag[rr];
    uint64_t pending = __ballot(unsure);
    while (pending) {
      const int src = __ffsll((unsigned long long)pending) - 1;
      const int sj = __shfl(j, src);
      const float* smu = a.mu ? a.mu + unit[rr] * kHeadDim : nullptr;
      const int64_t xbase = xb[rr];
      const bool r = exact_sign_nonneg_wave(
          limbs[wave],
          [&](int d) { return load_x_elem<FP32>(a, xbase + d); },
          [&](int d) { return load_elem<FP32>(a.W, (int64_t)d * ncol + sj); },
          [&](int d) { return smu ? (double)smu[d] : 0.0; }, smu != nullptr);
      if (lane == src) bit = r;
      pending &= pending - 1;
    }
    sbit[rr][cid] = (unsigned char)(bit && col_ok);
  }
  __syncthreads();
  // regroup: item (row, plane b, table beta) reads the bit of column beta*K + b
  const int items = nrow * a.K * 32;
  const int Wd = table_words(a.L);
  for (int p0 = 0; p0 < items; p0 += 512) {
    const int p = p0 + tid;
    const bool on = p < items;
    const int row = on && p >= a.K * 32 ? 1 : 0;          // at most two rows
    const int rem = on ? p - row * (a.K * 32) : 0;
    const int pb = rem >> 5, beta = rem & 31;
    const bool v = on && sbit[row][beta * a.K + pb];
    const uint64_t m = __ballot(v);
    uint32_t word = (lane >> 5) ? (uint32_t)(m >> 32) : (uint32_t)m;
    if (on && beta == 0) {
      const int x = w * a.K + pb;
      if (a.query_layout) {
        if (w == Wd - 1 && (a.L & 31)) word |= ~0u << (a.L & 31);  // padding tables never collide
        a.codes[(r0 + row) * a.NQ + x] = word;
      } else if (w < Wd - 1) {
        const int64_t blk = unit[row] * a.blocks_cap + key[row] / kBlockKeys;
        a.codes[blk * (kBlockKeys * (int64_t)a.NW) + slot_in_block(a.NW, x, (int)(key[row] % kBlockKeys))] = word;
      }
    }
  }
  if (!a.query_layout && w == Wd - 1) {
    // keys, last table group: the K planes are stored as one bit string of tail_tables bits
    // each; item (row, packed word e, bit) reads the sign bit at string position 32 e + bit
    const int Lt = tail_tables(a.L), xs = tail_begin(a.K, a.L), nt = a.NW - xs;
    const int titems = nrow * nt * 32;
    for (int p0 = 0; p0 < titems; p0 += 512) {
      const int p = p0 + tid;
      const bool on = p < titems;
      const int row = on ? p / (nt * 32) : 0;
      const int pos = on ? p % (nt * 32) : 0;
      const int pb = pos / Lt, tb = pos % Lt;            // plane, table inside the group
      const bool v = on && pb < a.K && sbit[row][tb * a.K + pb];
      const uint64_t m = __ballot(v);
      const uint32_t word = (lane >> 5) ? (uint32_t)(m >> 32) : (uint32_t)m;
      if (on && (pos & 31) == 0) {
        const int64_t blk = unit[row] * a.blocks_cap + key[row] / kBlockKeys;
        a.codes[blk * (kBlockKeys * (int64_t)a.NW) + slot_in_block(a.NW, xs + (pos >> 5), (int)(key[row] % kBlockKeys))] = word;
      }
    }
  }
}

// `b` may be null (one set of vectors); both sets share K, L, the projector and the element type.
hipError_t launch_hash_rows(const HashDirectArgs& a, const HashDirectArgs* b, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const int64_t rows0 = a.total_rows > 0 ? a.total_rows : 0, rows1 = b && b->total_rows > 0 ? b->total_rows : 0;
  if (rows0 + rows1 <= 0) return hipSuccess;
  const int pairs0 = (int)(a.mu ? rows0 : (rows0 + 1) / 2);           // workgroups of the first set
  const int pairs1 = (int)(b && b->mu ? rows1 : (rows1 + 1) / 2);
  const dim3 grid((unsigned)table_words(a.L), (unsigned)(pairs0 + pairs1)), block(512);
  const HashDirectArgs& a1 = b ? *b : a;
  const bool quad = (a.K * a.L) % 4 == 0;     // four columns per load (16-byte aligned base, checked by the caller)
  // (with events the launch carries the kernel's own begin / end timestamps)
  auto go = [&](auto kernel) {
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, start, stop, 0, a, a1, pairs0);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, a, a1, pairs0);
  };
  if (a.is_fp32) {
    if (quad) go(hash_rows_kernel<true, true>);
    else go(hash_rows_kernel<true, false>);
  } else {
    if (quad) go(hash_rows_kernel<false, true>);
    else go(hash_rows_kernel<false, false>);
  }
  return hipGetLastError();
}

hipError_t launch_hash_direct(const HashDirectArgs& a, hipStream_t s) {
  if (a.total_rows <= 0) return hipSuccess;
  const int64_t groups = (a.total_rows + 7) / 8;
  // few vectors (queries): one workgroup per (8 vectors, word); many (keys): words looped
  const unsigned ny = groups >= 4096 ? 1u : (unsigned)(a.query_layout ? a.NQ : tail_begin(a.K, a.L) + 1);
  // behind the matrix-core path the kernel normally only reads its flag and leaves: a capped
  // grid keeps that cheap, and the groups are walked in a loop if it does have to run
  const unsigned nx = (unsigned)(a.run_flag && groups > 2048 ? 2048 : groups);
  if (a.is_fp32) hipLaunchKernelGGL(hash_direct_kernel<true>, dim3(nx, ny), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(hash_direct_kernel<false>, dim3(nx, ny), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
