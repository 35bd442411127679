// SimHash coding of a few bf16 vectors on the matrix cores: the queries of a decode step
// (Algorithm 1 "Encode(q, W)") and the newest keys of every (batch, KV head), which join the hash
// structure behind the frozen centering vector (Sec. 4.3 "Data pre-processing"; Sec. 4.4 (3)).
//
// The step is latency-bound (a few thousand vectors at most against 384 KB of projector), so the
// kernel is built around one memory round trip.  The projector is read in a prepared form
// (magicpig_prepare_projector, once per model): MFMA A fragments, 16 bytes per lane and load,
// grouped so that a workgroup = one group of 32 tables and a wavefront = two of its bit planes.
// A wavefront requests its two A tiles and up to 64 vectors (B operand, lane%32 = vector) at
// once, multiplies (v_mfma_f32_32x32x16_bf16), and has the 32 sign bits of a plane word inside
// one lane as in the key-hashing kernel.  Keys enter with the prepared initial accumulators
// -fl(mu.W_j) (magicpig_prepare_centering, once per sequence: the mean is frozen).
//
// Bit-exactness: as in hash_keys_mfma.hip a projection with |acc| <= kGamma (|x| + |mu|) max|W_j|
// is re-evaluated exactly.  Here the re-evaluation never leaves the compute unit: the vector and
// the projector column sit in the wavefront's registers, the two lanes that hold each write them
// to LDS, every lane forms the exact float64 products of two elements (the centering vector was
// staged in LDS at the start), a butterfly adds them, and what float64 cannot decide goes to the
// exact accumulator (exact_dot.h).  The owning lane patches its bit before the word is stored,
// so there is no list, no overflow and no atomic.
#include "mp_common.h"
#include "exact_dot.h"
#include "device_utils.h"
#include <hip/hip_ext.h>

namespace mp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Row rho of tile tau of a plane pair: plane 2p + eta, bit beta of the plane word (table 32w + beta).
// Accumulator register r = 4*(rho/8) + rho%4 of lane half eta; inserted most significant bit first.
__host__ __device__ inline void few_row_to_bit(int tau, int rho, int* eta, int* beta) {
  *eta = (rho >> 2) & 1;
  *beta = 31 - (16 * tau + 4 * (rho >> 3) + (rho & 3));
}

__global__ void prep_few_header_kernel(uint32_t* header, int K, int L) {
  if (threadIdx.x == 0) {
    header[0] = kPreparedMagic;
    header[1] = (uint32_t)K;
    header[2] = (uint32_t)L;
    header[3] = 0u;                                        // largest column norm: raised by the next kernel
  }
}

// One thread per (tile row, 8-element piece of d): fragment, transposed copy, column norm.
__global__ __launch_bounds__(256) void prep_few_fragments_kernel(const uint16_t* W, uint32_t* header, uint4* frag,
                                                                 uint4* wt, int K, int L) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  const int P = (K + 1) / 2, Wd = table_words(L);
  const int row = gid >> 4, piece = gid & 15;              // row = ((w*P + p)*2 + tau)*32 + rho
  const bool row_in = row < Wd * P * 64;
  const int rho = row & 31, tau = (row >> 5) & 1, wp = row >> 6;
  const int p = wp % P, w = wp / P;
  int eta, beta;
  few_row_to_bit(tau, rho, &eta, &beta);
  const int b = 2 * p + eta, t = 32 * w + beta;
  const bool real = row_in && b < K && t < L;
  const int ncol = K * L, j = real ? t * K + b : 0;
  uint16_t v[8];
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = real ? W[(int64_t)(piece * 8 + e) * ncol + j] : (uint16_t)0;
    const float f = __uint_as_float((uint32_t)v[e] << 16);
    ss += f * f;
  }
  uint4 pk;
  pk.x = v[0] | ((uint32_t)v[1] << 16); pk.y = v[2] | ((uint32_t)v[3] << 16);
  pk.z = v[4] | ((uint32_t)v[5] << 16); pk.w = v[6] | ((uint32_t)v[7] << 16);
  const int s = piece >> 1, lane = (piece & 1) * 32 + rho;
  if (row_in) frag[((int64_t)(row >> 5) * 8 + s) * 64 + lane] = pk;
  if (real) wt[(int64_t)j * 16 + piece] = pk;
  ss = row_sum16(ss);                                      // the 16 pieces of a row sit in one DPP row
  if (real && piece == 0) atomicMax(&header[3], __float_as_uint(sqrtf(ss) * 1.000001f));   // (non-negative floats order like integers)
}

__global__ __launch_bounds__(256) void prep_few_copy_kernel(const uint4* src, uint4* dst, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// Per (batch, KV head): initial accumulators -fl(mu.W_j) in fragment order, and |mu|.
__global__ __launch_bounds__(256) void prep_centering_kernel(const float* mu_all, const uint16_t* wt, float* thr,
                                                             float* munorm, int K, int L) {
  const int unit = blockIdx.y;
  const int row = blockIdx.x * 256 + threadIdx.x;
  const int P = (K + 1) / 2, Wd = table_words(L);
  const float* mu = mu_all + (int64_t)unit * kHeadDim;
  if (row == 0) {
    double ss = 0.0;
    for (int d = 0; d < kHeadDim; ++d) ss += (double)mu[d] * (double)mu[d];
    munorm[unit] = (float)sqrt(ss) * 1.000001f;
  }
  if (row >= Wd * P * 64) return;
  const int rho = row & 31, tau = (row >> 5) & 1, wp = row >> 6;
  const int p = wp % P, w = wp / P;
  int eta, beta;
  few_row_to_bit(tau, rho, &eta, &beta);
  const int b = 2 * p + eta, t = 32 * w + beta;
  float c = 0.f;                                           // rows outside the projector are masked by the kernel
  if (b < K && t < L) {
    const uint16_t* wr = wt + (int64_t)(t * K + b) * kHeadDim;
    double th = 0.0;
    for (int d = 0; d < kHeadDim; ++d) th += (double)mu[d] * (double)__uint_as_float((uint32_t)wr[d] << 16);
    c = 0.0f - (float)th;                                  // +0 when the threshold is zero
  }
  const int r = 4 * (rho >> 3) + (rho & 3);
  thr[((((int64_t)unit * Wd * P + wp) * 2 + tau) * 2 + eta) * 16 + r] = c;
}

__global__ __launch_bounds__(512) void hash_few_mfma_kernel(HashFewArgs a) {
  __shared__ uint32_t sTail[16][32];                       // plane words of the last table group, [plane][key]
  __shared__ float sMu[32][kHeadDim];                      // centering vectors of the 32 keys of a key group
  __shared__ uint4 sX[8][16], sW[8][16];                   // per wavefront: a vector / a projector column being re-evaluated
  __shared__ long long sLimbs[8][kLimbs];
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int kap = lane & 31, hh = lane >> 5;
  const int w = blockIdx.x, p = wave;
  const bool is_key = (int)blockIdx.y >= a.q_groups;
  const int grp = is_key ? (int)blockIdx.y - a.q_groups : (int)blockIdx.y;
  int64_t first_key = a.first_key;
  if (is_key && a.n_dev) {                                 // the newest keys of a context whose length lives in device memory
    first_key = *a.n_dev - a.n_keys;
    if (first_key < 0 || first_key + a.n_keys > a.n_cap) return;    // (uniform in the workgroup, before any barrier)
  }
  if (lane < kLimbs) sLimbs[wave][lane] = 0;

  // ---- everything the wavefront needs from memory, requested at once ----
  bf16x8 A[2][8], B[2][8];
  const uint4* fr = reinterpret_cast<const uint4*>(a.frag) + (int64_t)(w * a.P + p) * 2 * 8 * 64 + lane;
#pragma unroll
  for (int tau = 0; tau < 2; ++tau)
#pragma unroll
    for (int s = 0; s < 8; ++s) A[tau][s] = __builtin_bit_cast(bf16x8, fr[(tau * 8 + s) * 64]);
  bool ok[2] = {false, false};
  const uint16_t* rp[2];
  int64_t unit = 0, key = 0;
  if (!is_key) {
#pragma unroll
    for (int bt = 0; bt < 2; ++bt) {
      const int v = grp * 64 + bt * 32 + kap;
      ok[bt] = v < a.n_q;
      rp[bt] = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)(ok[bt] ? v : 0) * kHeadDim;
    }
  } else {
    const int r = grp * 32 + kap;
    ok[0] = r < a.n_krows;
    const int64_t rr = ok[0] ? r : 0;
    unit = rr / a.n_keys;
    key = first_key + rr % a.n_keys;
    rp[0] = reinterpret_cast<const uint16_t*>(a.Kc) + (unit / a.n_kv_heads) * a.stride_b +
            (unit % a.n_kv_heads) * a.stride_h + key * a.stride_n;
    rp[1] = rp[0];
  }
  const bool key8 = is_key && a.kv_fp8;                    // the key rows are e4m3 bytes (wave-uniform)
  const bool two = !is_key && grp * 64 + 32 < a.n_q;       // a second tile of vectors (wave-uniform)
  if (key8) {
    // (same element offset, one byte per element; widened to the same values in bf16)
    const uint8_t* row8 = reinterpret_cast<const uint8_t*>(a.Kc) + (rp[0] - reinterpret_cast<const uint16_t*>(a.Kc)) + hh * 8;
    uint2 r8[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) r8[s] = *reinterpret_cast<const uint2*>(row8 + s * 16);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      B[0][s] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(r8[s].x, r8[s].y));
      B[1][s] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
    }
  } else {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      B[0][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(rp[0] + s * 16 + hh * 8));
      if (two) B[1][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(rp[1] + s * 16 + hh * 8));
      else B[1][s] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
    }
  }
  const bool centered = is_key && a.mu != nullptr;
  f32x16 acc[2][2];
#pragma unroll
  for (int tau = 0; tau < 2; ++tau)
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[tau][0][r] = 0.f; acc[tau][1][r] = 0.f; }
  float munorm = 0.f;
  if (centered) {
    const float* tp = a.thr + ((((int64_t)unit * a.Wd * a.P + (w * a.P + p)) * 2) * 2 + hh) * 16;
#pragma unroll
    for (int tau = 0; tau < 2; ++tau)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const float4 t4 = *reinterpret_cast<const float4*>(tp + tau * 32 + v4 * 4);
        acc[tau][0][v4 * 4] = t4.x; acc[tau][0][v4 * 4 + 1] = t4.y; acc[tau][0][v4 * 4 + 2] = t4.z; acc[tau][0][v4 * 4 + 3] = t4.w;
      }
    munorm = a.munorm[unit];
    // the centering vectors themselves, for the exact re-evaluation
    for (int i = tid; i < 32 * 32; i += blockDim.x) {
      const int kk = i >> 5, piece = i & 31;
      const int r = grp * 32 + kk;
      if (r < a.n_krows)
        reinterpret_cast<float4*>(sMu[kk])[piece] =
            reinterpret_cast<const float4*>(a.mu + (int64_t)(r / a.n_keys) * kHeadDim)[piece];
    }
  }
  const float wmax = __uint_as_float(a.header[3]);

  // ---- error bound per vector: kGamma (|x| + |mu|) max|W_j| ----
  // (|x|^2 by v_dot2_f32_bf16, two exact products per instruction, float32 accumulation: the
  // relative error of the norm, below 1e-5, is inside the margin of kGamma)
  float bnd[2] = {-1.f, -1.f};
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    if (bt == 1 && !two) break;
    float ss = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const uint4 raw = __builtin_bit_cast(uint4, B[bt][s]);
      const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bf16x2 v2 = __builtin_bit_cast(bf16x2, u[i]);
        ss = __builtin_amdgcn_fdot2_f32_bf16(v2, v2, ss, false);
      }
    }
    ss += __shfl_xor(ss, 32);                              // the other half of the row
    const float xnorm = sqrtf(ss) * 1.00002f;
    bnd[bt] = ok[bt] ? (kGamma * (xnorm + munorm) * wmax) * 1.000001f + 1e-30f : -1.f;
  }

  // ---- multiply ----
#pragma unroll
  for (int tau = 0; tau < 2; ++tau)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      acc[tau][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[tau][s], B[0][s], acc[tau][0], 0, 0, 0);
      if (two) acc[tau][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[tau][s], B[1][s], acc[tau][1], 0, 0, 0);
    }
  // sign bits and "too close to zero" flags, most significant bit first (bit beta of the plane
  // word): neg = 1 where the projection is negative.  The accumulator starts from +0 or a
  // non-zero threshold and round-to-nearest never produces -0 from a sum, so the sign bit is the
  // test "< 0".
  // The flags cost as much as the signs and are almost always all zero: the smallest |acc| of a
  // lane is compared with its bound first, and the per-bit flags are formed only by wavefronts
  // in which some lane has one below it.
  uint32_t neg[2] = {0, 0}, fl[2] = {0, 0};
  bool close_lane = false;
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    if (bt == 1 && !two) break;
    float lo = INFINITY;
#pragma unroll
    for (int tau = 0; tau < 2; ++tau)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        neg[bt] = __builtin_amdgcn_alignbit(neg[bt], __float_as_uint(acc[tau][bt][r]), 31);
        lo = fminf(lo, fabsf(acc[tau][bt][r]));
      }
    close_lane |= lo < bnd[bt];
  }
  if (__ballot(close_lane)) {
#pragma unroll
    for (int bt = 0; bt < 2; ++bt) {
      if (bt == 1 && !two) break;
#pragma unroll
      for (int tau = 0; tau < 2; ++tau)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          fl[bt] = __builtin_amdgcn_alignbit(fl[bt], __float_as_uint(fabsf(acc[tau][bt][r]) - bnd[bt]), 31);
    }
  }
  // this lane half's plane and the tables that exist in this group
  const int b_my = 2 * p + hh;
  const uint32_t tmask = (w == a.Wd - 1 && (a.L & 31)) ? (1u << (a.L & 31)) - 1u : ~0u;
  const uint32_t vmask = b_my < a.K ? tmask : 0u;
  fl[0] &= vmask;
  fl[1] &= two ? vmask : 0u;
  // the centering vectors of a key group are staged by the whole workgroup; a wavefront's own
  // accumulator cells only need the wavefront's own writes to have landed
  if (centered) __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();

  // ---- exact re-evaluation of the flagged projections, one at a time, in LDS and registers ----
  uint64_t has = __ballot((fl[0] | fl[1]) != 0u);
  while (has) {
    const int src = __ffsll((unsigned long long)has) - 1;                    // wave-uniform
    const uint32_t f0 = __builtin_amdgcn_readlane(fl[0], src), f1 = __builtin_amdgcn_readlane(fl[1], src);
    const int bt = f0 ? 0 : 1;
    const int beta = __ffs(f0 ? f0 : f1) - 1;
    const int el = 31 - beta, tau = el >> 4, r = el & 15;
    const int hsrc = src >> 5, kap0 = src & 31;
    const int rho = 8 * (r >> 2) + 4 * hsrc + (r & 3);                        // tile row of the projection
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
      if (tt == tau && kap == rho) {
#pragma unroll
        for (int s = 0; s < 8; ++s) sW[wave][s * 2 + hh] = __builtin_bit_cast(uint4, A[tt][s]);
      }
#pragma unroll
    for (int bb = 0; bb < 2; ++bb)
      if (bb == bt && kap == kap0) {
#pragma unroll
        for (int s = 0; s < 8; ++s) sX[wave][s * 2 + hh] = __builtin_bit_cast(uint4, B[bb][s]);
      }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    const uint16_t* xs16 = reinterpret_cast<const uint16_t*>(sX[wave]);
    const uint16_t* ws16 = reinterpret_cast<const uint16_t*>(sW[wave]);
    auto xv = [&](int d) { return (double)__uint_as_float((uint32_t)xs16[d] << 16); };
    auto wv = [&](int d) { return (double)__uint_as_float((uint32_t)ws16[d] << 16); };
    auto mv = [&](int d) { return centered ? (double)sMu[kap0][d] : 0.0; };
    const double w0 = wv(lane), w1 = wv(lane + 64);
    const double p0 = xv(lane) * w0, p1 = xv(lane + 64) * w1;                 // exact products
    double t = p0 + p1, g = fabs(p0) + fabs(p1);
    if (centered) {
      const double m0 = mv(lane) * w0, m1 = mv(lane + 64) * w1;               // exact products
      t -= m0 + m1;
      g += fabs(m0) + fabs(m1);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      t += __shfl_xor(t, o);
      g += __shfl_xor(g, o);
    }
    bool bit = t >= 0.0;
    if (g > 0.0 && fabs(t) <= kF64Slack * g) bit = exact_sign_nonneg_wave(sLimbs[wave], xv, wv, mv, centered);
    if (lane == src) {
      const uint32_t m = 1u << beta;
      if (bt == 0) { fl[0] &= ~m; neg[0] = bit ? (neg[0] & ~m) : (neg[0] | m); }
      else { fl[1] &= ~m; neg[1] = bit ? (neg[1] & ~m) : (neg[1] | m); }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
    has = __ballot((fl[0] | fl[1]) != 0u);
  }

  // ---- store ----
  if (!is_key) {
    // queries: plane words as they are, the tables beyond L set to 1 (they never collide)
    const uint32_t pad = b_my < a.K ? ~tmask : 0u;
    const uint32_t c0 = (~neg[0] & vmask) | pad, c1 = (~neg[1] & vmask) | pad;
    // lanes < 32 hold plane 2p of vectors kap / 32 + kap, lanes >= 32 plane 2p + 1: one half-swap
    // leaves lane l with both words of vector l
    const auto sw = __builtin_amdgcn_permlane32_swap(c0, c1, false, false);
    const int v = grp * 64 + lane;
    if (v < a.n_q) {
      uint32_t* dst = a.qcodes + (int64_t)v * a.NQ + w * a.K + 2 * p;
      dst[0] = sw[0];
      if (2 * p + 1 < a.K) dst[1] = sw[1];
    }
    return;
  }
  const uint32_t code = ~neg[0] & vmask;
  uint32_t* kdst = a.kcodes + (unit * a.blocks_cap + key / kBlockKeys) * (kBlockKeys * (int64_t)a.NW);
  const int kr = (int)(key % kBlockKeys);
  if (w < a.Wd - 1) {
    if (ok[0] && b_my < a.K) kdst[slot_in_block(a.NW, w * a.K + b_my, kr)] = code;
    return;
  }
  // keys, last table group: the K planes are stored as one bit string of tail_tables bits each
  sTail[b_my][kap] = code;                                 // b_my < 2P <= 16
  __syncthreads();
  if (wave == 0 && hh == 0 && ok[0]) {
    const int Lt = tail_tables(a.L);
    BitString bs;
    int xo = tail_begin(a.K, a.L);
    for (int b = 0; b < a.K; ++b) {
      uint32_t full;
      if (bs.append(sTail[b][kap], Lt, &full)) kdst[slot_in_block(a.NW, xo++, kr)] = full;
    }
    if (bs.nbits > 0) kdst[slot_in_block(a.NW, xo, kr)] = (uint32_t)bs.acc;
  }
}

hipError_t launch_prepare_projector(const void* W, void* prepared, int K, int L, hipStream_t s) {
  const PreparedLayout l = prepared_layout(K, L, false);
  char* base = reinterpret_cast<char*>(prepared);
  uint32_t* header = reinterpret_cast<uint32_t*>(base);
  hipLaunchKernelGGL(prep_few_header_kernel, dim3(1), dim3(64), 0, s, header, K, L);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rows = l.Wd * l.P * 64;
  hipLaunchKernelGGL(prep_few_fragments_kernel, dim3((unsigned)((rows * 16 + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(W), header, reinterpret_cast<uint4*>(base + l.frag_off),
                     reinterpret_cast<uint4*>(base + l.wt_off), K, L);
  return hipGetLastError();
}

hipError_t launch_prepare_projector_fp32(const void* W, void* prepared, int K, int L, hipStream_t s) {
  const PreparedLayout l = prepared_layout(K, L, true);
  char* base = reinterpret_cast<char*>(prepared);
  hipLaunchKernelGGL(prep_few_header_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(base), K, L);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t count = (int64_t)K * L * kHeadDim * 4 / 16;     // K*L*128 floats: a whole number of 16-byte pieces
  hipLaunchKernelGGL(prep_few_copy_kernel, dim3(64), dim3(256), 0, s, reinterpret_cast<const uint4*>(W),
                     reinterpret_cast<uint4*>(base + l.wt_off), count);
  return hipGetLastError();
}

hipError_t launch_prepare_centering(const float* mu, const void* prepared, void* centering, int K, int L, int units,
                                    hipStream_t s) {
  if (units <= 0) return hipSuccess;
  const PreparedLayout l = prepared_layout(K, L, false);
  const CenteringLayout c = centering_layout(K, L, (size_t)units);
  const char* pb = reinterpret_cast<const char*>(prepared);
  char* cb = reinterpret_cast<char*>(centering);
  const int rows = l.Wd * l.P * 64;
  hipLaunchKernelGGL(prep_centering_kernel, dim3((unsigned)((rows + 255) / 256), (unsigned)units), dim3(256), 0, s, mu,
                     reinterpret_cast<const uint16_t*>(pb + l.wt_off), reinterpret_cast<float*>(cb + c.thr_off),
                     reinterpret_cast<float*>(cb + c.munorm_off), K, L);
  return hipGetLastError();
}

hipError_t launch_hash_few(const HashFewArgs& a0, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  HashFewArgs a = a0;
  a.q_groups = (a.n_q + 63) / 64;
  const int k_groups = (a.n_krows + 31) / 32;
  if (a.q_groups + k_groups <= 0) return hipSuccess;
  const dim3 grid((unsigned)a.Wd, (unsigned)(a.q_groups + k_groups)), block(64 * a.P);
  if (start || stop) hipExtLaunchKernelGGL(hash_few_mfma_kernel, grid, block, 0, s, start, stop, 0, a);
  else hipLaunchKernelGGL(hash_few_mfma_kernel, grid, block, 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
