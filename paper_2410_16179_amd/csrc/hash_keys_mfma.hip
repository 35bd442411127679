// SimHash coding of cached bf16 keys on the matrix cores (Sec. 4.3 "Hash function
// selection"; Sec. 4.4 (3): the K*L random projections are the compute-bound step).
//
// The projection is a [keys x 128] x [128 x K*L] contraction.  It runs as bf16 MFMA
// (v_mfma_f32_32x32x16_bf16) with the projector as the A operand and 32 keys as the B
// operand, so an accumulator register of a lane holds one (projection, key) pair with
// lane%32 = key: the 32 sign bits of a code word are assembled inside one lane with one
// funnel shift per element and no cross-lane traffic.  Rows of the A operand are
// arranged (prep_projector_kernel) so that the two lane halves of two consecutive MFMA
// tiles produce two complete code words; one half-swap then gives every lane the four
// words of "its" key and a wavefront stores a contiguous kilobyte of the code layout.
//
// Bit-exactness.  The hash bit is the sign of the exact sum  k.W_j - mu.W_j.  The MFMA
// result acc ~ k.W_j - fl(mu.W_j) (the threshold enters as the initial accumulator) differs
// from it by at most  bound_i = kGamma * (|k_i| + |mu|) * max_j |W_j|:  every bf16 product is
// exact in float32, the accumulation inside the matrix core loses at most kGamma of the sum of
// magnitudes whatever its order and grouping (mp_common.h), and sum|terms| <= (|k_i| + |mu|) |W_j|
// by Cauchy-Schwarz.
// Elements with |acc| <= bound_i (a few in ten thousand) are listed in LDS and re-evaluated
// at the end of the workgroup in float64 with the exact fallback of exact_dot.h, which
// patches the bit.  Pairs beyond the LDS list go to a global list and recheck_kernel; if that
// overflows too, a flag makes the direct float64 kernel redo the whole call.
#include "mp_common.h"
#include "exact_dot.h"
#include "device_utils.h"

namespace mp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kListCapLocal = 1536;       // flagged elements a workgroup can hold in LDS

// Projection handled by row rho (0..31) of MFMA tile T: tile pair T/2 makes code words
// x = 2*(T/2) + eta, eta = (rho/4)%2 being the lane half that receives the row; the row is
// accumulator register r = 4*(rho/8) + rho%4 of that half, inserted as element 16*(T%2) + r
// of the word, most significant bit first.
__host__ __device__ inline void tile_row_to_bit(int T, int rho, int* x, int* beta) {
  const int eta = (rho >> 2) & 1;
  const int r = 4 * (rho >> 3) + (rho & 3);
  *x = 2 * (T >> 1) + eta;
  *beta = 31 - (16 * (T & 1) + r);
}

// A-operand fragments, transposed bf16 copy of W for the recheck, norm of every projector
// column (by tile row).  One thread per (tile row, 8-element piece of d).  Also clears the
// counters the later kernels of the call add to.
__global__ __launch_bounds__(256) void prep_projector_kernel(HashMfmaArgs a) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  if (gid == 0) {
    *a.list_count = 0u;
    *a.overflow = 0;
    *a.flagged_total = 0u;
    *a.wmax_bits = 0u;                                   // largest column norm: raised by the threshold kernel
  }
  const int row = gid >> 4, piece = gid & 15;        // row = T*32 + rho
  if (row >= a.ntiles * 32) return;
  const int T = row >> 5, rho = row & 31;
  int x, beta;
  tile_row_to_bit(T, rho, &x, &beta);
  const int t = 32 * (x / a.K) + beta;
  const bool real = x < a.NQ && t < a.L;
  const int j = real ? t * a.K + x % a.K : 0;
  const int ncol = a.K * a.L;
  const uint16_t* W = reinterpret_cast<const uint16_t*>(a.W);
  uint16_t v[8];
  float ss = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    v[e] = real ? W[(int64_t)(piece * 8 + e) * ncol + j] : (uint16_t)0;
    const float f = __uint_as_float((uint32_t)v[e] << 16);
    ss += f * f;
  }
  // fragment order: k-step s = piece/2, lane = (piece%2)*32 + rho, eight bf16 per lane
  const int s = piece >> 1, lane = (piece & 1) * 32 + rho;
  uint4 pk;
  pk.x = v[0] | ((uint32_t)v[1] << 16); pk.y = v[2] | ((uint32_t)v[3] << 16);
  pk.z = v[4] | ((uint32_t)v[5] << 16); pk.w = v[6] | ((uint32_t)v[7] << 16);
  reinterpret_cast<uint4*>(a.afrag)[((int64_t)T * 8 + s) * 64 + lane] = pk;
  if (real) reinterpret_cast<uint4*>(a.wt)[(int64_t)j * 16 + piece] = pk;
  ss = row_sum16(ss);                                  // the 16 pieces of a row sit in one DPP row
  if (piece == 0) a.rownorm[row] = sqrtf(ss) * 1.000001f;   // 0 for padding rows
}

// Per (batch, KV head): initial accumulators -fl(mu.W_j) in fragment order, and |mu|.
__global__ __launch_bounds__(256) void prep_threshold_kernel(HashMfmaArgs a) {
  const int unit = blockIdx.y;
  const int row = blockIdx.x * 256 + threadIdx.x;
  const float* mu = a.mu ? a.mu + (int64_t)unit * kHeadDim : nullptr;
  if (row == 0) {
    double ss = 0.0;
    if (mu) for (int d = 0; d < kHeadDim; ++d) ss += (double)mu[d] * (double)mu[d];
    a.munorm[unit] = (float)sqrt(ss) * 1.000001f;
  }
  if (row >= a.ntiles * 32) return;
  // the largest column norm of the projector, once per call (non-negative floats order like integers)
  if (unit == 0) atomicMax(a.wmax_bits, __float_as_uint(a.rownorm[row]));
  const int T = row >> 5, rho = row & 31;
  int x, beta;
  tile_row_to_bit(T, rho, &x, &beta);
  const int t = 32 * (x / a.K) + beta;
  const bool real = x < a.NQ && t < a.L;
  float c = -INFINITY;                                 // pad rows: never >= 0, never flagged
  if (real) {
    const int j = t * a.K + x % a.K;
    double th = 0.0, mg = 0.0;
    if (mu) {
      const uint16_t* wt = reinterpret_cast<const uint16_t*>(a.wt) + (int64_t)j * kHeadDim;
      for (int d = 0; d < kHeadDim; ++d) {
        const double pm = (double)mu[d] * (double)__uint_as_float((uint32_t)wt[d] << 16);   // exact
        th += pm;
        mg += fabs(pm);
      }
    }
    c = 0.0f - (float)th;                              // +0 when the threshold is zero
    // for the exact re-evaluation: the same sum in float64 and a float32 upper bound of its magnitude sum
    a.thr64[(int64_t)unit * a.K * a.L + j] = th;
    a.magmu[(int64_t)unit * a.K * a.L + j] = (float)mg * 1.000001f;
  }
  const int eta = (rho >> 2) & 1, r = 4 * (rho >> 3) + (rho & 3);
  a.thr[(((int64_t)unit * a.ntiles + T) * 2 + eta) * 16 + r] = c;
}

// Float64 / exact re-evaluation of listed (key, projection) pairs, for one wavefront: pairs
// first, first + step, ... below count, 64/LPP of them per sweep (step = 64/LPP * wavefronts).
// LPP lanes share a pair (128/LPP elements each, read in 16-byte pieces from the key row and
// from the transposed projector row); their float64 partial sums are combined by shuffles.
// Any summation order is covered by the float64 error bound; what it cannot decide is summed
// exactly.  The bit is then set or cleared in the stored code word.
// List entry: unit (16 bits) | key (32 bits) | code word x (11 bits) | bit of the word (5 bits).
template <int LPP, class GetEntry>
__device__ inline void recheck_pairs(const HashMfmaArgs& a, long long* limb, uint64_t count,
                                     uint64_t first, uint64_t step, GetEntry get) {
  constexpr int kPieces = 16 / LPP;                      // 8-element pieces per lane
  const int lane = threadIdx.x & 63;
  const uint16_t* Kc = reinterpret_cast<const uint16_t*>(a.Kc);
  const uint16_t* WT = reinterpret_cast<const uint16_t*>(a.wt);
  const int grp = lane / LPP, sl = lane % LPP;
  for (uint64_t i0 = first; i0 < count; i0 += step) {
    const uint64_t i = i0 + grp;
    const bool on = i < count;
    const unsigned long long e = get(on ? i : i0);
    const int x = (int)((e >> 5) & 0x7ff), tbit = (int)(e & 31);
    const int j = (32 * (x / a.K) + tbit) * a.K + x % a.K;
    const int64_t unit = (int64_t)(e >> 48);
    const int64_t k = (int64_t)((e >> 16) & 0xffffffffull);
    const int ub = (int)unit / a.n_kv_heads, uh = (int)unit % a.n_kv_heads;
    const int64_t xoff = (int64_t)ub * a.stride_b + (int64_t)uh * a.stride_h + k * a.stride_n;
    // Products of two bf16 values are exact in float32; they are added in float64 (at most 128
    // roundings of 2^-53 of the magnitude sum) and the centering term mu.W_j comes ready-made in
    // float64 from the threshold kernel, with the same kind of error on its own magnitude sum:
    // |s - exact| < 2^-45 (sum|k w| + sum|mu w|).  The magnitude sums are float32 upper bounds.
    uint4 kraw[kPieces], wraw[kPieces];
#pragma unroll
    for (int p = 0; p < kPieces; ++p) {
      const int d0 = (p * LPP + sl) * 8;
      if (a.kv_fp8) {                                    // e4m3 bytes, widened to the same values in bf16
        const uint2 r8 = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint8_t*>(a.Kc) + xoff + d0);
        kraw[p] = fp8x8_to_bf16x8(r8.x, r8.y);
      } else {
        kraw[p] = *reinterpret_cast<const uint4*>(Kc + xoff + d0);
      }
      wraw[p] = *reinterpret_cast<const uint4*>(WT + (int64_t)j * kHeadDim + d0);
    }
    double s = 0.0;
    float magf = 0.f;
#pragma unroll
    for (int p = 0; p < kPieces; ++p) {
      const uint32_t ku[4] = {kraw[p].x, kraw[p].y, kraw[p].z, kraw[p].w};
      const uint32_t wu[4] = {wraw[p].x, wraw[p].y, wraw[p].z, wraw[p].w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float p0 = __uint_as_float(ku[t] << 16) * __uint_as_float(wu[t] << 16);                 // exact
        const float p1 = __uint_as_float(ku[t] & 0xffff0000u) * __uint_as_float(wu[t] & 0xffff0000u);   // exact
        s += (double)p0;
        s += (double)p1;
        magf += fabsf(p0);
        magf += fabsf(p1);
      }
    }
#pragma unroll
    for (int o = LPP / 2; o > 0; o >>= 1) {
      s += __shfl_xor(s, o);
      magf += __shfl_xor(magf, o);
    }
    double mag = (double)(magf * 1.0001f);
    if (a.mu) {
      s -= a.thr64[unit * (a.K * a.L) + j];
      mag += (double)a.magmu[unit * (a.K * a.L) + j];
    }
    bool bit = s >= 0.0;
    // (1e-42: float32 products below 2^-126 are rounded to multiples of 2^-149; 128 of them)
    const bool unsure = on && sl == 0 && mag > 0.0 && fabs(s) <= kF64Slack * mag + 1e-42;
    uint64_t pending = __ballot(unsure);
    while (pending) {
      const int src = __ffsll((unsigned long long)pending) - 1;
      const int64_t sx = ((int64_t)__shfl((int)(xoff >> 32), src) << 32) | (uint32_t)__shfl((int)(xoff & 0xffffffff), src);
      const int sj = __shfl(j, src);
      const int64_t su = ((int64_t)__shfl((int)(unit >> 32), src) << 32) | (uint32_t)__shfl((int)(unit & 0xffffffff), src);
      const float* smu = a.mu ? a.mu + su * kHeadDim : nullptr;
      const bool r = exact_sign_nonneg_wave(
          limb,
          [&](int d) {
            return a.kv_fp8 ? (double)fp8_to_float(reinterpret_cast<const uint8_t*>(a.Kc)[sx + d])
                            : (double)__uint_as_float((uint32_t)Kc[sx + d] << 16);
          },
          [&](int d) { return (double)__uint_as_float((uint32_t)WT[(int64_t)sj * kHeadDim + d] << 16); },
          [&](int d) { return smu ? (double)smu[d] : 0.0; }, smu != nullptr);
      if (lane == src) bit = r;
      pending &= pending - 1;
    }
    if (on && sl == 0) {
      int kword, kbit;
      key_bit_position(a.K, a.L, x, tbit, &kword, &kbit);
      const uint32_t mask = 1u << kbit;
      uint32_t* word = a.codes + (unit * a.blocks_cap + k / kBlockKeys) * (kBlockKeys * (int64_t)a.NW) +
                       slot_in_block(a.NW, kword, (int)(k % kBlockKeys));
      if (bit) atomicOr(word, mask);
      else atomicAnd(word, ~mask);
    }
  }
}

// One pair of tiles (2 tiles x 8 k-steps x 64 lanes x 16 bytes = 16 KB of fragments), global -> LDS
// without passing through registers: lane l of a wavefront supplies the address of its 16
// bytes, the hardware writes them to (wave-uniform LDS base) + 16 l.  The caller waits for
// the vector-memory counter before the barrier that publishes the stage.
__device__ inline void stage_pair(const uint4* gpair, uint4* stage, int tid, int wave) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(gpair + i * 256 + tid),
        (__attribute__((address_space(3))) void*)(stage + i * 256 + wave * 64), 16, 0, 0);
}

// Three workgroups per compute unit: 152 registers, 46 KB of LDS (two 16 KB stages, the list).
// With stages of four tiles (80 KB, two workgroups per compute unit) the kernel was 10 % slower:
// a workgroup goes through its phases (load and norm the keys, sweep, queue, re-evaluate) one
// after the other, and a third resident workgroup fills more of the gaps.
__global__ __launch_bounds__(256, 3) void hash_keys_mfma_kernel(HashMfmaArgs a) {
  __shared__ uint4 sA0[2 * 8 * 64], sA1[2 * 8 * 64];     // two stages of a tile pair: 2 tiles x 8 k-steps each
  __shared__ float sThr[2][4 * 2 * 16];
  __shared__ unsigned long long sList[kListCapLocal];
  __shared__ unsigned sCount;
  __shared__ long long sLimbs[4][kLimbs];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int unit = blockIdx.y;
  const int kap = lane & 31, hh = lane >> 5;
  const int64_t first = a.first_key, last = a.first_key + a.n_keys;   // [first, last)
  const int64_t cb = first / kBlockKeys + (int64_t)blockIdx.x * 4 + wave;   // my code block
  const bool wave_on = cb * kBlockKeys < last;
  if (tid == 0) sCount = 0;

  const int nquads = a.ntiles / 4;                       // the fragment array holds whole quads
  const uint4* gA = reinterpret_cast<const uint4*>(a.afrag);
  const float* gThr = a.thr + (int64_t)unit * a.ntiles * 32;
  stage_pair(gA, sA0, tid, wave);
  if (tid < 128) sThr[0][tid] = gThr[tid];

  // ---- B operand: my 64 keys, resident in registers for the whole kernel ----
  const uint16_t* Kc = reinterpret_cast<const uint16_t*>(a.Kc);
  const int64_t ubase = (int64_t)(unit / a.n_kv_heads) * a.stride_b + (int64_t)(unit % a.n_kv_heads) * a.stride_h;
  bf16x8 B[2][8];
  float bnd[2];
  int64_t key[2];
  bool key_ok[2];
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    key[bt] = cb * kBlockKeys + bt * 32 + kap;
    key_ok[bt] = wave_on && key[bt] >= first && key[bt] < last;
    const int64_t krow = key_ok[bt] ? key[bt] : first;  // any valid row for masked lanes
    if (a.kv_fp8) {                                      // e4m3 bytes, widened to the same values in bf16
      const uint8_t* row8 = reinterpret_cast<const uint8_t*>(a.Kc) + ubase + krow * a.stride_n + hh * 8;
      uint2 r8[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) r8[s] = *reinterpret_cast<const uint2*>(row8 + s * 16);
#pragma unroll
      for (int s = 0; s < 8; ++s) B[bt][s] = __builtin_bit_cast(bf16x8, fp8x8_to_bf16x8(r8[s].x, r8[s].y));
    } else {
#pragma unroll
      for (int s = 0; s < 8; ++s)
        B[bt][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Kc + ubase + krow * a.stride_n + s * 16 + hh * 8));
    }
  }
  // largest column norm of the projector (from the threshold kernel; requested together with the keys)
  const float wmax = __uint_as_float(*a.wmax_bits);
  const float munorm = a.munorm[unit];
  float knorm[2];
#pragma unroll
  for (int bt = 0; bt < 2; ++bt) {
    // |k|^2 by v_dot2_f32_bf16 (two exact products per instruction, float32 accumulation: the
    // relative error of the norm, below 1e-5, is inside the margin of kGamma)
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
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
    ss += __shfl_xor(ss, 32);                            // the other half of the row
    knorm[bt] = sqrtf(ss) * 1.00002f;
  }

  const int NW = a.NW;
  uint32_t* blk_codes = a.codes + ((int64_t)unit * a.blocks_cap + cb) * (kBlockKeys * (int64_t)NW);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // flagged iff |acc| < bnd, bnd being just above the rigorous bound (so "<=" is covered)
#pragma unroll
  for (int bt = 0; bt < 2; ++bt)
    bnd[bt] = key_ok[bt] ? (kGamma * (knorm[bt] + munorm) * wmax) * 1.000001f + 1e-30f : -1.f;

  // The four words a quad produces are stored one quad later, so that the wait for the
  // staged fragments at the end of a quad does not also wait for a store just issued.
  uint4 pend = make_uint4(0, 0, 0, 0);
  const int64_t mykey = cb * kBlockKeys + lane;
  const bool store_on = wave_on && mykey >= first && mykey < last;
  // Plane words below the last table group are stored as they are (whole quads as 16 bytes);
  // the planes of the last group go through a bit string that keeps only the real tables.
  const int xs = tail_begin(a.K, a.L), Lt = tail_tables(a.L), NQ = a.NQ;
  BitString tail;
  int tail_x = xs;                                       // next key word the bit string fills
  uint4 tbuf = make_uint4(0, 0, 0, 0);                   // words of the 16-byte group being filled
  // Words leave in increasing order, starting at a group boundary: whole groups of four are
  // stored as 16 bytes, the words of the final 1-3 word group one by one.
  auto emit = [&](int x, uint32_t wv) {
    if ((x >> 2) < (NW >> 2)) {
      switch (x & 3) {
        case 0: tbuf.x = wv; break;
        case 1: tbuf.y = wv; break;
        case 2: tbuf.z = wv; break;
        default:
          tbuf.w = wv;
          if (store_on) *reinterpret_cast<uint4*>(blk_codes + (x >> 2) * 256 + lane * 4) = tbuf;
      }
    } else if (store_on) {
      blk_codes[slot_in_block(NW, x, lane)] = wv;
    }
  };
  auto store_quad = [&](int q) {
    const int x0 = q * 4;
    if (x0 + 4 <= xs) {
      if (store_on) *reinterpret_cast<uint4*>(blk_codes + q * 256 + lane * 4) = pend;
      return;
    }
    const uint32_t w4[4] = {pend.x, pend.y, pend.z, pend.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int x = x0 + i;
      if (x >= NQ) break;
      if (x < xs) {
        emit(x, w4[i]);
      } else {
        uint32_t full;
        if (tail.append(w4[i], Lt, &full)) emit(tail_x++, full);
      }
    }
    if (x0 + 4 >= NQ && tail.nbits > 0) emit(tail_x, (uint32_t)tail.acc);   // last quad: the rest
  };
  // One quad: 4 MFMA tiles (2 pairs = 4 code words) against the 64 keys of this wavefront.  The
  // fragments travel in stages of a pair: pair 2q sits in sA0 when the quad starts (published by
  // the last barrier), pair 2q + 1 goes to sA1 while the first pair is multiplied, and the first
  // pair of the next quad goes to sA0 while the second is.
  auto do_quad = [&](int q) {
    const int cur = q & 1;
    const bool more = q + 1 < nquads;
    float stt = -INFINITY;
    if (q > 0) store_quad(q - 1);
    stage_pair(gA + ((int64_t)q * 2 + 1) * 1024, sA1, tid, wave);
    if (more && tid < 128) stt = gThr[(q + 1) * 128 + tid];

    uint32_t wd[2][2];                                   // [pair][key tile] inverted bits, MSB first
    uint32_t fl[2][2];                                   // same bit positions: |acc| <= bound
#pragma unroll
    for (int pair = 0; pair < 2; ++pair) {
      wd[pair][0] = 0; wd[pair][1] = 0;
      fl[pair][0] = 0; fl[pair][1] = 0;
      if (pair == 1) {
        // (every wavefront of the workgroup, working or not, passes here) the second pair has
        // landed in sA1 and everybody is done with sA0: the first pair of the next quad may go there
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (more) stage_pair(gA + ((int64_t)q * 2 + 2) * 1024, sA0, tid, wave);
      }
      if (wave_on) {
        const uint4* sTile = pair ? sA1 : sA0;
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
          const int tile = pair * 2 + tau;
          f32x16 c;
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4) {
            const float4 t4 = *reinterpret_cast<const float4*>(&sThr[cur][(tile * 2 + hh) * 16 + v4 * 4]);
            c[v4 * 4] = t4.x; c[v4 * 4 + 1] = t4.y; c[v4 * 4 + 2] = t4.z; c[v4 * 4 + 3] = t4.w;
          }
          f32x16 acc0 = c, acc1 = c;
          // the A fragment of k-step s + 2 is requested from LDS before the MFMAs of step s are
          // issued (left to itself the compiler emits read, wait, two MFMAs, read, wait, ...)
          bf16x8 ring[3];
          ring[0] = __builtin_bit_cast(bf16x8, sTile[(tau * 8) * 64 + lane]);
          ring[1] = __builtin_bit_cast(bf16x8, sTile[(tau * 8 + 1) * 64 + lane]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            if (s + 2 < 8) ring[(s + 2) % 3] = __builtin_bit_cast(bf16x8, sTile[(tau * 8 + s + 2) * 64 + lane]);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[s % 3], B[0][s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[s % 3], B[1][s], acc1, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            // funnel shift: word = (word << 1) | sign(x).  For the code bit x = acc: the sign
            // is exact for ">= 0" because the accumulator starts from +0 or a non-zero
            // threshold, never -0.  For the flag x = |acc| - bound', negative iff |acc| <= bound.
            wd[pair][0] = __builtin_amdgcn_alignbit(wd[pair][0], __float_as_uint(acc0[r]), 31);
            wd[pair][1] = __builtin_amdgcn_alignbit(wd[pair][1], __float_as_uint(acc1[r]), 31);
            fl[pair][0] = __builtin_amdgcn_alignbit(fl[pair][0], __float_as_uint(fabsf(acc0[r]) - bnd[0]), 31);
            fl[pair][1] = __builtin_amdgcn_alignbit(fl[pair][1], __float_as_uint(fabsf(acc1[r]) - bnd[1]), 31);
          }
        }
        wd[pair][0] = ~wd[pair][0];
        wd[pair][1] = ~wd[pair][1];
      }
    }
    if (wave_on) {
      // lanes < 32 hold words x0 (pair 0) and x0+2 (pair 1) of keys kap / 32+kap, lanes >= 32
      // hold x0+1 and x0+3: one half-swap per pair leaves lane l with the words of key l
      const auto s0 = __builtin_amdgcn_permlane32_swap(wd[0][0], wd[0][1], false, false);
      const auto s1 = __builtin_amdgcn_permlane32_swap(wd[1][0], wd[1][1], false, false);
      pend = make_uint4(s0[0], s0[1], s1[0], s1[1]);     // stored at the start of the next quad
      // Projections too close to zero are queued once per quad, after the staged fragments
      // have landed (the list lives in LDS too).
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      const int nfl = __popc(fl[0][0]) + __popc(fl[0][1]) + __popc(fl[1][0]) + __popc(fl[1][1]);
      if (__ballot(nfl != 0)) {
        unsigned pos = 0;
        if (nfl) pos = atomicAdd(&sCount, (unsigned)nfl);  // one reservation per lane and quad
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
          const unsigned xw = (unsigned)(2 * (q * 2 + pair) + hh) << 5;   // code word of this lane half
#pragma unroll
          for (int bt = 0; bt < 2; ++bt) {
            uint32_t f = fl[pair][bt];
            while (f) {
              const int beta = __ffs(f) - 1;
              f &= f - 1;
              const unsigned long long ent =
                  ((unsigned long long)unit << 48) | ((unsigned long long)key[bt] << 16) | (xw + (unsigned)beta);
              if (pos < kListCapLocal) {
                sList[pos] = ent;
              } else {                                   // rare: the workgroup's list is full
                const unsigned gpos = atomicAdd(a.list_count, 1u);
                if (gpos < a.list_cap) a.list[gpos] = ent;
                else *a.overflow = 1;
              }
              ++pos;
            }
          }
        }
      }
    }

    if (more && tid < 128) sThr[cur ^ 1][tid] = stt;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the next stage has landed in LDS
    __syncthreads();
  };
  for (int q = 0; q < nquads; ++q) do_quad(q);
  store_quad(nquads - 1);

  // ---- re-evaluate this workgroup's flagged pairs while its key rows are still in L2 ----
  // The code words were stored above; the wait holds until L2 has them, the barrier makes
  // that true for all four wavefronts, so the atomic patches below land on top of them.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (lane < kLimbs) sLimbs[wave][lane] = 0;
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  const unsigned cnt = sCount;
  const unsigned keep = cnt < kListCapLocal ? cnt : kListCapLocal;
  if (tid == 0 && cnt) atomicAdd(a.flagged_total, cnt);    // statistics only
  recheck_pairs<4>(a, sLimbs[wave], keep, (uint64_t)wave * 16, 64, [&](uint64_t i) { return sList[i]; });
}

// Re-evaluates the pairs that did not fit a workgroup's own list (normally none).
__global__ __launch_bounds__(256) void recheck_kernel(HashMfmaArgs a) {
  __shared__ long long limbs[4][kLimbs];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (lane < kLimbs) limbs[wave][lane] = 0;
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  if (*a.overflow) return;                               // the direct kernel redoes everything
  const uint64_t count = *a.list_count < a.list_cap ? *a.list_count : a.list_cap;
  recheck_pairs<16>(a, limbs[wave], count, ((uint64_t)blockIdx.x * 4 + wave) * 4, (uint64_t)gridDim.x * 16,
                [&](uint64_t i) { return a.list[i]; });
}

hipError_t launch_hash_keys_mfma(const HashMfmaArgs& a, hipStream_t s) {
  const int rows = a.ntiles * 32;
  hipLaunchKernelGGL(prep_projector_kernel, dim3((unsigned)((rows * 16 + 255) / 256)), dim3(256), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(prep_threshold_kernel, dim3((unsigned)((rows + 255) / 256), (unsigned)a.units), dim3(256), 0, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const int64_t first_blk = a.first_key / kBlockKeys;
  const int64_t last_blk = (a.first_key + a.n_keys - 1) / kBlockKeys;
  const int64_t nblk = last_blk - first_blk + 1;
  hipLaunchKernelGGL(hash_keys_mfma_kernel, dim3((unsigned)((nblk + 3) / 4), (unsigned)a.units), dim3(256), 0, s, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(recheck_kernel, dim3(256), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
