// Pieces shared by the decode kernels: inclusion probability, code-block loads.
#pragma once
#include "mp_common.h"
#include "device_utils.h"

namespace mp {

typedef const uint32_t __attribute__((address_space(4))) * const_u32_ptr;

// acos(c), |c| <= 1, by the seven-degree polynomial of Abramowitz & Stegun 4.4.46:
// acos(x) = sqrt(1 - x) * poly(x) on [0, 1] with |error| <= 2e-8, reflected for negative x.
__device__ inline float acos_poly(float c) {
  const float x = fabsf(c);
  float p = -0.0012624911f;
  p = fmaf(p, x, 0.0066700901f);
  p = fmaf(p, x, -0.0170881256f);
  p = fmaf(p, x, 0.0308918810f);
  p = fmaf(p, x, -0.0501743046f);
  p = fmaf(p, x, 0.0889789874f);
  p = fmaf(p, x, -0.2145988016f);
  p = fmaf(p, x, 1.5707963050f);
  const float r = __builtin_sqrtf(1.f - x) * p;
  return c < 0.f ? 3.14159265358979f - r : r;
}

// u = P[Binomial(L, x) >= tau], x = p^K, p = 1 - acos(cos)/pi (Eq. "lsh sampling probability",
// Eq. "close form"), in float32 without cancellation: the complement 1 - P[< tau] when that
// is below one half, otherwise the positive upper-tail terms.  With term_j = C(L,j) x^j
// (1-x)^(L-j): term_0 = exp(L log(1-x)), term_{j+1} = term_j * (L-j)/(j+1) * x/(1-x).  The
// ratios (L-j)/(j+1) come from the host (AttnArgs::head_ratio / tail_ratio, scalar operands).
// For min_hits <= kFastTau the upper tail is the nested product term_tau * (1 + rho_tau * (1 +
// rho_tau+1 * ( ... ))) over kTailTerms terms, branch-free: it is only used when
// P[< tau] >= 1/2, i.e. L x is below about tau, where the neglected terms are below 1e-8 of
// the sum.  Larger min_hits sum the tail term by term until it no longer changes the sum.
// log(1-x) is its series below x = 1/8 (8 terms, truncation 7e-9 relative) and the hardware
// logarithm above, where 150 log errors of 1e-7 no longer matter (P[< tau] is tiny there).
// Overall u is accurate to a few 1e-6 relative, which moves log u by as much: three orders
// below the output tolerance.
__device__ inline float inclusion_probability(float cosv, const AttnArgs& a) {
  const int K = a.K, L = a.L, tau = a.tau;
  const float c = fminf(fmaxf(cosv, -1.f), 1.f);
  const float p = 1.f - acos_poly(c) * 0.31830988618379067f;
  float x = 1.f;
  for (int i = 0; i < K; ++i) x *= p;
  if (x >= 1.f) return L >= tau ? 1.f : 0.f;
  if (!(x > 0.f)) return 0.f;
  const float r = __fdividef(x, 1.f - x);
  float lg = 1.f / 9.f;
  lg = fmaf(lg, x, 1.f / 8.f);
  lg = fmaf(lg, x, 1.f / 7.f);
  lg = fmaf(lg, x, 1.f / 6.f);
  lg = fmaf(lg, x, 1.f / 5.f);
  lg = fmaf(lg, x, 1.f / 4.f);
  lg = fmaf(lg, x, 1.f / 3.f);
  lg = fmaf(lg, x, 1.f / 2.f);
  lg = fmaf(lg, x, 1.f);
  lg = x < 0.125f ? -x * lg : __logf(1.f - x);
  float t = __expf((float)L * lg);           // term j = 0
  float head = 0.f;
  if (tau <= kFastTau) {
#pragma unroll
    for (int j = 0; j < kFastTau; ++j) {                   // (constant indices: the ratios are scalar operands)
      if (j < tau) {
        head += t;
        t *= a.head_ratio[j] * r;
      }
    }
    float s = 1.f;
#pragma unroll
    for (int i = kTailTerms - 1; i >= 0; --i) s = fmaf(a.tail_ratio[i] * r, s, 1.f);
    return head < 0.5f ? 1.f - head : t * s;
  }
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

// The context length of the step: the launch-time value, or - when the caller keeps it in device
// memory (a decode loop replayed from a captured graph) - what that word holds now, clamped to
// the value the launch was sized for.  The static set follows it.
// (The kernel arguments themselves are never copied or modified: they stay in the constant
// argument segment, where the compiler reads them with scalar loads, dynamic indices included.)
struct Ctx {
  int64_t n, n_static;
};
__device__ inline Ctx resolve_context(const AttnArgs& a) {
  Ctx c{a.n, a.n_static};
  if (a.n_dev) {
    int64_t n = *a.n_dev;
    n = n < 0 ? 0 : (n > a.n ? a.n : n);
    c.n = n;
    const int64_t st = (int64_t)a.n_sink + a.n_local;
    c.n_static = st < n ? st : n;
  }
  return c;
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
    kw[4 * full] = __builtin_nontemporal_load(blkp + full * 256 + lane);
  } else if constexpr (rem == 2) {
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(blkp + full * 256 + lane * 2));
    kw[4 * full] = v.x; kw[4 * full + 1] = v.y;
  } else if constexpr (rem == 3) {
    kw[4 * full] = __builtin_nontemporal_load(blkp + full * 256 + lane * 3);
    kw[4 * full + 1] = __builtin_nontemporal_load(blkp + full * 256 + lane * 3 + 1);
    kw[4 * full + 2] = __builtin_nontemporal_load(blkp + full * 256 + lane * 3 + 2);
  }
}

// Lanes of block `blk` that hold a real key outside the static set (lane = key): what a query
// head can sample there.
__device__ inline uint64_t eligible_keys(const AttnArgs& a, const Ctx& c, int64_t blk, int lane) {
  const int64_t i = blk * kBlockKeys + lane;
  return __ballot(i < c.n && !(i < a.n_sink || i >= c.n - a.n_local));
}

// The keys of block `blk` that query head `head` samples, as a ballot (lane = key, cnt = its
// number of colliding tables, eligible = eligible_keys of the block); with DBG also the optional
// debug outputs (DBG = false keeps their pointers out of the scalar registers).
template <bool DBG>
__device__ inline uint64_t report_block(const AttnArgs& a, const Ctx& c, int64_t head, int64_t blk, int lane, uint32_t cnt,
                                        uint64_t eligible) {
  const uint64_t m = a.tau <= 0 ? eligible : (__ballot((int)cnt >= a.tau) & eligible);
  if constexpr (DBG) {
    const int64_t i = blk * kBlockKeys + lane;
    const bool hit = (m >> lane) & 1;
    if (a.dbg_counts && i < c.n) a.dbg_counts[head * a.dbg_stride + i] = (uint16_t)cnt;
    if (a.dbg_cand && hit) {
      const int pos = atomicAdd(&a.dbg_ncand[head], 1);
      if (pos < a.dbg_cand_cap) a.dbg_cand[head * a.dbg_cand_cap + pos] = (int32_t)i;
    }
  }
  return m;
}

// One wavefront compares BPW consecutive 64-key code blocks (lane = key) of KV unit `unit`,
// starting at block blk0 < key_blocks(n), with the codes of the query heads h_begin .. h_end-1
// of the unit's G, and hands emit(h, blk, ballot) the sampled keys of every (head, block).
// KT, WDT, LT: compile-time K, ceil(L/32) and tables in the last group for the tuned
// instantiations, 0 for the generic one.
// BPW: all code words of the blocks are requested before the first comparison, and each
// scalar-loaded query word serves BPW keys per lane.
template <int KT, int WDT, int LT, int BPW, bool DBG, class Emit>
__device__ inline void scan_blocks(const AttnArgs& a, const Ctx& c, int unit, int64_t blk0, int lane, int h_begin, int h_end, Emit emit) {
  constexpr bool kGeneric = (KT == 0);
  const int64_t nblk = key_blocks(c.n);
  const int G = a.Hq / a.Hkv;
  const int K = kGeneric ? a.K : KT;
  const int Wd = kGeneric ? a.Wd : WDT;
  const int NQ = K * Wd;                                 // plane words of a query code
  constexpr int kTailWords = kGeneric ? 0 : (KT * LT + 31) / 32;
  constexpr int kNWT = kGeneric ? 1 : KT * (WDT - 1) + kTailWords;   // words of a key code
  const int NW = kGeneric ? a.NW : kNWT;
  const int64_t head0 = (int64_t)(unit / a.Hkv) * a.Hq + (int64_t)(unit % a.Hkv) * G;
  // Query codes are wave-uniform and constant during the kernel: read through the constant
  // address space they are scalar loads into SGPRs and feed the bit operations directly.
  const const_u32_ptr qc = (const_u32_ptr)(a.qcodes + head0 * NQ);
  const uint32_t* blkp = a.kcodes + ((int64_t)unit * a.blocks_cap + blk0) * (kBlockKeys * (int64_t)NW);

  [[maybe_unused]] uint32_t kw[BPW][kNWT];
  // the planes of the last table group, taken out of their bit string once per key
  [[maybe_unused]] uint32_t kt[BPW][kGeneric ? 1 : KT];
  if constexpr (!kGeneric) {
#pragma unroll
    for (int j = 0; j < BPW; ++j) {
      if (blk0 + j < nblk) load_code_block<kNWT>(blkp + j * (kBlockKeys * (int64_t)NW), lane, kw[j]);
#pragma unroll
      for (int p = 0; p < KT; ++p) {
        constexpr int xs = KT * (WDT - 1);
        const int off = p * LT, wi = xs + off / 32, sh = off % 32;
        if (sh == 0) kt[j][p] = kw[j][wi];
        else if (sh + LT <= 32) kt[j][p] = kw[j][wi] >> sh;
        else kt[j][p] = __builtin_amdgcn_alignbit(kw[j][wi + 1], kw[j][wi], sh);
      }
    }
  }

  uint64_t eligible[BPW];
#pragma unroll
  for (int j = 0; j < BPW; ++j) eligible[j] = blk0 + j < nblk ? eligible_keys(a, c, blk0 + j, lane) : 0ull;
#pragma unroll 1
  for (int h = h_begin; h < h_end; ++h) {
    const const_u32_ptr qh = qc + h * NQ;
    uint32_t cnt[BPW];
#pragma unroll
    for (int j = 0; j < BPW; ++j) cnt[j] = 0;
    if constexpr (!kGeneric) {
#pragma unroll
      for (int w = 0; w < WDT; ++w) {
        const bool tail = w == WDT - 1;
        uint32_t same[BPW];
#pragma unroll
        for (int j = 0; j < BPW; ++j) same[j] = ~((tail ? kt[j][0] : kw[j][w * KT]) ^ qh[w * KT]);
#pragma unroll
        for (int p = 1; p < KT; ++p) {
#pragma unroll
          for (int j = 0; j < BPW; ++j)
            same[j] &= ~((tail ? kt[j][p] : kw[j][w * KT + p]) ^ qh[w * KT + p]);   // one 3-input op
        }
        // beyond the real tables of the last group the key planes hold bits of the next plane
        if (tail && LT < 32) {
#pragma unroll
          for (int j = 0; j < BPW; ++j) same[j] &= (1u << (LT & 31)) - 1u;
        }
#pragma unroll
        for (int j = 0; j < BPW; ++j) cnt[j] += __popc(same[j]);
      }
    } else {
      for (int w = 0; w < Wd; ++w) {
        uint32_t same = ~0u;
        for (int p = 0; p < K; ++p) {
          const int x = w * K + p;
          same &= ~(load_plane_word(blkp, NW, K, a.L, x, lane) ^ qh[x]);
        }
        if (w == Wd - 1 && (a.L & 31)) same &= (1u << (a.L & 31)) - 1u;
        cnt[0] += __popc(same);
      }
    }
#pragma unroll
    for (int j = 0; j < BPW; ++j) {
      const int64_t blk = blk0 + j;
      if (blk < nblk) emit(h, blk, report_block<DBG>(a, c, head0 + h, blk, lane, cnt[j], eligible[j]));
    }
  }
}

// j-th key of the static set T: the sink keys, then the local window (every key when the
// context is no longer than n_sink + n_local).
__device__ inline int64_t static_key_of(int64_t n, int64_t n_static, int n_sink, int n_local, int64_t j) {
  const int64_t sink_keys = n_static < n ? n_sink : n_static;
  return j < sink_keys ? j : j + (n - n_local - n_sink);
}
__device__ inline int64_t static_key(const AttnArgs& a, const Ctx& c, int64_t j) {
  return static_key_of(c.n, c.n_static, a.n_sink, a.n_local, j);
}

// The static set dealt over `slots` gather wavefronts of a head: slot s takes the static keys
// s, s + slots, s + 2 slots, ... (at long contexts at most one each), which ride along in the
// batch of its sampled keys instead of costing batches of their own.
__device__ inline int static_share_of(int64_t n_static, int slot, int slots) {
  // (n_static <= n_sink + n_local, two 32-bit counts: a 32-bit division)
  return slot < n_static ? (int)(((uint32_t)n_static - (uint32_t)slot + (uint32_t)slots - 1u) / (uint32_t)slots) : 0;
}
__device__ inline int static_share(const Ctx& c, int slot, int slots) {
  return static_share_of(c.n_static, slot, slots);
}

// The query row and the centering vector of a wavefront's head, eight elements per lane (the
// 16 lanes of a quarter wavefront hold a row).  Requested at the start of the kernel, so that
// they travel together with the ballots instead of after them.
template <bool FP32>
struct HeadVectors {
  Frag q;
  float4 mu0, mu1;
};
template <bool FP32>
__device__ inline void request_head_vectors(const AttnArgs& a, int unit, int64_t bh, HeadVectors<FP32>& hv) {
  const int sl = threadIdx.x & 15;
  frag_load<FP32>(a.q, bh * kHeadDim + sl * 8, hv.q);
  hv.mu0 = make_float4(0.f, 0.f, 0.f, 0.f);
  hv.mu1 = hv.mu0;
  if (a.mu) {
    const float4* mp4 = reinterpret_cast<const float4*>(a.mu + (int64_t)unit * kHeadDim + sl * 8);
    hv.mu0 = mp4[0];
    hv.mu1 = mp4[1];
  }
}

// One wavefront attends the keys key_of(0) .. key_of(total - 1) of query head bh (KV unit
// `unit`) and stores one (output[128], max, sum) partial at `pp`.  A quarter wavefront holds
// one 128-element row; all K and V rows of a batch (kIters rows per quarter wavefront) are
// requested before any is used; q.k, q.(k-mu), |k-mu|^2 are reduced over the 16 lanes of a
// row; the inclusion probability and the logit q.k/sqrt(d) - log u are evaluated once per key
// (the first n_sampled keys only: the keys behind them, static ones, enter with u = 1); an
// online max/sum softmax accumulates the weighted V rows.
// ET: element type of the K / V caches (kBF16, kFP32, or kFP8 with bf16 queries).
template <int ET, int kIters, class KeyOf>
__device__ inline void gather_estimate_wave(const AttnArgs& a, int unit, int64_t bh, int total, int n_sampled,
                                            const HeadVectors<ET == kFP32>& hv, KeyOf key_of, float* pp) {
  static_assert(kIters >= 1 && kIters <= 16, "one lane of a quarter wavefront per row of a batch");
  constexpr bool FP32 = ET == kFP32;
  const int lane = threadIdx.x & 63;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int qd = lane >> 4, sl = lane & 15;
  const int64_t kbase = (int64_t)b * a.ks_b + (int64_t)g * a.ks_h + sl * 8;
  const int64_t vbase = (int64_t)b * a.vs_b + (int64_t)g * a.vs_h + sl * 8;
  float o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // row strides are below 2^31 elements (checked by the host): one 32 x 32 -> 64-bit
  // multiply-add per address
  const uint32_t ksn = (uint32_t)a.ks_n, vsn = (uint32_t)a.vs_n;
  for (int base = 0; base < total; base += 4 * kIters) {
    Frag kf[kIters], vf[kIters];
    bool ok[kIters];
    // quarter-wavefront rounds of this batch that hold at least one row (wave-uniform): the
    // work of the others is skipped
    const int rounds = (total - base + 3) >> 2;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int cc = base + it * 4 + qd;
      ok[it] = cc < total;
      if (it < rounds) {
        const uint32_t idx = (uint32_t)key_of(ok[it] ? cc : base);
        if (ok[it]) {
          frag_load<ET>(a.Kc, kbase + (int64_t)((uint64_t)idx * ksn), kf[it]);
          frag_load<ET>(a.Vc, vbase + (int64_t)((uint64_t)idx * vsn), vf[it]);
        } else {
          frag_zero<ET>(kf[it]);
          frag_zero<ET>(vf[it]);
        }
      } else {
        frag_zero<ET>(kf[it]);
        frag_zero<ET>(vf[it]);
      }
    }
    // (first use of the query and the centering vector: after the rows have been requested)
    const float muf[8] = {hv.mu0.x, hv.mu0.y, hv.mu0.z, hv.mu0.w, hv.mu1.x, hv.mu1.y, hv.mu1.z, hv.mu1.w};
    float qf[8];
    frag_to_float<FP32>(hv.q, qf);
    float qq = 0.f, qm = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { qq += qf[e] * qf[e]; qm += qf[e] * muf[e]; }
    const float qnorm = sqrtf(row_sum16(qq));
    const float qmu = row_sum16(qm);                       // q.(k - mu) = q.k - q.mu
    // lane sl == it of quarter qd keeps candidate base + 4*it + qd
    float my_dq = 0.f, my_nn = 0.f;
    bool my_ok = false;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      if (it >= rounds) break;
      float kv[8];
      frag_to_float<ET>(kf[it], kv);
      float dq = 0.f, nn = 0.f;
      if constexpr (ET != kBF16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) dq += qf[e] * kv[e];
      } else {
        // q.k straight from the stored bf16 pairs (v_dot2c_f32_bf16: two products per instruction)
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        const uint32_t kr[4] = {kf[it].a.x, kf[it].a.y, kf[it].a.z, kf[it].a.w};
        const uint32_t qr[4] = {hv.q.a.x, hv.q.a.y, hv.q.a.z, hv.q.a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          dq = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, kr[e]), __builtin_bit_cast(bf16x2, qr[e]), dq, false);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float kc = kv[e] - muf[e];
        nn += kc * kc;
      }
      dq = row_sum16(dq);
      nn = row_sum16(nn);
      if (sl == it) { my_dq = dq; my_nn = nn; my_ok = ok[it]; }
    }
    const float my_dc = my_dq - qmu;
    float logit = -INFINITY;
    if (sl < kIters && my_ok) {
      logit = my_dq * a.scale;
      if (base + 4 * sl + qd < n_sampled && a.tau > 0) {   // this lane's key: base + 4*sl + qd
        const float den = qnorm * sqrtf(my_nn);
        const float cosv = den > 0.f ? my_dc / den : 0.f;
        const float u = fmaxf(inclusion_probability(cosv, a), 1.17549435e-38f);
        logit -= __logf(u);
      }
    }
    const float m_new = fmaxf(m_run, wave_max(logit));   // finite: the batch is not empty
    const float alpha = __expf(m_run - m_new);           // m_run = -inf gives 0
    const float wgt = logit > -INFINITY ? __expf(logit - m_new) : 0.f;
    l_run = l_run * alpha + wave_sum(wgt);
    m_run = m_new;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      if (it >= rounds) break;
      const float wv = row_bcast16(wgt, it);               // the weight of this quarter wavefront's row
      float vv[8];
      frag_to_float<ET>(vf[it], vv);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] += wv * vv[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    o[e] += __shfl_xor(o[e], 16);
    o[e] += __shfl_xor(o[e], 32);
  }
  if (lane < 16) {
    *reinterpret_cast<float4*>(pp + sl * 8) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(pp + sl * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
  }
  if (lane == 0) { pp[128] = m_run; pp[129] = l_run; }
}

}  // namespace mp
