// One decode step of LSH-sampled attention (Algorithm 1 "MagicPIG Decoding"; Eq. "lsh
// sampling probability"; Eq. "close form"), HBM-bound.
//
// A workgroup owns a chunk of consecutive keys of one (batch, KV head) and serves all G
// query heads of that KV head.
//  1. Collision scan: lane = key.  A wavefront reads one 64-key code block (contiguous
//     256*NW bytes, 16-byte vectors per lane); for every table word the K bit planes are
//     XNOR-ed with the query's and AND-ed together, and a popcount adds the number of
//     colliding tables.  Code traffic is read once and shared by the G heads.
//  2. Compaction: keys with count >= min_hits (and the static sink/local keys) are
//     ballot-compacted into per-head index lists in LDS.
//  3. Gather + estimator: one wavefront per head walks its list, four rows per step (a
//     quarter wavefront holds one 128-element row), 16 K rows and 16 V rows in flight;
//     q.k, q.(k-mu), |k-mu|^2 are reduced across the 16 lanes of a row, the inclusion
//     probability u_i and the logit q.k/sqrt(d) - log u_i are evaluated once per candidate,
//     and an online max/sum softmax accumulates the weighted V rows.
//  4. Each workgroup writes (max, sum, unnormalised output) per head; a merge kernel
//     combines the chunks (the "recursive attention" merge of Sec. 4.4).
#include "mp_common.h"
#include "device_utils.h"

namespace mp {

constexpr int kSegCap = kMaxChunkBlocks / kAttnWaves * kBlockKeys;   // list entries per (head, wave)

// u = P[Binomial(L, x) >= tau], x = p^K, in float32 without cancellation: the complement
// 1 - P[< tau] when that is below one half, otherwise the positive upper-tail terms.
__device__ inline float inclusion_probability(float cosv, int K, int L, int tau) {
  const float c = fminf(fmaxf(cosv, -1.f), 1.f);
  const float p = 1.f - acosf(c) * 0.31830988618379067f;
  float x = 1.f;
  for (int i = 0; i < K; ++i) x *= p;
  if (x >= 1.f) return L >= tau ? 1.f : 0.f;
  if (!(x > 0.f)) return 0.f;
  const float r = x / (1.f - x);
  float t = expf((float)L * log1pf(-x));   // term j = 0
  float head = 0.f;
  for (int j = 0; j < tau; ++j) {
    head += t;
    t *= (float)(L - j) / (float)(j + 1) * r;
  }
  if (head < 0.5f) return 1.f - head;
  float sum = 0.f;
  for (int j = tau; j <= L; ++j) {
    sum += t;
    t *= (float)(L - j) / (float)(j + 1) * r;
    if (t < 1e-9f * sum) break;
  }
  return sum;
}

template <int NW>
__device__ inline void load_code_block(const uint32_t* blkp, int lane, uint32_t (&kw)[NW]) {
  constexpr int full = NW / 4, rem = NW % 4;
#pragma unroll
  for (int g4 = 0; g4 < full; ++g4) {
    const uint4 v = *reinterpret_cast<const uint4*>(blkp + g4 * 256 + lane * 4);
    kw[4 * g4] = v.x; kw[4 * g4 + 1] = v.y; kw[4 * g4 + 2] = v.z; kw[4 * g4 + 3] = v.w;
  }
  if constexpr (rem == 1) {
    kw[4 * full] = blkp[full * 256 + lane];
  } else if constexpr (rem == 2) {
    const uint2 v = *reinterpret_cast<const uint2*>(blkp + full * 256 + lane * 2);
    kw[4 * full] = v.x; kw[4 * full + 1] = v.y;
  } else if constexpr (rem == 3) {
    kw[4 * full] = blkp[full * 256 + lane * 3];
    kw[4 * full + 1] = blkp[full * 256 + lane * 3 + 1];
    kw[4 * full + 2] = blkp[full * 256 + lane * 3 + 2];
  }
}

// FP32: element type of q/K/V.  G: query heads per KV head.  KT, WDT: compile-time K and
// ceil(L/32) for the tuned instantiations, 0 for the generic one (run-time K, L).
template <bool FP32, int G, int KT, int WDT>
__global__ __launch_bounds__(kAttnWaves * 64) void sampled_attention_kernel(AttnArgs a) {
  __shared__ uint16_t list[G][kAttnWaves][kSegCap];
  __shared__ int segcnt[G][kAttnWaves];
  constexpr bool kGeneric = (KT == 0);
  __shared__ uint32_t qlds[kGeneric ? G * 256 : 1];

  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t nblk = key_blocks(a.n);
  const int64_t blk0 = (int64_t)chunk * a.chunk_blocks;
  const int64_t blk1 = blk0 + a.chunk_blocks < nblk ? blk0 + a.chunk_blocks : nblk;
  const int K = kGeneric ? a.K : KT;
  const int Wd = kGeneric ? a.Wd : WDT;
  const int NW = K * Wd;
  const int64_t head0 = (int64_t)b * a.Hq + (int64_t)g * G;
  const uint32_t* qc = a.qcodes + head0 * NW;

  if constexpr (kGeneric) {
    for (int i = threadIdx.x; i < G * NW; i += kAttnWaves * 64) qlds[i] = qc[i];
    __syncthreads();
  }

  // ---- 1 + 2: collision scan and compaction ----
  int mycnt[G];
#pragma unroll
  for (int h = 0; h < G; ++h) mycnt[h] = 0;
  const int64_t local_lo = a.n - a.n_local;

  for (int64_t blk = blk0 + wave; blk < blk1; blk += kAttnWaves) {
    const uint32_t* blkp = a.kcodes + ((int64_t)unit * a.blocks_cap + blk) * (kBlockKeys * (int64_t)NW);
    uint32_t cnt[G];
#pragma unroll
    for (int h = 0; h < G; ++h) cnt[h] = 0;
    if constexpr (!kGeneric) {
      uint32_t kw[KT * WDT];
      load_code_block<KT * WDT>(blkp, lane, kw);
#pragma unroll
      for (int w = 0; w < WDT; ++w) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
          uint32_t same = ~(kw[w * KT] ^ qc[h * NW + w * KT]);
#pragma unroll
          for (int p = 1; p < KT; ++p) {
            same &= ~(kw[w * KT + p] ^ qc[h * NW + w * KT + p]);   // one three-input bit op
          }
          cnt[h] += __popc(same);
        }
      }
    } else {
      for (int w = 0; w < Wd; ++w) {
        uint32_t same[G];
#pragma unroll
        for (int h = 0; h < G; ++h) same[h] = ~0u;
        for (int p = 0; p < K; ++p) {
          const int x = w * K + p;
          const uint32_t kwv = blkp[slot_in_block(NW, x, lane)];
#pragma unroll
          for (int h = 0; h < G; ++h) same[h] &= ~(kwv ^ qlds[h * NW + x]);
        }
#pragma unroll
        for (int h = 0; h < G; ++h) cnt[h] += __popc(same[h]);
      }
    }
    const int64_t i = blk * kBlockKeys + lane;
    const bool valid = i < a.n;
    const bool in_T = i < a.n_sink || i >= local_lo;
    const uint16_t rel = (uint16_t)(i - blk0 * kBlockKeys);
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const bool hit = valid && (in_T || a.tau <= 0 || (int)cnt[h] >= a.tau);
      const uint64_t m = __ballot(hit);
      if (hit) {
        const int pos = mycnt[h] + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
        list[h][wave][pos] = rel;
      }
      mycnt[h] += __popcll(m);
      if (a.dbg_counts && valid) a.dbg_counts[(head0 + h) * a.n + i] = (uint16_t)cnt[h];
      if (a.dbg_cand && hit && !in_T) {
        const int pos = atomicAdd(&a.dbg_ncand[head0 + h], 1);
        if (pos < a.dbg_cand_cap) a.dbg_cand[(head0 + h) * a.dbg_cand_cap + pos] = (int32_t)i;
      }
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h) segcnt[h][wave] = mycnt[h];
  }
  __syncthreads();

  // ---- 3: gather + estimator, one wavefront per head ----
  const int qd = lane >> 4, sl = lane & 15;
  const int64_t kbase = (int64_t)b * a.ks_b + (int64_t)g * a.ks_h + sl * 8;
  const int64_t vbase = (int64_t)b * a.vs_b + (int64_t)g * a.vs_h + sl * 8;
  float muf[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) muf[e] = a.mu ? a.mu[(int64_t)unit * kHeadDim + sl * 8 + e] : 0.f;

  for (int h = wave; h < G; h += kAttnWaves) {
    float qf[8];
    {
      Frag f;
      frag_load<FP32>(a.q, (head0 + h) * kHeadDim + sl * 8, f);
      frag_to_float<FP32>(f, qf);
    }
    float qq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) qq += qf[e] * qf[e];
    const float qnorm = sqrtf(row_sum16(qq));

    float m_run = -INFINITY, l_run = 0.f;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;

    for (int seg = 0; seg < kAttnWaves; ++seg) {
      const int nseg = segcnt[h][seg];
      for (int base = 0; base < nseg; base += 16) {
        Frag kf[4], vf[4];
        int64_t idx[4];
        bool ok[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int c = base + it * 4 + qd;
          ok[it] = c < nseg;
          idx[it] = blk0 * kBlockKeys + (ok[it] ? list[h][seg][c] : 0);
          if (ok[it]) {
            frag_load<FP32>(a.Kc, kbase + idx[it] * a.ks_n, kf[it]);
            frag_load<FP32>(a.Vc, vbase + idx[it] * a.vs_n, vf[it]);
          } else {
            frag_zero<FP32>(kf[it]);
            frag_zero<FP32>(vf[it]);
          }
        }
        // per-candidate reductions; lane sl == it of quarter qd keeps candidate base + 4*it + qd
        float my_dq = 0.f, my_dc = 0.f, my_nn = 0.f;
        int64_t my_i = 0;
        bool my_ok = false;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          float kv[8];
          frag_to_float<FP32>(kf[it], kv);
          float dq = 0.f, dc = 0.f, nn = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float kc = kv[e] - muf[e];
            dq += qf[e] * kv[e];
            dc += qf[e] * kc;
            nn += kc * kc;
          }
          dq = row_sum16(dq);
          dc = row_sum16(dc);
          nn = row_sum16(nn);
          if (sl == it) { my_dq = dq; my_dc = dc; my_nn = nn; my_i = idx[it]; my_ok = ok[it]; }
        }
        float logit = -INFINITY;
        if (sl < 4 && my_ok) {
          logit = my_dq * a.scale;
          const bool in_T = my_i < a.n_sink || my_i >= local_lo;
          if (!in_T && a.tau > 0) {
            const float den = qnorm * sqrtf(my_nn);
            const float cosv = den > 0.f ? my_dc / den : 0.f;
            const float u = fmaxf(inclusion_probability(cosv, a.K, a.L, a.tau), 1.17549435e-38f);
            logit -= logf(u);
          }
        }
        const float m_new = fmaxf(m_run, wave_max(logit));   // finite: at least one candidate is valid
        const float alpha = expf(m_run - m_new);             // m_run = -inf gives 0
        const float wgt = logit > -INFINITY ? expf(logit - m_new) : 0.f;
        l_run = l_run * alpha + wave_sum(wgt);
        m_run = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const float wv = __shfl(wgt, (lane & 48) | it);
          float vv[8];
          frag_to_float<FP32>(vf[it], vv);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += wv * vv[e];
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[e] += __shfl_xor(o[e], 16);
      o[e] += __shfl_xor(o[e], 32);
    }
    float* pp = a.partial + ((head0 + h) * a.nchunk + chunk) * kPartialStride;
    if (lane < 16) {
      *reinterpret_cast<float4*>(pp + sl * 8) = make_float4(o[0], o[1], o[2], o[3]);
      *reinterpret_cast<float4*>(pp + sl * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
    if (lane == 0) { pp[128] = m_run; pp[129] = l_run; }
  }
}

// Combines the per-chunk (max, sum, output) triples of one query head.
__global__ __launch_bounds__(kHeadDim) void merge_partials_kernel(AttnArgs a) {
  const int64_t bh = blockIdx.x;
  const float* pp = a.partial + bh * a.nchunk * kPartialStride;
  float M = -INFINITY;
  for (int c = 0; c < a.nchunk; ++c) M = fmaxf(M, pp[c * kPartialStride + 128]);
  float acc = 0.f, l = 0.f;
  if (M > -INFINITY) {
    for (int c = 0; c < a.nchunk; ++c) {
      const float m = pp[c * kPartialStride + 128];
      if (m > -INFINITY) {
        const float s = expf(m - M);
        acc += s * pp[c * kPartialStride + threadIdx.x];
        l += s * pp[c * kPartialStride + 129];
      }
    }
  }
  a.out[bh * kHeadDim + threadIdx.x] = l > 0.f ? acc / l : 0.f;
}

template <bool FP32, int G>
static hipError_t launch_for_group(const AttnArgs& a, hipStream_t s) {
  const dim3 grid((unsigned)a.nchunk, (unsigned)(a.B * a.Hkv)), block(kAttnWaves * 64);
#define MP_TUNED(KT, WDT)                                                                    \
  if (a.K == KT && a.Wd == WDT) {                                                            \
    hipLaunchKernelGGL((sampled_attention_kernel<FP32, G, KT, WDT>), grid, block, 0, s, a);  \
    return hipGetLastError();                                                                \
  }
  if constexpr (!FP32) {
    if constexpr (G == 4) { MP_TUNED(10, 5) MP_TUNED(9, 4) }
    if constexpr (G == 8) { MP_TUNED(10, 6) }
  } else {
    if constexpr (G == 1) { MP_TUNED(8, 3) }
  }
#undef MP_TUNED
  hipLaunchKernelGGL((sampled_attention_kernel<FP32, G, 0, 0>), grid, block, 0, s, a);
  return hipGetLastError();
}

template <bool FP32>
static hipError_t launch_for_dtype(const AttnArgs& a, hipStream_t s) {
  switch (a.Hq / a.Hkv) {
    case 1: return launch_for_group<FP32, 1>(a, s);
    case 2: return launch_for_group<FP32, 2>(a, s);
    case 4: return launch_for_group<FP32, 4>(a, s);
    case 8: return launch_for_group<FP32, 8>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_sampled_attention(const AttnArgs& a, hipStream_t s) {
  if (a.B * a.Hq <= 0) return hipSuccess;
  if (a.nchunk > 0) {
    const hipError_t e = a.is_fp32 ? launch_for_dtype<true>(a, s) : launch_for_dtype<false>(a, s);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)(a.B * a.Hq)), dim3(kHeadDim), 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
