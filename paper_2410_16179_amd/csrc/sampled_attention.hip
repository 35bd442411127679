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
//  4. Each workgroup writes one (max, sum, unnormalised output) partial per head; a merge
//     kernel combines them (the "recursive attention" merge of Sec. 4.4).
#include "mp_common.h"
#include "device_utils.h"

namespace mp {

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

// FP32: element type of q/K/V.  KT, WDT: compile-time K and ceil(L/32) for the tuned
// instantiations, 0 for the generic one (run-time K, L).  NWAVES: wavefronts per workgroup,
// at least the number G of query heads per KV head.
//
// A workgroup owns the key blocks [part*blocks_per_part, ...) of one (batch, KV head) and
// walks them in chunks of at most NWAVES*kWaveChunkBlocks blocks.  Wavefront v scans blocks
// v, v+NWAVES, ... ; the code words of its next block are requested as soon as the current
// ones have been consumed, so a load is in flight while it compacts and gathers.  Wavefront
// h < G also owns query head h: its running softmax state lives in registers across chunks
// and is written out once, as one (max, sum, output) partial per (head, part).
template <bool FP32, int KT, int WDT, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) void sampled_attention_kernel(AttnArgs a) {
  constexpr int kWaveChunkBlocks = 32 / NWAVES;
  constexpr int kSeg = kWaveChunkBlocks * kBlockKeys;     // list entries per (head, wavefront, chunk)
  constexpr bool kGeneric = (KT == 0);
  constexpr int kIters = FP32 ? 4 : 8;                    // rows per quarter-wavefront and batch
  __shared__ uint16_t list[NWAVES][NWAVES][kSeg];
  __shared__ int segcnt[NWAVES][NWAVES];
  __shared__ uint32_t qlds[kGeneric ? NWAVES * 256 : 1];

  const int unit = blockIdx.y, part = blockIdx.x;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int G = a.Hq / a.Hkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t nblk = key_blocks(a.n);
  const int64_t b0 = (int64_t)part * a.blocks_per_part;
  const int64_t b1 = b0 + a.blocks_per_part < nblk ? b0 + a.blocks_per_part : nblk;
  const int K = kGeneric ? a.K : KT;
  const int Wd = kGeneric ? a.Wd : WDT;
  const int NW = K * Wd;
  const int64_t head0 = (int64_t)b * a.Hq + (int64_t)g * G;
  // Query codes are wave-uniform and constant during the kernel: read through the constant
  // address space they become scalar loads into SGPRs.
  typedef const uint32_t __attribute__((address_space(4))) * const_u32_ptr;
  const const_u32_ptr qc = (const_u32_ptr)(a.qcodes + head0 * NW);
  const uint32_t* ucodes = a.kcodes + (int64_t)unit * a.blocks_cap * (kBlockKeys * (int64_t)NW);
  const int64_t local_lo = a.n - a.n_local;

  if constexpr (kGeneric) {
    for (int i = threadIdx.x; i < G * NW; i += NWAVES * 64) qlds[i] = a.qcodes[head0 * NW + i];
    __syncthreads();
  }

  // gather-side state of this wavefront's head
  const int qd = lane >> 4, sl = lane & 15;
  const int64_t kbase = (int64_t)b * a.ks_b + (int64_t)g * a.ks_h + sl * 8;
  const int64_t vbase = (int64_t)b * a.vs_b + (int64_t)g * a.vs_h + sl * 8;
  const bool owner = wave < G;
  float muf[8], qf[8], o[8];
  float qnorm = 0.f, m_run = -INFINITY, l_run = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { muf[e] = 0.f; qf[e] = 0.f; o[e] = 0.f; }
  if (owner) {
    if (a.mu) {
#pragma unroll
      for (int e = 0; e < 8; ++e) muf[e] = a.mu[(int64_t)unit * kHeadDim + sl * 8 + e];
    }
    Frag f;
    frag_load<FP32>(a.q, (head0 + wave) * kHeadDim + sl * 8, f);
    frag_to_float<FP32>(f, qf);
    float qq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) qq += qf[e] * qf[e];
    qnorm = sqrtf(row_sum16(qq));
  }

  [[maybe_unused]] uint32_t kw[kGeneric ? 1 : KT * WDT];
  int64_t blk = b0 + wave;
  if constexpr (!kGeneric) {
    if (blk < b1) load_code_block<KT * WDT>(ucodes + blk * (kBlockKeys * (int64_t)NW), lane, kw);
  }

  for (int64_t c0 = b0; c0 < b1; c0 += NWAVES * kWaveChunkBlocks) {
    const int64_t c1 = c0 + NWAVES * kWaveChunkBlocks < b1 ? c0 + NWAVES * kWaveChunkBlocks : b1;
    // ---- collision scan + compaction of this chunk ----
    int cntv = 0;                                   // lane h: entries of head h in my segment
    for (; blk < c1; blk += NWAVES) {
      const uint32_t* blkp = ucodes + blk * (kBlockKeys * (int64_t)NW);
      const int64_t i = blk * kBlockKeys + lane;
      const bool valid = i < a.n;
      const bool in_T = i < a.n_sink || i >= local_lo;
      const uint16_t rel = (uint16_t)(i - c0 * kBlockKeys);
#pragma unroll 1
      for (int h = 0; h < G; ++h) {
        uint32_t cnt = 0;
        if constexpr (!kGeneric) {
          const const_u32_ptr qh = qc + h * (KT * WDT);
#pragma unroll
          for (int w = 0; w < WDT; ++w) {
            uint32_t same = ~(kw[w * KT] ^ qh[w * KT]);
#pragma unroll
            for (int p = 1; p < KT; ++p) same &= ~(kw[w * KT + p] ^ qh[w * KT + p]);   // one 3-input op
            cnt += __popc(same);
          }
        } else {
          for (int w = 0; w < Wd; ++w) {
            uint32_t same = ~0u;
            for (int p = 0; p < K; ++p) {
              const int x = w * K + p;
              same &= ~(blkp[slot_in_block(NW, x, lane)] ^ qlds[h * NW + x]);
            }
            cnt += __popc(same);
          }
        }
        const bool hit = valid && (in_T || a.tau <= 0 || (int)cnt >= a.tau);
        const uint64_t m = __ballot(hit);
        const int base = __builtin_amdgcn_readlane(cntv, h);
        if (hit) {
          const int pos = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
          list[h][wave][pos] = rel;
        }
        if (lane == h) cntv += __popcll(m);
        if (a.dbg_counts && valid) a.dbg_counts[(head0 + h) * a.n + i] = (uint16_t)cnt;
        if (a.dbg_cand && hit && !in_T) {
          const int pos = atomicAdd(&a.dbg_ncand[head0 + h], 1);
          if (pos < a.dbg_cand_cap) a.dbg_cand[(head0 + h) * a.dbg_cand_cap + pos] = (int32_t)i;
        }
      }
      if constexpr (!kGeneric) {                      // request my next block's code words
        if (blk + NWAVES < b1)
          load_code_block<KT * WDT>(ucodes + (blk + NWAVES) * (kBlockKeys * (int64_t)NW), lane, kw);
      }
    }
    if (lane < G) segcnt[lane][wave] = cntv;
    __syncthreads();

    // ---- gather + estimator: wavefront h serves head h ----
    if (owner) {
      for (int seg = 0; seg < NWAVES; ++seg) {
        const int nseg = segcnt[wave][seg];
        for (int base = 0; base < nseg; base += 4 * kIters) {
          Frag kf[kIters], vf[kIters];
          int64_t idx[kIters];
          bool ok[kIters];
#pragma unroll
          for (int it = 0; it < kIters; ++it) {
            const int c = base + it * 4 + qd;
            ok[it] = c < nseg;
            idx[it] = c0 * kBlockKeys + (ok[it] ? list[wave][seg][c] : 0);
            if (ok[it]) {
              frag_load<FP32>(a.Kc, kbase + idx[it] * a.ks_n, kf[it]);
              frag_load<FP32>(a.Vc, vbase + idx[it] * a.vs_n, vf[it]);
            } else {
              frag_zero<FP32>(kf[it]);
              frag_zero<FP32>(vf[it]);
            }
          }
          // lane sl == it of quarter qd keeps candidate base + 4*it + qd
          float my_dq = 0.f, my_dc = 0.f, my_nn = 0.f;
          int64_t my_i = 0;
          bool my_ok = false;
#pragma unroll
          for (int it = 0; it < kIters; ++it) {
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
          if (sl < kIters && my_ok) {
            logit = my_dq * a.scale;
            const bool in_T = my_i < a.n_sink || my_i >= local_lo;
            if (!in_T && a.tau > 0) {
              const float den = qnorm * sqrtf(my_nn);
              const float cosv = den > 0.f ? my_dc / den : 0.f;
              const float u = fmaxf(inclusion_probability(cosv, a.K, a.L, a.tau), 1.17549435e-38f);
              logit -= logf(u);
            }
          }
          const float m_new = fmaxf(m_run, wave_max(logit));   // finite: the batch is not empty
          const float alpha = expf(m_run - m_new);             // m_run = -inf gives 0
          const float wgt = logit > -INFINITY ? expf(logit - m_new) : 0.f;
          l_run = l_run * alpha + wave_sum(wgt);
          m_run = m_new;
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
          for (int it = 0; it < kIters; ++it) {
            const float wv = __shfl(wgt, (lane & 48) | it);
            float vv[8];
            frag_to_float<FP32>(vf[it], vv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += wv * vv[e];
          }
        }
      }
    }
    __syncthreads();
  }

  if (owner) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      o[e] += __shfl_xor(o[e], 16);
      o[e] += __shfl_xor(o[e], 32);
    }
    float* pp = a.partial + ((head0 + wave) * a.nparts + part) * kPartialStride;
    if (lane < 16) {
      *reinterpret_cast<float4*>(pp + sl * 8) = make_float4(o[0], o[1], o[2], o[3]);
      *reinterpret_cast<float4*>(pp + sl * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
    if (lane == 0) { pp[128] = m_run; pp[129] = l_run; }
  }
}

// Combines the (max, sum, output) partials of one query head: four wavefronts take every
// fourth partial with an online rescale, lane = two output elements; LDS joins the four.
__global__ __launch_bounds__(256) void merge_partials_kernel(AttnArgs a) {
  __shared__ float sm[4], sl_[4], so[4][kHeadDim];
  const int64_t bh = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float* pp = a.partial + bh * a.nparts * kPartialStride;
  float m = -INFINITY, l = 0.f, ox = 0.f, oy = 0.f;
#pragma unroll 4
  for (int c = wave; c < a.nparts; c += 4) {
    const float mc = pp[c * kPartialStride + 128];
    const float lc = pp[c * kPartialStride + 129];
    const float2 oc = *reinterpret_cast<const float2*>(pp + c * kPartialStride + 2 * lane);
    const float mn = fmaxf(m, mc);
    if (mn > -INFINITY) {
      const float sa = expf(m - mn), sb = expf(mc - mn);
      ox = ox * sa + oc.x * sb;
      oy = oy * sa + oc.y * sb;
      l = l * sa + lc * sb;
      m = mn;
    }
  }
  if (lane == 0) { sm[wave] = m; sl_[wave] = l; }
  so[wave][2 * lane] = ox;
  so[wave][2 * lane + 1] = oy;
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    const float M = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float acc = 0.f, lt = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        if (sm[w] > -INFINITY) {
          const float s = expf(sm[w] - M);
          acc += s * so[w][threadIdx.x];
          lt += s * sl_[w];
        }
      }
    }
    a.out[bh * kHeadDim + threadIdx.x] = lt > 0.f ? acc / lt : 0.f;
  }
}

template <bool FP32, int NWAVES>
static hipError_t launch_main(const AttnArgs& a, hipStream_t s) {
  const dim3 grid((unsigned)a.nparts, (unsigned)(a.B * a.Hkv)), block(NWAVES * 64);
#define MP_TUNED(KT, WDT)                                                                        \
  if (a.K == KT && a.Wd == WDT) {                                                                \
    hipLaunchKernelGGL((sampled_attention_kernel<FP32, KT, WDT, NWAVES>), grid, block, 0, s, a); \
    return hipGetLastError();                                                                    \
  }
  if constexpr (!FP32) {
    if constexpr (NWAVES == 4) { MP_TUNED(10, 5) MP_TUNED(9, 4) }
    if constexpr (NWAVES == 8) { MP_TUNED(10, 6) }
  } else {
    if constexpr (NWAVES == 4) { MP_TUNED(8, 3) }
  }
#undef MP_TUNED
  hipLaunchKernelGGL((sampled_attention_kernel<FP32, 0, 0, NWAVES>), grid, block, 0, s, a);
  return hipGetLastError();
}

hipError_t launch_sampled_attention(const AttnArgs& a, hipStream_t s) {
  if (a.B * a.Hq <= 0) return hipSuccess;
  if (a.nparts > 0) {
    const int G = a.Hq / a.Hkv;
    hipError_t e;
    if (G > 4) e = a.is_fp32 ? launch_main<true, 8>(a, s) : launch_main<false, 8>(a, s);
    else e = a.is_fp32 ? launch_main<true, 4>(a, s) : launch_main<false, 4>(a, s);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)(a.B * a.Hq)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace mp
