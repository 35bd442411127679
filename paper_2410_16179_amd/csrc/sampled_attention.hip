// One decode step of LSH-sampled attention (Algorithm 1 "MagicPIG Decoding"; Eq. "lsh
// sampling probability"; Eq. "close form"), HBM-bound.
//
// Retrieval by scanning the packed codes of every key (magicpig_sampled_attention):
//   scan_gather_kernel, then merge_partials_kernel.
// Retrieval through the hash tables (magicpig_sampled_attention_tables):
//   lookup_gather_kernel (hash_tables.hip: lookup, gather, scan of the few appended keys in one
//   launch), merge_partials_kernel; or, with many heads, for the count output and for other
//   min_hits: table lookup [+ collision_scan_kernel over the keys appended since the build],
//   gather_estimate_kernel, merge_partials_kernel.
//
// collision scan (scan_blocks)
//   One wavefront per 64-key code block, lane = key: the block is a contiguous 256*NW-byte
//   read, 16 bytes per lane and load.  For each of the G query heads of the KV head the K
//   bit planes of every table word are XNOR-ed with the query's (scalar operands) and
//   AND-ed together; a popcount adds the number of colliding tables.  Keys outside the
//   static set with count >= min_hits are reported as one 64-bit ballot per (head, block).
//   No LDS, no barrier, about 60 VGPRs.
// gather and estimate (gather_estimate_wave)
//   One wavefront per (query head, run of key blocks): the sampled keys are an index list in
//   LDS (gather_estimate_kernel expands the ballots by a wavefront prefix sum; scan_gather_kernel
//   appends to the list while it compares); the static sink and local-window keys ride
//   along in these batches, or, in gather_estimate_kernel, are taken 32 each by wavefronts of
//   their own; rows are gathered four at a time (a quarter wavefront holds one 128-element row)
//   with up to 32 K rows and 32 V rows in flight; q.k, q.(k-mu), |k-mu|^2 are reduced over
//   the 16 lanes of a row, the inclusion probability u_i and the logit q.k/sqrt(d) - log u_i
//   are evaluated once per candidate, and an online max/sum softmax accumulates the weighted
//   V rows.  The wavefront stores a (max, sum, output) partial.
// scan_gather_kernel does both for a run of 4 to 24 key blocks (chosen by the host) in one workgroup;
// collision_scan_kernel / gather_estimate_kernel are the two as separate launches, joined by
// the ballots in HBM.
// merge_partials_kernel combines a head's partials (the "recursive attention" merge of
//   Sec. 4.4) and writes the output row.
#include "attention_common.h"
#include <hip/hip_ext.h>

#ifndef MP_SCAN_BPW
#define MP_SCAN_BPW 1
#endif

namespace mp {

template <int KT, int WDT, int LT, int BPW>
__global__ __launch_bounds__(256) void collision_scan_kernel(AttnArgs a) {
  const Ctx c = resolve_context(a);
  // readfirstlane tells the compiler that the wavefront index (and everything derived from
  // it: KV head, query-code address) is uniform, so those loads become scalar
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t nblk = key_blocks(c.n);
  const int unit = blockIdx.y;
  const int64_t blk0 = a.blk_begin + ((int64_t)blockIdx.x * 4 + wave) * BPW;
  if (blk0 >= nblk) return;
  const int G = a.Hq / a.Hkv;
  const int64_t head0 = (int64_t)(unit / a.Hkv) * a.Hq + (int64_t)(unit % a.Hkv) * G;
  scan_blocks<KT, WDT, LT, BPW, true>(a, c, unit, blk0, lane, 0, G, [&](int h, int64_t blk, uint64_t m) {
    if (lane == 0) a.masks[(head0 + h) * nblk + blk] = m;
  });
}

// rows per quarter wavefront and batch of the stand-alone gather: 32 K and 32 V rows in flight
template <int ET> constexpr int kGatherIters = ET == kFP32 ? 4 : 8;

// One wavefront = one (query head, run of kRangeBlocks key blocks).  blockDim = 64 * G:
// the G wavefronts of a workgroup serve the G heads of one KV head on the same run.
template <int ET>
__global__ __launch_bounds__(512) void gather_estimate_kernel(AttnArgs a) {
  constexpr bool FP32 = ET == kFP32;
  __shared__ uint16_t lists[8][kRangeBlocks * kBlockKeys];
  const Ctx c = resolve_context(a);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int unit = blockIdx.y, range = blockIdx.x;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int G = a.Hq / a.Hkv;
  const int64_t bh = (int64_t)b * a.Hq + (int64_t)g * G + wave;
  const int64_t nblk = key_blocks(c.n);
  const int64_t blk0 = (int64_t)range * kRangeBlocks;
  uint16_t* list = lists[wave];
  HeadVectors<FP32> hv;
  request_head_vectors<FP32>(a, unit, bh, hv);

  // Ranges below nscan cover 16 key blocks of sampled keys; the ranges after them cover the
  // static set T (sink + local window), kStaticPerRange keys each, taken exactly (u = 1).
  const bool is_static = range >= a.nscan;
  int total;
  int64_t static_first = 0;
  if (!is_static) {
    // ---- expand the scan's ballots into an index list (wavefront prefix sum) ----
    uint64_t m = 0;
    if (lane < kRangeBlocks && blk0 + lane < nblk) m = a.masks[bh * nblk + blk0 + lane];
    const int pc = __popcll(m);
    static_assert(kRangeBlocks <= 16, "the ballots of a range are summed over one row of 16 lanes");
    const int incl = row_prefix_sum16(pc);
    total = __builtin_amdgcn_readlane(incl, kRangeBlocks - 1);
    int pos = incl - pc;
    while (m) {
      const int bit = __ffsll((unsigned long long)m) - 1;
      list[pos++] = (uint16_t)(lane * kBlockKeys + bit);
      m &= m - 1;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
  } else {
    static_first = (int64_t)(range - a.nscan) * kStaticPerRange;
    const int64_t left = c.n_static - static_first;
    total = (int)(left < kStaticPerRange ? left : kStaticPerRange);
  }
  float* pp = a.partial + (bh * a.nranges + range) * kPartialStride;
  if (!is_static) {
    gather_estimate_wave<ET, kGatherIters<ET>>(a, unit, bh, total, total, hv,
                               [&](int cc) { return blk0 * kBlockKeys + (int64_t)list[cc]; }, pp);
  } else {
    gather_estimate_wave<ET, kGatherIters<ET>>(a, unit, bh, total, 0, hv,
                               [&](int cc) { return static_key(a, c, static_first + cc); }, pp);
  }
}

// Scan and gather in one launch (the whole context is scanned, no hash tables): a workgroup of
// four wavefronts compares a run of up to kFusedBlocks = 24 consecutive code blocks with the G
// heads' codes (scan_blocks, f_wave_blocks blocks per wavefront one after the other), appends
// the keys each head samples to that head's list in LDS as it goes, and wavefront h then gathers
// and weighs the keys that head h samples from the
// run (16 blocks: about 17 at a sampling rate of 1.6 %, one batch of the 32-row gather).  As
// separate launches the gather follows the scan with two dependent round trips of its own
// (ballots, then rows) on an idle memory system; here the rows of one workgroup travel while
// the others still stream codes, and only the gather of the last workgroups is exposed
// (measured at 32 heads x 98304 keys: 33 us against 25.6 + 13.7 us).  The host picks the run
// length, 4 to 24 blocks: the shortest whose workgroups are all resident at once (16 blocks at
// that shape).  Shorter runs measured the same kernel time there but cost more partials and
// gather batches.  What remains exposed there, after the last block of codes has arrived
// (time stamps): 0.7 us until the four wavefronts meet, 0.6 us candidate positions and row
// addresses, 1.6 us for the rows, 1.3 us estimator, 0.7 us weighted V rows and the partial;
// until then the kernel moves its bytes at the rate of a plain read of the same codes.
// OCC: workgroups per compute unit the kernel is compiled for (see launch_scan_gather_as).
// The grid is one workgroup per run (at 8 KV heads x 98304 keys: 768, exactly what is resident
// at once; workgroups that start late end last).  The keys of the static set T are dealt over
// the runs of their KV head (key j to run j mod runs) and join the gather batches there, so
// they cost neither workgroups nor batches nor partials of their own.
// One partial per (head, run).
// DBG: with the debug outputs (counts, candidate lists).
// ET: element type of the caches (kBF16, kFP32, or kFP8 with bf16 queries).
template <int KT, int WDT, int LT, int ET, bool DBG, int OCC>
__global__ __launch_bounds__(256, OCC) void scan_gather_kernel(AttnArgs a) {
  constexpr bool FP32 = ET == kFP32;
  constexpr int kIt = FP32 ? (kFusedIters + 1) / 2 : kFusedIters;   // the same registers per batch
  constexpr int kSeg = kFusedWaveBlocks * kBlockKeys;      // most keys one wavefront can report for a head
  // seg[h][w]: the keys of the run that head h samples among the blocks of wavefront w, in key
  // order (position in the run, 11 bits); seg_n[h][w]: how many.  Written while the blocks are
  // compared, so that nothing but the row gather is left to do after the last block.
  __shared__ uint16_t seg[8][4][kSeg];
  __shared__ int seg_n[8][4];
  const Ctx c = resolve_context(a);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int unit = blockIdx.y, run = blockIdx.x;
  const int nruns = gridDim.x;                             // = f_nranges
  const int G = a.Hq / a.Hkv;
  const int64_t head0 = (int64_t)(unit / a.Hkv) * a.Hq + (int64_t)(unit % a.Hkv) * G;
  const int64_t nblk = key_blocks(c.n);
  const int wave_blocks = a.f_wave_blocks;                 // 1 .. kFusedWaveBlocks key blocks per wavefront
  const int run_blocks = 4 * wave_blocks;
  const int64_t blk0 = (int64_t)run * run_blocks;
  int found = 0;                                           // lane h: keys of head h found so far by this wavefront
  uint64_t last_found = 0;                                 // keys of the wavefront's last block that some head samples
#pragma unroll 1
  for (int j = 0; j < wave_blocks; ++j) {
    const int bi = wave * wave_blocks + j;
    if (blk0 + bi < nblk) {
      scan_blocks<KT, WDT, LT, 1, DBG>(a, c, unit, blk0 + bi, lane, 0, G, [&](int h, int64_t, uint64_t m) {
        if (m) {                                           // (wave-uniform)
          const int at = __builtin_amdgcn_readlane(found, h);
          const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
          if ((m >> lane) & 1) seg[h][wave][at + below] = (uint16_t)(bi * kBlockKeys + lane);
          if (lane == h) found = at + __popcll(m);
        }
        if (j == wave_blocks - 1) last_found |= m;
      });
    }
  }
  if (lane < G) seg_n[lane][wave] = found;
  // The gather reads its arguments from the kernel argument segment again, through a pointer the
  // compiler cannot trace back: otherwise it loads them all at the start of the kernel and keeps
  // them in scalar registers across the scan, whose query words then no longer fit (50 spills,
  // a reload on every third instruction of the compare loop).
  typedef const AttnArgs __attribute__((address_space(4))) * const_args_ptr;
  const_args_ptr kp = (const_args_ptr)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(kp));
  const AttnArgs& ga = *(const AttnArgs*)kp;
  // ... and all of them here, in one batch of scalar loads that is back before the barrier opens
  // (requested where they are used they cost four dependent round trips at the end of the kernel)
  asm volatile("" ::"s"(ga.q), "s"(ga.Kc), "s"(ga.Vc), "s"(ga.mu), "s"(ga.partial), "s"(ga.Hq), "s"(ga.Hkv), "s"(ga.K), "s"(ga.L),
               "s"(ga.tau), "s"(ga.n_sink), "s"(ga.n_local), "s"(ga.ks_b), "s"(ga.ks_h), "s"(ga.ks_n), "s"(ga.vs_b), "s"(ga.vs_h),
               "s"(ga.vs_n), "s"(ga.f_nranges), "s"(ga.f_touch), "s"(ga.scale));
  asm volatile("" ::"s"(ga.head_ratio[0]), "s"(ga.head_ratio[1]), "s"(ga.head_ratio[2]), "s"(ga.head_ratio[3]), "s"(ga.tail_ratio[0]),
               "s"(ga.tail_ratio[1]), "s"(ga.tail_ratio[2]), "s"(ga.tail_ratio[3]), "s"(ga.tail_ratio[4]), "s"(ga.tail_ratio[5]),
               "s"(ga.tail_ratio[6]), "s"(ga.tail_ratio[7]), "s"(ga.tail_ratio[8]), "s"(ga.tail_ratio[9]), "s"(ga.tail_ratio[10]),
               "s"(ga.tail_ratio[11]), "s"(ga.tail_ratio[12]), "s"(ga.tail_ratio[13]), "s"(ga.tail_ratio[14]), "s"(ga.tail_ratio[15]));
  static_assert(kFastTau == 4 && kTailTerms == 16, "the list above names every ratio");
  // When the workgroups of a launch come in several rounds the memory system is busy whenever one
  // of them reaches its gather, and its rows then take as long as a block of codes.  The rows of
  // the keys found in the last block are requested last of all (block compared, barrier, candidate
  // positions, only then the request): a wavefront touches one word of each of their cache lines
  // here already, so that the gather finds them in, or on their way to, the L2 (measured at batch
  // 16 x 65536 keys: 284 -> 276 us; with all workgroups resident at once it costs half a
  // microsecond instead, and touching the rows of every block costs 10 %).  The touches are
  // loads with a destination, consumed at the end of the kernel; the barrier does not wait for them.
  constexpr int kLines = ET == kFP32 ? 4 : (ET == kFP8 ? 1 : 2);            // 128-byte lines per row
  uint32_t touched[2 * kLines];
#pragma unroll
  for (int l = 0; l < 2 * kLines; ++l) touched[l] = 0;
  if (ga.f_touch && ((last_found >> lane) & 1)) {
    const int64_t key = (blk0 + wave * wave_blocks + wave_blocks - 1) * kBlockKeys + lane;
    const int b = unit / ga.Hkv, g = unit % ga.Hkv;
    const char* kr = (const char*)ga.Kc + ((int64_t)b * ga.ks_b + (int64_t)g * ga.ks_h + key * ga.ks_n) * (kLines * 128 / kHeadDim);
    const char* vr = (const char*)ga.Vc + ((int64_t)b * ga.vs_b + (int64_t)g * ga.vs_h + key * ga.vs_n) * (kLines * 128 / kHeadDim);
#pragma unroll
    for (int l = 0; l < kLines; ++l) {
      touched[2 * l] = *reinterpret_cast<const uint32_t*>(kr + 128 * l);
      touched[2 * l + 1] = *reinterpret_cast<const uint32_t*>(vr + 128 * l);
    }
  }
  // (the barrier orders the LDS writes above: it waits for them, not for loads in flight)
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  for (int h = wave; h < G; h += 4) {
    HeadVectors<FP32> hv;
    request_head_vectors<FP32>(ga, unit, head0 + h, hv);
    // the four wavefronts' keys of head h, one after the other: candidate cc is entry cc - s_w of
    // the last wavefront w whose first candidate s_w is not beyond cc
    const int s1 = __builtin_amdgcn_readfirstlane(seg_n[h][0]);
    const int s2 = s1 + __builtin_amdgcn_readfirstlane(seg_n[h][1]);
    const int s3 = s2 + __builtin_amdgcn_readfirstlane(seg_n[h][2]);
    const int total = s3 + __builtin_amdgcn_readfirstlane(seg_n[h][3]);
    const uint16_t* segh = &seg[h][0][0];
    // static keys run, run + nruns, ... ride along behind the sampled ones
    const int nst = static_share(c, run, nruns);
    gather_estimate_wave<ET, kIt>(ga, unit, head0 + h, total + nst, total, hv,
                                    [&](int cc) {
                                      if (cc >= total) return static_key(ga, c, run + (int64_t)(cc - total) * nruns);
                                      const int w = (cc >= s1) + (cc >= s2) + (cc >= s3);
                                      const int first = w == 0 ? 0 : (w == 1 ? s1 : (w == 2 ? s2 : s3));
                                      return blk0 * kBlockKeys + (int64_t)segh[w * kSeg + cc - first];
                                    },
                                    ga.partial + ((head0 + h) * ga.f_nranges + run) * kPartialStride);
  }
#pragma unroll
  for (int l = 0; l < 2 * kLines; ++l) asm volatile("" ::"v"(touched[l]));
}

// Merges the (max, sum, output) partials of one query head (NWAVES wavefronts: wavefront w takes
// every NWAVES-th group of partials, lane = two output elements).  Every load of a pass is
// issued before any is used - their addresses do not depend on the data - so a pass costs
// one memory round trip; LDS joins the wavefronts.
template <int NWAVES>
__global__ __launch_bounds__(64 * NWAVES) void merge_partials_kernel(AttnArgs a) {
  constexpr int kPer = 16;                    // partials per wavefront and pass
  __shared__ float sm[NWAVES], sl_[NWAVES], so[NWAVES][kHeadDim];
  const int64_t bh = blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const float* hp = a.partial + bh * a.nranges * kPartialStride;
  float m = -INFINITY, l = 0.f, ox = 0.f, oy = 0.f;
  for (int r0 = wave * kPer; r0 < a.nranges; r0 += NWAVES * kPer) {
    float2 oc[kPer];
    float mr[kPer], lr[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const bool ok = r0 + j < a.nranges;
      const float* pp = hp + (int64_t)(ok ? r0 + j : r0) * kPartialStride;
      oc[j] = *reinterpret_cast<const float2*>(pp + 2 * lane);
      mr[j] = ok ? pp[128] : -INFINITY;
      lr[j] = pp[129];
    }
    float mn = m;
#pragma unroll
    for (int j = 0; j < kPer; ++j) mn = fmaxf(mn, mr[j]);
    if (mn > -INFINITY) {
      const float sa = expf(m - mn);
      ox *= sa; oy *= sa; l *= sa;
#pragma unroll
      for (int j = 0; j < kPer; ++j) {
        const float sb = mr[j] > -INFINITY ? expf(mr[j] - mn) : 0.f;
        ox += sb * oc[j].x;
        oy += sb * oc[j].y;
        l += sb * lr[j];
      }
      m = mn;
    }
  }
  if (lane == 0) { sm[wave] = m; sl_[wave] = l; }
  so[wave][2 * lane] = ox;
  so[wave][2 * lane + 1] = oy;
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    float M = sm[0];
#pragma unroll
    for (int w = 1; w < NWAVES; ++w) M = fmaxf(M, sm[w]);
    float acc = 0.f, lt = 0.f;
    if (M > -INFINITY) {
#pragma unroll
      for (int w = 0; w < NWAVES; ++w) {
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

__global__ void zero_output_kernel(float* out, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) out[i] = 0.f;
}

// Ordinary launch, or - when events are given - a launch whose events carry the kernel's own
// begin / end timestamps (what a profiler reports), not the stream's dispatch times.
template <class F, class... Args>
static void launch_timed(F kernel, dim3 grid, dim3 block, hipStream_t s, hipEvent_t start, hipEvent_t stop, Args... args) {
  if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, start, stop, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}

static hipError_t launch_scan(const AttnArgs& a, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  constexpr int kBPW = MP_SCAN_BPW;
  const dim3 block(256);
  const int64_t nscanned = key_blocks(a.n) - a.blk_begin;   // > 0
  const dim3 grid_t((unsigned)((nscanned + 4 * kBPW - 1) / (4 * kBPW)), (unsigned)(a.B * a.Hkv));
#define MP_TUNED(KT, LL)                                                                            \
  if (a.K == KT && a.L == LL) {                                                                     \
    launch_timed(collision_scan_kernel<KT, (LL + 31) / 32, LL - 32 * ((LL + 31) / 32 - 1), kBPW>,  \
                 grid_t, block, s, start, stop, a);                                                 \
    return hipGetLastError();                                                                       \
  }
  MP_TUNED(10, 150) MP_TUNED(9, 120) MP_TUNED(10, 170) MP_TUNED(8, 75) MP_TUNED(10, 220) MP_TUNED(11, 300)
#undef MP_TUNED
  const dim3 grid((unsigned)((nscanned + 3) / 4), (unsigned)(a.B * a.Hkv));
  launch_timed(collision_scan_kernel<0, 0, 0, 1>, grid, block, s, start, stop, a);
  return hipGetLastError();
}

// a wavefront merges 16 partials per pass: enough wavefronts for one pass where that fits
static hipError_t launch_merge(const AttnArgs& a, int64_t heads, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const dim3 grid((unsigned)heads);
  if (a.nranges <= 64) launch_timed(merge_partials_kernel<4>, grid, dim3(256), s, start, stop, a);
  else if (a.nranges <= 128) launch_timed(merge_partials_kernel<8>, grid, dim3(512), s, start, stop, a);
  else launch_timed(merge_partials_kernel<16>, grid, dim3(1024), s, start, stop, a);
  return hipGetLastError();
}

// Workgroups per compute unit the kernel is compiled for: three (up to 168 registers) when the
// whole grid is resident at once - there the fourth could not be used, and the looser register
// allocation measured 0.4 us faster at 32 heads x 98304 keys - and four (128 registers) when the
// workgroups come in several rounds (batch 16 x 65536 keys: 283 against 285 us, and 275 with the
// early touches, which only pay at that occupancy).
template <int KT, int WDT, int LT, int ET, bool DBG>
static void launch_scan_gather_as(const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const dim3 block(256);
  if (a.f_touch) launch_timed(scan_gather_kernel<KT, WDT, LT, ET, DBG, 4>, grid, block, s, start, stop, a);
  else launch_timed(scan_gather_kernel<KT, WDT, LT, ET, DBG, 3>, grid, block, s, start, stop, a);
}

template <int KT, int WDT, int LT>
static void launch_scan_gather_for(const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const bool dbg = a.dbg_counts || a.dbg_cand;
  if (a.is_fp32) {
    if (dbg) launch_scan_gather_as<KT, WDT, LT, kFP32, true>(a, grid, s, start, stop);
    else launch_scan_gather_as<KT, WDT, LT, kFP32, false>(a, grid, s, start, stop);
  } else if (a.kv_fp8) {
    if (dbg) launch_scan_gather_as<KT, WDT, LT, kFP8, true>(a, grid, s, start, stop);
    else launch_scan_gather_as<KT, WDT, LT, kFP8, false>(a, grid, s, start, stop);
  } else {
    if (dbg) launch_scan_gather_as<KT, WDT, LT, kBF16, true>(a, grid, s, start, stop);
    else launch_scan_gather_as<KT, WDT, LT, kBF16, false>(a, grid, s, start, stop);
  }
}

static hipError_t launch_scan_gather(const AttnArgs& a, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const dim3 grid((unsigned)a.f_nranges, (unsigned)(a.B * a.Hkv));
  if (a.K == 10 && a.L == 150) launch_scan_gather_for<10, 5, 22>(a, grid, s, start, stop);
  else if (a.K == 9 && a.L == 120) launch_scan_gather_for<9, 4, 24>(a, grid, s, start, stop);
  else if (a.K == 10 && a.L == 170) launch_scan_gather_for<10, 6, 10>(a, grid, s, start, stop);
  else if (a.K == 8 && a.L == 75) launch_scan_gather_for<8, 3, 11>(a, grid, s, start, stop);
  else if (a.K == 10 && a.L == 220) launch_scan_gather_for<10, 7, 28>(a, grid, s, start, stop);   // App. E (K, L) study
  else if (a.K == 11 && a.L == 300) launch_scan_gather_for<11, 10, 12>(a, grid, s, start, stop);
  else launch_scan_gather_for<0, 0, 0>(a, grid, s, start, stop);
  return hipGetLastError();
}

hipError_t launch_sampled_attention(const AttnArgs& a, const TableArgs* tables, hipStream_t s, hipEvent_t const* ev) {
  const int64_t heads = (int64_t)a.B * a.Hq;
  if (heads <= 0) return hipSuccess;
  if (a.nranges <= 0) {      // no keys: the output is defined as the zero vector
    hipLaunchKernelGGL(zero_output_kernel, dim3((unsigned)((heads * kHeadDim + 255) / 256)), dim3(256), 0, s,
                       a.out, heads * kHeadDim);
    return hipGetLastError();
  }
  hipError_t e;
  // retrieval: stream every key's code, or look the query's codes up in the hash tables and
  // stream only the codes of the keys appended since the tables were built
  if (tables) {
    AttnArgs b = a;
    b.blk_begin = key_blocks(tables->n);                 // tables->n is a.n or a multiple of the block size
    const bool lookup = tables->n > 0, scan = b.blk_begin < key_blocks(a.n);
    const int nslices = (int)((b.blk_begin + kLgSliceBlocks - 1) / kLgSliceBlocks);
    const int app_runs = (int)((key_blocks(a.n) - b.blk_begin + 15) / 16);
    // One launch for lookup, gather, the static set and the few keys appended since the build
    // pays while its workgroups (one per head and slice, one per compute unit at a time) are
    // resident all at once: it removes launches and round trips from a latency-bound step.  Beyond
    // that a second round of workgroups costs more than the launches saved (64 heads x 98304
    // keys: 42.9 against 37.9 us per step), and with many heads the step is throughput-bound:
    // separate lookup and gather launches, each filling the chip with its own kind of work,
    // measured 35-40 % faster (batch 16 x 65536 keys, batch 8 x 131072).
    const bool few = heads * nslices <= kNumCU;
    if (lookup && few && !a.dbg_counts && (a.tau == 1 || a.tau == 2) && app_runs <= nslices) {
      b.nranges = nslices * 16;
      if ((e = launch_lookup_gather(b, *tables, nslices, app_runs, s, ev ? ev[0] : nullptr, ev ? ev[1] : nullptr)) != hipSuccess)
        return e;
      if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
      return launch_merge(b, heads, s, ev ? ev[4] : nullptr, ev ? ev[3] : nullptr);
    }
    if (lookup) {
      e = launch_table_lookup(a, *tables, s, ev ? ev[0] : nullptr, ev && !scan ? ev[1] : nullptr);
      if (e != hipSuccess) return e;
    }
    if (scan) {
      e = launch_scan(b, s, ev && !lookup ? ev[0] : nullptr, ev ? ev[1] : nullptr);
      if (e != hipSuccess) return e;
    }
  } else {
    // whole-context scan: scan and gather in one launch, then the merge over its partials
    if ((e = launch_scan_gather(a, s, ev ? ev[0] : nullptr, ev ? ev[1] : nullptr)) != hipSuccess) return e;
    if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
    AttnArgs b = a;
    b.nranges = a.f_nranges;
    if ((e = launch_merge(b, heads, s, ev ? ev[4] : nullptr, ev ? ev[3] : nullptr)) != hipSuccess) return e;
    return hipGetLastError();
  }
  const dim3 grid((unsigned)a.nranges, (unsigned)(a.B * a.Hkv)), block(64 * (a.Hq / a.Hkv));
  if (a.is_fp32) launch_timed(gather_estimate_kernel<kFP32>, grid, block, s, nullptr, ev ? ev[2] : nullptr, a);
  else if (a.kv_fp8) launch_timed(gather_estimate_kernel<kFP8>, grid, block, s, nullptr, ev ? ev[2] : nullptr, a);
  else launch_timed(gather_estimate_kernel<kBF16>, grid, block, s, nullptr, ev ? ev[2] : nullptr, a);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return launch_merge(a, heads, s, ev ? ev[4] : nullptr, ev ? ev[3] : nullptr);
}

}  // namespace mp
