// Bucketed LSH hash tables in HBM (Algorithm 1: S = Query(HT, q_code); Sec. 4.4 (4)
// "Retrieval"; App. E.2: L tables per key-value head, one key index per key and table).
//
// Per (batch, KV head) and table t the keys are counting-sorted by their K-bit code:
// offsets[t][c] .. offsets[t][c+1] delimits, inside indices[t][], the keys whose code in table
// t is c.  A decode step then touches only the L buckets its query codes select (about
// L*n/2^K indices per head) instead of every key's code: the same sample S as the collision
// scan at a small fraction of its bytes.
//   ht_build_kernel<false>: histogram of the codes of 32 (or fewer) tables in LDS -> offsets.
//   ht_build_kernel<true> : second pass, scatters key indices to their buckets.
//   With a large workspace the first pass also writes every key's code per table (16 bits,
//   table-major) and the bucket fill levels at the start of every window of 16384 keys, and
//   ht_place_kernel replaces the second pass: one workgroup places one window of one table, so
//   the 4-byte stores to a bucket come close together in time and combine into whole lines in
//   L2 (the one-pass scatter keeps thousands of lines half written per workgroup and writes
//   each store to HBM on its own).
//   lookup_gather_kernel  : the decode step's retrieval for min_hits 1 or 2: one workgroup per
//       (query head, slice of 16384 keys: one window of the build) reads the L buckets, marks the keys of its slice in
//       LDS bitmaps and gathers and weighs them right away; the few keys appended since the
//       build are found by the collision scan in the same workgroups.
//   table_lookup_kernel, table_lookup_bitmap_kernel: the lookup alone (hit counts per key in
//       LDS byte counters, or seen / seen-twice bitmaps): they emit the same 64-bit ballots
//       (count >= min_hits, key not static) that collision_scan_kernel emits, for the separate
//       gather and merge kernels; used for the count output, other min_hits, and when more
//       keys were appended than the one-launch form takes.
#include "attention_common.h"
#include <hip/hip_ext.h>

namespace mp {

// 64-key blocks per workgroup of the counting lookup: 32 KB of hit counters, one byte per key up
// to 255 tables, two bytes beyond (a key can collide in every table)
template <int BITS> constexpr int kLookupRunBlocks = 512 * 8 / BITS;

// tables handled by one build workgroup: as many histograms of 2^K counters as fit 64 KB of LDS
__host__ __device__ inline int ht_tables_per_pass(int K) {
  const int fit = (64 * 1024) / (4 << K);
  return fit >= 32 ? 32 : (fit >= 16 ? 16 : (fit >= 8 ? 8 : 4));
}

// SCATTER = false: count codes, write offsets.  SCATTER = true: read offsets, place indices.
template <bool SCATTER>
__global__ __launch_bounds__(256) void ht_build_kernel(TableArgs a) {
  extern __shared__ uint32_t hist[];                  // [tables in this pass][2^K]
  const int unit = blockIdx.y;
  const int tpp = ht_tables_per_pass(a.K);
  const int passes = 32 / tpp;
  const int w = blockIdx.x / passes, beta0 = (blockIdx.x % passes) * tpp;
  const int nb = 1 << a.K;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  uint32_t* offs = a.offsets + (int64_t)unit * a.L * (nb + 1);
  uint32_t* idxs = a.indices + (int64_t)unit * a.L * a.n_cap;

  for (int i = tid; i < tpp * nb; i += 256) {
    const int t = 32 * w + beta0 + i / nb;
    hist[i] = (SCATTER && t < a.L) ? offs[(int64_t)t * (nb + 1) + i % nb] : 0u;
  }
  __syncthreads();

  const int64_t nblk = key_blocks(a.n);
  const uint32_t* ucodes = a.kcodes + (int64_t)unit * a.blocks_cap * (kBlockKeys * (int64_t)a.NW);
  const bool windowed = !SCATTER && a.codes16 != nullptr;
  // (the lookup reads from the header whether the buckets are ordered by window)
  if (!SCATTER && blockIdx.x == 0 && blockIdx.y == 0 && tid == 0) a.header[0] = windowed ? (uint32_t)a.windows : 0u;
  constexpr int64_t kWinBlocks = kBuildWindow / kBlockKeys;
  const int64_t nwin = windowed ? a.windows : 1;
  for (int64_t win = 0; win < nwin; ++win) {
  if (windowed) {
    // fill levels of the buckets before this window (cumulative histogram so far)
    __syncthreads();
    for (int i = tid; i < tpp * nb; i += 256) {
      const int t = 32 * w + beta0 + i / nb;
      if (t < a.L) a.wincum[(((int64_t)unit * a.L + t) * a.windows + win) * nb + i % nb] = hist[i];
    }
    __syncthreads();
  }
  const int64_t blk_lo = windowed ? win * kWinBlocks : 0;
  const int64_t blk_hi = windowed ? (nblk < blk_lo + kWinBlocks ? nblk : blk_lo + kWinBlocks) : nblk;
  for (int64_t blk = blk_lo + wave; blk < blk_hi; blk += 4) {
    const int64_t key = blk * kBlockKeys + lane;
    const uint32_t* blkp = ucodes + blk * (kBlockKeys * (int64_t)a.NW);
    uint32_t kw[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) kw[b] = b < a.K ? load_plane_word(blkp, a.NW, a.K, a.L, w * a.K + b, lane) : 0u;
    if (key < a.n) {
      for (int bb = 0; bb < tpp; ++bb) {
        const int beta = beta0 + bb;
        if (32 * w + beta >= a.L) break;
        uint32_t code = 0;
#pragma unroll
        for (int b = 0; b < 16; ++b) code |= ((kw[b] >> beta) & 1u) << b;
        const uint32_t pos = atomicAdd(&hist[bb * nb + code], 1u);
        if (SCATTER) idxs[(int64_t)(32 * w + beta) * a.n_cap + pos] = (uint32_t)key;
        if (windowed) a.codes16[((int64_t)unit * a.L + 32 * w + beta) * (a.blocks_cap * kBlockKeys) + key] = (uint16_t)code;
      }
    }
  }
  }
  if (SCATTER) return;
  __syncthreads();
  // exclusive prefix sum of every table's histogram -> offsets (one wavefront per table)
  for (int bb = wave; bb < tpp; bb += 4) {
    const int t = 32 * w + beta0 + bb;
    if (t >= a.L) break;
    const int per = (nb + 63) / 64;                   // consecutive bins per lane
    uint32_t local = 0;
    for (int j = 0; j < per; ++j) {
      const int c = lane * per + j;
      if (c < nb) local += hist[bb * nb + c];
    }
    uint32_t incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t v = __shfl_up(incl, o);
      if (lane >= o) incl += v;
    }
    uint32_t run = incl - local;
    for (int j = 0; j < per; ++j) {
      const int c = lane * per + j;
      if (c < nb) {
        offs[(int64_t)t * (nb + 1) + c] = run;
        run += hist[bb * nb + c];
      }
    }
    if (lane == 63) offs[(int64_t)t * (nb + 1) + nb] = incl;
  }
}

// Places the keys of one window into the buckets of one table.  The window is counting-sorted
// by bucket in LDS (its bucket sizes are the differences of the fill levels the first pass
// left), then every bucket's piece is copied to its place - offsets[c] + keys of bucket c in
// earlier windows - by one wavefront with consecutive lanes on consecutive entries, so the
// index array is written in whole contiguous pieces.
__global__ __launch_bounds__(256) void ht_place_kernel(TableArgs a) {
  extern __shared__ uint32_t lds[];
  const int nb = 1 << a.K;
  uint32_t* cursor = lds;                                              // [2^K] next free slot of the bucket's piece
  uint16_t* cnt = reinterpret_cast<uint16_t*>(lds + nb);               // [2^K] keys of the bucket in this window
  uint16_t* sorted = cnt + nb;                                         // [kBuildWindow] key offsets, bucket-major
  __shared__ uint32_t wsum[4];
  const int win = blockIdx.x, t = blockIdx.y, unit = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const uint32_t* offs = a.offsets + ((int64_t)unit * a.L + t) * (nb + 1);
  const uint32_t* cum = a.wincum + (((int64_t)unit * a.L + t) * a.windows + win) * nb;
  const bool last = win == a.windows - 1;
  // bucket sizes of the window and their exclusive prefix sums (thread = run of consecutive buckets)
  const int per = nb / 256 > 0 ? nb / 256 : 1;                         // nb is a power of two
  uint32_t run = 0;
  for (int j = 0; j < per; ++j) {
    const int c = tid * per + j;
    if (c < nb) {
      const uint32_t after = last ? offs[c + 1] - offs[c] : cum[nb + c];
      const uint32_t n_c = after - cum[c];
      cnt[c] = (uint16_t)n_c;
      run += n_c;
    }
  }
  uint32_t incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t v = __shfl_up(incl, o);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  uint32_t base = incl - run;
  for (int v = 0; v < wave; ++v) base += wsum[v];
  for (int j = 0; j < per; ++j) {
    const int c = tid * per + j;
    if (c < nb) {
      cursor[c] = base;
      base += cnt[c];
    }
  }
  __syncthreads();
  // counting sort of the window's keys
  const uint16_t* codes = a.codes16 + ((int64_t)unit * a.L + t) * (a.blocks_cap * kBlockKeys);   // rows of whole blocks
  const int64_t k0 = (int64_t)win * kBuildWindow;
  const int64_t k1 = k0 + kBuildWindow < a.n ? k0 + kBuildWindow : a.n;
  for (int64_t kb = k0 + (int64_t)tid * 8; kb < k1; kb += 256 * 8) {
    const uint4 raw = *reinterpret_cast<const uint4*>(codes + kb);
    const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t code = (u[e >> 1] >> (16 * (e & 1))) & 0xffffu;
      if (kb + e < k1) sorted[atomicAdd(&cursor[code], 1u)] = (uint16_t)(kb + e - k0);
    }
  }
  __syncthreads();
  // copy out: wavefront v takes the buckets of every fourth group of 64; cursor[c] now marks
  // the end of bucket c's piece
  uint32_t* idxs = a.indices + ((int64_t)unit * a.L + t) * a.n_cap;
  for (int c0 = wave * 64; c0 < nb; c0 += 256) {
    const int c = c0 + lane;
    uint32_t gb = 0, le = 0, n_c = 0;
    if (c < nb) {
      gb = offs[c] + cum[c];
      le = cursor[c];
      n_c = cnt[c];
    }
    for (int j = 0; j < 64 && c0 + j < nb; ++j) {
      const uint32_t g = __shfl(gb, j), e = __shfl(le, j), m = __shfl(n_c, j);
      for (uint32_t i = lane; i < m; i += 64) idxs[g + i] = (uint32_t)k0 + sorted[e - m + i];
    }
  }
}

template <int BITS>
__global__ __launch_bounds__(1024) void table_lookup_kernel(AttnArgs a, TableArgs tb) {
  constexpr int kLookupRunKeys = kLookupRunBlocks<BITS> * kBlockKeys;
  constexpr int kPerWord = 32 / BITS;                  // counters per 32-bit LDS word
  constexpr uint32_t kCntMask = (1u << BITS) - 1u;
  __shared__ uint32_t counters[kLookupRunKeys / kPerWord];
  __shared__ uint32_t bstart[512], blen[512];
  const Ctx cx = resolve_context(a);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int run = blockIdx.x;
  const int64_t bh = blockIdx.y;
  const int G = a.Hq / a.Hkv;
  const int64_t unit = (bh / a.Hq) * a.Hkv + (bh % a.Hq) / G;
  const int nb = 1 << a.K;
  const uint32_t* offs = tb.offsets + unit * a.L * (nb + 1);
  const uint32_t* idxs = tb.indices + unit * a.L * tb.n_cap;
  const int64_t key0 = (int64_t)run * kLookupRunKeys;

  __shared__ uint32_t qs[256];
  for (int i = tid; i < kLookupRunKeys / kPerWord; i += 1024) counters[i] = 0u;
  if (tid < a.NQ) qs[tid] = a.qcodes[bh * a.NQ + tid];   // one round trip for the query's words
  __syncthreads();
  // bucket of every table: the query's K-bit code of table t selects offsets[t][code..code+1]
  for (int t = tid; t < a.L; t += 1024) {
    const uint32_t* qw = qs + (t >> 5) * a.K;
    uint32_t code = 0;
    for (int b = 0; b < a.K; ++b) code |= ((qw[b] >> (t & 31)) & 1u) << b;
    const uint32_t s0 = offs[(int64_t)t * (nb + 1) + code], s1 = offs[(int64_t)t * (nb + 1) + code + 1];
    bstart[t] = s0;
    blen[t] = s1 - s0;
  }
  __syncthreads();

  // wavefront v reads tables v, v+16, ...: up to 128 entries of each bucket are requested
  // before any is used; longer buckets are finished in a loop
  constexpr int kMaxB = 32;                           // L <= 512 tables over 16 wavefronts
  uint32_t e0[kMaxB], e1[kMaxB];
  const uint32_t ukey0 = (uint32_t)key0;
  const int nbk = (a.L - wave + 15) >> 4;             // buckets of this wavefront
#pragma unroll
  for (int k = 0; k < kMaxB; ++k) {
    e0[k] = 0xffffffffu; e1[k] = 0xffffffffu;
    if (k < nbk) {
      const int t = wave + 16 * k;
      const uint32_t len = blen[t];
      const uint32_t* p = idxs + (int64_t)t * tb.n_cap + bstart[t];
      if ((uint32_t)lane < len) e0[k] = p[lane];
      if ((uint32_t)lane + 64 < len) e1[k] = p[lane + 64];
    }
  }
  // a key outside this run (or the "no entry" marker) wraps to a value >= kLookupRunKeys
  auto count_key = [&](uint32_t key) {
    const uint32_t rel = key - ukey0;
    if (rel < (uint32_t)kLookupRunKeys) atomicAdd(&counters[rel / kPerWord], 1u << (BITS * (rel % kPerWord)));
  };
#pragma unroll
  for (int k = 0; k < kMaxB; ++k) {
    if (k < nbk) {
      count_key(e0[k]);
      count_key(e1[k]);
      const int t = wave + 16 * k;
      if (blen[t] > 128) {
        const uint32_t* p = idxs + (int64_t)t * tb.n_cap + bstart[t];
        for (uint32_t j = 128 + lane; j < blen[t]; j += 64) count_key(p[j]);
      }
    }
  }
  __syncthreads();

  // ballots of the blocks the tables cover: a thread takes 32 consecutive keys (half a block)
  const int64_t nblk = key_blocks(cx.n);
  for (int part = tid; part < kLookupRunKeys / 32; part += 1024) {
    const int64_t kfirst = key0 + (int64_t)part * 32;
    if (kfirst >= key_blocks(tb.n) * kBlockKeys) break;
    // positions of this thread's keys that are real and outside the static set
    const int64_t lo = (a.n_sink > kfirst ? a.n_sink : kfirst) - kfirst;
    const int64_t hi_key = cx.n - a.n_local < cx.n ? cx.n - a.n_local : cx.n;
    const int64_t hi = (hi_key < kfirst + 32 ? hi_key : kfirst + 32) - kfirst;
    uint32_t elig = 0;
    if (hi > lo) elig = (hi - lo >= 32 ? 0xffffffffu : ((1u << (hi - lo)) - 1u)) << lo;
    auto count_of = [&](int j) { return (int)((counters[(part * 32 + j) / kPerWord] >> (BITS * (j % kPerWord))) & kCntMask); };
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) bits |= (uint32_t)(a.tau <= 0 || count_of(j) >= a.tau) << j;
    bits &= elig;
    reinterpret_cast<uint32_t*>(a.masks)[(bh * nblk) * 2 + kfirst / 32] = bits;
    if (a.dbg_counts || a.dbg_cand) {                 // debug outputs only
      for (int j = 0; j < 32; ++j) {
        const int64_t i = kfirst + j;
        if (a.dbg_counts && i < cx.n) a.dbg_counts[bh * a.dbg_stride + i] = (uint16_t)count_of(j);
        if (a.dbg_cand && ((bits >> j) & 1u)) {
          const int pos = atomicAdd(&a.dbg_ncand[bh], 1);
          if (pos < a.dbg_cand_cap) a.dbg_cand[bh * a.dbg_cand_cap + pos] = (int32_t)i;
        }
      }
    }
  }
}

// Production form of the lookup for min_hits 1 or 2 (no count output): one workgroup per query
// head marks every key it meets in a "seen" bitmap of the whole indexed range and, when it was
// already marked, in a "seen twice" bitmap (both in LDS, a bit per key); the ballots are those
// bitmaps.  No bucket is read more than once per head, whatever the context length.
__global__ __launch_bounds__(1024) void table_lookup_bitmap_kernel(AttnArgs a, TableArgs tb) {
  extern __shared__ uint32_t bitmap[];                  // seen[nw], twice[nw]
  __shared__ uint32_t bstart[512], blen[512];
  __shared__ uint32_t qs[256];
  const Ctx cx = resolve_context(a);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int64_t bh = blockIdx.x;
  const int G = a.Hq / a.Hkv;
  const int64_t unit = (bh / a.Hq) * a.Hkv + (bh % a.Hq) / G;
  const int nb = 1 << a.K;
  const uint32_t* offs = tb.offsets + unit * a.L * (nb + 1);
  const uint32_t* idxs = tb.indices + unit * a.L * tb.n_cap;
  const int nw = (int)key_blocks(tb.n) * 2;             // 32-key words of the indexed range
  uint32_t* seen = bitmap;
  uint32_t* twice = bitmap + nw;
  for (int i = tid; i < 2 * nw; i += 1024) bitmap[i] = 0u;
  if (tid < a.NQ) qs[tid] = a.qcodes[bh * a.NQ + tid];
  __syncthreads();
  for (int t = tid; t < a.L; t += 1024) {
    const uint32_t* qw = qs + (t >> 5) * a.K;
    uint32_t code = 0;
    for (int b = 0; b < a.K; ++b) code |= ((qw[b] >> (t & 31)) & 1u) << b;
    const uint32_t s0 = offs[(int64_t)t * (nb + 1) + code], s1 = offs[(int64_t)t * (nb + 1) + code + 1];
    bstart[t] = s0;
    blen[t] = s1 - s0;
  }
  __syncthreads();
  // wavefront v reads tables v, v+16, ...: up to 128 entries of each bucket are requested before
  // any is used; longer buckets are finished in a loop
  constexpr int kMaxB = 32;                             // L <= 512 tables over 16 wavefronts
  uint32_t e0[kMaxB], e1[kMaxB];
  const int nbk = (a.L - wave + 15) >> 4;
#pragma unroll
  for (int k = 0; k < kMaxB; ++k) {
    e0[k] = 0xffffffffu; e1[k] = 0xffffffffu;
    if (k < nbk) {
      const int t = wave + 16 * k;
      const uint32_t len = blen[t];
      const uint32_t* p = idxs + (int64_t)t * tb.n_cap + bstart[t];
      if ((uint32_t)lane < len) e0[k] = p[lane];
      if ((uint32_t)lane + 64 < len) e1[k] = p[lane + 64];
    }
  }
  auto mark = [&](uint32_t key) {
    if (key != 0xffffffffu) {
      const uint32_t bit = 1u << (key & 31);
      if (atomicOr(&seen[key >> 5], bit) & bit) atomicOr(&twice[key >> 5], bit);
    }
  };
#pragma unroll
  for (int k = 0; k < kMaxB; ++k) {
    if (k < nbk) {
      mark(e0[k]);
      mark(e1[k]);
      const int t = wave + 16 * k;
      if (blen[t] > 128) {
        const uint32_t* p = idxs + (int64_t)t * tb.n_cap + bstart[t];
        for (uint32_t j = 128 + lane; j < blen[t]; j += 64) mark(p[j]);
      }
    }
  }
  __syncthreads();
  // ballots of the indexed range, 32 keys per word, static keys and keys beyond n masked out
  const int64_t nblk = key_blocks(cx.n);
  const uint32_t* hit = a.tau >= 2 ? twice : seen;
  uint32_t* mout = reinterpret_cast<uint32_t*>(a.masks) + bh * nblk * 2;
  const int64_t hi_key = cx.n - a.n_local < cx.n ? cx.n - a.n_local : cx.n;
  for (int i = tid; i < nw; i += 1024) {
    const int64_t kfirst = (int64_t)i * 32;
    const int64_t lo = (a.n_sink > kfirst ? a.n_sink : kfirst) - kfirst;
    const int64_t hi = (hi_key < kfirst + 32 ? hi_key : kfirst + 32) - kfirst;
    uint32_t elig = 0;
    if (hi > lo) elig = (hi - lo >= 32 ? 0xffffffffu : ((1u << (hi - lo)) - 1u)) << lo;
    const uint32_t bits = hit[i] & elig;
    mout[i] = bits;
    if (a.dbg_cand) {                                    // debug output only
      for (uint32_t f = bits; f; f &= f - 1) {
        const int pos = atomicAdd(&a.dbg_ncand[bh], 1);
        if (pos < a.dbg_cand_cap) a.dbg_cand[bh * a.dbg_cand_cap + pos] = (int32_t)(kfirst + __ffs(f) - 1);
      }
    }
  }
}

hipError_t launch_build_tables(const TableArgs& t, hipStream_t s) {
  if (t.units <= 0 || t.L <= 0) return hipSuccess;
  const int tpp = ht_tables_per_pass(t.K);
  const int passes = 32 / tpp;
  const size_t lds = (size_t)tpp * (4u << t.K);
  const dim3 grid((unsigned)(table_words(t.L) * passes), (unsigned)t.units);
  hipLaunchKernelGGL(ht_build_kernel<false>, grid, dim3(256), lds, s, t);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (t.codes16 && t.n > 0) {
    const size_t place_lds = ((size_t)6 << t.K) + (size_t)kBuildWindow * sizeof(uint16_t);   // <= 56 KB at K = 12
    hipLaunchKernelGGL(ht_place_kernel, dim3((unsigned)t.windows, (unsigned)t.L, (unsigned)t.units), dim3(256),
                       place_lds, s, t);
  } else {
    hipLaunchKernelGGL(ht_build_kernel<true>, grid, dim3(256), lds, s, t);
  }
  return hipGetLastError();
}

// Lookup and gather in one launch for min_hits 1 or 2: a workgroup of 16 wavefronts per (query
// head, slice of kLgSliceBlocks key blocks of the indexed range).  It reads the L buckets of the
// head: of window-ordered tables (the build with a workspace) only the pieces that hold the
// keys of its slice, which is a build window, so that a head's buckets are read once in all;
// otherwise whole buckets, of which it keeps the keys of its slice.  The keys are marked in
// "seen" / "seen twice" bitmaps in LDS, and wavefront v then expands the bits of its
// kLgWaveBlocks blocks into an index list and gathers and weighs those keys
// (gather_estimate_wave) without the ballots ever leaving the compute unit: one partial per
// (head, slice, wavefront).  The keys of the static set T are dealt over these wavefronts (key
// j to wavefront j mod their number) and join the batches.  The keys appended since the build,
// 16 code blocks per slice, are found by the collision scan in the workgroups of slice 0, 1,
// ... and join the gather batches there.
// KT, WDT, LT: the collision scan's compile-time K, ceil(L/32) and tables of the last group (0: any).
template <int KT, int WDT, int LT, int ET>
__global__ __launch_bounds__(1024) void lookup_gather_kernel(AttnArgs a, TableArgs tb) {
  constexpr bool FP32 = ET == kFP32;
  constexpr int kSliceWords = kLgSliceBlocks * 2;       // 32-key words of a slice
  constexpr int kWaveWords = kLgWaveBlocks * 2;
  __shared__ uint32_t seen[kSliceWords], twice[kSliceWords];
  __shared__ uint32_t qs[256];
  __shared__ uint16_t lists[16][kLgWaveBlocks * kBlockKeys + kBlockKeys];
  const Ctx cx = resolve_context(a);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int slice = blockIdx.x;
  const int64_t bh = blockIdx.y;
  const int G = a.Hq / a.Hkv;
  const int unit = (int)((bh / a.Hq) * a.Hkv + (bh % a.Hq) / G);
  const int nb = 1 << a.K;
  const uint32_t* offs = tb.offsets + (int64_t)unit * a.L * (nb + 1);
  const uint32_t* idxs = tb.indices + (int64_t)unit * a.L * tb.n_cap;
  const uint32_t key_lo = (uint32_t)slice * (kLgSliceBlocks * kBlockKeys);
  const uint32_t qword = tid < a.NQ ? a.qcodes[bh * a.NQ + tid] : 0u;      // (requested, not yet used)
  for (int i = tid; i < kSliceWords; i += 1024) { seen[i] = 0u; twice[i] = 0u; }
  // ---- keys appended since the build: run `slice` of 16 of their code blocks, one per
  // wavefront, compared with this head's code while the query code is on its way; the
  // wavefront gathers what its block samples with its own batch ----
  uint64_t app_mask = 0;
  const int64_t app_blk = a.blk_begin + (int64_t)slice * 16 + wave;
  if (slice < a.lg_app_runs && app_blk < key_blocks(cx.n)) {
    const int hg = (int)(bh % a.Hq) % G;
    scan_blocks<KT, WDT, LT, 1, true>(a, cx, unit, app_blk, lane, hg, hg + 1, [&](int, int64_t, uint64_t m) { app_mask = m; });
  }
  if (tid < a.NQ) qs[tid] = qword;
  __syncthreads();
  // wavefront v reads tables v, v+16, ...: lane k finds the bucket of table v + 16 k (its code
  // from the query's plane words, then two offsets); the descriptors reach the other lanes as
  // scalars.  Up to 128 entries of each bucket are requested before any is used; longer
  // buckets are finished in a loop.
  constexpr int kMaxB = 32;                             // L <= 512 tables over 16 wavefronts
  const int nbk = (a.L - wave + 15) >> 4;
  // 0: buckets in no particular order (also taken when the tables were built over another number
  // of keys than this call says: whole buckets are then read, never a piece that is not there)
  const int windows = (int)tb.header[0] == a.lg_nslices ? a.lg_nslices : 0;
  uint32_t my_start = 0, my_len = 0;
  if (lane < nbk) {
    const int t = wave + 16 * lane;
    const uint32_t* qw = qs + (t >> 5) * a.K;
    uint32_t code = 0;
    for (int b = 0; b < a.K; ++b) code |= ((qw[b] >> (t & 31)) & 1u) << b;
    const uint32_t* o = offs + (int64_t)t * (nb + 1) + code;
    my_start = o[0];
    uint32_t my_end = o[1];
    if (windows > 0) {
      // window-ordered buckets: only the piece that holds the keys of this slice
      const uint32_t* wc = tb.wincum + (((int64_t)unit * a.L + t) * windows + slice) * nb + code;
      if (slice + 1 < windows) my_end = my_start + wc[nb];
      my_start += wc[0];
    }
    my_len = my_end - my_start;
  }
  constexpr uint32_t kSliceKeys = kLgSliceBlocks * kBlockKeys;
  auto mark = [&](uint32_t key) {
    const uint32_t rel = key - key_lo;                  // absent entries and other slices: out of range
    if (rel < kSliceKeys) {
      const uint32_t bit = 1u << (rel & 31);
      if (atomicOr(&seen[rel >> 5], bit) & bit) atomicOr(&twice[rel >> 5], bit);
    }
  };
  if (windows > 0) {
    // Window-ordered tables: a piece holds about 16 keys (n 2^-K per window of 16384 keys), so
    // half a wavefront reads a piece: lanes 0..31 that of table v + 32 j, lanes 32..63 that of
    // table v + 32 j + 16.  The first atomics of all pieces are issued together and their
    // answers (was the key seen before?) used afterwards, so the LDS round trips overlap.
    // Pieces of more than 32 keys are finished in a loop.
    const int half = lane >> 5, li = lane & 31;
    uint32_t e[kMaxB / 2];
#pragma unroll
    for (int j = 0; j < kMaxB / 2; ++j) {
      e[j] = 0xffffffffu;
      if (2 * j < nbk) {
        const int k = 2 * j + half;
        const uint32_t start = __shfl(my_start, k), len = __shfl(my_len, k);   // (0 for k >= nbk)
        const uint32_t* p = idxs + (int64_t)(wave + 16 * k) * tb.n_cap + start;
        if ((uint32_t)li < len) e[j] = p[li];
      }
    }
    uint32_t before[kMaxB / 2];
#pragma unroll
    for (int j = 0; j < kMaxB / 2; ++j) {
      const uint32_t rel = e[j] - key_lo;
      before[j] = 0u;
      if (2 * j < nbk && rel < kSliceKeys) before[j] = atomicOr(&seen[rel >> 5], 1u << (rel & 31));
    }
#pragma unroll
    for (int j = 0; j < kMaxB / 2; ++j) {
      const uint32_t rel = e[j] - key_lo;
      if (2 * j < nbk && rel < kSliceKeys && ((before[j] >> (rel & 31)) & 1u)) atomicOr(&twice[rel >> 5], 1u << (rel & 31));
    }
    // (rare: the wavefront knows at once whether any of its pieces is that long)
    for (uint64_t f = __ballot(my_len > 32); f; f &= f - 1) {
      const int k = __ffsll((unsigned long long)f) - 1;
      const uint32_t len = __builtin_amdgcn_readlane(my_len, k);
      const uint32_t* p = idxs + (int64_t)(wave + 16 * k) * tb.n_cap + __builtin_amdgcn_readlane(my_start, k);
      for (uint32_t j = 32 + lane; j < len; j += 64) mark(p[j]);
    }
  } else {
    // Buckets in no particular order: up to 128 entries of each bucket are requested before any
    // is used; longer buckets are finished in a loop.
    uint32_t e0[kMaxB], e1[kMaxB];
#pragma unroll
    for (int k = 0; k < kMaxB; ++k) {
      e0[k] = 0xffffffffu; e1[k] = 0xffffffffu;
      if (k < nbk) {
        const uint32_t start = __builtin_amdgcn_readlane(my_start, k), len = __builtin_amdgcn_readlane(my_len, k);
        const uint32_t* p = idxs + (int64_t)(wave + 16 * k) * tb.n_cap + start;
        if ((uint32_t)lane < len) e0[k] = p[lane];
        if ((uint32_t)lane + 64 < len) e1[k] = p[lane + 64];
      }
    }
    // Marking: absent entries and keys of other slices fall out of range.  The first atomics of
    // eight buckets are issued together and their answers (was the key seen before?) used
    // afterwards, so the LDS round trips overlap instead of following each other.
#pragma unroll
    for (int c0 = 0; c0 < kMaxB; c0 += 8) {
      if (c0 < nbk) {
        uint32_t before[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const uint32_t rel = ((i & 1) ? e1[c0 + (i >> 1)] : e0[c0 + (i >> 1)]) - key_lo;
          before[i] = 0u;
          if (rel < kSliceKeys) before[i] = atomicOr(&seen[rel >> 5], 1u << (rel & 31));
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const uint32_t rel = ((i & 1) ? e1[c0 + (i >> 1)] : e0[c0 + (i >> 1)]) - key_lo;
          if (rel < kSliceKeys && ((before[i] >> (rel & 31)) & 1u)) atomicOr(&twice[rel >> 5], 1u << (rel & 31));
        }
      }
    }
    for (uint64_t f = __ballot(my_len > 128); f; f &= f - 1) {
      const int k = __ffsll((unsigned long long)f) - 1;
      const uint32_t len = __builtin_amdgcn_readlane(my_len, k);
      const uint32_t* p = idxs + (int64_t)(wave + 16 * k) * tb.n_cap + __builtin_amdgcn_readlane(my_start, k);
      for (uint32_t j = 128 + lane; j < len; j += 64) mark(p[j]);
    }
  }
  __syncthreads();
  // ---- gather: wavefront v takes blocks v*kLgWaveBlocks .. of the slice ----
  const uint32_t* hit = a.tau >= 2 ? twice : seen;
  const int64_t hi_key = cx.n - a.n_local < tb.n ? cx.n - a.n_local : tb.n;   // indexed, not in the local window
  const int64_t wave_key0 = (int64_t)key_lo + (int64_t)wave * (kLgWaveBlocks * kBlockKeys);
  uint16_t* list = lists[wave];
  HeadVectors<FP32> hv;
  request_head_vectors<FP32>(a, unit, bh, hv);
  uint32_t bits = 0;
  if (lane < kWaveWords) {
    const int64_t kfirst = wave_key0 + (int64_t)lane * 32;
    const int64_t lo = (a.n_sink > kfirst ? a.n_sink : kfirst) - kfirst;
    const int64_t hi = (hi_key < kfirst + 32 ? hi_key : kfirst + 32) - kfirst;
    uint32_t elig = 0;
    if (hi > lo) elig = (hi - lo >= 32 ? 0xffffffffu : ((1u << (hi - lo)) - 1u)) << lo;
    bits = hit[wave * kWaveWords + lane] & elig;
  }
  if (a.dbg_cand) {                                      // debug output only
    for (uint32_t f = bits; f; f &= f - 1) {
      const int pos = atomicAdd(&a.dbg_ncand[bh], 1);
      if (pos < a.dbg_cand_cap)
        a.dbg_cand[bh * a.dbg_cand_cap + pos] = (int32_t)(wave_key0 + lane * 32 + __ffs(f) - 1);
    }
  }
  const int c = __popc(bits);
  const int incl = half_prefix_sum32(c);                 // kWaveWords <= 32
  const int in_slice = __builtin_amdgcn_readlane(incl, 31);
  int pos = incl - c;
  for (uint32_t f = bits; f; f &= f - 1) list[pos++] = (uint16_t)(lane * 32 + __ffs(f) - 1);
  // behind them the sampled keys of the wavefront's appended block (lane = key of the block)
  if ((app_mask >> lane) & 1)
    list[in_slice + __popcll(app_mask & ((1ull << lane) - 1ull))] = (uint16_t)lane;
  const int n_sampled = in_slice + __popcll(app_mask);
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  __builtin_amdgcn_wave_barrier();
  // static keys slot, slot + slots, ... ride along behind the sampled ones
  const int slots = a.lg_nslices * 16, slot = slice * 16 + wave;
  const int nst = static_share(cx, slot, slots);
  gather_estimate_wave<ET, (FP32 ? 4 : 8)>(a, unit, bh, n_sampled + nst, n_sampled, hv,
                                            [&](int cc) {
                                              if (cc >= n_sampled) return static_key(a, cx, slot + (int64_t)(cc - n_sampled) * slots);
                                              return (cc < in_slice ? wave_key0 : app_blk * kBlockKeys) + (int64_t)list[cc];
                                            },
                                            a.partial + (bh * a.nranges + slot) * kPartialStride);
}

template <int KT, int WDT, int LT>
static void launch_lookup_gather_for(const AttnArgs& a, const TableArgs& t, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  auto go = [&](auto kernel) {
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, dim3(1024), 0, s, start, stop, 0, a, t);
    else hipLaunchKernelGGL(kernel, grid, dim3(1024), 0, s, a, t);
  };
  if (a.is_fp32) go(lookup_gather_kernel<KT, WDT, LT, kFP32>);
  else if (a.kv_fp8) go(lookup_gather_kernel<KT, WDT, LT, kFP8>);
  else go(lookup_gather_kernel<KT, WDT, LT, kBF16>);
}

hipError_t launch_lookup_gather(const AttnArgs& a0, const TableArgs& t, int nslices, int appended_runs, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  AttnArgs a = a0;
  a.lg_nslices = nslices;
  a.lg_app_runs = appended_runs;                       // <= nslices
  const dim3 grid((unsigned)nslices, (unsigned)((int64_t)a.B * a.Hq));
  // the scan of the appended keys has the same tuned forms as collision_scan_kernel
  if (a.K == 10 && a.L == 150) launch_lookup_gather_for<10, 5, 22>(a, t, grid, s, start, stop);
  else if (a.K == 9 && a.L == 120) launch_lookup_gather_for<9, 4, 24>(a, t, grid, s, start, stop);
  else if (a.K == 10 && a.L == 170) launch_lookup_gather_for<10, 6, 10>(a, t, grid, s, start, stop);
  else if (a.K == 8 && a.L == 75) launch_lookup_gather_for<8, 3, 11>(a, t, grid, s, start, stop);
  else if (a.K == 10 && a.L == 220) launch_lookup_gather_for<10, 7, 28>(a, t, grid, s, start, stop);
  else if (a.K == 11 && a.L == 300) launch_lookup_gather_for<11, 10, 12>(a, t, grid, s, start, stop);
  else launch_lookup_gather_for<0, 0, 0>(a, t, grid, s, start, stop);
  return hipGetLastError();
}

hipError_t launch_table_lookup(const AttnArgs& a, const TableArgs& t, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  const int64_t nblk = key_blocks(t.n);
  // two bits per key in LDS: up to 196608 indexed keys in 48 KB (5 KB more are static)
  const size_t bitmap_bytes = (size_t)nblk * 2 * 2 * sizeof(uint32_t);
  if (!a.dbg_counts && (a.tau == 1 || a.tau == 2) && bitmap_bytes <= 48 * 1024) {
    const dim3 grid((unsigned)((int64_t)a.B * a.Hq));
    if (start || stop) hipExtLaunchKernelGGL(table_lookup_bitmap_kernel, grid, dim3(1024), bitmap_bytes, s, start, stop, 0, a, t);
    else hipLaunchKernelGGL(table_lookup_bitmap_kernel, grid, dim3(1024), bitmap_bytes, s, a, t);
    return hipGetLastError();
  }
  auto go = [&](auto kernel, int run_blocks) {
    const dim3 grid((unsigned)((nblk + run_blocks - 1) / run_blocks), (unsigned)((int64_t)a.B * a.Hq));
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, dim3(1024), 0, s, start, stop, 0, a, t);
    else hipLaunchKernelGGL(kernel, grid, dim3(1024), 0, s, a, t);
  };
  if (a.L <= 255) go(table_lookup_kernel<8>, kLookupRunBlocks<8>);
  else go(table_lookup_kernel<16>, kLookupRunBlocks<16>);
  return hipGetLastError();
}

}  // namespace mp
