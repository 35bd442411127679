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
//   table_lookup_kernel   : one workgroup per (query head, run of 32768 keys): reads the L
//       buckets, counts hits per key in LDS byte counters, and emits the same 64-bit ballots
//       (count >= min_hits, key not static) that collision_scan_kernel emits, so the gather
//       and merge kernels are shared by both retrieval forms.
#include "attention_common.h"
#include <hip/hip_ext.h>

namespace mp {

constexpr int kLookupRunBlocks = 512;                 // 64-key blocks per lookup workgroup
constexpr int kLookupRunKeys = kLookupRunBlocks * kBlockKeys;

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

__global__ __launch_bounds__(1024) void table_lookup_kernel(AttnArgs a, TableArgs tb) {
  __shared__ uint32_t counters[kLookupRunKeys / 4];   // one byte per key of the run
  __shared__ uint32_t bstart[512], blen[512];
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
  for (int i = tid; i < kLookupRunKeys / 4; i += 1024) counters[i] = 0u;
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
    if (rel < (uint32_t)kLookupRunKeys) atomicAdd(&counters[rel >> 2], 1u << (8 * (rel & 3)));
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

  // ballots of the blocks the tables cover: thread = 32 consecutive keys (half a block)
  const int64_t nblk = key_blocks(a.n);
  const int64_t kfirst = key0 + (int64_t)tid * 32;
  if (kfirst < key_blocks(tb.n) * kBlockKeys) {
    // positions of this thread's keys that are real and outside the static set
    const int64_t lo = (a.n_sink > kfirst ? a.n_sink : kfirst) - kfirst;
    const int64_t hi_key = a.n - a.n_local < a.n ? a.n - a.n_local : a.n;
    const int64_t hi = (hi_key < kfirst + 32 ? hi_key : kfirst + 32) - kfirst;
    uint32_t elig = 0;
    if (hi > lo) elig = (hi - lo >= 32 ? 0xffffffffu : ((1u << (hi - lo)) - 1u)) << lo;
    uint32_t bits = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t cw = counters[tid * 8 + j];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int cnt = (cw >> (8 * q)) & 0xff;
        bits |= (uint32_t)(a.tau <= 0 || cnt >= a.tau) << (j * 4 + q);
      }
    }
    bits &= elig;
    reinterpret_cast<uint32_t*>(a.masks)[(bh * nblk) * 2 + kfirst / 32] = bits;
    if (a.dbg_counts || a.dbg_cand) {                 // debug outputs only
      for (int j = 0; j < 32; ++j) {
        const int64_t i = kfirst + j;
        const int cnt = (counters[tid * 8 + (j >> 2)] >> (8 * (j & 3))) & 0xff;
        if (a.dbg_counts && i < a.n) a.dbg_counts[bh * a.n + i] = (uint16_t)cnt;
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
  const int64_t nblk = key_blocks(a.n);
  const uint32_t* hit = a.tau >= 2 ? twice : seen;
  uint32_t* mout = reinterpret_cast<uint32_t*>(a.masks) + bh * nblk * 2;
  const int64_t hi_key = a.n - a.n_local < a.n ? a.n - a.n_local : a.n;
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
  const dim3 grid((unsigned)((nblk + kLookupRunBlocks - 1) / kLookupRunBlocks), (unsigned)((int64_t)a.B * a.Hq));
  if (start || stop) hipExtLaunchKernelGGL(table_lookup_kernel, grid, dim3(1024), 0, s, start, stop, 0, a, t);
  else hipLaunchKernelGGL(table_lookup_kernel, grid, dim3(1024), 0, s, a, t);
  return hipGetLastError();
}

}  // namespace mp
