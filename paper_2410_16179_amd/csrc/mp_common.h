// Shared declarations of the gfx950 library for LSH-sampled decode attention.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "magicpig.h"

namespace mp {

constexpr int kHeadDim = 128;
constexpr int kBlockKeys = 64;   // keys per code block = lanes per wavefront
constexpr int kNumCU = 256;      // MI355X

// ---- packed code layout (documented in magicpig.h) ----
// Plane word w*K + b holds sign bit b of tables 32w .. 32w+31.  Query codes are stored as
// plane words.  Key codes store the plane words of the first Wd-1 table groups as they are
// and the last group densely: its K planes, tail_tables(L) bits each, as one bit string.
__host__ __device__ inline int table_words(int L) { return (L + 31) >> 5; }
__host__ __device__ inline int plane_words(int K, int L) { return K * table_words(L); }
__host__ __device__ inline int tail_tables(int L) { return L - 32 * (table_words(L) - 1); }      // 1..32
__host__ __device__ inline int tail_begin(int K, int L) { return K * (table_words(L) - 1); }
__host__ __device__ inline int code_words(int K, int L) {
  return tail_begin(K, L) + (K * tail_tables(L) + 31) / 32;
}
__host__ __device__ inline int64_t key_blocks(int64_t n) { return (n + kBlockKeys - 1) / kBlockKeys; }
__host__ __device__ inline int slot_in_block(int NW, int x, int r) {
  const int full = NW >> 2, rem = NW & 3;
  const int gq = x >> 2;
  return gq < full ? gq * 256 + r * 4 + (x & 3) : full * 256 + r * rem + (x & 3);
}
// Key word and bit inside it that hold bit `beta` of plane word x.
__host__ __device__ inline void key_bit_position(int K, int L, int x, int beta, int* word, int* bit) {
  const int xs = tail_begin(K, L);
  if (x < xs) { *word = x; *bit = beta; return; }
  const int pos = (x - xs) * tail_tables(L) + beta;
  *word = xs + (pos >> 5);
  *bit = pos & 31;
}
// Plane word x of key r of a code block, read from memory (bits of tables >= L may be set in
// the last group: they belong to the next plane; callers mask or ignore them).
__device__ inline uint32_t load_plane_word(const uint32_t* blkp, int NW, int K, int L, int x, int r) {
  const int xs = tail_begin(K, L);
  if (x < xs) return blkp[slot_in_block(NW, x, r)];
  const int pos = (x - xs) * tail_tables(L);
  const int wi = xs + (pos >> 5), sh = pos & 31;
  const uint32_t lo = blkp[slot_in_block(NW, wi, r)];
  if (sh + tail_tables(L) <= 32) return lo >> sh;
  const uint32_t hi = blkp[slot_in_block(NW, wi + 1, r)];
  return (lo >> sh) | (hi << (32 - sh));
}
// Appends bit fields to a string of 32-bit words (every lane of a wavefront carries its own
// string; lengths and counts are wave-uniform).
struct BitString {
  uint64_t acc = 0;
  int nbits = 0;
  // returns true when a word was completed: it is in *out and must be stored by the caller
  __host__ __device__ inline bool append(uint32_t field, int len, uint32_t* out) {
    const uint32_t f = len >= 32 ? field : field & ((1u << len) - 1u);
    acc |= (uint64_t)f << nbits;
    nbits += len;
    if (nbits < 32) return false;
    *out = (uint32_t)acc;
    acc >>= 32;
    nbits -= 32;
    return true;
  }
};

// Launch description of the direct (float64 + exact fallback) SimHash kernel.
struct HashDirectArgs {
  const void* X;        // vectors to hash
  const void* W;        // [128, K*L] row-major
  const float* mu;      // per (b,g) [128] or nullptr
  uint32_t* codes;
  int is_fp32;          // element type of X and W
  int x_fp8;            // the vectors X are rows of an e4m3 K cache (W is bf16)
  int K, L, NW, NQ;     // NW: words per key code, NQ: plane words (= words per query code)
  int query_layout;     // 1: codes[row][NQ] plane words, pad bits 1;  0: blocked key layout, pad bits 0
  // key addressing: row r in [0, units*n_keys): unit = r / n_keys, i = first_key + r % n_keys
  int64_t n_keys, first_key;
  int n_kv_heads;       // unit = b*n_kv_heads + g
  int64_t stride_b, stride_h, stride_n;   // element strides (query layout: stride_n = 128, others 0)
  int64_t blocks_cap;   // code blocks per unit
  int64_t total_rows;
  const int* run_flag;  // if not null the kernel does nothing unless *run_flag != 0
  // hash_rows_kernel only: if not null, the context length in device memory; the vectors are then
  // the newest n_keys keys [*n_dev - n_keys, *n_dev) of every unit instead of first_key ..
  // (nothing is coded when that range does not lie inside [0, n_cap))
  const int64_t* n_dev;
  int64_t n_cap;
};

// Launch description of the matrix-core key hashing (bf16 keys).
struct HashMfmaArgs {
  const void* Kc; const void* W; const float* mu; uint32_t* codes;
  int K, L, NW, NQ, ntiles, units, n_kv_heads;
  int kv_fp8;                  // the K cache holds e4m3 bytes
  int64_t n_keys, first_key, n_cap, blocks_cap;
  int64_t stride_b, stride_h, stride_n;
  // workspace pieces
  void* afrag;                 // projector in MFMA A-fragment order, bf16
  void* wt;                    // projector transposed [K*L][128], bf16
  float* thr;                  // [units][ntiles][2][16] initial accumulators
  double* thr64;               // [units][K*L] mu.W_j in float64 (exact products, 128 roundings of 2^-53)
  float* magmu;                // [units][K*L] an upper bound of sum_d |mu_d W_dj|
  float* munorm;               // [units]
  float* rownorm;              // [ntiles*32] norm of the projector column behind each tile row
  unsigned* wmax_bits;         // max column norm of W (float bits), kept for the statistics
  unsigned* list_count; int* overflow; unsigned* flagged_total;
  unsigned long long* list; uint64_t list_cap;
};

// Matrix-core projections (bf16 products are exact in float32; float32 accumulation): whatever the
// order and grouping of the 128 products and the initial value inside the matrix core, with each
// alignment or rounding step losing at most 2^-23 of the running magnitude, the result is within
// kGamma * sum|terms| of the exact sum.  A fused 16-term block with truncating alignment gives
// (16 + 2) * 8 * 2^-23 = 2^-15.8; 2^-15 leaves a factor of 1.8.
constexpr float kGamma = 3.0517578125e-5f;

// The projector in the form the few-vectors matrix-core hashing reads (magicpig_prepare_projector):
// [256-byte header | fragments | transposed copy].  Header words: magic, K, L, float bits of the
// largest column norm.  Fragments: for table group w (32 tables) and plane pair p (planes 2p, 2p+1)
// two MFMA A tiles of 32 rows x 128, tile row rho of tile tau being plane 2p + (rho/4)%2 of table
// 32w + 31 - (16 tau + 4 (rho/8) + rho%4), in the lane order of v_mfma_f32_32x32x16_bf16: k-step s,
// lane (rho, half) holds elements 16 s + 8 half .. + 7.  Transposed copy: [K*L][128] bf16.
// float32 projectors: header and a plain copy.
constexpr uint32_t kPreparedMagic = 0x4d505731u;
struct PreparedLayout { size_t frag_off, wt_off, total; int P, Wd; };
__host__ __device__ inline PreparedLayout prepared_layout(int K, int L, bool fp32) {
  PreparedLayout l{};
  l.P = (K + 1) / 2;
  l.Wd = table_words(L);
  l.frag_off = 256;
  if (fp32) {
    l.wt_off = 256;
    l.total = 256 + (((size_t)K * L * kHeadDim * 4 + 255) & ~(size_t)255);
    return l;
  }
  const size_t frag = (size_t)l.Wd * l.P * 2 * 8 * 64 * 16;
  l.wt_off = l.frag_off + ((frag + 255) & ~(size_t)255);
  l.total = l.wt_off + (((size_t)K * L * kHeadDim * 2 + 255) & ~(size_t)255);
  return l;
}
// Centering prepared for the few-vectors hashing (magicpig_prepare_centering): per (batch, KV head)
// the initial accumulators -fl(mu.W_j) in the order of the fragments above
// ([unit][w][p][tau][lane half][16]), then |mu| per unit.
struct CenteringLayout { size_t thr_off, munorm_off, total; };
__host__ __device__ inline CenteringLayout centering_layout(int K, int L, size_t units) {
  CenteringLayout c{};
  const size_t thr = units * (size_t)table_words(L) * ((K + 1) / 2) * 64 * sizeof(float);
  c.thr_off = 0;
  c.munorm_off = (thr + 255) & ~(size_t)255;
  c.total = c.munorm_off + ((units * sizeof(float) + 255) & ~(size_t)255);
  return c;
}

// Launch description of the few-vectors matrix-core hashing (bf16): the queries of a decode step
// and / or the newest keys of every (batch, KV head).
struct HashFewArgs {
  const uint32_t* header; const void* frag; const void* wt;    // prepared projector
  const float* thr; const float* munorm;                        // prepared centering, or null (no centering)
  const void* q; uint32_t* qcodes; int n_q;                     // query vectors [n_q][128], codes [n_q][NQ]
  const void* Kc; const float* mu; uint32_t* kcodes;            // key vectors: key first_key + r % n_keys of unit r / n_keys
  int n_krows;                                                  // units * n_keys (0: no keys)
  int kv_fp8;                                                   // the K cache holds e4m3 bytes
  int64_t n_keys, first_key, n_cap, blocks_cap;
  const int64_t* n_dev;                                         // see HashDirectArgs::n_dev
  int n_kv_heads;
  int64_t stride_b, stride_h, stride_n;
  int K, L, Wd, P, NQ, NW;
  int q_groups;                                                 // grid rows that take queries (64 each); the rest take keys (32 each)
};

struct MeanArgs {
  const void* Kc; float* mu; double* partial;
  int is_fp32; int kv_fp8; int n_kv_heads; int units; int64_t n; int nchunk; int64_t rows_per_chunk;
  int64_t stride_b, stride_h, stride_n;
};

constexpr int kFastTau = 4;      // largest min_hits whose inclusion probability takes the branch-free form
constexpr int kTailTerms = 16;   // terms of its upper-tail series

struct AttnArgs {
  const void* q; const void* Kc; const void* Vc; const float* mu;
  const uint32_t* kcodes; const uint32_t* qcodes;
  float* partial; float* out;
  uint64_t* masks;        // [B*Hq][key blocks] ballots of sampled + static keys
  uint16_t* dbg_counts; int32_t* dbg_cand; int32_t* dbg_ncand; int64_t dbg_cand_cap;
  int64_t dbg_stride;     // keys per head in dbg_counts (the launch-time context length)
  int is_fp32;            // q, K, V are float32 (else q is bf16)
  int kv_fp8;             // K and V caches hold e4m3 bytes (q is bf16)
  int B, Hq, Hkv, K, L, Wd, NW, NQ, tau, n_sink, n_local;
  int64_t n, blocks_cap;
  // if not null: the context length in device memory, read by the kernels when they run (a decode
  // loop replayed from a captured graph); `n` is then the largest value it may hold, for which
  // grids and workspace were sized
  const int64_t* n_dev;
  int64_t blk_begin;         // first key block the collision scan covers (blocks before it: table lookup)
  int64_t ks_b, ks_h, ks_n, vs_b, vs_h, vs_n;
  int nranges;               // partials per head: nscan runs of kRangeBlocks key blocks + static runs
  int nscan;                 // runs of kRangeBlocks key blocks per head
  int64_t n_static;          // keys in the static set T
  // scan and gather in one launch: one workgroup, and one partial per head, for every run of
  // 4 * f_wave_blocks key blocks (f_wave_blocks: key blocks per wavefront, 1 .. kFusedWaveBlocks)
  int f_nranges, f_wave_blocks;
  int f_touch;               // 1: its workgroups come in several rounds (wavefronts touch the rows of the keys of their last block)
  // lookup + gather in one launch: slices of the indexed range; the first lg_app_runs of them
  // also take a run of 16 appended key blocks each
  int lg_nslices, lg_app_runs;
  // ratios of consecutive binomial terms, (L-j)/(j+1) (0 from j = L on): j = 0 .. kFastTau-1,
  // and j = tau .. tau+kTailTerms-1 (filled when tau <= kFastTau)
  float head_ratio[kFastTau], tail_ratio[kTailTerms];
  float scale;
};

// Bucketed hash tables of the cached keys.
struct TableArgs {
  const uint32_t* kcodes;      // packed key codes (build only)
  uint32_t* header;            // word 0: windows of the window-ordered build, 0 when buckets are unordered
  uint32_t* offsets;           // [units][L][2^K + 1]
  uint32_t* indices;           // [units][L][n_cap]
  int K, L, NW, units;
  int64_t n, n_cap, blocks_cap;   // n: keys [0, n) are in the tables
  // build with a large workspace: per-table codes of every key and, for every window of
  // kBuildWindow keys, the number of keys of each bucket in the windows before it
  uint16_t* codes16;           // [units][L][n_cap] (workspace), or null (one-pass scatter)
  uint32_t* wincum;            // [units][L][windows][2^K], part of the tables: with it the piece of a
                               // bucket that holds the keys of one window can be read alone
  int windows;
};
constexpr int kBuildWindow = 16384;   // keys one workgroup places into the buckets of one table

constexpr int kPartialStride = 132;   // 128 output elements, running max, running sum, pad
constexpr int kRangeBlocks = 16;      // key blocks per gather wavefront (1024 keys)
constexpr int kStaticPerRange = 32;   // static (sink / local) keys per gather wavefront
constexpr int kLgWaveBlocks = 16;     // lookup + gather in one launch: key blocks per wavefront,
constexpr int kLgSliceBlocks = 16 * kLgWaveBlocks;   // and per workgroup (16 wavefronts): one build window
static_assert(kLgSliceBlocks * kBlockKeys == kBuildWindow, "a lookup slice is a window of the table build");
// the one-launch scan + gather: four wavefronts per workgroup
constexpr int kFusedWaveBlocks = 6;           // most key blocks a wavefront scans, one after the other
constexpr int kFusedBlocks = 4 * kFusedWaveBlocks;        // most key blocks per workgroup
constexpr int kFusedFill = 768;               // workgroups of it that are resident at once (3 per compute unit)
constexpr int kFusedIters = 8;             // its gather batch: rows per quarter wavefront

// host-side launchers (defined next to their kernels)
hipError_t launch_hash_direct(const HashDirectArgs& a, hipStream_t s);
hipError_t launch_hash_rows(const HashDirectArgs& a, const HashDirectArgs* b, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_hash_keys_mfma(const HashMfmaArgs& a, hipStream_t s);
hipError_t launch_key_mean(const MeanArgs& a, hipStream_t s);
hipError_t launch_prepare_projector(const void* W, void* prepared, int K, int L, hipStream_t s);
hipError_t launch_prepare_projector_fp32(const void* W, void* prepared, int K, int L, hipStream_t s);
hipError_t launch_prepare_centering(const float* mu, const void* prepared, void* centering, int K, int L, int units, hipStream_t s);
hipError_t launch_hash_few(const HashFewArgs& a, hipStream_t s, hipEvent_t start = nullptr, hipEvent_t stop = nullptr);
hipError_t launch_sampled_attention(const AttnArgs& a, const TableArgs* tables, hipStream_t s, hipEvent_t const* stage_events);
hipError_t launch_build_tables(const TableArgs& t, hipStream_t s);
hipError_t launch_table_lookup(const AttnArgs& a, const TableArgs& t, hipStream_t s, hipEvent_t start, hipEvent_t stop);
hipError_t launch_lookup_gather(const AttnArgs& a, const TableArgs& t, int nslices, int appended_runs, hipStream_t s, hipEvent_t start, hipEvent_t stop);


}  // namespace mp
