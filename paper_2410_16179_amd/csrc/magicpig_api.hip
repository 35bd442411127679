// C ABI of the library: argument validation, workspace carving and kernel launches.
// Validation touches no HIP call so that it can be exercised on a host without a GPU.
#include "mp_common.h"

#include <mutex>
#include <string>

// Scratch of magicpig_sampled_attention_noalloc: device memory that belongs to the library's
// code object, one copy per GPU, there from the moment the library is loaded until the process
// ends.  In host code this name only stands for the symbol; the device address of a GPU's copy
// comes from hipGetSymbolAddress (static_scratch() below) and that is what kernels are given.
static __device__ __align__(256) unsigned char scratch[MAGICPIG_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_last_hip_error;
constexpr int kStageEvents = 7;
thread_local hipEvent_t g_stage_events[kStageEvents];
thread_local bool g_have_stage_events = false;

int fail_hip(hipError_t e) {
  g_last_hip_error = hipGetErrorString(e);
  return MAGICPIG_LAUNCH_FAILED;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Device address of the current GPU's copy of `scratch`, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e);
  if (dev < 0 || dev >= kMaxDevices) return MAGICPIG_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e);
    if (!ptr) return MAGICPIG_LAUNCH_FAILED;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MAGICPIG_OK;
}

int check_params(const magicpig_params* p) {
  if (!p) return MAGICPIG_INVALID_ARG;
  if (p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0) return MAGICPIG_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return MAGICPIG_INVALID_ARG;
  if (p->n_ctx < 0 || p->n_cap < p->n_ctx) return MAGICPIG_INVALID_ARG;
  if (p->n_sink < 0 || p->n_local < 0 || p->min_hits < 0) return MAGICPIG_INVALID_ARG;
  if (p->n_sink > (1 << 30) || p->n_local > (1 << 30)) return MAGICPIG_INVALID_ARG;   // their sum is handled in 32 bits
  if (p->head_dim != mp::kHeadDim) return MAGICPIG_UNSUPPORTED;
  if (p->K < 1 || p->K > 16 || p->L < 1 || p->L > 512) return MAGICPIG_UNSUPPORTED;
  if (p->dtype != MAGICPIG_BF16 && p->dtype != MAGICPIG_FP32) return MAGICPIG_UNSUPPORTED;
  if (p->kv_dtype != MAGICPIG_KV_SAME && p->kv_dtype != MAGICPIG_KV_FP8_E4M3) return MAGICPIG_UNSUPPORTED;
  if (p->kv_dtype == MAGICPIG_KV_FP8_E4M3 && p->dtype != MAGICPIG_BF16) return MAGICPIG_UNSUPPORTED;
  const int G = p->n_q_heads / p->n_kv_heads;
  if (G > 8) return MAGICPIG_UNSUPPORTED;                 // a workgroup keeps the ballots of at most eight heads
  if (p->n_cap > (int64_t)1 << 31) return MAGICPIG_UNSUPPORTED;
  // one grid row per (batch, KV head); the few-vectors hashing takes two query vectors per grid row
  if ((int64_t)p->batch * p->n_kv_heads > 65535) return MAGICPIG_UNSUPPORTED;
  if ((int64_t)p->batch * p->n_q_heads > 2 * 65535) return MAGICPIG_UNSUPPORTED;
  return MAGICPIG_OK;
}

// strides must keep every 8-element row fragment 16-byte aligned and rows in bounds
int check_strides(int64_t sb, int64_t sh, int64_t sn) {
  if (sb < 0 || sh < 0 || sn < mp::kHeadDim) return MAGICPIG_INVALID_ARG;
  if ((sb | sh | sn) & 7) return MAGICPIG_UNSUPPORTED;
  return MAGICPIG_OK;
}

constexpr int64_t kMeanRowsPerChunk = 256;
constexpr int64_t kFewRows = 128;   // key vectors per call up to which magicpig_hash_keys takes the few-rows kernel

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t ws_mean(const magicpig_params* p) {
  const int64_t units = (int64_t)p->batch * p->n_kv_heads;
  const int64_t nchunk = (p->n_ctx + kMeanRowsPerChunk - 1) / kMeanRowsPerChunk;
  return align256((size_t)(units * nchunk * mp::kHeadDim) * sizeof(double));
}

// key-hashing workspace (bf16, matrix cores):
// [A fragments | W transposed | thresholds | thresholds in float64 | their magnitude sums | |mu| |
//  column norms | scalars | flagged-element list]
struct HashWs { size_t afrag_off, wt_off, thr_off, thr64_off, magmu_off, munorm_off, rownorm_off, scalar_off, list_off, total; int ntiles; uint64_t list_cap; };
HashWs ws_hash_layout(const magicpig_params* p) {
  HashWs w{};
  const int NQ = mp::plane_words(p->K, p->L);
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const size_t nquads = (NQ + 3) / 4;                    // one tile pair makes two plane words
  w.ntiles = (int)(4 * nquads);                          // whole quads, padded with empty rows
  w.afrag_off = 0;
  w.wt_off = align256(nquads * 4 * 8 * 64 * 16);
  w.thr_off = w.wt_off + align256((size_t)p->K * p->L * mp::kHeadDim * 2);
  w.thr64_off = w.thr_off + align256(units * w.ntiles * 32 * sizeof(float));
  w.magmu_off = w.thr64_off + align256(units * (size_t)p->K * p->L * sizeof(double));
  w.munorm_off = w.magmu_off + align256(units * (size_t)p->K * p->L * sizeof(float));
  w.rownorm_off = w.munorm_off + align256(units * sizeof(float));
  w.scalar_off = w.rownorm_off + align256((size_t)w.ntiles * 32 * sizeof(float));
  w.list_off = w.scalar_off + 256;
  // room for one flagged element in 512 (a few in ten thousand are expected), at least 64K
  const uint64_t elems = (uint64_t)units * (uint64_t)p->n_cap * (uint64_t)(p->K * p->L);
  w.list_cap = elems / 512 > 65536 ? elems / 512 : 65536;
  w.total = w.list_off + align256(w.list_cap * sizeof(unsigned long long));
  return w;
}
size_t ws_hash(const magicpig_params* p) { return p->dtype == MAGICPIG_BF16 ? ws_hash_layout(p).total : 0; }
// what magicpig_hash_keys needs for n_keys keys per (batch, KV head): only the matrix-core path
// (bf16, more vectors than the few-vectors kernel takes) uses scratch
size_t ws_hash_for(const magicpig_params* p, int64_t n_keys) {
  return (int64_t)p->batch * p->n_kv_heads * n_keys > kFewRows ? ws_hash(p) : 0;
}

// decode workspace: [partials | ballots]
struct AttnWs { size_t partial_off, masks_off, total; int nranges, nscan, f_nranges, f_wave_blocks, f_touch; int64_t n_static; };
AttnWs ws_attention_layout(const magicpig_params* p) {
  AttnWs w{};
  const int64_t nblk = mp::key_blocks(p->n_ctx);
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  w.nscan = (int)((nblk + mp::kRangeBlocks - 1) / mp::kRangeBlocks);
  const int64_t st = (int64_t)p->n_sink + p->n_local;
  w.n_static = st < p->n_ctx ? st : p->n_ctx;
  w.nranges = w.nscan + (int)((w.n_static + mp::kStaticPerRange - 1) / mp::kStaticPerRange);
  // the one-launch scan + gather: one partial per run and head
  // The shortest runs (4 wave_blocks key blocks per workgroup) whose workgroups are all resident
  // at once, give or take a dozen: a second, mostly empty round of workgroups would
  // start late and end last (measured at 8 KV heads: 100000 keys 48.6 -> 44.8 us per step, 65536
  // keys 36.1 -> 33.7, 32768 keys 27.4 -> 23.9 against runs of 16, 8 or 4 blocks chosen to fill
  // the chip at least once).  When even the longest runs do not fit (large batches) the rounds
  // are many anyway: the longest runs, 24 blocks (fewer partials; batch 16 x 65536 keys: 275 ->
  // 272.5 us against 16 blocks), and the wavefronts touch the rows of their last block early.
  const int64_t units = (int64_t)p->batch * p->n_kv_heads;
  auto groups = [&](int wb) { return units * ((nblk + 4 * wb - 1) / (4 * wb)); };
  const int64_t fits = mp::kFusedFill + mp::kFusedFill / 64;   // 780: a dozen late workgroups cost less than longer runs
  w.f_wave_blocks = 1;
  while (w.f_wave_blocks < mp::kFusedWaveBlocks && groups(w.f_wave_blocks) > fits) ++w.f_wave_blocks;
  w.f_touch = 0;
  if (groups(w.f_wave_blocks) > fits) { w.f_wave_blocks = mp::kFusedWaveBlocks; w.f_touch = 1; }
  w.f_nranges = (int)((nblk + 4 * w.f_wave_blocks - 1) / (4 * w.f_wave_blocks));
  // lookup + gather in one launch: 16 partials per slice
  const int lg = (int)((nblk + mp::kLgSliceBlocks - 1) / mp::kLgSliceBlocks) * 16;
  size_t most = (size_t)(w.f_nranges > w.nranges ? w.f_nranges : w.nranges);
  if ((size_t)lg > most) most = (size_t)lg;
  w.partial_off = 0;
  w.masks_off = align256(heads * most * mp::kPartialStride * sizeof(float));
  w.total = w.masks_off + align256(heads * (size_t)nblk * sizeof(uint64_t));
  return w;
}
size_t ws_attention(const magicpig_params* p) { return ws_attention_layout(p).total; }

bool tables_supported(const magicpig_params* p) {
  // bucket offsets are 2^K + 1 words per table (the build keeps whole histograms in LDS); one grid row per head
  return p->K <= 12 && (int64_t)p->batch * p->n_q_heads <= 65535;
}

// workspace of the two-pass table build: the code of every key in every table
struct BuildWs { size_t codes_off, total; int windows; };
BuildWs ws_build_layout(const magicpig_params* p) {
  BuildWs w{};
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const int64_t n = p->n_ctx > 0 ? p->n_ctx : 1;
  w.windows = (int)((n + mp::kBuildWindow - 1) / mp::kBuildWindow);
  w.codes_off = 0;
  w.total = align256(units * p->L * (size_t)mp::key_blocks(p->n_cap) * mp::kBlockKeys * sizeof(uint16_t));
  return w;
}

// tables: [header | bucket offsets | key indices | bucket fill levels at the start of every window]
struct TableLayout { size_t header_off, offsets_off, indices_off, wincum_off, total; };
TableLayout table_layout(const magicpig_params* p) {
  TableLayout t{};
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const size_t nb = (size_t)1 << p->K;
  const size_t windows_cap = (size_t)((p->n_cap + mp::kBuildWindow - 1) / mp::kBuildWindow);
  t.header_off = 0;
  t.offsets_off = 256;
  t.indices_off = t.offsets_off + align256(units * p->L * (nb + 1) * 4);
  t.wincum_off = t.indices_off + align256(units * p->L * (size_t)p->n_cap * 4);
  t.total = t.wincum_off + align256(units * p->L * (windows_cap > 0 ? windows_cap : 1) * nb * 4);
  return t;
}

void fill_table_args(const magicpig_params* p, const void* tables, mp::TableArgs* t) {
  const size_t units = (size_t)p->batch * p->n_kv_heads;
  const TableLayout tl = table_layout(p);
  char* base = reinterpret_cast<char*>(const_cast<void*>(tables));
  t->kcodes = nullptr;
  t->header = reinterpret_cast<uint32_t*>(base + tl.header_off);
  t->offsets = reinterpret_cast<uint32_t*>(base + tl.offsets_off);
  t->indices = reinterpret_cast<uint32_t*>(base + tl.indices_off);
  t->wincum = reinterpret_cast<uint32_t*>(base + tl.wincum_off);
  t->K = p->K; t->L = p->L; t->NW = mp::code_words(p->K, p->L); t->units = (int)units;
  t->n = p->n_ctx; t->n_cap = p->n_cap; t->blocks_cap = mp::key_blocks(p->n_cap);
  t->codes16 = nullptr; t->windows = 1;
}

int check_hash_keys_args(const magicpig_params* p, const void* K_cache, const float* mu, const void* W,
                         int64_t first_key, int64_t n_keys, const uint32_t* key_codes, const void* workspace,
                         size_t workspace_bytes) {
  int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if ((st = check_strides(p->k_stride_b, p->k_stride_h, p->k_stride_n)) != MAGICPIG_OK) return st;
  if (first_key < 0 || n_keys < 0 || first_key + n_keys > p->n_cap) return MAGICPIG_INVALID_ARG;
  if (!W || !key_codes || (!K_cache && n_keys > 0 && p->batch > 0)) return MAGICPIG_INVALID_ARG;
  if (!aligned16(K_cache) || !aligned16(W) || !aligned16(key_codes) || !aligned16(workspace) ||
      (mu && !aligned16(mu)))
    return MAGICPIG_INVALID_ARG;
  const size_t need = ws_hash_for(p, n_keys);
  if (need > 0 && (!workspace || workspace_bytes < need)) return MAGICPIG_WORKSPACE_TOO_SMALL;
  return MAGICPIG_OK;
}

int check_hash_query_args(const magicpig_params* p, const void* q, const void* W, const uint32_t* q_codes,
                          const void* workspace, size_t workspace_bytes) {
  const int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  // (query hashing uses no scratch: any workspace, NULL included, will do)
  (void)workspace; (void)workspace_bytes;
  if (!W || !q_codes || (!q && p->batch > 0)) return MAGICPIG_INVALID_ARG;
  if (!aligned16(q) || !aligned16(W) || !aligned16(q_codes)) return MAGICPIG_INVALID_ARG;
  return MAGICPIG_OK;
}

// keys [first_key, first_key + n_keys) of every (batch, KV head) as a set of vectors to code
mp::HashDirectArgs key_rows(const magicpig_params* p, const void* K_cache, const float* mu, const void* W,
                            int64_t first_key, int64_t n_keys, uint32_t* key_codes) {
  mp::HashDirectArgs a{};
  a.X = K_cache; a.W = W; a.mu = mu; a.codes = key_codes;
  a.is_fp32 = p->dtype == MAGICPIG_FP32;
  a.x_fp8 = p->kv_dtype == MAGICPIG_KV_FP8_E4M3;
  a.K = p->K; a.L = p->L; a.NW = mp::code_words(p->K, p->L); a.NQ = mp::plane_words(p->K, p->L);
  a.query_layout = 0;
  a.n_keys = n_keys > 0 ? n_keys : 1; a.first_key = first_key;
  a.n_kv_heads = p->n_kv_heads;
  a.stride_b = p->k_stride_b; a.stride_h = p->k_stride_h; a.stride_n = p->k_stride_n;
  a.blocks_cap = mp::key_blocks(p->n_cap);
  a.total_rows = (int64_t)p->batch * p->n_kv_heads * n_keys;
  a.run_flag = nullptr;
  a.n_dev = nullptr; a.n_cap = p->n_cap;
  return a;
}

// the query vectors of a decode step: one unit holding every query row
mp::HashDirectArgs query_rows(const magicpig_params* p, const void* q, const void* W, uint32_t* q_codes) {
  mp::HashDirectArgs a{};
  a.X = q; a.W = W; a.mu = nullptr; a.codes = q_codes;
  a.is_fp32 = p->dtype == MAGICPIG_FP32;
  a.K = p->K; a.L = p->L; a.NW = mp::code_words(p->K, p->L); a.NQ = mp::plane_words(p->K, p->L);
  a.query_layout = 1;
  a.total_rows = (int64_t)p->batch * p->n_q_heads;
  a.n_keys = a.total_rows > 0 ? a.total_rows : 1; a.first_key = 0;
  a.n_kv_heads = 1;
  a.stride_b = 0; a.stride_h = 0; a.stride_n = mp::kHeadDim;
  a.blocks_cap = 0;
  a.run_flag = nullptr;
  a.n_dev = nullptr; a.n_cap = 0;
  return a;
}

// Validation and launch of a decode step.  `scratch` receives the partials (and, for the separate
// lookup / scan / gather launches, the ballots): scratch_bytes must cover ws_attention(p), or
// only its partial region when ballots_needed is false (the one-launch scan + gather).
int run_attention_impl(const magicpig_params* p, const void* q, const void* K_cache,
                       const void* V_cache, const float* mu, const uint32_t* key_codes,
                       const void* tables, int64_t n_indexed, const uint32_t* q_codes, float* out, uint16_t* dbg_counts,
                       int32_t* dbg_cand, int32_t* dbg_ncand, int64_t dbg_cand_cap,
                       void* workspace, size_t workspace_bytes, bool ballots_needed, bool use_static_scratch,
                       void* hip_stream) {
  int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if ((st = check_strides(p->k_stride_b, p->k_stride_h, p->k_stride_n)) != MAGICPIG_OK) return st;
  if ((st = check_strides(p->v_stride_b, p->v_stride_h, p->v_stride_n)) != MAGICPIG_OK) return st;
  // the gather forms row addresses from 32-bit row strides
  if (p->k_stride_n > INT32_MAX || p->v_stride_n > INT32_MAX) return MAGICPIG_UNSUPPORTED;
  const bool has_keys = p->n_ctx > 0 && p->batch > 0;
  if (!out || (!workspace && !use_static_scratch) || (!q && p->batch > 0)) return MAGICPIG_INVALID_ARG;
  if (has_keys && (!K_cache || !V_cache || (!key_codes && !tables) || !q_codes)) return MAGICPIG_INVALID_ARG;
  if (tables) {
    if (!tables_supported(p)) return MAGICPIG_UNSUPPORTED;
    // the tables cover whole code blocks, or everything
    if (n_indexed < 0 || n_indexed > p->n_ctx || (n_indexed != p->n_ctx && n_indexed % mp::kBlockKeys != 0))
      return MAGICPIG_INVALID_ARG;
    if (has_keys && !key_codes && mp::key_blocks(n_indexed) < mp::key_blocks(p->n_ctx)) return MAGICPIG_INVALID_ARG;
  }
  if ((dbg_cand != nullptr) != (dbg_ncand != nullptr) || dbg_cand_cap < 0) return MAGICPIG_INVALID_ARG;
  if (!aligned16(q) || !aligned16(K_cache) || !aligned16(V_cache) || !aligned16(key_codes) || !aligned16(tables) ||
      !aligned16(q_codes) || !aligned16(out) || !aligned16(workspace) || (mu && !aligned16(mu)))
    return MAGICPIG_INVALID_ARG;
  const AttnWs wl = ws_attention_layout(p);
  if (use_static_scratch) {
    // everything above ran without a GPU call; the library's own scratch replaces the workspace
    if (wl.masks_off > (size_t)MAGICPIG_STATIC_SCRATCH_BYTES) return MAGICPIG_SCRATCH_TOO_SMALL;
    if (p->batch == 0) return MAGICPIG_OK;
    if ((st = static_scratch(&workspace)) != MAGICPIG_OK) return st;
  } else if (workspace_bytes < (ballots_needed ? wl.total : wl.masks_off)) {
    return MAGICPIG_WORKSPACE_TOO_SMALL;
  }
  mp::AttnArgs a{};
  a.q = q; a.Kc = K_cache; a.Vc = V_cache; a.mu = mu; a.kcodes = key_codes; a.qcodes = q_codes;
  char* wsb = reinterpret_cast<char*>(workspace);
  a.partial = reinterpret_cast<float*>(wsb + wl.partial_off); a.out = out;
  a.masks = reinterpret_cast<uint64_t*>(wsb + wl.masks_off);
  a.nranges = wl.nranges; a.nscan = wl.nscan; a.n_static = wl.n_static;
  a.f_nranges = wl.f_nranges; a.f_wave_blocks = wl.f_wave_blocks; a.f_touch = wl.f_touch;
  a.dbg_counts = dbg_counts; a.dbg_cand = dbg_cand; a.dbg_ncand = dbg_ncand; a.dbg_cand_cap = dbg_cand_cap;
  a.dbg_stride = p->n_ctx; a.n_dev = p->n_ctx_dev;
  a.is_fp32 = p->dtype == MAGICPIG_FP32;
  a.kv_fp8 = p->kv_dtype == MAGICPIG_KV_FP8_E4M3;
  a.B = p->batch; a.Hq = p->n_q_heads; a.Hkv = p->n_kv_heads; a.K = p->K; a.L = p->L;
  a.Wd = mp::table_words(p->L); a.NW = mp::code_words(p->K, p->L); a.NQ = mp::plane_words(p->K, p->L);
  a.tau = p->min_hits; a.n_sink = p->n_sink; a.n_local = p->n_local;
  a.n = p->n_ctx; a.blocks_cap = mp::key_blocks(p->n_cap);
  a.ks_b = p->k_stride_b; a.ks_h = p->k_stride_h; a.ks_n = p->k_stride_n;
  a.vs_b = p->v_stride_b; a.vs_h = p->v_stride_h; a.vs_n = p->v_stride_n;
  a.scale = 0.08838834764831845f;   // 1/sqrt(128)
  {
    auto ratio = [&](int j) { return j < p->L ? (float)((double)(p->L - j) / (double)(j + 1)) : 0.f; };
    for (int j = 0; j < mp::kFastTau; ++j) a.head_ratio[j] = ratio(j);
    for (int i = 0; i < mp::kTailTerms; ++i) a.tail_ratio[i] = ratio(p->min_hits + i);
  }
  mp::TableArgs t{};
  if (tables) {
    fill_table_args(p, tables, &t);
    t.n = n_indexed;
  }
  const hipError_t e = mp::launch_sampled_attention(a, tables ? &t : nullptr, reinterpret_cast<hipStream_t>(hip_stream),
                                                    g_have_stage_events ? g_stage_events : nullptr);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

}  // namespace

extern "C" {

size_t magicpig_code_words_per_key(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  return (size_t)mp::code_words(p->K, p->L);
}

size_t magicpig_code_words_per_query(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  return (size_t)mp::plane_words(p->K, p->L);
}

size_t magicpig_key_code_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  return (size_t)p->batch * p->n_kv_heads * (size_t)mp::key_blocks(p->n_cap) * mp::kBlockKeys *
         mp::code_words(p->K, p->L) * sizeof(uint32_t);
}

size_t magicpig_query_code_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  return (size_t)p->batch * p->n_q_heads * mp::plane_words(p->K, p->L) * sizeof(uint32_t);
}

size_t magicpig_key_code_index(const magicpig_params* p, int32_t b, int32_t g, int64_t key, int32_t word) {
  if (check_params(p) != MAGICPIG_OK) return (size_t)-1;
  const int NW = mp::code_words(p->K, p->L);
  if (b < 0 || b >= p->batch || g < 0 || g >= p->n_kv_heads || key < 0 || key >= p->n_cap ||
      word < 0 || word >= NW)
    return (size_t)-1;
  const int64_t blk = ((int64_t)b * p->n_kv_heads + g) * mp::key_blocks(p->n_cap) + key / mp::kBlockKeys;
  return (size_t)(blk * mp::kBlockKeys * NW + mp::slot_in_block(NW, word, (int)(key % mp::kBlockKeys)));
}

size_t magicpig_hash_keys_stats_offset(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK || p->dtype != MAGICPIG_BF16) return (size_t)-1;
  return ws_hash_layout(p).scalar_off;
}

size_t magicpig_workspace_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  size_t m = ws_mean(p);
  if (ws_attention(p) > m) m = ws_attention(p);
  if (ws_hash(p) > m) m = ws_hash(p);
  return m < 256 ? 256 : m;
}

int magicpig_key_mean(const magicpig_params* p, const void* K_cache, float* mu_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if ((st = check_strides(p->k_stride_b, p->k_stride_h, p->k_stride_n)) != MAGICPIG_OK) return st;
  if (!mu_out || !workspace || (!K_cache && p->n_ctx > 0 && p->batch > 0)) return MAGICPIG_INVALID_ARG;
  if (!aligned16(K_cache) || !aligned16(workspace)) return MAGICPIG_INVALID_ARG;
  if (workspace_bytes < ws_mean(p)) return MAGICPIG_WORKSPACE_TOO_SMALL;
  mp::MeanArgs a{};
  a.Kc = K_cache; a.mu = mu_out; a.partial = reinterpret_cast<double*>(workspace);
  a.is_fp32 = p->dtype == MAGICPIG_FP32;
  a.kv_fp8 = p->kv_dtype == MAGICPIG_KV_FP8_E4M3;
  a.n_kv_heads = p->n_kv_heads; a.units = p->batch * p->n_kv_heads; a.n = p->n_ctx;
  a.rows_per_chunk = kMeanRowsPerChunk;
  a.nchunk = (int)((p->n_ctx + kMeanRowsPerChunk - 1) / kMeanRowsPerChunk);
  a.stride_b = p->k_stride_b; a.stride_h = p->k_stride_h; a.stride_n = p->k_stride_n;
  const hipError_t e = mp::launch_key_mean(a, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_hash_keys(const magicpig_params* p, const void* K_cache, const float* mu, const void* W,
                       int64_t first_key, int64_t n_keys, uint32_t* key_codes, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  const int st = check_hash_keys_args(p, K_cache, mu, W, first_key, n_keys, key_codes, workspace, workspace_bytes);
  if (st != MAGICPIG_OK) return st;
  if (n_keys == 0 || p->batch == 0) return MAGICPIG_OK;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  mp::HashDirectArgs a = key_rows(p, K_cache, mu, W, first_key, n_keys, key_codes);
  if (a.total_rows <= kFewRows) {
    // a few appended keys (a decode step): one latency-bound kernel instead of the prefill pipeline
    const hipError_t e = mp::launch_hash_rows(a, nullptr, stream);
    return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
  }
  if (p->dtype == MAGICPIG_BF16) {
    // matrix-core path; the direct kernel runs afterwards only if its list overflowed
    const HashWs wl = ws_hash_layout(p);
    char* wsb = reinterpret_cast<char*>(workspace);
    mp::HashMfmaArgs m{};
    m.Kc = K_cache; m.W = W; m.mu = mu; m.codes = key_codes;
    m.K = p->K; m.L = p->L; m.NW = a.NW; m.NQ = a.NQ; m.ntiles = wl.ntiles;
    m.units = p->batch * p->n_kv_heads; m.n_kv_heads = p->n_kv_heads;
    m.kv_fp8 = p->kv_dtype == MAGICPIG_KV_FP8_E4M3;
    m.n_keys = n_keys; m.first_key = first_key; m.n_cap = p->n_cap; m.blocks_cap = a.blocks_cap;
    m.stride_b = p->k_stride_b; m.stride_h = p->k_stride_h; m.stride_n = p->k_stride_n;
    m.afrag = wsb + wl.afrag_off; m.wt = wsb + wl.wt_off;
    m.thr = reinterpret_cast<float*>(wsb + wl.thr_off);
    m.thr64 = reinterpret_cast<double*>(wsb + wl.thr64_off);
    m.magmu = reinterpret_cast<float*>(wsb + wl.magmu_off);
    m.munorm = reinterpret_cast<float*>(wsb + wl.munorm_off);
    m.rownorm = reinterpret_cast<float*>(wsb + wl.rownorm_off);
    m.wmax_bits = reinterpret_cast<unsigned*>(wsb + wl.scalar_off);
    m.list_count = m.wmax_bits + 1;
    m.overflow = reinterpret_cast<int*>(m.wmax_bits + 2);
    m.flagged_total = m.wmax_bits + 3;
    m.list = reinterpret_cast<unsigned long long*>(wsb + wl.list_off); m.list_cap = wl.list_cap;
    const hipError_t e = mp::launch_hash_keys_mfma(m, stream);
    if (e != hipSuccess) return fail_hip(e);
    a.run_flag = m.overflow;
  }
  const hipError_t e = mp::launch_hash_direct(a, stream);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_hash_query(const magicpig_params* p, const void* q, const void* W, uint32_t* q_codes,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  const int st = check_hash_query_args(p, q, W, q_codes, workspace, workspace_bytes);
  if (st != MAGICPIG_OK) return st;
  const mp::HashDirectArgs a = query_rows(p, q, W, q_codes);
  const hipError_t e = mp::launch_hash_rows(a, nullptr, reinterpret_cast<hipStream_t>(hip_stream),
                                            g_have_stage_events ? g_stage_events[5] : nullptr,
                                            g_have_stage_events ? g_stage_events[6] : nullptr);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_hash_decode_step(const magicpig_params* p, const void* q, const void* K_cache, const float* mu,
                              const void* W, int64_t first_key, int64_t n_keys, uint32_t* key_codes,
                              uint32_t* q_codes, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_hash_query_args(p, q, W, q_codes, workspace, workspace_bytes);
  if (st != MAGICPIG_OK) return st;
  const bool live = p->n_ctx_dev != nullptr;             // the newest n_keys keys, wherever the context ends now
  if (live) first_key = 0;
  if ((st = check_hash_keys_args(p, K_cache, mu, W, first_key, n_keys, key_codes, workspace, workspace_bytes)) != MAGICPIG_OK)
    return st;
  if (live && (n_keys < 1 || (int64_t)p->batch * p->n_kv_heads * n_keys > kFewRows)) return MAGICPIG_UNSUPPORTED;
  if ((int64_t)p->batch * p->n_kv_heads * n_keys > kFewRows) {   // many keys: the two calls one after the other
    st = magicpig_hash_keys(p, K_cache, mu, W, first_key, n_keys, key_codes, workspace, workspace_bytes, hip_stream);
    if (st != MAGICPIG_OK) return st;
    return magicpig_hash_query(p, q, W, q_codes, workspace, workspace_bytes, hip_stream);
  }
  const mp::HashDirectArgs aq = query_rows(p, q, W, q_codes);
  mp::HashDirectArgs ak = key_rows(p, K_cache, mu, W, first_key, n_keys, key_codes);
  ak.n_dev = p->n_ctx_dev;
  const hipError_t e = mp::launch_hash_rows(aq, &ak, reinterpret_cast<hipStream_t>(hip_stream),
                                            g_have_stage_events ? g_stage_events[5] : nullptr,
                                            g_have_stage_events ? g_stage_events[6] : nullptr);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

size_t magicpig_prepared_projector_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  return mp::prepared_layout(p->K, p->L, p->dtype == MAGICPIG_FP32).total;
}

int magicpig_prepare_projector(const magicpig_params* p, const void* W, void* prepared, void* hip_stream) {
  const int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if (!W || !prepared || !aligned16(W) || !aligned16(prepared)) return MAGICPIG_INVALID_ARG;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  const hipError_t e = p->dtype == MAGICPIG_FP32 ? mp::launch_prepare_projector_fp32(W, prepared, p->K, p->L, stream)
                                                 : mp::launch_prepare_projector(W, prepared, p->K, p->L, stream);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

size_t magicpig_centering_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK) return 0;
  if (p->dtype == MAGICPIG_FP32) return 256;               // float32 keys are coded from mu itself
  const size_t n = mp::centering_layout(p->K, p->L, (size_t)p->batch * p->n_kv_heads).total;
  return n < 256 ? 256 : n;
}

int magicpig_prepare_centering(const magicpig_params* p, const float* mu, const void* prepared, void* centering,
                               void* hip_stream) {
  const int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if (!mu || !prepared || !centering || !aligned16(mu) || !aligned16(prepared) || !aligned16(centering))
    return MAGICPIG_INVALID_ARG;
  if (p->dtype == MAGICPIG_FP32) return MAGICPIG_OK;       // nothing to prepare
  const hipError_t e = mp::launch_prepare_centering(mu, prepared, centering, p->K, p->L, p->batch * p->n_kv_heads,
                                                    reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_hash_decode_step_prepared(const magicpig_params* p, const void* q, const void* K_cache, const float* mu,
                                       const void* centering, const void* prepared, int64_t first_key, int64_t n_keys,
                                       uint32_t* key_codes, uint32_t* q_codes, void* hip_stream) {
  int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if (!prepared || !aligned16(prepared)) return MAGICPIG_INVALID_ARG;
  const bool fp32 = p->dtype == MAGICPIG_FP32;
  const void* W = reinterpret_cast<const char*>(prepared) + mp::prepared_layout(p->K, p->L, fp32).wt_off;   // (float32: the copy)
  const bool with_q = q_codes != nullptr, with_k = n_keys > 0;
  if (!with_q && !with_k) return MAGICPIG_OK;
  if (with_q && (st = check_hash_query_args(p, q, W, q_codes, nullptr, 0)) != MAGICPIG_OK) return st;
  const bool live = p->n_ctx_dev != nullptr;
  if (live) first_key = 0;
  if (with_k) {
    if ((st = check_hash_keys_args(p, K_cache, mu, W, first_key, n_keys, key_codes, nullptr, 0)) != MAGICPIG_OK &&
        st != MAGICPIG_WORKSPACE_TOO_SMALL)
      return st;
    // the few-vectors kernel only: a prefill goes through magicpig_hash_keys
    if ((int64_t)p->batch * p->n_kv_heads * n_keys > kFewRows) return MAGICPIG_UNSUPPORTED;
    if (mu && !fp32 && (!centering || !aligned16(centering))) return MAGICPIG_INVALID_ARG;
  }
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (fp32) {
    mp::HashDirectArgs aq = query_rows(p, q, W, q_codes);
    mp::HashDirectArgs ak = key_rows(p, K_cache, mu, W, first_key, n_keys, key_codes);
    ak.n_dev = p->n_ctx_dev;
    if (!with_k) ak.total_rows = 0;
    if (!with_q) aq.total_rows = 0;
    const hipError_t e = with_q ? mp::launch_hash_rows(aq, with_k ? &ak : nullptr, stream) : mp::launch_hash_rows(ak, nullptr, stream);
    return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
  }
  const mp::PreparedLayout pl = mp::prepared_layout(p->K, p->L, false);
  const char* pb = reinterpret_cast<const char*>(prepared);
  mp::HashFewArgs a{};
  a.header = reinterpret_cast<const uint32_t*>(pb);
  a.frag = pb + pl.frag_off; a.wt = pb + pl.wt_off;
  if (with_k && mu) {
    const mp::CenteringLayout cl = mp::centering_layout(p->K, p->L, (size_t)p->batch * p->n_kv_heads);
    const char* cb = reinterpret_cast<const char*>(centering);
    a.thr = reinterpret_cast<const float*>(cb + cl.thr_off);
    a.munorm = reinterpret_cast<const float*>(cb + cl.munorm_off);
    a.mu = mu;
  }
  a.q = q; a.qcodes = q_codes; a.n_q = with_q ? p->batch * p->n_q_heads : 0;
  a.Kc = K_cache; a.kcodes = key_codes;
  a.kv_fp8 = p->kv_dtype == MAGICPIG_KV_FP8_E4M3;
  a.n_krows = with_k ? (int)((int64_t)p->batch * p->n_kv_heads * n_keys) : 0;
  a.n_keys = n_keys > 0 ? n_keys : 1; a.first_key = first_key; a.n_cap = p->n_cap;
  a.blocks_cap = mp::key_blocks(p->n_cap); a.n_dev = p->n_ctx_dev;
  a.n_kv_heads = p->n_kv_heads;
  a.stride_b = p->k_stride_b; a.stride_h = p->k_stride_h; a.stride_n = p->k_stride_n;
  a.K = p->K; a.L = p->L; a.Wd = pl.Wd; a.P = pl.P;
  a.NQ = mp::plane_words(p->K, p->L); a.NW = mp::code_words(p->K, p->L);
  const hipError_t e = mp::launch_hash_few(a, stream, g_have_stage_events ? g_stage_events[5] : nullptr,
                                           g_have_stage_events ? g_stage_events[6] : nullptr);
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_hash_query_prepared(const magicpig_params* p, const void* q, const void* prepared, uint32_t* q_codes,
                                 void* hip_stream) {
  if (!q_codes) return MAGICPIG_INVALID_ARG;
  return magicpig_hash_decode_step_prepared(p, q, nullptr, nullptr, nullptr, prepared, 0, 0, nullptr, q_codes, hip_stream);
}

int magicpig_sampled_attention(const magicpig_params* p, const void* q, const void* K_cache,
                               const void* V_cache, const float* mu, const uint32_t* key_codes,
                               const uint32_t* q_codes, float* out, uint16_t* dbg_counts,
                               int32_t* dbg_cand, int32_t* dbg_ncand, int64_t dbg_cand_cap,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (p && p->n_ctx > 0 && p->batch > 0 && !key_codes) return MAGICPIG_INVALID_ARG;
  return run_attention_impl(p, q, K_cache, V_cache, mu, key_codes, nullptr, 0, q_codes, out, dbg_counts, dbg_cand,
                            dbg_ncand, dbg_cand_cap, workspace, workspace_bytes, false, false, hip_stream);
}

int magicpig_sampled_attention_noalloc(const magicpig_params* p, const void* q, const void* K_cache,
                                       const void* V_cache, const float* mu, const uint32_t* key_codes,
                                       const uint32_t* q_codes, float* out, void* hip_stream) {
  if (p && p->n_ctx > 0 && p->batch > 0 && !key_codes) return MAGICPIG_INVALID_ARG;
  return run_attention_impl(p, q, K_cache, V_cache, mu, key_codes, nullptr, 0, q_codes, out, nullptr, nullptr,
                            nullptr, 0, nullptr, 0, false, true, hip_stream);
}

size_t magicpig_table_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK || !tables_supported(p)) return 0;
  return table_layout(p).total;
}

size_t magicpig_table_build_workspace_bytes(const magicpig_params* p) {
  if (check_params(p) != MAGICPIG_OK || !tables_supported(p)) return 0;
  return ws_build_layout(p).total;
}

int magicpig_build_tables(const magicpig_params* p, const uint32_t* key_codes, void* tables,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  int st = check_params(p);
  if (st != MAGICPIG_OK) return st;
  if (!tables_supported(p)) return MAGICPIG_UNSUPPORTED;
  if (!key_codes || !tables || !aligned16(key_codes) || !aligned16(tables)) return MAGICPIG_INVALID_ARG;
  mp::TableArgs t{};
  fill_table_args(p, tables, &t);
  t.kcodes = key_codes;
  // with room for the per-table codes the keys are placed window by window (several times faster)
  const BuildWs bw = ws_build_layout(p);
  if (workspace && aligned16(workspace) && workspace_bytes >= bw.total) {
    char* wsb = reinterpret_cast<char*>(workspace);
    t.codes16 = reinterpret_cast<uint16_t*>(wsb + bw.codes_off);
    t.windows = bw.windows;
  }
  const hipError_t e = mp::launch_build_tables(t, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MAGICPIG_OK : fail_hip(e);
}

int magicpig_sampled_attention_tables(const magicpig_params* p, const void* q, const void* K_cache,
                                      const void* V_cache, const float* mu, const void* tables,
                                      int64_t n_indexed, const uint32_t* key_codes,
                                      const uint32_t* q_codes, float* out, uint16_t* dbg_counts,
                                      int32_t* dbg_cand, int32_t* dbg_ncand, int64_t dbg_cand_cap,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (p && p->n_ctx > 0 && p->batch > 0 && !tables) return MAGICPIG_INVALID_ARG;
  return run_attention_impl(p, q, K_cache, V_cache, mu, key_codes, tables, n_indexed, q_codes, out, dbg_counts, dbg_cand,
                            dbg_ncand, dbg_cand_cap, workspace, workspace_bytes, true, false, hip_stream);
}

void magicpig_profile_stage_events(void* const* events) {
  g_have_stage_events = events != nullptr;
  if (events)
    for (int i = 0; i < kStageEvents; ++i) g_stage_events[i] = reinterpret_cast<hipEvent_t>(events[i]);
}

const char* magicpig_status_string(int status) {
  switch (status) {
    case MAGICPIG_OK: return "ok";
    case MAGICPIG_INVALID_ARG: return "invalid argument";
    case MAGICPIG_UNSUPPORTED: return "unsupported configuration";
    case MAGICPIG_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MAGICPIG_LAUNCH_FAILED: return "HIP launch failed";
    case MAGICPIG_SCRATCH_TOO_SMALL:
      return "the decode step needs more scratch than the library's static array holds: use the call that takes a workspace";
    default: return "unknown status";
  }
}

const char* magicpig_last_hip_error(void) { return g_last_hip_error.c_str(); }

}  // extern "C"
