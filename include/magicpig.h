/*
 * magicpig.h - C ABI of the MI355X (gfx950) library for LSH-sampled decode attention,
 * the method of "MagicPIG: LSH Sampling for Efficient LLM Generation" (arXiv 2410.16179).
 *
 * The calls follow the paper's problem statement (Algorithm 1 "MagicPIG Decoding"):
 * inputs K, V in R^{n x d}, q in R^{1 x d}, random projectors W in R^{d x (K*L)}, a hash
 * structure over the cached keys, and a static set T of sink + local tokens.  Here the
 * hash structure is the array of packed SimHash codes of all keys, kept in HBM and
 * scanned on every decode step, or bucketed hash tables built from those codes and
 * looked up on every step; both give the same sample S.
 *
 * Conventions for every call
 *  - `params` is HOST memory, read during the call only.  Every other pointer is a
 *    DEVICE pointer owned by the caller (the library allocates and frees nothing; the
 *    only state it keeps is the per-thread event setting of
 *    magicpig_profile_stage_events, the last HIP error, and the static scratch array of
 *    magicpig_sampled_attention_noalloc).  `workspace` is caller-owned device scratch, 16-byte
 *    aligned; magicpig_workspace_bytes(params) bytes are enough for every call (each call
 *    checks only what it needs itself: query hashing and the hashing of a few appended keys
 *    need none and accept NULL); its contents need not be preserved or initialised between
 *    calls, and two calls that share it must be ordered on one stream.
 *  - `hip_stream` is a hipStream_t (NULL = default stream).  Calls enqueue work and
 *    return without synchronising.
 *  - Return value: MAGICPIG_OK or a negative status.  Arguments are validated before any
 *    GPU call, so INVALID_ARG / UNSUPPORTED / WORKSPACE_TOO_SMALL can be observed on a
 *    host without a GPU.  No C++ exception crosses this boundary.
 *  - Tensors: q [batch, n_q_heads, 128]; K/V cache [batch, n_kv_heads, n, 128] addressed
 *    through element strides (innermost dimension contiguous); W [128, K*L] row-major,
 *    column t*K + b being hyperplane b of table t; mu [batch, n_kv_heads, 128] float32.
 *    q, K, V, W share the element type `dtype` (bf16 or float32), unless kv_dtype gives the
 *    caches a storage type of their own.
 *  - Grouped-query attention: query head h uses KV head h / (n_q_heads / n_kv_heads).
 */
#ifndef MAGICPIG_H
#define MAGICPIG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden symbol visibility; these entry points are what it exports. */
#define MAGICPIG_API __attribute__((visibility("default")))

enum { MAGICPIG_BF16 = 0, MAGICPIG_FP32 = 1 };
/* storage type of the K / V cache (magicpig_params.kv_dtype) */
enum { MAGICPIG_KV_SAME = 0,        /* the caches hold `dtype` elements                          */
       MAGICPIG_KV_FP8_E4M3 = 1 };  /* the caches hold OCP e4m3 bytes (quantised K / V, the
                                       paper's App. "Limitations and future work"); needs dtype
                                       BF16 for q and W                                          */

enum {
  MAGICPIG_OK = 0,
  MAGICPIG_INVALID_ARG = -1,         /* null pointer, negative size, heads not divisible ... */
  MAGICPIG_UNSUPPORTED = -2,         /* head_dim != 128, K or L out of range, unknown dtype  */
  MAGICPIG_WORKSPACE_TOO_SMALL = -3,
  MAGICPIG_LAUNCH_FAILED = -4,       /* a HIP call failed; see magicpig_last_hip_error()      */
  MAGICPIG_SCRATCH_TOO_SMALL = -5    /* magicpig_sampled_attention_noalloc: the step needs more
                                        than MAGICPIG_STATIC_SCRATCH_BYTES of scratch          */
};

typedef struct magicpig_params {
  int32_t batch, n_q_heads, n_kv_heads;
  int32_t head_dim;   /* must be 128 */
  int32_t K;          /* sign bits per table, 1..16 */
  int32_t L;          /* tables, 1..512 */
  int32_t min_hits;   /* a key is sampled iff it collides in >= min_hits tables; the paper
                         uses 2 (Sec. 4.3).  0: every eligible key is sampled with u = 1,
                         which makes the result exact attention. */
  int32_t n_sink;     /* first n_sink and last n_local keys form the static set T, attended */
  int32_t n_local;    /* exactly and excluded from sampling (Sec. 4.4 "On-device cache");
                         each 0 .. 2^30, else MAGICPIG_INVALID_ARG */
  int32_t dtype;      /* MAGICPIG_BF16 | MAGICPIG_FP32: element type of q, K, V, W */
  int64_t n_ctx;      /* keys per sequence seen by the decode step (all sequences alike)    */
  int64_t n_cap;      /* key capacity of the code buffer per (batch, KV head), >= n_ctx     */
  int64_t k_stride_b, k_stride_h, k_stride_n;   /* element strides of the K cache */
  int64_t v_stride_b, v_stride_h, v_stride_n;   /* element strides of the V cache; the decode
                         step needs row strides (*_stride_n) below 2^31 elements */
  const int64_t* n_ctx_dev;   /* NULL, or a DEVICE pointer to the context length of the running
                         decode loop (Algorithm 1 is run once per generated token: the context grows
                         by one key per step).  When set, magicpig_hash_decode_step and
                         magicpig_sampled_attention[_tables|_noalloc] read the length from there when
                         their kernels run, so that one captured HIP graph serves every step of the
                         loop; n_ctx is then the largest value the word may hold (grids and
                         workspace are sized for it; larger values are clamped to it).  The other
                         calls ignore it. */
  int32_t kv_dtype;   /* MAGICPIG_KV_SAME | MAGICPIG_KV_FP8_E4M3.  An e4m3 cache element stands for
                         the value its byte decodes to (no scale): every result - hash codes, sample,
                         probabilities, output - is defined on those values exactly as for the other
                         types (each e4m3 value is also a bf16 value).  Strides stay in elements. */
} magicpig_params;

/* ---- packed code layout (part of the contract: the caller stores codes between calls) ----
 * Codes are bit planes over groups of 32 tables: plane word w*K + b holds, in bit beta, the
 * sign bit b (SimHash, Sec. 2.2: 1 iff the projection is >= 0) of table t = 32*w + beta.
 * A query's code is its NQ = K * ceil(L/32) plane words, [batch, n_q_heads, NQ] row-major,
 * with the bits of tables t >= L set to 1.
 * A key's code is NW words: the K*(ceil(L/32) - 1) plane words of the complete table groups
 * as they are, then the last group (Lt = L - 32*(ceil(L/32) - 1) tables) as one bit string:
 * bit b*Lt + beta of the string, counted from bit 0 of word K*(ceil(L/32) - 1), is bit b of
 * table 32*(ceil(L/32) - 1) + beta; the string ends with zeros, NW = K*(ceil(L/32) - 1) +
 * ceil(K*Lt/32).  At (K, L) = (10, 150) that is 47 words = 188 bytes for 1500 sign bits.
 * Key codes are stored in blocks of 64 consecutive keys of one (batch, KV head):
 * word x of key i lives at u32 index
 *     ((b*n_kv_heads + g)*ceil(n_cap/64) + i/64) * 64*NW + slot(x, i%64),
 *     slot(x, r) = (x/4)*256 + r*4 + x%4              for x <  4*(NW/4),
 *                = (NW/4)*256 + r*(NW%4) + x%4        otherwise,
 * i.e. each lane of a 64-wide wavefront reads its key's words as 16-byte vectors and a
 * wavefront reads a contiguous 256*NW-byte block.  magicpig_key_code_index() evaluates
 * this formula.
 */
MAGICPIG_API size_t magicpig_code_words_per_key(const magicpig_params* params);     /* NW */
MAGICPIG_API size_t magicpig_code_words_per_query(const magicpig_params* params);   /* NQ */
MAGICPIG_API size_t magicpig_key_code_bytes(const magicpig_params* params);    /* whole key-code buffer  */
MAGICPIG_API size_t magicpig_query_code_bytes(const magicpig_params* params);
/* u32 index of word x of key i of (b, g) in the key-code buffer; (size_t)-1 if out of range */
MAGICPIG_API size_t magicpig_key_code_index(const magicpig_params* params, int32_t b, int32_t g,
                               int64_t key, int32_t word);
/* Scratch that is enough for any of the calls below with these params (0 on invalid params):
 * the largest of what the key mean, the prefill key hashing (which grows with n_cap) and the
 * decode step need. */
MAGICPIG_API size_t magicpig_workspace_bytes(const magicpig_params* params);

/* Key centering vector (Sec. 4.3 "Data pre-processing"): mu[b,g,:] = (1/n_ctx) sum_i k_i over
 * keys [0, n_ctx) of each (batch, KV head), accumulated in float32 per row group and float64
 * across groups, rounded to float32.  mu_out [batch, n_kv_heads, 128] float32. */
MAGICPIG_API int magicpig_key_mean(const magicpig_params* params, const void* K_cache, float* mu_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* SimHash codes of cached keys (Sec. 4.3 "Hash function selection"; Algorithm 1 input HT):
 * for keys first_key <= i < first_key + n_keys of every (batch, KV head),
 *   bit(i, t, b) = [ sum_d (k_{i,d} - mu_d) * W_{d, t*K+b} >= 0 ],
 * the sign being that of the exact real sum over the stored values (independent of
 * summation order).  mu may be NULL (no centering).  Requires first_key + n_keys <= n_cap;
 * n_ctx is not consulted, so keys can be appended with a frozen mu.  Writes only the words
 * of those keys. */
MAGICPIG_API int magicpig_hash_keys(const magicpig_params* params, const void* K_cache, const float* mu,
                       const void* W, int64_t first_key, int64_t n_keys, uint32_t* key_codes,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Byte offset, inside the workspace a bf16 magicpig_hash_keys call used, of four uint32
 * statistics of that call: { float bits of max_j |W_j|; number of (key, projection) pairs that
 * did not fit a workgroup's own re-evaluation list and went through the global one; 1 if the
 * global list overflowed and the whole call was redone by the float64 kernel; total number of
 * pairs whose matrix-core result was too close to zero and was re-evaluated exactly }.
 * (size_t)-1 when the params are invalid or not bf16. */
MAGICPIG_API size_t magicpig_hash_keys_stats_offset(const magicpig_params* params);

/* SimHash codes of the decode queries (Algorithm 1 "Encode(q, W)"); queries are not centered. */
MAGICPIG_API int magicpig_hash_query(const magicpig_params* params, const void* q, const void* W,
                        uint32_t* q_codes, void* workspace, size_t workspace_bytes,
                        void* hip_stream);

/* The hashing of one decode step in a single launch (Algorithm 1: the new token's key joins the
 * hash structure, "Encode(q, W)" codes its query): magicpig_hash_keys for the keys
 * [first_key, first_key + n_keys) (normally the one key the step appended) together with
 * magicpig_hash_query, same arguments, same results.  With more than 128 key vectors
 * (batch * n_kv_heads * n_keys) it simply makes the two calls one after the other.
 * With params->n_ctx_dev set the keys are the newest n_keys >= 1 keys of the context as it stands
 * when the kernel runs, [*n_ctx_dev - n_keys, *n_ctx_dev), and first_key is ignored (nothing is
 * coded if that range does not lie inside [0, n_cap)); at most 128 key vectors then. */
MAGICPIG_API int magicpig_hash_decode_step(const magicpig_params* params, const void* q, const void* K_cache,
                              const float* mu, const void* W, int64_t first_key, int64_t n_keys,
                              uint32_t* key_codes, uint32_t* q_codes, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/* ---- the hashing of a decode step from a prepared projector --------------------------------
 * The decode step codes a handful of vectors against the whole projector and is bound by memory
 * latency; reading W in a layout made for it (matrix-core fragments for bf16; Sec. 4.4 (3): the
 * projections belong on the matrix units) takes the step from three dependent round trips to one.
 * magicpig_prepare_projector writes that form once per model into `prepared`
 * (magicpig_prepared_projector_bytes, 256-byte aligned, caller-owned; K, L, dtype of params are
 * baked in; an opaque format).  magicpig_prepare_centering writes, once per sequence after
 * magicpig_key_mean (the mean is frozen afterwards), the per-projection thresholds mu.W_j and
 * |mu| of every (batch, KV head) into `centering` (magicpig_centering_bytes).
 * magicpig_hash_query_prepared and magicpig_hash_decode_step_prepared then give the same codes,
 * bit for bit, as magicpig_hash_query and magicpig_hash_decode_step (the sign of the exact sum:
 * matrix-core results too close to zero are re-evaluated exactly inside the kernel).  They need
 * no workspace.  In magicpig_hash_decode_step_prepared mu and centering go together (both NULL:
 * no centering), q_codes may be NULL (keys only), n_keys may be 0 (queries only); at most 128 key
 * vectors; params->n_ctx_dev is honoured as in magicpig_hash_decode_step. */
MAGICPIG_API size_t magicpig_prepared_projector_bytes(const magicpig_params* params);
MAGICPIG_API int magicpig_prepare_projector(const magicpig_params* params, const void* W, void* prepared,
                                            void* hip_stream);
MAGICPIG_API size_t magicpig_centering_bytes(const magicpig_params* params);
MAGICPIG_API int magicpig_prepare_centering(const magicpig_params* params, const float* mu, const void* prepared,
                                            void* centering, void* hip_stream);
MAGICPIG_API int magicpig_hash_query_prepared(const magicpig_params* params, const void* q, const void* prepared,
                                              uint32_t* q_codes, void* hip_stream);
MAGICPIG_API int magicpig_hash_decode_step_prepared(const magicpig_params* params, const void* q,
                                                    const void* K_cache, const float* mu, const void* centering,
                                                    const void* prepared, int64_t first_key, int64_t n_keys,
                                                    uint32_t* key_codes, uint32_t* q_codes, void* hip_stream);

/* One decode step of sampled attention (Algorithm 1; Eq. "lsh sampling probability" and Eq.
 * "close form"): for every query head h with KV head g,
 *   count(h,i) = #{ t : code_q(h,t) == code_k(g,i,t) },
 *   T = [0,n_sink) U [n_ctx-n_local, n_ctx)   (all keys if n_ctx <= n_sink + n_local),
 *   S_h = { i not in T : count(h,i) >= min_hits },
 *   p_i = 1 - arccos(cos(q, k_i - mu))/pi,  u_i = P[Binomial(L, p_i^K) >= min_hits],
 *   out_h = softmax_{i in S_h U T}( q.k_i/sqrt(128) - [i in S_h] log u_i ) V.
 * out [batch, n_q_heads, 128] float32 (zero vector when S_h U T is empty).  mu may be NULL.
 * Optional debug outputs (NULL in production): dbg_counts [batch, n_q_heads, n_ctx] uint16;
 * dbg_cand [batch, n_q_heads, dbg_cand_cap] int32 receives S_h in unspecified order and
 * dbg_ncand [batch, n_q_heads] int32 its size (entries beyond the capacity are counted but
 * not stored; dbg_ncand must be zeroed by the caller). */
MAGICPIG_API int magicpig_sampled_attention(const magicpig_params* params, const void* q, const void* K_cache,
                               const void* V_cache, const float* mu, const uint32_t* key_codes,
                               const uint32_t* q_codes, float* out, uint16_t* dbg_counts,
                               int32_t* dbg_cand, int32_t* dbg_ncand, int64_t dbg_cand_cap,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory or carry a workspace around - code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc: the same decode step as
 * magicpig_sampled_attention (same kernels, same result bit for bit, no debug outputs) with the
 * scratch for its partial results in a static device array of MAGICPIG_STATIC_SCRATCH_BYTES that
 * belongs to the library (each GPU the library runs on holds one until the process ends).  The
 * call allocates and frees nothing.  A step that needs more scratch (4 * 132 bytes per query
 * head and run of key blocks; batch 1 with 32 heads at 98304 keys needs 1.6 MB) is refused with
 * MAGICPIG_SCRATCH_TOO_SMALL before anything is launched.  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (different streams or threads) race; order them.
 * The first call on a GPU looks up the array's device address (once per GPU, with that GPU
 * current) and should not itself be made under stream capture. */
#define MAGICPIG_STATIC_SCRATCH_BYTES (8u << 20)
MAGICPIG_API int magicpig_sampled_attention_noalloc(const magicpig_params* params, const void* q,
                                                    const void* K_cache, const void* V_cache, const float* mu,
                                                    const uint32_t* key_codes, const uint32_t* q_codes, float* out,
                                                    void* hip_stream);

/* ---- bucketed hash tables (the paper's retrieval structure: Algorithm 1 "Query(HT, q_code)";
 * App. E.2: L tables per key-value head, one key index per key and table) ----
 * For every (batch, KV head) and table the keys [0, n_ctx) are grouped by their K-bit code:
 * a decode step then reads only the L buckets selected by the query's codes instead of every
 * key's code, and obtains the same counts on the keys it touches and the same sample S.
 * Supported for K <= 12, batch * n_q_heads <= 65535 (otherwise the size is 0 and the
 * calls return MAGICPIG_UNSUPPORTED).  The buffer holds, each part 256-byte aligned: a header of
 * 256 bytes (word 0: number of 16384-key windows when the buckets are ordered by window, else
 * 0); [batch*n_kv_heads][L][2^K + 1] uint32 bucket offsets; [batch*n_kv_heads][L][n_cap] uint32
 * key indices; [batch*n_kv_heads][L][windows][2^K] uint32 fill levels of the buckets at the
 * start of every window (room for ceil(n_cap / 16384) windows).  A build with the large
 * workspace orders every bucket by window (keys of window 0 first, ...), which lets a decode
 * step read, for a range of keys, only the piece of a bucket that holds them; inside a
 * window's piece, and in buckets of the one-pass build, the order is unspecified.  Tables are
 * rebuilt from the packed
 * key codes; they are not extended incrementally: keys appended after a build are found by
 * scanning their packed codes (see n_indexed below) until the next build. */
MAGICPIG_API size_t magicpig_table_bytes(const magicpig_params* params);
/* magicpig_build_tables works with any workspace (NULL included).  Given one of at least
 * magicpig_table_build_workspace_bytes(params) bytes (2 bytes per key and table; 0 if tables
 * are unsupported) it first writes every key's
 * code per table there and then places the keys window by window, which is several times faster
 * than scattering them in one pass.  The resulting tables hold the same buckets either way. */
MAGICPIG_API size_t magicpig_table_build_workspace_bytes(const magicpig_params* params);
MAGICPIG_API int magicpig_build_tables(const magicpig_params* params, const uint32_t* key_codes, void* tables,
                          void* workspace, size_t workspace_bytes, void* hip_stream);
/* magicpig_sampled_attention with the collision scan replaced by the table lookup for the keys
 * [0, n_indexed) the tables were built over (magicpig_build_tables with n_ctx = n_indexed and
 * the same n_cap); the keys [n_indexed, n_ctx) appended since are found by the collision scan
 * of their packed codes.  n_indexed is n_ctx or a multiple of 64 (one code block) below it;
 * key_codes may be NULL when no block lies behind the indexed keys.  Every other argument,
 * the result and the debug outputs are as in magicpig_sampled_attention (dbg_counts is 0 for
 * indexed keys that share no bucket with the query, which is also their true count). */
MAGICPIG_API int magicpig_sampled_attention_tables(const magicpig_params* params, const void* q, const void* K_cache,
                                      const void* V_cache, const float* mu, const void* tables,
                                      int64_t n_indexed, const uint32_t* key_codes,
                                      const uint32_t* q_codes, float* out, uint16_t* dbg_counts,
                                      int32_t* dbg_cand, int32_t* dbg_ncand, int64_t dbg_cand_cap,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Profiling aid, and the only setting the library keeps: a per-thread (thread_local) list of
 * events, empty unless this function was called on the calling host thread; production callers
 * never call it and pay one thread-local test per call.  When `events` is non-NULL it points to
 * seven hipEvent_t handles which the later decode-step calls of this host thread attach to their
 * kernels, so that the events carry the kernels' own begin / end timestamps (what a profiler
 * reports) rather than dispatch times: magicpig_sampled_attention[_tables|_noalloc]: events[0] /
 * events[1] begin / end of the retrieval kernel (collision scan or table lookup), events[2] end of
 * the gather / estimator kernel, events[4] / events[3] begin / end of the merge kernel
 * (magicpig_sampled_attention scans and gathers in one kernel: events[0] / events[1] are its
 * begin / end and events[2] is recorded on the stream right behind it);
 * magicpig_hash_query[_prepared] and magicpig_hash_decode_step[_prepared] (few-vectors kernels):
 * events[5] / events[6] begin / end of the hashing kernel.  NULL switches it off. */
MAGICPIG_API void magicpig_profile_stage_events(void* const* events);

MAGICPIG_API const char* magicpig_status_string(int status);
/* Text of the HIP error behind the most recent MAGICPIG_LAUNCH_FAILED on this thread. */
MAGICPIG_API const char* magicpig_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MAGICPIG_H */
