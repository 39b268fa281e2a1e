/*
 * efim.h -- C ABI of the EFIM cache-hit attention library for AMD MI355X (gfx950).
 *
 * EFIM (Sec. 1, Sec. 3.1 step 4 of the paper) reorders an infilling prompt to
 * <P>prefix<S>suffix<M>inc so that the serving engine's cross-request KV cache
 * covers prefix and suffix and only the incremental tokens `inc` are computed.
 * Per attention layer this leaves, for every request r of a serving step,
 *   C_r  cached tokens  (everything in front of `inc`; 0 when nothing is reused --
 *        the "Baseline" scheme of Sec. 4.2), and
 *   N_r  new tokens     (`inc`, or the whole prompt on a miss),
 * and two operations, which are the two calls below:
 *   1. rotary-embed the new tokens at positions C_r + i and append their K/V to
 *      the paged cache;
 *   2. let the new queries attend causally over the cached pages plus themselves.
 * The paper changes nothing in the model (Sec. 3), so both are the standard
 * definitions; the cache is the paged cache of the engine it serves with (Sec. 4.2).
 *
 * General conventions
 *  - Every function returns EFIM_OK (0) or a negative efim_status_t.  No exceptions,
 *    no errno, nothing is printed.
 *  - All device buffers are owned by the caller.  The library allocates no device
 *    memory at run time.  It keeps a small ring of pinned host staging buffers (host
 *    memory only) for the work list it sends to the device, and its code object carries
 *    static device memory: 2 MiB of arrival counters (one block per launch in flight) with
 *    which the workgroups of a split key range elect the one that combines them, and two
 *    2 MiB buffers that hold the work lists of batches launched more than once.
 *    If a kernel is killed half-way (device fault, reset) the counters may be left
 *    non-zero; after such an event the process should not keep using the library.
 *  - The calls that take a batch description plan their work on the host and rotate
 *    host-side state (staging buffers, blocks of counters, completion events): they may not
 *    be captured into a HIP graph.  The plan-object calls at the end of this header launch
 *    kernels only and may be captured.
 *  - A stream handed to a call must stay valid until efim_stream_release(stream) has been
 *    called or the process ends: completion of the calls on it is tracked lazily (an event is
 *    recorded on the stream of earlier calls when a later call needs it).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    enqueue work and return; they do not wait for the device.
 *  - Host arrays named in efim_batch_t are read before the call returns and may be
 *    reused or freed immediately afterwards.
 *  - bf16 tensors are raw 16-bit patterns; all tensor base pointers must be 16-byte
 *    aligned.  Offsets are computed in 64 bits.
 *  - Contents of device arrays (block_table entries) are not validated.
 */
#ifndef EFIM_H_
#define EFIM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum efim_status {
  EFIM_OK = 0,
  EFIM_ERR_INVALID_ARG = -1, /* NULL pointer, negative size, misaligned pointer, Hq % Hkv != 0 ... */
  EFIM_ERR_UNSUPPORTED = -2, /* head_dim not in {64,128}, page_size not a power of two in [8,256], batch too large */
  EFIM_ERR_WORKSPACE = -3,   /* workspace NULL/misaligned or smaller than efim_extend_workspace_bytes */
  EFIM_ERR_LAUNCH = -4       /* a HIP call failed; efim_last_hip_error() holds its hipError_t     */
} efim_status_t;

/*
 * One serving step's ragged batch (plain data, caller-owned, read-only).
 *
 * New-token tensors are packed: the rows of request r start at sum_{s<r} new_len[s];
 * T = sum_r new_len[r] is the total number of new tokens.
 * Logical position p of request r is stored in physical page
 * block_table[r * max_pages_per_req + p / page_size] at slot p % page_size.
 * Entries [0, ceil((C_r + N_r) / page_size)) of row r must be valid page ids in
 * [0, num_pages); later entries are never dereferenced.
 * A request with new_len 0 contributes no rows and causes no reads or writes.
 */
typedef struct efim_batch {
  int32_t batch;             /* B >= 0                                                   */
  int32_t num_q_heads;       /* Hq, a multiple of num_kv_heads                           */
  int32_t num_kv_heads;      /* Hkv >= 1                                                 */
  int32_t head_dim;          /* D: 64 or 128                                             */
  int32_t page_size;         /* P: a power of two, 8 <= P <= 256 (16 in the paper's engine)  */
  int32_t max_pages_per_req; /* row stride of block_table                                */
  int64_t num_pages;         /* pages in each of k_cache and v_cache                     */
  const int32_t* cached_len; /* HOST  [B]  C_r >= 0                                      */
  const int32_t* new_len;    /* HOST  [B]  N_r >= 0                                      */
  const int32_t* block_table;/* DEVICE [B, max_pages_per_req] int32 physical page ids    */
} efim_batch_t;

/*
 * efim_rope_append -- rotary embedding at offset positions + paged KV append.
 *
 * For new token i of request r, position pos = C_r + i (its index in the reordered
 * prompt, Sec. 1), and for pair j < D/2 with angle pos * rope_base^(-2j/D):
 *   rotate-half pairing (rope_interleaved = 0): (x[j], x[j + D/2])
 *   interleaved pairing (rope_interleaved = 1): (x[2j], x[2j + 1])
 * The rotation is evaluated in fp64 and rounded once to bf16 (nearest even).
 *
 *   q        DEVICE bf16 [T, Hq, D]   in/out: rotated in place.  May be NULL (keys only).
 *   k_new    DEVICE bf16 [T, Hkv, D]  raw keys of the new tokens (read only)
 *   v_new    DEVICE bf16 [T, Hkv, D]  values of the new tokens (read only, copied bit for bit)
 *   k_cache  DEVICE bf16 [num_pages, Hkv, P, D]  receives the rotated keys
 *   v_cache  DEVICE bf16 [num_pages, Hkv, P, D]  receives the values
 * Exactly the slots [C_r, C_r + N_r) of every request are written; no other byte of
 * the caches changes.  Pages written by one call must not be shared between requests.
 * B = 0 or T = 0: returns EFIM_OK without launching.
 */
int efim_rope_append(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                     void* k_cache, void* v_cache, double rope_base, int rope_interleaved,
                     void* stream);

/*
 * efim_rope_append_table -- the same with the rotary variants of the models the paper serves
 * (Sec. 4: their public configurations scale the frequencies for long contexts or rotate
 * only part of a head): pair j rotates by pos * inv_freq[j], and only the leading rotary_dim
 * elements of every head row take part -- pairs (x[j], x[j + rotary_dim/2]) or, interleaved,
 * (x[2j], x[2j + 1]), j < rotary_dim/2; elements rotary_dim .. D-1 are copied bit for bit.
 *   inv_freq    HOST double[rotary_dim / 2], finite; read before the call returns
 *   rotary_dim  multiple of 16, 16 <= rotary_dim <= head_dim
 * efim_rope_append(.., rope_base, ..) is this call with inv_freq[j] = rope_base^(-2j/D) and
 * rotary_dim = D.  Everything else (buffers, slots written, errors) as efim_rope_append;
 * EFIM_ERR_INVALID_ARG also for a NULL or non-finite table or a bad rotary_dim.
 */
int efim_rope_append_table(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                           int rope_interleaved, void* stream);

/*
 * efim_extend_workspace_bytes -- device workspace efim_extend_attention needs for this
 * batch (the partial results of split key ranges; at least 256).  Pure host function;
 * returns 0 for an invalid batch.  The size depends only on the host fields of `batch`
 * and on the tuning knobs in force.
 */
size_t efim_extend_workspace_bytes(const efim_batch_t* batch);

/*
 * efim_extend_attention -- causal softmax attention of the new tokens over the cached
 * pages plus themselves.
 *
 * New row i of request r and query head a (kv head a / (Hq/Hkv)) sees keys 0 .. C_r + i:
 *   s_j = sm_scale * <q_i, k_j>,  p = softmax_j(s),  out_i = sum_j p_j v_j.
 * Scores and outputs are accumulated in fp32 from bf16 operands; out is rounded to bf16.
 *
 *   q        DEVICE bf16 [T, Hq, D]  queries, already rotated (efim_rope_append's output)
 *   k_cache  DEVICE bf16 [num_pages, Hkv, P, D]  must already hold slots [0, C_r + N_r)
 *   v_cache  DEVICE bf16 [num_pages, Hkv, P, D]
 *   out      DEVICE bf16 [T, Hq, D]  must not alias q or the caches
 *   sm_scale softmax scale; 0 selects 1/sqrt(D)
 *   workspace DEVICE, 256-byte aligned, at least efim_extend_workspace_bytes(batch) bytes;
 *            its contents are scratch and it must not be used by an overlapping call
 * Slots at or beyond C_r + N_r in a request's last page, and pages not named in the used
 * part of its block-table row, may hold anything (NaN included) and do not influence out.
 * B = 0 or T = 0: returns EFIM_OK without launching.
 */
int efim_extend_attention(const efim_batch_t* batch, const void* q, const void* k_cache,
                          const void* v_cache, void* out, float sm_scale, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * efim_extend_attention_static -- efim_extend_attention for callers that cannot allocate device
 * memory or hold a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same result bit for
 * bit.  The work list and the partial results of split key ranges live in a fixed 32 MiB array
 * inside the library's code object (held by every device the library runs on until the process
 * ends); the call allocates nothing -- no hipMalloc, hipHostMalloc or hipFree -- after its
 * first use on a device has looked the array's address up.
 * Limits: the batch's work list must fit 2 MiB and its partial results
 * efim_extend_static_limit_bytes() (30 MiB; efim_extend_workspace_bytes(batch) tells what a
 * batch needs); otherwise EFIM_ERR_WORKSPACE and nothing is launched -- use
 * efim_extend_attention then.
 * All calls on one device share the array: calls that overlap on a device (different streams,
 * no ordering between them) race; calls on one stream, or ordered by events, do not.  A change
 * of batch waits on the host for the previous upload of a work list (a few microseconds of
 * copy), never for a kernel.  Other errors as efim_extend_attention.
 */
size_t efim_extend_static_limit_bytes(void);
int efim_extend_attention_static(const efim_batch_t* batch, const void* q, const void* k_cache,
                                 const void* v_cache, void* out, float sm_scale, void* stream);

/* Records what the library still has to record on `stream` (the completion event shared by
 * its latest calls there).  Call it before destroying a stream that was handed to the library.
 * Returns EFIM_OK or EFIM_ERR_LAUNCH. */
int efim_stream_release(void* stream);

const char* efim_status_string(int status);
int efim_last_hip_error(void); /* hipError_t of the most recent EFIM_ERR_LAUNCH on this thread */
int efim_version(void);        /* major * 10000 + minor * 100 + patch */
/* SHA-256 (hex) over the library's source files as they were when it was built; "" if the
 * build did not record one.  Lets a loader tell a stale binary from a current one. */
const char* efim_source_digest(void);

/* ---------------------------------------------------------------------------------------
 * Decode step, and other short steps, in one launch.  After the prompt, the engine generates
 * the answer one token per request and step (Sec. 2.2, the prefill / decode breakdown; Sec. 4.2:
 * 128 output tokens per request); and a cache hit on prefix and suffix leaves only a few
 * incremental tokens per request to compute (Sec. 1, Sec. 3.1).  For a batch of such requests --
 * every r has 1 <= new_len[r] <= 16 and new_len[r] * (num_q_heads / num_kv_heads) <= 32 --
 * efim_decode_step computes what
 *     efim_rope_append(batch, q, k_new, v_new, k_cache, v_cache, rope_base, rope_interleaved)
 *     efim_extend_attention(batch, q, k_cache, v_cache, out, sm_scale, ...)
 * compute, with one kernel: same cache contents bit for bit, same `out`.  The one difference:
 * q is read only -- it is rotated on the fly and NOT rewritten in place.
 *
 * workspace: DEVICE, 256-byte aligned, at least efim_decode_workspace_bytes(batch) bytes,
 * contents irrelevant (as for efim_extend_attention).
 * Errors: as efim_extend_attention / efim_rope_append; EFIM_ERR_UNSUPPORTED if some request
 * has no new token, more than 16 of them, or more than 32 query rows (new tokens x query heads)
 * per kv head.
 * efim_decode_workspace_bytes returns 0 for a batch efim_decode_step would reject.
 * ------------------------------------------------------------------------------------- */
size_t efim_decode_workspace_bytes(const efim_batch_t* batch);
int efim_decode_step(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                     void* k_cache, void* v_cache, void* out, double rope_base, int rope_interleaved,
                     float sm_scale, void* workspace, size_t workspace_bytes, void* stream);
/* The same with the rotary variants of efim_rope_append_table (inv_freq: HOST double[rotary_dim / 2];
 * rotary_dim a multiple of 16 in [16, head_dim]): what efim_rope_append_table followed by
 * efim_extend_attention compute, in one launch. */
int efim_decode_step_table(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, void* out, const double* inv_freq, int rotary_dim,
                           int rope_interleaved, float sm_scale, void* workspace, size_t workspace_bytes,
                           void* stream);

/* ---------------------------------------------------------------------------------------
 * 8-bit KV cache.  The paper serves unmodified models on a stock engine (Sec. 4.2) and does
 * not discuss the cache's number format; these three calls are the calls above for the common
 * engine option of a cache held in 8-bit floating point, which halves the bytes the cache-hit
 * attention reads.
 *
 * Format: OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
 * largest finite value 448), one byte per element, same [num_pages, Hkv, P, D] layout, one
 * scale per tensor:  value = code_value * scale.
 *   k_cache, v_cache  DEVICE  uint8 [num_pages, Hkv, P, D]
 *   k_scale, v_scale  finite, > 0
 * Append: what the bf16 call would have stored (the rotated key after its rounding to bf16,
 * the value as given) is divided by the scale in binary32 and rounded to the nearest code,
 * ties to the even code, magnitudes of 448 and above saturating to +-448.  q is rotated in
 * place exactly as by efim_rope_append.
 * Attention: as efim_extend_attention with code_value * scale in place of the bf16 cache
 * entries; q and out stay bf16.  Workspace as for the bf16 calls (same size queries).
 * Errors: as the bf16 calls; EFIM_ERR_INVALID_ARG for a scale that is not finite and positive.
 * ------------------------------------------------------------------------------------- */
int efim_rope_append_fp8(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, double rope_base, int rope_interleaved,
                         float k_scale, float v_scale, void* stream);
int efim_extend_attention_fp8(const efim_batch_t* batch, const void* q, const void* k_cache,
                              const void* v_cache, void* out, float sm_scale, float k_scale, float v_scale,
                              void* workspace, size_t workspace_bytes, void* stream);
int efim_decode_step_fp8(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, void* out, double rope_base, int rope_interleaved,
                         float sm_scale, float k_scale, float v_scale, void* workspace, size_t workspace_bytes,
                         void* stream);
/* The 8-bit append and decode step with the caller's frequency table over the first rotary_dim
 * features (arguments as efim_rope_append_table / efim_decode_step_table, scales as above). */
int efim_rope_append_fp8_table(const efim_batch_t* batch, void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, const double* inv_freq, int rotary_dim,
                               int rope_interleaved, float k_scale, float v_scale, void* stream);
int efim_decode_step_fp8_table(const efim_batch_t* batch, const void* q, const void* k_new, const void* v_new,
                               void* k_cache, void* v_cache, void* out, const double* inv_freq, int rotary_dim,
                               int rope_interleaved, float sm_scale, float k_scale, float v_scale,
                               void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Session pool: the FIM -> EFIM prompt rewrite in front of the engine (Sec. 3.1, steps 1-5
 * of the prompt transformation figure).  Host code only; no device is touched.
 *
 * A pool maps a user id to that user's session: the prefix and suffix of the previous
 * request as they were laid out in the prompt, and the prompt itself.  For a new request
 * (prefix, suffix), both sequences of token ids that contain none of the three marker ids:
 *   step 1/2  no session: PSM order  <P> prefix <S> suffix <M>; the session is created;
 *   step 3/4  same suffix and the prefix extends the session's: EFIM order
 *             <P> common <S> suffix <M> inc  with common = the session's prefix; the session
 *             keeps (common, suffix), so the next EFIM prompt extends this one;
 *   step 5    anything else (the paper names growth at the head of the suffix): PSM order with
 *             the new prefix and suffix, which replace the session.  A request identical to
 *             the session keeps its previous layout.
 * What a prefix-matching paged KV cache then reuses is reported alongside: cached_len is the
 * longest common token prefix of this prompt and the user's previous one, rounded down to
 * reuse_granularity tokens and at most prompt_len - 1; new_len = prompt_len - cached_len.
 * These are the C_r and N_r of efim_batch_t for this request.
 * ------------------------------------------------------------------------------------- */
typedef struct efim_session_pool efim_session_pool_t;

enum { EFIM_ORDER_PSM = 0, EFIM_ORDER_EFIM = 1 };

typedef struct {
  int32_t order;       /* EFIM_ORDER_PSM or EFIM_ORDER_EFIM                           */
  int32_t reserved;
  int64_t common_len;  /* tokens between <P> and <S>                                  */
  int64_t inc_len;     /* tokens behind <M> (0 in PSM order)                          */
  int64_t suffix_len;
  int64_t prompt_len;  /* common_len + suffix_len + inc_len + 3                       */
  int64_t cached_len;  /* reusable leading tokens (see above)                         */
  int64_t new_len;     /* prompt_len - cached_len >= 1                                */
} efim_prompt_info_t;

/* Creates an empty pool.  tok_p/tok_s/tok_m are the ids of <P>, <S>, <M> (pairwise
 * different); reuse_granularity >= 1 (16 for a cache with 16-token pages, 1 for exact
 * token reuse); always_psm != 0 switches steps 4 off (PSM order with cache reuse: the
 * "FIM" scheme of Sec. 4.2).  Returns NULL on invalid arguments or allocation failure.
 * The caller owns the pool and releases it with efim_session_pool_destroy (NULL is ok).
 * A pool may be used from several threads; calls on one pool are serialised. */
efim_session_pool_t* efim_session_pool_create(int32_t tok_p, int32_t tok_s, int32_t tok_m,
                                              int32_t reuse_granularity, int32_t always_psm);
void efim_session_pool_destroy(efim_session_pool_t* pool);

/* Steps 1-5 for one request.  prefix/suffix: HOST arrays of n_prefix/n_suffix token ids
 * (may be NULL when the length is 0), read before the call returns.  Fills *info and stores
 * the prompt in the session.  EFIM_ERR_INVALID_ARG for NULL pool/info, negative lengths, a
 * NULL array with a positive length, or a marker id inside prefix or suffix (the session is
 * left untouched). */
int efim_session_transform(efim_session_pool_t* pool, uint64_t user, const int32_t* prefix,
                           int64_t n_prefix, const int32_t* suffix, int64_t n_suffix,
                           efim_prompt_info_t* info);

/* Copies the prompt last built for `user` into dst (HOST, capacity tokens; at most capacity
 * are written, dst may be NULL when capacity is 0) and returns its full length, 0 if the
 * user has no session, or EFIM_ERR_INVALID_ARG. */
int64_t efim_session_prompt(efim_session_pool_t* pool, uint64_t user, int32_t* dst, int64_t capacity);

/* Forgets one user's session (returns 1 if there was one, 0 if not) / counts the sessions.
 * Both return EFIM_ERR_INVALID_ARG for a NULL pool. */
int efim_session_drop(efim_session_pool_t* pool, uint64_t user);
int64_t efim_session_count(efim_session_pool_t* pool);


/* ---------------------------------------------------------------------------------------
 * Plan objects: the attention call and the decode step as pure kernel launches.
 *
 * The calls above plan a batch's work on the host every time the batch changes and keep the
 * result in process-wide state.  A plan object is the same plan with an explicit owner: built
 * once from the host fields of a batch (the per-request lengths of Sec. 1's problem statement),
 * written once into a workspace the caller owns, and from then on every launch reads it from
 * there.  The planned calls keep no state in the library, touch no host-side ring, record no
 * event and never wait for the device: they may run from any thread and may be captured into a
 * HIP graph (they enqueue kernels only, no memset or copy).  This is how an engine replays the
 * decode step of Sec. 2.2 / Sec. 4.2 (128 output tokens per request) without a launch gap per
 * kernel.
 *
 *   efim_plan_create          HOST only.  Reads batch->cached_len / new_len and the scalar fields
 *                             (block_table is not looked at); decode != 0 plans a step for
 *                             efim_decode_step_planned (the batches efim_decode_step takes, else
 *                             NULL).
 *                             Returns NULL for an invalid or unsupported batch.  The caller owns
 *                             the plan and releases it with efim_plan_destroy (NULL is ok).
 *   efim_plan_workspace_bytes bytes of DEVICE workspace the plan needs (work list, arrival
 *                             counters, partial results of split key ranges), at least 256.
 *   efim_plan_upload          enqueues on `stream` the copy of the work list into `workspace`
 *                             (DEVICE, 256-byte aligned) and a kernel that clears the arrival
 *                             counters.  The plan keeps the host image of the list alive, so the
 *                             call returns at once; the workspace is usable by planned calls
 *                             enqueued behind it on the same stream (or ordered behind it by
 *                             events).  Not capturable (it copies).  One workspace belongs to
 *                             one plan; launches that use the same workspace at the same time
 *                             race, launches on one stream or in one graph do not.
 *   efim_extend_attention_planned / efim_decode_step_planned
 *                             efim_extend_attention / efim_decode_step for the planned batch:
 *                             same arguments minus the batch description, plus the batch's
 *                             DEVICE block table (same layout and row stride as when the plan
 *                             was created).  Same result bit for bit.
 * Errors: EFIM_ERR_INVALID_ARG (NULL or misaligned pointers, a decode call on an attention plan
 * or the reverse), EFIM_ERR_WORKSPACE (workspace NULL, misaligned or too small at upload),
 * EFIM_ERR_LAUNCH.
 * ------------------------------------------------------------------------------------- */
typedef struct efim_plan efim_plan_t;

efim_plan_t* efim_plan_create(const efim_batch_t* batch, int decode);
void efim_plan_destroy(efim_plan_t* plan);
size_t efim_plan_workspace_bytes(const efim_plan_t* plan);
int efim_plan_upload(efim_plan_t* plan, void* workspace, size_t workspace_bytes, void* stream);
int efim_extend_attention_planned(const efim_plan_t* plan, const int32_t* block_table, const void* q,
                                  const void* k_cache, const void* v_cache, void* out, float sm_scale,
                                  void* workspace, void* stream);
int efim_decode_step_planned(const efim_plan_t* plan, const int32_t* block_table, const void* q,
                             const void* k_new, const void* v_new, void* k_cache, void* v_cache, void* out,
                             double rope_base, int rope_interleaved, float sm_scale, void* workspace,
                             void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EFIM_H_ */
