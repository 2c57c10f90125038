/*
 * libadapshot -- MI355X (gfx950) hot path of AdapShot's semantics-aware KV-cache reuse.
 *
 * The path, per query (AdapShot paper, Method section):
 *   1. gather the cached K/V blocks of the selected shots from the global pool
 *      into one contiguous many-shot cache, in relevance order
 *      (Semantically-Aware KV Cache; Eq. prefill defines what the pool holds);
 *   2. re-encode every gathered key to its new position with the RoPE
 *      compensation rotation (Position Decoupling and Re-encoding,
 *      Eq. rope_encoding / Eq. rope_compensation), fused into the gather;
 *   3. let the probe/query tokens attend over the assembled cache plus their own
 *      tokens (softmax(q k^T / sqrt(d)) v, the scaling of Eq. attention_score;
 *      context layout of Eq. probe_context);
 *   4. reduce each probe's output logits to the entropy of its distribution
 *      (Eq. entropy), the quantity compared with the threshold tau.
 *
 * General conventions
 *   - Plain C ABI.  Pointers marked DEVICE are HIP device pointers owned by the
 *     caller (the library never frees or reallocates them); pointers marked HOST
 *     are ordinary host memory read before the call returns.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All kernels of a call are enqueued on it; calls return without waiting for
 *     the GPU.  A context owns device scratch (RoPE tables, tile descriptors,
 *     split partials), so calls on ONE context must be issued in stream order on
 *     one stream at a time; use one context per concurrent stream.
 *   - Allocation and waiting.  adapshot_create allocates the RoPE tables (hipMalloc and two
 *     blocking copies).  adapshot_query_attn, adapshot_query_attn_pool, the batched attention calls, adapshot_probe_entropy,
 *     adapshot_probe_entropy_tokens and adapshot_rank_shots keep grow-only workspaces: a call that
 *     needs more than any earlier call on the context calls hipMalloc (an outgrown buffer is kept
 *     until adapshot_destroy, never freed in a call, so no call waits for the device); a call that
 *     fits the existing workspaces allocates nothing.  adapshot_assemble, adapshot_query_attn_pool, the batched
 *     calls and adapshot_rank_shots write small tables into a ring of 8 pinned host buffers (hipHostMalloc
 *     when one must grow); the ninth such call in flight waits for the first one's kernels.  No
 *     call synchronises the device or the stream otherwise.  adapshot_probe_entropy_static is the
 *     variant of the entropy call that never allocates.
 *   - Every function validates its arguments on the host BEFORE launching
 *     anything: a call that returns an error has written nothing to device
 *     memory.  The reason is kept per context (adapshot_last_error).
 *   - Tensor layouts are row-major with the last index contiguous:
 *       pool     K, V : [n_layers][layer_stride_tokens][n_kv_heads][head_dim]
 *       cache    K, V : [n_layers][capacity]           [n_kv_heads][head_dim]
 *       queries  Q    : [t_q][n_q_heads][head_dim]
 *       self     K, V : [t_q][n_kv_heads][head_dim]
 *     element type = desc.dtype (fp32, or bf16 as 16-bit patterns).  Base
 *     pointers must be 16-byte aligned and head_dim * sizeof(element) a multiple
 *     of 32 bytes.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - RoPE uses the half-split pairing (i, i + head_dim/2) with
 *     theta_i = rope_theta^(-2i/head_dim); angles come from tables built in fp64.
 */
#ifndef ADAPSHOT_H_
#define ADAPSHOT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adapshot_ctx adapshot_ctx; /* opaque, host side */

typedef enum {
    ADAPSHOT_OK = 0,
    ADAPSHOT_EINVAL = 1,    /* null pointer, bad size, unsupported shape, misaligned pointer */
    ADAPSHOT_ESHOT = 2,     /* shot id or order entry out of range */
    ADAPSHOT_ECAPACITY = 3, /* cache capacity or max_position exceeded */
    ADAPSHOT_ESTATE = 4,    /* no pool registered, or n_ctx beyond the assembled length */
    ADAPSHOT_EDEVICE = 5    /* a HIP runtime call failed (no GPU, out of memory, ...) */
} adapshot_status;

typedef enum { ADAPSHOT_F32 = 0, ADAPSHOT_BF16 = 1 } adapshot_dtype;

/* How the pool's keys were stored.
 *   UNROTATED     : keys carry no position; the re-encode angle is p_new * theta.
 *   ROTATED_LOCAL : each shot was prefilled on its own at positions 0..T-1 (the
 *                   paper's offline phase); the re-encode angle is
 *                   Delta * theta with Delta = p_new - t (Eq. rope_compensation). */
typedef enum { ADAPSHOT_KEYS_UNROTATED = 0, ADAPSHOT_KEYS_ROTATED_LOCAL = 1 } adapshot_key_state;

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim;
    double rope_theta;            /* RoPE base (1e4 in Eq. rope_encoding; model dependent) */
    int32_t dtype;                /* adapshot_dtype */
    int32_t key_state;            /* adapshot_key_state */
    int64_t max_position;         /* largest position + 1 any token may take; 0 = 1048576 */
} adapshot_model_desc;

/* Create a context for one model shape on the current HIP device: validates the
 * shape (n_q_heads % n_kv_heads == 0, head_dim even, 16-byte row chunks), builds the
 * RoPE tables in fp64 and uploads them.  *out is NULL on failure. */
adapshot_status adapshot_create(const adapshot_model_desc* desc, adapshot_ctx** out);
void adapshot_destroy(adapshot_ctx* ctx);
/* Text of the last error on this context ("" if none).  Valid until the next call. */
const char* adapshot_last_error(const adapshot_ctx* ctx);
/* Library version / build string. */
const char* adapshot_version(void);

/* Register the global shot pool (offline phase, Eq. prefill): k_pool / v_pool are
 * DEVICE pointers BORROWED for the life of the context; shot_offsets is HOST
 * int64[n_shots + 1], non-decreasing, shot i owning pool tokens
 * [shot_offsets[i], shot_offsets[i+1]); it is copied.  layer_stride_tokens is the
 * token count between consecutive layers (>= shot_offsets[n_shots]). */
adapshot_status adapshot_pool_register(adapshot_ctx* ctx, const void* k_pool, const void* v_pool,
                                       const int64_t* shot_offsets, int32_t n_shots,
                                       int64_t layer_stride_tokens);

/* The assembled many-shot cache of one query.  k, v: DEVICE, caller-owned,
 * [n_layers][capacity][n_kv_heads][head_dim].  len (HOST, in/out) is the number of
 * slots already filled; assemble appends at slot len.  slot_shot / slot_tok /
 * slot_pos are optional DEVICE arrays of `capacity` entries (NULL to skip) that
 * receive, per slot, the pool shot id, the token index inside that shot and the
 * position the key was re-encoded to. */
typedef struct {
    void* k;
    void* v;
    int64_t capacity;
    int64_t len;
    int32_t* slot_shot;
    int32_t* slot_tok;
    int64_t* slot_pos;
} adapshot_cache;

/* Gather + re-encode (steps 1 and 2).  shot_ids, order: HOST int32[m].  Slot
 * group j (j = 0..m-1) receives shot shot_ids[order[j]] (order == NULL: identity);
 * duplicates are allowed and m == 0 is a no-op.  The first appended token lands in
 * slot cache->len and takes position pos0 + cache->len, later tokens follow
 * contiguously (pos0 = length of the instruction prefix I of Eq. probe_context).
 * V rows are bit copies; K rows are rotated in fp32 and rounded to nearest-even.
 * On success cache->len is advanced.  Errors: ESTATE (no pool), ESHOT,
 * ECAPACITY (capacity or max_position), EINVAL. */
adapshot_status adapshot_assemble(adapshot_ctx* ctx, adapshot_cache* cache, const int32_t* shot_ids,
                                  const int32_t* order, int32_t m, int64_t pos0, void* hip_stream);

/* Query-over-cache attention for one layer (step 3).  Row j (0..t_q-1) attends to
 * cache slots [0, n_ctx) in full and to self tokens 0..j causally.  q, k_self,
 * v_self (DEVICE) are given WITHOUT rotation: the library rotates row j of q and
 * k_self to position q_pos0 + j.  n_ctx <= cache->len.  out: DEVICE
 * [t_q][n_q_heads][head_dim] in desc.dtype.  Scores and the online softmax are kept
 * in fp32; bf16 models use bf16 MFMA for q k^T and p v with fp32 accumulation, and the
 * partial outputs of the context splits are exchanged as fp16 rows scaled by their
 * largest element (error <= 2^-11 of that element, below the bf16 rounding of out).
 * Accuracy of the bf16 path depends on the data: the rotated, pre-scaled query and the keys are bf16
 * matrix operands, so a score carries about 2^-9 of its own magnitude as error and the output error
 * grows with the spread of the scores.  With N(0,1) queries, keys and values the outputs stay within
 * 2e-2 (max-abs) of the exact result; keys three times as large were measured at 1.9e-2, eight times
 * as large at 6e-2.  Accumulation, maxima and sums are fp32 throughout.
 * Errors, all found before anything is launched (out is then untouched): EINVAL (null or
 * misaligned pointer, t_q < 1, layer out of range, n_ctx < 0, q_pos0 < 0, a q of 2 GiB or more, or a
 * context or query whose K/V rows span more than 4 GiB in one layer), ESTATE (n_ctx beyond
 * cache->len), ECAPACITY (q_pos0 + t_q beyond max_position). */
adapshot_status adapshot_query_attn(adapshot_ctx* ctx, const adapshot_cache* cache, int32_t layer,
                                    int64_t n_ctx, const void* q, const void* k_self,
                                    const void* v_self, int32_t t_q, int64_t q_pos0, void* out,
                                    void* hip_stream);

/* Zero-copy form of steps 1-3 for one layer: the query rows attend over the selected shots where they lie in
 * the pool, without an assembled cache.  The result is what adapshot_assemble(shot_ids, order, m, pos0) into an
 * empty cache followed by adapshot_query_attn over all of it (n_ctx = the shots' total length) gives, up to
 * rounding: the attention kernel gathers every 64-slot tile of the context row by row through a slot -> pool
 * token table and rotates its keys to the positions pos0 + slot inside the key loop, in LDS, before the first
 * product reads them (Position Decoupling and Re-encoding: R(a)R(b) = R(a+b), so the rotation of a tile's
 * first position and the rotation of the row's index inside the tile compose; Eq. rope_compensation).  Worth
 * it for a context that is attended once; a context that is attended again (further layers' probes, every
 * decode step) is cheaper assembled once.  shot_ids, order: HOST int32[m] as in adapshot_assemble; q, k_self,
 * v_self, out, q_pos0 as in adapshot_query_attn.  Two launches besides the merge of the split partials: a small
 * one that expands the plan, and the attention.  Pools registered with ADAPSHOT_KEYS_UNROTATED only (ESTATE
 * otherwise).  bf16 models with head_dim 128 run the matrix-core kernel described above, for which a pool layer
 * must stay below 4 GiB (ECAPACITY); other shapes run a plain kernel that gathers and rotates key by key. */
adapshot_status adapshot_query_attn_pool(adapshot_ctx* ctx, int32_t layer, const int32_t* shot_ids,
                                         const int32_t* order, int32_t m, int64_t pos0, const void* q,
                                         const void* k_self, const void* v_self, int32_t t_q, int64_t q_pos0,
                                         void* out, void* hip_stream);

/* Batched forms (several independent queries per call, e.g. the adaptive probe sweep over nested
 * prefixes, or the queries of a decode batch).  Every item is validated before anything is launched:
 * a call that returns an error has written nothing.
 *
 * adapshot_assemble_batched: cache b receives shot_ids[b][orders[b][j]], j = 0..m[b]-1, appended at
 * caches[b].len, first position pos0 + caches[b].len.  shot_ids / orders / m are HOST arrays of n_caches
 * entries (orders, or any orders[b], may be NULL).  The caches must be distinct buffers. */
adapshot_status adapshot_assemble_batched(adapshot_ctx* ctx, adapshot_cache* caches, int32_t n_caches,
                                          const int32_t* const* shot_ids, const int32_t* const* orders,
                                          const int32_t* m, int64_t pos0, void* hip_stream);

/* One attention problem of a batch: rows of q (t_q tokens at positions q_pos0 + j) over slots [0, n_ctx)
 * of caches[cache_index] plus their own tokens, as in adapshot_query_attn.  Several items may use the
 * same cache with different n_ctx: probes over nested prefixes (tree-structured multi-probe of the
 * Probe-based Dynamic Evaluation section) need no re-assembly because a prefix keeps its positions.
 * For bf16 models with head_dim 128 the whole batch runs as two launches (one attention grid over all items,
 * whose workgroups rotate the query rows they need themselves, and one combine grid): the context splits
 * have one common length, so
 * probes over nested prefixes of one cache read identical leading slices, and those workgroups are
 * scheduled next to each other.  Other shapes run item by item.  The outputs of distinct items must not
 * overlap; inputs may be shared between items.  A call whose arguments other than `layer` equal the previous
 * batched call's on this context (the same items, caches, pointers and lengths: the next layer of a forward pass)
 * reuses the tables the previous call left in device memory and only launches; nothing the caller does between
 * the two calls can make that wrong except freeing or moving the buffers the items name. */
typedef struct {
    const void* q;       /* DEVICE [t_q][n_q_heads][head_dim] */
    const void* k_self;  /* DEVICE [t_q][n_kv_heads][head_dim] */
    const void* v_self;  /* DEVICE [t_q][n_kv_heads][head_dim] */
    void* out;           /* DEVICE [t_q][n_q_heads][head_dim] */
    int64_t n_ctx;
    int64_t q_pos0;
    int32_t t_q;
    int32_t cache_index;
} adapshot_attn_item;
adapshot_status adapshot_query_attn_batched(adapshot_ctx* ctx, const adapshot_cache* caches, int32_t n_caches,
                                            int32_t layer, const adapshot_attn_item* items, int32_t n_items,
                                            void* hip_stream);

/* Zero-copy form of adapshot_query_attn_batched: the items' contexts are prefixes of n_lists shot lists, read
 * where the shots lie in the pool (no assembled cache; keys re-encoded inside the attention kernel by the
 * composition property of Position Decoupling and Re-encoding, as in adapshot_query_attn_pool).  List l is
 * shot_ids[l][orders[l][j]], j = 0..m[l]-1, its first token at position pos0 (shot_ids / orders / m: HOST arrays
 * of n_lists entries; orders, or any orders[l], may be NULL).  An item's cache_index names its list and its
 * n_ctx is a token count, at most the list's length: the probes of one query over nested prefixes of its ranked
 * list (Probe-based Dynamic Evaluation) are items of one list, and no shot is copied for a prefix that the stopping
 * rule then rejects.  Out[i] is what adapshot_query_attn_batched gives over caches assembled from the same lists
 * (same kernels' arithmetic; parity bar of adapshot_query_attn).  Three launches (two when the lists equal
 * the previous call's: the plan is kept for the next layer): the plan of all lists, the attention grid over
 * all items, the merge of the partials (bf16 models with head_dim 128, for which a pool layer
 * must stay below 4 GiB, ECAPACITY; other shapes run item by item).  Pools registered with ADAPSHOT_KEYS_UNROTATED
 * only (ESTATE otherwise). */
adapshot_status adapshot_query_attn_pool_batched(adapshot_ctx* ctx, int32_t layer, const int32_t* const* shot_ids,
                                                 const int32_t* const* orders, const int32_t* m, int32_t n_lists,
                                                 int64_t pos0, const adapshot_attn_item* items, int32_t n_items,
                                                 void* hip_stream);

/* Decode step (final answer generation after the shot count is chosen): append ONE new token to each
 * cache.  k_new, v_new: DEVICE [n_layers][n_caches][n_kv_heads][head_dim], keys WITHOUT rotation (as the
 * model produces them before RoPE, whatever desc.key_state says about the pool).  Token b lands in slot
 * caches[b].len, its key rotated to position pos0 + caches[b].len (Eq. rope_encoding); slot_shot gets -1.
 * On success every caches[b].len is advanced by one.  Errors: ECAPACITY if any cache is full. */
adapshot_status adapshot_decode_append(adapshot_ctx* ctx, adapshot_cache* caches, int32_t n_caches,
                                       const void* k_new, const void* v_new, int64_t pos0, void* hip_stream);

/* Entropy of softmax(logits) per row, natural log (step 4; Eq. entropy taken over
 * the whole output vocabulary).  logits: DEVICE fp32, row r at logits + r*row_stride
 * (row_stride >= vocab, in elements); entropy_out: DEVICE fp32[n_rows].  A logit of
 * -inf contributes 0; a row with a NaN, a +inf or no finite logit gives NaN. */
adapshot_status adapshot_probe_entropy(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                       int32_t n_rows, int32_t vocab, float* entropy_out,
                                       void* hip_stream);

/* adapshot_probe_entropy for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results; the
 * chunk partials go to a 768 KiB array that lives in the library's code object on every GPU it runs on
 * (held until the process ends) instead of a workspace of the context, and nothing is allocated, freed or
 * waited for, on the host or the device.  The array holds 65536 partials, one per (row, chunk of a row);
 * rows are cut into chunks of 8192 logits, or of 4096, 2048 or 1024 while that leaves fewer than four
 * workgroups per compute unit, so e.g. 128 x 128256 logits need 2048 partials and 4096 x 128256 need 65536.
 * A call that needs more returns ECAPACITY and launches nothing; ESTATE if the context's device is not the
 * current one.  All contexts of a process share one GPU's array: calls that overlap on the same GPU (two
 * streams, two contexts) race and must be ordered by the caller; calls in one stream are ordered already.
 * The launches of this entry point are not recorded by adapshot_profile_enable. */
adapshot_status adapshot_probe_entropy_static(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                              int32_t n_rows, int32_t vocab, float* entropy_out,
                                              void* hip_stream);

/* Eq. (entropy) as printed: H = -sum_{c in C} p_c ln p_c over a set C of answer tokens (the probe's
 * "Yes" / "No").  Two readings of p are offered, because the case study prints entropies above ln 2:
 *   ADAPSHOT_ENTROPY_FULL_P        p_c is token c's probability under the softmax over the whole
 *                                  vocabulary (the other tokens' terms are left out; at most |C|/e);
 *   ADAPSHOT_ENTROPY_RENORMALISED  p is renormalised over C (at most ln |C|).
 * token_ids: HOST, n_tokens distinct indices in [0, vocab), 1 <= n_tokens <= 16.  logits and entropy_out
 * as in adapshot_probe_entropy.  A term with p_c = 0 contributes 0; a row with a NaN, a +inf or no
 * finite logit gives NaN, and so does, in the renormalised reading, a row whose C-logits are all -inf. */
typedef enum { ADAPSHOT_ENTROPY_FULL_P = 0, ADAPSHOT_ENTROPY_RENORMALISED = 1 } adapshot_entropy_mode;
adapshot_status adapshot_probe_entropy_tokens(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                              int32_t n_rows, int32_t vocab, const int32_t* token_ids,
                                              int32_t n_tokens, int32_t mode, float* entropy_out,
                                              void* hip_stream);

/* Relevance of every shot of the pool to a query (Attention-based retrieval, Eq. attention_score): the
 * query attends to the cached keys of ALL pool tokens at one representative layer, and a shot's score is
 * the attention it receives averaged over heads, query tokens and the shot's tokens,
 *     s_i = 1 / (t_q * n_q_heads * T_i) * sum_{j, h} sum_{u in shot i} A_h[j, u].
 * The softmax runs over the whole pool (read inside one shot only, as printed, every row sums to 1 and
 * the average is 1 / T_i whatever the content).  Keys are taken as a cache holds them: encoded at their
 * position inside the shot (Eq. prefill); for a pool registered with ADAPSHOT_KEYS_UNROTATED the library
 * builds that encoding of the layer once and keeps it, together with one more layer-sized buffer, until
 * another layer is ranked, the pool is registered again or the context is destroyed.  The kept state is
 * tied to the registration, not to the bytes: after rewriting pool contents in place, call
 * adapshot_pool_register again before ranking.  The query is encoded on its own: token j at position
 * q_pos0 + j.  The reduction order is fixed: the same inputs give bit-identical scores.
 * q: DEVICE [t_q][n_q_heads][head_dim] without rotation; scores_out: DEVICE fp32 [n_shots].
 * Every shot must hold at least one token.  bf16 models with head_dim 128 run the matrix-core attention kernel
 * over the pool (a pool layer must stay below 4 GiB, ECAPACITY); other shapes run a plain kernel (one wavefront
 * per query token and head over the whole layer: for small models and checks, not tuned), head_dim <= 1024. */
adapshot_status adapshot_rank_shots(adapshot_ctx* ctx, int32_t layer, const void* q, int32_t t_q, int64_t q_pos0,
                                    float* scores_out, void* hip_stream);

/* The k most relevant shots, best first; equal scores keep the lower shot id first.  scores: HOST
 * fp32 [n_shots] (a NaN is EINVAL), shot_ids_out: HOST int32 [k].  Host logic, nothing is launched;
 * ctx may be NULL.  The result is what adapshot_assemble takes as shot_ids (with order = NULL). */
adapshot_status adapshot_top_k(adapshot_ctx* ctx, const float* scores, int32_t n_shots, int32_t k,
                               int32_t* shot_ids_out);

/* Stopping rule of the probe iteration (Probe-based Dynamic Evaluation): candidate i activates
 * shot_counts[i] shots and its probe gave entropy[i]; it passes when entropy[i] <= tau.  *picked receives
 * the smallest passing shot count, or -1 when no candidate passes (probe larger counts next).  A NaN
 * entropy never passes.  Host arrays, host logic: nothing is launched.  ctx may be NULL. */
adapshot_status adapshot_pick_shots(adapshot_ctx* ctx, const float* entropy, const int32_t* shot_counts,
                                    int32_t n_candidates, float tau, int32_t* picked);

/* Test and tuning aid (not a step of the method): fixes the number of context splits the attention
 * planner cuts a context into (1..64; 0 gives the choice back to the planner, which sizes the splits to
 * the compute units).  A batched call gives the longest item that many splits and every other item the
 * same split length.  The result of the attention does not depend on the split count beyond the
 * summation order of the partials. */
adapshot_status adapshot_set_attn_splits(adapshot_ctx* ctx, int32_t n_split);

/* The split plan adapshot_query_attn uses for t_q query tokens over n_ctx context slots on a GPU with
 * n_compute_units compute units (host logic, nothing is launched, no GPU needed): the context is cut into
 * *n_split pieces of *keys_per_split slots (a multiple of 64; the last piece may be shorter; an empty context
 * has no piece), and the query's own tokens form one more.  EINVAL on a bad description or argument. */
adapshot_status adapshot_attn_split_plan(const adapshot_model_desc* desc, int32_t n_compute_units, int32_t t_q,
                                         int64_t n_ctx, int32_t* n_split, int64_t* keys_per_split);

/* Measurement aid (not a step of the method).  While enabled, every kernel the context
 * launches carries a pair of HIP events attached to its dispatch on the launch stream, whose
 * difference is the kernel's own execution time (events recorded before and after a launch
 * would add about 2.5 us of command-processor round trips).  adapshot_profile_read waits for
 * the recorded launches of one kernel kind, returns their summed duration in milliseconds
 * and their count, and forgets them.  Whole-path throughput is measured with profiling off. */
typedef enum {
    ADAPSHOT_KERNEL_ASSEMBLE = 0,       /* fused gather + re-encode */
    ADAPSHOT_KERNEL_ROPE_ROWS = 1,      /* rotation of the query rows and their own keys */
    ADAPSHOT_KERNEL_ATTN = 2,           /* split-K attention proper */
    ADAPSHOT_KERNEL_ATTN_COMBINE = 3,   /* merge of the split partials */
    ADAPSHOT_KERNEL_ENTROPY_CHUNK = 4,  /* vocabulary pass */
    ADAPSHOT_KERNEL_ENTROPY_FINISH = 5, /* merge of the chunk partials */
    ADAPSHOT_KERNEL_KINDS = 6
} adapshot_kernel_kind;
adapshot_status adapshot_profile_enable(adapshot_ctx* ctx, int32_t enable);
adapshot_status adapshot_profile_read(adapshot_ctx* ctx, int32_t kind, double* total_ms, int64_t* launches);
/* The same, every launch on its own: the first min(*launches, capacity) durations in milliseconds, in launch
 * order, go to ms_out (HOST); *launches is the number recorded, all of which are forgotten. */
adapshot_status adapshot_profile_read_each(adapshot_ctx* ctx, int32_t kind, float* ms_out, int64_t capacity,
                                           int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* ADAPSHOT_H_ */
