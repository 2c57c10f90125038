// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "adapshot.h"

namespace adapshot {

// ---- RoPE tables --------------------------------------------------------------
// Angle multiplier a (a position or a position offset) is split as a = 64*hi + lo.
// tab_hi[hi][i] = (cos, sin)(64*hi*theta_i), tab_lo[lo][i] = (cos, sin)(lo*theta_i),
// both evaluated in fp64 and rounded once to fp32.  cos/sin(a*theta_i) follows by one
// angle addition in fp32 (error ~3e-7 absolute), see Eq. (rope_compensation).
constexpr int kRopeLoBits = 6;
constexpr int kRopeLo = 1 << kRopeLoBits;

// ---- assemble tiles -------------------------------------------------------------
// One tile = up to kTileTok consecutive tokens of ONE shot: contiguous in the pool
// and contiguous in the cache.  Angle of token tau in the tile: angle0 + tau*angle_step.
// A launch serves up to kAssembleBatch caches: a tile names its cache, and the caches'
// buffers travel in the kernel arguments.
constexpr int kTileTok = 32;
struct TileDesc {
    int32_t src_tok;     // first pool token (index inside a layer)
    int32_t dst_slot;    // first cache slot; the token's new position is the cache's pos0 + slot
    int32_t angle0;      // angle multiplier of the first token
    int32_t n_tok;       // 1..kTileTok
    int32_t angle_step;  // 1: keys un-rotated (angle = position); 0: rotated at local positions (angle = shot offset)
    int32_t shot;        // pool shot id
    int32_t tok0;        // index of the first token inside its shot
    int32_t cache;       // index into AssembleParams::dst
};
static_assert(sizeof(TileDesc) == 32, "TileDesc is read as two 16-byte words");

constexpr int kAssembleBatch = 48;
struct AssembleDst {  // one cache of the launch
    char* k_out;
    char* v_out;
    int32_t* slot_shot;
    int32_t* slot_tok;
    int64_t* slot_pos;
    int64_t layer_stride_bytes;
    int64_t pos0;
};

struct AssembleParams {
    const char* k_pool;
    const char* v_pool;
    const TileDesc* tiles;  // pinned host memory, read by the kernel
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t pool_layer_stride_bytes;
    int64_t n_tokens;      // tokens of all tiles together
    int32_t n_tiles;
    int32_t n_layers;
    int32_t n_dst;         // caches of this launch (entries of dst in use)
    int32_t wg_tok;        // tokens of a tile per workgroup: a power of two <= kTileTok (kTileTok / wg_tok workgroups per tile;
                           // kTileTok: the host has cut the shots into one-workgroup tiles already)
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;
    AssembleDst dst[kAssembleBatch];
};
hipError_t launch_assemble(const AssembleParams& p, hipStream_t stream);

// One decode step: cache i of this launch receives token row [layer][first + i] of k_new / v_new at
// slot[i], the key rotated to pos[i].  Pointer tables travel in the kernel arguments.
constexpr int kDecodeBatch = 32;
struct DecodeAppendParams {
    const char* k_new;  // [n_layers][n_total][h_kv][d], un-rotated
    const char* v_new;
    const float2* tab_lo;
    const float2* tab_hi;
    char* k_out[kDecodeBatch];
    char* v_out[kDecodeBatch];
    int32_t* slot_shot[kDecodeBatch];
    int32_t* slot_tok[kDecodeBatch];
    int64_t* slot_pos[kDecodeBatch];
    int32_t capacity[kDecodeBatch];
    int32_t slot[kDecodeBatch];
    int32_t pos[kDecodeBatch];
    int32_t n_layers, n_kv_heads, head_dim, dtype;
    int32_t n_total, first, count;
};
hipError_t launch_decode_append(const DecodeAppendParams& p, hipStream_t stream);

// ---- attention --------------------------------------------------------------------
struct RopeRowsParams {
    const void* q;       // [t_q][h_q][d]
    const void* k_self;  // [t_q][h_kv][d]
    void* q_rot;         // [t_q][h_q][d], scaled by log2(e)/sqrt(d)
    void* k_rot;         // [t_q][h_kv][d]
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t q_pos0;
    int32_t t_q, n_q_heads, n_kv_heads, head_dim, dtype;
    float q_scale;
};
hipError_t launch_rope_rows(const RopeRowsParams& p, hipStream_t stream);

// Split plan: splits 0..n_split-1 cover context keys [s*keys_per_split, ...) and
// split n_split is the causal self part.  Partials are indexed [split][kv head][row]
// with row = j*g + (h % g).
// What only the MFMA kernel's prologue (and its zero-copy form) reads.  Kept apart from AttnParams so that none
// of it occupies scalar registers during the key loop.
struct AttnFold {
    // The kernel rotates the rows it needs itself (Eq. rope_encoding at position q_pos0 + j), the query rows
    // scaled by q_scale = log2(e)/sqrt(d) on the way into its fragments, the query's own keys on the way into LDS.
    const void* q_raw;       // [t_q][h_q][d] as the caller gave it
    const void* k_self_raw;  // [t_q][h_kv][d] as the caller gave it
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t q_pos0;
    float q_scale;
    int32_t pool_tokens;  // zero-copy form: tokens in a pool layer (gathered rows are clamped to it)
    // Zero-copy form (template parameter POOL): k_cache / v_cache are the POOL's layer, context slot u holds pool
    // token slot_src[u], and its key is rotated to position pos0 + u inside the key loop;
    // tile_rot[i][f] = (cos, sin)((pos0 + 64 i) theta_f) for every 64-slot tile of the context.  slot_src is 16-byte
    // aligned and readable for 256 entries past the context's last slot (the kernel fetches it 1 KB at a time).
    const int32_t* slot_src;
    const float2* tile_rot;
};

struct AttnParams {
    const void* k_cache;  // one layer [>=n_ctx][h_kv][d]
    const void* v_cache;
    const void* q_rot;       // generic kernel: rows rotated and scaled by rope_rows
    const void* k_self_rot;  // generic kernel: the query's own keys rotated by rope_rows
    const void* v_self;
    // Partials, indexed [n_split+1][h_kv][rows]: part_mlf = (reference maximum in log2 units, row sum l,
    // factor f, unused) and a row O' of d values with  sum_k p_k v_k = f * O'.
    //   part_half = 0: O' is the unnormalised fp32 accumulator, f = 1 (generic kernel);
    //   part_half = 1: O' = accumulator / (l * a) in fp16 with a = the largest |accumulator| / l of the row,
    //                  so |O'| <= 1 whatever the range of V, and f = l * a (MFMA kernel): half the bytes,
    //                  error per element <= 2^-11 of the row's largest partial output.
    void* part_o;
    float4* part_mlf;
    int32_t part_half;
    // Ranking over the pool (MFMA kernel only): context splits with explicit key bounds
    // [split_bounds[s], split_bounds[s+1]) instead of equal lengths, and no self part.
    int32_t no_self;
    int32_t v_blocks;  // 32-column blocks of a V row that carry data: 4, or 1 when every window holds <= 32 shots
    const int64_t* split_bounds;
    void* out;       // [t_q][h_q][d]
    int64_t n_ctx;
    int64_t keys_per_split;
    int32_t n_split;
    int32_t t_q, n_q_heads, n_kv_heads, head_dim, dtype;
    // Batched launches only: k_cache / v_cache point at layer 0 of the item's context and the launch names the
    // layer, so that the tables of a batch serve every layer of a model (0 for single calls).
    int64_t layer_stride_bytes;
};
constexpr int kAttnRowTile = 256;  // query rows per workgroup of the MFMA kernel
// With at most this many rows per kv head half of a workgroup's wavefronts only move tiles and the launch is bound
// by the memory path, not by the matrix cores: its tile loads are then marked non-temporal (when no other workgroup
// reads the same tiles).
constexpr int kAttnStreamRows = 128;
struct GenericPool {  // zero-copy form of the generic kernel; slot_src == nullptr: the context is an assembled cache
    const int32_t* slot_src;
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t pos0;  // position of context slot 0
};
hipError_t launch_attn_generic(const AttnParams& p, const GenericPool& pool, hipStream_t stream);
hipError_t launch_attn_mfma(const AttnParams& p, const AttnFold& f, hipStream_t stream);
hipError_t launch_attn_mfma_pool(const AttnParams& p, const AttnFold& f, hipStream_t stream);  // zero-copy form
// Expands the per-shot segments of a zero-copy context into slot_src and builds tile_rot.
struct PoolSeg {
    int32_t slot0, src_tok0, len, pad;
};
struct PoolPlanParams {
    const PoolSeg* segs;  // pinned host memory, read by the kernel
    int32_t* slot_src;
    float2* tile_rot;
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t pos0;
    int32_t n_segs, n_tiles, head_dim;
};
hipError_t launch_pool_plan(const PoolPlanParams& p, hipStream_t stream);
bool attn_mfma_supported(const adapshot_model_desc& d);
hipError_t launch_attn_combine(const AttnParams& p, hipStream_t stream);

// ---- a batch of attention problems in two launches (attend, combine) ------------------------
// The tables live in device memory for the duration of the launches; every workgroup reads its own
// entry.  The probes of one query over nested prefixes of one cache, the queries of a decode step and
// the queries of a probe sweep are all such batches (Probe-based Dynamic Evaluation).
struct AttnBatchItem {
    AttnParams attn;
    AttnFold fold;
};
struct AttnWork {  // one workgroup of the batched MFMA kernel
    int32_t item, hk, row_tile, split;
};
struct CombineWork {  // one workgroup of the batched combine kernel: 16 (kv head, row) pairs from pair0 on (fp16 partials)
    int32_t item, pair0;
};
// Tables written by the host into pinned memory are brought to device memory by a kernel (a DMA copy
// between two kernels of a stream costs more than the copy itself).  bytes is a multiple of 16.
hipError_t launch_copy_table(void* dst, const void* src_pinned, size_t bytes, hipStream_t stream);
// stream_tiles: no two items read the same context and none has more than kAttnStreamRows rows per kv head
hipError_t launch_attn_mfma_batched(const AttnBatchItem* items, const AttnWork* work, int n_work, bool pool,
                                    bool stream_tiles, int layer, hipStream_t stream);
// max_partials: the most partial rows that any item merges per output row (its context splits + 1)
hipError_t launch_attn_combine_batched(const AttnBatchItem* items, const CombineWork* work, int n_work, int dtype,
                                       int max_partials, hipStream_t stream);

// ---- relevance ranking over the pool (Eq. attention_score) ----------------------------------
// The query attends over the locally encoded keys of ALL pool tokens at one layer with a one-hot "value"
// row per token: column = the token's shot, counted from the first shot of its window of <= head_dim
// consecutive shots.  A context split is one window, so the MFMA kernel's partial of (split, row) holds
// the attention mass of every shot of that window; the two kernels below turn the partials into scores.
struct RankPrepareParams {
    const char* k_pool;      // one layer [tokens][h_kv][d], un-rotated
    char* k_out;             // same layout, every key rotated to its position inside its shot; null: not needed
    char* v_out;             // one-hot rows
    const int32_t* tok_local;  // [tokens] index of the token inside its shot
    const int32_t* tok_col;    // [tokens] shot index inside its window
    const float2* tab_lo;
    const float2* tab_hi;
    int64_t n_tok;
    int32_t n_kv_heads, head_dim;
};
hipError_t launch_rank_prepare(const RankPrepareParams& p, hipStream_t stream);
struct RankReduceParams {
    const void* part_o;       // [n_split][pairs][d] fp16
    const float4* part_mlf;   // [n_split][pairs]
    float* weights;           // [n_split][pairs] scratch
    float* block_part;        // [n_split][ceil(pairs / 256)][128] scratch: per-row-block sums of every shot slot
    float* scores;            // [n_shots]
    const int32_t* split_shot0;  // [n_split + 1] first shot of every window
    const int32_t* shot_split;   // [n_shots] window of every shot
    const float* inv_len;     // [n_shots] 1 / T_i
    float inv_rows;           // 1 / (t_q * n_q_heads)
    int32_t n_split, n_pairs, head_dim, n_shots;
};
hipError_t launch_rank_weights(const RankReduceParams& p, hipStream_t stream);  // merge weights of the windows
hipError_t launch_rank_reduce(const RankReduceParams& p, hipStream_t stream);   // weighted sum over blocks of rows
hipError_t launch_rank_finish(const RankReduceParams& p, hipStream_t stream);   // row blocks added in a fixed order

// Ranking for the shapes the matrix-core kernel does not cover: one wavefront per (query token, head) walks the
// whole pool layer twice (normaliser, then the mass of every shot), a second kernel adds the rows in a fixed order.
struct RankGenericParams {
    const void* k_pool;       // one layer [tokens][h_kv][d]
    const void* q_rot;        // [t_q][h_q][d] rotated to q_pos0 + j, scaled by log2(e)/sqrt(d)
    const int64_t* shot_off;  // DEVICE [n_shots + 1]
    const float2* tab_lo;
    const float2* tab_hi;
    float* mass;              // [t_q * h_q][n_shots] scratch: attention received by every shot from one row
    float* scores;            // [n_shots]
    int32_t n_shots, t_q, n_q_heads, n_kv_heads, head_dim, dtype, key_state;
};
hipError_t launch_rank_generic(const RankGenericParams& p, hipStream_t stream);

// ---- entropy ------------------------------------------------------------------------
struct EntropyParams {
    const float* logits;
    float* out;
    float* partials;  // [n_rows][n_chunks][3] = (max, sum exp, sum (z-max) exp)
    int64_t row_stride;
    int32_t n_rows, vocab, chunk, n_chunks;
};
// The file-scope device array behind adapshot_probe_entropy_static: room for this many (row, chunk) partials.
constexpr int kStaticEntropyPartials = 65536;
// Device address of that array on the CURRENT device (looked up once per device, then remembered).
hipError_t entropy_static_scratch(float** out);
hipError_t launch_entropy_chunk(const EntropyParams& p, hipStream_t stream);
hipError_t launch_entropy_finish(const EntropyParams& p, hipStream_t stream);
// Eq. (entropy) over a set C of answer tokens, from the same vocabulary-wide partials.
constexpr int kMaxAnswerTokens = 16;
struct AnswerTokens {
    int32_t n;
    int32_t mode;  // ADAPSHOT_ENTROPY_FULL_P / ADAPSHOT_ENTROPY_RENORMALISED
    int32_t id[kMaxAnswerTokens];
};
hipError_t launch_entropy_finish_tokens(const EntropyParams& p, const AnswerTokens& c, hipStream_t stream);
// Whole rows in one launch (one workgroup per row); c == nullptr: the vocabulary-wide entropy.
hipError_t launch_entropy_rows(const EntropyParams& p, const AnswerTokens* c, hipStream_t stream);

// ---- host-side helpers -----------------------------------------------------------------
struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
    hipError_t reserve(size_t need, std::vector<void*>& retired);  // grow-only; an outgrown buffer is parked in `retired`
    void release();
};

struct PinnedRing {
    static constexpr int kSlots = 8;
    void* host[kSlots] = {};
    size_t bytes[kSlots] = {};
    hipEvent_t ev[kSlots] = {};
    bool pending[kSlots] = {};
    int next = 0;
    // Returns a pinned buffer of at least `need` bytes that no enqueued kernel still reads.
    hipError_t acquire(size_t need, int* slot, void** ptr);
    hipError_t mark_in_use(int slot, hipStream_t stream);
    void release();
};

// Timing events of the launch in progress.  When set, launch_kernel attaches them to the dispatch itself
// (hipExtLaunchKernelGGL): their difference is then the kernel's own execution time as its completion
// signal records it, without the two command-processor round trips that events recorded around a launch
// add (about 2.5 us on this part).  One dispatch consumes the pair.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local LaunchEvents g_launch_events;

template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream, Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    if (g_launch_events.start) {
        const LaunchEvents ev = g_launch_events;
        g_launch_events = LaunchEvents{};
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, ev.start, ev.stop, 0, static_cast<KArgs>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, static_cast<KArgs>(args)...);
    }
}

// Optional per-kernel timing with HIP events on the launch stream (measurement aid).
struct Profiler {
    struct Rec {
        int kind;
        hipEvent_t start, stop;
    };
    bool on = false;
    std::vector<Rec> recs;
    std::vector<hipEvent_t> free_events;
    hipError_t begin(int kind, hipStream_t stream);
    hipError_t end(hipStream_t stream);
    void release();
};

}  // namespace adapshot

struct adapshot_ctx {
    adapshot_model_desc desc;
    int device = -1;
    int elem_bytes = 0;
    int64_t row_bytes = 0;  // n_kv_heads * head_dim * elem_bytes
    int64_t max_position = 0;
    // pool
    const void* k_pool = nullptr;
    const void* v_pool = nullptr;
    std::vector<int64_t> shot_offsets;
    int64_t pool_layer_stride_tokens = 0;
    int32_t n_shots = 0;
    // tables
    float2* tab_lo = nullptr;
    float2* tab_hi = nullptr;
    float* static_ent = nullptr;  // this device's copy of the static entropy scratch array (not owned)
    // scratch
    adapshot::PinnedRing tile_ring;
    adapshot::DevBuf q_rot, k_rot, part_o, part_ml, ent_part, batch_tab, pool_src, pool_rot;
    // What the device-side tables of the last batched attention call (batch_tab) and of the last zero-copy plan
    // (pool_src, pool_rot) were built from: a call with the same inputs -- the next layer of the same batch --
    // reuses them instead of planning and uploading again.  Empty = nothing to reuse.
    std::vector<unsigned char> batch_key, pool_key;
    int64_t batch_n_attn = 0, batch_n_comb = 0;
    int32_t batch_max_partials = 0;
    size_t batch_attn_off = 0, batch_comb_off = 0;
    // ranking state of one pool layer, built on first use
    int32_t rank_layer = -1;
    int32_t rank_n_split = 0;
    adapshot::DevBuf rank_k, rank_v, rank_tab, rank_w, rank_part;
    const int32_t* rank_tok = nullptr;       // views into rank_tab
    const int64_t* rank_bounds = nullptr;
    const int32_t* rank_shot0 = nullptr;
    const int32_t* rank_shot_split = nullptr;
    const float* rank_inv_len = nullptr;
    std::vector<void*> retired;  // outgrown workspaces, freed when the context is destroyed
    adapshot::Profiler prof;
    int n_cu = 256;
    int32_t assemble_wg_tok = adapshot::kTileTok;  // tokens of a tile per assemble workgroup
    int32_t force_splits = 0;  // adapshot_set_attn_splits: 0 = the planner chooses
    int32_t entropy_rows_min = 256;  // from this many rows on, probe entropy runs one workgroup per row in one launch
    std::string last_error;
};
