// Host side of libadapshot: contexts, argument validation, the integer plan
// (prefix sums -> tile descriptors) and kernel launches.  No device code here.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "adapshot_internal.h"

using namespace adapshot;

namespace adapshot {

thread_local LaunchEvents g_launch_events;

// Grow-only.  A buffer that is too small is not freed here: kernels already enqueued (on any stream) may
// still use it, and hipFree would stall the whole device.  It is parked in `retired` until the context is
// destroyed; the new one is at least half as large again as the old, so the parked memory stays below
// twice the final size.  Contents are not carried over: every workspace is rewritten by the call that
// reserves it.
hipError_t DevBuf::reserve(size_t need, std::vector<void*>& retired) {
    if (need <= bytes) return hipSuccess;
    size_t want = std::max(std::max(need, bytes + bytes / 2), (size_t)1 << 16);
    want = (want + 255) & ~(size_t)255;
    void* fresh = nullptr;
    hipError_t e = hipMalloc(&fresh, want);
    if (e != hipSuccess) return e;
    if (p) retired.push_back(p);
    p = fresh;
    bytes = want;
    return hipSuccess;
}

void DevBuf::release() {
    if (p) (void)hipFree(p);
    p = nullptr;
    bytes = 0;
}

hipError_t PinnedRing::acquire(size_t need, int* slot, void** ptr) {
    int s = next;
    next = (next + 1) % kSlots;
    if (pending[s]) {
        hipError_t e = hipEventSynchronize(ev[s]);
        if (e != hipSuccess) return e;
        pending[s] = false;
    }
    if (bytes[s] < need) {
        if (host[s]) (void)hipHostFree(host[s]);
        host[s] = nullptr;
        bytes[s] = 0;
        size_t want = std::max(need, (size_t)1 << 16);
        hipError_t e = hipHostMalloc(&host[s], want, hipHostMallocDefault);
        if (e != hipSuccess) {
            host[s] = nullptr;
            return e;
        }
        bytes[s] = want;
    }
    if (!ev[s]) {
        hipError_t e = hipEventCreateWithFlags(&ev[s], hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    *slot = s;
    *ptr = host[s];
    return hipSuccess;
}

hipError_t PinnedRing::mark_in_use(int slot, hipStream_t stream) {
    hipError_t e = hipEventRecord(ev[slot], stream);
    if (e == hipSuccess) pending[slot] = true;
    return e;
}

void PinnedRing::release() {
    for (int s = 0; s < kSlots; ++s) {
        if (pending[s] && ev[s]) (void)hipEventSynchronize(ev[s]);
        if (ev[s]) (void)hipEventDestroy(ev[s]);
        if (host[s]) (void)hipHostFree(host[s]);
        ev[s] = nullptr;
        host[s] = nullptr;
        bytes[s] = 0;
        pending[s] = false;
    }
}

hipError_t Profiler::begin(int kind, hipStream_t stream) {
    if (!on) return hipSuccess;
    Rec r;
    r.kind = kind;
    hipEvent_t* ev[2] = {&r.start, &r.stop};
    for (auto e : ev) {
        if (!free_events.empty()) {
            *e = free_events.back();
            free_events.pop_back();
        } else {
            hipError_t err = hipEventCreate(e);
            if (err != hipSuccess) return err;
        }
    }
    recs.push_back(r);
    g_launch_events.start = r.start;  // the next launch_kernel on this thread attaches the pair to its dispatch
    g_launch_events.stop = r.stop;
    (void)stream;
    return hipSuccess;
}

hipError_t Profiler::end(hipStream_t stream) {
    if (!on || recs.empty()) return hipSuccess;
    if (!g_launch_events.start) return hipSuccess;  // consumed by the launch
    // nothing was launched (an empty problem): record the pair around nothing so that it can be read back
    g_launch_events = LaunchEvents{};
    hipError_t e = hipEventRecord(recs.back().start, stream);
    if (e != hipSuccess) return e;
    return hipEventRecord(recs.back().stop, stream);
}

void Profiler::release() {
    for (auto& r : recs) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (auto e : free_events) (void)hipEventDestroy(e);
    recs.clear();
    free_events.clear();
}

}  // namespace adapshot

// Launch exactly one kernel; when profiling is on its dispatch carries a pair of timing events.
template <typename F>
static hipError_t timed_launch(adapshot_ctx* ctx, int kind, hipStream_t stream, F&& launch) {
    hipError_t e = ctx->prof.begin(kind, stream);
    if (e != hipSuccess) return e;
    e = launch();
    if (e != hipSuccess) {
        g_launch_events = LaunchEvents{};  // a launch that failed before its dispatch leaves no pair behind
        return e;
    }
    return ctx->prof.end(stream);
}

static adapshot_status fail(adapshot_ctx* ctx, adapshot_status st, const char* fmt, ...) {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->last_error = buf;
    }
    return st;
}

static adapshot_status fail_hip(adapshot_ctx* ctx, const char* what, hipError_t e) {
    (void)hipGetLastError();  // clear the sticky error so that it is not reported twice
    return fail(ctx, ADAPSHOT_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

extern "C" const char* adapshot_version(void) { return "libadapshot 0.1 (gfx950)"; }

extern "C" const char* adapshot_last_error(const adapshot_ctx* ctx) {
    return ctx ? ctx->last_error.c_str() : "null context";
}

// Validation of a model description; no device access.
static const char* check_desc(const adapshot_model_desc& d) {
    if (d.n_layers < 1 || d.n_layers > 65535) return "n_layers must be in [1, 65535]";
    if (d.n_kv_heads < 1 || d.n_q_heads < 1) return "head counts must be >= 1";
    if (d.n_q_heads % d.n_kv_heads != 0) return "n_q_heads must be a multiple of n_kv_heads";
    if (d.dtype != ADAPSHOT_F32 && d.dtype != ADAPSHOT_BF16) return "dtype must be ADAPSHOT_F32 or ADAPSHOT_BF16";
    if (d.key_state != ADAPSHOT_KEYS_UNROTATED && d.key_state != ADAPSHOT_KEYS_ROTATED_LOCAL)
        return "key_state must be ADAPSHOT_KEYS_UNROTATED or ADAPSHOT_KEYS_ROTATED_LOCAL";
    if (d.head_dim < 2 || d.head_dim % 2 != 0 || d.head_dim > 256) return "head_dim must be even and in [2, 256]";
    int e = d.dtype == ADAPSHOT_F32 ? 4 : 2;
    int half_bytes = d.head_dim / 2 * e;
    if (half_bytes % 16 != 0) return "head_dim * sizeof(element) must be a multiple of 32 bytes";
    int ch = half_bytes / 16;
    if (ch != 1 && ch != 2 && ch != 4 && ch != 8 && ch != 16) return "head_dim/2 must span 1, 2, 4, 8 or 16 16-byte chunks";
    if (!(d.rope_theta > 1.0) || !isfinite(d.rope_theta)) return "rope_theta must be finite and > 1";
    if (d.max_position < 0 || d.max_position > ((int64_t)1 << 30)) return "max_position must be in [0, 2^30]";
    return nullptr;
}

extern "C" adapshot_status adapshot_create(const adapshot_model_desc* desc, adapshot_ctx** out) {
    if (out) *out = nullptr;
    if (!desc || !out) return ADAPSHOT_EINVAL;
    if (check_desc(*desc)) return ADAPSHOT_EINVAL;
    adapshot_ctx* ctx = new (std::nothrow) adapshot_ctx();
    if (!ctx) return ADAPSHOT_EDEVICE;
    ctx->desc = *desc;
    ctx->elem_bytes = desc->dtype == ADAPSHOT_F32 ? 4 : 2;
    ctx->row_bytes = (int64_t)desc->n_kv_heads * desc->head_dim * ctx->elem_bytes;
    ctx->max_position = desc->max_position ? desc->max_position : ((int64_t)1 << 20);
    ctx->desc.max_position = ctx->max_position;
    // tokens of a tile per assemble workgroup: about 16 KB per layer and operand
    int wg_tok = kTileTok;
    while (wg_tok > 1 && (int64_t)wg_tok * ctx->row_bytes > 16384) wg_tok /= 2;
    ctx->assemble_wg_tok = wg_tok;

    hipError_t e = hipGetDevice(&ctx->device);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        delete ctx;
        return ADAPSHOT_EDEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, ctx->device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->n_cu = prop.multiProcessorCount;
    // One workgroup per row keeps the memory system busy once there are as many rows as compute units (256 rows of
    // 128256 logits: 24.4 us in one launch against 26.3 us for chunks + merge; 4096 rows: 303 against 318 us, 6.9 TB/s;
    // 128 rows: 16.5 against 16.1 us, 48 rows: 14.8 against 10.4 us -- a lone workgroup streams ~40 GB/s).
    ctx->entropy_rows_min = ctx->n_cu;

    // RoPE tables in fp64, rounded once to fp32.
    const int half = desc->head_dim / 2;
    const int64_t n_hi = (ctx->max_position + kRopeLo - 1) / kRopeLo + 1;
    std::vector<float2> lo((size_t)kRopeLo * half), hi((size_t)n_hi * half);
    std::vector<double> theta(half);
    for (int i = 0; i < half; ++i) theta[i] = pow(desc->rope_theta, -2.0 * (double)i / (double)desc->head_dim);
    for (int r = 0; r < kRopeLo; ++r)
        for (int i = 0; i < half; ++i) {
            double a = (double)r * theta[i];
            lo[(size_t)r * half + i] = make_float2((float)cos(a), (float)sin(a));
        }
    for (int64_t r = 0; r < n_hi; ++r)
        for (int i = 0; i < half; ++i) {
            double a = (double)(r * kRopeLo) * theta[i];
            hi[(size_t)r * half + i] = make_float2((float)cos(a), (float)sin(a));
        }
    e = hipMalloc((void**)&ctx->tab_lo, lo.size() * sizeof(float2));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->tab_hi, hi.size() * sizeof(float2));
    if (e == hipSuccess) e = hipMemcpy(ctx->tab_lo, lo.data(), lo.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ctx->tab_hi, hi.data(), hi.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = entropy_static_scratch(&ctx->static_ent);  // set-up: the current device is the context's
    if (e != hipSuccess) {
        (void)hipGetLastError();
        adapshot_destroy(ctx);
        return ADAPSHOT_EDEVICE;
    }
    *out = ctx;
    return ADAPSHOT_OK;
}

extern "C" void adapshot_destroy(adapshot_ctx* ctx) {
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    ctx->prof.release();
    ctx->tile_ring.release();
    ctx->q_rot.release();
    ctx->k_rot.release();
    ctx->part_o.release();
    ctx->part_ml.release();
    ctx->ent_part.release();
    ctx->batch_tab.release();
    ctx->pool_src.release();
    ctx->pool_rot.release();
    ctx->rank_k.release();
    ctx->rank_v.release();
    ctx->rank_w.release();
    ctx->rank_part.release();
    ctx->rank_tab.release();
    for (void* q : ctx->retired) (void)hipFree(q);
    ctx->retired.clear();
    if (ctx->tab_lo) (void)hipFree(ctx->tab_lo);
    if (ctx->tab_hi) (void)hipFree(ctx->tab_hi);
    delete ctx;
}

extern "C" adapshot_status adapshot_pool_register(adapshot_ctx* ctx, const void* k_pool, const void* v_pool,
                                                  const int64_t* shot_offsets, int32_t n_shots,
                                                  int64_t layer_stride_tokens) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (!k_pool || !v_pool || !shot_offsets) return fail(ctx, ADAPSHOT_EINVAL, "pool_register: null pointer");
    if (n_shots < 0) return fail(ctx, ADAPSHOT_EINVAL, "pool_register: n_shots < 0");
    if (!aligned16(k_pool) || !aligned16(v_pool))
        return fail(ctx, ADAPSHOT_EINVAL, "pool_register: pool pointers must be 16-byte aligned");
    if (shot_offsets[0] < 0) return fail(ctx, ADAPSHOT_EINVAL, "pool_register: shot_offsets[0] < 0");
    for (int32_t i = 0; i < n_shots; ++i)
        if (shot_offsets[i + 1] < shot_offsets[i])
            return fail(ctx, ADAPSHOT_EINVAL, "pool_register: shot_offsets decreases at %d", i);
    if (shot_offsets[n_shots] > layer_stride_tokens)
        return fail(ctx, ADAPSHOT_EINVAL, "pool_register: layer_stride_tokens %lld < pool tokens %lld",
                    (long long)layer_stride_tokens, (long long)shot_offsets[n_shots]);
    if (layer_stride_tokens > INT32_MAX)
        return fail(ctx, ADAPSHOT_EINVAL, "pool_register: more than 2^31-1 tokens per layer");
    ctx->k_pool = k_pool;
    ctx->v_pool = v_pool;
    ctx->shot_offsets.assign(shot_offsets, shot_offsets + n_shots + 1);
    ctx->n_shots = n_shots;
    ctx->pool_layer_stride_tokens = layer_stride_tokens;
    ctx->rank_layer = -1;  // ranking state belongs to the previous pool
    ctx->batch_key.clear();  // so do the tables kept for the next layer of a batch
    ctx->pool_key.clear();
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

// How the shots of an assemble call are cut into tiles.  Few layers: tiles of kTileTok tokens, and the grid gives every
// tile kTileTok / wg_tok workgroups (a shot's last tile leaves some of them empty or nearly so, but the list is
// short: the host plans 49 us per call at the headline size as it is, and a workgroup's first act is to fetch its
// descriptor from host memory).  Many layers: the host cuts the shots into pieces of wg_tok tokens itself, one
// workgroup per piece and layer, what is left over of a shot joined to its last piece when the two fit a tile's
// table -- no empty workgroups and none that runs for a handful of tokens, four times the descriptors, read again by
// every layer's workgroups (28 layers of the decode caches -5 %, 80 layers of the 70B shape -2 %, the sweep's 32
// layers 0 to -14 % from process to process; a single layer +5 %, and its planning would overtake the GPU).
constexpr int kAssemblePieceLayers = 8;
static inline int64_t assemble_unit(const adapshot_ctx* ctx) {
    return ctx->desc.n_layers >= kAssemblePieceLayers ? ctx->assemble_wg_tok : kTileTok;
}
static inline int64_t shot_tiles(int64_t len, int64_t unit) {
    if (len <= 0) return 0;
    const int64_t q = len / unit, r = len - q * unit;
    if (q == 0) return 1;
    return r != 0 && unit + r > kTileTok ? q + 1 : q;
}

// Validation + integer plan totals of one assemble call; nothing is launched or written.
static adapshot_status check_assemble(adapshot_ctx* ctx, const adapshot_cache* cache, const int32_t* shot_ids,
                                      const int32_t* order, int32_t m, int64_t pos0, int64_t* total_out,
                                      int64_t* n_tiles_out) {
    if (!cache) return fail(ctx, ADAPSHOT_EINVAL, "assemble: null cache");
    if (m < 0) return fail(ctx, ADAPSHOT_EINVAL, "assemble: m < 0");
    if (m > 0 && !shot_ids) return fail(ctx, ADAPSHOT_EINVAL, "assemble: null shot_ids");
    if (!ctx->k_pool) return fail(ctx, ADAPSHOT_ESTATE, "assemble: no pool registered");
    if (!cache->k || !cache->v) return fail(ctx, ADAPSHOT_EINVAL, "assemble: null cache buffers");
    if (!aligned16(cache->k) || !aligned16(cache->v))
        return fail(ctx, ADAPSHOT_EINVAL, "assemble: cache pointers must be 16-byte aligned");
    if (cache->capacity < 0 || cache->capacity > INT32_MAX || cache->len < 0 || cache->len > cache->capacity)
        return fail(ctx, ADAPSHOT_EINVAL, "assemble: bad cache capacity/len");
    if (pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "assemble: pos0 < 0");
    int64_t total = 0, n_tiles = 0;
    for (int32_t j = 0; j < m; ++j) {
        int32_t oj = order ? order[j] : j;
        if (oj < 0 || oj >= m) return fail(ctx, ADAPSHOT_ESHOT, "assemble: order[%d] = %d out of range", j, oj);
        int32_t s = shot_ids[oj];
        if (s < 0 || s >= ctx->n_shots) return fail(ctx, ADAPSHOT_ESHOT, "assemble: shot id %d out of range", s);
        int64_t len = ctx->shot_offsets[s + 1] - ctx->shot_offsets[s];
        total += len;
        n_tiles += shot_tiles(len, assemble_unit(ctx));
    }
    if (cache->len + total > cache->capacity)
        return fail(ctx, ADAPSHOT_ECAPACITY, "assemble: %lld + %lld tokens exceed capacity %lld",
                    (long long)cache->len, (long long)total, (long long)cache->capacity);
    if (pos0 + cache->len + total > ctx->max_position)
        return fail(ctx, ADAPSHOT_ECAPACITY, "assemble: position %lld exceeds max_position %lld",
                    (long long)(pos0 + cache->len + total), (long long)ctx->max_position);
    if (n_tiles > INT32_MAX) return fail(ctx, ADAPSHOT_EINVAL, "assemble: too many tiles");
    *total_out = total;
    *n_tiles_out = n_tiles;
    return ADAPSHOT_OK;
}

// One validated assemble job of a batch.
struct AssembleJob {
    adapshot_cache* cache;
    const int32_t* shot_ids;
    const int32_t* order;
    int32_t m;
    int64_t total, n_tiles;
};

// Plan (prefix sums -> tile descriptors) and launch of validated assemble jobs: one launch per group of
// up to kAssembleBatch caches, the tiles of a group's caches in one descriptor list.
static adapshot_status run_assemble(adapshot_ctx* ctx, AssembleJob* jobs, int32_t n_jobs, int64_t pos0,
                                    hipStream_t stream) {
    const bool local = ctx->desc.key_state == ADAPSHOT_KEYS_ROTATED_LOCAL;
    for (int32_t j0 = 0; j0 < n_jobs; j0 += kAssembleBatch) {
        const int32_t j1 = std::min<int32_t>(n_jobs, j0 + kAssembleBatch);
        int64_t group_tiles = 0;
        for (int32_t b = j0; b < j1; ++b) group_tiles += jobs[b].n_tiles;
        if (group_tiles == 0) continue;
        if (group_tiles > INT32_MAX / kTileTok) return fail(ctx, ADAPSHOT_EINVAL, "assemble: too many tiles");
        int slot;
        void* host;
        hipError_t e = ctx->tile_ring.acquire((size_t)group_tiles * sizeof(TileDesc), &slot, &host);
        if (e != hipSuccess) return fail_hip(ctx, "assemble: pinned tile buffer", e);
        TileDesc* tiles = (TileDesc*)host;
        AssembleParams p;
        const int64_t unit = assemble_unit(ctx);
        int64_t nt = 0, n_tok_group = 0;
        for (int32_t b = j0; b < j1; ++b) {
            const AssembleJob& jb = jobs[b];
            AssembleDst& dc = p.dst[b - j0];
            dc.k_out = (char*)jb.cache->k;
            dc.v_out = (char*)jb.cache->v;
            dc.slot_shot = jb.cache->slot_shot;
            dc.slot_tok = jb.cache->slot_tok;
            dc.slot_pos = jb.cache->slot_pos;
            dc.layer_stride_bytes = jb.cache->capacity * ctx->row_bytes;
            dc.pos0 = pos0;
            // slot group j starts at off_j = sum of the lengths before it
            int64_t slot0 = jb.cache->len;
            for (int32_t j = 0; j < jb.m; ++j) {
                const int32_t s = jb.shot_ids[jb.order ? jb.order[j] : j];
                const int64_t src = ctx->shot_offsets[s], len = ctx->shot_offsets[s + 1] - src;
                const int64_t n_here = shot_tiles(len, unit);
                for (int64_t i = 0, t0 = 0; i < n_here; ++i, t0 += unit) {
                    TileDesc& d = tiles[nt++];
                    d.src_tok = (int32_t)(src + t0);
                    d.dst_slot = (int32_t)(slot0 + t0);
                    d.angle0 = (int32_t)(local ? pos0 + slot0 : pos0 + slot0 + t0);
                    d.angle_step = local ? 0 : 1;
                    d.n_tok = (int32_t)(i + 1 == n_here ? len - t0 : unit);  // the last tile takes what is left
                    d.shot = s;
                    d.tok0 = (int32_t)t0;
                    d.cache = b - j0;
                }
                slot0 += len;
                n_tok_group += len;
            }
        }
        for (int32_t i = j1 - j0; i < kAssembleBatch; ++i) p.dst[i] = AssembleDst{};
        p.k_pool = (const char*)ctx->k_pool;
        p.v_pool = (const char*)ctx->v_pool;
        p.tiles = tiles;
        p.tab_lo = ctx->tab_lo;
        p.tab_hi = ctx->tab_hi;
        p.pool_layer_stride_bytes = ctx->pool_layer_stride_tokens * ctx->row_bytes;
        p.n_tiles = (int32_t)nt;
        p.n_tokens = n_tok_group;
        p.n_layers = ctx->desc.n_layers;
        p.n_dst = j1 - j0;
        p.wg_tok = unit == kTileTok ? ctx->assemble_wg_tok : kTileTok;  // pieces cut by the host: one workgroup each
        p.n_kv_heads = ctx->desc.n_kv_heads;
        p.head_dim = ctx->desc.head_dim;
        p.dtype = ctx->desc.dtype;
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ASSEMBLE, stream, [&] { return launch_assemble(p, stream); });
        if (e != hipSuccess) return fail_hip(ctx, "assemble: launch", e);
        e = ctx->tile_ring.mark_in_use(slot, stream);
        if (e != hipSuccess) return fail_hip(ctx, "assemble: event record", e);
        for (int32_t b = j0; b < j1; ++b) jobs[b].cache->len += jobs[b].total;
    }
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_assemble(adapshot_ctx* ctx, adapshot_cache* cache, const int32_t* shot_ids,
                                             const int32_t* order, int32_t m, int64_t pos0, void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    AssembleJob job{cache, shot_ids, order, m, 0, 0};
    adapshot_status st = check_assemble(ctx, cache, shot_ids, order, m, pos0, &job.total, &job.n_tiles);
    if (st != ADAPSHOT_OK) return st;
    st = run_assemble(ctx, &job, 1, pos0, (hipStream_t)hip_stream);
    if (st == ADAPSHOT_OK) ctx->last_error.clear();
    return st;
}

extern "C" adapshot_status adapshot_assemble_batched(adapshot_ctx* ctx, adapshot_cache* caches, int32_t n_caches,
                                                     const int32_t* const* shot_ids, const int32_t* const* orders,
                                                     const int32_t* m, int64_t pos0, void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (n_caches < 0) return fail(ctx, ADAPSHOT_EINVAL, "assemble_batched: n_caches < 0");
    if (n_caches > 0 && (!caches || !shot_ids || !m)) return fail(ctx, ADAPSHOT_EINVAL, "assemble_batched: null pointer");
    std::vector<AssembleJob> jobs((size_t)n_caches);
    for (int32_t b = 0; b < n_caches; ++b) {  // every item is validated before anything is launched
        for (int32_t c = 0; c < b; ++c)
            if (caches[c].k == caches[b].k || caches[c].v == caches[b].v)
                return fail(ctx, ADAPSHOT_EINVAL, "assemble_batched: caches %d and %d share a buffer", c, b);
        jobs[(size_t)b] = AssembleJob{&caches[b], shot_ids[b], orders ? orders[b] : nullptr, m[b], 0, 0};
        adapshot_status st = check_assemble(ctx, &caches[b], shot_ids[b], orders ? orders[b] : nullptr, m[b], pos0,
                                            &jobs[(size_t)b].total, &jobs[(size_t)b].n_tiles);
        if (st != ADAPSHOT_OK) return st;
    }
    adapshot_status st = run_assemble(ctx, jobs.data(), n_caches, pos0, (hipStream_t)hip_stream);
    if (st != ADAPSHOT_OK) return st;
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_decode_append(adapshot_ctx* ctx, adapshot_cache* caches, int32_t n_caches,
                                                  const void* k_new, const void* v_new, int64_t pos0,
                                                  void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (n_caches < 0) return fail(ctx, ADAPSHOT_EINVAL, "decode_append: n_caches < 0");
    if (n_caches == 0) {
        ctx->last_error.clear();
        return ADAPSHOT_OK;
    }
    if (!caches || !k_new || !v_new) return fail(ctx, ADAPSHOT_EINVAL, "decode_append: null pointer");
    if (!aligned16(k_new) || !aligned16(v_new))
        return fail(ctx, ADAPSHOT_EINVAL, "decode_append: k_new / v_new must be 16-byte aligned");
    if (pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "decode_append: pos0 < 0");
    for (int32_t b = 0; b < n_caches; ++b) {
        const adapshot_cache& c = caches[b];
        if (!c.k || !c.v || !aligned16(c.k) || !aligned16(c.v))
            return fail(ctx, ADAPSHOT_EINVAL, "decode_append: cache %d has null or misaligned buffers", b);
        if (c.capacity < 0 || c.capacity > INT32_MAX || c.len < 0 || c.len > c.capacity)
            return fail(ctx, ADAPSHOT_EINVAL, "decode_append: cache %d has bad capacity/len", b);
        if (c.len + 1 > c.capacity) return fail(ctx, ADAPSHOT_ECAPACITY, "decode_append: cache %d is full", b);
        if (pos0 + c.len + 1 > ctx->max_position)
            return fail(ctx, ADAPSHOT_ECAPACITY, "decode_append: position exceeds max_position");
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    for (int32_t b0 = 0; b0 < n_caches; b0 += kDecodeBatch) {
        DecodeAppendParams p;
        p.k_new = (const char*)k_new;
        p.v_new = (const char*)v_new;
        p.tab_lo = ctx->tab_lo;
        p.tab_hi = ctx->tab_hi;
        p.n_layers = ctx->desc.n_layers;
        p.n_kv_heads = ctx->desc.n_kv_heads;
        p.head_dim = ctx->desc.head_dim;
        p.dtype = ctx->desc.dtype;
        p.n_total = n_caches;
        p.first = b0;
        p.count = std::min<int32_t>(kDecodeBatch, n_caches - b0);
        for (int32_t i = 0; i < p.count; ++i) {
            const adapshot_cache& c = caches[b0 + i];
            p.k_out[i] = (char*)c.k;
            p.v_out[i] = (char*)c.v;
            p.capacity[i] = (int32_t)c.capacity;
            p.slot[i] = (int32_t)c.len;
            p.pos[i] = (int32_t)(pos0 + c.len);
            p.slot_shot[i] = c.slot_shot;
            p.slot_tok[i] = c.slot_tok;
            p.slot_pos[i] = c.slot_pos;
        }
        hipError_t e = timed_launch(ctx, ADAPSHOT_KERNEL_ASSEMBLE, stream, [&] { return launch_decode_append(p, stream); });
        if (e != hipSuccess) return fail_hip(ctx, "decode_append: launch", e);
    }
    for (int32_t b = 0; b < n_caches; ++b) caches[b].len += 1;
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

static adapshot_status check_query_attn(adapshot_ctx* ctx, const adapshot_cache* cache, int32_t layer, int64_t n_ctx,
                                        const void* q, const void* k_self, const void* v_self, int32_t t_q,
                                        int64_t q_pos0, const void* out) {
    if (!cache || !q || !k_self || !v_self || !out) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: null pointer");
    if (t_q < 1) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: t_q < 1");
    if (layer < 0 || layer >= ctx->desc.n_layers) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: layer out of range");
    if (n_ctx < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: n_ctx < 0");
    if (n_ctx > cache->len || cache->len > cache->capacity)
        return fail(ctx, ADAPSHOT_ESTATE, "query_attn: n_ctx %lld beyond assembled length %lld", (long long)n_ctx,
                    (long long)cache->len);
    if (n_ctx > 0 && (!cache->k || !cache->v)) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: null cache buffers");
    if (q_pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn: q_pos0 < 0");
    if (q_pos0 + t_q > ctx->max_position)
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn: query positions exceed max_position");
    if (!aligned16(q) || !aligned16(k_self) || !aligned16(v_self) || !aligned16(out) || !aligned16(cache->k) ||
        !aligned16(cache->v))
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn: pointers must be 16-byte aligned");

    if ((uint64_t)std::max<int64_t>(n_ctx, t_q) * (uint64_t)ctx->row_bytes > 0xffffffffull)
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn: context rows span more than 4 GiB per layer");
    // the kernels address a query row by a 32-bit byte offset
    if ((uint64_t)t_q * (uint64_t)ctx->desc.n_q_heads * (uint64_t)ctx->desc.head_dim * (uint64_t)ctx->elem_bytes > 0x7fffffffull)
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn: query rows span 2 GiB or more");
    return ADAPSHOT_OK;
}

// Split count of one MFMA attention launch.  The grid is `units` (kv head, row tile) pairs times the context
// splits, plus one workgroup per unit for the query's own tokens; one workgroup occupies a compute unit, and
// the self workgroups are dispatched first.  A handful of candidate counts -- everything in one round beside
// the self workgroups, one context split per compute unit with the last of them starting when the self
// workgroups are done, and two to four rounds of that -- are priced in 64-key tiles plus a fixed
// per-workgroup cost, and the cheapest wins (the smaller count on a tie).  A short context fits everything into
// one round (26k tokens, 16 units: 15 splits of 29 tiles beside the 16 self workgroups); a long one does not
// leave the self workgroups' compute units idle (127k tokens, 64 units: 4 splits of 495 tiles, not 3 of 660).
static int64_t plan_mfma_splits(int64_t n_cu, int64_t units, int64_t key_tiles, int64_t self_tiles) {
    const double fixed = 2.5;  // launch, first tile round trip and partial write-out of a workgroup, in tiles
    const int64_t s_max = std::min<int64_t>(key_tiles, 64);
    const double ls = (double)self_tiles + fixed;
    auto price = [&](int64_t s) {
        const double l = (double)((key_tiles + s - 1) / s) + fixed;
        const int64_t n = units * s;
        double t;
        if (units + n <= n_cu) t = std::max(l, ls);          // one round
        else if (n <= n_cu && units <= n_cu) t = ls + l;      // the context workgroups that do not fit wait for the self ones
        else t = ceil(((double)n * l + (double)units * ls) / ((double)n_cu * l)) * l;  // whole rounds
        return t + 0.02 * (double)s;                           // partials cost a little too
    };
    const int64_t one_round = (n_cu - units) / units, per_cu = n_cu / units;
    const int64_t cand[6] = {1, one_round, per_cu, 2 * per_cu, 3 * per_cu, 4 * per_cu};
    int64_t best = 1;
    double best_t = price(1);
    for (int64_t c : cand) {
        int64_t sc = std::max<int64_t>(1, std::min<int64_t>(c, s_max));
        sc = (key_tiles + ((key_tiles + sc - 1) / sc) - 1) / ((key_tiles + sc - 1) / sc);  // the count this split length gives
        const double t = price(sc);
        if (t < best_t - 1e-9 || (t < best_t + 1e-9 && sc < best)) {
            best = sc;
            best_t = t;
        }
    }
    return best;
}

// Split the context of one attention call so that (kv heads x row tiles x splits) fills the chip: once for the
// MFMA kernel (one 8-wave workgroup per compute unit), several times for the one-wave generic kernel.  Keys per
// split is a multiple of the 64-key tile; an empty context has no split.
static void plan_single_attn(const adapshot_model_desc& d, int64_t n_cu, int32_t force_splits, int32_t t_q, int64_t n_ctx,
                             int64_t* n_split_out, int64_t* keys_per_split_out) {
    const bool mfma = attn_mfma_supported(d);
    const int64_t rows = (int64_t)t_q * (d.n_q_heads / d.n_kv_heads);
    const int64_t row_tile = mfma ? kAttnRowTile : 1;
    const int64_t units = d.n_kv_heads * ((rows + row_tile - 1) / row_tile);
    const int64_t key_tiles = (n_ctx + 63) / 64;
    int64_t n_split = 0, keys_per_split = 64;
    if (key_tiles > 0) {
        if (mfma) {
            n_split = plan_mfma_splits(n_cu, units, key_tiles, ((int64_t)t_q + 63) / 64);
        } else {
            const int64_t target = std::max<int64_t>(1, n_cu * 8 / units);
            n_split = std::min<int64_t>(std::min<int64_t>(target, key_tiles), 64);
        }
        if (force_splits > 0) n_split = std::min<int64_t>(force_splits, key_tiles);
        keys_per_split = ((key_tiles + n_split - 1) / n_split) * 64;
        n_split = (n_ctx + keys_per_split - 1) / keys_per_split;
    }
    *n_split_out = n_split;
    *keys_per_split_out = keys_per_split;
}

// k_ctx / v_ctx: one layer of the context the rows attend over -- the assembled cache, or, for the zero-copy form
// (slot_src and tile_rot given), one layer of the pool.
static adapshot_status run_query_attn_on(adapshot_ctx* ctx, const void* k_ctx, const void* v_ctx, int64_t n_ctx,
                                         const void* q, const void* k_self, const void* v_self, int32_t t_q,
                                         int64_t q_pos0, void* out, const int32_t* slot_src, const float2* tile_rot,
                                         hipStream_t stream, int64_t ctx_pos0 = 0);

static adapshot_status run_query_attn(adapshot_ctx* ctx, const adapshot_cache* cache, int32_t layer, int64_t n_ctx,
                                      const void* q, const void* k_self, const void* v_self, int32_t t_q,
                                      int64_t q_pos0, void* out, hipStream_t stream) {
    const int64_t layer_off = (int64_t)layer * cache->capacity * ctx->row_bytes;
    return run_query_attn_on(ctx, (const char*)cache->k + layer_off, (const char*)cache->v + layer_off, n_ctx, q, k_self,
                             v_self, t_q, q_pos0, out, nullptr, nullptr, stream);
}

static adapshot_status run_query_attn_on(adapshot_ctx* ctx, const void* k_ctx, const void* v_ctx, int64_t n_ctx,
                                         const void* q, const void* k_self, const void* v_self, int32_t t_q,
                                         int64_t q_pos0, void* out, const int32_t* slot_src, const float2* tile_rot,
                                         hipStream_t stream, int64_t ctx_pos0) {
    const adapshot_model_desc& d = ctx->desc;
    const int g = d.n_q_heads / d.n_kv_heads;
    const int64_t rows = (int64_t)t_q * g;
    const bool mfma = attn_mfma_supported(d);

    int64_t n_split = 0, keys_per_split = 64;
    plan_single_attn(d, ctx->n_cu, ctx->force_splits, t_q, n_ctx, &n_split, &keys_per_split);

    const size_t esz = (size_t)ctx->elem_bytes;
    hipError_t e = hipSuccess;
    const bool fold = mfma;  // the matrix-core kernels rotate the query rows (and the query's own keys) themselves
    if (!fold) {
        e = ctx->q_rot.reserve((size_t)t_q * d.n_q_heads * d.head_dim * esz, ctx->retired);
        if (e == hipSuccess) e = ctx->k_rot.reserve((size_t)t_q * d.n_kv_heads * d.head_dim * esz, ctx->retired);
    }
    if (e == hipSuccess)
        e = ctx->part_o.reserve((size_t)(n_split + 1) * d.n_kv_heads * rows * d.head_dim * (mfma ? 2 : 4), ctx->retired);
    if (e == hipSuccess) e = ctx->part_ml.reserve((size_t)(n_split + 1) * d.n_kv_heads * rows * sizeof(float4), ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn: workspace", e);

    RopeRowsParams rp;
    rp.q = q;
    rp.k_self = k_self;
    rp.q_rot = ctx->q_rot.p;
    rp.k_rot = ctx->k_rot.p;
    rp.tab_lo = ctx->tab_lo;
    rp.tab_hi = ctx->tab_hi;
    rp.q_pos0 = q_pos0;
    rp.t_q = t_q;
    rp.n_q_heads = d.n_q_heads;
    rp.n_kv_heads = d.n_kv_heads;
    rp.head_dim = d.head_dim;
    rp.dtype = d.dtype;
    rp.q_scale = (float)(1.4426950408889634 / sqrt((double)d.head_dim));
    if (!fold) {
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ROPE_ROWS, stream, [&] { return launch_rope_rows(rp, stream); });
        if (e != hipSuccess) return fail_hip(ctx, "query_attn: rope launch", e);
    }

    AttnParams ap;
    ap.k_cache = k_ctx;
    ap.v_cache = v_ctx;
    AttnFold af;
    af.slot_src = slot_src;
    af.tile_rot = tile_rot;
    ap.q_rot = ctx->q_rot.p;
    ap.k_self_rot = ctx->k_rot.p;
    ap.v_self = v_self;
    af.q_raw = q;
    af.k_self_raw = k_self;
    af.tab_lo = ctx->tab_lo;
    af.tab_hi = ctx->tab_hi;
    af.q_pos0 = q_pos0;
    af.q_scale = rp.q_scale;
    af.pool_tokens = (int32_t)std::min<int64_t>(ctx->shot_offsets.empty() ? 0 : ctx->shot_offsets.back(), INT32_MAX);
    ap.part_o = ctx->part_o.p;
    ap.part_mlf = (float4*)ctx->part_ml.p;
    ap.part_half = mfma ? 1 : 0;
    ap.no_self = 0;
    ap.v_blocks = 4;
    ap.split_bounds = nullptr;
    ap.out = out;
    ap.n_ctx = n_ctx;
    ap.keys_per_split = keys_per_split;
    ap.n_split = (int32_t)n_split;
    ap.t_q = t_q;
    ap.n_q_heads = d.n_q_heads;
    ap.n_kv_heads = d.n_kv_heads;
    ap.head_dim = d.head_dim;
    ap.dtype = d.dtype;
    ap.layer_stride_bytes = 0;
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN, stream, [&] {
        if (!mfma) return launch_attn_generic(ap, GenericPool{slot_src, ctx->tab_lo, ctx->tab_hi, ctx_pos0}, stream);
        return slot_src ? launch_attn_mfma_pool(ap, af, stream) : launch_attn_mfma(ap, af, stream);
    });
    if (e != hipSuccess) return fail_hip(ctx, "query_attn: attention launch", e);
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream, [&] { return launch_attn_combine(ap, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "query_attn: combine launch", e);
    return ADAPSHOT_OK;
}

// Common split length (in 64-key tiles) of a batch.  The longest item is cut into n equal splits, every other item
// into splits of that length plus a remainder; n is the candidate whose work list finishes first when the
// workgroups, sorted longest first, are dealt round-robin over the compute units (the first workgroup of every
// round is the longest of that round, so the finish time is the sum of those), or rather the fewest splits that come
// within 12 % of it: whole rounds of equal workgroups win
// over an average that leaves a few compute units one workgroup more (32 queries x 4 kv heads x 16k tokens: 4 splits,
// 512 workgroups in two rounds, 199 us; the 4-or-5 splits of an average-based length: 210 us; 3 splits: 230 us).
struct BatchShape {
    int64_t units, key_tiles, self_tiles;
};
static int64_t plan_batch_split_tiles(int64_t n_cu, const std::vector<BatchShape>& shapes, int32_t force_splits) {
    int64_t longest = 1;
    for (const BatchShape& b : shapes) longest = std::max(longest, b.key_tiles);
    if (force_splits > 0) return (longest + force_splits - 1) / force_splits;
    const double fixed = 2.5;  // launch, first tile round trip and partial write-out of a workgroup, in tiles
    struct Class {
        double cost;
        int64_t count;
    };
    std::vector<Class> cls;
    int64_t best_st = longest;
    double best_t = 1e300;
    static const int kCand[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 20, 24, 32, 48, 64};
    int64_t cand_st[sizeof(kCand) / sizeof(kCand[0])];
    double cand_t[sizeof(kCand) / sizeof(kCand[0])];
    int n_cand = 0;
    int64_t last_st = -1;
    for (int n : kCand) {
        int64_t st = (longest + n - 1) / n;
        if (st < 8 && longest >= 8) st = 8;  // shorter splits are all prologue
        if (st == last_st) continue;
        last_st = st;
        cls.clear();
        int64_t partials = 0;
        for (const BatchShape& b : shapes) {
            const int64_t full = b.key_tiles / st, rem = b.key_tiles - full * st;
            if (full > 0) cls.push_back(Class{(double)st + fixed, full * b.units});
            if (rem > 0) cls.push_back(Class{(double)rem + fixed, b.units});
            cls.push_back(Class{(double)b.self_tiles + fixed, b.units});
            partials += (full + (rem > 0)) * b.units;
        }
        std::sort(cls.begin(), cls.end(), [](const Class& a, const Class& b) { return a.cost > b.cost; });
        // finish time of the compute unit that gets the first workgroup of every round
        double t = 0.0;
        int64_t rank = 0, next_pick = 0;  // workgroups dealt so far; rank of the next round's first workgroup
        for (const Class& c : cls) {
            while (next_pick < rank + c.count) {
                t += c.cost;
                next_pick += n_cu;
            }
            rank += c.count;
        }
        t += 0.0005 * (double)partials;  // the partials are written and merged too
        cand_st[n_cand] = st;
        cand_t[n_cand++] = t;
        best_t = std::min(best_t, t);
    }
    // The fewest splits within 12 % of the best: the chip clocks higher while some compute units idle, so a finer
    // cut gains less than its balance promises, and every extra workgroup has a prologue, an epilogue and a
    // partial of its own (the probe sweep's 48 items: 4-5 splits of the longest item 850 us, 8-16 splits 872-887 us).
    for (int i = 0; i < n_cand; ++i)
        if (cand_t[i] <= 1.12 * best_t) return cand_st[i];
    return best_st;
}

// All items of a batch in two launches: one MFMA attention grid over the work list of all (item, kv head,
// row tile, split) workgroups (each rotates the query rows it needs itself), one combine grid.  Items are validated
// by the caller.  The context is cut into splits of one common length (plan_batch_split_tiles: whole rounds of
// equal workgroups over the chip); the work list is ordered longest first.
// With `pool` given the items' contexts are shot lists read where they lie in the pool (zero-copy form): an item's
// cache_index names a list, and its context is the first n_ctx slots of that list's slot table.
struct PoolBatch {
    const char* k_layer;        // the layer to attend in (what the item-by-item path of other shapes reads)
    const char* v_layer;
    const int32_t* slot_src;    // device: the lists' slot tables, one after the other
    const int64_t* list_base;   // host: first entry of every list in slot_src
    const float2* tile_rot;     // device: (cos, sin) of position pos0 + 64 i for every 64-slot tile, shared by the lists
};
static adapshot_status run_query_attn_batch(adapshot_ctx* ctx, const adapshot_cache* caches, int32_t layer,
                                            const adapshot_attn_item* items, int32_t n_items, hipStream_t stream,
                                            const PoolBatch* pool = nullptr) {
    const adapshot_model_desc& d = ctx->desc;
    const int g = d.n_q_heads / d.n_kv_heads;

    // ---- the same batch as the last call (the next layer of a model)?  Then the tables in device memory still
    // hold: they name layer 0 of every context, and the launch names the layer.
    std::vector<unsigned char> key;
    {
        auto put = [&](const void* ptr, size_t n) { key.insert(key.end(), (const unsigned char*)ptr, (const unsigned char*)ptr + n); };
        key.reserve(16 + (size_t)n_items * (sizeof(adapshot_attn_item) + 3 * sizeof(void*)));
        const int32_t head[4] = {pool ? 1 : 0, ctx->force_splits, n_items, ctx->n_cu};
        put(head, sizeof(head));
        put(items, (size_t)n_items * sizeof(adapshot_attn_item));
        for (int32_t i = 0; i < n_items; ++i) {
            if (pool) {
                const void* id[3] = {ctx->k_pool, pool->slot_src + pool->list_base[items[i].cache_index], pool->tile_rot};
                put(id, sizeof(id));
            } else {
                const adapshot_cache& c = caches[items[i].cache_index];
                const void* id[2] = {c.k, c.v};
                put(id, sizeof(id));
                put(&c.capacity, sizeof(c.capacity));
            }
        }
    }
    // Few rows per kv head and every context read by one item only: the launch streams its tiles.
    bool stream_tiles = pool == nullptr;
    if (stream_tiles) {
        std::vector<int32_t> seen;
        seen.reserve((size_t)n_items);
        for (int32_t i = 0; i < n_items && stream_tiles; ++i) {
            if ((int64_t)items[i].t_q * g > kAttnStreamRows) stream_tiles = false;
            if (items[i].n_ctx > 0) seen.push_back(items[i].cache_index);
        }
        if (stream_tiles) {
            std::sort(seen.begin(), seen.end());
            stream_tiles = std::adjacent_find(seen.begin(), seen.end()) == seen.end();
        }
    }
    if (!ctx->batch_key.empty() && key == ctx->batch_key) {
        const AttnBatchItem* dit = (const AttnBatchItem*)ctx->batch_tab.p;
        const AttnWork* daw = (const AttnWork*)((const char*)ctx->batch_tab.p + ctx->batch_attn_off);
        const CombineWork* dcw = (const CombineWork*)((const char*)ctx->batch_tab.p + ctx->batch_comb_off);
        hipError_t e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN, stream, [&] {
            return launch_attn_mfma_batched(dit, daw, (int)ctx->batch_n_attn, pool != nullptr, stream_tiles, layer, stream);
        });
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: attention launch", e);
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream,
                         [&] { return launch_attn_combine_batched(dit, dcw, (int)ctx->batch_n_comb, d.dtype, ctx->batch_max_partials, stream); });
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: combine launch", e);
        return ADAPSHOT_OK;
    }
    ctx->batch_key.clear();  // the tables are about to be rewritten

    // ---- split plan
    std::vector<BatchShape> shapes((size_t)n_items);
    for (int32_t i = 0; i < n_items; ++i) {
        const int64_t rows = (int64_t)items[i].t_q * g;
        shapes[(size_t)i].units = d.n_kv_heads * ((rows + kAttnRowTile - 1) / kAttnRowTile);
        shapes[(size_t)i].key_tiles = (items[i].n_ctx + 63) / 64;
        shapes[(size_t)i].self_tiles = ((int64_t)items[i].t_q + 63) / 64;
    }
    const int64_t split_tiles_common = plan_batch_split_tiles(ctx->n_cu, shapes, ctx->force_splits);

    struct Plan {
        int64_t rows, n_row_tiles, n_split, keys_per_split;
        size_t po_off, pml_off;
    };
    std::vector<Plan> plan((size_t)n_items);
    size_t po_bytes = 0, pml_bytes = 0;
    int64_t n_attn = 0, n_comb = 0;
    int32_t max_partials = 1;
    for (int32_t i = 0; i < n_items; ++i) {
        const adapshot_attn_item& it = items[i];
        Plan& pl = plan[(size_t)i];
        pl.rows = (int64_t)it.t_q * g;
        pl.n_row_tiles = (pl.rows + kAttnRowTile - 1) / kAttnRowTile;
        const int64_t key_tiles = (it.n_ctx + 63) / 64;
        pl.n_split = 0;
        pl.keys_per_split = 64;
        if (key_tiles > 0) {
            int64_t st = split_tiles_common;
            if ((key_tiles + st - 1) / st > 64) st = (key_tiles + 63) / 64;  // at most 64 context splits per item
            pl.keys_per_split = st * 64;
            pl.n_split = (it.n_ctx + pl.keys_per_split - 1) / pl.keys_per_split;
        }
        auto up = [](size_t v) { return (v + 255) & ~(size_t)255; };
        pl.po_off = po_bytes;
        po_bytes += up((size_t)(pl.n_split + 1) * d.n_kv_heads * pl.rows * d.head_dim * 2);  // fp16 rows
        pl.pml_off = pml_bytes;
        pml_bytes += up((size_t)(pl.n_split + 1) * d.n_kv_heads * pl.rows * sizeof(float4));
        n_attn += d.n_kv_heads * pl.n_row_tiles * (pl.n_split + 1);
        max_partials = std::max<int32_t>(max_partials, (int32_t)pl.n_split + 1);
        n_comb += (d.n_kv_heads * pl.rows + 15) / 16;
    }
    if (n_attn > INT32_MAX || n_comb > INT32_MAX)
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn_batched: batch too large for one launch");

    // ---- workspace and tables
    hipError_t e = ctx->part_o.reserve(po_bytes, ctx->retired);
    if (e == hipSuccess) e = ctx->part_ml.reserve(pml_bytes, ctx->retired);
    const size_t items_bytes = (size_t)n_items * sizeof(AttnBatchItem);
    const size_t attn_off = (items_bytes + 255) & ~(size_t)255;
    const size_t comb_off = (attn_off + (size_t)n_attn * sizeof(AttnWork) + 255) & ~(size_t)255;
    const size_t tab_bytes = (comb_off + (size_t)n_comb * sizeof(CombineWork) + 15) & ~(size_t)15;
    if (e == hipSuccess) e = ctx->batch_tab.reserve(tab_bytes, ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: workspace", e);
    int slot = -1;
    void* host = nullptr;
    e = ctx->tile_ring.acquire(tab_bytes, &slot, &host);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: pinned tables", e);

    AttnBatchItem* hit = (AttnBatchItem*)host;
    AttnWork* haw = (AttnWork*)((char*)host + attn_off);
    CombineWork* hcw = (CombineWork*)((char*)host + comb_off);
    struct Key {
        int64_t tiles;
        int32_t cache;
        AttnWork w;
    };
    std::vector<Key> keys;
    keys.reserve((size_t)n_attn);
    int64_t ic = 0;
    for (int32_t i = 0; i < n_items; ++i) {
        const adapshot_attn_item& it = items[i];
        const Plan& pl = plan[(size_t)i];
        AttnBatchItem& b = hit[i];
        if (pool) {  // layer 0 of the context; the launch names the layer
            b.attn.k_cache = ctx->k_pool;
            b.attn.v_cache = ctx->v_pool;
            b.attn.layer_stride_bytes = ctx->pool_layer_stride_tokens * ctx->row_bytes;
            b.fold.slot_src = pool->slot_src + pool->list_base[it.cache_index];
            b.fold.tile_rot = pool->tile_rot;
        } else {
            const adapshot_cache& c = caches[it.cache_index];
            b.attn.k_cache = c.k;
            b.attn.v_cache = c.v;
            b.attn.layer_stride_bytes = c.capacity * ctx->row_bytes;
            b.fold.slot_src = nullptr;
            b.fold.tile_rot = nullptr;
        }
        b.attn.q_rot = nullptr;
        b.attn.k_self_rot = nullptr;
        b.attn.v_self = it.v_self;
        b.fold.q_raw = it.q;
        b.fold.k_self_raw = it.k_self;
        b.fold.tab_lo = ctx->tab_lo;
        b.fold.tab_hi = ctx->tab_hi;
        b.fold.q_pos0 = it.q_pos0;
        b.fold.q_scale = (float)(1.4426950408889634 / sqrt((double)d.head_dim));
        b.fold.pool_tokens = (int32_t)std::min<int64_t>(ctx->shot_offsets.empty() ? 0 : ctx->shot_offsets.back(), INT32_MAX);
        b.attn.part_o = (char*)ctx->part_o.p + pl.po_off;
        b.attn.part_mlf = (float4*)((char*)ctx->part_ml.p + pl.pml_off);
        b.attn.part_half = 1;
        b.attn.no_self = 0;
        b.attn.v_blocks = 4;
        b.attn.split_bounds = nullptr;
        b.attn.out = it.out;
        b.attn.n_ctx = it.n_ctx;
        b.attn.keys_per_split = pl.keys_per_split;
        b.attn.n_split = (int32_t)pl.n_split;
        b.attn.t_q = it.t_q;
        b.attn.n_q_heads = d.n_q_heads;
        b.attn.n_kv_heads = d.n_kv_heads;
        b.attn.head_dim = d.head_dim;
        b.attn.dtype = d.dtype;
        for (int64_t sp = 0; sp <= pl.n_split; ++sp) {
            int64_t tiles;
            if (sp == pl.n_split) tiles = (it.t_q + 63) / 64;
            else tiles = (std::min<int64_t>(it.n_ctx, (sp + 1) * pl.keys_per_split) - sp * pl.keys_per_split + 63) / 64;
            for (int64_t rt = 0; rt < pl.n_row_tiles; ++rt)
                for (int32_t hk = 0; hk < d.n_kv_heads; ++hk)
                    keys.push_back(Key{tiles, sp == pl.n_split ? -1 : it.cache_index, AttnWork{i, hk, (int32_t)rt, (int32_t)sp}});
        }
        const int64_t pairs = d.n_kv_heads * pl.rows;
        for (int64_t p0 = 0; p0 < pairs; p0 += 16) hcw[ic++] = CombineWork{i, (int32_t)p0};
    }
    // Longest workgroups first.  Among equal lengths, the workgroups that read the same slice of the same
    // cache (probes over nested prefixes of one ordering share their leading splits, because the split
    // length is common) are adjacent, kv head fastest: they start together on the XCD that serves that head
    // and the later ones find the slice in its L2 -- the shared prefix of a probe tree is fetched once.
    std::stable_sort(keys.begin(), keys.end(), [](const Key& a, const Key& b) {
        if (a.tiles != b.tiles) return a.tiles > b.tiles;
        if (a.cache != b.cache) return a.cache < b.cache;
        if (a.cache >= 0 && a.w.split != b.w.split) return a.w.split < b.w.split;
        return false;
    });
    for (size_t k = 0; k < keys.size(); ++k) haw[k] = keys[k].w;

    e = launch_copy_table(ctx->batch_tab.p, host, tab_bytes, stream);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: table copy", e);
    e = ctx->tile_ring.mark_in_use(slot, stream);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: event record", e);
    const AttnBatchItem* dit = (const AttnBatchItem*)ctx->batch_tab.p;
    const AttnWork* daw = (const AttnWork*)((const char*)ctx->batch_tab.p + attn_off);
    const CombineWork* dcw = (const CombineWork*)((const char*)ctx->batch_tab.p + comb_off);
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN, stream,
                     [&] { return launch_attn_mfma_batched(dit, daw, (int)n_attn, pool != nullptr, stream_tiles, layer, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: attention launch", e);
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream,
                     [&] { return launch_attn_combine_batched(dit, dcw, (int)n_comb, d.dtype, max_partials, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_batched: combine launch", e);
    ctx->batch_key.swap(key);
    ctx->batch_n_attn = n_attn;
    ctx->batch_max_partials = max_partials;
    ctx->batch_n_comb = n_comb;
    ctx->batch_attn_off = attn_off;
    ctx->batch_comb_off = comb_off;
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_query_attn(adapshot_ctx* ctx, const adapshot_cache* cache, int32_t layer,
                                               int64_t n_ctx, const void* q, const void* k_self,
                                               const void* v_self, int32_t t_q, int64_t q_pos0, void* out,
                                               void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    adapshot_status st = check_query_attn(ctx, cache, layer, n_ctx, q, k_self, v_self, t_q, q_pos0, out);
    if (st != ADAPSHOT_OK) return st;
    st = run_query_attn(ctx, cache, layer, n_ctx, q, k_self, v_self, t_q, q_pos0, out, (hipStream_t)hip_stream);
    if (st == ADAPSHOT_OK) ctx->last_error.clear();
    return st;
}

// Zero-copy form: the rows attend over the selected shots where they lie in the pool.
extern "C" adapshot_status adapshot_query_attn_pool(adapshot_ctx* ctx, int32_t layer, const int32_t* shot_ids,
                                                    const int32_t* order, int32_t m, int64_t pos0, const void* q,
                                                    const void* k_self, const void* v_self, int32_t t_q,
                                                    int64_t q_pos0, void* out, void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    const adapshot_model_desc& d = ctx->desc;
    if (d.key_state != ADAPSHOT_KEYS_UNROTATED)
        return fail(ctx, ADAPSHOT_ESTATE, "query_attn_pool: needs a pool registered with ADAPSHOT_KEYS_UNROTATED");
    if (!ctx->k_pool) return fail(ctx, ADAPSHOT_ESTATE, "query_attn_pool: no pool registered");
    if (m < 0 || (m > 0 && !shot_ids)) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: bad shot list");
    if (!q || !k_self || !v_self || !out) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: null pointer");
    if (!aligned16(q) || !aligned16(k_self) || !aligned16(v_self) || !aligned16(out))
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: pointers must be 16-byte aligned");
    if (t_q < 1) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: t_q < 1");
    if (layer < 0 || layer >= d.n_layers) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: layer out of range");
    if (pos0 < 0 || q_pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: negative position");
    if (q_pos0 + t_q > ctx->max_position)
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool: query positions exceed max_position");
    int64_t total = 0;
    for (int32_t j = 0; j < m; ++j) {
        const int32_t oj = order ? order[j] : j;
        if (oj < 0 || oj >= m) return fail(ctx, ADAPSHOT_ESHOT, "query_attn_pool: order[%d] = %d out of range", j, oj);
        const int32_t s = shot_ids[oj];
        if (s < 0 || s >= ctx->n_shots) return fail(ctx, ADAPSHOT_ESHOT, "query_attn_pool: shot id %d out of range", s);
        total += ctx->shot_offsets[s + 1] - ctx->shot_offsets[s];
    }
    if (total > INT32_MAX) return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool: context longer than 2^31 - 1 tokens");
    if (pos0 + total > ctx->max_position)
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool: position %lld exceeds max_position %lld",
                    (long long)(pos0 + total), (long long)ctx->max_position);
    // a lane of the matrix-core kernel addresses its key row by a 32-bit byte offset inside the pool's layer
    if (attn_mfma_supported(d) &&
        ((uint64_t)ctx->shot_offsets[(size_t)ctx->n_shots] * (uint64_t)ctx->row_bytes > 0xffffffffull ||
         (uint64_t)std::max<int64_t>(total, t_q) * (uint64_t)ctx->row_bytes > 0xffffffffull))
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool: a pool layer of 4 GiB or more is not supported");
    if ((uint64_t)t_q * (uint64_t)d.n_q_heads * (uint64_t)d.head_dim * (uint64_t)ctx->elem_bytes > 0x7fffffffull)
        return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool: query rows span 2 GiB or more");
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t layer_off = (int64_t)layer * ctx->pool_layer_stride_tokens * ctx->row_bytes;
    const char* k_layer = (const char*)ctx->k_pool + layer_off;
    const char* v_layer = (const char*)ctx->v_pool + layer_off;
    if (total == 0) {  // nothing but the query's own tokens
        adapshot_status st = run_query_attn_on(ctx, k_layer, v_layer, 0, q, k_self, v_self, t_q, q_pos0, out, nullptr, nullptr,
                                               stream);
        if (st == ADAPSHOT_OK) ctx->last_error.clear();
        return st;
    }

    // the plan of the same shots at the same positions (the previous layer's call) still holds
    std::vector<unsigned char> pkey;
    {
        auto put = [&](const void* ptr, size_t n) { pkey.insert(pkey.end(), (const unsigned char*)ptr, (const unsigned char*)ptr + n); };
        pkey.reserve(sizeof(int64_t) * 2 + sizeof(int32_t) * (size_t)(m + 1));
        const int64_t head[2] = {-1, pos0};  // -1: a single list at the start of the table (a batched plan names its list count)
        put(head, sizeof(head));
        put(&m, sizeof(m));
        for (int32_t j = 0; j < m; ++j) {
            const int32_t sid = shot_ids[order ? order[j] : j];
            put(&sid, sizeof(sid));
        }
    }
    if (!ctx->pool_key.empty() && pkey == ctx->pool_key) {
        adapshot_status st = run_query_attn_on(ctx, k_layer, v_layer, total, q, k_self, v_self, t_q, q_pos0, out,
                                               (const int32_t*)ctx->pool_src.p, (const float2*)ctx->pool_rot.p, stream, pos0);
        if (st == ADAPSHOT_OK) ctx->last_error.clear();
        return st;
    }
    ctx->pool_key.clear();  // the tables are about to be rewritten, and a batch's tables point into them
    ctx->batch_key.clear();
    const int64_t n_tiles = (total + 63) / 64;
    hipError_t e = ctx->pool_src.reserve((size_t)(total + 256) * sizeof(int32_t), ctx->retired);  // the kernel reads it 1 KB at a time
    if (e == hipSuccess) e = ctx->pool_rot.reserve((size_t)n_tiles * (d.head_dim / 2) * sizeof(float2), ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool: workspace", e);
    int slot = -1;
    void* host = nullptr;
    e = ctx->tile_ring.acquire((size_t)std::max<int32_t>(m, 1) * sizeof(PoolSeg), &slot, &host);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool: pinned segments", e);
    PoolSeg* segs = (PoolSeg*)host;
    int64_t slot0 = 0;
    int32_t n_segs = 0;
    for (int32_t j = 0; j < m; ++j) {  // slot group j starts at off_j = sum of the lengths before it
        const int32_t s = shot_ids[order ? order[j] : j];
        const int64_t src = ctx->shot_offsets[s], len = ctx->shot_offsets[s + 1] - src;
        if (len > 0) segs[n_segs++] = PoolSeg{(int32_t)slot0, (int32_t)src, (int32_t)len, 0};
        slot0 += len;
    }
    PoolPlanParams pp;
    pp.segs = segs;
    pp.slot_src = (int32_t*)ctx->pool_src.p;
    pp.tile_rot = (float2*)ctx->pool_rot.p;
    pp.tab_lo = ctx->tab_lo;
    pp.tab_hi = ctx->tab_hi;
    pp.pos0 = pos0;
    pp.n_segs = n_segs;
    pp.n_tiles = (int32_t)n_tiles;
    pp.head_dim = d.head_dim;
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ROPE_ROWS, stream, [&] { return launch_pool_plan(pp, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool: plan launch", e);
    e = ctx->tile_ring.mark_in_use(slot, stream);
    if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool: event record", e);
    adapshot_status st = run_query_attn_on(ctx, k_layer, v_layer, total, q, k_self, v_self, t_q, q_pos0, out,
                                           (const int32_t*)ctx->pool_src.p, (const float2*)ctx->pool_rot.p, stream, pos0);
    if (st == ADAPSHOT_OK) {
        ctx->pool_key.swap(pkey);
        ctx->last_error.clear();
    }
    return st;
}

// Zero-copy form of the batched call: every item attends over a prefix of one of n_lists shot lists, read where
// the shots lie in the pool.
extern "C" adapshot_status adapshot_query_attn_pool_batched(adapshot_ctx* ctx, int32_t layer,
                                                            const int32_t* const* shot_ids,
                                                            const int32_t* const* orders, const int32_t* m,
                                                            int32_t n_lists, int64_t pos0,
                                                            const adapshot_attn_item* items, int32_t n_items,
                                                            void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    const adapshot_model_desc& d = ctx->desc;
    if (d.key_state != ADAPSHOT_KEYS_UNROTATED)
        return fail(ctx, ADAPSHOT_ESTATE, "query_attn_pool_batched: needs a pool registered with ADAPSHOT_KEYS_UNROTATED");
    if (!ctx->k_pool) return fail(ctx, ADAPSHOT_ESTATE, "query_attn_pool_batched: no pool registered");
    if (n_items < 0 || n_lists < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: negative count");
    if (n_lists > 0 && (!shot_ids || !m)) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: null list arrays");
    if (n_items > 0 && !items) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: null items");
    if (layer < 0 || layer >= d.n_layers) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: layer out of range");
    if (pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: negative position");
    if (attn_mfma_supported(d) && (uint64_t)ctx->shot_offsets[(size_t)ctx->n_shots] * (uint64_t)ctx->row_bytes > 0xffffffffull)
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool_batched: a pool layer of 4 GiB or more is not supported");

    // ---- the lists: lengths, and where each one's slot table starts
    std::vector<int64_t> list_base((size_t)n_lists + 1, 0), list_len((size_t)n_lists, 0);
    int64_t n_segs = 0, longest = 0;
    for (int32_t l = 0; l < n_lists; ++l) {
        if (m[l] < 0 || (m[l] > 0 && !shot_ids[l]))
            return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: list %d: bad shot list", l);
        const int32_t* order = orders ? orders[l] : nullptr;
        int64_t total = 0;
        for (int32_t j = 0; j < m[l]; ++j) {
            const int32_t oj = order ? order[j] : j;
            if (oj < 0 || oj >= m[l])
                return fail(ctx, ADAPSHOT_ESHOT, "query_attn_pool_batched: list %d: order[%d] = %d out of range", l, j, oj);
            const int32_t s = shot_ids[l][oj];
            if (s < 0 || s >= ctx->n_shots)
                return fail(ctx, ADAPSHOT_ESHOT, "query_attn_pool_batched: list %d: shot id %d out of range", l, s);
            total += ctx->shot_offsets[s + 1] - ctx->shot_offsets[s];
        }
        if (pos0 + total > ctx->max_position)
            return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool_batched: list %d: position %lld exceeds max_position %lld", l,
                        (long long)(pos0 + total), (long long)ctx->max_position);
        if ((uint64_t)total * (uint64_t)ctx->row_bytes > 0xffffffffull)
            return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool_batched: list %d: context rows span more than 4 GiB", l);
        list_len[(size_t)l] = total;
        list_base[(size_t)l + 1] = (list_base[(size_t)l] + total + 63) & ~(int64_t)63;  // every list's table starts 16-byte aligned
        n_segs += m[l];
        longest = std::max(longest, total);
    }
    if (list_base[(size_t)n_lists] > INT32_MAX || n_segs > INT32_MAX)
        return fail(ctx, ADAPSHOT_ECAPACITY, "query_attn_pool_batched: the lists hold more than 2^31 - 1 tokens");
    // ---- the items, each against its list standing in for an assembled cache of the list's length
    for (int32_t i = 0; i < n_items; ++i) {
        const adapshot_attn_item& it = items[i];
        if (it.cache_index < 0 || it.cache_index >= n_lists)
            return fail(ctx, ADAPSHOT_EINVAL, "query_attn_pool_batched: item %d: list index out of range", i);
        adapshot_cache as_cache{};
        as_cache.k = const_cast<void*>(ctx->k_pool);
        as_cache.v = const_cast<void*>(ctx->v_pool);
        as_cache.len = as_cache.capacity = list_len[(size_t)it.cache_index];
        adapshot_status st = check_query_attn(ctx, &as_cache, layer, it.n_ctx, it.q, it.k_self, it.v_self, it.t_q, it.q_pos0,
                                              it.out);
        if (st != ADAPSHOT_OK) {
            ctx->last_error = "query_attn_pool_batched: item " + std::to_string(i) + ": " + ctx->last_error;
            return st;
        }
    }
    if (n_items == 0) {
        ctx->last_error.clear();
        return ADAPSHOT_OK;
    }

    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t layer_off = (int64_t)layer * ctx->pool_layer_stride_tokens * ctx->row_bytes;
    PoolBatch pb;
    pb.k_layer = (const char*)ctx->k_pool + layer_off;
    pb.v_layer = (const char*)ctx->v_pool + layer_off;
    pb.list_base = list_base.data();
    pb.slot_src = nullptr;
    pb.tile_rot = nullptr;
    // the slot tables and rotation rows of the same lists at the same positions (the previous layer's call) still hold
    std::vector<unsigned char> pkey;
    {
        auto put = [&](const void* ptr, size_t n) { pkey.insert(pkey.end(), (const unsigned char*)ptr, (const unsigned char*)ptr + n); };
        pkey.reserve(sizeof(int64_t) * 2 + sizeof(int32_t) * (size_t)(n_lists + n_segs));
        const int64_t head[2] = {n_lists, pos0};
        put(head, sizeof(head));
        put(m, (size_t)n_lists * sizeof(int32_t));
        for (int32_t l = 0; l < n_lists; ++l) {
            const int32_t* order = orders ? orders[l] : nullptr;
            for (int32_t j = 0; j < m[l]; ++j) {
                const int32_t sid = shot_ids[l][order ? order[j] : j];
                put(&sid, sizeof(sid));
            }
        }
    }
    const bool plan_holds = longest > 0 && !ctx->pool_key.empty() && pkey == ctx->pool_key;
    if (plan_holds) {
        pb.slot_src = (const int32_t*)ctx->pool_src.p;
        pb.tile_rot = (const float2*)ctx->pool_rot.p;
    } else if (longest > 0) {
        ctx->pool_key.clear();
        ctx->batch_key.clear();  // its tables point into what is rewritten now
        const int64_t n_tiles = (longest + 63) / 64;
        hipError_t e = ctx->pool_src.reserve((size_t)(list_base[(size_t)n_lists] + 256) * sizeof(int32_t), ctx->retired);
        if (e == hipSuccess) e = ctx->pool_rot.reserve((size_t)n_tiles * (d.head_dim / 2) * sizeof(float2), ctx->retired);
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool_batched: workspace", e);
        int slot = -1;
        void* host = nullptr;
        e = ctx->tile_ring.acquire((size_t)std::max<int64_t>(n_segs, 1) * sizeof(PoolSeg), &slot, &host);
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool_batched: pinned segments", e);
        PoolSeg* segs = (PoolSeg*)host;
        int32_t ns = 0;
        for (int32_t l = 0; l < n_lists; ++l) {
            const int32_t* order = orders ? orders[l] : nullptr;
            int64_t slot0 = list_base[(size_t)l];
            for (int32_t j = 0; j < m[l]; ++j) {
                const int32_t s = shot_ids[l][order ? order[j] : j];
                const int64_t src = ctx->shot_offsets[s], len = ctx->shot_offsets[s + 1] - src;
                if (len > 0) segs[ns++] = PoolSeg{(int32_t)slot0, (int32_t)src, (int32_t)len, 0};
                slot0 += len;
            }
        }
        PoolPlanParams pp;
        pp.segs = segs;
        pp.slot_src = (int32_t*)ctx->pool_src.p;
        pp.tile_rot = (float2*)ctx->pool_rot.p;
        pp.tab_lo = ctx->tab_lo;
        pp.tab_hi = ctx->tab_hi;
        pp.pos0 = pos0;
        pp.n_segs = ns;
        pp.n_tiles = (int32_t)n_tiles;
        pp.head_dim = d.head_dim;
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ROPE_ROWS, stream, [&] { return launch_pool_plan(pp, stream); });
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool_batched: plan launch", e);
        e = ctx->tile_ring.mark_in_use(slot, stream);
        if (e != hipSuccess) return fail_hip(ctx, "query_attn_pool_batched: event record", e);
        pb.slot_src = (const int32_t*)ctx->pool_src.p;
        pb.tile_rot = (const float2*)ctx->pool_rot.p;
        ctx->pool_key.swap(pkey);
    }
    adapshot_status st = ADAPSHOT_OK;
    if (attn_mfma_supported(d)) {
        // with nothing but empty lists every item has its own tokens only, and the kernel never looks at the tables
        st = run_query_attn_batch(ctx, nullptr, layer, items, n_items, stream, &pb);
    } else {  // other shapes run item by item through the generic kernel
        for (int32_t i = 0; i < n_items && st == ADAPSHOT_OK; ++i) {
            const adapshot_attn_item& it = items[i];
            st = run_query_attn_on(ctx, pb.k_layer, pb.v_layer, it.n_ctx, it.q, it.k_self, it.v_self, it.t_q, it.q_pos0, it.out,
                                   it.n_ctx > 0 ? pb.slot_src + list_base[(size_t)it.cache_index] : nullptr, pb.tile_rot, stream,
                                   pos0);
        }
    }
    if (st == ADAPSHOT_OK) ctx->last_error.clear();
    return st;
}

extern "C" adapshot_status adapshot_query_attn_batched(adapshot_ctx* ctx, const adapshot_cache* caches,
                                                       int32_t n_caches, int32_t layer,
                                                       const adapshot_attn_item* items, int32_t n_items,
                                                       void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (n_items < 0 || n_caches < 0) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_batched: negative count");
    if (n_items > 0 && (!items || !caches)) return fail(ctx, ADAPSHOT_EINVAL, "query_attn_batched: null pointer");
    for (int32_t i = 0; i < n_items; ++i) {  // every item is validated before anything is launched
        const adapshot_attn_item& it = items[i];
        if (it.cache_index < 0 || it.cache_index >= n_caches)
            return fail(ctx, ADAPSHOT_EINVAL, "query_attn_batched: item %d: cache_index out of range", i);
        adapshot_status st = check_query_attn(ctx, &caches[it.cache_index], layer, it.n_ctx, it.q, it.k_self, it.v_self,
                                              it.t_q, it.q_pos0, it.out);
        if (st != ADAPSHOT_OK) {  // say which item it was
            ctx->last_error = "query_attn_batched: item " + std::to_string(i) + ": " + ctx->last_error;
            return st;
        }
    }
    if (n_items > 0 && attn_mfma_supported(ctx->desc)) {
        adapshot_status st = run_query_attn_batch(ctx, caches, layer, items, n_items, (hipStream_t)hip_stream);
        if (st != ADAPSHOT_OK) return st;
    } else {
        for (int32_t i = 0; i < n_items; ++i) {
            const adapshot_attn_item& it = items[i];
            adapshot_status st = run_query_attn(ctx, &caches[it.cache_index], layer, it.n_ctx, it.q, it.k_self,
                                                it.v_self, it.t_q, it.q_pos0, it.out, (hipStream_t)hip_stream);
            if (st != ADAPSHOT_OK) return st;
        }
    }
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

// Validation and chunk plan shared by the entropy entry points; nothing is launched.
static adapshot_status plan_probe_entropy(adapshot_ctx* ctx, const float* logits, int64_t row_stride, int32_t n_rows,
                                          int32_t vocab, const float* entropy_out, EntropyParams* out) {
    if (n_rows < 0 || vocab < 1) return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: n_rows < 0 or vocab < 1");
    if (vocab > (1 << 30)) return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: vocab beyond 2^30");
    if (n_rows == 0) return ADAPSHOT_OK;
    if (!logits || !entropy_out) return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: null pointer");
    if (row_stride < vocab) return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: row_stride < vocab");
    if (((uintptr_t)logits & 3u) || ((uintptr_t)entropy_out & 3u))
        return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: pointers must be 4-byte aligned");
    EntropyParams& p = *out;
    p.logits = logits;
    p.out = const_cast<float*>(entropy_out);
    p.partials = nullptr;
    p.row_stride = row_stride;
    p.n_rows = n_rows;
    p.vocab = vocab;
    // Chunk of a row per workgroup: large when there are many rows, small when a few rows
    // must still be spread over all compute units.  Multiple of 1024 floats.
    int64_t chunk = 8192;
    while (chunk > 1024 && (int64_t)n_rows * ((vocab + chunk - 1) / chunk) < (int64_t)ctx->n_cu * 4) chunk /= 2;
    p.chunk = (int32_t)chunk;
    p.n_chunks = (int32_t)((vocab + chunk - 1) / chunk);
    if ((int64_t)n_rows * p.n_chunks > INT32_MAX)
        return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy: n_rows x vocab chunks beyond 2^31 - 1 workgroups");
    return ADAPSHOT_OK;
}

// Vocabulary-wide pass shared by both entropy entry points; `answer` selects the epilogue.
static adapshot_status run_probe_entropy(adapshot_ctx* ctx, const float* logits, int64_t row_stride, int32_t n_rows,
                                         int32_t vocab, const AnswerTokens* answer, float* entropy_out,
                                         void* hip_stream) {
    EntropyParams p;
    adapshot_status st = plan_probe_entropy(ctx, logits, row_stride, n_rows, vocab, entropy_out, &p);
    if (st != ADAPSHOT_OK) return st;
    if (n_rows == 0) {
        ctx->last_error.clear();
        return ADAPSHOT_OK;
    }
    hipStream_t stream = (hipStream_t)hip_stream;
    if (n_rows >= ctx->entropy_rows_min && vocab >= 16384) {  // enough rows of at least one full step for one workgroup each: one launch, no partials
        hipError_t e1 = timed_launch(ctx, ADAPSHOT_KERNEL_ENTROPY_CHUNK, stream, [&] { return launch_entropy_rows(p, answer, stream); });
        if (e1 != hipSuccess) return fail_hip(ctx, "probe_entropy: launch", e1);
        ctx->last_error.clear();
        return ADAPSHOT_OK;
    }
    hipError_t e = ctx->ent_part.reserve((size_t)n_rows * p.n_chunks * 3 * sizeof(float), ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "probe_entropy: workspace", e);
    p.partials = (float*)ctx->ent_part.p;
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ENTROPY_CHUNK, stream, [&] { return launch_entropy_chunk(p, stream); });
    if (e == hipSuccess)
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ENTROPY_FINISH, stream, [&] {
            return answer ? launch_entropy_finish_tokens(p, *answer, stream) : launch_entropy_finish(p, stream);
        });
    if (e != hipSuccess) return fail_hip(ctx, "probe_entropy: launch", e);
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_probe_entropy(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                                  int32_t n_rows, int32_t vocab, float* entropy_out,
                                                  void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    return run_probe_entropy(ctx, logits, row_stride, n_rows, vocab, nullptr, entropy_out, hip_stream);
}

// The same two kernels over the file-scope device array instead of a workspace of the context: no
// allocation of any kind on this path (no hipMalloc, no event creation: the launches are not profiled).
extern "C" adapshot_status adapshot_probe_entropy_static(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                                         int32_t n_rows, int32_t vocab, float* entropy_out,
                                                         void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    EntropyParams p;
    adapshot_status st = plan_probe_entropy(ctx, logits, row_stride, n_rows, vocab, entropy_out, &p);
    if (st != ADAPSHOT_OK) return st;
    if (n_rows == 0) {
        ctx->last_error.clear();
        return ADAPSHOT_OK;
    }
    if ((int64_t)n_rows * p.n_chunks > kStaticEntropyPartials)
        return fail(ctx, ADAPSHOT_ECAPACITY,
                    "probe_entropy_static: %d rows x %d chunks of %d logits need %lld partials, the static scratch holds %d",
                    n_rows, p.n_chunks, p.chunk, (long long)n_rows * p.n_chunks, kStaticEntropyPartials);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device || !ctx->static_ent)
        return fail(ctx, ADAPSHOT_ESTATE, "probe_entropy_static: the context's device must be current");
    p.partials = ctx->static_ent;  // every (row, chunk) triple is written by the first kernel before the second reads it
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e = launch_entropy_chunk(p, stream);
    if (e == hipSuccess) e = launch_entropy_finish(p, stream);
    if (e != hipSuccess) return fail_hip(ctx, "probe_entropy_static: launch", e);
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_probe_entropy_tokens(adapshot_ctx* ctx, const float* logits, int64_t row_stride,
                                                         int32_t n_rows, int32_t vocab, const int32_t* token_ids,
                                                         int32_t n_tokens, int32_t mode, float* entropy_out,
                                                         void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (!token_ids || n_tokens < 1 || n_tokens > kMaxAnswerTokens)
        return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy_tokens: need 1..%d answer tokens", kMaxAnswerTokens);
    if (mode != ADAPSHOT_ENTROPY_FULL_P && mode != ADAPSHOT_ENTROPY_RENORMALISED)
        return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy_tokens: unknown mode %d", mode);
    AnswerTokens c;
    c.n = n_tokens;
    c.mode = mode;
    for (int32_t i = 0; i < kMaxAnswerTokens; ++i) c.id[i] = 0;
    for (int32_t i = 0; i < n_tokens; ++i) {
        if (token_ids[i] < 0 || token_ids[i] >= vocab)
            return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy_tokens: token id %d outside the vocabulary", token_ids[i]);
        for (int32_t k = 0; k < i; ++k)
            if (token_ids[k] == token_ids[i])
                return fail(ctx, ADAPSHOT_EINVAL, "probe_entropy_tokens: token id %d listed twice", token_ids[i]);
        c.id[i] = token_ids[i];
    }
    return run_probe_entropy(ctx, logits, row_stride, n_rows, vocab, &c, entropy_out, hip_stream);
}

// Shots per window: their one-hot columns fill one 32-column block of a V row, so the second product of
// the attention kernel needs a quarter of its matrix instructions.
constexpr int kRankWindowShots = 32;

// Ranking state of one pool layer: windows of consecutive shots (at most kRankWindowShots shots and about
// total / (2 n_cu / n_kv_heads) keys each, so that one query makes a few rounds of workgroups), per-token
// tables, the locally encoded keys (when the pool stores them un-rotated) and the one-hot rows.

static adapshot_status rank_prepare(adapshot_ctx* ctx, int32_t layer, hipStream_t stream) {
    const adapshot_model_desc& d = ctx->desc;
    const int64_t n_tok = ctx->shot_offsets[(size_t)ctx->n_shots];
    const int64_t target_windows = std::max<int64_t>(1, 2 * (int64_t)ctx->n_cu / d.n_kv_heads);
    const int64_t keys_target = std::max<int64_t>(512, ((n_tok + target_windows - 1) / target_windows + 63) / 64 * 64);
    std::vector<int64_t> bounds;
    std::vector<int32_t> shot0;
    std::vector<int32_t> shot_split((size_t)ctx->n_shots);
    bounds.push_back(0);
    shot0.push_back(0);
    {
        int64_t keys = 0;
        int32_t first = 0;
        for (int32_t i = 0; i < ctx->n_shots; ++i) {
            const int64_t len = ctx->shot_offsets[(size_t)i + 1] - ctx->shot_offsets[(size_t)i];
            if (i > first && (i - first >= kRankWindowShots || keys + len > keys_target)) {  // close the window before shot i
                bounds.push_back(ctx->shot_offsets[(size_t)i]);
                shot0.push_back(i);
                first = i;
                keys = 0;
            }
            keys += len;
            shot_split[(size_t)i] = (int32_t)shot0.size() - 1;
        }
    }
    bounds.push_back(n_tok);
    shot0.push_back(ctx->n_shots);
    const int32_t n_split = (int32_t)bounds.size() - 1;

    // One table blob, written into a pinned buffer and brought over by a kernel on the caller's stream:
    // [bounds int64 | local index of every token | window column of every token | first shot of every
    //  window | window of every shot | 1 / T_i], every part 16-byte aligned.
    auto up16 = [](size_t v) { return (v + 15) & ~(size_t)15; };
    const size_t off_bounds = 0;
    const size_t off_tok = up16(off_bounds + bounds.size() * sizeof(int64_t));
    const size_t off_shot0 = up16(off_tok + (size_t)(2 * n_tok) * sizeof(int32_t));
    const size_t off_split = up16(off_shot0 + shot0.size() * sizeof(int32_t));
    const size_t off_inv = up16(off_split + shot_split.size() * sizeof(int32_t));
    const size_t tab_bytes = up16(off_inv + (size_t)ctx->n_shots * sizeof(float));

    const size_t layer_bytes = (size_t)n_tok * ctx->row_bytes;
    const bool rotate = d.key_state == ADAPSHOT_KEYS_UNROTATED;
    hipError_t e = ctx->rank_v.reserve(layer_bytes, ctx->retired);
    if (e == hipSuccess && rotate) e = ctx->rank_k.reserve(layer_bytes, ctx->retired);
    if (e == hipSuccess) e = ctx->rank_tab.reserve(tab_bytes, ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: workspace", e);
    int slot = -1;
    void* host = nullptr;
    e = ctx->tile_ring.acquire(tab_bytes, &slot, &host);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: pinned tables", e);
    memcpy((char*)host + off_bounds, bounds.data(), bounds.size() * sizeof(int64_t));
    int32_t* tok = (int32_t*)((char*)host + off_tok);
    float* inv_len = (float*)((char*)host + off_inv);
    for (int32_t i = 0; i < ctx->n_shots; ++i) {
        const int64_t t0 = ctx->shot_offsets[(size_t)i], len = ctx->shot_offsets[(size_t)i + 1] - t0;
        const int32_t col = i - shot0[(size_t)shot_split[(size_t)i]];
        inv_len[i] = len > 0 ? 1.0f / (float)len : 0.f;
        for (int64_t t = 0; t < len; ++t) {
            tok[t0 + t] = (int32_t)t;
            tok[n_tok + t0 + t] = col;
        }
    }
    memcpy((char*)host + off_shot0, shot0.data(), shot0.size() * sizeof(int32_t));
    memcpy((char*)host + off_split, shot_split.data(), shot_split.size() * sizeof(int32_t));
    e = launch_copy_table(ctx->rank_tab.p, host, tab_bytes, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: table copy", e);
    e = ctx->tile_ring.mark_in_use(slot, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: event record", e);
    const char* tab = (const char*)ctx->rank_tab.p;
    ctx->rank_bounds = (const int64_t*)(tab + off_bounds);
    ctx->rank_tok = (const int32_t*)(tab + off_tok);
    ctx->rank_shot0 = (const int32_t*)(tab + off_shot0);
    ctx->rank_shot_split = (const int32_t*)(tab + off_split);
    ctx->rank_inv_len = (const float*)(tab + off_inv);

    RankPrepareParams rp;
    rp.k_pool = (const char*)ctx->k_pool + (int64_t)layer * ctx->pool_layer_stride_tokens * ctx->row_bytes;
    rp.k_out = rotate ? (char*)ctx->rank_k.p : nullptr;
    rp.v_out = (char*)ctx->rank_v.p;
    rp.tok_local = ctx->rank_tok;
    rp.tok_col = ctx->rank_tok + n_tok;
    rp.tab_lo = ctx->tab_lo;
    rp.tab_hi = ctx->tab_hi;
    rp.n_tok = n_tok;
    rp.n_kv_heads = d.n_kv_heads;
    rp.head_dim = d.head_dim;
    e = launch_rank_prepare(rp, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: prepare launch", e);
    ctx->rank_layer = layer;
    ctx->rank_n_split = n_split;
    return ADAPSHOT_OK;
}

// Ranking for the shapes the matrix-core kernel does not cover (arguments validated by the caller).
static adapshot_status rank_shots_generic(adapshot_ctx* ctx, int32_t layer, const void* q, int32_t t_q, int64_t q_pos0,
                                          float* scores_out, hipStream_t stream) {
    const adapshot_model_desc& d = ctx->desc;
    if (d.head_dim > 1024) return fail(ctx, ADAPSHOT_ESTATE, "rank_shots: head_dim above 1024 is not supported");
    const size_t off_bytes = ((size_t)(ctx->n_shots + 1) * sizeof(int64_t) + 15) & ~(size_t)15;
    const size_t rows = (size_t)t_q * d.n_q_heads;
    hipError_t e = ctx->q_rot.reserve(rows * d.head_dim * (size_t)ctx->elem_bytes, ctx->retired);
    if (e == hipSuccess) e = ctx->rank_tab.reserve(off_bytes, ctx->retired);
    if (e == hipSuccess) e = ctx->rank_w.reserve(rows * (size_t)ctx->n_shots * sizeof(float), ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: workspace", e);
    ctx->rank_layer = -1;  // the table buffer is shared with the matrix-core path's prepared state
    int slot = -1;
    void* host = nullptr;
    e = ctx->tile_ring.acquire(off_bytes, &slot, &host);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: pinned tables", e);
    memcpy(host, ctx->shot_offsets.data(), (size_t)(ctx->n_shots + 1) * sizeof(int64_t));
    e = launch_copy_table(ctx->rank_tab.p, host, off_bytes, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: table copy", e);
    e = ctx->tile_ring.mark_in_use(slot, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: event record", e);

    RopeRowsParams rp;
    rp.q = q;
    rp.k_self = nullptr;
    rp.q_rot = ctx->q_rot.p;
    rp.k_rot = nullptr;
    rp.tab_lo = ctx->tab_lo;
    rp.tab_hi = ctx->tab_hi;
    rp.q_pos0 = q_pos0;
    rp.t_q = t_q;
    rp.n_q_heads = d.n_q_heads;
    rp.n_kv_heads = d.n_kv_heads;
    rp.head_dim = d.head_dim;
    rp.dtype = d.dtype;
    rp.q_scale = (float)(1.4426950408889634 / sqrt((double)d.head_dim));
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ROPE_ROWS, stream, [&] { return launch_rope_rows(rp, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: rope launch", e);

    RankGenericParams gp;
    gp.k_pool = (const char*)ctx->k_pool + (int64_t)layer * ctx->pool_layer_stride_tokens * ctx->row_bytes;
    gp.q_rot = ctx->q_rot.p;
    gp.shot_off = (const int64_t*)ctx->rank_tab.p;
    gp.tab_lo = ctx->tab_lo;
    gp.tab_hi = ctx->tab_hi;
    gp.mass = (float*)ctx->rank_w.p;
    gp.scores = scores_out;
    gp.n_shots = ctx->n_shots;
    gp.t_q = t_q;
    gp.n_q_heads = d.n_q_heads;
    gp.n_kv_heads = d.n_kv_heads;
    gp.head_dim = d.head_dim;
    gp.dtype = d.dtype;
    gp.key_state = d.key_state;
    e = launch_rank_generic(gp, stream);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: launch", e);
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_rank_shots(adapshot_ctx* ctx, int32_t layer, const void* q, int32_t t_q,
                                               int64_t q_pos0, float* scores_out, void* hip_stream) {
    if (!ctx) return ADAPSHOT_EINVAL;
    const adapshot_model_desc& d = ctx->desc;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!ctx->k_pool) return fail(ctx, ADAPSHOT_ESTATE, "rank_shots: no pool registered");
    if (layer < 0 || layer >= d.n_layers) return fail(ctx, ADAPSHOT_EINVAL, "rank_shots: layer out of range");
    if (!q || !scores_out) return fail(ctx, ADAPSHOT_EINVAL, "rank_shots: null pointer");
    if (!aligned16(q) || ((uintptr_t)scores_out & 3u)) return fail(ctx, ADAPSHOT_EINVAL, "rank_shots: q must be 16-byte aligned");
    if (t_q < 1 || t_q > 65536) return fail(ctx, ADAPSHOT_EINVAL, "rank_shots: t_q must be in [1, 65536]");
    if (q_pos0 < 0) return fail(ctx, ADAPSHOT_EINVAL, "rank_shots: q_pos0 < 0");
    if (q_pos0 + t_q > ctx->max_position)
        return fail(ctx, ADAPSHOT_ECAPACITY, "rank_shots: query positions exceed max_position");
    const int64_t n_tok = ctx->shot_offsets[(size_t)ctx->n_shots];
    if (ctx->n_shots < 1 || n_tok < 1) return fail(ctx, ADAPSHOT_ESTATE, "rank_shots: empty pool");
    for (int32_t i = 0; i < ctx->n_shots; ++i) {
        const int64_t len = ctx->shot_offsets[(size_t)i + 1] - ctx->shot_offsets[(size_t)i];
        if (len < 1) return fail(ctx, ADAPSHOT_ESTATE, "rank_shots: shot %d is empty", i);
        if (len > ctx->max_position) return fail(ctx, ADAPSHOT_ECAPACITY, "rank_shots: shot %d longer than max_position", i);
    }
    if (!attn_mfma_supported(d)) return rank_shots_generic(ctx, layer, q, t_q, q_pos0, scores_out, stream);
    if (n_tok * ctx->row_bytes >= ((int64_t)1 << 32))
        return fail(ctx, ADAPSHOT_ECAPACITY, "rank_shots: a pool layer of 4 GiB or more is not supported");
    if (ctx->rank_layer != layer) {
        adapshot_status st = rank_prepare(ctx, layer, stream);
        if (st != ADAPSHOT_OK) return st;
    }
    const int g = d.n_q_heads / d.n_kv_heads;
    const int64_t rows = (int64_t)t_q * g;
    const int64_t n_pairs = rows * d.n_kv_heads;
    const int32_t n_split = ctx->rank_n_split;
    const size_t esz = (size_t)ctx->elem_bytes;
    hipError_t e = ctx->q_rot.reserve((size_t)t_q * d.n_q_heads * d.head_dim * esz, ctx->retired);
    if (e == hipSuccess) e = ctx->part_o.reserve((size_t)n_split * n_pairs * d.head_dim * 2, ctx->retired);
    if (e == hipSuccess) e = ctx->part_ml.reserve((size_t)n_split * n_pairs * sizeof(float4), ctx->retired);
    if (e == hipSuccess) e = ctx->rank_w.reserve((size_t)n_split * n_pairs * sizeof(float), ctx->retired);
    if (e == hipSuccess)
        e = ctx->rank_part.reserve((size_t)n_split * (size_t)((n_pairs + 255) / 256) * 128 * sizeof(float), ctx->retired);
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: workspace", e);

    RopeRowsParams rp;  // the query rows rotated to q_pos0 + j and scaled, in a launch of their own
    rp.q = q;
    rp.k_self = nullptr;
    rp.q_rot = ctx->q_rot.p;
    rp.k_rot = nullptr;
    rp.tab_lo = ctx->tab_lo;
    rp.tab_hi = ctx->tab_hi;
    rp.q_pos0 = q_pos0;
    rp.t_q = t_q;
    rp.n_q_heads = d.n_q_heads;
    rp.n_kv_heads = d.n_kv_heads;
    rp.head_dim = d.head_dim;
    rp.dtype = d.dtype;
    rp.q_scale = (float)(1.4426950408889634 / sqrt((double)d.head_dim));
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ROPE_ROWS, stream, [&] { return launch_rope_rows(rp, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: rope launch", e);

    AttnParams ap;
    ap.k_cache = d.key_state == ADAPSHOT_KEYS_UNROTATED
                     ? ctx->rank_k.p
                     : (const void*)((const char*)ctx->k_pool + (int64_t)layer * ctx->pool_layer_stride_tokens * ctx->row_bytes);
    ap.v_cache = ctx->rank_v.p;
    AttnFold af;
    af.slot_src = nullptr;
    af.tile_rot = nullptr;
    ap.q_rot = ctx->q_rot.p;
    ap.k_self_rot = nullptr;
    ap.v_self = nullptr;
    af.q_raw = q;
    af.k_self_raw = nullptr;
    af.tab_lo = ctx->tab_lo;
    af.tab_hi = ctx->tab_hi;
    af.q_pos0 = q_pos0;
    af.q_scale = (float)(1.4426950408889634 / sqrt((double)d.head_dim));
    ap.part_o = ctx->part_o.p;
    ap.part_mlf = (float4*)ctx->part_ml.p;
    ap.part_half = 1;
    ap.no_self = 1;
    ap.v_blocks = 1;  // rank_prepare closes a window after kRankWindowShots = 32 shots: one block of columns
    ap.split_bounds = ctx->rank_bounds;
    ap.out = nullptr;
    ap.n_ctx = n_tok;
    ap.keys_per_split = 64;
    ap.n_split = n_split;
    ap.t_q = t_q;
    ap.n_q_heads = d.n_q_heads;
    ap.n_kv_heads = d.n_kv_heads;
    ap.head_dim = d.head_dim;
    ap.dtype = d.dtype;
    ap.layer_stride_bytes = 0;
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN, stream, [&] { return launch_attn_mfma(ap, af, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: attention launch", e);

    RankReduceParams rr;
    rr.part_o = ctx->part_o.p;
    rr.part_mlf = (const float4*)ctx->part_ml.p;
    rr.weights = (float*)ctx->rank_w.p;
    rr.block_part = (float*)ctx->rank_part.p;
    rr.scores = scores_out;
    rr.split_shot0 = ctx->rank_shot0;
    rr.shot_split = ctx->rank_shot_split;
    rr.inv_len = ctx->rank_inv_len;
    rr.inv_rows = 1.0f / ((float)t_q * (float)d.n_q_heads);
    rr.n_split = n_split;
    rr.n_pairs = (int32_t)n_pairs;
    rr.head_dim = d.head_dim;
    rr.n_shots = ctx->n_shots;
    e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream, [&] { return launch_rank_weights(rr, stream); });
    if (e == hipSuccess)
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream, [&] { return launch_rank_reduce(rr, stream); });
    if (e == hipSuccess)
        e = timed_launch(ctx, ADAPSHOT_KERNEL_ATTN_COMBINE, stream, [&] { return launch_rank_finish(rr, stream); });
    if (e != hipSuccess) return fail_hip(ctx, "rank_shots: reduce launch", e);
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

// Host logic: the k best shots by score, best first; equal scores keep the lower shot id first.
extern "C" adapshot_status adapshot_top_k(adapshot_ctx* ctx, const float* scores, int32_t n_shots, int32_t k,
                                          int32_t* shot_ids_out) {
    if (n_shots < 0 || k < 0 || k > n_shots || (n_shots > 0 && !scores) || (k > 0 && !shot_ids_out))
        return fail(ctx, ADAPSHOT_EINVAL, "top_k: bad arguments");
    for (int32_t i = 0; i < n_shots; ++i)
        if (scores[i] != scores[i]) return fail(ctx, ADAPSHOT_EINVAL, "top_k: score %d is NaN", i);
    std::vector<int32_t> idx((size_t)n_shots);
    for (int32_t i = 0; i < n_shots; ++i) idx[(size_t)i] = i;
    std::partial_sort(idx.begin(), idx.begin() + k, idx.end(), [&](int32_t a, int32_t b) {
        return scores[a] > scores[b] || (scores[a] == scores[b] && a < b);
    });
    for (int32_t i = 0; i < k; ++i) shot_ids_out[i] = idx[(size_t)i];
    if (ctx) ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_pick_shots(adapshot_ctx* ctx, const float* entropy, const int32_t* shot_counts,
                                               int32_t n_candidates, float tau, int32_t* picked) {
    if (!picked || n_candidates < 0 || (n_candidates > 0 && (!entropy || !shot_counts)))
        return fail(ctx, ADAPSHOT_EINVAL, "pick_shots: null pointer or negative count");
    int32_t best = -1;
    for (int32_t i = 0; i < n_candidates; ++i) {
        if (shot_counts[i] < 0) return fail(ctx, ADAPSHOT_EINVAL, "pick_shots: negative shot count");
        if (entropy[i] <= tau && (best < 0 || shot_counts[i] < best)) best = shot_counts[i];
    }
    *picked = best;
    if (ctx) ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_set_attn_splits(adapshot_ctx* ctx, int32_t n_split) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (n_split < 0 || n_split > 64) return fail(ctx, ADAPSHOT_EINVAL, "set_attn_splits: n_split must be in [0, 64]");
    ctx->force_splits = n_split;
    ctx->last_error.clear();
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_attn_split_plan(const adapshot_model_desc* desc, int32_t n_compute_units,
                                                    int32_t t_q, int64_t n_ctx, int32_t* n_split,
                                                    int64_t* keys_per_split) {
    if (!desc || !n_split || !keys_per_split || n_compute_units < 1 || t_q < 1 || n_ctx < 0) return ADAPSHOT_EINVAL;
    if (check_desc(*desc) != nullptr) return ADAPSHOT_EINVAL;
    int64_t ns = 0, kps = 64;
    plan_single_attn(*desc, n_compute_units, 0, t_q, n_ctx, &ns, &kps);
    *n_split = (int32_t)ns;
    *keys_per_split = kps;
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_profile_enable(adapshot_ctx* ctx, int32_t enable) {
    if (!ctx) return ADAPSHOT_EINVAL;
    ctx->prof.on = enable != 0;
    return ADAPSHOT_OK;
}

// Shared by the two read calls: waits for the recorded launches of one kind, hands every duration to `sink`
// in launch order and forgets the records.
template <typename Sink>
static adapshot_status profile_drain(adapshot_ctx* ctx, int32_t kind, Sink&& sink) {
    hipError_t err = hipSuccess;
    std::vector<Profiler::Rec> keep;
    for (auto& r : ctx->prof.recs) {
        if (r.kind != kind) {
            keep.push_back(r);
            continue;
        }
        hipError_t e = hipEventSynchronize(r.stop);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        // a record is consumed whether or not it could be read: its events go back to the free list exactly once
        ctx->prof.free_events.push_back(r.start);
        ctx->prof.free_events.push_back(r.stop);
        if (e != hipSuccess) {
            if (err == hipSuccess) err = e;
            continue;
        }
        sink(ms);
    }
    ctx->prof.recs.swap(keep);
    if (err != hipSuccess) return fail_hip(ctx, "profile_read", err);
    return ADAPSHOT_OK;
}

extern "C" adapshot_status adapshot_profile_read(adapshot_ctx* ctx, int32_t kind, double* total_ms, int64_t* launches) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (kind < 0 || kind >= ADAPSHOT_KERNEL_KINDS || !total_ms || !launches)
        return fail(ctx, ADAPSHOT_EINVAL, "profile_read: bad kind or null pointer");
    double tot = 0.0;
    int64_t n = 0;
    adapshot_status st = profile_drain(ctx, kind, [&](float ms) {
        tot += ms;
        ++n;
    });
    *total_ms = tot;
    *launches = n;
    return st;
}

extern "C" adapshot_status adapshot_profile_read_each(adapshot_ctx* ctx, int32_t kind, float* ms_out, int64_t capacity,
                                                      int64_t* launches) {
    if (!ctx) return ADAPSHOT_EINVAL;
    if (kind < 0 || kind >= ADAPSHOT_KERNEL_KINDS || !launches || capacity < 0 || (capacity > 0 && !ms_out))
        return fail(ctx, ADAPSHOT_EINVAL, "profile_read_each: bad kind, capacity or null pointer");
    int64_t n = 0;
    adapshot_status st = profile_drain(ctx, kind, [&](float ms) {
        if (n < capacity) ms_out[n] = ms;
        ++n;
    });
    *launches = n;
    return st;
}
