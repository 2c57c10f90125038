// Fused gather + RoPE re-encode (Semantically-Aware KV Cache: concatenation in rank
// order; Position Decoupling and Re-encoding, Eq. rope_compensation).
//
// A tile is up to kTileTok consecutive tokens of one shot: contiguous in the pool and
// contiguous in the cache, so both sides of the copy are dense byte ranges and every
// wavefront access is a run of full 128-byte lines.  HBM-bound: per token and layer
// the kernel reads one K row and one V row and writes one of each.
//
//   blockIdx.x = (tile, part of the tile), blockIdx.y = layer, blockIdx.z = 0: K, 1: V.
// One layer per workgroup, layer slowest in the dispatch order: the workgroups in flight then work on one or two
// layers, i.e. on two narrow address windows, instead of walking all layers each at its own pace (a multi-layer
// gather copy of the same blocks: 5.47 TB/s against 5.10 TB/s; this kernel on 28..32 layers: +1.5 .. +6 %).
// A workgroup takes wg_tok consecutive tokens of a tile, about 16 KB per layer and operand, and keeps 64 bytes
// per lane in flight with 58 registers (8 wavefronts per SIMD): many small workgroups stream faster on this part
// than few large ones (plain gather copies into 2 GB: 5.5 TB/s in 16 KB blocks, 5.2 TB/s in 64 KB and larger
// blocks).  The tile's cache -- its buffers, its
// layer stride, its position base -- comes from the table in the kernel arguments, so one launch fills the
// caches of a whole batch of queries.
//
// K workgroups first form cos/sin(a*theta_i) for every (token, frequency) of the tile
// ONCE into LDS -- one fp32 angle addition of two fp64-built table entries,
// a = 64*hi + lo -- and then stream all heads and layers through it: a lane owns the
// two 16-byte chunks that hold the pair partners (i, i + d/2), rotates them in fp32 and
// stores both.  V workgroups are a plain 128-bit copy.  Both streams keep their loads one step ahead of
// their stores, and the first K step is requested before the angle table is built.
#include "adapshot_internal.h"

namespace adapshot {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int64_t kAssembleStreamBytes = 256ll << 20;  // launches that write more than this use non-temporal stores

__device__ __forceinline__ u32x4 ld16(const char* p) { return __builtin_nontemporal_load((const u32x4*)p); }
// Plain stores when what the launch writes fits the 256 MB last-level cache (attention reads the cache next, and
// non-temporal stores were ~10 % slower for the pair); non-temporal stores for the launches that stream past it.
template <bool NT>
__device__ __forceinline__ void st16(char* p, u32x4 v) {
    if (NT) __builtin_nontemporal_store(v, (u32x4*)p);
    else *(u32x4*)p = v;
}

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xffff0000u); }
// Two fp32 -> packed bf16, round to nearest even (hardware conversion on gfx950).
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}

// Rotate the pair partners held in chunks a (first half of the head) and b (second half).
// cs points at the (cos, sin) entries of this chunk's frequencies in LDS.
template <int DTYPE>
__device__ __forceinline__ void rotate_chunks(u32x4& a, u32x4& b, const float2* cs) {
    if (DTYPE == ADAPSHOT_BF16) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float2 c0 = cs[2 * w], c1 = cs[2 * w + 1];
            float x1l = bf16_lo(a[w]), x1h = bf16_hi(a[w]);
            float x2l = bf16_lo(b[w]), x2h = bf16_hi(b[w]);
            float y1l = x1l * c0.x - x2l * c0.y, y2l = x2l * c0.x + x1l * c0.y;
            float y1h = x1h * c1.x - x2h * c1.y, y2h = x2h * c1.x + x1h * c1.y;
            a[w] = pack_bf16(y1l, y1h);
            b[w] = pack_bf16(y2l, y2h);
        }
    } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float2 c = cs[w];
            float x1 = __uint_as_float(a[w]), x2 = __uint_as_float(b[w]);
            a[w] = __float_as_uint(x1 * c.x - x2 * c.y);
            b[w] = __float_as_uint(x2 * c.x + x1 * c.y);
        }
    }
}

// DTYPE: element type; CH: 16-byte chunks per half head (head_dim/2 * elem / 16).
template <int DTYPE, int CH, bool NT>
__global__ __launch_bounds__(256) void assemble_reencode_kernel(AssembleParams p) {
    constexpr int E = DTYPE == ADAPSHOT_BF16 ? 2 : 4;
    constexpr int NP = 16 / E;            // pairs per chunk
    constexpr int HALF = CH * NP;         // head_dim / 2
    constexpr int HEAD_BYTES = 2 * CH * 16;
    __shared__ float2 cs[kTileTok * HALF];

    const int tid = threadIdx.x;
    const int parts = kTileTok / p.wg_tok;
    const TileDesc td = p.tiles[blockIdx.x / parts];
    const int t_first = (int)(blockIdx.x % parts) * p.wg_tok;  // this workgroup's tokens of the tile: t_first .. t_first + n_tok - 1
    const int n_tok = td.n_tok - t_first < p.wg_tok ? td.n_tok - t_first : p.wg_tok;
    if (n_tok <= 0) return;  // a ragged tile's last parts are empty (workgroup-uniform)
    // the first cache's entry is read without waiting for the descriptor: a launch for one cache needs no other
    AssembleDst dc = p.dst[0];
    if (p.n_dst != 1) dc = p.dst[__builtin_amdgcn_readfirstlane(td.cache)];
    const int64_t row_bytes = (int64_t)p.n_kv_heads * HEAD_BYTES;
    const int64_t src_off = (int64_t)(td.src_tok + t_first) * row_bytes;
    const int64_t dst_off = (int64_t)(td.dst_slot + t_first) * row_bytes;

    if (blockIdx.z == 1) {
        // ---- V: dense copy of n_tok rows per layer, one step (4 x 16 bytes per lane) ahead ----
        const int n16 = (int)((n_tok * row_bytes) >> 4);
        auto vload = [&](int l, int i0, u32x4(&r)[4]) __attribute__((always_inline)) {
            const char* src = p.v_pool + (int64_t)l * p.pool_layer_stride_bytes + src_off;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + 256 * u < n16) r[u] = ld16(src + ((int64_t)(i0 + 256 * u) << 4));
        };
        auto vstore = [&](int l, int i0, u32x4(&r)[4]) __attribute__((always_inline)) {
            char* dst = dc.v_out + (int64_t)l * dc.layer_stride_bytes + dst_off;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + 256 * u < n16) st16<NT>(dst + ((int64_t)(i0 + 256 * u) << 4), r[u]);
        };
        const int l = blockIdx.y;
        u32x4 cur[4];
        vload(l, tid, cur);
        for (int i0 = tid; i0 - tid < n16; i0 += 1024) {
            const bool more = i0 + 1024 - tid < n16;  // workgroup-uniform
            u32x4 nxt[4];
            if (more) vload(l, i0 + 1024, nxt);
            vstore(l, i0, cur);
#pragma unroll
            for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
        }
        return;
    }

    // ---- K ----
    if (blockIdx.y == 0 && tid < n_tok) {
        const int slot = td.dst_slot + t_first + tid;
        if (dc.slot_shot) dc.slot_shot[slot] = td.shot;
        if (dc.slot_tok) dc.slot_tok[slot] = td.tok0 + t_first + tid;
        if (dc.slot_pos) dc.slot_pos[slot] = dc.pos0 + slot;
    }

    const int rpt = p.n_kv_heads * CH;  // lane items per token: (head, chunk)
    const int n_items = n_tok * rpt;
    // One step of the K stream: up to KI (head, chunk) items per lane, both pair partners of each
    // (2 * KI 16-byte loads in flight per lane, the same as a V step).
    constexpr int KI = 2;
    struct Step {
        u32x4 a[KI], b[KI];
        int64_t off[KI];
        int csi[KI];
    };
    auto load_step = [&](const char* src, int base, Step& st) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < KI; ++u) {
            const int f = base + u * 256 + tid;
            if (f < n_items) {
                const int tau = f / rpt;
                const int r = f - tau * rpt;
                const int h = r / CH;
                const int c = r - h * CH;
                st.off[u] = (int64_t)tau * row_bytes + h * HEAD_BYTES + c * 16;
                st.csi[u] = tau * HALF + c * NP;
                st.a[u] = ld16(src + st.off[u]);
                st.b[u] = ld16(src + st.off[u] + CH * 16);
            }
        }
    };
    auto store_step = [&](char* dst, int base, Step& st) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < KI; ++u) {
            const int f = base + u * 256 + tid;
            if (f < n_items) {
                rotate_chunks<DTYPE>(st.a[u], st.b[u], cs + st.csi[u]);
                st16<NT>(dst + st.off[u], st.a[u]);
                st16<NT>(dst + st.off[u] + CH * 16, st.b[u]);
            }
        }
    };
    // The first keys are requested before the angle table is built, so that the table's own loads and
    // arithmetic run under their latency.
    const int l = blockIdx.y;
    const char* ksrc = p.k_pool + (int64_t)l * p.pool_layer_stride_bytes + src_off;
    char* kdst = dc.k_out + (int64_t)l * dc.layer_stride_bytes + dst_off;
    Step first;
    load_step(ksrc, 0, first);

    // cos/sin of every (token, frequency) of the tile, two frequencies per step.
    for (int it = tid; it < n_tok * (HALF / 2); it += 256) {
        const int tau = it / (HALF / 2);
        const int f2 = it - tau * (HALF / 2);
        const int a = td.angle0 + (t_first + tau) * td.angle_step;
        const f32x4 h = *(const f32x4*)(p.tab_hi + (int64_t)(a >> kRopeLoBits) * HALF + 2 * f2);
        const f32x4 l = *(const f32x4*)(p.tab_lo + (a & (kRopeLo - 1)) * HALF + 2 * f2);
        f32x4 r;
        r[0] = h[0] * l[0] - h[1] * l[1];  // cos(A+B)
        r[1] = h[1] * l[0] + h[0] * l[1];  // sin(A+B)
        r[2] = h[2] * l[2] - h[3] * l[3];
        r[3] = h[3] * l[2] + h[2] * l[3];
        *(f32x4*)(cs + tau * HALF + 2 * f2) = r;
    }
    __syncthreads();

    // The stream runs one step ahead: the loads of the next KI * 256 items are in flight while the current ones
    // are rotated and stored.
    Step cur = first;
    for (int base = 0; base < n_items; base += KI * 256) {
        const bool more = base + KI * 256 < n_items;
        Step nxt;
        if (more) load_step(ksrc, base + KI * 256, nxt);
        store_step(kdst, base, cur);
        cur = nxt;
    }
}

template <int DTYPE, int CH>
static hipError_t launch_t(const AssembleParams& p, hipStream_t stream) {
    dim3 grid((unsigned)p.n_tiles * (unsigned)(kTileTok / p.wg_tok), (unsigned)p.n_layers, 2);
    // what the launch writes, K and V
    const int64_t e = DTYPE == ADAPSHOT_BF16 ? 2 : 4;
    const int64_t written = 2 * p.n_tokens * p.n_kv_heads * p.head_dim * e * p.n_layers;
    if (written > kAssembleStreamBytes)
        launch_kernel((assemble_reencode_kernel<DTYPE, CH, true>), grid, dim3(256), stream, p);
    else
        launch_kernel((assemble_reencode_kernel<DTYPE, CH, false>), grid, dim3(256), stream, p);
    return hipGetLastError();
}

hipError_t launch_assemble(const AssembleParams& p, hipStream_t stream) {
    const int e = p.dtype == ADAPSHOT_BF16 ? 2 : 4;
    const int ch = p.head_dim / 2 * e / 16;
    if (p.n_tiles <= 0) return hipSuccess;
    if (p.wg_tok < 1 || p.wg_tok > kTileTok || (p.wg_tok & (p.wg_tok - 1)) != 0) return hipErrorInvalidValue;
    if ((int64_t)p.n_tiles * (kTileTok / p.wg_tok) > INT32_MAX) return hipErrorInvalidValue;
    if (p.dtype == ADAPSHOT_BF16) {
        switch (ch) {
            case 1: return launch_t<ADAPSHOT_BF16, 1>(p, stream);
            case 2: return launch_t<ADAPSHOT_BF16, 2>(p, stream);
            case 4: return launch_t<ADAPSHOT_BF16, 4>(p, stream);
            case 8: return launch_t<ADAPSHOT_BF16, 8>(p, stream);
            case 16: return launch_t<ADAPSHOT_BF16, 16>(p, stream);
        }
    } else {
        switch (ch) {
            case 1: return launch_t<ADAPSHOT_F32, 1>(p, stream);
            case 2: return launch_t<ADAPSHOT_F32, 2>(p, stream);
            case 4: return launch_t<ADAPSHOT_F32, 4>(p, stream);
            case 8: return launch_t<ADAPSHOT_F32, 8>(p, stream);
            case 16: return launch_t<ADAPSHOT_F32, 16>(p, stream);
        }
    }
    return hipErrorInvalidValue;
}

// ---- decode append ------------------------------------------------------------------------------
// One new token per cache: its key rotated to the token's position (the keys of a decode step come
// from the model un-rotated, whatever the pool's key state), its value copied.  grid = (caches of this
// launch, layers); a lane owns one (head, chunk) item exactly as in the tile kernel.
template <int DTYPE, int CH>
__global__ __launch_bounds__(128) void decode_append_kernel(DecodeAppendParams p) {
    constexpr int E = DTYPE == ADAPSHOT_BF16 ? 2 : 4;
    constexpr int NP = 16 / E;
    constexpr int HALF = CH * NP;
    constexpr int HEAD_BYTES = 2 * CH * 16;
    const int i = blockIdx.x, l = blockIdx.y;
    const int64_t row_bytes = (int64_t)p.n_kv_heads * HEAD_BYTES;
    const char* ksrc = p.k_new + ((int64_t)l * p.n_total + p.first + i) * row_bytes;
    const char* vsrc = p.v_new + ((int64_t)l * p.n_total + p.first + i) * row_bytes;
    const int64_t dst = ((int64_t)l * p.capacity[i] + p.slot[i]) * row_bytes;
    char* kdst = p.k_out[i] + dst;
    char* vdst = p.v_out[i] + dst;
    const int a = p.pos[i];
    if (l == 0 && threadIdx.x == 0) {
        if (p.slot_shot[i]) p.slot_shot[i][p.slot[i]] = -1;  // not a pool shot
        if (p.slot_tok[i]) p.slot_tok[i][p.slot[i]] = 0;
        if (p.slot_pos[i]) p.slot_pos[i][p.slot[i]] = a;
    }
    const int n_items = p.n_kv_heads * CH;
    for (int f = threadIdx.x; f < n_items; f += 128) {
        const int h = f / CH, c = f - h * CH;
        const int64_t off = (int64_t)h * HEAD_BYTES + c * 16;
        u32x4 x1 = ld16(ksrc + off), x2 = ld16(ksrc + off + CH * 16);
        float2 cs[NP];
#pragma unroll
        for (int w = 0; w < NP; ++w) {
            const float2 hi = p.tab_hi[(int64_t)(a >> kRopeLoBits) * HALF + c * NP + w];
            const float2 lo = p.tab_lo[(a & (kRopeLo - 1)) * HALF + c * NP + w];
            cs[w] = make_float2(hi.x * lo.x - hi.y * lo.y, hi.y * lo.x + hi.x * lo.y);
        }
        rotate_chunks<DTYPE>(x1, x2, cs);
        st16<false>(kdst + off, x1);
        st16<false>(kdst + off + CH * 16, x2);
        st16<false>(vdst + off, ld16(vsrc + off));
        st16<false>(vdst + off + CH * 16, ld16(vsrc + off + CH * 16));
    }
}

template <int DTYPE, int CH>
static hipError_t launch_decode_t(const DecodeAppendParams& p, hipStream_t stream) {
    launch_kernel((decode_append_kernel<DTYPE, CH>), dim3((unsigned)p.count, (unsigned)p.n_layers), dim3(128), stream, p);
    return hipGetLastError();
}

hipError_t launch_decode_append(const DecodeAppendParams& p, hipStream_t stream) {
    const int e = p.dtype == ADAPSHOT_BF16 ? 2 : 4;
    const int ch = p.head_dim / 2 * e / 16;
    if (p.count <= 0) return hipSuccess;
    if (p.dtype == ADAPSHOT_BF16) {
        switch (ch) {
            case 1: return launch_decode_t<ADAPSHOT_BF16, 1>(p, stream);
            case 2: return launch_decode_t<ADAPSHOT_BF16, 2>(p, stream);
            case 4: return launch_decode_t<ADAPSHOT_BF16, 4>(p, stream);
            case 8: return launch_decode_t<ADAPSHOT_BF16, 8>(p, stream);
            case 16: return launch_decode_t<ADAPSHOT_BF16, 16>(p, stream);
        }
    } else {
        switch (ch) {
            case 1: return launch_decode_t<ADAPSHOT_F32, 1>(p, stream);
            case 2: return launch_decode_t<ADAPSHOT_F32, 2>(p, stream);
            case 4: return launch_decode_t<ADAPSHOT_F32, 4>(p, stream);
            case 8: return launch_decode_t<ADAPSHOT_F32, 8>(p, stream);
            case 16: return launch_decode_t<ADAPSHOT_F32, 16>(p, stream);
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace adapshot
