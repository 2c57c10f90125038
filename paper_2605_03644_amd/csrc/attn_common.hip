// Query-over-cache attention, the parts shared by every shape:
//   rope_rows     -- rotate the probe/query rows and their own keys to positions
//                    q_pos0 + j (Eq. rope_encoding) and fold the softmax scale
//                    log2(e)/sqrt(d) (Eq. attention_score's 1/sqrt(d)) into q, for the
//                    generic kernel (the MFMA kernel rotates its rows itself);
//   attn_generic  -- a straightforward fp32 split-K kernel (one wavefront per query
//                    row, head and split) used for fp32 models and for shapes the
//                    MFMA kernel does not cover;
//   attn_combine  -- merges the per-split (max, sum, unnormalised output) partials.
#include <algorithm>
#include <type_traits>

#include "adapshot_internal.h"

namespace adapshot {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int DTYPE>
__device__ __forceinline__ float load_elem(const void* base, int64_t i) {
    if (DTYPE == ADAPSHOT_BF16) return __uint_as_float(((unsigned)((const unsigned short*)base)[i]) << 16);
    return ((const float*)base)[i];
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
    __bf16 b = (__bf16)f;
    return __builtin_bit_cast(unsigned short, b);
}

template <int DTYPE>
__device__ __forceinline__ void store_elem(void* base, int64_t i, float v) {
    if (DTYPE == ADAPSHOT_BF16) ((unsigned short*)base)[i] = f32_to_bf16_rne(v);
    else ((float*)base)[i] = v;
}

// ---- rope_rows ----------------------------------------------------------------------
// One thread per pair of 16-byte chunks holding rotation partners (i, i + d/2), i = NP*ci .. NP*ci + NP - 1.
// Rows 0..t_q*h_q-1 are query rows, the rest self-key rows.
template <int DTYPE>
__device__ __forceinline__ void rope_rows_block(const RopeRowsParams& p, int64_t block) {
    constexpr int NP = DTYPE == ADAPSHOT_BF16 ? 8 : 4;  // pairs per chunk
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const int half = p.head_dim >> 1;
    const int cpr = half / NP;  // chunk pairs per row
    const int64_t n_q = (int64_t)p.t_q * p.n_q_heads;
    const int64_t n_k = p.k_self ? (int64_t)p.t_q * p.n_kv_heads : 0;  // ranking rotates the query only
    const int64_t idx = block * 256 + threadIdx.x;
    if (idx >= (n_q + n_k) * cpr) return;
    const int64_t row = idx / cpr;
    const int ci = (int)(idx - row * cpr);
    const bool is_q = row < n_q;
    const int64_t r = is_q ? row : row - n_q;
    const int j = (int)(r / (is_q ? p.n_q_heads : p.n_kv_heads));
    const int64_t a = p.q_pos0 + j;
    const float2* th = p.tab_hi + (a >> kRopeLoBits) * half + ci * NP;
    const float2* tl = p.tab_lo + (a & (kRopeLo - 1)) * half + ci * NP;
    const char* src = (const char*)(is_q ? p.q : p.k_self);
    char* dst = (char*)(is_q ? p.q_rot : p.k_rot);
    const int64_t o = (r * p.head_dim + ci * NP) * (DTYPE == ADAPSHOT_BF16 ? 2 : 4);
    const int64_t ho = (int64_t)half * (DTYPE == ADAPSHOT_BF16 ? 2 : 4);
    u32x4 x1 = *(const u32x4*)(src + o), x2 = *(const u32x4*)(src + o + ho);
    const float sc = is_q ? p.q_scale : 1.0f;
    float y1[NP], y2[NP];
#pragma unroll
    for (int w = 0; w < NP; ++w) {
        const float2 h = th[w], l = tl[w];
        const float c = h.x * l.x - h.y * l.y;
        const float s = h.y * l.x + h.x * l.y;
        float a1, a2;
        if (DTYPE == ADAPSHOT_BF16) {
            const unsigned w1 = x1[w >> 1], w2 = x2[w >> 1];
            a1 = (w & 1) ? __uint_as_float(w1 & 0xffff0000u) : __uint_as_float(w1 << 16);
            a2 = (w & 1) ? __uint_as_float(w2 & 0xffff0000u) : __uint_as_float(w2 << 16);
        } else {
            a1 = __uint_as_float(x1[w]);
            a2 = __uint_as_float(x2[w]);
        }
        y1[w] = (a1 * c - a2 * s) * sc;
        y2[w] = (a2 * c + a1 * s) * sc;
    }
    if (DTYPE == ADAPSHOT_BF16) {
#pragma unroll
        for (int w = 0; w < NP; w += 2) {
            x1[w >> 1] = (unsigned)f32_to_bf16_rne(y1[w]) | ((unsigned)f32_to_bf16_rne(y1[w + 1]) << 16);
            x2[w >> 1] = (unsigned)f32_to_bf16_rne(y2[w]) | ((unsigned)f32_to_bf16_rne(y2[w + 1]) << 16);
        }
    } else {
#pragma unroll
        for (int w = 0; w < NP; ++w) {
            x1[w] = __float_as_uint(y1[w]);
            x2[w] = __float_as_uint(y2[w]);
        }
    }
    *(u32x4*)(dst + o) = x1;
    *(u32x4*)(dst + o + ho) = x2;
}

template <int DTYPE>
__global__ __launch_bounds__(256) void rope_rows_kernel(RopeRowsParams p) {
    rope_rows_block<DTYPE>(p, blockIdx.x);
}

hipError_t launch_rope_rows(const RopeRowsParams& p, hipStream_t stream) {
    const int np = p.dtype == ADAPSHOT_BF16 ? 8 : 4;
    const int64_t n = (int64_t)p.t_q * (p.n_q_heads + (p.k_self ? p.n_kv_heads : 0)) * (p.head_dim / 2 / np);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (p.dtype == ADAPSHOT_BF16)
        launch_kernel(rope_rows_kernel<ADAPSHOT_BF16>, dim3(blocks), dim3(256), stream, p);
    else
        launch_kernel(rope_rows_kernel<ADAPSHOT_F32>, dim3(blocks), dim3(256), stream, p);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_table_kernel(u32x4_t* dst, const u32x4_t* src, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy_table(void* dst, const void* src_pinned, size_t bytes, hipStream_t stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 512);
    launch_kernel(copy_table_kernel, dim3(blocks), dim3(256), stream, (u32x4_t*)dst, (const u32x4_t*)src_pinned, n16);
    return hipGetLastError();
}

// ---- plan of a zero-copy context ----------------------------------------------------------
// Blocks 0 .. n_segs-1 expand one shot each into slot_src (context slot -> pool token); the blocks after them
// form tile_rot[i][f] = (cos, sin)((pos0 + 64 i) theta_f) for every 64-slot tile, one fp32 angle addition of the
// two fp64-built table entries.
__global__ __launch_bounds__(256) void pool_plan_kernel(PoolPlanParams p) {
    if ((int)blockIdx.x < p.n_segs) {
        const PoolSeg sg = p.segs[blockIdx.x];
        for (int t = threadIdx.x; t < sg.len; t += 256) p.slot_src[sg.slot0 + t] = sg.src_tok0 + t;
        return;
    }
    const int half = p.head_dim >> 1;
    const int64_t idx = (int64_t)(blockIdx.x - p.n_segs) * 256 + threadIdx.x;
    if (idx >= (int64_t)p.n_tiles * half) return;
    const int64_t tile = idx / half;
    const int f = (int)(idx - tile * half);
    const int64_t a = p.pos0 + tile * 64;
    const float2 h = p.tab_hi[(a >> kRopeLoBits) * half + f], l = p.tab_lo[(a & (kRopeLo - 1)) * half + f];
    p.tile_rot[idx] = make_float2(h.x * l.x - h.y * l.y, h.y * l.x + h.x * l.y);
}

hipError_t launch_pool_plan(const PoolPlanParams& p, hipStream_t stream) {
    const int64_t rot_blocks = ((int64_t)p.n_tiles * (p.head_dim / 2) + 255) / 256;
    const int64_t blocks = p.n_segs + rot_blocks;
    if (blocks <= 0) return hipSuccess;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    launch_kernel(pool_plan_kernel, dim3((unsigned)blocks), dim3(256), stream, p);
    return hipGetLastError();
}

// ---- wavefront reductions --------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---- generic fp32 kernel -----------------------------------------------------------------
// grid = (t_q * h_q, n_split + 1); one wavefront each.  Lanes run over 64 keys for the
// scores and over the head dimension for p.v.  Works in log2 units: q is pre-scaled by
// log2(e)/sqrt(d), so p = 2^(s - m).
// With pool.slot_src given (zero-copy form) the context is one layer of the POOL: slot u holds pool token
// slot_src[u], and its key is rotated to position pos0 + u on the way into the score (Eq. rope_compensation;
// rounded to the storage type, as the assembled cache would hold it).
template <int DTYPE>
__global__ __launch_bounds__(64) void attn_generic_kernel(AttnParams p, GenericPool pool) {
    __shared__ float q_s[256];
    __shared__ float p_s[64];
    __shared__ int tok_s[64];
    const int lane = threadIdx.x;
    const int d = p.head_dim;
    const int g = p.n_q_heads / p.n_kv_heads;
    const int j = blockIdx.x / p.n_q_heads;
    const int h = blockIdx.x - j * p.n_q_heads;
    const int hk = h / g;
    const int split = blockIdx.y;
    const bool self = split == p.n_split;
    const int64_t rows = (int64_t)p.t_q * g;
    const int64_t row = (int64_t)j * g + (h - hk * g);

    for (int e = lane; e < d; e += 64) q_s[e] = load_elem<DTYPE>(p.q_rot, ((int64_t)j * p.n_q_heads + h) * d + e);
    __syncthreads();

    const void* kbase = self ? p.k_self_rot : p.k_cache;
    const void* vbase = self ? p.v_self : p.v_cache;
    int64_t k0 = self ? 0 : (int64_t)split * p.keys_per_split;
    int64_t k1 = self ? (int64_t)j + 1 : (k0 + p.keys_per_split < p.n_ctx ? k0 + p.keys_per_split : p.n_ctx);

    float m = -INFINITY, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int64_t kb = k0; kb < k1; kb += 64) {
        const int64_t u = kb + lane;
        const bool gather = pool.slot_src && !self;
        float s = -INFINITY;
        if (u < k1) {
            const int64_t tok = gather ? (int64_t)pool.slot_src[u] : u;
            tok_s[lane] = (int)tok;
            const int64_t o = (tok * p.n_kv_heads + hk) * d;
            float dot = 0.f;
            if (gather) {
                const int half = d >> 1;
                const int64_t a = pool.pos0 + u;
                const float2* th = pool.tab_hi + (a >> kRopeLoBits) * half;
                const float2* tl = pool.tab_lo + (a & (kRopeLo - 1)) * half;
                for (int i = 0; i < half; ++i) {
                    const float2 hh = th[i], ll = tl[i];
                    const float c = hh.x * ll.x - hh.y * ll.y, sn = hh.y * ll.x + hh.x * ll.y;
                    const float x1 = load_elem<DTYPE>(kbase, o + i), x2 = load_elem<DTYPE>(kbase, o + i + half);
                    float y1 = x1 * c - x2 * sn, y2 = x2 * c + x1 * sn;
                    if (DTYPE == ADAPSHOT_BF16) {
                        y1 = __uint_as_float((unsigned)f32_to_bf16_rne(y1) << 16);
                        y2 = __uint_as_float((unsigned)f32_to_bf16_rne(y2) << 16);
                    }
                    dot += q_s[i] * y1 + q_s[i + half] * y2;
                }
            } else {
                for (int e = 0; e < d; ++e) dot += q_s[e] * load_elem<DTYPE>(kbase, o + e);
            }
            s = dot;
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float alpha = exp2f(m - m_new);  // m = -inf on the first block: 0
        const float pe = (u < k1) ? exp2f(s - m_new) : 0.f;
        l = l * alpha + wave_sum(pe);
        m = m_new;
        p_s[lane] = pe;
        __syncthreads();
        const int nk = (int)((k1 - kb) < 64 ? (k1 - kb) : 64);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int e = lane + 64 * c;
            if (e < d) {
                float a = acc[c] * alpha;
                for (int t = 0; t < nk; ++t)
                    a += p_s[t] * load_elem<DTYPE>(vbase, ((int64_t)(gather ? tok_s[t] : kb + t) * p.n_kv_heads + hk) * d + e);
                acc[c] = a;
            }
        }
        __syncthreads();
    }
    const int64_t pr = ((int64_t)split * p.n_kv_heads + hk) * rows + row;
    if (lane == 0) p.part_mlf[pr] = make_float4(m, l, 1.0f, 0.f);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int e = lane + 64 * c;
        if (e < d) ((float*)p.part_o)[pr * d + e] = acc[c];
    }
}

hipError_t launch_attn_generic(const AttnParams& p, const GenericPool& pool, hipStream_t stream) {
    dim3 grid((unsigned)(p.t_q * p.n_q_heads), (unsigned)(p.n_split + 1));
    if (p.dtype == ADAPSHOT_BF16)
        launch_kernel(attn_generic_kernel<ADAPSHOT_BF16>, grid, dim3(64), stream, p, pool);
    else
        launch_kernel(attn_generic_kernel<ADAPSHOT_F32>, grid, dim3(64), stream, p, pool);
    return hipGetLastError();
}

// ---- combine --------------------------------------------------------------------------------
// out = sum_s 2^(m_s - M) f_s O'_s / sum_s 2^(m_s - M) l_s with M = max_s m_s.  HBM-bound on the partials.
// Lanes per (kv head, row) pair and elements per lane and step: 32 x 4 fp32 or 16 x 8 fp16 (16 bytes per
// lane either way), so a workgroup of 256 lanes handles 8 or 16 pairs; the partial rows of 8 splits are
// requested together before any is used.  The self split always holds at least one visible key, so the
// denominator is > 0.
template <int DTYPE, bool HALF, int NV, int SB>
__device__ __forceinline__ void attn_combine_rows(const AttnParams& p, int64_t pair0) {
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    typedef float f32x8 __attribute__((ext_vector_type(8)));
    typedef typename std::conditional<HALF, f16x8, f32x4>::type ROW;  // 16 bytes of a partial row
    constexpr int LP = HALF ? 16 : 32;  // lanes per pair
    constexpr int EL = HALF ? 8 : 4;    // elements per lane and step; NV steps cover head_dim <= NV * 128
    const int d = p.head_dim;
    const int g = p.n_q_heads / p.n_kv_heads;
    const int64_t rows = (int64_t)p.t_q * g;
    const int64_t n_pairs = rows * p.n_kv_heads;
    const int64_t pair = pair0 + (threadIdx.x / LP);
    if (pair >= n_pairs) return;
    const int c = threadIdx.x % LP;
    const int hk = (int)(pair / rows);
    const int64_t row = pair - (int64_t)hk * rows;
    const int j = (int)(row / g);
    const int h = hk * g + (int)(row - (int64_t)j * g);
    const int ns = p.n_split + 1;
    const int64_t split_stride = (int64_t)p.n_kv_heads * rows;  // pairs per split
    const float4* mlf = p.part_mlf + pair;
    const char* po = (const char*)p.part_o + pair * d * (HALF ? 2 : 4);

    // One round of loads per SB splits: their (m, l, f) and their rows are requested together; the running
    // maximum M is raised afterwards and what has been accumulated is rescaled (nothing yet: factor 0).
    float M = -INFINITY, L = 0.f;
    f32x8 acc[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[v][i] = 0.f;
    for (int s0 = 0; s0 < ns; s0 += SB) {
        float4 mv[SB];
        ROW o[SB][NV];
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const bool on = s0 + u < ns;
            const int64_t so = (int64_t)(s0 + u) * split_stride;
            mv[u] = on ? mlf[so] : make_float4(-INFINITY, 0.f, 0.f, 0.f);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int e = EL * (c + LP * v);
#pragma unroll
                for (int i = 0; i < EL; ++i) o[u][v][i] = 0;
                if (on && e < d) o[u][v] = __builtin_nontemporal_load((const ROW*)(po + (so * d + e) * (HALF ? 2 : 4)));
            }
        }
        float cm = mv[0].x;
#pragma unroll
        for (int u = 1; u < SB; ++u) cm = fmaxf(cm, mv[u].x);
        const float M_new = fmaxf(M, cm);
        const float r = M == -INFINITY ? 0.f : exp2f(M - M_new);
        M = M_new;
        L *= r;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < EL; ++i) acc[v][i] *= r;
#pragma unroll
        for (int u = 0; u < SB; ++u) {
            const float w = mv[u].x == -INFINITY ? 0.f : exp2f(mv[u].x - M);  // empty or absent split: 0
            L += w * mv[u].y;
            const float wf = w * mv[u].z;
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int i = 0; i < EL; ++i) acc[v][i] += wf * (float)o[u][v][i];
        }
    }
    const float inv = 1.0f / L;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = EL * (c + LP * v);
        if (e < d) {
            const int64_t oo = ((int64_t)j * p.n_q_heads + h) * d + e;
            if (DTYPE == ADAPSHOT_BF16) {
                typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
                for (int q4 = 0; q4 < EL / 4; ++q4) {
                    const f32x4 r = {acc[v][4 * q4] * inv, acc[v][4 * q4 + 1] * inv, acc[v][4 * q4 + 2] * inv,
                                     acc[v][4 * q4 + 3] * inv};
                    *(bf16x4*)((unsigned short*)p.out + oo + 4 * q4) = __builtin_convertvector(r, bf16x4);
                }
            } else {
#pragma unroll
                for (int q4 = 0; q4 < EL / 4; ++q4) {
                    const f32x4 r = {acc[v][4 * q4] * inv, acc[v][4 * q4 + 1] * inv, acc[v][4 * q4 + 2] * inv,
                                     acc[v][4 * q4 + 3] * inv};
                    *(f32x4*)((float*)p.out + oo + 4 * q4) = r;
                }
            }
        }
    }
}

// One kernel per (row type, head width, splits in flight): the register count follows the splits in flight (16
// partial rows and their (m, l, f) are 128 registers), and a launch with thousands of workgroups -- the combine of
// a probe sweep -- lives on how many of them fit a compute unit (one kernel for all forms: 244 registers, two
// wavefronts per SIMD, 40 us for the sweep's 6144 workgroups).
// SB splits in flight: 8 when the problem has at most 8 partials per row, else 16 (fp16 rows) or 8 (fp32 rows).
template <int DTYPE, bool HALF, int NV, int SB>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnParams p) {
    attn_combine_rows<DTYPE, HALF, NV, SB>(p, (int64_t)blockIdx.x * (HALF ? 16 : 8));
}

template <int DTYPE, bool HALF, int NV, int SB>
__global__ __launch_bounds__(256) void attn_combine_batched_kernel(const AttnBatchItem* items, const CombineWork* work) {
    const CombineWork w = work[blockIdx.x];
    attn_combine_rows<DTYPE, HALF, NV, SB>(items[w.item].attn, w.pair0);
}

template <int DTYPE, bool HALF, int NV, int SB>
static void launch_combine_form(const AttnParams* p, const AttnBatchItem* items, const CombineWork* work, unsigned blocks,
                                hipStream_t stream) {
    if (p) launch_kernel((attn_combine_kernel<DTYPE, HALF, NV, SB>), dim3(blocks), dim3(256), stream, *p);
    else launch_kernel((attn_combine_batched_kernel<DTYPE, HALF, NV, SB>), dim3(blocks), dim3(256), stream, items, work);
}
template <int DTYPE>
static void launch_combine_dtype(const AttnParams* p, const AttnBatchItem* items, const CombineWork* work, unsigned blocks,
                                 bool half, bool wide, bool many, hipStream_t stream) {
    if (half) {
        if (many) {
            if (wide) launch_combine_form<DTYPE, true, 2, 16>(p, items, work, blocks, stream);
            else launch_combine_form<DTYPE, true, 1, 16>(p, items, work, blocks, stream);
        } else {
            if (wide) launch_combine_form<DTYPE, true, 2, 8>(p, items, work, blocks, stream);
            else launch_combine_form<DTYPE, true, 1, 8>(p, items, work, blocks, stream);
        }
    } else {
        if (wide) launch_combine_form<DTYPE, false, 2, 8>(p, items, work, blocks, stream);
        else launch_combine_form<DTYPE, false, 1, 8>(p, items, work, blocks, stream);
    }
}

hipError_t launch_attn_combine(const AttnParams& p, hipStream_t stream) {
    const int g = p.n_q_heads / p.n_kv_heads;
    const int64_t n_pairs = (int64_t)p.n_kv_heads * p.t_q * g;
    const int per_wg = p.part_half ? 16 : 8;
    const unsigned blocks = (unsigned)((n_pairs + per_wg - 1) / per_wg);
    const bool wide = p.head_dim > 128, many = p.n_split + 1 > 8;
    if (p.dtype == ADAPSHOT_BF16)
        launch_combine_dtype<ADAPSHOT_BF16>(&p, nullptr, nullptr, blocks, p.part_half != 0, wide, many, stream);
    else
        launch_combine_dtype<ADAPSHOT_F32>(&p, nullptr, nullptr, blocks, p.part_half != 0, wide, many, stream);
    return hipGetLastError();
}

// All items of a batch have fp16 partial rows of 128 columns (the matrix-core kernel's); max_partials is the largest
// number of partial rows that any item merges per output row.
hipError_t launch_attn_combine_batched(const AttnBatchItem* items, const CombineWork* work, int n_work, int dtype,
                                       int max_partials, hipStream_t stream) {
    if (n_work <= 0) return hipSuccess;
    if (dtype == ADAPSHOT_BF16)
        launch_combine_dtype<ADAPSHOT_BF16>(nullptr, items, work, (unsigned)n_work, true, false, max_partials > 8, stream);
    else
        launch_combine_dtype<ADAPSHOT_F32>(nullptr, items, work, (unsigned)n_work, true, false, max_partials > 8, stream);
    return hipGetLastError();
}

}  // namespace adapshot
