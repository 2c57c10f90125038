// bf16 MFMA query-over-cache attention for head_dim 128 (split-K, flash style).
//
// The probe/query rows of one KV head (all g query heads of its group packed as rows
// j*g + h%g) attend over a slice of the assembled cache; Eq. (attention_score) gives the
// 1/sqrt(d) scale, folded with log2(e) into q by rope_rows, so p = 2^(s - m).
//
// Work decomposition: workgroup = (kv head, tile of 128*NR rows, split of the context);
// 4 wavefronts, each owning 32*NR rows for the whole key loop.  The extra split index
// n_split is the causal part over the query's own tokens.
//
// Everything is computed TRANSPOSED so that a query row lives in one lane column:
//   S^T = K . Q^T   A = K tile from LDS (16-byte reads), B = Q fragments held in registers;
//                   v_mfma_f32_32x32x16_bf16 leaves lane l with row (l % 32) and 16 keys;
//   softmax         per-lane max/sum over its 32 keys of the tile, one exchange with lane^32;
//                   the rescale factor is a per-lane scalar for the O^T accumulators;
//   O^T += V^T . P^T  B = P^T straight from the S^T registers (rounded to bf16), A = V^T read
//                   from the row-major V tile in LDS with the transposing ds_read_b64_tr_b16.
// The k-slot order of the second product is the key order the S^T registers already have:
// slot 8*(l/32)+e of 16-key step ks  <->  key 16*ks + 8*(e/4) + 4*(l/32) + e%4.
#include "adapshot_internal.h"

namespace adapshot {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;             // head_dim
constexpr int kTileKeys = 64;
constexpr int kKStride = 272;       // bytes per K row in LDS: 256 + 16 (16-byte reads of 16 rows hit 16 bank groups)
constexpr int kVStride = 320;       // bytes per V row in LDS: 4 rows x 64 B of a transposing read tile all 64 banks
constexpr int kKBytes = kTileKeys * kKStride;
constexpr int kVBytes = kTileKeys * kVStride;

bool attn_mfma_supported(const adapshot_model_desc& d) { return d.dtype == ADAPSHOT_BF16 && d.head_dim == kD; }

__device__ __forceinline__ float xchg32(float v) {
    // value held by lane ^ 32
    return __shfl_xor(v, 32, 64);
}

__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(unsigned, b);
}

template <int NR>
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnParams p, int n_row_tiles) {
    __shared__ __attribute__((aligned(16))) char k_s[kKBytes];
    __shared__ __attribute__((aligned(16))) char v_s[kVBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int hh = lane >> 5;

    // blockIdx.x -> (kv head fastest: workgroups round-robin over the 8 XCDs, so with 8 kv heads every
    // XCD's L2 sees the K/V of one head only), row tile, split
    const int hk = blockIdx.x % p.n_kv_heads;
    const int rest = blockIdx.x / p.n_kv_heads;
    const int row_tile = rest % n_row_tiles;
    const int split = rest / n_row_tiles;
    const bool self = split == p.n_split;

    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int row0 = row_tile * (128 * NR) + wave * (32 * NR);

    // ---- Q fragments (B operand): lane holds row l32, d = 16*kk + 8*hh .. +7
    bf16x8 qf[NR][8];
    int jrow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int row = row0 + 32 * rb + l32;
        const bool valid = row < rows;
        const int j = valid ? row / g : 0;
        const int gq = valid ? row - j * g : 0;
        jrow[rb] = valid ? j : 0x7fffffff;
        const char* qrow = (const char*)p.q_rot + ((int64_t)(j * p.n_q_heads + hk * g + gq) * kD) * 2;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (valid) w = *(const u32x4*)(qrow + (16 * kk + 8 * hh) * 2);
            qf[rb][kk] = __builtin_bit_cast(bf16x8, w);
        }
    }

    // ---- key range of this split
    const char* kbase = (const char*)(self ? p.k_self_rot : p.k_cache) + hk * (kD * 2);
    const char* vbase = (const char*)(self ? p.v_self : p.v_cache) + hk * (kD * 2);
    const int64_t kv_stride = (int64_t)p.n_kv_heads * (kD * 2);
    const int64_t k0 = self ? 0 : (int64_t)split * p.keys_per_split;
    const int64_t k1 = self ? (int64_t)p.t_q : (k0 + p.keys_per_split < p.n_ctx ? k0 + p.keys_per_split : p.n_ctx);
    const int n_tiles = (int)((k1 - k0 + kTileKeys - 1) / kTileKeys);

    f32x16 o[4][NR];
    float m_run[NR], l_run[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][rb][r] = 0.f;
    }

    // ---- global -> register prefetch of one 64-key tile (rows clamped to the last valid key)
    const int ld_row = tid >> 4;   // 0..15
    const int ld_chunk = tid & 15; // 16-byte chunk of the 256-byte row
    u32x4 kreg[4], vreg[4];
    auto prefetch = [&](int t) {
#pragma unroll
        for (int ps = 0; ps < 4; ++ps) {
            int64_t key = k0 + (int64_t)t * kTileKeys + 16 * ps + ld_row;
            key = key < k1 ? key : k1 - 1;
            const int64_t off = key * kv_stride + ld_chunk * 16;
            kreg[ps] = *(const u32x4*)(kbase + off);
            vreg[ps] = *(const u32x4*)(vbase + off);
        }
    };
    if (n_tiles > 0) prefetch(0);

    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();  // all waves are done reading the previous tile
#pragma unroll
        for (int ps = 0; ps < 4; ++ps) {
            *(u32x4*)(k_s + (16 * ps + ld_row) * kKStride + ld_chunk * 16) = kreg[ps];
            *(u32x4*)(v_s + (16 * ps + ld_row) * kVStride + ld_chunk * 16) = vreg[ps];
        }
        __syncthreads();
        if (t + 1 < n_tiles) prefetch(t + 1);

        // ---- S^T = K . Q^T : s[kb][rb], lane: row l32, keys 32*kb + 8*(r/4) + 4*hh + r%4
        f32x16 s[2][NR];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int rb = 0; rb < NR; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][rb][r] = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const u32x4 aw = *(const u32x4*)(k_s + (32 * kb + l32) * kKStride + 32 * kk + 16 * hh);
                const bf16x8 a = __builtin_bit_cast(bf16x8, aw);
#pragma unroll
                for (int rb = 0; rb < NR; ++rb)
                    s[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], s[kb][rb], 0, 0, 0);
            }

        // ---- masks: keys past the end of the split; causal part over the query's own tokens
        const int64_t tile_k0 = k0 + (int64_t)t * kTileKeys;
        if (self || tile_k0 + kTileKeys > k1) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t key = tile_k0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
#pragma unroll
                    for (int rb = 0; rb < NR; ++rb) {
                        const bool vis = key < k1 && (!self || key <= (int64_t)jrow[rb]);
                        if (!vis) s[kb][rb][r] = -INFINITY;
                    }
                }
        }

        // ---- online softmax per row block
#pragma unroll
        for (int rb = 0; rb < NR; ++rb) {
            float mx = s[0][rb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][rb][r]);
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][rb][r]);
            mx = fmaxf(mx, xchg32(mx));
            const float m_new = fmaxf(m_run[rb], mx);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;  // fully masked so far: p = 0, no NaN
            const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_use);
            m_run[rb] = m_new;
            float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = __builtin_amdgcn_exp2f(s[kb][rb][r] - m_use);
                    s[kb][rb][r] = e;
                    sum += e;
                }
            l_run[rb] = l_run[rb] * alpha + sum;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][rb][r] *= alpha;
            }
        }

        // ---- O^T += V^T . P^T
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 pb[NR];
#pragma unroll
            for (int rb = 0; rb < NR; ++rb) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] = pack2_bf16(s[ks >> 1][rb][8 * (ks & 1) + 2 * e], s[ks >> 1][rb][8 * (ks & 1) + 2 * e + 1]);
                pb[rb] = __builtin_bit_cast(bf16x8, w);
            }
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                // transposing read: 16-lane group i -> row kbase + i/4, 4 columns at dbase + 4*(i%4);
                // lane i receives column dbase + i of rows kbase .. kbase+3
                const int i16 = lane & 15;
                const int krow = 16 * ks + 4 * hh + (i16 >> 2);
                const int dcol = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
                const char* va = v_s + krow * kVStride + dcol * 2;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(va));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4*)(va + 8 * kVStride));
                const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                for (int rb = 0; rb < NR; ++rb)
                    o[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[rb], o[db][rb], 0, 0, 0);
            }
        }
    }

    // ---- partials: unnormalised O (row-major [row][d]), running max and sum
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        const int row = row0 + 32 * rb + l32;
        const float l_tot = l_run[rb] + xchg32(l_run[rb]);
        if (row < rows) {
            const int64_t pr = ((int64_t)split * p.n_kv_heads + hk) * rows + row;
            if (hh == 0) p.part_ml[pr] = make_float2(m_run[rb], l_tot);
            float* orow = p.part_o + pr * kD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    f32x4 w = {o[db][rb][4 * rq], o[db][rb][4 * rq + 1], o[db][rb][4 * rq + 2], o[db][rb][4 * rq + 3]};
                    *(f32x4*)(orow + 32 * db + 8 * rq + 4 * hh) = w;
                }
        }
    }
}

hipError_t launch_attn_mfma(const AttnParams& p, hipStream_t stream) {
    constexpr int NR = 1;
    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int n_row_tiles = (rows + 128 * NR - 1) / (128 * NR);
    const unsigned blocks = (unsigned)(p.n_kv_heads * n_row_tiles * (p.n_split + 1));
    hipLaunchKernelGGL((attn_mfma_kernel<NR>), dim3(blocks), dim3(256), 0, stream, p, n_row_tiles);
    return hipGetLastError();
}

}  // namespace adapshot
