// bf16 MFMA query-over-cache attention for head_dim 128 (split-K, flash style).
//
// The probe/query rows of one KV head (all g query heads of its group packed as rows
// j*g + h%g) attend over a slice of the assembled cache; Eq. (attention_score) gives the
// 1/sqrt(d) scale, folded with log2(e) into q by rope_rows, so p = 2^(s - m).
//
// Work decomposition: workgroup = (kv head, tile of 256 rows, split of the context);
// 8 wavefronts, each owning 32 rows for the whole key loop.  The extra split index
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
#include <stdio.h>

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

// ---- LDS fragment reads --------------------------------------------------------------------
// K fragment (A operand of S^T): key row 32*kb + l32, 16 bytes at d = 16*kk + 8*hh.
__device__ __forceinline__ bf16x8 k_frag(const char* kt, int l32, int hh, int kb, int kk) {
    const u32x4 w = *(const u32x4*)(kt + (32 * kb + l32) * kKStride + 32 * kk + 16 * hh);
    return __builtin_bit_cast(bf16x8, w);
}
// V^T fragment (A operand of O^T): two transposing reads.  In a 16-lane group, lane i addresses row
// kbase + i/4, 4 columns at dbase + 4*(i%4), and receives column dbase + i of rows kbase .. kbase+3.
__device__ __forceinline__ bf16x8 v_frag(const char* vt, int lane, int hh, int ks, int db) {
#ifdef ADAPSHOT_EXPERIMENT_VT
    const u32x4 w = *(const u32x4*)(vt + ks * 4096 + (32 * db + (lane & 31)) * 32 + hh * 16);
    return __builtin_bit_cast(bf16x8, w);
#endif
    const int i16 = lane & 15;
    const int krow = 16 * ks + 4 * hh + (i16 >> 2);
    const int dcol = 32 * db + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
    const char* va = vt + krow * kVStride + dcol * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(va));
    const s16x4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(va + 8 * kVStride));
    const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, av);
}

// 8 wavefronts of 32 rows each, two per SIMD, run as two groups (waves 0-3 and 4-7) that are kept
// one phase apart: a wave alternates an MFMA phase M_t = { O^T += V^T P^T of tile t-1 ; S^T of tile t }
// with a softmax phase V_t on the VALU, with a workgroup barrier after every phase, and group B
// starts one barrier late -- so while one wave of a SIMD feeds the matrix core the other one runs
// its exponentials.  K and V tiles are double buffered in LDS; M_t also moves K(t+1) and V(t) from
// registers into LDS and starts the global loads of K(t+2) and V(t+1).
#ifdef ADAPSHOT_EXPERIMENT_TIMING
#define TSTAMP(slot)                                                                      \
    do {                                                                                  \
        if (blockIdx.x == 40 && lane == 0 && (wave == 0 || wave == 4) && (slot) < 256)     \
            dbg[(wave ? 256 : 0) + (slot)] = __builtin_readcyclecounter();                \
    } while (0)
#else
#define TSTAMP(slot)
#endif

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void attn_mfma_kernel(AttnParams p, int n_row_tiles
#ifdef ADAPSHOT_EXPERIMENT_TIMING
                                                               , unsigned long long* dbg
#endif
) {
    constexpr int THREADS = WAVES * 64;
    constexpr int PASSES = (kTileKeys * 16) / THREADS;  // 16-byte chunks of a tile per thread
    static_assert(PASSES * THREADS == kTileKeys * 16, "tile must divide over the threads");
    __shared__ __attribute__((aligned(16))) char k_s[2][kKBytes];
    __shared__ __attribute__((aligned(16))) char v_s[2][kVBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l32 = lane & 31;
    const int hh = lane >> 5;
    TSTAMP(240);
    const bool group_b = wave >= WAVES / 2;

    // blockIdx.x -> (kv head fastest: workgroups round-robin over the 8 XCDs, so with 8 kv heads every
    // XCD's L2 sees the K/V of one head only), row tile, split
    const int hk = blockIdx.x % p.n_kv_heads;
    const int rest = blockIdx.x / p.n_kv_heads;
    const int row_tile = rest % n_row_tiles;
    const int split = rest / n_row_tiles;
    const bool self = split == p.n_split;

    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int row = row_tile * (32 * WAVES) + wave * 32 + l32;
    const bool row_valid = row < rows;
    const int jrow = row_valid ? row / g : 0x7fffffff;

    // ---- Q fragments (B operand): lane holds row l32, d = 16*kk + 8*hh .. +7
    bf16x8 qf[8];
    {
        const int j = row_valid ? jrow : 0;
        const int gq = row_valid ? row - j * g : 0;
        const char* qrow = (const char*)p.q_rot + ((int64_t)(j * p.n_q_heads + hk * g + gq) * kD) * 2;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (row_valid) w = *(const u32x4*)(qrow + (16 * kk + 8 * hh) * 2);
            qf[kk] = __builtin_bit_cast(bf16x8, w);
        }
    }

    TSTAMP(241);
    // ---- key range of this split
    const char* kbase = (const char*)(self ? p.k_self_rot : p.k_cache) + hk * (kD * 2);
    const char* vbase = (const char*)(self ? p.v_self : p.v_cache) + hk * (kD * 2);
    const int64_t kv_stride = (int64_t)p.n_kv_heads * (kD * 2);
    const int64_t k0 = self ? 0 : (int64_t)split * p.keys_per_split;
    const int64_t k1 = self ? (int64_t)p.t_q : (k0 + p.keys_per_split < p.n_ctx ? k0 + p.keys_per_split : p.n_ctx);
    const int n_tiles = (int)((k1 - k0 + kTileKeys - 1) / kTileKeys);  // >= 1

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_run = -INFINITY;  // reference maximum of the exponentials (log2 units); may lag the true maximum by < 8
    float l_run = 0.f;        // this lane's share of the row sum

    // ---- global -> register -> LDS staging of 64-key tiles (rows clamped to the last valid key)
    u32x4 kreg[PASSES], vreg[PASSES];
    auto gload = [&](const char* base, int t, u32x4(&reg)[PASSES]) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int c = ps * THREADS + tid;
            int64_t key = k0 + (int64_t)t * kTileKeys + (c >> 4);
            key = key < k1 ? key : k1 - 1;
            reg[ps] = *(const u32x4*)(base + key * kv_stride + (c & 15) * 16);
        }
    };
    auto stage = [&](char* buf, int stride, const u32x4(&reg)[PASSES]) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int c = ps * THREADS + tid;
            *(u32x4*)(buf + (c >> 4) * stride + (c & 15) * 16) = reg[ps];
        }
    };

    gload(kbase, 0, kreg);
    stage(k_s[0], kKStride, kreg);
    gload(vbase, 0, vreg);
    if (n_tiles > 1) gload(kbase, 1, kreg);
    TSTAMP(242);
    __syncthreads();
    TSTAMP(243);
    if (group_b) __syncthreads();  // group B runs one phase behind group A

    f32x16 s[2];
    bf16x8 pb[4];  // P^T of the previous tile, one B operand per 16-key step

    // K(t+1) and V(t) move from registers to the buffers nobody reads in this or the next phase;
    // then the loads of K(t+2) and V(t+1) start (two phases of latency cover)
    auto stage_and_load = [&](int t) {
        if (t + 1 < n_tiles) stage(k_s[(t + 1) & 1], kKStride, kreg);
        stage(v_s[t & 1], kVStride, vreg);
#ifndef ADAPSHOT_EXPERIMENT_NO_GLOAD
        if (t + 2 < n_tiles) gload(kbase, t + 2, kreg);
        if (t + 1 < n_tiles) gload(vbase, t + 1, vreg);
#endif
    };
    auto zero_s = [&]() {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
    };
    // V_t: masks and online softmax on the VALU; leaves P^T(t) in pb
    auto softmax_phase = [&](int t) {
        const int64_t tile_k0 = k0 + (int64_t)t * kTileKeys;
        if (self || tile_k0 + kTileKeys > k1) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t key = tile_k0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const bool vis = key < k1 && (!self || key <= (int64_t)jrow);
                    if (!vis) s[kb][r] = -INFINITY;
                }
        }
        float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
        mx = fmaxf(mx, xchg32(mx));
        if (__builtin_amdgcn_ballot_w64(mx > m_run + 8.0f || (m_run == -INFINITY && mx > -INFINITY))) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        }
        const float m_use = m_run == -INFINITY ? 0.f : m_run;  // nothing visible yet: p = 2^(-inf) = 0
        float sum = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float e0 = __builtin_amdgcn_exp2f(s[ks >> 1][8 * (ks & 1) + 2 * e] - m_use);
                const float e1 = __builtin_amdgcn_exp2f(s[ks >> 1][8 * (ks & 1) + 2 * e + 1] - m_use);
                sum += e0 + e1;
                w[e] = pack2_bf16(e0, e1);
            }
            pb[ks] = __builtin_bit_cast(bf16x8, w);
        }
        l_run += sum;
    };

    // =========================== M_0: S(0) only
    {
        const char* kt = k_s[0];
        zero_s();
        bf16x8 fr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fr[i] = k_frag(kt, l32, hh, i & 1, i >> 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const bf16x8 a = fr[i & 3];
            if (i + 4 < 16) fr[i & 3] = k_frag(kt, l32, hh, (i + 4) & 1, (i + 4) >> 1);
            s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[i >> 1], s[i & 1], 0, 0, 0);
        }
        stage_and_load(0);
        __syncthreads();
        softmax_phase(0);
        __syncthreads();
    }
    TSTAMP(0);

    for (int t = 1; t < n_tiles; ++t) {
        // =========================== M_t: PV(t-1) and S(t) on the matrix core: 32 MFMAs alternating the
        // two products; operand fragments are read from LDS 4 steps ahead
        const char* kt = k_s[t & 1];
        const char* vt = v_s[(t + 1) & 1];  // tile t-1
        {
            f32x16 sn[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sn[kb][r] = 0.f;
            bf16x8 fr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                fr[i] = (i & 1) ? k_frag(kt, l32, hh, (i >> 1) & 1, i >> 2) : v_frag(vt, lane, hh, i >> 3, (i >> 1) & 3);
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int u = i >> 1;  // PV: ks = u/4, db = u%4;  S: kk = u/2, kb = u%2
                const bf16x8 a = fr[i & 3];
                if (i + 4 < 32) {
                    const int n = i + 4, un = n >> 1;
                    fr[i & 3] = (n & 1) ? k_frag(kt, l32, hh, un & 1, un >> 1) : v_frag(vt, lane, hh, un >> 2, un & 3);
                }
                if (i & 1)
                    sn[u & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[u >> 1], sn[u & 1], 0, 0, 0);
                else
                    o[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[u >> 2], o[u & 3], 0, 0, 0);
            }
            s[0] = sn[0];
            s[1] = sn[1];
        }
        TSTAMP(4 * t + 0);
        stage_and_load(t);
        TSTAMP(4 * t + 1);
        __syncthreads();
        TSTAMP(4 * t + 2);
        softmax_phase(t);
        TSTAMP(4 * t + 3);
        __syncthreads();
        TSTAMP(4 * t + 4);
    }

    // =========================== M_n: PV(n-1) only
    {
        const char* vt = v_s[(n_tiles + 1) & 1];
        bf16x8 fr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fr[i] = v_frag(vt, lane, hh, i >> 2, i & 3);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const bf16x8 a = fr[i & 3];
            if (i + 4 < 16) fr[i & 3] = v_frag(vt, lane, hh, (i + 4) >> 2, (i + 4) & 3);
            o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[i >> 2], o[i & 3], 0, 0, 0);
        }
        __syncthreads();
    }
    TSTAMP(244);
    if (!group_b) __syncthreads();  // every wave passes the same number of barriers

    // ---- partials: unnormalised O (row-major [row][d]), reference maximum and row sum
    const float l_tot = l_run + xchg32(l_run);
    if (row_valid) {
        const int64_t pr = ((int64_t)split * p.n_kv_heads + hk) * rows + row;
        if (hh == 0) p.part_ml[pr] = make_float2(m_run, l_tot);
        float* orow = p.part_o + pr * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                f32x4 w = {o[db][4 * rq], o[db][4 * rq + 1], o[db][4 * rq + 2], o[db][4 * rq + 3]};
                *(f32x4*)(orow + 32 * db + 8 * rq + 4 * hh) = w;
            }
    }
#ifdef ADAPSHOT_EXPERIMENT_TIMING
    __builtin_amdgcn_s_waitcnt(0);
#endif
    TSTAMP(245);
}

hipError_t launch_attn_mfma(const AttnParams& p, hipStream_t stream) {
    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int n_row_tiles = (rows + kAttnRowTile - 1) / kAttnRowTile;
    const unsigned blocks = (unsigned)(p.n_kv_heads * n_row_tiles * (p.n_split + 1));
#ifdef ADAPSHOT_EXPERIMENT_TIMING
    static unsigned long long* dbg = nullptr;
    if (!dbg) { (void)hipMalloc(&dbg, 512 * 8); (void)hipMemset(dbg, 0, 512 * 8); }
    hipLaunchKernelGGL((attn_mfma_kernel<kAttnRowTile / 32>), dim3(blocks), dim3(kAttnRowTile * 2), 0, stream, p,
                       n_row_tiles, dbg);
    (void)hipDeviceSynchronize();
    unsigned long long h[512];
    (void)hipMemcpy(h, dbg, sizeof h, hipMemcpyDeviceToHost);
    static int once = 0;
    if (!once++) {
        for (int w = 0; w < 2; ++w) {
            printf("wave %d:", w * 4);
            for (int i = 5; i < 14; ++i) printf(" %lld", (long long)(h[w * 256 + i] - h[w * 256 + 4]));
            printf("\n  coarse: qload %lld  k0stage %lld  barrier %lld  loop %lld  epilogue %lld\n",
                   (long long)(h[w * 256 + 241] - h[w * 256 + 240]), (long long)(h[w * 256 + 242] - h[w * 256 + 241]),
                   (long long)(h[w * 256 + 243] - h[w * 256 + 242]), (long long)(h[w * 256 + 244] - h[w * 256 + 243]),
                   (long long)(h[w * 256 + 245] - h[w * 256 + 244]));
        }
    }
#else
    hipLaunchKernelGGL((attn_mfma_kernel<kAttnRowTile / 32>), dim3(blocks), dim3(kAttnRowTile * 2), 0, stream, p,
                       n_row_tiles);
#endif
    return hipGetLastError();
}

}  // namespace adapshot
