// Relevance ranking of the pool's shots for a query (Eq. attention_score, Attention-based retrieval).
//
// The attention itself runs in the MFMA kernel: keys = the locally encoded keys of every pool token at
// the representative layer, "values" = one-hot rows that mark each token's shot inside its window of at
// most head_dim consecutive shots, one context split per window, softmax normalised over the whole pool
// when the splits are merged.  This file holds what surrounds it:
//   rank_prepare   once per pool layer: rotate every key to its position inside its shot (a pool that
//                  stores un-rotated keys; Eq. prefill caches them encoded) and write the one-hot rows;
//   rank_weights   per (kv head, row): merge the splits' (m, l) into the row's global normaliser and
//                  leave  w[s][row] = f_s 2^(m_s - M) / L  for every split;
//   rank_reduce    per (window, block of 256 rows, shot slot): sum w[s][row] * O'[s][row][slot] over the
//                  block's rows into a partial;
//   rank_finish    per shot: add the row blocks' partials in a fixed order (the same query gives the same
//                  bits every time) and scale by 1 / (T_q H_q T_i).
#include "adapshot_internal.h"

namespace adapshot {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One thread per (token, kv head, chunk pair): bf16, 8 pairs per 16-byte chunk.
__global__ __launch_bounds__(256) void rank_prepare_kernel(RankPrepareParams p) {
    const int half = p.head_dim >> 1;
    const int cpr = half / 8;  // chunk pairs per head
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n = p.n_tok * p.n_kv_heads * cpr;
    if (idx >= n) return;
    const int ci = (int)(idx % cpr);
    const int64_t th = idx / cpr;
    const int hk = (int)(th % p.n_kv_heads);
    const int64_t u = th / p.n_kv_heads;
    const int64_t o = ((u * p.n_kv_heads + hk) * p.head_dim + ci * 8) * 2;
    const int64_t ho = (int64_t)half * 2;
    if (p.k_out) {
        const int a = p.tok_local[u];
        const float2* thi = p.tab_hi + (int64_t)(a >> kRopeLoBits) * half + ci * 8;
        const float2* tlo = p.tab_lo + (a & (kRopeLo - 1)) * half + ci * 8;
        u32x4 x1 = *(const u32x4*)(p.k_pool + o), x2 = *(const u32x4*)(p.k_pool + o + ho);
        float y1[8], y2[8];
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const float2 h = thi[w], l = tlo[w];
            const float c = h.x * l.x - h.y * l.y;
            const float s = h.y * l.x + h.x * l.y;
            const unsigned w1 = x1[w >> 1], w2 = x2[w >> 1];
            const float a1 = (w & 1) ? __uint_as_float(w1 & 0xffff0000u) : __uint_as_float(w1 << 16);
            const float a2 = (w & 1) ? __uint_as_float(w2 & 0xffff0000u) : __uint_as_float(w2 << 16);
            y1[w] = a1 * c - a2 * s;
            y2[w] = a2 * c + a1 * s;
        }
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int w = 0; w < 8; w += 2) {
            const f32x2 f1 = {y1[w], y1[w + 1]}, f2 = {y2[w], y2[w + 1]};
            x1[w >> 1] = __builtin_bit_cast(unsigned, __builtin_convertvector(f1, bf16x2));  // round to nearest even
            x2[w >> 1] = __builtin_bit_cast(unsigned, __builtin_convertvector(f2, bf16x2));
        }
        *(u32x4*)(p.k_out + o) = x1;
        *(u32x4*)(p.k_out + o + ho) = x2;
    }
    // one-hot row of this token (the same for every head): bf16 1.0 at column tok_col[u]
    const int col = p.tok_col[u];
    u32x4 z1 = {0u, 0u, 0u, 0u}, z2 = {0u, 0u, 0u, 0u};
    const int e1 = col - ci * 8, e2 = col - half - ci * 8;
    if (e1 >= 0 && e1 < 8) z1[e1 >> 1] = (e1 & 1) ? 0x3f800000u : 0x00003f80u;
    if (e2 >= 0 && e2 < 8) z2[e2 >> 1] = (e2 & 1) ? 0x3f800000u : 0x00003f80u;
    *(u32x4*)(p.v_out + o) = z1;
    *(u32x4*)(p.v_out + o + ho) = z2;
}

hipError_t launch_rank_prepare(const RankPrepareParams& p, hipStream_t stream) {
    const int64_t n = p.n_tok * p.n_kv_heads * (p.head_dim / 16);
    if (n <= 0) return hipSuccess;
    launch_kernel(rank_prepare_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), stream, p);
    return hipGetLastError();
}

// 16 lanes per (kv head, row) pair, lane sl taking splits sl, sl + 16, ...
__global__ __launch_bounds__(256) void rank_weights_kernel(RankReduceParams p) {
    const int sl = threadIdx.x & 15;
    const int64_t pair = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool on = pair < p.n_pairs;  // whole 16-lane groups are on or off together
    float M = -INFINITY;
    if (on)
        for (int s = sl; s < p.n_split; s += 16) M = fmaxf(M, p.part_mlf[(int64_t)s * p.n_pairs + pair].x);
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
    float L = 0.f;
    if (on)
        for (int s = sl; s < p.n_split; s += 16) {
            const float4 v = p.part_mlf[(int64_t)s * p.n_pairs + pair];
            L += v.x == -INFINITY ? 0.f : exp2f(v.x - M) * v.y;
        }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) L += __shfl_xor(L, o, 64);
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    if (on)
        for (int s = sl; s < p.n_split; s += 16) {
            const float4 v = p.part_mlf[(int64_t)s * p.n_pairs + pair];
            p.weights[(int64_t)s * p.n_pairs + pair] = v.x == -INFINITY ? 0.f : exp2f(v.x - M) * v.z * inv;
        }
}

// grid = (n_split, ceil(n_pairs / 256)); 256 threads = 64 row groups x 4 lanes, a lane owning 8 shot slots
// (16 bytes of a partial row: a window holds at most 32 shots, so only the first 32 of a row's 128 columns
// carry data, and the attention kernel writes only those).  Row group rg takes rows pair0 + rg, + 64, ...;
// the 64 partial sums of a slot meet in LDS and leave as block_part[window][row block][slot].
__global__ __launch_bounds__(256) void rank_reduce_kernel(RankReduceParams p) {
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    __shared__ float red[64][33];
    const int s = blockIdx.x;
    const int lane4 = threadIdx.x & 3, rg = threadIdx.x >> 2;
    const int shot0 = p.split_shot0[s];
    const int n_here = p.split_shot0[s + 1] - shot0;
    const int64_t pair0 = (int64_t)blockIdx.y * 256;
    const int64_t pair1 = pair0 + 256 < p.n_pairs ? pair0 + 256 : p.n_pairs;
    const _Float16* o = (const _Float16*)p.part_o + ((int64_t)s * p.n_pairs) * 128 + lane4 * 8;
    const float* w = p.weights + (int64_t)s * p.n_pairs;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t r = pair0 + rg; r < pair1; r += 64) {
        const f16x8 v = __builtin_nontemporal_load((const f16x8*)(o + r * 128));
        const float wr = w[r];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] += wr * (float)v[i];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[rg][lane4 * 8 + i] = acc[i];
    __syncthreads();
    const int c = threadIdx.x;
    if (c < 32 && c < n_here) {
        float t = 0.f;
#pragma unroll
        for (int g = 0; g < 64; ++g) t += red[g][c];
        p.block_part[((int64_t)s * gridDim.y + blockIdx.y) * 128 + c] = t;
    }
}

// One thread per shot: its window's row-block partials added in index order.
__global__ __launch_bounds__(256) void rank_finish_kernel(RankReduceParams p, int n_blocks) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= p.n_shots) return;
    const int s = p.shot_split[i];
    const int c = i - p.split_shot0[s];
    const float* part = p.block_part + (int64_t)s * n_blocks * 128 + c;
    float t = 0.f;
    for (int b = 0; b < n_blocks; ++b) t += part[(int64_t)b * 128];
    p.scores[i] = t * p.inv_rows * p.inv_len[i];
}

hipError_t launch_rank_weights(const RankReduceParams& p, hipStream_t stream) {
    if (p.n_split <= 0 || p.n_pairs <= 0) return hipSuccess;
    launch_kernel(rank_weights_kernel, dim3((unsigned)((p.n_pairs + 15) / 16)), dim3(256), stream, p);
    return hipGetLastError();
}

hipError_t launch_rank_reduce(const RankReduceParams& p, hipStream_t stream) {
    if (p.n_split <= 0 || p.n_pairs <= 0) return hipSuccess;
    if (p.head_dim != 128) return hipErrorInvalidValue;
    launch_kernel(rank_reduce_kernel, dim3((unsigned)p.n_split, (unsigned)((p.n_pairs + 255) / 256)), dim3(256), stream, p);
    return hipGetLastError();
}

hipError_t launch_rank_finish(const RankReduceParams& p, hipStream_t stream) {
    if (p.n_split <= 0 || p.n_pairs <= 0 || p.n_shots <= 0) return hipSuccess;
    launch_kernel(rank_finish_kernel, dim3((unsigned)((p.n_shots + 255) / 256)), dim3(256), stream, p,
                  (int)((p.n_pairs + 255) / 256));
    return hipGetLastError();
}

// ---- shapes the matrix-core kernel does not cover ------------------------------------------------------
template <int DTYPE>
__device__ __forceinline__ float rank_load(const void* base, int64_t i) {
    if (DTYPE == ADAPSHOT_BF16) return __uint_as_float(((unsigned)((const unsigned short*)base)[i]) << 16);
    return ((const float*)base)[i];
}
__device__ __forceinline__ float rank_wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float rank_wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wavefront per (query token j, head h).  score(u) = q~ . k~_u in log2 units, k~_u = the key of pool token u
// as a cache holds it: encoded at its position inside its shot and rounded to the storage type (a pool that
// stores un-rotated keys), or as stored.  Pass 1: the row's maximum and sum over the whole pool; pass 2: the
// normalised mass of every shot.
template <int DTYPE>
__global__ __launch_bounds__(64) void rank_generic_kernel(RankGenericParams p) {
    __shared__ float q_s[1024];
    const int lane = threadIdx.x;
    const int d = p.head_dim, half = d >> 1;
    const int g = p.n_q_heads / p.n_kv_heads;
    const int r = blockIdx.x;  // j * h_q + h
    const int h = r % p.n_q_heads;
    const int hk = h / g;
    for (int e = lane; e < d; e += 64) q_s[e] = rank_load<DTYPE>(p.q_rot, (int64_t)r * d + e);
    __syncthreads();
    auto score = [&](int64_t u, int64_t t_local) -> float {
        const int64_t o = (u * p.n_kv_heads + hk) * d;
        float dot = 0.f;
        if (p.key_state == ADAPSHOT_KEYS_UNROTATED) {
            const float2* th = p.tab_hi + (t_local >> kRopeLoBits) * half;
            const float2* tl = p.tab_lo + (t_local & (kRopeLo - 1)) * half;
            for (int i = 0; i < half; ++i) {
                const float2 hh = th[i], ll = tl[i];
                const float c = hh.x * ll.x - hh.y * ll.y, sn = hh.y * ll.x + hh.x * ll.y;
                const float x1 = rank_load<DTYPE>(p.k_pool, o + i), x2 = rank_load<DTYPE>(p.k_pool, o + i + half);
                float y1 = x1 * c - x2 * sn, y2 = x2 * c + x1 * sn;
                if (DTYPE == ADAPSHOT_BF16) {
                    y1 = __uint_as_float((unsigned)__builtin_bit_cast(unsigned short, (__bf16)y1) << 16);
                    y2 = __uint_as_float((unsigned)__builtin_bit_cast(unsigned short, (__bf16)y2) << 16);
                }
                dot += q_s[i] * y1 + q_s[i + half] * y2;
            }
        } else {
            for (int e = 0; e < d; ++e) dot += q_s[e] * rank_load<DTYPE>(p.k_pool, o + e);
        }
        return dot;
    };
    float m = -INFINITY, l = 0.f;  // per lane; merged below
    for (int i = 0; i < p.n_shots; ++i) {
        const int64_t t0 = p.shot_off[i], t1 = p.shot_off[i + 1];
        for (int64_t u = t0 + lane; u < t1; u += 64) {
            const float s = score(u, u - t0);
            const float mn = fmaxf(m, s);
            l = l * exp2f(m - mn) + exp2f(s - mn);
            m = mn;
        }
    }
    const float M = rank_wave_max(m);
    const float L = rank_wave_sum(m == -INFINITY ? 0.f : l * exp2f(m - M));
    const float inv_l = 1.0f / L;
    for (int i = 0; i < p.n_shots; ++i) {
        const int64_t t0 = p.shot_off[i], t1 = p.shot_off[i + 1];
        float a = 0.f;
        for (int64_t u = t0 + lane; u < t1; u += 64) a += exp2f(score(u, u - t0) - M);
        a = rank_wave_sum(a);
        if (lane == 0) p.mass[(int64_t)r * p.n_shots + i] = a * inv_l;
    }
}

// One thread per shot: the rows' masses added in row order, scaled by 1 / (T_q H_q T_i).
__global__ __launch_bounds__(256) void rank_generic_finish_kernel(RankGenericParams p) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= p.n_shots) return;
    const int n_rows = p.t_q * p.n_q_heads;
    float a = 0.f;
    for (int r = 0; r < n_rows; ++r) a += p.mass[(int64_t)r * p.n_shots + i];
    const float len = (float)(p.shot_off[i + 1] - p.shot_off[i]);
    p.scores[i] = a / ((float)n_rows * len);
}

hipError_t launch_rank_generic(const RankGenericParams& p, hipStream_t stream) {
    if (p.head_dim > 1024) return hipErrorInvalidValue;
    const unsigned rows = (unsigned)(p.t_q * p.n_q_heads);
    if (p.dtype == ADAPSHOT_BF16)
        launch_kernel(rank_generic_kernel<ADAPSHOT_BF16>, dim3(rows), dim3(64), stream, p);
    else
        launch_kernel(rank_generic_kernel<ADAPSHOT_F32>, dim3(rows), dim3(64), stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    launch_kernel(rank_generic_finish_kernel, dim3((unsigned)((p.n_shots + 255) / 256)), dim3(256), stream, p);
    return hipGetLastError();
}

}  // namespace adapshot
