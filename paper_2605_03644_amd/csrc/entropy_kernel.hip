// Entropy of softmax(logits) over the whole vocabulary (Eq. entropy), natural log.
//
// With m = max z, e_v = exp(z_v - m), s = sum e_v, t = sum (z_v - m) e_v:
//     H = ln s - t / s.
// One HBM pass: a workgroup reduces one chunk of one row to (m, s, t) with an online
// rescale per 16-element batch; a second tiny kernel merges the chunks of a row.
// Partials re-base as  s' = s * exp(m - M),  t' = (t + (m - M) * s) * exp(m - M).
#include <mutex>

#include "adapshot_internal.h"

namespace adapshot {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Chunk partials of the entry point that allocates nothing: kStaticEntropyPartials (row, chunk) triples,
// 768 KiB, held by every GPU the library runs on until the process ends.  Host code never uses this name as
// an address: entropy_static_scratch() asks the runtime where the current device keeps its copy.
static __device__ __align__(256) float g_entropy_scratch[(size_t)kStaticEntropyPartials * 3];

hipError_t entropy_static_scratch(float** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static float* ptr_of_device[kMaxDevices] = {};
    *out = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {  // once per device, with that device current
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_entropy_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr_of_device[dev] = (float*)p;
    }
    *out = ptr_of_device[dev];
    return hipSuccess;
}

struct Mst {
    float m, s, t;
};

// Merge b into a.  -inf maxima (empty parts) are handled by the w == 0 branches.
__device__ __forceinline__ Mst mst_merge(Mst a, Mst b) {
    const float M = fmaxf(a.m, b.m);
    Mst r;
    r.m = M;
    if (M == -INFINITY) {  // both empty so far (or all -inf): keep sums as they are (0, or NaN markers)
        r.s = a.s + b.s;
        r.t = a.t + b.t;
        return r;
    }
    const float da = a.m - M, db = b.m - M;  // <= 0, may be -inf
    const float wa = __expf(da), wb = __expf(db);
    const float ta = wa > 0.f ? (a.t + da * a.s) * wa : 0.f;
    const float tb = wb > 0.f ? (b.t + db * b.s) * wb : 0.f;
    r.s = a.s * wa + b.s * wb;
    r.t = ta + tb;
    return r;
}

__device__ __forceinline__ Mst mst_wave_reduce(Mst v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        Mst w;
        w.m = __shfl_xor(v.m, o, 64);
        w.s = __shfl_xor(v.s, o, 64);
        w.t = __shfl_xor(v.t, o, 64);
        v = mst_merge(v, w);
    }
    return v;
}

// a * b with 0 * anything = 0 (v_mul_legacy_f32)
__device__ __forceinline__ float mul_legacy(float a, float b) {
    float r;
    asm("v_mul_legacy_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Fold a batch of N values into the running (m, s, t).  A NaN logit poisons s through exp(NaN); a -inf
// logit gives e = 0 and must contribute 0 to t although dz = -inf: the legacy multiply returns 0 for
// 0 * anything, which is exactly the limit p ln p -> 0.
template <int N>
__device__ __forceinline__ void mst_add_batch(Mst& acc, const float (&z)[N]) {
    float bm = z[0];
#pragma unroll
    for (int i = 1; i < N; ++i) bm = fmaxf(bm, z[i]);
    const float M = fmaxf(acc.m, bm);
    if (M == INFINITY) {  // +inf logit: the row has no distribution
        acc.m = M;
        acc.s = NAN;
        acc.t = NAN;
        return;
    }
    if (M == -INFINITY) {  // nothing but -inf so far, unless a NaN hides behind the maximum (fmaxf skips NaN)
        bool nan = false;
#pragma unroll
        for (int i = 0; i < N; ++i) nan |= (z[i] != z[i]);
        if (nan) {
            acc.s = NAN;
            acc.t = NAN;
        }
        return;
    }
    if (M > acc.m) {
        const float dm = acc.m - M;
        const float w = __expf(dm);  // acc.m = -inf -> 0
        acc.t = w > 0.f ? (acc.t + dm * acc.s) * w : 0.f;
        acc.s *= w;
        acc.m = M;
    }
    float s = 0.f, t = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const float dz = z[i] - M;
        const float e = __expf(dz);
        s += e;
        t += mul_legacy(e, dz);
    }
    acc.s += s;
    acc.t += t;
}

// grid = n_rows * n_chunks workgroups (chunk fastest), 256 threads.  VEC: rows are 16-byte aligned -> float4 loads.
template <bool VEC>
__global__ __launch_bounds__(256) void entropy_chunk_kernel(EntropyParams p) {
    __shared__ Mst red[4];
    const int tid = threadIdx.x;
    const int row = blockIdx.x / p.n_chunks;
    const int chunk = blockIdx.x - row * p.n_chunks;
    const float* z = p.logits + (int64_t)row * p.row_stride;
    const int c0 = chunk * p.chunk;
    const int c1 = min(c0 + p.chunk, p.vocab);
    Mst acc = {-INFINITY, 0.f, 0.f};
    if (VEC) {
        // 4 float4 per thread per step, each load instruction covering 4 KB contiguous per workgroup.  Full
        // steps (the common case) take a branch-free path and the next step's loads are issued before this
        // step's values are used; the ragged last step of a row checks every element.
        auto load_full = [&](int base, float (&v)[16]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const f32x4 x = __builtin_nontemporal_load((const f32x4*)(z + base + u * 1024 + tid * 4));
#pragma unroll
                for (int k = 0; k < 4; ++k) v[4 * u + k] = x[k];
            }
        };
        int base = c0;
        if (base + 4096 <= c1) {
            float cur[16];
            load_full(base, cur);
            base += 4096;
            while (base + 4096 <= c1) {
                float nxt[16];
                load_full(base, nxt);
                base += 4096;
                mst_add_batch<16>(acc, cur);
#pragma unroll
                for (int k = 0; k < 16; ++k) cur[k] = nxt[k];
            }
            mst_add_batch<16>(acc, cur);
        }
        for (; base < c1; base += 4096) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * 1024 + tid * 4;
                f32x4 x = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                if (i + 3 < c1) {
                    x = __builtin_nontemporal_load((const f32x4*)(z + i));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (i + k < c1) x[k] = z[i + k];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) v[4 * u + k] = x[k];
            }
            mst_add_batch<16>(acc, v);
        }
    } else {
        for (int base = c0; base < c1; base += 1024) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * 256 + tid;
                v[u] = i < c1 ? z[i] : -INFINITY;
            }
            mst_add_batch<4>(acc, v);
        }
    }
    acc = mst_wave_reduce(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        Mst r = mst_merge(mst_merge(red[0], red[1]), mst_merge(red[2], red[3]));
        float* o = p.partials + (int64_t)blockIdx.x * 3;
        o[0] = r.m;
        o[1] = r.s;
        o[2] = r.t;
    }
}

// Whole rows in one launch: a workgroup of 1024 threads reduces one row and writes its entropy (or, with answer
// tokens, Eq. (entropy) over those) itself.  The same per-thread stream and merge as the chunk kernel; used when
// there are enough rows to keep the memory system busy with one workgroup per row, which saves the second launch.
template <bool VEC, bool TOKENS>
__global__ __launch_bounds__(1024) void entropy_row_kernel(EntropyParams p, AnswerTokens c) {
    __shared__ Mst red[16];
    const int tid = threadIdx.x;
    const int row = blockIdx.x;
    const float* z = p.logits + (int64_t)row * p.row_stride;
    const int c1 = p.vocab;
    Mst acc = {-INFINITY, 0.f, 0.f};
    if (VEC) {
        auto load_full = [&](int base, float (&v)[16]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const f32x4 x = __builtin_nontemporal_load((const f32x4*)(z + base + u * 4096 + tid * 4));
#pragma unroll
                for (int k = 0; k < 4; ++k) v[4 * u + k] = x[k];
            }
        };
        // one step (16384 logits) ahead; more in flight does not help a lone workgroup (a compute unit alone sustains
        // about 40 GB/s: 12.8 us for a 513 KB row, 14.5 us with three steps in flight)
        int base = 0;
        if (base + 16384 <= c1) {
            float cur[16];
            load_full(base, cur);
            base += 16384;
            while (base + 16384 <= c1) {
                float nxt[16];
                load_full(base, nxt);
                base += 16384;
                mst_add_batch<16>(acc, cur);
#pragma unroll
                for (int k = 0; k < 16; ++k) cur[k] = nxt[k];
            }
            mst_add_batch<16>(acc, cur);
        }
        for (; base < c1; base += 16384) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * 4096 + tid * 4;
                f32x4 x = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                if (i + 3 < c1) {
                    x = __builtin_nontemporal_load((const f32x4*)(z + i));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (i + k < c1) x[k] = z[i + k];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) v[4 * u + k] = x[k];
            }
            mst_add_batch<16>(acc, v);
        }
    } else {
        for (int base = 0; base < c1; base += 4096) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * 1024 + tid;
                v[u] = i < c1 ? z[i] : -INFINITY;
            }
            mst_add_batch<4>(acc, v);
        }
    }
    acc = mst_wave_reduce(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid >= 64) return;
    const int lane = tid;
    Mst r = {-INFINITY, 0.f, 0.f};
    if (lane < 16) r = red[lane];
    r = mst_wave_reduce(r);
    if (!TOKENS) {
        if (lane == 0) {
            float h;
            if (r.m == -INFINITY || r.m == INFINITY) h = NAN;  // no finite logit, or a +inf logit
            else h = logf(r.s) - r.t / r.s;                   // NaN sums propagate
            p.out[row] = h;
        }
        return;
    }
    // Eq. (entropy) over the answer tokens, as in entropy_finish_tokens_kernel
    const bool row_bad = r.m == -INFINITY || r.m == INFINITY || r.s != r.s;
    const float zc = lane < c.n ? z[c.id[lane]] : -INFINITY;
    float lse;
    if (c.mode == ADAPSHOT_ENTROPY_FULL_P) {
        lse = r.m + logf(r.s);
    } else {
        float mc = zc;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mc = fmaxf(mc, __shfl_xor(mc, o, 64));
        float sc = mc == -INFINITY ? 0.f : expf(zc - mc);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sc += __shfl_xor(sc, o, 64);
        lse = mc + logf(sc);
        if (mc == -INFINITY) lse = NAN;
    }
    const float lp = zc - lse;
    const float pc = expf(lp);
    float h = (lane < c.n && pc > 0.f) ? -pc * lp : 0.f;
    if (lse != lse) h = NAN;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) h += __shfl_xor(h, o, 64);
    if (lane == 0) p.out[row] = row_bad ? NAN : h;
}

hipError_t launch_entropy_rows(const EntropyParams& p, const AnswerTokens* c, hipStream_t stream) {
    const bool vec = (((uintptr_t)p.logits & 15u) == 0) && (p.row_stride % 4 == 0);
    const dim3 grid((unsigned)p.n_rows);
    const AnswerTokens none{};
    if (c) {
        if (vec) launch_kernel((entropy_row_kernel<true, true>), grid, dim3(1024), stream, p, *c);
        else launch_kernel((entropy_row_kernel<false, true>), grid, dim3(1024), stream, p, *c);
    } else {
        if (vec) launch_kernel((entropy_row_kernel<true, false>), grid, dim3(1024), stream, p, none);
        else launch_kernel((entropy_row_kernel<false, false>), grid, dim3(1024), stream, p, none);
    }
    return hipGetLastError();
}

// One wavefront per row merges its chunk partials and writes H.
__global__ __launch_bounds__(64) void entropy_finish_kernel(EntropyParams p) {
    const int row = blockIdx.x;
    const int lane = threadIdx.x;
    Mst acc = {-INFINITY, 0.f, 0.f};
    for (int c = lane; c < p.n_chunks; c += 64) {
        const float* o = p.partials + ((int64_t)row * p.n_chunks + c) * 3;
        Mst b = {o[0], o[1], o[2]};
        acc = mst_merge(acc, b);
    }
    acc = mst_wave_reduce(acc);
    if (lane == 0) {
        float h;
        if (acc.m == -INFINITY || acc.m == INFINITY) h = NAN;  // no finite logit, or a +inf logit
        else h = logf(acc.s) - acc.t / acc.s;                 // NaN sums propagate
        p.out[row] = h;
    }
}

// Eq. (entropy) as printed, summed over the answer tokens C only.  One wavefront per row merges the
// chunk partials into the vocabulary-wide log-sum-exp; lane c < |C| then holds token c.
//   full-p reading:      H = -sum_c p_c ln p_c,  ln p_c = z_c - lse
//   renormalised reading: the same with the log-sum-exp taken over C
// A term with p_c = 0 contributes 0.
__global__ __launch_bounds__(64) void entropy_finish_tokens_kernel(EntropyParams p, AnswerTokens c) {
    const int row = blockIdx.x;
    const int lane = threadIdx.x;
    Mst acc = {-INFINITY, 0.f, 0.f};
    for (int k = lane; k < p.n_chunks; k += 64) {
        const float* o = p.partials + ((int64_t)row * p.n_chunks + k) * 3;
        Mst b = {o[0], o[1], o[2]};
        acc = mst_merge(acc, b);
    }
    acc = mst_wave_reduce(acc);
    const bool row_bad = acc.m == -INFINITY || acc.m == INFINITY || acc.s != acc.s;  // as in the full entropy
    const float z = lane < c.n ? p.logits[(int64_t)row * p.row_stride + c.id[lane]] : -INFINITY;
    float lse;
    if (c.mode == ADAPSHOT_ENTROPY_FULL_P) {
        lse = acc.m + logf(acc.s);
    } else {
        float mc = z;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mc = fmaxf(mc, __shfl_xor(mc, o, 64));
        float sc = mc == -INFINITY ? 0.f : expf(z - mc);  // lanes past |C| hold -inf: 0
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sc += __shfl_xor(sc, o, 64);
        lse = mc + logf(sc);  // all of C at -inf: -inf + (-inf) -> handled below
        if (mc == -INFINITY) lse = NAN;
    }
    const float lp = z - lse;
    const float pc = expf(lp);
    float h = (lane < c.n && pc > 0.f) ? -pc * lp : 0.f;
    if (lse != lse) h = NAN;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) h += __shfl_xor(h, o, 64);
    if (lane == 0) p.out[row] = row_bad ? NAN : h;
}

hipError_t launch_entropy_finish_tokens(const EntropyParams& p, const AnswerTokens& c, hipStream_t stream) {
    launch_kernel(entropy_finish_tokens_kernel, dim3((unsigned)p.n_rows), dim3(64), stream, p, c);
    return hipGetLastError();
}

hipError_t launch_entropy_chunk(const EntropyParams& p, hipStream_t stream) {
    if ((int64_t)p.n_chunks * p.n_rows > INT32_MAX) return hipErrorInvalidValue;  // the host checks this first
    dim3 grid((unsigned)((int64_t)p.n_chunks * p.n_rows));
    const bool vec = (((uintptr_t)p.logits & 15u) == 0) && (p.row_stride % 4 == 0);
    if (vec)
        launch_kernel(entropy_chunk_kernel<true>, grid, dim3(256), stream, p);
    else
        launch_kernel(entropy_chunk_kernel<false>, grid, dim3(256), stream, p);
    return hipGetLastError();
}

hipError_t launch_entropy_finish(const EntropyParams& p, hipStream_t stream) {
    launch_kernel(entropy_finish_kernel, dim3((unsigned)p.n_rows), dim3(64), stream, p);
    return hipGetLastError();
}

}  // namespace adapshot
