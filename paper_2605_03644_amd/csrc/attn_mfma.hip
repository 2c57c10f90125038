// bf16 MFMA query-over-cache attention for head_dim 128 (split-K, flash style).
//
// The probe/query rows of one KV head (all g query heads of its group packed as rows
// j*g + h%g) attend over a slice of the assembled cache; Eq. (attention_score) gives the
// 1/sqrt(d) scale, folded with log2(e) into q when a workgroup rotates its query rows to their positions
// (Eq. rope_encoding) on the way into the fragments, so p = 2^(s - m).
//
// Work decomposition: workgroup = (kv head, tile of 256 rows, split of the context);
// 8 wavefronts (two per SIMD), each owning 32 rows for the whole key loop.  The extra split
// index n_split is the causal part over the query's own tokens.  The host picks the split count
// so that all workgroups, self parts included, fit the compute units in one round.
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
//
// The two wavefronts of a SIMD run the same three phases per 64-key tile -- S^T (matrix core),
// softmax (VALU), O^T accumulation (matrix core) -- but rotated against each other: wavefronts 0-3 go
// S(t), softmax(t), PV(t); wavefronts 4-7 go PV(t-1), S(t), softmax(t).  While one of them runs
// its exponentials the other one feeds the matrix core, with one workgroup barrier per tile.  A wave
// raises its issue priority for its matrix-core phases (s_setprio): when both waves of a SIMD have an
// instruction ready, the MFMA goes first and the other wave's vector work fills the gaps (-6 % time).
//
// The S^T accumulators start from -m (m = the row's reference maximum, in registers) instead of zero,
// so the scores leave the matrix core already shifted and the exponentials need no subtraction; the
// reference moves only when a score exceeds it by more than 8 (log2 units), then O^T, the row sum and
// the current scores are rescaled.  The key loop is unrolled four times so that every LDS buffer
// offset is an instruction immediate and the tile pointers advance in scalar registers: the per-tile
// vector ALU work is the maxima, the exponentials, the row sums and the bf16 packing only.
//
// K/V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane), four
// tiles deep for K and for V, with an XOR swizzle of the 16-byte chunks instead of row padding:
//   K row r keeps chunk c at position c ^ (r & 15)      (16 rows of a 16-byte read: 16 bank groups)
//   V row r keeps chunk c at position c ^ ((r & 3) << 2) (4 rows x 64 B of a transposing read: 64 banks)
// The query rows come in and the partial rows go out through LDS as well, as whole rows: a lane's own share of a
// row is 32 bytes of a fragment and 8 bytes of an accumulator quad, and memory instructions that touch 32 rows for
// that little each cost 5 % of the kernel when every workgroup of the grid issues them at the same moment.

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

constexpr int kD = 128;  // head_dim
constexpr int kTileKeys = 64;
constexpr int kRowBytes = kD * 2;
constexpr int kTileBytes = kTileKeys * kRowBytes;  // 16 KB, no padding
constexpr int kNBuf = 4;                           // tiles in LDS per operand
constexpr int kAttnWaves = 8;                      // wavefronts per workgroup, two per SIMD, 32 rows each
constexpr int kPD = 4;                             // LDS fragment reads in flight ahead of the MFMAs

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int kWaitVm0 = 0x0f70;  // vmcnt(0), other counters untouched

bool attn_mfma_supported(const adapshot_model_desc& d) { return d.dtype == ADAPSHOT_BF16 && d.head_dim == kD; }

// max / sum over the two lanes l and l^32 without going through LDS
__device__ __forceinline__ float max_xhalf(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xhalf(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(unsigned, b);
}

// max of three in one instruction.  fmaxf() chains compile to twice as many instructions because every
// input is first canonicalised; the scores here are MFMA outputs or -inf, never signalling NaNs.
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands at lds_base + 16*l
// (lds_base is wave-uniform and goes through M0; the source is a uniform base plus a 32-bit lane offset).
// Issued as inline assembly so that the key loop keeps control of the wait counters: the loads complete
// in order and are awaited with vmcnt in barrier_keep_one_group(), tiles after they were issued.
// NT marks the data as read once (the instruction's non-temporal bit): a launch whose workgroups stream their
// context with one or two working wavefronts is bound by the memory path, and tiles that are not kept in the L2
// for a reader that never comes move 10 % faster (5.9 -> 6.45 TB/s for the bare tile stream of a decode step).
template <bool NT = false>
__device__ __forceinline__ void load_lds_16(const char* gbase, unsigned goff, unsigned lds_base) {
    unsigned saved_m0;
    if (NT)
        asm volatile(
            "s_mov_b32 %0, m0\n\t"
            "s_mov_b32 m0, %3\n\t"
            "global_load_lds_dwordx4 %1, %2 nt\n\t"
            "s_mov_b32 m0, %0"
            : "=&s"(saved_m0)
            : "v"(goff), "s"(gbase), "s"(lds_base)
            : "memory");
    else
        asm volatile(
            "s_mov_b32 %0, m0\n\t"
            "s_mov_b32 m0, %3\n\t"
            "global_load_lds_dwordx4 %1, %2\n\t"
            "s_mov_b32 m0, %0"
            : "=&s"(saved_m0)
            : "v"(goff), "s"(gbase), "s"(lds_base)
            : "memory");
}
__device__ __forceinline__ unsigned lds_addr(const void* p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// Workgroup barrier of the key loop.  __syncthreads() would drain every tile load still in flight
// (they write LDS); here only the group issued two tiles ago must have landed (the younger
// group stays outstanding), this wave's own LDS reads must be complete, and the
// compiler may not move memory operations across.
template <int LOADS_PER_GROUP>
__device__ __forceinline__ void barrier_keep_one_group() {
    static_assert(LOADS_PER_GROUP == 4 || LOADS_PER_GROUP == 8, "vmcnt immediate");
    if (LOADS_PER_GROUP == 4)
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// A wave-uniform record from device memory into scalar registers.
template <typename T>
__device__ __forceinline__ T load_uniform(const T* ptr) {
    static_assert(sizeof(T) % 4 == 0, "whole dwords");
    T out;
    const unsigned* src = (const unsigned*)ptr;
    unsigned* dst = (unsigned*)&out;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) / 4); ++i) dst[i] = __builtin_amdgcn_readfirstlane(src[i]);
    return out;
}

// WAVES wavefronts, each owning NR blocks of 32 rows for the whole key loop.  BATCHED: the workgroup takes
// its problem and its (kv head, row tile, split) from the work list instead of the launch arguments.
// PVB: 32-column blocks of V that carry data (4 = the whole head; ranking's one-hot rows use 1).
// POOL: the zero-copy form.  The context is not an assembled cache but the pool itself, read through the
// table slot_src (context slot -> pool token): every 64-slot tile is gathered row by row into LDS, and its
// keys are rotated there, in place, to the positions pos0 + slot before the first product reads them
// (R(a)R(b) = R(a+b): tile_rot holds (cos, sin) of the tile's first position, every thread keeps the entries of
// the 64-row second-level table that its share of a tile needs).  The key loop is the plain form's -- four K
// tiles in LDS, one workgroup barrier per tile, the two wavefronts of a SIMD in rotated phase order -- with
// three additions: K(t+1), which the pipeline has landed a tile early anyway, is rotated by all 512 threads
// during tile t; the slot table entries and the rotation row of a tile arrive through the same direct-to-LDS
// path as the tiles (one more load per tile for wavefronts 0 and 1, which changes their wait counts, nothing
// else); and V keeps three tiles in LDS instead of four, which pays for the tables (V(t+1) has one tile of
// time to land instead of two).  What a context split computes is what the plain form computes over the
// assembled cache.
// FOLD: the workgroup rotates its query rows (and the self split its keys) itself; otherwise rope_rows has
// done that in a launch of its own and the kernel reads q_rot / k_self_rot.  Folding saves the launch: at the
// headline size the rotation repeated in every context split costs the kernel 1.4 us and the launch it replaces
// cost the step 3 us.  Ranking, whose one block of columns needs no keys of the query, keeps the launch.
// NT: the K/V tile loads of the plain form carry the non-temporal bit (see load_lds_16).
template <int WAVES, int NR, bool BATCHED, int PVB, bool POOL, bool FOLD, bool NT = false>
__global__ __launch_bounds__(WAVES * 64) void attn_mfma_kernel(AttnParams p_arg, AttnFold f_arg,
                                                               int n_row_tiles_arg, const AttnBatchItem* items,
                                                               const AttnWork* work) {
    // n_row_tiles_arg: row tiles per kv head of the single problem; for a batch, the layer to attend in
    constexpr int PASSES = (kTileKeys * 16) / (WAVES * 64);  // 1 KB blocks of a tile per wavefront
    static_assert(PASSES * WAVES * 64 == kTileKeys * 16, "tile must divide over the threads");
    static_assert(WAVES * NR * 32 == kAttnRowTile && NR == 1, "row tile");
    static_assert(!(NT && POOL), "pool tokens are shared by the lists that select them: they stay cacheable");
    // LDS: the K ring at byte 0, the V ring at 64 KB; the zero-copy form adds, after its shorter V ring, the ring of
    // slot-table pieces (8 x 1 KB), the ring of rotation rows (4 x 1 KB) and the threads' second-level table entries.
    constexpr int kVBuf = POOL ? 3 : kNBuf;
    constexpr int kIdxSlots = 8, kRotSlots = 4;
    constexpr int kLoBytes = WAVES * 64 * 64;
    constexpr int kPoolBytes = POOL ? (kIdxSlots + kRotSlots) * 1024 + kLoBytes : 0;
    // The plain form adds 4 KB per wavefront through which the partial rows leave (the zero-copy form reuses its
    // threads' table entries for that).
    constexpr int kStageBytes = POOL ? 0 : WAVES * 4096;
    __shared__ __attribute__((aligned(65536))) char lds_all[(kNBuf + kVBuf) * kTileBytes + kPoolBytes + kStageBytes];
    static_assert(sizeof(lds_all) <= 160 * 1024, "LDS of a compute unit");
    char (*const k_s)[kTileBytes] = (char (*)[kTileBytes])lds_all;
    char (*const v_s)[kTileBytes] = (char (*)[kTileBytes])(lds_all + kNBuf * kTileBytes);
    char* const idx_s = lds_all + (kNBuf + kVBuf) * kTileBytes;
    char* const rot_s = idx_s + kIdxSlots * 1024;
    char* const lo_s = rot_s + kRotSlots * 1024;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int hh = lane >> 5;

    AttnParams p;
    int hk, row_tile, split;
    int item = 0;
    if (BATCHED) {
        const AttnWork w = load_uniform(work + blockIdx.x);
        item = w.item;
        p = load_uniform(&items[w.item].attn);
        p.k_cache = (const char*)p.k_cache + (int64_t)n_row_tiles_arg * p.layer_stride_bytes;
        p.v_cache = (const char*)p.v_cache + (int64_t)n_row_tiles_arg * p.layer_stride_bytes;
        hk = w.hk;
        row_tile = w.row_tile;
        split = w.split;
    } else {
        // blockIdx.x -> (kv head fastest: workgroups round-robin over the 8 XCDs, so with 8 kv heads every
        // XCD's L2 sees the K/V of one head only), row tile, split
        p = p_arg;
        hk = blockIdx.x % p.n_kv_heads;
        const int rest = blockIdx.x / p.n_kv_heads;
        row_tile = rest % n_row_tiles_arg;
        split = rest / n_row_tiles_arg;
        // the self split is dispatched first: its workgroups are short, and what the grid has beyond one
        // workgroup per compute unit then starts as soon as they are done
        if (!p.no_self) split = split == 0 ? p.n_split : split - 1;
    }
    const bool self = !p.no_self && split == p.n_split;
    // the prologue-only arguments are fetched where they are used, not held through the key loop
    auto fold = [&]() __attribute__((always_inline)) -> AttnFold {
        if (BATCHED) return load_uniform(&items[item].fold);
        return f_arg;
    };

    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    int row[NR], jrow[NR];
#pragma unroll
    for (int rb = 0; rb < NR; ++rb) {
        row[rb] = row_tile * kAttnRowTile + (wave * NR + rb) * 32 + l32;
        jrow[rb] = row[rb] < rows ? row[rb] / g : 0x7fffffff;
    }

    // ---- key range of this split
    // context splits; a folding kernel's self split has a path of its own
    const char* kbase = (const char*)(!FOLD && self ? p.k_self_rot : p.k_cache) + hk * kRowBytes;
    const char* vbase = (const char*)(self ? p.v_self : p.v_cache) + hk * kRowBytes;
    const int64_t kv_stride = (int64_t)p.n_kv_heads * kRowBytes;
    int64_t k0, k1;
    if (self) {
        k0 = 0;
        k1 = p.t_q;
    } else if (p.split_bounds) {  // explicit bounds (ranking: one window of shots per split)
        const unsigned* b = (const unsigned*)(p.split_bounds + split);
        k0 = (int64_t)(((uint64_t)__builtin_amdgcn_readfirstlane(b[1]) << 32) | __builtin_amdgcn_readfirstlane(b[0]));
        k1 = (int64_t)(((uint64_t)__builtin_amdgcn_readfirstlane(b[3]) << 32) | __builtin_amdgcn_readfirstlane(b[2]));
    } else {
        k0 = (int64_t)split * p.keys_per_split;
        k1 = k0 + p.keys_per_split < p.n_ctx ? k0 + p.keys_per_split : p.n_ctx;
    }
    const int n_tiles = (int)((k1 - k0 + kTileKeys - 1) / kTileKeys);  // >= 1
    const int n_keys = (int)(k1 - k0);

    // ---- tile loads: wavefront w moves the 1 KB blocks (4 rows) w, w+WAVES, ...; lane = (row in block, chunk).
    // Every lane keeps the byte offset of its chunks inside a tile; the tile itself is addressed by a
    // wave-uniform pointer that advances by one tile per load.  The last tile (whose rows may run past the
    // end of the split) and the tiles past the end (loaded anyway so that the number of loads in flight
    // stays the same in every iteration; they land in buffers nobody reads any more) take their offsets
    // from the start of the cache with the row clamped to the last valid key.
    const unsigned tile_step = (unsigned)(kTileKeys * kv_stride);
    unsigned k_loff[PASSES], v_loff[PASSES];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
        const unsigned row_off = (unsigned)(r * kv_stride);
        k_loff[ps] = row_off + (((lane & 15) ^ (r & 15)) << 4);
        v_loff[ps] = row_off + (((lane & 15) ^ ((r & 3) << 2)) << 4);
    }
    const char* k_tile = kbase + k0 * kv_stride;  // next K tile to load
    const char* v_tile = vbase + k0 * kv_stride;  // next V tile to load
    auto clamped_off = [&](int ps, bool is_v) __attribute__((always_inline)) -> unsigned {
        const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
        int64_t key = k0 + (int64_t)(n_tiles - 1) * kTileKeys + r;
        key = key < k1 ? key : k1 - 1;
        const unsigned sw = is_v ? ((lane & 15) ^ ((r & 3) << 2)) : ((lane & 15) ^ (r & 15));
        return (unsigned)(key * kv_stride) + (sw << 4);
    };
    int next_k_tile = 0, next_v_tile = 0;
    // buf is a compile-time constant at every call site, so the LDS destination is an immediate
    auto issue_k = [&](int buf) __attribute__((always_inline)) {
        if (next_k_tile >= n_tiles - 1) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                load_lds_16<NT>(kbase, clamped_off(ps, false),
                            __builtin_amdgcn_readfirstlane(lds_addr(k_s[buf] + (ps * WAVES + wave) * 1024)));
        } else {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                load_lds_16<NT>(k_tile, k_loff[ps],
                            __builtin_amdgcn_readfirstlane(lds_addr(k_s[buf] + (ps * WAVES + wave) * 1024)));
            k_tile += tile_step;
        }
        ++next_k_tile;
    };
    auto issue_v = [&](int buf) __attribute__((always_inline)) {
        if (next_v_tile >= n_tiles - 1) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                load_lds_16<NT>(vbase, clamped_off(ps, true),
                            __builtin_amdgcn_readfirstlane(lds_addr(v_s[buf] + (ps * WAVES + wave) * 1024)));
        } else {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
                load_lds_16<NT>(v_tile, v_loff[ps],
                            __builtin_amdgcn_readfirstlane(lds_addr(v_s[buf] + (ps * WAVES + wave) * 1024)));
            v_tile += tile_step;
        }
        ++next_v_tile;
    };
    // K(0) and V(0) of a context split start now; the other tiles of the pipeline follow once these have
    // landed.  (The split over the query's own tokens moves its tiles through registers, see below.)
    // ---- zero-copy form: gathered tile loads
    AttnFold pf{};
    if (POOL) pf = fold();
    // Byte offsets (inside the pool's layer) of this lane's rows of tile T, from the ring of slot-table pieces.
    // The tiles past the end of the split stand for its last tile (their loads keep the number in flight the same
    // and land where nobody reads any more); rows past the last key repeat it (the softmax masks them).
    auto pool_rows = [&](int T, unsigned (&off)[PASSES]) __attribute__((always_inline)) {
        const int Tc = T < n_tiles ? T : n_tiles - 1;
        const char* piece = idx_s + (T & (kIdxSlots - 1)) * 1024;
        const int last = n_keys - 1 - Tc * kTileKeys;
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
            unsigned tok = *(const unsigned*)(piece + (r < last ? r : last) * 4);
            tok = tok < (unsigned)pf.pool_tokens ? tok : (unsigned)pf.pool_tokens - 1u;  // never outside the pool
            off[ps] = tok * (unsigned)kv_stride;  // the host keeps a pool layer below 4 GiB
        }
    };
    // the same offsets straight from the table in memory (prologue: tiles 0 and 1)
    auto pool_rows_direct = [&](int T, unsigned (&off)[PASSES]) __attribute__((always_inline)) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
            int64_t key = k0 + (int64_t)T * kTileKeys + r;
            key = key < k1 ? key : k1 - 1;
            unsigned tok = (unsigned)pf.slot_src[key];
            tok = tok < (unsigned)pf.pool_tokens ? tok : (unsigned)pf.pool_tokens - 1u;
            off[ps] = tok * (unsigned)kv_stride;
        }
    };
    // lds_dst: LDS byte address of the destination tile (wave-uniform)
    auto pool_gather_k = [&](const unsigned (&off)[PASSES], unsigned lds_dst) __attribute__((always_inline)) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
            load_lds_16(kbase, off[ps] + (((lane & 15) ^ (r & 15)) << 4),
                        __builtin_amdgcn_readfirstlane(lds_dst + (ps * WAVES + wave) * 1024));
        }
    };
    auto pool_gather_v = [&](const unsigned (&off)[PASSES], unsigned lds_dst) __attribute__((always_inline)) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
            const int r = 4 * (ps * WAVES + wave) + (lane >> 4);
            load_lds_16(vbase, off[ps] + (((lane & 15) ^ ((r & 3) << 2)) << 4),
                        __builtin_amdgcn_readfirstlane(lds_dst + (ps * WAVES + wave) * 1024));
        }
    };
    // one wavefront: 1 KB of the slot table starting at tile T's first slot (the tile's 64 entries and 192 more;
    // the host pads the table by that much) into piece T % 8
    auto issue_idx = [&](int T) __attribute__((always_inline)) {
        const int Tc = T < n_tiles ? T : n_tiles - 1;
        load_lds_16((const char*)(pf.slot_src + k0 + (int64_t)Tc * kTileKeys), (unsigned)lane * 16u,
                    __builtin_amdgcn_readfirstlane(lds_addr(idx_s + (T & (kIdxSlots - 1)) * 1024)));
    };
    // one wavefront: the rotation row of tile T (512 bytes, lanes 0-31; lanes 32-63 bring the next row along)
    // into slot T % 4
    auto issue_rot = [&](int T) __attribute__((always_inline)) {
        const int64_t last = (p.n_ctx - 1) / kTileKeys;
        int64_t gt = k0 / kTileKeys + T + (lane >> 5);
        gt = gt < last ? gt : last;
        load_lds_16((const char*)pf.tile_rot, (unsigned)(gt * 512 + (lane & 31) * 16),
                    __builtin_amdgcn_readfirstlane(lds_addr(rot_s + (T & (kRotSlots - 1)) * 1024)));
    };
    // rotate the keys of tile T, landed in K buffer `buf` (= T % 4), in place: thread = (row r, chunk pair cp), the
    // same pairing as the assemble kernel; position of row r = (tile's first position) + r
    auto pool_rotate = [&](int T, int buf) __attribute__((always_inline)) {
        static_assert(!POOL || WAVES * 64 == kTileKeys * 8, "one (row, chunk pair) per thread");
        if (T >= n_tiles) return;
        __builtin_amdgcn_s_setprio(0);
        const int r = tid >> 3, cp = tid & 7;
        const f32x4* hi = (const f32x4*)(rot_s + buf * 1024 + cp * 64);
        u32x4* a1 = (u32x4*)(k_s[buf] + r * kRowBytes + ((cp ^ (r & 15)) << 4));
        u32x4* a2 = (u32x4*)(k_s[buf] + r * kRowBytes + (((cp + 8) ^ (r & 15)) << 4));
        u32x4 x1 = *a1, x2 = *a2;
#pragma unroll
        for (int w = 0; w < 4; ++w) {  // word w holds elements 2w, 2w+1 of the chunk: frequencies 8 cp + 2w, + 2w + 1
            const f32x4 h = hi[w], l = *(const f32x4*)(lo_s + w * (WAVES * 64 * 16) + tid * 16);
            const float c0 = h[0] * l[0] - h[1] * l[1], s0 = h[1] * l[0] + h[0] * l[1];
            const float c1 = h[2] * l[2] - h[3] * l[3], s1 = h[3] * l[2] + h[2] * l[3];
            const float a1l = __uint_as_float(x1[w] << 16), a1h = __uint_as_float(x1[w] & 0xffff0000u);
            const float a2l = __uint_as_float(x2[w] << 16), a2h = __uint_as_float(x2[w] & 0xffff0000u);
            x1[w] = pack2_bf16(a1l * c0 - a2l * s0, a1h * c1 - a2h * s1);
            x2[w] = pack2_bf16(a2l * c0 + a1l * s0, a2h * c1 + a1h * s1);
        }
        *a1 = x1;
        *a2 = x2;
    };
    if (!self || !FOLD) {
        if (POOL) {
            // this thread's entries of the second-level table: (cos, sin)(r theta_f), f = 8 cp .. 8 cp + 7
            const f32x4* tl = (const f32x4*)(pf.tab_lo + (tid >> 3) * (kD / 2) + 8 * (tid & 7));
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) *(f32x4*)(lo_s + e2 * (WAVES * 64 * 16) + tid * 16) = tl[e2];
            // K(0), V(0), K(1); the slot-table pieces of tiles 1-4 and the rotation rows of tiles 0-2
            unsigned off[PASSES];
            pool_rows_direct(0, off);
            pool_gather_k(off, lds_addr(k_s[0]));
            pool_gather_v(off, lds_addr(v_s[0]));
            pool_rows_direct(1, off);
            pool_gather_k(off, lds_addr(k_s[1]));
            if (wave == 0) {
                issue_idx(1);
                issue_idx(2);
                issue_idx(3);
                issue_idx(4);
            }
            if (wave == 1) {
                issue_rot(0);
                issue_rot(1);
                issue_rot(2);
            }
        } else {
            // the second tile is requested with the first: the memory system is idle at this point, and the first
            // two tiles then run without waiting for a round trip that only started after the first barrier
            issue_k(0);
            issue_v(0);
            issue_k(1);
            issue_v(1);
        }
    }

    // Eight (cos, sin) of position `a` for the frequencies f0 .. f0+7: one fp32 angle addition of the two
    // fp64-built table entries (a = 64*hi + lo).
    auto cos_sin8 = [&](const AttnFold& f, int64_t a, int f0, float (&c)[8], float (&sn)[8]) __attribute__((always_inline)) {
        const f32x4* th = (const f32x4*)(f.tab_hi + (a >> kRopeLoBits) * (kD / 2) + f0);
        const f32x4* tl = (const f32x4*)(f.tab_lo + (a & (kRopeLo - 1)) * (kD / 2) + f0);
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const f32x4 h = th[e2], l = tl[e2];  // two frequencies: (cos, sin, cos, sin)
            c[2 * e2] = h[0] * l[0] - h[1] * l[1];
            sn[2 * e2] = h[1] * l[0] + h[0] * l[1];
            c[2 * e2 + 1] = h[2] * l[2] - h[3] * l[3];
            sn[2 * e2 + 1] = h[3] * l[2] + h[2] * l[3];
        }
    };
    // Rotate the pair partners held in two 16-byte chunks (elements i .. i+7 and i+64 .. i+71 of a row),
    // scale, round to bf16 (nearest even).
    auto rotate8 = [&](u32x4& x1, u32x4& x2, const float (&c)[8], const float (&sn)[8], float sc) __attribute__((always_inline)) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a1l = __uint_as_float(x1[w] << 16), a1h = __uint_as_float(x1[w] & 0xffff0000u);
            const float a2l = __uint_as_float(x2[w] << 16), a2h = __uint_as_float(x2[w] & 0xffff0000u);
            const float y1l = (a1l * c[2 * w] - a2l * sn[2 * w]) * sc, y2l = (a2l * c[2 * w] + a1l * sn[2 * w]) * sc;
            const float y1h = (a1h * c[2 * w + 1] - a2h * sn[2 * w + 1]) * sc, y2h = (a2h * c[2 * w + 1] + a1h * sn[2 * w + 1]) * sc;
            x1[w] = pack2_bf16(y1l, y1h);
            x2[w] = pack2_bf16(y2l, y2h);
        }
    };

    // ---- Q fragments (B operand): lane holds row l32, d = 16*kk + 8*hh .. +7.  Fragments kk and kk + 4 hold
    // rotation partners (d, d + 64), so a lane rotates its own row to position q_pos0 + j and folds the
    // softmax scale in, without another pass over Q in memory.
    // The wavefront's 32 rows come whole through LDS: 8 KB of the tile ring that no tile uses before the first
    // barrier, filled by the direct-to-LDS path 4 rows (1 KB of whole 256-byte rows) per instruction, 16-byte
    // pieces permuted by the row number like the K tiles'.  Read straight from memory a fragment is 32 bytes of
    // each of 32 rows per instruction, and with every context split of a query fetching the same rows at the
    // same moment that cost 2 % of the kernel at the headline size.  Rows past the last one stand for it.
    bf16x8 qf[8];
    {
        AttnFold f{};
        if (FOLD) f = fold();
        const bool valid = row[0] < rows;
        const int j = valid ? jrow[0] : 0;
        const char* qbase = (const char*)(FOLD ? f.q_raw : p.q_rot);
        const int r_last = rows - 1, j_last = r_last / g;
        const int jc = valid ? j : j_last, gc = valid ? row[0] - j * g : r_last - j_last * g;
        const unsigned qoff = (unsigned)(((jc * p.n_q_heads + hk * g + gc) * kD) * 2);  // the host keeps Q below 2 GiB
        char* const qst = wave < WAVES / 2 ? k_s[2] + wave * 8192 : v_s[kVBuf - 2] + (wave - WAVES / 2) * 8192;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rl = 4 * i + (lane >> 4);  // row of the wavefront that this lane fetches a piece of
            const unsigned off_r = (unsigned)__builtin_amdgcn_ds_bpermute(rl * 4, (int)qoff);
            load_lds_16(qbase, off_r + (((lane & 15) ^ (rl & 15)) << 4),
                        __builtin_amdgcn_readfirstlane(lds_addr(qst + i * 1024)));
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // these rows, and the first tiles requested above
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4 x1 = {0u, 0u, 0u, 0u}, x2 = {0u, 0u, 0u, 0u};
            if (valid) {
                x1 = *(const u32x4*)(qst + l32 * 256 + (((2 * kk + hh) ^ (l32 & 15)) << 4));
                x2 = *(const u32x4*)(qst + l32 * 256 + (((2 * (kk + 4) + hh) ^ (l32 & 15)) << 4));
                if (FOLD) {
                    float c[8], sn[8];
                    cos_sin8(f, f.q_pos0 + j, 16 * kk + 8 * hh, c, sn);
                    rotate8(x1, x2, c, sn, f.q_scale);
                }
            }
            qf[kk] = __builtin_bit_cast(bf16x8, x1);
            qf[kk + 4] = __builtin_bit_cast(bf16x8, x2);
        }
    }

    // ---- per-lane LDS read addresses.  The K tiles occupy LDS bytes [0, 64K) and the V tiles
    // [64K, 128K), four 16 KB buffers each.
    // K fragment kk of key block kb: row 32*kb + l32, chunk (2*kk + hh) ^ (l32 & 15)
    unsigned ka[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
        ka[kk] = lds_addr(&k_s[0][0]) + (unsigned)(l32 * kRowBytes + (((2 * kk + hh) ^ (l32 & 15)) << 4));
    // V^T fragment (db, ks): two transposing reads.  In a 16-lane group, lane i addresses row
    // kbase + i/4, 8 bytes at element column dbase + 4*(i%4), and receives column dbase + i of rows
    // kbase .. kbase+3.  Row = 16*ks + 4*hh + i/4 (+8), so (row & 3) = i/4.
    unsigned va[4];
    {
        const int i16 = lane & 15;
        const int r3 = i16 >> 2;
#pragma unroll
        for (int db = 0; db < 4; ++db)
            va[db] = lds_addr(&v_s[0][0]) + (unsigned)((4 * hh + r3) * kRowBytes + ((db ^ r3) << 6) +
                                                       (((lane >> 4) & 1) << 5) + ((i16 & 3) << 3));
    }
    typedef __attribute__((address_space(3))) char lds_char;
    lds_char* kp[8];
    lds_char* vp[4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) kp[kk] = (lds_char*)(uintptr_t)ka[kk];
#pragma unroll
    for (int db = 0; db < 4; ++db) vp[db] = (lds_char*)(uintptr_t)va[db];
    // buf and the block indices are compile-time constants at every call site: they fold into the
    // 16-bit offset field of the LDS instruction, so the address registers never change.
    auto k_frag = [&](int buf, int kb, int kk) __attribute__((always_inline)) -> bf16x8 {
        const u32x4 w = *(const __attribute__((address_space(3))) u32x4*)(kp[kk] + buf * kTileBytes + kb * (32 * kRowBytes));
        return __builtin_bit_cast(bf16x8, w);
    };
    auto v_frag = [&](int buf, int ks, int db, unsigned voff) __attribute__((always_inline)) -> bf16x8 {
        lds_char* a = vp[db] + voff + buf * kTileBytes + ks * (16 * kRowBytes);
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)a);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a + 8 * kRowBytes));
        const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, av);
    };

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_run = -INFINITY;  // reference maximum of the exponentials (log2 units); may lag the true maximum by < 8
    float l_run = 0.f;        // this lane's share of the row sum
    f32x16 s[2];              // S^T of the current tile minus the reference maximum, key blocks 0 and 1
    f32x16 negm;              // -(reference maximum): the value the S^T accumulators start from, so that the
                              // exponentials need no subtraction; rewritten only when the reference moves
#pragma unroll
    for (int r = 0; r < 16; ++r) negm[r] = 0.f;
    u32x4 pb[4];              // P^T of the current tile (packed bf16), one B operand per 16-key step

    // S^T(t) - m = K(t) . Q^T - m from K buffer `buf`: 16 MFMAs, fragments read kPD steps ahead
    constexpr int kFD = POOL ? 2 : kPD;  // fragment reads in flight (the zero-copy form has fewer registers to spare)
    auto s_phase = [&](int buf) __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(1);  // matrix-core phases win the issue arbitration over the other wave's softmax
        bf16x8 fr[kFD];
#pragma unroll
        for (int i = 0; i < kFD; ++i) fr[i] = k_frag(buf, i & 1, i >> 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) {  // kk = i/2, kb = i%2
            const bf16x8 a = fr[i % kFD];
            if (i + kFD < 16) fr[i % kFD] = k_frag(buf, (i + kFD) & 1, (i + kFD) >> 1);
            if (i < 2) s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0], negm, 0, 0, 0);
            else s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[i >> 1], s[i & 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, kFD, 0);  // the first kFD fragment reads, then MFMA / read pairs
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + kFD < 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    };
    // O^T += V^T . P^T from V buffer `buf` (plus voff bytes, the zero-copy form's run-time ring position):
    // 4 * PVB MFMAs, 2 transposing reads per fragment
    auto pv_phase = [&](int buf, unsigned voff = 0u) __attribute__((always_inline)) {
        constexpr int NPV = 4 * PVB;
        constexpr int PD = kFD < NPV ? kFD : NPV;
        __builtin_amdgcn_s_setprio(1);
        bf16x8 fr[PD];
#pragma unroll
        for (int i = 0; i < PD; ++i) fr[i] = v_frag(buf, i / PVB, i % PVB, voff);
#pragma unroll
        for (int i = 0; i < NPV; ++i) {  // ks = i / PVB, db = i % PVB
            const bf16x8 a = fr[i % PD];
            if (i + PD < NPV) fr[i % PD] = v_frag(buf, (i + PD) / PVB, (i + PD) % PVB, voff);
            o[i % PVB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pb[i / PVB]), o[i % PVB], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * PD, 0);
#pragma unroll
        for (int i = 0; i < NPV; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + PD < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
    };
    // masks + online softmax of tile t with a lazily updated reference maximum; leaves P^T(t) in pb
    // Key visibility in 32-bit arithmetic relative to k0: a key of this lane is visible while its index
    // 64*t + 32*kb + 8*(r/4) + (r%4) stays below lim (the 4*hh of the lane is folded into lim).
    const int lim = (self ? (jrow[0] < n_keys ? jrow[0] + 1 : n_keys) : n_keys) - 4 * hh;
    auto softmax_phase = [&](int t) __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(0);
        if (self || (t + 1) * kTileKeys > n_keys) {
            const int lim_t = lim - t * kTileKeys;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * kb + 8 * (r >> 2) + (r & 3) >= lim_t) s[kb][r] = -INFINITY;
        }
        // s holds S - m_use; mx is relative to the reference
        float mx = max3(s[0][0], s[1][0], s[0][1]);
#pragma unroll
        for (int r = 1; r < 15; ++r) mx = max3(mx, s[1][r], s[0][r + 1]);
        mx = max_xhalf(fmaxf(mx, s[1][15]));
        if (__builtin_amdgcn_ballot_w64(mx > 8.0f || (m_run == -INFINITY && mx > -INFINITY))) {
            const float m_use_old = m_run == -INFINITY ? 0.f : m_run;  // nothing visible yet: the reference is 0
            const float m_new = fmaxf(m_run, mx + m_use_old);
            const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
            const float m_use_new = m_new == -INFINITY ? 0.f : m_new;
            const float delta = m_use_new - m_use_old;
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] -= delta;
#pragma unroll
            for (int r = 0; r < 16; ++r) negm[r] = -m_use_new;
        }
        float sum = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float e0 = __builtin_amdgcn_exp2f(s[ks >> 1][8 * (ks & 1) + 2 * e]);
                const float e1 = __builtin_amdgcn_exp2f(s[ks >> 1][8 * (ks & 1) + 2 * e + 1]);
                sum += e0 + e1;
                pb[ks][e] = pack2_bf16(e0, e1);
            }
        l_run += sum;
    };
    // End of tile t (b = t % 4): K(t+1) and V(t+1) have landed (the younger group may stay in flight); the buffers
    // of K(t) and V(t-1), which every wave has finished reading, are refilled with K(t+4) and V(t+3).
    auto end_of_tile = [&](int b) __attribute__((always_inline)) {
        barrier_keep_one_group<2 * PASSES>();
        issue_k(b);            // K(t+4)
        issue_v((b + 3) & 3);  // V(t+3)
    };

    // ---- prologue: the first two tiles (the zero-copy form: K(0) V(0) K(1)) have landed and the Q fragments
    // are in registers (every wavefront has read its rows out of the ring buffers that the loads below fill).
    // The Q registers pass through the wait statement so that the compiler places no counter wait of its own
    // after the loads below, which it cannot see (it would drain them).  Then the rest of the pipeline starts:
    // K(2) V(2) K(3), in the order the tiles are needed, so that "all but the youngest four loads" covers K(t+1)
    // and V(t+1) at the end of every tile t from the first one on.
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(qf[0]), "+v"(qf[1]), "+v"(qf[2]), "+v"(qf[3]), "+v"(qf[4]), "+v"(qf[5]), "+v"(qf[6]), "+v"(qf[7])
                 :
                 : "memory");
    __syncthreads();
    // A wavefront whose 32 rows all lie past the last query row (a decode step has fewer rows than one
    // wavefront owns) only moves tiles and keeps the barriers.
    const bool wave_idle = row_tile * kAttnRowTile + wave * NR * 32 >= rows;
    if (self && FOLD) {
        // ---- the query's own tokens: a few tiles at most, moved through registers so that the keys can be
        // rotated to their positions q_pos0 + u on the way (the caller gives them un-rotated).  One tile at a
        // time in buffer 0, two workgroup barriers per tile.  Thread = (row r, chunk pair cp) for K, two
        // (row, chunk) items for V; rows past the last token are zero-filled (and masked by the softmax).
        const AttnFold f = fold();
        const char* ksbase = (const char*)f.k_self_raw + hk * kRowBytes;
        const int r = tid >> 3, cp = tid & 7;
        for (int t = 0; t < n_tiles; ++t) {
            const int u = t * kTileKeys + r;
            u32x4 x1 = {0u, 0u, 0u, 0u}, x2 = {0u, 0u, 0u, 0u};
            if (u < n_keys) {
                const char* krow = ksbase + (int64_t)u * kv_stride;
                x1 = *(const u32x4*)(krow + cp * 16);
                x2 = *(const u32x4*)(krow + (cp + 8) * 16);
                float c[8], sn[8];
                cos_sin8(f, f.q_pos0 + u, 8 * cp, c, sn);
                rotate8(x1, x2, c, sn, 1.0f);
            }
            *(u32x4*)(k_s[0] + r * kRowBytes + ((cp ^ (r & 15)) << 4)) = x1;
            *(u32x4*)(k_s[0] + r * kRowBytes + (((cp + 8) ^ (r & 15)) << 4)) = x2;
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int rv = 4 * (ps * WAVES + wave) + (lane >> 4), cv = lane & 15;
                const int uv = t * kTileKeys + rv;
                u32x4 xv = {0u, 0u, 0u, 0u};
                if (uv < n_keys) xv = *(const u32x4*)(vbase + (int64_t)uv * kv_stride + cv * 16);
                *(u32x4*)(v_s[0] + rv * kRowBytes + ((cv ^ ((rv & 3) << 2)) << 4)) = xv;
            }
            __syncthreads();
            if (!wave_idle) {
                s_phase(0);
                softmax_phase(t);
                pv_phase(0);
            }
            __syncthreads();
        }
    } else if (POOL) {
        // ---- zero-copy key loop.  K(0), K(1), V(0), the table pieces and rotation rows requested so far have
        // landed (wait and barrier above).  K(0) is rotated now; the rest of the pipeline starts in the order the
        // waits below assume: K(2), then the group V(1), K(3) and the extra load of wavefronts 0 and 1.
        pool_rotate(0, 0);
        {
            unsigned off[PASSES];
            pool_rows(2, off);
            pool_gather_k(off, lds_addr(k_s[2]));
            pool_rows(1, off);
            pool_gather_v(off, lds_addr(v_s[1]));
            pool_rows(3, off);
            pool_gather_k(off, lds_addr(k_s[3]));
            if (wave == 0) issue_idx(5);
            if (wave == 1) issue_rot(3);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // the rotated K(0) is visible
        // V ring positions (bytes from V buffer 0) of V(t) and V(t-1); the third buffer holds V(t+1)
        unsigned vo_cur = 0u, vo_prev = 2u * kTileBytes;
        // End of tile t (b = t % 4).  Every load but the last K tile's (and the extra one behind it) has landed:
        // V(t+1), K(t+2) with its rotation row, the table pieces up to tile t+5.  The buffers of V(t-1) and K(t)
        // are refilled with V(t+2) and K(t+4); piece (t+6) % 8 and rotation slot (t+4) % 4 were last read tiles ago.
        auto end_of_tile_z = [&](int t, int b) __attribute__((always_inline)) {
            if (wave < 2) asm volatile("s_waitcnt vmcnt(3) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(2) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            unsigned off[PASSES];
            pool_rows(t + 2, off);
            pool_gather_v(off, lds_addr(v_s[0]) + vo_prev);
            pool_rows(t + 4, off);
            pool_gather_k(off, lds_addr(k_s[b]));
            if (wave == 0) issue_idx(t + 6);
            if (wave == 1) issue_rot(t + 4);
            const unsigned vo_next = 3u * kTileBytes - vo_cur - vo_prev;
            vo_prev = vo_cur;
            vo_cur = vo_next;
        };
        if (wave_idle) {
            for (int t = 0; t < n_tiles; ++t) {
                pool_rotate(t + 1, (t + 1) & 3);
                end_of_tile_z(t, t & 3);
            }
        } else if (wave < WAVES / 2) {
            // order A: S(t), softmax(t), PV(t), rotate K(t+1)
            auto tile_a = [&](int t, int b) __attribute__((always_inline)) {
                s_phase(b);
                softmax_phase(t);
                pv_phase(0, vo_cur);
                pool_rotate(t + 1, (b + 1) & 3);
                end_of_tile_z(t, b);
            };
            int t = 0;
            for (; t + 4 <= n_tiles; t += 4) {
                tile_a(t, 0);
                tile_a(t + 1, 1);
                tile_a(t + 2, 2);
                tile_a(t + 3, 3);
            }
            for (; t < n_tiles; ++t) tile_a(t, t & 3);
        } else {
            // order B: PV(t-1), rotate K(t+1), S(t), softmax(t)
            auto tile_b = [&](int t, int b) __attribute__((always_inline)) {
                pv_phase(0, vo_prev);
                pool_rotate(t + 1, (b + 1) & 3);
                s_phase(b);
                softmax_phase(t);
                end_of_tile_z(t, b);
            };
            pool_rotate(1, 1);
            s_phase(0);
            softmax_phase(0);
            end_of_tile_z(0, 0);
            int t = 1;
            for (; t + 4 <= n_tiles; t += 4) {
                tile_b(t, 1);
                tile_b(t + 1, 2);
                tile_b(t + 2, 3);
                tile_b(t + 3, 0);
            }
            for (; t < n_tiles; ++t) tile_b(t, t & 3);
            pv_phase(0, vo_prev);
        }
    } else {
    issue_k(2);
    issue_v(2);
    issue_k(3);

    // The key loop is unrolled four times so that the LDS buffer of every access is a compile-time constant;
    // the last n_tiles % 4 tiles take the buffer index at run time.
    if (wave_idle) {
        for (int t = 0; t < n_tiles; ++t) end_of_tile(t & 3);
    } else if (wave < WAVES / 2) {
        // order A: S(t), softmax(t), PV(t)
        auto tile_a = [&](int t, int b) __attribute__((always_inline)) {
            s_phase(b);
            softmax_phase(t);
            pv_phase(b);
            end_of_tile(b);
        };
        int t = 0;
        for (; t + 4 <= n_tiles; t += 4) {
            tile_a(t, 0);
            tile_a(t + 1, 1);
            tile_a(t + 2, 2);
            tile_a(t + 3, 3);
        }
        for (; t < n_tiles; ++t) tile_a(t, t & 3);
    } else {
        // order B: PV(t-1), S(t), softmax(t); the same number of barriers as order A
        auto tile_b = [&](int t, int b) __attribute__((always_inline)) {
            pv_phase((b + 3) & 3);
            s_phase(b);
            softmax_phase(t);
            end_of_tile(b);
        };
        s_phase(0);
        softmax_phase(0);
        end_of_tile(0);
        int t = 1;
        for (; t + 4 <= n_tiles; t += 4) {
            tile_b(t, 1);
            tile_b(t + 1, 2);
            tile_b(t + 2, 3);
            tile_b(t + 3, 0);
        }
        for (; t < n_tiles; ++t) tile_b(t, t & 3);
        pv_phase((n_tiles - 1) & 3);
    }
    }
    __builtin_amdgcn_s_waitcnt(kWaitVm0);  // the loads of the tiles past the end must land before LDS is released

    // ---- partials: the row's reference maximum, sum l and factor f = l * a, and O' = O / (l * a) in fp16, where
    // a is the largest |O| / l of the row: |O'| <= 1 whatever the range of V (row-major [row][d]).
    const float l_tot = sum_xhalf(l_run);
    float amax = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(o[db][r]));
    amax = max_xhalf(amax);
    const bool some = amax > 0.f && amax < INFINITY;  // all-zero row (or overflow): plain scale 1
    const float scale = some ? 1.0f / amax : 1.0f;
    if (row[0] < rows && hh == 0)
        p.part_mlf[((int64_t)split * p.n_kv_heads + hk) * rows + row[0]] = make_float4(m_run, l_tot, some ? amax : 1.0f, 0.f);
    // The rows leave through 4 KB of LDS that only this wavefront touches, half a row (64 columns) at a time: a lane
    // holds 4 consecutive columns of its row per register quad, and stored from there every instruction would write
    // 8 bytes to each of 32 rows (the write-out took 3.4 of the kernel's 57 us at the headline size, 2.6 of them
    // for that); read back row-wise, an instruction writes 128 contiguous bytes of each of eight rows.  Row r of
    // the piece is 128 bytes whose 16-byte slots are permuted by (r / 2) % 8, which spreads both directions over
    // the banks.  The plain form has the space to spare; the zero-copy form reuses the wavefront's share of the
    // second-level table entries (four 1 KB pieces, one per plane), which the key loop is done with.
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    auto stage_row = [&](int r) __attribute__((always_inline)) -> char* {
        if (POOL) return lo_s + (r >> 3) * (WAVES * 64 * 16) + wave * 1024 + (r & 7) * 128;
        return lds_all + (kNBuf + kVBuf) * kTileBytes + kPoolBytes + wave * 4096 + r * 128;
    };
    const int row0 = row_tile * kAttnRowTile + wave * NR * 32;  // first row of this wavefront
    char* const obase = (char*)p.part_o + ((((int64_t)split * p.n_kv_heads + hk) * rows + row0) * kD) * 2;
    // (ranking's one block of columns: the first 64 bytes of every row are written and read, nothing else)
    constexpr int kHalves = PVB == 1 ? 1 : 2, kBlocks = PVB == 1 ? 1 : 2, kSlots = PVB == 1 ? 4 : 8;
#pragma unroll
    for (int half = 0; half < kHalves; ++half) {
#pragma unroll
        for (int dbl = 0; dbl < kBlocks; ++dbl)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int db = 2 * half + dbl;
                const f32x4 w = {o[db][4 * rq] * scale, o[db][4 * rq + 1] * scale, o[db][4 * rq + 2] * scale,
                                 o[db][4 * rq + 3] * scale};
                const int slot = (4 * dbl + rq) ^ ((l32 >> 1) & 7);
                *(f16x4*)(stage_row(l32) + slot * 16 + hh * 8) = __builtin_convertvector(w, f16x4);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // written by other lanes of the wavefront, read below
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 8 * j + (lane >> 3), sl = lane & 7;
            const u32x4 v = *(const u32x4*)(stage_row(r) + ((sl ^ ((r >> 1) & 7)) << 4));
            if (row0 + r < rows && sl < kSlots) *(u32x4*)(obase + (int64_t)r * (kD * 2) + half * 128 + sl * 16) = v;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // read before the second half overwrites the piece
    }
}

hipError_t launch_attn_mfma(const AttnParams& p, const AttnFold& f, hipStream_t stream) {
    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int n_row_tiles = (rows + kAttnRowTile - 1) / kAttnRowTile;
    const unsigned blocks = (unsigned)(p.n_kv_heads * n_row_tiles * (p.n_split + (p.no_self ? 0 : 1)));
    if (blocks == 0) return hipSuccess;
    if (p.v_blocks == 1)
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), false, 1, false, false>), dim3(blocks),
                      dim3(kAttnWaves * 64), stream, p, f, n_row_tiles, (const AttnBatchItem*)nullptr,
                      (const AttnWork*)nullptr);
    else if (rows <= kAttnStreamRows)  // every tile is read by one workgroup per kv head, which has few rows to feed
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), false, 4, false, true, true>),
                      dim3(blocks), dim3(kAttnWaves * 64), stream, p, f, n_row_tiles, (const AttnBatchItem*)nullptr,
                      (const AttnWork*)nullptr);
    else
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), false, 4, false, true>), dim3(blocks),
                      dim3(kAttnWaves * 64), stream, p, f, n_row_tiles, (const AttnBatchItem*)nullptr,
                      (const AttnWork*)nullptr);
    return hipGetLastError();
}

hipError_t launch_attn_mfma_pool(const AttnParams& p, const AttnFold& f, hipStream_t stream) {
    const int g = p.n_q_heads / p.n_kv_heads;
    const int rows = p.t_q * g;
    const int n_row_tiles = (rows + kAttnRowTile - 1) / kAttnRowTile;
    const unsigned blocks = (unsigned)(p.n_kv_heads * n_row_tiles * (p.n_split + 1));
    if (blocks == 0) return hipSuccess;
    if (p.no_self || p.split_bounds || !f.slot_src || !f.tile_rot || p.keys_per_split % kTileKeys != 0)
        return hipErrorInvalidValue;
    launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), false, 4, true, true>), dim3(blocks),
                  dim3(kAttnWaves * 64), stream, p, f, n_row_tiles, (const AttnBatchItem*)nullptr, (const AttnWork*)nullptr);
    return hipGetLastError();
}

hipError_t launch_attn_mfma_batched(const AttnBatchItem* items, const AttnWork* work, int n_work, bool pool,
                                    bool stream_tiles, int layer, hipStream_t stream) {
    if (n_work <= 0) return hipSuccess;
    if (pool)
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), true, 4, true, true>), dim3((unsigned)n_work),
                      dim3(kAttnWaves * 64), stream, AttnParams{}, AttnFold{}, layer, items, work);
    else if (stream_tiles)
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), true, 4, false, true, true>),
                      dim3((unsigned)n_work), dim3(kAttnWaves * 64), stream, AttnParams{}, AttnFold{}, layer, items, work);
    else
        launch_kernel((attn_mfma_kernel<kAttnWaves, kAttnRowTile / (32 * kAttnWaves), true, 4, false, true>), dim3((unsigned)n_work),
                      dim3(kAttnWaves * 64), stream, AttnParams{}, AttnFold{}, layer, items, work);
    return hipGetLastError();
}

}  // namespace adapshot
