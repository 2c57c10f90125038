/*
 * adapshot_oracle.c -- plain CPU oracle for the AdapShot KV-reuse hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the HIP
 * library can be checked element by element against a slow, obviously correct
 * implementation.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  It shares no code, header, table or constant with the HIP
 * path and is never a fallback for it.
 *
 * Everything is written as the defining formula, in straight loops, with fp64
 * arithmetic.  Stored tensors are either fp32 or bf16 (bf16 passed as uint16 bit
 * patterns); both convert exactly to fp64 on load, and a result is rounded once,
 * to nearest-even, when it is stored back in the storage type.  OpenMP is used
 * only across independent units (tokens, (row, head) pairs, logit rows).
 *
 * What each function follows (AdapShot paper):
 *   plan      -- Position Decoupling and Re-encoding: the two-shot concatenation
 *                example (shot_B after shot_A gets positions T_A .. T_A+T_B-1),
 *                and Eq. (probe_context): instruction prefix, then shots in order.
 *   rot       -- Eq. (rope_encoding) / Eq. (rope_compensation):
 *                x * cos(a*theta) + rotate_half(x) * sin(a*theta),
 *                theta_i = base^(-2i/d), halves paired as (i, i + d/2).
 *   assemble  -- Semantically-Aware KV Cache (concatenate cached blocks in rank
 *                order) + Eq. (rope_compensation) applied to every key.
 *   attention -- softmax(q k^T / sqrt(d)) v as in Eq. (attention_score), for the
 *                probe/query tokens of Eq. (probe_context) over the assembled
 *                context plus their own tokens (causal).
 *   entropy   -- Eq. (entropy), H = -sum p log p, here over the whole vocabulary
 *                of one output distribution, natural log.
 *   rot_rows  -- rot applied row by row with stored input/output (decode-step append).
 *   entropy_subset -- Eq. (entropy) as printed: the sum runs over a set C of answer
 *                tokens only (Yes / No), in two readings of p (see the function).
 *   rank_scores -- relevance of every pool shot to a query (Eq. attention_score), the
 *                quantity the examples are sorted by; the reading is stated at the function.
 *   pick_shots -- the stopping rule of the probe iteration: the smallest candidate
 *                shot count whose probe entropy is <= tau (Probe-based Dynamic
 *                Evaluation; parallel multi-probe selects the minimum passing count).
 *
 * Parity pins for every function live in tests/test_oracle_*.py; none of the
 * functions below is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_KEYS_UNROTATED = 0, ORC_KEYS_ROTATED_LOCAL = 1 };

int32_t adapshot_oracle_threads(void) {
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- storage <-> fp64 ------------------------------------------------------ */

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f; /* exact */
}

/* Round an fp64 value to bf16 (8 significant bits, fp32 exponent range) with
 * round-to-nearest-even, in ONE rounding step (not via fp32). */
uint16_t adapshot_oracle_double_to_bf16(double x) {
    if (isnan(x)) return 0x7FC0u;
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double ax = fabs(x);
    if (isinf(ax)) return (uint16_t)(sign | 0x7F80u);
    if (ax == 0.0) return sign;
    int e;
    (void)frexp(ax, &e);          /* ax = f * 2^e, f in [0.5, 1) */
    int q = e - 8;                /* spacing of bf16 numbers near ax is 2^(e-8) */
    if (q < -133) q = -133;       /* bf16 subnormal spacing: 2^-126 * 2^-7 */
    double r = rint(ldexp(ax, -q)); /* rint: current mode = nearest-even */
    double y = ldexp(r, q);       /* exactly a bf16 value (or 2^128 on overflow) */
    float f = (float)y;           /* exact, or +inf */
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(sign | (uint16_t)(u >> 16));
}

static double load_elem(const void* base, int dtype, int64_t idx) {
    if (dtype == ORC_BF16) return bf16_bits_to_double(((const uint16_t*)base)[idx]);
    return (double)((const float*)base)[idx];
}

static void store_elem(void* base, int dtype, int64_t idx, double v) {
    if (dtype == ORC_BF16) ((uint16_t*)base)[idx] = adapshot_oracle_double_to_bf16(v);
    else ((float*)base)[idx] = (float)v; /* C conversion: correctly rounded, nearest-even */
}

/* ---- plan: slot / position indexing ------------------------------------------ */

/* Slot j of the appended context (j = 0..m-1) holds shot s_j = shot_ids[order[j]]
 * (order == NULL: identity).  With off_0 = 0 and off_j = sum_{r<j} T_{s_r}, token t
 * of that shot lands at slot slot0 + off_j + t and gets position pos0 + slot.
 * Outputs are indexed by the appended token (0 .. n-1):
 *   slot_shot = pool shot id, slot_tok = t, slot_pos = new position,
 *   slot_src  = token index inside the pool (shot_offsets[s] + t).
 * Returns n (the number of appended tokens), or -1 for a shot id or an order
 * entry out of range.  Output pointers may be NULL (then only n is computed). */
int64_t adapshot_oracle_plan(const int64_t* shot_offsets, int32_t n_shots,
                             const int32_t* shot_ids, const int32_t* order, int32_t m,
                             int64_t slot0, int64_t pos0,
                             int32_t* slot_shot, int32_t* slot_tok,
                             int64_t* slot_pos, int64_t* slot_src) {
    int64_t off = 0;
    for (int32_t j = 0; j < m; ++j) {
        int32_t oj = order ? order[j] : j;
        if (oj < 0 || oj >= m) return -1;
        int32_t s = shot_ids[oj];
        if (s < 0 || s >= n_shots) return -1;
        int64_t len = shot_offsets[s + 1] - shot_offsets[s];
        for (int64_t t = 0; t < len; ++t) {
            int64_t i = off + t;
            if (slot_shot) slot_shot[i] = s;
            if (slot_tok) slot_tok[i] = (int32_t)t;
            if (slot_pos) slot_pos[i] = pos0 + slot0 + off + t;
            if (slot_src) slot_src[i] = shot_offsets[s] + t;
        }
        off += len;
    }
    return off;
}

/* ---- rot: RoPE at angle multiplier a ----------------------------------------- */

/* y = x (.) cos(a*theta) + rotate_half(x) (.) sin(a*theta), where theta has d/2
 * entries theta_i = base^(-2i/d), cos/sin are tiled over both halves, and
 * rotate_half(x) = [-x_{d/2..d-1}, x_{0..d/2-1}].  Written per pair (i, i+d/2). */
void adapshot_oracle_rot(const double* x, int32_t d, double base, double a, double* y) {
    int32_t h = d / 2;
    for (int32_t i = 0; i < h; ++i) {
        double theta_i = pow(base, -2.0 * (double)i / (double)d);
        double phi = a * theta_i;
        double c = cos(phi), s = sin(phi);
        double x1 = x[i], x2 = x[i + h];
        y[i] = x1 * c + (-x2) * s;
        y[i + h] = x2 * c + x1 * s;
    }
}

/* Rotate n_rows stored rows of length d, row r by angle multiplier a[r] (rot above), and store them
 * rounded once to the storage type; y_exact (optional, fp64 [n_rows][d]) gets the unrounded rows.
 * This is the decode-step append: a new token's key from the model, brought to its position
 * (Eq. rope_encoding with p = position). */
void adapshot_oracle_rot_rows(const void* x, int dtype, int64_t n_rows, int32_t d, double base,
                              const double* a, void* y, double* y_exact) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        double xi[1024], yo[1024];
        if (d > 1024) continue;
        for (int32_t e = 0; e < d; ++e) xi[e] = load_elem(x, dtype, r * d + e);
        adapshot_oracle_rot(xi, d, base, a[r], yo);
        for (int32_t e = 0; e < d; ++e) {
            store_elem(y, dtype, r * d + e, yo[e]);
            if (y_exact) y_exact[r * d + e] = yo[e];
        }
    }
}

/* ---- assemble: gather + re-encode --------------------------------------------- */

/* For every layer l and appended token i (0..n_new-1), with slot = slot0 + i:
 *   V_out[l, slot, :, :] = V_pool[l, slot_src[i], :, :]           (bit copy)
 *   K_out[l, slot, h, :] = rot(K_pool[l, slot_src[i], h, :], a_i)
 * where a_i = slot_pos[i] if the pool keys carry no rotation (UNROTATED), or
 * a_i = slot_pos[i] - slot_tok[i] (= Delta, the shot's offset) if they were
 * prefilled at local positions 0..T-1 (ROTATED_LOCAL), Eq. (rope_compensation).
 * Pool layout [L][pool_layer_stride_tokens][h_kv][d]; output [L][capacity][h_kv][d].
 * k_exact (optional, fp64 [L][n_new][h_kv][d]) receives the keys before rounding.
 * Returns 0, or -1 if slot0 + n_new > capacity. */
int adapshot_oracle_assemble(const void* k_pool, const void* v_pool, int dtype,
                             int32_t n_layers, int64_t pool_layer_stride_tokens,
                             int32_t h_kv, int32_t d, double base, int key_state,
                             const int64_t* slot_src, const int32_t* slot_tok,
                             const int64_t* slot_pos, int64_t n_new, int64_t slot0,
                             void* k_out, void* v_out, int64_t capacity, double* k_exact) {
    if (slot0 < 0 || slot0 + n_new > capacity) return -1;
    if (d <= 0 || d % 2 != 0 || d > 1024) return -1;
    int64_t row = (int64_t)h_kv * d;
    for (int32_t l = 0; l < n_layers; ++l) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n_new; ++i) {
            double x[1024], y[1024];
            int64_t src = ((int64_t)l * pool_layer_stride_tokens + slot_src[i]) * row;
            int64_t dst = ((int64_t)l * capacity + slot0 + i) * row;
            double a = (key_state == ORC_KEYS_ROTATED_LOCAL)
                           ? (double)(slot_pos[i] - (int64_t)slot_tok[i])
                           : (double)slot_pos[i];
            for (int32_t h = 0; h < h_kv; ++h) {
                for (int32_t e = 0; e < d; ++e) x[e] = load_elem(k_pool, dtype, src + (int64_t)h * d + e);
                adapshot_oracle_rot(x, d, base, a, y);
                for (int32_t e = 0; e < d; ++e) {
                    store_elem(k_out, dtype, dst + (int64_t)h * d + e, y[e]);
                    if (k_exact) k_exact[((int64_t)l * n_new + i) * row + (int64_t)h * d + e] = y[e];
                }
                for (int32_t e = 0; e < d; ++e)
                    store_elem(v_out, dtype, dst + (int64_t)h * d + e,
                               load_elem(v_pool, dtype, src + (int64_t)h * d + e));
            }
        }
    }
    return 0;
}

/* ---- attention: query rows over the assembled context + causal self ------------- */

/* One layer.  k_cache / v_cache: [>= n_ctx][h_kv][d] (keys already at their
 * positions).  q: [t_q][h_q][d], k_self / v_self: [t_q][h_kv][d], all given
 * WITHOUT rotation; row j is rotated to position q_pos0 + j here.  Query head h
 * uses kv head h / (h_q / h_kv).  Row j sees context slots 0..n_ctx-1 and self
 * tokens 0..j.  Score = q~ . k / sqrt(d); softmax over all visible keys; output
 * = sum p * v.  If `pairs` is NULL all (j, h) are computed into out[t_q][h_q][d];
 * otherwise pairs holds n_pairs (j, h) couples and out is [n_pairs][d].
 * Returns 0, -1 on bad arguments. */
int adapshot_oracle_query_attn(const void* k_cache, const void* v_cache, int dtype, int64_t n_ctx,
                               const void* q, const void* k_self, const void* v_self,
                               int32_t t_q, int32_t h_q, int32_t h_kv, int32_t d, double base,
                               int64_t q_pos0, const int32_t* pairs, int64_t n_pairs, double* out) {
    if (h_kv <= 0 || h_q % h_kv != 0 || d <= 0 || d % 2 != 0 || d > 1024 || t_q < 0 || n_ctx < 0) return -1;
    int32_t g = h_q / h_kv;
    int64_t n_units = pairs ? n_pairs : (int64_t)t_q * h_q;
    double inv_sqrt_d = 1.0 / sqrt((double)d);

    /* rotate the self keys once: ks_rot[j][hk][:] = rot(k_self[j][hk][:], q_pos0 + j) */
    double* ks_rot = (double*)malloc(sizeof(double) * (size_t)(t_q > 0 ? t_q : 1) * h_kv * d);
    if (!ks_rot) return -1;
    for (int32_t j = 0; j < t_q; ++j)
        for (int32_t hk = 0; hk < h_kv; ++hk) {
            double x[1024];
            int64_t o = ((int64_t)j * h_kv + hk) * d;
            for (int32_t e = 0; e < d; ++e) x[e] = load_elem(k_self, dtype, o + e);
            adapshot_oracle_rot(x, d, base, (double)(q_pos0 + j), ks_rot + o);
        }

    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < n_units; ++u) {
        int32_t j = pairs ? pairs[2 * u] : (int32_t)(u / h_q);
        int32_t h = pairs ? pairs[2 * u + 1] : (int32_t)(u % h_q);
        double* o = out + u * d;
        if (j < 0 || j >= t_q || h < 0 || h >= h_q) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        int32_t hk = h / g;
        int64_t n_keys = n_ctx + j + 1;
        double* sc = (double*)malloc(sizeof(double) * (size_t)n_keys);
        if (!sc) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        double x[1024], qr[1024];
        for (int32_t e = 0; e < d; ++e) x[e] = load_elem(q, dtype, ((int64_t)j * h_q + h) * d + e);
        adapshot_oracle_rot(x, d, base, (double)(q_pos0 + j), qr);

        double mx = -INFINITY;
        for (int64_t c = 0; c < n_keys; ++c) {
            double dot = 0.0;
            if (c < n_ctx) {
                int64_t ko = (c * h_kv + hk) * d;
                for (int32_t e = 0; e < d; ++e) dot += qr[e] * load_elem(k_cache, dtype, ko + e);
            } else {
                const double* kr = ks_rot + ((c - n_ctx) * h_kv + hk) * d;
                for (int32_t e = 0; e < d; ++e) dot += qr[e] * kr[e];
            }
            sc[c] = dot * inv_sqrt_d;
            if (sc[c] > mx) mx = sc[c];
        }
        double denom = 0.0;
        for (int64_t c = 0; c < n_keys; ++c) {
            sc[c] = exp(sc[c] - mx);
            denom += sc[c];
        }
        for (int32_t e = 0; e < d; ++e) o[e] = 0.0;
        for (int64_t c = 0; c < n_keys; ++c) {
            double p = sc[c] / denom;
            if (c < n_ctx) {
                int64_t vo = (c * h_kv + hk) * d;
                for (int32_t e = 0; e < d; ++e) o[e] += p * load_elem(v_cache, dtype, vo + e);
            } else {
                int64_t vo = ((c - n_ctx) * h_kv + hk) * d;
                for (int32_t e = 0; e < d; ++e) o[e] += p * load_elem(v_self, dtype, vo + e);
            }
        }
        free(sc);
    }
    free(ks_rot);
    return failed ? -1 : 0;
}

/* ---- entropy of softmax(logits) ------------------------------------------------- */

/* H = -sum_v p_v ln p_v with p = softmax(z).  With m = max z, e_v = exp(z_v - m),
 * s = sum e_v:  ln p_v = (z_v - m) - ln s, so H = ln s - (sum (z_v - m) e_v) / s.
 * A term with e_v == 0 contributes 0 (p ln p -> 0 as p -> 0), which also covers
 * logits equal to -infinity.  A row holding a NaN, +infinity, or only -infinity
 * has no defined distribution and yields NaN. */
void adapshot_oracle_entropy(const float* logits, int64_t row_stride, int32_t n_rows,
                             int32_t vocab, double* entropy_out) {
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < n_rows; ++r) {
        const float* z = logits + (int64_t)r * row_stride;
        double m = -INFINITY;
        int bad = (vocab <= 0);
        for (int32_t v = 0; v < vocab; ++v) {
            double zv = (double)z[v];
            if (isnan(zv) || zv == INFINITY) bad = 1;
            if (zv > m) m = zv;
        }
        if (bad || m == -INFINITY) {
            entropy_out[r] = NAN;
            continue;
        }
        double s = 0.0, t = 0.0;
        for (int32_t v = 0; v < vocab; ++v) {
            double dz = (double)z[v] - m;
            double e = exp(dz);
            s += e;
            if (e > 0.0) t += dz * e;
        }
        entropy_out[r] = log(s) - t / s;
    }
}

/* ---- Eq. (entropy) over a set C of answer tokens ------------------------------------ */

/* H = -sum_{c in C} p_c ln p_c.
 * mode 0: p_c is the probability of token c under the softmax over the WHOLE vocabulary
 *         (the sum simply leaves the other tokens' terms out; it can reach 2/e for |C| = 2,
 *         which is what the values above ln 2 printed in the case study need);
 * mode 1: p is renormalised over C, p_c = e^{z_c} / sum_{c' in C} e^{z_c'} (a proper
 *         |C|-class entropy, at most ln |C|).
 * ids are distinct token indices in [0, vocab).  A row holding a NaN, +infinity or only
 * -infinity yields NaN; in mode 1 a row whose C-logits are all -infinity yields NaN too. */
void adapshot_oracle_entropy_subset(const float* logits, int64_t row_stride, int32_t n_rows,
                                    int32_t vocab, const int32_t* ids, int32_t n_ids, int32_t mode,
                                    double* entropy_out) {
    for (int32_t r = 0; r < n_rows; ++r) {
        const float* z = logits + (int64_t)r * row_stride;
        double m = -INFINITY;
        int bad = (vocab <= 0);
        for (int32_t v = 0; v < vocab; ++v) {
            double zv = (double)z[v];
            if (isnan(zv) || zv == INFINITY) bad = 1;
            if (zv > m) m = zv;
        }
        if (bad || m == -INFINITY) {
            entropy_out[r] = NAN;
            continue;
        }
        double h = 0.0;
        if (mode == 0) {
            double s = 0.0;
            for (int32_t v = 0; v < vocab; ++v) s += exp((double)z[v] - m);
            const double lse = m + log(s);
            for (int32_t c = 0; c < n_ids; ++c) {
                const double lp = (double)z[ids[c]] - lse; /* ln p_c */
                const double pc = exp(lp);
                if (pc > 0.0) h -= pc * lp;
            }
        } else {
            double mc = -INFINITY;
            for (int32_t c = 0; c < n_ids; ++c)
                if ((double)z[ids[c]] > mc) mc = (double)z[ids[c]];
            if (mc == -INFINITY) {
                entropy_out[r] = NAN;
                continue;
            }
            double s = 0.0;
            for (int32_t c = 0; c < n_ids; ++c) s += exp((double)z[ids[c]] - mc);
            const double lse = mc + log(s);
            for (int32_t c = 0; c < n_ids; ++c) {
                const double lp = (double)z[ids[c]] - lse;
                const double pc = exp(lp);
                if (pc > 0.0) h -= pc * lp;
            }
        }
        entropy_out[r] = h;
    }
}

/* ---- stopping rule of the probe iteration ----------------------------------------- */

/* counts[i] shots gave probe entropy h[i].  A candidate passes when h[i] <= tau; the
 * answer is the smallest passing count, or -1 when none passes (the caller then probes
 * larger counts).  A NaN entropy never passes. */
int32_t adapshot_oracle_pick_shots(const double* h, const int32_t* counts, int32_t n, double tau) {
    int32_t best = -1;
    for (int32_t i = 0; i < n; ++i)
        if (h[i] <= tau && (best < 0 || counts[i] < best)) best = counts[i];
    return best;
}

/* ---- relevance of the pool's shots to a query (Eq. attention_score) ----------------- */

/* The query attends to the cached keys of the pool at one representative layer; the
 * attention a shot receives, averaged over heads, query tokens and the shot's tokens,
 * is its relevance s^(i).
 *
 * Reading.  As printed, the softmax runs over one shot's own T_i keys; each row of that
 * matrix sums to 1, so its average over all T_q x T_i entries is 1/T_i whatever the
 * content.  Here the softmax runs over the keys of the WHOLE pool (the shots compete for
 * the query's attention), and
 *     s^(i) = 1 / (T_q H_q T_i) * sum_{j, h} sum_{u in shot i} A_h[j, u].
 * Keys are what the cache holds: the key of token t of a shot encoded at its local
 * position t (Eq. prefill; for an un-rotated pool it is rotated here and rounded to the
 * storage type, as a cache would hold it).  The query is encoded on its own: token j at
 * position q_pos0 + j.  Score = q~ . k~ / sqrt(d), kv head = h / (h_q / h_kv).
 * k_pool: one layer [tokens][h_kv][d]; scores: [n_shots].  Returns 0, -1 on bad arguments. */
int adapshot_oracle_rank_scores(const void* k_pool, int dtype, const int64_t* shot_offsets, int32_t n_shots,
                                const void* q, int32_t t_q, int32_t h_q, int32_t h_kv, int32_t d, double base,
                                int key_state, int64_t q_pos0, double* scores) {
    if (h_kv <= 0 || h_q % h_kv != 0 || d <= 0 || d % 2 != 0 || d > 1024 || t_q <= 0 || n_shots <= 0) return -1;
    const int32_t g = h_q / h_kv;
    const int64_t n_tok = shot_offsets[n_shots];
    if (n_tok <= 0) return -1;
    double* kc = (double*)malloc(sizeof(double) * (size_t)n_tok * h_kv * d);
    int32_t* shot_of = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_tok);
    if (!kc || !shot_of) {
        free(kc);
        free(shot_of);
        return -1;
    }
    for (int32_t i = 0; i < n_shots; ++i)
        for (int64_t u = shot_offsets[i]; u < shot_offsets[i + 1]; ++u) {
            shot_of[u] = i;
            for (int32_t hk = 0; hk < h_kv; ++hk) {
                double x[1024], y[1024];
                const int64_t o = (u * h_kv + hk) * d;
                for (int32_t e = 0; e < d; ++e) x[e] = load_elem(k_pool, dtype, o + e);
                if (key_state == ORC_KEYS_UNROTATED) {
                    adapshot_oracle_rot(x, d, base, (double)(u - shot_offsets[i]), y);
                    for (int32_t e = 0; e < d; ++e) /* what a cache of this storage type holds */
                        kc[o + e] = dtype == ORC_BF16 ? bf16_bits_to_double(adapshot_oracle_double_to_bf16(y[e]))
                                                      : (double)(float)y[e];
                } else {
                    for (int32_t e = 0; e < d; ++e) kc[o + e] = x[e];
                }
            }
        }
    for (int32_t i = 0; i < n_shots; ++i) scores[i] = 0.0;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    int failed = 0;
#pragma omp parallel
    {
        double* acc = (double*)calloc((size_t)n_shots, sizeof(double));
        double* sc = (double*)malloc(sizeof(double) * (size_t)n_tok);
        if (!acc || !sc) {
#pragma omp atomic write
            failed = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < (int64_t)t_q * h_q; ++r) {
                const int32_t j = (int32_t)(r / h_q), h = (int32_t)(r % h_q), hk = h / g;
                double x[1024], qr[1024];
                for (int32_t e = 0; e < d; ++e) x[e] = load_elem(q, dtype, ((int64_t)j * h_q + h) * d + e);
                adapshot_oracle_rot(x, d, base, (double)(q_pos0 + j), qr);
                double mx = -INFINITY;
                for (int64_t u = 0; u < n_tok; ++u) {
                    const double* k = kc + (u * h_kv + hk) * d;
                    double dot = 0.0;
                    for (int32_t e = 0; e < d; ++e) dot += qr[e] * k[e];
                    sc[u] = dot * inv_sqrt_d;
                    if (sc[u] > mx) mx = sc[u];
                }
                double denom = 0.0;
                for (int64_t u = 0; u < n_tok; ++u) {
                    sc[u] = exp(sc[u] - mx);
                    denom += sc[u];
                }
                for (int64_t u = 0; u < n_tok; ++u) acc[shot_of[u]] += sc[u] / denom;
            }
#pragma omp critical
            for (int32_t i = 0; i < n_shots; ++i) scores[i] += acc[i];
        }
        free(acc);
        free(sc);
    }
    for (int32_t i = 0; i < n_shots; ++i)
        scores[i] /= (double)t_q * (double)h_q * (double)(shot_offsets[i + 1] - shot_offsets[i]);
    free(kc);
    free(shot_of);
    return failed ? -1 : 0;
}
