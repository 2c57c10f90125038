"""Mutation check of the oracle's pins (CPU only).

Each case plants one plausible mistake in a scratch copy of the oracle's C source -- a wrong sign, a
dropped term, a swapped operand or index -- compiles it, and runs the pin suite against that copy in a
child process.  Every mutant has to be caught by at least one pin; an unmodified copy has to pass.
Nothing here touches the GPU or the product library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "adapshot_oracle.c")

# (name, text to find, replacement, which occurrence)
MUTANTS = [
    ("rot_first_sign", "y[i] = x1 * c + (-x2) * s;", "y[i] = x1 * c + x2 * s;", 0),
    ("rot_second_sign", "y[i + h] = x2 * c + x1 * s;", "y[i + h] = x2 * c - x1 * s;", 0),
    ("rot_frequency_exponent", "-2.0 * (double)i / (double)d", "-1.0 * (double)i / (double)d", 0),
    ("rot_cos_sin_swapped", "double c = cos(phi), s = sin(phi);", "double c = sin(phi), s = cos(phi);", 0),
    ("rot_adjacent_pairs", "double x1 = x[i], x2 = x[i + h];", "double x1 = x[i], x2 = x[(i + h + 1) % d];", 0),
    ("plan_position_without_slot0", "slot_pos[i] = pos0 + slot0 + off + t;", "slot_pos[i] = pos0 + off + t;", 0),
    ("plan_order_ignored", "int32_t oj = order ? order[j] : j;", "int32_t oj = j;", 0),
    ("plan_source_is_slot", "slot_src[i] = shot_offsets[s] + t;", "slot_src[i] = off + t;", 0),
    ("plan_positions_restart_per_shot", "slot_pos[i] = pos0 + slot0 + off + t;", "slot_pos[i] = pos0 + slot0 + t;", 0),
    ("assemble_delta_sign", "(double)(slot_pos[i] - (int64_t)slot_tok[i])", "(double)(slot_pos[i] + (int64_t)slot_tok[i])", 0),
    ("assemble_key_states_swapped", "(key_state == ORC_KEYS_ROTATED_LOCAL)", "(key_state != ORC_KEYS_ROTATED_LOCAL)", 0),
    ("assemble_values_from_key_pool", "load_elem(v_pool, dtype, src + (int64_t)h * d + e));",
     "load_elem(k_pool, dtype, src + (int64_t)h * d + e));", 0),
    ("assemble_heads_reversed", "store_elem(k_out, dtype, dst + (int64_t)h * d + e, y[e]);",
     "store_elem(k_out, dtype, dst + (int64_t)(h_kv - 1 - h) * d + e, y[e]);", 0),
    ("assemble_layer_stride", "int64_t dst = ((int64_t)l * capacity + slot0 + i) * row;",
     "int64_t dst = ((int64_t)l * n_new + slot0 + i) * row;", 0),
    ("attn_scale", "double inv_sqrt_d = 1.0 / sqrt((double)d);", "double inv_sqrt_d = 1.0 / (double)d;", 0),
    ("attn_not_causal", "int64_t n_keys = n_ctx + j + 1;", "int64_t n_keys = n_ctx + t_q;", 0),
    ("attn_kv_head_mapping", "int32_t hk = h / g;", "int32_t hk = h % h_kv;", 0),
    ("attn_self_keys_at_local_position", "(double)(q_pos0 + j), ks_rot + o);", "(double)j, ks_rot + o);", 0),
    ("attn_query_not_rotated", "adapshot_oracle_rot(x, d, base, (double)(q_pos0 + j), qr);",
     "adapshot_oracle_rot(x, d, base, 0.0, qr);", 0),
    ("attn_query_read_transposed", "x[e] = load_elem(q, dtype, ((int64_t)j * h_q + h) * d + e);",
     "x[e] = load_elem(q, dtype, ((int64_t)h * t_q + j) * d + e);", 0),
    ("attn_self_values_from_self_keys", "o[e] += p * load_elem(v_self, dtype, vo + e);",
     "o[e] += p * load_elem(k_self, dtype, vo + e);", 0),
    ("attn_not_normalised", "double p = sc[c] / denom;", "double p = sc[c];", 0),
    ("attn_context_key_head", "int64_t ko = (c * h_kv + hk) * d;", "int64_t ko = (c * h_kv) * d;", 0),
    ("entropy_sign", "entropy_out[r] = log(s) - t / s;", "entropy_out[r] = log(s) + t / s;", 0),
    ("entropy_zero_probability_term", "if (e > 0.0) t += dz * e;", "t += dz * e;", 0),
    ("entropy_without_log_sum", "entropy_out[r] = log(s) - t / s;", "entropy_out[r] = -t / s;", 0),
    ("subset_modes_swapped", "if (mode == 0) {", "if (mode != 0) {", 0),
    ("subset_lse_without_max", "const double lse = m + log(s);", "const double lse = log(s);", 0),
    ("subset_renormalised_over_vocab", "const double lse = mc + log(s);", "const double lse = m + log(s);", 0),
    ("pick_strict_threshold", "if (h[i] <= tau &&", "if (h[i] < tau &&", 0),
    ("pick_largest_passing", "counts[i] < best", "counts[i] > best", 0),
    ("rank_not_per_token", " * (double)(shot_offsets[i + 1] - shot_offsets[i]);", ";", 0),
    ("rank_keys_at_pool_position", "(double)(u - shot_offsets[i]), y);", "(double)u, y);", 0),
    ("rank_query_not_rotated", "adapshot_oracle_rot(x, d, base, (double)(q_pos0 + j), qr);",
     "adapshot_oracle_rot(x, d, base, 0.0, qr);", 1),
    ("rank_rotated_keys_not_rounded", "kc[o + e] = dtype == ORC_BF16 ?", "kc[o + e] = dtype == 77 ?", 0),
    ("rank_key_states_swapped", "if (key_state == ORC_KEYS_UNROTATED) {", "if (key_state != ORC_KEYS_UNROTATED) {", 0),
    ("rank_scale", "double inv_sqrt_d = 1.0 / sqrt((double)d);", "double inv_sqrt_d = 1.0;", 1),
    ("attn_context_value_head", "int64_t vo = (c * h_kv + hk) * d;", "int64_t vo = (c * h_kv) * d;", 0),
    ("attn_self_value_head", "int64_t vo = ((c - n_ctx) * h_kv + hk) * d;", "int64_t vo = ((c - n_ctx) * h_kv) * d;", 0),
    ("attn_self_key_head", "ks_rot + ((c - n_ctx) * h_kv + hk) * d;", "ks_rot + ((c - n_ctx) * h_kv) * d;", 0),
    ("assemble_pool_layer_stride", "((int64_t)l * pool_layer_stride_tokens + slot_src[i]) * row;",
     "((int64_t)l * n_new + slot_src[i]) * row;", 0),
    ("assemble_exact_fit_rejected", "slot0 + n_new > capacity) return -1;", "slot0 + n_new >= capacity) return -1;", 0),
    ("rot_rows_one_angle", "adapshot_oracle_rot(xi, d, base, a[r], yo);", "adapshot_oracle_rot(xi, d, base, a[0], yo);", 0),
    ("plan_token_index", "slot_tok[i] = (int32_t)t;", "slot_tok[i] = (int32_t)i;", 0),
    ("plan_shot_is_order_entry", "slot_shot[i] = s;", "slot_shot[i] = oj;", 0),
    ("subset_full_p_zero_term", "if (pc > 0.0) h -= pc * lp;", "h -= pc * lp;", 0),
    ("subset_renormalised_zero_term", "if (pc > 0.0) h -= pc * lp;", "h -= pc * lp;", 1),
    ("rank_mass_not_normalised", "acc[shot_of[u]] += sc[u] / denom;", "acc[shot_of[u]] += sc[u];", 0),
    ("rank_not_averaged_over_heads", "scores[i] /= (double)t_q * (double)h_q *", "scores[i] /= (double)t_q *", 0),
    ("rank_kv_head_mapping", ", hk = h / g;", ", hk = h % h_kv;", 0),
    ("bf16_sign_lost", "uint16_t sign = signbit(x) ? 0x8000u : 0u;", "uint16_t sign = 0u;", 0),
    ("bf16_subnormal_spacing", "if (q < -133) q = -133;", "if (q < -1000) q = -1000;", 0),
    ("bf16_truncates", "double r = rint(ldexp(ax, -q));", "double r = floor(ldexp(ax, -q));", 0),
    ("bf16_seven_bits", "int q = e - 8; ", "int q = e - 7; ", 0),
]


def _mutate(text, find, repl, nth):
    parts = text.split(find)
    assert len(parts) - 1 > nth, f"pattern not found often enough: {find!r}"
    line = find.join(parts[:nth + 1]).rsplit("\n", 1)[-1].strip()
    assert not line.startswith(("*", "/*")), f"pattern {find!r} #{nth} sits in a comment"
    return find.join(parts[:nth + 1]) + repl + find.join(parts[nth + 1:])


def _run_pins(src_path):
    env = dict(os.environ, ADAPSHOT_ORACLE_SRC=src_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    return r.returncode, r.stdout


def _compile(src_path):
    lib = os.path.join(os.path.dirname(src_path), "libadapshot_oracle.so")
    subprocess.run(["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", src_path, "-o", lib, "-lm"],
                   check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)


def test_names_are_unique():
    names = [m[0] for m in MUTANTS]
    assert len(set(names)) == len(names)


def test_every_planted_mistake_is_caught_by_a_pin(tmp_path):
    text = open(SRC).read()
    jobs = [("unmodified", text)]
    for name, find, repl, nth in MUTANTS:
        mutated = _mutate(text, find, repl, nth)
        assert mutated != text
        jobs.append((name, mutated))

    def work(job):
        name, body = job
        d = tmp_path / name
        d.mkdir()
        src = str(d / "adapshot_oracle.c")
        with open(src, "w") as f:
            f.write(body)
        _compile(src)
        return name, *_run_pins(src)

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(work, jobs))
    report = {name: (rc, out) for name, rc, out in results}
    rc, out = report.pop("unmodified")
    assert rc == 0, "the pin suite fails on an unmodified copy of the oracle:\n" + out[-2000:]
    survivors = [n for n, (rc, _) in report.items() if rc == 0]
    assert not survivors, f"no pin notices these planted mistakes: {survivors}"
    broken = {n: out[-800:] for n, (rc, out) in report.items() if rc not in (0, 1)}
    assert not broken, f"the pin run itself broke (not a test failure): {broken}"
