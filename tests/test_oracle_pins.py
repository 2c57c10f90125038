"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- the paper's worked example, closed forms, invariants,
library routines on the special cases that reduce to them, and brute force on
tiny inputs.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _constants():
    out = {}
    for line in open(os.path.join(GOLD, "constants.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v)
    return out


# ---------------------------------------------------------------- bf16 rounding

def test_bf16_rounding_matches_library_on_fp32_inputs(oracle_mod):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32),
                        (rng.standard_normal(500) * 1e-30).astype(np.float32),
                        (rng.standard_normal(500) * 1e30).astype(np.float32),
                        (rng.standard_normal(500) * 3e-39).astype(np.float32),   # bf16 subnormals
                        np.array([0.0, -0.0, 1.0, -1.0, 3.3895314e38, 1e-40, -1e-40, 9.2e-41], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle_mod.double_to_bf16(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want)


def test_bf16_rounding_ties_and_single_step(oracle_mod):
    f = oracle_mod.double_to_bf16
    assert f(1.0) == 0x3F80
    assert f(1.0 + 2.0 ** -8) == 0x3F80           # tie -> even mantissa
    assert f(1.0 + 3 * 2.0 ** -8) == 0x3F82       # tie -> even mantissa
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81   # just above the tie: one rounding, not two
    assert f(1.0 + 2.0 ** -8 - 2.0 ** -40) == 0x3F80
    assert f(float("inf")) == 0x7F80 and f(float("-inf")) == 0xFF80
    assert f(3.4e38) == 0x7F80                    # above the largest bf16 (3.3895e38) + half spacing
    assert f(2.0 ** -133) == 0x0001 and f(2.0 ** -135) == 0x0000
    # subnormal range: the spacing stays 2^-133, ties go to the even code
    assert f(0.75 * 2.0 ** -133) == 0x0001 and f(1.75 * 2.0 ** -133) == 0x0002
    assert f(1.5 * 2.0 ** -133) == 0x0002 and f(2.5 * 2.0 ** -133) == 0x0002 and f(-3.5 * 2.0 ** -133) == 0x8004
    assert f(127.5 * 2.0 ** -133) == 0x0080      # rounds up into the smallest normal number
    assert oracle_mod.bf16_bits_to_f64(np.array([0x3F81], np.uint16))[0] == 1.0078125


# ---------------------------------------------------------------- plan / indexing

def test_plan_paper_two_shot_example(oracle_mod):
    rows = [list(map(int, l.split())) for l in open(os.path.join(GOLD, "two_shot_positions.txt"))
            if l.strip() and not l.startswith("#")]
    rows = np.array(rows)
    offsets = np.array([0, 5, 8], np.int64)        # pool: shot A (5 tokens) then shot B (3 tokens)
    pl = oracle_mod.plan(offsets, [0, 1], None)
    assert pl["n"] == 8
    assert np.array_equal(pl["slot_shot"], rows[:, 1])
    assert np.array_equal(pl["slot_tok"], rows[:, 2])
    assert np.array_equal(pl["slot_pos"], rows[:, 3])
    assert np.array_equal(pl["slot_pos"] - pl["slot_tok"], rows[:, 4])
    # B before A: B now starts at 0 and A is shifted by T_B
    pl = oracle_mod.plan(offsets, [0, 1], [1, 0])
    assert list(pl["slot_shot"]) == [1, 1, 1, 0, 0, 0, 0, 0]
    assert list(pl["slot_pos"] - pl["slot_tok"]) == [0, 0, 0, 3, 3, 3, 3, 3]
    assert list(pl["slot_src"]) == [5, 6, 7, 0, 1, 2, 3, 4]


def test_plan_bruteforce_concatenation(oracle_mod):
    rng = np.random.default_rng(7)
    for trial in range(20):
        n = int(rng.integers(1, 12))
        lens = rng.integers(1, 9, size=n)
        offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        m = int(rng.integers(0, 10))
        ids = rng.integers(0, n, size=m).astype(np.int32)          # duplicates allowed
        order = rng.permutation(m).astype(np.int32)
        slot0, pos0 = int(rng.integers(0, 5)), int(rng.integers(0, 100))
        pl = oracle_mod.plan(offsets, ids, order, slot0=slot0, pos0=pos0)
        shot, tok, src = [], [], []
        for j in range(m):
            s = int(ids[order[j]])
            for t in range(int(lens[s])):
                shot.append(s); tok.append(t); src.append(int(offsets[s]) + t)
        assert pl["n"] == len(shot)
        assert list(pl["slot_shot"]) == shot and list(pl["slot_tok"]) == tok and list(pl["slot_src"]) == src
        assert list(pl["slot_pos"]) == [pos0 + slot0 + i for i in range(len(shot))]


def test_plan_rejects_bad_ids(oracle_mod):
    offsets = np.array([0, 2, 5], np.int64)
    with pytest.raises(ValueError):
        oracle_mod.plan(offsets, [0, 2], None)
    with pytest.raises(ValueError):
        oracle_mod.plan(offsets, [-1], None)
    with pytest.raises(ValueError):
        oracle_mod.plan(offsets, [0, 1], [0, 2])
    assert oracle_mod.plan(offsets, [], None)["n"] == 0


# ---------------------------------------------------------------- rot

def _rot_complex(x, base, a):
    """Brute force: the pair (x_i, x_{i+d/2}) as a complex number times e^{i a theta_i}."""
    d = x.shape[-1]
    h = d // 2
    z = x[..., :h] + 1j * x[..., h:]
    theta = np.array([base ** (-2.0 * i / d) for i in range(h)])
    w = z * np.exp(1j * a * theta)
    return np.concatenate([w.real, w.imag], axis=-1)


@pytest.mark.parametrize("d,base", [(64, 1.0e4), (128, 5.0e5), (128, 1.0e6), (2, 10000.0), (6, 123.0)])
def test_rot_bruteforce_complex(oracle_mod, d, base):
    rng = np.random.default_rng(d)
    for a in [0, 1, 17, 4095, 26000, 131071]:
        x = rng.standard_normal(d)
        assert np.allclose(oracle_mod.rot(x, base, a), _rot_complex(x, base, a), rtol=0, atol=1e-11)


def test_rot_closed_forms(oracle_mod):
    c = _constants()
    e0 = np.zeros(8); e0[0] = 1.0
    y = oracle_mod.rot(e0, 10000.0, 1.0)             # theta_0 = 1: pair (0, 4) turns by 1 rad
    want = np.zeros(8); want[0] = c["cos1"]; want[4] = c["sin1"]
    assert np.allclose(y, want, atol=1e-15)
    y = oracle_mod.rot(e0, 500000.0, 2.0)
    want = np.zeros(8); want[0] = c["cos2"]; want[4] = c["sin2"]
    assert np.allclose(y, want, atol=1e-15)
    # second half of the pair: (0,1) turns to (-sin, cos)
    e4 = np.zeros(8); e4[4] = 1.0
    y = oracle_mod.rot(e4, 10000.0, 1.0)
    want = np.zeros(8); want[0] = -c["sin1"]; want[4] = c["cos1"]
    assert np.allclose(y, want, atol=1e-15)
    # theta_1 = base^(-2/d): d = 4, base = 1e4 -> 0.01, so a = 100 turns pair (1, 3) by 1 rad
    e1 = np.zeros(4); e1[1] = 1.0
    y = oracle_mod.rot(e1, 10000.0, 100.0)
    assert np.allclose(y, [0.0, c["cos1"], 0.0, c["sin1"]], atol=1e-13)
    # quarter turn maps x_i -> x_{i+d/2}
    y = oracle_mod.rot(np.array([1.0, 0.0]), 7.0, math.pi / 2)
    assert np.allclose(y, [0.0, 1.0], atol=1e-15)


def test_rot_invariants(oracle_mod):
    rng = np.random.default_rng(3)
    d, base = 128, 5.0e5
    x = rng.standard_normal(d)
    assert np.array_equal(oracle_mod.rot(x, base, 0.0), x)                     # R(0) = I
    for a, b in [(3, 5), (100, 26500), (70000, 61071), (12345, -12345)]:
        ab = oracle_mod.rot(oracle_mod.rot(x, base, a), base, b)
        assert np.allclose(ab, oracle_mod.rot(x, base, a + b), atol=1e-10)     # R(a)R(b) = R(a+b)
    y = oracle_mod.rot(x, base, 9999)
    h = d // 2
    assert np.allclose(x[:h] ** 2 + x[h:] ** 2, y[:h] ** 2 + y[h:] ** 2, atol=1e-12)  # pair norms kept
    # q~ . k~ depends on the position difference only
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    s0 = oracle_mod.rot(q, base, 500) @ oracle_mod.rot(k, base, 123)
    s1 = oracle_mod.rot(q, base, 500 + 77777) @ oracle_mod.rot(k, base, 123 + 77777)
    assert abs(s0 - s1) < 1e-9


def test_rot_rows_bruteforce_and_rounding(oracle_mod):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 4, 16)).astype(np.float32)
    ang = np.arange(12, dtype=np.float64) * 977 + 3
    y, ex = oracle_mod.rot_rows(x, "f32", 5.0e5, ang, want_exact=True)
    for r in range(12):
        want = _rot_complex(x.reshape(12, 16)[r].astype(np.float64), 5.0e5, ang[r])
        assert np.allclose(ex.reshape(12, 16)[r], want, atol=1e-11)
        assert np.array_equal(y.reshape(12, 16)[r], want.astype(np.float32))
    xb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    yb, exb = oracle_mod.rot_rows(xb, "bf16", 5.0e5, ang, want_exact=True)
    assert np.all(np.abs(oracle_mod.bf16_bits_to_f64(yb) - exb) <= 2.0 ** -8 * np.abs(exb) + 1e-40)
    assert np.array_equal(oracle_mod.rot_rows(xb, "bf16", 5.0e5, np.zeros(12)), xb)      # angle 0: identity


# ---------------------------------------------------------------- assemble

def _tiny_pool(rng, L, n_shots, hkv, d, lo=2, hi=7):
    lens = rng.integers(lo, hi, size=n_shots, endpoint=True)
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    k = rng.standard_normal((L, int(offsets[-1]), hkv, d)).astype(np.float32)
    v = rng.standard_normal((L, int(offsets[-1]), hkv, d)).astype(np.float32)
    return offsets, k, v


def test_assemble_bruteforce_f32(oracle_mod):
    rng = np.random.default_rng(11)
    L, hkv, d, base = 2, 2, 8, 100.0
    offsets, k, v = _tiny_pool(rng, L, 6, hkv, d)
    ids, order = [4, 1, 1, 5], [2, 0, 3, 1]
    pos0 = 9
    pl = oracle_mod.plan(offsets, ids, order, slot0=0, pos0=pos0)
    cap = pl["n"] + 3
    ko, vo, kx = oracle_mod.assemble(k, v, "f32", base, oracle_mod.KEYS_UNROTATED, pl, 0, cap, want_exact=True)
    slot = 0
    for j in range(4):
        s = ids[order[j]]
        for t in range(int(offsets[s + 1] - offsets[s])):
            src = int(offsets[s]) + t
            for l in range(L):
                assert np.array_equal(vo[l, slot], v[l, src])                   # bit copy
                want = _rot_complex(k[l, src].astype(np.float64), base, pos0 + slot)
                assert np.allclose(kx[l, slot], want, atol=1e-12)
                assert np.array_equal(ko[l, slot], want.astype(np.float32))     # rounded once
            slot += 1
    assert slot == pl["n"]
    assert not ko[:, slot:].any() and not vo[:, slot:].any()                    # nothing written past the end


def test_assemble_rotated_local_equals_unrotated(oracle_mod):
    """Keys cached at local positions 0..T-1 and shifted by Delta = offset give the same
    result as un-rotated keys rotated to the new position (Eq. rope_compensation)."""
    rng = np.random.default_rng(12)
    L, hkv, d, base = 1, 2, 16, 1.0e4
    offsets, k, v = _tiny_pool(rng, L, 5, hkv, d)
    k64 = k.astype(np.float64)
    k_local = np.empty_like(k64)
    for s in range(5):
        for t in range(int(offsets[s + 1] - offsets[s])):
            k_local[0, offsets[s] + t] = _rot_complex(k64[0, offsets[s] + t], base, t)
    ids, order = [3, 0, 4], [1, 2, 0]
    pl = oracle_mod.plan(offsets, ids, order, slot0=0, pos0=2)
    _, _, kx_u = oracle_mod.assemble(k, v, "f32", base, oracle_mod.KEYS_UNROTATED, pl, 0, pl["n"], want_exact=True)
    _, _, kx_r = oracle_mod.assemble(k_local.astype(np.float32), v, "f32", base, oracle_mod.KEYS_ROTATED_LOCAL,
                                     pl, 0, pl["n"], want_exact=True)
    assert np.allclose(kx_u, kx_r, atol=2e-6)       # k_local was rounded to fp32 once


def test_assemble_bf16_storage_and_append(oracle_mod):
    rng = np.random.default_rng(13)
    L, hkv, d, base = 1, 1, 8, 1.0e4
    offsets, k, v = _tiny_pool(rng, L, 4, hkv, d)
    kb = torch.from_numpy(k).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    vb = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    pl1 = oracle_mod.plan(offsets, [2, 0], None, slot0=0, pos0=0)
    pl2 = oracle_mod.plan(offsets, [3], None, slot0=pl1["n"], pos0=0)
    cap = pl1["n"] + pl2["n"]
    ko, vo, _ = oracle_mod.assemble(kb, vb, "bf16", base, 0, pl1, 0, cap)
    ko, vo, _ = oracle_mod.assemble(kb, vb, "bf16", base, 0, pl2, pl1["n"], cap, k_out=ko, v_out=vo)
    # one-shot assembly of all three gives the same cache (append keeps positions contiguous)
    pl = oracle_mod.plan(offsets, [2, 0, 3], None)
    ko2, vo2, kx = oracle_mod.assemble(kb, vb, "bf16", base, 0, pl, 0, cap, want_exact=True)
    assert np.array_equal(ko, ko2) and np.array_equal(vo, vo2)
    # stored keys are the exact keys rounded to bf16: within half a spacing (<= 2^-8 relative)
    got = oracle_mod.bf16_bits_to_f64(ko2)
    assert np.all(np.abs(got - kx) <= 2.0 ** -8 * np.abs(kx) + 1e-40)
    with pytest.raises(ValueError):
        oracle_mod.assemble(kb, vb, "bf16", base, 0, pl, 0, cap - 1)


# ---------------------------------------------------------------- attention

def _naive_attention(kc, vc, n_ctx, q, ks, vs, base, q_pos0):
    """Brute force in numpy matrix form with complex-number RoPE (independent of the C loops)."""
    t_q, h_q, d = q.shape
    h_kv = ks.shape[1]
    g = h_q // h_kv
    out = np.zeros((t_q, h_q, d))
    qr = np.stack([_rot_complex(q[j].astype(np.float64), base, q_pos0 + j) for j in range(t_q)])
    kr = np.stack([_rot_complex(ks[j].astype(np.float64), base, q_pos0 + j) for j in range(t_q)])
    for h in range(h_q):
        hk = h // g
        keys = np.concatenate([kc[:n_ctx, hk].astype(np.float64), kr[:, hk]], axis=0)
        vals = np.concatenate([vc[:n_ctx, hk].astype(np.float64), vs[:, hk].astype(np.float64)], axis=0)
        s = qr[:, h] @ keys.T / math.sqrt(d)
        mask = np.ones_like(s, dtype=bool)
        for j in range(t_q):
            mask[j, n_ctx + j + 1:] = False
        s = np.where(mask, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h] = p @ vals
    return out


def _rand_attn_inputs(rng, n_ctx, t_q, h_q, h_kv, d):
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return f(n_ctx, h_kv, d), f(n_ctx, h_kv, d), f(t_q, h_q, d), f(t_q, h_kv, d), f(t_q, h_kv, d)


@pytest.mark.parametrize("n_ctx,t_q,h_q,h_kv,d", [(13, 5, 4, 2, 8), (0, 4, 2, 2, 4), (40, 1, 7, 1, 16), (9, 6, 6, 3, 64)])
def test_attention_bruteforce(oracle_mod, n_ctx, t_q, h_q, h_kv, d):
    rng = np.random.default_rng(n_ctx * 31 + t_q)
    kc, vc, q, ks, vs = _rand_attn_inputs(rng, n_ctx, t_q, h_q, h_kv, d)
    got = oracle_mod.query_attn(kc, vc, "f32", n_ctx, q, ks, vs, 1.0e4, q_pos0=n_ctx + 3)
    want = _naive_attention(kc, vc, n_ctx, q, ks, vs, 1.0e4, n_ctx + 3)
    assert np.allclose(got, want, atol=1e-12)
    pairs = np.array([[t_q - 1, h_q - 1], [0, 0], [t_q // 2, 1]], np.int32)
    sub = oracle_mod.query_attn(kc, vc, "f32", n_ctx, q, ks, vs, 1.0e4, n_ctx + 3, pairs=pairs)
    for i, (j, h) in enumerate(pairs):
        assert np.array_equal(sub[i], got[j, h])


def test_attention_reduces_to_library_sdpa(oracle_mod):
    """One query token at position 0 (rotation angle 0), one head: textbook softmax(q K^T / sqrt d) V."""
    rng = np.random.default_rng(21)
    n_ctx, d = 50, 32
    kc, vc, q, ks, vs = _rand_attn_inputs(rng, n_ctx, 1, 1, 1, d)
    got = oracle_mod.query_attn(kc, vc, "f32", n_ctx, q, ks, vs, 5.0e5, q_pos0=0)
    K = torch.from_numpy(np.concatenate([kc[:, 0], ks[:, 0]])).double()[None, None]
    V = torch.from_numpy(np.concatenate([vc[:, 0], vs[:, 0]])).double()[None, None]
    Q = torch.from_numpy(q[:, 0]).double()[None, None]
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V)[0, 0].numpy()
    assert np.allclose(got[:, 0], want, atol=1e-12)


def test_attention_library_sdpa_causal_block(oracle_mod):
    """No context, several tokens from position 0: plain causal self-attention of a rotated sequence.
    The library routine gets keys/queries rotated by the complex-number brute force."""
    rng = np.random.default_rng(22)
    t_q, h, d, base = 7, 2, 16, 1.0e4
    kc, vc, q, ks, vs = _rand_attn_inputs(rng, 0, t_q, h, h, d)
    got = oracle_mod.query_attn(kc, vc, "f32", 0, q, ks, vs, base, q_pos0=0)
    qr = np.stack([_rot_complex(q[j].astype(np.float64), base, j) for j in range(t_q)])
    kr = np.stack([_rot_complex(ks[j].astype(np.float64), base, j) for j in range(t_q)])
    Q = torch.from_numpy(qr).permute(1, 0, 2)[None]
    K = torch.from_numpy(kr).permute(1, 0, 2)[None]
    V = torch.from_numpy(vs.astype(np.float64)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, atol=1e-12)


def test_attention_zero_keys_gives_mean_of_visible_values(oracle_mod):
    rng = np.random.default_rng(23)
    n_ctx, t_q, h_q, h_kv, d = 11, 4, 4, 2, 8
    kc, vc, q, ks, vs = _rand_attn_inputs(rng, n_ctx, t_q, h_q, h_kv, d)
    kc[:] = 0; ks[:] = 0
    got = oracle_mod.query_attn(kc, vc, "f32", n_ctx, q, ks, vs, 1.0e4, q_pos0=n_ctx)
    for j in range(t_q):
        for h in range(h_q):
            hk = h // 2
            want = (vc[:, hk].astype(np.float64).sum(0) + vs[: j + 1, hk].astype(np.float64).sum(0)) / (n_ctx + j + 1)
            assert np.allclose(got[j, h], want, atol=1e-13)


def test_attention_needle_and_group_symmetry(oracle_mod):
    rng = np.random.default_rng(24)
    n_ctx, t_q, h_q, h_kv, d = 64, 2, 4, 1, 16
    kc, vc, q, ks, vs = _rand_attn_inputs(rng, n_ctx, t_q, h_q, h_kv, d)
    q[:, 1] = q[:, 0]; q[:, 2] = q[:, 0]; q[:, 3] = q[:, 0]
    # plant a key parallel to the rotated query of row 0: its score dwarfs the rest
    qr0 = _rot_complex(q[0, 0].astype(np.float64), 1.0e4, 100)
    kc[17, 0] = (50.0 * qr0 / np.linalg.norm(qr0)).astype(np.float32)
    got = oracle_mod.query_attn(kc, vc, "f32", n_ctx, q, ks, vs, 1.0e4, q_pos0=100)
    assert np.allclose(got[0, 0], vc[17, 0], atol=1e-6)
    for h in range(1, 4):
        assert np.array_equal(got[:, h], got[:, 0])     # same q in a group -> same output


def test_chain_relative_position_invariance(oracle_mod):
    """Shifting pos0 and q_pos0 by the same constant leaves the attention output unchanged."""
    rng = np.random.default_rng(25)
    L, hkv, d, base = 1, 2, 16, 1.0e4
    offsets, k, v = _tiny_pool(rng, L, 6, hkv, d)
    ids, order = [5, 2, 0], [2, 0, 1]
    q = rng.standard_normal((3, 4, d)).astype(np.float32)
    ks = rng.standard_normal((3, hkv, d)).astype(np.float32)
    vs = rng.standard_normal((3, hkv, d)).astype(np.float32)
    outs = []
    for shift in (0, 4321):
        pl = oracle_mod.plan(offsets, ids, order, slot0=0, pos0=shift)
        _, vo, kx = oracle_mod.assemble(k, v, "f32", base, 0, pl, 0, pl["n"], want_exact=True)
        # feed the un-rounded keys so that only the rotation is tested
        outs.append(_naive_attention(kx[0], vo[0], pl["n"], q, ks, vs, base, shift + pl["n"]))
        o = oracle_mod.query_attn(kx[0].astype(np.float32), vo[0], "f32", pl["n"], q, ks, vs, base, shift + pl["n"])
        assert np.allclose(o, outs[-1], atol=1e-5)
    assert np.allclose(outs[0], outs[1], atol=1e-9)


def test_attention_bf16_inputs_widen_exactly(oracle_mod):
    rng = np.random.default_rng(26)
    n_ctx, t_q, h_q, h_kv, d = 10, 3, 2, 1, 8
    arrs = _rand_attn_inputs(rng, n_ctx, t_q, h_q, h_kv, d)
    bf = [torch.from_numpy(a).to(torch.bfloat16) for a in arrs]
    bits = [b.view(torch.int16).numpy().view(np.uint16) for b in bf]
    back = [b.float().numpy() for b in bf]
    a = oracle_mod.query_attn(bits[0], bits[1], "bf16", n_ctx, bits[2], bits[3], bits[4], 5.0e5, 10)
    b = oracle_mod.query_attn(back[0], back[1], "f32", n_ctx, back[2], back[3], back[4], 5.0e5, 10)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- entropy

def test_entropy_closed_forms(oracle_mod):
    c = _constants()
    assert abs(oracle_mod.entropy(np.zeros((1, 1000), np.float32))[0] - c["ln1000"]) < 1e-12
    assert abs(oracle_mod.entropy(np.full((1, 128256), 3.25, np.float32))[0] - c["ln128256"]) < 1e-11
    z = np.zeros((2, 128256), np.float32)
    z[0, 77] = 1.0e4
    z[1, :] = -np.inf; z[1, 5] = 0.0
    h = oracle_mod.entropy(z)
    assert h[0] == 0.0 and h[1] == 0.0
    # n entries at level a, the rest at 0
    V, n, a = 5000, 37, 4.5
    z = np.zeros((1, V), np.float32); z[0, 100:100 + n] = a
    Z = n * math.exp(a) + (V - n)
    want = math.log(Z) - n * a * math.exp(a) / Z
    assert abs(oracle_mod.entropy(z)[0] - want) < 1e-12
    # two classes: binary entropy of sigmoid(z1 - z0)
    z = np.array([[0.3, -1.1]], np.float32)
    p = 1.0 / (1.0 + math.exp(float(z[0, 1]) - float(z[0, 0])))
    assert abs(oracle_mod.entropy(z)[0] - (-(p * math.log(p) + (1 - p) * math.log(1 - p)))) < 1e-14


def test_entropy_library_and_shift(oracle_mod):
    import scipy.special
    import scipy.stats
    rng = np.random.default_rng(31)
    z = (rng.standard_normal((6, 3001)) * 3).astype(np.float32)
    want = scipy.stats.entropy(scipy.special.softmax(z.astype(np.float64), axis=1), axis=1)
    got = oracle_mod.entropy(z)
    assert np.allclose(got, want, atol=1e-12)
    # logits that are exact in fp32 after the shift: invariance is exact up to fp64 rounding
    zi = rng.integers(-8, 8, size=(3, 500)).astype(np.float32)
    assert np.allclose(oracle_mod.entropy(zi), oracle_mod.entropy(zi + 64.0), atol=1e-12)
    # strided rows
    big = np.zeros((4, 4000), np.float32); big[:, :3001] = z[:4]
    assert np.allclose(oracle_mod.entropy(big[:, :3001]), got[:4], atol=0)


def test_entropy_invalid_rows_are_nan(oracle_mod):
    z = np.zeros((3, 16), np.float32)
    z[0, 3] = np.nan
    z[1, 3] = np.inf
    z[2, :] = -np.inf
    assert np.all(np.isnan(oracle_mod.entropy(z)))


def test_entropy_gaussian_logits_statistic(oracle_mod):
    """iid N(0, s2) logits: E[H] ~ ln V - s2/2 (variance 2 -> ln V - 1), far from the std-2 reading."""
    from paper_2605_03644_amd import workloads as wl
    w = wl.WORKLOADS["llama8b_1layer"]
    z = wl.make_logits(w, "cpu", n_rows=8).numpy()
    h = oracle_mod.entropy(z)
    assert abs(h.mean() - (math.log(w.vocab) - 1.0)) < 0.05


# ---- Eq. (entropy) over the answer tokens, and the stopping rule -------------------------------

def _case_study():
    rounds, tau, picked = {}, None, None
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "case_study_probe_rounds.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a = line.split()
        if a[0] == "tau":
            tau, picked = float(a[1]), int(a[2])
        else:
            rounds.setdefault(int(a[0]), []).append((int(a[1]), float(a[2])))
    return rounds, tau, picked


def test_pick_shots_reproduces_the_case_study(oracle_mod):
    """The paper's worked example: no first-round probe passes, the second round selects 28 of {28, 32}."""
    rounds, tau, picked = _case_study()
    k1, h1 = zip(*rounds[1])
    k2, h2 = zip(*rounds[2])
    assert oracle_mod.pick_shots(h1, k1, tau) == -1
    assert oracle_mod.pick_shots(h2, k2, tau) == picked == 28
    # the order in which the candidates are listed does not matter, NaN never passes, equality passes
    assert oracle_mod.pick_shots(h2[::-1], k2[::-1], tau) == 28
    assert oracle_mod.pick_shots([float("nan"), 0.7], [4, 8], tau) == -1
    assert oracle_mod.pick_shots([0.65, 0.1], [8, 16], 0.65) == 8


def test_case_study_values_need_the_full_vocabulary_reading(oracle_mod):
    """Two printed entropies exceed ln 2, the ceiling of a renormalised two-class entropy in nats; the sum of
    two terms of a larger distribution can reach 2/e.  Both ceilings are attained by the oracle."""
    rounds, _, _ = _case_study()
    hs = [h for r in rounds.values() for _, h in r]
    assert max(hs) > math.log(2.0) and max(hs) < 2.0 / math.e
    V = 1000
    # full-vocabulary reading: p_yes = p_no = 1/e, the rest spread evenly
    z = np.full((1, V), math.log((1.0 - 2.0 / math.e) / (V - 2)), np.float32)
    z[0, 3] = z[0, 7] = -1.0
    h = oracle_mod.entropy_subset(z, [3, 7], oracle_mod.ENTROPY_FULL_P)[0]
    assert abs(h - 2.0 / math.e) < 1e-6
    # any other split of the same mass gives less
    z2 = z.copy(); z2[0, 3] = math.log(0.5); z2[0, 7] = math.log(2.0 / math.e - 0.5)
    assert oracle_mod.entropy_subset(z2, [3, 7], oracle_mod.ENTROPY_FULL_P)[0] < h
    # renormalised reading: equal logits give ln 2 whatever the rest of the vocabulary holds
    assert abs(oracle_mod.entropy_subset(z, [3, 7], oracle_mod.ENTROPY_RENORMALISED)[0] - math.log(2.0)) < 1e-12


def test_entropy_subset_closed_forms(oracle_mod):
    V = 512
    rng = np.random.default_rng(11)
    # uniform logits: p_c = 1/V, so the full-vocabulary reading gives |C| ln(V) / V
    z = np.full((2, V), 0.37, np.float32)
    ids = [5, 100, 511]
    h = oracle_mod.entropy_subset(z, ids, oracle_mod.ENTROPY_FULL_P)
    assert np.allclose(h, 3 * math.log(V) / V, rtol=1e-12)
    assert np.allclose(oracle_mod.entropy_subset(z, ids, oracle_mod.ENTROPY_RENORMALISED), math.log(3), rtol=1e-12)
    # C = whole vocabulary: both readings are the full entropy
    z = (rng.standard_normal((3, 64)) * 2).astype(np.float32)
    full = oracle_mod.entropy(z)
    for mode in (oracle_mod.ENTROPY_FULL_P, oracle_mod.ENTROPY_RENORMALISED):
        assert np.allclose(oracle_mod.entropy_subset(z, np.arange(64), mode), full, rtol=1e-12)
    # all mass on C (the other logits are -inf): both readings equal the binary entropy of sigmoid(z_a - z_b)
    z = np.full((1, V), -np.inf, np.float32)
    z[0, 10], z[0, 20] = 1.25, -0.5
    p = 1.0 / (1.0 + math.exp(-1.75))
    hb = -(p * math.log(p) + (1 - p) * math.log(1 - p))
    for mode in (oracle_mod.ENTROPY_FULL_P, oracle_mod.ENTROPY_RENORMALISED):
        assert abs(oracle_mod.entropy_subset(z, [10, 20], mode)[0] - hb) < 1e-12


def test_entropy_subset_against_library_softmax(oracle_mod):
    """Random rows against scipy's log-softmax, written out term by term."""
    from scipy.special import log_softmax
    rng = np.random.default_rng(12)
    z = (rng.standard_normal((5, 3000)) * math.sqrt(2.0)).astype(np.float32)
    z[2, 17] = -np.inf
    ids = np.array([17, 2999, 0, 1234], np.int32)
    lp = log_softmax(z.astype(np.float64), axis=1)[:, ids]
    with np.errstate(invalid="ignore"):
        ref_full = -np.where(np.isfinite(lp), np.exp(lp) * lp, 0.0).sum(1)
    lq = log_softmax(z.astype(np.float64)[:, ids], axis=1)
    with np.errstate(invalid="ignore"):
        ref_ren = -np.where(np.isfinite(lq), np.exp(lq) * lq, 0.0).sum(1)
    assert np.allclose(oracle_mod.entropy_subset(z, ids, oracle_mod.ENTROPY_FULL_P), ref_full, rtol=1e-11, atol=1e-14)
    assert np.allclose(oracle_mod.entropy_subset(z, ids, oracle_mod.ENTROPY_RENORMALISED), ref_ren, rtol=1e-11, atol=1e-14)


def test_entropy_subset_degenerate_rows(oracle_mod):
    z = np.zeros((4, 16), np.float32)
    z[0, 3] = np.nan
    z[1, 4] = np.inf
    z[2, :] = -np.inf
    z[3, [1, 2]] = -np.inf
    for mode in (oracle_mod.ENTROPY_FULL_P, oracle_mod.ENTROPY_RENORMALISED):
        h = oracle_mod.entropy_subset(z, [1, 2], mode)
        assert np.isnan(h[0]) and np.isnan(h[1]) and np.isnan(h[2])
    assert oracle_mod.entropy_subset(z, [1, 2], oracle_mod.ENTROPY_FULL_P)[3] == 0.0       # both terms vanish
    assert np.isnan(oracle_mod.entropy_subset(z, [1, 2], oracle_mod.ENTROPY_RENORMALISED)[3])  # nothing to renormalise


# ---- Eq. (attention_score): relevance ranking over the pool ---------------------------------------

def _rank_case(seed, n_shots=7, h_q=4, h_kv=2, d=16, t_q=5, lo=3, hi=9):
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi, n_shots, endpoint=True)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    k = rng.standard_normal((int(off[-1]), h_kv, d)).astype(np.float32)
    q = rng.standard_normal((t_q, h_q, d)).astype(np.float32)
    return off, k, q


def _rank_numpy(off, k, q, base, rotate_keys, q_pos0, store=None):
    """Eq. (attention_score) with the softmax over the whole pool, written with numpy and the closed-form
    rotation matrix, not with the oracle's rot().  `store` rounds a rotated key to the cache's storage type
    (default: fp32)."""
    if store is None:
        store = lambda y: y.astype(np.float32).astype(np.float64)
    T, h_kv, d = k.shape
    t_q, h_q, _ = q.shape
    half = d // 2
    theta = base ** (-2.0 * np.arange(half) / d)

    def rot(x, a):  # x [..., d]
        ang = a * theta
        c, s = np.cos(ang), np.sin(ang)
        x1, x2 = x[..., :half], x[..., half:]
        return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], -1)

    kk = k.astype(np.float64)
    if rotate_keys:
        kk = kk.copy()
        for i in range(len(off) - 1):
            for t in range(off[i + 1] - off[i]):
                # the cache holds the rotated key in the storage type (fp32 here)
                kk[off[i] + t] = store(rot(k[off[i] + t].astype(np.float64), float(t)))
    g = h_q // h_kv
    s = np.zeros(len(off) - 1)
    for j in range(t_q):
        for h in range(h_q):
            qr = rot(q[j, h].astype(np.float64), float(q_pos0 + j))
            sc = kk[:, h // g, :] @ qr / math.sqrt(d)
            p = np.exp(sc - sc.max()); p /= p.sum()
            s += np.add.reduceat(p, off[:-1])
    return s / (t_q * h_q * np.diff(off))


@pytest.mark.parametrize("key_state", [0, 1])
def test_rank_scores_match_numpy_brute_force(oracle_mod, key_state):
    off, k, q = _rank_case(21)
    got = oracle_mod.rank_scores(k, "f32", off, q, 1.0e4, key_state, q_pos0=3)
    want = _rank_numpy(off, k, q, 1.0e4, rotate_keys=(key_state == 0), q_pos0=3)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-15)
    # the un-rotated pool ranked with local positions differs from treating the same numbers as already rotated
    other = oracle_mod.rank_scores(k, "f32", off, q, 1.0e4, 1 - key_state, q_pos0=3)
    assert np.abs(other - got).max() > 1e-4 * got.max()


def test_rank_scores_invariants(oracle_mod):
    off, k, q = _rank_case(22, n_shots=9)
    s = oracle_mod.rank_scores(k, "f32", off, q, 1.0e4, 0)
    lens = np.diff(off)
    # all attention mass lands on some shot: sum_i T_i s_i = 1
    assert abs(float((s * lens).sum()) - 1.0) < 1e-12
    assert (s > 0).all()
    # zero queries -> uniform attention -> every shot scores 1 / T_pool whatever its length
    s0 = oracle_mod.rank_scores(k, "f32", off, np.zeros_like(q), 1.0e4, 0)
    assert np.allclose(s0, 1.0 / off[-1], rtol=1e-12)
    # the literal reading (softmax inside one shot) could not rank: it gives 1/T_i for any content
    # (stated here as the reason for the reading; computed directly)
    i = 3
    sc = np.random.default_rng(0).standard_normal((5, lens[i]))
    p = np.exp(sc) / np.exp(sc).sum(1, keepdims=True)
    assert abs(p.mean() - 1.0 / lens[i]) < 1e-15


def test_rank_scores_find_the_planted_shot(oracle_mod):
    """A shot whose keys align with the query direction at the matching relative rotation must rank first."""
    off, k, q = _rank_case(23, n_shots=8, d=16, t_q=4)
    k = k * 0.1
    # rotated-local pool: keys are used as stored, so plant the (rotated) query direction itself
    half = 8
    theta = 1.0e4 ** (-2.0 * np.arange(half) / 16)
    def rot(x, a):
        c, s = np.cos(a * theta), np.sin(a * theta)
        return np.concatenate([x[:half] * c - x[half:] * s, x[half:] * c + x[:half] * s])
    target = 5
    for hk in range(k.shape[1]):
        qbar = np.mean([rot(q[j, h].astype(np.float64), j) for j in range(q.shape[0]) for h in (2 * hk, 2 * hk + 1)], 0)
        k[off[target]:off[target + 1], hk, :] = (3.0 * qbar).astype(np.float32)
    s = oracle_mod.rank_scores(k, "f32", off, q, 1.0e4, 1)
    assert int(np.argmax(s)) == target and s[target] > 2 * np.delete(s, target).max()


def test_rank_scores_bf16_storage_rounds_rotated_keys(oracle_mod):
    """bf16 pool, un-rotated: the rotated key is rounded to bf16 before the dot product (a cache holds bf16)."""
    off, k, q = _rank_case(24)
    kb = (k.view(np.uint32) >> 16).astype(np.uint16)          # truncate to bf16 bit patterns
    qb = (q.view(np.uint32) >> 16).astype(np.uint16)
    got = oracle_mod.rank_scores(kb, "bf16", off, qb, 1.0e4, 0)
    kf = (kb.astype(np.uint32) << 16).view(np.float32)
    qf = (qb.astype(np.uint32) << 16).view(np.float32)
    # with the rotated keys rounded to bf16 by the library's own conversion the scores match; with the
    # rotated keys kept in fp32 they differ by the size of a bf16 rounding, not by nothing
    to_bf16 = lambda y: torch.from_numpy(y).to(torch.bfloat16).to(torch.float64).numpy()
    want = _rank_numpy(off, kf, qf, 1.0e4, rotate_keys=True, q_pos0=0, store=to_bf16)
    assert np.allclose(got, want, rtol=1e-9, atol=0)
    exact = _rank_numpy(off, kf, qf, 1.0e4, rotate_keys=True, q_pos0=0)   # rounds rotated keys to fp32 only
    assert 1e-6 * exact.max() < np.abs(got - exact).max() < 2e-2 * exact.max()
    assert abs(float((got * np.diff(off)).sum()) - 1.0) < 1e-12
