"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Bars: indexing bit-exact; fp32 re-encode 1e-5 relative per rotation pair;
bf16 keys >= 99 % identical to the oracle's rounding and each within
half a bf16 spacing + 1e-5 relative of the exact key; attention 2e-2 max-abs and
1e-2 relative Frobenius (bf16), 1e-4 / 1e-5 (fp32 path); entropy 1e-4."""
import ctypes
import math

import numpy as np
import pytest
import torch

from paper_2605_03644_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_03644_amd import binding
    binding.load_library()          # raises if the HIP library is not built: no fallback
    return binding


def _pool_numpy(k, v):
    return H.to_storage(k), H.to_storage(v)


def _run_assemble_case(ad, oracle_mod, w, key_state, pos0, splits, n_layers=None, ids=None, order=None):
    """Assemble on the GPU (possibly as several appends) and with the oracle; compare everything."""
    dev = "cuda"
    L = w.n_layers if n_layers is None else n_layers
    k_pool, v_pool, off = wl.make_pool(w, dev, n_layers=L)
    if ids is None:
        ids, order = wl.selection(w)
    ctx = ad.Context.for_workload(w, key_state=key_state, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    seq = [int(ids[o]) for o in order] if order is not None else [int(i) for i in ids]
    total = int(sum(off[s + 1] - off[s] for s in seq))
    cap = total + 5
    cache = ad.Cache(ctx, cap)
    canary_k = cache.k[:, total:].clone()
    # appends: the first uses (ids, order) sliced through `order`; later ones pass explicit id lists
    bounds = [0] + [int(len(seq) * f) for f in splits] + [len(seq)]
    for a, b in zip(bounds[:-1], bounds[1:]):
        if a == 0 and b == len(seq) and order is not None:
            ctx.assemble(cache, ids, order, pos0=pos0)
        else:
            ctx.assemble(cache, seq[a:b], None, pos0=pos0)
    torch.cuda.synchronize()
    assert cache.len == total

    kp, vp = _pool_numpy(k_pool, v_pool)
    pl = oracle_mod.plan(off, ids, order, slot0=0, pos0=pos0)
    assert pl["n"] == total
    ko, vo, kx = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, key_state, pl, 0, cap, want_exact=True)

    # indexing: bit exact
    assert np.array_equal(cache.slot_shot[:total].cpu().numpy(), pl["slot_shot"])
    assert np.array_equal(cache.slot_tok[:total].cpu().numpy(), pl["slot_tok"])
    assert np.array_equal(cache.slot_pos[:total].cpu().numpy(), pl["slot_pos"])
    assert (cache.slot_shot[total:] == -1).all() and (cache.slot_pos[total:] == -1).all()
    # V: bit copy; nothing written past the end
    kg, vg = H.to_storage(cache.k), H.to_storage(cache.v)
    assert np.array_equal(vg[:, :total], vo[:, :total])
    assert not vg[:, total:].any()
    assert torch.equal(cache.k[:, total:], canary_k)
    # K
    if w.dtype == "f32":
        src = kp[:, pl["slot_src"]]
        worst = H.check_reencode_f32(kg[:, :total], kx, src, rel=1e-5)
        return dict(worst_rel=worst, total=total)
    frac = H.check_reencode_bf16(kg[:, :total], ko[:, :total], kx, kp[:, pl["slot_src"]])
    ctx.close()
    return dict(frac_equal=frac, total=total)


@pytest.mark.parametrize("key_state", [0, 1])
@pytest.mark.parametrize("pos0,splits", [(0, []), (11, [0.4]), (100000, [0.25, 0.5]), (1048576 - 300, [])])
def test_assemble_tiny_fp32(ad, oracle_mod, key_state, pos0, splits):
    w = wl.WORKLOADS["tiny_fp32"]
    _run_assemble_case(ad, oracle_mod, w, key_state, pos0, splits)


def test_assemble_tiny_fp32_multilayer_duplicates(ad, oracle_mod):
    w = wl.WORKLOADS["tiny_fp32"]
    ids = np.array([3, 3, 15, 0, 7, 3], np.int32)
    order = np.array([5, 0, 2, 1, 4, 3], np.int32)
    _run_assemble_case(ad, oracle_mod, w, 0, 7, [], n_layers=3, ids=ids, order=order)


@pytest.mark.parametrize("key_state", [0, 1])
def test_assemble_llama8b_bf16_full(ad, oracle_mod, key_state):
    """Config 2 at full size (256 of 2000 shots, ~26k tokens), the launch shape the benchmark times."""
    w = wl.WORKLOADS["llama8b_1layer"]
    r = _run_assemble_case(ad, oracle_mod, w, key_state, 0, [])
    assert r["total"] > 20000


def test_assemble_qwen_shape_bf16_two_layers(ad, oracle_mod):
    """4 KV heads (half a wavefront per token row), theta 1e6, two layers, three appends."""
    w = wl.WORKLOADS["qwen7b_decode"]
    _run_assemble_case(ad, oracle_mod, w, 0, 3, [0.3, 0.9], n_layers=2)


@pytest.mark.parametrize("key_state", [0, 1])
def test_assemble_many_layers_host_cut_pieces(ad, oracle_mod, key_state):
    """From 8 layers on the host cuts every shot into one-workgroup pieces (8 tokens for this row size) and joins
    what is left over to the last piece: shot lengths 1..70 cover shots shorter than a piece, shots with no
    remainder and every remainder 1..7; three appends."""
    import dataclasses
    w = dataclasses.replace(wl.WORKLOADS["llama8b_1layer"], name="llama8b_pieces", n_layers=8, n_shots=90, len_lo=1,
                            len_hi=70, m_select=60)
    lens = wl.shot_lengths(w)
    assert lens.min() == 1 and lens.max() == 70 and len({int(x) % 8 for x in lens}) == 8
    r = _run_assemble_case(ad, oracle_mod, w, key_state, 5, [0.2, 0.7])
    assert r["total"] > 1000


def test_assemble_errors_write_nothing(ad):
    w = wl.WORKLOADS["tiny_fp32"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda")
    ctx = ad.Context.for_workload(w, max_position=4096)
    cache = ad.Cache(ctx, 64)
    with pytest.raises(ad.AdapshotError) as e:
        ctx.assemble(cache, [0, 1])
    assert e.value.status == ad.ESTATE
    ctx.pool_register(k_pool, v_pool, off)
    for ids, order, pos0, status in [([0, 16], None, 0, ad.ESHOT), ([-1], None, 0, ad.ESHOT),
                                     ([0, 1], [0, 2], 0, ad.ESHOT), ([0, 1, 2, 3], None, 0, ad.ECAPACITY),
                                     ([0], None, 4090, ad.ECAPACITY), ([0], None, -1, ad.EINVAL)]:
        with pytest.raises(ad.AdapshotError) as e:
            ctx.assemble(cache, ids, order, pos0=pos0)
        assert e.value.status == status, (ids, e.value)
        assert ctx.last_error()
    torch.cuda.synchronize()
    assert cache.len == 0 and not cache.k.any() and not cache.v.any() and (cache.slot_shot == -1).all()
    ctx.assemble(cache, [], None)          # m = 0 is a no-op
    assert cache.len == 0
    ctx.assemble(cache, [2])
    assert cache.len == int(off[3] - off[2]) and ctx.last_error() == ""
    ctx.close()


# ------------------------------------------------------------------------------ entropy

def _entropy_case(ad, oracle_mod, z: torch.Tensor, tol=1e-4):
    ctx = ad.Context(1, 4, 2, 64, 1.0e4, ad.F32)
    got = ctx.probe_entropy(z).cpu().numpy().astype(np.float64)
    want = oracle_mod.entropy(z.cpu().numpy())
    ctx.close()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    if (~nan).any():
        err = np.abs(got[~nan] - want[~nan]).max()
        assert err <= tol, f"entropy error {err:.3e}"
    return got, want


def test_entropy_workloads(ad, oracle_mod):
    for name in ("tiny_fp32", "llama8b_1layer"):
        w = wl.WORKLOADS[name]
        z = wl.make_logits(w, "cuda")
        got, want = _entropy_case(ad, oracle_mod, z)
        assert abs(want.mean() - (math.log(w.vocab) - 1.0)) < 0.2


@pytest.mark.parametrize("rows,vocab", [(1, 128256), (48, 128256), (3, 1), (5, 7), (2, 1023), (2, 1025), (7, 4099),
                                        (2, 152064), (300, 333)])
def test_entropy_shapes(ad, oracle_mod, rows, vocab):
    g = torch.Generator(device="cuda"); g.manual_seed(rows * 1000003 + vocab)
    z = torch.randn(rows, vocab, device="cuda", generator=g) * 3.0
    _entropy_case(ad, oracle_mod, z)


@pytest.mark.parametrize("rows,vocab", [(256, 128256), (300, 16387), (512, 16389), (257, 16384), (700, 40000)])
def test_entropy_many_rows_one_workgroup_per_row(ad, oracle_mod, rows, vocab):
    """From as many rows as the GPU has compute units on, a row is reduced by one workgroup in one launch: full
    steps, ragged tails, unaligned rows, degenerate rows and the answer-token epilogue on that path."""
    g = torch.Generator(device="cuda"); g.manual_seed(rows * 7919 + vocab)
    z = torch.randn(rows, vocab, device="cuda", generator=g) * 3.0
    z[1] = -float("inf"); z[1, vocab - 1] = 2.0       # single finite logit: H = 0
    z[2, vocab // 2] = float("nan")
    z[3, 0] = float("inf")
    z[4] = -float("inf")
    z[5, : vocab // 3] = -float("inf")
    got, want = _entropy_case(ad, oracle_mod, z)
    assert got[1] == 0.0
    _entropy_case(ad, oracle_mod, z[:, 1:vocab - 2])   # base pointer off by 4 bytes, stride > vocab
    ctx = ad.Context(1, 4, 2, 64, 1.0e4, ad.F32)
    ids = [0, vocab - 1, vocab // 2, 7]
    zz = z[6:]                                         # rows without planted infinities
    for mode in (0, 1):
        got = ctx.probe_entropy_tokens(zz, ids, mode).cpu().numpy().astype(np.float64)
        want = oracle_mod.entropy_subset(zz.cpu().numpy(), ids, mode)
        assert np.all(np.isfinite(want)) and float(np.abs(got - want).max()) < 1e-4
    ctx.close()


def test_entropy_strided_and_unaligned_rows(ad, oracle_mod):
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    big = torch.randn(6, 5003, device="cuda", generator=g)
    _entropy_case(ad, oracle_mod, big[:, :5001])           # row stride 5003: rows not 16-byte aligned
    _entropy_case(ad, oracle_mod, big[:, 1:4097])          # base pointer off by 4 bytes
    big2 = torch.randn(4, 8192, device="cuda", generator=g)
    _entropy_case(ad, oracle_mod, big2[:, :8000])          # aligned rows, stride > vocab


def test_entropy_closed_forms_and_degenerate_rows(ad, oracle_mod):
    V = 128256
    z = torch.zeros(8, V, device="cuda")
    z[1] = 3.25
    z[2, 77] = 1.0e4                      # one-hot: H = 0
    z[3] = -float("inf"); z[3, 5] = 0.0   # single finite logit: H = 0
    z[4, 100] = float("nan")
    z[5, V - 1] = float("inf")
    z[6] = -float("inf")
    z[7, :40000] = -float("inf")          # -inf entries contribute 0
    got, want = _entropy_case(ad, oracle_mod, z)
    assert abs(got[0] - math.log(V)) < 1e-4 and abs(got[1] - math.log(V)) < 1e-4
    assert got[2] == 0.0 and got[3] == 0.0
    assert abs(got[7] - math.log(V - 40000)) < 1e-4
    ctx = ad.Context(1, 4, 2, 64, 1.0e4, ad.F32)
    with pytest.raises(ad.AdapshotError):
        ctx.lib.adapshot_probe_entropy.restype  # keep linters quiet
        ctx._check(ctx.lib.adapshot_probe_entropy(ctx._h, z.data_ptr(), 10, 1, 100, z.data_ptr(), None))
    ctx.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_entropy_over_answer_tokens(ad, oracle_mod, mode):
    """Eq. (entropy) over the probe's answer tokens, both readings, at the bench's logit shape and on small,
    strided and degenerate rows, against the oracle."""
    ctx = ad.Context(1, 4, 2, 64, 1.0e4, ad.F32)
    w = wl.WORKLOADS["llama8b_1layer"]
    z = wl.make_logits(w, "cuda")
    z[:, 9891] += 9.0   # two likely answer tokens, as a probe prompt would make them
    z[:, 2822] += 8.5 + torch.linspace(-3, 3, z.shape[0], device="cuda")
    cases = [(z, [9891, 2822]), (z, [0, w.vocab - 1, 77, 9891]), (z[:5, :1001], [1000]),
             (z[3:40, 1:4098], list(range(16)))]
    for zz, ids in cases:
        got = ctx.probe_entropy_tokens(zz, ids, mode).cpu().numpy().astype(np.float64)
        want = oracle_mod.entropy_subset(zz.cpu().numpy(), ids, mode)
        assert np.all(np.isfinite(want)) and float(np.abs(got - want).max()) < 1e-4, (ids, np.abs(got - want).max())
    h2 = oracle_mod.entropy_subset(z.cpu().numpy(), [9891, 2822], mode)
    assert h2.max() > 0.3 and h2.min() < h2.max() - 0.05      # the rows do differ: not a constant
    # degenerate rows
    d = torch.zeros(6, 4096, device="cuda")
    d[0, 3] = float("nan"); d[1, 4] = float("inf"); d[2] = -float("inf")
    d[3, [1, 2]] = -float("inf")
    d[4, 1] = 50.0                  # all mass on one answer token: H = 0
    d[5] = -float("inf"); d[5, 1] = 0.3; d[5, 2] = -0.9   # all mass on C: binary entropy in both readings
    got = ctx.probe_entropy_tokens(d, [1, 2], mode).cpu().numpy().astype(np.float64)
    want = oracle_mod.entropy_subset(d.cpu().numpy(), [1, 2], mode)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.allclose(got[~np.isnan(got)], want[~np.isnan(want)], atol=1e-5)
    assert np.isnan(got[:3]).all() and got[4] < 1e-6
    # argument errors are reported before anything is launched
    out = torch.full((6,), 7.0, device="cuda")
    for bad in ([1, 1], [4096], [-1], [], list(range(17))):
        with pytest.raises(ad.AdapshotError):
            ctx.probe_entropy_tokens(d, bad, mode, out=out)
    with pytest.raises(ad.AdapshotError):
        ctx.probe_entropy_tokens(d, [1, 2], 5, out=out)
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0
    ctx.close()


def test_adaptive_rounds_end_to_end(ad, oracle_mod):
    """Two rounds of four parallel probes as in the case study: entropies of each round's logits on the GPU,
    the stopping rule on the host, against the oracle doing the same."""
    ctx = ad.Context(1, 4, 2, 64, 1.0e4, ad.F32)
    g = torch.Generator(device="cuda"); g.manual_seed(77)
    V, yes, no, tau = 32000, 9454, 2822, 0.65
    rounds = [[4, 8, 12, 16], [20, 24, 28, 32]]
    margins = [[0.2, -0.1, 0.05, 0.3], [0.1, 0.25, 1.4, 1.1]]   # confidence grows only late in the second round
    picked = -1
    for counts, mg in zip(rounds, margins):
        z = torch.randn(4, V, device="cuda", generator=g) * 1.4142
        z[:, yes] = 11.0 + torch.tensor(mg, device="cuda")
        z[:, no] = 11.0
        h = ctx.probe_entropy_tokens(z, [yes, no], ad.ENTROPY_FULL_P)
        h_ref = oracle_mod.entropy_subset(z.cpu().numpy(), [yes, no], oracle_mod.ENTROPY_FULL_P)
        assert float(np.abs(h.cpu().numpy() - h_ref).max()) < 1e-4
        assert np.abs(h_ref - tau).min() > 1e-3     # no candidate sits on the threshold
        picked = ctx.pick_shots(h.cpu().numpy(), counts, tau)
        assert picked == oracle_mod.pick_shots(h_ref, counts, tau)
        if picked >= 0:
            break
    assert picked == 28
    ctx.close()


# ------------------------------------------------------------------------------ attention

def _attention_case(ad, oracle_mod, w, n_shots_sel, t_q, pos0=0, q_pos0=None, n_ctx=None, max_abs=2e-2,
                    rel_fro=1e-2, mutate=None, pairs=None, seed_q=0):
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ids, order = wl.selection(w)
    ids, order = ids[:n_shots_sel], np.argsort(np.argsort(order[:n_shots_sel])).astype(np.int32)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    cache = ad.Cache(ctx, max(total, 1), with_index=False)
    ctx.assemble(cache, ids, order, pos0=pos0)
    n_ctx = total if n_ctx is None else n_ctx
    q_pos0 = pos0 + n_ctx if q_pos0 is None else q_pos0
    q, ks, vs = wl.make_query(w, "cuda", query=seed_q, t_q=t_q)
    if mutate is not None:
        mutate(cache, q, ks, vs, q_pos0)
    out = ctx.query_attn(cache, 0, n_ctx, q, ks, vs, q_pos0)
    torch.cuda.synchronize()
    # the oracle attends over the GPU-assembled cache (assemble parity is tested on its own)
    kc, vc = H.to_storage(cache.k[0]), H.to_storage(cache.v[0])
    ref = oracle_mod.query_attn(kc, vc, w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                w.rope_theta, q_pos0, pairs=pairs)
    got = out.float().cpu().numpy()
    if pairs is not None:
        got = np.stack([got[j, h] for j, h in pairs])
    res = H.check_attention(got, ref, max_abs=max_abs, rel_fro=rel_fro)
    ctx.close()
    return res, got, ref


def test_attention_tiny_fp32(ad, oracle_mod):
    w = wl.WORKLOADS["tiny_fp32"]
    _attention_case(ad, oracle_mod, w, 8, 16, max_abs=1e-4, rel_fro=1e-5)
    _attention_case(ad, oracle_mod, w, 8, 16, pos0=5000, max_abs=1e-4, rel_fro=1e-5)
    _attention_case(ad, oracle_mod, w, 3, 1, max_abs=1e-4, rel_fro=1e-5)


def test_attention_tiny_fp32_no_context_and_prefix(ad, oracle_mod):
    w = wl.WORKLOADS["tiny_fp32"]
    _attention_case(ad, oracle_mod, w, 8, 16, n_ctx=0, q_pos0=0, max_abs=1e-4, rel_fro=1e-5)
    _attention_case(ad, oracle_mod, w, 8, 5, n_ctx=77, max_abs=1e-4, rel_fro=1e-5)   # a prefix of the cache


def test_attention_needle_tiny(ad, oracle_mod):
    """One context key made parallel to a rotated query and scaled x50: the output is that key's value row."""
    w = wl.WORKLOADS["tiny_fp32"]

    def mutate(cache, q, ks, vs, q_pos0):
        qr = oracle_mod.rot(q[0, 0].double().cpu().numpy(), w.rope_theta, q_pos0)   # row 0 sits at q_pos0
        cache.k[0, 100, 0, :] = torch.from_numpy(50.0 * qr / np.linalg.norm(qr)).to(cache.k.dtype).cuda()

    (_, _), got, ref = _attention_case(ad, oracle_mod, w, 8, 4, max_abs=1e-4, rel_fro=1e-5, mutate=mutate)
    assert np.abs(ref).max() > 0.5          # outputs are O(1) somewhere, so the max-abs bar has teeth


# ------------------------------------------------------------------------------ bf16 MFMA attention

@pytest.mark.parametrize("name,n_sel,t_q", [("llama8b_1layer", 3, 16), ("llama8b_1layer", 9, 128), ("llama8b_1layer", 5, 37),
                                            ("llama8b_1layer", 1, 1), ("qwen7b_decode", 7, 1), ("qwen7b_decode", 4, 19),
                                            ("llama70b_128k", 6, 40)])
def test_attention_bf16_small(ad, oracle_mod, name, n_sel, t_q):
    """A few shots (several 64-key tiles plus a ragged tail), ragged row tiles, g = 4, 7 and 8."""
    w = wl.WORKLOADS[name]
    _attention_case(ad, oracle_mod, w, n_sel, t_q)


def test_attention_bf16_no_context_prefix_and_shift(ad, oracle_mod):
    w = wl.WORKLOADS["llama8b_1layer"]
    _attention_case(ad, oracle_mod, w, 4, 70, n_ctx=0, q_pos0=0)           # causal self part only
    _attention_case(ad, oracle_mod, w, 6, 33, n_ctx=129)                    # prefix of the cache
    _attention_case(ad, oracle_mod, w, 6, 33, pos0=90000)                   # far positions


def test_attention_bf16_needle(ad, oracle_mod):
    w = wl.WORKLOADS["llama8b_1layer"]

    def mutate(cache, q, ks, vs, q_pos0):
        for j, slot in ((0, 200), (5, 3)):
            qr = oracle_mod.rot(q[j, 2].double().cpu().numpy(), w.rope_theta, q_pos0 + j)
            cache.k[0, slot, 0, :] = torch.from_numpy(50.0 * qr / np.linalg.norm(qr)).to(cache.k.dtype).cuda()

    (_, _), got, ref = _attention_case(ad, oracle_mod, w, 8, 8, mutate=mutate)
    assert np.abs(ref).max() > 0.5


def test_attention_bf16_zero_keys_mean_of_values(ad, oracle_mod):
    """K = 0 everywhere: every visible key gets the same weight, so O is the mean of the visible V rows
    (closed form, independent of the oracle) -- checks the causal counts n_ctx + j + 1."""
    w = wl.WORKLOADS["llama8b_1layer"]

    def mutate(cache, q, ks, vs, q_pos0):
        cache.k.zero_(); ks.zero_()
        mutate.v = cache.v[0, :cache.len].double().cpu().numpy(); mutate.vs = vs.double().cpu().numpy()

    (_, _), got, ref = _attention_case(ad, oracle_mod, w, 5, 21, mutate=mutate)
    n_ctx = mutate.v.shape[0]
    for j in (0, 7, 20):
        for h in (0, 13, 31):
            want = (mutate.v[:, h // 4].sum(0) + mutate.vs[: j + 1, h // 4].sum(0)) / (n_ctx + j + 1)
            assert np.abs(got[j, h] - want).max() < 2e-3


def test_attention_llama8b_bf16_full(ad, oracle_mod):
    """Config 2 at full size: 128 query tokens x 32 heads over ~26k assembled tokens, every output checked."""
    w = wl.WORKLOADS["llama8b_1layer"]
    (mx, fro), got, ref = _attention_case(ad, oracle_mod, w, w.m_select, w.t_q)
    assert np.linalg.norm(ref) > 0


def test_attention_bf16_context_length_sweep(ad, oracle_mod):
    """Context lengths around every boundary of the key loop (64-key tiles, the four-tile unroll, split edges)
    and query lengths around the 32-row and 256-row edges, sampled outputs against the oracle; one cache,
    single calls and one batched call over the same cases."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ids, order = wl.selection(w)
    ids, order = ids[:48], np.argsort(np.argsort(order[:48])).astype(np.int32)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    cache = ad.Cache(ctx, total, with_index=False)
    ctx.assemble(cache, ids, order)
    kc, vc = H.to_storage(cache.k[0]), H.to_storage(cache.v[0])
    g = torch.Generator(device="cuda"); g.manual_seed(31337)
    cases = [(1, 1), (63, 7), (64, 8), (65, 9), (127, 33), (129, 64), (255, 65), (257, 1), (320, 2), (511, 5),
             (1000, 3), (1025, 70), (2048, 4), (4097, 1), (total, 6)]
    rng = np.random.default_rng(8)
    items, refs = [], []
    for n_ctx, t_q in cases:
        q = torch.randn(t_q, w.n_q_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        ks = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        vs = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        pairs = np.stack([rng.integers(0, t_q, 4), rng.integers(0, w.n_q_heads, 4)], 1).astype(np.int32)
        pairs[0] = (t_q - 1, w.n_q_heads - 1)
        ref = oracle_mod.query_attn(kc, vc, w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                    w.rope_theta, n_ctx, pairs=pairs)
        out = ctx.query_attn(cache, 0, n_ctx, q, ks, vs, n_ctx).float().cpu().numpy()
        H.check_attention(np.stack([out[j, h] for j, h in pairs]), ref)
        items.append((0, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q)))
        refs.append((pairs, ref))
    ctx.query_attn_batched([cache], 0, items)
    torch.cuda.synchronize()
    for it, (pairs, ref) in zip(items, refs):
        out = it[6].float().cpu().numpy()
        H.check_attention(np.stack([out[j, h] for j, h in pairs]), ref)
    ctx.close()


def test_attention_entropy_and_ranking_errors_launch_nothing(ad):
    """Every bad argument is reported with its status before anything is launched: the output buffers keep
    their sentinel, also when only one item of a batch is bad."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1, max_position=4096)
    q, ks, vs = wl.make_query(w, "cuda", t_q=8)
    with pytest.raises(ad.AdapshotError) as e:   # no pool yet
        ctx.rank_shots(0, q)
    assert e.value.status == ad.ESTATE
    ctx.pool_register(k_pool, v_pool, off)
    cache = ad.Cache(ctx, 512)
    ctx.assemble(cache, [3, 5])
    n = cache.len
    out = torch.full_like(q, 7.0)

    def bad(status, **kw):
        a = dict(layer=0, n_ctx=n, q_pos0=n)
        a.update(kw)
        with pytest.raises(ad.AdapshotError) as e:
            ctx.query_attn(cache, a["layer"], a["n_ctx"], a.get("q", q), ks, vs, a["q_pos0"], out=out)
        assert e.value.status == status, (kw, e.value)
        assert ctx.last_error()

    bad(ad.ESTATE, n_ctx=n + 1)              # beyond the assembled length
    bad(ad.EINVAL, n_ctx=-1)
    bad(ad.EINVAL, layer=1)
    bad(ad.EINVAL, layer=-1)
    bad(ad.ECAPACITY, q_pos0=4096 - 4)       # the query's positions run past max_position
    bad(ad.EINVAL, q_pos0=-1)
    bad(ad.EINVAL, q=q.view(-1)[1:1 + 7 * q.shape[1] * q.shape[2]].view(7, q.shape[1], q.shape[2]))  # not 16-byte aligned
    # a query of 2 GiB or more (the kernels address its rows by 32-bit offsets); found from the sizes alone
    ctx2 = ad.Context.for_workload(w, n_layers=1, max_position=1 << 20)
    cache2 = ad.Cache(ctx2, 64)
    t_big = (1 << 31) // (w.n_q_heads * w.head_dim * 2) + 1
    with pytest.raises(ad.AdapshotError) as e:
        ctx2._check(ctx2.lib.adapshot_query_attn(ctx2._h, ctypes.byref(cache2.c), 0, 0, q.data_ptr(), ks.data_ptr(),
                                                 vs.data_ptr(), t_big, 0, out.data_ptr(), None))
    assert e.value.status == ad.EINVAL and "2 GiB" in e.value.message
    ctx2.close()
    # a batch with one bad item among good ones launches nothing at all
    outs = [torch.full_like(q, 7.0) for _ in range(3)]
    items = [(0, n, q, ks, vs, n, outs[0]), (0, n + 1, q, ks, vs, n, outs[1]), (0, n // 2, q, ks, vs, n // 2, outs[2])]
    with pytest.raises(ad.AdapshotError) as e:
        ctx.query_attn_batched([cache], 0, items)
    assert e.value.status == ad.ESTATE and "item 1" in e.value.message
    with pytest.raises(ad.AdapshotError) as e:
        ctx.query_attn_batched([cache], 0, [(1, n, q, ks, vs, n, outs[0])])   # cache index out of range
    assert e.value.status == ad.EINVAL
    # entropy
    z = wl.make_logits(w, "cuda", n_rows=4)
    h = torch.full((4,), 7.0, device="cuda")
    for ids, mode in (([w.vocab], 0), ([-1], 0), ([5, 5], 0), ([], 0), (list(range(17)), 0), ([1, 2], 2)):
        with pytest.raises(ad.AdapshotError) as e:
            ctx.probe_entropy_tokens(z, ids, mode, out=h)
        assert e.value.status == ad.EINVAL, (ids, mode)
    with pytest.raises(ad.AdapshotError) as e:   # rows overlap: row stride shorter than the vocabulary
        ctx._check(ctx.lib.adapshot_probe_entropy(ctx._h, z.data_ptr(), w.vocab - 1, 4, w.vocab, h.data_ptr(), None))
    assert e.value.status == ad.EINVAL
    # ranking
    sc = torch.full((w.n_shots,), 7.0, device="cuda")
    for layer, pos in ((1, 0), (0, 4096 - 4), (0, -1)):
        with pytest.raises(ad.AdapshotError):
            ctx.rank_shots(layer, q, q_pos0=pos, out=sc)
    torch.cuda.synchronize()
    assert (out == 7.0).all() and all((o == 7.0).all() for o in outs) and (h == 7.0).all() and (sc == 7.0).all()
    # and the same context still works afterwards
    ok = ctx.query_attn(cache, 0, n, q, ks, vs, n, out=out)
    torch.cuda.synchronize()
    assert torch.isfinite(ok.float()).all() and not (ok == 7.0).all() and ctx.last_error() == ""
    ctx.close()


def test_pool_and_batched_assemble_errors_change_nothing(ad, oracle_mod):
    """A rejected pool leaves the registered one in place; a batch of assemblies with one bad member writes to
    no cache and moves no length."""
    w = wl.WORKLOADS["tiny_fp32"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda")
    ctx = ad.Context.for_workload(w, max_position=4096)
    ctx.pool_register(k_pool, v_pool, off)
    bad_off = off.copy()
    bad_off[3] = bad_off[2] - 1                                  # decreasing
    for o, kp in ((bad_off, k_pool), (off, k_pool[:, : int(off[-1]) - 1].contiguous())):   # second: pool shorter than the offsets say
        with pytest.raises(ad.AdapshotError) as e:
            ctx.pool_register(kp, kp.clone(), o)
        assert e.value.status == ad.EINVAL
    assert ctx.n_shots == w.n_shots
    c0, c1 = ad.Cache(ctx, 200), ad.Cache(ctx, 200)
    for ids, orders, status in (([[0, 1], [2, 99]], None, ad.ESHOT),
                                ([[0, 1], [2, 3]], [None, [0, 5]], ad.ESHOT),
                                ([[0, 1], list(range(12))], None, ad.ECAPACITY)):
        with pytest.raises(ad.AdapshotError) as e:
            ctx.assemble_batched([c0, c1], ids, orders)
        assert e.value.status == status, (ids, e.value)
    with pytest.raises(ad.AdapshotError) as e:                    # the same cache twice in one batch
        ctx.assemble_batched([c0, c0], [[0], [1]])
    assert e.value.status == ad.EINVAL
    torch.cuda.synchronize()
    for c in (c0, c1):
        assert c.len == 0 and not c.k.any() and not c.v.any() and (c.slot_shot == -1).all()
    # the pool registered first is still the one in use
    ctx.assemble_batched([c0, c1], [[0, 1], [2, 3]])
    torch.cuda.synchronize()
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    for c, ids in ((c0, [0, 1]), (c1, [2, 3])):
        pl = oracle_mod.plan(off, ids, None)
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, 200)
        assert c.len == pl["n"] and np.array_equal(H.to_storage(c.v), vo)
        assert np.abs(H.to_storage(c.k).astype(np.float64) - ko).max() < 1e-4
    ctx.close()


def test_calls_are_ordered_on_the_callers_stream(ad, oracle_mod):
    """The inputs are produced on a side stream behind several milliseconds of other work, and the library is called
    with that stream right away: it sees the right inputs only if its kernels are ordered on that stream too.
    The results are read back after synchronising that stream alone."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    ids, order = wl.selection(w)
    ids, order = ids[:6], np.argsort(np.argsort(order[:6])).astype(np.int32)
    z_src = wl.make_logits(w, "cuda", n_rows=8)
    q_src, ks, vs = wl.make_query(w, "cuda", t_q=16)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    cache = ad.Cache(ctx, 1024)
    z = torch.zeros_like(z_src)
    q = torch.zeros_like(q_src)
    with torch.cuda.stream(s):
        a = torch.randn(4096, 4096, device="cuda")
        for _ in range(40):                      # a few milliseconds of work ahead of the inputs
            a = torch.tanh(a @ a * 1e-3)
        z.copy_(z_src)
        q.copy_(q_src)
        ctx.assemble(cache, ids, order, stream=s)
        n = cache.len
        out = ctx.query_attn(cache, 0, n, q, ks, vs, n, stream=s)
        h = ctx.probe_entropy(z, stream=s)
        h2 = ctx.probe_entropy_tokens(z, [11, 22], ad.ENTROPY_FULL_P, stream=s)
    s.synchronize()
    want_h = oracle_mod.entropy(z_src.cpu().numpy())
    assert np.abs(h.cpu().numpy() - want_h).max() < 1e-4
    assert np.abs(h2.cpu().numpy() - oracle_mod.entropy_subset(z_src.cpu().numpy(), [11, 22], 0)).max() < 1e-4
    ref = oracle_mod.query_attn(H.to_storage(cache.k[0]), H.to_storage(cache.v[0]), w.dtype, n, H.to_storage(q_src),
                                H.to_storage(ks), H.to_storage(vs), w.rope_theta, n)
    H.check_attention(out.float().cpu().numpy(), ref)
    ctx.close()


def test_two_contexts_on_two_streams(ad, oracle_mod):
    """One context per concurrent stream: two contexts over the same borrowed pool, each with its own cache and
    query, are driven from two streams at once, several rounds, and both match the oracle."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs, caches, sels, qs, outs = [], [], [], [], []
    for i in range(2):
        c = ad.Context.for_workload(w, n_layers=1)
        c.pool_register(k_pool, v_pool, off)
        ids, order = wl.selection(w, query=i)
        m = 5 + 3 * i
        sels.append((ids[:m], np.argsort(np.argsort(order[:m])).astype(np.int32)))
        ctxs.append(c)
        caches.append(ad.Cache(c, 2048))
        qs.append(wl.make_query(w, "cuda", query=i, t_q=24 + 8 * i))
        outs.append(torch.empty_like(qs[i][0]))
    torch.cuda.synchronize()
    for rnd in range(4):
        for i in range(2):
            caches[i].reset()
            ctxs[i].assemble(caches[i], sels[i][0], sels[i][1], stream=streams[i])
            n = caches[i].len
            ctxs[i].query_attn(caches[i], 0, n, *qs[i], n, out=outs[i], stream=streams[i])
    for s in streams:
        s.synchronize()
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    for i in range(2):
        pl = oracle_mod.plan(off, sels[i][0], sels[i][1])
        n = pl["n"]
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, n)
        assert caches[i].len == n and np.array_equal(H.to_storage(caches[i].v[:, :n]), vo)
        q, ks, vs = qs[i]
        ref = oracle_mod.query_attn(H.to_storage(caches[i].k[0]), H.to_storage(caches[i].v[0]), w.dtype, n,
                                    H.to_storage(q), H.to_storage(ks), H.to_storage(vs), w.rope_theta, n)
        H.check_attention(outs[i].float().cpu().numpy(), ref)
        ctxs[i].close()


@pytest.mark.parametrize("dtype,d,hq,hkv", [("f32", 8, 2, 1), ("f32", 32, 4, 4), ("f32", 128, 6, 2),
                                            ("bf16", 16, 2, 2), ("bf16", 64, 8, 2), ("bf16", 256, 4, 1)])
def test_other_head_shapes(ad, oracle_mod, dtype, d, hq, hkv):
    """Every head_dim the library accepts besides the workloads' own (fp32: 8..128, bf16: 16..256 in powers of
    two), with grouped, ungrouped and single kv heads: assemble in both key states, then attention over the
    result (the one-wavefront kernel serves every shape the matrix-core kernel does not)."""
    import dataclasses
    w = dataclasses.replace(wl.WORKLOADS["tiny_fp32"], name=f"shape_{dtype}_{d}", n_q_heads=hq, n_kv_heads=hkv,
                            head_dim=d, dtype=dtype, rope_theta=5.0e5)
    for key_state in (0, 1):
        res = _run_assemble_case(ad, oracle_mod, w, key_state, 17, [0.5])
        assert res["total"] > 0
    if dtype == "f32":
        _attention_case(ad, oracle_mod, w, 8, 16, max_abs=1e-4, rel_fro=1e-5)
        _attention_case(ad, oracle_mod, w, 3, 1, pos0=1000, max_abs=1e-4, rel_fro=1e-5)
    else:
        _attention_case(ad, oracle_mod, w, 8, 16)
        _attention_case(ad, oracle_mod, w, 3, 1, pos0=1000)


@pytest.mark.parametrize("hq,hkv,t_q", [(4, 4, 300), (3, 3, 40), (32, 2, 20), (5, 1, 60), (48, 6, 33), (16, 16, 1)])
def test_matrix_core_kernel_other_groupings(ad, oracle_mod, hq, hkv, t_q):
    """bf16, head_dim 128 with group sizes 1, 5, 8 and 16 and kv head counts that are not multiples of the XCD count;
    row counts t_q * g that end inside a wavefront's 32 rows, inside a 256-row tile, and in a second tile."""
    import dataclasses
    w = dataclasses.replace(wl.WORKLOADS["llama8b_1layer"], name=f"grouping_{hq}_{hkv}", n_q_heads=hq, n_kv_heads=hkv)
    _attention_case(ad, oracle_mod, w, 7, t_q)
    _attention_case(ad, oracle_mod, w, 2, t_q, n_ctx=65, pos0=3)


@pytest.mark.parametrize("direction", ["rising", "falling", "spikes"])
def test_attention_bf16_wide_score_range(ad, oracle_mod, direction):
    """Keys scaled by a factor that changes along the context (0.05 .. 3): the row maxima keep rising from tile to
    tile (the reference maximum is moved and everything accumulated rescaled again and again), or fall so that
    late tiles underflow to nothing, or jump at isolated keys.  The scores now span some twenty powers of two,
    and the bf16 rounding of the rotated query, which every bf16 attention carries into its scores, grows with
    them (about 2^-9 of a score): the bars are 1.5 times the ones for N(0,1) keys."""
    w = wl.WORKLOADS["llama8b_1layer"]

    def mutate(cache, q, ks, vs, q_pos0):
        n = cache.len
        u = torch.arange(n, device="cuda", dtype=torch.float32) / max(n - 1, 1)
        if direction == "rising":
            f = 0.05 + 2.95 * u
        elif direction == "falling":
            f = 3.0 - 2.95 * u
        else:
            f = torch.full_like(u, 0.3)
            f[::97] = 3.0
        cache.k[0, :n] = (cache.k[0, :n].float() * f[:, None, None]).to(cache.k.dtype)

    (worst, fro), got, ref = _attention_case(ad, oracle_mod, w, 9, 40, mutate=mutate, max_abs=3e-2, rel_fro=1.5e-2)
    print(f"{direction}: max-abs {worst:.3e}, rel-Frobenius {fro:.3e}")
    assert np.isfinite(got).all() and np.abs(ref).max() > 0.5
