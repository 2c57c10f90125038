"""GPU parity at the sizes bench.py times, against an oracle chain that takes nothing from the GPU path:
the oracle plans, assembles its own cache from the pool and attends over it.

  * the Llama-3-8B single-layer workload in full (every output of assemble, attention and entropy);
  * the probe sweep at its real batch: 8 queries x nested prefixes {16..512} of their own 512-shot ordering
    (up to ~53k tokens), 64 probe tokens, all 48 probes in one adapshot_query_attn_batched call;
  * the decode workload at its real batch: 32 queries x 200 shots (~16k tokens), 64 appended tokens each,
    single-token attention through the batched call at the first step and the last two;
  * relevance ranking over the whole 2000-shot pool.
One layer each (layers are independent and identical in shape); contexts and batches are NOT reduced, only
the outputs compared are sampled where the oracle would otherwise need hours."""
import sys

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
    binding.load_library()
    return binding


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


def test_llama8b_1layer_pure_oracle_chain(ad, oracle_mod):
    """The benchmark's step at its full size, every output: plan, gathered values (bit-exact), re-encoded keys,
    attention of all 128 x 32 rows over the ORACLE's own assembled cache, entropy of all 128 rows."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda")
    ids, order = wl.selection(w)
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    cache = ad.Cache(ctx, total)
    ctx.assemble(cache, ids, order)
    q, ks, vs = wl.make_query(w, "cuda")
    out = ctx.query_attn(cache, 0, total, q, ks, vs, total)
    z = wl.make_logits(w, "cuda")
    h = ctx.probe_entropy(z)
    torch.cuda.synchronize()

    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    pl = oracle_mod.plan(off, ids, order)
    assert pl["n"] == total
    assert np.array_equal(cache.slot_shot.cpu().numpy(), pl["slot_shot"])
    assert np.array_equal(cache.slot_tok.cpu().numpy(), pl["slot_tok"])
    assert np.array_equal(cache.slot_pos.cpu().numpy(), pl["slot_pos"])
    ko, vo, kx = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, total, want_exact=True)
    assert np.array_equal(H.to_storage(cache.v), vo)
    H.check_reencode_bf16(H.to_storage(cache.k), ko, kx, kp[:, pl["slot_src"]])
    ref = oracle_mod.query_attn(ko[0], vo[0], w.dtype, total, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                w.rope_theta, total)
    err, fro = H.check_attention(out.float().cpu().numpy(), ref)
    _say(f"llama8b_1layer pure-oracle chain: attention max-abs {err:.2e}, rel-Frobenius {fro:.2e}")
    herr = np.abs(h.cpu().numpy().astype(np.float64) - oracle_mod.entropy(z.cpu().numpy())).max()
    assert herr <= 1e-4, herr
    ctx.close()


def test_probe_sweep_full_batch_against_oracle(ad, oracle_mod):
    """Config 3's batch on one layer: 8 caches of 512 shots assembled in one adapshot_assemble_batched call,
    48 probes (8 queries x 6 nested prefixes, 64 tokens each) in one adapshot_query_attn_batched call.
    1056 sampled (probe, row, head) outputs, 22 per probe, against the oracle's own assembly of each ordering
    (a k-shot prefix of it IS the k-shot assembly: checked on the integer plan)."""
    w = wl.WORKLOADS["llama8b_sweep"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, query=qi) for qi in range(w.n_queries)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    assert len(sels) == 8 and max(totals) > 50000
    caches = [ad.Cache(ctx, t, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    assert [c.len for c in caches] == totals
    items, meta = [], []
    for qi in range(w.n_queries):
        ids, order = sels[qi]
        seq = [int(ids[o]) for o in order]
        q, ks, vs = wl.make_query(w, "cuda", query=qi, layer=0)
        for k in w.prefixes:
            n_ctx = int(sum(off[s + 1] - off[s] for s in seq[:k]))
            out = torch.empty_like(q)
            items.append((qi, n_ctx, q, ks, vs, n_ctx, out))
            meta.append((qi, k, n_ctx, q, ks, vs, out))
    assert len(items) == 48
    ctx.query_attn_batched(caches, 0, items)
    torch.cuda.synchronize()

    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    rng = np.random.default_rng(3)
    worst, n_checked = 0.0, 0
    got_all, ref_all = [], []
    for qi in range(w.n_queries):
        ids, order = sels[qi]
        pl = oracle_mod.plan(off, ids, order)
        ko, vo, kx = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, totals[qi], want_exact=True)
        # the batched assemble at this size: values bit-exact, keys to the re-encode bar
        assert np.array_equal(H.to_storage(caches[qi].v), vo)
        H.check_reencode_bf16(H.to_storage(caches[qi].k), ko, kx, kp[:, pl["slot_src"]])
        del kx
        seq = [int(ids[o]) for o in order]
        for (mq, k, n_ctx, q, ks, vs, out) in meta:
            if mq != qi:
                continue
            plk = oracle_mod.plan(off, seq[:k], None)   # assembling the first k shots from scratch ...
            assert plk["n"] == n_ctx
            assert np.array_equal(plk["slot_src"], pl["slot_src"][:n_ctx])  # ... reads the same pool tokens
            assert np.array_equal(plk["slot_pos"], pl["slot_pos"][:n_ctx])  # ... to the same positions
            pairs = np.stack([rng.integers(0, w.t_q, 22), rng.integers(0, w.n_q_heads, 22)], axis=1).astype(np.int32)
            pairs[0] = (0, 0)
            pairs[1] = (w.t_q - 1, w.n_q_heads - 1)
            ref = oracle_mod.query_attn(ko[0], vo[0], w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks),
                                        H.to_storage(vs), w.rope_theta, n_ctx, pairs=pairs)
            o = out.float().cpu().numpy()
            got = np.stack([o[j, h] for j, h in pairs])
            assert np.isfinite(o).all()
            err, _ = H.check_attention(got, ref)
            worst = max(worst, err)
            n_checked += len(pairs)
            got_all.append(got)
            ref_all.append(ref)
        _say(f"probe sweep full batch: query {qi} checked ({totals[qi]} tokens)")
    assert n_checked >= 1000
    H.check_attention(np.concatenate(got_all), np.concatenate(ref_all))
    _say(f"probe sweep full batch: {n_checked} sampled outputs, worst max-abs {worst:.2e}")
    ctx.close()


def test_decode_full_batch_against_oracle(ad, oracle_mod):
    """Config 5's batch on one layer: 32 caches of 200 shots (~16k tokens) assembled in one call, then 64
    decode steps of adapshot_decode_append; at steps 0, 62 and 63 the 32 single-token queries attend through
    adapshot_query_attn_batched (7 query heads per kv head: rows per kv head = 7) and EVERY output
    (3 x 32 x 28 rows) is compared with the oracle attending over its own cache."""
    w = wl.WORKLOADS["qwen7b_decode"]
    nq, steps = w.n_queries, w.decode_steps
    assert nq == 32 and steps == 64
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, query=qi) for qi in range(nq)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    assert np.mean(totals) > 14000
    caches = [ad.Cache(ctx, t + steps, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    ref_k, ref_v = [], []
    for qi in range(nq):
        pl = oracle_mod.plan(off, sels[qi][0], sels[qi][1])
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, totals[qi] + steps)
        ref_k.append(ko)
        ref_v.append(vo)
    _say("decode full batch: oracle caches assembled")
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed + 177)
    n_checked, worst = 0, 0.0
    for s in range(steps):
        k_new = torch.randn(1, nq, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
        v_new = torch.randn(1, nq, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
        lens = [c.len for c in caches]
        ctx.decode_append(caches, k_new, v_new)
        kn, vn = H.to_storage(k_new), H.to_storage(v_new)
        for qi in range(nq):
            ref_k[qi][0, lens[qi]] = oracle_mod.rot_rows(kn[0, qi], w.dtype, w.rope_theta,
                                                         np.full(w.n_kv_heads, float(lens[qi])))
            ref_v[qi][0, lens[qi]] = vn[0, qi]
        if s not in (0, steps - 2, steps - 1):
            continue
        items = []
        for qi in range(nq):
            q, ks, vs = wl.make_query(w, "cuda", query=qi * 100 + s, layer=0)
            items.append((qi, caches[qi].len, q, ks, vs, caches[qi].len, torch.empty_like(q)))
        ctx.query_attn_batched(caches, 0, items)
        torch.cuda.synchronize()
        got_all, ref_all = [], []
        for qi, n_ctx, q, ks, vs, _, out in items:
            ref = oracle_mod.query_attn(ref_k[qi][0], ref_v[qi][0], w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks),
                                        H.to_storage(vs), w.rope_theta, n_ctx)
            got = out.float().cpu().numpy()
            err, _ = H.check_attention(got, ref)
            worst = max(worst, err)
            n_checked += got.shape[0] * got.shape[1]
            got_all.append(got)
            ref_all.append(ref)
        H.check_attention(np.concatenate(got_all), np.concatenate(ref_all))
        _say(f"decode full batch: step {s} checked")
    assert n_checked >= 1000
    _say(f"decode full batch: {n_checked} outputs, worst max-abs {worst:.2e}")
    torch.cuda.synchronize()
    for qi in range(nq):
        n = caches[qi].len
        assert n == totals[qi] + steps
        kg, vg = H.to_storage(caches[qi].k), H.to_storage(caches[qi].v)
        assert np.array_equal(vg[:, :n], ref_v[qi][:, :n])
        assert (kg[:, :n] == ref_k[qi][:, :n]).mean() > 0.99
        assert np.abs(H.storage_to_f64(kg[:, :n]) - H.storage_to_f64(ref_k[qi][:, :n])).max() < 0.05
    ctx.close()


def test_rank_full_pool_against_oracle(ad, oracle_mod):
    """Relevance of all 2000 shots of config 2's pool (~209k tokens) to the 128-token query: every score
    against the oracle's whole-pool softmax."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda")
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    q, _, _ = wl.make_query(w, "cuda")
    got = ctx.rank_shots(0, q).cpu().numpy().astype(np.float64)
    again = ctx.rank_shots(0, q).cpu().numpy().astype(np.float64)
    _say("rank full pool: GPU done, oracle running")
    want = oracle_mod.rank_scores(H.to_storage(k_pool)[0], "bf16", off, H.to_storage(q), w.rope_theta, 0)
    lens = np.diff(off)
    assert abs(float((want * lens).sum()) - 1.0) < 1e-9
    assert abs(float((got * lens).sum()) - 1.0) < 2e-3
    err = np.abs(got - want)
    assert float(err.max()) <= 2e-2 * want.max() and float((err / want).mean()) < 5e-3, (err.max(), want.max())
    assert np.array_equal(again, got)   # fixed summation order: the same query gives the same bits
    ids = ctx.top_k(got, 16)
    order = np.argsort(-want, kind="stable")
    margin = 4 * float(err.max())
    for r, i in enumerate(ids):
        assert want[i] >= want[order[r]] - margin
    _say(f"rank full pool: worst error {err.max():.3e} of max score {want.max():.3e}")
    ctx.close()
