"""GPU parity on the multi-query workloads: the nested-prefix probe sweep (config 3), the 128k-token
context (config 4, sampled outputs) and the decode loop (config 5), all through the C ABI."""
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


def test_probe_sweep_nested_prefixes_batched(ad, oracle_mod):
    """Config 3 shape, 2 layers, 3 queries: each query assembles its own 64-shot ordering once
    (adapshot_assemble_batched); probes at prefixes k = 16, 32, 64 attend over slots [0, off_k) of that cache
    (adapshot_query_attn_batched) -- a prefix keeps its positions, so this equals re-assembling k shots."""
    w = wl.WORKLOADS["llama8b_sweep"]
    L, n_q, ks_list, m_max = 2, 3, (16, 32, 64), 64
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=L)
    ctx = ad.Context.for_workload(w, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    sels = []
    for qi in range(n_q):
        ids, order = wl.selection(w, query=qi)
        ids, order = ids[:m_max], np.argsort(np.argsort(order[:m_max])).astype(np.int32)
        sels.append((ids, order))
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    caches = [ad.Cache(ctx, t) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    assert [c.len for c in caches] == totals
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)

    for layer in range(L):
        items, meta = [], []
        for qi in range(n_q):
            ids, order = sels[qi]
            seq = [int(ids[o]) for o in order]
            q, ks, vs = wl.make_query(w, "cuda", query=qi, layer=layer)
            for k in ks_list:
                n_ctx = int(sum(off[s + 1] - off[s] for s in seq[:k]))
                out = torch.empty_like(q)
                items.append((qi, n_ctx, q, ks, vs, n_ctx, out))
                meta.append((qi, k, n_ctx, q, ks, vs, out))
        ctx.query_attn_batched(caches, layer, items)
        torch.cuda.synchronize()
        for qi, k, n_ctx, q, ks, vs, out in meta:
            ids, order = sels[qi]
            # oracle: assemble exactly the first k shots from scratch, then attend
            seq = [int(ids[o]) for o in order][:k]
            pl = oracle_mod.plan(off, seq, None)
            assert pl["n"] == n_ctx
            ko, vo, _ = oracle_mod.assemble(kp[layer:layer + 1], vp[layer:layer + 1], w.dtype, w.rope_theta, 0, pl, 0, n_ctx)
            pairs = np.array([[j, h] for j in (0, 17, w.t_q - 1) for h in (0, 9, 31)], np.int32)
            ref = oracle_mod.query_attn(ko[0], vo[0], w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                        w.rope_theta, n_ctx, pairs=pairs)
            got = np.stack([out.float().cpu().numpy()[j, h] for j, h in pairs])
            H.check_attention(got, ref)
            # the prefix of the incrementally assembled cache is bit-identical to the from-scratch assembly
            assert (H.to_storage(caches[qi].k[layer, :n_ctx]) == ko[0]).mean() > 0.99
            assert np.array_equal(H.to_storage(caches[qi].v[layer, :n_ctx]), vo[0])
    # a bad item anywhere fails the whole batch before anything runs
    out0 = items[0][6].clone()
    bad = list(items)
    bad[-1] = (0, totals[0] + 1, *items[-1][2:])
    with pytest.raises(ad.AdapshotError) as e:
        ctx.query_attn_batched(caches, 0, bad)
    assert e.value.status == ad.ESTATE
    torch.cuda.synchronize()
    assert torch.equal(items[0][6], out0)
    ctx.close()


def test_llama70b_128k_context_sampled(ad, oracle_mod):
    """Config 4 at full context size on one layer: 1000 of 4000 shots (~128k tokens), 256 query tokens,
    64 q heads / 8 kv heads.  Assemble is checked in full; attention on 1000 sampled (row, head) outputs
    (each one a 127k-key softmax for the oracle)."""
    w = wl.WORKLOADS["llama70b_128k"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ids, order = wl.selection(w)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    assert total > 120000
    cache = ad.Cache(ctx, total)
    ctx.assemble(cache, ids, order)
    q, ks, vs = wl.make_query(w, "cuda")
    out = ctx.query_attn(cache, 0, total, q, ks, vs, total)
    torch.cuda.synchronize()
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    pl = oracle_mod.plan(off, ids, order)
    assert np.array_equal(cache.slot_pos.cpu().numpy(), pl["slot_pos"])
    assert np.array_equal(cache.slot_shot.cpu().numpy(), pl["slot_shot"])
    ko, vo, kx = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, total, want_exact=True)
    kg, vg = H.to_storage(cache.k), H.to_storage(cache.v)
    assert np.array_equal(vg, vo)
    H.check_reencode_bf16(kg, ko, kx, kp[:, pl["slot_src"]])
    rng = np.random.default_rng(4)
    n_s = 1000
    pairs = np.stack([rng.integers(0, w.t_q, n_s), rng.integers(0, w.n_q_heads, n_s)], axis=1).astype(np.int32)
    pairs[0] = (0, 0); pairs[1] = (w.t_q - 1, w.n_q_heads - 1)
    ref = oracle_mod.query_attn(kg[0], vg[0], w.dtype, total, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                w.rope_theta, total, pairs=pairs)
    got = np.stack([out.float().cpu().numpy()[j, h] for j, h in pairs])
    H.check_attention(got, ref)
    ctx.close()


def test_qwen_decode_loop(ad, oracle_mod):
    """Config 5 shape, 2 layers, 4 queries with their own 12-shot orderings, 5 decode steps: every step appends
    one token per query (adapshot_decode_append) and attends with a single query token (g = 7 rows per kv head)."""
    w = wl.WORKLOADS["qwen7b_decode"]
    L, n_q, steps, m = 2, 4, 5, 12
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=L)
    ctx = ad.Context.for_workload(w, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, query=qi) for qi in range(n_q)]
    sels = [(ids[:m], np.argsort(np.argsort(order[:m])).astype(np.int32)) for ids, order in sels]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    caches = [ad.Cache(ctx, t + steps) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    # oracle caches
    ref_k, ref_v = [], []
    for qi in range(n_q):
        pl = oracle_mod.plan(off, sels[qi][0], sels[qi][1])
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl, 0, totals[qi] + steps)
        ref_k.append(ko); ref_v.append(vo)
    g = torch.Generator(device="cuda"); g.manual_seed(w.seed + 77)
    for s in range(steps):
        k_new = torch.randn(L, n_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
        v_new = torch.randn(L, n_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
        lens = [c.len for c in caches]
        ctx.decode_append(caches, k_new, v_new)
        assert [c.len for c in caches] == [n + 1 for n in lens]
        # oracle append: rotate the new key of query qi to position lens[qi]
        kn, vn = H.to_storage(k_new), H.to_storage(v_new)
        for qi in range(n_q):
            rot = oracle_mod.rot_rows(kn[:, qi], w.dtype, w.rope_theta, np.full(L * w.n_kv_heads, float(lens[qi])))
            ref_k[qi][:, lens[qi]] = rot
            ref_v[qi][:, lens[qi]] = vn[:, qi]
        # one query token per query attends over its whole cache (the token it just appended included)
        for layer in range(L):
            items, meta = [], []
            for qi in range(n_q):
                q, ks, vs = wl.make_query(w, "cuda", query=qi * 100 + s, layer=layer)
                out = torch.empty_like(q)
                n_ctx = caches[qi].len
                items.append((qi, n_ctx, q, ks, vs, n_ctx, out))
                meta.append((qi, n_ctx, q, ks, vs, out))
            ctx.query_attn_batched(caches, layer, items)
            torch.cuda.synchronize()
            for qi, n_ctx, q, ks, vs, out in meta:
                kc, vc = H.to_storage(caches[qi].k[layer]), H.to_storage(caches[qi].v[layer])
                ref = oracle_mod.query_attn(kc, vc, w.dtype, n_ctx, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                            w.rope_theta, n_ctx)
                H.check_attention(out.float().cpu().numpy(), ref)
    torch.cuda.synchronize()
    for qi in range(n_q):
        n = caches[qi].len
        kg, vg = H.to_storage(caches[qi].k), H.to_storage(caches[qi].v)
        assert np.array_equal(vg[:, :n], ref_v[qi][:, :n])
        assert (kg[:, :n] == ref_k[qi][:, :n]).mean() > 0.99
        assert np.array_equal(caches[qi].slot_pos[:n].cpu().numpy(), np.arange(n))
        assert (caches[qi].slot_shot[totals[qi]:n] == -1).all()
    # a full cache is refused and nothing is appended anywhere
    lens = [c.len for c in caches]
    with pytest.raises(ad.AdapshotError) as e:
        ctx.decode_append(caches, k_new, v_new)
    assert e.value.status == ad.ECAPACITY and [c.len for c in caches] == lens
    ctx.close()


def test_batched_attention_edge_items_match_single_calls(ad, oracle_mod):
    """One batch mixing an empty context, a one-token query, a ragged query length and a long context, over two
    caches: every item equals its single-call result (same kernels, different split plan) within the bf16
    output rounding, and the empty-context item is checked against the oracle."""
    w = wl.WORKLOADS["llama8b_sweep"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    sels = []
    for qi in range(2):
        ids, order = wl.selection(w, query=qi)
        ids, order = ids[:40], np.argsort(np.argsort(order[:40])).astype(np.int32)
        sels.append((ids, order))
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    caches = [ad.Cache(ctx, t) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    g = torch.Generator(device="cuda"); g.manual_seed(4242)

    def qkv(t_q):
        q = torch.randn(t_q, w.n_q_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        ks = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        vs = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        return q, ks, vs

    specs = [(0, 0, 5), (1, totals[1], 1), (0, totals[0], 37), (1, 777, 64), (0, 63, 3), (1, 65, 130)]
    items, singles = [], []
    for ci, n_ctx, t_q in specs:
        q, ks, vs = qkv(t_q)
        items.append((ci, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q)))
        singles.append(ctx.query_attn(caches[ci], 0, n_ctx, q, ks, vs, n_ctx).float().cpu().numpy())
    ctx.query_attn_batched(caches, 0, items)
    ctx.query_attn_batched(caches, 0, [])          # an empty batch is a no-op
    torch.cuda.synchronize()
    for (ci, n_ctx, t_q), it, one in zip(specs, items, singles):
        got = it[6].float().cpu().numpy()
        assert np.isfinite(got).all()
        assert float(np.abs(got - one).max()) <= 2.0 ** -7 * max(1.0, float(np.abs(one).max())), (ci, n_ctx, t_q)
    # the empty-context item attends to its own tokens only
    ci, n_ctx, t_q = specs[0]
    q, ks, vs = items[0][2], items[0][3], items[0][4]
    ref = oracle_mod.query_attn(H.to_storage(caches[0].k[0]), H.to_storage(caches[0].v[0]), w.dtype, 0, H.to_storage(q),
                                H.to_storage(ks), H.to_storage(vs), w.rope_theta, 0)
    H.check_attention(items[0][6].float().cpu().numpy(), ref)
    ctx.close()


def test_byte_offsets_beyond_4gib_in_pool_and_cache(ad, oracle_mod):
    """Six layers of the config-4 shape.  The pool holds 1.07 GB per layer and operand and the cache is given
    a capacity of 520k tokens, so layer 3 starts beyond byte offset 2^31 and layer 5 beyond 2^32 in both.
    Those two layers are checked: assemble on every selected token, untouched rows around them, attention
    over the assembled context, and one appended decode token."""
    w = wl.WORKLOADS["llama70b_128k"]
    L, m, t_q, cap = 6, 48, 16, 520_000
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=L)
    row_bytes = w.n_kv_heads * w.head_dim * 2
    assert 3 * int(off[-1]) * row_bytes > 2 ** 31 and 5 * int(off[-1]) * row_bytes > 2 ** 32
    assert 3 * cap * row_bytes > 2 ** 31 and 5 * cap * row_bytes > 2 ** 32
    ids, order = wl.selection(w)
    ids = ids[:m]
    order = np.argsort(np.argsort(order[:m])).astype(np.int32)
    ctx = ad.Context.for_workload(w, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    cache = ad.Cache(ctx, cap)
    ctx.assemble(cache, ids, order)
    torch.cuda.synchronize()
    pl = oracle_mod.plan(off, ids, order)
    assert np.array_equal(cache.slot_pos[:total].cpu().numpy(), pl["slot_pos"])
    src = torch.from_numpy(pl["slot_src"]).cuda()
    small = dict(pl, slot_src=np.arange(total, dtype=np.int64))   # the same plan over the gathered rows only
    q, ks, vs = wl.make_query(w, "cuda", t_q=t_q)
    g = torch.Generator(device="cuda"); g.manual_seed(w.seed + 5)
    k_new = torch.randn(L, 1, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
    v_new = torch.randn(L, 1, w.n_kv_heads, w.head_dim, device="cuda", generator=g).to(torch.bfloat16)
    for layer in (3, 5):
        kp, vp = H.to_storage(k_pool[layer:layer + 1, src]), H.to_storage(v_pool[layer:layer + 1, src])
        ko, vo, kx = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, small, 0, total, want_exact=True)
        kg, vg = H.to_storage(cache.k[layer:layer + 1, :total]), H.to_storage(cache.v[layer:layer + 1, :total])
        assert np.array_equal(vg, vo)
        H.check_reencode_bf16(kg, ko, kx, kp)
        # nothing was written past the assembled rows of this layer or before the first row of the next one
        assert not cache.k[layer, total:total + 4096].any() and not cache.v[layer, total:total + 4096].any()
        assert not cache.k[layer, cap - 4096:].any() and not cache.v[layer, cap - 4096:].any()
        out = ctx.query_attn(cache, layer, total, q, ks, vs, total)
        ref = oracle_mod.query_attn(kg[0], vg[0], w.dtype, total, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                    w.rope_theta, total)
        H.check_attention(out.float().cpu().numpy(), ref)
    ctx.decode_append([cache], k_new, v_new)
    torch.cuda.synchronize()
    assert cache.len == total + 1
    kn, vn = H.to_storage(k_new), H.to_storage(v_new)
    for layer in (3, 5):
        rot = oracle_mod.rot_rows(kn[layer, 0], w.dtype, w.rope_theta, np.full(w.n_kv_heads, float(total)))
        got = H.to_storage(cache.k[layer, total])
        assert (got == rot).mean() > 0.99 and np.abs(H.storage_to_f64(got) - H.storage_to_f64(rot)).max() < 0.05
        assert np.array_equal(H.to_storage(cache.v[layer, total]), vn[layer, 0])
        assert not cache.k[layer, total + 1:total + 4096].any()
    ctx.close()


def test_assemble_batched_many_caches_one_call(ad, oracle_mod):
    """53 caches in one adapshot_assemble_batched call (more than one launch's table of caches holds): ragged
    selections, an empty one, duplicates, appended after a first call; every cache against the oracle."""
    w = wl.WORKLOADS["tiny_fp32"]
    L = 2
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=L)
    ctx = ad.Context.for_workload(w, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    rng = np.random.default_rng(53)
    n_c = 53
    first = [rng.integers(0, w.n_shots, rng.integers(0, 4)).astype(np.int32) for _ in range(n_c)]
    second = [rng.integers(0, w.n_shots, rng.integers(1, 5)).astype(np.int32) for _ in range(n_c)]
    first[7] = np.zeros(0, np.int32)                      # nothing to append for this cache
    lens = lambda ids: int(sum(off[i + 1] - off[i] for i in ids))
    caches = [ad.Cache(ctx, lens(a) + lens(b) + 3) for a, b in zip(first, second)]
    ctx.assemble_batched(caches, first, None, pos0=5)
    ctx.assemble_batched(caches, second, [np.argsort(rng.random(len(b))).astype(np.int32) for b in second], pos0=5)
    torch.cuda.synchronize()
    kp, vp = H.to_storage(k_pool), H.to_storage(v_pool)
    rng = np.random.default_rng(53)                        # replay the draws to recover the second call's orders
    _ = [rng.integers(0, w.n_shots, rng.integers(0, 4)) for _ in range(n_c)]
    _ = [rng.integers(0, w.n_shots, rng.integers(1, 5)) for _ in range(n_c)]
    orders = [np.argsort(rng.random(len(b))).astype(np.int32) for b in second]
    for ci in range(n_c):
        n1, n2 = lens(first[ci]), lens(second[ci])
        assert caches[ci].len == n1 + n2
        cap = caches[ci].capacity
        pl1 = oracle_mod.plan(off, first[ci], None, slot0=0, pos0=5)
        pl2 = oracle_mod.plan(off, second[ci], orders[ci], slot0=n1, pos0=5)
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl1, 0, cap, want_exact=False)
        ko, vo, _ = oracle_mod.assemble(kp, vp, w.dtype, w.rope_theta, 0, pl2, n1, cap, k_out=ko, v_out=vo)
        kg, vg = H.to_storage(caches[ci].k), H.to_storage(caches[ci].v)
        assert np.array_equal(vg, vo), ci
        assert np.abs(kg.astype(np.float64) - ko.astype(np.float64)).max() <= 2e-5, ci   # fp32 keys, |k| < 6
        want_pos = np.concatenate([pl1["slot_pos"], pl2["slot_pos"]])
        assert np.array_equal(caches[ci].slot_pos[:n1 + n2].cpu().numpy(), want_pos), ci
        assert np.array_equal(caches[ci].slot_shot[:n1 + n2].cpu().numpy(), np.concatenate([pl1["slot_shot"], pl2["slot_shot"]]))
        assert (caches[ci].slot_pos[n1 + n2:] == -1).all()
    ctx.close()


def test_context_at_the_4gib_per_layer_limit(ad, oracle_mod):
    """The attention kernels address a key row by a 32-bit byte offset inside its layer.  A context of 2 097 151
    Llama-shaped rows (4 GiB - 2 KiB per operand) is the largest one accepted: its sampled outputs are checked
    against the oracle (the last context split works at offsets just below 2^32); one more row is refused
    before anything is launched."""
    w = wl.WORKLOADS["llama8b_1layer"]
    n_max = (1 << 32) // (w.n_kv_heads * w.head_dim * 2) - 1
    assert n_max == 2097151
    ctx = ad.Context.for_workload(w, n_layers=1, max_position=1 << 22)
    cache = ad.Cache(ctx, n_max + 17, with_index=False)
    cache.k = wl.normal_tensor(tuple(cache.k.shape), torch.bfloat16, "cuda", 901)     # any keys will do: the oracle sees the same bits
    cache.v = wl.normal_tensor(tuple(cache.v.shape), torch.bfloat16, "cuda", 902)
    cache.c.k, cache.c.v = cache.k.data_ptr(), cache.v.data_ptr()
    cache.c.len = n_max + 17
    t_q = 3
    q, ks, vs = wl.make_query(w, "cuda", t_q=t_q)
    q[1, 5] = (cache.k[0, n_max - 1, 1].float() * 0.5).bfloat16()     # a row that looks at the very last key (un-rotated: close enough to matter)
    out = torch.full_like(q, 7.0)
    with pytest.raises(ad.AdapshotError) as e:
        ctx.query_attn(cache, 0, n_max + 1, q, ks, vs, n_max + 1, out=out)
    assert e.value.status == ad.EINVAL and "4 GiB" in e.value.message
    torch.cuda.synchronize()
    assert float(out.float().min()) == 7.0 and float(out.float().max()) == 7.0
    ctx.query_attn(cache, 0, n_max, q, ks, vs, n_max, out=out)
    torch.cuda.synchronize()
    pairs = np.array([[0, 0], [1, 5], [2, 31], [0, 17], [2, 8], [1, 30]], np.int32)
    ref = oracle_mod.query_attn(H.to_storage(cache.k[0]), H.to_storage(cache.v[0]), w.dtype, n_max, H.to_storage(q),
                                H.to_storage(ks), H.to_storage(vs), w.rope_theta, n_max, pairs=pairs)
    o = out.float().cpu().numpy()
    H.check_attention(np.stack([o[j, h] for j, h in pairs]), ref)
    ctx.close()
