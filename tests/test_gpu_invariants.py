"""Properties of the GPU path that hold whatever the plan: the attention result does not depend on the number
of context splits, and the same inputs give the same bits on every run (fixed split plan, fixed reduction
orders, no atomics on floating-point data)."""
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


def _setup(ad, w, n_sel, with_index=False):
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ids, order = wl.selection(w)
    ids, order = ids[:n_sel], np.argsort(np.argsort(order[:n_sel])).astype(np.int32)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    cache = ad.Cache(ctx, total, with_index=with_index)
    ctx.assemble(cache, ids, order)
    return ctx, cache, total, (k_pool, v_pool, off, ids, order)


@pytest.mark.parametrize("name,n_sel,t_q", [("llama8b_1layer", 256, 128), ("tiny_fp32", 8, 16)])
def test_attention_does_not_depend_on_the_split_count(ad, oracle_mod, name, n_sel, t_q):
    """Split counts 1, 2 and 7 and the planner's own choice: each within the parity bar of the oracle (which
    assembles its own cache), and within output rounding of each other."""
    w = wl.WORKLOADS[name]
    ctx, cache, total, (k_pool, v_pool, off, ids, order) = _setup(ad, w, n_sel)
    q, ks, vs = wl.make_query(w, "cuda", t_q=t_q)
    pl = oracle_mod.plan(off, ids, order)
    ko, vo, _ = oracle_mod.assemble(H.to_storage(k_pool), H.to_storage(v_pool), w.dtype, w.rope_theta, 0, pl, 0, total)
    rng = np.random.default_rng(11)
    n_s = min(200, t_q * w.n_q_heads)
    flat = rng.choice(t_q * w.n_q_heads, n_s, replace=False)
    pairs = np.stack([flat // w.n_q_heads, flat % w.n_q_heads], axis=1).astype(np.int32)
    ref = oracle_mod.query_attn(ko[0], vo[0], w.dtype, total, H.to_storage(q), H.to_storage(ks), H.to_storage(vs),
                                w.rope_theta, total, pairs=pairs)
    bars = dict(max_abs=2e-2, rel_fro=1e-2) if w.dtype == "bf16" else dict(max_abs=1e-4, rel_fro=1e-5)
    outs = {}
    for n_split in (0, 1, 2, 7):
        ctx.set_attn_splits(n_split)
        o = ctx.query_attn(cache, 0, total, q, ks, vs, total).float().cpu().numpy()
        H.check_attention(np.stack([o[j, h] for j, h in pairs]), ref, **bars)
        outs[n_split] = o
    step = 2.0 ** -7 if w.dtype == "bf16" else 1e-5      # one rounding step of the output type at its largest value
    scale = max(1.0, float(np.abs(outs[0]).max()))
    for n_split in (1, 2, 7):
        assert float(np.abs(outs[n_split] - outs[0]).max()) <= step * scale, n_split
    with pytest.raises(ad.AdapshotError):
        ctx.set_attn_splits(65)
    ctx.set_attn_splits(0)
    ctx.close()


def test_batched_attention_does_not_depend_on_the_split_count(ad):
    """The batched planner with the longest item cut into 1, 2 and 7 splits against its own choice."""
    w = wl.WORKLOADS["llama8b_sweep"]
    ctx, cache, total, _ = _setup(ad, w, 48)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    items = []
    for n_ctx, t_q in ((total, 64), (total // 3, 64), (777, 5), (0, 9), (total - 1, 1)):
        q = torch.randn(t_q, w.n_q_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        ks = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        vs = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        items.append((0, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q)))
    outs = {}
    for n_split in (0, 1, 2, 7):
        ctx.set_attn_splits(n_split)
        ctx.query_attn_batched([cache], 0, items)
        torch.cuda.synchronize()
        outs[n_split] = [it[6].float().cpu().numpy().copy() for it in items]
    for n_split in (1, 2, 7):
        for a, b in zip(outs[n_split], outs[0]):
            assert np.isfinite(a).all()
            assert float(np.abs(a - b).max()) <= 2.0 ** -7 * max(1.0, float(np.abs(b).max())), n_split
    ctx.close()


def test_same_inputs_give_the_same_bits(ad):
    """Assemble, attention (single and batched), entropy and ranking, run twice on the same inputs into fresh
    buffers: bit-identical outputs (the plan is a function of the shapes only; partials are merged in index
    order)."""
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ids, order = wl.selection(w)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    q, ks, vs = wl.make_query(w, "cuda")
    z = wl.make_logits(w, "cuda", n_rows=16)
    runs = []
    for _ in range(2):
        cache = ad.Cache(ctx, total)
        ctx.assemble(cache, ids, order)
        o = ctx.query_attn(cache, 0, total, q, ks, vs, total)
        items = [(0, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q)) for n_ctx in (total, total // 2, 100)]
        ctx.query_attn_batched([cache], 0, items)
        h = ctx.probe_entropy(z)
        s = ctx.rank_shots(0, q)
        torch.cuda.synchronize()
        runs.append((cache.k.clone(), cache.v.clone(), cache.slot_pos.clone(), o.clone(),
                     [it[6].clone() for it in items], h.clone(), s.clone()))
    a, b = runs
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16))
    assert torch.equal(a[1].view(torch.int16), b[1].view(torch.int16))
    assert torch.equal(a[2], b[2])
    assert torch.equal(a[3].view(torch.int16), b[3].view(torch.int16))
    for x, y in zip(a[4], b[4]):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))
    assert torch.equal(a[5].view(torch.int32), b[5].view(torch.int32))
    assert torch.equal(a[6].view(torch.int32), b[6].view(torch.int32))
    ctx.close()


def test_batch_tables_kept_for_the_next_layer_give_the_same_bits(ad):
    """A batched attention call whose inputs equal the previous call's (the next layer of a model) reuses the tables
    in device memory; every such result must be bit-identical to what a fresh context computes for that layer alone,
    for assembled caches and for the zero-copy form, and anything that changes the batch must drop the tables."""
    w = wl.WORKLOADS["llama8b_sweep"]
    L = 3
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=L)
    lists = []
    for qi in range(3):
        ids, order = wl.selection(w, query=qi)
        lists.append((ids[:20 + 5 * qi], np.argsort(np.argsort(order[:20 + 5 * qi])).astype(np.int32)))
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in lists]
    g = torch.Generator(device="cuda")
    g.manual_seed(321)

    def make_items(n_ctx_of):
        its = []
        for li, n_ctx, t_q in n_ctx_of:
            q = torch.randn(t_q, w.n_q_heads, w.head_dim, device="cuda", generator=g).bfloat16()
            ks = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
            vs = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
            its.append((li, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q)))
        return its

    specs = [(0, totals[0], 64), (0, totals[0] // 2, 64), (1, totals[1], 7), (2, totals[2], 1), (2, 0, 3)]
    items = make_items(specs)

    def fresh(layer, its, zero_copy):
        """The same batch on a context that has seen nothing else."""
        c2 = ad.Context.for_workload(w, n_layers=L)
        c2.pool_register(k_pool, v_pool, off)
        outs = [(li, n, q, ks, vs, qp, torch.empty_like(q)) for (li, n, q, ks, vs, qp, _) in its]
        if zero_copy:
            c2.query_attn_pool_batched(layer, ([l[0] for l in lists], [l[1] for l in lists]), outs)
        else:
            cs = [ad.Cache(c2, t, with_index=False) for t in totals]
            c2.assemble_batched(cs, [l[0] for l in lists], [l[1] for l in lists])
            c2.query_attn_batched(cs, layer, outs)
        torch.cuda.synchronize()
        res = [o[6].clone() for o in outs]
        c2.close()
        return res

    def same(its, ref):
        torch.cuda.synchronize()
        return all(torch.equal(a[6].view(torch.int16), b.view(torch.int16)) for a, b in zip(its, ref))

    ctx = ad.Context.for_workload(w, n_layers=L)
    ctx.pool_register(k_pool, v_pool, off)
    caches = [ad.Cache(ctx, t, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [l[0] for l in lists], [l[1] for l in lists])
    packed_lists = ctx.pack_shot_lists([l[0] for l in lists], [l[1] for l in lists])
    for zero_copy in (False, True):
        call = (lambda layer, its: ctx.query_attn_pool_batched(layer, packed_lists, its)) if zero_copy else \
               (lambda layer, its: ctx.query_attn_batched(caches, layer, its))
        packed = ctx.pack_attn_items(items)
        for layer in (0, 1, 2, 1):                          # layers 1, 2, 1 reuse the tables of the first call
            call(layer, packed)
            assert same(items, fresh(layer, items, zero_copy)), (zero_copy, layer)
        # another split count, another batch, another single call in between: each drops the tables
        ctx.set_attn_splits(3)
        call(2, packed)
        ctx.set_attn_splits(0)
        call(2, packed)
        assert same(items, fresh(2, items, zero_copy))
        items2 = make_items([(1, totals[1] - 5, 64), (0, totals[0], 64)])
        call(1, items2)
        assert same(items2, fresh(1, items2, zero_copy))
        call(1, packed)
        assert same(items, fresh(1, items, zero_copy))
        q1, ks1, vs1 = items[0][2], items[0][3], items[0][4]
        if zero_copy:
            ctx.query_attn_pool(0, lists[2][0], lists[2][1], q1, ks1, vs1, totals[2])   # rewrites the slot tables
        else:
            ctx.query_attn(caches[1], 0, totals[1], q1, ks1, vs1, totals[1])
        call(0, packed)
        assert same(items, fresh(0, items, zero_copy))
        ctx.pool_register(k_pool, v_pool, off)              # a new registration drops them too
        call(2, packed)
        assert same(items, fresh(2, items, zero_copy))
    ctx.close()


def test_streamed_tile_loads_give_the_same_bits(ad):
    """A batch whose items have few rows per kv head and contexts of their own reads its K/V tiles with the
    non-temporal cache policy; one more item on a cache that is already in the batch switches the launch back to the
    default policy.  The policy is not arithmetic: with the split length pinned, the items the two batches share
    must come out bit-identical."""
    w = wl.WORKLOADS["llama8b_sweep"]
    k_pool, v_pool, off = wl.make_pool(w, "cuda", n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    lists = []
    for qi in range(2):
        ids, order = wl.selection(w, query=qi)
        lists.append((ids[:30 + 9 * qi], np.argsort(np.argsort(order[:30 + 9 * qi])).astype(np.int32)))
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in lists]
    caches = [ad.Cache(ctx, t, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [l[0] for l in lists], [l[1] for l in lists])
    g = torch.Generator(device="cuda")
    g.manual_seed(2718)
    rows_limit = 128 // (w.n_q_heads // w.n_kv_heads)  # query tokens that still make a streaming launch

    def item(ci, n_ctx, t_q):
        q = torch.randn(t_q, w.n_q_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        ks = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        vs = torch.randn(t_q, w.n_kv_heads, w.head_dim, device="cuda", generator=g).bfloat16()
        return (ci, n_ctx, q, ks, vs, n_ctx, torch.empty_like(q))

    shared = [item(0, totals[0], 1), item(1, totals[1] - 37, rows_limit)]
    extra = item(0, totals[0] // 2, 3)
    ctx.set_attn_splits(3)  # the longest item is the same in both batches, so every shared item gets the same splits
    ctx.query_attn_batched(caches, 0, shared)
    torch.cuda.synchronize()
    streamed = [it[6].clone() for it in shared]
    for it in shared:
        it[6].zero_()
    ctx.query_attn_batched(caches, 0, shared + [extra])
    torch.cuda.synchronize()
    for a, it in zip(streamed, shared):
        assert torch.isfinite(a.float()).all() and float(a.float().abs().max()) > 0
        assert torch.equal(a.view(torch.int16), it[6].view(torch.int16))
    # the single call of such a problem streams too; it runs another instantiation (its rows are rotated by a launch
    # of their own), so it agrees to rounding, not bit for bit
    _, n_ctx, q, ks, vs, qp, _ = shared[1]
    ctx.set_attn_splits(0)
    one = ctx.query_attn(caches[1], 0, n_ctx, q, ks, vs, qp)
    torch.cuda.synchronize()
    ref = streamed[1].float()
    assert float((one.float() - ref).abs().max()) <= 2.0 ** -6 * max(1.0, float(ref.abs().max()))
    ctx.close()
