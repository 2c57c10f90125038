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
