"""The entropy entry point that allocates nothing (adapshot_probe_entropy_static) against the ordinary one
(adapshot_probe_entropy), through the C ABI: two calls in a row, the second with a smaller input, so that
what the first call left in the shared static scratch array would show."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2605_03644_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ad():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_03644_amd import binding
    binding.load_library()
    return binding


def _call(ad, ctx, name, z, out):
    """One raw C-ABI call of an entropy entry point on torch's current stream."""
    f = getattr(ctx.lib, name)
    rows, vocab = z.shape
    return f(ctx._h, ctypes.c_void_p(z.data_ptr()), ctypes.c_int64(z.stride(0)), ctypes.c_int32(rows),
             ctypes.c_int32(vocab), ctypes.c_void_p(out.data_ptr()),
             ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


def test_static_entropy_matches_the_allocating_entry_point(ad, oracle_mod):
    w = wl.WORKLOADS["llama8b_1layer"]
    ctx = ad.Context.for_workload(w)
    big = wl.make_logits(w, "cuda", n_rows=128)                 # 128 x 128256: 2048 partials
    small = wl.make_logits(w, "cuda", n_rows=5, variant=3)[:, :4099].contiguous()   # 5 x 4099, ragged tail
    for z in (big, small):                                     # the second call is the smaller one
        rows = z.shape[0]
        want = torch.full((rows + 2,), -7.0, device="cuda")
        got = torch.full((rows + 2,), -7.0, device="cuda")
        assert _call(ad, ctx, "adapshot_probe_entropy", z, want) == ad.OK
        assert _call(ad, ctx, "adapshot_probe_entropy_static", z, got) == ad.OK, ctx.last_error()
        torch.cuda.synchronize()
        w_np, g_np = want.cpu().numpy(), got.cpu().numpy()
        assert (g_np[rows:] == -7.0).all()                      # nothing written past the rows
        assert np.abs(g_np[:rows].astype(np.float64) - w_np[:rows]).max() <= 1e-4
        # and against the oracle directly, to the entropy bar
        ref = oracle_mod.entropy(z.cpu().numpy())
        assert np.abs(g_np[:rows].astype(np.float64) - ref).max() <= 1e-4
    # the big one once more after the small one: the array is reused, not stale
    got = torch.empty(128, device="cuda")
    want = torch.empty(128, device="cuda")
    assert _call(ad, ctx, "adapshot_probe_entropy_static", big, got) == ad.OK
    assert _call(ad, ctx, "adapshot_probe_entropy", big, want) == ad.OK
    torch.cuda.synchronize()
    assert np.abs(got.cpu().numpy().astype(np.float64) - want.cpu().numpy()).max() <= 1e-4
    ctx.close()


def test_static_entropy_rejects_what_does_not_fit_and_empty_is_a_no_op(ad):
    w = wl.WORKLOADS["tiny_fp32"]
    ctx = ad.Context.for_workload(w)
    rows = 65536 + 1                                            # one chunk per row: one partial too many
    z = torch.zeros(rows, 8, device="cuda")
    out = torch.full((rows,), 3.0, device="cuda")
    st = _call(ad, ctx, "adapshot_probe_entropy_static", z, out)
    assert st == ad.ECAPACITY and "static scratch" in ctx.last_error()
    torch.cuda.synchronize()
    assert float(out.min()) == 3.0 and float(out.max()) == 3.0  # nothing was launched
    assert _call(ad, ctx, "adapshot_probe_entropy_static", z[:65536], out) == ad.OK   # exactly the limit fits
    torch.cuda.synchronize()
    assert np.allclose(out[:65536].cpu().numpy(), np.log(8.0), atol=1e-5) and float(out[65536]) == 3.0
    assert _call(ad, ctx, "adapshot_probe_entropy_static", z[:0], out) == ad.OK
    ctx.close()
