"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad model descriptions before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2605_03644_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2605_03644_amd import build
        build.build()
    return binding.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "adapshot.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adapshot_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    from paper_2605_03644_amd import binding
    names = _declared_symbols()
    assert "adapshot_assemble" in names and "adapshot_query_attn" in names and "adapshot_probe_entropy" in names
    assert "adapshot_pool_register" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in adapshot.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_build_returns_the_library_path(monkeypatch, tmp_path):
    """build() hands back the path it wrote (the driver's build step checks that the file exists) and
    raises with the compiler's output when hipcc fails; hipcc itself is stubbed out here."""
    import subprocess
    from paper_2605_03644_amd import build
    seen = {}

    class Done:
        def __init__(self, rc):
            self.returncode, self.stdout = rc, "warning: something\nerror: boom\n"

    def fake_run(cmd, **kw):
        seen["cmd"] = cmd
        return Done(seen["rc"])

    monkeypatch.setattr(subprocess, "run", fake_run)
    seen["rc"] = 0
    target = str(tmp_path / "lib.so")
    assert build.build(out=target) == target
    assert seen["cmd"][-2:] == ["-o", target] and "--offload-arch=gfx950" in seen["cmd"]
    assert all(any(c.endswith(s) for c in seen["cmd"]) for s in build.SOURCES)
    i = seen["cmd"].index("-packed-fp32-ops")
    assert seen["cmd"][i - 3:i] == ["-Xclang", "-target-feature", "-Xclang"]
    assert build.build() == build.LIB
    seen["rc"] = 1
    with pytest.raises(RuntimeError, match="boom"):
        build.build(out=target)


def test_version_and_null_context(lib):
    assert b"adapshot" in lib.adapshot_version()
    assert lib.adapshot_last_error(None) == b"null context"
    lib.adapshot_destroy(None)


@pytest.mark.parametrize("field,value", [("n_layers", 0), ("n_q_heads", 5), ("head_dim", 6), ("head_dim", 512),
                                         ("dtype", 7), ("key_state", 3), ("rope_theta", 0.5), ("max_position", -1)])
def test_create_rejects_bad_descriptions_on_host(lib, field, value):
    from paper_2605_03644_amd import binding
    d = binding.ModelDesc(1, 4, 2, 64, 1.0e4, binding.F32, binding.KEYS_UNROTATED, 0)
    setattr(d, field, value)
    h = ctypes.c_void_p(1234)
    assert lib.adapshot_create(ctypes.byref(d), ctypes.byref(h)) == binding.EINVAL
    assert not h.value
    assert lib.adapshot_create(None, ctypes.byref(h)) == binding.EINVAL


def test_pick_shots_is_host_logic_and_matches_the_case_study(lib, oracle_mod):
    """The stopping rule needs no device: called with a null context on the case study's printed entropies
    (tests/golden/case_study_probe_rounds.txt) and on random candidates against the oracle's rule."""
    import numpy as np
    i32, f32 = ctypes.c_int32, ctypes.c_float

    def pick(h, k, tau):
        h = np.ascontiguousarray(h, np.float32)
        k = np.ascontiguousarray(k, np.int32)
        out = i32(7)
        st = lib.adapshot_pick_shots(None, h.ctypes.data_as(ctypes.c_void_p), k.ctypes.data_as(ctypes.c_void_p),
                                     i32(h.size), f32(tau), ctypes.byref(out))
        assert st == 0
        return out.value

    assert pick([0.6731, 0.7023, 0.7044, 0.6671], [4, 8, 12, 16], 0.65) == -1
    assert pick([0.6862, 0.6884, 0.6232, 0.6450], [20, 24, 28, 32], 0.65) == 28
    assert pick([], [], 0.65) == -1
    assert pick([float("nan"), 0.2], [4, 8], 0.65) == 8
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 9))
        h = rng.uniform(0.4, 0.9, n).astype(np.float32)
        k = rng.permutation(64)[:n].astype(np.int32)
        tau = float(rng.uniform(0.4, 0.9))
        assert pick(h, k, tau) == oracle_mod.pick_shots(h.astype(np.float64), k, float(np.float32(tau)))
    out = i32(0)
    assert lib.adapshot_pick_shots(None, None, None, i32(3), f32(0.5), ctypes.byref(out)) != 0


def test_top_k_is_host_logic(lib):
    """Best first, lower shot id first among equal scores, errors for NaN scores and k out of range."""
    import numpy as np
    i32 = ctypes.c_int32

    def top_k(scores, k):
        sc = np.ascontiguousarray(scores, np.float32)
        out = np.full(max(k, 1), -7, np.int32)
        st = lib.adapshot_top_k(None, sc.ctypes.data_as(ctypes.c_void_p), i32(sc.size), i32(k),
                                out.ctypes.data_as(ctypes.c_void_p))
        return st, out[:k]

    st, ids = top_k([0.1, 0.5, 0.3, 0.5, 0.2], 3)
    assert st == 0 and ids.tolist() == [1, 3, 2]
    st, ids = top_k([0.25] * 6, 4)
    assert st == 0 and ids.tolist() == [0, 1, 2, 3]
    st, ids = top_k([0.3, 0.1], 0)
    assert st == 0 and ids.size == 0
    rng = np.random.default_rng(5)
    for _ in range(20):
        n = int(rng.integers(1, 200))
        sc = rng.integers(0, 50, n).astype(np.float32) / 50.0       # many ties
        k = int(rng.integers(0, n + 1))
        st, ids = top_k(sc, k)
        want = sorted(range(n), key=lambda i: (-sc[i], i))[:k]
        assert st == 0 and ids.tolist() == want
    assert top_k([0.1, float("nan")], 1)[0] != 0
    assert top_k([0.1, 0.2], 3)[0] != 0
    assert lib.adapshot_top_k(None, None, i32(2), i32(1), None) != 0
    # the device entry point refuses a null context before touching anything
    assert lib.adapshot_rank_shots(None, i32(0), None, i32(1), ctypes.c_int64(0), None, None) != 0


def test_attn_split_plan_properties(lib):
    """The attention split planner is host logic: checked here without a GPU.  Whatever the shape, the splits cover
    the context exactly once in pieces of one length that is a multiple of the 64-key tile, at most 64 of them; the
    two workloads the kernel was sized on get the plans their measurements were made with."""
    import numpy as np
    from paper_2605_03644_amd import binding as ad
    # the headline workload: 32 q / 8 kv heads, 128 query tokens (16 units), ~27k context on 256 compute units:
    # 15 splits of 29 tiles share one round with the 16 self workgroups
    assert ad.attn_split_plan(32, 8, 128, ad.BF16, 256, 128, 27189) == (15, 29 * 64)
    # 64 q / 8 kv heads, 256 query tokens (64 units), 126617 slots: one context split per compute unit
    assert ad.attn_split_plan(64, 8, 128, ad.BF16, 256, 256, 126617) == (4, 495 * 64)
    assert ad.attn_split_plan(32, 8, 128, ad.BF16, 256, 128, 0) == (0, 64)
    rng = np.random.default_rng(3)
    shapes = [(32, 8, 128, ad.BF16), (28, 4, 128, ad.BF16), (4, 2, 64, ad.F32), (8, 8, 128, ad.F32), (64, 8, 128, ad.BF16)]
    for _ in range(400):
        hq, hkv, d, dt = shapes[rng.integers(len(shapes))]
        n_cu = int(rng.choice([1, 8, 64, 104, 256, 304]))
        t_q = int(rng.choice([1, 2, 7, 64, 128, 300, 4096]))
        n_ctx = int(rng.choice([1, 63, 64, 65, 1000, 27189, 126617, 2_000_000]))
        ns, kps = ad.attn_split_plan(hq, hkv, d, dt, n_cu, t_q, n_ctx)
        assert 1 <= ns <= 64 and kps % 64 == 0 and kps >= 64
        assert ns * kps >= n_ctx and (ns - 1) * kps < n_ctx, (hq, hkv, d, n_cu, t_q, n_ctx, ns, kps)
    # more compute units never mean fewer, longer splits for the same problem beyond one round
    assert ad.attn_split_plan(32, 8, 128, ad.BF16, 64, 128, 27189)[0] <= ad.attn_split_plan(32, 8, 128, ad.BF16, 256, 128, 27189)[0]
    with pytest.raises(ad.AdapshotError):
        ad.attn_split_plan(32, 7, 128, ad.BF16, 256, 128, 100)      # heads do not divide
    with pytest.raises(ad.AdapshotError):
        ad.attn_split_plan(32, 8, 128, ad.BF16, 0, 128, 100)
    with pytest.raises(ad.AdapshotError):
        ad.attn_split_plan(32, 8, 128, ad.BF16, 256, 128, -1)
