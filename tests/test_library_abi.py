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
