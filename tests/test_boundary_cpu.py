"""Boundary checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and its host-only logic (schedule, status strings, argument checks that
precede any device call) behaves as documented."""
import ctypes
import os
import re

import pytest

from oracle import cacheblend_oracle as O
from workloads.configs import WORKLOADS, ModelShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cacheblend.h")
LIB = os.path.join(ROOT, "paper_2405_16444_amd", "libcacheblend.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2405_16444_amd import build
        build.build()
    import torch  # noqa: F401  (the binding loads torch's HIP runtime first; do the same here)
    return ctypes.CDLL(LIB)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cb_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert {"cb_realign_rope", "cb_fuse_layer", "cb_fuse_prefill", "cb_create", "cb_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2405_16444_amd import binding
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert callable(getattr(binding, n))


def test_schedule_matches_oracle_on_every_workload():
    import paper_2405_16444_amd as P
    for w in WORKLOADS.values():
        for flat in (False, True):
            got = P.cb_default_schedule(w.model.n_layers, w.n_ctx, w.ratio, w.ratio_first, flat)
            ref = O.default_schedule(w.model.n_layers, w.n_ctx, w.ratio, w.ratio_first,
                                     "flat" if flat else "gradual")
            assert got == ref, w.name
    for r in (0.0, 0.05, 0.3, 1.0):
        assert P.cb_default_schedule(7, 1001, r) == O.default_schedule(7, 1001, r)


def test_status_strings_and_host_side_rejections(lib):
    import paper_2405_16444_amd as P
    from paper_2405_16444_amd.binding import CacheBlendError
    assert P.cb_strerror(0) == "ok" and "workspace" in P.cb_strerror(-3)
    with pytest.raises(CacheBlendError) as e:
        P.cb_default_schedule(0, 10, 0.1)
    assert e.value.status == -1
    with pytest.raises(CacheBlendError) as e:
        P.cb_default_schedule(3, 10, 1.5)
    assert e.value.status == -1
    # geometry checks come before any device call, so they work without a GPU
    bad = ModelShape(2, 256, 4, 2, 96, 688, 1e-5, 1e4, "f32")
    with pytest.raises(CacheBlendError) as e:
        P.cb_create(bad, 64)
    assert e.value.status == -4
    with pytest.raises(CacheBlendError) as e:
        P.cb_create(ModelShape(2, 256, 5, 2, 64, 688, 1e-5, 1e4, "f32"), 64)
    assert e.value.status == -4
    with pytest.raises(CacheBlendError) as e:
        P.cb_create(ModelShape(0, 256, 4, 2, 64, 688, 1e-5, 1e4, "f32"), 64)
    assert e.value.status == -1
    from paper_2405_16444_amd.binding import _ModelDesc
    desc, handle = _ModelDesc(2, 256, 4, 2, 64, 688, 1e-5, 1e4, 0, 7), ctypes.c_void_p()   # no such rotary order
    assert lib.cb_create(ctypes.byref(desc), 64, ctypes.byref(handle)) == -1 and not handle.value
    lib.cb_layer_workspace_bytes.restype = ctypes.c_size_t
    assert lib.cb_layer_workspace_bytes(None, 10) == 0


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2405_16444_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f
    src = open(os.path.join(ROOT, "oracle", "cacheblend_oracle.py")).read()
    assert "paper_2405_16444_amd" not in src and "ctypes" not in src


def test_loading_controller_matches_oracle():
    """Host arithmetic of Sec. 5.1 through the C ABI against the oracle's definitions."""
    import itertools
    import paper_2405_16444_amd as P
    from oracle import cacheblend_oracle as O
    for r, pf in itertools.product([0.0, 0.05, 0.15, 1.0], [0.5, 20.0, 3000.0]):
        assert P.cb_recompute_delay(r, pf) == O.recompute_delay(r, pf)
    for kv, n, bw in itertools.product([4096.0, 16384.0, 131072.0], [1, 3136, 32896], [4.8e9, 64e9]):
        assert P.cb_load_delay(kv, n, bw) == O.load_delay(kv, n, bw)
    assert P.cb_load_delay(1.0, 1.0, 0.0) == float("inf")
    for pf, ld, rmin in itertools.product([1.0, 20.0, 46.7], [0.5, 4.0, 16.0, 100.0], [0.0, 0.15, 0.3]):
        assert P.cb_pick_recompute_ratio(pf, ld, rmin) == O.pick_recompute_ratio(pf, ld, rmin)
    cases = [(3.0, [0.5, 2.5, 16.0], [9.0, 3.0, 1.0]), (20.0, [0.5, 2.5, 16.0], [9.0, 3.0, 1.0]),
             (0.1, [0.5, 2.5, 16.0], [9.0, 3.0, 1.0]), (3.0, [1.0, 1.0], [2.0, 2.0]), (1.0, [], [])]
    for t, loads, costs in cases:
        assert P.cb_pick_storage_device(t, loads, costs) == O.pick_storage_device(t, loads, costs)
