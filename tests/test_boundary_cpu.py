"""Host-side checks of the C boundary that need no GPU: the library loads,
exports every declared symbol, sizes workspaces, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2110_00625_amd import kavg
from paper_2110_00625_amd.configs import WORKLOADS, num_params

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kavg.LIB_PATH):
        from paper_2110_00625_amd import build
        build.build(verbose=False)
    return kavg.load_library()


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "kavg.h")).read()
    declared = set(re.findall(r"\b(kavg_[a-z_]+)\s*\(", text))
    declared.discard("kavg_workspace_bytes(...)")
    assert declared == set(kavg.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_num_params_matches_the_layout(lib):
    for w in WORKLOADS.values():
        if w.dims:
            assert kavg.kavg_num_params(w.dims) == num_params(w.dims)
    assert kavg.kavg_num_params((3072, 4096, 4096, 1000)) == 33_465_320
    assert kavg.kavg_num_params((3072, 64, 10)) == 197_322


def test_workspace_holds_state_and_replicas(lib):
    for w in WORKLOADS.values():
        if not w.dims:
            continue
        n = num_params(w.dims)
        need = kavg.kavg_workspace_bytes(w.P, w.K, w.B, w.dims, w.dtype)
        # global model + momentum + P replicas, 4 bytes each (in bf16 mode a replica is two 16-bit planes)
        floor = (w.P + 2) * n * 4
        assert need >= floor
        assert need < floor * 1.5 + (64 << 20)
    assert kavg.kavg_workspace_bytes(0, 1, 1, (8, 8), 0) == 0
    assert kavg.kavg_workspace_bytes(1, 1, 1, (8, 5, 3), 1) == 0      # bf16 wants multiples of 8
    assert kavg.kavg_workspace_bytes(1, 1, 1, (8, 16, 3), 1) > 0


@pytest.mark.parametrize("kw, code", [
    (dict(P=0), kavg.KAVG_EINVAL), (dict(K=0), kavg.KAVG_EINVAL), (dict(B=0), kavg.KAVG_EINVAL),
    (dict(B=70000), kavg.KAVG_EINVAL), (dict(lr=-0.1), kavg.KAVG_EINVAL), (dict(mu=1.0), kavg.KAVG_EINVAL),
    (dict(mu=-0.1), kavg.KAVG_EINVAL), (dict(dtype=7), kavg.KAVG_EINVAL), (dict(dims=(8, 0, 2)), kavg.KAVG_EINVAL),
    (dict(dims=(8, 12, 2), dtype=1), kavg.KAVG_EINVAL), (dict(ws=0), kavg.KAVG_EINVAL),
    (dict(ws=4096 + 8), kavg.KAVG_EINVAL), (dict(nbytes=1024), kavg.KAVG_ENOMEM),
])
def test_init_rejects_bad_arguments_without_touching_the_device(lib, kw, code):
    a = dict(P=2, K=2, lr=0.1, mu=0.9, dims=(8, 8, 2), B=4, dtype=0, ws=4096, nbytes=1 << 30)
    a.update(kw)
    ctx = ctypes.c_void_p()
    rc = lib.kavg_init(ctypes.byref(ctx), a["P"], a["K"], a["lr"], a["mu"], len(a["dims"]) - 1,
                       kavg._dims_array(a["dims"]), a["B"], a["dtype"], 0, a["ws"], a["nbytes"], None)
    assert rc == code
    assert not ctx.value
    assert len(lib.kavg_last_error(None)) > 0


def test_flat_meta_update_rejects_bad_arguments(lib):
    f = lib.kavg_meta_update_flat
    assert f(None, 4096, 4096, 8, None, 0, 2, 8, 0.5, None) == kavg.KAVG_EINVAL
    assert f(4096, 4096, 4096, 4, None, 0, 2, 8, 0.5, None) == kavg.KAVG_EINVAL     # stride < n
    assert f(4096, 4096, 4096, 8, None, 0, 0, 8, 0.5, None) == kavg.KAVG_EINVAL     # P < 1
    assert f(4096, 4096, 4096, 8, None, 0, 2, 8, 1.0, None) == kavg.KAVG_EINVAL     # mu = 1
    assert f(4096, 4096, 4096, 8, None, 0, 2, 0, 0.5, None) == kavg.KAVG_EINVAL     # n = 0


def test_null_context_is_an_error(lib):
    for name in ("kavg_local_steps", "kavg_meta_update", "kavg_destroy"):
        assert getattr(lib, name)(None) == kavg.KAVG_EINVAL
