"""Host-side checks of the C boundary that need no GPU: the library loads,
exports every declared symbol, sizes workspaces, and rejects bad arguments
before touching the device."""
import ctypes
import os
import re
import subprocess

import numpy as np

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


def test_split_storage_contract_on_the_host(tmp_path):
    """The library keeps a learner's fp32 parameter as two 16-bit planes (csrc/split.h).  Contract,
    stated here and checked on the header's own functions compiled for the host:
      hi   = top 16 bits of (pattern + 0x8000): the nearest bf16 value, exact ties away from zero;
      lo   = low 16 bits of the pattern;
      join(hi, lo) returns the pattern, whatever it is.
    hi differs from the nearest-even conversion only on exact ties (lo == 0x8000 with an even kept
    mantissa), where it is one bf16 unit further from zero."""
    src = tmp_path / "shim.cpp"
    src.write_text(
        '#include "%s"\n'
        'extern "C" void split_all(const unsigned* in, unsigned* hi, unsigned* lo, unsigned* back, long n) {\n'
        '  for (long i = 0; i < n; ++i) { hi[i] = kavg::split_hi(in[i]); lo[i] = kavg::split_lo(in[i]);\n'
        '                                 back[i] = kavg::split_join(hi[i], lo[i]); } }\n'
        % os.path.join(ROOT, "paper_2110_00625_amd", "csrc", "split.h"))
    so = tmp_path / "shim.so"
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", str(src), "-o", str(so)], check=True)
    shim = ctypes.CDLL(str(so))
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 1 << 32, size=400000, dtype=np.uint64).astype(np.uint32)
    bits &= np.uint32(0xBFFFFFFF)                                  # finite values
    keep = np.arange(0x3F00, 0x4100, dtype=np.uint32)
    ties = (keep << np.uint32(16)) | np.uint32(0x8000)
    near = np.concatenate([ties - 1, ties + 1, ties | np.uint32(0x80000000), keep << np.uint32(16),
                           (keep << np.uint32(16)) | np.uint32(0xFFFF)])
    bits = np.concatenate([bits, ties, near, np.array([0, 0x80000000, 0x00800000, 0x0000FFFF], dtype=np.uint32)])
    hi, lo, back = (np.empty_like(bits) for _ in range(3))
    vp = ctypes.c_void_p
    shim.split_all.argtypes = [vp, vp, vp, vp, ctypes.c_long]
    shim.split_all(bits.ctypes.data, hi.ctypes.data, lo.ctypes.data, back.ctypes.data, bits.size)
    assert np.array_equal(back, bits)
    assert np.array_equal(hi, ((bits.astype(np.uint64) + 0x8000) >> 16).astype(np.uint32) & np.uint32(0xFFFF))
    assert np.array_equal(lo, bits & np.uint32(0xFFFF))
    # against the nearest-even conversion (the oracle's): equal except on ties with an even kept mantissa
    import torch
    rne = torch.from_numpy(bits.view(np.float32).copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    differ = hi.astype(np.uint16) != rne
    is_tie_even = ((bits & np.uint32(0xFFFF)) == 0x8000) & (((bits >> np.uint32(16)) & 1) == 0)
    assert np.array_equal(differ, is_tie_even)
    assert np.all(hi[differ].astype(np.int64) - rne[differ].astype(np.int64) == 1)


def test_static_workspace_init_rejects_oversize_before_any_device_call(lib):
    """kavg_init_static sizes the configuration against the library's own block first: a
    configuration that does not fit is refused with KAVG_ENOMEM (no device needed to say so),
    a bad shape with KAVG_EINVAL."""
    ctx = ctypes.c_void_p()
    big = (3072, 1024, 1024, 10)
    assert kavg.kavg_workspace_bytes(16, 8, 128, big, 1) > kavg.STATIC_WORKSPACE_BYTES
    rc = lib.kavg_init_static(ctypes.byref(ctx), 16, 8, 0.1, 0.9, 3, kavg._dims_array(big), 128, 1, 0, None)
    assert rc == kavg.KAVG_ENOMEM and not ctx.value
    assert b"kavg_init" in lib.kavg_last_error(None)
    rc = lib.kavg_init_static(ctypes.byref(ctx), 0, 8, 0.1, 0.9, 3, kavg._dims_array(big), 128, 1, 0, None)
    assert rc == kavg.KAVG_EINVAL and not ctx.value
    text = open(os.path.join(ROOT, "include", "kavg.h")).read()
    assert "#define KAVG_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)" in text and kavg.STATIC_WORKSPACE_BYTES == 32 << 20


def test_image_generator_is_seeded_padded_and_on_the_bf16_grid():
    from paper_2110_00625_amd import synth
    a = synth.make_image_dataset(40, 6, 5, 3, 8, 4, seed_data=5, seed_texture=6)
    b = synth.make_image_dataset(40, 6, 5, 3, 8, 4, seed_data=5, seed_texture=6)
    assert np.array_equal(a["Xbits"], b["Xbits"]) and np.array_equal(a["y"], b["y"])
    X = a["X32"].reshape(40, 6, 5, 8)
    assert np.all(X[..., 3:] == 0) and np.any(X[..., :3] != 0)
    assert np.array_equal(X.view(np.uint32) & 0xFFFF, np.zeros(X.shape, dtype=np.uint32))        # exactly representable in bf16
    assert np.array_equal((X.view(np.uint32) >> 16).astype(np.uint16), a["Xbits"].reshape(X.shape))
    assert a["y"].min() >= 0 and a["y"].max() < 4
    w0 = synth.he_normal_conv_params((8, 16), (16, 4), 7)
    assert w0.size == 16 * 72 + 16 + 4 * 16 + 4 and np.all(w0[16 * 72:16 * 72 + 16] == 0)


def test_multiply_shift_division_is_exact_over_its_stated_range(tmp_path):
    """csrc/fastdiv.h replaces n / d by (n * m) >> s in the index arithmetic of the convolution loaders.  Its
    own functions, compiled for the host, against integer division: every divisor below 2^14, with the
    numerators where a wrong constant shows first (multiples of d and their neighbours up to 2^30) and
    random ones."""
    src = tmp_path / "fd.cpp"
    src.write_text(
        '#include "%s"\n'
        'extern "C" long check(const unsigned* n, long count, unsigned dmax) {\n'
        '  long bad = 0;\n'
        '  for (unsigned d = 1; d < dmax; ++d) { unsigned m; int s; kavg::fastdiv_make(d, &m, &s);\n'
        '    for (long i = 0; i < count; ++i) bad += kavg::fastdiv(n[i], m, s) != n[i] / d;\n'
        '    const unsigned top = (1u << 30) - 1; const unsigned q = top / d;\n'
        '    for (unsigned k = 0; k < 64 && k <= q; ++k) { const unsigned a = (q - k) * d;\n'
        '      bad += kavg::fastdiv(a, m, s) != a / d; if (a) bad += kavg::fastdiv(a - 1, m, s) != (a - 1) / d;\n'
        '      if (a + d - 1 <= top) bad += kavg::fastdiv(a + d - 1, m, s) != (a + d - 1) / d; }\n'
        '    bad += kavg::fastdiv(top, m, s) != top / d; }\n'
        '  return bad; }\n'
        % os.path.join(ROOT, "paper_2110_00625_amd", "csrc", "fastdiv.h"))
    so = tmp_path / "fd.so"
    subprocess.run(["g++", "-O2", "-shared", "-fPIC", str(src), "-o", str(so)], check=True)
    lib = ctypes.CDLL(str(so))
    lib.check.restype = ctypes.c_long
    lib.check.argtypes = [ctypes.c_void_p, ctypes.c_long, ctypes.c_uint]
    rng = np.random.default_rng(11)
    n = np.concatenate([rng.integers(0, 1 << 30, size=3000, dtype=np.uint64), np.arange(0, 70000, 7, dtype=np.uint64)]).astype(np.uint32)
    assert lib.check(n.ctypes.data, n.size, 1 << 14) == 0
