"""The entry point that allocates nothing (kavg_init_static): a context that works in the library's
own device block must give exactly what a context on a caller workspace gives, call after call."""
import numpy as np
import pytest

from paper_2110_00625_amd import kavg, synth

pytestmark = pytest.mark.gpu


def _run(static, P, K, B, dims, bf16, seed, rounds=2):
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    data = synth.make_dataset(400, dims[0], dims[-1], bf16=bf16, seed_data=seed, seed_teacher=seed + 1,
                              teacher_hidden=32)
    w0 = synth.he_normal_params(dims, seed + 2)
    g = kavg.MAvg(P, K, 0.05, 0.9, dims, B, kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32, index_seed=seed + 3,
                  static_workspace=static)
    X = torch.from_numpy(data["Xbits"].view(np.int16) if bf16 else data["X32"]).cuda()
    g.set_data(X, torch.from_numpy(data["y"]).cuda())
    g.set_params(w0)
    out = []
    for _ in range(rounds):
        g.local_steps()
        reps = [g.replica(j) for j in range(P)]
        g.meta_update()
        out.append((g.indices(), g.losses(), reps, g.params(), g.momentum()))
    g.close()
    return out


def _same(a, b):
    for ra, rb in zip(a, b):
        assert np.array_equal(ra[0], rb[0]) and np.array_equal(ra[1], rb[1])
        for x, y in zip(ra[2], rb[2]):
            assert np.array_equal(x, y)
        assert np.array_equal(ra[3], rb[3]) and np.array_equal(ra[4], rb[4])


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_static_workspace_context_matches_caller_workspace_context(bf16):
    """Two contexts in a row in the library's block, the second smaller than the first (it finds
    the first one's leftovers there), each against the same run on a caller workspace.  The fp32
    shape has a long first contraction, so its forward pass goes through the partial-tile scratch
    piece of the workspace."""
    big = (1000, 136, 72, 10) if not bf16 else (264, 200, 136, 10)
    small = (200, 72, 10) if not bf16 else (136, 72, 24)
    first = _run(True, 5, 2, 40, big, bf16, 11)
    second = _run(True, 2, 3, 9, small, bf16, 21)
    _same(first, _run(False, 5, 2, 40, big, bf16, 11))
    _same(second, _run(False, 2, 3, 9, small, bf16, 21))


def test_static_workspace_is_one_context_per_device_and_has_a_size_limit():
    import torch
    assert torch.cuda.is_available()
    a = kavg.MAvg(2, 2, 0.1, 0.5, (40, 24, 6), 8, static_workspace=True)
    with pytest.raises(kavg.KavgError) as ei:
        kavg.MAvg(2, 2, 0.1, 0.5, (40, 24, 6), 8, static_workspace=True)
    assert ei.value.code == kavg.KAVG_ESTATE
    a.close()
    b = kavg.MAvg(2, 2, 0.1, 0.5, (40, 24, 6), 8, static_workspace=True)     # free again after destroy
    b.close()
    with pytest.raises(kavg.KavgError) as ei:
        kavg.MAvg(16, 8, 0.1, 0.9, (3072, 1024, 1024, 10), 128, kavg.KAVG_BF16, static_workspace=True)
    assert ei.value.code == kavg.KAVG_ENOMEM
