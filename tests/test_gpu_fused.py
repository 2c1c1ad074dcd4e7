"""Small fp32 models: all K local steps of Algorithm 1 in one launch (kavg_fused) against the oracle
and against the launch-per-layer path of the same library."""
import numpy as np
import pytest

from paper_2110_00625_amd import kavg
from tests.test_gpu_small import TOL_FP32, _pair, _run_and_compare, _torch
from tests.util import flat_error

pytestmark = pytest.mark.gpu

CASES = [
    # P, K, B, dims
    (4, 4, 32, (3072, 64, 10)),        # the shape of the smallest workload: 16 workgroups of 192 columns per learner
    (3, 3, 19, (200, 40, 7)),          # ragged everywhere: last chunk 8 columns wide, odd batch, 40 units
    (2, 2, 64, (64, 64, 16)),          # one workgroup per learner, every limit reached
    (5, 3, 7, (132, 8, 3)),            # last chunk 4 columns wide, fewer rows than a matrix-instruction block
    (1, 5, 33, (1000, 33, 2)),         # a single learner, batch one over half the tile
    (2, 3, 64, (4000, 64, 16)),        # 21 chunks of 192 columns (the last one 160 wide), full batch
    (3, 2, 50, (1600, 48, 9)),         # 13 chunks of 128 columns (the last one 64 wide)
]


@pytest.mark.parametrize("P,K,B,dims", CASES, ids=[str(c[3]) for c in CASES])
def test_fused_steps_match_the_oracle(P, K, B, dims):
    g, o = _pair(P, K, 0.05, 0.9, dims, B, False, 91)
    assert g.fused
    _run_and_compare(g, o, dims, 4, TOL_FP32, "fused %s" % (dims,))


@pytest.mark.parametrize("P,K,B,dims", CASES[:3], ids=[str(c[3]) for c in CASES[:3]])
def test_fused_steps_match_the_launch_per_layer_path(P, K, B, dims):
    g, _ = _pair(P, K, 0.05, 0.9, dims, B, False, 92)
    h, _ = _pair(P, K, 0.05, 0.9, dims, B, False, 92)
    h.set_fused(False)
    assert g.fused and not h.fused
    for r in range(3):
        g.local_steps()
        h.local_steps()
        for j in range(P):
            assert flat_error(g.replica(j), h.replica(j)) < 2e-6, (r, j)
        assert np.max(np.abs(g.losses() - h.losses())) < 1e-5
        g.meta_update()
        h.meta_update()
    assert flat_error(g.params(), h.params()) < 2e-6


def test_fused_steps_with_caller_indices():
    torch = _torch()
    P, K, B, dims = 3, 3, 20, (264, 48, 10)
    g, o = _pair(P, K, 0.05, 0.9, dims, B, False, 93)
    assert g.fused
    rng = np.random.default_rng(5)
    for r in range(3):
        idx = rng.integers(0, 600, size=(P, K, B)).astype(np.int32)
        g.set_indices(torch.from_numpy(idx).cuda())
        o.set_indices(idx)
        g.local_steps()
        o.local_steps()
        assert np.array_equal(g.indices(), idx)
        for j in range(P):
            assert flat_error(g.replica(j), o.replica(j)) < TOL_FP32
        g.meta_update()
        o.meta_update()
    assert flat_error(g.params(), o.params()) < TOL_FP32


def test_a_wait_that_gives_up_ends_the_launch_and_is_reported():
    """With a limit of one poll a workgroup does not wait for the others: the launch still runs to its end
    (nothing hangs), a wait that found its data missing is reported once as KAVG_EDEVICE, and the context
    works again after the parameters have been installed anew."""
    P, K, B, dims = 4, 4, 32, (3072, 64, 10)
    g, o = _pair(P, K, 0.05, 0.9, dims, B, False, 94)
    w0 = g.params().copy()
    g.set_wait_limit(1)
    reported = 0
    for _ in range(3):
        g.local_steps()
        try:
            g.losses()
        except kavg.KavgError as e:
            assert e.code == kavg.KAVG_EDEVICE
            reported += 1
    print("launches with a wait that gave up: %d of 3" % reported)
    g.set_wait_limit(1 << 20)
    g.set_state(w0, np.zeros_like(w0), 0)                     # parameters, momentum and the index stream as at the start
    _run_and_compare(g, o, dims, 2, TOL_FP32, "after a wait limit of one poll")


def test_fused_path_is_taken_only_where_it_fits():
    _torch()
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (64, 65, 10), 8, kavg.KAVG_FP32).fused          # hidden layer too wide
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (64, 32, 17), 8, kavg.KAVG_FP32).fused          # too many classes
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (64, 32, 10), 65, kavg.KAVG_FP32).fused         # batch too large
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (66, 32, 10), 8, kavg.KAVG_FP32).fused          # d_0 not a multiple of 4
    assert not kavg.MAvg(17, 2, 0.1, 0.5, (3072, 32, 10), 8, kavg.KAVG_FP32).fused       # 17 x 16 workgroups: more than compute units
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (64, 32, 32, 10), 8, kavg.KAVG_FP32).fused      # two hidden layers
    assert not kavg.MAvg(2, 33, 0.1, 0.5, (64, 32, 10), 32, kavg.KAVG_FP32).fused        # K*B beyond the index table
    assert not kavg.MAvg(2, 2, 0.1, 0.5, (64, 32, 10), 8, kavg.KAVG_BF16).fused          # mixed precision
    g = kavg.MAvg(2, 2, 0.1, 0.5, (64, 32, 10), 8, kavg.KAVG_FP32)
    assert g.fused
    g.set_learner_momentum(0.9)
    assert not g.fused
    g.set_learner_momentum(0.0)
    assert g.fused
