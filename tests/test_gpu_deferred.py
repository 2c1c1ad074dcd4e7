"""Deferred weight updates (kavg_set_refresh): the stored replicas are refreshed every m local steps,
products in between use the pending rank-B terms.  Same iterates as Algorithm 1 in exact arithmetic."""
import numpy as np
import pytest

from oracle import mavg_oracle as O
from paper_2110_00625_amd import kavg, synth
from tests.util import flat_error, replica_error, worst_error

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _setup(P, K, B, dims, seed, m, N=600, lr=0.05, mu=0.9):
    torch = _torch()
    data = synth.make_dataset(N, dims[0], dims[-1], bf16=True, seed_data=seed, seed_teacher=seed + 1, teacher_hidden=32)
    w0 = synth.he_normal_params(dims, seed + 2)
    g = kavg.MAvg(P, K, lr, mu, dims, B, kavg.KAVG_BF16, index_seed=seed + 3)
    g.set_data(torch.from_numpy(data["Xbits"].view(np.int16)).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(w0)
    if m > 1:
        g.set_refresh(m)
    o = O.MAvgOracle(P, K, lr, mu, dims, B, bf16=True, index_seed=seed + 3)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    return g, o


CASES = [
    # P, K, B, dims, m
    (3, 4, 40, (264, 200, 136, 10), 4),        # head kernels for the last layer, refresh once per round
    (3, 5, 40, (264, 200, 136, 10), 2),        # K not a multiple of m: the last segment is shorter
    (2, 3, 70, (136, 328, 150), 3),            # generic last layer (150 classes), ragged batch
    (2, 4, 16, (72, 264, 8, 24), 4),           # a hidden layer narrower than any tile, 24 classes
    (2, 3, 9, (40, 24), 3),                    # single generic layer
    (2, 3, 9, (40, 3), 3),                     # single layer with head kernels: nothing is deferred
]


@pytest.mark.parametrize("P,K,B,dims,m", CASES, ids=[str(c[3]) + "-m%d" % c[4] for c in CASES])
def test_deferred_updates_match_the_oracle(P, K, B, dims, m):
    g, o = _setup(P, K, B, dims, 51, m)
    for r in range(3):
        g.local_steps()
        o.local_steps()
        assert np.array_equal(g.indices(), o.indices())
        for j in range(P):
            e = replica_error(g.replica(j), o.replica(j), dims)
            assert e < TOL_BF16, "replica %d after the local steps of round %d: %.3g" % (j, r, e)
        gl, ol = g.losses(), o.losses()
        assert np.max(np.abs(gl - ol) / np.maximum(np.abs(ol), 1e-3)) < 50 * TOL_BF16
        g.meta_update()
        o.meta_update()
        e = replica_error(g.params(), o.params(), dims)
        assert e < TOL_BF16, "global model after round %d: %.3g" % (r, e)
        assert np.array_equal(g.replica(P - 1), g.params())
    g.close()


def test_deferred_and_immediate_paths_agree_and_differ_only_in_rounding():
    dims, P, K, B = (264, 200, 136, 24), 3, 4, 40
    a, _ = _setup(P, K, B, dims, 61, 1)
    b, _ = _setup(P, K, B, dims, 61, 4)
    for _r in range(2):
        for g in (a, b):
            g.local_steps()
            g.meta_update()
    e = replica_error(b.params(), a.params(), dims)
    print("deferred vs immediate after two rounds: %.3g" % e)
    assert 0.0 < e < 5e-3
    # the biases of deferred layers are stepped with the same sums in the same order: first round, first step equal
    a.close()
    b.close()


def test_refresh_period_one_is_the_plain_path_bit_for_bit_and_can_be_switched():
    dims, P, K, B = (136, 72, 10), 2, 3, 16
    a, _ = _setup(P, K, B, dims, 71, 1)
    b, _ = _setup(P, K, B, dims, 71, 3)
    b.set_refresh(1)                                   # back to the plain path before any step
    for g in (a, b):
        g.local_steps()
        g.meta_update()
    assert np.array_equal(a.params(), b.params())
    b.set_refresh(3)                                   # and on again in the middle of a run
    b.local_steps()
    b.meta_update()
    a.local_steps()
    a.meta_update()
    assert replica_error(b.params(), a.params(), dims) < 5e-3
    a.close()
    b.close()


def test_two_calls_without_a_meta_step_do_not_share_weights():
    """kavg_local_steps twice in a row is 2K local steps; in the second call the stored replicas differ
    from learner to learner from the start (they were refreshed at the end of the first call), so the
    first segment must read every learner's own weights."""
    dims, P, K, B = (136, 200, 24), 3, 2, 24
    g, _ = _setup(P, K, B, dims, 81, 2)
    o = None
    data = synth.make_dataset(600, dims[0], dims[-1], bf16=True, seed_data=81, seed_teacher=82, teacher_hidden=32)
    o = O.MAvgOracle(P, 2 * K, 0.05, 0.9, dims, B, bf16=True, index_seed=84)          # one call of 2K steps
    o.set_data(data["X32"], data["y"])
    o.set_params(synth.he_normal_params(dims, 83))
    g.local_steps()
    g.local_steps()
    o.local_steps()
    for j in range(P):
        assert replica_error(g.replica(j), o.replica(j), dims) < TOL_BF16
    # the replicas have drifted apart, so sharing learner 0's weights would have been visible
    assert replica_error(g.replica(1), g.replica(0), dims) > 1e-3
    g.close()


def test_refresh_argument_errors():
    torch = _torch()
    g = kavg.MAvg(2, 3, 0.1, 0.5, (40, 24, 6), 8, kavg.KAVG_BF16)
    for bad in (0, 4):
        with pytest.raises(kavg.KavgError) as ei:
            g.set_refresh(bad)
        assert ei.value.code == kavg.KAVG_EINVAL
    f = kavg.MAvg(2, 3, 0.1, 0.5, (40, 24, 6), 8, kavg.KAVG_FP32)
    with pytest.raises(kavg.KavgError) as ei:
        f.set_refresh(2)
    assert ei.value.code == kavg.KAVG_EINVAL
    g.set_learner_momentum(0.5)
    with pytest.raises(kavg.KavgError) as ei:
        g.set_refresh(2)
    assert ei.value.code == kavg.KAVG_ESTATE
    g.close()
    f.close()


def test_cifar_mlp_one_round_with_deferred_updates():
    """cifar_mlp at full shape with the replicas refreshed once per round (m = K = 8): one whole meta
    round against the oracle, strict per-tensor metric."""
    from paper_2110_00625_amd.configs import CIFAR_MLP as w
    torch = _torch()
    data = synth.make_workload_inputs(w)
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, kavg.KAVG_BF16, index_seed=w.seeds["index"])
    g.set_data(torch.from_numpy(data["Xbits"].view(np.int16)).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(data["w0"])
    g.set_refresh(w.K)
    o = O.MAvgOracle(w.P, w.K, w.lr, w.mu, w.dims, w.B, bf16=True, index_seed=w.seeds["index"])
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    for r in range(2):
        g.local_steps()
        from tests.test_gpu_workloads import _oracle_local_steps
        _oracle_local_steps(o)
        assert np.array_equal(g.indices(), o.indices())
        g.meta_update()
        o.meta_update()
        e = worst_error(g.params(), o.params(), w.dims, verbose=True)
        print("cifar_mlp, deferred updates, round %d: max relative error %.3g" % (r, e))
        assert e < TOL_BF16
    g.close()
