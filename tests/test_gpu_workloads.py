"""GPU parity at the sizes of the workload table."""
import numpy as np
import pytest

from oracle import mavg_oracle as O
from paper_2110_00625_amd import kavg, synth
from paper_2110_00625_amd.configs import TINY, META_ONLY
from tests.util import bf16_plane_bits, flat_error, matmul_in_float32, replica_error, worst_error

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def test_tiny_workload_all_rounds():
    """Tiny: P=4, K=4, B=32, MLP 3072-64-10, fp32, 20 meta rounds, free running."""
    torch = _torch()
    w = TINY
    data = synth.make_workload_inputs(w)
    g = kavg.MAvg(w.P, w.K, w.lr, w.mu, w.dims, w.B, kavg.KAVG_FP32, index_seed=w.seeds["index"])
    g.set_data(torch.from_numpy(data["X32"]).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(data["w0"])
    o = O.MAvgOracle(w.P, w.K, w.lr, w.mu, w.dims, w.B, index_seed=w.seeds["index"])
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    worst = 0.0
    for r in range(w.rounds):
        g.local_steps()
        o.local_steps()
        g.meta_update()
        o.meta_update()
        e = worst_error(g.params(), o.params(), w.dims)
        worst = max(worst, e)
        assert e < 1e-4, "round %d: %.3g" % (r, e)
    assert np.array_equal(g.indices(), o.indices())
    first, last = o.losses()[0].mean(), None
    assert np.max(np.abs(g.losses() - o.losses())) < 1e-3
    print("tiny: worst relative error over %d rounds = %.3g" % (w.rounds, worst))
    g.close()


def test_meta_only_workload_full_size_200_passes():
    """P=64 replicas of an 11.2M-parameter fp32 vector, 200 fused passes; the oracle's
    meta step is elementwise, so the full vector is compared (not a sample)."""
    torch = _torch()
    w = META_ONLY
    n, P = w.flat_n, w.P
    inp = synth.make_meta_only_inputs(P, n, seed=w.seeds["data"])
    stride = (n + 63) // 64 * 64
    wt = torch.from_numpy(inp["w_tilde"]).cuda()
    v = torch.from_numpy(inp["v"]).cuda()
    reps = torch.empty((P, stride), device="cuda")
    reps[:, :n] = torch.from_numpy(inp["replicas"]).cuda()
    wo, vo = O.meta_step(inp["w_tilde"].astype(np.float64), inp["v"].astype(np.float64),
                         inp["replicas"].astype(np.float64), w.mu)
    v1 = vo.copy()
    kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
    torch.cuda.synchronize()
    assert flat_error(wt.cpu().numpy(), wo) < 1e-6
    assert flat_error(v.cpu().numpy(), vo) < 1e-5
    for k in range(2, w.rounds + 1):
        kavg.kavg_meta_update_flat(wt, v, reps, w.mu)
        # the oracle's later passes: all replicas equal w~ (they were just rebroadcast)
        a = wo.copy()                       # mean of P copies of w~
        vo = w.mu * vo + (a - wo)
        wo = wo + vo
    torch.cuda.synchronize()
    got = wt.cpu().numpy()
    assert flat_error(got, wo) < 1e-4
    closed = inp["w_tilde"].astype(np.float64) + v1 * (1 - w.mu ** w.rounds) / (1 - w.mu)
    assert flat_error(got, closed) < 1e-4
    assert np.array_equal(reps[P - 1, :n].cpu().numpy(), got)


# ---------------------------------------------------------------------------
# bf16 workloads at their full shapes (P, K, B, layer widths, N as benchmarked), every learner
# walked by the oracle.  Tolerance: 2e-2 on every tensor of the global model after a meta round.
#
# Two mixed-precision runs that differ only in accumulation order and width (fp32 on the matrix
# cores, float64 in the oracle) do not stay together for ever: now and then a bf16 rounding of an
# activation falls the other way, which flips ReLU masks one layer on, and block momentum carries
# every such difference forward.  What is asserted is therefore
#   * free running from w~_1 over the horizon where the tolerance holds with margin (the first 10
#     of the 50 rounds of cifar_mlp; one whole round -- K steps of all P learners plus the meta
#     step -- of the two big workloads), and
#   * single rounds from a shared state at points spread over the whole run (cifar_mlp: the GPU
#     runs all 50 rounds on its own; at the listed rounds the oracle is set to the GPU's global
#     model, momentum buffer and round counter and both take that round).
# ---------------------------------------------------------------------------
import functools  # noqa: E402

from paper_2110_00625_amd.configs import CIFAR_MLP, NOISY_WIDE, LARGE, WORKLOADS, num_params  # noqa: E402

TOL_BF16 = 2e-2
HOST_CORES = 16            # the GPU machine's CPU share


def _oracle_local_steps(o, learners=None):
    """The oracle's K local steps with its learners walked by up to HOST_CORES threads (they are
    independent between meta steps) and the BLAS pool narrowed so that the two do not oversubscribe."""
    from threadpoolctl import threadpool_limits
    n = o.P if learners is None else len(learners)
    workers = max(1, min(n, HOST_CORES))
    with threadpool_limits(limits=max(1, HOST_CORES // workers)):
        o.local_steps(learners=learners, workers=workers)


@functools.lru_cache(maxsize=1)
def _inputs(name, N):
    return synth.make_workload_inputs(WORKLOADS[name], N=N)


def _bf16_pair(w, N, K=None, P=None):
    torch = _torch()
    K = w.K if K is None else K
    P = w.P if P is None else P
    data = _inputs(w.name, N)
    g = kavg.MAvg(P, K, w.lr, w.mu, w.dims, w.B, kavg.KAVG_BF16, index_seed=w.seeds["index"])
    g.set_data(torch.from_numpy(data["Xbits"].view(np.int16)).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(data["w0"])
    o = O.MAvgOracle(P, K, w.lr, w.mu, w.dims, w.B, bf16=True, index_seed=w.seeds["index"])
    o.set_data(data["X32"], data["y"])
    o.set_params(data["w0"])
    return g, o


def test_cifar_mlp_free_running_first_10_rounds():
    """P=16, K=8, B=128, MLP 3072-1024-1024-10, bf16 operands, N=50000: every learner, global model
    compared after each of the first 10 meta rounds, free running from w~_1 (no re-sync)."""
    w = CIFAR_MLP
    g, o = _bf16_pair(w, w.N)
    for r in range(10):
        g.local_steps()
        _oracle_local_steps(o)
        assert np.array_equal(g.indices(), o.indices())
        if r == 0:
            e = max(replica_error(g.replica(j), o.replica(j), w.dims) for j in range(w.P))
            print("cifar_mlp round 0: worst replica after the K local steps %.3g" % e)
            assert e < TOL_BF16
            assert np.max(np.abs(g.losses() - o.losses()) / np.maximum(o.losses(), 1.0)) < 1e-2
        g.meta_update()
        o.meta_update()
        e = worst_error(g.params(), o.params(), w.dims)
        print("cifar_mlp free-running round %d: max relative error %.3g (momentum buffer %.3g)" % (
            r, e, flat_error(g.momentum(), o.momentum())))
        assert e < TOL_BF16, "global model after round %d: %.3g" % (r, e)
    g.close()


def test_cifar_mlp_single_rounds_spread_over_all_50():
    """The GPU runs all 50 meta rounds on its own.  At six of them the oracle is set to the GPU's
    state before the round (global model, momentum buffer, round counter: the whole state of
    Algorithm 1 between rounds) and both take the round: K local steps of the 16 learners plus the
    meta step, late in training as well as at its start."""
    w = CIFAR_MLP
    g, o = _bf16_pair(w, w.N)
    checked = (0, 9, 19, 29, 39, 49)
    for r in range(w.rounds):
        if r in checked:
            o.set_state(g.params(), g.momentum(), g.round())
            assert g.round() == r
        g.local_steps()
        g.meta_update()
        if r in checked:
            _oracle_local_steps(o)
            assert np.array_equal(g.indices(), o.indices())
            o.meta_update()
            e = worst_error(g.params(), o.params(), w.dims)
            ev = flat_error(g.momentum(), o.momentum())
            print("cifar_mlp round %d from a shared state: model %.3g, momentum buffer %.3g, mean loss %.4f" % (
                r, e, ev, float(o.losses().mean())))
            assert e < TOL_BF16 and ev < 5e-2
    assert g.round() == w.rounds
    g.close()


LARGE_DIVERGES = (
    "large (lr = 0.2, 1000 classes, B = 256) starts violently -- the minibatch loss climbs from 7.7 to 30-110 in "
    "its first four steps before it settles -- and in that phase single ReLU masks that fall the other way under "
    "fp32 instead of float64 accumulation move weight rows by several per cent; the learners never re-converge "
    "within K = 32.  A CPU run of the same reading that only accumulates in fp32 leaves the oracle exactly as "
    "fast (test_large_leaves_the_oracle_no_faster_than_a_cpu_fp32_twin), so the 2e-2 of a whole free-running "
    "round is out of reach of any fp32-accumulating implementation on this workload (measured: 0.37)")


@pytest.mark.parametrize("w", [NOISY_WIDE, pytest.param(LARGE, marks=pytest.mark.xfail(reason=LARGE_DIVERGES, strict=False))],
                         ids=["noisy_wide", "large"])
def test_big_workloads_one_full_round_every_learner(w):
    """Full P, K, B, layer widths and N; one whole meta round of Algorithm 1 from w~_1: K local
    steps of every learner, then the meta step; global model within tolerance, tensor by tensor."""
    g, o = _bf16_pair(w, w.N)
    g.local_steps()
    _oracle_local_steps(o)
    assert np.array_equal(g.indices(), o.indices())
    reps = [replica_error(g.replica(j), o.replica(j), w.dims) for j in range(w.P)]
    print("%s: single replicas after K=%d local steps: median %.3g, worst %.3g" % (
        w.name, w.K, float(np.median(reps)), max(reps)))
    gl, ol = g.losses(), o.losses()
    assert np.all(np.isfinite(gl))
    print("%s: minibatch losses, worst relative difference %.3g" % (
        w.name, float(np.max(np.abs(gl - ol) / np.maximum(ol, 1.0)))))
    g.meta_update()
    o.meta_update()
    print("%s: global model after the meta step, per tensor:" % w.name)
    e = worst_error(g.params(), o.params(), w.dims, verbose=True)
    print("%s: worst %.3g, momentum buffer %.3g" % (w.name, e, flat_error(g.momentum(), o.momentum())))
    assert e < TOL_BF16, "%s: global model after one round: %.3g" % (w.name, e)
    if w is NOISY_WIDE:
        # the same round with the stored replicas refreshed once (deferred updates, m = K), against the same oracle
        g2, _unused = _bf16_pair(w, w.N)
        g2.set_refresh(w.K)
        g2.local_steps()
        assert np.array_equal(g2.indices(), o.indices())
        g2.meta_update()
        e2 = worst_error(g2.params(), o.params(), w.dims)
        print("%s with deferred updates (m = %d): worst %.3g; against the plain path %.3g" % (
            w.name, w.K, e2, worst_error(g2.params(), g.params(), w.dims)))
        assert e2 < TOL_BF16
        g2.close()
    wt, v = g.params(), g.momentum()
    assert np.array_equal(g.replica(0), wt) and np.array_equal(g.replica(w.P - 1), wt)      # rebroadcast
    # first round from v = 0: w~_2 = w~_1 + v_2 holds to one fp32 rounding
    assert np.max(np.abs((wt - _inputs(w.name, w.N)["w0"]) - v)) <= 2e-7 * np.max(np.abs(wt))
    g.close()


@pytest.mark.parametrize("w,N,sample", [(NOISY_WIDE, 20000, (5, 31)), (LARGE, 20000, (0, 7))],
                         ids=["noisy_wide", "large"])
def test_big_workloads_first_step_is_tight(w, N, sample):
    """One local step from identical state at the full launch shapes: nothing but accumulation order
    and fp32 master rounding separates the two sides."""
    g, o = _bf16_pair(w, N, K=1)
    g.local_steps()
    o.local_steps(learners=list(sample))
    for j in sample:
        e = replica_error(g.replica(j), o.replica(j), w.dims)
        print("%s learner %d after one local step: max relative error %.3g" % (w.name, j, e))
        assert e < 5e-3          # a single flipped ReLU mask already costs about 2e-3 here
        assert abs(g.losses()[0, j] - o.losses()[0, j]) < 1e-3 * max(1.0, o.losses()[0, j])
    g.close()


def _fp32_twin_gradient(wv, dims, Xb, yb, bf16=False):
    """The oracle's minibatch gradient with one change: every matrix product is numpy's float32
    product of the same (bf16-rounded) operands instead of the float64 one."""
    q, mm = O.rne_bf16, matmul_in_float32
    Ws, bs = O.unpack(wv, dims)
    Wq = [q(W) for W in Ws]
    L = len(Ws)
    Zs, As = [], [Xb]
    for l in range(L):
        Zs.append(mm(As[-1], Wq[l].T) + bs[l])
        if l < L - 1:
            As.append(q(np.maximum(Zs[-1], 0.0)))
    loss, dZL = O.softmax_cross_entropy(Zs[-1], yb)
    dZ = q(dZL)
    pieces = [None] * L
    for l in range(L - 1, -1, -1):
        pieces[l] = np.concatenate([mm(dZ.T, As[l]).ravel(), dZ.sum(axis=0)])
        if l > 0:
            dZ = q(mm(dZ, Wq[l]) * (Zs[l - 1] > 0.0))
    return float(loss.mean()), np.concatenate(pieces)


def test_large_leaves_the_oracle_no_faster_than_a_cpu_fp32_twin(monkeypatch):
    """The first 8 local steps of two learners of `large`, free running from w~_1, three ways: the
    oracle (float64 products), a CPU twin that differs from it only in accumulating the products
    in fp32, and the GPU.  Step by step the GPU is about as far from the oracle as the twin is
    (both correct implementations of the same reading); neither stays within 2e-2."""
    w, N, learners, steps = LARGE, 20000, [0, 1], 8
    g, o = _bf16_pair(w, N, K=1)
    _, twin = _bf16_pair(w, N, K=1)
    _.close()
    worst_gpu = worst_twin = 0.0
    for k in range(steps):
        g.local_steps()                                   # K = 1 and no meta step: step k of the round
        _oracle_local_steps(o, learners)
        with monkeypatch.context() as m:
            m.setattr(O, "minibatch_gradient", _fp32_twin_gradient)
            _oracle_local_steps(twin, learners)
        for j in learners:
            eg = replica_error(g.replica(j), o.replica(j), w.dims)
            et = replica_error(twin.replica(j), o.replica(j), w.dims)
            print("large step %d learner %d: GPU vs oracle %.3g, fp32 twin vs oracle %.3g, loss %.2f" % (
                k, j, eg, et, o.losses()[0, j]))
            assert eg < 2.0 * et + 1e-2, "step %d learner %d: GPU %.3g, twin %.3g" % (k, j, eg, et)
            worst_gpu, worst_twin = max(worst_gpu, eg), max(worst_twin, et)
    assert worst_twin > 2e-2, "the fp32 twin stayed within tolerance: the divergence would be the GPU's own"
    g.close()


# Launch shapes that only large problems select (128x128 and 64x128 forward / backward-data tiles,
# the 128x64 backward-data tile, the streaming 64x128 update and the 128x128 update of batches
# above 128), on extents that are multiples of none of them: widths 3080 / 4104, batches 70, 60
# and 200, 24 classes.
@pytest.mark.parametrize("P,B,sample", [(32, 70, (0, 31)), (16, 60, (3, 15)), (4, 200, (0, 3)), (8, 200, (0, 7))],
                         ids=["tiles128x128", "tiles64x128", "bwd128x64", "update128x128"])
def test_large_tile_shapes_on_ragged_extents(P, B, sample):
    torch = _torch()
    dims, N, lr = (3080, 4104, 4104, 24), 1500, 0.05
    data = synth.make_dataset(N, dims[0], dims[-1], bf16=True, seed_data=77, seed_teacher=78, teacher_hidden=32)
    w0 = synth.he_normal_params(dims, 79)
    g = kavg.MAvg(P, 1, lr, 0.9, dims, B, kavg.KAVG_BF16, index_seed=80)
    g.set_data(torch.from_numpy(data["Xbits"].view(np.int16)).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(w0)
    o = O.MAvgOracle(P, 1, lr, 0.9, dims, B, bf16=True, index_seed=80)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    g.local_steps()
    o.local_steps(learners=list(sample))
    for j in sample:
        assert np.array_equal(g.indices()[j], o.indices()[j])
        e = replica_error(g.replica(j), o.replica(j), dims)
        print("ragged large tiles P=%d B=%d learner %d: %.3g" % (P, B, j, e))
        assert e < 2e-3
        assert abs(g.losses()[0, j] - o.losses()[0, j]) < 1e-3 * max(1.0, o.losses()[0, j])
    # untouched learners of the oracle still hold w0; on the GPU every learner has moved
    assert not np.array_equal(g.replica((sample[0] + 1) % P), w0)
    g.close()


# The 256x128 forward tile whose slices are brought in by loader wavefronts through a ring of LDS buffers
# (batches that are multiples of 256, contraction lengths that are multiples of 64, at least 192 tiles):
# the shortest contractions it takes (two and three slices: fewer than the ring is deep), a ragged last
# column tile (3000 = 23 x 128 + 56), gathered rows in layer 1, two row tiles per learner.
@pytest.mark.parametrize("P,B,dims", [(8, 256, (128, 3000, 24)), (8, 256, (192, 3000, 24)), (4, 512, (448, 3000, 3008, 16))],
                         ids=["two_slices", "three_slices", "two_row_tiles"])
def test_ring_forward_tile_on_short_and_ragged_extents(P, B, dims):
    torch = _torch()
    N, lr = 1200, 0.05
    data = synth.make_dataset(N, dims[0], dims[-1], bf16=True, seed_data=91, seed_teacher=92, teacher_hidden=32)
    w0 = synth.he_normal_params(dims, 93)
    g = kavg.MAvg(P, 1, lr, 0.9, dims, B, kavg.KAVG_BF16, index_seed=94)
    g.set_data(torch.from_numpy(data["Xbits"].view(np.int16)).cuda(), torch.from_numpy(data["y"]).cuda())
    g.set_params(w0)
    o = O.MAvgOracle(P, 1, lr, 0.9, dims, B, bf16=True, index_seed=94)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    g.local_steps()
    sample = (0, P - 1)
    o.local_steps(learners=list(sample))
    for j in sample:
        e = replica_error(g.replica(j), o.replica(j), dims)
        print("ring forward P=%d B=%d dims=%s learner %d: %.3g" % (P, B, dims, j, e))
        assert e < 2e-3
        assert abs(g.losses()[0, j] - o.losses()[0, j]) < 1e-3 * max(1.0, o.losses()[0, j])
    g.close()


@pytest.mark.parametrize("w", [CIFAR_MLP, NOISY_WIDE, LARGE], ids=lambda w: w.name)
def test_meta_step_at_workload_size_with_shadows(w):
    torch = _torch()
    n, P = num_params(w.dims), w.P
    stride = (n + 63) // 64 * 64
    rng = np.random.default_rng(w.seeds["data"])
    base = rng.standard_normal(n, dtype=np.float32) * np.float32(0.05)
    v0 = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
    wt = torch.from_numpy(base).cuda()
    v = torch.from_numpy(v0).cuda()
    reps = torch.empty((P, stride), device="cuda")
    acc = np.zeros(n, dtype=np.float64)
    for j in range(P):                                  # replica by replica: the oracle's sum in the same order
        rj = base + rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
        reps[j, :n] = torch.from_numpy(rj).cuda()
        acc += rj
    sh = torch.zeros((P, stride), dtype=torch.int16, device="cuda")
    kavg.kavg_meta_update_flat(wt, v, reps, w.mu, shadow=sh)
    torch.cuda.synchronize()
    a = acc * (1.0 / P)
    vo = w.mu * v0.astype(np.float64) + (a - base)
    wo = base + vo
    got = wt.cpu().numpy()
    assert flat_error(got, wo) < 1e-6
    assert flat_error(v.cpu().numpy(), vo) < 1e-5
    for j in (0, P - 1):
        assert np.array_equal(reps[j, :n].cpu().numpy(), got)
        # bf16 copies: the library's documented storage rule (stated in tests/util.py)
        assert np.array_equal(sh[j, :n].cpu().numpy().view(np.uint16), bf16_plane_bits(got))
