"""GPU parity, small shapes: the HIP path against the CPU oracle, element by
element, on the same seeded inputs.  Shapes span several tiles and ragged
tails in every dimension and finish in seconds on the oracle."""
import numpy as np
import pytest

from oracle import mavg_oracle as O
from paper_2110_00625_amd import kavg, synth
from tests.util import bf16_plane_bits, flat_error, replica_error, worst_error

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4      # max relative error of fp32 parameters after each meta round
TOL_BF16 = 2e-2      # the same for bf16-operand configurations


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _dataset(N, dims, bf16, seed):
    return synth.make_dataset(N, dims[0], dims[-1], bf16=bf16, seed_data=seed, seed_teacher=seed + 1,
                              teacher_hidden=32)


def _to_device(data, bf16):
    torch = _torch()
    if bf16:
        X = torch.from_numpy(data["Xbits"].view(np.int16)).cuda()
    else:
        X = torch.from_numpy(data["X32"]).cuda()
    return X, torch.from_numpy(data["y"]).cuda()


def _pair(P, K, lr, mu, dims, B, bf16, seed, N=600):
    data = _dataset(N, dims, bf16, seed)
    w0 = synth.he_normal_params(dims, seed + 2)
    g = kavg.MAvg(P, K, lr, mu, dims, B, kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32, index_seed=seed + 3)
    X, y = _to_device(data, bf16)
    g.set_data(X, y)
    g.set_params(w0)
    o = O.MAvgOracle(P, K, lr, mu, dims, B, bf16=bf16, index_seed=seed + 3)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    return g, o


def _run_and_compare(g, o, dims, rounds, tol, tag):
    """Small made-up shapes (few learners, batches down to 1): kernel correctness on tile tails.  A
    bias element is a sum over a handful of samples here, so biases are measured on their layer's
    scale (replica_error) for the global model too; the workload tests use the strict per-tensor
    metric."""
    for r in range(rounds):
        g.local_steps()
        o.local_steps()
        assert np.array_equal(g.indices(), o.indices()), "%s: index stream differs in round %d" % (tag, r)
        for j in range(o.P):
            e = replica_error(g.replica(j), o.replica(j), dims)
            assert e < tol, "%s: replica %d after local steps of round %d: %.3g" % (tag, j, r, e)
        gl, ol = g.losses(), o.losses()
        assert np.max(np.abs(gl - ol) / np.maximum(np.abs(ol), 1e-3)) < 50 * tol, "%s: losses" % tag
        g.meta_update()
        o.meta_update()
        e = replica_error(g.params(), o.params(), dims)
        assert e < tol, "%s: global model after round %d: %.3g" % (tag, r, e)
        ev = flat_error(g.momentum(), o.momentum())
        assert ev < 50 * tol, "%s: momentum after round %d: %.3g" % (tag, r, ev)
        for j in (0, o.P - 1):
            assert np.array_equal(g.replica(j), g.params()), "%s: rebroadcast" % tag
    assert g.round() == rounds


# ----------------------------------------------------------------- index stream
@pytest.mark.parametrize("P,K,B,N", [(3, 2, 5, 97), (16, 8, 128, 50000), (2, 3, 64, 200000)])
def test_index_stream_is_bit_exact(P, K, B, N):
    torch = _torch()
    dims = (8, 8, 4)
    g = kavg.MAvg(P, K, 0.0, 0.0, dims, B, kavg.KAVG_FP32, index_seed=4002)
    X = torch.zeros((N, 8), device="cuda")
    y = torch.zeros(N, dtype=torch.int32, device="cuda")
    g.set_data(X, y)
    g.set_params(np.zeros(g.n, dtype=np.float32))
    for call in range(2):                                    # second call: step counter has advanced by K
        g.local_steps()
        got = g.indices()
        for j in range(P):
            for k in range(K):
                want = O.minibatch_indices(4002, j, call * K + k, B, N)
                assert np.array_equal(got[j, k], want)
    g.close()


# ----------------------------------------------------------------- meta step
@pytest.mark.parametrize("P,n,shadow", [(1, 1, False), (3, 1003, False), (64, 4098, False), (5, 777, True),
                                        (16, 40000, True)])
def test_meta_update_flat_matches_oracle(P, n, shadow):
    torch = _torch()
    inp = synth.make_meta_only_inputs(P, n, seed=P * 1000 + n)
    stride = (n + 63) // 64 * 64
    w = torch.from_numpy(inp["w_tilde"]).cuda()
    v = torch.from_numpy(inp["v"]).cuda()
    reps = torch.zeros((P, stride), device="cuda")
    reps[:, :n] = torch.from_numpy(inp["replicas"]).cuda()
    sh = torch.zeros((P, stride), dtype=torch.int16, device="cuda") if shadow else None
    wo, vo, ro = inp["w_tilde"].astype(np.float64), inp["v"].astype(np.float64), inp["replicas"].astype(np.float64)
    for it in range(3):
        kavg.kavg_meta_update_flat(w, v, reps, 0.9, shadow=sh)
        wo, vo = O.meta_step(wo, vo, ro, 0.9)
        ro = np.tile(wo, (P, 1))
        torch.cuda.synchronize()
        assert flat_error(w.cpu().numpy(), wo) < 1e-6
        assert flat_error(v.cpu().numpy(), vo) < 1e-5
        rg = reps.cpu().numpy()
        assert np.array_equal(rg[:, :n], np.tile(w.cpu().numpy(), (P, 1)))
        assert np.all(rg[:, n:] == 0)                                 # padding untouched
        if shadow:
            # the bf16 copies follow the library's documented storage rule (stated in tests/util.py)
            want_bits = bf16_plane_bits(w.cpu().numpy())
            got_bits = sh.cpu().numpy().view(np.uint16)
            assert np.array_equal(got_bits[:, :n], np.tile(want_bits, (P, 1)))


def test_meta_update_flat_unaligned_views_take_the_scalar_path():
    torch = _torch()
    P, n = 4, 1001
    inp = synth.make_meta_only_inputs(P, n, seed=5)
    wbuf = torch.zeros(n + 1, device="cuda")
    vbuf = torch.zeros(n + 1, device="cuda")
    rbuf = torch.zeros((P, n + 3), device="cuda")
    w, v, reps = wbuf[1:], vbuf[1:], rbuf[:, 1:n + 1]
    w.copy_(torch.from_numpy(inp["w_tilde"]))
    v.copy_(torch.from_numpy(inp["v"]))
    reps.copy_(torch.from_numpy(inp["replicas"]))
    kavg.kavg_meta_update_flat(w, v, reps, 0.5)
    torch.cuda.synchronize()
    wo, vo = O.meta_step(inp["w_tilde"].astype(np.float64), inp["v"].astype(np.float64),
                         inp["replicas"].astype(np.float64), 0.5)
    assert flat_error(w.cpu().numpy(), wo) < 1e-6 and flat_error(v.cpu().numpy(), vo) < 1e-5
    assert float(wbuf[0]) == 0.0 and float(rbuf[0, 0]) == 0.0 and float(rbuf[0, n + 1]) == 0.0


# ----------------------------------------------------------------- learner loop, fp32
@pytest.mark.parametrize("P,K,B,dims", [
    (3, 3, 40, (200, 136, 72, 10)),       # ragged in every dimension, three layers
    (2, 2, 7, (33, 5)),                    # single layer (softmax regression)
    (4, 2, 65, (96, 130, 3)),
])
def test_fp32_learner_loop_and_meta_step(P, K, B, dims):
    g, o = _pair(P, K, 0.05, 0.9, dims, B, False, seed=11)
    _run_and_compare(g, o, dims, rounds=3, tol=TOL_FP32, tag="fp32 %s" % (dims,))
    g.close()


# ----------------------------------------------------------------- learner loop, bf16 operands
@pytest.mark.parametrize("P,K,B,dims", [
    (3, 3, 40, (264, 200, 136, 10)),      # ragged tiles in every dimension, B below one row tile
    (2, 2, 150, (136, 328, 150)),          # B spans two row tiles, class count spans two tiles
    (2, 2, 64, (72, 264, 8, 10)),          # the 64-row tile, a hidden layer narrower than any tile
    (2, 2, 9, (40, 3)),                    # single layer
])
def test_bf16_learner_loop_and_meta_step(P, K, B, dims):
    g, o = _pair(P, K, 0.05, 0.9, dims, B, True, seed=51)
    _run_and_compare(g, o, dims, rounds=3, tol=TOL_BF16, tag="bf16 %s" % (dims,))
    g.close()


def test_bf16_one_step_is_tight():
    """A single local step from identical state: only accumulation order and the fp32
    master rounding separate the two sides, far below the free-running tolerance."""
    dims = (264, 200, 136, 10)
    g, o = _pair(2, 1, 0.05, 0.0, dims, 40, True, seed=61)
    g.local_steps()
    o.local_steps()
    for j in range(2):
        e = replica_error(g.replica(j), o.replica(j), dims)
        assert e < 2e-4, e
    g.close()


def test_lr0_is_bit_exact_on_the_gpu():
    dims = (64, 48, 10)
    g, o = _pair(3, 2, 0.0, 0.9, dims, 16, False, seed=21)
    w0 = g.params()
    for _ in range(2):
        g.local_steps()
        g.meta_update()
    assert np.array_equal(g.params(), w0)
    assert np.array_equal(g.momentum(), np.zeros_like(w0))
    assert np.array_equal(g.replica(2), w0)
    g.close()


def test_two_runs_are_bit_identical():
    dims = (200, 136, 72, 10)
    outs = []
    for _ in range(2):
        g, _o = _pair(3, 3, 0.05, 0.9, dims, 40, False, seed=31)
        for _r in range(2):
            g.local_steps()
            g.meta_update()
        outs.append((g.params(), g.momentum(), g.losses()))
        g.close()
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


def test_caller_supplied_indices_and_range_check():
    torch = _torch()
    dims = (40, 24, 6)
    P, K, B, N = 2, 2, 9, 50
    g, o = _pair(P, K, 0.1, 0.5, dims, B, False, seed=41, N=N)
    idx = np.random.default_rng(0).integers(0, N, size=(P, K, B)).astype(np.int32)
    g.set_indices(torch.from_numpy(idx).cuda())
    o.set_indices(idx)
    _run_and_compare(g, o, dims, rounds=2, tol=TOL_FP32, tag="user idx")
    bad = idx.copy()
    bad[1, 0, 3] = N                                                   # one past the end
    g.set_indices(torch.from_numpy(bad).cuda())
    g.local_steps()
    with pytest.raises(kavg.KavgError) as ei:
        g.params()
    assert ei.value.code == kavg.KAVG_EINVAL
    g.close()


def test_state_errors():
    torch = _torch()
    g = kavg.MAvg(2, 2, 0.1, 0.5, (8, 8, 2), 4)
    with pytest.raises(kavg.KavgError) as ei:
        g.local_steps()
    assert ei.value.code == kavg.KAVG_ESTATE
    g.set_params(np.zeros(g.n, dtype=np.float32))
    with pytest.raises(kavg.KavgError) as ei:
        g.local_steps()                                                # no data yet
    assert ei.value.code == kavg.KAVG_ESTATE
    X = torch.zeros((10, 8), device="cuda")
    ybad = torch.full((10,), 2, dtype=torch.int32, device="cuda")      # class id == d_L
    with pytest.raises(kavg.KavgError) as ei:
        g.set_data(X, ybad)
    assert ei.value.code == kavg.KAVG_EINVAL
    g.close()


# ----------------------------------------------------------------- edge cases
@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("P,K,B,dims", [
    (1, 1, 1, (8, 8, 2)),                  # one learner, one step, one sample
    (1, 3, 2, (16, 3)),                    # single layer, fewer classes than any tile
    (5, 1, 3, (1000, 72, 10)),             # long first contraction (split over workgroups in fp32)
])
def test_degenerate_shapes(bf16, P, K, B, dims):
    g, o = _pair(P, K, 0.05, 0.5, dims, B, bf16, seed=71, N=37)
    _run_and_compare(g, o, dims, rounds=2, tol=TOL_BF16 if bf16 else TOL_FP32, tag="edge %s" % (dims,))
    g.close()


def test_bf16_two_runs_are_bit_identical():
    dims = (264, 200, 136, 10)
    outs = []
    for _ in range(2):
        g, _o = _pair(3, 3, 0.05, 0.9, dims, 40, True, seed=81)
        for _r in range(2):
            g.local_steps()
            g.meta_update()
        outs.append((g.params(), g.momentum(), g.losses(), g.replica(1)))
        g.close()
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
def test_resume_from_saved_state_continues_bit_identically(bf16):
    dims = (72, 40, 6)
    g, o = _pair(3, 2, 0.05, 0.9, dims, 12, bf16, seed=91)
    for _ in range(2):
        g.local_steps()
        g.meta_update()
    w, v, r = g.params(), g.momentum(), g.round()
    g.local_steps()
    g.meta_update()
    want_w, want_v, want_idx = g.params(), g.momentum(), g.indices()
    g.close()
    h, _o = _pair(3, 2, 0.05, 0.9, dims, 12, bf16, seed=91)      # same data, same index seed
    h.set_state(w, v, r)
    assert h.round() == 2
    h.local_steps()
    h.meta_update()
    assert np.array_equal(h.indices(), want_idx)                 # the stream resumes at step round*K
    assert np.array_equal(h.params(), want_w) and np.array_equal(h.momentum(), want_v)
    h.close()


def test_mu_zero_is_plain_averaging():
    """mu = 0: M-AVG reduces to K-AVG (remark after Theorem 1): the new global model is the
    average of the replicas."""
    dims = (40, 24, 6)
    g, o = _pair(4, 2, 0.1, 0.0, dims, 9, False, seed=95)
    g.local_steps()
    reps = np.stack([g.replica(j) for j in range(4)]).astype(np.float64)
    g.meta_update()
    assert flat_error(g.params(), reps.mean(axis=0)) < 1e-6
    g.close()


@pytest.mark.parametrize("dims,fwd_per_step", [((40, 24, 6), 1), ((40, 24, 20), 2)],
                         ids=["head_kernels", "generic_last_layer"])
def test_profile_counts_launches(dims, fwd_per_step):
    # up to 16 classes the last layer's forward runs inside the loss kernel (one forward launch less)
    g, _o = _pair(2, 3, 0.1, 0.5, dims, 9, False, seed=97)
    g.set_fused(False)          # the launch-per-layer path is what is counted (a model this small would run its K steps in one launch)
    g.profile(["forward", "update", "meta", "head"], every=1)
    g.local_steps()
    g.meta_update()
    got = g.profile_read()
    assert got["forward"][1] == 3 * fwd_per_step and got["update"][1] == 3 * fwd_per_step and got["meta"][1] == 1
    assert got["head"][1] == (3 * 2 if fwd_per_step == 1 else 0)
    assert got["backward"][1] == 0 and got["forward"][0] > 0.0
    g.profile(["update"], every=2)
    g.local_steps()
    assert g.profile_read()["update"][1] == (2 if fwd_per_step == 1 else 3)   # every second launch of 3 / 6
    g.profile([])
    g.close()


# ----------------------------------------------------------------- learner-level momentum
@pytest.mark.parametrize("bf16", [False, True], ids=["fp32", "bf16"])
@pytest.mark.parametrize("dims", [(200, 136, 72, 10), (136, 200, 24)], ids=["head_kernels", "generic_last_layer"])
def test_learner_momentum_matches_oracle(bf16, dims):
    P, K, B, lr, mu, beta = 3, 3, 40, 0.02, 0.9, 0.8
    data = _dataset(600, dims, bf16, 101)
    w0 = synth.he_normal_params(dims, 103)
    g = kavg.MAvg(P, K, lr, mu, dims, B, kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32, index_seed=104)
    X, y = _to_device(data, bf16)
    g.set_data(X, y)
    g.set_learner_momentum(beta)
    g.set_params(w0)
    o = O.MAvgOracle(P, K, lr, mu, dims, B, bf16=bf16, index_seed=104, learner_momentum=beta)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    tol = TOL_BF16 if bf16 else TOL_FP32
    for r in range(3):
        g.local_steps()
        o.local_steps()
        for j in range(P):
            assert replica_error(g.replica(j), o.replica(j), dims) < tol
            assert replica_error(g.velocity(j), o.velocity(j), dims) < 10 * tol   # velocities persist across rounds
        g.meta_update()
        o.meta_update()
        assert replica_error(g.params(), o.params(), dims) < tol
    # the momentum run differs from the plain one (the check is not vacuous) ...
    plain = O.MAvgOracle(P, K, lr, mu, dims, B, bf16=bf16, index_seed=104)
    plain.set_data(data["X32"], data["y"])
    plain.set_params(w0)
    plain.local_steps()
    o2 = O.MAvgOracle(P, K, lr, mu, dims, B, bf16=bf16, index_seed=104, learner_momentum=beta)
    o2.set_data(data["X32"], data["y"])
    o2.set_params(w0)
    o2.local_steps()
    assert worst_error(o2.replica(0), plain.replica(0), dims) > 5e-3
    # ... and switching it off returns to Algorithm 1 as printed
    g.set_learner_momentum(0.0)
    g.set_params(w0)
    g.local_steps()
    assert replica_error(g.replica(0), plain.replica(0), dims) < tol
    with pytest.raises(kavg.KavgError) as ei:
        g.velocity(0)
    assert ei.value.code == kavg.KAVG_ESTATE
    g.close()


# ----------------------------------------------------------------- K-AVG vs M-AVG sweep harness
def test_sweep_harness_runs_and_is_consistent_with_the_oracle():
    """The sweep only loops over configurations of the library; check its bookkeeping on a tiny
    grid (non-power-of-two P) and one of its loss curves against the oracle."""
    from paper_2110_00625_amd import sweep
    dims, K, B, lr, rounds, N, seed = (40, 24, 5), 2, 8, 0.05, 4, 300, 7
    out = sweep.sweep([3, 6], [0.0, 0.7], K=K, B=B, lr=lr, rounds=rounds, dims=dims, N=N, seed=seed, quiet=True)
    assert len(out["runs"]) == 4 and all(len(r["curve"]) == rounds for r in out["runs"])
    assert all(np.isfinite(r["final_loss"]) for r in out["runs"])
    assert "| 3 |" in sweep.table(out) and "| 6 |" in sweep.table(out)
    data = synth.make_dataset(N, dims[0], dims[-1], bf16=False, seed_data=seed, seed_teacher=seed + 1, teacher_hidden=64)
    o = O.MAvgOracle(6, K, lr, 0.7, dims, B, index_seed=seed + 3)
    o.set_data(data["X32"], data["y"])
    o.set_params(synth.he_normal_params(dims, seed + 2))
    want = []
    for _ in range(rounds):
        o.local_steps()
        o.meta_update()
        want.append(o.losses().mean())
    got = [r for r in out["runs"] if r["P"] == 6 and r["mu"] == 0.7][0]["curve"]
    assert np.max(np.abs(np.array(got) - np.array(want))) < 1e-4


# ----------------------------------------------------------------- graph replay of the K local steps
GRAPH_CASES = [
    ("fp32-head", (96, 72, 10), False, 3, 3, 20, 0.0),
    ("bf16-head", (264, 200, 136, 10), True, 4, 2, 24, 0.0),
    ("bf16-generic", (136, 72, 40), True, 3, 3, 16, 0.0),
    ("bf16-learner-momentum", (264, 200, 10), True, 3, 2, 24, 0.8),
]


@pytest.mark.parametrize("tag,dims,bf16,P,K,B,beta", GRAPH_CASES, ids=[c[0] for c in GRAPH_CASES])
def test_graph_replay_matches_the_eager_path_bit_for_bit(tag, dims, bf16, P, K, B, beta):
    """The recorded sequence is replayed many times, with the program's own eager work and waits
    between the replays (parameter read-backs, meta steps, a profiled round, a change of data set);
    every round must leave exactly what the eager path leaves."""
    torch = _torch()
    dtype = kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32
    data = _dataset(500, dims, bf16, 31)
    data2 = _dataset(300, dims, bf16, 37)
    w0 = synth.he_normal_params(dims, 33)
    side = torch.cuda.Stream()
    runs = []
    for use_graph in (False, True):
        with torch.cuda.stream(side):
            g = kavg.MAvg(P, K, 0.05, 0.6, dims, B, dtype, index_seed=35)
            X, y = _to_device(data, bf16)
            X2, y2 = _to_device(data2, bf16)
            torch.cuda.synchronize()
            g.set_data(X, y)
            if beta > 0:
                g.set_learner_momentum(beta)
            g.set_params(w0)
            if use_graph:
                g.graph(True)
            trace = []
            for r in range(9):
                if r == 5:
                    g.set_data(X2, y2)                  # the recording must be dropped and made again
                if r == 7:
                    g.profile(("forward", "update"))     # a profiled round runs eagerly
                g.local_steps()
                if r == 7:
                    g.profile(())
                reps = [g.replica(j) for j in range(P)]
                losses = g.losses()
                g.meta_update()
                trace.append((g.indices(), reps, losses, g.params(), g.momentum()))
            g.close()
        runs.append(trace)
    for r, (a, b) in enumerate(zip(*runs)):
        assert np.array_equal(a[0], b[0]), "%s round %d: indices" % (tag, r)
        for j in range(P):
            assert np.array_equal(a[1][j], b[1][j]), "%s round %d: replica %d" % (tag, r, j)
        assert np.array_equal(a[2], b[2]), "%s round %d: losses" % (tag, r)
        assert np.array_equal(a[3], b[3]), "%s round %d: global model" % (tag, r)
        assert np.array_equal(a[4], b[4]), "%s round %d: momentum" % (tag, r)


def test_graph_replay_against_the_oracle():
    torch = _torch()
    dims = (96, 72, 10)
    with torch.cuda.stream(torch.cuda.Stream()):
        g, o = _pair(3, 3, 0.05, 0.5, dims, 20, False, 41)
        g.graph(True)
        _run_and_compare(g, o, dims, 5, TOL_FP32, "graph")
        g.close()


def test_graph_needs_a_stream_of_its_own():
    g, _ = _pair(2, 2, 0.05, 0.5, (40, 24, 10), 8, False, 43)
    with pytest.raises(kavg.KavgError) as e:
        g.graph(True)
    assert e.value.code == kavg.KAVG_ESTATE
    g.local_steps()                                      # the context keeps working eagerly
    g.graph(False)
    g.close()


# ----------------------------------------------------------------- split storage of the fp32 master
def test_split_storage_returns_every_fp32_pattern_exactly():
    """Mixed precision keeps a learner's fp32 parameters as a bf16 plane plus a 16-bit remainder plane.
    Whatever fp32 values go in must come back bit for bit: ties of the bf16 rounding in both signs,
    remainders just below and above one half, carries into the exponent, zeros, tiny and large values."""
    dims, P = (40, 24, 6), 3
    n = kavg.kavg_num_params(dims)
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    bits &= np.uint32(0xBFFFFFFF)                              # keep exponents away from inf / nan
    special = np.array([0x3F808000, 0xBF808000, 0x3F818000, 0xBF818000, 0x3F807FFF, 0x3F808001,
                        0x3FFFFFFF, 0xBFFFFFFF, 0x3FFF8000, 0x00000000, 0x80000000, 0x00800000,
                        0x3F800000, 0x3F80FFFF, 0x7F000000 & 0x7EFFFFFF, 0x0000FFFF, 0x00008000], dtype=np.uint32)
    bits[:special.size] = special
    w0 = bits.view(np.float32).copy()
    data = _dataset(64, dims, True, 3)
    g = kavg.MAvg(P, 2, 0.0, 0.5, dims, 8, kavg.KAVG_BF16, index_seed=1)
    X, y = _to_device(data, True)
    g.set_data(X, y)
    g.set_params(w0)
    for j in range(P):
        assert np.array_equal(g.replica(j).view(np.uint32), bits), "replica %d after set_params" % j
    assert np.array_equal(g.params().view(np.uint32), bits)
    g.close()


# ----------------------------------------------------------------- random ragged shapes
@pytest.mark.parametrize("bf16", [True, False], ids=["bf16", "fp32"])
def test_random_ragged_shapes(bf16):
    """Forty seeded random models (1-3 layers; widths any multiple of 8 up to 312 in mixed precision, any
    width up to 199 in fp32; class counts on both sides of the head-kernel limit; batches from 1 to 130;
    1-5 learners): two meta rounds each against the oracle.  Covers tile tails in every dimension of
    every kernel, and the clamped loads behind them."""
    _torch()
    rng = np.random.default_rng(123)
    tol = TOL_BF16 if bf16 else TOL_FP32
    dtype = kavg.KAVG_BF16 if bf16 else kavg.KAVG_FP32
    for case in range(40):
        L = int(rng.integers(1, 4))
        widths = [int(rng.integers(1, 40)) * 8 if bf16 else int(rng.integers(1, 200)) for _ in range(L)]
        dims = widths + [int(rng.choice([2, 3, 7, 10, 13, 16, 17, 24, 33]))]
        P, K = int(rng.integers(1, 6)), int(rng.integers(1, 4))
        B = int(rng.choice([1, 5, 16, 33, 64, 70, 130]))
        data = synth.make_dataset(300, dims[0], dims[-1], bf16=bf16, seed_data=case, seed_teacher=case + 1,
                                  teacher_hidden=16)
        w0 = synth.he_normal_params(dims, case + 2)
        g = kavg.MAvg(P, K, 0.05, 0.7, dims, B, dtype, index_seed=case + 3)
        X, y = _to_device(data, bf16)
        g.set_data(X, y)
        g.set_params(w0)
        o = O.MAvgOracle(P, K, 0.05, 0.7, dims, B, bf16=bf16, index_seed=case + 3)
        o.set_data(data["X32"], data["y"])
        o.set_params(w0)
        tag = "case %d dims %s P=%d K=%d B=%d" % (case, dims, P, K, B)
        for r in range(2):
            g.local_steps()
            o.local_steps()
            assert np.array_equal(g.indices(), o.indices()), tag
            for j in range(P):
                e = replica_error(g.replica(j), o.replica(j), dims)
                assert e < tol, "%s: replica %d round %d: %.3g" % (tag, j, r, e)
            g.meta_update()
            o.meta_update()
            e = replica_error(g.params(), o.params(), dims)
            assert e < tol, "%s: global model round %d: %.3g" % (tag, r, e)
        g.close()
