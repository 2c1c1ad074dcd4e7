"""Pins for the oracle's learner loop and meta step (Algorithm 1, eq. (2),
the z-sequence of the proof of Theorem 1, the geometric form of v)."""
import numpy as np
import pytest
import torch

from oracle import mavg_oracle as O


def _problem(dims, N, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, dims[0]))
    y = rng.integers(0, dims[-1], size=N).astype(np.int32)
    w0 = rng.standard_normal(O.num_params(dims)) * 0.3
    return X, y, w0


def _torch_sgd(w0, dims, X, y, batches, lr):
    """Plain minibatch SGD with a library autograd; batches: list of index arrays."""
    w = torch.tensor(w0, dtype=torch.float64)
    L = len(dims) - 1
    for ib in batches:
        wt = w.clone().requires_grad_(True)
        a = torch.tensor(X[ib], dtype=torch.float64)
        o = 0
        for l in range(1, L + 1):
            W = wt[o:o + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1])
            o += dims[l] * dims[l - 1]
            b = wt[o:o + dims[l]]
            o += dims[l]
            a = torch.nn.functional.linear(a, W, b)
            if l < L:
                a = torch.relu(a)
        loss = torch.nn.functional.cross_entropy(a, torch.tensor(y[ib], dtype=torch.long))
        loss.backward()
        w = w - lr * wt.grad
    return w.numpy()


DIMS = (10, 9, 7, 4)


def test_K1_mu0_equals_synchronous_sgd_at_batch_PB():
    P, B, rounds, lr = 4, 6, 5, 0.2
    X, y, w0 = _problem(DIMS, 200, 0)
    o = O.MAvgOracle(P, 1, lr, 0.0, DIMS, B, index_seed=99)
    o.set_params(w0)
    o.set_data(X, y)
    big_batches = []
    for _ in range(rounds):
        o.local_steps()
        o.meta_update()
        big_batches.append(o.indices().reshape(-1))        # the P batches of this round, concatenated
    want = _torch_sgd(w0, DIMS, X, y, big_batches, lr)
    assert np.max(np.abs(o.params() - want)) < 1e-13
    assert np.max(np.abs(want - w0)) > 1e-3


def test_P1_mu0_equals_plain_sgd():
    K, B, rounds, lr = 3, 5, 4, 0.15
    X, y, w0 = _problem(DIMS, 100, 1)
    o = O.MAvgOracle(1, K, lr, 0.0, DIMS, B, index_seed=5)
    o.set_params(w0)
    o.set_data(X, y)
    batches = []
    for _ in range(rounds):
        o.local_steps()
        batches += [o.indices()[0, k] for k in range(K)]
        o.meta_update()
    want = _torch_sgd(w0, DIMS, X, y, batches, lr)
    assert np.max(np.abs(o.params() - want)) < 1e-13
    # the stream continues across rounds: step counter t = round*K + k
    assert np.array_equal(batches[K + 1], O.minibatch_indices(5, 0, K + 1, B, 100))


def test_learners_use_their_own_streams_and_local_counter():
    X, y, w0 = _problem(DIMS, 64, 2)
    o = O.MAvgOracle(3, 2, 0.1, 0.5, DIMS, 4, index_seed=17)
    o.set_params(w0)
    o.set_data(X, y)
    o.local_steps()
    o.meta_update()
    o.local_steps()
    idx = o.indices()
    for j in range(3):
        for k in range(2):
            assert np.array_equal(idx[j, k], O.minibatch_indices(17, j, 2 + k, 4, 64))


def test_lr0_leaves_everything_fixed():
    # a = (1/P) sum_j w^j of P equal numbers is w only up to the rounding of the
    # running sum, so "fixed" means: to a few units in the last place of float64.
    X, y, w0 = _problem(DIMS, 64, 3)
    o = O.MAvgOracle(4, 3, 0.0, 0.9, DIMS, 5, index_seed=1)
    o.set_params(w0)
    o.set_data(X, y)
    for _ in range(3):
        o.local_steps()
        o.meta_update()
    scale = np.max(np.abs(w0))
    assert np.max(np.abs(o.params() - w0)) < 1e-15 * scale
    assert np.max(np.abs(o.momentum())) < 1e-15 * scale
    for j in range(4):
        assert np.array_equal(o.replica(j), o.params())
    # with a single learner the average is exact and nothing moves at all
    o1 = O.MAvgOracle(1, 3, 0.0, 0.9, DIMS, 5, index_seed=1)
    o1.set_params(w0)
    o1.set_data(X, y)
    o1.local_steps()
    o1.meta_update()
    assert np.array_equal(o1.params(), w0) and np.array_equal(o1.momentum(), np.zeros_like(w0))


def test_identical_replicas_average_to_themselves():
    rng = np.random.default_rng(4)
    n = 1000
    w = rng.standard_normal(n)
    v = rng.standard_normal(n) * 0.1
    for P in (1, 2, 8, 64):
        reps = np.tile(w, (P, 1))
        w1, v1 = O.meta_step(w, v, reps, 0.9)
        if P <= 2:                                          # w, w + w: exact sums, d = 0 exactly
            assert np.array_equal(v1, 0.9 * v)
            assert np.array_equal(w1, w + 0.9 * v)
        assert np.max(np.abs(v1 - 0.9 * v)) < P * 2.3e-16 * np.max(np.abs(w))
        assert np.max(np.abs(w1 - (w + 0.9 * v))) < P * 2.3e-16 * np.max(np.abs(w))
    # mu = 0: the new global model is the plain average (K-AVG, remark after Theorem 1)
    reps = rng.standard_normal((6, n))
    w1, v1 = O.meta_step(w, v, reps, 0.0)
    assert np.max(np.abs(w1 - reps.mean(axis=0))) < 1e-15


def test_displacement_is_minus_lr_times_K_step_average_gradient():
    """eq. (2): d = a - w~ = -lr * G_n with G_n = (1/P) sum_j sum_t (mean minibatch gradient)."""
    P, K, B, lr = 3, 4, 5, 0.07
    X, y, w0 = _problem(DIMS, 80, 5)
    o = O.MAvgOracle(P, K, lr, 0.6, DIMS, B, index_seed=3)
    o.set_params(w0)
    o.set_data(X, y)
    o.local_steps()
    # recompute G_n from the recorded batches with the library autograd, walking each learner
    G = np.zeros_like(w0)
    idx = o.indices()
    for j in range(P):
        w = w0.copy()
        for k in range(K):
            w_next = _torch_sgd(w, DIMS, X, y, [idx[j, k]], lr)
            G += (w - w_next) / lr
            w = w_next
    G /= P
    a = np.mean([o.replica(j) for j in range(P)], axis=0)
    assert np.max(np.abs((a - w0) + lr * G)) < 1e-14
    assert np.max(np.abs(o.grad_sum / P - G)) < 1e-12
    v_before = o.momentum()
    o.meta_update()
    assert np.max(np.abs(o.momentum() - (0.6 * v_before - lr * G))) < 1e-14
    assert np.max(np.abs(o.params() - (w0 + o.momentum()))) < 1e-15


def test_z_sequence_identity():
    """z_n = w~_n + mu/(1-mu) v_n obeys z_{n+1} - z_n = d_n/(1-mu) for any model."""
    P, K, B, lr, mu = 4, 2, 4, 0.1, 0.8
    X, y, w0 = _problem(DIMS, 80, 6)
    o = O.MAvgOracle(P, K, lr, mu, DIMS, B, index_seed=8)
    o.set_params(w0)
    o.set_data(X, y)
    z = o.params() + mu / (1 - mu) * o.momentum()
    for _ in range(5):
        w_before = o.params()
        o.local_steps()
        a = np.mean([o.replica(j) for j in range(P)], axis=0)
        d = a - w_before
        o.meta_update()
        z_new = o.params() + mu / (1 - mu) * o.momentum()
        assert np.max(np.abs((z_new - z) * (1 - mu) - d)) < 1e-14
        assert np.max(np.abs(d)) > 1e-5
        z = z_new
        for j in range(P):                                   # learners restart from w~_{n+1}, not from a
            assert np.array_equal(o.replica(j), o.params())


def test_v_is_the_geometric_sum_of_displacements():
    rng = np.random.default_rng(7)
    n, P, mu, rounds = 300, 5, 0.7, 9
    w = rng.standard_normal(n)
    v = np.zeros(n)
    w_start = w.copy()
    ds = []
    for r in range(rounds):
        reps = w + rng.standard_normal((P, n)) * 0.01
        ds.append(reps.mean(axis=0) - w)
        w, v = O.meta_step(w, v, reps, mu)
        v_closed = sum(mu ** i * ds[r - i] for i in range(r + 1))
        assert np.max(np.abs(v - v_closed)) < 1e-15
    # total displacement: each d_i enters w~ with weight Gamma = (1 - mu^m)/(1 - mu)
    w_closed = w_start + sum(ds[i] * (1 - mu ** (rounds - i)) / (1 - mu) for i in range(rounds))
    assert np.max(np.abs(w - w_closed)) < 1e-14


def test_repeated_passes_closed_form():
    """Meta-only workload: after the first pass all replicas equal w~, so d = 0 and
    v_k = mu^(k-1) v_1, w~_k = w~_0 + v_1 (1 - mu^k)/(1 - mu)."""
    rng = np.random.default_rng(8)
    n, P, mu = 500, 64, 0.9
    w0 = rng.standard_normal(n) * 0.05
    v0 = rng.standard_normal(n) * 1e-3
    reps = w0 + rng.standard_normal((P, n)) * 1e-3
    w, v = O.meta_step(w0, v0, reps, mu)
    v1 = v.copy()
    assert np.max(np.abs(v1 - (mu * v0 + reps.mean(axis=0) - w0))) < 1e-16
    for k in range(2, 201):
        w, v = O.meta_step(w, v, np.tile(w, (P, 1)), mu)
    # d of the later passes is zero only up to the rounding of the running sum
    # over P equal values (<= P/2 ulp of w~); through v <- mu v + d it settles at
    # no more than that bound divided by (1 - mu).
    noise = P * 1.2e-16 * np.max(np.abs(w0)) / (1 - mu)
    assert np.max(np.abs(v - mu ** 199 * v1)) < noise
    assert np.max(np.abs(w - (w0 + v1 * (1 - mu ** 200) / (1 - mu)))) < 200 * noise
    assert 200 * noise < 1e-4 * np.max(np.abs(v1))          # the bound still resolves v_1


def test_set_indices_overrides_the_stream():
    X, y, w0 = _problem(DIMS, 50, 9)
    idx = np.random.default_rng(0).integers(0, 50, size=(2, 3, 4)).astype(np.int32)
    o = O.MAvgOracle(2, 3, 0.1, 0.0, DIMS, 4, index_seed=0)
    o.set_params(w0)
    o.set_data(X, y)
    o.set_indices(idx)
    o.local_steps()
    assert np.array_equal(o.indices(), idx)
    for j in range(2):
        want = _torch_sgd(w0, DIMS, X, y, [idx[j, k] for k in range(3)], 0.1)
        assert np.max(np.abs(o.replica(j) - want)) < 1e-14


# ---------------------------------------------------------------------------
# The pins above must notice plausible mistakes: plant some in copies of the
# oracle's functions (on the CPU) and see the corresponding check fail.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("mistake", ["sign_d", "mu_on_d", "restart_from_a", "w_plus_d"])
def test_planted_meta_mistakes_are_caught(monkeypatch, mistake):
    def bad_meta(w, v, reps, mu):
        a = reps.mean(axis=0)
        d = a - w
        if mistake == "sign_d":
            vn = mu * v - d
            return w + vn, vn
        if mistake == "mu_on_d":
            vn = mu * (v + d)
            return w + vn, vn
        if mistake == "w_plus_d":
            vn = mu * v + d
            return w + d, vn
        vn = mu * v + d
        return a, vn                                          # forgets the momentum extrapolation

    monkeypatch.setattr(O, "meta_step", bad_meta)
    with pytest.raises(AssertionError):
        test_z_sequence_identity()


@pytest.mark.parametrize("mistake", ["no_mean", "mask_ge", "transposed_gw", "post_update_w"])
def test_planted_backprop_mistakes_are_caught(monkeypatch, mistake):
    import tests.test_oracle_model as TM
    if mistake == "no_mean":
        orig = O.softmax_cross_entropy
        monkeypatch.setattr(O, "softmax_cross_entropy", lambda Z, y: (orig(Z, y)[0], orig(Z, y)[1] * Z.shape[0]))
    elif mistake == "mask_ge":
        def bad_backward(Ws, Zs, As, dZL, q=lambda x: x):
            L = len(Ws)
            gWs, gbs = [None] * L, [None] * L
            dZ = dZL
            for l in range(L - 1, -1, -1):
                gWs[l] = dZ.T @ As[l]
                gbs[l] = dZ.sum(axis=0)
                if l > 0:
                    dZ = (dZ @ Ws[l]) * (Zs[l - 1] >= -0.5)
            return gWs, gbs
        monkeypatch.setattr(O, "backward", bad_backward)
    elif mistake == "transposed_gw":
        orig_b = O.backward

        def bad_backward(Ws, Zs, As, dZL, q=lambda x: x):
            gWs, gbs = orig_b(Ws, Zs, As, dZL, q)
            return [g.T.reshape(g.shape) for g in gWs], gbs
        monkeypatch.setattr(O, "backward", bad_backward)
    else:
        orig_b = O.backward

        def bad_backward(Ws, Zs, As, dZL, q=lambda x: x):
            return orig_b([W * 1.01 for W in Ws], Zs, As, dZL, q)
        monkeypatch.setattr(O, "backward", bad_backward)
    with pytest.raises(AssertionError):
        TM.test_backprop_three_layers_central_differences()


# ---------------------------------------------------------------------------
# learner-level momentum (Section 2: momentum "can also" be added at the learner level)
# ---------------------------------------------------------------------------
def _torch_momentum_sgd(w0, dims, X, y, batches, lr, beta):
    """Library reference: torch.optim.SGD(momentum=beta) (heavy ball, no dampening, no Nesterov)."""
    w = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([w], lr=lr, momentum=beta)
    L = len(dims) - 1
    for ib in batches:
        opt.zero_grad()
        a = torch.tensor(X[ib], dtype=torch.float64)
        o = 0
        for l in range(1, L + 1):
            W = w[o:o + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1])
            o += dims[l] * dims[l - 1]
            b = w[o:o + dims[l]]
            o += dims[l]
            a = torch.nn.functional.linear(a, W, b)
            if l < L:
                a = torch.relu(a)
        torch.nn.functional.cross_entropy(a, torch.tensor(y[ib], dtype=torch.long)).backward()
        opt.step()
    return w.detach().numpy()


def test_learner_momentum_matches_library_heavy_ball():
    # one learner, K steps, no meta momentum, ONE round: the replica is momentum SGD on its stream
    K, B, lr, beta = 6, 5, 0.1, 0.8
    X, y, w0 = _problem(DIMS, 100, 11)
    o = O.MAvgOracle(1, K, lr, 0.0, DIMS, B, index_seed=5, learner_momentum=beta)
    o.set_params(w0)
    o.set_data(X, y)
    o.local_steps()
    want = _torch_momentum_sgd(w0, DIMS, X, y, [o.indices()[0, k] for k in range(K)], lr, beta)
    assert np.max(np.abs(o.replica(0) - want)) < 1e-13
    assert np.max(np.abs(want - _torch_sgd(w0, DIMS, X, y, [o.indices()[0, k] for k in range(K)], lr))) > 1e-3


def test_learner_velocity_persists_across_rounds_and_is_per_learner():
    P, K, B, lr, beta = 2, 2, 4, 0.1, 0.5
    X, y, w0 = _problem(DIMS, 60, 12)
    o = O.MAvgOracle(P, K, lr, 0.0, DIMS, B, index_seed=6, learner_momentum=beta)
    o.set_params(w0)
    o.set_data(X, y)
    o.local_steps()
    u_after_round1 = [o.velocity(j) for j in range(P)]
    assert np.max(np.abs(u_after_round1[0] - u_after_round1[1])) > 1e-4          # own streams, own velocities
    o.meta_update()
    start = o.params()
    o.local_steps()
    # first step of round 2 for learner 0: u = beta*u_prev + g(start), w = start - lr*u
    idx = o.indices()[0, 0]
    _, g = O.minibatch_gradient(start, DIMS, X[idx], y[idx])
    u1 = beta * u_after_round1[0] + g
    w1 = start - lr * u1
    idx = o.indices()[0, 1]
    _, g2 = O.minibatch_gradient(w1, DIMS, X[idx], y[idx])
    u2 = beta * u1 + g2
    assert np.max(np.abs(o.velocity(0) - u2)) < 1e-14
    assert np.max(np.abs(o.replica(0) - (w1 - lr * u2))) < 1e-14


def test_learner_momentum_zero_is_algorithm_1():
    X, y, w0 = _problem(DIMS, 60, 13)
    a = O.MAvgOracle(3, 2, 0.1, 0.7, DIMS, 4, index_seed=7)
    b = O.MAvgOracle(3, 2, 0.1, 0.7, DIMS, 4, index_seed=7, learner_momentum=0.0)
    for o in (a, b):
        o.set_params(w0)
        o.set_data(X, y)
        for _ in range(2):
            o.local_steps()
            o.meta_update()
    assert np.array_equal(a.params(), b.params())


# ------------------------------------------------------------------ resume (set_state)
@pytest.mark.parametrize("bf16", [False, True], ids=["fp64", "bf16"])
def test_set_state_resumes_the_run_where_it_stopped(bf16):
    """Global model, momentum buffer and round counter are the whole state of Algorithm 1 between
    rounds (every learner restarts from the global model): a run cut after round 2 and resumed from
    those three continues exactly like the uninterrupted one, including the minibatches it draws
    (learner j's step counter is round * K)."""
    P, K, B, lr, mu = 3, 2, 4, 0.1, 0.8
    X, y, w0 = _problem(DIMS, 120, 21)
    a = O.MAvgOracle(P, K, lr, mu, DIMS, B, bf16=bf16, index_seed=5)
    a.set_params(w0)
    a.set_data(X, y)
    for _ in range(2):
        a.local_steps()
        a.meta_update()
    w, v, r = a.params(), a.momentum(), a.round
    assert r == 2
    b = O.MAvgOracle(P, K, lr, mu, DIMS, B, bf16=bf16, index_seed=5)
    b.set_data(X, y)
    b.set_state(w, v, r)
    for j in range(P):
        assert np.array_equal(b.replica(j), w)                 # learners restart from the global model
    for _ in range(2):
        a.local_steps()
        a.meta_update()
        b.local_steps()
        b.meta_update()
        assert np.array_equal(a.indices(), b.indices())
        assert np.array_equal(a.params(), b.params()) and np.array_equal(a.momentum(), b.momentum())
        assert np.array_equal(a.losses(), b.losses())
    assert b.round == 4
    # the resumed run's draws are those of steps round*K .. : not the first steps' again
    for j in range(P):
        for k in range(K):
            assert np.array_equal(b.indices()[j, k], O.minibatch_indices(5, j, 3 * K + k, B, 120))
    assert not np.array_equal(b.indices()[0, 0], O.minibatch_indices(5, 0, 0, B, 120))


def test_set_state_at_round_zero_with_zero_momentum_is_set_params():
    X, y, w0 = _problem(DIMS, 80, 22)
    a = O.MAvgOracle(2, 2, 0.1, 0.9, DIMS, 3, index_seed=9)
    a.set_params(w0)
    b = O.MAvgOracle(2, 2, 0.1, 0.9, DIMS, 3, index_seed=9)
    b.set_state(w0, np.zeros_like(w0), 0)
    for o in (a, b):
        o.set_data(X, y)
        o.local_steps()
        o.meta_update()
    assert np.array_equal(a.params(), b.params()) and np.array_equal(a.momentum(), b.momentum())
    # a momentum buffer handed in is used: the next global model moves by mu * v more
    c = O.MAvgOracle(2, 2, 0.1, 0.9, DIMS, 3, index_seed=9)
    c.set_state(w0, np.full_like(w0, 0.01), 0)
    c.set_data(X, y)
    c.local_steps()
    c.meta_update()
    assert np.allclose(c.params() - a.params(), 0.9 * 0.01, rtol=0, atol=1e-12)


def test_learners_walked_by_threads_give_the_same_run():
    X, y, w0 = _problem(DIMS, 150, 23)
    runs = []
    for workers in (1, 3):
        o = O.MAvgOracle(5, 3, 0.1, 0.9, DIMS, 4, index_seed=3)
        o.set_params(w0)
        o.set_data(X, y)
        for _ in range(2):
            o.local_steps(workers=workers)
            o.meta_update()
        runs.append((o.params(), o.momentum(), o.losses(), o.indices(), o.grad_sum))
    for a, b in zip(*runs):
        assert np.array_equal(a, b)


# ------------------------------------------------------------------ local steps as low-rank terms
def test_local_steps_are_rank_B_terms_on_top_of_the_round_start_weights():
    """Algorithm 1: a learner's k-th local step subtracts lr * dZ_k^T A_k (a rank-B matrix) from each
    weight matrix.  So along the oracle's own trajectory  W_k = W_0 - lr sum_{i<k} dZ_i^T A_i, and a
    product with W_k can be formed without W_k:  A W_k^T = A W_0^T - lr sum_{i<k} (A A_i^T) dZ_i  and
    dZ W_k = dZ W_0 - lr sum_{i<k} (dZ dZ_i^T) A_i.  Checked layer by layer against the replica the
    oracle has actually stepped (the GPU's deferred-update mode relies on exactly this)."""
    P, K, B, lr = 1, 4, 5, 0.1
    X, y, w0 = _problem(DIMS, 60, 31)
    o = O.MAvgOracle(P, 1, lr, 0.0, DIMS, B, index_seed=7)
    o.set_params(w0)
    o.set_data(X, y)
    W0, b0 = O.unpack(w0.copy(), DIMS)
    hist = []                                       # per step: (inputs of every layer, dZ of every layer)
    rng = np.random.default_rng(0)
    for k in range(K):
        Wk, bk = O.unpack(o.replica(0), DIMS)       # the oracle's current weights
        ib = O.minibatch_indices(7, 0, k, B, 60)
        Zs, As = O.forward(Wk, bk, X[ib])
        for l in range(len(Wk)):
            # the stepped weights are the round-start ones plus the pending rank-B terms
            want = W0[l] - lr * sum((dZ[l].T @ A[l] for A, dZ in hist), np.zeros_like(W0[l]))
            assert np.max(np.abs(Wk[l] - want)) < 1e-14
            # forward product without W_k
            low_rank = As[l] @ W0[l].T - lr * sum(((As[l] @ A[l].T) @ dZ[l] for A, dZ in hist), 0.0)
            assert np.max(np.abs(As[l] @ Wk[l].T - low_rank)) < 1e-12
            # data-gradient product without W_k
            g = rng.standard_normal((B, DIMS[l + 1]))
            low_rank = g @ W0[l] - lr * sum(((g @ dZ[l].T) @ A[l] for A, dZ in hist), 0.0)
            assert np.max(np.abs(g @ Wk[l] - low_rank)) < 1e-12
        # this step's dZ_l, recomputed from the definition (the oracle's backward pass keeps none)
        _, dZL = O.softmax_cross_entropy(Zs[-1], y[ib])
        dZs = [None] * len(Wk)
        dZ = dZL
        for l in range(len(Wk) - 1, -1, -1):
            dZs[l] = dZ
            if l > 0:
                dZ = (dZ @ Wk[l]) * (Zs[l - 1] > 0)
        hist.append((As, dZs))
        o.local_steps()                             # K = 1 per call: one more local step, no meta step
    assert len(hist) == K and np.max(np.abs(o.replica(0) - w0)) > 1e-3
