"""Pins for the oracle's model arithmetic (forward, softmax-CE, backprop)."""
import math

import numpy as np
import torch

from oracle import mavg_oracle as O


def _rand_problem(dims, B, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(O.num_params(dims)) * 0.5
    X = rng.standard_normal((B, dims[0]))
    y = rng.integers(0, dims[-1], size=B)
    return w, X, y


def _torch_loss_and_grad(w, dims, X, y):
    """Library reference: torch float64 linear/relu/cross_entropy + autograd."""
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(X, dtype=torch.float64)
    o = 0
    L = len(dims) - 1
    for l in range(1, L + 1):
        W = wt[o:o + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1])
        o += dims[l] * dims[l - 1]
        b = wt[o:o + dims[l]]
        o += dims[l]
        a = torch.nn.functional.linear(a, W, b)
        if l < L:
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), wt.grad.numpy()


def test_backprop_matches_central_differences():
    dims, B = (5, 4, 3), 3
    w, X, y = _rand_problem(dims, B, 0)
    loss, g = O.minibatch_gradient(w, dims, X, y)
    h = 1e-5
    fd = np.zeros_like(w)
    for i in range(w.size):
        wp, wm = w.copy(), w.copy()
        wp[i] += h
        wm[i] -= h
        fd[i] = (O.minibatch_gradient(wp, dims, X, y)[0] - O.minibatch_gradient(wm, dims, X, y)[0]) / (2 * h)
    assert np.max(np.abs(fd - g)) < 1e-8 * max(1.0, np.max(np.abs(g)))
    assert np.max(np.abs(g)) > 1e-3          # the check is not vacuous


def test_backprop_three_layers_central_differences():
    dims, B = (6, 5, 4, 3), 4
    w, X, y = _rand_problem(dims, B, 1)
    _, g = O.minibatch_gradient(w, dims, X, y)
    h = 1e-5
    rng = np.random.default_rng(2)
    for i in rng.choice(w.size, size=40, replace=False):
        wp, wm = w.copy(), w.copy()
        wp[i] += h
        wm[i] -= h
        fd = (O.minibatch_gradient(wp, dims, X, y)[0] - O.minibatch_gradient(wm, dims, X, y)[0]) / (2 * h)
        assert abs(fd - g[i]) < 1e-8 * max(1.0, abs(g[i]))


def test_one_step_matches_library_autograd():
    for dims, B, seed in (((7, 6, 5), 4, 3), ((9, 8, 8, 4), 6, 4), ((5, 3), 2, 5)):
        w, X, y = _rand_problem(dims, B, seed)
        loss, g = O.minibatch_gradient(w, dims, X, y)
        tl, tg = _torch_loss_and_grad(w, dims, X, y)
        assert abs(loss - tl) < 1e-12 * max(1.0, abs(tl))
        assert np.max(np.abs(g - tg)) < 1e-12


def test_hand_expanded_two_two_two_net():
    """2-2-2 net, B=1, every quantity expanded in Python floats."""
    W1 = [[0.3, -0.2], [0.1, 0.4]]
    b1 = [0.05, -0.6]
    W2 = [[0.7, -0.5], [-0.3, 0.2]]
    b2 = [0.1, -0.1]
    x = [1.5, -0.5]
    y = 1
    w = np.array(W1[0] + W1[1] + b1 + W2[0] + W2[1] + b2)
    # forward
    z1 = [W1[i][0] * x[0] + W1[i][1] * x[1] + b1[i] for i in range(2)]
    a1 = [max(z, 0.0) for z in z1]
    assert a1[0] > 0 and a1[1] == 0.0          # one live, one dead unit
    z2 = [W2[i][0] * a1[0] + W2[i][1] * a1[1] + b2[i] for i in range(2)]
    e = [math.exp(z) for z in z2]
    p = [v / (e[0] + e[1]) for v in e]
    loss = -math.log(p[y])
    dz2 = [p[0], p[1] - 1.0]
    gW2 = [[dz2[i] * a1[k] for k in range(2)] for i in range(2)]
    gb2 = dz2
    da1 = [dz2[0] * W2[0][k] + dz2[1] * W2[1][k] for k in range(2)]
    dz1 = [da1[0], 0.0]                         # dead unit passes nothing back
    gW1 = [[dz1[i] * x[k] for k in range(2)] for i in range(2)]
    gb1 = dz1
    want = np.array(gW1[0] + gW1[1] + gb1 + gW2[0] + gW2[1] + gb2)
    got_loss, got = O.minibatch_gradient(w, (2, 2, 2), np.array([x]), np.array([y]))
    assert abs(got_loss - loss) < 1e-15
    assert np.max(np.abs(got - want)) < 1e-15


def test_softmax_ce_special_cases():
    rng = np.random.default_rng(7)
    Z = rng.standard_normal((6, 10)) * 3
    y = rng.integers(0, 10, size=6)
    loss, dZ = O.softmax_cross_entropy(Z, y)
    assert np.max(np.abs(dZ.sum(axis=1))) < 1e-16              # rows sum to zero
    loss2, dZ2 = O.softmax_cross_entropy(Z + 123.0, y)          # shift invariance
    assert np.allclose(loss, loss2, rtol=0, atol=1e-12) and np.allclose(dZ, dZ2, rtol=0, atol=1e-14)
    for C in (10, 1000):                                        # zero logits: uniform p, loss ln C
        l0, d0 = O.softmax_cross_entropy(np.zeros((4, C)), np.array([0, 1, 2, 3]))
        assert np.allclose(l0, math.log(C), rtol=1e-15)
        want = np.full((4, C), 1.0 / C)
        want[np.arange(4), np.arange(4)] -= 1.0
        assert np.allclose(d0, want / 4, rtol=0, atol=1e-17)
    big, _ = O.softmax_cross_entropy(np.array([[1000.0, -1000.0]]), np.array([1]))
    assert np.isfinite(big[0]) and abs(big[0] - 2000.0) < 1e-9   # no overflow


def test_zero_last_layer_gives_ln_C_loss():
    dims, B = (12, 8, 10), 5
    w, X, y = _rand_problem(dims, B, 9)
    Ws, bs = O.unpack(w, dims)
    Ws[-1][:] = 0.0
    bs[-1][:] = 0.0
    loss, _ = O.minibatch_gradient(w, dims, X, y)
    assert abs(loss - math.log(10)) < 1e-14


def test_flat_layout_is_weights_then_bias_per_layer():
    dims = (3, 2, 4)
    w = np.arange(O.num_params(dims), dtype=np.float64)
    Ws, bs = O.unpack(w, dims)
    assert O.num_params(dims) == 3 * 2 + 2 + 2 * 4 + 4
    assert Ws[0].shape == (2, 3) and Ws[0][1, 0] == 3.0          # row-major, output-major
    assert list(bs[0]) == [6.0, 7.0]
    assert Ws[1].shape == (4, 2) and Ws[1][0, 0] == 8.0
    assert list(bs[1]) == [16.0, 17.0, 18.0, 19.0]


# ------------------------------------------------------------------ mixed precision reading
def _bf(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def test_bf16_mode_rounding_points_against_library_casts():
    """Re-derive one minibatch gradient with torch's bf16 conversion as the
    rounding primitive at the points the mixed-precision reading names."""
    dims, B = (16, 24, 8, 5), 7
    rng = np.random.default_rng(11)
    w = (rng.standard_normal(O.num_params(dims)) * 0.3).astype(np.float32).astype(np.float64)
    X = _bf(torch.tensor(rng.standard_normal((B, dims[0])))).numpy()
    y = rng.integers(0, dims[-1], size=B)
    loss, g = O.minibatch_gradient(w, dims, X, y, bf16=True)

    Ws, bs = O.unpack(w, dims)
    Wq = [_bf(torch.tensor(W)) for W in Ws]
    bt = [torch.tensor(b) for b in bs]
    A = [torch.tensor(X)]
    Z = []
    for l in range(3):
        z = A[-1] @ Wq[l].T + bt[l]
        Z.append(z)
        if l < 2:
            A.append(_bf(torch.relu(z)))
    p = torch.softmax(Z[-1], dim=1)
    oh = torch.nn.functional.one_hot(torch.tensor(y), dims[-1]).to(torch.float64)
    dZ = _bf((p - oh) / B)
    pieces = [None] * 3
    for l in (2, 1, 0):
        pieces[l] = torch.cat([(dZ.T @ A[l]).reshape(-1), dZ.sum(0)])
        if l > 0:
            dZ = _bf((dZ @ Wq[l]) * (Z[l - 1] > 0))
    want = torch.cat(pieces).numpy()
    assert np.max(np.abs(g - want)) < 1e-15 + 1e-13 * np.max(np.abs(want))
    # and the mixed-precision gradient stays close to the exact one
    _, g_exact = O.minibatch_gradient(w, dims, X, y, bf16=False)
    assert np.max(np.abs(g - g_exact)) < 2e-2 * np.max(np.abs(g_exact))
    assert np.max(np.abs(g - g_exact)) > 0.0


def test_bf16_mode_rounds_weight_ties_to_even():
    """Weights that sit exactly between two bf16 values (constructed: low half of the fp32 pattern =
    0x8000, odd and even kept mantissas, both signs) enter the products rounded to the even
    neighbour: the gradient agrees with a derivation that uses the library's cast for the weights
    and differs from one that sends the ties away from zero."""
    dims, B = (8, 6, 4), 5
    rng = np.random.default_rng(13)
    n = O.num_params(dims)
    keep = rng.integers(0x3E00, 0x3F80, size=n).astype(np.uint32)            # magnitudes 0.125 .. 1
    sign = rng.integers(0, 2, size=n).astype(np.uint32) << np.uint32(31)
    w32 = (((keep << np.uint32(16)) | np.uint32(0x8000)) | sign).view(np.float32)
    w = w32.astype(np.float64)
    X = _bf(torch.tensor(rng.standard_normal((B, dims[0])))).numpy()
    y = rng.integers(0, dims[-1], size=B)
    _, g = O.minibatch_gradient(w, dims, X, y, bf16=True)

    def derive(round_w):
        Ws, bs = O.unpack(w, dims)
        W1, W2 = round_w(torch.tensor(Ws[0])), round_w(torch.tensor(Ws[1]))
        z1 = torch.tensor(X) @ W1.T + torch.tensor(bs[0])
        a1 = _bf(torch.relu(z1))
        z2 = a1 @ W2.T + torch.tensor(bs[1])
        oh = torch.nn.functional.one_hot(torch.tensor(y), dims[-1]).to(torch.float64)
        dz2 = _bf((torch.softmax(z2, dim=1) - oh) / B)
        dz1 = _bf((dz2 @ W2) * (z1 > 0))
        return torch.cat([(dz1.T @ torch.tensor(X)).reshape(-1), dz1.sum(0),
                          (dz2.T @ a1).reshape(-1), dz2.sum(0)]).numpy()

    def away(t):                                   # add half a unit to the magnitude, cut to 16 bits
        bits = t.to(torch.float32).numpy().view(np.uint32).astype(np.uint64)
        return torch.tensor((((bits + 0x8000) >> 16) << 16).astype(np.uint32).view(np.float32).astype(np.float64))

    want = derive(_bf)
    assert np.max(np.abs(g - want)) < 1e-15 + 1e-13 * np.max(np.abs(want))
    other = derive(away)
    assert np.max(np.abs(g - other)) > 1e-4 * np.max(np.abs(want))            # the tie rule is visible here
