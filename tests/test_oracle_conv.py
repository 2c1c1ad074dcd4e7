"""Pins for the convolutional instance of the oracle (oracle/conv_oracle.py)."""
import numpy as np
import torch

from oracle import conv_oracle as C
from oracle import mavg_oracle as O


def _problem(spec, B, seed, scale=0.4):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(spec.num_params()) * scale
    X = rng.standard_normal((B, spec.H * spec.W * spec.channels[0]))
    y = rng.integers(0, spec.dims[-1], size=B)
    return w, X, y


def test_gradient_matches_central_differences_on_every_parameter():
    spec = C.ConvSpec(4, 3, (2, 3, 2), (2, 4, 3))
    w, X, y = _problem(spec, 3, 0)
    loss, g = C.minibatch_gradient(w, spec, X, y)
    h = 1e-6
    fd = np.zeros_like(w)
    for i in range(w.size):
        wp, wm = w.copy(), w.copy()
        wp[i] += h
        wm[i] -= h
        fd[i] = (C.minibatch_gradient(wp, spec, X, y)[0] - C.minibatch_gradient(wm, spec, X, y)[0]) / (2 * h)
    assert np.max(np.abs(g - fd)) < 1e-7 * max(1.0, np.max(np.abs(fd)))
    assert np.max(np.abs(g)) > 1e-3


def _torch_model(w, spec, X, y):
    """The same network with a library convolution (channels-first tensors) and autograd, float64."""
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    x = torch.tensor(X, dtype=torch.float64).reshape(-1, spec.H, spec.W, spec.channels[0]).permute(0, 3, 1, 2)
    o = 0
    for t in range(1, len(spec.channels)):
        co, ci = spec.channels[t], spec.channels[t - 1]
        Wc = wt[o:o + co * 9 * ci].reshape(co, 3, 3, ci).permute(0, 3, 1, 2)          # -> [out][in][kh][kw]
        o += co * 9 * ci
        b = wt[o:o + co]
        o += co
        x = torch.relu(torch.nn.functional.conv2d(x, Wc, b, stride=1, padding=1))
    a = x.mean(dim=(2, 3))
    L = len(spec.dims) - 1
    for l in range(1, L + 1):
        W = wt[o:o + spec.dims[l] * spec.dims[l - 1]].reshape(spec.dims[l], spec.dims[l - 1])
        o += spec.dims[l] * spec.dims[l - 1]
        b = wt[o:o + spec.dims[l]]
        o += spec.dims[l]
        a = torch.nn.functional.linear(a, W, b)
        if l < L:
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(y, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), wt.grad.numpy()


def test_gradient_matches_a_library_convolution_with_autograd():
    for spec, B, seed in ((C.ConvSpec(5, 6, (3, 4, 5), (5, 6, 4)), 4, 1), (C.ConvSpec(3, 3, (1, 2), (2, 3)), 2, 2),
                          (C.ConvSpec(8, 8, (8, 16, 16), (16, 10)), 3, 3)):
        w, X, y = _problem(spec, B, seed)
        loss, g = C.minibatch_gradient(w, spec, X, y)
        want_loss, want = _torch_model(w, spec, X, y)
        assert abs(loss - want_loss) < 1e-12
        assert np.max(np.abs(g - want)) < 1e-12 * max(1.0, np.max(np.abs(want)))


def test_single_channel_convolution_expanded_by_hand():
    """A 3x3 one-channel image and one 3x3 filter: every output pixel is the filter laid over the
    zero-padded image, written out with plain loops."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 3, 3, 1))
    Wc = rng.standard_normal((1, 3, 3, 1))
    b = np.array([0.25])
    want = np.zeros((3, 3))
    for h in range(3):
        for w in range(3):
            s = b[0]
            for kh in range(3):
                for kw in range(3):
                    hh, ww = h + kh - 1, w + kw - 1
                    if 0 <= hh < 3 and 0 <= ww < 3:
                        s += x[0, hh, ww, 0] * Wc[0, kh, kw, 0]
            want[h, w] = s
    assert np.max(np.abs(C.conv3x3(x, Wc, b)[0, :, :, 0] - want)) < 1e-15
    # centre tap only: the convolution is a per-pixel scaling; corner tap: a shift with zero fill
    Wc0 = np.zeros((1, 3, 3, 1))
    Wc0[0, 1, 1, 0] = 2.0
    assert np.allclose(C.conv3x3(x, Wc0, np.zeros(1)), 2.0 * x)
    Wc1 = np.zeros((1, 3, 3, 1))
    Wc1[0, 0, 0, 0] = 1.0                                   # out[h][w] = x[h-1][w-1]
    out = C.conv3x3(x, Wc1, np.zeros(1))[0, :, :, 0]
    assert np.allclose(out[1:, 1:], x[0, :2, :2, 0]) and np.all(out[0, :] == 0) and np.all(out[:, 0] == 0)


def test_flat_layout_and_parameter_count():
    spec = C.ConvSpec(4, 4, (2, 3), (3, 5))
    assert spec.num_params() == 3 * 9 * 2 + 3 + 5 * 3 + 5
    w = np.arange(spec.num_params(), dtype=np.float64)
    convs, Ws, bs = C.unpack(w, spec)
    assert convs[0][0].shape == (3, 3, 3, 2) and convs[0][0][1, 0, 0, 0] == 18.0      # [out][kh][kw][in]
    assert convs[0][0][0, 0, 1, 0] == 2.0 and list(convs[0][1]) == [54.0, 55.0, 56.0]
    assert Ws[0].shape == (5, 3) and Ws[0][0, 0] == 57.0


def _bf(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def test_mixed_precision_rounding_points_against_library_casts():
    spec = C.ConvSpec(4, 4, (2, 3, 2), (2, 3))
    rng = np.random.default_rng(9)
    w = (rng.standard_normal(spec.num_params()) * 0.4).astype(np.float32).astype(np.float64)
    X = _bf(torch.tensor(rng.standard_normal((3, 4 * 4 * 2)))).numpy()
    y = rng.integers(0, 3, size=3)
    _, g = C.minibatch_gradient(w, spec, X, y, bf16=True)
    # the same with torch tensors and torch's cast as the rounding primitive, convolutions by autograd-free formulas
    convs, Ws, bs = C.unpack(w, spec)
    x0 = torch.tensor(X).reshape(3, 4, 4, 2)

    def conv(x, Wc, b):
        return torch.nn.functional.conv2d(x.permute(0, 3, 1, 2), torch.tensor(Wc).permute(0, 3, 1, 2), torch.tensor(b),
                                          padding=1).permute(0, 2, 3, 1)
    W1, W2 = _bf(torch.tensor(convs[0][0])).numpy(), _bf(torch.tensor(convs[1][0])).numpy()
    z1 = conv(x0, W1, convs[0][1])
    a1 = _bf(torch.relu(z1))
    z2 = conv(a1, W2, convs[1][1])
    a2 = _bf(torch.relu(z2))
    pooled = _bf(a2.mean(dim=(1, 2)))
    Wd = _bf(torch.tensor(Ws[0]))
    logits = pooled @ Wd.T + torch.tensor(bs[0])
    oh = torch.nn.functional.one_hot(torch.tensor(y), 3).to(torch.float64)
    dz = _bf((torch.softmax(logits, dim=1) - oh) / 3)
    gWd, gbd = dz.T @ pooled, dz.sum(0)
    dpool = _bf(dz @ Wd)
    dz2 = _bf((dpool[:, None, None, :] / 16.0) * (z2 > 0))
    gW2, gb2, dx2 = C.conv3x3_gradients(a1.numpy(), W2, dz2.numpy(), True)
    dz1 = _bf(torch.tensor(dx2) * (z1 > 0))
    gW1, gb1, _ = C.conv3x3_gradients(x0.numpy(), W1, dz1.numpy(), False)
    want = np.concatenate([gW1.ravel(), gb1, gW2.ravel(), gb2, gWd.numpy().ravel(), gbd.numpy()])
    assert np.max(np.abs(g - want)) < 1e-15 + 1e-12 * np.max(np.abs(want))
    _, g_exact = C.minibatch_gradient(w, spec, X, y, bf16=False)
    assert 0.0 < np.max(np.abs(g - g_exact)) < 3e-2 * np.max(np.abs(g_exact))


def test_mavg_on_the_convolutional_model_K1_mu0_is_synchronous_sgd():
    """Algorithm 1 does not depend on the model: K = 1, mu = 0 on P learners equals one SGD step on the
    concatenated batch (gradient by the library)."""
    spec = C.ConvSpec(4, 4, (2, 3), (3, 4))
    rng = np.random.default_rng(11)
    N, P, B, lr = 40, 3, 4, 0.2
    X = rng.standard_normal((N, 4 * 4 * 2))
    y = rng.integers(0, 4, size=N).astype(np.int32)
    w0 = rng.standard_normal(spec.num_params()) * 0.4
    o = C.make_oracle(P, 1, lr, 0.0, spec, B, index_seed=13)
    o.set_params(w0)
    o.set_data(X, y)
    o.local_steps()
    o.meta_update()
    idx = o.indices().reshape(-1)
    _, g = _torch_model(w0, spec, X[idx], y[idx])
    assert np.max(np.abs(o.params() - (w0 - lr * g))) < 1e-13
