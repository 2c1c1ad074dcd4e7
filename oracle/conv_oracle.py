"""Plain CPU oracle of a small convolutional classifier, the second instance of the objective
F(w) = (1/n) sum_i loss(y_i, f(x_i, w)) of Section 2 that M-AVG (Algorithm 1) is run on.

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's CPU-baseline
leg, never by the product path; shares no code with the HIP kernels.

The paper trains convolutional networks on 32x32x3 images (Section 4); it prints no architecture of
its own, so the model here is the plainest member of that family:

    x [H][W][c_0]  ->  M times ( 3x3 convolution, stride 1, zero padding 1, bias, ReLU )
                   ->  mean over the H*W positions  ->  MLP (ReLU hidden layers)  ->  softmax cross-entropy

written from the definitions, in float64, with numpy's matmul as the only library step:
  convolution   out[n,h,w,o] = b[o] + sum_{kh,kw,c} xpad[n,h+kh,w+kw,c] * W[o,kh,kw,c]     (kh, kw = 0..2)
  its gradients gW[o,kh,kw,c] = sum_{n,h,w} dZ[n,h,w,o] * xpad[n,h+kh,w+kw,c],  gb[o] = sum dZ[...,o],
                dxpad[n,h+kh,w+kw,c] += sum_o dZ[n,h,w,o] * W[o,kh,kw,c]
Layout: images are [H][W][channels] (channels last); flat parameters: for every convolution its
weights [c_out][3][3][c_in] then its bias, then the MLP's layers as in mavg_oracle (W row-major, bias).

Mixed precision (bf16=True) rounds, to nearest even, what the matrix products read and what is stored
between layers: the weights as multiplied, every stored activation (convolution outputs after ReLU,
the pooled vector, hidden MLP activations) and every back-propagated gradient that is stored (dZ of each
layer, the gradient of the pooled vector).  Sums, biases, softmax and the update stay unrounded.

Pins (tests/test_oracle_conv.py): central differences on every parameter of a tiny net; a library
convolution with autograd in float64; a hand-expanded single-channel 3x3 image; the mixed-precision
rounding points re-derived with a library cast.
"""
import numpy as np

from . import mavg_oracle as O


class ConvSpec:
    """H, W: image size; channels: c_0 (input) .. c_M; dims: c_M, hidden widths ..., classes."""

    def __init__(self, H, W, channels, dims):
        self.H, self.W = int(H), int(W)
        self.channels = tuple(int(c) for c in channels)
        self.dims = tuple(int(d) for d in dims)
        assert len(self.channels) >= 2 and self.dims[0] == self.channels[-1]

    def num_params(self):
        n = sum(self.channels[t] * 9 * self.channels[t - 1] + self.channels[t] for t in range(1, len(self.channels)))
        return n + O.num_params(self.dims)


def unpack(w, spec):
    """([(Wc [c_out][3][3][c_in], b [c_out])], MLP weights, MLP biases) as views into w."""
    convs, o = [], 0
    for t in range(1, len(spec.channels)):
        co, ci = spec.channels[t], spec.channels[t - 1]
        Wc = w[o:o + co * 9 * ci].reshape(co, 3, 3, ci)
        o += co * 9 * ci
        convs.append((Wc, w[o:o + co]))
        o += co
    Ws, bs = O.unpack(w[o:], spec.dims)
    return convs, Ws, bs


def conv3x3(x, Wc, b):
    """x [n][H][W][c_in] -> [n][H][W][c_out], zero padding 1, stride 1."""
    n, H, W, _ = x.shape
    xpad = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    out = np.zeros((n, H, W, Wc.shape[0])) + b
    for kh in range(3):
        for kw in range(3):
            out += xpad[:, kh:kh + H, kw:kw + W, :] @ Wc[:, kh, kw, :].T
    return out


def conv3x3_gradients(x, Wc, dZ, need_dx):
    n, H, W, _ = x.shape
    xpad = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    gW = np.zeros_like(Wc)
    dxpad = np.zeros_like(xpad) if need_dx else None
    flat = dZ.reshape(-1, dZ.shape[-1])
    for kh in range(3):
        for kw in range(3):
            patch = xpad[:, kh:kh + H, kw:kw + W, :]
            gW[:, kh, kw, :] = flat.T @ patch.reshape(-1, patch.shape[-1])
            if need_dx:
                dxpad[:, kh:kh + H, kw:kw + W, :] += dZ @ Wc[:, kh, kw, :]
    gb = flat.sum(axis=0)
    return gW, gb, (dxpad[:, 1:-1, 1:-1, :] if need_dx else None)


def minibatch_gradient(w, spec, Xb, yb, bf16=False):
    """(mean loss, flat gradient) of the minibatch objective; Xb [B][H*W*c_0] (channels last)."""
    q = O.rne_bf16 if bf16 else (lambda a: a)
    convs, Ws, bs = unpack(w, spec)
    Bn = Xb.shape[0]
    x = np.asarray(Xb, dtype=np.float64).reshape(Bn, spec.H, spec.W, spec.channels[0])
    acts, pre = [x], []
    for Wc, b in convs:                                  # convolution stack
        Z = conv3x3(acts[-1], q(Wc), b)
        pre.append(Z)
        acts.append(q(np.maximum(Z, 0.0)))
    pooled = q(acts[-1].mean(axis=(1, 2)))               # mean over the positions
    Wq = [q(W) for W in Ws]
    Zs, As = O.forward(Wq, bs, pooled, q)                # MLP
    loss, dZL = O.softmax_cross_entropy(Zs[-1], yb)
    L = len(Ws)
    gWs, gbs = [None] * L, [None] * L
    dZ = q(dZL)
    for l in range(L - 1, -1, -1):
        gWs[l] = dZ.T @ As[l]
        gbs[l] = dZ.sum(axis=0)
        dA = dZ @ Wq[l]
        if l > 0:
            dZ = q(dA * (Zs[l - 1] > 0.0))
    dpool = q(dA)                                        # gradient of the pooled vector, stored
    dZc = q((dpool[:, None, None, :] * (1.0 / (spec.H * spec.W))) * (pre[-1] > 0.0))
    gconv = [None] * len(convs)
    for t in range(len(convs) - 1, -1, -1):
        gW, gb, dx = conv3x3_gradients(acts[t], q(convs[t][0]), dZc, need_dx=t > 0)
        gconv[t] = (gW, gb)
        if t > 0:
            dZc = q(dx * (pre[t - 1] > 0.0))
    pieces = []
    for gW, gb in gconv:
        pieces += [gW.ravel(), gb]
    for gW, gb in zip(gWs, gbs):
        pieces += [gW.ravel(), gb]
    return float(loss.mean()), np.concatenate(pieces)


def make_oracle(P, K, lr, mu, spec, B, bf16=False, index_seed=0):
    """M-AVG (mavg_oracle.MAvgOracle) on this model."""
    return O.MAvgOracle(P, K, lr, mu, spec.dims, B, bf16=bf16, index_seed=index_seed,
                        gradient=lambda w, Xb, yb, b16: minibatch_gradient(w, spec, Xb, yb, b16),
                        n_params=spec.num_params())
