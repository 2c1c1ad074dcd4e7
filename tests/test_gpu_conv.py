"""The convolutional learner (kavg_init_conv) against the oracle of the same model: 3x3 convolutions,
ReLU, mean over the positions, MLP, softmax cross-entropy, under Algorithm 1."""
import numpy as np
import pytest

from oracle import conv_oracle as C
from paper_2110_00625_amd import kavg, synth

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def conv_slices(spec):
    """(name, slice, kind) of every tensor of the flat vector, in order."""
    out, o = [], 0
    for t in range(1, len(spec.channels)):
        nw = spec.channels[t] * 9 * spec.channels[t - 1]
        out.append(("conv%d.W" % t, slice(o, o + nw)))
        o += nw
        out.append(("conv%d.b" % t, slice(o, o + spec.channels[t])))
        o += spec.channels[t]
    for l in range(1, len(spec.dims)):
        nw = spec.dims[l] * spec.dims[l - 1]
        out.append(("fc%d.W" % l, slice(o, o + nw)))
        o += nw
        out.append(("fc%d.b" % l, slice(o, o + spec.dims[l])))
        o += spec.dims[l]
    assert o == spec.num_params()
    return out


def conv_error(got, want, spec, verbose=False):
    """Largest per-tensor error; weights against their own largest magnitude, a bias against the
    larger of its own and its layer's weight scale (one ReLU mask that falls the other way moves a
    single learner's bias element by several per cent of itself, however exact the arithmetic)."""
    worst, wscale = 0.0, 1.0
    for name, sl in conv_slices(spec):
        w = np.asarray(want[sl], dtype=np.float64)
        g = np.asarray(got[sl], dtype=np.float64)
        scale = float(np.max(np.abs(w)))
        if name.endswith(".W"):
            wscale = scale
        else:
            scale = max(scale, wscale)
        e = float(np.max(np.abs(g - w))) / max(scale, 1e-30)
        if verbose:
            print("   %-8s %.3g" % (name, e))
        worst = max(worst, e)
    return worst


def _setup(P, K, B, H, W, channels, dims, seed, N=300, lr=0.05, mu=0.9):
    torch = _torch()
    spec = C.ConvSpec(H, W, channels, dims)
    data = synth.make_image_dataset(N, H, W, min(3, channels[0]), channels[0], dims[-1], seed_data=seed, seed_texture=seed + 1)
    w0 = synth.he_normal_conv_params(channels, dims, seed + 2)
    assert w0.size == spec.num_params()
    g = kavg.MAvg(P, K, lr, mu, dims, B, kavg.KAVG_BF16, index_seed=seed + 3, conv=(H, W, channels))
    assert g.n == spec.num_params()
    X = torch.from_numpy(data["Xbits"].view(np.int16).reshape(N, H, W, channels[0])).cuda()
    g.set_data(X, torch.from_numpy(data["y"]).cuda())
    g.set_params(w0)
    o = C.make_oracle(P, K, lr, mu, spec, B, bf16=True, index_seed=seed + 3)
    o.set_data(data["X32"], data["y"])
    o.set_params(w0)
    return g, o, spec


CASES = [
    # P, K, B, H, W, channels, dims
    (2, 3, 16, 8, 8, (8, 16, 24), (24, 40, 10)),       # two convolutions, head kernels for the last MLP layer
    (3, 2, 10, 6, 5, (8, 8), (8, 10)),                  # one convolution, a one-layer MLP, odd image
    (2, 2, 12, 7, 9, (8, 24, 16, 32), (32, 48, 24)),    # three convolutions, 24 classes (generic last layer)
    (2, 2, 32, 16, 16, (8, 32, 64), (64, 10)),          # 8192 positions per learner: the weight gradient is split
    (1, 2, 2, 128, 128, (8, 16, 8), (8, 10)),           # 2^14 positions per image: every convolution on explicit patches
    # images 32 pixels wide: the weight gradients of convolutions 2.. come from the all-taps kernel
    (2, 2, 8, 32, 32, (8, 32, 64, 128), (128, 10)),     # the shapes of the cifar_conv workload: 32->64 and 64->128
    (3, 1, 4, 6, 32, (8, 32, 32), (32, 10)),            # three slices per image, one image per workgroup: borders everywhere
    (2, 1, 6, 4, 32, (8, 64, 64, 32), (32, 10)),        # three images per workgroup; 64->64 and 64->32
    (2, 1, 4, 8, 32, (8, 32, 128), (128, 10)),          # 32->128
    # ... and, with heights that are multiples of 8, their forward pass and data gradient from the tile kernels
    (2, 1, 3, 8, 32, (8, 32, 32, 64, 64, 32), (32, 10)),  # 32->32, 32->64, 64->64, 64->32: every remaining channel pairing
    (1, 2, 2, 16, 32, (8, 128, 32), (32, 10)),          # 128 contraction channels forward: two channel groups
    (2, 2, 4, 8, 32, (8, 64, 32), (32, 10)),            # first convolution 8->64 straight from the gathered images (8->32: above)
]


@pytest.mark.parametrize("P,K,B,H,W,channels,dims", CASES, ids=["%dx%d-%s-%s" % (c[3], c[4], c[5], c[6]) for c in CASES])
def test_conv_learner_matches_the_oracle(P, K, B, H, W, channels, dims):
    g, o, spec = _setup(P, K, B, H, W, channels, dims, 71)
    for r in range(2):
        print("round", r, flush=True)
        g.local_steps()
        o.local_steps()
        assert np.array_equal(g.indices(), o.indices())
        for j in range(P):
            e = conv_error(g.replica(j), o.replica(j), spec, verbose=True)
            assert e < TOL_BF16, "replica %d after the local steps of round %d: %.3g" % (j, r, e)
        gl, ol = g.losses(), o.losses()
        assert np.max(np.abs(gl - ol) / np.maximum(np.abs(ol), 1e-3)) < TOL_BF16, (gl, ol)
        g.meta_update()
        o.meta_update()
        e = conv_error(g.params(), o.params(), spec)
        assert e < TOL_BF16, "global model after round %d: %.3g" % (r, e)


def test_cifar_conv_launch_configuration_one_step_sampled_learners():
    """The benchmark's convolutional workload at its full launch configuration (P = 16 learners of B = 64 images of
    32x32, channels 8-32-64-128: 256 or 512 image ranges per weight gradient, 4096 tiles per forward pass), one local
    step; the oracle walks the first and the last learner."""
    from paper_2110_00625_amd.configs import CIFAR_CONV as w
    g, o, spec = _setup(w.P, 1, w.B, w.H, w.W, w.channels, w.dims, 73, N=600, lr=w.lr, mu=w.mu)
    g.local_steps()
    sample = [0, w.P - 1]
    o.local_steps(learners=sample)
    for j in sample:
        assert np.array_equal(g.indices()[j], o.indices()[j])
        e = conv_error(g.replica(j), o.replica(j), spec, verbose=True)
        print("cifar_conv learner %d after one local step: %.3g" % (j, e))
        assert e < 2e-4, e                 # measured 2e-6 .. 4e-6
        assert abs(g.losses()[0, j] - o.losses()[0, j]) < 1e-3 * max(1.0, o.losses()[0, j])
    g.close()


def test_cifar_conv_whole_round_every_learner():
    """One whole meta round of the benchmark's convolutional workload (P = 16, K = 8, B = 64), free running from
    w~_1: every replica after the local steps, the per-step losses, and the global model after the meta step."""
    from paper_2110_00625_amd.configs import CIFAR_CONV as w
    g, o, spec = _setup(w.P, w.K, w.B, w.H, w.W, w.channels, w.dims, 74, N=2000, lr=w.lr, mu=w.mu)
    g.local_steps()
    o.local_steps(workers=8)
    assert np.array_equal(g.indices(), o.indices())
    worst = 0.0
    for j in range(w.P):
        worst = max(worst, conv_error(g.replica(j), o.replica(j), spec))
    print("cifar_conv, replicas after %d local steps: worst %.3g" % (w.K, worst))
    assert worst < TOL_BF16
    gl, ol = g.losses(), o.losses()
    assert np.max(np.abs(gl - ol) / np.maximum(np.abs(ol), 1e-3)) < TOL_BF16
    g.meta_update()
    o.meta_update()
    e = conv_error(g.params(), o.params(), spec, verbose=True)
    print("cifar_conv, global model after the round: %.3g" % e)
    assert e < TOL_BF16
    g.close()


def test_conv_first_step_is_tight():
    """One step of one learner from bf16-exact inputs.  The step itself (replica minus start, i.e.
    -lr times the minibatch gradient) is compared tensor by tensor on ITS OWN scale, so a gradient that
    is small next to the weights cannot hide behind them."""
    g, o, spec = _setup(1, 1, 16, 8, 8, (8, 16, 16), (16, 10), 72, lr=0.1)
    w0 = g.params().astype(np.float64)
    g.local_steps()
    o.local_steps()
    e = conv_error(g.replica(0), o.replica(0), spec, verbose=True)
    assert e < 4e-3, e
    got, want = g.replica(0).astype(np.float64) - w0, o.replica(0).astype(np.float64) - w0
    for name, sl in conv_slices(spec):
        scale = float(np.max(np.abs(want[sl])))
        assert scale > 0, name
        es = float(np.max(np.abs(got[sl] - want[sl]))) / scale
        print("   step of %-8s %.3g (scale %.3g)" % (name, es, scale))
        assert es < TOL_BF16, (name, es)


def test_conv_argument_errors():
    torch = _torch()
    with pytest.raises(kavg.KavgError):
        kavg.MAvg(2, 2, 0.1, 0.5, (16, 10), 8, kavg.KAVG_BF16, conv=(8, 8, (3, 16)))       # channels not a multiple of 8
    with pytest.raises(kavg.KavgError):
        kavg.MAvg(2, 2, 0.1, 0.5, (24, 10), 8, kavg.KAVG_BF16, conv=(8, 8, (8, 16)))       # d_0 != last channel count
    g = kavg.MAvg(2, 2, 0.1, 0.5, (16, 10), 8, kavg.KAVG_BF16, conv=(8, 8, (8, 16)))
    with pytest.raises(kavg.KavgError):
        g.set_learner_momentum(0.9)
    with pytest.raises(kavg.KavgError):
        g.set_refresh(2)
    del torch
