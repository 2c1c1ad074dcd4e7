"""Helpers shared by the parity tests (no arithmetic of the method)."""
import numpy as np


def layer_slices(dims):
    out, o = [], 0
    for l in range(1, len(dims)):
        out.append(("W%d" % l, slice(o, o + dims[l] * dims[l - 1])))
        o += dims[l] * dims[l - 1]
        out.append(("b%d" % l, slice(o, o + dims[l])))
        o += dims[l]
    return out


def tensor_errors(got, want, dims):
    """Per tensor T in {W_l, b_l}: max_i |got_i - want_i| / max(max_i |want_i|, 1e-30)."""
    errs = {}
    for name, sl in layer_slices(dims):
        w = np.asarray(want[sl], dtype=np.float64)
        g = np.asarray(got[sl], dtype=np.float64)
        errs[name] = float(np.max(np.abs(g - w)) / max(float(np.max(np.abs(w))), 1e-30))
    return errs


def worst_error(got, want, dims, verbose=False):
    """Largest per-tensor relative error, every W_l and b_l measured against its own largest
    magnitude in the oracle.  A bias tensor that is still numerically zero (max |b| < 1e-6: biases
    start at 0) has no scale of its own and is measured against its layer's weights instead."""
    worst = 0.0
    sl = dict(layer_slices(dims))
    for l in range(1, len(dims)):
        w = np.asarray(want[sl["W%d" % l]], dtype=np.float64)
        g = np.asarray(got[sl["W%d" % l]], dtype=np.float64)
        wscale = float(np.max(np.abs(w)))
        ew = float(np.max(np.abs(g - w))) / max(wscale, 1e-30)
        b = np.asarray(want[sl["b%d" % l]], dtype=np.float64)
        gb = np.asarray(got[sl["b%d" % l]], dtype=np.float64)
        bscale = float(np.max(np.abs(b)))
        if bscale < 1e-6:
            bscale = wscale
        eb = float(np.max(np.abs(gb - b))) / max(bscale, 1e-30)
        if verbose:
            print("    W%d %.3g  b%d %.3g" % (l, ew, l, eb))
        worst = max(worst, ew, eb)
    return worst


def replica_error(got, want, dims):
    """Error of ONE learner's replica between two meta steps (an intermediate state of Algorithm 1;
    the stated tolerance is for the parameters after a meta round, see worst_error).  Weights as in
    worst_error.  A bias element of a single learner is a sum over the ~B/2 active samples of one
    minibatch, so ONE ReLU mask that falls the other way (the two sides accumulate in different
    precision) moves it by about (B/2)^-1/2 of itself -- several per cent, however exact the
    arithmetic.  A bias tensor is therefore measured against the larger of its own scale and its
    layer's weight scale: the scale on which it enters z = W a + b."""
    worst = 0.0
    sl = dict(layer_slices(dims))
    for l in range(1, len(dims)):
        w = np.asarray(want[sl["W%d" % l]], dtype=np.float64)
        g = np.asarray(got[sl["W%d" % l]], dtype=np.float64)
        wscale = float(np.max(np.abs(w)))
        worst = max(worst, float(np.max(np.abs(g - w))) / max(wscale, 1e-30))
        b = np.asarray(want[sl["b%d" % l]], dtype=np.float64)
        gb = np.asarray(got[sl["b%d" % l]], dtype=np.float64)
        bscale = max(float(np.max(np.abs(b))), wscale)
        worst = max(worst, float(np.max(np.abs(gb - b))) / max(bscale, 1e-30))
    return worst


def matmul_in_float32(a, b):
    """numpy's float32 product of the same operands, returned as float64: what separates a CPU
    "twin" of the oracle that accumulates in fp32 from the oracle itself."""
    return (np.asarray(a, dtype=np.float32) @ np.asarray(b, dtype=np.float32)).astype(np.float64)


def bf16_plane_bits(x32):
    """The 16-bit patterns the library documents for its bf16 copies of fp32 values (include/kavg.h):
    nearest bf16, exact ties away from zero, i.e. the top half of (pattern + 0x8000)."""
    bits = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((bits + 0x8000) >> 16) & 0xFFFF).astype(np.uint16)


def flat_error(got, want):
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / max(float(np.max(np.abs(want))), 1e-30))
