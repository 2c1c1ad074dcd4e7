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


def worst_error(got, want, dims):
    """Largest per-tensor error over the weight matrices and over bias vectors that have moved
    away from zero (a bias tensor that is still ~0 has no scale to be relative to: it is
    measured against the scale of its layer's weights instead)."""
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


def flat_error(got, want):
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - want)) / max(float(np.max(np.abs(want))), 1e-30))
