"""Seeded synthetic inputs, shared by the CPU oracle's tests and the GPU path.

Nothing here belongs to the method (no SGD, no averaging, no momentum): the
module only manufactures datasets, teacher labels, initial parameters and the
meta-only replica sets, all on the host from numpy's seeded ``Generator``.
The same arrays are handed to the oracle and to the HIP library, so a choice
made here can never hide a disagreement between the two.

Recipe (stands in for CIFAR-10 / ImageNet-1K of the paper's Section 4, which
are not available -- only shape and first/second moments are kept):
  * inputs x ~ N(0,1), i.i.d. per feature (a per-channel-normalised image of
    3x32x32 flattened has d_0 = 3072 features);
  * labels = argmax of a fixed random ReLU teacher MLP d_0-256-C (He-normal
    weights, no bias), evaluated in fp64, lowest index on ties; optionally a
    fraction of labels is replaced by a uniformly drawn *different* class;
  * initial parameters: He-normal W_l ~ N(0, 2/d_{l-1}) for every layer, b = 0;
  * for bf16 workloads the dataset is *defined* on the bf16 grid: every x is
    snapped to the nearest bf16 value here, once, so both sides start from
    bit-identical operands.
"""
import numpy as np

from .configs import Workload, num_params, layer_offsets


def snap_to_bf16_grid(x32: np.ndarray):
    """Return (bits uint16, value float32) of the nearest-even bf16 of x32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    bits = r.astype(np.uint16)
    val = (r << np.uint32(16)).view(np.float32)
    return bits, val


def he_normal_params(dims, seed) -> np.ndarray:
    """Flat fp32 vector: W_l ~ N(0, 2/d_{l-1}) row-major [d_l][d_{l-1}], b_l = 0."""
    rng = np.random.default_rng(seed)
    w = np.zeros(num_params(dims), dtype=np.float32)
    for l, (wo, bo) in enumerate(layer_offsets(dims), start=1):
        fan_in = dims[l - 1]
        w[wo:bo] = rng.standard_normal(dims[l] * fan_in, dtype=np.float32) * np.float32(
            np.sqrt(2.0 / fan_in))
    return w


def teacher_labels(X32: np.ndarray, n_classes: int, hidden: int, seed: int,
                   chunk: int = 8192) -> np.ndarray:
    rng = np.random.default_rng(seed)
    d0 = X32.shape[1]
    T1 = rng.standard_normal((d0, hidden)) * np.sqrt(2.0 / d0)
    T2 = rng.standard_normal((hidden, n_classes)) * np.sqrt(2.0 / hidden)
    y = np.empty(X32.shape[0], dtype=np.int32)
    for s in range(0, X32.shape[0], chunk):
        h = np.maximum(X32[s:s + chunk].astype(np.float64) @ T1, 0.0)
        y[s:s + chunk] = np.argmax(h @ T2, axis=1).astype(np.int32)
    return y


def flip_labels(y: np.ndarray, n_classes: int, frac: float, seed: int) -> np.ndarray:
    """Replace each label independently with probability frac by another class."""
    if frac <= 0.0:
        return y
    rng = np.random.default_rng(seed)
    hit = rng.random(y.shape[0]) < frac
    shift = rng.integers(1, n_classes, size=y.shape[0], dtype=np.int32)
    out = y.copy()
    out[hit] = (y[hit] + shift[hit]) % n_classes
    return out


def make_dataset(N, d0, n_classes, *, bf16, seed_data, seed_teacher,
                 teacher_hidden=256, label_flip=0.0, seed_noise=0):
    """Returns dict(X32 [N][d0] float32, Xbits uint16 or None, y int32 [N])."""
    rng = np.random.default_rng(seed_data)
    X32 = rng.standard_normal((N, d0), dtype=np.float32)
    bits = None
    if bf16:
        bits, X32 = snap_to_bf16_grid(X32)
    y = teacher_labels(X32, n_classes, teacher_hidden, seed_teacher)
    y = flip_labels(y, n_classes, label_flip, seed_noise)
    return {"X32": X32, "Xbits": bits, "y": y}


def make_workload_inputs(w: Workload, N=None):
    """Dataset and initial parameters of a training workload (N may be reduced)."""
    N = w.N if N is None else N
    data = make_dataset(N, w.dims[0], w.n_classes, bf16=(w.dtype == 1),
                        seed_data=w.seeds["data"], seed_teacher=w.seeds["teacher"],
                        teacher_hidden=w.teacher_hidden, label_flip=w.label_flip,
                        seed_noise=w.seeds["noise"])
    data["w0"] = he_normal_params(w.dims, w.seeds["init"])
    return data


def make_image_dataset(N, H, W, c_real, c_pad, n_classes, *, seed_data, seed_texture):
    """Textured-noise images for the convolutional workload, channels last.

    Class k owns a random 3x3 filter bank F_k [c_real][3][3][c_real]; an image of class k is white
    Gaussian noise filtered with F_k (circular shifts), so classes differ in their local statistics,
    which is what 3x3 convolutions followed by a mean over the positions can pick up.  Channels
    c_real..c_pad-1 are zero (the kernels want channel counts that are multiples of 8).
    Returns dict(X32 [N][H*W*c_pad] float32 on the bf16 grid, Xbits uint16, y int32 [N])."""
    rng = np.random.default_rng(seed_data)
    y = rng.integers(0, n_classes, size=N).astype(np.int32)
    F = np.random.default_rng(seed_texture).standard_normal((n_classes, c_real, 3, 3, c_real)) / np.sqrt(9.0 * c_real)
    X = np.zeros((N, H, W, c_pad), dtype=np.float32)
    bits = np.zeros((N, H, W, c_pad), dtype=np.uint16)
    chunk = 4096
    for s in range(0, N, chunk):
        noise = rng.standard_normal((min(chunk, N - s), H, W, c_real))
        out = np.zeros_like(noise)
        yc = y[s:s + chunk]
        for kh in range(3):
            for kw in range(3):
                shifted = np.roll(noise, (1 - kh, 1 - kw), axis=(1, 2))
                for k in range(n_classes):
                    sel = yc == k
                    part = shifted[sel]
                    out[sel] += (part.reshape(-1, c_real) @ F[k, :, kh, kw, :].T).reshape(part.shape)
        b, v = snap_to_bf16_grid((out * 1.5).astype(np.float32))
        X[s:s + chunk, :, :, :c_real] = v
        bits[s:s + chunk, :, :, :c_real] = b
    return {"X32": X.reshape(N, -1), "Xbits": bits.reshape(N, -1), "y": y}


def he_normal_conv_params(channels, dims, seed) -> np.ndarray:
    """Flat fp32 vector of a convolutional net: per 3x3 convolution W ~ N(0, 2/(9 c_in)) laid out
    [c_out][3][3][c_in], then its zero bias; then the MLP as in he_normal_params."""
    rng = np.random.default_rng(seed)
    pieces = []
    for t in range(1, len(channels)):
        fan_in = 9 * channels[t - 1]
        pieces.append(rng.standard_normal(channels[t] * fan_in, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in)))
        pieces.append(np.zeros(channels[t], dtype=np.float32))
    pieces.append(he_normal_params(dims, seed + 1))
    return np.concatenate(pieces)


def make_conv_workload_inputs(w: Workload, N=None):
    """Images, labels and initial parameters of a convolutional workload (N may be reduced)."""
    N = w.N if N is None else N
    data = make_image_dataset(N, w.H, w.W, w.c_real, w.channels[0], w.n_classes,
                              seed_data=w.seeds["data"], seed_texture=w.seeds["teacher"])
    data["w0"] = he_normal_conv_params(w.channels, w.dims, w.seeds["init"])
    return data


def make_meta_only_inputs(P, n, seed, base_std=0.05, pert_std=1e-3, v_std=1e-3):
    """Meta-only workload: global model = base ~ N(0, base_std^2); replica j =
    base + N(0, pert_std^2); momentum buffer ~ N(0, v_std^2). All fp32."""
    rng = np.random.default_rng(seed)
    base = rng.standard_normal(n, dtype=np.float32) * np.float32(base_std)
    v = rng.standard_normal(n, dtype=np.float32) * np.float32(v_std)
    reps = np.empty((P, n), dtype=np.float32)
    for j in range(P):
        reps[j] = base + rng.standard_normal(n, dtype=np.float32) * np.float32(pert_std)
    return {"w_tilde": base, "v": v, "replicas": reps}
