"""Workload table: the synthetic configurations the M-AVG hot path is
checked and measured on (five MLP / flat-vector ones and a convolutional one).

Each entry fixes the hyper-parameters of Algorithm 1 (P learners, K local
steps, batch B, step size lr, block momentum mu, number of meta rounds), the
MLP the learners train, and the recipe of the synthetic data that stands in
for the image-classification sets the paper trained on (Section 4: CIFAR-10,
ImageNet-1K -- neither is available, only their shapes are kept).

This module holds no arithmetic of the method; it is shared by the tests, the
benchmark and the seeded generators in ``synth``.
"""
from dataclasses import dataclass, field
from typing import Tuple

DTYPE_FP32 = 0   # fp32 everywhere
DTYPE_BF16 = 1   # bf16 GEMM operands, fp32 accumulation, fp32 master parameters


@dataclass(frozen=True)
class Workload:
    name: str
    P: int                  # learners ("processors", Section 2 notation)
    K: int                  # local SGD steps per meta round
    B: int                  # per-learner minibatch size
    mu: float               # block momentum parameter
    lr: float               # step size (gamma_n = eta_n, held fixed)
    rounds: int             # meta rounds N
    dims: Tuple[int, ...]   # d_0, ..., d_L of the MLP (empty: flat vector)
    dtype: int
    N: int                  # dataset size
    teacher_hidden: int = 256
    label_flip: float = 0.0  # fraction of labels replaced by a different class
    flat_n: int = 0         # meta-only workload: length of the flat vector
    seeds: dict = field(default_factory=dict)
    # convolutional workload: 3x3 convolutions on H x W images in front of the MLP
    # (channels[0] = input channels padded to a multiple of 8, of which c_real carry data)
    H: int = 0
    W: int = 0
    channels: Tuple[int, ...] = ()
    c_real: int = 0

    @property
    def n_classes(self) -> int:
        return self.dims[-1]


def _seeds(c: int) -> dict:
    return {"data": 1000 + c, "teacher": 2000 + c, "init": 3000 + c,
            "index": 4000 + c, "noise": 5000 + c}


TINY = Workload("tiny", P=4, K=4, B=32, mu=0.9, lr=0.05, rounds=20,
                dims=(3072, 64, 10), dtype=DTYPE_FP32, N=4096, seeds=_seeds(1))

CIFAR_MLP = Workload("cifar_mlp", P=16, K=8, B=128, mu=0.9, lr=0.1, rounds=50,
                     dims=(3072, 1024, 1024, 10), dtype=DTYPE_BF16, N=50000,
                     seeds=_seeds(2))

NOISY_WIDE = Workload("noisy_wide", P=32, K=16, B=64, mu=0.9, lr=0.05, rounds=30,
                      dims=(3072, 4096, 4096, 10), dtype=DTYPE_BF16, N=100000,
                      label_flip=0.1, seeds=_seeds(3))

META_ONLY = Workload("meta_only", P=64, K=0, B=0, mu=0.9, lr=0.0, rounds=200,
                     dims=(), dtype=DTYPE_FP32, N=0, flat_n=11_173_962,
                     seeds=_seeds(4))

LARGE = Workload("large", P=8, K=32, B=256, mu=0.95, lr=0.2, rounds=10,
                 dims=(3072, 4096, 4096, 1000), dtype=DTYPE_BF16, N=200000,
                 seeds=_seeds(5))

# CIFAR-shaped images (32x32x3, Section 4) through three 3x3 convolutions, the mean over the
# positions and a small MLP
CIFAR_CONV = Workload("cifar_conv", P=16, K=8, B=64, mu=0.9, lr=0.05, rounds=20,
                      dims=(128, 256, 10), dtype=DTYPE_BF16, N=10000, seeds=_seeds(6),
                      H=32, W=32, channels=(8, 32, 64, 128), c_real=3)

WORKLOADS = {w.name: w for w in (TINY, CIFAR_MLP, NOISY_WIDE, META_ONLY, LARGE)}
CONV_WORKLOADS = {w.name: w for w in (CIFAR_CONV,)}


def conv_num_params(channels, dims) -> int:
    """Flat length of a convolutional net: per convolution W [c_out][3][3][c_in] and bias, then the MLP."""
    return sum(channels[t] * 9 * channels[t - 1] + channels[t] for t in range(1, len(channels))) + num_params(dims)


def conv_flops_per_learner_step(H, W, channels, dims, B) -> int:
    """Dense-product flops of one learner step: per convolution forward, weight gradient and (from the
    second one on) data gradient, 2 flops per weight and position each; the MLP with a data gradient
    in every layer (its first layer hands the gradient of the pooled vector on)."""
    rows = B * H * W
    tot = 0
    for t in range(1, len(channels)):
        tot += (6 if t > 1 else 4) * rows * 9 * channels[t - 1] * channels[t]
    for l in range(1, len(dims)):
        tot += 6 * B * dims[l] * dims[l - 1]
    return tot


def num_params(dims) -> int:
    """Length of the flat parameter vector: per layer W_l [d_l][d_{l-1}] then b_l [d_l]."""
    return sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims)))


def layer_offsets(dims):
    """[(w_off, b_off)] of every layer inside the flat parameter vector."""
    offs, o = [], 0
    for l in range(1, len(dims)):
        w = o
        o += dims[l] * dims[l - 1]
        b = o
        o += dims[l]
        offs.append((w, b))
    return offs


def flops_per_learner_step(dims, B) -> int:
    """Forward 2, weight-gradient 2, data-gradient 2 flops per weight and
    sample; the first layer has no data gradient."""
    tot = 0
    for l in range(1, len(dims)):
        tot += 6 * B * dims[l] * dims[l - 1]
    tot -= 2 * B * dims[1] * dims[0]
    return tot
