"""Plain CPU oracle of M-AVG (K-step averaging SGD with block momentum).

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
of what the GPU library has to compute.  It is imported by the tests, by the
smoke check and by the benchmark's CPU-baseline leg, never by the product
path, and it shares no code with the HIP kernels or their Python binding.

What it follows
---------------
* Algorithm 1 (M-AVG) of the paper, Section 2: every one of P learners starts
  a round at the global model w~_n, takes K minibatch-SGD steps
      w <- w - (gamma/B) * sum_s grad F(w; xi_s),
  then the meta level forms
      a = (1/P) sum_j w^j,   d = a - w~_n,   v <- mu v + d,   w~_{n+1} = w~_n + v,
  and the learners restart from w~_{n+1}.
* The objective is the one of Section 2, F(w) = (1/n) sum_i loss(y_i, f(x_i, w)),
  instantiated on an MLP with ReLU hidden layers, affine layers with bias, and
  softmax cross-entropy, mean over the minibatch.

An iteration has no closed form to fall back on, so the oracle takes the
algorithm's steps in the paper's order.  All state and arithmetic are float64.
Matrix products use numpy's matmul as a library step; nothing is blocked,
fused or reordered.

Readings where the paper is silent (each repeated in the design notes):
* step size: gamma_n of Algorithm 1 and eta_n of eq. (2) are one fixed lr;
* "randomly sample a mini-batch": i.i.d. uniform with replacement over the
  whole data set, from a counter-based stream (SplitMix64, see below);
* ReLU derivative at 0 is 0;
* momentum exactly as printed: no dampening, no Nesterov, block step 1;
  v persists across rounds;
* 1/P is applied as a multiplication of the sum by the reciprocal.
* learner-level momentum (Section 2 only says that momentum "can also" be added
  at the learner level): heavy-ball inside each learner, u <- beta u + g,
  w <- w - lr u, with g the mean minibatch gradient; every learner keeps its
  own u across meta rounds (it is not reset when the learner restarts from
  w~), u = 0 initially.  beta = 0 is Algorithm 1 as printed.
* mixed precision ("bf16" mode): the operands of every matrix product are
  rounded to bf16, nearest with ties to even (the IEEE default conversion):
  the weights as used in forward and data-gradient products, the stored
  hidden activations, and the gradient dZ_l that flows backward through
  layer l (used for the weight gradient, the bias gradient and the data
  gradient alike).  Accumulation, logits, softmax,
  loss, the SGD update of the master parameters and the whole meta step stay
  in full precision.  The data set itself is given on the bf16 grid.

Pins (tests/test_oracle_*.py): SplitMix64 published vector; bf16 rounding vs
constructed ties and a library conversion; backprop vs central differences,
vs a library autograd, vs a hand-expanded scalar net; K=1/mu=0 = synchronous
SGD at batch P*B; P=1/mu=0 = plain SGD; lr=0 and identical-replica identities;
d = -lr*G_n of eq. (2); the z-sequence identity of the proof of Theorem 1;
the geometric closed form of v.  The convergence bounds of Theorem 1 and
Lemmas 1-5 are not checked anywhere: parity unpinned for those (they are
inequalities with unknown constants, not part of the computation).
"""
import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


# --------------------------------------------------------------------------
# minibatch sampling (Algorithm 1: "randomly sample a mini-batch of size B")
# --------------------------------------------------------------------------
def splitmix64_output(state: np.ndarray) -> np.ndarray:
    """Output function of SplitMix64 (Steele, Lea, Flood 2014; Vigna's
    reference implementation) applied to already-advanced 64-bit states."""
    z = state.astype(np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def minibatch_indices(seed: int, j: int, t: int, B: int, N: int) -> np.ndarray:
    """Sample indices xi_{t,s}^j, s = 0..B-1, of learner j at its t-th local step.

    Counter c = j*2^40 + t*2^16 + s (j < 2^24, t < 2^24, s < 2^16); the draw is
    the (c+1)-th output of a SplitMix64 generator seeded with `seed`, i.e. the
    output function applied to seed + (c+1)*golden (mod 2^64), reduced mod N.
    """
    assert 0 <= j < (1 << 24) and 0 <= t < (1 << 24) and 0 < B <= (1 << 16)
    out = np.empty(B, dtype=np.int32)
    for s in range(B):
        c = (j << 40) | (t << 16) | s
        state = (seed + (c + 1) * _GOLDEN) & _MASK64
        z = int(splitmix64_output(np.array([state], dtype=np.uint64))[0])
        out[s] = z % N
    return out


# --------------------------------------------------------------------------
# bf16 rounding (mixed-precision reading)
# --------------------------------------------------------------------------
def rne_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bf16 value (8 significant bits, ties to even) of each float64.
    Written from the definition: x = m * 2^e with 0.5 <= |m| < 1, keep 8 bits
    of m.  Normal range only (no overflow / subnormal handling is needed for
    the magnitudes that occur)."""
    m, e = np.frexp(np.asarray(x, dtype=np.float64))
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


def _identity(x):
    return x


# --------------------------------------------------------------------------
# the model: MLP, ReLU, softmax cross-entropy  (Section 2, F(w))
# --------------------------------------------------------------------------
def num_params(dims) -> int:
    return sum(dims[l] * dims[l - 1] + dims[l] for l in range(1, len(dims)))


def unpack(w: np.ndarray, dims):
    """Views (W_l [d_l][d_{l-1}], b_l [d_l]) for l = 1..L into the flat vector:
    per layer the weight matrix row-major (output-major), then the bias."""
    Ws, bs, o = [], [], 0
    for l in range(1, len(dims)):
        Ws.append(w[o:o + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1]))
        o += dims[l] * dims[l - 1]
        bs.append(w[o:o + dims[l]])
        o += dims[l]
    return Ws, bs


def forward(Ws, bs, A0, q=_identity):
    """Z_l = A_{l-1} W_l^T + b_l; A_l = q(max(Z_l, 0)) for hidden layers.
    Ws are the weights as used in the products (already rounded if needed)."""
    Zs, As = [], [A0]
    L = len(Ws)
    for l in range(L):
        Z = As[-1] @ Ws[l].T + bs[l]
        Zs.append(Z)
        if l < L - 1:
            As.append(q(np.maximum(Z, 0.0)))
    return Zs, As


def softmax_cross_entropy(ZL, y):
    """Per-sample loss -log softmax(Z_L)[y] and its gradient w.r.t. Z_L for the
    MEAN over the batch: dZ_L = (softmax(Z_L) - onehot(y)) / B."""
    Bn = ZL.shape[0]
    m = ZL.max(axis=1, keepdims=True)
    e = np.exp(ZL - m)
    S = e.sum(axis=1, keepdims=True)
    p = e / S
    rows = np.arange(Bn)
    loss = -(ZL[rows, y] - m[:, 0] - np.log(S[:, 0]))
    onehot = np.zeros_like(p)
    onehot[rows, y] = 1.0
    return loss, (p - onehot) / Bn


def backward(Ws, Zs, As, dZL, q=_identity):
    """Gradients of the mean minibatch loss: gW_l = dZ_l^T A_{l-1},
    gb_l = column sums of dZ_l, dZ_{l-1} = (dZ_l W_l) * [Z_{l-1} > 0]."""
    L = len(Ws)
    gWs, gbs = [None] * L, [None] * L
    dZ = q(dZL)
    for l in range(L - 1, -1, -1):
        gWs[l] = dZ.T @ As[l]
        gbs[l] = dZ.sum(axis=0)
        if l > 0:
            dA = dZ @ Ws[l]
            dZ = q(dA * (Zs[l - 1] > 0.0))
    return gWs, gbs


def minibatch_gradient(w, dims, Xb, yb, bf16=False):
    """(mean loss, flat gradient) of the minibatch objective at w."""
    q = rne_bf16 if bf16 else _identity
    Ws, bs = unpack(w, dims)
    Wq = [q(W) for W in Ws]
    Zs, As = forward(Wq, bs, Xb, q)
    loss, dZL = softmax_cross_entropy(Zs[-1], yb)
    gWs, gbs = backward(Wq, Zs, As, dZL, q)
    g = np.concatenate([np.concatenate([gW.ravel(), gb]) for gW, gb in zip(gWs, gbs)])
    return float(loss.mean()), g


# --------------------------------------------------------------------------
# meta level (Algorithm 1, the four assignments after the K local steps)
# --------------------------------------------------------------------------
def meta_step(w_tilde, v, replicas, mu):
    """Returns (w~_{n+1}, v_{n+1}) from w~_n, v_n and the P learner results."""
    P = replicas.shape[0]
    a = replicas.sum(axis=0) * (1.0 / P)
    d = a - w_tilde
    v_new = mu * v + d
    return w_tilde + v_new, v_new


class MAvgOracle:
    """State machine with the same call names as the C library."""

    def __init__(self, P, K, lr, mu, dims, B, bf16=False, index_seed=0, learner_momentum=0.0,
                 gradient=None, n_params=None):
        """gradient / n_params: another instance of the objective F(w) of Section 2 than the MLP
        (a function (w, Xb, yb, bf16) -> (mean loss, flat gradient) and its parameter count);
        Algorithm 1 itself does not depend on the model."""
        assert P >= 1 and K >= 1 and B >= 1 and lr >= 0.0 and 0.0 <= mu < 1.0
        assert 0.0 <= learner_momentum < 1.0
        self.beta = float(learner_momentum)
        self.P, self.K, self.lr, self.mu = P, K, float(lr), float(mu)
        self.dims, self.B, self.bf16, self.seed = tuple(dims), B, bool(bf16), int(index_seed)
        self.gradient = gradient
        self.n = num_params(self.dims) if n_params is None else int(n_params)
        self.w_tilde = None
        self.v = None
        self.reps = None
        self.X = self.y = None
        self.user_idx = None
        self.t0 = 0            # local steps every learner has taken so far
        self.round = 0
        self.last_idx = None
        self.last_losses = None
        self.grad_sum = None   # sum over learners and local steps of minibatch gradients

    def set_params(self, w0):
        self.w_tilde = np.asarray(w0, dtype=np.float64).copy()
        assert self.w_tilde.shape == (self.n,)
        self.v = np.zeros(self.n)
        self.reps = np.tile(self.w_tilde, (self.P, 1))
        self.u = np.zeros((self.P, self.n)) if self.beta > 0.0 else None
        self.t0 = 0
        self.round = 0

    def set_state(self, w, v, round_):
        self.w_tilde = np.asarray(w, dtype=np.float64).copy()
        self.v = np.asarray(v, dtype=np.float64).copy()
        self.reps = np.tile(self.w_tilde, (self.P, 1))
        self.u = np.zeros((self.P, self.n)) if self.beta > 0.0 else None
        self.round = int(round_)
        self.t0 = self.round * self.K

    def set_data(self, X, y):
        self.X = np.asarray(X)
        self.y = np.asarray(y)
        assert self.gradient is not None or self.X.shape[1] == self.dims[0]

    def set_indices(self, idx):
        """idx [P][K][B] to use in every following local_steps call, or None
        to draw from the seeded stream."""
        self.user_idx = None if idx is None else np.asarray(idx, dtype=np.int32).reshape(
            self.P, self.K, self.B)

    def _learner_steps(self, j):
        """The K local steps of learner j on its own replica (Algorithm 1, inner loop).  Touches
        nothing but replica j (and velocity j); returns its indices, losses and gradient sum."""
        N = self.X.shape[0]
        idx = np.zeros((self.K, self.B), dtype=np.int32)
        losses = np.zeros(self.K)
        gsum = np.zeros(self.n)
        w = self.reps[j]
        for k in range(self.K):
            if self.user_idx is not None:
                ib = self.user_idx[j, k]
            else:
                ib = minibatch_indices(self.seed, j, self.t0 + k, self.B, N)
            idx[k] = ib
            Xb = self.X[ib].astype(np.float64)
            yb = self.y[ib]
            if self.gradient is not None:
                loss, g = self.gradient(w, Xb, yb, self.bf16)
            else:
                loss, g = minibatch_gradient(w, self.dims, Xb, yb, self.bf16)
            losses[k] = loss
            gsum += g
            if self.beta > 0.0:
                self.u[j] = self.beta * self.u[j] + g
                w -= self.lr * self.u[j]
            else:
                w -= self.lr * g      # in place: w is a view of replica j
        return idx, losses, gsum

    def local_steps(self, learners=None, workers=1):
        """K minibatch-SGD steps on every learner (or only on the listed ones).  The learners of
        Algorithm 1 work independently between two meta steps ("in parallel"), so with workers > 1
        they are walked by that many threads; nothing a learner computes depends on that."""
        todo = list(range(self.P) if learners is None else learners)
        if workers > 1 and len(todo) > 1:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=workers) as pool:
                results = list(pool.map(self._learner_steps, todo))
        else:
            results = [self._learner_steps(j) for j in todo]
        idx = np.zeros((self.P, self.K, self.B), dtype=np.int32)
        losses = np.zeros((self.K, self.P))
        self.grad_sum = np.zeros(self.n)
        for j, (idx_j, losses_j, gsum_j) in zip(todo, results):
            idx[j] = idx_j
            losses[:, j] = losses_j
            self.grad_sum += gsum_j
        self.t0 += self.K
        self.last_idx, self.last_losses = idx, losses

    def meta_update(self):
        self.w_tilde, self.v = meta_step(self.w_tilde, self.v, self.reps, self.mu)
        self.reps = np.tile(self.w_tilde, (self.P, 1))
        self.round += 1

    def params(self):
        return self.w_tilde.copy()

    def momentum(self):
        return self.v.copy()

    def replica(self, j):
        return self.reps[j].copy()

    def velocity(self, j):
        return self.u[j].copy()

    def losses(self):
        return self.last_losses.copy()

    def indices(self):
        return self.last_idx.copy()
