"""Pins for the oracle's minibatch index stream and its bf16 rounding."""
import os

import numpy as np
import torch

from oracle import mavg_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = 0x9E3779B97F4A7C15
M64 = (1 << 64) - 1


def _golden_vector():
    with open(os.path.join(HERE, "golden", "splitmix64_seed1234567.txt")) as f:
        return [int(l) for l in f if l.strip() and not l.startswith("#")]


def test_splitmix64_published_vector():
    want = _golden_vector()
    states = np.array([(1234567 + (i + 1) * GOLDEN) & M64 for i in range(5)], dtype=np.uint64)
    got = [int(z) for z in O.splitmix64_output(states)]
    assert got == want


def test_indices_are_the_sequential_stream_for_learner0_step0():
    # counter c = s for j = 0, t = 0: the s-th draw is the (s+1)-th generator output
    want = _golden_vector()
    N = 1_000_003
    got = O.minibatch_indices(1234567, 0, 0, 5, N)
    assert got.dtype == np.int32
    assert list(got) == [z % N for z in want]


def test_counter_layout_against_a_sequential_generator():
    # run the stateful reference recurrence 2^16 + 4 times: the draw with
    # (j=0, t=1, s=3) must be output number 2^16 + 3 + 1.
    seed = 42
    s = seed
    outs = {}
    for i in range(1, (1 << 16) + 5):
        s = (s + GOLDEN) & M64
        if i in (1, (1 << 16) + 4):
            z = s
            z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
            z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
            outs[i] = z ^ (z >> 31)
    N = 50000
    assert O.minibatch_indices(seed, 0, 0, 1, N)[0] == outs[1] % N
    assert O.minibatch_indices(seed, 0, 1, 4, N)[3] == outs[(1 << 16) + 4] % N


def test_learner_field_sits_at_bit_40():
    # learner j, step 0, slot 0 == learner 0 stream advanced by j * 2^40 draws,
    # i.e. a generator seeded with seed + j*2^40*golden.
    seed, N = 7, 4096
    for j in (1, 5, 300):
        shifted_seed = (seed + ((j << 40) * GOLDEN)) & M64
        assert np.array_equal(O.minibatch_indices(seed, j, 3, 8, N),
                              O.minibatch_indices(shifted_seed, 0, 3, 8, N))


def test_indices_in_range_and_roughly_uniform():
    N = 97
    draws = np.concatenate([O.minibatch_indices(4001, j, t, 64, N)
                            for j in range(4) for t in range(40)])
    assert draws.min() >= 0 and draws.max() < N
    counts = np.bincount(draws, minlength=N)
    expect = draws.size / N
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 160.0          # 96 dof: mean 96, 160 is far beyond the 99.99 % point
    # streams of different learners / steps differ
    assert not np.array_equal(O.minibatch_indices(1, 0, 0, 32, N), O.minibatch_indices(1, 1, 0, 32, N))
    assert not np.array_equal(O.minibatch_indices(1, 0, 0, 32, N), O.minibatch_indices(1, 0, 1, 32, N))


# ------------------------------------------------------------------ bf16
def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (1e-6, 1e-2, 1.0, 300.0)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.rne_bf16(x.astype(np.float64)), want)


def test_bf16_ties_go_to_even():
    # 1 + 2^-8 lies exactly between 1 and 1 + 2^-7 -> even mantissa = 1.0
    assert O.rne_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # 1 + 3*2^-8 lies between 1+2^-7 (odd) and 1+2^-6 (even)
    assert O.rne_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # just above / below the tie
    assert O.rne_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1.0 + 2.0 ** -7
    assert O.rne_bf16(np.array([1.0 + 2.0 ** -8 - 2.0 ** -30]))[0] == 1.0
    assert O.rne_bf16(np.array([-(1.0 + 2.0 ** -8)]))[0] == -1.0
    assert O.rne_bf16(np.array([0.0]))[0] == 0.0
    # mantissa carry into the exponent
    assert O.rne_bf16(np.array([2.0 - 2.0 ** -9]))[0] == 2.0


def test_bf16_rounding_idempotent_monotone_and_close():
    rng = np.random.default_rng(1)
    x = np.sort(rng.standard_normal(5000))
    r = O.rne_bf16(x)
    assert np.array_equal(O.rne_bf16(r), r)
    assert np.all(np.diff(r) >= 0)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_bf16_rounding_of_constructed_ties_in_fp32_bit_patterns():
    """Exact ties between two bf16 neighbours (low 16 bits of the fp32 pattern = 0x8000) go to the
    neighbour whose last kept bit is 0, for 2000 consecutive mantissas and both signs; checked on
    the bit patterns, without the library conversion."""
    keep = np.arange(1, 2001, dtype=np.uint32) + np.uint32(0x3F80)          # top 16 bits
    ties = ((keep << np.uint32(16)) | np.uint32(0x8000)).view(np.float32)
    even = np.where(keep & 1, keep + 1, keep).astype(np.uint32)                # odd -> up, even -> stay
    want = (even << np.uint32(16)).view(np.float32).astype(np.float64)
    assert np.array_equal(O.rne_bf16(ties.astype(np.float64)), want)
    assert np.array_equal(O.rne_bf16(-ties.astype(np.float64)), -want)
