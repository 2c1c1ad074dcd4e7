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


def test_weight_rounding_is_nearest_with_ties_away_from_zero():
    # exact ties go away from zero, in both signs ...
    assert O.rna_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0 + 2.0 ** -7
    assert O.rna_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert O.rna_bf16(np.array([-(1.0 + 2.0 ** -8)]))[0] == -(1.0 + 2.0 ** -7)
    assert O.rna_bf16(np.array([2.0 - 2.0 ** -9]))[0] == 2.0            # carries into the exponent
    assert O.rna_bf16(np.array([0.0]))[0] == 0.0
    # ... everything else is plain nearest: same as ties-to-even off the ties
    rng = np.random.default_rng(5)
    x = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))
    assert np.array_equal(O.rna_bf16(x), O.rne_bf16(x))
    # on float32 inputs it is "add half a unit to the bit pattern, keep the top 16 bits"
    x32 = (rng.standard_normal(100000) * np.exp(rng.uniform(-10, 10, 100000))).astype(np.float32)
    ties = (np.arange(1, 2001, dtype=np.uint32) * np.uint32(0x10000) + np.uint32(0x3F808000)).view(np.float32)
    x32 = np.concatenate([x32, ties, -ties])
    bits = x32.view(np.uint32).astype(np.uint64)
    want = (((bits + 0x8000) >> 16) << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    assert np.array_equal(O.rna_bf16(x32.astype(np.float64)), want)
    r = O.rna_bf16(x)
    assert np.array_equal(O.rna_bf16(r), r)                                # idempotent
