"""CPU pins of the oracle's expert-diversify step (Stage 1; Algorithm 1's loop e_i <- diversify(e, i))."""
import os

import numpy as np

from oracle import evomoe_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _shared(F=48, d=40, seed=5):
    rng = np.random.default_rng(seed)
    W1 = rng.standard_normal((F, d)).astype(np.float32) + 3.0     # no zeros of its own
    W2 = rng.standard_normal((d, F)).astype(np.float32) + 3.0
    b1 = rng.standard_normal(F).astype(np.float32)
    b2 = rng.standard_normal(d).astype(np.float32)
    return W1, b1, W2, b2


def test_generator_reproduces_the_published_vectors():
    want = [int(l) for l in open(os.path.join(HERE, "golden", "splitmix64_seed1234567.txt")) if not l.startswith("#")]
    got = [int(orc.splitmix64_output(1234567, n)) for n in range(len(want))]
    assert got == want
    assert [int(v) for v in orc.splitmix64_output(1234567, np.arange(5))] == want      # array form


def test_ratio_zero_copies_and_ratio_one_clears():
    W1, b1, W2, b2 = _shared()
    o = orc.diversify(W1, b1, W2, b2, 5, seed=9, mask_ratio=0.0)
    for i in range(5):          # no masking: every expert IS the shared expert (Algorithm 1 before line "diversify")
        assert np.array_equal(o[0][i], W1) and np.array_equal(o[2][i], W2)
        assert np.array_equal(o[1][i], b1) and np.array_equal(o[3][i], b2)
    z = orc.diversify(W1, b1, W2, b2, 3, seed=9, mask_ratio=1.0)
    assert not z[0].any() and not z[2].any()
    assert np.array_equal(z[1][2], b1) and np.array_equal(z[3][0], b2)                  # biases are never masked


def test_masked_fraction_kept_values_and_diversity():
    W1, b1, W2, b2 = _shared(F=256, d=192)
    E, ratio = 6, 0.3
    oW1, ob1, oW2, ob2 = orc.diversify(W1, b1, W2, b2, E, seed=2021, mask_ratio=ratio)
    n = W1.size
    sd = np.sqrt(ratio * (1 - ratio) / n)
    for i in range(E):
        for got, src in ((oW1[i], W1), (oW2[i], W2)):
            zero = got == 0
            assert abs(zero.mean() - ratio) < 5 * sd                    # a binomial fraction of the weights is masked
            assert np.array_equal(got[~zero], src[~zero])               # the rest are the shared expert's, bit for bit
    # "different masks": any two experts' masks agree only as often as independent draws would
    for i in range(E):
        for j in range(i + 1, E):
            agree = ((oW1[i] == 0) == (oW1[j] == 0)).mean()
            assert abs(agree - (ratio ** 2 + (1 - ratio) ** 2)) < 0.02
    # W1's and W2's masks are different draws too (same shape after a transpose: compare flat)
    assert ((oW1[0] == 0).ravel() != (oW2[0] == 0).ravel()).mean() > 0.3
    # deterministic in (seed, ratio); another seed gives another mask
    again = orc.diversify(W1, b1, W2, b2, E, seed=2021, mask_ratio=ratio)
    assert np.array_equal(again[0], oW1) and np.array_equal(again[2], oW2)
    other = orc.diversify(W1, b1, W2, b2, E, seed=2022, mask_ratio=ratio)
    assert ((other[0] == 0) != (oW1 == 0)).mean() > 0.3


def test_masks_are_nested_in_the_ratio_and_follow_the_counter_layout():
    """A weight masked at ratio r stays masked at every larger ratio (one draw per weight, compared with a
    threshold), and the draw of weight j of tensor t of expert i is output number (t << 62 | i << 48 | j)."""
    keep_lo = orc.diversify_keep_mask(7, 0.2, 1, 3, 5000)
    keep_hi = orc.diversify_keep_mask(7, 0.6, 1, 3, 5000)
    assert not (keep_hi & ~keep_lo).any()
    j = 1234
    draw = int(orc.splitmix64_output(7, (1 << 62) | (3 << 48) | j)) >> 40
    assert bool(keep_lo[j]) == (draw >= int(np.floor(np.float64(np.float32(0.2)) * 2 ** 24)))
