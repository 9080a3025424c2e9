"""Host-side check of the arithmetic fact the build's update step relies on when it sums a large
cluster in several runs instead of member by member: if the addends are storage-type values whose
exponent fields span emax - emin and there are n of them, with
    emax - emin + ceil(log2 n) <= 52 - (mantissa bits of the storage type),
then no fp64 addition of any subset in any order rounds, so every summation order gives the exact
sum.  Beyond that bound orders can differ, which is why the kernel then falls back to the
reference's one-by-one order."""
from fractions import Fraction

import numpy as np


def _bf16_values(rng, n, e_lo, e_hi):
    """n random bf16 numbers (as fp64) with unbiased exponents in [e_lo, e_hi] and random signs."""
    e = rng.integers(e_lo, e_hi + 1, size=n)
    mant = 1.0 + rng.integers(0, 128, size=n) / 128.0      # 7 mantissa bits
    sign = rng.choice([-1.0, 1.0], size=n)
    return sign * mant * np.exp2(e.astype(np.float64))


def _sequential(x):
    s = 0.0
    for v in x:
        s += float(v)
    return s


def _in_runs(x, runs):
    per = -(-len(x) // runs)
    parts = [_sequential(x[i * per:(i + 1) * per]) for i in range(runs)]
    return _sequential(parts)


def _exact(x):
    return sum((Fraction(float(v)) for v in x), Fraction(0))


def test_sums_within_the_exponent_bound_are_exact_in_any_order():
    rng = np.random.default_rng(7)
    for n, spread in ((129, 37), (1060, 34), (4096, 33), (16, 41)):
        assert spread + int(np.ceil(np.log2(n))) <= 45
        for _ in range(20):
            x = _bf16_values(rng, n, -spread, 0)
            exact = _exact(x)
            assert Fraction(_sequential(x)) == exact
            assert Fraction(_in_runs(x, 16)) == exact
            assert Fraction(_sequential(x[::-1])) == exact
            assert Fraction(float(np.sum(x))) == exact          # numpy's pairwise order


def test_sums_beyond_the_bound_can_depend_on_the_order():
    """The bound is not idle: with a wide exponent range different orders do differ, so the
    split sum must not be used there."""
    rng = np.random.default_rng(8)
    differs = 0
    for _ in range(50):
        x = _bf16_values(rng, 1060, -70, 0)
        differs += int(_sequential(x) != _in_runs(x, 16))
    assert differs > 0
