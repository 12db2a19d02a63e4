"""The seeded input generators (no GPU): the 'special' recipe must really produce the corner cases it names,
otherwise the GPU parity tests that use it would prove less than they claim."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import numeric
from paper_2201_11840_amd import inputs


def _exact(a, dtype):
    with np.errstate(invalid="ignore"):
        return numeric.to_float64(a, dtype)


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_special_recipe_meets_its_classes(dtype):
    n = 30000
    ranks = inputs.make_special(3, n, dtype, 77)
    cls = inputs.special_classes(n, 77)
    vals = [_exact(a, dtype) for a in ranks]
    _, ebits, mbits = inputs.FORMAT[dtype]
    smallest_normal = 2.0 ** (2 - (1 << (ebits - 1)))
    name = inputs.SPECIAL_CLASSES.index
    assert all(np.count_nonzero(cls == k) > n // 12 for k in range(len(inputs.SPECIAL_CLASSES)))
    tiny = cls == name("tiny")
    assert np.all(np.abs(vals[0][tiny]) < 8 * smallest_normal)
    assert np.count_nonzero(np.abs(vals[0][tiny]) < smallest_normal) > tiny.sum() // 6          # subnormal operands
    huge = cls == name("huge")
    assert np.all(np.isfinite(vals[0][huge]))
    largest = float(2.0 ** (1 << (ebits - 1))) * (1 - 2.0 ** -(mbits + 2))
    assert np.count_nonzero(np.abs(vals[0][huge] + vals[1][huge]) > largest) > huge.sum() // 8   # sums that overflow
    zeros = cls == name("zeros")
    z0, z1 = vals[0][zeros], vals[1][zeros]
    both = (z0 == 0) & (z1 == 0)
    assert np.count_nonzero(both & np.signbit(z0) & np.signbit(z1)) > 0                        # -0 + -0
    assert np.count_nonzero(both & (np.signbit(z0) != np.signbit(z1))) > 0                     # +0 + -0
    infnan = cls == name("inf_nan")
    assert np.count_nonzero(np.isnan(vals[0][infnan])) > 0 and np.count_nonzero(np.isinf(vals[0][infnan])) > 0
    assert np.count_nonzero(np.isinf(vals[0][infnan]) & np.isinf(vals[1][infnan]) &
                            (np.signbit(vals[0][infnan]) != np.signbit(vals[1][infnan]))) > 0      # inf - inf
    # ties: the exact sum of rank 0's and rank 1's value lies exactly half-way between two neighbouring
    # representable values (checked in rational arithmetic on a sample)
    ties = np.flatnonzero(cls == name("ties"))[:400]
    halfway = 0
    for i in ties:
        a, b = Fraction(float(vals[0][i])), Fraction(float(vals[1][i]))
        s = a + b
        if s == 0:
            continue
        e = 0
        while Fraction(2) ** (e + 1) <= abs(s):
            e += 1
        while Fraction(2) ** e > abs(s):
            e -= 1
        ulp = Fraction(2) ** (e - mbits)
        q = s / ulp
        if q.denominator == 2:            # an odd multiple of half a unit in the last place
            halfway += 1
    assert halfway > len(ties) * 0.8


def test_generators_are_seeded_and_rank_dependent():
    for dist in ("int8", "uniform", "normal", "special"):
        a = inputs.make_inputs(2, 1000, "f16", dist, 5)
        b = inputs.make_inputs(2, 1000, "f16", dist, 5)
        assert all(x.tobytes() == y.tobytes() for x, y in zip(a, b))
        assert a[0].tobytes() != a[1].tobytes()
        assert a[0].dtype == inputs.STORAGE["f16"]
    assert inputs.make_inputs(1, 64, "bf16", "special", 1)[0].dtype == np.uint16
    assert inputs.make_inputs(1, 64, "f32", "special", 1)[0].dtype == np.float32
