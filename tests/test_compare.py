"""The checker checked: oracle.compare decides every parity verdict, so its accept / reject
behaviour is pinned here with hand-typed numbers taken from the stated tolerance
(sum, mean: |C - Cref| <= 1e-5 * Sabs + 1e-6 per element; max, min: the bits of the oracle's
double result rounded once to fp32), not with the function's own formula.
"""
import numpy as np
import pytest

import oracle


def one(value):
    return np.array([[value]], dtype=np.float32)


# (Sabs, largest accepted error, smallest rejected error): bound = 1e-5 * Sabs + 1e-6, typed by hand
BOUNDS = [
    (0.0, 0.99e-6, 1.01e-6),                 # only the absolute floor
    (1.0, 1.09e-5, 1.11e-5),                 # 1e-5 + 1e-6 = 1.1e-5
    (100.0, 1.0009e-3, 1.0011e-3),           # 1e-3 + 1e-6 = 1.001e-3
    (5.0e9, 4.9999e4, 5.0001e4),             # the absolute floor is invisible: 5e4
]


@pytest.mark.parametrize("op", ["sum", "mean"])
@pytest.mark.parametrize("sabs,inside,outside", BOUNDS)
@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_sum_tolerance_edges(op, sabs, inside, outside, sign):
    C = one(1.5 if sabs < 1e6 else 2.0 ** 33)            # exactly representable in fp32
    exact = float(C[0, 0])
    S = np.array([[sabs]])
    ok, worst = oracle.compare(op, C, np.array([[exact - sign * inside]]), S)
    assert ok and 0.9 < worst <= 1.0
    ok, worst = oracle.compare(op, C, np.array([[exact - sign * outside]]), S)
    assert not ok and worst > 1.0


def test_sum_one_bad_element_among_many_is_found():
    rng = np.random.default_rng(0)
    Cref = rng.standard_normal((50, 7))
    Sabs = np.abs(Cref) + 1.0
    C = Cref.astype(np.float32)
    assert oracle.compare("sum", C, Cref, Sabs)[0]
    for i, j in ((0, 0), (49, 6), (17, 3)):
        bad = C.copy()
        bad[i, j] += np.float32(3e-5 * Sabs[i, j])         # three times the relative bound
        ok, worst = oracle.compare("sum", bad, Cref, Sabs)
        assert not ok and worst > 1.5


@pytest.mark.parametrize("op", ["sum", "mean"])
@pytest.mark.parametrize("poison", [np.nan, np.inf, -np.inf])
def test_sum_rejects_non_finite_results(op, poison):
    Cref = np.ones((3, 4))
    Sabs = np.ones((3, 4))
    C = np.ones((3, 4), dtype=np.float32)
    C[1, 2] = poison
    assert not oracle.compare(op, C, Cref, Sabs)[0]
    # ... also when the reference bound itself is infinite (a NaN would pass "err <= inf" otherwise)
    assert not oracle.compare(op, C, Cref, np.full((3, 4), np.inf))[0]


def test_sum_non_finite_references_must_be_matched_exactly():
    Cref = np.array([[np.inf, -np.inf, np.nan, 1.0]])
    Sabs = np.array([[np.inf, np.inf, np.inf, 1.0]])
    good = np.array([[np.inf, -np.inf, np.nan, 1.0]], dtype=np.float32)
    assert oracle.compare("sum", good, Cref, Sabs) == (True, 0.0)
    for j, wrong in ((0, -np.inf), (0, np.nan), (0, 3.0e38), (1, np.inf), (1, np.nan), (2, np.inf), (2, 0.0)):
        bad = good.copy()
        bad[0, j] = wrong
        assert not oracle.compare("sum", bad, Cref, Sabs)[0], (j, wrong)
    bad = good.copy()
    bad[0, 3] = 1.1                                        # the finite elements are still checked
    assert not oracle.compare("sum", bad, Cref, Sabs)[0]


def test_mean_bound_uses_the_row_length():
    """A row of four entries (1, 2, 3, 4) against ones: sum of magnitudes 10, mean 2.5, and the scale
    of the mean's bound is 10 / 4, so an error of 2.0e-5 passes for sum's scale but fails for mean's."""
    rowptr = np.array([0, 4], dtype=np.int32)
    colind = np.array([0, 1, 2, 3], dtype=np.int32)
    vals = np.array([1, 2, 3, 4], dtype=np.float32)
    B = np.ones((4, 1), dtype=np.float32)
    Cs, Ss = oracle.spmm(rowptr, colind, vals, B, "sum")
    Cm, Sm = oracle.spmm(rowptr, colind, vals, B, "mean")
    assert Cs[0, 0] == 10.0 and Ss[0, 0] == 10.0 and Cm[0, 0] == 2.5 and Sm[0, 0] == 2.5
    # bound for mean: 1e-5 * 2.5 + 1e-6 = 2.6e-5; for the same error against the sum's scale it would be 1.01e-4
    assert oracle.compare("mean", one(2.5 + 2.0e-5), Cm, Sm)[0]
    assert not oracle.compare("mean", one(2.5 + 4.0e-5), Cm, Sm)[0]
    assert oracle.compare("sum", one(10.0 + 4.0e-5), Cs, Ss)[0]


@pytest.mark.parametrize("op", ["max", "min"])
def test_extremes_are_compared_bit_for_bit(op):
    Cref = np.array([[1.0, -2.5, 3.0e-40, 0.1]])           # 0.1 is not representable: rounded once to fp32
    good = Cref.astype(np.float32)
    assert oracle.compare(op, good, Cref, None) == (True, 0)
    for j in range(4):
        bad = good.copy()
        bad.view(np.uint32)[0, j] ^= 1                      # last mantissa bit flipped
        assert oracle.compare(op, bad, Cref, None) == (False, 1)
    # signed zeros differ
    z = np.array([[0.0, -0.0]])
    assert oracle.compare(op, np.array([[0.0, -0.0]], dtype=np.float32), z, None)[0]
    assert oracle.compare(op, np.array([[-0.0, -0.0]], dtype=np.float32), z, None) == (False, 1)
    assert oracle.compare(op, np.array([[0.0, 0.0]], dtype=np.float32), z, None) == (False, 1)
    # a NaN never matches a number, infinities must match exactly
    assert not oracle.compare(op, np.array([[np.nan]], dtype=np.float32), np.array([[1.0]]), None)[0]
    assert oracle.compare(op, np.array([[np.inf]], dtype=np.float32), np.array([[np.inf]]), None)[0]
    assert not oracle.compare(op, np.array([[np.inf]], dtype=np.float32), np.array([[-np.inf]]), None)[0]
    assert not oracle.compare(op, np.array([[3.4e38]], dtype=np.float32), np.array([[np.inf]]), None)[0]


def test_compare_refuses_wrong_types_and_shapes():
    Cref = np.zeros((2, 2))
    with pytest.raises(AssertionError):
        oracle.compare("sum", np.zeros((2, 2), dtype=np.float64), Cref, Cref)
    with pytest.raises(AssertionError):
        oracle.compare("max", np.zeros((2, 3), dtype=np.float32), Cref, None)
    assert oracle.compare("sum", np.zeros((0, 4), dtype=np.float32), np.zeros((0, 4)), np.zeros((0, 4))) == (True, 0.0)
