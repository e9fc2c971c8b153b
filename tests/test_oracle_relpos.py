"""Pins for the oracle's relative-position bucket function (CPU only)."""
from decimal import Decimal, getcontext

import numpy as np
import pytest

from conftest import read_golden_pairs
from oracle import t5_oracle as O


@pytest.mark.parametrize("fname,bidir", [("relpos_bidirectional_32_128.txt", True),
                                         ("relpos_unidirectional_32_128.txt", False)])
def test_worked_values(fname, bidir):
    rows = read_golden_pairs(fname)
    assert len(rows) >= 18
    for rp, want in rows:
        assert O.relpos_bucket_scalar(int(rp), bidir, 32, 128) == int(want), (rp, want)


def test_first_n_of_each_bucket():
    for mode, bucket, first_n in read_golden_pairs("relpos_first_n_32_128.txt"):
        bidir = mode == "bi"
        b, n = int(bucket), int(first_n)
        assert O.relpos_bucket_scalar(-n, bidir, 32, 128) == b
        assert O.relpos_bucket_scalar(-(n - 1), bidir, 32, 128) == b - 1


def _log_form(n, n_side, max_distance):
    """High-precision evaluation of the textbook log form, 60 significant digits."""
    getcontext().prec = 60
    e = n_side // 2
    if n < e:
        return n
    val = (Decimal(n) / Decimal(e)).ln() / (Decimal(max_distance) / Decimal(e)).ln() * (n_side - e)
    # exact integers (n a rational power of D/E) come out within 1e-50 of the integer
    k = int((val + Decimal(10) ** -40).to_integral_value(rounding="ROUND_FLOOR"))
    return min(n_side - 1, e + k)


@pytest.mark.parametrize("nb,md", [(32, 128), (16, 64), (8, 20), (64, 1000)])
def test_integer_form_equals_high_precision_log_form(nb, md):
    for rp in range(-2047, 2048):
        # bidirectional
        want = _log_form(abs(rp), nb // 2, md) + (nb // 2 if rp > 0 else 0)
        assert O.relpos_bucket_scalar(rp, True, nb, md) == want, (rp, nb, md)
        # unidirectional
        want = _log_form(max(-rp, 0), nb, md)
        assert O.relpos_bucket_scalar(rp, False, nb, md) == want, (rp, nb, md)


def test_structure():
    rp = np.arange(-3000, 3001)
    bi = O.relpos_bucket(rp, True, 32, 128)
    uni = O.relpos_bucket(rp, False, 32, 128)
    assert bi.min() == 0 and bi.max() == 31 and uni.min() == 0 and uni.max() == 31
    neg = bi[rp <= 0][::-1]        # n = 0, 1, 2, ...
    pos = bi[rp >= 0]
    assert np.all(np.diff(neg) >= 0) and np.all(np.diff(pos[1:]) >= 0)
    # sign symmetry: bucket(+n) = bucket(-n) + 16 for n > 0
    assert np.array_equal(pos[1:], neg[1:] + 16)
    assert np.all(neg[91:] == 15) and neg[90] == 14
    un = uni[rp <= 0][::-1]
    assert np.all(np.diff(un) >= 0)
    assert np.all(un[113:] == 31) and un[112] == 30
    assert np.all(uni[rp > 0] == 0)
    # every bucket is used, except bidirectional 16 ("key after query at distance 0" cannot occur)
    assert set(bi.tolist()) == set(range(32)) - {16} and set(uni.tolist()) == set(range(32))


def test_bias_is_toeplitz_and_indexed_key_minus_query():
    rng = np.random.default_rng(3)
    table = rng.standard_normal((32, 3))
    bias, bucket = O.relpos_bias(table, 40, True, 32, 128)
    assert bias.shape == (3, 40, 40)
    for i in range(39):
        assert np.array_equal(bias[:, i, :-1], bias[:, i + 1, 1:])
    # query 5, key 7 -> rp = +2 -> bucket 18 ; query 7, key 5 -> rp = -2 -> bucket 2
    assert bucket[5, 7] == 18 and bucket[7, 5] == 2
    assert np.array_equal(bias[:, 5, 7], table[18]) and np.array_equal(bias[:, 7, 5], table[2])
