"""Pins for the oracle's row statistics (max, first argmax, softmax normaliser).

The oracle's hand-written fp64 loops are checked against library routines,
closed forms and invariants; nothing here comes from the GPU path.
"""
import math

import numpy as np
import pytest
import scipy.special

from gen import bf16_bits_to_f32, f32_to_bf16_bits
from oracle import csd_oracle as O


def _rand_rows(rng, rows, V, dtype):
    z = (rng.standard_normal((rows, V)) * 3.0).astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(z).reshape(rows, V)
    return z


def _widen(z):
    return bf16_bits_to_f32(z).astype(np.float64) if z.dtype == np.uint16 else z.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1, 2, 7, 64, 1000, 4099])
def test_rows_match_library_routines(dtype, V):
    """Special case: the statistics are numpy.max / first-occurrence argmax / logsumexp in fp64."""
    rng = np.random.default_rng(100 + V)
    z = _rand_rows(rng, 9, V, dtype)
    m, t, S = O.row_stats(z)
    zd = _widen(z)
    np.testing.assert_array_equal(m, zd.max(axis=1))
    np.testing.assert_array_equal(t, zd.argmax(axis=1))            # numpy returns the first maximum
    lse = scipy.special.logsumexp(zd, axis=1)
    np.testing.assert_allclose(np.log(S) + m, lse, rtol=0, atol=1e-12)


def test_bf16_ties_resolve_to_lowest_id():
    """bf16 rows have many exactly equal values; the lowest id must win."""
    rng = np.random.default_rng(5)
    z = _rand_rows(rng, 50, 3000, "bf16")
    zd = _widen(z)
    top = zd.max(axis=1)
    # force at least a double maximum in every row at known places
    for r in range(z.shape[0]):
        a, b = sorted(rng.choice(3000, size=2, replace=False))
        hi = f32_to_bf16_bits(np.array([top[r] + 1.0], dtype=np.float32))[0]
        z[r, a] = hi
        z[r, b] = hi
        m, t, S = O.row_stats(z[r:r + 1])
        assert t[0] == a


def test_signed_zero_compares_equal():
    z = np.array([[-1.0, -0.0, 0.0, -2.0]], dtype=np.float32)
    m, t, S = O.row_stats(z)
    assert t[0] == 1 and m[0] == 0.0
    z = np.array([[-1.0, 0.0, -0.0, -2.0]], dtype=np.float32)
    m, t, S = O.row_stats(z)
    assert t[0] == 1


def test_closed_form_constant_row():
    for V in (1, 5, 1000):
        z = np.full((1, V), 2.5, dtype=np.float32)
        m, t, S = O.row_stats(z)
        assert m[0] == 2.5 and t[0] == 0
        assert S[0] == float(V)


def test_closed_form_single_spike():
    V, h = 5000, 7.0
    for pos in (0, 1234, V - 1):
        z = np.zeros((1, V), dtype=np.float32)
        z[0, pos] = h
        m, t, S = O.row_stats(z)
        assert t[0] == pos and m[0] == h
        assert S[0] == pytest.approx(1.0 + (V - 1) * math.exp(-h), rel=1e-13)


def test_closed_form_two_equal_peaks():
    z = np.zeros((1, 100), dtype=np.float32)
    z[0, 70] = 4.0
    z[0, 30] = 4.0
    m, t, S = O.row_stats(z)
    assert t[0] == 30
    assert S[0] == pytest.approx(2.0 + 98 * math.exp(-4.0), rel=1e-13)


def test_masked_vocab_minus_inf():
    z = np.full((1, 64), -np.inf, dtype=np.float32)
    z[0, 10] = 1.0
    z[0, 20] = 0.0
    m, t, S = O.row_stats(z)
    assert t[0] == 10 and m[0] == 1.0
    assert S[0] == pytest.approx(1.0 + math.exp(-1.0), rel=1e-15)


def test_shift_invariance_and_probabilities_sum_to_one():
    rng = np.random.default_rng(11)
    z = _rand_rows(rng, 4, 777, "f32")
    m, t, S = O.row_stats(z)
    # exact shift by a power of two keeps every difference exact
    z2 = (z.astype(np.float64) + 16.0).astype(np.float32)
    m2, t2, S2 = O.row_stats(z2)
    np.testing.assert_array_equal(t, t2)
    np.testing.assert_allclose(m2 - 16.0, m, rtol=0, atol=1e-5)
    np.testing.assert_allclose(S2, S, rtol=1e-5)
    for r in range(4):
        p = [math.exp(O.logit(z[r], v) - m[r]) / S[r] for v in range(z.shape[1])]
        assert sum(p) == pytest.approx(1.0, abs=1e-12)


def test_permutation_moves_argmax_keeps_m_and_S():
    rng = np.random.default_rng(12)
    z = _rand_rows(rng, 1, 513, "f32")
    m, t, S = O.row_stats(z)
    perm = rng.permutation(513)
    zp = np.ascontiguousarray(z[:, perm])
    mp, tp, Sp = O.row_stats(zp)
    assert mp[0] == m[0]
    assert perm[tp[0]] == t[0]
    assert Sp[0] == pytest.approx(S[0], rel=1e-12)


def test_threads_do_not_change_results():
    rng = np.random.default_rng(13)
    z = _rand_rows(rng, 37, 300, "bf16").reshape(37, 1, 300)
    a = O.row_stats(z, threads=1)
    b = O.row_stats(z, threads=5)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_eq3_ratio_identity_and_temperature_invariance():
    """Eq. 3: p(draft)/p(t*) from full softmax probabilities equals exp(z_draft - z_t*);
    the gate uses temperature-1 logits whatever the sampling temperature."""
    rng = np.random.default_rng(14)
    V, k = 300, 6
    z = _rand_rows(rng, k + 1, V, "f32").reshape(1, k + 1, V)
    draft = rng.integers(0, V, size=(1, k)).astype(np.int32)
    orc = O.CSDOracle()
    res = orc.verify_step(z, draft, tau=0.3, lam=2)
    P = scipy.special.softmax(z.astype(np.float64), axis=-1)
    for i in range(k):
        tstar = int(np.argmax(z[0, i]))
        full = P[0, i, draft[0, i]] / P[0, i, tstar]
        assert res.ratio[0, i] == pytest.approx(full, rel=1e-12)
        assert res.p_draft[0, i] == pytest.approx(P[0, i, draft[0, i]], rel=1e-12)
        assert 1.0 / res.row_sumexp[0, i] == pytest.approx(P[0, i, tstar], rel=1e-12)
        # a sampling temperature of 0.5 would square the ratio; the oracle must not do that
        if draft[0, i] != tstar:
            P_half = scipy.special.softmax(z[0, i].astype(np.float64) / 0.5)
            assert res.ratio[0, i] != pytest.approx(P_half[draft[0, i]] / P_half[tstar], rel=1e-6)
