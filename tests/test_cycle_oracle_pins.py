"""Pins for the per-cycle oracle: special cases and closed forms that the reading fixes."""
import math

import numpy as np

from oracle import aggregate_stats
from oracle.cycle_oracle import EXTRA, HEAD, cycle_summary, summary_count


def one_stats(seed, K=3, P=500, off=None, b=(32, 57, 132)):
    rng = np.random.default_rng(seed)
    g = [rng.standard_normal(P).astype(np.float32) for _ in range(K)]
    return aggregate_stats(g, list(b), off)[1]


def test_single_iteration_is_the_record_itself():
    st = one_stats(1)
    out = cycle_summary([st], 3, 0, [32, 57, 132], eta=0.5, delta=0.25)
    R = HEAD + 6
    assert out.shape == (summary_count(3, 0),) == (R + EXTRA + 3,)
    assert np.array_equal(out[:R], st[0])
    # with one iteration the pooled ratios are the record's own ratios (recomputed in double)
    for got, want in ((out[R + 0], st[0, 3]), (out[R + 1], st[0, 5]), (out[R + 2], st[0, 6])):
        assert math.isclose(got, want, rel_tol=1e-14)
    assert out[R + 3] == -0.5 * (st[0, 5] + st[0, 6])


def test_identical_iterations_average_to_themselves():
    st = one_stats(2, off=[0, 100, 500])
    out = cycle_summary([st] * 7, 3, 2, [32, 57, 132], eta=1.0, delta=1.0)
    R = HEAD + 6
    for r in range(3):
        np.testing.assert_allclose(out[r * (R + EXTRA):r * (R + EXTRA) + R], st[r], rtol=1e-15)
    two = cycle_summary([st] * 2, 3, 2, [32, 57, 132], eta=1.0, delta=1.0)   # x + x, / 2: exact
    for r in range(3):
        assert np.array_equal(two[r * (R + EXTRA):r * (R + EXTRA) + R], st[r])


def test_mean_matches_numpy_and_pooled_ratios_use_mean_sums():
    sts = [one_stats(10 + i) for i in range(5)]
    b = [32, 57, 132]
    out = cycle_summary(sts, 3, 0, b, eta=2.0, delta=0.1)
    R = HEAD + 6
    M = np.mean(np.stack([s[0] for s in sts]), axis=0)
    np.testing.assert_allclose(out[:R], M, rtol=1e-15)
    B = float(sum(b))
    assert math.isclose(out[R + 0], M[1] / (M[0] - M[1] / B), rel_tol=1e-14)
    assert math.isclose(out[R + 1], M[1] / (B * M[0]), rel_tol=1e-14)
    assert math.isclose(out[R + 2], math.sqrt(M[1] / (B * M[0])), rel_tol=1e-14)
    assert math.isclose(out[R + 3], -2.0 * (M[5] + M[6]), rel_tol=1e-14)
    # a mean of ratios is not the ratio of means: the two differ on varying data
    assert out[R + 0] != M[3]


def test_batch_regulariser_closed_form():
    out = cycle_summary([one_stats(3, K=4, b=(32, 64, 1024, 8))], 4, 0, [32, 64, 1024, 8],
                        eta=0.0, delta=0.5)
    tail = out[-4:]
    assert tail[0] == 0.0            # the constant 5 is log2 of the smallest batch size, 32
    assert tail[1] == -0.5 and tail[2] == -2.5 and tail[3] == 1.0
    mid = cycle_summary([one_stats(3)], 3, 0, [32, 57, 132], eta=0.0, delta=1.0)[-3:]
    assert math.isclose(mid[1], -(math.log(57) / math.log(2) - 5.0), rel_tol=1e-14)


def test_degenerate_records_propagate():
    st = one_stats(4)
    z = st.copy()
    z[0, :] = 0.0
    out = cycle_summary([z], 3, 0, [32, 57, 132], eta=1.0, delta=1.0)
    R = HEAD + 6
    assert np.isnan(out[R + 0]) and np.isnan(out[R + 1]) and out[R + 2] == 0.0
