"""Pins for the CPU oracle: what the mathematics fixes, checked without the HIP path.

The paper gives no formula and no worked example for the aggregation or the gradient
statistics, so every pin is a closed form, a library routine on a special case, an invariant,
or exact-rational brute force.  Each is chosen so that a plausible slip in the oracle (uniform
instead of batch-size weights, K instead of K-1, a dropped b_k in T, deviations taken from the
wrong mean, swapped n/d slots, a segment range off by one) fails at least one of them.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import HEAD, IDX, aggregate_stats, widen
from oracle.bruteforce import exact_record
from paper_2510_08522_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rel(a, b):
    return abs(a - b) / abs(b)


def rnd(rng, K, P, scale=1.0):
    return [(rng.standard_normal(P) * scale).astype(np.float32) for _ in range(K)]


def to_bf16_bits(x32):
    return torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f64(u16):
    return (u16.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ---------------------------------------------------------------- hand-worked example
def test_hand_example():
    ex = json.load(open(os.path.join(GOLD, "hand_example_k2.json")))
    g = [np.asarray(r, dtype=np.float32) for r in ex["grads"]]
    agg, st = aggregate_stats(g, ex["batch_sizes"])
    K = 2
    assert agg.tolist() == ex["agg"]
    for name, i in IDX.items():
        if name == "count":
            assert st[0, i] == 2
        else:
            assert st[0, i] == pytest.approx(ex[name], rel=1e-15), name
    assert st[0, HEAD:HEAD + K].tolist() == ex["worker_sqnorm"]
    assert st[0, HEAD + K:HEAD + 2 * K].tolist() == ex["worker_dev_sqnorm"]


# ---------------------------------------------------------------- special cases
def test_single_worker_is_identity():
    rng = np.random.default_rng(1)
    g = rnd(rng, 1, 1001)
    agg, st = aggregate_stats(g, [77])
    assert np.array_equal(agg, g[0].astype(np.float64))        # bit for bit after widening
    assert st[0, IDX["tr_sigma"]] == 0.0
    assert st[0, HEAD + 1] == 0.0                               # d_0
    assert st[0, IDX["agg_sqnorm"]] == st[0, HEAD]              # A == n_0
    assert st[0, IDX["agg_sqnorm_unbiased"]] == st[0, IDX["agg_sqnorm"]]
    assert st[0, IDX["noise_scale"]] == 0.0 and st[0, IDX["sigma_norm"]] == 0.0


def test_identical_workers_have_zero_variance():
    rng = np.random.default_rng(2)
    g0 = rnd(rng, 1, 4097)[0]
    # batch sizes that sum to a power of two keep the weighted mean of equal values exact
    agg, st = aggregate_stats([g0, g0.copy(), g0.copy()], [32, 32, 64])
    assert np.array_equal(agg, g0.astype(np.float64))
    assert np.all(st[0, HEAD + 3:HEAD + 6] == 0.0)
    assert st[0, IDX["tr_sigma"]] == 0.0 and st[0, IDX["noise_scale"]] == 0.0
    # any batch sizes: deviations vanish to rounding
    agg, st = aggregate_stats([g0, g0.copy(), g0.copy()], [33, 50, 100])
    assert st[0, IDX["tr_sigma"]] <= 1e-30 * st[0, IDX["agg_sqnorm"]]


def test_equal_batch_sizes_reduce_to_library_mean_and_variance():
    rng = np.random.default_rng(3)
    K, P, b = 6, 5003, 48
    g = rnd(rng, K, P)
    M = np.stack(g).astype(np.float64)
    agg, st = aggregate_stats(g, [b] * K)
    np.testing.assert_allclose(agg, M.mean(axis=0), rtol=1e-14, atol=1e-300)
    T_lib = b * M.var(axis=0, ddof=1).sum()
    assert rel(st[0, IDX["tr_sigma"]], T_lib) < 1e-13
    for k in range(K):
        assert rel(st[0, HEAD + k], float(np.dot(M[k], M[k]))) < 1e-13
        dev = M[k] - M.mean(axis=0)
        assert rel(st[0, HEAD + K + k], float(np.dot(dev, dev))) < 1e-13
    assert rel(st[0, IDX["agg_sqnorm"]], float(np.dot(M.mean(axis=0), M.mean(axis=0)))) < 1e-13


def test_two_workers_closed_form():
    rng = np.random.default_rng(4)
    g = rnd(rng, 2, 3001)
    b = [40, 300]
    _, st = aggregate_stats(g, b)
    diff = g[0].astype(np.float64) - g[1].astype(np.float64)
    B = sum(b)
    wd = b[0] * st[0, HEAD + 2] + b[1] * st[0, HEAD + 3]
    assert rel(wd, b[0] * b[1] / B * float(np.dot(diff, diff))) < 1e-13
    assert rel(st[0, IDX["tr_sigma"]], wd) < 1e-15           # K-1 == 1
    # each worker sits at the other's share of the difference
    assert rel(st[0, HEAD + 2], (b[1] / B) ** 2 * float(np.dot(diff, diff))) < 1e-13
    assert rel(st[0, HEAD + 3], (b[0] / B) ** 2 * float(np.dot(diff, diff))) < 1e-13


def test_weighted_variance_identity():
    # sum_k b_k d_k == sum_k b_k n_k - B A   (expand the square around the weighted mean)
    rng = np.random.default_rng(5)
    K, P = 7, 2500
    g = rnd(rng, K, P)
    b = rng.integers(8, 1025, size=K)
    _, st = aggregate_stats(g, b)
    lhs = float(np.dot(b, st[0, HEAD + K:HEAD + 2 * K]))
    rhs = float(np.dot(b, st[0, HEAD:HEAD + K])) - b.sum() * st[0, IDX["agg_sqnorm"]]
    assert rel(lhs, rhs) < 1e-11
    assert rel(st[0, IDX["tr_sigma"]], lhs / (K - 1)) < 1e-15


def test_derived_scalars_follow_their_definitions():
    rng = np.random.default_rng(6)
    K = 5
    g = rnd(rng, K, 777)
    b = np.array([32, 57, 132, 1024, 8])
    _, st = aggregate_stats(g, b)
    A, T, B = st[0, 0], st[0, 1], float(b.sum())
    assert rel(st[0, 2], A - T / B) < 1e-14
    assert rel(st[0, 3], T / (A - T / B)) < 1e-13
    assert rel(st[0, 4], T / A) < 1e-14
    assert rel(st[0, 5], st[0, 4] / B) < 1e-14
    assert rel(st[0, 6], np.sqrt(st[0, 5])) < 1e-14
    assert st[0, 7] == 777


# ---------------------------------------------------------------- invariances
def test_scale_and_permutation():
    rng = np.random.default_rng(7)
    K, P = 5, 1234
    g = rnd(rng, K, P)
    b = rng.integers(8, 513, size=K)
    agg, st = aggregate_stats(g, b)
    agg2, st2 = aggregate_stats([x * np.float32(4.0) for x in g], b)   # exact scaling
    np.testing.assert_allclose(agg2, 4.0 * agg, rtol=1e-15)
    for i in (0, 1, 2):
        assert rel(st2[0, i], 16.0 * st[0, i]) < 1e-15
    for i in (3, 4, 5, 6):
        assert rel(st2[0, i], st[0, i]) < 1e-14
    np.testing.assert_allclose(st2[0, HEAD:], 16.0 * st[0, HEAD:], rtol=1e-15)
    perm = rng.permutation(K)
    agg3, st3 = aggregate_stats([g[p] for p in perm], b[perm])
    np.testing.assert_allclose(agg3, agg, rtol=1e-13, atol=1e-18)
    np.testing.assert_allclose(st3[0, :HEAD], st[0, :HEAD], rtol=1e-12)
    np.testing.assert_allclose(st3[0, HEAD:HEAD + K], st[0, HEAD:HEAD + K][perm], rtol=1e-15)
    np.testing.assert_allclose(st3[0, HEAD + K:], st[0, HEAD + K:][perm], rtol=1e-12)


def test_batch_size_scaling_leaves_mean_unchanged():
    # only the ratios b_k / B enter G and d_k; T and the noise scales grow with the common factor
    rng = np.random.default_rng(8)
    g = rnd(rng, 4, 900)
    b = np.array([10, 20, 30, 45])
    agg, st = aggregate_stats(g, b)
    agg2, st2 = aggregate_stats(g, 3 * b)
    np.testing.assert_allclose(agg2, agg, rtol=1e-15, atol=1e-300)
    np.testing.assert_allclose(st2[0, HEAD:], st[0, HEAD:], rtol=1e-14)
    assert rel(st2[0, 1], 3 * st[0, 1]) < 1e-14
    assert rel(st2[0, 2], st[0, 2]) < 1e-13       # A - T/B: both T and B scale by 3
    assert rel(st2[0, 5], st[0, 5]) < 1e-13       # sigma2_norm = T/(B A)


# ---------------------------------------------------------------- exact brute force, tiny P
def test_widening_of_every_16_bit_pattern():
    """The oracle's value of every fp16 and bf16 bit pattern against the conversions of numpy
    (binary16) and torch (bfloat16), which share no code with it."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for got, ref in [(widen(bits.view(np.float16)), bits.view(np.float16).astype(np.float64)),
                     (widen(bits), torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
                      .to(torch.float64).numpy())]:
        nan = np.isnan(ref)
        assert (np.isnan(got) == nan).all()
        assert (got[~nan] == ref[~nan]).all()
        assert (np.signbit(got[~nan]) == np.signbit(ref[~nan])).all()     # -0.0 stays -0.0
    x = np.random.default_rng(1).standard_normal(1000).astype(np.float32)
    assert (widen(x) == x.astype(np.float64)).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("K,P,threads", [(1, 5, 1), (2, 1, 1), (3, 64, 1), (5, 37, 3), (8, 64, 4)])
def test_bruteforce_exact_rationals(dtype, K, P, threads):
    rng = np.random.default_rng(100 + K * 64 + P)
    g32 = rnd(rng, K, P, scale=3.0)
    b = rng.integers(1, 1025, size=K)
    if dtype == "bf16":
        g = [to_bf16_bits(x) for x in g32]
        vals = [bf16_bits_to_f64(x) for x in g]
    elif dtype == "f16":
        g = [x.astype(np.float16) for x in g32]
        g[0][::7] = np.float16(3e-6)                       # a few subnormals
        vals = [x.astype(np.float64) for x in g]
    else:
        g = g32
        vals = [x.astype(np.float64) for x in g]
    cols = [[float(v) for v in x] for x in vals]
    cuts = sorted(set([0, P] + ([1, P // 2, P - 1] if P > 3 else [])))
    off = np.asarray(cuts, dtype=np.int64)
    agg, st = aggregate_stats(g, b, off, threads=threads)
    ranges = [(0, P)] + list(zip(cuts[:-1], cuts[1:]))
    for r, (lo, hi) in enumerate(ranges):
        ex = exact_record(cols, b, lo, hi)
        if r == 0:
            for i in range(P):
                assert agg[i] == float(ex["G"][i]), i          # correctly rounded
        tol = 4e-16

        def close(got, frac):
            f = float(frac)
            return got == f or abs(got - f) <= tol * abs(f)
        assert close(st[r, 0], ex["A"])
        assert close(st[r, 1], ex["T"])
        # A - T/B can cancel: compare with the rounding of its two parts
        assert abs(st[r, 2] - float(ex["A_unb"])) <= tol * (float(ex["A"]) + float(ex["T"] / ex["B"]))
        assert st[r, 7] == hi - lo
        for k in range(K):
            assert close(st[r, HEAD + k], ex["n"][k])
            assert close(st[r, HEAD + K + k], ex["d"][k])
        if K > 1 and ex["A"] != 0:
            assert close(st[r, 4], ex["T"] / ex["A"])
            assert close(st[r, 5], ex["T"] / (ex["B"] * ex["A"]))
            if abs(float(ex["A_unb"])) > 1e-3 * float(ex["A"]):
                assert abs(st[r, 3] - float(ex["T"] / ex["A_unb"])) <= 1e-12 * abs(float(ex["T"] / ex["A_unb"]))


# ---------------------------------------------------------------- segments and threads
def test_segment_records_add_up_and_match_slices():
    rng = np.random.default_rng(9)
    K, P = 4, 10007
    g = rnd(rng, K, P)
    b = rng.integers(16, 257, size=K)
    off = np.array([0, 1, 2, 130, 131, 4099, 4100, 9001, P])
    agg, st = aggregate_stats(g, b, off)
    S = len(off) - 1
    assert st.shape == (1 + S, HEAD + 2 * K)
    for i in [0, 1, 7] + list(range(HEAD, HEAD + 2 * K)):   # additive entries (same B, same K-1)
        assert rel(st[1:, i].sum(), st[0, i]) < 1e-12, i
    for j in range(S):     # a segment record is the global record of the slice on its own
        _, sj = aggregate_stats([x[off[j]:off[j + 1]] for x in g], b)
        np.testing.assert_array_equal(sj[0], st[1 + j])


def test_thread_count_does_not_matter():
    rng = np.random.default_rng(10)
    g = rnd(rng, 3, 50001)
    b = [100, 125, 225]
    a1, s1 = aggregate_stats(g, b, [0, 17, 50001], threads=1)
    a5, s5 = aggregate_stats(g, b, [0, 17, 50001], threads=5)
    assert np.array_equal(a1, a5)
    np.testing.assert_allclose(s5, s1, rtol=1e-15)


def test_argument_checks():
    g = [np.ones(4, dtype=np.float32)] * 2
    with pytest.raises(ValueError):
        aggregate_stats(g, [1, 0])
    with pytest.raises(ValueError):
        aggregate_stats(g, [1, 2], [0, 2, 2, 4])
    with pytest.raises(ValueError):
        aggregate_stats(g, [1, 2], [0, 2, 3])
    with pytest.raises(TypeError):
        aggregate_stats([np.ones(4)] * 2, [1, 2])


# ---------------------------------------------------------------- generator closed forms
def _closed_form_check(w, st_row, P, sigma, musq, nsig=5.0):
    K, b = w.K, w.batch_sizes.astype(np.float64)
    B = b.sum()
    T, A, A_unb = st_row[1], st_row[0], st_row[2]
    # T estimates tr(Sigma) = P sigma^2; (K-1) T / (P sigma^2) is chi-square with (K-1) P dof
    sdT = np.sqrt(2.0 / ((K - 1) * P))
    assert abs(T / (P * sigma ** 2) - 1.0) < nsig * sdT + 2e-5
    # A_unb estimates the realised |mu|^2
    sdA = np.sqrt(4 * musq * sigma ** 2 / B + 2 * P * sigma ** 4 / B ** 2 + (sdT * P * sigma ** 2 / B) ** 2)
    assert abs(A_unb - musq) < nsig * sdA + 1e-5 * musq
    # the raw |G|^2 is biased up by tr(Sigma)/B
    assert abs(A - (musq + P * sigma ** 2 / B)) < nsig * sdA + 1e-5 * A
    ns = P * sigma ** 2 / musq
    assert abs(st_row[3] / ns - 1.0) < nsig * (sdT + sdA / musq) + 3e-5
    nsb = P * sigma ** 2 / (musq + P * sigma ** 2 / B)
    assert abs(st_row[4] / nsb - 1.0) < nsig * (sdT + sdA / A) + 3e-5


def test_generator_closed_form_c1():
    w = W.config("C1")
    _, st = aggregate_stats(w.host_arrays(), w.batch_sizes, threads=8)
    _closed_form_check(w, st[0], w.P, float(w.sigma[0]), float(w.mu_sqnorm[0]))
    assert abs(st[0, 3] - 100.0) < 2.0                    # sigma=1e-2, mean std 1e-3
    # independent cross-check: n_k = |mu|^2 + P sigma^2 / b_k + noise; fit a line in 1/b_k
    n = st[0, HEAD:HEAD + w.K]
    x = 1.0 / w.batch_sizes.astype(np.float64)
    slope, icpt = np.polyfit(x, n, 1)
    assert abs(slope / (w.P * w.sigma[0] ** 2) - 1.0) < 0.02
    assert abs(icpt / w.mu_sqnorm[0] - 1.0) < 0.02


def test_generator_closed_form_bf16_recipe():
    w = W.config("C3", P=1_500_000)
    _, st = aggregate_stats(w.host_arrays(), w.batch_sizes, threads=8)
    # bf16 storage adds ~2^-18/3 relative variance per element: far below the sampling spread
    _closed_form_check(w, st[0], w.P, float(w.sigma[0]), float(w.mu_sqnorm[0]))
    assert abs(st[0, 3] / 2000.0 - 1.0) < 0.05


def test_generator_closed_form_per_segment():
    w = W.config("C5", P=1_000_000)
    _, st = aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets, threads=8)
    sizes = np.diff(w.segment_offsets)
    checked = 0
    for j in range(w.S):
        if sizes[j] >= 2000:
            _closed_form_check(w, st[1 + j], int(sizes[j]), float(w.sigma[j]),
                               float(w.mu_sqnorm[1 + j]), nsig=6.0)
            checked += 1
    assert checked >= 20
    trS = float((sizes * w.sigma ** 2).sum())
    assert abs(st[0, 1] / trS - 1.0) < 0.01
