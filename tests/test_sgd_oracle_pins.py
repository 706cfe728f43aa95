"""Pins for the oracle's model update p <- p - lr (G + wd p): special cases, closed forms and the
library optimizer on the same gradient."""
import numpy as np
import torch

from oracle import aggregate_stats, sgd_step


def data(seed, K=3, P=257):
    rng = np.random.default_rng(seed)
    g = [rng.standard_normal(P).astype(np.float32) for _ in range(K)]
    p = rng.standard_normal(P).astype(np.float32)
    return g, p


def test_zero_learning_rate_and_zero_gradient():
    g, p = data(1)
    agg, _ = aggregate_stats(g, [32, 64, 96])
    assert np.array_equal(sgd_step(agg, p, 0.0, 0.3), p.astype(np.float64))
    assert np.array_equal(sgd_step(np.zeros_like(agg), p, 0.5, 0.0), p.astype(np.float64))


def test_closed_forms_with_exact_numbers():
    # powers of two keep every product and sum exact
    agg = np.array([1.0, -2.0, 0.5, 0.0])
    p = np.array([4.0, 4.0, -1.0, 8.0], dtype=np.float32)
    assert sgd_step(agg, p, 0.5, 0.0).tolist() == [3.5, 5.0, -1.25, 8.0]
    # weight decay alone shrinks towards zero: p (1 - lr wd)
    assert sgd_step(np.zeros(4), p, 0.5, 0.25).tolist() == [3.5, 3.5, -0.875, 7.0]
    # both: p - lr (G + wd p)
    assert sgd_step(agg, p, 0.5, 0.25).tolist() == [3.0, 4.5, -1.125, 7.0]
    # lr = 1, wd = 0, p = G: the step lands on zero
    assert not sgd_step(agg, agg.astype(np.float32), 1.0, 0.0).any()


def test_matches_the_library_optimizer_on_the_aggregate():
    g, p = data(2, K=4, P=1000)
    agg, _ = aggregate_stats(g, [16, 48, 100, 256])
    for lr, wd in [(0.1, 0.0), (0.05, 5e-4), (1.5, 0.1)]:
        w = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
        opt = torch.optim.SGD([w], lr=lr, weight_decay=wd)
        w.grad = torch.from_numpy(agg.copy())
        opt.step()
        np.testing.assert_allclose(sgd_step(agg, p, lr, wd), w.detach().numpy(), rtol=1e-14,
                                   atol=1e-16)


def test_single_worker_is_plain_sgd_on_its_gradient():
    g, p = data(3, K=1)
    agg, _ = aggregate_stats(g, [77])
    ref = p.astype(np.float64) - 0.25 * g[0].astype(np.float64)
    np.testing.assert_allclose(sgd_step(agg, p, 0.25, 0.0), ref, rtol=1e-15, atol=0)
