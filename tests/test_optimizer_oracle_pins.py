"""Pins for the oracle's momentum-SGD and Adam steps: exact closed forms in binary-exact numbers,
special cases that reduce to the plain SGD step or to the identity, and the library optimizers
(in float64, over several steps with the state carried) on the same gradients."""
import numpy as np
import pytest
import torch

from oracle import adam_step, aggregate_stats, sgd_momentum_step, sgd_step


def data(seed, K=3, P=257):
    rng = np.random.default_rng(seed)
    g = [rng.standard_normal(P).astype(np.float32) for _ in range(K)]
    p = rng.standard_normal(P).astype(np.float32)
    return g, p


# ------------------------------------------------------------------ SGD with momentum
def test_momentum_closed_forms_with_exact_numbers():
    agg = np.array([1.0, -2.0, 0.5, 0.0])
    p = np.array([4.0, 4.0, -1.0, 8.0], dtype=np.float32)
    buf = np.array([2.0, 0.0, -4.0, 1.0], dtype=np.float32)
    # buf' = mu buf + G ; p' = p - lr buf'
    np_, nb = sgd_momentum_step(agg, p, buf, 0.5, 0.0, 0.5, False)
    assert nb.tolist() == [2.0, -2.0, -1.5, 0.5]
    assert np_.tolist() == [3.0, 5.0, -0.25, 7.75]
    # Nesterov: step = G + mu buf'
    np_, nb = sgd_momentum_step(agg, p, buf, 0.5, 0.0, 0.5, True)
    assert nb.tolist() == [2.0, -2.0, -1.5, 0.5]
    assert np_.tolist() == [4.0 - 0.5 * 2.0, 4.0 - 0.5 * -3.0, -1.0 - 0.5 * -0.25, 8.0 - 0.5 * 0.25]
    # weight decay enters the gradient before the buffer: g' = G + wd p
    np_, nb = sgd_momentum_step(agg, p, buf, 0.5, 0.25, 0.5, False)
    assert nb.tolist() == [3.0, -1.0, -1.75, 2.5]
    assert np_.tolist() == [2.5, 4.5, -0.125, 6.75]


def test_momentum_special_cases():
    g, p = data(1)
    agg, _ = aggregate_stats(g, [32, 64, 96])
    zero = np.zeros_like(p)
    rng = np.random.default_rng(5)
    buf = rng.standard_normal(p.shape[0]).astype(np.float32)
    # zero momentum, or a zero buffer without Nesterov, is the plain SGD step
    for nesterov in (False, True):
        np_, nb = sgd_momentum_step(agg, p, buf, 0.25, 0.01, 0.0, nesterov)
        assert np.array_equal(np_, sgd_step(agg, p, 0.25, 0.01))
    np_, nb = sgd_momentum_step(agg, p, zero, 0.25, 0.01, 0.9, False)
    assert np.array_equal(np_, sgd_step(agg, p, 0.25, 0.01))
    np.testing.assert_allclose(nb, agg + 0.01 * p.astype(np.float64), rtol=1e-15)
    # zero learning rate leaves the parameters alone and still advances the buffer
    np_, nb = sgd_momentum_step(agg, p, buf, 0.0, 0.0, 0.5, True)
    assert np.array_equal(np_, p.astype(np.float64))
    np.testing.assert_allclose(nb, 0.5 * buf.astype(np.float64) + agg, rtol=1e-15, atol=1e-18)


@pytest.mark.parametrize("nesterov", [False, True])
@pytest.mark.parametrize("wd", [0.0, 5e-4])
def test_momentum_matches_the_library_optimizer_over_steps(nesterov, wd):
    rng = np.random.default_rng(7)
    P = 500
    p = rng.standard_normal(P).astype(np.float32)
    w = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
    opt = torch.optim.SGD([w], lr=0.1, momentum=0.9, weight_decay=wd, nesterov=nesterov)
    cur_p, cur_b = p.astype(np.float64), np.zeros(P)
    for step in range(4):
        g = [rng.standard_normal(P).astype(np.float32) for _ in range(3)]
        agg, _ = aggregate_stats(g, [16, 48, 100])
        w.grad = torch.from_numpy(agg.copy())
        opt.step()
        # the oracle takes float32 state: feed it the rounded state, and the library the same
        p32, b32 = cur_p.astype(np.float32), cur_b.astype(np.float32)
        cur_p, cur_b = sgd_momentum_step(agg, p32, b32, 0.1, wd, 0.9, nesterov)
        ref_p = w.detach().numpy()
        # (the library carries float64 state; the oracle was restarted from float32 roundings of
        # its own state, which differ from the library's by at most a float32 rounding per step)
        np.testing.assert_allclose(cur_p, ref_p, rtol=0, atol=2e-6 * (step + 1))
    # one step from identical float32 state agrees to double rounding
    w2 = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
    opt2 = torch.optim.SGD([w2], lr=0.1, momentum=0.9, weight_decay=wd, nesterov=nesterov)
    b0 = rng.standard_normal(P).astype(np.float32)
    w2.grad = torch.from_numpy(agg.copy())
    opt2.state[w2]["momentum_buffer"] = torch.from_numpy(b0.astype(np.float64))
    opt2.step()
    np_, nb = sgd_momentum_step(agg, p, b0, 0.1, wd, 0.9, nesterov)
    np.testing.assert_allclose(np_, w2.detach().numpy(), rtol=1e-14, atol=1e-16)
    np.testing.assert_allclose(nb, opt2.state[w2]["momentum_buffer"].numpy(), rtol=1e-14, atol=1e-16)


# ------------------------------------------------------------------ Adam
def test_adam_first_step_is_a_signed_step_of_the_learning_rate():
    # zero moments, eps = 0, t = 1: m-hat = g, v-hat = g^2, so p' = p - lr sign(g); with
    # beta1 = 1/2 and beta2 = 3/4 every intermediate is exact
    agg = np.array([1.0, -2.0, 0.5, 4.0])
    p = np.array([4.0, 4.0, -1.0, 8.0], dtype=np.float32)
    z = np.zeros(4, dtype=np.float32)
    np_, nm, nv = adam_step(agg, p, z, z, 0.25, 0.5, 0.75, 0.0, 0.0, False, 1)
    assert nm.tolist() == [0.5, -1.0, 0.25, 2.0]
    assert nv.tolist() == [0.25, 1.0, 0.0625, 4.0]
    assert np_.tolist() == [3.75, 4.25, -1.25, 7.75]
    # eps enters the denominator after the root: |g| + eps
    np_, _, _ = adam_step(agg, p, z, z, 0.25, 0.5, 0.75, 1.0, 0.0, False, 1)
    assert np_.tolist() == [4.0 - 0.25 * 0.5, 4.0 + 0.25 * 2.0 / 3.0, -1.0 - 0.25 * 0.5 / 1.5, 8.0 - 0.25 * 0.8]


def test_adam_closed_forms_at_a_later_step():
    # t = 2, beta1 = beta2 = 1/2: corrections 1 - 1/4 = 3/4
    agg = np.array([2.0, -4.0])
    p = np.array([1.0, 1.0], dtype=np.float32)
    m = np.array([1.0, 2.0], dtype=np.float32)
    v = np.array([4.0, 16.0], dtype=np.float32)
    np_, nm, nv = adam_step(agg, p, m, v, 0.5, 0.5, 0.5, 0.0, 0.0, False, 2)
    assert nm.tolist() == [1.5, -1.0] and nv.tolist() == [4.0, 16.0]
    want = [1.0 - 0.5 * (1.5 / 0.75) / np.sqrt(4.0 / 0.75), 1.0 - 0.5 * (-1.0 / 0.75) / np.sqrt(16.0 / 0.75)]
    np.testing.assert_allclose(np_, want, rtol=1e-15)
    # L2 weight decay enters the gradient; decoupled decay shrinks the parameter and leaves the
    # moments those of the plain gradient
    _, nm2, _ = adam_step(agg, p, m, v, 0.5, 0.5, 0.5, 0.0, 2.0, False, 2)
    assert nm2.tolist() == [0.5 * 1.0 + 0.5 * 4.0, 0.5 * 2.0 + 0.5 * -2.0]
    np3, nm3, nv3 = adam_step(agg, p, m, v, 0.5, 0.5, 0.5, 0.0, 0.5, True, 2)
    assert nm3.tolist() == nm.tolist() and nv3.tolist() == nv.tolist()
    np.testing.assert_allclose(np3, np.asarray(want) - 0.25, rtol=1e-15)     # p (1 - lr wd) = 0.75


@pytest.mark.parametrize("decoupled", [False, True])
def test_adam_matches_the_library_optimizer_over_steps(decoupled):
    rng = np.random.default_rng(11)
    P = 400
    p = rng.standard_normal(P).astype(np.float32)
    lr, b1, b2, eps, wd = 1e-2, 0.9, 0.999, 1e-8, 0.01
    w = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
    cls = torch.optim.AdamW if decoupled else torch.optim.Adam
    opt = cls([w], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    cur = (p.astype(np.float64), np.zeros(P), np.zeros(P))
    for step in range(1, 6):
        g = [rng.standard_normal(P).astype(np.float32) for _ in range(4)]
        agg, _ = aggregate_stats(g, [16, 48, 100, 256])
        w.grad = torch.from_numpy(agg.copy())
        # one step from the library's own state, rounded to float32 on both sides
        st = opt.state[w]
        if st:
            m32 = st["exp_avg"].numpy().astype(np.float32)
            v32 = st["exp_avg_sq"].numpy().astype(np.float32)
            st["exp_avg"].copy_(torch.from_numpy(m32.astype(np.float64)))
            st["exp_avg_sq"].copy_(torch.from_numpy(v32.astype(np.float64)))
        else:
            m32 = v32 = np.zeros(P, dtype=np.float32)
        p32 = w.detach().numpy().astype(np.float32)
        with torch.no_grad():
            w.copy_(torch.from_numpy(p32.astype(np.float64)))
        opt.step()
        np_, nm, nv = adam_step(agg, p32, m32, v32, lr, b1, b2, eps, wd, decoupled, step)
        np.testing.assert_allclose(np_, w.detach().numpy(), rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(nm, opt.state[w]["exp_avg"].numpy(), rtol=1e-13, atol=1e-17)
        np.testing.assert_allclose(nv, opt.state[w]["exp_avg_sq"].numpy(), rtol=1e-13, atol=1e-17)


def test_adam_special_cases():
    g, p = data(4)
    agg, _ = aggregate_stats(g, [8, 100, 33])
    rng = np.random.default_rng(6)
    m = rng.standard_normal(p.shape[0]).astype(np.float32)
    v = (rng.standard_normal(p.shape[0]) ** 2).astype(np.float32)
    # zero learning rate: parameters untouched, moments advance
    np_, nm, nv = adam_step(agg, p, m, v, 0.0, 0.9, 0.999, 1e-8, 0.0, False, 3)
    assert np.array_equal(np_, p.astype(np.float64))
    np.testing.assert_allclose(nm, 0.9 * m.astype(np.float64) + (1 - 0.9) * agg, rtol=1e-14, atol=1e-17)
    np.testing.assert_allclose(nv, 0.999 * v.astype(np.float64) + (1 - 0.999) * agg ** 2, rtol=1e-12, atol=1e-17)
    # beta1 = beta2 = 0: no memory, p' = p - lr g / (|g| + eps) at any step
    np_, nm, nv = adam_step(agg, p, m, v, 0.125, 0.0, 0.0, 0.5, 0.0, False, 7)
    assert np.array_equal(nm, agg)
    np.testing.assert_allclose(nv, agg * agg, rtol=4e-16, atol=0)
    np.testing.assert_allclose(np_, p - 0.125 * agg / (np.abs(agg) + 0.5), rtol=1e-15, atol=1e-17)
    # scaling gradient and root of the second moment together leaves the step unchanged (eps = 0)
    a1, _, _ = adam_step(agg, p, m, v, 0.01, 0.5, 0.75, 0.0, 0.0, False, 2)
    a2, _, _ = adam_step(agg * 4.0, p, m * 4.0, v * 16.0, 0.01, 0.5, 0.75, 0.0, 0.0, False, 2)
    np.testing.assert_allclose(a1, a2, rtol=1e-15, atol=1e-17)
