"""Host side of an adjustment cycle (no GPU): pins of the numpy oracle against the paper's
numbers, closed forms and a library network, then the library's C functions against the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from oracle import policy_oracle as O


# ------------------------------------------------------------------ oracle pins
def test_action_set_and_clamp_are_the_papers():
    # "Action space and batch size adjustment": {-100, -25, 0, +25, +100}, range [32, 1024]
    assert O.ACTIONS == (-100, -25, 0, 25, 100)
    assert O.step_batch_sizes([32, 32, 100, 1000, 1024, 500], [0, 1, 0, 4, 3, 2]) == \
        [32, 32, 32, 1024, 1024, 500]
    assert O.step_batch_sizes([132, 57, 999], [0, 3, 3]) == [32, 82, 1024]
    assert O.step_batch_sizes([64], [4], b_min=16, b_max=128) == [128]


def test_reward_closed_forms():
    # "Reward function design": the regulariser vanishes at the minimum batch size of 32 and is
    # -5 delta at 1024; only positive accuracy gains count; the optimizer penalty is eta (s2 + s)
    r = O.rewards([0.5], [0.1], [2.0], [32], alpha=2.0, beta=0.25, delta=7.0)
    assert r == [0.5 + 0.2 - 0.5]
    r = O.rewards([0.5, 0.5], [-0.3, 0.0], [0.0, 0.0], [1024, 64], alpha=9.0, beta=1.0, delta=0.5)
    assert r == [0.5 - 2.5, 0.5 - 0.5]
    sgd = O.rewards([0.75], [0.0], [1.0], [128], 1.0, 0.5, 0.25, eta=4.0, sigma2_norm=0.0625, sigma_norm=0.25)
    adam = O.rewards([0.75], [0.0], [1.0], [128], 1.0, 0.5, 0.25, eta=4.0, sigma2_norm=0.0625,
                     sigma_norm=0.25, adaptive=True)
    assert sgd == [0.75 - 0.5 - 0.5] and adam == [sgd[0] - 1.25]
    assert O.discounted_return([1.0, 2.0, 4.0], 0.5) == 1.0 + 1.0 + 1.0
    assert O.discounted_return([3.0, 5.0], 0.0) == 3.0 and O.discounted_return([3.0, 5.0], 1.0) == 8.0


def test_policy_special_cases():
    sizes = [3, 4, 5]
    n = 3 * 4 + 4 + 4 * 5 + 5
    # all-zero parameters: the uniform policy
    p = O.policy_probs(np.zeros(n), sizes, [[1.0, -2.0, 3.0]])
    assert np.allclose(p, 0.2) and p.shape == (1, 5)
    # zero matrices, output biases log(1..5): probabilities 1/15 .. 5/15 whatever the state
    w = np.zeros(n)
    w[-5:] = np.log([1.0, 2.0, 3.0, 4.0, 5.0])
    p = O.policy_probs(w, sizes, [[7.0, 7.0, 7.0], [0.0, 1.0, 2.0]])
    np.testing.assert_allclose(p, np.tile(np.arange(1, 6) / 15.0, (2, 1)), rtol=1e-14)
    # one linear layer: softmax(W s + b) written out
    W = np.arange(10, dtype=np.float64).reshape(5, 2) / 10.0
    b = np.array([0.0, 0.1, 0.0, -0.1, 0.0])
    s = np.array([1.0, -1.0])
    z = W @ s + b
    want = np.exp(z) / np.exp(z).sum()
    np.testing.assert_allclose(O.policy_probs(np.concatenate([W.ravel(), b]), [2, 5], [s])[0], want,
                               rtol=1e-14)
    # a large common shift of the logits changes nothing (no overflow)
    b2 = b + 1000.0
    np.testing.assert_allclose(O.policy_probs(np.concatenate([W.ravel(), b2]), [2, 5], [s])[0], want,
                               rtol=1e-12)


def test_policy_matches_a_library_network():
    torch.manual_seed(0)
    sizes = [11, 16, 8, 5]
    net = torch.nn.Sequential(torch.nn.Linear(11, 16), torch.nn.Tanh(), torch.nn.Linear(16, 8),
                              torch.nn.Tanh(), torch.nn.Linear(8, 5)).double()
    flat = np.concatenate([np.concatenate([m.weight.detach().numpy().ravel(), m.bias.detach().numpy()])
                           for m in net if isinstance(m, torch.nn.Linear)])
    states = np.random.default_rng(1).standard_normal((6, 11))
    want = torch.softmax(net(torch.from_numpy(states)), dim=1).detach().numpy()
    np.testing.assert_allclose(O.policy_probs(flat, sizes, states), want, rtol=1e-13)


def test_choice_of_actions():
    p = [[0.1, 0.2, 0.4, 0.2, 0.1], [0.25, 0.25, 0.2, 0.15, 0.15], [0.0, 0.0, 0.0, 0.0, 1.0]]
    assert O.choose(p) == [2, 0, 4]
    assert O.choose(p, [0.0, 0.2499, 0.999]) == [0, 0, 4]
    assert O.choose(p, [0.1, 0.25, 0.0]) == [1, 1, 4]         # boundaries belong to the next action
    assert O.choose(p, [0.95, 0.99, 0.5]) == [4, 4, 4]
    # frequencies follow the probabilities
    rng = np.random.default_rng(2)
    u = rng.random(20000)
    picks = O.choose([p[0]] * 20000, u)
    freq = np.bincount(picks, minlength=5) / 20000.0
    assert np.abs(freq - np.asarray(p[0])).max() < 0.012


# ------------------------------------------------------------------ the library against the oracle
def network(seed, sizes):
    rng = np.random.default_rng(seed)
    n = sum(a * b + b for a, b in zip(sizes[:-1], sizes[1:]))
    return (rng.standard_normal(n) * 0.5).astype(np.float32)


@pytest.mark.parametrize("sizes", [[4, 5], [9, 16, 5], [12, 32, 32, 5], [1, 1, 5]])
def test_library_policy_forward(sizes):
    w = network(3, sizes)
    assert D.dynamix_policy_weight_count(sizes) == w.size
    states = np.random.default_rng(4).standard_normal((7, sizes[0])).astype(np.float32)
    got = D.dynamix_policy_forward(w, sizes, states)
    want = O.policy_probs(w, sizes, states)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-9)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-6)
    # greedy and sampled choices agree with the oracle's on the library's own probabilities
    assert D.dynamix_policy_choose(got).tolist() == O.choose(got)
    u = np.random.default_rng(5).random(7).astype(np.float32)
    assert D.dynamix_policy_choose(got, u).tolist() == O.choose(got, u)


def test_library_choice_boundaries_and_batch_size_step():
    p = np.array([[0.125, 0.125, 0.25, 0.25, 0.25]] * 6, dtype=np.float32)
    u = np.array([0.0, 0.125, 0.2499, 0.25, 0.75, 0.99999], dtype=np.float32)
    assert D.dynamix_policy_choose(p, u).tolist() == O.choose(p, u) == [0, 1, 1, 2, 4, 4]
    b = [32, 57, 132, 999, 1024, 500, 64]
    a = [0, 3, 0, 3, 4, 2, 1]
    assert D.dynamix_batch_sizes_step(b, a).tolist() == O.step_batch_sizes(b, a)
    assert D.dynamix_batch_sizes_step([64], [4], 16, 128).tolist() == [128]
    for bad in (lambda: D.dynamix_batch_sizes_step([64], [5]), lambda: D.dynamix_batch_sizes_step([64], [-1]),
                lambda: D.dynamix_batch_sizes_step([64], [1], 100, 50),
                lambda: D.dynamix_policy_choose(p[:1], [1.0])):
        with pytest.raises(D.DynamixError):
            bad()
    assert D.dynamix_policy_weight_count([4]) == -1 and D.dynamix_policy_weight_count([4, 0, 5]) == -1
    with pytest.raises(D.DynamixError):      # the last layer must have one output per action
        D.binding._check(D.binding.load().dynamix_policy_forward(
            network(1, [4, 6]).ctypes.data, np.array([4, 6], dtype=np.int32).ctypes.data, 2,
            np.zeros(4, dtype=np.float32).ctypes.data, 1, np.zeros(5, dtype=np.float32).ctypes.data))


def test_library_rewards_and_return():
    rng = np.random.default_rng(6)
    K = 9
    A, dA, T = rng.random(K), rng.standard_normal(K) * 0.1, rng.random(K) * 3
    b = rng.integers(32, 1025, size=K)
    for adaptive in (False, True):
        got = D.dynamix_cycle_rewards(A, dA, T, b, 1.5, 0.2, 0.05, 0.7, 0.031, 0.176, adaptive)
        want = O.rewards(A, dA, T, b, 1.5, 0.2, 0.05, 0.7, 0.031, 0.176, adaptive)
        np.testing.assert_allclose(got, want, rtol=1e-15, atol=1e-16)
    r = rng.standard_normal(50)
    assert abs(D.dynamix_discounted_return(r, 0.95) - O.discounted_return(r, 0.95)) < 1e-13


def test_a_cycle_end_to_end_on_the_host():
    # state rows = a worker's local metrics followed by the shared global ones; one decision step
    K, local, shared = 8, 6, 3
    sizes = [local + shared, 16, 5]
    w = network(8, sizes)
    rng = np.random.default_rng(9)
    states = np.concatenate([rng.standard_normal((K, local)),
                             np.tile(rng.standard_normal(shared), (K, 1))], axis=1).astype(np.float32)
    b = rng.integers(32, 1025, size=K).astype(np.int32)
    probs = D.dynamix_policy_forward(w, sizes, states)
    u = rng.random(K).astype(np.float32)
    acts = D.dynamix_policy_choose(probs, u)
    nxt = D.dynamix_batch_sizes_step(b, acts)
    assert nxt.tolist() == O.step_batch_sizes(b, O.choose(O.policy_probs(w, sizes, states), u))
    assert ((nxt >= 32) & (nxt <= 1024)).all()
    for before, after in zip(b.tolist(), nxt.tolist()):     # a listed move, or a clamped one
        assert after in {min(max(before + a, 32), 1024) for a in O.ACTIONS}


# ------------------------------------------------------------------ the policy update
def decisions(seed, sizes, n):
    rng = np.random.default_rng(seed)
    w = network(seed, sizes).astype(np.float64)
    states = rng.standard_normal((n, sizes[0]))
    actions = rng.integers(0, 5, size=n)
    signal = rng.standard_normal(n) * 2.0
    old = O.policy_probs(w, sizes, states)[np.arange(n), actions] * np.exp(rng.uniform(-0.4, 0.4, n))
    return w, states, actions, signal, np.minimum(old, 0.99)


def torch_objective(w, sizes, states, actions, signal, old=None, eps=0.2):
    """The same objective through a library network and automatic differentiation."""
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    h, pos = torch.from_numpy(np.asarray(states, dtype=np.float64)), 0
    for i, (n_in, n_out) in enumerate(zip(sizes[:-1], sizes[1:])):
        W = wt[pos:pos + n_out * n_in].reshape(n_out, n_in)
        pos += n_out * n_in
        b = wt[pos:pos + n_out]
        pos += n_out
        h = h @ W.T + b
        if i + 2 < len(sizes):
            h = torch.tanh(h)
    logp = torch.log_softmax(h, dim=1)[torch.arange(len(actions)), torch.from_numpy(np.asarray(actions))]
    sg = torch.from_numpy(np.asarray(signal, dtype=np.float64))
    if old is None:
        J = (sg * logp).mean()
    else:
        r = torch.exp(logp) / torch.from_numpy(np.asarray(old, dtype=np.float64))
        J = torch.minimum(r * sg, torch.clamp(r, 1 - eps, 1 + eps) * sg).mean()
    J.backward()
    return float(J.detach()), wt.grad.numpy()


@pytest.mark.parametrize("sizes", [[3, 5], [6, 8, 5], [4, 7, 6, 5]])
def test_oracle_gradient_matches_automatic_differentiation(sizes):
    w, st, a, sg, old = decisions(21, sizes, 40)
    for o in (None, old):
        J, g = torch_objective(w, sizes, st, a, sg, o)
        assert abs(O.objective(w, sizes, st, a, sg, o) - J) < 1e-13
        np.testing.assert_allclose(O.objective_gradient(w, sizes, st, a, sg, o), g, rtol=1e-10, atol=1e-14)


def test_oracle_gradient_closed_forms():
    # one linear layer, one decision, zero parameters: p = 1/5 everywhere, so the bias gradient of
    # R log p_a is R (onehot - 1/5) and the matrix gradient its outer product with the state
    sizes, s, R = [2, 5], np.array([[2.0, -1.0]]), 3.0
    g = O.objective_gradient(np.zeros(15), sizes, s, [3], [R])
    want_b = R * (np.eye(5)[3] - 0.2)
    np.testing.assert_allclose(g[10:], want_b, rtol=1e-15)
    np.testing.assert_allclose(g[:10].reshape(5, 2), np.outer(want_b, s[0]), rtol=1e-15)
    # clipped surrogate: with a positive advantage and a ratio above 1 + eps the objective is flat
    # (gradient zero); with a negative advantage it still follows the ratio
    old = [0.1]                                     # p = 0.2, r = 2 > 1.2
    assert not O.objective_gradient(np.zeros(15), sizes, s, [3], [1.0], old).any()
    gneg = O.objective_gradient(np.zeros(15), sizes, s, [3], [-1.0], old)
    np.testing.assert_allclose(gneg[10:], -1.0 * 2.0 * (np.eye(5)[3] - 0.2), rtol=1e-15)
    assert O.objective(np.zeros(15), sizes, s, [3], [1.0], old) == 1.2
    assert O.objective(np.zeros(15), sizes, s, [3], [-1.0], old) == -2.0
    # inside the clip range the two terms coincide: gradient A r (onehot - p)
    gin = O.objective_gradient(np.zeros(15), sizes, s, [3], [1.0], [0.2])
    np.testing.assert_allclose(gin[10:], np.eye(5)[3] - 0.2, rtol=1e-15)


def test_oracle_gradient_against_finite_differences():
    sizes = [5, 6, 5]
    w, st, a, sg, old = decisions(22, sizes, 16)
    g = O.objective_gradient(w, sizes, st, a, sg)
    rng = np.random.default_rng(0)
    for i in rng.choice(len(w), size=12, replace=False):
        e = np.zeros_like(w)
        e[i] = 1e-6
        fd = (O.objective(w + e, sizes, st, a, sg) - O.objective(w - e, sizes, st, a, sg)) / 2e-6
        assert abs(fd - g[i]) < 1e-7 * max(1.0, abs(g[i]))


@pytest.mark.parametrize("sizes", [[3, 5], [9, 16, 5], [6, 12, 8, 5]])
def test_library_policy_update(sizes):
    w, st, a, sg, old = decisions(23, sizes, 64)
    w32 = w.astype(np.float32)
    st32, old32 = st.astype(np.float32), old.astype(np.float32)
    for o in (None, old32):
        new, J = D.dynamix_policy_update(w32, sizes, st32, a, sg, 0.05, old_probs=o)
        want = O.update(w32, sizes, st32, a, sg, 0.05, o)
        assert abs(J - O.objective(w32, sizes, st32, a, sg, o)) < 1e-12
        np.testing.assert_allclose(new, want, rtol=2e-7, atol=1e-8)
        assert np.abs(new - w32).max() > 1e-4                   # it did move
    # ascent: a small step on the return-weighted objective does not lower it
    new, J0 = D.dynamix_policy_update(w32, sizes, st32, a, sg, 1e-3)
    assert O.objective(new, sizes, st32, a, sg) >= J0
    with pytest.raises(D.DynamixError):
        D.dynamix_policy_update(w32, sizes, st32, np.full(64, 5), sg, 0.05)
