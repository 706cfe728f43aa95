"""TEST INFRASTRUCTURE -- plain numpy oracle of the host side of an adjustment cycle.

The paper's agent (Problem Formulation: "Reinforcement learning framework", "Action space and
batch size adjustment", "Reward function design"; Algorithm 1, the action and batch-size steps)
maps every worker's state to one of the adjustments {-100, -25, 0, +25, +100} with a policy whose
parameters all workers share, moves the batch size by it, clamps it to [x_min, x_max], and scores
the cycle with

    r = A_mean + alpha max(0, dA) - beta T_iter - delta (log2 b - 5)  [- eta (sigma_norm^2 + sigma_norm)]

and the discounted sum J = sum_t gamma^t r_t.  The paper prints neither the network's shape nor a
coefficient.  Readings: a multi-layer perceptron, tanh between layers, softmax over the five
actions; sampling by the inverse cumulative distribution at a uniform draw handed in by the caller.
Everything in float64, one worker at a time, no vectorisation tricks.  Shares no code with the
library and never imports it.
"""
import numpy as np

ACTIONS = (-100, -25, 0, 25, 100)


def unpack(weights, layer_sizes):
    """[(W, b), ...] from the flat parameter vector: per layer a row-major out x in matrix, then
    out biases."""
    w = np.asarray(weights, dtype=np.float64)
    layers, pos = [], 0
    for n_in, n_out in zip(layer_sizes[:-1], layer_sizes[1:]):
        W = w[pos:pos + n_out * n_in].reshape(n_out, n_in)
        pos += n_out * n_in
        b = w[pos:pos + n_out]
        pos += n_out
        layers.append((W, b))
    assert pos == w.size
    return layers


def policy_probs(weights, layer_sizes, states):
    """Action probabilities, one row per worker: pi_theta(. | s_i, s_global)."""
    layers = unpack(weights, layer_sizes)
    out = []
    for s in np.asarray(states, dtype=np.float64):
        h = s
        for i, (W, b) in enumerate(layers):
            h = W @ h + b
            if i + 1 < len(layers):
                h = np.tanh(h)
        e = np.exp(h - h.max())
        out.append(e / e.sum())
    return np.asarray(out)


def choose(probs, uniforms=None):
    """Index of the chosen action per worker: the most probable (first of equals), or the inverse
    of the cumulative distribution at the given uniform draw."""
    picks = []
    for k, p in enumerate(np.asarray(probs, dtype=np.float64)):
        if uniforms is None:
            picks.append(int(np.argmax(p)))
        else:
            c = np.cumsum(p)
            a = int(np.searchsorted(c, float(uniforms[k]) * c[-1], side="right"))
            picks.append(min(a, len(p) - 1))
    return picks


def step_batch_sizes(batch_sizes, picks, b_min=32, b_max=1024):
    return [max(min(int(b) + ACTIONS[a], b_max), b_min) for b, a in zip(batch_sizes, picks)]


def rewards(mean_acc, acc_gain, t_iter, batch_sizes, alpha, beta, delta, eta=0.0, sigma2_norm=0.0,
            sigma_norm=0.0, adaptive=False):
    out = []
    for A, dA, T, b in zip(mean_acc, acc_gain, t_iter, batch_sizes):
        r = A + alpha * max(0.0, dA) - beta * T - delta * (np.log2(float(b)) - 5.0)
        if adaptive:
            r -= eta * (sigma2_norm + sigma_norm)
        out.append(r)
    return out


def discounted_return(r, gamma):
    return sum(gamma ** t * x for t, x in enumerate(r))


def objective(weights, layer_sizes, states, actions, signal, old_probs=None, clip_eps=0.2):
    """Mean over the recorded decisions of signal * log pi(a | s) (the paper's simplified rule:
    the cumulative reward weighs each decision) or, with old_probs, of the clipped surrogate
    min(r A, clip(r, 1 - eps, 1 + eps) A), r = pi(a | s) / old_prob (the PPO objective, Eq. 1)."""
    p = policy_probs(weights, layer_sizes, states)
    total = 0.0
    for j, a in enumerate(actions):
        if old_probs is None:
            total += signal[j] * np.log(p[j, a])
        else:
            r = p[j, a] / float(old_probs[j])
            total += min(r * signal[j], min(max(r, 1 - clip_eps), 1 + clip_eps) * signal[j])
    return total / len(actions)


def objective_gradient(weights, layer_sizes, states, actions, signal, old_probs=None, clip_eps=0.2):
    """Gradient of `objective` with respect to the flat parameter vector, by the chain rule written
    out layer by layer (float64)."""
    layers = unpack(weights, layer_sizes)
    grads = [(np.zeros_like(W), np.zeros_like(b)) for W, b in layers]
    n = len(actions)
    for j, a in enumerate(actions):
        hs = [np.asarray(states[j], dtype=np.float64)]
        for i, (W, b) in enumerate(layers):
            z = W @ hs[-1] + b
            hs.append(np.tanh(z) if i + 1 < len(layers) else z)
        e = np.exp(hs[-1] - hs[-1].max())
        p = e / e.sum()
        onehot = np.zeros(len(p))
        onehot[a] = 1.0
        if old_probs is None:
            scale = signal[j]                       # d(R log p_a)/dz = R (onehot - p)
        else:
            r = p[a] / float(old_probs[j])
            held = min(max(r, 1 - clip_eps), 1 + clip_eps)
            # the minimum moves with r only where the unclipped term is the smaller one
            scale = signal[j] * r if r * signal[j] <= held * signal[j] else 0.0
        delta = scale * (onehot - p) / n
        for i in range(len(layers) - 1, -1, -1):
            W, _ = layers[i]
            grads[i][0][...] += np.outer(delta, hs[i])
            grads[i][1][...] += delta
            delta = W.T @ delta
            if i > 0:
                delta = delta * (1.0 - hs[i] ** 2)  # tanh'
    return np.concatenate([np.concatenate([gW.ravel(), gb]) for gW, gb in grads])


def update(weights, layer_sizes, states, actions, signal, lr, old_probs=None, clip_eps=0.2):
    """One ascent step; returns the new flat parameters (float64)."""
    g = objective_gradient(weights, layer_sizes, states, actions, signal, old_probs, clip_eps)
    return np.asarray(weights, dtype=np.float64) + lr * g
