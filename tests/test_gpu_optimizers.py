"""Fused model updates that carry optimizer state (SGD with momentum, Adam) against the CPU
oracle (needs an MI355X).  Each step starts from the float32 state the GPU holds, so that the
comparison is of one step at a time and nothing drifts."""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W
from parity_util import aggregate_error_bound, compare, compare_adam, compare_momentum

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
F = lambda x: float(np.float32(x))       # hyper-parameters as the C ABI's floats hold them


def randn(P, seed, scale):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    return torch.randn(P, generator=gen, device=DEV, dtype=torch.float32) * scale


def oracle_aggregate(oracle_mod, w):
    ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                           threads=16)
    dg = aggregate_error_bound(w.host_arrays(), w.batch_sizes, oracle_mod.widen)
    return ragg, rst, dg


def momentum_case(oracle_mod, w, lr, wd, mu, nesterov, steps, where, agg=None):
    print("case", where, "K", w.K, "P", w.P, w.dtype, "S", w.S, flush=True)
    ragg, rst, dg = agg or oracle_aggregate(oracle_mod, w)
    is_bf16 = w.dtype == torch.bfloat16
    p, buf = randn(w.P, 900 + w.K, 0.05), torch.zeros(w.P, dtype=torch.float32, device=DEV)
    for step in range(steps):
        p0, b0 = p.cpu().numpy(), buf.cpu().numpy()
        st = D.dynamix_grad_aggregate_stats_sgd_momentum(w.grads, w.batch_sizes, p, buf, lr, wd, mu,
                                                         nesterov, w.segment_offsets)
        torch.cuda.synchronize()
        rp, rb = oracle_mod.sgd_momentum_step(ragg, p0, b0, lr, wd, mu, nesterov)
        compare_momentum(p.cpu().numpy(), buf.cpu().numpy(), rp, rb, p0, b0, ragg, dg, lr, wd, mu,
                         nesterov, is_bf16=is_bf16, where="%s step %d" % (where, step))
        compare(None, st.cpu().numpy(), ragg, rst, w.batch_sizes, is_bf16=is_bf16, where=where)


def adam_case(oracle_mod, w, lr, b1, b2, eps, wd, decoupled, steps, where, agg=None, first_step=1):
    print("case", where, "K", w.K, "P", w.P, w.dtype, "S", w.S, flush=True)
    ragg, rst, dg = agg or oracle_aggregate(oracle_mod, w)
    is_bf16 = w.dtype == torch.bfloat16
    p = randn(w.P, 950 + w.K, 0.05)
    m = torch.zeros(w.P, dtype=torch.float32, device=DEV)
    v = torch.zeros(w.P, dtype=torch.float32, device=DEV)
    for step in range(first_step, first_step + steps):
        p0, m0, v0 = p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()
        st = D.dynamix_grad_aggregate_stats_adam(w.grads, w.batch_sizes, p, m, v, lr, step, b1, b2,
                                                 eps, wd, decoupled, w.segment_offsets)
        torch.cuda.synchronize()
        ref = oracle_mod.adam_step(ragg, p0, m0, v0, lr, b1, b2, eps, wd, decoupled, step)
        compare_adam((p.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()), ref, p0, m0, v0, ragg, dg,
                     lr, b1, b2, eps, wd, decoupled, step, is_bf16=is_bf16,
                     where="%s step %d" % (where, step))
        compare(None, st.cpu().numpy(), ragg, rst, w.batch_sizes, is_bf16=is_bf16, where=where)


CASES = [(1, torch.float32), (2, torch.bfloat16), (3, torch.float16), (8, torch.float32),
         (9, torch.bfloat16), (16, torch.float32), (17, torch.float16), (24, torch.float32),
         (24, torch.bfloat16), (25, torch.float32), (32, torch.float32), (32, torch.bfloat16)]


@pytest.mark.parametrize("K,dtype", CASES)
def test_fused_momentum_steps(oracle_mod, K, dtype):
    rng = np.random.default_rng(400 + K)
    P = int(rng.integers(150_000, 250_000)) * 4 + int(rng.integers(1, 4))
    w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, 1e-2, seed=60 + K, device=DEV)
    agg = oracle_aggregate(oracle_mod, w)
    momentum_case(oracle_mod, w, F(0.1), F(5e-4), F(0.9), False, 3, "momentum K=%d" % K, agg)
    momentum_case(oracle_mod, w, F(0.05), 0.0, F(0.8), True, 2, "nesterov K=%d" % K, agg)


@pytest.mark.parametrize("K,dtype", CASES)
def test_fused_adam_steps(oracle_mod, K, dtype):
    rng = np.random.default_rng(500 + K)
    P = int(rng.integers(150_000, 250_000)) * 4 + int(rng.integers(1, 4))
    w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, 1e-2, seed=80 + K, device=DEV)
    agg = oracle_aggregate(oracle_mod, w)
    adam_case(oracle_mod, w, F(1e-3), F(0.9), F(0.999), F(1e-8), F(1e-2), False, 3,
              "adam K=%d" % K, agg)
    adam_case(oracle_mod, w, F(1e-3), F(0.9), F(0.99), F(1e-6), F(1e-2), True, 2,
              "adamw K=%d" % K, agg, first_step=7)


def test_stateful_updates_with_segments_and_shared_tail(oracle_mod, monkeypatch):
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "8")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    rng = np.random.default_rng(12)
    for K, dtype, tile in [(24, torch.float32, 1024), (8, torch.bfloat16, 256 * 2 * 8),
                           (32, torch.float32, 512)]:
        P = (8 * 40 + 2) * tile - 3
        cuts = sorted({int(c) for c in rng.integers(1, P, size=5)} | {P - 3 * tile - 7, P - 9})
        off = [0] + cuts + [P]
        sig = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), size=len(off) - 1))
        w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, sig, seed=660 + K,
                   device=DEV, segment_offsets=off, one_allocation=False)
        agg = oracle_aggregate(oracle_mod, w)
        momentum_case(oracle_mod, w, F(0.1), F(1e-4), F(0.9), True, 2, "momentum tail K=%d" % K, agg)
        adam_case(oracle_mod, w, F(1e-3), F(0.9), F(0.999), F(1e-8), 0.0, False, 2,
                  "adam tail K=%d" % K, agg)


def test_first_momentum_step_is_plain_sgd():
    # a zero buffer: the fused momentum step equals the fused plain step, and the buffer becomes
    # the decayed gradient; both up to the order of the sums only in the statistics
    w = W.config("C2", device=DEV, P=1_000_003)
    p0 = randn(w.P, 3, 0.05)
    p1, p2, buf = p0.clone(), p0.clone(), torch.zeros_like(p0)
    D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p1, F(0.25), F(0.01))
    D.dynamix_grad_aggregate_stats_sgd_momentum(w.grads, w.batch_sizes, p2, buf, F(0.25), F(0.01),
                                                F(0.9), False)
    torch.cuda.synchronize()
    assert torch.equal(p1, p2)
    agg, _ = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes)
    torch.cuda.synchronize()
    a64, p64 = agg.double().cpu().numpy(), p0.double().cpu().numpy()
    assert (np.abs(buf.double().cpu().numpy() - (a64 + F(0.01) * p64))
            <= 2.0 ** -23 * (np.abs(a64) + F(0.01) * np.abs(p64))).all()


def test_stateful_update_argument_checks():
    w = W.config("C1", device=DEV, P=10_000)
    p, a, b = randn(w.P, 1, 0.1), torch.zeros(w.P, device=DEV), torch.zeros(w.P, device=DEV)
    with pytest.raises(D.DynamixError):
        D.dynamix_grad_aggregate_stats_sgd_momentum(w.grads, w.batch_sizes, p, a, float("nan"))
    with pytest.raises(D.DynamixError):
        D.dynamix_grad_aggregate_stats_adam(w.grads, w.batch_sizes, p, a, b, 1e-3, 0)     # step < 1
    with pytest.raises(D.DynamixError):
        D.dynamix_grad_aggregate_stats_adam(w.grads, w.batch_sizes, p, a, b, 1e-3, 1, beta1=1.0)
    with pytest.raises(ValueError):
        D.dynamix_grad_aggregate_stats_adam(w.grads, w.batch_sizes, p, a[:-1], b, 1e-3, 1)
    # more workers than the stateful kernels are built for
    K = D.DYNAMIX_K_MAX_STATEFUL + 1
    w25 = W.make(K, 5000, torch.float32, [32] * K, 1e-3, 1e-2, seed=2, device=DEV)
    p = randn(5000, 1, 0.1)
    a = torch.zeros(5000, device=DEV)
    with pytest.raises(D.DynamixError) as e:
        D.dynamix_grad_aggregate_stats_sgd_momentum(w25.grads, w25.batch_sizes, p, a, 0.1)
    assert e.value.status == D.binding.DYNAMIX_ERR_ARG
    torch.cuda.synchronize()
    assert not a.any()
