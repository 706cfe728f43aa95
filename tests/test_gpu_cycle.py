"""Per-cycle aggregation on the GPU against its CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from oracle.cycle_oracle import EXTRA, HEAD, cycle_summary
from paper_2510_08522_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def close(gpu, ref, rtol):
    gpu, ref = np.asarray(gpu), np.asarray(ref)
    assert gpu.shape == ref.shape
    assert (np.isnan(gpu) == np.isnan(ref)).all()
    fin = ~np.isnan(ref)
    np.testing.assert_allclose(gpu[fin], ref[fin], rtol=rtol, atol=0)


@pytest.mark.parametrize("K,S,iters", [(4, 0, 1), (4, 0, 7), (8, 5, 4), (32, 148, 3), (64, 2, 2)])
def test_cycle_matches_oracle_on_the_same_records(oracle_mod, K, S, iters):
    # the statistics records fed to both sides come from the CPU oracle on seeded inputs
    rng = np.random.default_rng(K * 1000 + S)
    P = 2000 + 13 * S
    b = rng.integers(8, 1025, size=K)
    off = None
    if S:
        off = np.concatenate([[0], np.sort(rng.choice(np.arange(1, P), S - 1, replace=False)), [P]])
    records = []
    for it in range(iters):
        g = [rng.standard_normal(P).astype(np.float32) * 1e-2 for _ in range(K)]
        records.append(oracle_mod.aggregate_stats(g, b, off)[1])
    window = None
    for it, st in enumerate(records):
        window = D.dynamix_cycle_accumulate(torch.from_numpy(st).to(DEV), window, first=(it == 0))
    summ = D.dynamix_cycle_summary(window, K, S, b, eta=0.3, delta=0.05)
    torch.cuda.synchronize()
    ref = cycle_summary(records, K, S, b, eta=0.3, delta=0.05)
    w = window.cpu().numpy()
    assert w[-1] == iters
    # same additions in the same order: the running sums agree to the last bit
    tot = np.zeros_like(records[0])
    for st in records:
        tot = tot + st
    assert np.array_equal(w[:-1], tot.ravel())
    close(summ.cpu().numpy(), ref, rtol=4e-16 * 8)


def test_cycle_restart_and_reuse():
    st1 = torch.arange(1, 17, dtype=torch.float64, device=DEV).reshape(1, 16)
    st2 = st1 * 3.0
    w = D.dynamix_cycle_accumulate(st1, None, first=True)
    D.dynamix_cycle_accumulate(st2, w)
    torch.cuda.synchronize()
    assert w[-1].item() == 2 and torch.equal(w[:-1], (st1 + st2).ravel())
    D.dynamix_cycle_accumulate(st2, w, first=True)           # a new cycle overwrites the window
    torch.cuda.synchronize()
    assert w[-1].item() == 1 and torch.equal(w[:-1], st2.ravel())


def test_end_to_end_cycle_from_gradients(oracle_mod):
    # gradients -> statistics -> cycle summary, every step on the GPU, against the two oracles
    base = W.config("C5", device=DEV, P=300_007)
    K, S, b = base.K, base.S, base.batch_sizes
    recs, window = [], None
    for it in range(4):
        w = W.make(K, base.P, torch.float32, b, 1e-3, base.sigma, seed=900 + it, device=DEV,
                   segment_offsets=base.segment_offsets)
        _, st = D.dynamix_grad_aggregate_stats_ex(w.grads, b, w.segment_offsets)
        window = D.dynamix_cycle_accumulate(st, window, first=(it == 0))
        recs.append(oracle_mod.aggregate_stats(w.host_arrays(), b, w.segment_offsets, threads=8)[1])
    summ = D.dynamix_cycle_summary(window, K, S, b, eta=1.0, delta=1.0).cpu().numpy()
    ref = cycle_summary(recs, K, S, b, eta=1.0, delta=1.0)
    R = HEAD + 2 * K
    for r in range(1 + S):
        g, o = summ[r * (R + EXTRA):(r + 1) * (R + EXTRA)], ref[r * (R + EXTRA):(r + 1) * (R + EXTRA)]
        big = o[7] >= 4096
        tol = 1e-5 if big else 1e-3      # tiny segments: single cancelling entries (see parity_util)
        for i in (0, 1, R + 1, R + 2, R + 3):
            assert abs(g[i] - o[i]) <= tol * abs(o[i]) + 1e-300, (r, i, g[i], o[i])
        np.testing.assert_allclose(g[HEAD:HEAD + K], o[HEAD:HEAD + K], rtol=1e-5)
        if big and abs(o[2]) > 0.05 * (o[0] + o[1] / b.sum()):
            assert abs(g[R] - o[R]) <= 1e-4 * abs(o[R])
    np.testing.assert_allclose(summ[-K:], ref[-K:], rtol=1e-15)
