"""Fused model update (plain SGD on the aggregate) against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W
from parity_util import compare, compare_sgd

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def params_for(P, seed):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    return torch.randn(P, generator=gen, device=DEV, dtype=torch.float32) * 0.05


def check_step(oracle_mod, w, lr, wd, where):
    print("case", where, "K", w.K, "P", w.P, w.dtype, "S", w.S, flush=True)
    p0 = params_for(w.P, 77 + w.K)
    p = p0.clone()
    st = D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p, lr, wd, w.segment_offsets)
    torch.cuda.synchronize()
    ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                           threads=16)
    ref = oracle_mod.sgd_step(ragg, p0.cpu().numpy(), lr, wd)
    compare_sgd(p.cpu().numpy(), ref, p0.cpu().numpy(), ragg, lr,
                is_bf16=(w.dtype == torch.bfloat16), where=where)
    # the statistics are those of the plain call
    compare(None, st.cpu().numpy(), ragg, rst, w.batch_sizes, is_bf16=(w.dtype == torch.bfloat16),
            where=where)
    return p0, p, st


@pytest.mark.parametrize("K,dtype", [(1, torch.float32), (4, torch.float32), (8, torch.bfloat16),
                                     (16, torch.bfloat16), (32, torch.float32), (33, torch.float32),
                                     (49, torch.float32), (64, torch.bfloat16),
                                     (2, torch.float16), (48, torch.float16)])
def test_fused_sgd_step(oracle_mod, K, dtype):
    rng = np.random.default_rng(300 + K)
    P = int(rng.integers(150_000, 250_000)) * 4 + int(rng.integers(1, 4))
    w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, 1e-2, seed=50 + K, device=DEV)
    check_step(oracle_mod, w, lr=0.1, wd=5e-4, where="sgd K=%d" % K)


@pytest.mark.parametrize("one_allocation", [True, False])
def test_fused_sgd_across_the_staging_phases(oracle_mod, monkeypatch, one_allocation):
    """One block, enough tiles to fill the LDS and both register banks more than once, so that
    updated parameters pass through every staging place before they are written."""
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "1")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")
    rng = np.random.default_rng(9)
    for K, dtype, tiles, tile in [(32, torch.float32, 2 * 102 + 38 + 3, 1024),
                                  (8, torch.bfloat16, 2 * 25 + 9 + 2, 256 * 4 * 8)]:
        w = W.make(K, tiles * tile - 5, dtype, rng.integers(8, 1025, size=K), 1e-3, 1e-2,
                   seed=600 + K, device=DEV, one_allocation=one_allocation)
        check_step(oracle_mod, w, lr=0.1, wd=5e-4, where="sgd phases K=%d" % K)


def test_fused_sgd_with_shared_tail_pieces(oracle_mod, monkeypatch):
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "8")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    rng = np.random.default_rng(10)
    for K, dtype, tile in [(32, torch.float32, 1024), (8, torch.bfloat16, 256 * 4 * 8)]:
        P = (8 * 40 + 2) * tile - 3
        assert (D.dynamix_plan_describe(K, P, 0 if dtype == torch.float32 else 1, None, 8)[:, 5]
                < 0).sum() >= 16
        w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, 1e-2, seed=640 + K,
                   device=DEV, one_allocation=False)
        check_step(oracle_mod, w, lr=0.1, wd=5e-4, where="sgd shared tail K=%d" % K)


def test_fused_sgd_with_segments(oracle_mod):
    w = W.config("C5", device=DEV, P=1_500_007)
    check_step(oracle_mod, w, lr=0.05, wd=0.0, where="sgd segments")


def test_fused_sgd_headline_shape(oracle_mod):
    w = W.config("C4", device=DEV)
    check_step(oracle_mod, w, lr=0.1, wd=1e-4, where="sgd C4")


def test_fused_update_equals_aggregate_then_update():
    # the fused result is the fp32 update applied to the very aggregate the plain call writes
    w = W.config("C2", device=DEV, P=2_000_003)
    agg, st = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes)
    p0 = params_for(w.P, 5)
    p = p0.clone()
    st2 = D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p, 0.25, 0.01)
    torch.cuda.synchronize()
    assert torch.equal(st, st2)
    want = torch.addcmul(p0, torch.addcmul(agg, p0, torch.tensor(0.01, device=DEV)),
                         torch.tensor(-0.25, device=DEV))
    np.testing.assert_allclose(p.cpu().numpy(), want.cpu().numpy(), rtol=3e-7, atol=1e-9)
    # zero learning rate leaves the parameters untouched, bit for bit
    q = p0.clone()
    D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, q, 0.0, 0.3)
    torch.cuda.synchronize()
    assert torch.equal(q, p0)


def test_fused_sgd_argument_checks():
    w = W.config("C1", device=DEV, P=10_000)
    p = params_for(w.P, 1)
    with pytest.raises(D.DynamixError):
        D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p, float("nan"))
    with pytest.raises(ValueError):
        D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p[:-1], 0.1)
