"""More than 64 workers: the two-sweep kernel against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W
from parity_util import HEAD, compare

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check(oracle_mod, w, where):
    print("case", where, "K", w.K, "P", w.P, w.dtype, "S", w.S, flush=True)
    agg, st = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets)
    torch.cuda.synchronize()
    ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                           threads=16)
    compare(agg.cpu().numpy(), st.cpu().numpy(), ragg, rst, w.batch_sizes,
            is_bf16=(w.dtype == torch.bfloat16), where=where)
    # statistics only: the same sums bit for bit; and again with the aggregate: same bits
    _, st2 = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets,
                                               stats_only=True)
    agg3, st3 = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets)
    torch.cuda.synchronize()
    assert torch.equal(st, st2) and torch.equal(st, st3) and torch.equal(agg, agg3), where
    return agg, st


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K", [65, 80, 96, 128, 200, 256])
def test_wide_worker_counts(oracle_mod, K, dtype):
    rng = np.random.default_rng(7000 + K)
    # several super-tiles of 32 block iterations per block, ragged end, one odd segment cut
    P = int(rng.integers(700_000, 900_000)) * 4 + int(rng.integers(1, 4))
    cut = int(rng.integers(P // 3, P // 2)) | 1
    w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, [1e-2, 3e-2], seed=7100 + K,
               device=DEV, segment_offsets=[0, cut, P], one_allocation=bool(K % 2))
    _, st = check(oracle_mod, w, "wide K=%d" % K)
    assert st.shape == (3, HEAD + 2 * K)


@pytest.mark.parametrize("P", [1, 3, 5, 1023, 1025, 8193, 262_145])
def test_wide_tiny_and_boundary_lengths(oracle_mod, P):
    for dtype in (torch.float32, torch.float16):
        w = W.make(70, P, dtype, np.arange(70) + 8, 1e-3, 1e-2, seed=7200 + P, device=DEV)
        check(oracle_mod, w, "wide P=%d" % P)


def test_wide_one_block_through_several_super_tiles(oracle_mod, monkeypatch):
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "1")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")
    rng = np.random.default_rng(71)
    for dtype, vec in ((torch.float32, 4), (torch.bfloat16, 8)):
        tile = 256 * vec
        for tiles in (31, 32, 33, 64, 97):
            P = tiles * tile - int(rng.integers(0, vec + 2))
            w = W.make(72, P, dtype, rng.integers(8, 1025, size=72), 1e-3, 1e-2, seed=7300 + tiles,
                       device=DEV)
            assert len(D.dynamix_plan_describe(72, P, 0 if dtype == torch.float32 else 1, None, 1)) == 1
            check(oracle_mod, w, "wide one block, %d tiles" % tiles)


def test_wide_shared_tail_and_many_segments(oracle_mod, monkeypatch):
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "8")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    rng = np.random.default_rng(72)
    K, tile = 100, 1024
    P = (8 * 40 + 3) * tile - 5
    cuts = sorted({int(c) for c in rng.integers(1, P, size=9)} | {P - 3 * tile - 7, P - 9, 1, 2})
    off = [0] + cuts + [P]
    pcs = D.dynamix_plan_describe(K, P, 0, off, 8)
    assert (pcs[:, 5] < 0).sum() >= 16
    sig = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), size=len(off) - 1))
    w = W.make(K, P, torch.float32, rng.integers(8, 1025, size=K), 1e-3, sig, seed=7400, device=DEV,
               segment_offsets=off, one_allocation=False)
    agg, st = check(oracle_mod, w, "wide shared tail")
    for rep in range(3):
        a2, s2 = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets)
        torch.cuda.synchronize()
        assert torch.equal(agg, a2) and torch.equal(st, s2), rep


def test_wide_has_no_fused_update():
    K = 65
    w = W.make(K, 5000, torch.float32, [32] * K, 1e-3, 1e-2, seed=3, device=DEV)
    p = torch.zeros(5000, device=DEV)
    with pytest.raises(D.DynamixError) as e:
        D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p, 0.1)
    assert e.value.status == D.binding.DYNAMIX_ERR_ARG
