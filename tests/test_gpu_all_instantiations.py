"""Every shipped instantiation of the streaming pass against the CPU oracle (needs an MI355X).

The kernel is compiled once per worker count K = 1..64 and storage type (192 kernels).  Each one
is run here through the C ABI in its three modes (aggregate written, statistics only, fused SGD
step) on an input that one block walks alone, long enough to take the kernel through every
staging place of the aggregate (LDS, first and second register bank, timed and forced flushes)
more than twice, with a segment cut at an odd element and a ragged last vector.
"""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W
from parity_util import (aggregate_error_bound, compare, compare_adam, compare_momentum,
                         compare_sgd)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DTYPES = [torch.float32, torch.bfloat16, torch.float16]
CODE = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}


def kernel_shape(K, dtype, opt=0):
    """Elements per block iteration and the tile capacities of the staging places, as the kernel
    derives them from K, the storage type and the number of optimizer state vectors it carries:
    (tile elements, LDS tiles, second-bank tiles, tiles per flush cycle)."""
    lw = 4 if K <= 32 else 2 if K <= 48 else 1          # 32-bit words per lane and load
    if opt and K > 24:
        lw = 2                                            # the updates with state: 8-byte loads
    q = 1 if dtype == torch.float32 else 2               # stores per vector of the aggregate
    if opt == 0:
        u = 8 if K <= 2 else 4 if K <= 8 else 2 if K <= 16 else 1
    else:
        u = 4 if K <= 2 else 2 if K <= 8 else 1
    slots = 152 * 1024 // (256 * lw * 4)
    per_tile = u * q * (1 + opt)                          # one vector per stream written
    nb = slots // per_tile
    nb2 = (256 - nb * per_tile * lw) // (per_tile * lw)
    cycle = 2 * nb + nb2 if K <= 44 else nb
    return 256 * u * lw * q, nb, nb2, cycle


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("K", range(1, 65))
def test_instantiation(oracle_mod, monkeypatch, K, dtype):
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "1")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")
    tile, nb, nb2, cycle = kernel_shape(K, dtype)
    rng = np.random.default_rng(8000 + 3 * K + CODE[dtype])
    # first segment: two flush cycles and a bit; second: starts at an odd element, fills the LDS
    # once and spills into the first bank
    cut = (2 * cycle + 2) * tile + 3
    P = cut + (nb + 2) * tile - int(rng.integers(1, 6))
    off = [0, cut, P]
    assert len(D.dynamix_plan_describe(K, P, CODE[dtype], off, 1)) == 2
    b = rng.integers(8, 1025, size=K)
    w = W.make(K, P, dtype, b, 1e-3, [1e-2, 3e-2], seed=8100 + K, device=DEV, segment_offsets=off,
               one_allocation=bool(K % 2))      # rows of one slab, or K aligned allocations
    is_bf16 = dtype == torch.bfloat16
    where = "K=%d %s" % (K, str(dtype).split(".")[1])
    print("case", where, "P", P, "aggregate written", flush=True)
    agg, st = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets)
    torch.cuda.synchronize()
    ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                           threads=16)
    compare(agg.cpu().numpy(), st.cpu().numpy(), ragg, rst, w.batch_sizes, is_bf16=is_bf16,
            where=where)

    print("case", where, "statistics only", flush=True)
    _, st2 = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets,
                                               stats_only=True)
    torch.cuda.synchronize()
    assert torch.equal(st, st2), where

    print("case", where, "fused SGD", flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(8200 + K)
    p0 = torch.randn(P, generator=gen, device=DEV, dtype=torch.float32) * 0.05
    p = p0.clone()
    st3 = D.dynamix_grad_aggregate_stats_sgd(w.grads, w.batch_sizes, p, 0.1, 5e-4,
                                             w.segment_offsets)
    torch.cuda.synchronize()
    assert torch.equal(st, st3), where
    compare_sgd(p.cpu().numpy(), oracle_mod.sgd_step(ragg, p0.cpu().numpy(), 0.1, 5e-4),
                p0.cpu().numpy(), ragg, 0.1, is_bf16=is_bf16, where=where)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("K", range(1, D.DYNAMIX_K_MAX_STATEFUL + 1))
def test_stateful_instantiation(oracle_mod, monkeypatch, K, dtype):
    """The kernels that carry optimizer state (momentum: one state vector, Adam: two), one block
    through two flush cycles and a segment cut, as above."""
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "1")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")
    F = lambda x: float(np.float32(x))
    is_bf16 = dtype == torch.bfloat16
    for opt in (1, 2):
        tile, nb, nb2, cycle = kernel_shape(K, dtype, opt)
        rng = np.random.default_rng(9000 + 7 * K + 3 * CODE[dtype] + opt)
        cut = (2 * cycle + 2) * tile + 3
        P = cut + (nb + 2) * tile - int(rng.integers(1, 6))
        off = [0, cut, P]
        w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, [1e-2, 3e-2], seed=9100 + K,
                   device=DEV, segment_offsets=off, one_allocation=bool(K % 2))
        where = "K=%d %s opt=%d" % (K, str(dtype).split(".")[1], opt)
        print("case", where, "P", P, flush=True)
        ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                               threads=16)
        dg = aggregate_error_bound(w.host_arrays(), w.batch_sizes, oracle_mod.widen)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(9200 + K)
        p = torch.randn(P, generator=gen, device=DEV, dtype=torch.float32) * 0.05
        s1 = torch.randn(P, generator=gen, device=DEV, dtype=torch.float32) * 1e-3
        s2 = torch.rand(P, generator=gen, device=DEV, dtype=torch.float32) * 1e-5
        p0, a0, b0 = p.cpu().numpy(), s1.cpu().numpy(), s2.cpu().numpy()
        if opt == 1:
            st = D.dynamix_grad_aggregate_stats_sgd_momentum(
                w.grads, w.batch_sizes, p, s1, F(0.1), F(5e-4), F(0.9), bool(K % 2),
                w.segment_offsets)
            torch.cuda.synchronize()
            rp, rb = oracle_mod.sgd_momentum_step(ragg, p0, a0, F(0.1), F(5e-4), F(0.9), bool(K % 2))
            compare_momentum(p.cpu().numpy(), s1.cpu().numpy(), rp, rb, p0, a0, ragg, dg, F(0.1),
                             F(5e-4), F(0.9), bool(K % 2), is_bf16=is_bf16, where=where)
        else:
            st = D.dynamix_grad_aggregate_stats_adam(
                w.grads, w.batch_sizes, p, s1, s2, F(1e-3), 3, F(0.9), F(0.999), F(1e-8), F(1e-2),
                bool(K % 2), w.segment_offsets)
            torch.cuda.synchronize()
            ref = oracle_mod.adam_step(ragg, p0, a0, b0, F(1e-3), F(0.9), F(0.999), F(1e-8),
                                       F(1e-2), bool(K % 2), 3)
            compare_adam((p.cpu().numpy(), s1.cpu().numpy(), s2.cpu().numpy()), ref, p0, a0, b0,
                         ragg, dg, F(1e-3), F(0.9), F(0.999), F(1e-8), F(1e-2), bool(K % 2), 3,
                         is_bf16=is_bf16, where=where)
        compare(None, st.cpu().numpy(), ragg, rst, w.batch_sizes, is_bf16=is_bf16, where=where)
