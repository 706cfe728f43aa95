"""The entry point that allocates nothing (workspace in the library's static device array)
against the allocating entry point it is a variant of (needs an MI355X).

Both run the same kernels on the same work decomposition, so the results must agree bit for bit,
which is stricter than the tolerance against the oracle that the allocating entry point is held
to elsewhere.  The static array keeps the last call's tables: the calls here change shape from one
to the next (a smaller input after a larger one, then the larger one again) and repeat a shape.
"""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(w, stats_only=False):
    """(aggregate, statistics) of the allocating and of the static entry point, on caller-owned
    outputs pre-filled with a pattern."""
    outs = []
    for entry in (D.dynamix_grad_aggregate_stats_ex, D.dynamix_grad_aggregate_stats_static):
        agg = None if stats_only else torch.full((w.P,), 7.0, dtype=torch.float32, device=DEV)
        st = torch.full((1 + w.S, D.DYNAMIX_STATS_HEAD + 2 * w.K), 7.0, dtype=torch.float64,
                        device=DEV)
        entry(w.grads, w.batch_sizes, w.segment_offsets, out_agg=agg, out_stats=st,
              stats_only=stats_only)
        torch.cuda.synchronize()
        outs.append((None if agg is None else agg.cpu().numpy(), st.cpu().numpy()))
    return outs


def same(pair):
    (a0, s0), (a1, s1) = pair
    assert np.array_equal(s0, s1, equal_nan=True)
    if a0 is not None:
        assert np.array_equal(a0, a1, equal_nan=True)


def test_static_entry_matches_the_allocating_one_on_two_calls_in_a_row(oracle_mod):
    print("case static: C5 recipe, 3M elements, 148 segments", flush=True)
    big = W.config("C5", device=DEV, P=3_000_011, one_allocation=False)
    same(both(big))
    print("case static: smaller input right after (K=32, 700k elements, no segments)", flush=True)
    rng = np.random.default_rng(5)
    small = W.make(32, 700_001, torch.float32, rng.integers(16, 257, size=32), 1e-3, 1e-2,
                   seed=77, device=DEV)
    pair = both(small)
    same(pair)
    # and the static result is the oracle's, to the usual tolerance
    from parity_util import compare
    ragg, rst = oracle_mod.aggregate_stats(small.host_arrays(), small.batch_sizes, threads=16)
    compare(pair[1][0], pair[1][1], ragg, rst, small.batch_sizes, where="static small")
    print("case static: the same shape again, then the large one again, then bf16", flush=True)
    same(both(small))
    same(both(big, stats_only=True))
    same(both(big))
    w16 = W.config("C3", device=DEV, P=1_000_003)
    same(both(w16))


def test_static_entry_with_a_shared_tail_and_sliced_final_reduction(monkeypatch):
    # long spans: tail pieces drawn from the counter in the static array, record 0 folded in slices
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "64")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    K, tile = 32, 1024
    P = 64 * 100 * tile + 777
    off = [0, 5, 13 * tile + 1, 1000 * tile - 3, 5200 * tile + 2, P]
    assert len(D.dynamix_plan_describe(K, P, 0, off, 64)) >= 4 * 96
    rng = np.random.default_rng(6)
    w = W.make(K, P, torch.float32, rng.integers(8, 1025, size=K), 1e-3,
               [1e-2, 2e-2, 5e-3, 1e-2, 3e-2], seed=78, device=DEV, segment_offsets=off,
               one_allocation=False)
    print("case static: shared tail, sliced final reduction", flush=True)
    for rep in range(3):
        same(both(w))


def test_static_entry_rejects_what_does_not_fit():
    # one-element segments: 6 MB of tables and partial sums
    K, P = 4, 60_000
    w = W.make(K, P, torch.float32, [32, 64, 96, 128], 1e-3, 1e-2, seed=79, device=DEV,
               segment_offsets=list(range(P + 1)))
    st = torch.full((1 + w.S, D.DYNAMIX_STATS_HEAD + 2 * K), 7.0, dtype=torch.float64, device=DEV)
    agg = torch.full((P,), 7.0, dtype=torch.float32, device=DEV)
    print("case static: capacity error", flush=True)
    with pytest.raises(D.DynamixError) as e:
        D.dynamix_grad_aggregate_stats_static(w.grads, w.batch_sizes, w.segment_offsets,
                                              out_agg=agg, out_stats=st)
    assert e.value.status == D.DYNAMIX_ERR_CAPACITY
    torch.cuda.synchronize()
    assert (agg == 7.0).all() and (st == 7.0).all()        # nothing was enqueued
    # the allocating entry point takes the same call, and the static one still works afterwards
    D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, w.segment_offsets, out_agg=agg,
                                      out_stats=st)
    small = W.config("C1", device=DEV, P=50_001)
    same(both(small))


def test_static_entry_recorded_into_a_graph_without_a_call_before(oracle_mod):
    """The use the entry point is for: the very first call with a shape is made under stream
    capture, in the capture mode that rejects allocations.  Replays are interleaved with eager
    calls of another shape, which overwrite the tables in the static array in between; every
    replay and every eager call must still give the allocating entry point's bits."""
    wa = W.make(12, 900_001, torch.float32, np.arange(12) * 7 + 16, 1e-3, 1e-2, seed=90, device=DEV,
                one_allocation=False)
    wb = W.config("C1", device=DEV, P=333_337)
    ref_a = D.dynamix_grad_aggregate_stats_ex(wa.grads, wa.batch_sizes)
    ref_b = D.dynamix_grad_aggregate_stats_ex(wb.grads, wb.batch_sizes)
    torch.cuda.synchronize()
    agg_a = torch.empty(wa.P, dtype=torch.float32, device=DEV)
    st_a = torch.empty((1, D.DYNAMIX_STATS_HEAD + 2 * wa.K), dtype=torch.float64, device=DEV)
    agg_b, st_b = torch.empty_like(ref_b[0]), torch.empty_like(ref_b[1])
    print("case static: first call with a shape recorded into a graph", flush=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        D.dynamix_grad_aggregate_stats_static(wa.grads, wa.batch_sizes, out_agg=agg_a,
                                              out_stats=st_a, stream=torch.cuda.current_stream())
    for rep in range(3):
        print("case static: replay", rep, flush=True)
        agg_a.fill_(7.0)
        st_a.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(agg_a, ref_a[0]) and torch.equal(st_a, ref_a[1]), rep
        # an eager call of another shape in between overwrites the array's tables
        D.dynamix_grad_aggregate_stats_static(wb.grads, wb.batch_sizes, out_agg=agg_b, out_stats=st_b)
        torch.cuda.synchronize()
        assert torch.equal(agg_b, ref_b[0]) and torch.equal(st_b, ref_b[1]), rep
    # an eager call of the recorded shape after all that
    agg_a.fill_(7.0)
    D.dynamix_grad_aggregate_stats_static(wa.grads, wa.batch_sizes, out_agg=agg_a, out_stats=st_a)
    torch.cuda.synchronize()
    assert torch.equal(agg_a, ref_a[0]) and torch.equal(st_a, ref_a[1])
