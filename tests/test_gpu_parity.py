"""Parity of the HIP path with the CPU oracle on the same seeded inputs (needs an MI355X).

Every call goes through the C ABI (ctypes binding); the oracle runs on the host copy of the very
same tensors.
"""
import numpy as np
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import workloads as W
from parity_util import HEAD, compare

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THREADS = 16


def run_gpu(w, entry=None, **kw):
    entry = entry or D.dynamix_grad_aggregate_stats_ex
    agg, st = entry(w.grads, w.batch_sizes, w.segment_offsets, **kw)
    torch.cuda.synchronize()
    return (None if agg is None else agg.cpu().numpy()), st.cpu().numpy()


def run_oracle(oracle_mod, w, want_agg=True):
    return oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, w.segment_offsets,
                                      want_agg=want_agg, threads=THREADS)


def check(oracle_mod, w, where):
    print("case", where, "K", w.K, "P", w.P, w.dtype, "S", w.S, flush=True)
    agg, st = run_gpu(w)
    ragg, rst = run_oracle(oracle_mod, w)
    compare(agg, st, ragg, rst, w.batch_sizes, is_bf16=(w.dtype == torch.bfloat16), where=where)
    return agg, st, ragg, rst


# ------------------------------------------------------------------ the named configurations
@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_config_full_size(oracle_mod, name):
    w = W.config(name, device=DEV)
    _, st, _, _ = check(oracle_mod, w, name)
    expected = 2000.0 if name == "C3" else 100.0
    assert abs(st[0, D.STAT["noise_scale"]] / expected - 1.0) < 0.05


def test_config_c4_full_size_headline(oracle_mod):
    # K=32, P=138M fp32 in K allocations made one by one: the shape, buffer layout and launch
    # configuration the benchmark times
    w = W.config("C4", device=DEV, one_allocation=False)
    assert all(g.data_ptr() % 256 == 0 for g in w.grads)
    _, st, _, _ = check(oracle_mod, w, "C4")
    assert abs(st[0, D.STAT["noise_scale"]] / 100.0 - 1.0) < 0.02


def test_config_c5_full_size_segments(oracle_mod):
    w = W.config("C5", device=DEV)
    assert w.S == 148
    check(oracle_mod, w, "C5")


# ------------------------------------------------------------------ shapes: every K, ragged tails
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 31, 32, 33, 48, 63, 64])
def test_worker_counts_and_ragged_tail(oracle_mod, K, dtype):
    rng = np.random.default_rng(1000 + K)
    # several tiles per block iteration plus a tail that is not a whole vector
    P = int(rng.integers(60_000, 90_000)) * 4 + int(rng.integers(1, 4))
    b = rng.integers(8, 1025, size=K)
    w = W.make(K, P, dtype, b, 1e-3, 1e-2, seed=7 + K, device=DEV)
    check(oracle_mod, w, "K=%d" % K)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 8, 9, 255, 1023, 1024, 1025, 4097, 262_145])
def test_tiny_and_boundary_lengths(oracle_mod, P, dtype):
    w = W.make(3, P, dtype, [32, 57, 132], 1e-3, 1e-2, seed=P, device=DEV)
    check(oracle_mod, w, "P=%d" % P)


def test_all_64_workers_large(oracle_mod):
    rng = np.random.default_rng(64)
    w = W.make(64, 3_000_001, torch.float32, rng.integers(32, 1025, size=64), 1e-3, 1e-2,
               seed=64, device=DEV)
    check(oracle_mod, w, "K=64 large")


# ------------------------------------------------------------------ segments
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
def test_segments_at_odd_offsets(oracle_mod, dtype):
    P = 1_200_007
    off = [0, 1, 2, 3, 7, 8, 130, 131, 4099, 4100, 65_537, 262_143, 262_145, 700_001, P - 1, P]
    rng = np.random.default_rng(3)
    sig = np.exp(rng.uniform(np.log(1e-4), np.log(1e-1), size=len(off) - 1))
    w = W.make(6, P, dtype, [16, 48, 100, 125, 256, 1024], 1e-3, sig, seed=11, device=DEV,
               segment_offsets=off)
    _, st, _, rst = check(oracle_mod, w, "odd segments")
    assert st.shape == (len(off), HEAD + 12)
    # the entry point that finds the number of segments itself gives the same bits
    _, st2 = run_gpu(w, entry=D.dynamix_grad_aggregate_stats)
    assert np.array_equal(st, st2)


RANDOM_K = [1, 2, 3, 5, 8, 9, 16, 17, 31, 32, 33, 40, 48, 49, 57, 64]   # every unroll / load width


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K", RANDOM_K)
def test_random_segmentations_for_every_kernel_shape(oracle_mod, K, dtype):
    """Random lengths and random segment cuts (neighbouring cuts, cuts inside one vector, cuts at
    tile edges) for every combination of unroll factor, load width and storage type."""
    rng = np.random.default_rng(5000 + K * 3 + [torch.float32, torch.bfloat16, torch.float16].index(dtype))
    for rep in range(2):
        P = int(rng.integers(1, 40)) if (rep == 1 and K % 3 == 0) else int(rng.integers(5_000, 400_000))
        S = int(min(P, rng.integers(1, 25)))
        cuts = set(int(c) for c in rng.choice(np.arange(1, P), size=S - 1, replace=False)) if S > 1 else set()
        for c in list(cuts)[:3]:                    # one-element segments and a cut at a tile edge
            if c + 1 < P:
                cuts.add(c + 1)
        tile_elems = 512 * 4
        if P > tile_elems + 1:
            cuts.add(tile_elems)
        off = [0] + sorted(cuts) + [P]
        sig = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), size=len(off) - 1))
        b = rng.integers(1, 1025, size=K)
        w = W.make(K, P, dtype, b, 1e-3, sig, seed=900 + K + rep, device=DEV, segment_offsets=off)
        check(oracle_mod, w, "random K=%d P=%d S=%d" % (K, P, len(off) - 1))


@pytest.mark.parametrize("K,dtype,U,NB,NB2", [(32, torch.float32, 1, 38, 26), (8, torch.float32, 4, 9, 7),
                                              (16, torch.bfloat16, 2, 9, 7), (2, torch.float16, 8, 2, 2),
                                              (40, torch.float32, 1, 76, 52), (44, torch.bfloat16, 1, 38, 26)])
@pytest.mark.parametrize("one_allocation", [True, False])
def test_tile_counts_around_the_staging_phases(oracle_mod, monkeypatch, K, dtype, U, NB, NB2,
                                               one_allocation):
    """One block walks the whole vector, so that the number of tiles it parks is known: just below,
    at and just above each hand-over (LDS full -> first register bank -> second bank -> flush),
    with a ragged last tile."""
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "1")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")       # the one block walks all of it in order
    vec = (4 if K <= 32 else 2) * (1 if dtype == torch.float32 else 2)   # elements per vector
    tile = 256 * U * vec                                   # elements per block iteration
    cycle = 2 * NB + NB2
    rng = np.random.default_rng(77 + K)
    for t in [1, NB - 1, NB, NB + 1, NB + NB2 - 1, NB + NB2, NB + NB2 + 1, cycle - 1, cycle,
              cycle + 1, cycle + NB, 2 * cycle + NB + NB2 + 1]:
        if t < 1:
            continue
        P = t * tile - int(rng.integers(0, vec + 2))       # sometimes whole, sometimes ragged
        b = rng.integers(8, 1025, size=K)
        w = W.make(K, P, dtype, b, 1e-3, 1e-2, seed=500 + t, device=DEV,
                   one_allocation=one_allocation)
        assert len(D.dynamix_plan_describe(K, P, {torch.float32: 0, torch.bfloat16: 1,
                                                  torch.float16: 2}[dtype], None, 1)) == 1
        check(oracle_mod, w, "phases K=%d tiles=%d" % (K, t))


@pytest.mark.parametrize("K,dtype,U", [(32, torch.float32, 1), (24, torch.float16, 1),
                                        (16, torch.bfloat16, 2), (8, torch.float32, 4),
                                        (2, torch.float16, 8)])
@pytest.mark.parametrize("blocks", ["1", "0"])
def test_interleaved_tile_order(oracle_mod, monkeypatch, K, dtype, U, blocks):
    """Buffers that start on 256-byte boundaries (allocations of their own) are read in groups of
    16 tiles whose chunks interleave; the groups start at multiples of 256 vectors, with a short
    tile in front where a segment starts elsewhere, and what is left after the last whole group is
    taken in consecutive tiles.  With DYNAMIX_SPREAD=0 the same call takes consecutive tiles: the
    aggregate must be the same bit for bit, the sums equal up to their order."""
    if blocks != "0":
        monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", blocks)
    vec = 4 * (1 if dtype == torch.float32 else 2)
    tile = 256 * U * vec
    group = 16 * tile
    rng = np.random.default_rng(31 + K)
    # three segments: a short one, one that starts at an odd element and holds two whole groups
    # and a ragged rest, and one of less than a group
    c1 = 5 * vec + 3
    c2 = c1 + 2 * group + 7 * tile + 11 * vec + 1
    P = c2 + 9 * tile - 2 - (vec if blocks == "0" else 0)   # (a shape of its own: plans are cached)
    b = rng.integers(8, 1025, size=K)
    w = W.make(K, P, dtype, b, 1e-3, [1e-2, 3e-2, 1e-3], seed=40 + K, device=DEV,
               segment_offsets=[0, c1, c2, P], one_allocation=False)
    assert all(g.data_ptr() % 256 == 0 for g in w.grads)
    agg, st, _, _ = check(oracle_mod, w, "interleaved K=%d blocks=%s" % (K, blocks))
    monkeypatch.setenv("DYNAMIX_SPREAD", "0")
    agg0, st0 = run_gpu(w)
    assert np.array_equal(agg, agg0)
    np.testing.assert_allclose(st, st0, rtol=1e-4 if dtype == torch.float32 else 1e-3)
    # the same buffers a vector off the boundary: consecutive tiles again, same results
    monkeypatch.delenv("DYNAMIX_SPREAD")
    w.grads = [torch.cat([g.new_zeros(vec), g])[vec:] for g in w.grads]
    assert all(g.data_ptr() % 256 == 16 for g in w.grads)
    agg1, st1 = run_gpu(w)
    assert np.array_equal(agg, agg1) and np.array_equal(st0, st1)


DTYPE_CODE = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}


@pytest.mark.parametrize("K,dtype,U,vec", [(32, torch.float32, 1, 4), (8, torch.float32, 4, 4),
                                            (16, torch.bfloat16, 2, 8), (2, torch.float16, 8, 8),
                                            (40, torch.float32, 1, 2), (64, torch.bfloat16, 1, 2)])
def test_shared_tail_pieces(oracle_mod, monkeypatch, K, dtype, U, vec):
    """The end of a long input is cut into short pieces that the blocks draw from a counter (here
    forced on a short input: a quarter of it, eight blocks).  Which block takes which piece varies
    from launch to launch; the results may not: every piece yields its own partial record."""
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "8")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    tile = 256 * U * vec
    rng = np.random.default_rng(61 + K)
    P = (8 * 40 + 3) * tile - 5
    cuts = sorted({int(c) for c in rng.integers(1, P, size=6)} | {P - 3 * tile - 7, P - 9})
    off = [0] + cuts + [P]
    pcs = D.dynamix_plan_describe(K, P, DTYPE_CODE[dtype], off, 8)
    assert (pcs[:, 5] < 0).sum() >= 16 and (pcs[:, 5] >= 0).sum() >= 8
    sig = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), size=len(off) - 1))
    w = W.make(K, P, dtype, rng.integers(8, 1025, size=K), 1e-3, sig, seed=70 + K, device=DEV,
               segment_offsets=off, one_allocation=False)
    agg, st, _, _ = check(oracle_mod, w, "shared tail K=%d" % K)
    for rep in range(3):
        agg2, st2 = run_gpu(w)
        assert np.array_equal(agg, agg2) and np.array_equal(st, st2), rep
    _, st3 = run_gpu(w, stats_only=True)
    assert np.array_equal(st, st3)


@pytest.mark.parametrize("K,U", [(8, 4), (32, 1)])
def test_pieces_that_start_off_the_group_boundaries(oracle_mod, K, U):
    """Many segments that start at odd elements: each piece first takes the vectors up to the next
    multiple of 256 as a short tile of its own, whose idle lanes may neither read nor write (the
    flush addresses the whole piece through one descriptor).  A stray write would race with the
    real one, so the aggregate is also compared over repeated launches."""
    tile = 256 * U * 4
    rng = np.random.default_rng(91 + K)
    sizes = rng.integers(17 * tile, 40 * tile, size=60) + rng.integers(1, 1000, size=60)
    off = [0] + [int(x) for x in np.cumsum(sizes)]
    P = off[-1]
    w = W.make(K, P, torch.float32, rng.integers(8, 1025, size=K), 1e-3,
               np.full(60, 1e-2), seed=17 + K, device=DEV, segment_offsets=off,
               one_allocation=False)
    agg, st, _, _ = check(oracle_mod, w, "short tiles in front K=%d" % K)
    for rep in range(5):
        agg2, st2 = run_gpu(w)
        assert np.array_equal(agg, agg2) and np.array_equal(st, st2), rep


def test_final_reduction_shared_by_several_blocks(oracle_mod, monkeypatch):
    """With some hundred pieces record 0 is folded by several blocks, the last of which to finish
    adds their sums in a fixed order: same bits in every launch, whichever block that is."""
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "64")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    K, tile = 32, 1024
    P = 64 * 100 * tile + 777
    off = [0, 5, 13 * tile + 1, 1000 * tile - 3, 5200 * tile + 2, P]
    assert len(D.dynamix_plan_describe(K, P, 0, off, 64)) >= 4 * 96     # four blocks for record 0
    rng = np.random.default_rng(123)
    w = W.make(K, P, torch.float32, rng.integers(8, 1025, size=K), 1e-3,
               [1e-2, 2e-2, 5e-3, 1e-2, 3e-2], seed=321, device=DEV, segment_offsets=off,
               one_allocation=False)
    agg, st, _, _ = check(oracle_mod, w, "final reduction in slices")
    for rep in range(6):
        _, st2 = run_gpu(w, stats_only=True)
        assert np.array_equal(st, st2), rep


def test_many_one_element_segments(oracle_mod):
    P = 3000
    w = W.make(4, P, torch.float32, [32, 64, 96, 128], 1e-3, 1e-2, seed=5, device=DEV,
               segment_offsets=list(range(P + 1)))
    check(oracle_mod, w, "one-element segments")


def test_c5_recipe_small(oracle_mod):
    w = W.config("C5", device=DEV, P=2_000_003)
    check(oracle_mod, w, "C5 small")


# ------------------------------------------------------------------ special and degenerate inputs
def test_single_worker_identity_is_bitwise(oracle_mod):
    w = W.make(1, 100_003, torch.float32, [77], 1e-3, 1e-2, seed=1, device=DEV)
    agg, st, _, _ = check(oracle_mod, w, "K=1")
    assert np.array_equal(agg, w.grads[0].cpu().numpy())
    assert st[0, 1] == 0.0 and st[0, HEAD + 1] == 0.0


def test_identical_workers(oracle_mod):
    w = W.make(1, 500_001, torch.float32, [64], 1e-3, 1e-2, seed=2, device=DEV)
    w.grads = [w.grads[0], w.grads[0].clone(), w.grads[0].clone(), w.grads[0].clone()]
    w.K, w.batch_sizes = 4, np.array([32, 32, 64, 128], dtype=np.int32)    # B = 256: exact weights
    agg, st, _, _ = check(oracle_mod, w, "identical")
    assert np.array_equal(agg, w.grads[0].cpu().numpy())
    assert st[0, 1] == 0.0 and (st[0, HEAD + 4:] == 0.0).all()
    w.batch_sizes = np.array([33, 50, 100, 77], dtype=np.int32)             # inexact weights
    _, st, _, _ = check(oracle_mod, w, "identical, inexact weights")
    assert st[0, 1] <= 1e-10 * st[0, 0] * w.batch_sizes.sum()


def test_all_zero_gradients(oracle_mod):
    w = W.make(3, 10_001, torch.float32, [32, 64, 96], 0.0, 0.0, seed=3, device=DEV)
    agg, st, _, rst = check(oracle_mod, w, "zeros")
    assert not agg.any() and np.isnan(st[0, 3]) and np.isnan(rst[0, 3])


def test_wide_dynamic_range(oracle_mod):
    w = W.make(5, 300_001, torch.float32, [8, 32, 100, 512, 1024], 1e-3, 1e-2, seed=4, device=DEV)
    scale = torch.exp(torch.linspace(-20.0, 20.0, w.P, device=DEV))
    w.grads = [(g * scale).contiguous() for g in w.grads]
    check(oracle_mod, w, "dynamic range")


def test_non_finite_inputs_propagate():
    w = W.make(3, 50_000, torch.float32, [32, 64, 96], 1e-3, 1e-2, seed=6, device=DEV)
    w.grads[1][12_345] = float("inf")
    w.grads[2][40_000] = float("nan")
    agg, st = run_gpu(w)
    assert np.isinf(agg[12_345]) and np.isnan(agg[40_000])
    assert np.isfinite(np.delete(agg, [12_345, 40_000])).all()
    assert np.isfinite(st[0, HEAD]) and np.isinf(st[0, HEAD + 1]) and np.isnan(st[0, HEAD + 2])


def test_fp16_subnormals_and_loss_scale_overflow(oracle_mod):
    """fp16 gradients are held to the fp32 tolerances (widening is exact, subnormals included).
    Unscaled they sit in the subnormal range; scaled by 2^16 one worker overflows to Inf, which
    shows in that worker's squared norm alone."""
    K, P = 6, 700_003
    w = W.make(K, P, torch.float32, [16, 32, 64, 64, 128, 256], 1e-6, 2e-5, seed=21, device=DEV)
    small = [g.to(torch.float16) for g in w.grads]
    sub = sum(int(((g != 0) & (g.abs() < 6.2e-5)).sum()) for g in small)
    assert sub > K * P // 2                                   # mostly subnormal values
    w.grads, w.dtype = small, torch.float16
    check(oracle_mod, w, "fp16 subnormal")

    w.grads = [(g.float() * 65536.0).to(torch.float16) for g in small]
    check(oracle_mod, w, "fp16 loss-scaled")
    w.grads[3][123_456] = float("inf")                        # what an overflowing scale leaves
    _, st = run_gpu(w, stats_only=True)
    n = st[0, HEAD:HEAD + K]
    assert np.isinf(n[3]) and np.isfinite(np.delete(n, 3)).all()
    assert not np.isfinite(st[0, 0]) and not np.isfinite(st[0, HEAD + K:]).any()


# ------------------------------------------------------------------ behaviour of the entry point
def test_bitwise_reproducible_and_stats_only():
    w = W.config("C2", device=DEV, P=3_000_001)
    a1, s1 = run_gpu(w)
    a2, s2 = run_gpu(w)
    assert np.array_equal(a1, a2) and np.array_equal(s1, s2)
    a3, s3 = run_gpu(w, stats_only=True)
    assert a3 is None and np.array_equal(s1, s3)


def test_other_stream_and_caller_buffers(oracle_mod):
    w = W.config("C1", device=DEV, P=400_003)
    out_agg = torch.full((w.P,), 7.0, dtype=torch.float32, device=DEV)
    out_st = torch.full((1, HEAD + 2 * w.K), 7.0, dtype=torch.float64, device=DEV)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        for _ in range(3):          # steady state reuses the cached plan and workspace
            a, st = D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, out_agg=out_agg,
                                                      out_stats=out_st, stream=s)
    s.synchronize()
    assert a is out_agg and st is out_st
    ragg, rst = run_oracle(oracle_mod, w)
    compare(out_agg.cpu().numpy(), out_st.cpu().numpy(), ragg, rst, w.batch_sizes, where="stream")
    assert D.dynamix_release_cached() == 0
    a2, st2 = run_gpu(w)
    assert np.array_equal(a2, out_agg.cpu().numpy())


def test_permuting_workers_permutes_their_entries(oracle_mod):
    w = W.config("C2", device=DEV, P=500_001)
    _, st = run_gpu(w)
    perm = np.random.default_rng(0).permutation(w.K)
    w2 = W.Workload(name="perm", K=w.K, P=w.P, dtype=w.dtype, batch_sizes=w.batch_sizes[perm],
                    grads=[w.grads[p] for p in perm], segment_offsets=None, m=w.m,
                    sigma=w.sigma, mu_sqnorm=w.mu_sqnorm)
    _, st2 = run_gpu(w2)
    # a worker's own squared norm does not depend on its slot; the aggregate only to rounding
    assert np.array_equal(st2[0, HEAD:HEAD + w.K], st[0, HEAD:HEAD + w.K][perm])
    np.testing.assert_allclose(st2[0, :7], st[0, :7], rtol=1e-5)


def test_kernel_timing_slots():
    w = W.config("C1", device=DEV, P=200_000)
    D.dynamix_timing_begin(2)
    for _ in range(3):                       # the third call finds no free slot and is not timed
        run_gpu(w)
    assert D.dynamix_timing_count() == 2
    for i in range(2):
        t_stream, t_final = D.dynamix_timing_read(i)
        assert 0.0 < t_stream < 50.0 and 0.0 < t_final < 50.0
    with pytest.raises(D.DynamixError):
        D.dynamix_timing_read(2)
    # only every third call timed: calls 0, 3 and 6 of seven
    D.dynamix_timing_every(3)
    D.dynamix_timing_begin(10)
    for _ in range(7):
        run_gpu(w)
    assert D.dynamix_timing_count() == 3
    assert all(0.0 < D.dynamix_timing_read(i)[0] < 50.0 for i in range(3))
    D.dynamix_timing_every(1)
    D.dynamix_timing_begin(0)
    assert D.dynamix_timing_count() == 0


def test_many_shapes_outlive_the_plan_cache(oracle_mod):
    # more distinct shapes than the cache keeps: the oldest plans are dropped and rebuilt
    w = W.config("C1", device=DEV, P=40_000)
    first = None
    for i in range(140):
        P = 20_000 + 7 * i
        sub = W.Workload(name="sub", K=w.K, P=P, dtype=w.dtype, batch_sizes=w.batch_sizes,
                         grads=[g[:P] for g in w.grads], segment_offsets=None, m=w.m,
                         sigma=w.sigma, mu_sqnorm=w.mu_sqnorm)
        agg, st = run_gpu(sub)
        if i == 0:
            first = (agg.copy(), st.copy(), sub)
    agg, st = run_gpu(first[2])              # its plan was evicted meanwhile
    assert np.array_equal(agg, first[0]) and np.array_equal(st, first[1])
    ragg, rst = run_oracle(oracle_mod, first[2])
    compare(agg, st, ragg, rst, w.batch_sizes, where="after eviction")


def test_buffers_allocated_one_by_one(oracle_mod):
    # same values whether the K buffers are rows of one allocation or K allocations
    w1 = W.config("C2", device=DEV, P=1_000_003)
    w2 = W.config("C2", device=DEV, P=1_000_003, one_allocation=False)
    assert all(torch.equal(a, b) for a, b in zip(w1.grads, w2.grads))
    a1, s1 = run_gpu(w1)
    a2, s2 = run_gpu(w2)
    # (rows of the slab are not 256-byte aligned here, the allocations are: the order in which
    # the sums are taken differs, the aggregate does not)
    assert np.array_equal(a1, a2)
    np.testing.assert_allclose(s1, s2, rtol=1e-4)
    check(oracle_mod, w2, "separate allocations")


def test_steady_state_call_can_be_captured_in_a_graph(oracle_mod, monkeypatch):
    # once its plan exists, a call only launches kernels: it can be recorded into a HIP graph and
    # replayed; every replay is checked against an eager call on the same (changed) inputs
    # (with a shared tail, so that the replays also depend on its counter being set back)
    monkeypatch.setenv("DYNAMIX_MAX_BLOCKS", "16")
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    w = W.config("C1", device=DEV, P=3_000_001)
    assert (D.dynamix_plan_describe(w.K, w.P, 0, None, 16)[:, 5] < 0).sum() >= 16
    out_agg = torch.empty(w.P, dtype=torch.float32, device=DEV)
    out_st = torch.empty((1, HEAD + 2 * w.K), dtype=torch.float64, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up on the capture stream builds the plan
        D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, out_agg=out_agg,
                                          out_stats=out_st, stream=side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, out_agg=out_agg,
                                          out_stats=out_st, stream=torch.cuda.current_stream())
    for rep in range(3):
        for g in w.grads:                   # new gradients in the same buffers
            g.mul_(1.0 + 0.25 * rep).add_(1e-4 * rep)
        torch.cuda.synchronize()
        out_agg.zero_()
        out_st.zero_()
        graph.replay()
        torch.cuda.synchronize()
        a_graph, s_graph = out_agg.cpu().numpy().copy(), out_st.cpu().numpy().copy()
        a_eager, s_eager = run_gpu(w)
        assert np.array_equal(a_graph, a_eager) and np.array_equal(s_graph, s_eager), rep
    ragg, rst = run_oracle(oracle_mod, w)
    compare(a_graph, s_graph, ragg, rst, w.batch_sizes, where="graph replay")


def test_recorded_call_carries_its_table_upload(oracle_mod):
    """A call recorded into a graph right after its plan was built, before any eager call has put
    the tables on the device for good: the replays must not depend on what ran eagerly."""
    w = W.config("C2", device=DEV, P=777_001)
    out_agg = torch.empty(w.P, dtype=torch.float32, device=DEV)
    out_st = torch.empty((1, HEAD + 2 * w.K), dtype=torch.float64, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    # the plan of a stream is built by the first call on it; the capture mode that tolerates the
    # allocation lets that first call be the recorded one
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side, capture_error_mode="relaxed"):
        D.dynamix_grad_aggregate_stats_ex(w.grads, w.batch_sizes, out_agg=out_agg,
                                          out_stats=out_st, stream=torch.cuda.current_stream())
    ragg, rst = run_oracle(oracle_mod, w)
    for rep in range(3):
        out_agg.zero_()
        out_st.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        compare(out_agg.cpu().numpy(), out_st.cpu().numpy(), ragg, rst, w.batch_sizes,
                where="recorded first call, replay %d" % rep)
        a_eager, s_eager = run_gpu(w)
        assert np.array_equal(out_agg.cpu().numpy(), a_eager) and np.array_equal(out_st.cpu().numpy(), s_eager)


def test_more_than_two_to_the_31_elements(oracle_mod):
    # indices beyond 32 bits: two workers, 2^31 + 4099 fp32 elements each (8.6 GB per buffer)
    P = (1 << 31) + 4099
    w = W.make(2, P, torch.float32, [48, 200], 1e-3, 1e-2, seed=31, device=DEV)
    agg, st = run_gpu(w)
    ragg, rst = oracle_mod.aggregate_stats(w.host_arrays(), w.batch_sizes, threads=THREADS)
    compare(agg, st, ragg, rst, w.batch_sizes, where="P > 2^31")
    assert st[0, 7] == float(P)
    # the last elements, beyond the 32-bit range, are written
    assert np.array_equal(agg[-5:].astype(np.float32), agg[-5:]) and np.abs(agg[-5:]).max() > 0


def test_two_streams_at_once():
    # calls on different streams use different plans and workspaces and may overlap
    w1 = W.config("C2", device=DEV, P=3_000_017)
    w2 = W.config("C1", device=DEV, P=3_000_017)
    ref1, ref2 = run_gpu(w1), run_gpu(w2)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for rep in range(4):
        with torch.cuda.stream(s1):
            o1 = D.dynamix_grad_aggregate_stats_ex(w1.grads, w1.batch_sizes, stream=s1)
        with torch.cuda.stream(s2):
            o2 = D.dynamix_grad_aggregate_stats_ex(w2.grads, w2.batch_sizes, stream=s2)
        outs.append((o1, o2))
    torch.cuda.synchronize()
    for o1, o2 in outs:
        assert np.array_equal(o1[0].cpu().numpy(), ref1[0]) and np.array_equal(o1[1].cpu().numpy(), ref1[1])
        assert np.array_equal(o2[0].cpu().numpy(), ref2[0]) and np.array_equal(o2[1].cpu().numpy(), ref2[1])
