"""Host-side checks of the C ABI that need no GPU: the library loads and exports what the header
declares, argument validation happens before any HIP call, and the work decomposition covers
every element exactly once."""
import ctypes
import os
import re
import shutil
import subprocess

import numpy as np
import pytest

import paper_2510_08522_amd as D
from paper_2510_08522_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dynamix.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dynamix_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"dynamix_grad_aggregate_stats", "dynamix_grad_aggregate_stats_ex",
            "dynamix_stats_count", "dynamix_status_string", "dynamix_release_cached",
            "dynamix_plan_describe"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    # the Python layer carries the same names
    for n in names:
        assert hasattr(D, n), n


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_header_is_plain_c_and_links_from_a_c_program(tmp_path):
    """The boundary is a C ABI: a strict C99 translation unit that includes the header, takes the
    address of every declared function and calls the two that need no device."""
    names = declared_functions()
    src = tmp_path / "use_dynamix.c"
    src.write_text(
        '#include "dynamix.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    const void* fns[] = {%s};\n"
        '    printf("%%d %%lld %%s\\n", (int)(sizeof fns / sizeof fns[0]),\n'
        "           (long long)dynamix_stats_count(32, 148), dynamix_status_string(DYNAMIX_ERR_ALIGN));\n"
        "    return fns[0] == 0;\n}\n" % ", ".join("(const void*)%s" % n for n in names))
    exe = tmp_path / "use_dynamix"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-Wno-pedantic",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-ldynamix", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 2)
    assert int(out[0]) == len(names) and int(out[1]) == 149 * 72
    assert out[2].strip() == "misaligned pointer"


def test_stats_count_and_status_strings():
    assert D.dynamix_stats_count(4, 0) == 16
    assert D.dynamix_stats_count(32, 148) == 149 * 72
    assert D.dynamix_stats_count(0, 0) == -1 and D.dynamix_stats_count(257, 0) == -1
    assert D.dynamix_stats_count(256, 1) == 2 * 520
    assert D.dynamix_stats_count(4, -1) == -1
    seen = {D.dynamix_status_string(i) for i in range(8)}
    assert len(seen) == 8 and D.dynamix_status_string(0) == "ok"
    assert D.dynamix_status_string(99) == "unknown status"


A16, ST = 0x1000, 0x2000     # fake, suitably aligned "device" addresses: never dereferenced


def raw(ptrs, b, K, P, dtype=0, off=None, S=0, agg=A16, stats=ST, explicit=True):
    return B.call_raw(ptrs, b, K, P, dtype, off, S, agg, stats, None, explicit_count=explicit)


def test_validation_precedes_any_device_work():
    ok_p, ok_b = [A16, A16 + 64], [32, 64]
    assert raw(None, ok_b, 2, 100) == B.DYNAMIX_ERR_NULL
    assert raw(ok_p, None, 2, 100) == B.DYNAMIX_ERR_NULL
    assert raw(ok_p, ok_b, 2, 100, stats=None) == B.DYNAMIX_ERR_NULL
    assert raw([A16, None], ok_b, 2, 100) == B.DYNAMIX_ERR_NULL
    assert raw(ok_p, ok_b, 0, 100) == B.DYNAMIX_ERR_ARG
    assert raw([A16] * 257, [1] * 257, 257, 100) == B.DYNAMIX_ERR_ARG
    assert raw(ok_p, ok_b, 2, 0) == B.DYNAMIX_ERR_ARG
    assert raw(ok_p, ok_b, 2, 100, dtype=3) == B.DYNAMIX_ERR_ARG
    assert raw(ok_p, ok_b, 2, 100, dtype=-1) == B.DYNAMIX_ERR_ARG
    assert raw(ok_p, [32, 0], 2, 100) == B.DYNAMIX_ERR_ARG
    assert raw(ok_p, [32, -5], 2, 100) == B.DYNAMIX_ERR_ARG
    assert raw([A16, A16 + 4], ok_b, 2, 100) == B.DYNAMIX_ERR_ALIGN
    assert raw(ok_p, ok_b, 2, 100, agg=A16 + 8) == B.DYNAMIX_ERR_ALIGN
    assert raw(ok_p, ok_b, 2, 100, stats=ST + 4) == B.DYNAMIX_ERR_ALIGN


def test_stateful_update_validation_precedes_any_device_work():
    lib = B.load()
    K = 3
    ptrs = (ctypes.c_void_p * K)(A16, A16 + 64, A16 + 128)
    b = (ctypes.c_int32 * K)(32, 64, 96)

    def momentum(params=A16 + 256, buf=A16 + 512, lr=0.1, k=K, pp=ptrs, bb=b):
        return lib.dynamix_grad_aggregate_stats_sgd_momentum(pp, bb, k, 100, 0, None, 0, params, buf,
                                                             lr, 0.0, 0.9, 0, ST, None)

    def adam(params=A16 + 256, m=A16 + 512, v=A16 + 768, lr=1e-3, b1=0.9, b2=0.999, step=1):
        return lib.dynamix_grad_aggregate_stats_adam(ptrs, b, K, 100, 0, None, 0, params, m, v, lr, b1,
                                                     b2, 1e-8, 0.0, 0, step, ST, None)

    assert momentum(params=None) == B.DYNAMIX_ERR_NULL and momentum(buf=None) == B.DYNAMIX_ERR_NULL
    assert momentum(lr=float("nan")) == B.DYNAMIX_ERR_ARG
    assert momentum(buf=A16 + 516) == B.DYNAMIX_ERR_ALIGN
    many = B.DYNAMIX_K_MAX_STATEFUL + 1
    assert momentum(k=many, pp=(ctypes.c_void_p * many)(*[A16 + 64 * i for i in range(many)]),
                    bb=(ctypes.c_int32 * many)(*[32] * many)) == B.DYNAMIX_ERR_ARG
    assert adam(m=None) == B.DYNAMIX_ERR_NULL and adam(v=None) == B.DYNAMIX_ERR_NULL
    assert adam(step=0) == B.DYNAMIX_ERR_ARG and adam(b1=1.0) == B.DYNAMIX_ERR_ARG
    assert adam(b2=-0.1) == B.DYNAMIX_ERR_ARG and adam(lr=float("nan")) == B.DYNAMIX_ERR_ARG
    assert adam(v=A16 + 772) == B.DYNAMIX_ERR_ALIGN


def test_segment_offsets_validation():
    p, b = [A16, A16 + 64], [32, 64]
    bad = B.DYNAMIX_ERR_SEGMENTS
    assert raw(p, b, 2, 100, off=[1, 50, 100], S=2) == bad          # does not start at 0
    assert raw(p, b, 2, 100, off=[0, 50, 50, 100], S=3) == bad      # empty segment
    assert raw(p, b, 2, 100, off=[0, 60, 50, 100], S=3) == bad      # decreasing
    assert raw(p, b, 2, 100, off=[0, 50, 99], S=2) == bad           # does not end at P
    assert raw(p, b, 2, 100, off=[0, 50, 100], S=0) == bad          # offsets without a count
    assert raw(p, b, 2, 100, off=None, S=2) == bad                  # count without offsets
    assert raw(p, b, 2, 100, off=[0, 50, 100], S=-1) == bad
    # the entry point that scans for the terminating entry
    assert raw(p, b, 2, 100, off=[0, 50, 120], explicit=False) == bad
    assert raw(p, b, 2, 100, off=[0, 50, 50, 100], explicit=False) == bad
    assert raw(p, b, 2, 100, off=[5, 50, 100], explicit=False) == bad
    assert raw(p, b, 2, 0, off=[0, 50, 100], explicit=False) == B.DYNAMIX_ERR_ARG


def unroll_for(K):
    return 8 if K <= 2 else 4 if K <= 8 else 2 if K <= 16 else 1


def check_cover(K, P, dtype, off, max_blocks):
    """Replay the kernel's iteration space on the host: the body of whole vectors of every piece
    plus its boundary vectors must touch each element exactly once."""
    vec = (1 if K > 48 else 2 if K > 32 else 4) * (1 if dtype == 0 else 2)   # elements per lane and load
    tile = 256 * unroll_for(K)                              # vectors per block iteration
    pcs = D.dynamix_plan_describe(K, P, dtype, off, max_blocks)
    assert len(pcs) >= 1
    own = pcs[pcs[:, 5] >= 0]                                   # pieces that belong to a block
    assert pcs[0, 5] == 0                                       # (the rest: the shared tail)
    assert (np.diff(own[:, 5]) >= 0).all()                      # pieces sorted by owning block
    assert own[:, 5].max() < max_blocks
    assert set(own[:, 5].tolist()) == set(range(int(own[:, 5].max()) + 1))   # no idle block index
    assert (np.diff(pcs[:, 3]) > 0).all()                       # and all of them by position
    cover = np.zeros(P, dtype=np.int32)
    for vb, ve, step, elo, ehi, _ in pcs.tolist():
        assert 0 <= vb < ve and step == tile
        assert vb * vec <= elo < ehi <= min(P, ve * vec)
        assert elo < (vb + 1) * vec and ehi > (ve - 1) * vec    # only the end vectors are cut
        body_b, body_e = vb, ve
        head_cut, tail_cut = elo > vb * vec, ehi < ve * vec
        if head_cut:
            body_b += 1
            cover[elo:min(ehi, (vb + 1) * vec)] += 1
        if tail_cut and ve - 1 >= body_b:
            body_e -= 1
            cover[(ve - 1) * vec:ehi] += 1
        if body_b < body_e:
            cover[body_b * vec:body_e * vec] += 1
    assert (cover == 1).all()
    if off is not None:                                          # pieces never straddle a segment
        seg_of = np.searchsorted(np.asarray(off), pcs[:, 3], side="right") - 1
        assert (np.asarray(off)[seg_of + 1] >= pcs[:, 4]).all()
        assert (np.diff(seg_of) >= 0).all()
    return pcs


@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_plan_covers_every_element_once(dtype):
    rng = np.random.default_rng(5)
    for K, P, mb in [(1, 1, 512), (4, 3, 512), (4, 1_000_000, 512), (8, 1_000_003, 1024),
                     (32, 777_777, 512), (64, 300_001, 256), (16, 2_000_001, 7), (3, 65_537, 1)]:
        check_cover(K, P, dtype, None, mb)
        S = int(min(P, rng.integers(1, 40)))
        cuts = np.sort(rng.choice(np.arange(1, P), size=S - 1, replace=False)) if S > 1 else []
        off = [0] + [int(c) for c in cuts] + [P]
        check_cover(K, P, dtype, off, mb)
    # one-element segments and boundaries inside a single vector
    check_cover(4, 5000, dtype, [0, 1, 2, 130, 131, 4099, 4100, 5000], 4)
    check_cover(5, 20, dtype, list(range(21)), 512)


def test_plan_for_the_headline_shape_is_balanced():
    pcs = check_cover(32, 138_000_000, 0, None, 256)
    own = pcs[pcs[:, 5] >= 0]
    assert len(own) == 256                                       # one span per compute unit
    spans = np.diff(np.append(own[:, 0], pcs[-1, 1]))           # (a block's part and its tail pieces)
    tiles = -(-spans // 256)
    assert tiles.max() - tiles.min() <= 1


def test_spans_start_on_wave_boundaries_and_small_inputs_use_every_unit():
    for K, P, dtype in [(4, 1_000_000, 0), (16, 25_600_000, 1), (33, 999_999, 2), (64, 123_457, 0)]:
        pcs = check_cover(K, P, dtype, None, 256)
        gran = 256 if 8 <= K <= 32 else 64       # 4 KB where the kernel interleaves chunks
        assert (pcs[:, 0] % gran == 0).all()
        n = pcs[:, 1] - pcs[:, 0]
        assert n[:-1].max() - n[:-1].min() <= gran and n[-1] <= n[:-1].max()
    assert len(check_cover(4, 1_000_000, 0, None, 256)) == 256      # 122 tiles, 256 spans
    assert len(check_cover(4, 2_047, 0, None, 256)) == 1            # one block per 512 vectors
    assert len(check_cover(4, 4_096, 0, None, 256)) == 2


def test_long_spans_end_in_shared_tail_pieces(monkeypatch):
    """The last 3 % of every long span belong to no block: they are cut into ever shorter
    pieces, down to two tiles, which any block draws when its own part is done."""
    K, P, tile, grid = 32, 138_000_000, 256, 256
    pcs = check_cover(K, P, 0, None, grid)
    own = pcs[:, 5] >= 0
    assert own.sum() == grid
    n = (pcs[:, 1] - pcs[:, 0])
    starts = np.where(own)[0]
    for b in (0, 1, 100, 255):
        mine = pcs[starts[b]:(starts[b + 1] if b + 1 < grid else len(pcs))]
        tiles = int((mine[-1, 1] - mine[0, 0]) // tile)          # 526 or 527 (the last: 525 and a rest)
        assert tiles in (525, 526, 527)
        sizes = (mine[:, 1] - mine[:, 0]) // tile
        assert sizes.tolist() == [tiles - 15, 7, 4, 2, 2]      # each half of what is left
        assert mine[:, 5].tolist() == [b, -1, -2, -3, -4]        # the round in which it is drawn
        assert (mine[1:, 0] % tile == 0).all()
    assert pcs[-1, 1] == -(-P // 4)
    # short inputs have none; the environment can force or forbid one
    assert (check_cover(K, 256 * 60 * 1024, 0, None, 256)[:, 5] >= 0).all()
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "0")
    assert (check_cover(K, P, 0, None, 256)[:, 5] >= 0).all()
    monkeypatch.setenv("DYNAMIX_TAIL_PERMILLE", "250")
    rng = np.random.default_rng(8)
    for K, P, dtype, mb in [(4, 1_000_003, 0, 16), (16, 3_000_001, 1, 7), (33, 999_999, 2, 5),
                            (64, 300_001, 0, 3), (8, 5_000_000, 0, 1)]:
        pcs = check_cover(K, P, dtype, None, mb)
        assert mb <= (pcs[:, 5] < 0).sum() <= 12 * mb            # halving: few pieces per span
        cuts = np.sort(rng.choice(np.arange(1, P), size=37, replace=False))
        pcs = check_cover(K, P, dtype, [0] + [int(c) for c in cuts] + [P], mb)
        assert (pcs[:, 5] < 0).sum() >= mb


def test_long_spans_are_cut_into_pieces_of_bounded_length():
    # a lane adds a piece's squares in fp32 before they reach the fp64 partial sums, and the kernel
    # addresses the aggregate of a piece with 32-bit byte offsets: 2^18 vectors at most
    P = (1 << 20) + 5
    pcs = check_cover(64, P, 0, None, 1)
    assert (pcs[:, 1] - pcs[:, 0]).max() == 1 << 18 and (pcs[:, 5] >= 0).sum() == 4
    assert len(pcs) < 40                                         # the tail: a piece per halving
    pcs = check_cover(64, P, 0, [0, 7, (1 << 19) + 9, P], 2)
    assert (pcs[:, 1] - pcs[:, 0]).max() <= 1 << 18
    pcs = check_cover(4, (1 << 22) + 77, 1, None, 1)             # 8 elements per vector
    assert (pcs[:, 1] - pcs[:, 0]).max() == 1 << 18


def test_plan_describe_rejects_bad_shapes():
    with pytest.raises(D.DynamixError):
        D.dynamix_plan_describe(0, 10, 0)
    with pytest.raises(D.DynamixError):
        D.dynamix_plan_describe(4, 10, 0, [0, 5, 9])


def test_cycle_entry_points_validate_on_the_host():
    assert D.dynamix_cycle_summary_count(4, 0) == 16 + 4 + 4
    assert D.dynamix_cycle_summary_count(32, 148) == 149 * 76 + 32
    assert D.dynamix_cycle_summary_count(0, 0) == -1 and D.dynamix_cycle_summary_count(4, -1) == -1
    lib = B.load()
    i32 = ctypes.c_int32
    b_ok, b_bad = (i32 * 2)(32, 64), (i32 * 2)(32, 0)
    assert lib.dynamix_cycle_accumulate(None, 16, ST, 1, None) == B.DYNAMIX_ERR_NULL
    assert lib.dynamix_cycle_accumulate(A16, 16, None, 1, None) == B.DYNAMIX_ERR_NULL
    assert lib.dynamix_cycle_accumulate(A16, 0, ST, 1, None) == B.DYNAMIX_ERR_ARG
    assert lib.dynamix_cycle_accumulate(A16 + 4, 16, ST, 1, None) == B.DYNAMIX_ERR_ALIGN
    assert lib.dynamix_cycle_summary(None, 2, 0, b_ok, 1.0, 1.0, ST, None) == B.DYNAMIX_ERR_NULL
    assert lib.dynamix_cycle_summary(A16, 2, 0, None, 1.0, 1.0, ST, None) == B.DYNAMIX_ERR_NULL
    assert lib.dynamix_cycle_summary(A16, 2, 0, b_ok, 1.0, 1.0, None, None) == B.DYNAMIX_ERR_NULL
    assert lib.dynamix_cycle_summary(A16, 0, 0, b_ok, 1.0, 1.0, ST, None) == B.DYNAMIX_ERR_ARG
    assert lib.dynamix_cycle_summary(A16, 2, 0, b_bad, 1.0, 1.0, ST, None) == B.DYNAMIX_ERR_ARG
    assert lib.dynamix_cycle_summary(A16, 2, -1, b_ok, 1.0, 1.0, ST, None) == B.DYNAMIX_ERR_SEGMENTS
    assert lib.dynamix_cycle_summary(A16, 2, 0, b_ok, 1.0, 1.0, ST + 4, None) == B.DYNAMIX_ERR_ALIGN


def test_fused_sgd_entry_validates_on_the_host():
    lib = B.load()
    ptrs = (ctypes.c_void_p * 2)(A16, A16 + 64)
    b = (ctypes.c_int32 * 2)(32, 64)

    def call(params, lr=0.1, wd=0.0, K=2, P=100, stats=ST):
        return lib.dynamix_grad_aggregate_stats_sgd(ptrs, b, K, P, 0, None, 0, params, lr, wd,
                                                    stats, None)
    assert call(None) == B.DYNAMIX_ERR_NULL
    assert call(A16 + 8) == B.DYNAMIX_ERR_ALIGN
    assert call(A16, lr=float("nan")) == B.DYNAMIX_ERR_ARG
    assert call(A16, wd=float("nan")) == B.DYNAMIX_ERR_ARG
    assert call(A16, K=0) == B.DYNAMIX_ERR_ARG
    assert call(A16, P=0) == B.DYNAMIX_ERR_ARG
    assert call(A16, stats=None) == B.DYNAMIX_ERR_NULL


def test_build_check_of_register_allocation():
    """The build refuses a streaming-pass instantiation that spills or that has values placed in
    accumulation registers other than its two banks (256 of them for K <= 44, none above)."""
    from paper_2510_08522_amd import build as Bd
    assert [Bd._bank_registers(K, d, U) for K, d, U in
            [(1, 0, 8), (8, 0, 4), (16, 1, 2), (32, 0, 1), (32, 2, 1), (33, 0, 1), (44, 1, 1), (45, 0, 1),
             (64, 1, 1)]] == [256, 256, 256, 256, 256, 256, 256, 0, 0]
    # the updates with state park two or three streams per tile
    assert [Bd._bank_registers(K, d, U, o) for K, d, U, o in
            [(24, 0, 1, 2), (24, 1, 1, 2), (2, 1, 4, 2), (8, 1, 2, 2), (8, 0, 2, 1), (32, 0, 1, 2),
             (32, 1, 1, 1)]] == [252, 240, 192, 240, 256, 252, 256]
    tag = "[-Rpass-analysis=kernel-resource-usage]"
    fn = "x.hip:1:1: remark: Function Name: _ZN7dynamix18stream_pass_kernelILi%dELi0ELi1ELi0EEEvNS_10StreamArgsE " + tag

    def remarks(K, agprs, scratch, spilled=0):
        return "\n".join([fn % K, "x.hip:1:1: remark:     VGPRs: 246 " + tag,
                          "x.hip:1:1: remark:     AGPRs: %d %s" % (agprs, tag),
                          "x.hip:1:1: remark:     ScratchSize [bytes/lane]: %d %s" % (scratch, tag),
                          "x.hip:1:1: remark:     VGPRs Spill: %d %s" % (spilled, tag)])
    assert Bd._check_resources(remarks(32, 256, 0), "x.hip") == []
    assert Bd._check_resources(remarks(50, 0, 0), "x.hip") == []
    for bad in (remarks(32, 152, 0), remarks(32, 256, 8, 1), remarks(50, 6, 0), remarks(8, 256, 0, 2)):
        with pytest.raises(RuntimeError):
            Bd._check_resources(bad, "x.hip")
    # a private segment that no vector register was spilled to is reported for a look at the code
    assert Bd._check_resources(remarks(32, 256, 36), "x.hip") == [(32, 0, 1, 0)]
    assert Bd._uses_scratch("\tv_add_f32 v1, v2, v3\n\tscratch_store_dword off, v249, off\n")
    assert not Bd._uses_scratch("\tbuffer_store_dwordx4 v[1:4], v5, s[8:11], 0 offen nt\n"
                                "\t.amdhsa_private_segment_fixed_size 36\n")
