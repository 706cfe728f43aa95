"""The plain streaming kernels used to measure the memory system (needs an MI355X): they must
touch what they claim to touch, or the ceilings they give would mean nothing."""
import pytest
import torch

import paper_2510_08522_amd as D
from paper_2510_08522_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_probe_copy_copies_and_write_writes():
    n = 3 * (1 << 20) + 4096                       # bytes; whole tiles of the copy kernel
    src = torch.randn(n // 4, device=DEV)
    dst = torch.zeros(n // 4, device=DEV)
    print("case probe copy", flush=True)
    B.dynamix_hbm_probe([src, dst], n // 32768 * 32768, B.DYNAMIX_PROBE_COPY, 7)
    torch.cuda.synchronize()
    m = n // 32768 * 32768 // 4
    assert torch.equal(dst[:m], src[:m]) and not dst[m:].any()
    print("case probe write", flush=True)
    B.dynamix_hbm_probe([dst], n, B.DYNAMIX_PROBE_WRITE, 5)
    torch.cuda.synchronize()
    words = dst.view(torch.int32)
    assert (words[2::4] == 2).all() and (words[3::4] == 3).all()
    assert torch.equal(words[1::4], torch.arange(n // 4096, device=DEV, dtype=torch.int32)
                       .repeat_interleave(256))
    print("case probe read", flush=True)
    before = src.clone()
    for mode in (B.DYNAMIX_PROBE_READ, B.DYNAMIX_PROBE_READ_SPREAD, B.DYNAMIX_PROBE_READ_SPREAD_128B,
                 B.DYNAMIX_PROBE_READ_SPREAD_512B):
        for k in (1, 2, 4, 8, 16, 32):
            B.dynamix_hbm_probe([src] * k, n, mode, 3)
    torch.cuda.synchronize()
    assert torch.equal(src, before)


def test_probe_argument_checks():
    t = torch.zeros(4096, device=DEV)
    for bad in (lambda: B.dynamix_hbm_probe([t] * 3, 4096, B.DYNAMIX_PROBE_READ, 1),
                lambda: B.dynamix_hbm_probe([t], 4096, B.DYNAMIX_PROBE_COPY, 1),
                lambda: B.dynamix_hbm_probe([t[1:]], 4096, B.DYNAMIX_PROBE_WRITE, 1),
                lambda: B.dynamix_hbm_probe([t], 4096, 9, 1),
                lambda: B.dynamix_hbm_probe([t], 4096, B.DYNAMIX_PROBE_WRITE, 0)):
        with pytest.raises(D.DynamixError):
            bad()
