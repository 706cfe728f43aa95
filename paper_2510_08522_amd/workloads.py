"""Seeded synthetic gradients shaped like the paper's workloads.

The paper trains VGG and ResNet models on CIFAR with 8 to 32 workers whose batch sizes move in
[32, 1024] (Evaluation, "Scalability"; Problem Formulation, "Action space and batch size
adjustment").  Neither the data sets nor real gradients are needed here: only the sizes and the
batch-size ranges matter.  Each worker k draws

    g_k = mu + eps_k,   mu ~ N(0, m^2) shared by all workers,
                        eps_k ~ N(0, sigma^2 / b_k) independent per element,

i.e. a mean over b_k examples whose per-example gradient has mean mu and covariance
sigma^2 I, cast to the storage dtype last.  With contiguous segments, sigma may differ per
segment.

This module only produces inputs (and the generator's own parameters, such as the realised
|mu|^2, which tests use for closed-form checks).  It holds none of the aggregation or statistics
arithmetic and serves both the HIP path and the CPU oracle's tests, so that both sides see
bit-identical data.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

BASE_SEED = 20251008


@dataclass
class Workload:
    name: str
    K: int
    P: int
    dtype: torch.dtype
    batch_sizes: np.ndarray               # int32[K]
    grads: List[torch.Tensor]             # K separate 1-d tensors of P elements
    segment_offsets: Optional[np.ndarray]  # int64[S+1] or None
    m: float                              # std of the shared mean
    sigma: np.ndarray                     # per-segment (or [1]) per-example std
    mu_sqnorm: np.ndarray                 # realised |mu|^2: [0] global, [1..S] per segment
    seed: int = 0
    extra: dict = field(default_factory=dict)

    @property
    def S(self):
        return 0 if self.segment_offsets is None else len(self.segment_offsets) - 1

    @property
    def itemsize(self):
        return 4 if self.dtype == torch.float32 else 2

    @property
    def bytes_read(self):
        return self.K * self.P * self.itemsize

    def host_arrays(self, lo=0, hi=None):
        """The K inputs (or the slice [lo, hi) of each) as numpy arrays the oracle accepts:
        float32, float16, or uint16 holding the bf16 bit patterns."""
        out = []
        for g in self.grads:
            t = g[lo:hi].detach().cpu().contiguous()
            if t.dtype == torch.bfloat16:
                out.append(t.view(torch.int16).numpy().view(np.uint16))
            else:
                out.append(t.numpy())
        return out


def _segment_sizes(rng, P, S, lo, hi):
    """S sizes, log-uniform in [lo, hi], scaled to sum to P (floor, remainder to the largest,
    every size at least 1)."""
    raw = np.exp(rng.uniform(np.log(lo), np.log(hi), size=S))
    sizes = np.maximum(1, np.floor(raw * (P / raw.sum())).astype(np.int64))
    sizes[np.argmax(sizes)] += P - sizes.sum()
    assert sizes.sum() == P and sizes.min() >= 1
    return sizes


def make(K, P, dtype, batch_sizes, m, sigma, seed, device="cpu", segment_offsets=None,
         name="custom", one_allocation=True, stagger_elems=0):
    """Draw one workload.  sigma is a scalar, or one value per segment.

    The K buffers are independent as far as the aggregation entry point is concerned (it takes
    K pointers).  With one_allocation they are rows of a single allocation made before anything
    else (rows padded to a multiple of 16 bytes, so most rows start off the 256-byte boundaries
    the kernel's interleaved tile order needs), otherwise K allocations made one by one (which
    torch places on 512-byte boundaries)."""
    dev = torch.device(device)
    store = None
    if one_allocation:
        row = (P + 7) // 8 * 8
        store = torch.empty((K, row), dtype=dtype, device=dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(seed))
    b = np.asarray(batch_sizes, dtype=np.int32)
    assert b.shape == (K,) and (b > 0).all()
    sig = np.atleast_1d(np.asarray(sigma, dtype=np.float64))
    off = None
    if segment_offsets is not None:
        off = np.asarray(segment_offsets, dtype=np.int64)
        assert off[0] == 0 and off[-1] == P and (np.diff(off) > 0).all()
    mu = torch.randn(P, generator=gen, device=dev, dtype=torch.float32) * float(m)
    if sig.size > 1:
        assert off is not None and sig.size == len(off) - 1
        sizes = torch.from_numpy(np.diff(off)).to(dev)
        sig_el = torch.repeat_interleave(
            torch.from_numpy(sig.astype(np.float32)).to(dev), sizes)
    else:
        sig_el = None
    grads = []
    for k in range(K):
        eps = torch.randn(P, generator=gen, device=dev, dtype=torch.float32)
        if sig_el is None:
            eps.mul_(float(sig[0] / np.sqrt(float(b[k]))))
        else:
            eps.mul_(sig_el).mul_(float(1.0 / np.sqrt(float(b[k]))))
        eps.add_(mu)
        if store is None and stagger_elems:
            # buffer k starts k * stagger_elems elements into an allocation of its own
            own = torch.empty(P + K * stagger_elems, dtype=dtype, device=dev)
            own[k * stagger_elems:k * stagger_elems + P].copy_(eps)
            grads.append(own[k * stagger_elems:k * stagger_elems + P])
        elif store is None:
            grads.append(eps.to(dtype).contiguous())
        else:
            store[k, :P].copy_(eps)           # same rounding as .to(dtype)
            grads.append(store[k, :P])
        del eps
    mu64 = mu.double()
    musq = [float((mu64 * mu64).sum().item())]
    if off is not None:
        for j in range(len(off) - 1):
            s = mu64[int(off[j]):int(off[j + 1])]
            musq.append(float((s * s).sum().item()))
    del mu, mu64, sig_el
    return Workload(name=name, K=K, P=P, dtype=dtype, batch_sizes=b, grads=grads,
                    segment_offsets=off, m=float(m), sigma=sig, mu_sqnorm=np.asarray(musq),
                    seed=int(seed), extra={"one_allocation": bool(one_allocation)})


#: (K, P, dtype, segments) of the five named configurations
SHAPES = {
    "C1": (4, 1_000_000, torch.float32, 0),
    "C2": (8, 11_700_000, torch.float32, 0),       # ResNet-18-sized
    "C3": (16, 25_600_000, torch.bfloat16, 0),     # ResNet-50-sized
    "C4": (32, 138_000_000, torch.float32, 0),     # VGG-16-sized, 32-node scale
    "C5": (8, 124_000_000, torch.float32, 148),    # 148 layer segments
}


def config(name, device="cpu", P=None, one_allocation=True, stagger_elems=0):
    """One of the named configurations C1..C5.  P overrides the length (the batch sizes, the
    generator parameters and the segment structure stay those of the configuration), so that
    CPU tests can use the same recipe at a size the oracle finishes quickly."""
    K, P0, dtype, S = SHAPES[name]
    P = int(P0 if P is None else P)
    c = int(name[1])
    seed = BASE_SEED + c
    rng = np.random.default_rng(seed)
    m, sigma, off = 1e-3, 1e-2, None
    if name == "C1":
        b = [32, 64, 96, 128]
    elif name in ("C2", "C5"):
        b = rng.integers(1, 17, size=K) * 16                 # {16, 32, ..., 256}
    elif name == "C3":
        b = np.rint(np.exp(rng.uniform(np.log(8.0), np.log(512.0), size=K)))
        sigma = 5e-3
        m = sigma / np.sqrt(2000.0)                          # expected noise scale 2000
    elif name == "C4":
        b = rng.integers(16, 257, size=K)                    # integers in [16, 256]
    if name == "C5":
        scale = P / P0
        sizes = _segment_sizes(rng, P, S, max(1.0, 1e3 * scale), max(2.0, 4e7 * scale))
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        sigma = np.exp(rng.uniform(np.log(1e-4), np.log(1e-1), size=S))
    w = make(K, P, dtype, np.asarray(b, dtype=np.int32), m, sigma, seed, device=device,
             segment_offsets=off, name=name, one_allocation=one_allocation,
             stagger_elems=stagger_elems)
    return w
