"""Seeded synthetic inputs for the group-synchronous parameter update.

This module only *draws* inputs: parameter / momentum / gradient buffers and
the stream of worker groups.  It contains none of the method's arithmetic and
is the one module the GPU path's tests, the CPU oracle's tests and the
benchmark all share.

What the inputs stand in for.  The paper trains ten CIFAR-10 / WikiText-2
models under a parameter-server architecture (Section 3, experiment settings);
the update path itself never looks at the data, only at W gradient buffers of
the shard's length and at which workers form the group of each update
(Section 1, items (2) and (4); Section 4.2).  The five workloads below are
shard-sized buffers with the stated Gaussian statistics and group-size mixes.
"N(0, s)" means standard deviation s.

Tensor draws use ``torch.Generator`` (CPU or CUDA; the two give different but
equally valid streams, and a consumer that needs the values on the host copies
them back).  Update streams use ``numpy.random.default_rng`` on the host.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    P: int                 # shard length (elements)
    W: int                 # workers
    grad_dtype: str        # "f32" | "bf16"
    grad_std: float
    param_std: float
    U: int                 # updates per call
    calls: int             # calls per step (state carried in params/momentum)
    group_rule: str        # see make_update_stream
    wmode: str             # "mean" | "stale"
    max_staleness: int
    lr: float
    momentum: float
    weight_decay: float
    norms: bool
    heavy_frac: float = 0.0   # fraction of workers whose whole row is scaled x10
    fresh_grads_per_call: bool = False

    def scaled(self, P: int, name: Optional[str] = None) -> "Workload":
        """Same structure at another shard length (for oracle-sized parity cases)."""
        return dataclasses.replace(self, P=int(P), name=name or f"{self.name}@P={P}")

    @property
    def grad_bytes(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2

    def algorithmic_bytes_per_call(self, w_used: Optional[int] = None) -> int:
        """Bytes the method must move per call: every referenced gradient row
        once, params and momentum read once and written once."""
        w = self.W if w_used is None else w_used
        return self.P * (w * self.grad_bytes + 16)


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny", 1_048_576, 4, "f32", 1e-2, 0.02, 10, 1, "fixed2", "mean", 0,
                 0.1, 0.9, 1e-4, False),
        Workload("resnet50", 25_557_032, 8, "f32", 1e-3, 0.02, 64, 1, "cycle248", "mean", 0,
                 0.1, 0.9, 5e-5, False),
        Workload("bert_base", 110_000_000, 16, "f32", 1e-3, 0.02, 64, 1, "uniform1toW", "stale", 4,
                 0.01, 0.9, 1e-4, True, heavy_frac=0.05),
        Workload("vgg16", 138_357_544, 32, "bf16", 1e-3, 0.02, 128, 1, "alt_full_4", "mean", 0,
                 0.01, 0.9, 0.0, False),
        Workload("bert_large", 340_000_000, 16, "bf16", 5e-4, 0.02, 64, 4, "uniform2toW", "stale", 8,
                 0.01, 0.9, 1e-4, True, fresh_grads_per_call=True),
    ]
}
ORDER = ["tiny", "resnet50", "bert_base", "vgg16", "bert_large"]


def _rng(seed: int, purpose: int, call: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(purpose), int(call)])


def make_update_stream(wl: Workload, seed: int = 0, call: int = 0) -> dict:
    """Draw the U worker groups of one call.

    Returns a dict with int32 ``offsets`` [U+1], int32 ``members`` and, for the
    staleness-weighted workloads, int32 ``staleness`` (same length as members,
    uniform in 0..max_staleness); ``staleness`` is None otherwise.  Members of a
    group are distinct and listed in the order drawn (not sorted).
    """
    rg = _rng(seed, 2, call)
    rs = _rng(seed, 3, call)
    rz = _rng(seed, 4, call)
    W, U = wl.W, wl.U
    sizes: List[int] = []
    for u in range(U):
        if wl.group_rule == "fixed2":
            y = 2
        elif wl.group_rule == "cycle248":
            y = (2, 4, 8)[u % 3]
        elif wl.group_rule == "uniform1toW":
            y = int(rz.integers(1, W + 1))
        elif wl.group_rule == "uniform2toW":
            y = int(rz.integers(2, W + 1))
        elif wl.group_rule == "alt_full_4":
            y = W if u % 2 == 0 else 4
        else:
            raise ValueError(wl.group_rule)
        sizes.append(min(y, W))
    offsets = np.zeros(U + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(sizes)
    members = np.empty(int(offsets[-1]), dtype=np.int32)
    for u, y in enumerate(sizes):
        members[offsets[u]:offsets[u + 1]] = rg.permutation(W)[:y]
    staleness = None
    if wl.wmode == "stale":
        staleness = rs.integers(0, wl.max_staleness + 1, size=members.shape[0]).astype(np.int32)
    return {"offsets": offsets, "members": members, "staleness": staleness}


def heavy_workers(wl: Workload, seed: int = 0) -> List[int]:
    """Workers whose gradient row is scaled x10 (heavy tail)."""
    if wl.heavy_frac <= 0:
        return []
    n = max(1, int(round(wl.heavy_frac * wl.W)))
    return sorted(int(x) for x in _rng(seed, 5).permutation(wl.W)[:n])


def _normal(n: int, std: float, seed_words, device, dtype=torch.float32, chunk: int = 1 << 26):
    g = torch.Generator(device=device)
    s = 0
    for wd in seed_words:                       # small injective-ish mix of the words
        s = (s * 1_000_003 + int(wd) + 12345) % (2 ** 62)
    g.manual_seed(s)
    out = torch.empty(n, dtype=dtype, device=device)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        x = torch.randn(hi - lo, generator=g, device=device, dtype=torch.float32)
        x.mul_(std)
        out[lo:hi] = x.to(dtype)               # bf16: round-to-nearest-even of the fp32 draw
    return out


def make_params(wl: Workload, seed: int = 0, device="cpu") -> torch.Tensor:
    return _normal(wl.P, wl.param_std, (seed, 1), device)


def make_momentum(wl: Workload, device="cpu") -> torch.Tensor:
    return torch.zeros(wl.P, dtype=torch.float32, device=device)


def make_grad_rows(wl: Workload, seed: int = 0, call: int = 0, device="cpu") -> List[torch.Tensor]:
    """W gradient rows of length P (fp32 or bf16), one tensor per worker."""
    dtype = torch.float32 if wl.grad_dtype == "f32" else torch.bfloat16
    heavy = set(heavy_workers(wl, seed))
    rows = []
    for w in range(wl.W):
        std = wl.grad_std * (10.0 if w in heavy else 1.0)
        rows.append(_normal(wl.P, std, (seed, 100 + 1000 * call + w), device, dtype))
    return rows


def rows_to_numpy(rows: List[torch.Tensor]) -> List[np.ndarray]:
    """Host copies in the oracle's input format: float32 arrays, or uint16 bit
    patterns for bf16 rows."""
    out = []
    for r in rows:
        if r.dtype == torch.bfloat16:
            out.append(r.detach().cpu().view(torch.int16).numpy().view(np.uint16).copy())
        else:
            out.append(r.detach().cpu().numpy().copy())
    return out
