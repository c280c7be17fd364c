"""Seeded synthetic inputs of the five benchmark workloads.

This module only produces DATA (gradients, parameters, block partitions, the
prior update norm that starts the alpha recurrence); it contains none of the
method's arithmetic.  Tests hand the same bits to the HIP library and to the
CPU oracle (device -> host copy), so no cross-device RNG agreement is needed.

The paper trains ResNet18/CIFAR-10 and an LSTM/Wikitext-2 (Section 5.1); those
datasets are not used here.  The workloads below are synthetic stand-ins with
the flat-vector sizes of a ResNet-50, a BERT-base and a 1.3 B-parameter model.
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional

import torch

ROUND_NEAREST_EVEN = 0
ROUND_STOCHASTIC = 1
_CHUNK = 1 << 26  # coordinates generated per pass (bounds temporaries)


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    d: int
    n: int
    rounding: int
    wire: int
    clip: int
    steps: int
    grad_kind: str                 # "normal" | "student_t3" | "mixture"
    sigma: float                   # scale of the gradient distribution
    eta: float = 0.1
    beta: float = 0.9
    eps: float = 1e-8
    philox_seed: int = 0
    block_offsets: Optional[List[int]] = None
    first_normsq: List[float] = field(default_factory=list)  # ||x^1 - x^0||^2 per block

    @property
    def num_blocks(self):
        return 1 if self.block_offsets is None else len(self.block_offsets) - 1

    def scaled(self, d, block_offsets=None):
        """Same recipe on a smaller vector (tests)."""
        var = self.grad_variance()
        if block_offsets is None:
            first = [self.first_normsq[0] * d / self.d] if self.config_id == 1 else \
                [self.eta ** 2 * d * var / self.n]
        else:
            first = [self.eta ** 2 * (b - a) * var / self.n
                     for a, b in zip(block_offsets[:-1], block_offsets[1:])]
        return replace(self, d=d, block_offsets=block_offsets, first_normsq=first,
                       name=self.name + "-scaled")

    def grad_variance(self):
        if self.grad_kind == "normal":
            return self.sigma ** 2
        if self.grad_kind == "student_t3":
            return 3.0 * self.sigma ** 2          # Var of t(3) is 3
        if self.grad_kind == "mixture":
            return 0.99 * (1e-4) ** 2 + 0.01 * (1e-2) ** 2
        raise ValueError(self.grad_kind)


def bert_base_block_sizes():
    """161 tensors with BERT-base layer shapes: 12 layers of {4 x 768x768, 768x3072,
    3072x768, 7 x 768}, then the 30522x768 embedding and 4 x 768 (108,443,136 coordinates)."""
    sizes = []
    for _ in range(12):
        sizes += [768 * 768] * 4 + [768 * 3072, 3072 * 768] + [768] * 7
    sizes += [30522 * 768] + [768] * 4
    assert len(sizes) == 161
    return sizes


def _offsets(sizes):
    off = [0]
    for s in sizes:
        off.append(off[-1] + s)
    return off


def _int32_clip(n):
    return (2 ** 31 - 1) // n


def config(config_id: int, per_bucket: bool = True, rounding: Optional[int] = None) -> Workload:
    """Workload `config_id`; `rounding` overrides the recipe's rounding mode (workload 4 does
    not name one: randomized is its default here, nearest-even the variant)."""
    w = _config(config_id, per_bucket)
    if rounding is not None and rounding != w.rounding:
        suffix = "-stochastic" if rounding == ROUND_STOCHASTIC else "-nearest-even"
        w = replace(w, rounding=rounding, name=w.name + suffix)
    return w


def _config(config_id: int, per_bucket: bool) -> Workload:
    eta = 0.1
    if config_id == 1:
        d, n = 1_048_576, 4
        return Workload("cfg1-oracle-sized", 1, d, n, ROUND_STOCHASTIC, 32, _int32_clip(n), 1,
                        "normal", 0.01, first_normsq=[1e-6])
    if config_id == 2:
        d, n = 25_557_032, 16
        return Workload("cfg2-resnet50-det-int32", 2, d, n, ROUND_NEAREST_EVEN, 32, _int32_clip(n),
                        100, "normal", 1e-3, first_normsq=[eta ** 2 * d * 1e-6 / n])
    if config_id == 3:
        d, n = 25_557_032, 8
        return Workload("cfg3-int8-student-t", 3, d, n, ROUND_STOCHASTIC, 8, 127, 20,
                        "student_t3", 1e-3, first_normsq=[eta ** 2 * d * 3e-6 / n])
    if config_id == 4:
        sizes = bert_base_block_sizes()
        off = _offsets(sizes)
        d, n = off[-1], 8
        if per_bucket:
            first = [eta ** 2 * s * 1e-6 / n for s in sizes]
            return Workload("cfg4-bert-base-per-bucket", 4, d, n, ROUND_STOCHASTIC, 32,
                            _int32_clip(n), 10, "normal", 1e-3, block_offsets=off,
                            first_normsq=first)
        return Workload("cfg4-bert-base-global", 4, d, n, ROUND_STOCHASTIC, 32, _int32_clip(n), 10,
                        "normal", 1e-3, first_normsq=[eta ** 2 * d * 1e-6 / n])
    if config_id == 5:
        d, n = 1_300_000_000, 8
        var = 0.99 * 1e-8 + 0.01 * 1e-4
        return Workload("cfg5-1.3B-mixture", 5, d, n, ROUND_STOCHASTIC, 32, _int32_clip(n), 5,
                        "mixture", 1e-3, first_normsq=[eta ** 2 * d * var / n])
    raise ValueError("config_id must be 1..5")


def _generator(w: Workload, step: int, worker: int, device):
    g = torch.Generator(device=device)
    g.manual_seed(((w.config_id * 1_000_003 + step) * 1_000_033 + worker) & (2 ** 63 - 1))
    return g


def make_params(w: Workload, device, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x^k ~ iid N(0, 1), fp32 (written into `out`, d floats, if given)."""
    x = out if out is not None else torch.empty(w.d, dtype=torch.float32, device=device)
    assert x.shape == (w.d,) and x.dtype == torch.float32
    g = _generator(w, 0, 1 << 20, device)
    for a in range(0, w.d, _CHUNK):
        x[a:a + _CHUNK].normal_(0.0, 1.0, generator=g)
    return x


def fill_gradient(w: Workload, step: int, worker: int, out: torch.Tensor):
    """Worker `worker`'s fp32 gradient of step `step`, written into `out` (d floats)."""
    g = _generator(w, step, worker, out.device)
    for a in range(0, w.d, _CHUNK):
        v = out[a:a + _CHUNK]
        if w.grad_kind == "normal":
            v.normal_(0.0, w.sigma, generator=g)
        elif w.grad_kind == "student_t3":
            # t(3) = Z / sqrt(chi2_3 / 3), chi2_3 = sum of three squared normals
            v.normal_(0.0, 1.0, generator=g)
            chi = torch.zeros_like(v)
            tmp = torch.empty_like(v)
            for _ in range(3):
                tmp.normal_(0.0, 1.0, generator=g)
                chi.addcmul_(tmp, tmp)
            v.div_(chi.div_(3.0).sqrt_()).mul_(w.sigma)
        elif w.grad_kind == "mixture":
            # 0.99 N(0, 1e-4^2) + 0.01 N(0, 1e-2^2)
            v.normal_(0.0, 1.0, generator=g)
            pick = torch.empty_like(v).uniform_(0.0, 1.0, generator=g)
            scale = torch.where(pick < 0.01, torch.full_like(v, 1e-2), torch.full_like(v, 1e-4))
            v.mul_(scale)
        else:
            raise ValueError(w.grad_kind)
    return out


def row_stride(d: int, skew_bytes: int = 0) -> int:
    """Floats between the starts of two workers' gradients in one buffer: d rounded up
    so that every row starts on a 256-byte boundary (each worker would own a separately
    allocated, aligned gradient buffer), plus an optional skew (a multiple of 256 bytes)."""
    assert skew_bytes % 256 == 0
    return (d + 63) // 64 * 64 + skew_bytes // 4


def make_gradients(w: Workload, step: int, device, out: Optional[torch.Tensor] = None,
                   skew_bytes: int = 0):
    """-> (buffer [n, row_stride(d)], list of the n row views of d floats)."""
    stride = row_stride(w.d, skew_bytes)
    buf = out if out is not None else torch.empty((w.n, stride), dtype=torch.float32, device=device)
    assert buf.shape == (w.n, stride)
    rows = [buf[i, :w.d] for i in range(w.n)]
    for i, row in enumerate(rows):
        fill_gradient(w, step, i, row)
    return buf, rows
