"""Helpers shared by the GPU parity tests: bit/ulp comparison and adversarial inputs."""
import numpy as np
import torch

F32 = np.float32

# Values that exercise every branch of the rounding / clip contract.
ADVERSARIAL = np.array(
    [0.0, -0.0, 1e-45, -1e-45, 1e-39, 0.5, -0.5, 1.5, 2.5, -2.5, 126.5, 127.49, 127.5, -127.5, 128.0,
     1e9, -1e9, 16777216.0, 16777217.0, -16777216.0, 2147483648.0, -2147483648.0, 2147483520.0, 4e9,
     -4e9, np.inf, -np.inf, np.nan, 0.99999994, -0.99999994, 3.4e38, -3.4e38], dtype=F32)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def u64(t: torch.Tensor) -> np.ndarray:
    """Device int64 tensor holding uint64 bits -> numpy uint64."""
    return host(t).view(np.uint64)


def ordered(a: np.ndarray) -> np.ndarray:
    """fp32 bit patterns mapped to integers that are monotone in the float value."""
    i = np.ascontiguousarray(a, dtype=F32).view(np.int32).astype(np.int64)
    return np.where(i < 0, -(i & 0x7FFFFFFF), i)


def ulp_diff(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in fp32 ulps; NaN vs NaN counts as 0, NaN vs number as a huge value."""
    a = np.ascontiguousarray(a, dtype=F32)
    b = np.ascontiguousarray(b, dtype=F32)
    dist = np.abs(ordered(a) - ordered(b))
    an, bn = np.isnan(a), np.isnan(b)
    dist = np.where(an & bn, 0, dist)
    dist = np.where(an ^ bn, 1 << 40, dist)
    return dist


def assert_within_ulp(got, want, max_ulp=1, what="value"):
    dist = ulp_diff(got, want)
    worst = int(dist.max()) if dist.size else 0
    assert worst <= max_ulp, "%s: worst distance %d ulp at index %d (got %r want %r)" % (
        what, worst, int(dist.argmax()), got[int(dist.argmax())], want[int(dist.argmax())])
    return int((dist != 0).sum())


def rel_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.maximum(np.abs(want), 1e-300)
    return float(np.max(np.abs(got - want) / den)) if got.size else 0.0


def sprinkle_adversarial(rng, g: np.ndarray, alpha: float, frac=0.02) -> np.ndarray:
    """Overwrites a fraction of g with values whose SCALED image alpha*g hits the
    adversarial list (so that ties, clip edges and non-finite inputs really occur)."""
    g = g.copy()
    flat = g.reshape(-1)
    k = max(1, int(frac * flat.size))
    idx = rng.choice(flat.size, k, replace=False)
    vals = rng.choice(ADVERSARIAL, k)
    with np.errstate(all="ignore"):
        flat[idx] = (vals.astype(np.float64) / float(alpha)).astype(F32)
    # and some raw ones (tiny / huge regardless of alpha)
    idx2 = rng.choice(flat.size, k, replace=False)
    flat[idx2] = rng.choice(ADVERSARIAL, k)
    return g
