"""The entry point that allocates nothing (intsgd_step_fused_static) against the entry point
it is a variant of (intsgd_step_fused_next_alpha), through the C ABI: same x, norm, counts,
r and next alpha, on consecutive calls that share the library's static scratch array."""
import numpy as np
import pytest
import torch

import paper_2102_08374_amd as P
from tests.gpu_util import F32, host, rel_err, sprinkle_adversarial, u64

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _inputs(d, n, B, seed):
    rng = np.random.default_rng(seed)
    alpha = rng.uniform(50.0, 2000.0, B).astype(F32)
    g = rng.normal(0.0, 0.01, (n, d)).astype(F32)
    g = sprinkle_adversarial(rng, g, float(alpha[0]))          # ties, clip edges, NaN, Inf
    x = rng.normal(0.0, 1.0, d).astype(F32)
    r = rng.uniform(1e-6, 1e-3, B)
    return alpha, g, x, r


def _run(entry, desc, alpha, g_rows, x, r, eta, eta_next, ws):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    d_a, d_x, d_r = t(alpha), t(x), t(r)
    d_ns = torch.full((desc.num_blocks,), -1.0, dtype=torch.float64, device=DEV)
    d_cnt = torch.full((desc.n,), -1, dtype=torch.int64, device=DEV)
    if entry == "static":
        P.intsgd_step_fused_static(desc, g_rows, d_a, eta, d_x, d_r, 0.9, 1e-8, d_ns, d_cnt,
                                   eta_next=eta_next)
    else:
        P.intsgd_step_fused_next_alpha(desc, g_rows, d_a, eta, d_x, d_r, 0.9, 1e-8, d_ns, d_cnt, ws,
                                       eta_next=eta_next)
    torch.cuda.synchronize()
    return host(d_x), host(d_ns), u64(d_cnt), host(d_r), host(d_a)


def _compare(desc, seed, eta=0.1, eta_next=0.07):
    B = desc.num_blocks
    alpha, g, x, r = _inputs(desc.d, desc.n, B, seed)
    rows = [torch.from_numpy(g[i]).to(DEV) for i in range(desc.n)]
    ws = P.new_workspace(desc, DEV)
    want = _run("workspace", desc, alpha, rows, x, r, eta, eta_next, ws)
    got = _run("static", desc, alpha, rows, x, r, eta, eta_next, None)
    assert np.array_equal(got[0].view(np.uint32), want[0].view(np.uint32)), "x"     # <= 1 ulp bar: equal bits
    assert rel_err(got[1], want[1]) <= 1e-5 and np.array_equal(got[1], want[1]), "norm"
    assert got[2].tolist() == want[2].tolist(), "clip counts"
    assert want[2].sum() > 0, "the adversarial values must clip"
    assert np.array_equal(got[3], want[3]), "r"
    assert np.array_equal(got[4].view(np.uint32), want[4].view(np.uint32)), "next alpha"


@pytest.mark.parametrize("rounding", [P.ROUND_STOCHASTIC, P.ROUND_NEAREST_EVEN])
def test_static_scratch_step_equals_workspace_step_on_consecutive_calls(rounding):
    """Two calls in a row, the second on a smaller input (which finds the first call's flags,
    partials and count rows in the array), then a larger one again."""
    for k, (d, n) in enumerate([(300_007, 9), (41_003, 5), (1 << 22 | 4, 16)]):
        desc = P.Desc(d, n, rounding=rounding, clip=1000, seed=11, step=k + 1)
        P.intsgd_prepare(desc)
        _compare(desc, seed=100 * rounding + k)


def test_static_scratch_step_with_blocks_needs_a_prepared_partition():
    offsets = [0, 5, 1030, 1031, 40000, 70001]
    desc = P.Desc(70001, 6, rounding=P.ROUND_STOCHASTIC, clip=127, seed=3, step=2, block_offsets=offsets,
                  opts=P.LaunchOpts(tile_coords=3072))        # a tiling no other call has prepared
    alpha, g, x, r = _inputs(desc.d, desc.n, desc.num_blocks, 5)
    rows = [torch.from_numpy(g[i]).to(DEV) for i in range(desc.n)]
    with pytest.raises(P.IntSGDError) as err:
        _run("static", desc, alpha, rows, x, r, 0.1, 0.1, None)
    assert err.value.status == -6                              # INTSGD_ENOPLAN: it must not build one
    P.intsgd_prepare(desc)
    _compare(desc, seed=5)
    _compare(P.Desc(8191, 3, rounding=P.ROUND_NEAREST_EVEN, clip=50, seed=3, step=3), seed=6)   # smaller again


def test_static_scratch_step_refuses_what_does_not_fit():
    """(12 + 8 n) bytes per tile: 2^26 coordinates in tiles of 1024 at n = 128 need 65 MiB."""
    n = 128
    big = P.Desc(1 << 26, n, rounding=P.ROUND_STOCHASTIC, clip=1000, opts=P.LaunchOpts(tile_coords=1024))
    assert (12 + 8 * n) * ((1 << 26) // 1024) > P.STATIC_SCRATCH_BYTES
    tiny = torch.zeros(4, dtype=torch.float32, device=DEV)     # never touched: refused before any launch
    b = P.binding
    status = b._lib.intsgd_step_fused_static(big.ref(), b._ptr_array([tiny] * n), b._ptr(tiny), 0.1, 0.1,
                                             b._ptr(tiny), b._ptr(tiny), 0.9, 1e-8, b._ptr(tiny),
                                             b._ptr(tiny), None)
    assert status == -5                                        # INTSGD_EWORKSPACE
    torch.cuda.synchronize()
