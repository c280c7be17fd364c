"""The largest integer in the aggregate (Appendix A.2 reports it per iteration): every call whose
sweep forms S writes max |S_j| per block into the descriptor's optional output, bit-exact
against the oracle's value on the oracle's aggregate."""
import numpy as np
import pytest
import torch

import oracle
import paper_2102_08374_amd as P
from tests.gpu_util import F32, host, sprinkle_adversarial

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [
    # d, n, block offsets (None = one block), tile
    (10007, 3, None, 1024),
    (70001, 9, [0, 5, 1030, 1031, 40000, 70001], 1024),
    (20480, 16, [0, 768, 8192, 20480], 4096),
    (2, 1, None, 1024),
    (5003, 128, None, 2048),
    (4099, 127, [0, 1, 2050, 4099], 1024),
]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def case(d, n, offsets, seed, adversarial=True):
    rng = np.random.default_rng(seed)
    B = 1 if offsets is None else len(offsets) - 1
    alpha = rng.uniform(50.0, 2000.0, B).astype(F32)
    g = rng.normal(0.0, 0.01, (n, d)).astype(F32)
    if adversarial:
        g = sprinkle_adversarial(rng, g, float(alpha[0]))
    x = rng.normal(0.0, 1.0, d).astype(F32)
    return alpha, g, x


def sentinel(B):
    return torch.full((B,), -12345, dtype=torch.int32, device=DEV)


def u32(t):
    return host(t).view(np.uint32).tolist()


@pytest.mark.parametrize("rounding", [P.ROUND_NEAREST_EVEN, P.ROUND_STOCHASTIC])
@pytest.mark.parametrize("clip", [None, 15])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "d%d-n%d" % (s[0], s[1]))
def test_every_sweep_that_forms_the_aggregate_reports_its_largest_entry(shape, clip, rounding):
    d, n, offsets, tile = shape
    L = P.default_clip(n) if clip is None else clip
    seed, step, eta = 77, 5, 0.1
    alpha, g, x = case(d, n, offsets, seed=d + n + rounding)
    B = alpha.size
    off_np = None if offsets is None else np.array(offsets, np.uint64)
    kw = dict(rounding=rounding, L=L, seed=seed, step=step, offsets=off_np)
    out = oracle.step(list(g), alpha, x, eta=eta, **kw)
    want = oracle.max_abs_sum(out["S"], offsets=off_np, B=B).tolist()
    assert max(want) <= n * L

    desc = P.Desc(d, n, rounding=rounding, clip=L, seed=seed, step=step, block_offsets=offsets,
                  opts=P.LaunchOpts(tile_coords=tile))
    ws = P.new_workspace(desc, DEV)
    d_g = [dev(g[i]) for i in range(n)]
    d_alpha = dev(alpha)
    cnt = torch.zeros(n, dtype=torch.int64, device=DEV)
    ns = torch.zeros(B, dtype=torch.float64, device=DEV)

    # F1
    big = sentinel(B)
    desc.largest_sum = big
    S = torch.zeros(d, dtype=torch.int32, device=DEV)
    P.intsgd_compress_sum(desc, d_g, d_alpha, S, cnt, ws)
    assert np.array_equal(host(S), out["S"])
    assert u32(big) == want
    # the calls that are handed S instead of forming it leave the output alone
    big.fill_(-12345)
    P.intsgd_decode_update_norm(desc, S, d_alpha, eta, dev(x), ns, ws)
    P.intsgd_update_norm(desc, dev(x), dev(x), ns, ws)
    assert host(big).tolist() == [-12345] * B
    # F3
    P.intsgd_step_fused(desc, d_g, d_alpha, eta, dev(x), ns, cnt, ws)
    assert u32(big) == want
    # F3 + a8 in one call, workspace form and static-scratch form
    for static in (False, True):
        big.fill_(-12345)
        r = torch.zeros(B, dtype=torch.float64, device=DEV)
        a_io = d_alpha.clone()
        if static:
            P.intsgd_prepare(desc)
            P.intsgd_step_fused_static(desc, d_g, a_io, eta, dev(x), r, 0.9, 1e-8, ns, cnt)
        else:
            P.intsgd_step_fused_next_alpha(desc, d_g, a_io, eta, dev(x), r, 0.9, 1e-8, ns, cnt, ws)
        assert u32(big) == want
    # momentum form (the aggregate is the same)
    big.fill_(-12345)
    m = torch.zeros(d, dtype=torch.float32, device=DEV)
    P.intsgd_step_momentum(desc, d_g, d_alpha, eta, 0.9, 1e-4, dev(x), m, None, 0.9, 1e-8, ns, cnt, ws)
    assert u32(big) == want
    # without the output nothing is written anywhere near it
    desc.largest_sum = None
    big.fill_(-12345)
    P.intsgd_step_fused(desc, d_g, d_alpha, eta, dev(x), ns, cnt, ws)
    assert host(big).tolist() == [-12345] * B


@pytest.mark.parametrize("rounding", [P.ROUND_NEAREST_EVEN, P.ROUND_STOCHASTIC])
@pytest.mark.parametrize("shape", SHAPES[:3] + SHAPES[5:], ids=lambda s: "d%d-n%d" % (s[0], s[1]))
def test_diana_step_reports_the_largest_aggregated_difference(shape, rounding):
    d, n, offsets, tile = shape
    L = P.default_clip(n)
    alpha, g, x = case(d, n, offsets, seed=d + 3 * n + rounding)
    B = alpha.size
    rng = np.random.default_rng(d)
    hl = rng.normal(0.0, 0.01, (n, d)).astype(F32)
    h = hl.astype(np.float64).mean(axis=0).astype(F32)
    off_np = None if offsets is None else np.array(offsets, np.uint64)
    out = oracle.diana_step(list(g), list(hl), alpha, x, h, rounding=rounding, L=L, eta=0.1, seed=9,
                            step=2, offsets=off_np)
    want = oracle.max_abs_sum(out["S"], offsets=off_np, B=B).tolist()
    desc = P.Desc(d, n, rounding=rounding, clip=L, seed=9, step=2, block_offsets=offsets,
                  opts=P.LaunchOpts(tile_coords=tile))
    ws = P.new_workspace(desc, DEV)
    big = sentinel(B)
    desc.largest_sum = big
    cnt = torch.zeros(n, dtype=torch.int64, device=DEV)
    ns = torch.zeros(B, dtype=torch.float64, device=DEV)
    P.intsgd_diana_step(desc, [dev(g[i]) for i in range(n)], [dev(hl[i]) for i in range(n)], dev(alpha),
                        0.1, dev(x), dev(h), None, 0.0, 0.0, ns, cnt, ws)
    assert u32(big) == want


@pytest.mark.parametrize("rounding", [P.ROUND_NEAREST_EVEN, P.ROUND_STOCHASTIC])
@pytest.mark.parametrize("n", [2, 9])
def test_two_phase_forms_report_the_same_largest_entry(n, rounding):
    """d just past 2^22 with a ragged end: the persistent two-phase sweeps (F3, F3 with momentum,
    F1) against the oracle and against the tile sweeps; the extreme value sits in the last
    coordinates, which the d mod 4 tail of the two-phase form handles."""
    d = (1 << 22) + 1027
    L = P.default_clip(n)
    alpha, g, x = case(d, n, None, seed=n + rounding, adversarial=False)
    g[:, d - 2] = F32(3.0)                    # far above everything else, in the scalar tail
    g[0, 12345] = F32(-2.5)
    out = oracle.step(list(g), alpha, x, rounding=rounding, L=L, eta=0.1, seed=4, step=8)
    want = oracle.max_abs_sum(out["S"]).tolist()
    d_g = [dev(g[i]) for i in range(n)]
    cnt = torch.zeros(n, dtype=torch.int64, device=DEV)
    ns = torch.zeros(1, dtype=torch.float64, device=DEV)
    for form in (1, 2):
        desc = P.Desc(d, n, rounding=rounding, clip=L, seed=4, step=8, opts=P.LaunchOpts(two_phase=form))
        assert P.intsgd_fused_step_form(desc) == form
        ws = P.new_workspace(desc, DEV)
        big = sentinel(1)
        desc.largest_sum = big
        P.intsgd_step_fused(desc, d_g, dev(alpha), 0.1, dev(x), ns, cnt, ws)
        assert u32(big) == want, form
        big.fill_(-12345)
        S = torch.zeros(d, dtype=torch.int32, device=DEV)
        P.intsgd_compress_sum(desc, d_g, dev(alpha), S, cnt, ws)
        assert u32(big) == want, form
        big.fill_(-12345)
        m = torch.zeros(d, dtype=torch.float32, device=DEV)
        P.intsgd_step_momentum(desc, d_g, dev(alpha), 0.1, 0.9, 1e-4, dev(x), m, None, 0.9, 1e-8, ns, cnt, ws)
        assert u32(big) == want, form


def test_two_level_final_reduction_over_a_long_tile_list():
    """More than 16 K tiles in one block: the final maximum goes through the chunk level.  The
    extreme is planted in the last chunk, a runner-up in the first."""
    d, n = 1024 * 20000 + 77, 1
    rng = np.random.default_rng(5)
    g = rng.normal(0.0, 0.01, (n, d)).astype(F32)
    g[0, 1000] = F32(1.5)
    g[0, d - 50] = F32(-2.0)
    alpha = np.array([100.0], F32)
    x = np.zeros(d, F32)
    out = oracle.step(list(g), alpha, x, rounding=0, L=10**6, eta=0.1)
    want = oracle.max_abs_sum(out["S"]).tolist()
    assert want == [200]
    desc = P.Desc(d, n, rounding=0, clip=10**6, opts=P.LaunchOpts(tile_coords=1024, two_phase=1))
    ws = P.new_workspace(desc, DEV)
    big = sentinel(1)
    desc.largest_sum = big
    cnt = torch.zeros(n, dtype=torch.int64, device=DEV)
    ns = torch.zeros(1, dtype=torch.float64, device=DEV)
    P.intsgd_step_fused(desc, [dev(g[0])], dev(alpha), 0.1, dev(x), ns, cnt, ws)
    assert u32(big) == want


def test_everything_clips_to_the_bound():
    """alpha = +Inf: every finite non-zero coordinate clips to +-L, so the largest entry is n L
    wherever all workers agree in sign (planted), and the count says so."""
    d, n, L = 9001, 4, 127
    rng = np.random.default_rng(8)
    g = rng.normal(0.0, 1.0, (n, d)).astype(F32)
    g[:, 4242] = np.abs(g[:, 4242]) + F32(0.5)
    alpha = np.array([np.inf], F32)
    out = oracle.step(list(g), alpha, np.zeros(d, F32), rounding=1, L=L, eta=0.1, seed=1, step=1)
    want = oracle.max_abs_sum(out["S"]).tolist()
    assert want == [n * L]
    desc = P.Desc(d, n, rounding=1, wire=P.WIRE_INT8, clip=L, seed=1, step=1)
    ws = P.new_workspace(desc, DEV)
    big = sentinel(1)
    desc.largest_sum = big
    cnt = torch.zeros(n, dtype=torch.int64, device=DEV)
    ns = torch.zeros(1, dtype=torch.float64, device=DEV)
    P.intsgd_step_fused(desc, [dev(g[i]) for i in range(n)], dev(alpha), 0.1,
                        torch.zeros(d, dtype=torch.float32, device=DEV), ns, cnt, ws)
    assert u32(big) == want


def test_graph_replay_of_the_static_scratch_step_with_the_largest_entry():
    """The entry point for callers that cannot allocate, captured in a HIP graph with the
    largest-entry output attached, replayed with fresh gradients (randomized rounding, blocks):
    every replay equals the eager workspace form, the step counter being part of the capture."""
    d, n, offsets = 600_011, 5, [0, 100_003, 100_004, 600_011]
    B = len(offsets) - 1
    rng = np.random.default_rng(77)
    desc_g = P.Desc(d, n, rounding=P.ROUND_STOCHASTIC, clip=P.default_clip(n), seed=3, step=7,
                    block_offsets=offsets)
    desc_e = P.Desc(d, n, rounding=P.ROUND_STOCHASTIC, clip=P.default_clip(n), seed=3, step=7,
                    block_offsets=offsets)
    P.intsgd_prepare(desc_g)
    ws = P.new_workspace(desc_e, DEV)
    big_g, big_e = sentinel(B), sentinel(B)
    desc_g.largest_sum, desc_e.largest_sum = big_g, big_e
    rows = [torch.zeros(d, dtype=torch.float32, device=DEV) for _ in range(n)]
    x_g = torch.zeros(d, dtype=torch.float32, device=DEV)
    a_g = torch.full((B,), 500.0, dtype=torch.float32, device=DEV)
    r_g = torch.zeros(B, dtype=torch.float64, device=DEV)
    ns_g = torch.zeros(B, dtype=torch.float64, device=DEV)
    cnt_g = torch.zeros(n, dtype=torch.int64, device=DEV)
    x_e, a_e, r_e, ns_e, cnt_e = x_g.clone(), a_g.clone(), r_g.clone(), ns_g.clone(), cnt_g.clone()

    def call_static():
        P.intsgd_step_fused_static(desc_g, rows, a_g, 0.1, x_g, r_g, 0.9, 1e-8, ns_g, cnt_g)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call_static()                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    x_g.zero_()
    a_g.fill_(500.0)
    r_g.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call_static()
    for k in range(3):
        fresh = rng.normal(0.0, 0.01, (n, d)).astype(F32)
        for i in range(n):
            rows[i].copy_(torch.from_numpy(fresh[i]))      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        P.intsgd_step_fused_next_alpha(desc_e, rows, a_e, 0.1, x_e, r_e, 0.9, 1e-8, ns_e, cnt_e, ws)
        torch.cuda.synchronize()
        assert torch.equal(x_g, x_e), "replay %d" % k
        assert torch.equal(a_g, a_e) and torch.equal(r_g, r_e) and torch.equal(ns_g, ns_e)
        assert torch.equal(cnt_g, cnt_e)
        assert torch.equal(big_g, big_e) and host(big_g).min() > 0
