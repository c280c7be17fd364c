"""The region arena (placement.py): pieces are disjoint, aligned, inside their region, and the
fused step gives the oracle's result on buffers carved from it."""
import numpy as np
import pytest
import torch

import paper_2102_08374_amd as P
import oracle as O
from paper_2102_08374_amd import workloads as W
from tests.gpu_util import assert_within_ulp, host, rel_err, u64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_arena_hands_out_disjoint_aligned_pieces_by_region():
    free, total = torch.cuda.mem_get_info(DEV)
    if free < (8 << 30):
        pytest.skip("needs 8 GiB of free device memory")
    arena = P.Arena(DEV, nbytes=2 << 30, guard=1 << 20)
    try:
        assert len(arena.extent) == P.HBM_REGIONS
        assert arena.free_in(1) == 0 and arena.free_in(2) == 0      # 2 GiB end inside region 0
        a = arena.take(1000, 0)
        b = arena.take(4096, 0)
        assert a.data_ptr() % 256 == 0 and b.data_ptr() % 256 == 0
        assert b.data_ptr() >= a.data_ptr() + 1000
        with pytest.raises(MemoryError):
            arena.take(8, 1)
        with pytest.raises(MemoryError):
            arena.take(4 << 30, 0)
        arena.reset()
        assert arena.take(16, 0).data_ptr() == a.data_ptr()
    finally:
        del arena
        torch.cuda.empty_cache()


def test_fused_step_on_arena_pieces_matches_the_oracle():
    free, _ = torch.cuda.mem_get_info(DEV)
    if free < (8 << 30):
        pytest.skip("needs 8 GiB of free device memory")
    w = W.config(1)
    arena = P.Arena(DEV, nbytes=1 << 30, guard=1 << 20)
    try:
        stride = W.row_stride(w.d)
        buf = arena.take(4 * w.n * stride, 0).view(torch.float32).view(w.n, stride)
        _, rows = W.make_gradients(w, 1, DEV, out=buf)
        x = W.make_params(w, DEV, out=arena.take(4 * w.d, 0).view(torch.float32))
        x0 = host(x).copy()
        desc = P.Desc(w.d, w.n, rounding=w.rounding, wire=w.wire, clip=w.clip, seed=w.philox_seed,
                      block_offsets=w.block_offsets)
        desc.step = 1
        ws = P.new_workspace(desc, DEV)
        alpha = torch.full((w.num_blocks,), 900.0, dtype=torch.float32, device=DEV)
        ns = torch.zeros(w.num_blocks, dtype=torch.float64, device=DEV)
        cnt = torch.zeros(w.n, dtype=torch.int64, device=DEV)
        P.intsgd_step_fused(desc, rows, alpha, w.eta, x, ns, cnt, ws)
        torch.cuda.synchronize()
        ref = O.step([host(r) for r in rows], host(alpha), x0, rounding=w.rounding,
                     L=w.clip, eta=w.eta, seed=w.philox_seed, step=1, offsets=w.block_offsets)
        assert_within_ulp(host(x), ref["x_new"], 1, "x")
        assert u64(cnt).tolist() == ref["sat_count"].tolist()
        assert rel_err(host(ns), ref["normsq"]) <= 1e-5
    finally:
        del arena, buf, rows, x
        torch.cuda.empty_cache()
