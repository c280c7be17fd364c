"""Where in HBM the buffers of a step live (harness-side helper; no arithmetic of the method).

Measured on MI355X (288 GiB of HBM3E): device memory behaves as three regions of 96 GiB, most
likely the three ranks of the 12-high stacks, which share channels but own their banks.  A
sweep that reads its n gradient streams from one region and reads-modifies-writes x in ANOTHER
runs at 80-85 % of the HBM peak; with x in the SAME region as the gradients it runs at 73-80 %
(writes and reads then fight over the same banks: row conflicts and write-to-read turnarounds).
Offsets inside a region make no difference, only the region does (placement_map() below prints
the measurement).

Physical addresses are not visible to a process, and the driver does not hand out device memory
in address order once requests of different sizes mix.  One allocation that covers (nearly) all
of the free memory, made before anything else of size, IS laid out in address order: Arena takes
that allocation and hands out pieces of it by region, so that a trainer can keep what a sweep
only reads (gradients) and what it writes (parameters, momentum, shifts) in different regions.
"""
import torch

__all__ = ["Arena", "HBM_REGIONS", "placement_map"]

HBM_REGIONS = 3      # MI355X: 288 GiB behave as three regions of 96 GiB


class Arena:
    """One allocation over the free device memory, handed out piecewise by HBM region.

    Region k covers the physical addresses [k, k + 1) * total / HBM_REGIONS.  The arena starts
    behind whatever the process allocated before it (`total - free` bytes, taken to sit at the
    low addresses), and `guard` bytes on either side of a region boundary are never handed out,
    since that estimate of the arena's own start is only good to a few GiB.
    """

    def __init__(self, device="cuda:0", keep_free=6 << 30, guard=4 << 30, nbytes=None):
        """Takes all but `keep_free` bytes of the free device memory (or `nbytes`, if given:
        the regions beyond its end are then empty)."""
        free, total = torch.cuda.mem_get_info(device)
        nbytes = (free - keep_free) >> 30 << 30 if nbytes is None else int(nbytes)
        if nbytes <= 0 or nbytes > free:
            raise RuntimeError("no free device memory for an arena")
        self.buffer = torch.empty(nbytes, dtype=torch.uint8, device=device)
        base = total - free                          # bytes in use below the arena
        size = total // HBM_REGIONS
        self.extent = []                             # per region: [first offset, end offset)
        for k in range(HBM_REGIONS):
            lo = (max(0, k * size - base + (guard if k else 0)) + 255) // 256 * 256
            hi = min(nbytes, (k + 1) * size - base - (guard if k + 1 < HBM_REGIONS else 0))
            self.extent.append((min(lo, nbytes), max(min(lo, nbytes), hi)))
        self.reset()

    def reset(self):
        """Forgets every piece handed out so far (views of them stay valid memory, and will be
        handed out again)."""
        self.bounds = [[lo, hi] for lo, hi in self.extent]   # per region: [next free, end)

    def free_in(self, region):
        lo, hi = self.bounds[region]
        return hi - lo

    def take(self, nbytes, region):
        """-> a uint8 view of `nbytes` bytes in `region` (256-byte aligned); raises
        MemoryError when the region has less than that left."""
        nbytes = int(nbytes)
        lo, hi = self.bounds[region]
        if lo + nbytes > hi:
            raise MemoryError("region %d has %d bytes left, %d asked for" % (region, hi - lo, nbytes))
        self.bounds[region][0] = (lo + nbytes + 255) // 256 * 256
        return self.buffer[lo:lo + nbytes]


def placement_map(nchunks=40, chunk_bytes=6 << 30, n=8, device="cuda:0", out=print):
    """Prints how the fused sweep's rate depends on WHERE its streams live: device memory is
    filled with `nchunks` equal allocations; with the n gradient streams in chunk i and x in
    chunk j, one nearest-even fused step is timed (HIP events on its sweep kernel) and shown
    as a percentage of the HBM peak (8 TB/s).  python -m paper_2102_08374_amd.placement"""
    import ctypes as C

    from . import binding as B
    torch.zeros(1, device=device)
    hip = None
    with open("/proc/self/maps") as fh:
        for line in fh:
            if "libamdhip64" in line:
                hip = C.CDLL(line.split()[-1])
                break
    hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    hip.hipEventDestroy.argtypes = [C.c_void_p]
    d = chunk_bytes // 4 // n
    chunks = []
    for _ in range(nchunks):
        c = torch.empty(chunk_bytes // 4, dtype=torch.float32, device=device)
        c.normal_(0.0, 1e-3)
        chunks.append(c)
    opts = B.LaunchOpts()
    desc = B.Desc(d, n, rounding=B.ROUND_NEAREST_EVEN, clip=B.default_clip(n), opts=opts)
    ws = B.new_workspace(desc, device)
    alpha = torch.full((1,), 700.0, dtype=torch.float32, device=device)
    ns = torch.zeros(1, dtype=torch.float64, device=device)
    cnt = torch.zeros(n, dtype=torch.int64, device=device)

    def sweep_ms(gi, xi):
        rows = [chunks[gi][k * d:(k + 1) * d] for k in range(n)]
        x = chunks[xi][:d]
        B.intsgd_step_fused(desc, rows, alpha, 0.1, x, ns, cnt, ws)
        best = float("inf")
        for _ in range(3):
            a, b = C.c_void_p(), C.c_void_p()
            hip.hipEventCreate(C.byref(a))
            hip.hipEventCreate(C.byref(b))
            opts.set_events(a.value, b.value)
            B.intsgd_step_fused(desc, rows, alpha, 0.1, x, ns, cnt, ws)
            opts.set_events(None, None)
            torch.cuda.synchronize()
            ms = C.c_float()
            hip.hipEventElapsedTime(C.byref(ms), a, b)
            hip.hipEventDestroy(a)
            hip.hipEventDestroy(b)
            best = min(best, ms.value)
        return best

    at_peak_ms = (4 * n + 8) * d / 8e12 * 1e3
    out("%d chunks of %.1f GiB; d = %d, n = %d; entries: %% of 8 TB/s with x in chunk j (column)"
        % (nchunks, chunk_bytes / 2 ** 30, d, n))
    for gi in range(0, nchunks, max(1, nchunks // 8)):
        row = ["--" if xi == gi else "%2d" % round(100 * at_peak_ms / sweep_ms(gi, xi))
               for xi in range(nchunks)]
        out("gradients in chunk %2d: %s" % (gi, " ".join(row)))


if __name__ == "__main__":
    import sys
    placement_map(int(sys.argv[1]) if len(sys.argv) > 1 else 40)
