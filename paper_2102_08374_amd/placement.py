"""Where in HBM the written state lives (harness-side helper; no arithmetic of the method).

Measured on MI355X (288 GB of HBM3E): device memory behaves as three regions of 96 GB, most
likely the three ranks of the 12-high stacks, which share channels but own their banks.  A
sweep that reads its n gradient streams from one region and reads-modifies-writes x in ANOTHER
runs at 84-85 % of the HBM peak; with x in the SAME region as the gradients it runs at 79-80 %
(writes and reads then fight over the same banks: row conflicts and write-to-read turnarounds).
Offsets inside a region make no difference, only the region does.

Physical addresses are not visible to a process, and the driver does not hand out device memory
in address order once requests of different sizes mix, so the placement is found by timing:
spread a few candidate buffers over the free device memory (spacer allocations in between,
released afterwards), time the caller's own kernel on each, keep the fastest.  Done once at
set-up; a trainer that keeps its gradient and parameter buffers for the whole run pays it once.
"""
import torch

__all__ = ["allocate_apart", "HBM_REGIONS"]

HBM_REGIONS = 3      # MI355X: 288 GiB behave as three regions of 96 GiB


def allocate_apart(nbytes, device, time_fn, *, spread_bytes=48 << 30, keep_free=8 << 30,
                   max_candidates=7, choose=None, report=None):
    """-> a uint8 tensor of `nbytes` placed where `time_fn` runs fastest.

    time_fn(candidate) -> milliseconds (smaller is better), or a list of them (one per
    read-only buffer set the caller tries the candidate with): runs the caller's kernel(s)
    with the candidate as the written state and whatever read-only buffers the caller
    already holds.  Candidates are allocated one after the other with `spread_bytes` of
    spacer between them until less than `keep_free` bytes of device memory would remain, so
    that every region of the memory gets one.  choose(timings) -> index of the winner
    (default: smallest mean).  Everything but the winner is released (torch's cache
    included) before returning.  `report`, if given, receives the list of timings.
    """
    nbytes = int(nbytes)
    chunk = 4 << 30
    candidates, spacers, timings = [], [], []
    try:
        while len(candidates) < max_candidates:
            free, _ = torch.cuda.mem_get_info(device)
            if free - nbytes < keep_free:
                break
            c = torch.empty(nbytes, dtype=torch.uint8, device=device)
            c.zero_()
            candidates.append(c)
            left = spread_bytes
            while left > 0:
                free, _ = torch.cuda.mem_get_info(device)
                take = min(chunk, left)
                if free - take - nbytes < keep_free:
                    break
                spacers.append(torch.empty(take, dtype=torch.uint8, device=device))
                left -= take
        if not candidates:
            raise RuntimeError("not enough free device memory for %d bytes" % nbytes)
        for c in candidates:
            t = time_fn(c)
            timings.append([float(v) for v in t] if isinstance(t, (list, tuple)) else float(t))
    finally:
        spacers.clear()

    def mean(t):
        return sum(t) / len(t) if isinstance(t, list) else t

    best = choose(timings) if choose is not None else min(range(len(candidates)),
                                                          key=lambda i: mean(timings[i]))
    winner = candidates[best]
    candidates.clear()
    torch.cuda.empty_cache()
    if report is not None:
        report.extend(timings)
    return winner
