"""Plain copy of known size, used to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE
counters: run it under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) and compare
what the counter reports for the elementwise kernel with the bytes below.

  python -m paper_2102_08374_amd.copy_probe [MiB]
"""
import sys

import torch


def main():
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
    n = mib * 1024 * 1024 // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)      # one elementwise kernel: reads n*4 B, writes n*4 B
    torch.cuda.synchronize()
    print("copy_probe: each elementwise launch reads %d bytes and writes %d bytes" % (n * 4, n * 4))


if __name__ == "__main__":
    main()
