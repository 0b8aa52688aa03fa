"""Plain device-to-device copy of a known size: the reference the FETCH_SIZE / WRITE_SIZE counters of
rocprofv3 are scaled by (run it under `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`).

    python -m paper_2112_01801_amd.hbm_calib [MiB]

Copies MiB (default 1024) of float32 five times with torch's elementwise copy kernel; each launch reads
MiB and writes MiB of HBM (the buffers are far larger than the 256 MB last-level cache).
"""
import sys

import torch


def main():
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
    n = mib * 1024 * 1024 // 4
    a = torch.ones(n, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(5):
        b.copy_(a)
    torch.cuda.synchronize()
    print("copied %d MiB x5" % mib)


if __name__ == "__main__":
    main()
