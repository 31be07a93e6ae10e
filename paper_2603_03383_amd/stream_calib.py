"""Calibration runs for profiling: a plain copy of known size (to scale rocprofv3's FETCH_SIZE / WRITE_SIZE
counters) and the pure-read ceiling at a few sizes.

    python3 -m paper_2603_03383_amd.stream_calib copy      # three 1 GiB copies, nothing else on the GPU
    python3 -m paper_2603_03383_amd.stream_calib read      # prints GB/s of the read stream at several sizes
"""
from __future__ import annotations

import sys

import torch

from . import binding as B


def read_ceiling(sizes=(33_554_432, 154_500_000, 1_048_576_000), n_workgroups=256, reps=10, pool_bytes=6 << 30):
    """{size: GB/s}: HIP-event timed, rotating through a pool much larger than the caches."""
    dev = torch.device("cuda:0")
    pool = torch.zeros(pool_bytes, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4, dtype=torch.uint8, device=dev)
    out = {}
    for size in sizes:
        nrot = max(1, pool_bytes // size)
        nread = 0
        for r in range(2):                       # warm-up
            B.medusa_stream_read(pool[(r % nrot) * size:], size, n_workgroups, sink)
        # `reps` launches back to back between two events, each on a different part of the pool, so that the host's
        # launch latency is hidden behind the previous launch and nothing is re-read from a cache
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for r in range(reps):
            nread = B.medusa_stream_read(pool[((r + 2) % nrot) * size:], size, n_workgroups, sink)
        b.record()
        b.synchronize()
        out[size] = nread * reps / (a.elapsed_time(b) * 1e-3) / 1e9
    return out


def main():
    what = sys.argv[1] if len(sys.argv) > 1 else "read"
    dev = torch.device("cuda:0")
    if what == "copy":
        n = 1 << 30
        a = torch.ones(n, dtype=torch.uint8, device=dev)
        b = torch.empty(n, dtype=torch.uint8, device=dev)
        for _ in range(3):
            B.medusa_stream_copy(a, b, n)
        torch.cuda.synchronize()
        print(f"copied {n} bytes 3 times (stream_copy_kernel)")
    else:
        for size, gbps in read_ceiling().items():
            print(f"read {size / 1e6:9.1f} MB: {gbps:7.1f} GB/s")


if __name__ == "__main__":
    main()
