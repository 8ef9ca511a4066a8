"""Plain streaming copy through the library's copy kernel: the measured HBM ceiling of the box, and the
known-size kernel that hardware counters (FETCH_SIZE / WRITE_SIZE) are calibrated against.

    python -m paper_2205_05632_amd.copybench [--mib 1024] [--iters 20]

Prints one JSON line: bytes moved per launch (read + write) and the achieved GB/s.
"""
import argparse
import json
import time

import torch

from . import binding as B


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024, help="size of the source buffer")
    ap.add_argument("--iters", type=int, default=20)
    args = ap.parse_args()
    n = args.mib * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    src.random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(3):
        B.compams_copy(dst, src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.iters):
        B.compams_copy(dst, src)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.iters
    assert torch.equal(dst, src)
    print(json.dumps({"kernel": "k_copy16", "bytes_read": n, "bytes_written": n, "us_per_launch": dt * 1e6,
                      "gbps": 2 * n / dt / 1e9}))


if __name__ == "__main__":
    main()
