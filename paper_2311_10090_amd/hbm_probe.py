"""Achievable HBM bandwidth of this GPU with plain library kernels of known size.

Two uses: (1) the write-only and copy rates that the env-only rollout's roofline fraction is
put beside; (2) a kernel of exactly known traffic for scaling rocprofv3's FETCH_SIZE /
WRITE_SIZE counters (run this file under `rocprofv3 --pmc ...` and compare the counter of
the fill / copy dispatches with the byte counts printed here).

    python -m paper_2311_10090_amd.hbm_probe [--mib 1792] [--iters 20]
"""
import argparse
import json

import torch


def timed(fn, iters):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / iters * 1e-3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1792, help="buffer size (the cfg 2 trajectory is ~1792 MiB)")
    ap.add_argument("--iters", type=int, default=20)
    args = ap.parse_args()
    n = args.mib * (1 << 20) // 4
    x = torch.empty(n, dtype=torch.float32, device="cuda")
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    nbytes = n * 4
    t_fill = timed(lambda: x.fill_(1.0), args.iters)
    t_copy = timed(lambda: y.copy_(x), args.iters)
    print(json.dumps({
        "buffer_bytes": nbytes,
        "fill": {"bytes_written": nbytes, "seconds": t_fill, "GBs": nbytes / t_fill / 1e9},
        "copy": {"bytes_read": nbytes, "bytes_written": nbytes, "seconds": t_copy,
                 "GBs_read_plus_write": 2 * nbytes / t_copy / 1e9},
    }))


if __name__ == "__main__":
    main()
