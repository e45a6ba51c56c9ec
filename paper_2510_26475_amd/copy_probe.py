"""A plain device-to-device copy of known size, for calibrating rocprofv3 byte counters.

    python -m paper_2510_26475_amd.copy_probe [--mib 1024] [--iters 3]

The copy reads N bytes and writes N bytes; what FETCH_SIZE / WRITE_SIZE report for its
kernel, divided by N, is the scale factor applied to the same counters of the verify kernels.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=3)
    args = ap.parse_args()
    n = args.mib << 20
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {n} bytes x {args.iters}")


if __name__ == "__main__":
    main()
