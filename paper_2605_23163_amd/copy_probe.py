"""A plain device-to-device copy of known size, for calibrating HBM byte
counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE report KiB per dispatch;
dividing what they read for this copy by the bytes it really moves gives the
scale factor to apply to other kernels' readings).

    python -m paper_2605_23163_amd.copy_probe [--mib 1024] [--reps 5]

The copy kernel reads `mib` MiB and writes `mib` MiB per dispatch.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    n = a.mib << 20
    x = torch.empty(n, dtype=torch.uint8, device="cuda")
    x.random_(0, 255)
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        y.copy_(x)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps} (each dispatch reads {n} bytes and writes {n} bytes)")


if __name__ == "__main__":
    main()
