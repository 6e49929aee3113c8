"""A plain device-to-device copy of known size, used only to calibrate the rocprofv3 HBM counters
(FETCH_SIZE / WRITE_SIZE) that profiles/ reports for the join kernel.

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2508_21230_amd.copy_probe --mib 4096
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=4096)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    n = a.mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps} (each copy reads and writes {a.mib * 1024} KiB)")


if __name__ == "__main__":
    main()
