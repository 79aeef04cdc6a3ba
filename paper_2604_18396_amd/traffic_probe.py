"""Calibration aid for HBM traffic counters: a plain device copy of known size.

Run under `rocprofv3 --pmc FETCH_SIZE` (then `WRITE_SIZE`): the copy kernel reads and
writes exactly `--mib` MiB per launch, which gives the factor between the counter's unit
and bytes.  torch is used for the copy only (plumbing)."""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=3)
    a = ap.parse_args()
    n = a.mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.iters}")


if __name__ == "__main__":
    main()
