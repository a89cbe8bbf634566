"""A plain device-to-device copy of known size, for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE.

Run it under `rocprofv3 --pmc FETCH_SIZE` (then `WRITE_SIZE`): the copy kernel moves exactly
`--mib` MiB in and `--mib` MiB out per launch, so counter / (mib * 1024) is the factor by which
the counter over- or under-reports HBM KiB on this machine.  The buffer is larger than the 256 MB
Infinity Cache so that the copy really streams through HBM.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    src = torch.empty(a.mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps}")


if __name__ == "__main__":
    main()
