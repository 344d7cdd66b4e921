"""Plain device-to-device copies of a known size: the yardstick for the HBM byte counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE): the copy kernel of each repetition reads
and writes exactly `--mib` MiB, so counter / (mib * 1024) is the factor between the counter's unit
and KiB on this machine.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=4)
    a = ap.parse_args()
    n = a.mib * 1024 * 1024 // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps}")


if __name__ == "__main__":
    main()
