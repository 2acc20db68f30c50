"""A plain device-to-device copy of a known size, used to calibrate the FETCH_SIZE / WRITE_SIZE
hardware counters (run it under `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE`: the copy kernel
moves exactly `--mib` MiB in each direction)."""
import argparse

import torch

if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=256)
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    src = torch.empty(a.mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {a.mib} MiB x {a.reps}")
