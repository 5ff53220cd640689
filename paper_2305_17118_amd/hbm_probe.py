"""Plain device copy of known size, for calibrating HBM traffic counters.

``python -m paper_2305_17118_amd.hbm_probe --mib 1024 --reps 5`` copies a buffer of the given
size `reps` times with torch's own copy kernel (one dispatch each, reading and writing exactly
that many bytes) and prints the achieved copy bandwidth.  Run under
``rocprofv3 --pmc FETCH_SIZE`` / ``--pmc WRITE_SIZE`` it shows what the counters report for a
known number of bytes, which is the scale factor applied to the decode kernel's counters.
"""
import argparse
import time

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=1024)
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    n = a.mib * 2 ** 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.reps
    print("copy %d MiB: %.1f us per dispatch, %.1f GB/s read + %.1f GB/s write" % (
        a.mib, dt * 1e6, n / dt / 1e9, n / dt / 1e9))


if __name__ == "__main__":
    main()
