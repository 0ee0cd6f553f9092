#!/usr/bin/env python3
"""Known-size copy for calibrating rocprofv3's FETCH_SIZE / WRITE_SIZE counters (KiB per dispatch).

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out -- python3 tests/copy_calibration.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out -- python3 tests/copy_calibration.py

Each probe_copy_kernel dispatch reads and writes exactly --mib MiB; the ratio counter / (MiB * 1024) is the
factor by which the counters of the other kernels are scaled.  Also prints the achieved copy bandwidth."""
import argparse
import ctypes
import os
import time

import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mib", type=int, default=2048)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    lib = ctypes.CDLL(os.path.join(HERE, "libmsa_probe.so"))
    n = args.mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(args.reps):
        t0 = time.perf_counter()
        lib.probe_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), ctypes.c_ulonglong(n))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        print(f"copy {args.mib} MiB: {dt * 1e3:.3f} ms  {2 * n / dt / 1e9:.0f} GB/s (read + write)")
    assert torch.equal(src, dst)


if __name__ == "__main__":
    main()
