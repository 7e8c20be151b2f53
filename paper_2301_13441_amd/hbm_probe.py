"""Calibration run for HBM traffic counters: one device-to-device copy of a known size.

Under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) the copy kernel's counter value divided by
the bytes it is known to move gives the scale of the counter on this machine; the same factor
is then applied to the forest kernel's reading.
"""
import sys

import torch


def main() -> int:
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
    n = mib * 1024 * 1024 // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {mib} MiB three times (reads {mib} MiB, writes {mib} MiB per copy)")
    return 0


if __name__ == "__main__":
    sys.exit(main())
