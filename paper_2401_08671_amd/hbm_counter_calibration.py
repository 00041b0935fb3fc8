"""Plain device-to-device copy of a known size, for calibrating HBM traffic counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE): the counter value of the copy
kernel divided by the bytes it is known to move gives the scale that converts the same
counter on the attention kernels into bytes.

    python -m paper_2401_08671_amd.hbm_counter_calibration [GiB]
"""
import sys

import torch


def main():
    gib = float(sys.argv[1]) if len(sys.argv) > 1 else 2.0
    n = int(gib * (1 << 30))
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {n} bytes x3 (each launch reads {n} and writes {n} bytes)")


if __name__ == "__main__":
    main()
