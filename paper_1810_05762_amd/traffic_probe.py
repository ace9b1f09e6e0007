"""A plain device-to-device copy of known size, for calibrating HBM traffic counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE): the copy reads and writes
exactly SIZE_MIB MiB per dispatch, so counter / size gives the factor by which the same
counter over- or under-reports for other kernels.
"""
import sys

import torch

SIZE_MIB = 256


def main():
    if not torch.cuda.is_available():
        print("traffic_probe needs a GPU", file=sys.stderr)
        sys.exit(1)
    n = SIZE_MIB * 1024 * 1024 // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:1000], src[:1000])
    print(f"copied {SIZE_MIB} MiB x 5")


if __name__ == "__main__":
    main()
