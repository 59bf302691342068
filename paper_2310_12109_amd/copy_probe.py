"""Plain device-to-device copy of a known size, used to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE
counters (see profiles/): `python -m paper_2310_12109_amd.copy_probe [MiB]` copies a buffer 8 times."""
import sys

import torch


def main():
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 256
    n = mib * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(8):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {mib} MiB x 8")


if __name__ == "__main__":
    main()
