"""A plain device-to-device copy of known size, used to calibrate the FETCH_SIZE / WRITE_SIZE
hardware counters: `rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2305_04359_amd.copy_probe`
reads the counter for a kernel whose HBM traffic is known (it prints the byte count)."""
import sys

import torch


def main(mib: int = 1024) -> None:
    n = mib * (1 << 20) // 4
    a = torch.arange(n, dtype=torch.int32, device="cuda:0")
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)  # one elementwise copy kernel: reads n*4 bytes, writes n*4 bytes
    torch.cuda.synchronize()
    print(f"copy_probe: each copy kernel reads {n * 4} bytes and writes {n * 4} bytes")


if __name__ == "__main__":
    main(int(sys.argv[1]) if len(sys.argv) > 1 else 1024)
