"""A plain device-to-device copy of known size, for calibrating the HBM byte counters.

Run under `rocprofv3 --pmc FETCH_SIZE` (then `WRITE_SIZE`): the copy kernel reads and writes exactly
`BYTES` bytes per launch, so counter value / BYTES gives the factor by which the same counter of another
kernel is scaled.
"""
import torch

BYTES = 1 << 30


def main():
    src = torch.empty(BYTES // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copied {BYTES} bytes x3")


if __name__ == "__main__":
    main()
