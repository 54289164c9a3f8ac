"""Plain device-to-device copies of a known size, for calibrating rocprofv3's FETCH_SIZE /
WRITE_SIZE counters:

    rocprofv3 --pmc FETCH_SIZE -d out -o calib --output-format csv -- python3 -m paper_2602_21477_amd.calib_copy

Each copy reads and writes exactly SIZE bytes; whatever the counters report per copy
dispatch, divided into SIZE, is the factor the same counters are scaled by for the scan
kernel.
"""
import torch

SIZE = 1 << 30  # bytes per copy


def main():
    src = torch.empty(SIZE, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(4):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied", SIZE, "bytes x 4")


if __name__ == "__main__":
    main()
