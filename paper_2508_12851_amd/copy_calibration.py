"""Plain device-to-device copy of a known size, for calibrating rocprofv3's
FETCH_SIZE / WRITE_SIZE counters against a kernel whose HBM traffic is known:

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2508_12851_amd.copy_calibration

Copies 1 GiB (reads 1 GiB, writes 1 GiB) five times with torch's copy kernel.
"""
import torch

GIB = 1 << 30


def main():
    src = torch.full((GIB // 4,), 1.0, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied", GIB, "bytes x 5")


if __name__ == "__main__":
    main()
