"""Plain device copy of a known size, for scaling rocprofv3's FETCH_SIZE /
WRITE_SIZE readings:

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2508_15881_amd.traffic_calibration

Copies 1 GiB (float32) five times with an elementwise kernel; every launch
reads 1 GiB and writes 1 GiB.  The ratio known bytes / counter reading is
the factor applied to the decode kernel's counters.
"""
import torch


def main():
    n = (1 << 30) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    print("copied 5 x %d bytes" % (n * 4))


if __name__ == "__main__":
    main()
