"""Plain device-to-device copy of a known size, for calibrating the HBM byte
counters of rocprofv3 (FETCH_SIZE / WRITE_SIZE) against a known traffic:

    rocprofv3 --pmc FETCH_SIZE -- python3 -m paper_2605_12245_amd.copy_probe

copies 1 GiB five times with torch's element-wise copy kernel (1 GiB read and
1 GiB written per dispatch).
"""
import sys

import torch


def main(gib: float = 1.0, reps: int = 5) -> None:
    n = int(gib * (1 << 30)) // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        # a strided-free dtype-preserving copy: one vectorized elementwise kernel per call
        torch.add(src, 0, out=dst)
    torch.cuda.synchronize()
    print(f"copied {n * 4} bytes x {reps}")


if __name__ == "__main__":
    main(float(sys.argv[1]) if len(sys.argv) > 1 else 1.0)
