"""Counter calibration aid: a plain device-to-device copy of known size, so that what
rocprofv3's FETCH_SIZE / WRITE_SIZE read for it can scale the same counters read for the
FFN kernel.  Usage: python -m paper_2512_13525_amd.calib_copy [MiB] [repeats]"""
import sys

import torch


def main() -> None:
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 512
    reps = int(sys.argv[2]) if len(sys.argv) > 2 else 4
    n = mib << 20
    # distinct source buffers so that every copy reads from HBM, not from the memory-side cache
    srcs = [torch.full((n,), i + 1, dtype=torch.uint8, device="cuda") for i in range(reps)]
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for s in srcs:
        dst.copy_(s)
    torch.cuda.synchronize()
    print(f"copied {reps} x {mib} MiB ({n} bytes read + {n} bytes written per copy)")


if __name__ == "__main__":
    main()
