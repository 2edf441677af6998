"""Plain device-to-device copy of a known size, for calibrating rocprofv3 HBM counters.

``rocprofv3 --pmc FETCH_SIZE -- python -m paper_2401_02669_amd.hbm_probe --gib 4`` shows what the
counter reads for a kernel that fetches exactly ``gib`` GiB (and, with WRITE_SIZE, writes as much);
the ratio (known bytes / counter) scales the same counter's reading for the MicroAttention kernel.
"""
import argparse

import torch


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=float, default=4.0)
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    n = int(a.gib * (1 << 30)) // 4
    src = torch.arange(n, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(a.reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:1024], src[:1024])
    print("copied %d bytes x %d (read and written once each per copy)" % (n * 4, a.reps), flush=True)


if __name__ == "__main__":
    main()
