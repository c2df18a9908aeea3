"""A plain device-to-device copy of known size, to calibrate rocprofv3's
FETCH_SIZE / WRITE_SIZE counters: the factor (bytes really moved) / (counter
reading) found here scales the same counters read for the scoring kernels.

    rocprofv3 --pmc FETCH_SIZE -d out -o copy_fetch -- python3 -m paper_2511_12934_amd.profiling.copy_kernel

Copies ``MIB`` MiB (default 1024, far beyond the caches) ``REPS`` times with an
elementwise kernel (``dst = src * 1``: a same-type ``copy_`` could go through the
copy engines and never show up as a dispatch); each dispatch reads MIB MiB and
writes MIB MiB.
"""
from __future__ import annotations

import sys


def main(mib: int = 1024, reps: int = 5) -> None:
    import torch
    if not torch.cuda.is_available():
        sys.exit("copy_kernel needs a GPU")
    n = mib * (1 << 20) // 4
    src = torch.arange(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(reps):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    assert bool((dst[-5:] == src[-5:]).all())
    print(f"copied {mib} MiB x {reps}: each dispatch reads {mib * 1024} KiB and writes {mib * 1024} KiB")


if __name__ == "__main__":
    main(*(int(a) for a in sys.argv[1:3]))
