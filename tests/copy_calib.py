"""Counter calibration: one plain device-to-device copy of a known size (torch's copy kernel).

Run under `rocprofv3 --pmc FETCH_SIZE` (then `WRITE_SIZE`): the counter value of the copy dispatch divided by
the known bytes gives the factor by which the same counter of the library's kernels is scaled to HBM bytes.
"""
import sys

import torch

MIB = int(sys.argv[1]) if len(sys.argv) > 1 else 1024
src = torch.full((MIB << 20,), 1, dtype=torch.uint8, device="cuda:0")
dst = torch.empty_like(src)
torch.cuda.synchronize()
for _ in range(3):
    dst.copy_(src)          # reads MIB MiB, writes MIB MiB per launch
torch.cuda.synchronize()
print(f"copied {MIB} MiB x3")
