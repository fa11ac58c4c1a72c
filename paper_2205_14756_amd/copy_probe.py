"""Plain device-to-device copy of a known size, for calibrating the HBM traffic counters.

rocprofv3's FETCH_SIZE / WRITE_SIZE (KiB per dispatch) are read for this copy -- whose traffic is
known: `bytes` read and `bytes` written per launch -- and the ratio counter/known scales the
readings taken for the module's kernels in the same way.

    python3 -m paper_2205_14756_amd.copy_probe [MiB]
"""
import sys

import torch


def main():
    mib = int(sys.argv[1]) if len(sys.argv) > 1 else 512
    n = mib * 1024 * 1024 // 2
    src = torch.ones(n, device="cuda", dtype=torch.float16)
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(f"copy_probe: 5 copies of {mib} MiB (read {mib} MiB + write {mib} MiB per launch)")


if __name__ == "__main__":
    main()
