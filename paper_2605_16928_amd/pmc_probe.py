"""Small driver for hardware-counter runs (rocprofv3 --pmc): launches the decode kernels of
configuration 2 a few times, plus a plain device-to-device copy of known size whose counter reading
calibrates the byte counters.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d gpurun_out/pmc_fetch -o c2 --output-format csv \
        -- python3 -m paper_2605_16928_amd.pmc_probe
    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d gpurun_out/pmc_write -o c2 --output-format csv \
        -- python3 -m paper_2605_16928_amd.pmc_probe
"""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    from paper_2605_16928_amd import workloads as wl
    from paper_2605_16928_amd.pipeline import DecodeRun
    run = DecodeRun(wl.c2("cuda:0", seed=100))
    n = 1 << 28                                     # 1 GiB read + 1 GiB written per copy
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    for _ in range(5):
        run.step()
        run.dense_attn(run.out)
    torch.cuda.synchronize()
    print("copy bytes per launch:", n * 4, "read and", n * 4, "written")


if __name__ == "__main__":
    main()
