"""Small driver for hardware-counter runs (rocprofv3 --pmc), one counter set per run.

Decode (default): launches the decode kernels of configuration 2 a few times, plus a plain
device-to-device copy of known size whose counter reading calibrates the byte counters.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d gpurun_out/pmc_fetch -o c2 --output-format csv \
        -- python3 -m paper_2605_16928_amd.pmc_probe
    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d gpurun_out/pmc_write -o c2 --output-format csv \
        -- python3 -m paper_2605_16928_amd.pmc_probe

Prefill (argument `prefill`): the last 8192-query chunk of the 1,048,576-token configuration --
retrieval heads dense, retrieval heads with per-query top-p, local heads -- for the matrix-core counters.

    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_BUSY_CU_CYCLES GRBM_GUI_ACTIVE \
        --kernel-trace -d gpurun_out/pmc_mfma -o c4 --output-format csv -- python3 -m paper_2605_16928_amd.pmc_probe prefill
"""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def decode():
    from paper_2605_16928_amd import workloads as wl
    from paper_2605_16928_amd.pipeline import DecodeRun
    run = DecodeRun(wl.c2("cuda:0", seed=100))
    n = 1 << 28                                     # 1 GiB read + 1 GiB written per copy
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    for _ in range(5):
        run.step_one_stream()                       # score pass + rtp_decode_attention (local heads carried)
        run.step()                                  # selection + retrieval-head attention as one call, local heads apart
        run.step(fused=False)                       # ... and selection and attention as two calls
        run.dense_attn(run.out)
    torch.cuda.synchronize()
    print("copy bytes per launch:", n * 4, "read and", n * 4, "written")


def prefill():
    from paper_2605_16928_amd import rtp, workloads as wl
    from paper_2605_16928_amd.pipeline import PrefillRun
    w = wl.c4_chunk("cuda:0", chunk=127)
    run = PrefillRun(w)
    for _ in range(2):
        rtp.rtp_sparse_attn_prefill(run.desc, w.qI, w.q, None, w.kI, w.N * 16, run.Kp, run.Vp, run.rs, run.hs,
                                    w.chunk_start, w.T, 1.0, run.out, None, None, None, None, run.ws)
        run.sparse_prefill(p=0.9)
        run.local_attn()
    torch.cuda.synchronize()
    pairs = sum(w.chunk_start + t + 1 for t in range(w.T))
    print("causal (query, key) pairs per head in this chunk:", pairs, "; 512 flop per pair and head")


if __name__ == "__main__":
    prefill() if len(sys.argv) > 1 and sys.argv[1] == "prefill" else decode()
