"""Workload for hardware-counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE): a plain element-wise kernel of
known traffic (the scale reference), then verify passes of the bench shape so that every kernel of the path shows up
with its per-dispatch counters.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d out -o fetch -- python3 paper_2510_19705_amd/pmc_probe.py
"""
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2510_19705_amd import hsd, inputs  # noqa: E402

REF_MIB = 256


def main():
    shape = dict(inputs.SHAPES["1b"], n_layers=2)
    w = inputs.make_weights(shape, seed=3, bf16=True)
    model = hsd.Model(shape, hsd.BF16, 1024, 64, inputs.ROPE_BASE, inputs.EPS, rows_copy_layers=2)
    model.load(w)
    tok = torch.from_numpy(inputs.make_prompt(shape["vocab"], 600, seed=4)).cuda()
    for p0 in range(0, 512, 64):
        model.model_pass(tok[p0:p0 + 64], p0, 2, 0)
    # reference: reads REF_MIB MiB, writes REF_MIB MiB
    src = torch.ones(REF_MIB * (1 << 20) // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.add(src, 1.0, out=dst)
    torch.cuda.synchronize()
    for _ in range(10):
        model.model_pass(tok[512:518], 512, 2, 6)       # verify pass, 6 rows (tiled kernels)
    for _ in range(10):
        model.model_pass(tok[518:519], 518, 2, 1)       # draft step, 1 row (row kernel)
    torch.cuda.synchronize()
    print("pmc probe done: reference kernel moves %d MiB each way" % REF_MIB)


if __name__ == "__main__":
    main()
