"""Times every compiled instance on a range of problem shapes on the MI355X in this machine and writes
tests/golden/mi355x_shape_sweep.txt (performance measurements for the selector test; no expected values of the
parity tests come from here).  Run from the repository root:  python tests/golden/sweep_instances.py"""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
import paper_2511_16041_amd as atb  # noqa: E402

SHAPES = ([(8192, 8192, 8192), (4096, 4096, 4096), (8192, 14336, 4096), (3000, 5000, 4104)]
          + [(M, 2048, K) for M in (1024, 2048, 4096) for K in (2048, 4096, 8192)] + [(512, 512, 2048)]
          + [(M, 8192, 8192) for M in (16, 64, 128, 256, 512, 1024)])


def main():
    torch.manual_seed(0)
    inst = atb.instances()
    lines = ["# TFLOP/s of every compiled instance on a range of problem shapes, one MI355X, one session (normal-distributed A and B;",
             "# 20 timed launches after 10 for the large problems, 100 after 100 for the others, after a burn-in; HIP events).  Written by",
             "# tests/golden/sweep_instances.py; tests/test_abi_host.py checks the selector's pick against it.",
             "# columns: M N K, then one figure per instance in the order of atb_instance_get:",
             "# " + " ".join(",".join(map(str, t)) for t in inst)]
    for (M, N, K) in SHAPES:
        A_bfp = atb.bfp16_quantize(torch.randn(M, K, device="cuda"))
        B = torch.randn(K, N, device="cuda").bfloat16()
        C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        big = M * N * K > 1e11
        # the clock settles over the first tens of ms after an idle pause: burn in before the first instance is timed
        p = atb.Gemm(M, N, K, *inst[0])
        bench.time_plan(p, A_bfp, B, C, 1, 60 if big else 300)
        p.close()
        vals = []
        for t in inst:
            p = atb.Gemm(M, N, K, *t)
            _, kms = bench.time_plan(p, A_bfp, B, C, 20 if big else 100, 10 if big else 100)
            p.close()
            vals.append(2.0 * M * N * K / (kms * 1e-3) / 1e12)
        print((M, N, K), " ".join(f"{v:.1f}" for v in vals), flush=True)
        lines.append(f"{M} {N} {K}  " + " ".join(f"{v:.1f}" for v in vals))
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "mi355x_shape_sweep.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
