"""Run one GEMV configuration a few dozen times over distinct packed copies, for a profiler.

    rocprofv3 --kernel-trace --stats -d out -- python3 -m paper_2412_17560_amd.profile_case 14336 4096 0.3
    python3 -m paper_2412_17560_amd.profile_case N K sparsity [--bits 4|8] [--batch B] [--panels] [--calls 48]

Synthetic weights and activations of the benchmark's distributions (gqsa_inputs); 24 device
copies of the packed matrix are walked, so every call reads its weights from HBM.  Prints the
partition and the algorithmic bytes of a call.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    p = argparse.ArgumentParser()
    p.add_argument("N", type=int)
    p.add_argument("K", type=int)
    p.add_argument("sparsity", type=float)
    p.add_argument("--bits", type=int, default=4)
    p.add_argument("--batch", type=int, default=1)
    p.add_argument("--panels", action="store_true", help="build the second image and use the matrix-core kernel")
    p.add_argument("--calls", type=int, default=48)
    p.add_argument("--copies", type=int, default=24)
    args = p.parse_args()

    import torch

    import gqsa_inputs as gi
    import paper_2412_17560_amd as gq

    dev = torch.device("cuda:0")
    W = gi.dense_weight_chunked(args.N, args.K, seed=1, workers=min(16, os.cpu_count() or 8))
    x = torch.from_numpy(gi.activations(args.batch, args.K, seed=1)).to(dev)
    y = torch.empty((args.batch, args.N), dtype=torch.float16, device=dev)
    e = gq.gqsa_export(gq.gqsa_pack(W, 16, args.bits, args.sparsity))
    hs = []
    for _ in range(args.copies):
        h = gq.gqsa_import(e["rowIndex"], e["groups"], e["values"], e["scales"], e["zeros"], args.N, args.K, 16, args.bits)
        if args.panels:
            gq.gqsa_build_panels(h)
        gq.gqsa_upload(h)
        hs.append(h)
    for k in range(args.calls):
        gq.gqsa_gemv(hs[k % len(hs)], x, y, panels=args.panels)
    torch.cuda.synchronize()
    info = gq.gqsa_info(hs[0])
    print(f"{args.N}x{args.K} S={args.sparsity} W{args.bits} batch={args.batch} panels={args.panels}: partition "
          f"{gq.gqsa_partition(hs[0])}, {info['algorithmic_bytes']} algorithmic bytes, {args.calls} calls", flush=True)


if __name__ == "__main__":
    main()
