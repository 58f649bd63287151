"""Runs one bf16 GEMM shape through the C ABI a few times, for profiling it alone.

    python3 -m paper_2107_06925_amd.gemm_probe M N K fwd|dgrad|wgrad [tile] [iters]

tile: e.g. 128x128, 256x256 or auto (the library's own choice).  Use under
rocprofv3 (--kernel-trace --stats, or --pmc <counters>).
"""
import os
import sys

import torch

from paper_2107_06925_amd import binding as b


def main():
    if len(sys.argv) < 5:
        sys.exit(__doc__)
    m, n, k, layout = int(sys.argv[1]), int(sys.argv[2]), int(sys.argv[3]), sys.argv[4]
    tile = sys.argv[5] if len(sys.argv) > 5 else "auto"
    iters = int(sys.argv[6]) if len(sys.argv) > 6 else 5
    if tile != "auto":
        os.environ["CHIMERA_GEMM_TILE"] = tile
    a_kc, b_kc = {"fwd": (1, 0), "dgrad": (1, 1), "wgrad": (0, 0)}[layout]
    A = torch.randn((m, k) if a_kc else (k, m), device="cuda").bfloat16()
    B = torch.randn((n, k) if b_kc else (k, n), device="cuda").bfloat16()
    if layout == "wgrad":
        C, epi = torch.zeros((m, n), device="cuda"), b.EPI_ACCUM_F32
    else:
        C, epi = torch.empty((m, n), device="cuda", dtype=torch.bfloat16), b.EPI_NONE
    for _ in range(iters):
        b.chimera_op_gemm(A, B, C, m, n, k, a_kc, b_kc, epi, workspace=None)
    torch.cuda.synchronize()
    print("ran %d x gemm %dx%dx%d %s tile=%s" % (iters, m, n, k, layout, tile))


if __name__ == "__main__":
    main()
