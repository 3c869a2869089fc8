"""What operand traffic leaves of the matrix pipe (prints a Markdown table).

`sr_probe_mfma_under_loads` alternates sixteen register-resident 32x32x16 bf16 MFMAs per wavefront with 0, 2, 4 or 8
wavefront-wide 16-byte-per-lane loads from a small buffer, into registers or straight into LDS, with or without LDS
reads beside them.  Four loads per sixteen MFMAs is the operand traffic of a 256 x 256 x 32 GEMM step on eight
computing wavefronts, so the row for 4 is the rate a tiled GEMM of that shape cannot exceed on this chip.
Marshalling only: every number comes from the library's kernels and HIP events.

    python -m paper_2605_05802_amd.matrix_pipe_study
"""
from __future__ import annotations

import argparse

from . import sr_probe_mfma_under_loads


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--repeat", type=int, default=2)
    args = ap.parse_args()
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    scratch = torch.zeros(256 * 512, dtype=torch.float32, device="cuda")
    print("| buffer | path | loads per 16 MFMAs | LDS reads per 16 MFMAs | PFLOP/s | TB/s of loads |")
    print("|---|---|---|---|---|---|")
    for mib, where in ((1, "1 MiB (L2)"), (64, "64 MiB (memory-side cache)")):
        buf = torch.zeros(mib << 18, dtype=torch.int32, device="cuda")
        cases = [(0, 0, False), (0, 0, True), (2, 2, False), (2, 4, False), (2, 8, False), (2, 4, True),
                 (1, 2, False), (1, 4, False), (1, 8, False), (0, 0, False)]
        for path, loads, ds in cases:
            best = max(sr_probe_mfma_under_loads(buf, scratch, path, loads, ds) for _ in range(args.repeat))
            name = ("none", "into registers", "straight into LDS")[path]
            print(f"| {where} | {name} | {loads} | {12 if ds else 0} | {best[0] / 1e3:.2f} | {best[1] / 1e3:.1f} |", flush=True)


if __name__ == "__main__":
    main()
