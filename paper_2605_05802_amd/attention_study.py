"""Decode attention, one layer, phases apart (prints a Markdown table).

Times the shared-prompt phase, the private phase and the fused launch of `sr_decode_step`'s attention on
synthetic pages at the 7B attention shape through `sr_probe_decode_attention`, with the pages in HBM and
with every load a cache hit, so that bandwidth, latency chain and the cost of fusing the phases can be
told apart.  Marshalling only: every number comes from the library's kernels and HIP events.

    python -m paper_2605_05802_amd.attention_study               # the table
    python -m paper_2605_05802_amd.attention_study --phases 1     # one configuration, for a counter run
"""
from __future__ import annotations

import argparse

from . import sr_probe_decode_attention


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--groups", type=int, default=16)
    ap.add_argument("--G", type=int, default=8)
    ap.add_argument("--shared", type=int, default=1024)
    ap.add_argument("--phases", type=int, default=0, help="1 shared, 2 private, 3 fused, 7 fused + merge launch; 0 = the whole table")
    ap.add_argument("--priv", type=int, default=1000)
    ap.add_argument("--splits", type=int, default=2)
    ap.add_argument("--hot", action="store_true")
    args = ap.parse_args()
    import torch
    assert torch.cuda.is_available(), "needs a GPU"
    torch.zeros(1, device="cuda")
    if args.phases:
        us, nbytes = sr_probe_decode_attention(args.groups, args.G, args.shared, args.priv, args.splits, args.phases,
                                               args.hot)
        print(f"phases={args.phases} priv={args.priv} splits={args.splits} hot={int(args.hot)}: {us:.1f} us, "
              f"{nbytes / 1e6:.0f} MB, {nbytes / us / 1e6:.2f} TB/s")
        return
    M = args.groups * args.G
    print(f"| rows | private tokens | splits | phase | K/V MB | HBM us | TB/s | all hits us |")
    print("|---|---|---|---|---|---|---|---|")
    for groups in (args.groups, args.groups * 5 // 8):
        for priv, splits in ((100, 1), (500, 2), (1000, 2), (1900, 2 if groups == args.groups else 3)):
            for ph, name in ((1, "shared prompt"), (2, "private"), (3, "both, one launch"),
                             (7, "both, and the merge launch")):
                if ph == 1 and priv != 1000:
                    continue
                us, nbytes = sr_probe_decode_attention(groups, args.G, args.shared, priv, splits, ph, False)
                hot, _ = sr_probe_decode_attention(groups, args.G, args.shared, priv, splits, ph, True)
                print(f"| {groups * args.G} | {priv} | {splits} | {name} | {nbytes / 1e6:.0f} | {us:.1f} | "
                      f"{nbytes / us / 1e6:.2f} | {hot:.1f} |")


if __name__ == "__main__":
    main()
