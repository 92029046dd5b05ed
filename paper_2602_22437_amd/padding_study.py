"""Offline padding study with the library's planner (host only, no GPU needed).

The paper chooses the FSDP group size by simulating layouts offline so that rounding to block
multiples costs least, and reports the padding overhead of the plan against the FSDP size for row granularities
1x / 16x / 128x of the expert-MLP matrices (Section 6.4, padding figure).  This tool runs that
sweep on synthetic units shaped like the two models the section uses.

    python -m paper_2602_22437_amd.padding_study [--model deepseek|gpt_oss|gpt_oss_fused] [--order 0..3]
                                                 [--units all|listing|both]
    python -m paper_2602_22437_amd.padding_study --pick 480 544        # the FSDP sizes of a range with least padding
"""
from __future__ import annotations

import argparse
import time
from typing import Dict, List, Sequence, Tuple

from . import binding as B


def moe_unit(model: str, rows_per_block: int) -> List[Tuple[int, int, int, int]]:
    """(rows, cols, mode, g_explicit) per tensor: expert-MLP matrices with a sharding granularity of
    `rows_per_block` whole rows, everything else element-wise (g = 1)."""
    def mat(r, c):
        return (r, c, B.RS_BLOCK_EXPLICIT, rows_per_block * c)

    def plain(r, c):
        return (r, c, B.RS_BLOCK_EXPLICIT, 1)

    if model == "deepseek":
        h, inter, ne = 7168, 2048, 256
        ts = []
        for _ in range(ne + 1):                      # routed experts and the shared expert
            ts += [mat(inter, h), mat(inter, h), mat(h, inter)]
        return ts
    h, nq, nkv, hd, ne = 2880, 64, 8, 64, 128
    ts = [plain(nq * hd, h), plain(nkv * hd, h), plain(nkv * hd, h), plain(h, nq * hd), plain(ne, h)]
    if model == "gpt_oss":
        for _ in range(ne):
            ts += [mat(2 * h, h), mat(h, h)]
    elif model == "gpt_oss_fused":                   # all experts in one parameter tensor
        ts += [mat(ne * 2 * h, h), mat(ne * h, h)]
    else:
        raise ValueError("unknown model")
    return ts


def sweep(model: str, worlds: Sequence[int], granularities: Sequence[int] = (1, 16, 128),
          order: int = B.RS_ORDER_DEFAULT) -> Dict[int, Dict[int, Tuple[float, float]]]:
    """{rows_per_block: {world: (padding / payload, planner seconds)}}; `order` may carry
    B.RS_UNITS_LISTING to keep the search to the candidate units of Algorithm 1 as listed."""
    out: Dict[int, Dict[int, Tuple[float, float]]] = {}
    for g in granularities:
        unit = moe_unit(model, g)
        out[g] = {}
        for w in worlds:
            t0 = time.perf_counter()
            plan = B.rs_plan_create_ordered(unit, w, 16, 2, 0, order)
            dt = time.perf_counter() - t0
            out[g][w] = (B.rs_plan_padding_elems(plan) / B.rs_plan_payload_elems(plan), dt)
            B.rs_plan_destroy(plan)
    return out


def pick_world(model: str, lo: int, hi: int, rows_per_block: int,
               order: int = B.RS_ORDER_DEFAULT) -> List[Tuple[float, int]]:
    """The section's guideline as a tool: every FSDP size of [lo, hi] with its padding overhead,
    least padding first (equal overheads: smaller size first)."""
    unit = moe_unit(model, rows_per_block)
    found = []
    for w in range(lo, hi + 1):
        plan = B.rs_plan_create_ordered(unit, w, 16, 2, 0, order)
        found.append((B.rs_plan_padding_elems(plan) / B.rs_plan_payload_elems(plan), w))
        B.rs_plan_destroy(plan)
    return sorted(found)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="deepseek", choices=["deepseek", "gpt_oss", "gpt_oss_fused"])
    ap.add_argument("--order", type=int, default=B.RS_ORDER_DEFAULT)
    ap.add_argument("--units", default="both", choices=["all", "listing", "both"],
                    help="candidate units of the search: Algorithm 1 as listed, the library's wider set, or both")
    ap.add_argument("--worlds", default="8,16,32,64,96,128,192,256,384,512,768,1024")
    ap.add_argument("--pick", type=int, nargs=2, metavar=("LO", "HI"),
                    help="rank the FSDP sizes of [LO, HI] by padding overhead instead of sweeping --worlds")
    args = ap.parse_args()
    if args.pick:
        lo, hi = args.pick
        print(f"FSDP sizes {lo}..{hi} with the least padding, {args.model}-shaped MoE unit")
        for g in (1, 16, 128):
            ranked = pick_world(args.model, lo, hi, g, args.order)
            print(f"{g:>4d}x rows: " + ", ".join(f"{w} ({100 * p:.2f}%)" for p, w in ranked[:5])
                  + f"  ... worst {ranked[-1][1]} ({100 * ranked[-1][0]:.2f}%)")
        return
    worlds = [int(x) for x in args.worlds.split(",")]
    variants = {"all": [("the library's search", 0)], "listing": [("Algorithm 1 as listed", B.RS_UNITS_LISTING)],
                "both": [("Algorithm 1 as listed", B.RS_UNITS_LISTING), ("the library's wider search", 0)]}[args.units]
    print(f"padding overhead (padding / parameter elements), {args.model}-shaped MoE unit, bf16, 16-byte units")
    for label, flag in variants:
        res = sweep(args.model, worlds, order=args.order | flag)
        print(f"-- candidate units: {label}")
        print("FSDP size " + "".join(f"{w:>9d}" for w in worlds))
        for g, row in res.items():
            print(f"{g:>4d}x rows " + "".join(f"{100 * row[w][0]:8.2f}%" for w in worlds))
        print("planner s  " + "".join(f"{max(res[g][w][1] for g in res):9.3f}" for w in worlds))


if __name__ == "__main__":
    main()
