"""Where the streaming hint stops paying: the two constants of emb_bag_profile_reuse, one MI355X.

    python -m paper_2410_22249_amd.autotune hints [--tables 32] [--steps 60]

The paper picks a table's cache treatment from its access pattern (Sec. 4.3, Sec. 7 steps v-vi).
For uniform tables this sweeps how much of a table one batch draws (lookups per table / rows) over
several batch sizes and row widths, runs every case with all tables marked EMB_HINT_DEFAULT and
then EMB_HINT_STREAMING, and prints a markdown table: both kernel times, the cost of the
streaming hint in percent, the table size, and what the profiler's rule says for the first batch.
The rule's constants (rows in use beyond 256 MiB; fewer than 75 permille of the lookups expected
to repeat a row) are where the sign of that cost changes.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--tables", type=int, default=32)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--pooling", type=int, default=20)
    ap.add_argument("--shapes", default="64:2048,64:8192,128:8192,64:32768,128:32768,16:32768",
                    help="dim:batch pairs (fp32 rows)")
    ap.add_argument("--ratios", default="0.08,0.12,0.16,0.2,0.3,0.45,0.7",
                    help="lookups per table of one batch / rows of the table")
    a = ap.parse_args(argv)

    import torch
    from inputgen import gen
    from paper_2410_22249_amd import autotune

    T, L = a.tables, a.pooling
    print("| row bytes | lookups per table | lookups / rows | table MB | default us | streaming us | "
          "streaming costs | profiler says |")
    print("|---|---|---|---|---|---|---|---|")
    autotune.apply_tuning(autotune.NEUTRAL)
    for shape in a.shapes.split(","):
        D, B = (int(v) for v in shape.split(":"))
        for x in (float(v) for v in a.ratios.split(",")):
            R = int(B * L / x)
            if T * R * 4 * D > 0.6 * torch.cuda.get_device_properties(0).total_memory:
                continue    # the arena would not fit beside the batches
            wl = gen.Workload(name=f"hint_D{D}_B{B}", T=T, rows=(R,) * T, D=D, dtype="f32", B=B,
                              pooling=("fixed", L), dists=(("uniform",),) * T, seed=0x5EED1100 + D)
            state = autotune._setup_wl(wl, 4)
            hints = state[7]
            says = int(hints.sum().item())
            t = {}
            for name, v in (("default", 0), ("streaming", 1)):
                hints.fill_(v)
                t[name] = autotune._time(state, a.steps, a.warmup)
            print(f"| {4 * D} | {B * L} | {x:.2f} | {R * 4 * D / 1e6:.0f} | {t['default'] * 1e6:.1f} | "
                  f"{t['streaming'] * 1e6:.1f} | {100 * (t['streaming'] / t['default'] - 1):+.1f} % | "
                  f"{'streaming' if says == T else 'default' if says == 0 else f'{says} of {T} streaming'} |",
                  flush=True)
            del state, hints
            torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
