"""The two forward kernels over the pooling factor (lookups per bag) and the row width, one MI355X.

    python -m paper_2410_22249_amd.autotune pooling [--lookups 4000000] [--steps 15]

The paper fixes the pooling factor at 150 and studies it only for L2 pinning (Sec. 4.3, the
figure of speedup against pooling factor): short bags are where the per-bag chain bag bounds ->
indices -> rows (Sec. 3.1) cannot be hidden inside one bag.  For 26 fp32 tables of 1,000,000 rows
and each (row width, pooling factor) this runs the same batch (batch size chosen so that a launch
holds about `--lookups` lookups, uniform indices, every table marked streaming) through the
one-wavefront-per-bag kernel ("stream" = 0) and the short-bag stream kernel ("stream" = 1,
automatic bags per group), and prints a markdown table: kernel time, algorithmic GB/s (rows +
indices + bag bounds + output), the ratio, and which kernel the automatic choice takes.
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
    ap.add_argument("--lookups", type=int, default=4_000_000)
    ap.add_argument("--steps", type=int, default=15)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dims", default="32,64,128,256")
    ap.add_argument("--pooling", default="1,2,4,8,16,32,64")
    a = ap.parse_args(argv)

    import numpy as np
    import torch
    import paper_2410_22249_amd as emb
    from inputgen import gen
    from paper_2410_22249_amd import autotune, metrics

    T, R = 26, 1_000_000
    print("| row bytes | pooling | batch | wave kernel us | stream kernel us | wave / stream | "
          "algorithmic GB/s (faster) | automatic choice |")
    print("|---|---|---|---|---|---|---|---|")
    for D in [int(x) for x in a.dims.split(",")]:
        for L in [int(x) for x in a.pooling.split(",")]:
            B = max(1, a.lookups // (T * L))
            wl = gen.Workload(name=f"pool_D{D}_L{L}", T=T, rows=(R,) * T, D=D, dtype="f32", B=B,
                              pooling=("fixed", L), dists=(("uniform",),) * T, seed=0x5EED0F00 + D)
            state = autotune._setup_wl(wl, 2)
            t = {}
            for name, s in (("wave", 0), ("stream", 1), ("auto", -1)):
                autotune.apply_tuning({**autotune.NEUTRAL, "stream": s})
                t[name] = autotune._time(state, a.steps, a.warmup)
            autotune.apply_tuning(autotune.NEUTRAL)
            nl = float(np.mean([b.num_lookups for b in state[6]]))
            algo = metrics.algorithmic_bytes(nl, T, B, D, 4)
            best = min(t["wave"], t["stream"])
            if abs(t["wave"] - t["stream"]) < 0.03 * best:
                chose = "(tie)"     # the timing cannot tell which kernel ran
            else:
                chose = "stream" if abs(t["auto"] - t["stream"]) < abs(t["auto"] - t["wave"]) else "wave"
            print(f"| {4 * D} | {L} | {B} | {t['wave'] * 1e6:.1f} | {t['stream'] * 1e6:.1f} | "
                  f"{t['wave'] / t['stream']:.2f} | {algo / best / 1e9:.0f} | {chose} |", flush=True)
            del state
            torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
