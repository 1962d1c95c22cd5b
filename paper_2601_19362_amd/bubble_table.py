"""Bubble-rate estimate of the load-balancing strategies under both communication schemes
(paper Section 5.1 names the strategies, Eq. 1 gives the runtime under per-layer collectives,
Appendix F defines the bubble rate as idle time over total time, estimated by the packing
algorithm).

    python -m paper_2601_19362_amd.bubble_table --world 8 --samples-per-device 4

draws synthetic minibatches (sequence lengths clip(round(exp(mu + sigma Z)), lo, hi): a stand-in
for the long-tailed length histograms of the paper's datasets), plans each with LocalSort,
LB-Micro and LB-Mini through the native planner and prints, per strategy and scheme, the mean
estimated minibatch time relative to Collective + LocalSort and the mean bubble rate.  LB-Mini
gives devices different microbatch counts, so it exists only under ODC.  Host code only.
"""
from __future__ import annotations

import argparse
from typing import Dict, List, Tuple

import numpy as np

from . import packing

STRATEGIES = (("LocalSort", packing.LOCAL_SORT), ("LB-Micro", packing.LB_MICRO), ("LB-Mini", packing.LB_MINI))


def synthetic_lengths(n: int, seed: int, mu: float, sigma: float, lo: int, hi: int) -> List[int]:
    rng = np.random.default_rng(seed)
    return [int(v) for v in np.clip(np.rint(np.exp(mu + sigma * rng.standard_normal(n))), lo, hi)]


def estimate(world: int, samples_per_device: int, minibatches: int, max_tokens: int, hidden: int, seed: int,
             mu: float = 7.0, sigma: float = 1.0, lo: int = 128, hi: int = 32768) -> Dict[Tuple[str, str], Tuple[float, float]]:
    """{(scheme, strategy): (mean time relative to Collective + LocalSort, mean bubble rate)}."""
    acc: Dict[Tuple[str, str], List[Tuple[float, float]]] = {}
    for b in range(minibatches):
        seq = synthetic_lengths(world * samples_per_device, seed * 100003 + b, mu, sigma, lo, hi)
        base = None
        for name, mode in STRATEGIES:
            plan, _ = packing.plan_minibatch(seq, world, max_tokens, hidden, mode)
            t_coll, t_odc, _, bub_coll, bub_odc = packing.plan_runtime(seq, plan, hidden)
            if base is None:
                base = float(t_coll)          # Collective + LocalSort of this minibatch
            if mode != packing.LB_MINI:
                acc.setdefault(("Collective", name), []).append((t_coll / base, bub_coll))
            acc.setdefault(("ODC", name), []).append((t_odc / base, bub_odc))
    return {k: (float(np.mean([t for t, _ in v])), float(np.mean([x for _, x in v]))) for k, v in acc.items()}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--world", type=int, default=8)
    ap.add_argument("--samples-per-device", type=int, default=4)
    ap.add_argument("--minibatches", type=int, default=32)
    ap.add_argument("--max-tokens", type=int, default=32768)
    ap.add_argument("--hidden", type=int, default=3584)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args(argv)
    table = estimate(args.world, args.samples_per_device, args.minibatches, args.max_tokens, args.hidden, args.seed)
    print(f"{args.world} devices x {args.samples_per_device} samples, {args.minibatches} synthetic minibatches, "
          f"max {args.max_tokens} tokens per microbatch, cost(s) = s * (s + 6 * {args.hidden})")
    print(f"{'scheme':<11}{'strategy':<11}{'relative time':>14}{'bubble rate':>13}")
    for scheme in ("Collective", "ODC"):
        for name, _ in STRATEGIES:
            if (scheme, name) in table:
                t, bub = table[(scheme, name)]
                print(f"{scheme:<11}{name:<11}{t:>14.3f}{100 * bub:>12.1f}%")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
