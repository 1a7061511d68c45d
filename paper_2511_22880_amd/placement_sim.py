"""A small what-if for the placement routine: synthetic adapter demand on a group of servers, placed by
lora_place_assign and by the two static placements the paper compares with (Evaluation, "Baselines":
adapters spread at random; adapters sorted by rank and cut into equal runs).  No GPU needed.

Per server it reports the utilisation the placement leads to under two cost models of the LoRA delta:
  ragged  a token of a rank-r adapter costs 1 / op[r]            (this library: no token pays for
          another adapter's rank);
  padded  a token costs 1 / op[largest rank served on that server] (kernels sized to the largest rank
          in the batch, the effect the paper's motivation measures).
op[r] = tokens/s of the delta kernels alone at rank r, measured with this library on one MI355X
(token-heavy batch, 4096 -> 4096; see profiles/).  They are not end-to-end operating points under a
latency objective, which is what a deployment would profile; only their ratios matter here.

    python -m paper_2511_22880_amd.placement_sim [--servers 8] [--adapters 200] [--alpha 1.1] [--seed 0]
"""
from __future__ import annotations

import argparse

import numpy as np

from . import binding as L

def operating_points() -> dict:
    """{rank: tokens/s one GPU sustains through shrink + expand of a 4096 -> 4096 projection with every
    adapter at that rank}, measured with bench.py on the MI355X machine and kept in profiles/measured.json."""
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "measured.json")
    with open(path) as f:
        return {int(k): float(v) for k, v in json.load(f)["placement_operating_points_tokens_per_s"].items()}


def utilisation(phi: np.ndarray, ranks: np.ndarray, demand: np.ndarray, op: dict, padded: bool) -> np.ndarray:
    servers = phi.shape[1]
    out = np.zeros(servers)
    for s in range(servers):
        on = phi[:, s] > 0
        if not on.any():
            continue
        rmax = int(ranks[on].max())
        cost = np.array([1.0 / op[rmax if padded else int(r)] for r in ranks[on]])
        out[s] = float((phi[on, s] * demand[on] * cost).sum())
    return out


def static_placement(kind: str, servers: int, ranks: np.ndarray, g: np.random.Generator) -> np.ndarray:
    n = ranks.shape[0]
    phi = np.zeros((n, servers))
    if kind == "random":
        phi[np.arange(n), g.integers(0, servers, size=n)] = 1.0
    else:  # contiguous: by rank, equal counts
        order = np.argsort(ranks, kind="stable")
        for i, a in enumerate(order):
            phi[a, min(servers - 1, i * servers // n)] = 1.0
    return phi


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--servers", type=int, default=8)
    ap.add_argument("--adapters", type=int, default=200)
    ap.add_argument("--alpha", type=float, default=1.1, help="power-law exponent of adapter popularity")
    ap.add_argument("--load", type=float, default=0.7, help="total demand as a fraction of the group's ragged capacity")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    g = np.random.default_rng(args.seed)
    OP = operating_points()
    rank_set = np.array(sorted(OP))
    ranks = rank_set[g.permutation(args.adapters) % len(rank_set)].astype(np.int32)
    pop = (np.arange(args.adapters) + 1.0) ** -args.alpha
    pop = pop[g.permutation(args.adapters)]
    per_token = np.array([1.0 / OP[int(r)] for r in ranks])
    demand = pop / (pop * per_token).sum() * args.load * args.servers      # tokens/s
    placements = {
        "rank-aware (lora_place_assign)": L.lora_place_assign(args.servers, ranks, demand, OP)["phi"],
        "random": static_placement("random", args.servers, ranks, g),
        "contiguous by rank": static_placement("contiguous", args.servers, ranks, g),
    }
    print(f"{args.servers} servers, {args.adapters} adapters, popularity ~ k^-{args.alpha}, load {args.load:.2f}")
    print(f"{'placement':34s} {'ragged: max / mean util':>26s} {'padded: max / mean util':>26s} {'copies':>7s}")
    for name, phi in placements.items():
        ur = utilisation(phi, ranks, demand, OP, False)
        up = utilisation(phi, ranks, demand, OP, True)
        print(f"{name:34s} {ur.max():12.3f} / {ur.mean():.3f} {up.max():18.3f} / {up.mean():.3f} {int((phi > 0).sum()):7d}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
