"""A time-stepped what-if for the placement routine: synthetic adapter demand that drifts from step to
step, placed for every step by lora_place_extrapolate + lora_place_assign from what was observed up to
the step before (the paper's System Design, "Adapter Placement and Request Routing", Algorithm 1,
steps 1 to 5), next to the two static placements the paper compares with (Evaluation, "Baselines":
adapters spread at random; adapters sorted by rank and cut into equal runs).  No GPU needed.

Demand.  `adapters` adapters, ranks balanced over the measured rank set; inside a rank the adapters'
shares follow a power law (alpha = 1, the paper's annotation of its production trace); the ranks'
shares of the traffic follow one of the three shapes of Evaluation, "Traces":
  uniform      every rank the same share, all the time;
  shifting     at the start rank 128 has half the traffic and the other ranks share the rest equally;
               this shifts linearly until, at the end, rank 8 has half;
  exponential  the share halves from one rank to the next larger one, all the time.
Every adapter's demand carries seeded multiplicative noise (log-normal, `--noise`), so the projection of
step 1 has something to project.  Traces, datasets and a serving stack stay out of scope.

Per step the simulator reports, under the demand that really arrived in that step,
  peak / mean utilisation of the servers for two cost models of the LoRA delta:
     ragged  a token of a rank-r adapter costs 1 / op[r]            (this library: no token pays for
             another adapter's rank);
     padded  a token costs 1 / op[largest rank served on that server] (kernels sized to the largest rank
             in the batch, the effect the paper's motivation measures);
  adapters moved: (adapter, server) pairs of the step's table that the previous table did not have,
     i.e. copies some server has to fetch, counted and weighted by rank (bytes are proportional to it).
`--no-relabel` leaves out step 5 (no previous table is given to lora_place_assign), which shows what
the relabelling saves.  op[r] = tokens/s of the delta kernels alone at rank r, measured with this
library on one MI355X and kept in profiles/measured.json; they are not end-to-end operating points
under a latency objective, which is what a deployment would profile; only their ratios matter here.

    python -m paper_2511_22880_amd.placement_sim [--trace shifting] [--steps 48] [--servers 8] [--adapters 100]
"""
from __future__ import annotations

import argparse
import json
import os
from typing import Callable, Dict, Optional

import numpy as np

TRACES = ("uniform", "shifting", "exponential")


def operating_points() -> Dict[int, float]:
    """{rank: tokens/s one GPU sustains through shrink + expand of a 4096 -> 4096 projection with every
    adapter at that rank}, measured with bench.py on the MI355X machine and kept in profiles/measured.json."""
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "measured.json")
    with open(path) as f:
        return {int(k): float(v) for k, v in json.load(f)["placement_operating_points_tokens_per_s"].items()}


def rank_shares(trace: str, rank_set: np.ndarray, t: int, steps: int) -> np.ndarray:
    """Share of the traffic each rank of rank_set (ascending) gets in step t of `steps`."""
    n = len(rank_set)
    if trace == "uniform":
        return np.full(n, 1.0 / n)
    if trace == "exponential":
        w = 0.5 ** np.arange(n)
        return w / w.sum()
    if trace == "shifting":
        f = t / max(1, steps - 1)                      # 0 at the start, 1 at the end
        start = np.full(n, 0.5 / (n - 1)) if n > 1 else np.ones(1)
        end = start.copy()
        if n > 1:
            start[-1], end[0] = 0.5, 0.5
        return (1.0 - f) * start + f * end
    raise ValueError(f"unknown trace {trace!r}")


def make_demand(trace: str, steps: int, ranks: np.ndarray, op: Dict[int, float], servers: int, load: float,
                noise: float, seed: int) -> np.ndarray:
    """[steps][adapters] tokens/s.  The total is scaled so that the ragged cost of step t is load * servers."""
    g = np.random.default_rng([seed, 77])
    rank_set = np.array(sorted(set(int(r) for r in ranks)))
    within = np.zeros(len(ranks))
    for r in rank_set:
        idx = np.nonzero(ranks == r)[0]
        w = 1.0 / (np.arange(len(idx)) + 1.0)           # power law, alpha = 1
        within[idx] = w / w.sum()
    per_token = np.array([1.0 / op[int(r)] for r in ranks])
    out = np.zeros((steps, len(ranks)))
    for t in range(steps):
        share = rank_shares(trace, rank_set, t, steps)
        d = within * np.array([share[np.searchsorted(rank_set, r)] for r in ranks])
        if noise > 0:
            d = d * np.exp(noise * g.standard_normal(len(ranks)))
        out[t] = d / (d * per_token).sum() * load * servers
    return out


def utilisation(phi: np.ndarray, ranks: np.ndarray, demand: np.ndarray, op: Dict[int, float], padded: bool) -> np.ndarray:
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
    n = len(ranks)
    phi = np.zeros((n, servers))
    if kind == "random":
        phi[np.arange(n), g.integers(0, servers, size=n)] = 1.0
    else:  # contiguous: sorted by rank, cut into equal runs
        order = np.argsort(ranks, kind="stable")
        for i, a in enumerate(order):
            phi[a, min(servers - 1, i * servers // n)] = 1.0
    return phi


def moved(phi: np.ndarray, prev: Optional[np.ndarray], ranks: np.ndarray):
    """(copies to fetch, the same weighted by rank): pairs the table has that the previous one had not."""
    if prev is None:
        return 0, 0.0
    new = (phi > 0) & ~(prev > 0)
    return int(new.sum()), float((new * ranks[:, None]).sum())


def native_engine():
    from . import binding as L
    return L.lora_place_extrapolate, lambda s, r, d, op, prev: L.lora_place_assign(s, r, d, op, prev)["phi"]


def simulate(trace: str, steps: int, servers: int, ranks: np.ndarray, op: Dict[int, float], load: float = 0.7,
             noise: float = 0.1, seed: int = 0, relabel: bool = True, engine: Optional[tuple] = None,
             demand: Optional[np.ndarray] = None) -> dict:
    """Runs the placement over `steps` time steps.  engine = (extrapolate(history, current) -> float,
    assign(servers, ranks, demand, op, prev_phi) -> phi); default: the native library."""
    extrapolate, assign = engine or native_engine()
    if demand is None:
        demand = make_demand(trace, steps, ranks, op, servers, load, noise, seed)
    n = len(ranks)
    rows, phi_prev = [], None
    for t in range(steps):
        if t == 0:
            projected = demand[0].copy()                # nothing observed yet: the first step's own demand
        else:
            projected = np.array([extrapolate(demand[:t - 1, a], demand[t - 1, a]) for a in range(n)])
        phi = np.asarray(assign(servers, ranks, projected, op, phi_prev if relabel else None))
        ur, up = utilisation(phi, ranks, demand[t], op, False), utilisation(phi, ranks, demand[t], op, True)
        copies, weight = moved(phi, phi_prev, ranks)
        rows.append({"step": t, "peak_util": float(ur.max()), "mean_util": float(ur.mean()), "peak_util_padded": float(up.max()),
                     "copies_moved": copies, "rank_weight_moved": weight, "copies_held": int((phi > 0).sum())})
        phi_prev = phi
    return {"trace": trace, "relabel": relabel, "steps": rows, "demand": demand}


def summary(res: dict) -> dict:
    r = res["steps"]
    return {"peak_util_max": max(x["peak_util"] for x in r), "peak_util_mean": float(np.mean([x["peak_util"] for x in r])),
            "peak_util_padded_mean": float(np.mean([x["peak_util_padded"] for x in r])),
            "copies_moved": int(sum(x["copies_moved"] for x in r)), "rank_weight_moved": float(sum(x["rank_weight_moved"] for x in r))}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--trace", choices=TRACES + ("all",), default="all")
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--servers", type=int, default=8)
    ap.add_argument("--adapters", type=int, default=100)
    ap.add_argument("--load", type=float, default=0.7, help="mean utilisation of the servers under the ragged cost model")
    ap.add_argument("--noise", type=float, default=0.1, help="sigma of the log-normal factor on every adapter's demand per step")
    ap.add_argument("--no-relabel", action="store_true", help="leave out step 5 (no previous table given)")
    ap.add_argument("--per-step", action="store_true", help="print every step, not only the summary")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    op = operating_points()
    g = np.random.default_rng(args.seed)
    rank_set = np.array(sorted(op))
    ranks = rank_set[g.permutation(args.adapters) % len(rank_set)].astype(np.int32)
    print(f"{args.servers} servers, {args.adapters} adapters, {args.steps} steps, load {args.load:.2f}, noise {args.noise:.2f}")
    print(f"{'trace':12s} {'placement':30s} {'peak util: mean / max':>22s} {'padded: mean peak':>18s} {'copies moved':>13s} {'rank-weighted':>14s}")
    for trace in (TRACES if args.trace == "all" else (args.trace,)):
        demand = make_demand(trace, args.steps, ranks, op, args.servers, args.load, args.noise, args.seed)
        runs = {"Algorithm 1, steps 1-5": simulate(trace, args.steps, args.servers, ranks, op, demand=demand, relabel=True)}
        if not args.no_relabel:
            runs["Algorithm 1 without step 5"] = simulate(trace, args.steps, args.servers, ranks, op, demand=demand, relabel=False)
        for name, res in runs.items():
            sm = summary(res)
            print(f"{trace:12s} {name:30s} {sm['peak_util_mean']:12.3f} / {sm['peak_util_max']:.3f} {sm['peak_util_padded_mean']:18.3f} "
                  f"{sm['copies_moved']:13d} {sm['rank_weight_moved']:14.0f}")
            if args.per_step:
                for x in res["steps"]:
                    print(f"    step {x['step']:3d}: peak {x['peak_util']:.3f} mean {x['mean_util']:.3f} padded peak "
                          f"{x['peak_util_padded']:.3f} moved {x['copies_moved']:3d} held {x['copies_held']}")
        for kind in ("random", "contiguous"):
            phi = static_placement(kind, args.servers, ranks, np.random.default_rng([args.seed, 5]))
            ur = np.array([utilisation(phi, ranks, demand[t], op, False).max() for t in range(args.steps)])
            up = np.array([utilisation(phi, ranks, demand[t], op, True).max() for t in range(args.steps)])
            print(f"{trace:12s} {'static, ' + kind:30s} {ur.mean():12.3f} / {ur.max():.3f} {up.mean():18.3f} {0:13d} {0:14.0f}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
