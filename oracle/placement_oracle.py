"""Plain reference of the paper's adapter placement (System Design, "Adapter Placement and Request
Routing", Algorithm 1), steps 1-5, in the paper's order and names.  Test infrastructure: only tests
may import it; the native library shares no code with it.

Where the listing leaves a step open, the reading taken (the same ones the native library documents):
  R1 extrapolate: linear through the last recorded value and the current one, not below zero.
  R2 round: half away from zero (floor(x + 0.5)).
  R3 ranks are served in descending order; servers are handed out consecutively; a rank whose budget
     no longer fits gets the servers that are left.
  R4 fractionalBinPacking: the rank's adapters by descending demand (ties by id) fill the rank's
     servers one after the other up to targetUtil each; an adapter that does not fit the current
     server continues on the next (that is the fraction); what still remains of a started adapter
     after the rank's last server stays on that last server; adapters not started, and adapters with
     no demand, are left over.
  R5 allocateHighestMaxRank: left-over adapters by descending rank (ties: demand descending, id);
     servers that are empty or already serve a rank at least as high take the adapter without getting
     more heterogeneous: among them the least utilised wins (ties: higher max rank, lower id); if
     there is none, the server with the highest max rank (ties: least utilised, lower id).
  R6 permuteAssignment: servers are relabelled so that the rank-weighted number of (adapter, server)
     pairs kept from the previous assignment is largest (an assignment problem).
"""
from __future__ import annotations

import itertools
import math
from typing import Dict, List, Optional, Sequence

import numpy as np

EPS = 1e-12


def extrapolate(history: Sequence[float], current: float) -> float:
    """Step 1, per adapter: projected tokens/s of the next time step (R1)."""
    if len(history) == 0:
        return max(0.0, float(current))
    return max(0.0, float(current) + (float(current) - float(history[-1])))


def target_utilisation(ranks, demand, op: Dict[int, float], n_servers: int):
    """Step 1: utilisation each rank asks for, and the average per server."""
    rank_util: Dict[int, float] = {}
    for r in sorted(set(int(x) for x in ranks)):
        rank_util[r] = sum(float(d) for x, d in zip(ranks, demand) if int(x) == r) / op[r]
    return rank_util, sum(rank_util.values()) / n_servers


def server_budget(rank_util: Dict[int, float], target: float) -> Dict[int, int]:
    """Step 2: servers that can be dedicated to each rank (R2)."""
    return {r: (int(math.floor(u / target + 0.5)) if target > 0 else 0) for r, u in rank_util.items()}


def assign(n_servers: int, ranks, demand, op: Dict[int, float], prev_phi: Optional[np.ndarray] = None,
           step4: str = "fits"):
    """-> dict(phi [n_adapters][n_servers], server_util, server_max_rank, budget, target, phi_unpermuted).
    step4 = "fits" is reading R5; "literal" takes the listing's comment word for word (the server with the
    highest max rank, the least utilised among those), kept for the comparison in the tests."""
    ranks = [int(r) for r in ranks]
    demand = [float(d) for d in demand]
    n = len(ranks)
    rank_util, target = target_utilisation(ranks, demand, op, n_servers)
    budget = server_budget(rank_util, target)
    phi = np.zeros((n, n_servers))
    util = [0.0] * n_servers
    max_rank = [0] * n_servers
    started = [False] * n

    # Step 3: fractional bin packing per rank with a budget (R3, R4)
    next_server = 0
    for r in sorted(budget, reverse=True):
        bins = list(range(next_server, min(n_servers, next_server + budget[r])))
        next_server += len(bins)
        if not bins:
            continue
        order = sorted((a for a in range(n) if ranks[a] == r and demand[a] > 0), key=lambda a: (-demand[a], a))
        b = 0
        for a in order:
            if b >= len(bins):
                break
            load = demand[a] / op[r]
            left = load
            started[a] = True
            while left > EPS * max(1.0, load) and b < len(bins):
                s = bins[b]
                room = target - util[s]
                take = min(left, room)
                if take > 0:
                    phi[a, s] += take / load
                    util[s] += take
                    max_rank[s] = max(max_rank[s], r)
                    left -= take
                if util[s] >= target - EPS * max(1.0, target):
                    b += 1
            if left > EPS * max(1.0, load):     # the rank's servers are full: the rest stays on the last one
                s = bins[-1]
                phi[a, s] += left / load
                util[s] += left
            phi[a] /= phi[a].sum()

    # Step 4: left-over adapters, highest rank first (R5)
    leftovers = sorted((a for a in range(n) if not started[a]), key=lambda a: (-ranks[a], -demand[a], a))
    for a in leftovers:
        r = ranks[a]
        fits = [s for s in range(n_servers) if max_rank[s] == 0 or max_rank[s] >= r]
        if step4 == "literal":
            fits = []
        if fits:
            s = min(fits, key=lambda s: (util[s], -max_rank[s], s))
        else:
            s = min(range(n_servers), key=lambda s: (-max_rank[s], util[s], s))
        phi[a, s] = 1.0
        util[s] += demand[a] / op[r]
        max_rank[s] = max(max_rank[s], r)

    unpermuted = phi.copy()
    perm = list(range(n_servers))
    if prev_phi is not None:
        perm = best_permutation(phi, np.asarray(prev_phi), ranks)
        # new server i takes the label perm[i]
        out = np.zeros_like(phi)
        u2, m2 = [0.0] * n_servers, [0] * n_servers
        for i, lab in enumerate(perm):
            out[:, lab] = phi[:, i]
            u2[lab], m2[lab] = util[i], max_rank[i]
        phi, util, max_rank = out, u2, m2
    return {"phi": phi, "server_util": np.array(util), "server_max_rank": np.array(max_rank), "budget": budget,
            "target": target, "phi_unpermuted": unpermuted, "perm": perm}


def kept_weight(phi_new: np.ndarray, phi_prev: np.ndarray, ranks, perm) -> float:
    """Rank-weighted count of (adapter, server) pairs that stay where they were when new server i is
    given the label perm[i]."""
    total = 0.0
    for i, lab in enumerate(perm):
        both = (phi_new[:, i] > 0) & (phi_prev[:, lab] > 0)
        total += float(np.asarray(ranks, dtype=np.float64)[both].sum())
    return total


def best_permutation(phi_new, phi_prev, ranks) -> List[int]:
    """Step 5 (R6), by exhaustive search up to 7 servers, else the library assignment solver."""
    s = phi_new.shape[1]
    if s <= 7:
        return list(max(itertools.permutations(range(s)), key=lambda p: (kept_weight(phi_new, phi_prev, ranks, p),
                                                                           tuple(-x for x in p))))
    from scipy.optimize import linear_sum_assignment
    w = np.asarray(ranks, dtype=np.float64)
    overlap = ((phi_new > 0).T.astype(np.float64) * w) @ (phi_prev > 0).astype(np.float64)
    rows, cols = linear_sum_assignment(-overlap)
    perm = [0] * s
    for i, j in zip(rows, cols):
        perm[i] = int(j)
    return perm
