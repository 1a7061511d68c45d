"""Pins of the placement reference (oracle/placement_oracle.py) against what the paper's steps fix:
hand-worked cases, closed forms, invariants, brute force for the relabelling step."""
import itertools
import os

import numpy as np
import pytest

from oracle import placement_oracle as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "placement_hand_worked.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        head, ops, ads, phi = [f.strip() for f in line.split("|")]
        name, servers = head.split()
        op = {int(t.split(":")[0]): float(t.split(":")[1]) for t in ops.split()}
        ranks = [int(t.split(":")[0]) for t in ads.split()]
        demand = [float(t.split(":")[1]) for t in ads.split()]
        rows = np.array([[float(v) for v in row.split()] for row in phi.split(";")])
        out.append((name, int(servers), op, ranks, demand, rows))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c[0])
def test_hand_worked_placements(case):
    _, servers, op, ranks, demand, want = case
    got = P.assign(servers, ranks, demand, op)
    assert np.allclose(got["phi"], want, rtol=0, atol=1e-15)
    assert np.allclose(got["server_util"], 1.0) and got["target"] == pytest.approx(1.0)


def test_extrapolation_is_linear_and_not_negative():
    assert P.extrapolate([], 7.0) == 7.0
    assert P.extrapolate([3.0, 10.0], 14.0) == 18.0
    assert P.extrapolate([30.0], 10.0) == 0.0


def test_equal_adapters_of_one_rank_fill_every_server_to_the_target():
    servers, per = 5, 4
    ranks = [16] * (servers * per)
    demand = [25.0] * len(ranks)
    got = P.assign(servers, ranks, demand, {16: 200.0})
    assert got["budget"] == {16: servers} and got["target"] == pytest.approx(per * 25.0 / 200.0)
    assert np.allclose(got["server_util"], got["target"])
    assert np.all(got["server_max_rank"] == 16)
    assert np.array_equal((got["phi"] > 0).sum(axis=0), [per] * servers)      # nothing is split here


def _random_instance(seed, servers, n):
    g = np.random.default_rng(seed)
    rank_set = np.array([8, 16, 32, 64, 128])
    ranks = rank_set[g.integers(0, 5, size=n)]
    demand = g.zipf(1.5, size=n).astype(np.float64) * g.uniform(0.5, 1.5, size=n)
    demand[g.random(n) < 0.1] = 0.0
    op = {8: 1000.0, 16: 900.0, 32: 700.0, 64: 500.0, 128: 300.0}
    return ranks, demand, op


@pytest.mark.parametrize("seed,servers,n", [(0, 4, 40), (1, 7, 100), (2, 3, 9), (3, 12, 200), (4, 2, 5)])
def test_invariants_on_random_instances(seed, servers, n):
    ranks, demand, op = _random_instance(seed, servers, n)
    got = P.assign(servers, ranks, demand, op)
    phi = got["phi"]
    load = demand / np.array([op[int(r)] for r in ranks])
    assert np.all(phi >= 0) and np.allclose(phi.sum(axis=1), 1.0, atol=1e-12)          # every adapter fully routed
    assert np.allclose(phi.T @ load, got["server_util"], atol=1e-9)                     # utilisation adds up
    assert got["server_util"].sum() == pytest.approx(load.sum())
    assert got["target"] == pytest.approx(load.sum() / servers)
    for s in range(servers):
        on = phi[:, s] > 0
        assert got["server_max_rank"][s] == (ranks[on].max() if on.any() else 0)
    # step 2: the budget is the rounded share of each rank
    for r, b in got["budget"].items():
        share = load[ranks == r].sum() / got["target"]
        assert b == int(np.floor(share + 0.5))
    # step 3: an adapter is split over consecutive servers only, and only adapters with demand are split
    for a in range(n):
        used = np.nonzero(phi[a] > 0)[0]
        assert len(used) >= 1 and np.array_equal(used, np.arange(used[0], used[-1] + 1))
        if demand[a] == 0:
            assert len(used) == 1


def test_a_rank_without_budget_is_left_over_and_goes_where_it_adds_no_heterogeneity():
    # rank 64 asks for 1.9 servers' worth, rank 8 for 0.1: budgets 2 and 0
    op = {8: 100.0, 64: 100.0}
    ranks = [64, 64, 8, 8]
    demand = [100.0, 90.0, 6.0, 4.0]
    got = P.assign(2, ranks, demand, op)
    assert got["budget"] == {8: 0, 64: 2} and got["target"] == pytest.approx(1.0)
    # rank 64: adapter 0 fills server 0; adapter 1 (0.9) goes to server 1
    assert np.allclose(got["phi"][:2], [[1, 0], [0, 1]])
    # left over, by demand: adapter 2 to the less utilised server (1: 0.9), then adapter 3 to server 1 again (0.96 < 1.0)
    assert np.allclose(got["phi"][2:], [[0, 1], [0, 1]])
    assert np.allclose(got["server_util"], [1.0, 1.0])
    # a left-over adapter of a higher rank than any server serves: the server with the highest max rank
    got = P.assign(2, [8, 8, 8, 8, 128], [50.0, 50.0, 50.0, 50.0, 0.0], {8: 100.0, 128: 10.0})
    assert got["phi"][4].tolist() in ([1.0, 0.0], [0.0, 1.0]) and got["server_max_rank"].max() == 128


def test_relabelling_keeps_the_most_of_the_previous_assignment():
    ranks, demand, op = _random_instance(7, 5, 60)
    base = P.assign(5, ranks, demand, op)
    # the previous assignment is the same placement under other labels: relabelling must find it again
    shuffle = [3, 0, 4, 1, 2]
    prev = np.zeros_like(base["phi_unpermuted"])
    for i, lab in enumerate(shuffle):
        prev[:, lab] = base["phi_unpermuted"][:, i]
    got = P.assign(5, ranks, demand, op, prev_phi=prev)
    assert np.array_equal(got["phi"], prev)
    # the solver path (8 servers) against exhaustive search
    ranks, demand, op = _random_instance(8, 8, 90)
    new = P.assign(8, ranks, demand, op)["phi_unpermuted"]
    g = np.random.default_rng(1)
    prev = new[:, g.permutation(8)].copy()
    prev[g.random(prev.shape) < 0.2] = 0.0          # some adapters have moved away since
    perm = P.best_permutation(new, prev, ranks)
    best = max(P.kept_weight(new, prev, ranks, p) for p in itertools.permutations(range(8)))
    assert sorted(perm) == list(range(8)) and P.kept_weight(new, prev, ranks, perm) == best
