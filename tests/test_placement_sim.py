"""The time-stepped placement simulator (host only): its demand shapes, the pins of Algorithm 1's steps 1
and 5 over time, the native routine against the plain reference step by step, and what reading R5 of
step 4 buys over the listing's comment taken word for word."""
import numpy as np
import pytest

from oracle import placement_oracle as P
from paper_2511_22880_amd import binding as L
from paper_2511_22880_amd import placement_sim as S

OP = {8: 5000.0, 16: 4600.0, 32: 3900.0, 64: 3000.0, 128: 2000.0}


def _ranks(n, seed=0):
    g = np.random.default_rng(seed)
    rs = np.array(sorted(OP))
    return rs[g.permutation(n) % len(rs)].astype(np.int32)


def test_rank_shares_of_the_three_traces():
    rs = np.array([8, 16, 32, 64, 128])
    for trace in S.TRACES:
        for t in (0, 5, 11):
            sh = S.rank_shares(trace, rs, t, 12)
            assert abs(sh.sum() - 1.0) < 1e-12 and (sh > 0).all()
    assert np.allclose(S.rank_shares("uniform", rs, 3, 12), 0.2)
    first, last = S.rank_shares("shifting", rs, 0, 12), S.rank_shares("shifting", rs, 11, 12)
    assert first[-1] == 0.5 and np.allclose(first[:-1], 0.125)      # rank 128 has half the traffic at the start
    assert last[0] == 0.5 and np.allclose(last[1:], 0.125)          # rank 8 at the end
    mid = S.rank_shares("shifting", rs, 11, 23)                       # half-way: linear in between
    assert np.allclose(mid, 0.5 * (first + last))
    ex = S.rank_shares("exponential", rs, 0, 12)
    assert np.allclose(ex[:-1] / ex[1:], 2.0)                         # smaller ranks more popular


def test_demand_has_the_load_it_was_asked_for():
    ranks = _ranks(40)
    d = S.make_demand("shifting", 10, ranks, OP, servers=4, load=0.6, noise=0.2, seed=3)
    cost = (d / np.array([OP[int(r)] for r in ranks])).sum(axis=1)
    assert np.allclose(cost, 0.6 * 4) and (d >= 0).all()
    assert np.array_equal(d, S.make_demand("shifting", 10, ranks, OP, 4, 0.6, 0.2, 3))    # seeded


@pytest.mark.parametrize("trace", ["uniform", "exponential"])
def test_stationary_demand_moves_nothing_after_the_first_step(trace):
    """Step 1's projection of a constant series is that constant, the packing is deterministic, and
    step 5 finds the identity: no adapter is fetched anywhere from the second step on."""
    ranks = _ranks(60)
    for relabel in (True, False):
        res = S.simulate(trace, 8, 6, ranks, OP, noise=0.0, relabel=relabel)
        assert [x["copies_moved"] for x in res["steps"]] == [0] * 8
        peaks = [x["peak_util"] for x in res["steps"]]
        assert max(peaks) - min(peaks) < 1e-12


def test_a_relabelled_previous_table_moves_nothing():
    """If the previous table is the new placement with the servers renamed, step 5 renames them back."""
    ranks = _ranks(50, seed=2)
    g = np.random.default_rng(5)
    demand = g.uniform(0.0, 800.0, size=50)
    phi = L.lora_place_assign(7, ranks, demand, OP)["phi"]
    perm = g.permutation(7)
    prev = phi[:, perm]
    again = L.lora_place_assign(7, ranks, demand, OP, prev_phi=prev)["phi"]
    assert S.moved(again, prev, ranks) == (0, 0.0)
    assert np.allclose(again, prev)
    # without the previous table the same demand lands on other server names: that is what step 5 is for
    assert S.moved(phi, prev, ranks)[0] > 0


def test_relabelling_only_renames_servers():
    """Step 5 changes which server is which, not the load: same utilisation profile with and without it."""
    ranks = _ranks(60, seed=4)
    demand = S.make_demand("shifting", 12, ranks, OP, 6, 0.7, 0.15, 1)
    a = S.simulate("shifting", 12, 6, ranks, OP, demand=demand, relabel=True)
    b = S.simulate("shifting", 12, 6, ranks, OP, demand=demand, relabel=False)
    assert np.allclose([x["peak_util"] for x in a["steps"]], [x["peak_util"] for x in b["steps"]])
    assert sum(x["rank_weight_moved"] for x in a["steps"]) <= sum(x["rank_weight_moved"] for x in b["steps"])


@pytest.mark.parametrize("trace", S.TRACES)
def test_native_routine_follows_the_reference_over_time(trace):
    """lora_place_extrapolate + lora_place_assign(prev_phi) against the plain reference, driven over a
    drifting demand: same utilisation in every step, the same rank-weighted number of copies moved
    (relabellings can tie, so the tables themselves may name tied servers differently)."""
    ranks = _ranks(45, seed=7)
    demand = S.make_demand(trace, 10, ranks, OP, 5, 0.7, 0.2, 11)
    ref_engine = (P.extrapolate, lambda s, r, d, op, prev: P.assign(s, r, d, op, prev)["phi"])
    nat = S.simulate(trace, 10, 5, ranks, OP, demand=demand)
    ref = S.simulate(trace, 10, 5, ranks, OP, demand=demand, engine=ref_engine)
    for x, y in zip(nat["steps"], ref["steps"]):
        assert abs(x["peak_util"] - y["peak_util"]) < 1e-9 and abs(x["peak_util_padded"] - y["peak_util_padded"]) < 1e-9
        assert x["copies_held"] == y["copies_held"]
    # step 0 and 1 have no tie history; later steps may differ by tied relabellings only through the weight kept
    assert nat["steps"][1]["rank_weight_moved"] == ref["steps"][1]["rank_weight_moved"]


def test_step_four_reading_against_the_listing_comment_word_for_word():
    """Left-over adapters go to the least utilised server that is empty or already serves a rank at least
    as high (R5).  Word for word, the listing's comment sends them to the servers with the highest max
    rank, whatever their load.  On demands with many left-overs (adapters without projected demand, ranks
    without budget) R5 never makes a server more heterogeneous than it was either, and keeps the peak
    utilisation lower."""
    g = np.random.default_rng(9)
    worse, total = 0, 0
    for _ in range(40):
        n, servers = int(g.integers(20, 80)), int(g.integers(3, 9))
        ranks = _ranks(n, seed=int(g.integers(0, 1000)))
        demand = g.uniform(0.0, 600.0, size=n) * (g.uniform(size=n) < 0.6)       # 40 % of the adapters idle in the projection
        a, b = P.assign(servers, ranks, demand, OP), P.assign(servers, ranks, demand, OP, step4="literal")
        true_demand = np.where(demand > 0, demand, 120.0)                          # the idle ones wake up
        ua = S.utilisation(a["phi"], ranks, true_demand, OP, False).max()
        ub = S.utilisation(b["phi"], ranks, true_demand, OP, False).max()
        total += 1
        worse += ua > ub + 1e-12
        assert np.allclose(a["phi"].sum(axis=1), 1.0) and np.allclose(b["phi"].sum(axis=1), 1.0)
    assert worse <= total // 10, f"R5 gave the higher peak in {worse} of {total} instances"
