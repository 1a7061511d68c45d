"""The native placement routine (include/lora_placement.h) against the reference in oracle/: the same
routing table before relabelling, an equally good relabelling, the same budgets and target."""
import numpy as np
import pytest

from oracle import placement_oracle as P
from paper_2511_22880_amd import binding as L

OP = {8: 1000.0, 16: 900.0, 32: 700.0, 64: 500.0, 128: 300.0}


def _instance(seed, n):
    g = np.random.default_rng(seed)
    ranks = np.array([8, 16, 32, 64, 128])[g.integers(0, 5, size=n)].astype(np.int32)
    demand = g.zipf(1.4, size=n).astype(np.float64) * g.uniform(0.5, 1.5, size=n)
    demand[g.random(n) < 0.1] = 0.0
    return ranks, demand


@pytest.mark.parametrize("seed,servers,n", [(0, 4, 40), (1, 7, 100), (2, 3, 9), (3, 12, 200), (4, 2, 5), (5, 1, 3),
                                            (6, 16, 1000), (7, 5, 0)])
def test_native_placement_equals_the_reference(seed, servers, n):
    ranks, demand = _instance(seed, n)
    want = P.assign(servers, ranks, demand, OP)
    got = L.lora_place_assign(servers, ranks, demand, OP)
    assert np.allclose(got["phi"], want["phi"], rtol=0, atol=1e-12)
    assert np.allclose(got["server_util"], want["server_util"], rtol=1e-12, atol=1e-12)
    assert np.array_equal(got["server_max_rank"], want["server_max_rank"])
    assert got["target"] == pytest.approx(want["target"], rel=1e-13)
    for r, b in want["budget"].items():
        assert got["budget"][r] == b


@pytest.mark.parametrize("seed,servers,n", [(10, 4, 30), (11, 6, 80), (12, 9, 150), (13, 16, 400)])
def test_native_relabelling_keeps_as_much_as_the_reference(seed, servers, n):
    ranks, demand = _instance(seed, n)
    g = np.random.default_rng(seed)
    base = P.assign(servers, ranks, demand, OP)["phi_unpermuted"]
    prev = base[:, g.permutation(servers)].copy()
    prev[g.random(prev.shape) < 0.15] = 0.0
    want = P.assign(servers, ranks, demand, OP, prev_phi=prev)
    got = L.lora_place_assign(servers, ranks, demand, OP, prev_phi=prev)
    # several relabellings can be equally good: compare what is unique (the kept weight) and check that
    # the table is the unpermuted one with its columns renamed
    kept = lambda phi: float((np.asarray(ranks, dtype=np.float64)[:, None] * ((phi > 0) & (prev > 0))).sum())
    assert kept(got["phi"]) == kept(want["phi"])
    cols = sorted(map(tuple, np.round(got["phi"].T, 12)))
    assert cols == sorted(map(tuple, np.round(base.T, 12)))
    assert np.allclose(got["phi"].T @ (demand / np.array([OP[int(r)] for r in ranks])), got["server_util"], atol=1e-9)


def test_native_extrapolation_and_errors():
    assert L.lora_place_extrapolate([], 7.0) == 7.0
    assert L.lora_place_extrapolate([3.0, 10.0], 14.0) == 18.0
    assert L.lora_place_extrapolate([30.0], 10.0) == 0.0
    with pytest.raises(L.LoraError):
        L.lora_place_assign(2, [8, 24], [1.0, 1.0], OP)            # rank 24 has no operating point
    with pytest.raises(L.LoraError):
        L.lora_place_assign(0, [8], [1.0], OP)
    with pytest.raises(L.LoraError):
        L.lora_place_assign(2, [8], [-1.0], OP)


def test_what_if_script_balances_better_than_the_static_placements():
    """The demonstration script's numbers: under the ragged cost model every placement carries the
    same total utilisation, and the rank-aware one has the lowest peak on skewed popularity."""
    from paper_2511_22880_amd import placement_sim as S
    op = S.operating_points()
    for seed in (0, 1, 2):
        g = np.random.default_rng(seed)
        servers, n = 8, 200
        ranks = np.array(sorted(op))[g.permutation(n) % 5].astype(np.int32)
        pop = ((np.arange(n) + 1.0) ** -1.1)[g.permutation(n)]
        per_token = np.array([1.0 / op[int(r)] for r in ranks])
        demand = pop / (pop * per_token).sum() * 0.7 * servers
        ours = L.lora_place_assign(servers, ranks, demand, op)["phi"]
        peaks = {}
        for name, phi in (("ours", ours), ("random", S.static_placement("random", servers, ranks, g)),
                          ("contiguous", S.static_placement("contiguous", servers, ranks, g))):
            u = S.utilisation(phi, ranks, demand, op, padded=False)
            assert u.sum() == pytest.approx(0.7 * servers)
            peaks[name] = u.max()
        assert peaks["ours"] < peaks["random"] and peaks["ours"] < peaks["contiguous"]
