"""Host side of the C-ABI library, no GPU: the library loads and exports every symbol the header
declares, argument errors are reported before the device is touched, pool offsets follow the ragged
layout, and the planner's grouping and work units match a brute-force grouping."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_22880_amd import binding as L
from paper_2511_22880_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_ARENA = 0x7F0000000000  # 256-byte aligned address that is never dereferenced on the host


def make_pool(in_f=512, out_f=256, ranks=(8, 16, 3, 128), resident=True):
    ranks = np.asarray(ranks, dtype=np.int32)
    scales = (2.0 / np.maximum(ranks, 1)).astype(np.float32)
    n = L.lora_pool_bytes(in_f, out_f, ranks, scales)
    pool = L.lora_pool_create(in_f, out_f, ranks, scales, FAKE_ARENA, n)
    if resident:
        for a in range(len(ranks)):
            L.lora_pool_mark_resident(pool, a)
    return pool


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                     if h.endswith(".h"))
    declared = set(re.findall(r"\b(lora_[a-z_]+)\s*\(", header))
    assert declared == set(L.EXPORTS), declared ^ set(L.EXPORTS)
    lib = L.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert L.lora_status_string(0) == "LORA_OK" and L.lora_status_string(4) == "LORA_ERR_NOT_RESIDENT"


def test_pool_bytes_and_offsets_are_ragged():
    ranks = np.array([8, 16, 3, 128, 256], dtype=np.int32)
    in_f, out_f = 4096, 1024
    n = L.lora_pool_bytes(in_f, out_f, ranks, 2.0 / ranks)
    r8 = (ranks + 7) // 8 * 8
    assert n == int(2 * r8.sum() * (in_f + out_f))          # no padding to the largest rank
    assert n < 2 * 256 * len(ranks) * (in_f + out_f) / 2
    pool = L.lora_pool_create(in_f, out_f, ranks, 2.0 / ranks, FAKE_ARENA, n)
    off = 0
    for a, r in enumerate(ranks):
        info = L.lora_pool_adapter_info(pool, a)
        assert info["a_offset"] == off and info["b_offset"] == off + r8[a] * in_f
        assert info["rank"] == r and info["rank_padded"] == r8[a] and info["resident"] == 0
        assert info["scale"] == pytest.approx(2.0 / r)
        off += r8[a] * (in_f + out_f)
    L.lora_pool_destroy(pool)


@pytest.mark.parametrize("kwargs,status", [
    (dict(in_f=100), "LORA_ERR_SHAPE"),
    (dict(out_f=4097), "LORA_ERR_SHAPE"),
    (dict(ranks=(8, 0)), "LORA_ERR_SHAPE"),
    (dict(ranks=(8, 257)), "LORA_ERR_SHAPE"),
])
def test_pool_shape_errors(kwargs, status):
    with pytest.raises(L.LoraError) as e:
        make_pool(**kwargs)
    assert e.value.status_name == status and e.value.detail


def test_pool_argument_errors():
    ranks = np.array([8], dtype=np.int32)
    n = L.lora_pool_bytes(256, 256, ranks, [0.25])
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_create(256, 256, ranks, [0.25], FAKE_ARENA, n - 1)
    assert e.value.status_name == "LORA_ERR_OOM"
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_create(256, 256, ranks, [0.25], FAKE_ARENA + 8, n)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_create(256, 256, ranks, [0.25], 0, n)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    pool = make_pool()
    for bad in (-1, 4):
        with pytest.raises(L.LoraError) as e:
            L.lora_pool_evict(pool, bad)
        assert e.value.status_name == "LORA_ERR_INVALID_ARG"
        with pytest.raises(L.LoraError):
            L.lora_pool_adapter_info(pool, bad)
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_load(pool, 0, None, None, src_is_device=True)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    L.lora_pool_destroy(pool)


def test_plan_rejects_bad_routing_before_touching_the_device():
    pool = make_pool(resident=False)
    L.lora_pool_mark_resident(pool, 0)
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan(pool, [0, 1])
    assert e.value.status_name == "LORA_ERR_NOT_RESIDENT" and "adapter 1" in e.value.detail
    for bad in ([0, 4], [0, -2]):
        with pytest.raises(L.LoraError) as e:
            L.lora_segments_plan(pool, bad)
        assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    seg = L.lora_segments_plan(pool, [0, -1, 0])   # -1 is "no adapter", not an error
    assert L.lora_segments_info(seg)["n_active"] == 2
    L.lora_pool_evict(pool, 0)
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan(pool, [0])
    assert e.value.status_name == "LORA_ERR_NOT_RESIDENT"
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan_ranges(pool, [1, 2], [0])
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan_ranges(pool, [0, 5, 3], [-1, -1])
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_launch_checks_happen_on_the_host():
    pool = make_pool()
    seg = L.lora_segments_plan(pool, [0, 1, 3])
    # planned but never uploaded: refused, nothing is launched
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(pool, seg, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ldy=256, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "upload" in e.value.detail
    # evicting an adapter the batch does not use leaves the object alone (the refusal is still the missing upload)
    L.lora_pool_evict(pool, 2)
    with pytest.raises(L.LoraError) as e:
        L.lora_shrink(pool, seg, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "upload" in e.value.detail
    # evicting one it uses: not resident; declaring it resident again: another stamp, so the object is stale
    L.lora_pool_evict(pool, 1)
    with pytest.raises(L.LoraError) as e:
        L.lora_shrink(pool, seg, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_NOT_RESIDENT"
    L.lora_pool_mark_resident(pool, 1)
    with pytest.raises(L.LoraError) as e:
        L.lora_shrink(pool, seg, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    # a pool in which an adapter the batch uses has another rank (hence other places) is refused too
    other = make_pool(ranks=(8, 32, 3, 128))
    with pytest.raises(L.LoraError) as e:
        L.lora_expand(other, seg, FAKE_ARENA, FAKE_ARENA, ldy=256)
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    assert L.lora_apply_workspace_bytes(pool, seg) >= 4 * L.lora_segments_info(seg)["v_floats"]
    for o in (seg,):
        L.lora_segments_destroy(o)
    L.lora_pool_destroy(pool)
    L.lora_pool_destroy(other)


def brute_force_groups(ta):
    groups = {}
    for t, a in enumerate(ta):
        if a >= 0:
            groups.setdefault(int(a), []).append(t)
    return groups


@pytest.mark.parametrize("maker", [
    lambda: wl.cfg0_tiny(), lambda: wl.cfg1_decode(), lambda: wl.small_mixed(),
    lambda: wl.cfg4_skew(0, "9:1"), lambda: wl.cfg3_stack(length_scale=0.05), lambda: wl.cfg3_stack(length_scale=0.3),
    lambda: wl.cfg2_prefill(0, length_scale=0.1),
])
def test_planner_matches_brute_force_grouping(maker):
    b = maker()
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    seg = L.lora_segments_plan(pool, b.token_adapter)
    info, ex, units = L.lora_segments_info(seg), L.lora_segments_export(seg), L.lora_segments_export_units(seg)
    groups = brute_force_groups(b.token_adapter)
    r8 = (b.ranks + 7) // 8 * 8
    assert info["n_tokens"] == b.T and info["n_active"] == sum(len(g) for g in groups.values())
    assert info["n_segments"] == len(groups)
    assert list(ex["seg_adapter"]) == sorted(groups)
    # stable grouping: each group's tokens in batch order
    for s, a in enumerate(ex["seg_adapter"]):
        assert list(ex["perm"][ex["seg_start"][s]: ex["seg_start"][s + 1]]) == groups[int(a)]
    assert info["v_floats"] == sum(len(g) * int(r8[a]) for a, g in groups.items())
    assert info["weight_bytes"] == sum(2 * int(r8[a]) * (b.in_features + b.out_features) for a in groups)
    # v rows are disjoint and tile [0, v_floats)
    spans = sorted((int(ex["v_offset"][t]), int(r8[b.token_adapter[t]])) for t in range(b.T) if b.token_adapter[t] >= 0)
    pos = 0
    for off, ln in spans:
        assert off == pos
        pos += ln
    assert pos == info["v_floats"] and np.all(ex["v_offset"][b.token_adapter < 0] == -1)
    # shrink units cover every (token, rank row, k-slice) exactly once; expand units every (token, column)
    nsl = info["n_k_slices"]
    for s, a in enumerate(ex["seg_adapter"]):
        ntok, rr = len(groups[int(a)]), int(r8[a])
        token_heavy = ntok >= 32 and info["n_active"] >= 1024
        mine = units["shrink"][units["shrink"][:, 0] == s]
        # token tiles: all rank rows, and all of k or (launches of few such units) 2 or 4 slices of it
        cuts = int(mine[:, 5].max()) + 1 if token_heavy else nsl
        assert cuts in (1, 2, 4) and cuts <= max(nsl, 1)
        cover = np.zeros((ntok, rr, cuts), dtype=np.int32)
        for seg_i, tok0, nt, p0, pn, ks in mine:
            if token_heavy:
                assert 1 <= nt <= (32 if rr <= 64 else 64 if rr <= 128 else 16) and (p0, pn) == (0, rr) and 0 <= ks < cuts
                cover[tok0:tok0 + nt, :, ks] += 1
            else:
                assert 1 <= nt <= 16 and 1 <= pn <= 16
                cover[tok0:tok0 + nt, p0:p0 + pn, ks] += 1
        assert np.all(cover == 1)
        ecover = np.zeros((ntok, b.out_features), dtype=np.int32)
        for seg_i, tok0, nt, p0, pn, ks in units["expand"][units["expand"][:, 0] == s]:
            assert pn % 128 == 0 and 1 <= nt <= (64 if token_heavy else 16)
            ecover[tok0:tok0 + nt, p0:p0 + pn] += 1
        assert np.all(ecover == 1)
    # no unit's size depends on another adapter's rank: the bytes of B^T per unit are bounded by a
    # constant (one column pass of <= 64 KiB for small groups, four passes for token-heavy ones)
    eu = units["expand"]
    ub = eu[:, 4].astype(np.int64) * 2 * r8[ex["seg_adapter"][eu[:, 0]]]
    seg_tokens = np.diff(ex["seg_start"])[eu[:, 0]]
    heavy = (seg_tokens >= 32) & (info["n_active"] >= 1024)
    assert ub[~heavy].max(initial=0) <= 64 * 1024 and ub[heavy].max(initial=0) <= 256 * 1024
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_column_runs_of_64_token_expand_units_meet_few_xcds():
    """Work group b of a launch runs on XCD b mod 8.  The 64-token expand units of a group are listed
    in rows of 8 (each of the 4 column runs with 2 consecutive token tiles), so a column run of a
    group takes 2 of the 8 residues, whatever place the group starts at (a last row of 4 units, when
    the group has an odd number of token tiles, aside)."""
    b = wl.cfg2_prefill(0)
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    seg = L.lora_segments_plan(pool, b.token_adapter)
    ex, units = L.lora_segments_export(seg), L.lora_segments_export_units(seg)
    eu = units["expand"]
    ntok_of = np.diff(ex["seg_start"])[eu[:, 0]]
    big = eu[ntok_of >= 32]                  # every group of cfg2 is token-heavy and up to rank 128
    assert len(big) == len(eu) and big[:, 2].max() == 64
    ntiles = {int(s): (int(n) + 63) // 64 for s, n in enumerate(np.diff(ex["seg_start"]))}
    runs = {}
    for pos, (s, tok0, nt, p0, pn, ks) in enumerate(big):
        if ntiles[int(s)] % 2 and tok0 // 64 == ntiles[int(s)] - 1:
            continue                         # an odd tile count leaves a last row of 4 units
        runs.setdefault((int(s), int(p0)), set()).add(pos % 8)
    assert len({p0 for _, p0 in runs}) == 4
    assert max(len(r) for r in runs.values()) <= 2
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_token_heavy_units_are_cut_by_k_in_launches_of_few_units():
    """A mixed batch planned in k-slices: every 32-token tile of a token-heavy group gets 4 or 2 units
    (k-slices of the same rows) while the cut units stay at or below 320 (750 beyond 8192 input
    features), else one."""
    cases = ((wl.cfg3_stack(projection=6), 2), (wl.cfg3_stack(projection=0), 1), (wl.cfg2_prefill(2), 1),
             (wl.cfg3_stack(projection=0, length_scale=0.5), 2), (wl.cfg3_stack(projection=0, length_scale=0.25), 4),
             (wl.cfg3_stack(projection=6, length_scale=0.5), 4))
    for b, cuts in cases:
        n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
        pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
        for a in range(b.n_adapters):
            L.lora_pool_mark_resident(pool, a)
        seg = L.lora_segments_plan(pool, b.token_adapter)
        ex, units = L.lora_segments_export(seg), L.lora_segments_export_units(seg)
        sh = units["shrink"]
        assert np.all(sh[sh[:, 0] < 0][:, 2] == 0)              # places that only pad an XCD's list hold no tokens
        sh = sh[sh[:, 0] >= 0]
        heavy = sh[np.diff(ex["seg_start"])[sh[:, 0]] >= 32]
        tiles = {}
        for s_, tok0, nt, p0, pn, ks in heavy:
            tiles.setdefault((int(s_), int(tok0), int(nt), int(p0), int(pn)), []).append(int(ks))
        assert len(tiles) > 0
        limit = 750 if b.in_features > 8192 else 320
        assert len(tiles) * cuts <= limit or cuts == 1
        assert cuts == 4 or len(tiles) * cuts * 2 > limit
        for ks_list in tiles.values():
            assert sorted(ks_list) == list(range(cuts))
        L.lora_segments_destroy(seg)
        L.lora_pool_destroy(pool)


def test_whole_k_limit_switches_the_shrink_plan():
    b = wl.cfg1_decode()
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    got = {}
    L.lora_set_decode_single_launch(False)   # the two-launch plan; the one-launch form has a test of its own below
    try:
        for limit in (1024, 216, 0):
            L.lora_set_whole_k_limit(limit)
            seg = L.lora_segments_plan(pool, b.token_adapter)
            info = L.lora_segments_info(seg)
            got[limit] = (info["n_k_slices"], info["n_shrink_units"])
            L.lora_segments_destroy(seg)
        with pytest.raises(L.LoraError):
            L.lora_set_whole_k_limit(-1)
    finally:
        L.lora_set_whole_k_limit(1024)
        L.lora_set_decode_single_launch(True)
    # 217 whole-k units (16 rank rows x <= 16 tokens each) fit the default limit (32 of them, those of
    # 5 tokens and more, cut into two units of 8 rows: 249, within the 256 of one round); below it k is
    # cut in 4
    assert got[1024] == (1, 249) and got[216] == (4, 868) and got[0] == (4, 868)
    L.lora_pool_destroy(pool)


def test_whole_k_units_of_most_tokens_are_cut_into_row_halves():
    """In a whole-k plan of at most 256 units the 16-row units with the most tokens come as two units of
    8 rows on the same tokens (the same start of the row block in the pool, v offsets 8 apart), heaviest
    first, as many token counts as fit 256 units; the units still tile (token tile x rank rows) exactly."""
    for T in (256, 128, 64, 24):
        b = wl.cfg1_decode(n_tokens=T)
        n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
        pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
        for a in range(b.n_adapters):
            L.lora_pool_mark_resident(pool, a)
        L.lora_set_decode_single_launch(False)
        try:
            seg = L.lora_segments_plan(pool, b.token_adapter)
        finally:
            L.lora_set_decode_single_launch(True)
        info = L.lora_segments_info(seg)
        if info["n_k_slices"] != 1:
            L.lora_segments_destroy(seg)
            L.lora_pool_destroy(pool)
            continue
        u = L.lora_segments_export_units(seg)["shrink"]
        ex = L.lora_segments_export(seg)
        r8 = (b.ranks[ex["seg_adapter"]] + 7) // 8 * 8
        assert len(u) <= 256
        # exact tiling of every group's (tokens x padded rank rows)
        for si in range(info["n_segments"]):
            ntok = int(ex["seg_start"][si + 1] - ex["seg_start"][si])
            cover = np.zeros((ntok, int(r8[si])), dtype=np.int32)
            for seg_i, tok0, nt, p0, pn, ks in u[u[:, 0] == si]:
                cover[tok0:tok0 + nt, p0:p0 + pn] += 1
            assert (cover == 1).all()
        # halves: 8 rows inside a full 16-row block; the cut follows the token count
        in_full_block = (u[:, 4] == 8) & ((u[:, 3] % 16 == 8) | (r8[u[:, 0]] - u[:, 3] >= 16))
        whole = (u[:, 4] == 16)
        assert in_full_block.sum() % 2 == 0
        if in_full_block.any() and whole.any():
            assert u[in_full_block, 2].min() > u[whole, 2].max() - 1     # every cut unit has at least as many tokens as any whole one
            assert u[in_full_block, 2].min() >= u[whole, 2].max()
        uncut = len(u) - in_full_block.sum() // 2
        if whole.any():      # the next token count down would not have fitted
            m = int(u[whole, 2].max())
            assert len(u) + int((whole & (u[:, 2] == m)).sum()) > 256 or not in_full_block.any() and uncut > 256
        L.lora_segments_destroy(seg)
        L.lora_pool_destroy(pool)


def test_live_pool_places_frees_and_coalesces():
    """Space in a live pool: first fit, 256-byte granules, neighbours merge when freed."""
    in_f, out_f = 256, 256
    ranks = np.array([8, 16, 32, 8, 64, 16], dtype=np.int32)
    scales = (2.0 / ranks).astype(np.float32)
    size = lambda a: 2 * int((ranks[a] + 7) // 8 * 8) * (in_f + out_f)      # all multiples of 256 here
    arena = size(0) + size(1) + size(2) + size(3)                            # room for 0..3, not for 4
    pool = L.lora_pool_create_live(in_f, out_f, ranks, scales, FAKE_ARENA, arena)
    assert L.lora_pool_space(pool) == {"free_bytes": arena, "largest_free_bytes": arena}
    assert L.lora_pool_adapter_info(pool, 0)["a_offset"] == 2 ** 64 - 1     # no place yet
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_mark_resident(pool, 0)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    for a in (0, 1, 2, 3):
        L.lora_pool_reserve(pool, a)
        L.lora_pool_mark_resident(pool, a)
    offs = [L.lora_pool_adapter_info(pool, a)["a_offset"] * 2 for a in range(4)]
    assert offs == [0, size(0), size(0) + size(1), size(0) + size(1) + size(2)]
    info1 = L.lora_pool_adapter_info(pool, 1)
    assert info1["b_offset"] - info1["a_offset"] == 16 * in_f and info1["resident"] == 1
    assert L.lora_pool_space(pool) == {"free_bytes": 0, "largest_free_bytes": 0}
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_reserve(pool, 4)
    assert e.value.status_name == "LORA_ERR_OOM"
    # free 0 and 2: two separate pieces; 4 (rank 64) fits neither, and the message says compaction would not help
    L.lora_pool_evict(pool, 0)
    L.lora_pool_evict(pool, 2)
    assert L.lora_pool_space(pool) == {"free_bytes": size(0) + size(2), "largest_free_bytes": size(2)}
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_reserve(pool, 4)
    assert e.value.status_name == "LORA_ERR_OOM" and "compact" not in e.value.detail
    # free 1 as well: 0, 1, 2 merge into one piece, first fit puts 5 (rank 16) at the start
    L.lora_pool_evict(pool, 1)
    assert L.lora_pool_space(pool)["largest_free_bytes"] == size(0) + size(1) + size(2)
    L.lora_pool_reserve(pool, 5)
    assert L.lora_pool_adapter_info(pool, 5)["a_offset"] == 0
    # a segment object only depends on the adapters it uses
    seg = L.lora_segments_plan(pool, [3, 3, -1])
    L.lora_pool_mark_resident(pool, 5)
    L.lora_pool_evict(pool, 5)
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(pool, seg, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=in_f, ldy=out_f, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "upload" in e.value.detail
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan(pool, [5])
    assert e.value.status_name == "LORA_ERR_NOT_RESIDENT"
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_live_pool_reports_when_compaction_would_help():
    in_f, out_f = 256, 256
    ranks = np.array([8, 8, 8, 16], dtype=np.int32)
    scales = (2.0 / ranks).astype(np.float32)
    one = 2 * 8 * (in_f + out_f)
    pool = L.lora_pool_create_live(in_f, out_f, ranks, scales, FAKE_ARENA, 3 * one)
    for a in (0, 1, 2):
        L.lora_pool_reserve(pool, a)
    L.lora_pool_evict(pool, 0)
    L.lora_pool_evict(pool, 2)
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_reserve(pool, 3)            # 2 * one free in total, in two pieces
    assert e.value.status_name == "LORA_ERR_OOM" and "compact" in e.value.detail
    L.lora_pool_destroy(pool)


def test_multi_projection_plan_is_the_projections_plans_one_after_the_other():
    """q|k|v in one object: the unit lists of the three plans, expand columns shifted by the column base
    of each projection, v rows and counters of projection q after those of q - 1."""
    ranks = np.array([8, 16, 3, 128, 64], dtype=np.int32)
    scales = (2.0 / ranks).astype(np.float32)
    outs = (512, 128, 256)
    pools, addr = [], FAKE_ARENA
    for o in outs:
        n = L.lora_pool_bytes(512, o, ranks, scales)
        pools.append(L.lora_pool_create(512, o, ranks, scales, addr, n))
        addr += (n + 4095) // 4096 * 4096
        for a in range(len(ranks)):
            L.lora_pool_mark_resident(pools[-1], a)
    ta = np.array([0, 3, 3, -1, 4, 1, 3, 0, 2, 4, 4, 3] * 5, dtype=np.int32)
    multi = L.lora_segments_plan_multi(pools, ta)
    mi, mu = L.lora_segments_info(multi), L.lora_segments_export_units(multi)
    singles = [L.lora_segments_plan(p, ta) for p in pools]
    si = [L.lora_segments_info(s_) for s_ in singles]
    su = [L.lora_segments_export_units(s_) for s_ in singles]
    assert mi["v_floats"] == sum(i["v_floats"] for i in si) and mi["weight_bytes"] == sum(i["weight_bytes"] for i in si)
    assert mi["n_shrink_units"] == sum(i["n_shrink_units"] for i in si)
    assert mi["n_expand_units"] == sum(i["n_expand_units"] for i in si)
    assert np.array_equal(mu["shrink"], np.concatenate([u["shrink"] for u in su]))
    want, col = [], 0
    for u, o in zip(su, outs):
        e = u["expand"].copy()
        e[:, 3] += col              # first output column
        want.append(e)
        col += o
    assert np.array_equal(mu["expand"], np.concatenate(want))
    # the single-pool launch calls refuse such an object; pools that disagree in ranks cannot share one
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(pools[0], multi, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ldy=512, ws_bytes=1 << 20)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "lora_apply_multi" in e.value.detail
    with pytest.raises(L.LoraError) as e:
        L.lora_apply_multi(pools, multi, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ldy=sum(outs), ws_bytes=1 << 24)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "upload" in e.value.detail
    with pytest.raises(L.LoraError) as e:
        L.lora_apply_multi(pools[:2], multi, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ldy=sum(outs), ws_bytes=1 << 24)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    with pytest.raises(L.LoraError) as e:
        L.lora_apply_multi(pools[::-1], multi, FAKE_ARENA, FAKE_ARENA, FAKE_ARENA, ldx=512, ldy=sum(outs), ws_bytes=1 << 24)
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    other = make_pool(in_f=512, out_f=256, ranks=(8, 16, 3, 128, 32))
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan_multi([pools[0], other], ta)
    assert e.value.status_name == "LORA_ERR_SHAPE"
    for s_ in singles + [multi]:
        L.lora_segments_destroy(s_)
    for p_ in pools + [other]:
        L.lora_pool_destroy(p_)


def test_ranges_merge_requests_of_the_same_adapter():
    pool = make_pool()
    seg = L.lora_segments_plan_ranges(pool, [0, 3, 5, 9, 12], [1, -1, 0, 1])
    ex, info = L.lora_segments_export(seg), L.lora_segments_info(seg)
    assert info["n_tokens"] == 12 and info["n_active"] == 10 and info["n_segments"] == 2
    assert list(ex["seg_adapter"]) == [0, 1]
    assert list(ex["perm"]) == [5, 6, 7, 8, 0, 1, 2, 9, 10, 11]
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_empty_batches_plan():
    pool = make_pool()
    for ta in ([], [-1, -1, -1]):
        seg = L.lora_segments_plan(pool, np.asarray(ta, dtype=np.int32))
        info = L.lora_segments_info(seg)
        assert info["n_active"] == 0 and info["n_segments"] == 0 and info["v_floats"] == 0
        assert info["n_shrink_units"] == 0 and info["n_expand_units"] == 0
        L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_decode_shrink_units_of_a_group_share_an_xcd():
    """Launch order of the decode shrink units: work group b runs on XCD b mod 8, so a group's units
    (which all read the group's rows of x) are given places of one residue mod 8, the eight residues
    get the same number of units (a one-round launch stays one round) and about the same bytes."""
    b = wl.cfg1_decode()
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    seg = L.lora_segments_plan(pool, b.token_adapter)
    su = L.lora_segments_export_units(seg)["shrink"]
    res = np.arange(len(su)) % 8
    counts = np.bincount(res, minlength=8)
    assert counts.max() - counts.min() <= 1
    groups = np.unique(su[:, 0])
    together = sum(len(np.unique(res[su[:, 0] == g])) == 1 for g in groups)
    assert together >= 0.85 * len(groups)
    weight = (su[:, 2] + su[:, 4]).astype(np.int64)          # tokens + rank rows: bytes of x and A^T per k
    per_xcd = np.array([weight[res == q].sum() for q in range(8)])
    assert per_xcd.max() <= 1.15 * per_xcd.mean()
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_token_heavy_shrink_units_of_an_adapter_share_an_xcd_at_equal_cost():
    """Launch order of the token-heavy shrink units (cfg2): the tiles of one adapter on places of one
    residue mod 8 (one XCD fetches its A^T), the eight residues carrying the same bytes (tokens + rank
    rows of the units), the shorter lists padded at their end with places of no tokens."""
    b = wl.cfg2_prefill(0)
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    seg = L.lora_segments_plan(pool, b.token_adapter)
    ex, info = L.lora_segments_export(seg), L.lora_segments_info(seg)
    su = L.lora_segments_export_units(seg)["shrink"]
    count = np.diff(ex["seg_start"])
    n_small = int(np.sum((su[:, 0] >= 0) & (count[np.maximum(su[:, 0], 0)] < 32)))   # the small groups' units come first
    heavy = su[n_small:]
    assert len(heavy) % 8 == 0
    res = np.arange(len(heavy)) % 8
    real = heavy[:, 0] >= 0
    assert np.all(heavy[~real][:, 2] == 0) and np.all(heavy[real][:, 2] >= 1)
    for q in range(8):                                        # padding only at the end of a list
        mine = real[res == q]
        assert not np.any(mine[int(mine.sum()):])
    r8 = ((b.ranks + 7) // 8 * 8)[ex["seg_adapter"]]
    cost = np.where(real, heavy[:, 2] + heavy[:, 4], 0).astype(np.int64)       # rows of x + rows of A^T
    per_xcd = np.array([cost[res == q].sum() for q in range(8)])
    assert per_xcd.max() <= 1.03 * per_xcd.mean()
    groups = np.unique(heavy[real][:, 0])
    pairs = sum(len(np.unique(res[real & (heavy[:, 0] == g)])) for g in groups)
    assert pairs <= 1.35 * len(groups)                        # A^T fetched by 1.35 XCDs on average, not by 8
    tile = np.where(r8 <= 64, 32, 64)                       # tokens per unit: 64 above rank 64
    assert real.sum() == sum((c + t - 1) // t for c, t in zip(count, tile) if c >= 32)
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_token_heavy_units_above_rank_128():
    """Token-heavy groups above rank 128 are cut like the others: shrink units of 64 tokens up to rank 192
    and of 32 above, all rank rows each; expand units of up to 64 tokens (none of 16)."""
    ranks = np.array([160, 192, 256, 200, 8], dtype=np.int32)
    lens = [300, 260, 250, 130, 200]
    ta = np.concatenate([np.full(n, a, dtype=np.int32) for a, n in enumerate(lens)])
    pool = L.lora_pool_create(4096, 1024, ranks, (2.0 / ranks).astype(np.float32), FAKE_ARENA,
                              L.lora_pool_bytes(4096, 1024, ranks, (2.0 / ranks).astype(np.float32)))
    for a in range(len(ranks)):
        L.lora_pool_mark_resident(pool, a)
    seg = L.lora_segments_plan(pool, ta)
    ex = L.lora_segments_export(seg)
    units = L.lora_segments_export_units(seg)
    su = units["shrink"][units["shrink"][:, 0] >= 0]
    eu = units["expand"]
    rank_of = ranks[ex["seg_adapter"]]
    for g, r in enumerate(rank_of):
        n = lens[int(ex["seg_adapter"][g])]
        mine = su[su[:, 0] == g]
        tile = 32 if (r <= 64 or r > 192) else 64
        assert np.all(mine[:, 4] == (r + 7) // 8 * 8), (r, mine)
        slices = len(np.unique(mine[:, 5]))                   # a launch of few such units cuts each along k
        first = mine[mine[:, 5] == 0]
        assert len(mine) == slices * len(first)
        assert sorted(first[:, 1]) == list(range(0, n, tile)) and first[:, 2].sum() == n
        e = eu[eu[:, 0] == g]
        assert e[:, 2].max() > 16 and np.all(e[:, 2] <= 64)
        cols = np.unique(e[:, 3])
        assert sum(e[e[:, 3] == c][:, 2].sum() for c in cols) == n * len(cols)
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool)


def test_one_launch_decode_plan_keeps_every_tile_on_one_xcd():
    """The one-launch decode form hands v over through the L2 of one XCD, and work group b of a launch
    runs on the XCD of b mod 8: all units of a (group, token tile) sit at places of one residue mod 8.
    The shrink units (some cut into row halves) tile every group's (tokens x padded rank rows) exactly,
    the expand units its (tokens x columns); the launch is one round of at most 256 work groups."""
    cases = [wl.cfg1_decode(), wl.cfg1_decode(n_tokens=128), wl.cfg1_decode(in_features=2048, out_features=640, n_tokens=200),
             wl.cfg4_skew(0, "1:1", adapters_per_class=8), wl.cfg1_decode(n_tokens=300, n_adapters=40)]
    planned = 0
    for b in cases:
        n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
        pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
        for a in range(b.n_adapters):
            L.lora_pool_mark_resident(pool, a)
        seg = L.lora_segments_plan(pool, b.token_adapter)
        info = L.lora_segments_info(seg)
        if not info["single_launch"]:
            L.lora_segments_destroy(seg)
            L.lora_pool_destroy(pool)
            continue
        planned += 1
        g = info["launch_work_groups"]
        assert 8 <= g <= 256 and g % 8 == 0 and info["n_k_slices"] == 1
        lu = L.lora_segments_export_launch_units(seg)
        su, eu = lu["shrink"], lu["expand"]
        assert su.shape == (g, 7) and eu.shape == (4 * g, 7)
        ex = L.lora_segments_export(seg)
        r8 = (b.ranks[ex["seg_adapter"]] + 7) // 8 * 8
        xcd_of_tile = {}
        for place, u in enumerate(su):
            if u[2] > 0:
                assert xcd_of_tile.setdefault(int(u[6]), place % 8) == place % 8
        for place, u in enumerate(eu):
            if u[2] > 0:
                assert int(u[6]) in xcd_of_tile, "an expand unit reads a tile no shrink unit writes"
                assert xcd_of_tile[int(u[6])] == (place // 4) % 8
        for si in range(info["n_segments"]):
            ntok = int(ex["seg_start"][si + 1] - ex["seg_start"][si])
            cover = np.zeros((ntok, int(r8[si])), dtype=np.int32)
            for _s, tok0, nt, p0, pn, _ks, _t in su[(su[:, 0] == si) & (su[:, 2] > 0)]:
                assert pn in (8, 16) and tok0 % 16 == 0
                cover[tok0:tok0 + nt, p0:p0 + pn] += 1
            assert (cover == 1).all()
            cols = np.zeros((ntok, b.out_features), dtype=np.int32)
            for _s, tok0, nt, p0, pn, _ks, _t in eu[(eu[:, 0] == si) & (eu[:, 2] > 0)]:
                cols[tok0:tok0 + nt, p0:p0 + pn] += 1
            assert (cols == 1).all()
        L.lora_segments_destroy(seg)
        L.lora_pool_destroy(pool)
    assert planned >= 3


def test_plan_options_belong_to_the_object():
    """Settings given at planning stay with the segment object: two objects planned in one process with
    different settings differ, whatever the process-wide defaults are, and fields left at their default
    follow the lora_set_* value of the moment."""
    b = wl.cfg1_decode()
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
    for a in range(b.n_adapters):
        L.lora_pool_mark_resident(pool, a)
    plans = {}
    for name, opt in (("slices", L.plan_options(whole_k_limit=0)), ("two", L.plan_options(decode_single_launch=0)),
                      ("one", L.plan_options(decode_single_launch=1)), ("default", None)):
        seg = L.lora_segments_plan(pool, b.token_adapter, options=opt)
        plans[name] = L.lora_segments_info(seg)
        L.lora_segments_destroy(seg)
    assert plans["slices"]["n_k_slices"] == 4 and not plans["slices"]["single_launch"]
    assert plans["two"]["n_k_slices"] == 1 and not plans["two"]["single_launch"] and plans["two"]["n_shrink_units"] == 249
    assert plans["one"]["single_launch"] and plans["one"]["launch_work_groups"] == 256
    assert plans["default"]["single_launch"]
    L.lora_set_decode_single_launch(False)
    try:
        seg = L.lora_segments_plan(pool, b.token_adapter)
        assert not L.lora_segments_info(seg)["single_launch"]            # a default field follows the process-wide value
        L.lora_segments_destroy(seg)
        seg = L.lora_segments_plan(pool, b.token_adapter, options=L.plan_options(decode_single_launch=1))
        assert L.lora_segments_info(seg)["single_launch"]                # an explicit field does not
        L.lora_segments_destroy(seg)
    finally:
        L.lora_set_decode_single_launch(True)
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_plan(pool, b.token_adapter, options=L.plan_options(merged_launches=5))
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    L.lora_pool_destroy(pool)


def test_planner_thresholds_can_be_moved_per_object():
    """The size thresholds of the planner are fields of lora_plan_options_t: a batch can be planned on
    either side of each (what bench.py --plan does); -1 keeps the built-in value, anything below is refused."""
    def plan(b, **kw):
        n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
        pool = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, FAKE_ARENA, n)
        for a in range(b.n_adapters):
            L.lora_pool_mark_resident(pool, a)
        seg = L.lora_segments_plan(pool, b.token_adapter, options=L.plan_options(**kw) if kw else None)
        info, units = L.lora_segments_info(seg), L.lora_segments_export_units(seg)
        L.lora_segments_destroy(seg)
        L.lora_pool_destroy(pool)
        return info, units
    # in_features beyond the built-in limit of the whole-k plan: k-slices, unless the limit is raised
    b = wl.cfg1_decode(in_features=18496, out_features=512)
    assert plan(b)[0]["n_k_slices"] > 1 and plan(b, whole_k_max_in=32768)[0]["n_k_slices"] == 1
    b = wl.cfg1_decode(in_features=18432, out_features=512)
    assert plan(b)[0]["n_k_slices"] == 1 and plan(b, whole_k_max_in=4096)[0]["n_k_slices"] > 1
    # a 40-token group in a batch of 1000 tokens is cut like the small groups, unless the batch size that
    # makes groups token-heavy is lowered; in a batch of 1030 it is token-heavy, unless that size is raised
    for extra, kw in ((960, {"heavy_min_batch": 1000}), (990, {"heavy_min_batch": 100000})):
        b = wl.groups_batch(256, 256, [(1, 40, 64), (extra, 1, 0)])
        base, moved = plan(b)[1]["shrink"], plan(b, **kw)[1]["shrink"]
        big = lambda u: int((u[:, 2] > 16).sum())
        assert (big(base) > 0) == (extra == 990) and (big(moved) > 0) == (extra == 960)
    # groups of 31 tokens become token-heavy when the token threshold is lowered
    b = wl.groups_batch(256, 256, [(40, 31, 64), (800, 1, 0)])
    assert int((plan(b)[1]["shrink"][:, 2] > 16).sum()) == 0
    assert int((plan(b, heavy_min_tokens=31)[1]["shrink"][:, 2] > 16).sum()) == 40
    # 64-token expand units: 8 column runs within one round of work groups (512 units), else 4
    b = wl.groups_batch(256, 4096, [(4, 1024, 32)])
    assert len(plan(b)[1]["expand"]) == 64 * 8 and len(plan(b, big_runs_max_units=511)[1]["expand"]) == 64 * 4
    b = wl.groups_batch(256, 4096, [(5, 832, 32)])
    assert len(plan(b)[1]["expand"]) == 65 * 4 and len(plan(b, big_runs_max_units=520)[1]["expand"]) == 65 * 8
    with pytest.raises(L.LoraError):
        plan(b, heavy_k_cut_max_units=-2)
    with pytest.raises(L.LoraError):
        plan(b, heavy_min_tokens=0)


def test_handles_that_outlive_their_pool_are_refused():
    ranks = np.array([8, 64], dtype=np.int32)
    scales = (2.0 / ranks).astype(np.float32)
    n = L.lora_pool_bytes(512, 256, ranks, scales)
    pool = L.lora_pool_create(512, 256, ranks, scales, FAKE_ARENA, n)
    for a in range(2):
        L.lora_pool_mark_resident(pool, a)
    ta = np.array([0, 1, 1, -1], dtype=np.int32)
    seg = L.lora_segments_plan(pool, ta)
    assert L.lora_segments_table_bytes(seg) > 0 and L.lora_segments_table_bytes(seg) % 256 == 0
    handle = pool.handle.value
    L.lora_pool_destroy(pool)
    pool.handle = ctypes.c_void_p(handle)          # the stale handle, as a careless caller would keep it
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_rebuild(seg, ta)
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    with pytest.raises(L.LoraError) as e:
        L.lora_apply_workspace_bytes(pool, seg)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_adapter_info(pool, 0)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG"
    pool.handle = ctypes.c_void_p(None)
    L.lora_segments_destroy(seg)


def test_bench_reads_its_profiler_figures_from_the_data_file():
    """bench.py carries no profiler figure of its own: HBM traffic per launch, the read ceiling and the
    placement simulator's operating points come from profiles/measured.json, and the summaries beside
    it quote the same traffic figures."""
    import glob
    import importlib.util
    import json
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    with open(os.path.join(root, "profiles", "measured.json")) as f:
        data = json.load(f)
    assert bench.load_measured() == data
    assert data["read_ceiling_GBps"] > 0 and data["traffic_bytes"] and data["phase_kernels"]
    src = open(os.path.join(root, "bench.py")).read()
    assert "MEASURED_TRAFFIC" not in src and "28.49e6" not in src
    summaries = "".join(open(p).read() for p in glob.glob(os.path.join(root, "profiles", "*.md")))
    for key, nbytes in data["traffic_bytes"].items():
        assert f"{nbytes / 1e6:.2f}" in summaries or f"{nbytes / 1e6:.1f}" in summaries, f"{key}: {nbytes} is not quoted in profiles/*.md"
    from paper_2511_22880_amd import placement_sim
    ops = placement_sim.operating_points()
    assert ops == {int(k): v for k, v in data["placement_operating_points_tokens_per_s"].items()}
