"""GPU parity: the HIP path (through the C-ABI) against the fp64 CPU oracle on the same seeded bf16
inputs.  Bar: max per-row relative L2 error <= 5e-3 on rows with an adapter (y0 = 0, so the error is
measured on the delta itself); rows without an adapter bitwise untouched."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_22880_amd import binding as L
from paper_2511_22880_amd import workloads as wl

import gpu_util as G

pytestmark = pytest.mark.gpu


def _full_parity(batch, y0_kind="zero", ranges=None, tol=G.TOL):
    print(f"[case] {batch.name} T={batch.T} in={batch.in_features} out={batch.out_features} y0={y0_kind}", flush=True)
    dp = G.DevicePool(batch)
    x_bits, y0_bits = batch.x_bits(), batch.y0_bits(y0_kind)
    y_bits = G.apply_on_gpu(dp, x_bits, y0_bits, ranges=ranges)
    y_ref = G.oracle_apply(dp, x_bits, y0_bits)
    worst = G.check_parity(y_bits, y_ref, y0_bits, batch.token_adapter, tol=tol)
    n, _w, worst_el = G.check_all_rows(dp, x_bits, y0_bits, y_bits, token_adapter=batch.token_adapter, tol=tol)
    dp.close()
    print(f"[ok] {batch.name}: {n} rows, max row rel-L2 {worst:.3e}, max element error / bound {worst_el:.3f}", flush=True)
    return worst


def test_cfg0_tiny():
    _full_parity(wl.cfg0_tiny())


def test_cfg0_tiny_accumulates_into_small_y0():
    _full_parity(wl.cfg0_tiny(), y0_kind="small")


def test_small_mixed_ragged():
    """Odd ranks (1, 3, 12, 100 ...), tokens without adapter, prefill runs of awkward lengths and
    scattered decode tokens: several token tiles, row tiles and column tiles plus ragged tails."""
    _full_parity(wl.small_mixed())
    _full_parity(wl.small_mixed(seed=3, in_features=1280, out_features=640), y0_kind="small")


def test_decode_batches_up_to_the_widest_whole_k_plan():
    """Decode co-batches whose units take the whole of k up to 18,432 input features (the one-launch form
    and the two launches), and just beyond, where the planner goes to k-slices."""
    for in_f in (14336, 18432, 18496):
        b = wl.cfg1_decode(in_features=in_f, out_features=512, n_tokens=200)
        dp = G.DevicePool(b)
        seg = L.lora_segments_plan(dp.pool, b.token_adapter)
        assert (L.lora_segments_info(seg)["n_k_slices"] == 1) == (in_f <= 18432)
        L.lora_segments_destroy(seg)
        dp.close()
        _full_parity(b)
        L.lora_set_decode_single_launch(False)
        try:
            _full_parity(b, y0_kind="small")
        finally:
            L.lora_set_decode_single_launch(True)


def test_padded_control_pool():
    """The control layout (every adapter stored zero-padded at the largest rank, what a kernel sized to
    the largest rank needs) goes through the same entry points and gives the same rows."""
    for b in (wl.small_mixed(), wl.cfg4_skew(0, "1:1", adapters_per_class=2)):
        print(f"[case] padded pool {b.name} T={b.T}", flush=True)
        dp = G.DevicePool(b, padded=True)
        x_bits, y0_bits = b.x_bits(), b.y0_bits("zero")
        y_bits = G.apply_on_gpu(dp, x_bits, y0_bits)
        rows = np.arange(0, b.T, 4, dtype=np.int32)
        y_ref = G.oracle_apply(dp, x_bits, y0_bits, rows=rows)
        G.check_parity(y_bits, y_ref, y0_bits, b.token_adapter, rows=rows)
        dp.close()


def test_unit_y0_rounds_once():
    """With y0 ~ N(0,1) the delta is below one bf16 ulp of most outputs: the result must be the
    oracle's value rounded to bf16, within one bf16 ulp per element."""
    b = wl.cfg0_tiny()
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("unit")
    y_bits = G.apply_on_gpu(dp, x_bits, y0_bits)
    y_ref = G.oracle_apply(dp, x_bits, y0_bits)
    want = wl.f32_to_bf16_bits(y_ref.astype(np.float32))
    diff = np.abs(y_bits.astype(np.int32) - want.astype(np.int32))
    # same sign assumed for the ulp distance; values that straddle zero are tiny and compared in value
    same_sign = (y_bits >> 15) == (want >> 15)
    assert np.all(diff[same_sign] <= 1)
    assert np.allclose(wl.bf16_bits_to_f64(y_bits)[~same_sign], y_ref[~same_sign], atol=1e-2)
    assert (diff == 0).mean() > 0.9
    dp.close()


def test_cfg1_decode_full_size():
    _full_parity(wl.cfg1_decode())


def test_two_launch_apply_matches_fused_apply():
    """lora_apply as one launch (expand units wait on counters) and as two launches give the same
    bits: the arithmetic and its order are identical, only the hand-over of v differs."""
    L.lora_set_whole_k_limit(0)     # the single launch exists for the k-slice plan only
    try:
        for b in (wl.small_mixed(seed=4), wl.cfg1_decode(in_features=2048, out_features=512)):
            dp = G.DevicePool(b)
            x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
            y_two = G.apply_on_gpu(dp, x_bits, y0_bits)
            try:
                L.lora_set_fused_apply(True)
                y_fused = G.apply_on_gpu(dp, x_bits, y0_bits)
            finally:
                L.lora_set_fused_apply(False)
            assert np.array_equal(y_fused, y_two)
            G.check_parity(y_fused, G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
            dp.close()
    finally:
        L.lora_set_whole_k_limit(1024)


def test_one_launch_decode_apply_matches_two_launches_bitwise():
    """A whole-k decode batch runs as one launch by default (shrink units, then expand units that wait
    for their tile's v, in one grid of at most one work group per compute unit); with
    lora_set_decode_single_launch(0) as a shrink launch and an expand launch.  Same tiles, same order
    of additions: same bits.  Applied several times on one table: a launch leaves every counter at zero."""
    cases = (wl.cfg1_decode(), wl.cfg1_decode(in_features=2048, out_features=640, n_tokens=200),
             wl.cfg4_skew(0, "1:1", adapters_per_class=8), wl.small_mixed(seed=21, in_features=1024, out_features=384,
                                                                        decode_tokens=300, prefill_lens=(5, 17, 31)))
    for b in cases:
        print(f"[case] one launch vs two on {b.name} T={b.T} in={b.in_features} out={b.out_features}", flush=True)
        dp = G.DevicePool(b)
        x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
        x = G.bits_to_dev(x_bits)
        seg = L.lora_segments_build(dp.pool, b.token_adapter)
        assert L.lora_segments_info(seg)["n_k_slices"] == 1, "the case is meant to be on the whole-k plan"
        ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
        ys = {}
        for one in (True, False, True):
            L.lora_set_decode_single_launch(one)
            try:
                for rep in range(3):
                    y = G.bits_to_dev(y0_bits)
                    L.lora_apply(dp.pool, seg, x, y, ws)
                    torch.cuda.synchronize()
                    L.lora_segments_check(seg)
                    yb = G.dev_to_bits(y)
                    assert np.array_equal(ys.setdefault("first", yb), yb), f"one launch = {one}, repetition {rep}"
            finally:
                L.lora_set_decode_single_launch(True)
        rows = np.arange(0, b.T, 2, dtype=np.int32)
        G.check_parity(ys["first"], G.oracle_apply(dp, x_bits, y0_bits, rows=rows), y0_bits, b.token_adapter, rows=rows)
        L.lora_segments_destroy(seg)
        dp.close()


def test_whole_k_plan_matches_k_slice_plan_bitwise():
    """The two plans of the decode shrink (whole-k units of 16 wavefronts; k-slice units added up
    through counters) do the same arithmetic in the same order: same bits in y and in v."""
    # the last case has more whole-k units than the chip has compute units: those launches run as work
    # groups of 8 wavefronts, two per compute unit, each wavefront in two of the sixteen roles
    for b, more_than_a_round in ((wl.small_mixed(seed=5, in_features=2048), False),
                                 (wl.cfg1_decode(in_features=4096, out_features=256, n_tokens=96), False),
                                 (wl.cfg1_decode(in_features=3200, out_features=128, n_tokens=40), False),
                                 (wl.cfg1_decode(in_features=6144, out_features=128, n_tokens=512), True)):
        print(f"[case] plans on {b.name} T={b.T} in={b.in_features}", flush=True)
        dp = G.DevicePool(b)
        x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
        ys, vs = [], []
        for limit in (1024, 0):
            L.lora_set_whole_k_limit(limit)
            try:
                ys.append(G.apply_on_gpu(dp, x_bits, y0_bits))
                seg = L.lora_segments_build(dp.pool, b.token_adapter)
                info = L.lora_segments_info(seg)
                assert (info["n_k_slices"] == 1) == (limit == 1024)
                if limit == 1024:
                    assert (info["n_shrink_units"] > 256) == more_than_a_round, info["n_shrink_units"]
                v = torch.zeros(max(info["v_floats"], 1), dtype=torch.float32, device="cuda")
                ws = torch.empty(max(L.lora_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
                L.lora_shrink(dp.pool, seg, G.bits_to_dev(x_bits), v, ws)
                torch.cuda.synchronize()
                vs.append(v.cpu().numpy())
                L.lora_segments_destroy(seg)
            finally:
                L.lora_set_whole_k_limit(1024)
        assert np.array_equal(ys[0], ys[1]) and np.array_equal(vs[0].view(np.uint32), vs[1].view(np.uint32))
        G.check_parity(ys[0], G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
        dp.close()


@pytest.mark.parametrize("fused", [False, True])
def test_apply_repeated_on_one_table(fused):
    """The counters only grow; launch after launch on the same table must keep working (the epoch
    advances), also across a rebuild (counters and epoch start again)."""
    L.lora_set_fused_apply(fused)
    L.lora_set_whole_k_limit(0 if fused else 1024)
    try:
        _repeated_on_one_table()
    finally:
        L.lora_set_fused_apply(False)
        L.lora_set_whole_k_limit(1024)


def _repeated_on_one_table():
    b = wl.small_mixed(seed=6)
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("zero")
    x = G.bits_to_dev(x_bits)
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    y_ref = G.oracle_apply(dp, x_bits, y0_bits)
    # a second input on the same table: a stale v (cached from the launch before) would give the
    # other input's result
    x2_bits = wl.small_mixed(seed=7).x_bits()
    x2 = G.bits_to_dev(x2_bits)
    y2_ref = G.oracle_apply(dp, x2_bits, y0_bits)
    for it in range(9):
        if it == 4:
            L.lora_segments_rebuild(seg, b.token_adapter)
        if it == 6:
            ws.zero_()
        xin, ref = (x, y_ref) if it % 2 == 0 else (x2, y2_ref)
        y = G.bits_to_dev(y0_bits)
        L.lora_apply(dp.pool, seg, xin, y, ws)
        if it % 3 == 0:
            torch.cuda.synchronize()
        yb = G.dev_to_bits(y)
        L.lora_segments_check(seg)
        G.check_parity(yb, ref, y0_bits, b.token_adapter)
    L.lora_segments_destroy(seg)
    dp.close()


def test_token_heavy_batches_small():
    """Batches of >= 1024 tokens with groups of >= 32 tokens take the token-tile shrink and the
    64-token expand units; sized so the oracle finishes in seconds, with ragged tiles (lengths that
    are no multiple of 16, 64 or 128), every rank bucket, and decode tokens mixed in."""
    b = wl.cfg2_prefill(0, length_scale=0.08)
    b.in_features, b.out_features = 1024, 640
    assert b.T >= 1024
    _full_parity(b)
    b3 = wl.cfg3_stack(layer=1, projection=1, length_scale=0.12)   # k_proj: 4096 -> 1024
    b3.in_features = 512
    assert b3.T >= 1024
    _full_parity(b3, y0_kind="small")
    big = wl.small_mixed(seed=8, in_features=576, out_features=384, ranks=(1, 3, 4, 8, 12, 16, 24, 40, 100, 128, 200, 256),
                         decode_tokens=45, prefill_lens=(33, 130, 257, 64, 700, 31, 129))
    _full_parity(big)


@pytest.mark.parametrize("in_features", [2048, 3072, 4096])
def test_token_heavy_groups_of_every_rank_bucket(in_features):
    """One token-heavy group per rank bucket of the token-tile shrink (ranks that are no multiple of
    16 give an 8-row last block; 72..120, 136 and 200 leave row blocks beyond the rank; 64-token units
    up to rank 192, 32-token units above) at in_features of several k passes per wavefront, groups
    whose last unit is short, decode tokens beside them; all rows checked."""
    ranks = (8, 3, 12, 16, 24, 32, 40, 56, 64, 72, 100, 120, 128, 1, 136, 192, 200, 256, 161)
    lens = (33, 47, 64, 32, 95, 130, 40, 70, 36, 50, 65, 100, 81, 37, 70, 129, 45, 97, 64)
    b0 = wl.small_mixed(seed=in_features, in_features=in_features, out_features=256, n_adapters=len(ranks),
                        ranks=ranks, decode_tokens=240, prefill_lens=())
    ta = np.concatenate([np.full(n, a, dtype=np.int32) for a, n in enumerate(lens)] + [b0.token_adapter])
    b = wl.CoBatch("heavy_in%d" % in_features, in_features, 256, b0.ranks, b0.scales, ta, seed=in_features, config=9)
    assert int((b.token_adapter >= 0).sum()) >= 1024
    _full_parity(b, y0_kind="small" if in_features == 3072 else "zero")


def _long_k_mixed():
    """A mixed batch at 9216 input features with few token-heavy shrink units: they are cut along k."""
    ranks = (8, 40, 64, 128, 24, 100, 16, 3)
    lens = (200, 300, 150, 100)
    b0 = wl.small_mixed(seed=33, in_features=9216, out_features=256, n_adapters=len(ranks), ranks=ranks,
                        decode_tokens=330, prefill_lens=())
    ta = np.concatenate([np.full(n, a, dtype=np.int32) for a, n in enumerate(lens)] + [b0.token_adapter])
    b = wl.CoBatch("long_k_mixed", 9216, 256, b0.ranks, b0.scales, ta, seed=33, config=9)
    assert int((b.token_adapter >= 0).sum()) >= 1024
    return b


def test_token_heavy_units_cut_by_k():
    """Few token-heavy units: they are cut into k-slices whose sums meet through the tile's counter
    (apply after apply on one object: the counters only grow)."""
    b = _long_k_mixed()
    dp = G.DevicePool(b)
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    units, ex = L.lora_segments_export_units(seg), L.lora_segments_export(seg)
    sh = units["shrink"]
    sh = sh[sh[:, 0] >= 0]                                       # without the places that only pad an XCD's list
    heavy = sh[np.diff(ex["seg_start"])[sh[:, 0]] >= 32]
    assert set(int(k) for k in heavy[:, 5]) == {0, 1, 2, 3}      # 24 tiles: four slices each
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    x = G.bits_to_dev(x_bits)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    first = None
    for _ in range(4):
        y = G.bits_to_dev(y0_bits)
        L.lora_apply(dp.pool, seg, x, y, ws)
        torch.cuda.synchronize()
        bits = G.dev_to_bits(y)
        if first is None:
            first = bits
        assert np.array_equal(bits, first)
    L.lora_segments_check(seg)
    L.lora_segments_destroy(seg)
    y_ref = G.oracle_apply(dp, x_bits, y0_bits)
    G.check_parity(first, y_ref, y0_bits, b.token_adapter)
    dp.close()


@pytest.mark.parametrize("big", [False, True, "long_k"])
def test_shrink_and_expand_separately(big):
    if big == "long_k":
        b = _long_k_mixed()
    elif big:
        b = wl.small_mixed(seed=9, in_features=576, out_features=384, decode_tokens=40,
                           prefill_lens=(200, 470, 33, 350, 17))
        assert b.T >= 1024
    else:
        b = wl.small_mixed(seed=1)
    dp = G.DevicePool(b)
    x_bits = b.x_bits()
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    info = L.lora_segments_info(seg)
    ex = L.lora_segments_export(seg)
    x = G.bits_to_dev(x_bits)
    v = torch.full((max(info["v_floats"], 1),), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(L.lora_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_shrink(dp.pool, seg, x, v, ws)
    torch.cuda.synchronize()
    vh = v.cpu().numpy().astype(np.float64)
    v_ref = oracle.lora_shrink(x_bits, b.token_adapter, b.ranks, dp.A)
    worst = 0.0
    for t in range(b.T):
        a = b.token_adapter[t]
        if a < 0:
            assert ex["v_offset"][t] == -1
            continue
        r, r8 = int(b.ranks[a]), (int(b.ranks[a]) + 7) // 8 * 8
        row = vh[ex["v_offset"][t]: ex["v_offset"][t] + r8]
        assert not row[r:].any(), "padding entries of v must be zero"
        err = np.linalg.norm(row[:r] - v_ref[t, :r]) / np.linalg.norm(v_ref[t, :r])
        worst = max(worst, err)
    # fp32 accumulation of exact bf16 products: error ~ sqrt(in) * 2^-24 * sum|terms| / |sum|, which a
    # rank-1 row with cancellation can push to a few 1e-5
    assert worst < 2e-4, worst
    # expand from the oracle's v (rounded to fp32), into y0 = 0
    v_in = np.zeros(max(info["v_floats"], 1), dtype=np.float32)
    for t in range(b.T):
        a = b.token_adapter[t]
        if a >= 0:
            v_in[ex["v_offset"][t]: ex["v_offset"][t] + int(b.ranks[a])] = v_ref[t, : int(b.ranks[a])]
    y0_bits = b.y0_bits("zero")
    y = G.bits_to_dev(y0_bits)
    L.lora_expand(dp.pool, seg, torch.from_numpy(v_in).cuda(), y)
    torch.cuda.synchronize()
    y_ref = oracle.lora_expand(v_ref, b.token_adapter, b.ranks, b.scales, dp.B, b.out_features)
    G.check_parity(G.dev_to_bits(y), y_ref, y0_bits, b.token_adapter)
    L.lora_segments_destroy(seg)
    dp.close()


def test_expand_keeps_sixteen_bits_of_a_wide_ranged_v():
    """v reaches the expand MFMAs as two bf16 terms hi + lo (16 significant bits).  With a v whose
    entries span thirty binades (2^-20 .. 2^10, random mantissas, both signs) every element of y must
    stay within one rounding of y (2^-8) plus (2^-16 + (r + 2) 2^-24) of the sum of the absolute terms:
    a v cut to bf16 alone (8 bits) would miss that bound by two orders of magnitude on the rows where
    the large entries cancel."""
    for b in (wl.small_mixed(seed=41, in_features=256, out_features=640),
              wl.small_mixed(seed=42, in_features=256, out_features=512, decode_tokens=30, prefill_lens=(300, 500, 260))):
        dp = G.DevicePool(b)
        seg = L.lora_segments_build(dp.pool, b.token_adapter)
        info = L.lora_segments_info(seg)
        ex = L.lora_segments_export(seg)
        rng = np.random.default_rng(7)
        stride = int(b.ranks.max())
        v_ref = np.zeros((b.T, stride), dtype=np.float64)
        v_in = np.zeros(max(info["v_floats"], 1), dtype=np.float32)
        for t in range(b.T):
            a = b.token_adapter[t]
            if a < 0:
                continue
            r = int(b.ranks[a])
            vals = (rng.uniform(1.0, 2.0, r) * np.exp2(rng.integers(-20, 11, r)) * rng.choice([-1.0, 1.0], r)).astype(np.float32)
            v_in[ex["v_offset"][t]: ex["v_offset"][t] + r] = vals
            v_ref[t, :r] = vals.astype(np.float64)
        y0_bits = b.y0_bits("zero")
        y = G.bits_to_dev(y0_bits)
        L.lora_expand(dp.pool, seg, torch.from_numpy(v_in).cuda(), y)
        torch.cuda.synchronize()
        yg = wl.bf16_bits_to_f64(G.dev_to_bits(y))
        y_ref = oracle.lora_expand(v_ref, b.token_adapter, b.ranks, b.scales, dp.B, b.out_features)
        mag = oracle.lora_expand(np.abs(v_ref), b.token_adapter, b.ranks, b.scales,
                                 [None if m is None else G.abs_bits(m) for m in dp.B], b.out_features)
        act = b.token_adapter >= 0
        r8 = ((b.ranks.astype(np.int64) + 7) // 8 * 8)[b.token_adapter[act]].astype(np.float64)
        c = 2.0 ** -16 + (r8 + 2.0) * 2.0 ** -24
        bound = (G.U_BF16 * np.abs(y_ref[act]) + c[:, None] * mag[act]) * (1.0 + 2.0 ** -7)
        ratio = np.abs(yg[act] - y_ref[act]) / np.maximum(bound, 1e-300)
        assert ratio.max() <= 1.0, f"element error {ratio.max():.2f} x the hi + lo bound"
        # the bound is tight enough to tell 16 bits from 8: with v cut to bf16 the same check fails
        v_cut = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(v_ref.astype(np.float32)))
        y_cut = oracle.lora_expand(v_cut, b.token_adapter, b.ranks, b.scales, dp.B, b.out_features)
        assert (np.abs(y_cut[act] - y_ref[act]) / np.maximum(bound, 1e-300)).max() > 1.0
        assert not yg[~act].any()
        L.lora_segments_destroy(seg)
        dp.close()


def test_ranges_entry_point_matches_token_list():
    b = wl.cfg2_prefill(0, length_scale=0.02)
    b.in_features, b.out_features = 512, 256
    starts = np.array([s for s, _, _ in b.requests] + [b.T], dtype=np.int32)
    ads = np.array([a for _, _, a in b.requests], dtype=np.int32)
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("zero")
    y1 = G.apply_on_gpu(dp, x_bits, y0_bits)
    y2 = G.apply_on_gpu(dp, x_bits, y0_bits, ranges=(starts, ads))
    assert np.array_equal(y1, y2)
    y_ref = G.oracle_apply(dp, x_bits, y0_bits)
    G.check_parity(y1, y_ref, y0_bits, b.token_adapter)
    dp.close()


def test_token_order_invariance_on_gpu():
    """Permuting the batch permutes the result: each row's arithmetic does not depend on where the
    token sits in the batch, only on its group-mates' count (tile shapes), so compare to tolerance
    and require bitwise equality for a permutation that keeps every group's internal order."""
    b = wl.small_mixed(seed=2)
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    y = G.apply_on_gpu(dp, x_bits, y0_bits)
    # stable: sort tokens by adapter id (keeps order inside every group)
    p = np.argsort(b.token_adapter, kind="stable")
    yp = G.apply_on_gpu(dp, x_bits[p], y0_bits[p], token_adapter=b.token_adapter[p])
    assert np.array_equal(yp, y[p])
    q = np.random.default_rng(0).permutation(b.T)
    yq = G.apply_on_gpu(dp, x_bits[q], y0_bits[q], token_adapter=b.token_adapter[q])
    act = b.token_adapter[q] >= 0
    err = G.row_rel_l2(wl.bf16_bits_to_f64(yq)[act], wl.bf16_bits_to_f64(y[q])[act])
    assert err.max() < 5e-3
    dp.close()


def test_empty_and_all_inactive_batches():
    b = wl.cfg0_tiny()
    dp = G.DevicePool(b)
    y0_bits = b.y0_bits("small")
    none = np.full(b.T, -1, dtype=np.int32)
    y = G.apply_on_gpu(dp, b.x_bits(), y0_bits, token_adapter=none)
    assert np.array_equal(y, y0_bits)
    seg = L.lora_segments_build(dp.pool, np.zeros(0, dtype=np.int32))
    assert L.lora_segments_info(seg)["n_active"] == 0
    L.lora_apply(dp.pool, seg, None, None, None)  # nothing to do: no pointer is touched
    L.lora_segments_destroy(seg)
    dp.close()


def test_rebuild_reuses_the_object():
    b = wl.cfg0_tiny()
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("zero")
    x = G.bits_to_dev(x_bits)
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(5)
    for it in range(4):
        ta = rng.integers(-1, 4, size=b.T).astype(np.int32) if it else b.token_adapter
        L.lora_segments_rebuild(seg, ta)
        y = G.bits_to_dev(y0_bits)
        L.lora_apply(dp.pool, seg, x, y, ws)
        torch.cuda.synchronize()
        y_ref = G.oracle_apply(dp, x_bits, y0_bits, token_adapter=ta)
        G.check_parity(G.dev_to_bits(y), y_ref, y0_bits, ta)
    L.lora_segments_destroy(seg)
    dp.close()


def test_device_source_load_and_stale_segments():
    b = wl.cfg0_tiny()
    dp = G.DevicePool(b)
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    # reload adapter 2 from device memory with different weights: old segments must be refused
    other = wl.cfg0_tiny(seed=1)
    A2, B2 = other.adapter_bits(2)
    L.lora_pool_load(dp.pool, 2, G.bits_to_dev(A2), G.bits_to_dev(B2))
    torch.cuda.synchronize()
    x = G.bits_to_dev(b.x_bits())
    y = G.bits_to_dev(b.y0_bits("zero"))
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(dp.pool, seg, x, y, ws)
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    L.lora_segments_destroy(seg)
    dp.A[2], dp.B[2] = A2, B2
    y_bits = G.apply_on_gpu(dp, b.x_bits(), b.y0_bits("zero"))
    y_ref = G.oracle_apply(dp, b.x_bits(), b.y0_bits("zero"))
    G.check_parity(y_bits, y_ref, b.y0_bits("zero"), b.token_adapter)
    dp.close()


# ------------------------------------------------------------------------------------------------
# Full sizes, in the launch configuration bench.py times (lora_segments_build + lora_apply, two
# launches), checked on sampled rows the oracle computes one by one, plus the property that rows
# without an adapter and rows outside the sample's groups are untouched where that applies.
# ------------------------------------------------------------------------------------------------
def _sampled_parity(batch, n_rows=48, y0_kind="zero", seed=0, quick=False):
    """A full-size case: every active row against the oracle (row bar and element-wise bound), in row
    chunks; with --quick-parity only sampled rows (each group's first, middle and last token plus random
    ones) at the row bar."""
    print(f"[case] {batch.name} T={batch.T} in={batch.in_features} out={batch.out_features} "
          f"({'sampled rows' if quick else 'all rows'})", flush=True)
    dp = G.DevicePool(batch)
    x_bits, y0_bits = batch.x_bits(), batch.y0_bits(y0_kind)
    y_bits = G.apply_on_gpu(dp, x_bits, y0_bits)
    if y0_kind == "zero":
        # no row is left undone: every active row of a zero y0 must have become non-zero
        active_rows = batch.token_adapter >= 0
        assert np.all(y_bits[active_rows].any(axis=1)) and not y_bits[~active_rows].any()
    if not quick:
        n, worst_row, worst_el = G.check_all_rows(dp, x_bits, y0_bits, y_bits)
        assert n == int((batch.token_adapter >= 0).sum())
        dp.close()
        print(f"[ok] {batch.name}: {n} rows, max row rel-L2 {worst_row:.3e}, max element error / bound {worst_el:.3f}",
              flush=True)
        return
    rng = np.random.default_rng(seed)
    rows = set(rng.integers(0, batch.T, size=n_rows).tolist())
    for a in batch.used_adapters()[:: max(1, len(batch.used_adapters()) // 12)]:
        idx = np.nonzero(batch.token_adapter == a)[0]
        rows.update([int(idx[0]), int(idx[-1]), int(idx[len(idx) // 2])])
    rows = np.array(sorted(rows), dtype=np.int32)
    y_ref = G.oracle_apply(dp, x_bits, y0_bits, rows=rows)
    ta = batch.token_adapter[rows]
    yg = wl.bf16_bits_to_f64(y_bits[rows])
    act = ta >= 0
    assert np.array_equal(y_bits[rows][~act], y0_bits[rows][~act])
    err = G.row_rel_l2(yg[act], y_ref[act])
    assert err.max() <= G.TOL, f"max per-row relative L2 error {err.max():.3e}"
    dp.close()
    print(f"[ok] {batch.name}: max row rel-L2 {err.max():.3e} on {act.sum()} sampled rows", flush=True)


@pytest.mark.parametrize("shape", [0, 1, 2])
def test_cfg2_prefill_full_size(shape, quick_parity):
    _sampled_parity(wl.cfg2_prefill(shape), quick=quick_parity)


@pytest.mark.parametrize("layer,projection", [(0, 0), (5, 1), (17, 4), (31, 6)])
def test_cfg3_stack_full_size(layer, projection, quick_parity):
    """The mixed batch (8 prefills + 384 decode tokens, 256 adapters) on q, k, gate and down
    projections of four layers; all 224 projections share the token -> adapter map."""
    _sampled_parity(wl.cfg3_stack(layer=layer, projection=projection), seed=layer, quick=quick_parity)


def test_mixed_batch_forms_give_the_same_bits():
    """A mixed batch runs as two launches that hold both kinds of unit (the default), or as four
    launches with the decode-sized pair on the segment object's own stream between a fork and a join
    event, or as four launches on one stream.  Same bits in all three forms, on a non-default stream,
    apply after apply on one object (each reading the y the one before it wrote), with a dependent
    operation queued right behind the last apply."""
    b = wl.cfg3_stack(layer=3, projection=1)      # k_proj 4096 -> 1024: the quickest mixed batch
    dp = G.DevicePool(b)
    x = G.bits_to_dev(b.x_bits())
    results = []
    for merged, side in ((True, True), (False, True), (False, False)):
        L.lora_set_merged_launches(merged)
        L.lora_set_side_stream(side)
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                seg = L.lora_segments_build(dp.pool, b.token_adapter, stream=stream)
                info = L.lora_segments_info(seg)
                assert info["n_shrink_units"] > 32
                assert (info["n_k_slices"] > 1) == merged      # decode-sized groups in k-slices only when merged
                ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
                y = G.bits_to_dev(b.y0_bits("small"))
                for _ in range(6):
                    L.lora_apply(dp.pool, seg, x, y, ws, stream=stream)
                y_after = y.clone()           # ordered behind the last apply (and its join)
            stream.synchronize()
            L.lora_segments_check(seg, stream=stream)
            L.lora_segments_destroy(seg)
            results.append(G.dev_to_bits(y_after))
        finally:
            L.lora_set_merged_launches(True)
            L.lora_set_side_stream(True)
    assert np.array_equal(results[0], results[1]) and np.array_equal(results[1], results[2])
    # planned under one setting, applied under the other: still the same bits
    for planned in (True, False):
        try:
            L.lora_set_merged_launches(planned)
            seg = L.lora_segments_build(dp.pool, b.token_adapter)
            L.lora_set_merged_launches(not planned)
            ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
            y = G.bits_to_dev(b.y0_bits("small"))
            for _ in range(6):
                L.lora_apply(dp.pool, seg, x, y, ws)
            torch.cuda.synchronize()
            L.lora_segments_check(seg)
            L.lora_segments_destroy(seg)
        finally:
            L.lora_set_merged_launches(True)
        assert np.array_equal(G.dev_to_bits(y), results[0])
    # and the default form against the oracle, after one apply on y0
    y = G.bits_to_dev(b.y0_bits("small"))
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_apply(dp.pool, seg, x, y, ws)
    torch.cuda.synchronize()
    rows = np.arange(0, b.T, 16, dtype=np.int32)
    y_ref = G.oracle_apply(dp, b.x_bits(), b.y0_bits("small"), rows=rows)
    G.check_parity(G.dev_to_bits(y), y_ref, b.y0_bits("small"), b.token_adapter, rows=rows)
    L.lora_segments_destroy(seg)
    dp.close()


def test_mixed_batch_with_token_heavy_groups_up_to_rank_64():
    """A mixed batch whose token-heavy groups all have rank <= 64 takes the forms of the merged
    launches that fit four work groups per compute unit; the decode-sized groups beside them have
    any rank (1 .. 256, ranks that are no multiple of 8 or 16).  All rows checked."""
    ranks = (8, 16, 32, 64, 24, 40, 128, 100, 256, 3, 200, 12)
    lens = (300, 210, 170, 129, 95, 64)          # adapters 0..5 get token-heavy groups (ranks <= 64)
    b0 = wl.small_mixed(seed=21, in_features=1024, out_features=512, n_adapters=len(ranks), ranks=ranks,
                        decode_tokens=260, prefill_lens=())
    dec = b0.token_adapter.copy()
    dec[(dec >= 0) & (dec < 6)] += 6             # decode tokens only on adapters 6..11 (and -1)
    ta = np.concatenate([np.full(n, a, dtype=np.int32) for a, n in enumerate(lens)] + [dec])
    b = wl.CoBatch("mixed_low_rank_heavy", 1024, 512, b0.ranks, b0.scales, ta, seed=21, config=9)
    assert int((b.token_adapter >= 0).sum()) >= 1024
    dp = G.DevicePool(b)
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    info = L.lora_segments_info(seg)
    assert info["n_k_slices"] >= 1 and info["n_shrink_units"] > len(lens)
    L.lora_segments_destroy(seg)
    dp.close()
    _full_parity(b, y0_kind="small")


@pytest.mark.parametrize("shape,split", [(0, "9:1"), (0, "1:1"), (0, "1:9"), (1, "1:1"), (2, "1:1")])
def test_cfg4_skew_full_size(shape, split, quick_parity):
    _sampled_parity(wl.cfg4_skew(shape, split), n_rows=64, quick=quick_parity)


@pytest.mark.parametrize("split", ["9:1", "1:9"])
def test_cfg4_two_adapter_variant_full_size(split, quick_parity):
    """One rank-8 and one rank-256 adapter share the 512 tokens (the co-serving pair of the paper's
    motivation, Fig. 1): groups of up to 461 tokens on the decode-sized units."""
    _sampled_parity(wl.cfg4_skew(0, split, adapters_per_class=1), n_rows=64, quick=quick_parity)


def test_cfg4_isolated_class_equals_mixed_rows():
    """Rank-8 tokens get bitwise the same result whether or not rank-256 tokens share the batch:
    no unit of work of one adapter depends on another adapter's rank."""
    mixed = wl.cfg4_skew(0, "1:1")
    iso = wl.cfg4_skew(0, "1:1", only_class=0)
    dp = G.DevicePool(mixed)
    x_bits, y0_bits = mixed.x_bits(), mixed.y0_bits("zero")
    y_mixed = G.apply_on_gpu(dp, x_bits, y0_bits)
    y_iso = G.apply_on_gpu(dp, x_bits, y0_bits, token_adapter=iso.token_adapter)
    lo = iso.token_adapter >= 0
    assert lo.sum() == 256 and np.array_equal(y_mixed[lo], y_iso[lo]) and not y_iso[~lo].any()
    dp.close()


# ------------------------------------------------------------------------------------------------
# Live pool: which adapters are present changes between (and during) batches.
# ------------------------------------------------------------------------------------------------
def _apply_live(pool, b, ta, x, y0_bits):
    y = G.bits_to_dev(y0_bits)
    seg = L.lora_segments_build(pool, ta)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pool, seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_apply(pool, seg, x, y, ws)
    torch.cuda.synchronize()
    L.lora_segments_check(seg)
    return seg, G.dev_to_bits(y)


def test_live_pool_load_evict_compact():
    """An arena too small for all adapters: batches use what is loaded, evictions make room, a
    fragmented arena refuses a large adapter until it is compacted, moved adapters make old segment
    objects stale, and every batch still matches the oracle."""
    b = wl.small_mixed(seed=11, in_features=512, out_features=384)
    ranks = b.ranks                                   # (1, 3, 4, 8, 12, 16, 24, 32, 40, 64, 100, 128)
    size = lambda a: 2 * int((ranks[a] + 7) // 8 * 8) * (b.in_features + b.out_features)
    arena_bytes = size(11) + size(9) + size(7) + size(5) + size(3) + 4096
    arena = torch.zeros(arena_bytes, dtype=torch.uint8, device="cuda")
    pool = L.lora_pool_create_live(b.in_features, b.out_features, ranks, b.scales, arena)
    A, B = zip(*[b.adapter_bits(a) for a in range(b.n_adapters)])
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    x = G.bits_to_dev(x_bits)
    rng = np.random.default_rng(0)

    def batch_on(adapters):
        ta = b.token_adapter.copy()
        ta[ta >= 0] = rng.choice(np.asarray(adapters, dtype=np.int32), size=int((ta >= 0).sum()))
        return ta

    def check(ta, y_bits):
        y_ref = oracle.lora_apply(x_bits, ta, ranks, b.scales, list(A), list(B), y0=wl.bf16_bits_to_f64(y0_bits))
        G.check_parity(y_bits, y_ref, y0_bits, ta)

    first = [3, 5, 7, 9, 11]
    for a in first:
        L.lora_pool_load(pool, a, A[a], B[a])
    ta1 = batch_on(first)
    seg1, y1 = _apply_live(pool, b, ta1, x, y0_bits)
    check(ta1, y1)
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_load(pool, 10, A[10], B[10])                    # rank 100: no room
    assert e.value.status_name == "LORA_ERR_OOM"
    # evict 3 (rank 8) and 7 (rank 32): two holes with 5 between them; rank 40 needs more than either
    # hole and exactly as much as both
    L.lora_pool_evict(pool, 3)
    L.lora_pool_evict(pool, 7)
    sp = L.lora_pool_space(pool)
    assert sp["largest_free_bytes"] < size(8) <= sp["free_bytes"]
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_load(pool, 8, A[8], B[8])
    assert e.value.status_name == "LORA_ERR_OOM" and "compact" in e.value.detail
    # the old object used 3 and 7: refused; a batch on the remaining adapters still runs
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(pool, seg1, x, G.bits_to_dev(y0_bits), ws)
    assert e.value.status_name == "LORA_ERR_NOT_RESIDENT"
    ta2 = batch_on([5, 9, 11])
    seg2, y2 = _apply_live(pool, b, ta2, x, y0_bits)
    check(ta2, y2)
    # compaction without scratch: every move overlaps its source and goes in pieces
    before = {a: L.lora_pool_adapter_info(pool, a)["a_offset"] for a in (5, 9, 11)}
    moved = L.lora_pool_compact(pool)
    torch.cuda.synchronize()
    after = {a: L.lora_pool_adapter_info(pool, a)["a_offset"] for a in (5, 9, 11)}
    assert moved == 3 and all(after[a] < before[a] for a in before) and after[5] == 0
    sp = L.lora_pool_space(pool)
    assert sp["free_bytes"] == sp["largest_free_bytes"] >= size(8)
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(pool, seg2, x, G.bits_to_dev(y0_bits), ws)     # it uses adapters that were moved
    assert e.value.status_name == "LORA_ERR_STALE_SEGMENTS"
    L.lora_pool_load(pool, 8, A[8], B[8])
    ta3 = batch_on([5, 8, 9, 11])
    seg3, y3 = _apply_live(pool, b, ta3, x, y0_bits)
    check(ta3, y3)
    # ... and through a scratch buffer: evict the first adapter in the arena, compact again
    L.lora_pool_evict(pool, 5)
    scratch = torch.empty(size(11), dtype=torch.uint8, device="cuda")
    assert L.lora_pool_compact(pool, scratch) == 3
    torch.cuda.synchronize()
    ta4 = batch_on([8, 9, 11])
    seg4, y4 = _apply_live(pool, b, ta4, x, y0_bits)
    check(ta4, y4)
    for s in (seg1, seg2, seg3, seg4):
        L.lora_segments_destroy(s)
    L.lora_pool_destroy(pool)


def test_load_on_a_copy_stream_while_batches_run():
    """Adapters that the running batches do not use are loaded (packed by a device kernel) on a
    second stream meanwhile: the batches' results do not change by a bit, their segment object stays
    valid, and once the load has been ordered before it, a batch that uses the new adapters is right."""
    b = wl.cfg1_decode(in_features=2048, out_features=1024, n_tokens=128, n_adapters=48)
    ranks = b.ranks
    total = L.lora_pool_bytes(b.in_features, b.out_features, ranks, b.scales)
    arena = torch.zeros(total, dtype=torch.uint8, device="cuda")
    pool = L.lora_pool_create_live(b.in_features, b.out_features, ranks, b.scales, arena)
    used = [int(a) for a in b.used_adapters()]
    late = used[-4:]                                   # arrive while the first batches run
    early = [a for a in used if a not in late]
    A, B = {}, {}
    for a in used:
        A[a], B[a] = b.adapter_bits(a)
    for a in early:
        L.lora_pool_load(pool, a, A[a], B[a])
    ta_early = b.token_adapter.copy()
    ta_early[np.isin(ta_early, late)] = -1
    x_bits, y0_bits = b.x_bits(), b.y0_bits("zero")
    x = G.bits_to_dev(x_bits)
    seg, y_base = _apply_live(pool, b, ta_early, x, y0_bits)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pool, seg), 256), dtype=torch.uint8, device="cuda")
    dev_src = {a: (G.bits_to_dev(A[a]), G.bits_to_dev(B[a])) for a in late}
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    ys = []
    for it in range(12):
        y = G.bits_to_dev(y0_bits)
        compute.wait_stream(torch.cuda.current_stream())
        L.lora_apply(pool, seg, x, y, ws, stream=compute)
        if it % 3 == 0 and it // 3 < len(late):
            a = late[it // 3]
            L.lora_pool_load(pool, a, dev_src[a][0], dev_src[a][1], stream=copy)
        ys.append(y)
    loaded = torch.cuda.Event()
    loaded.record(copy)
    torch.cuda.synchronize()
    for y in ys:
        assert np.array_equal(G.dev_to_bits(y), y_base)
    # the late adapters' first batch: ordered after their loads
    compute.wait_event(loaded)
    y = G.bits_to_dev(y0_bits)
    seg_all = L.lora_segments_build(pool, b.token_adapter, stream=compute)
    ws2 = torch.empty(max(L.lora_apply_workspace_bytes(pool, seg_all), 256), dtype=torch.uint8, device="cuda")
    L.lora_apply(pool, seg_all, x, y, ws2, stream=compute)
    torch.cuda.synchronize()
    Al = [A.get(a) for a in range(b.n_adapters)]
    Bl = [B.get(a) for a in range(b.n_adapters)]
    y_ref = oracle.lora_apply(x_bits, b.token_adapter, ranks, b.scales, Al, Bl)
    G.check_parity(G.dev_to_bits(y), y_ref, y0_bits, b.token_adapter)
    L.lora_segments_destroy(seg)
    L.lora_segments_destroy(seg_all)
    L.lora_pool_destroy(pool)


# ------------------------------------------------------------------------------------------------
# Several projections that share x (q|k|v, gate|up) in one pass.
# ------------------------------------------------------------------------------------------------
def _multi_case(batch, outs, y0_kind="small"):
    """Pools of the same adapters (ranks, routing) with different out_features; weights per projection
    from the generator's projection key."""
    print(f"[case] multi {batch.name} T={batch.T} in={batch.in_features} outs={outs}", flush=True)
    batches = []
    for q, o in enumerate(outs):
        bq = wl.CoBatch(batch.name, batch.in_features, o, batch.ranks, batch.scales, batch.token_adapter,
                        seed=batch.seed, config=batch.config, layer=batch.layer, projection=q)
        batches.append(bq)
    sizes = [L.lora_pool_bytes(batch.in_features, o, batch.ranks, batch.scales) for o in outs]
    starts = np.concatenate([[0], np.cumsum([(n + 4095) // 4096 * 4096 for n in sizes])])
    arena = torch.zeros(int(starts[-1]), dtype=torch.uint8, device="cuda")
    pools, A, B = [], [], []
    used = [int(a) for a in batch.used_adapters()]
    for q, (bq, o) in enumerate(zip(batches, outs)):
        pool = L.lora_pool_create(batch.in_features, o, batch.ranks, batch.scales,
                                  arena[int(starts[q]): int(starts[q]) + sizes[q]])
        Aq, Bq = [None] * batch.n_adapters, [None] * batch.n_adapters
        for a in used:
            Aq[a], Bq[a] = bq.adapter_bits(a)
            L.lora_pool_load(pool, a, Aq[a], Bq[a])
        pools.append(pool)
        A.append(Aq)
        B.append(Bq)
    x_bits = batch.x_bits()
    x = G.bits_to_dev(x_bits)
    y0_bits = np.concatenate([bq.y0_bits(y0_kind) for bq in batches], axis=1)
    # all projections in one pass
    y = G.bits_to_dev(y0_bits)
    seg = L.lora_segments_build_multi(pools, batch.token_adapter)
    su, sx = L.lora_segments_export_units(seg)["shrink"], L.lora_segments_export(seg)
    heavy_cut = bool((su[np.diff(sx["seg_start"])[su[:, 0] % len(sx["seg_adapter"])] >= 32][:, 5] > 0).any())
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_apply_multi(pools, seg, x, y, ws)
    torch.cuda.synchronize()
    L.lora_segments_check(seg)
    y_multi = G.dev_to_bits(y)
    # a second pass on the same object after a rebuild must give the same bits
    L.lora_segments_rebuild(seg, batch.token_adapter)
    y2 = G.bits_to_dev(y0_bits)
    L.lora_apply_multi(pools, seg, x, y2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(G.dev_to_bits(y2), y_multi)
    L.lora_segments_destroy(seg)
    # the other forms of a mixed batch (four launches, with and without the side stream): same bits
    for side in (True, False):
        L.lora_set_merged_launches(False)
        L.lora_set_side_stream(side)
        try:
            seg = L.lora_segments_build_multi(pools, batch.token_adapter)
            ws2 = torch.empty(max(L.lora_apply_workspace_bytes(pools[0], seg), 256), dtype=torch.uint8, device="cuda")
            y3 = G.bits_to_dev(y0_bits)
            L.lora_apply_multi(pools, seg, x, y3, ws2)
            torch.cuda.synchronize()
            L.lora_segments_check(seg)
            L.lora_segments_destroy(seg)
        finally:
            L.lora_set_merged_launches(True)
            L.lora_set_side_stream(True)
        if heavy_cut:       # the merged plan also cut token-heavy units along k: other grouping of the sums
            d = wl.bf16_bits_to_f64(G.dev_to_bits(y3)) - wl.bf16_bits_to_f64(y_multi)
            ref = wl.bf16_bits_to_f64(y_multi)
            act = batch.token_adapter >= 0
            assert (np.linalg.norm(d[act], axis=1) / np.linalg.norm(ref[act], axis=1)).max() < G.TOL
        else:
            assert np.array_equal(G.dev_to_bits(y3), y_multi)
    # one projection at a time on the column blocks of the same matrix: the same bits; and the oracle
    y_sep = G.bits_to_dev(y0_bits)
    col = 0
    for q, o in enumerate(outs):
        s1 = L.lora_segments_build(pools[q], batch.token_adapter)
        w1 = torch.empty(max(L.lora_apply_workspace_bytes(pools[q], s1), 256), dtype=torch.uint8, device="cuda")
        L.lora_apply(pools[q], s1, x, y_sep[:, col: col + o], w1, ldy=y_sep.shape[1])
        torch.cuda.synchronize()
        L.lora_segments_destroy(s1)
        y_ref = oracle.lora_apply(x_bits, batch.token_adapter, batch.ranks, batch.scales, A[q], B[q],
                                  y0=wl.bf16_bits_to_f64(y0_bits[:, col: col + o]))
        G.check_parity(y_multi[:, col: col + o], y_ref, y0_bits[:, col: col + o], batch.token_adapter)
        col += o
    assert np.array_equal(G.dev_to_bits(y_sep), y_multi)
    for p in pools:
        L.lora_pool_destroy(p)


def test_multi_projection_apply_decode_and_prefill():
    _multi_case(wl.small_mixed(seed=12, in_features=1024), (512, 128, 256))
    _multi_case(wl.cfg1_decode(in_features=2048, out_features=128, n_tokens=160, n_adapters=64), (256, 256), "zero")
    heavy = wl.cfg2_prefill(0, length_scale=0.08)
    heavy.in_features = 1024
    assert heavy.T >= 1024
    _multi_case(heavy, (640, 128, 128), "zero")
    heavy2 = wl.cfg2_prefill(0, length_scale=0.08)      # 2048 input features: k-slices, token-heavy units cut along k
    heavy2.in_features = 2048
    _multi_case(heavy2, (256, 128), "zero")


def test_apply_replayed_from_a_captured_graph():
    """The two-launch applies leave the segment object's device table as they found it (the arrival
    counters of k-slice units go back to zero), so an apply captured into a graph can be replayed:
    y after n replays is bitwise y after n eager applies.  Decode batch on the whole-k plan, the same
    on the k-slice plan, and a mixed batch whose token-heavy units are cut along k; other work runs
    between the replays."""
    cases = [("whole-k", wl.cfg1_decode(in_features=1024, out_features=512, n_tokens=200, n_adapters=40), None),
             ("k-slices", wl.cfg1_decode(in_features=2048, out_features=512, n_tokens=200, n_adapters=40), 0),
             ("mixed", _long_k_mixed(), None),
             ("mixed, own stream", wl.cfg3_stack(layer=3, projection=1), None)]
    for name, b, limit in cases:
        print(f"[case] graph replay {name} T={b.T}", flush=True)
        if limit is not None:
            L.lora_set_whole_k_limit(limit)
        try:
            dp = G.DevicePool(b)
            seg = L.lora_segments_build(dp.pool, b.token_adapter)
        finally:
            L.lora_set_whole_k_limit(1024)
        assert (L.lora_segments_info(seg)["n_k_slices"] > 1) == (name != "whole-k")
        # the four-launch form of a mixed batch (decode-sized pair on the object's own stream, made at
        # the first apply: the eager applies below come before the capture) is chosen at apply time
        L.lora_set_merged_launches(name != "mixed, own stream")
        try:
            _graph_replay_case(name, b, dp, seg)
        finally:
            L.lora_set_merged_launches(True)
        L.lora_segments_destroy(seg)
        dp.close()


def _graph_replay_case(name, b, dp, seg):
    x = G.bits_to_dev(b.x_bits())
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    y0 = b.y0_bits("small")
    n_rep = 4
    y_eager = G.bits_to_dev(y0)
    for _ in range(n_rep):
        L.lora_apply(dp.pool, seg, x, y_eager, ws)
    torch.cuda.synchronize()
    want = G.dev_to_bits(y_eager)
    y_graph = G.bits_to_dev(y0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.lora_apply(dp.pool, seg, x, y_graph, ws, stream=torch.cuda.current_stream())
    y_graph.copy_(G.bits_to_dev(y0))          # whatever the capture did or did not execute
    scratch = torch.zeros(1 << 20, device="cuda")
    for _ in range(n_rep):
        graph.replay()
        scratch.add_(1.0)                     # eager work between the replays
        torch.cuda.synchronize()
    assert np.array_equal(G.dev_to_bits(y_graph), want), name
    # and an eager apply after the replays still finds the table in order
    y_after = G.bits_to_dev(y0)
    L.lora_apply(dp.pool, seg, x, y_after, ws)
    y_once = G.bits_to_dev(y0)
    L.lora_apply(dp.pool, seg, x, y_once, ws)
    torch.cuda.synchronize()
    assert np.array_equal(G.dev_to_bits(y_after), G.dev_to_bits(y_once))
    L.lora_segments_check(seg)
    del graph


# ------------------------------------------------------------------------------------------------
# Edges of the shape space and of the tiles.
# ------------------------------------------------------------------------------------------------
def _custom(name, in_f, out_f, ranks, ta, seed=0):
    ranks = np.asarray(ranks, dtype=np.int32)
    return wl.CoBatch(name, in_f, out_f, ranks, (2.0 / ranks).astype(np.float32), np.asarray(ta, dtype=np.int32),
                      seed=seed, config=8)


def test_smallest_shapes_and_single_tokens():
    """in = 64 and out = 128 (the smallest the library takes), rank 1 and rank 256, one token."""
    _full_parity(_custom("min_shape", 64, 128, [1, 256, 8], [1]))
    _full_parity(_custom("min_shape", 64, 128, [1, 256, 8], [0, 1, 2, -1, 1, 0]), y0_kind="small")
    _full_parity(_custom("one_token_wide", 4096, 4096, [128], [0]))
    _full_parity(_custom("ragged_in", 64 * 37, 128 * 3, [5, 72, 136, 256], [3, 2, 1, 0] * 9))


@pytest.mark.parametrize("ntok", [15, 16, 17, 31, 32, 33, 63, 64, 65, 129])
def test_group_sizes_around_the_token_tiles(ntok):
    """One group of exactly ntok tokens beside scattered others: the 16-token units of a small batch,
    and (in a batch of 1024+ tokens) the 32-token shrink and 64-token expand units."""
    ranks = [8, 24, 64, 128, 200]
    small = [a for a in (0, 1, 2, 3, 4) for _ in range(3)] + [2] * ntok + [-1, 4, 0]
    _full_parity(_custom(f"tiles_small_{ntok}", 576, 384, ranks, small, seed=ntok))
    for big_rank in (1, 3):
        heavy = [big_rank] * ntok + [0] * 700 + [4] * 40 + [2] * 300 + [-1] * 3 + [3, 1, 4]
        _full_parity(_custom(f"tiles_heavy_{ntok}_{big_rank}", 320, 256, ranks, heavy, seed=ntok + 100 * big_rank))


def _random_cobatch(seed):
    """A seeded co-batch of arbitrary structure: feature sizes anywhere on the library's grid, ranks
    anywhere in 1..256, groups from single tokens to more than a thousand, tokens without adapter,
    in contiguous runs or scattered."""
    rng = np.random.default_rng(10_000 + seed)
    in_f = 64 * int(rng.integers(1, 49))
    out_f = 128 * int(rng.integers(1, 25))
    n_adapters = int(rng.integers(1, 13))
    ranks = np.where(rng.random(n_adapters) < 0.5, rng.choice([8, 16, 32, 64, 128], n_adapters),
                     rng.integers(1, 257, n_adapters))
    sizes = []
    for a in range(n_adapters):
        kind = rng.random()
        if kind < 0.15:
            continue                                    # resident but unused
        hi = 20 if kind < 0.55 else 70 if kind < 0.75 else 400 if kind < 0.93 else 1500
        sizes.append((a, int(rng.integers(1, hi + 1))))
    if seed % 2 and sizes:                              # odd seeds: a batch large enough for token-heavy units
        a, n = sizes[int(rng.integers(0, len(sizes)))]
        sizes.append((a, int(rng.integers(600, 1500))))
    ta = np.concatenate([np.full(n, a, dtype=np.int32) for a, n in sizes]
                        + [np.full(int(rng.integers(0, 6)), -1, dtype=np.int32)])
    if rng.random() < 0.5:
        rng.shuffle(ta)
    return _custom(f"random_{seed}", in_f, out_f, ranks, ta, seed=seed)


@pytest.mark.parametrize("seed", range(20))
def test_random_cobatches_under_random_plan_settings(seed):
    """Seeded random co-batches, each under a seeded choice of the process-wide plan settings (whole-k
    limit, single-launch apply, merged launches of mixed batches, side stream): every combination has
    to meet the oracle."""
    rng = np.random.default_rng(20_000 + seed)
    b = _random_cobatch(seed)
    if b.T == 0:
        pytest.skip("the draw left no token")
    limit = int(rng.choice([0, 64, 1024]))
    fused, merged, side = (bool(rng.integers(0, 2)) for _ in range(3))
    print(f"[settings] whole_k_limit={limit} fused={fused} merged={merged} side_stream={side} ranks={b.ranks.tolist()}",
          flush=True)
    L.lora_set_whole_k_limit(limit)
    L.lora_set_fused_apply(fused)
    L.lora_set_merged_launches(merged)
    L.lora_set_side_stream(side)
    try:
        _full_parity(b, y0_kind="small" if seed % 2 else "zero")
    finally:
        L.lora_set_whole_k_limit(1024)
        L.lora_set_fused_apply(False)
        L.lora_set_merged_launches(True)
        L.lora_set_side_stream(True)


@pytest.mark.parametrize("seed", range(10))
def test_random_decode_batches_at_long_k(seed):
    """Seeded decode-sized co-batches (1..300 tokens over 4..64 adapters, uniform to very skewed
    popularity) at 2,048 .. 20,480 input features, mostly through the one-launch form, every launch the
    first on its pool: shrink units that end far apart, tiles of v that share cache lines."""
    rng = np.random.default_rng(99_000 + seed)
    in_f = 64 * int(rng.integers(32, 321))
    out_f = 128 * int(rng.integers(1, 9))
    n_ad = int(rng.integers(4, 65))
    ranks = np.where(rng.random(n_ad) < 0.6, rng.choice([8, 16, 32, 64, 128], n_ad), rng.integers(1, 257, n_ad))
    ntok = int(rng.integers(1, 301))
    p = (np.arange(n_ad) + 1.0) ** -float(rng.choice([0.0, 1.1, 2.0]))
    ta = rng.choice(n_ad, size=ntok, p=p / p.sum()).astype(np.int32)
    ta[rng.random(ntok) < 0.03] = -1
    b = _custom(f"long_k_decode_{seed}", in_f, out_f, ranks, ta, seed=seed)
    single, limit = bool(rng.integers(0, 4)), int(rng.choice([1024, 1024, 0]))
    print(f"[settings] decode_single_launch={single} whole_k_limit={limit}", flush=True)
    L.lora_set_decode_single_launch(single)
    L.lora_set_whole_k_limit(limit)
    try:
        _full_parity(b, y0_kind="small" if seed % 2 else "zero")
    finally:
        L.lora_set_decode_single_launch(True)
        L.lora_set_whole_k_limit(1024)


@pytest.mark.parametrize("seed", range(100, 112))
def test_random_cobatches_through_every_entry_point(seed):
    """Seeded random co-batches under seeded plan settings, through the calls a server makes on one
    segment object: apply on a non-default stream with x and y inside wider buffers (row strides above
    the feature sizes, guard columns that must stay as they are), a second apply on top of the first
    under other apply-time settings, shrink and expand on their own, then the same object rebuilt for another token->adapter map."""
    rng = np.random.default_rng(30_000 + seed)
    b = _random_cobatch(seed)
    if b.T == 0:
        pytest.skip("the draw left no token")
    limit = int(rng.choice([0, 64, 1024]))
    fused, merged, side = (bool(rng.integers(0, 2)) for _ in range(3))
    padx, pady = 8 * int(rng.integers(0, 5)), 8 * int(rng.integers(1, 5))
    print(f"[case] {b.name} T={b.T} in={b.in_features} out={b.out_features} ranks={b.ranks.tolist()} "
          f"whole_k_limit={limit} fused={fused} merged={merged} side_stream={side} padx={padx} pady={pady}", flush=True)
    L.lora_set_whole_k_limit(limit)
    L.lora_set_fused_apply(fused)
    L.lora_set_merged_launches(merged)
    L.lora_set_side_stream(side)
    try:
        dp = G.DevicePool(b)
        x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
        guard = np.uint16(0x7FC1)                     # a NaN pattern: any use of a guard column would show
        xw = np.full((b.T, b.in_features + padx), guard, dtype=np.uint16)
        xw[:, :b.in_features] = x_bits
        yw = np.full((b.T, b.out_features + 2 * pady), guard, dtype=np.uint16)
        yw[:, pady:pady + b.out_features] = y0_bits
        x_dev = G.bits_to_dev(xw)
        y_dev = G.bits_to_dev(yw)
        x_view, y_view = x_dev[:, :b.in_features], y_dev[:, pady:pady + b.out_features]
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            seg = L.lora_segments_build(dp.pool, b.token_adapter, stream=stream)
            ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
            L.lora_apply(dp.pool, seg, x_view, y_view, ws, stream=stream)
            y1 = y_dev.clone()
            # the settings that act when an apply is issued, drawn again: the object's plan stays
            L.lora_set_fused_apply(bool(rng.integers(0, 2)))
            L.lora_set_merged_launches(bool(rng.integers(0, 2)))
            L.lora_set_side_stream(bool(rng.integers(0, 2)))
            L.lora_apply(dp.pool, seg, x_view, y_view, ws, stream=stream)
            y2 = y_dev.clone()
        stream.synchronize()
        L.lora_segments_check(seg, stream=stream)
        y1w, y2w = G.dev_to_bits(y1), G.dev_to_bits(y2)
        for yw_after in (y1w, y2w):
            assert (yw_after[:, :pady] == guard).all() and (yw_after[:, pady + b.out_features:] == guard).all()
        y1_bits = np.ascontiguousarray(y1w[:, pady:pady + b.out_features])
        y2_bits = np.ascontiguousarray(y2w[:, pady:pady + b.out_features])
        G.check_parity(y1_bits, G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
        G.check_parity(y2_bits, G.oracle_apply(dp, x_bits, y1_bits), y1_bits, b.token_adapter)

        # shrink and expand on their own, same object, default stream
        info = L.lora_segments_info(seg)
        v = torch.full((max(info["v_floats"], 1),), float("nan"), dtype=torch.float32, device="cuda")
        ws2 = torch.empty(max(L.lora_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
        y_sep = G.bits_to_dev(y0_bits)
        L.lora_shrink(dp.pool, seg, x_view, v, ws2)
        L.lora_expand(dp.pool, seg, v, y_sep)
        torch.cuda.synchronize()
        assert not torch.isnan(v[:info["v_floats"]]).any(), "an entry of v was not written"
        G.check_parity(G.dev_to_bits(y_sep), G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)

        # the same object for another map over the same adapters (some tokens lose theirs)
        ta2 = b.token_adapter.copy()
        rng.shuffle(ta2)
        ta2[rng.random(b.T) < 0.1] = -1
        L.lora_segments_rebuild(seg, ta2)
        ws3 = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
        y3 = G.bits_to_dev(y0_bits)
        for _ in range(2):                       # twice from the same y0: the second must not see the first's counters
            y3.copy_(G.bits_to_dev(y0_bits))
            L.lora_apply(dp.pool, seg, x_view, y3, ws3)
        torch.cuda.synchronize()
        L.lora_segments_check(seg)
        G.check_parity(G.dev_to_bits(y3), G.oracle_apply(dp, x_bits, y0_bits, token_adapter=ta2), y0_bits, ta2)
        L.lora_segments_destroy(seg)
        dp.close()
    finally:
        L.lora_set_whole_k_limit(1024)
        L.lora_set_fused_apply(False)
        L.lora_set_merged_launches(True)
        L.lora_set_side_stream(True)


@pytest.mark.parametrize("seed", range(200, 208))
def test_random_cobatches_over_several_projections(seed):
    """Seeded random co-batches through lora_apply_multi over two or three projections of seeded widths:
    the same bits as one apply per projection, in every form of a mixed batch, and the oracle's values."""
    rng = np.random.default_rng(40_000 + seed)
    b = _random_cobatch(seed)
    if not (b.token_adapter >= 0).any():
        pytest.skip("the draw left no token with an adapter")
    outs = [128 * int(rng.integers(1, 13)) for _ in range(int(rng.integers(2, 4)))]
    _multi_case(b, outs, y0_kind="small" if seed % 2 else "zero")


def test_two_hundred_thousand_tokens():
    """A batch far beyond the configurations' sizes (200,003 tokens, two token-heavy groups and a few
    scattered tokens): thousands of units per launch, token offsets beyond 2^16 tiles, v beyond 2^24 floats."""
    ta = np.concatenate([np.full(150_000, 0), np.full(50_000, 1), [2, 3, -1]]).astype(np.int32)
    np.random.default_rng(7).shuffle(ta)
    b = _custom("many_tokens", 256, 256, [16, 128, 40, 200], ta, seed=7)
    _full_parity(b, y0_kind="small")


def test_adapters_placed_beyond_four_gigabytes():
    """A live pool over a 4.6 GB arena whose first 4.3 GB are reserved for other adapters: the adapters
    a batch uses lie beyond byte 2^32 (element offsets beyond 2^31).  A mixed batch (token-heavy units,
    64-token expand units, k-slice units) and a decode batch (whole-k units) against the oracle."""
    import types
    n_fill, in_f, out_f = 1040, 4096, 4096
    ranks = np.array([256] * n_fill + [128, 256, 64, 8], dtype=np.int32)
    a0 = n_fill
    heavy = [a0] * 1100 + [a0 + 1] * 40 + [a0 + 2] * 300 + [a0 + 3, a0 + 1, -1, a0 + 3] * 5
    for name, ta in (("mixed", heavy), ("decode", [a0, a0 + 1, a0 + 3, a0 + 2, a0 + 1, -1] * 5)):
        b = _custom(f"beyond_4g_{name}", in_f, out_f, ranks, ta, seed=11)
        arena = torch.empty(4_600_000_000, dtype=torch.uint8, device="cuda")
        pool = L.lora_pool_create_live(in_f, out_f, b.ranks, b.scales, arena)
        for a in range(n_fill):
            L.lora_pool_reserve(pool, a)
        A, B = [None] * b.n_adapters, [None] * b.n_adapters
        for a in range(a0, a0 + 4):
            A[a], B[a] = b.adapter_bits(a)
            L.lora_pool_load(pool, a, A[a], B[a])
            info = L.lora_pool_adapter_info(pool, a)
            assert 2 * min(info["a_offset"], info["b_offset"]) >= 1 << 32, info     # offsets count bf16 elements
        dp = types.SimpleNamespace(batch=b, pool=pool, A=A, B=B)
        x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
        print(f"[case] {b.name} T={b.T}", flush=True)
        y_bits = G.apply_on_gpu(dp, x_bits, y0_bits)
        G.check_parity(y_bits, G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
        L.lora_pool_destroy(pool)
        del arena


@pytest.mark.parametrize("kind", ["col", "row"])
def test_tensor_parallel_shard_shapes(kind):
    """One GPU's shard of the 70B shapes under 8-way tensor parallelism: 8192 -> 28672/8 (a column-parallel
    layer's columns of B) and 28672/8 -> 8192 (a row-parallel layer's rows of A), rank-skew routing."""
    import dataclasses
    if kind == "col":
        b = dataclasses.replace(wl.cfg4_skew(1, "1:1"), name="cfg4_tp8col", out_features=28672 // 8)
    else:
        b = dataclasses.replace(wl.cfg4_skew(2, "1:1"), name="cfg4_tp8row", in_features=28672 // 8)
    _full_parity(b, y0_kind="small")


@pytest.mark.parametrize("seed", range(6))
def test_live_pool_under_random_operations(seed):
    """A seeded sequence of loads, evictions, reloads with other weights, compactions (with and without
    a scratch buffer) and batches on an arena that holds about half of the adapters: every batch over
    the adapters resident at that moment matches the oracle on the weights loaded last, a load that
    does not fit says so, and the pool's free bytes follow the model."""
    rng = np.random.default_rng(60_000 + seed)
    in_f, out_f = 64 * int(rng.integers(2, 17)), 128 * int(rng.integers(1, 9))
    n = 14
    ranks = rng.integers(1, 257, n).astype(np.int32)
    size = lambda a: 2 * int((ranks[a] + 7) // 8 * 8) * (in_f + out_f)
    total = sum(size(a) for a in range(n))
    arena_bytes = (total // 2 + 4096) // 256 * 256
    ta0 = rng.integers(0, n, size=int(rng.integers(20, 200))).astype(np.int32)
    b = _custom(f"live_random_{seed}", in_f, out_f, ranks, ta0, seed=seed)
    arena = torch.zeros(arena_bytes, dtype=torch.uint8, device="cuda")
    pool = L.lora_pool_create_live(in_f, out_f, ranks, b.scales, arena)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    x = G.bits_to_dev(x_bits)
    A, B = [None] * n, [None] * n              # what each resident adapter holds now
    version = [0] * n
    resident = set()
    scratch = torch.empty(max(size(a) for a in range(n)), dtype=torch.uint8, device="cuda")
    segs, batches = [], 0
    print(f"[case] {b.name} in={in_f} out={out_f} ranks={ranks.tolist()} arena={arena_bytes}", flush=True)
    for step in range(60):
        op = rng.random()
        if op < 0.40:                                        # load (or reload with other weights)
            a = int(rng.integers(0, n))
            version[a] += 1
            src = _with_seed(b, 1000 * version[a] + seed)
            Aa, Ba = src.adapter_bits(a)
            free = L.lora_pool_space(pool)
            try:
                L.lora_pool_load(pool, a, Aa, Ba)
                A[a], B[a] = Aa, Ba
                resident.add(a)
            except L.LoraError as e:
                assert e.status_name == "LORA_ERR_OOM", e
                assert a not in resident and free["largest_free_bytes"] < size(a)
        elif op < 0.60 and resident:                         # evict
            a = int(rng.choice(sorted(resident)))
            L.lora_pool_evict(pool, a)
            resident.discard(a)
            A[a] = B[a] = None
        elif op < 0.70:                                      # compact
            L.lora_pool_compact(pool, scratch if rng.random() < 0.5 else None)
            sp = L.lora_pool_space(pool)
            assert sp["free_bytes"] == sp["largest_free_bytes"]
        elif resident:                                       # a batch over what is resident now
            ta = b.token_adapter.copy()
            ta[:] = rng.choice(np.asarray(sorted(resident), dtype=np.int32), size=b.T)
            ta[rng.random(b.T) < 0.05] = -1
            seg, y = _apply_live(pool, b, ta, x, y0_bits)
            segs.append(seg)
            y_ref = oracle.lora_apply(x_bits, ta, ranks, b.scales, A, B, y0=wl.bf16_bits_to_f64(y0_bits))
            G.check_parity(y, y_ref, y0_bits, ta)
            batches += 1
        used = sum(size(a) for a in resident)
        assert L.lora_pool_space(pool)["free_bytes"] <= arena_bytes - used
        assert L.lora_pool_space(pool)["free_bytes"] >= arena_bytes - used - 256 * (len(resident) + 1)
    assert batches >= 3
    for s in segs:
        L.lora_segments_destroy(s)
    L.lora_pool_destroy(pool)


def _with_seed(b, seed):
    import dataclasses
    return dataclasses.replace(b, seed=seed)


def test_callers_own_table_staging_and_load_buffers():
    """The allocation-free forms: the segment table in device memory and pinned staging of the caller's
    (lora_segments_upload_to, kept through lora_segments_rebuild), adapters loaded from host memory
    through a device staging buffer of the caller's (lora_pool_load_staged).  Same bits as the calls
    that allocate for the caller."""
    b = wl.small_mixed(seed=31, in_features=1024, out_features=512)
    dp = G.DevicePool(b)                     # loaded with lora_pool_load (library's staging)
    n = L.lora_pool_bytes(b.in_features, b.out_features, b.ranks, b.scales)
    arena2 = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pool2 = L.lora_pool_create(b.in_features, b.out_features, b.ranks, b.scales, arena2)
    stage = torch.empty(max(L.lora_pool_load_staging_bytes(pool2, int(a)) for a in b.used_adapters()),
                        dtype=torch.uint8, device="cuda")
    for a in b.used_adapters():
        L.lora_pool_load_staged(pool2, int(a), dp.A[int(a)], dp.B[int(a)], stage)
        torch.cuda.synchronize()             # one staging buffer for all: wait before it is written again
    assert torch.equal(arena2, dp.arena)
    with pytest.raises(L.LoraError) as e:
        L.lora_pool_load_staged(pool2, int(b.used_adapters()[0]), dp.A[int(b.used_adapters()[0])],
                                dp.B[int(b.used_adapters()[0])], stage[:64])
    assert e.value.status_name == "LORA_ERR_OOM"

    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    want = G.apply_on_gpu(dp, x_bits, y0_bits)
    seg = L.lora_segments_plan(pool2, b.token_adapter)
    need = L.lora_segments_table_bytes(seg)
    table = torch.empty(2 * need, dtype=torch.uint8, device="cuda")
    staging = torch.empty(2 * need, dtype=torch.uint8).pin_memory()
    with pytest.raises(L.LoraError) as e:
        L.lora_segments_upload_to(seg, table[:256], staging)
    assert e.value.status_name == "LORA_ERR_OOM"
    L.lora_segments_upload_to(seg, table, staging)
    x = G.bits_to_dev(x_bits)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pool2, seg), 256), dtype=torch.uint8, device="cuda")
    y = G.bits_to_dev(y0_bits)
    L.lora_apply(pool2, seg, x, y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(G.dev_to_bits(y), want)
    # another batch into the same object: the caller's buffers are used again
    ta2 = np.roll(b.token_adapter, 7)
    L.lora_segments_rebuild(seg, ta2)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(pool2, seg), 256), dtype=torch.uint8, device="cuda")
    y = G.bits_to_dev(y0_bits)
    L.lora_apply(pool2, seg, x, y, ws)
    torch.cuda.synchronize()
    want2 = G.apply_on_gpu(dp, x_bits, y0_bits, token_adapter=ta2)
    assert np.array_equal(G.dev_to_bits(y), want2)
    G.check_parity(want2, G.oracle_apply(dp, x_bits, y0_bits, token_adapter=ta2), y0_bits, ta2)
    # a batch whose table no longer fits the caller's buffers is refused, the object stays usable
    big = np.concatenate([b.token_adapter] * 40)
    if L.lora_segments_table_bytes(seg) * 20 > 2 * need:
        with pytest.raises(L.LoraError) as e:
            L.lora_segments_rebuild(seg, big)
        assert e.value.status_name == "LORA_ERR_OOM"
    L.lora_segments_destroy(seg)
    L.lora_pool_destroy(pool2)
    dp.close()


def test_plan_options_select_the_launch_form_per_object():
    """Two segment objects of one pool with different settings, applied one after the other: each keeps
    its own form (one launch / two launches / k-slices), all give the same bits."""
    b = wl.cfg1_decode(in_features=2048, out_features=1024, n_tokens=200)
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    x = G.bits_to_dev(x_bits)
    outs = []
    segs = [L.lora_segments_build(dp.pool, b.token_adapter, options=o) for o in
            (L.plan_options(decode_single_launch=1), L.plan_options(decode_single_launch=0), L.plan_options(whole_k_limit=0),
             L.plan_options(whole_k_limit=0, fused_apply=1))]
    infos = [L.lora_segments_info(sg) for sg in segs]
    assert infos[0]["single_launch"] and not infos[1]["single_launch"] and infos[2]["n_k_slices"] > 1
    for rep in range(2):
        for sg in segs:
            ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, sg), 256), dtype=torch.uint8, device="cuda")
            y = G.bits_to_dev(y0_bits)
            L.lora_apply(dp.pool, sg, x, y, ws)
            torch.cuda.synchronize()
            L.lora_segments_check(sg)
            outs.append(G.dev_to_bits(y))
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    G.check_parity(outs[0], G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
    for sg in segs:
        L.lora_segments_destroy(sg)
    dp.close()


def _linear_case(b, w_sigma, seed=0, check_elements=True, rows=None):
    """lora_linear (base GEMM with the delta in its epilogue) against oracle.lora_linear on every row
    (or, at sizes where the fp64 layer takes minutes, on the rows given)."""
    print(f"[case] lora_linear {b.name} T={b.T} in={b.in_features} out={b.out_features} sigma_W={w_sigma}", flush=True)
    dp = G.DevicePool(b)
    rng = np.random.default_rng([seed, 991])
    W_bits = wl.f32_to_bf16_bits((rng.standard_normal((b.in_features, b.out_features)) * w_sigma).astype(np.float32))
    wt = G.bits_to_dev(np.ascontiguousarray(W_bits.T))                      # W^T [out][in], a linear layer's weight
    wp = torch.empty(b.in_features * b.out_features * 2, dtype=torch.uint8, device="cuda")
    L.lora_linear_pack_weight(wt, b.in_features, b.out_features, wp)
    x_bits = b.x_bits()
    x = G.bits_to_dev(x_bits)
    y = torch.full((b.T, b.out_features), float("nan"), dtype=torch.bfloat16, device="cuda")   # y need not be initialised
    seg = L.lora_segments_build(dp.pool, b.token_adapter)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_linear(dp.pool, seg, x, wp, y, ws)
    torch.cuda.synchronize()
    L.lora_segments_check(seg)
    yg = wl.bf16_bits_to_f64(G.dev_to_bits(y))
    assert np.isfinite(yg).all(), "a row of y was not written"
    ta_all = b.token_adapter
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int32)
        yg = yg[rows]
    y_ref = oracle.lora_linear(x_bits, W_bits, b.token_adapter, b.ranks, b.scales, dp.A, dp.B, rows=rows)
    nz = np.linalg.norm(y_ref, axis=1) > 0
    err = G.row_rel_l2(yg[nz], y_ref[nz])
    assert err.max() <= G.TOL, f"max per-row relative L2 error {err.max():.3e}"
    assert not yg[~nz].any()
    worst_el = 0.0
    if check_elements:
        mag = oracle.lora_linear(G.abs_bits(x_bits), G.abs_bits(W_bits), b.token_adapter, b.ranks, b.scales,
                                 [None if m is None else G.abs_bits(m) for m in dp.A],
                                 [None if m is None else G.abs_bits(m) for m in dp.B], rows=rows)
        ta_sel = ta_all if rows is None else ta_all[rows]
        r8 = np.where(ta_sel >= 0, ((b.ranks.astype(np.int64) + 7) // 8 * 8)[np.maximum(ta_sel, 0)], 0)
        bound = G.elementwise_bound(y_ref, mag, b.in_features, r8)
        worst_el = float((np.abs(yg - y_ref) / np.maximum(bound, 1e-300)).max())
        assert worst_el <= 1.0, f"element error {worst_el:.2f} x the bound"
    L.lora_segments_destroy(seg)
    dp.close()
    print(f"[ok] lora_linear {b.name}: {len(yg)} rows, max row rel-L2 {err.max():.3e}, max element error / bound {worst_el:.3f}",
          flush=True)


def test_linear_with_delta_in_the_epilogue_small_shapes():
    """Ragged groups, odd ranks, tokens without adapter, several row tiles and column tiles; with W = 0
    (the delta alone goes through the epilogue), a small W (base and delta of the same size) and a W of
    the weights' own scale (the base dominates, as in a model)."""
    for w_sigma in (0.0, 0.0005, 0.02):
        _linear_case(wl.small_mixed(seed=51, in_features=256, out_features=384), w_sigma, seed=1)
        _linear_case(wl.small_mixed(seed=52, in_features=1024, out_features=128, decode_tokens=120,
                                    prefill_lens=(300, 500, 260, 40, 7)), w_sigma, seed=2)
    _linear_case(wl.cfg0_tiny(), 0.02)
    _linear_case(wl.cfg1_decode(in_features=2048, out_features=512, n_tokens=200), 0.0005)


def test_linear_on_a_token_heavy_batch_at_model_width():
    _linear_case(wl.cfg2_prefill(0, length_scale=0.12), 0.02, seed=3)


def test_linear_at_full_size_on_sampled_rows():
    """The shape bench.py --linear times (cfg2's 22,532 tokens, 4096 -> 4096): every group's first, middle
    and last row, the padded tail of the row order and every 61st row against the fp64 layer."""
    b = wl.cfg2_prefill(0)
    rows = set(range(0, b.T, 61)) | {b.T - 1}
    for a in b.used_adapters():
        idx = np.nonzero(b.token_adapter == a)[0]
        rows.update([int(idx[0]), int(idx[-1]), int(idx[len(idx) // 2])])
    _linear_case(b, 0.02, seed=4, rows=sorted(rows))


def test_plan_then_upload_and_the_measurement_hook():
    """lora_segments_plan + lora_segments_upload give the object lora_segments_build gives (same bits
    from an apply); a planned object that was never uploaded is refused; the measurement hook records
    its three events around the next apply's launches, in order, without changing the result."""
    import ctypes
    b = wl.cfg1_decode(in_features=2048, out_features=1024, n_tokens=100, n_adapters=30)
    dp = G.DevicePool(b)
    x, y0_bits = G.bits_to_dev(b.x_bits()), b.y0_bits("small")
    built = L.lora_segments_build(dp.pool, b.token_adapter)
    planned = L.lora_segments_plan(dp.pool, b.token_adapter)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, built), 256), dtype=torch.uint8, device="cuda")
    with pytest.raises(L.LoraError) as e:
        L.lora_apply(dp.pool, planned, x, G.bits_to_dev(y0_bits), ws)
    assert e.value.status_name == "LORA_ERR_INVALID_ARG" and "upload" in e.value.detail
    stream = torch.cuda.Stream()
    L.lora_segments_upload(planned, stream=stream)
    ys = []
    rt = ctypes.CDLL("libamdhip64.so")
    events = [ctypes.c_void_p() for _ in range(3)]
    for ev in events:
        assert rt.hipEventCreate(ctypes.byref(ev)) == 0
    with torch.cuda.stream(stream):
        for seg, hook in ((built, False), (planned, False), (planned, True), (planned, False)):
            y = G.bits_to_dev(y0_bits)
            if hook:
                L.lora_profile_next_apply(*events)
            L.lora_apply(dp.pool, seg, x, y, ws, stream=stream)
            ys.append(y)
    stream.synchronize()
    bits = [G.dev_to_bits(y) for y in ys]
    assert all(np.array_equal(bits[0], other) for other in bits[1:])
    G.check_parity(bits[0], G.oracle_apply(dp, b.x_bits(), y0_bits), y0_bits, b.token_adapter)
    ms = ctypes.c_float()
    for first, second in ((0, 1), (1, 2)):
        assert rt.hipEventElapsedTime(ctypes.byref(ms), events[first], events[second]) == 0
        assert 0.0 < ms.value < 50.0, ms.value         # one launch each: microseconds, not the whole loop
    for ev in events:
        rt.hipEventDestroy(ev)
    L.lora_segments_destroy(built)
    L.lora_segments_destroy(planned)
    dp.close()


def test_single_launch_apply_gives_up_waiting_and_says_so():
    """The failure path of the single-launch apply, reached from the host: with a wait limit of one poll
    the expand units give up before their shrink units are done, every wavefront still ends,
    lora_segments_check reports the apply as failed (and keeps reporting it), and after the object's
    table is uploaded again with the default limit the same object gives the right result."""
    b = wl.cfg1_decode(in_features=2048, out_features=512)
    dp = G.DevicePool(b)
    x_bits, y0_bits = b.x_bits(), b.y0_bits("small")
    x = G.bits_to_dev(x_bits)
    L.lora_set_whole_k_limit(0)
    L.lora_set_fused_apply(True)
    try:
        seg = L.lora_segments_build(dp.pool, b.token_adapter)
        assert L.lora_segments_info(seg)["n_k_slices"] > 1
        ws = torch.zeros(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
        L.lora_set_fused_wait_limit(1)
        L.lora_apply(dp.pool, seg, x, G.bits_to_dev(y0_bits), ws)
        for _ in range(2):
            with pytest.raises(L.LoraError) as e:
                L.lora_segments_check(seg)
            assert e.value.status_name == "LORA_ERR_DEVICE" and "waiting" in e.value.detail
        L.lora_set_fused_wait_limit(0)
        L.lora_segments_rebuild(seg, b.token_adapter)
        y = G.bits_to_dev(y0_bits)
        L.lora_apply(dp.pool, seg, x, y, ws)
        L.lora_segments_check(seg)
        G.check_parity(G.dev_to_bits(y), G.oracle_apply(dp, x_bits, y0_bits), y0_bits, b.token_adapter)
        L.lora_segments_destroy(seg)
    finally:
        L.lora_set_fused_wait_limit(0)
        L.lora_set_fused_apply(False)
        L.lora_set_whole_k_limit(1024)
    dp.close()
