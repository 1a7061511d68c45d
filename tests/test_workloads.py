"""The seeded input generators: bf16 rounding, shapes and distributions of the five configurations."""
import numpy as np
import torch

from paper_2511_22880_amd import workloads as wl


def test_bf16_rounding_is_nearest_even_and_matches_torch():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 65280.0, 1e-30], np.float32)])
    got = wl.f32_to_bf16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert got[20001] == 0x3F80 and got[20002] == 0x3F82
    back = wl.bf16_bits_to_f64(got)
    assert np.all(np.abs(back - a) <= np.abs(a) * 2.0 ** -8 + 1e-38)


def test_generators_are_deterministic_and_sliceable():
    b1, b2 = wl.cfg1_decode(in_features=256, out_features=128), wl.cfg1_decode(in_features=256, out_features=128)
    assert np.array_equal(b1.x_bits(), b2.x_bits())
    A1, B1 = b1.adapter_bits(5)
    A2, B2 = b2.adapter_bits(5)
    assert np.array_equal(A1, A2) and np.array_equal(B1, B2)
    assert A1.shape == (256, b1.ranks[5]) and B1.shape == (b1.ranks[5], 128)
    other = wl.cfg1_decode(layer=1, in_features=256, out_features=128)
    assert np.array_equal(other.token_adapter, b1.token_adapter) and np.array_equal(other.ranks, b1.ranks)
    assert not np.array_equal(other.x_bits(), b1.x_bits())
    assert not np.array_equal(other.adapter_bits(5)[0], A1)


def test_cfg0():
    b = wl.cfg0_tiny()
    assert (b.in_features, b.out_features, b.T) == (256, 256, 64)
    assert list(b.ranks) == [4, 8, 16, 32] and np.array_equal(b.token_adapter, np.arange(64) % 4)
    assert np.allclose(b.scales, 2.0 / b.ranks)
    x = wl.bf16_bits_to_f64(b.x_bits())
    assert abs(x.std() - 1.0) < 0.02
    A, B = b.adapter_bits(3)
    assert abs(wl.bf16_bits_to_f64(A).std() - 0.02) < 0.002 and abs(wl.bf16_bits_to_f64(B).std() - 0.02) < 0.002


def test_cfg1_routing_is_heavy_tailed_and_ranks_balanced():
    b = wl.cfg1_decode()
    assert b.T == 256 and b.n_adapters == 128
    counts = np.bincount(b.ranks, minlength=129)
    assert all(25 <= counts[r] <= 26 for r in wl.RANK_SET) and counts.sum() == 128
    used = b.used_adapters()
    assert 55 <= used.size <= 80
    top = np.sort(np.bincount(b.token_adapter, minlength=128))[::-1]
    assert top[0] >= 35 and top[:5].sum() >= 0.35 * 256
    # 2*r*(in+out) bytes per distinct adapter, x once, y read+write, v write+read
    r = b.ranks[used].astype(np.int64)
    assert b.weight_bytes_touched() == int(2 * r.sum() * 8192)
    rs = int(b.ranks[b.token_adapter].sum())
    assert b.algorithmic_bytes() == b.weight_bytes_touched() + 256 * 4096 * 2 + 256 * 4096 * 4 + 8 * rs


def test_cfg2_lengths_and_segments():
    for s, (i, o) in enumerate(wl.CFG2_SHAPES):
        b = wl.cfg2_prefill(s)
        assert (b.in_features, b.out_features) == (i, o)
        lens = np.array([n for _, n, _ in b.requests])
        assert lens.size == 32 and lens.min() >= 16 and lens.max() <= 4096 and b.T == lens.sum()
        assert 12000 < b.T < 45000
        assert sorted(a for _, _, a in b.requests) == list(range(32))
        for start, n, a in b.requests:
            assert np.all(b.token_adapter[start:start + n] == a)


def test_cfg3_and_cfg4_shapes():
    b = wl.cfg3_stack(layer=3, projection=6)
    assert (b.in_features, b.out_features) == (14336, 4096) and b.n_adapters == 256
    lens = [n for _, n, _ in b.requests]
    assert len(lens) == 392 and all(256 <= n <= 2048 for n in lens[:8]) and lens[8:] == [1] * 384
    assert np.array_equal(b.token_adapter, wl.cfg3_stack(layer=0, projection=0).token_adapter)
    for split, (lo, hi) in wl.CFG4_SPLITS.items():
        c = wl.cfg4_skew(0, split)
        assert c.T == 512 and (c.ranks[c.token_adapter] == 8).sum() == lo and (c.ranks[c.token_adapter] == 256).sum() == hi
        iso = wl.cfg4_skew(0, split, only_class=0)
        keep = iso.token_adapter >= 0
        assert keep.sum() == lo and np.array_equal(iso.token_adapter[keep], c.token_adapter[keep])


def test_small_mixed_has_ragged_everything():
    b = wl.small_mixed()
    assert (b.token_adapter < 0).any() and b.T == 37 + 5 + 17 + 33 + 70 + 129
    assert any(r % 8 for r in b.ranks)
