"""Seeded synthetic co-batches: the only code shared by the CPU oracle's tests and the HIP path's tests.

This module holds none of the method's arithmetic.  It draws random numbers, rounds them to bf16
bit patterns and decides which token uses which adapter.  Everything is host-side numpy; any slice
(one adapter of one projection of one layer) can be regenerated alone because each tensor has its
own ``SeedSequence`` key ``[seed, config, layer, projection, tensor_kind, adapter]``.

The paper measures on a production trace and on traces derived from a public dataset (Evaluation,
"Traces"); neither ships with it, so these inputs stand in for them.  They keep what the paper
states about those workloads: adapter ranks drawn from {8, 16, 32, 64, 128} (Evaluation, "Traces"),
heavy-tailed adapter popularity (Motivation, "LoRA in Production"; Evaluation, "Sensitivity to Rank
Skews": a power law over adapters), prompts of hundreds to thousands of tokens (Motivation, "Input
Sizes"), and LoRA applied to every adapted projection of every layer (Background, "Low-Rank
Adaptation").
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

RANK_SET = (8, 16, 32, 64, 128)

# tensor_kind values of the seed key
_K_RANKS, _K_ROUTE, _K_LENGTHS, _K_X, _K_A, _K_B, _K_Y0 = range(7)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(k) for k in key])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp64 (for reading results and building test inputs)."""
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _normal_bf16(key: Sequence[int], shape: Tuple[int, ...], sigma: float) -> np.ndarray:
    z = _rng(*key).standard_normal(size=shape, dtype=np.float32)
    return f32_to_bf16_bits(z * np.float32(sigma))


def balanced_ranks(n_adapters: int, rank_set: Sequence[int], key: Sequence[int]) -> np.ndarray:
    """Ranks "uniform over" a set: equal counts per rank, assigned through a seeded permutation of
    adapter ids so that rank is independent of popularity."""
    perm = _rng(*key).permutation(n_adapters)
    ranks = np.empty(n_adapters, dtype=np.int32)
    for i in range(n_adapters):
        ranks[i] = rank_set[int(perm[i]) % len(rank_set)]
    return ranks


def zipf_route(n_requests: int, n_adapters: int, alpha: float, key: Sequence[int]) -> np.ndarray:
    """One iid draw per request from P(adapter k) proportional to (k+1)^-alpha on k = 0..N-1."""
    p = (np.arange(n_adapters, dtype=np.float64) + 1.0) ** (-alpha)
    p /= p.sum()
    return _rng(*key).choice(n_adapters, size=n_requests, p=p).astype(np.int32)


@dataclass
class CoBatch:
    """One projection's co-batch: T tokens, each routed to one of N adapters (or to none, -1)."""

    name: str
    in_features: int
    out_features: int
    ranks: np.ndarray            # int32 [N]
    scales: np.ndarray           # float32 [N]
    token_adapter: np.ndarray    # int32 [T], -1 = no adapter
    seed: int = 0
    config: int = 0
    layer: int = 0
    projection: int = 0
    sigma_w: float = 0.02
    sigma_x: float = 1.0
    # contiguous (start, length, adapter) ranges when the batch was built from requests
    requests: List[Tuple[int, int, int]] = field(default_factory=list)

    @property
    def T(self) -> int:
        return int(self.token_adapter.shape[0])

    @property
    def n_adapters(self) -> int:
        return int(self.ranks.shape[0])

    def _key(self, kind: int, adapter: int = 0) -> List[int]:
        return [self.seed, self.config, self.layer, self.projection, kind, adapter]

    def x_bits(self) -> np.ndarray:
        """x [T][in] as bf16 bit patterns, x ~ N(0, sigma_x^2)."""
        return _normal_bf16(self._key(_K_X), (self.T, self.in_features), self.sigma_x)

    def x_rows_bits(self, rows: Sequence[int]) -> np.ndarray:
        """Selected rows of x; identical to ``x_bits()[rows]``."""
        return self.x_bits()[np.asarray(rows, dtype=np.int64)]

    def adapter_bits(self, a: int) -> Tuple[np.ndarray, np.ndarray]:
        """(A [in][r], B [r][out]) of adapter ``a`` as bf16 bit patterns, entries ~ N(0, sigma_w^2)."""
        r = int(self.ranks[a])
        A = _normal_bf16(self._key(_K_A, a), (self.in_features, r), self.sigma_w)
        B = _normal_bf16(self._key(_K_B, a), (r, self.out_features), self.sigma_w)
        return A, B

    def y0_bits(self, kind: str = "zero") -> np.ndarray:
        """Initial y [T][out] bf16 bits: 'zero', 'small' (N(0, 0.01^2), the delta's own scale) or
        'unit' (N(0,1), the scale of a base projection's output)."""
        if kind == "zero":
            return np.zeros((self.T, self.out_features), dtype=np.uint16)
        sigma = {"small": 0.01, "unit": 1.0}[kind]
        return _normal_bf16(self._key(_K_Y0), (self.T, self.out_features), sigma)

    def used_adapters(self) -> np.ndarray:
        u = np.unique(self.token_adapter)
        return u[u >= 0].astype(np.int32)

    def weight_bytes_touched(self) -> int:
        """Bytes of the distinct adapters this batch routes to, unpadded: 2*r*(in+out) each."""
        r = self.ranks[self.used_adapters()].astype(np.int64)
        return int(2 * r.sum() * (self.in_features + self.out_features))

    def algorithmic_bytes(self) -> int:
        """Unique adapter weights once + x once + y read + y write + v write + v read (fp32)."""
        act = self.token_adapter >= 0
        n_act = int(act.sum())
        rsum = int(self.ranks[self.token_adapter[act]].astype(np.int64).sum())
        return (self.weight_bytes_touched() + 2 * n_act * self.in_features
                + 4 * n_act * self.out_features + 8 * rsum)

    def flops(self) -> int:
        act = self.token_adapter >= 0
        rsum = int(self.ranks[self.token_adapter[act]].astype(np.int64).sum())
        return 2 * rsum * (self.in_features + self.out_features)


def _scales_for(ranks: np.ndarray) -> np.ndarray:
    return (np.float32(2.0) / ranks.astype(np.float32)).astype(np.float32)


# --------------------------------------------------------------------------------------------
# The five configurations
# --------------------------------------------------------------------------------------------

def cfg0_tiny(seed: int = 0) -> CoBatch:
    """in=out=256, 4 adapters of ranks (4, 8, 16, 32), 64 decode tokens round-robin, s = 2/r."""
    ranks = np.array([4, 8, 16, 32], dtype=np.int32)
    ta = (np.arange(64) % 4).astype(np.int32)
    return CoBatch("cfg0_tiny", 256, 256, ranks, _scales_for(ranks), ta, seed=seed, config=0)


def cfg1_decode(seed: int = 0, layer: int = 0, in_features: int = 4096, out_features: int = 4096,
                n_tokens: int = 256, n_adapters: int = 128) -> CoBatch:
    """Decode co-batch at the q_proj shape: one token per request, Zipf(1.1) request->adapter over
    128 resident adapters whose ranks are balanced over {8,16,32,64,128}.  Ranks and routing are the
    same for every layer (one request batch walks the whole stack); x and weights differ per layer."""
    ranks = balanced_ranks(n_adapters, RANK_SET, [seed, 1, 0, 0, _K_RANKS, 0])
    ta = zipf_route(n_tokens, n_adapters, 1.1, [seed, 1, 0, 0, _K_ROUTE, 0])
    return CoBatch("cfg1_decode", in_features, out_features, ranks, _scales_for(ranks), ta,
                   seed=seed, config=1, layer=layer)


CFG2_SHAPES = ((4096, 4096), (4096, 14336), (14336, 4096))


def lognormal_lengths(n: int, median: float, sigma: float, lo: int, hi: int, key: Sequence[int]) -> np.ndarray:
    z = _rng(*key).standard_normal(n)
    return np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi).astype(np.int64)


def _from_requests(name: str, in_f: int, out_f: int, ranks: np.ndarray, req_len: Sequence[int],
                   req_adapter: Sequence[int], **kw) -> CoBatch:
    ta = np.concatenate([np.full(int(n), int(a), dtype=np.int32) for n, a in zip(req_len, req_adapter)])
    reqs, start = [], 0
    for n, a in zip(req_len, req_adapter):
        reqs.append((start, int(n), int(a)))
        start += int(n)
    return CoBatch(name, in_f, out_f, ranks, _scales_for(ranks), ta, requests=reqs, **kw)


def groups_batch(in_features: int, out_features: int, groups: Sequence[Tuple[int, int, int]], seed: int = 0) -> CoBatch:
    """A batch given by its groups: (how many groups, tokens of each, rank of their adapters or 0 = the
    rank set in turn), every group with an adapter of its own and its tokens side by side.  For
    measurements at chosen sizes (a planner rule on either side of its threshold), not one of the
    paper's workloads."""
    lens, ranks = [], []
    for count, tokens, rank in groups:
        for _ in range(int(count)):
            lens.append(int(tokens))
            ranks.append(int(rank) if rank else RANK_SET[len(ranks) % len(RANK_SET)])
    ranks = np.asarray(ranks, dtype=np.int32)
    return _from_requests(f"groups_{in_features}x{out_features}_{len(lens)}", in_features, out_features, ranks, lens,
                          np.arange(len(lens)), seed=seed, config=9)


def cfg2_prefill(shape: int = 0, seed: int = 0, length_scale: float = 1.0) -> CoBatch:
    """32 prefill requests, prompt lengths lognormal (median 512, sigma 1, clipped 16..4096), one
    distinct adapter per request, ranks balanced over {8..128}.  ``shape`` indexes CFG2_SHAPES.
    ``length_scale`` < 1 shrinks every prompt (parity cases the oracle can finish in seconds)."""
    in_f, out_f = CFG2_SHAPES[shape]
    n = 32
    ranks = balanced_ranks(n, RANK_SET, [seed, 2, 0, 0, _K_RANKS, 0])
    lens = lognormal_lengths(n, 512.0, 1.0, 16, 4096, [seed, 2, 0, 0, _K_LENGTHS, 0])
    if length_scale != 1.0:
        lens = np.maximum(1, np.rint(lens * length_scale)).astype(np.int64)
    return _from_requests(f"cfg2_prefill_{in_f}x{out_f}", in_f, out_f, ranks, lens, np.arange(n),
                          seed=seed, config=2, projection=shape)


# (name, in, out) of the seven adapted projections of one Llama-3-8B layer
CFG3_PROJECTIONS = (("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
                    ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096))
CFG3_LAYERS = 32


def cfg3_stack(layer: int = 0, projection: int = 0, seed: int = 0, length_scale: float = 1.0) -> CoBatch:
    """Mixed batch of the full layer stack: 8 prefills (lengths uniform 256..2048) + 384 decode
    tokens, 256 resident adapters, every request routed by Zipf(1.1).  All 32 x 7 projections share
    the token->adapter map; each has its own x and weights."""
    n_ad = 256
    ranks = balanced_ranks(n_ad, RANK_SET, [seed, 3, 0, 0, _K_RANKS, 0])
    lens = _rng(seed, 3, 0, 0, _K_LENGTHS, 0).integers(256, 2049, size=8)
    if length_scale != 1.0:
        lens = np.maximum(1, np.rint(lens * length_scale)).astype(np.int64)
    route = zipf_route(8 + 384, n_ad, 1.1, [seed, 3, 0, 0, _K_ROUTE, 0])
    req_len = list(lens) + [1] * 384
    pname, in_f, out_f = CFG3_PROJECTIONS[projection]
    return _from_requests(f"cfg3_L{layer}_{pname}", in_f, out_f, ranks, req_len, route,
                          seed=seed, config=3, layer=layer, projection=projection)


CFG4_SHAPES = ((8192, 8192), (8192, 28672), (28672, 8192))
CFG4_SPLITS = {"9:1": (461, 51), "1:1": (256, 256), "1:9": (51, 461)}


def cfg4_skew(shape: int = 0, split: str = "1:1", adapters_per_class: int = 32, seed: int = 0,
              only_class: Optional[int] = None) -> CoBatch:
    """512 decode tokens split between rank-8 and rank-256 adapters.  Adapters 0..n-1 have rank 8,
    n..2n-1 rank 256; tokens are spread uniformly (seeded) inside their class.  ``only_class``
    (0 = rank 8, 1 = rank 256) routes the other class's tokens to no adapter, which gives the
    isolated run of one class on the same tokens."""
    in_f, out_f = CFG4_SHAPES[shape]
    n = adapters_per_class
    ranks = np.array([8] * n + [256] * n, dtype=np.int32)
    n_lo, n_hi = CFG4_SPLITS[split]
    g = _rng(seed, 4, 0, 0, _K_ROUTE, 0)
    lo = g.integers(0, n, size=n_lo).astype(np.int32)
    hi = (n + g.integers(0, n, size=n_hi)).astype(np.int32)
    ta = np.concatenate([lo, hi])
    ta = ta[g.permutation(ta.shape[0])]
    if only_class is not None:
        is_hi = ta >= n
        ta = np.where(is_hi == bool(only_class), ta, -1).astype(np.int32)
    return CoBatch(f"cfg4_skew_{in_f}x{out_f}_{split.replace(':', 'to')}", in_f, out_f, ranks,
                   _scales_for(ranks), ta, seed=seed, config=4, projection=shape)


def small_mixed(seed: int = 0, in_features: int = 512, out_features: int = 384, n_adapters: int = 12,
                ranks: Sequence[int] = (1, 3, 4, 8, 12, 16, 24, 32, 40, 64, 100, 128),
                decode_tokens: int = 37, prefill_lens: Sequence[int] = (5, 17, 33, 70, 129),
                config: int = 9) -> CoBatch:
    """A small ragged case for parity tests: odd ranks, tokens with no adapter, prefill runs of
    awkward lengths mixed with scattered decode tokens, several tiles plus ragged tails."""
    ranks = np.asarray(list(ranks)[:n_adapters], dtype=np.int32)
    g = _rng(seed, config, 0, 0, _K_ROUTE, 0)
    parts = [np.full(n, int(g.integers(0, n_adapters)), dtype=np.int32) for n in prefill_lens]
    dec = g.integers(-1, n_adapters, size=decode_tokens).astype(np.int32)
    ta = np.concatenate(parts + [dec])
    return CoBatch("small_mixed", in_features, out_features, ranks, _scales_for(ranks), ta,
                   seed=seed, config=config)
