"""Helpers for the GPU parity tests: put a seeded co-batch on the device, run the C-ABI path through
the Python binding, and compare with the CPU oracle.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2511_22880_amd import binding as L
from paper_2511_22880_amd import workloads as wl

TOL = 5e-3  # max per-row relative L2 error against the fp64 oracle (bf16 inputs, fp32 accumulation)


def bits_to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 patterns -> bf16 tensor on the GPU (bit copy, no conversion)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class DevicePool:
    """A pool for one CoBatch with the adapters the batch uses (or all of them) loaded from host."""

    def __init__(self, batch: wl.CoBatch, load="used", stream=None, padded=False):
        self.batch = batch
        # padded: the control layout, every adapter stored at the pool's largest rank with zero rows / columns
        ranks = np.full_like(batch.ranks, batch.ranks.max()) if padded else batch.ranks
        n = L.lora_pool_bytes(batch.in_features, batch.out_features, ranks, batch.scales)
        self.arena = torch.zeros(max(n, 256), dtype=torch.uint8, device="cuda")
        self.pool = L.lora_pool_create(batch.in_features, batch.out_features, ranks, batch.scales, self.arena)
        self.A = [None] * batch.n_adapters
        self.B = [None] * batch.n_adapters
        ids = batch.used_adapters() if load == "used" else range(batch.n_adapters)
        for a in ids:
            A, B = batch.adapter_bits(int(a))
            self.A[int(a)], self.B[int(a)] = A, B
            if padded:
                Ap = np.zeros((batch.in_features, int(ranks[a])), dtype=np.uint16)
                Bp = np.zeros((int(ranks[a]), batch.out_features), dtype=np.uint16)
                Ap[:, :A.shape[1]] = A
                Bp[:B.shape[0]] = B
                A, B = Ap, Bp
            L.lora_pool_load(self.pool, int(a), A, B, stream=stream)

    def close(self):
        L.lora_pool_destroy(self.pool)


def row_rel_l2(y_gpu: np.ndarray, y_ref: np.ndarray) -> np.ndarray:
    num = np.sqrt(((y_gpu - y_ref) ** 2).sum(axis=1))
    den = np.sqrt((y_ref ** 2).sum(axis=1))
    out = np.zeros_like(num)
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    out[~nz] = np.where(num[~nz] == 0, 0.0, np.inf)
    return out


def apply_on_gpu(dp: DevicePool, x_bits: np.ndarray, y0_bits: np.ndarray, token_adapter=None, ranges=None):
    """Runs lora_segments_build + lora_apply; returns y as bf16 bits [T][out]."""
    b = dp.batch
    x = bits_to_dev(x_bits)
    y = bits_to_dev(y0_bits)
    ta = b.token_adapter if token_adapter is None else token_adapter
    if ranges is not None:
        seg = L.lora_segments_build_ranges(dp.pool, ranges[0], ranges[1])
    else:
        seg = L.lora_segments_build(dp.pool, ta)
    ws = torch.empty(max(L.lora_apply_workspace_bytes(dp.pool, seg), 256), dtype=torch.uint8, device="cuda")
    L.lora_apply(dp.pool, seg, x, y, ws)
    torch.cuda.synchronize()
    L.lora_segments_check(seg)
    L.lora_segments_destroy(seg)
    return dev_to_bits(y)


def oracle_apply(dp: DevicePool, x_bits, y0_bits, token_adapter=None, rows=None):
    b = dp.batch
    ta = b.token_adapter if token_adapter is None else token_adapter
    y0 = wl.bf16_bits_to_f64(y0_bits)
    if rows is not None:
        y0 = y0[np.asarray(rows)]
    return oracle.lora_apply(x_bits, ta, b.ranks, b.scales, dp.A, dp.B, y0=y0, rows=rows)


def check_parity(y_bits: np.ndarray, y_ref: np.ndarray, y0_bits: np.ndarray, token_adapter: np.ndarray, rows=None,
                 tol: float = TOL):
    """Rows with an adapter: relative L2 <= tol.  Rows without: bitwise equal to y0."""
    ta = np.asarray(token_adapter)
    if rows is not None:
        rows = np.asarray(rows)
        y_bits, y0_bits, ta = y_bits[rows], y0_bits[rows], ta[rows]
    yg = wl.bf16_bits_to_f64(y_bits)
    act = ta >= 0
    assert np.array_equal(y_bits[~act], y0_bits[~act]), "rows without adapter were written"
    err = row_rel_l2(yg[act], y_ref[act])
    worst = float(err.max()) if err.size else 0.0
    assert worst <= tol, f"max per-row relative L2 error {worst:.3e} > {tol:.1e}"
    return worst


# ---- element-wise bound --------------------------------------------------------------------------------
# y_gpu = bf16_rne(fp32(y0) + s * acc), acc an fp32 sum of exact bf16 x bf16 products in some order, v
# handed to the expand as bf16 hi + lo (relative error <= 2^-16).  With M[t, o] = s * sum_j (sum_k |x_k|
# |A_kj|) |B_jo| (the same formula on absolute values, which the oracle computes from inputs whose sign bits
# are cleared), every element obeys
#     |y_gpu - y_ref| <= U_BF16 * |y_ref| + C * M,      C = 2^-16 + (in + r8 + 2) * 2^-24,
# both times (1 + 2^-7) for the second-order terms: 2^-8 is the one rounding to nearest of a format with 8
# significant bits (half a unit in the last place of a value just above a power of two), 2^-24 per
# fp32 addition in the worst case over in terms of the shrink and r8 of the expand, 2^-16 the hi + lo split
# (two roundings of 2^-8 each, the second on the remainder of the first).
# The bound follows from the arithmetic, not from what the kernels were seen to do; it is loose (errors of
# sums grow like the square root of their length, not linearly), and it holds for any summation order.
U_BF16 = 2.0 ** -8


def elementwise_bound(y_ref: np.ndarray, mag: np.ndarray, in_features: int, r8_of_row: np.ndarray) -> np.ndarray:
    c = 2.0 ** -16 + (in_features + r8_of_row.astype(np.float64) + 2.0) * 2.0 ** -24
    return (U_BF16 * np.abs(y_ref) + c[:, None] * mag) * (1.0 + 2.0 ** -7)


def abs_bits(bits: np.ndarray) -> np.ndarray:
    """bf16 patterns with the sign bit cleared."""
    return np.ascontiguousarray(bits) & np.uint16(0x7FFF)


def check_all_rows(dp: DevicePool, x_bits, y0_bits, y_bits, token_adapter=None, chunk_rows: int = 4096, tol: float = TOL):
    """Every row against the oracle, in chunks of rows: rows with an adapter within `tol` (relative L2) and
    inside the element-wise bound; rows without one bitwise equal to y0.  Returns (rows checked, worst row
    error, worst element error / bound)."""
    b = dp.batch
    ta = np.asarray(b.token_adapter if token_adapter is None else token_adapter)
    absA = [None if a is None else abs_bits(a) for a in dp.A]
    absB = [None if a is None else abs_bits(a) for a in dp.B]
    ax = abs_bits(x_bits)
    r8 = (b.ranks.astype(np.int64) + 7) // 8 * 8
    worst_row, worst_el, n_checked = 0.0, 0.0, 0
    for r0 in range(0, b.T, chunk_rows):
        rows = np.arange(r0, min(b.T, r0 + chunk_rows), dtype=np.int32)
        act = ta[rows] >= 0
        assert np.array_equal(y_bits[rows][~act], y0_bits[rows][~act]), "rows without adapter were written"
        if not act.any():
            continue
        rows = rows[act]
        y0 = wl.bf16_bits_to_f64(y0_bits[rows])
        y_ref = oracle.lora_apply(x_bits, ta, b.ranks, b.scales, dp.A, dp.B, y0=y0, rows=rows)
        mag = oracle.lora_apply(ax, ta, b.ranks, b.scales, absA, absB, rows=rows)
        yg = wl.bf16_bits_to_f64(y_bits[rows])
        err = row_rel_l2(yg, y_ref)
        worst_row = max(worst_row, float(err.max()))
        assert err.max() <= tol, f"row {int(rows[int(err.argmax())])}: relative L2 error {err.max():.3e} > {tol:.1e}"
        bound = elementwise_bound(y_ref, mag + np.abs(y0), b.in_features, r8[ta[rows]])
        ratio = np.abs(yg - y_ref) / np.maximum(bound, 1e-300)
        worst_el = max(worst_el, float(ratio.max()))
        if ratio.max() > 1.0:
            i, j = np.unravel_index(int(ratio.argmax()), ratio.shape)
            raise AssertionError(f"element ({int(rows[i])}, {j}): |y_gpu - y_ref| = {abs(yg[i, j] - y_ref[i, j]):.3e} "
                                 f"exceeds the bound {bound[i, j]:.3e}")
        n_checked += int(rows.size)
    return n_checked, worst_row, worst_el
