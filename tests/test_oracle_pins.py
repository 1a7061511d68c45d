"""Pins of the fp64 CPU oracle against things other than itself (no GPU).

Each test is chosen so that a plausible mistake in the oracle (a dropped term, a wrong sign or index,
a transposed operand, the scale applied twice or not at all, a row written that should not be)
fails at least one of them.  Shapes are never square so a transposed read cannot pass by accident.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2511_22880_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(a):
    """fp64 array of bf16-representable values -> bf16 bit patterns (checked to be exact)."""
    b = wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    assert np.array_equal(wl.bf16_bits_to_f64(b), np.asarray(a, dtype=np.float64)), "not bf16-exact"
    return b


def dyadic(rng, shape, span=8, denom=4):
    return rng.integers(-span, span + 1, size=shape).astype(np.float64) / denom


def random_problem(rng, T, in_f, out_f, ranks, allow_none=True):
    N = len(ranks)
    A = [wl.f32_to_bf16_bits(rng.standard_normal((in_f, r)).astype(np.float32) * 0.02) for r in ranks]
    B = [wl.f32_to_bf16_bits(rng.standard_normal((r, out_f)).astype(np.float32) * 0.02) for r in ranks]
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, in_f)).astype(np.float32))
    ta = rng.integers(-1 if allow_none else 0, N, size=T).astype(np.int32)
    scales = (2.0 / np.asarray(ranks, dtype=np.float32)).astype(np.float32)
    return x, ta, np.asarray(ranks, dtype=np.int32), scales, A, B


def test_hand_worked_example():
    """tests/golden/hand_worked_delta.txt: a pencil-and-paper evaluation of the definition."""
    want = np.loadtxt(os.path.join(GOLDEN, "hand_worked_delta.txt"), comments="#")
    A = [bits([[1], [2], [-1]]), bits([[1, 0], [0, 1], [2, -2]])]
    B = [bits([[0.5, -1]]), bits([[1, 2], [-4, 0.25]])]
    x = bits([[1, 2, 3], [2, -1, 4], [5, 5, 5]])
    y0 = np.array([[1, -1], [0, 0.25], [3, -7]], dtype=np.float64)
    y = oracle.lora_apply(x, [1, 0, -1], [1, 2], [2.0, 0.5], A, B, y0=y0)
    assert np.array_equal(y, want[:, 1:])
    v = oracle.lora_shrink(x, [1, 0, -1], [1, 2], A)
    assert np.array_equal(v, np.array([[7, -4], [-4, 0], [0, 0]], dtype=np.float64))


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_exact_on_dyadic_inputs(seed):
    """Materialise dW_a = s_a A_a B_a, then y0 + x[t] dW_a(t): a different evaluation order of the
    same definition.  Small dyadic values keep every fp64 operation exact, so equality is exact."""
    rng = np.random.default_rng(seed)
    in_f, out_f, T = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 12))
    ranks = [int(r) for r in rng.integers(1, 9, size=int(rng.integers(1, 5)))]
    Af = [dyadic(rng, (in_f, r)) for r in ranks]
    Bf = [dyadic(rng, (r, out_f)) for r in ranks]
    xf = dyadic(rng, (T, in_f))
    y0 = dyadic(rng, (T, out_f))
    scales = np.array([2.0 ** int(e) for e in rng.integers(-3, 2, size=len(ranks))], dtype=np.float32)
    ta = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    want = y0.copy()
    for t in range(T):
        a = ta[t]
        if a < 0:
            continue
        dW = np.zeros((in_f, out_f))
        for k in range(in_f):
            for o in range(out_f):
                for j in range(ranks[a]):
                    dW[k, o] += Af[a][k, j] * Bf[a][j, o]
        dW *= float(scales[a])
        for o in range(out_f):
            want[t, o] += sum(xf[t, k] * dW[k, o] for k in range(in_f))
    got = oracle.lora_apply(bits(xf), ta, ranks, scales, [bits(m) for m in Af], [bits(m) for m in Bf], y0=y0)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("r,in_f,out_f", [(8, 96, 40), (5, 33, 70), (128, 256, 192)])
def test_single_adapter_equals_merged_dense_product(r, in_f, out_f):
    """All tokens share one adapter: base output + delta equals x (W + s A B), the merged form the
    paper mentions for hot adapters.  numpy's fp64 matmul is a routine the oracle does not call."""
    rng = np.random.default_rng(100 + r)
    T = 19
    x, _, ranks, scales, A, B = random_problem(rng, T, in_f, out_f, [r], allow_none=False)
    ta = np.zeros(T, dtype=np.int32)
    W = rng.standard_normal((in_f, out_f))
    X = wl.bf16_bits_to_f64(x)
    y0 = X @ W
    merged = W + float(scales[0]) * (wl.bf16_bits_to_f64(A[0]) @ wl.bf16_bits_to_f64(B[0]))
    want = X @ merged
    got = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0)
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))
    # the delta alone must be non-trivial, otherwise the check above pins nothing
    assert np.max(np.abs(got - y0)) > 1e-6


def test_token_order_invariance_is_bitwise():
    rng = np.random.default_rng(7)
    x, ta, ranks, scales, A, B = random_problem(rng, 41, 72, 56, [3, 8, 16, 20])
    y0 = rng.standard_normal((41, 56))
    y = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0)
    p = rng.permutation(41)
    yp = oracle.lora_apply(x[p], ta[p], ranks, scales, A, B, y0=y0[p])
    assert np.array_equal(yp, y[p])


def test_rows_subset_matches_full():
    rng = np.random.default_rng(8)
    x, ta, ranks, scales, A, B = random_problem(rng, 30, 48, 24, [4, 8, 2])
    y0 = rng.standard_normal((30, 24))
    y = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0)
    rows = np.array([29, 0, 7, 7, 13], dtype=np.int32)
    ys = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0[rows], rows=rows)
    assert np.array_equal(ys, y[rows])


@pytest.mark.parametrize("r", [2, 8, 64])
def test_rank_r_equals_sum_of_two_half_rank_adapters(r):
    rng = np.random.default_rng(20 + r)
    T, in_f, out_f = 9, 80, 48
    x, _, ranks, scales, A, B = random_problem(rng, T, in_f, out_f, [r], allow_none=False)
    ta = np.zeros(T, dtype=np.int32)
    full = oracle.lora_apply(x, ta, ranks, scales, A, B)
    h = r // 2
    halves = np.zeros_like(full)
    for sl in (slice(0, h), slice(h, r)):
        halves += oracle.lora_apply(x, ta, [h], scales, [np.ascontiguousarray(A[0][:, sl])],
                                    [np.ascontiguousarray(B[0][sl, :])])
    assert np.max(np.abs(full - halves)) <= 1e-12 * np.max(np.abs(full))
    assert np.max(np.abs(full)) > 0


def test_zero_B_and_no_adapter_leave_y_bitwise_unchanged():
    rng = np.random.default_rng(3)
    x, ta, ranks, scales, A, B = random_problem(rng, 25, 40, 24, [4, 8, 16])
    B[1] = np.zeros_like(B[1])
    y0 = rng.standard_normal((25, 24))
    y = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0)
    untouched = (ta == 1) | (ta < 0)
    assert untouched.any() and (~untouched).any()
    assert np.array_equal(y[untouched], y0[untouched])
    assert np.all(np.any(y[~untouched] != y0[~untouched], axis=1))


def test_scale_is_applied_exactly_once():
    rng = np.random.default_rng(4)
    x, ta, ranks, scales, A, B = random_problem(rng, 12, 40, 24, [4, 8], allow_none=False)
    d1 = oracle.lora_apply(x, ta, ranks, scales, A, B)
    d2 = oracle.lora_apply(x, ta, ranks, scales * np.float32(2), A, B)
    assert np.array_equal(d2, 2.0 * d1)
    # and s really multiplies the product: with s = 1 the delta is (x A) B from numpy
    d0 = oracle.lora_apply(x, ta, ranks, np.ones(2, dtype=np.float32), A, B)
    X = wl.bf16_bits_to_f64(x)
    for t in range(12):
        a = ta[t]
        want = (X[t] @ wl.bf16_bits_to_f64(A[a])) @ wl.bf16_bits_to_f64(B[a])
        assert np.allclose(d0[t], want, rtol=1e-12, atol=1e-18)


def test_unit_vector_input_selects_one_row_of_A():
    """x = e_k gives s * A[k,:] B in closed form; catches a transposed A or an off-by-one in k."""
    rng = np.random.default_rng(5)
    in_f, out_f, r = 24, 10, 6
    _, _, ranks, scales, A, B = random_problem(rng, 1, in_f, out_f, [r], allow_none=False)
    Af, Bf = wl.bf16_bits_to_f64(A[0]), wl.bf16_bits_to_f64(B[0])
    xe = np.eye(in_f)
    y = oracle.lora_apply(bits(xe), np.zeros(in_f, dtype=np.int32), ranks, scales, A, B)
    v = oracle.lora_shrink(bits(xe), np.zeros(in_f, dtype=np.int32), ranks, A)
    assert np.array_equal(v, Af)
    for k in range(in_f):
        want = float(scales[0]) * (Af[k] @ Bf)
        assert np.allclose(y[k], want, rtol=1e-13, atol=0)


def test_shrink_and_expand_agree_with_numpy_matmul_per_adapter():
    rng = np.random.default_rng(6)
    T, in_f, out_f = 33, 72, 40
    x, ta, ranks, scales, A, B = random_problem(rng, T, in_f, out_f, [1, 5, 16, 32])
    X = wl.bf16_bits_to_f64(x)
    v = oracle.lora_shrink(x, ta, ranks, A)
    assert v.shape == (T, 32)
    for t in range(T):
        a = ta[t]
        if a < 0:
            assert not v[t].any()
            continue
        r = ranks[a]
        assert np.allclose(v[t, :r], X[t] @ wl.bf16_bits_to_f64(A[a]), rtol=1e-12, atol=1e-15)
        assert not v[t, r:].any()
    y0 = rng.standard_normal((T, out_f))
    vin = rng.standard_normal((T, 32))
    y = oracle.lora_expand(vin, ta, ranks, scales, B, out_f, y0=y0)
    for t in range(T):
        a = ta[t]
        if a < 0:
            assert np.array_equal(y[t], y0[t])
            continue
        r = ranks[a]
        want = y0[t] + float(scales[a]) * (vin[t, :r] @ wl.bf16_bits_to_f64(B[a]))
        assert np.allclose(y[t], want, rtol=1e-12, atol=1e-15)
    # composition of the two halves is the whole
    whole = oracle.lora_apply(x, ta, ranks, scales, A, B, y0=y0)
    comp = oracle.lora_expand(v, ta, ranks, scales, B, out_f, y0=y0)
    assert np.array_equal(whole, comp)


def test_each_token_uses_its_own_adapter():
    """Two adapters of equal rank but different weights: swapping the routing must swap results."""
    rng = np.random.default_rng(9)
    x, _, ranks, scales, A, B = random_problem(rng, 2, 24, 12, [4, 4], allow_none=False)
    x[1] = x[0]
    y01 = oracle.lora_apply(x, [0, 1], ranks, scales, A, B)
    y10 = oracle.lora_apply(x, [1, 0], ranks, scales, A, B)
    assert np.array_equal(y01[0], y10[1]) and np.array_equal(y01[1], y10[0])
    assert not np.array_equal(y01[0], y01[1])


def test_cfg0_delta_statistics():
    """cfg0 with its real distributions: the delta's variance has a closed form,
    E[d^2] = s^2 * in * r * sigma_x^2 * sigma_w^4, which a dropped scale or a wrong rank breaks."""
    b = wl.cfg0_tiny()
    AB = [b.adapter_bits(a) for a in range(b.n_adapters)]
    y = oracle.lora_apply(b.x_bits(), b.token_adapter, b.ranks, b.scales, [m[0] for m in AB], [m[1] for m in AB])
    for a in range(b.n_adapters):
        r = int(b.ranks[a])
        rows = y[b.token_adapter == a]
        want = (2.0 / r) ** 2 * b.in_features * r * (0.02 ** 4)
        assert 0.7 * want < np.mean(rows ** 2) < 1.4 * want


def test_oracle_rejects_bad_arguments():
    rng = np.random.default_rng(1)
    x, ta, ranks, scales, A, B = random_problem(rng, 4, 8, 6, [2, 3], allow_none=False)
    with pytest.raises(ValueError):
        oracle.lora_apply(x, ta, ranks, scales, [A[0], None], B)
    with pytest.raises(ValueError):
        oracle.lora_apply(x, ta, ranks, scales, [A[0], A[1].T.copy()], B)
    with pytest.raises(TypeError):
        oracle.lora_apply(x.astype(np.float32), ta, ranks, scales, A, B)


# ---- the adapted layer as a whole: base projection plus delta (oracle.lora_linear) ----------------------
def test_linear_hand_worked_example():
    """tests/golden/hand_worked_linear.txt: the hand-worked delta on top of a 3 x 2 base matrix."""
    want = np.loadtxt(os.path.join(GOLDEN, "hand_worked_linear.txt"), comments="#")
    A = [bits([[1], [2], [-1]]), bits([[1, 0], [0, 1], [2, -2]])]
    B = [bits([[0.5, -1]]), bits([[1, 2], [-4, 0.25]])]
    x = bits([[1, 2, 3], [2, -1, 4], [5, 5, 5]])
    W = bits([[1, 0.5], [-2, 1], [0, 3]])
    y = oracle.lora_linear(x, W, [1, 0, -1], [1, 2], [2.0, 0.5], A, B)
    assert np.array_equal(y, want[:, 1:])
    # a subset of rows, in another order
    assert np.array_equal(oracle.lora_linear(x, W, [1, 0, -1], [1, 2], [2.0, 0.5], A, B, rows=[2, 0]), want[[2, 0], 1:])


@pytest.mark.parametrize("seed", range(4))
def test_linear_equals_the_merged_dense_product(seed):
    """All tokens on one adapter: x W + s (x A) B = x (W + s A B), the merged weight of the paper's remark
    that an adapter can be folded into the base model; numpy's matmul in fp64 is the textbook routine."""
    rng = np.random.default_rng(100 + seed)
    T, in_f, out_f, r = 7, 24, 10, 5
    x, ta, ranks, scales, A, B = random_problem(rng, T, in_f, out_f, [r], allow_none=False)
    W = wl.f32_to_bf16_bits(rng.standard_normal((in_f, out_f)).astype(np.float32) * 0.05)
    y = oracle.lora_linear(x, W, ta, ranks, scales, A, B)
    Xf, Wf, Af, Bf = (wl.bf16_bits_to_f64(m) for m in (x, W, A[0], B[0]))
    merged = Xf @ (Wf + float(scales[0]) * (Af @ Bf))
    assert np.allclose(y, merged, rtol=1e-12, atol=1e-14)


def test_linear_with_a_zero_base_is_the_delta_and_rows_without_adapter_are_the_base():
    rng = np.random.default_rng(7)
    T, in_f, out_f = 9, 16, 6
    x, ta, ranks, scales, A, B = random_problem(rng, T, in_f, out_f, [3, 8, 1])
    ta[0], ta[1] = -1, 2
    zero_w = np.zeros((in_f, out_f), dtype=np.uint16)
    assert np.array_equal(oracle.lora_linear(x, zero_w, ta, ranks, scales, A, B), oracle.lora_apply(x, ta, ranks, scales, A, B))
    W = wl.f32_to_bf16_bits(rng.standard_normal((in_f, out_f)).astype(np.float32))
    y = oracle.lora_linear(x, W, ta, ranks, scales, A, B)
    base = wl.bf16_bits_to_f64(x) @ wl.bf16_bits_to_f64(W)
    none = ta < 0
    assert none.any() and np.allclose(y[none], base[none], rtol=1e-13, atol=1e-15)
    # base and delta add: y - x W is the delta on its own
    assert np.allclose(y - base, oracle.lora_apply(x, ta, ranks, scales, A, B), rtol=0, atol=1e-12)
    # the base part is linear in W: W scaled by 4 (exact in bf16) scales it by 4
    W4 = wl.f32_to_bf16_bits((wl.bf16_bits_to_f64(W) * 4.0).astype(np.float32))
    y4 = oracle.lora_linear(x, W4, ta, ranks, scales, A, B)
    assert np.allclose(y4 - y, 3.0 * base, rtol=1e-12, atol=1e-13)


def test_linear_reads_w_as_in_by_out():
    """A unit input row picks one row of W (not a column): x = e_k gives W[k, :] plus the delta of e_k."""
    in_f, out_f = 5, 3
    rng = np.random.default_rng(3)
    W = bits(dyadic(rng, (in_f, out_f)))
    A = [bits(dyadic(rng, (in_f, 2)))]
    B = [bits(dyadic(rng, (2, out_f)))]
    for k in range(in_f):
        e = np.zeros((1, in_f))
        e[0, k] = 1.0
        y = oracle.lora_linear(bits(e), W, [0], [2], [0.5], A, B)
        want = wl.bf16_bits_to_f64(W)[k] + 0.5 * (wl.bf16_bits_to_f64(A[0])[k] @ wl.bf16_bits_to_f64(B[0]))
        assert np.array_equal(y[0], want)
