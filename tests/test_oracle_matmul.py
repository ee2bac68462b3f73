"""Pins of the oracle's arithmetic: closed forms, special cases that reduce to a
library routine, and operand-order traps (non-square, asymmetric operands)."""
import numpy as np
import pytest

import workloads
from oracle import matmul as om


def test_identity_left_and_right():
    rng = np.random.default_rng(1)
    B = rng.standard_normal((7, 11))
    assert np.array_equal(om.matmul(np.eye(7), B), B)
    A = rng.standard_normal((5, 9))
    assert np.array_equal(om.matmul(A, np.eye(9)), A)


def test_all_ones_product_equals_k():
    for m, k, n in [(3, 17, 5), (8, 1, 8), (2, 300, 4)]:
        C = om.matmul(np.ones((m, k)), np.ones((k, n)))
        assert C.shape == (m, n) and (C == k).all()


def test_rank_one_operands():
    """A = u 1^T, B = 1 v^T  =>  C = K u v^T; u and v differ in length and
    content so a transposed or swapped operand cannot pass."""
    u = np.arange(1.0, 7.0)            # m = 6
    v = np.array([0.5, -2.0, 4.0])     # n = 3
    K = 16                             # powers of two: exact in fp64
    C = om.matmul(np.outer(u, np.ones(K)), np.outer(np.ones(K), v))
    assert np.array_equal(C, K * np.outer(u, v))


def test_unit_vectors_pick_single_entries():
    """e_i^T A' style: A with a single one at (i, l) selects row l of B into row i."""
    B = np.arange(20.0).reshape(4, 5)
    for i in range(3):
        for l in range(4):
            A = np.zeros((3, 4))
            A[i, l] = 1.0
            C = om.matmul(A, B)
            want = np.zeros((3, 5))
            want[i] = B[l]
            assert np.array_equal(C, want)


def test_linearity_and_library_agreement():
    rng = np.random.default_rng(2)
    A = rng.standard_normal((33, 47))
    B = rng.standard_normal((47, 29))
    C = om.matmul(A, B)
    np.testing.assert_allclose(C, A @ B, rtol=0, atol=1e-13 * 47)   # BLAS dgemm as the special case
    assert np.array_equal(om.matmul(4.0 * A, B), 4.0 * C)           # power-of-two scaling is exact
    A2 = rng.standard_normal((33, 47))
    np.testing.assert_allclose(om.matmul(A + A2, B), C + om.matmul(A2, B), rtol=0, atol=1e-12)


def test_integer_products_are_exact_in_every_input_type():
    """Small integers are exact in bf16, fp32 and fp64, so the three input types
    must give the same exact integer result as int64 arithmetic."""
    rng = np.random.default_rng(3)
    Ai = rng.integers(-8, 9, size=(10, 40))
    Bi = rng.integers(-8, 9, size=(40, 6))
    want = (Ai @ Bi).astype(np.float64)
    assert np.array_equal(om.matmul(Ai.astype(np.float64), Bi.astype(np.float64)), want)
    assert np.array_equal(om.matmul(Ai.astype(np.float32), Bi.astype(np.float32)), want)
    Ab = workloads.bf16_round(Ai.astype(np.float32))
    Bb = workloads.bf16_round(Bi.astype(np.float32))
    assert np.array_equal(om.matmul(Ab, Bb, bf16=True), want)


def test_bf16_bit_patterns_widen_exactly():
    """1 x 1 products against hand-decoded bf16 values (sign, exponent, 7-bit fraction)."""
    cases = {0x3F80: 1.0, 0xBF80: -1.0, 0x4000: 2.0, 0x3F00: 0.5, 0x3FC0: 1.5, 0x4049: 3.140625,
             0x0000: 0.0, 0x3C00: 2.0 ** -7, 0xC2F7: -123.5}
    one = np.array([[0x3F80]], dtype=np.uint16)
    for bits, val in cases.items():
        x = np.array([[bits]], dtype=np.uint16)
        assert om.matmul(x, one, bf16=True)[0, 0] == val
        assert om.matmul(one, x, bf16=True)[0, 0] == val


def test_bf16_rounding_helper_is_nearest_even():
    """The input generator's rounding, against hand-worked ties."""
    f = np.array([1.0, 1.00390625, 1.01171875, 1.005, -2.5, 3.0e-3], dtype=np.float32)
    # 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80);
    # 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    bits = workloads.bf16_round(f)
    assert bits[0] == 0x3F80 and bits[1] == 0x3F80 and bits[2] == 0x3F82
    back = workloads.bf16_to_f32(bits)
    assert np.all(np.abs(back - f) <= np.abs(f) * 2.0 ** -8)
    assert np.array_equal(workloads.bf16_round(back), bits)       # idempotent


def test_strided_rows_and_empty_dims():
    rng = np.random.default_rng(4)
    big = rng.standard_normal((12, 30))
    A = big[2:9, 3:14]            # row stride 30, width 11
    Bbig = rng.standard_normal((11, 40))
    B = Bbig[:, 5:22]
    np.testing.assert_allclose(om.matmul(A, B), np.array(A) @ np.array(B), rtol=0, atol=1e-12)
    assert om.matmul(np.zeros((0, 5)), np.zeros((5, 3))).shape == (0, 3)
    assert np.array_equal(om.matmul(np.zeros((4, 0)), np.zeros((0, 3))), np.zeros((4, 3)))


def test_sum_runs_in_ascending_k():
    """fp64 cancellation that depends on order: (1e16 + 1) - 1e16 = 0 left to
    right (1 is below half an ulp of 1e16), but 1 if the last two were paired
    first."""
    A = np.array([[1e16, 1.0, -1e16]])
    B = np.ones((3, 1))
    assert om.matmul(A, B)[0, 0] == 0.0
    A = np.array([[1e16, -1e16, 1.0]])
    assert om.matmul(A, B)[0, 0] == 1.0


def test_reduce_replicas_two_is_plain_fp32_add():
    rng = np.random.default_rng(5)
    a = rng.standard_normal((9, 13)).astype(np.float32)
    b = rng.standard_normal((9, 13)).astype(np.float32)
    assert np.array_equal(om.reduce_replicas([a, b]), a + b)
    assert np.array_equal(om.reduce_replicas([a]), a)


def test_reduce_replicas_order_and_precision():
    """fp32, left to right: (1e8 + 1) + (-1e8) = 0 in fp32, whereas fp64 or
    another order would give 1."""
    one = np.full((2, 2), 1.0, dtype=np.float32)
    big = np.full((2, 2), 1e8, dtype=np.float32)
    assert (om.reduce_replicas([big, one, -big]) == 0.0).all()
    assert (om.reduce_replicas([big, -big, one]) == 1.0).all()
    rng = np.random.default_rng(6)
    parts = [rng.standard_normal((5, 7)).astype(np.float32) for _ in range(4)]
    want = ((parts[0] + parts[1]) + parts[2]) + parts[3]
    assert np.array_equal(om.reduce_replicas(parts), want)


def test_thread_count_reported():
    assert om.num_threads() >= 1
