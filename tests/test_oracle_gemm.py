"""Pins for the oracle's integer GEMM (Sec. 3.3: int8 products, int32 accumulation)."""
import numpy as np
import pytest

import oracle


def rand_i8(rng, shape):
    return rng.integers(-127, 128, size=shape, dtype=np.int64).astype(np.int8)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (16, 9, 33), (40, 31, 130)])
def test_all_operand_forms_against_numpy_int64(M, N, K):
    rng = np.random.default_rng(M * 1000 + N * 10 + K)
    A, B = rand_i8(rng, (M, K)), rand_i8(rng, (K, N))
    want = A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(oracle.gemm(A, B), want)
    assert np.array_equal(oracle.gemm(np.ascontiguousarray(A.T), B, transA=True), want)
    assert np.array_equal(oracle.gemm(A, np.ascontiguousarray(B.T), transB=True), want)
    assert np.array_equal(oracle.gemm(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), transA=True, transB=True),
                          want)


def test_python_loop_bruteforce_tiny():
    rng = np.random.default_rng(1)
    A, B = rand_i8(rng, (4, 6)), rand_i8(rng, (6, 3))
    C = oracle.gemm(A, B)
    for i in range(4):
        for j in range(3):
            assert int(C[i, j]) == sum(int(A[i, k]) * int(B[k, j]) for k in range(6))


def test_identities():
    rng = np.random.default_rng(2)
    A = rand_i8(rng, (20, 20))
    eye = np.eye(20, dtype=np.int8)
    assert np.array_equal(oracle.gemm(A, eye), A.astype(np.int32))
    assert np.array_equal(oracle.gemm(eye, A), A.astype(np.int32))
    ones = np.ones((20, 5), np.int8)
    assert np.array_equal(oracle.gemm(A, ones), np.repeat(A.astype(np.int32).sum(1, keepdims=True), 5, 1))
    B = rand_i8(rng, (20, 11))
    assert np.array_equal(oracle.gemm(A, B).T, oracle.gemm(np.ascontiguousarray(B.T), np.ascontiguousarray(A.T)))


def test_extreme_values_at_the_longest_contraction():
    """+-127 everywhere at K = 25088 (the longest contraction of the workloads):
    16129 * K = 404 644 352 still fits int32."""
    K = 25088
    A = np.full((2, K), 127, np.int8)
    B = np.full((K, 2), -127, np.int8)
    C = oracle.gemm(A, B)
    assert C.dtype == np.int32 and np.all(C == -16129 * K)
    assert 16129 * 133144 < 2**31 <= 16129 * 133145      # the documented bound on the contraction length


def test_contractions_beyond_one_int32_sum_are_summed_exactly():
    """Past 133144 terms an int32 could wrap; the oracle then returns the exact int64 sums (all operand forms,
    against numpy's int64 matmul, with rows of +-127 whose sums do exceed 2^31)."""
    K = oracle.INT32_TERMS + 6857
    rng = np.random.default_rng(5)
    A, B = rand_i8(rng, (5, K)), rand_i8(rng, (K, 4))
    A[0], A[1], B[:, 0] = 127, -127, 127
    want = A.astype(np.int64) @ B.astype(np.int64)
    assert want[0, 0] == 16129 * K > 2**31 and want[1, 0] == -16129 * K
    AT, BT = np.ascontiguousarray(A.T), np.ascontiguousarray(B.T)
    for C in (oracle.gemm(A, B), oracle.gemm(AT, B, transA=True), oracle.gemm(A, BT, transB=True),
              oracle.gemm(AT, BT, transA=True, transB=True), oracle.gemm64(A, B)):
        assert C.dtype == np.int64 and np.array_equal(C, want)
    # at the bound itself the int32 path is still taken, and the 64-bit one agrees with it
    A, B = np.full((1, oracle.INT32_TERMS), 127, np.int8), np.full((oracle.INT32_TERMS, 1), 127, np.int8)
    C = oracle.gemm(A, B)
    assert C.dtype == np.int32 and int(C[0, 0]) == 16129 * oracle.INT32_TERMS == int(oracle.gemm64(A, B)[0, 0])


def test_empty_contraction_gives_zeros():
    C = oracle.gemm(np.zeros((3, 0), np.int8), np.zeros((0, 4), np.int8))
    assert C.shape == (3, 4) and np.all(C == 0)
