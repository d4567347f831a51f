"""Pins for the CPU oracle's matmul (row-major A, column-major B) and for the
int32 / fp32 accumulation semantics the paper attributes to the tensorized
instructions (Section III-A)."""
import numpy as np
import pytest

import oracle
from paper_2101_08458_amd import workloads as wl


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (16, 16, 16), (33, 17, 65), (1, 40, 96)])
def test_matmul_i8_vs_int64_library(M, N, K):
    A, B = wl.gemm_inputs_i8(M, N, K, 80, M)
    got = oracle.matmul_i8(A, B)
    ref = A.astype(np.int64) @ B.astype(np.int64).T
    assert np.array_equal(got.astype(np.int64), ref)


def test_matmul_identity_and_transpose():
    g = wl.rng(81)
    B = wl.int8_weights(g, (9, 12))                       # n=9 columns of k=12
    eye = np.eye(12, dtype=np.int8)
    # A = I (12x12): C[m,n] = B[k=m, n] = Bstored[n, m]
    assert np.array_equal(oracle.matmul_i8(eye, B), B.T.astype(np.int32))
    A = wl.int8_weights(g, (7, 12))
    # (A B)^T obtained by swapping the operands (both are "rows of k")
    assert np.array_equal(oracle.matmul_i8(A, B).T, oracle.matmul_i8(B, A))


def test_matmul_not_symmetric_in_layout():
    """A deliberately asymmetric hand-worked 2x3 * 3x2 case."""
    A = np.array([[1, 2, 3], [4, 5, 6]], np.int8)
    Bcols = np.array([[1, 0, -1], [2, 1, 0]], np.int8)    # column n of B is Bcols[n]
    assert np.array_equal(oracle.matmul_i8(A, Bcols), np.array([[-2, 4], [-2, 13]], np.int32))


def test_vnni_lane_semantics():
    """The VNNI description in Section III-A: 16 int32 lanes, lane i = c[i] + sum over
    j<4 of a[4i+j]*b[4i+j].  Lane i is the diagonal of a [16,4] x [4,16] product."""
    g = wl.rng(82)
    a = wl.int8_weights(g, (64,))
    b = wl.int8_weights(g, (64,))
    a[:4] = -128
    b[:4] = -128                                           # lane 0 = 65536: needs widening
    c = g.integers(-1000, 1000, size=16).astype(np.int32)
    lanes = np.diag(oracle.matmul_i8(np.ascontiguousarray(a.reshape(16, 4)),
                                     np.ascontiguousarray(b.reshape(16, 4)))) + c
    exp = [int(c[i]) + sum(int(a[4 * i + j]) * int(b[4 * i + j]) for j in range(4)) for i in range(16)]
    assert lanes.tolist() == exp and lanes[0] == 65536 + c[0]


def test_tensor_core_shape_f16():
    """16x16x16, fp16 in, fp32 accumulate (the Tensor Core description, Section III-A):
    small integers make every partial sum exact, so the answer is the integer product."""
    g = wl.rng(83)
    Ai = g.integers(-8, 9, size=(16, 16))
    Bi = g.integers(-8, 9, size=(16, 16))
    C = oracle.matmul_f16(wl.f16_bits(Ai), wl.f16_bits(Bi))
    assert np.array_equal(C.astype(np.int64), Ai @ Bi.T)


def test_matmul_f16_sequential_fp32_order():
    A, B = wl.gemm_inputs_f16(3, 4, 37, 84)
    got = oracle.matmul_f16(A, B)
    Af, Bf = A.view(np.float16).astype(np.float32), B.view(np.float16).astype(np.float32)
    for m in range(3):
        for n in range(4):
            acc = np.float32(0)
            for k in range(37):
                acc = np.float32(acc + np.float32(Af[m, k] * Bf[n, k]))
            assert got[m, n].view(np.uint32) == acc.view(np.uint32)


def test_matmul_f16_vs_float64_library_and_bound():
    A, B = wl.gemm_inputs_f16(20, 24, 300, 85)
    c32 = oracle.matmul_f16(A, B)
    c64, cabs = oracle.matmul_f16_f64(A, B)
    ref = A.view(np.float16).astype(np.float64) @ B.view(np.float16).astype(np.float64).T
    assert np.all(np.abs(ref - c64) <= 1e-13 * cabs)
    assert np.all(np.abs(c32 - c64) <= 300 * 2.0 ** -24 * cabs)
