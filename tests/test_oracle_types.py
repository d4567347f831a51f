"""Pins for the oracle's further operand types (u8 x i8 -> i32, bf16 x bf16 -> f32).

Same definitions as the int8 / binary16 functions with another element decoding, so the pins
are: the decoding against the format's definition, agreement with the already pinned functions
wherever the value sets overlap, float64 library contractions, and the offset identity
sum u*w = sum (u-128)*w + 128*sum w that ties the unsigned form to the signed one.
"""
import numpy as np
import pytest

import oracle
from paper_2101_08458_amd import workloads as wl


def test_bf16_decoding_all_patterns():
    bits = np.arange(65536, dtype=np.uint32)
    want = (bits << 16).view(np.float32)
    for b in list(range(0, 65536, 97)) + [0x0001, 0x007F, 0x0080, 0x7F7F, 0x7F80, 0x7FC0, 0x8000, 0xFF80, 0x3F80]:
        got = np.float32(oracle.bf16_to_float(b))
        assert got.view(np.uint32) == want[b].view(np.uint32) or (np.isnan(got) and np.isnan(want[b]))
    assert oracle.bf16_to_float(0x3F80) == 1.0 and oracle.bf16_to_float(0xC000) == -2.0
    assert oracle.bf16_to_float(0x3F81) == 1.0 + 2.0 ** -7          # 7 fraction bits


def test_bf16_rounding_of_generator():
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -0.3, 1e-3, 65504.0], np.float32)
    bits = wl.bf16_bits(vals)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2.0 ** -6      # ties to even
    assert np.all(np.abs(back - vals) <= np.abs(vals) * 2.0 ** -8)


@pytest.mark.parametrize("stride,pad", [((1, 1), (1, 1)), ((2, 2), (0, 0)), ((2, 1), (2, 1))])
def test_u8i8_conv(stride, pad):
    g = np.random.default_rng(31)
    x = wl.uint8_activations(g, (2, 5, 9, 8))
    w = wl.int8_weights(g, (4, 5, 3, 3))
    got = oracle.conv2d_u8i8(x, w, stride, pad)
    # offset identity: the unsigned conv is the signed conv of (x - 128) plus 128 times the
    # conv of an all-ones image (zero padded) -- ties it to the pinned int8 function
    xs = (x.astype(np.int16) - 128).astype(np.int8)
    ones = np.ones_like(xs)
    want = oracle.conv2d_i8(xs, w, stride, pad) + 128 * oracle.conv2d_i8(ones, w, stride, pad)
    assert np.array_equal(got, want)
    # float64 library contraction over explicit patches
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (pad[0], pad[0]), (pad[1], pad[1])))
    P, Q = got.shape[2:]
    ref = np.zeros(got.shape)
    for p in range(P):
        for q in range(Q):
            patch = xp[:, :, p * stride[0]:p * stride[0] + 3, q * stride[1]:q * stride[1] + 3]
            ref[:, :, p, q] = np.einsum("ncrs,kcrs->nk", patch, w.astype(np.float64))
    assert np.array_equal(got, ref.astype(np.int64))


def test_u8i8_small_values_equal_signed():
    g = np.random.default_rng(32)
    x = g.integers(0, 128, size=(1, 7, 6, 6), dtype=np.int64)
    w = wl.int8_weights(g, (3, 7, 3, 3))
    a = oracle.conv2d_u8i8(x.astype(np.uint8), w, (1, 1), (1, 1))
    b = oracle.conv2d_i8(x.astype(np.int8), w, (1, 1), (1, 1))
    assert np.array_equal(a, b)
    A = g.integers(0, 128, size=(5, 33), dtype=np.int64)
    B = wl.int8_weights(g, (4, 33))
    assert np.array_equal(oracle.matmul_u8i8(A.astype(np.uint8), B), oracle.matmul_i8(A.astype(np.int8), B))


def test_u8i8_matmul_extremes():
    K = 300
    A = np.full((2, K), 255, np.uint8)
    B = np.stack([np.full(K, -128, np.int8), np.full(K, 127, np.int8)])
    C = oracle.matmul_u8i8(A, B)
    assert C[0, 0] == -255 * 128 * K and C[0, 1] == 255 * 127 * K
    g = np.random.default_rng(33)
    A = wl.uint8_activations(g, (9, 70))
    B = wl.int8_weights(g, (6, 70))
    assert np.array_equal(oracle.matmul_u8i8(A, B), A.astype(np.int64) @ B.astype(np.int64).T)
    # operands are not interchangeable: the first is the unsigned one
    assert oracle.matmul_u8i8(np.array([[200]], np.uint8), np.array([[-3]], np.int8))[0, 0] == -600


def test_bf16_integer_valued_inputs_are_exact():
    # small integers are bf16 values and all partial sums stay below 2^24: fp32 accumulation is
    # exact and must equal the integer function bit for bit
    g = np.random.default_rng(34)
    xi = g.integers(-8, 9, size=(2, 6, 7, 7)).astype(np.int8)
    wi = g.integers(-8, 9, size=(5, 6, 3, 3)).astype(np.int8)
    y, y64, ya = oracle.conv2d_bf16(wl.bf16_bits(xi.astype(np.float32)), wl.bf16_bits(wi.astype(np.float32)),
                                    (1, 1), (1, 1))
    ref = oracle.conv2d_i8(xi, wi, (1, 1), (1, 1))
    assert np.array_equal(y, ref.astype(np.float32)) and np.array_equal(y64, ref.astype(np.float64))
    yabs_ref = oracle.conv2d_i8(np.abs(xi), np.abs(wi), (1, 1), (1, 1))
    assert np.array_equal(ya, yabs_ref.astype(np.float64))
    Ai = g.integers(-8, 9, size=(7, 40)).astype(np.int8)
    Bi = g.integers(-8, 9, size=(5, 40)).astype(np.int8)
    C, C64, Ca = oracle.matmul_bf16(wl.bf16_bits(Ai.astype(np.float32)), wl.bf16_bits(Bi.astype(np.float32)))
    assert np.array_equal(C, oracle.matmul_i8(Ai, Bi).astype(np.float32))
    assert np.array_equal(C64, (Ai.astype(np.int64) @ Bi.astype(np.int64).T).astype(np.float64))


def test_bf16_general_values():
    sh = wl.conv_shape(12, 9, 7, 3, 2, 1)
    x, w = wl.conv_inputs_bf16(sh, 2, 9, 1)
    y, y64, ya = oracle.conv2d_bf16(x, w, (2, 2), (1, 1))
    xf = (x.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    wf = (w.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    xp = np.pad(xf, ((0, 0), (0, 0), (1, 1), (1, 1)))
    P, Q = y.shape[2:]
    ref = np.zeros(y.shape)
    for p in range(P):
        for q in range(Q):
            ref[:, :, p, q] = np.einsum("ncrs,kcrs->nk", xp[:, :, 2 * p:2 * p + 3, 2 * q:2 * q + 3], wf)
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-12)
    kred = 12 * 9
    assert np.all(np.abs(y - y64) <= kred * 2.0 ** -24 * ya + 1e-30)
    A, B = wl.gemm_inputs_bf16(6, 5, 200)
    C, C64, Ca = oracle.matmul_bf16(A, B)
    Af = (A.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    Bf = (B.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.allclose(C64, Af @ Bf.T, rtol=1e-12, atol=1e-12)
    assert np.all(np.abs(C - C64) <= 200 * 2.0 ** -24 * Ca)
    # sequential order of the fp32 sum (not pairwise, not reversed)
    acc = np.float32(0)
    af, bf = Af[0].astype(np.float32), Bf[0].astype(np.float32)
    for k in range(200):
        acc = np.float32(acc + np.float32(af[k] * bf[k]))
    assert C[0, 0] == acc


# ------------------------------------------------------------------ fp8 (E4M3, finite-only)

def test_fp8_decoding_all_patterns():
    import torch
    bits = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(bits.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    for b in range(256):
        got = oracle.fp8_e4m3_to_float(b)
        assert (np.isnan(got) and np.isnan(lib[b])) or got == lib[b], b
    # the format's landmarks
    assert oracle.fp8_e4m3_to_float(0x7E) == 448.0 and oracle.fp8_e4m3_to_float(0xFE) == -448.0
    assert oracle.fp8_e4m3_to_float(0x38) == 1.0 and oracle.fp8_e4m3_to_float(0x01) == 2.0 ** -9
    assert oracle.fp8_e4m3_to_float(0x08) == 2.0 ** -6 and np.isnan(oracle.fp8_e4m3_to_float(0x7F))


def test_fp8_generator_rounding():
    import torch
    g = np.random.default_rng(35)
    vals = np.concatenate([g.standard_normal(4000) * 3, g.standard_normal(2000) * 0.01,
                           [0.0, 448.0, 1000.0, -1000.0, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, 1.1875]])
    bits = wl.fp8_e4m3_bits(vals)
    inside = np.abs(vals) <= 448
    lib = torch.from_numpy(vals[inside].astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(bits[inside], lib)
    assert bits[-7] == 0x7E and bits[-6] == 0x7E and bits[-5] == 0xFE     # saturation
    assert bits[-4] == 0x00 and bits[-3] == 0x02                           # ties to even among subnormals
    assert bits[-2] == 0x38 and bits[-1] == 0x3A                           # 1.0625 -> 1.0, 1.1875 -> 1.25


def test_fp8_integer_valued_inputs_are_exact():
    g = np.random.default_rng(36)
    xi = g.integers(-8, 9, size=(2, 6, 7, 7)).astype(np.int8)
    wi = g.integers(-8, 9, size=(5, 6, 3, 3)).astype(np.int8)
    y, y64, ya = oracle.conv2d_fp8(wl.fp8_e4m3_bits(xi), wl.fp8_e4m3_bits(wi), (1, 1), (1, 1))
    ref = oracle.conv2d_i8(xi, wi, (1, 1), (1, 1))
    assert np.array_equal(y, ref.astype(np.float32)) and np.array_equal(y64, ref.astype(np.float64))
    assert np.array_equal(ya, oracle.conv2d_i8(np.abs(xi), np.abs(wi), (1, 1), (1, 1)).astype(np.float64))
    Ai = g.integers(-8, 9, size=(7, 40)).astype(np.int8)
    Bi = g.integers(-8, 9, size=(5, 40)).astype(np.int8)
    C, C64, Ca = oracle.matmul_fp8(wl.fp8_e4m3_bits(Ai), wl.fp8_e4m3_bits(Bi))
    assert np.array_equal(C, oracle.matmul_i8(Ai, Bi).astype(np.float32))


def test_fp8_general_values():
    import torch
    A, B = wl.gemm_inputs_fp8(6, 5, 200)
    C, C64, Ca = oracle.matmul_fp8(A, B)
    Af = torch.from_numpy(A.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    Bf = torch.from_numpy(B.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.allclose(C64, Af @ Bf.T, rtol=1e-12, atol=1e-12)
    assert np.allclose(Ca, np.abs(Af) @ np.abs(Bf).T, rtol=1e-12, atol=1e-12)
    assert np.all(np.abs(C - C64) <= 200 * 2.0 ** -24 * Ca)
    acc = np.float32(0)
    for k in range(200):
        acc = np.float32(acc + np.float32(Af[0, k]) * np.float32(Bf[0, k]))
    assert C[0, 0] == acc
    sh = wl.conv_shape(10, 8, 6, 3, 2, 1)
    x, w = wl.conv_inputs_fp8(sh, 2, 9, 2)
    y, y64, ya = oracle.conv2d_fp8(x, w, (2, 2), (1, 1))
    xf = torch.from_numpy(x.copy()).view(torch.float8_e4m3fn).to(torch.float64)
    wf = torch.from_numpy(w.copy()).view(torch.float8_e4m3fn).to(torch.float64)
    ref = torch.nn.functional.conv2d(xf, wf, stride=2, padding=1).numpy()
    assert np.allclose(y64, ref, rtol=1e-12, atol=1e-12)
