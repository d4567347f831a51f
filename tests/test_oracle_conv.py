"""Pins for the CPU oracle's conv2d (int8 -> int32 and fp16 -> fp32).

None of these re-type the oracle's gather loop: they use a scatter-form brute
force in pure Python, closed forms, special cases with known answers, a float64
library convolution on integer-valued tensors and an independently written
im2col, chosen so that a dropped term, a flipped kernel, a swapped stride/pad
axis or a transposed operand fails at least one of them.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2101_08458_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def scatter_conv_py(x, w, stride, pad):
    """Pure-Python scatter form: every (input pixel, tap) pair adds into the one
    output it contributes to.  Works on Python ints / floats, arbitrary precision."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    sh, sw = stride
    ph, pw = pad
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    y = [[[[0 for _ in range(Q)] for _ in range(P)] for _ in range(K)] for _ in range(N)]
    for n, c, h, ww in itertools.product(range(N), range(C), range(H), range(W)):
        xv = x[n, c, h, ww].item()
        for r, s in itertools.product(range(R), range(S)):
            # h = p*sh + r - ph  =>  p = (h + ph - r)/sh when divisible
            tp, tq = h + ph - r, ww + pw - s
            if tp % sh or tq % sw:
                continue
            p, q = tp // sh, tq // sw
            if not (0 <= p < P and 0 <= q < Q):
                continue
            for k in range(K):
                y[n][k][p][q] += xv * w[k, c, r, s].item()
    return np.array(y)


def im2col_np(x, R, S, stride, pad):
    """[N,C,H,W] -> [N*P*Q, C*R*S] with numpy slicing (no per-element index math)."""
    N, C, H, W = x.shape
    sh, sw = stride
    ph, pw = pad
    xp = np.zeros((N, C, H + 2 * ph, W + 2 * pw), x.dtype)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    P = (H + 2 * ph - R) // sh + 1
    Q = (W + 2 * pw - S) // sw + 1
    cols = np.empty((N, P, Q, C, R, S), x.dtype)
    for r in range(R):
        for s in range(S):
            cols[:, :, :, :, r, s] = xp[:, :, r:r + sh * (P - 1) + 1:sh,
                                        s:s + sw * (Q - 1) + 1:sw].transpose(0, 2, 3, 1)
    return cols.reshape(N * P * Q, C * R * S), (N, P, Q)


TINY = [
    # N C H W K R S stride pad
    (1, 2, 4, 4, 2, 3, 3, (1, 1), (1, 1)),
    (2, 3, 5, 4, 2, 3, 2, (2, 1), (1, 0)),
    (1, 1, 6, 7, 3, 1, 1, (2, 3), (0, 0)),
    (1, 2, 5, 5, 2, 2, 3, (1, 2), (0, 2)),
    (1, 3, 7, 6, 1, 7, 5, (2, 2), (3, 2)),
]


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", TINY)
def test_conv_i8_brute_force(N, C, H, W, K, R, S, stride, pad):
    g = wl.rng(90, N * 100 + H)
    x = wl.int8_weights(g, (N, C, H, W))
    w = wl.int8_weights(g, (K, C, R, S))
    got = oracle.conv2d_i8(x, w, stride, pad)
    exp = scatter_conv_py(x, w, stride, pad)
    assert got.shape == exp.shape
    assert np.array_equal(got.astype(np.int64), exp)


@pytest.mark.parametrize("shape", [
    (2, 5, 9, 11, 7, 3, 3, (1, 1), (1, 1)),
    (1, 16, 14, 14, 8, 1, 1, (2, 2), (0, 0)),
    (1, 3, 23, 23, 4, 7, 7, (2, 2), (3, 3)),
    (3, 4, 8, 6, 5, 3, 1, (2, 1), (1, 0)),
])
def test_conv_i8_vs_float64_library(shape):
    """torch's CPU double conv is exact on integer-valued tensors (|acc| < 2^53)."""
    N, C, H, W, K, R, S, stride, pad = shape
    g = wl.rng(91, H)
    x = wl.int8_activations(g, (N, C, H, W))
    w = wl.int8_weights(g, (K, C, R, S))
    got = oracle.conv2d_i8(x, w, stride, pad)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)),
                                     torch.from_numpy(w.astype(np.float64)),
                                     stride=stride, padding=pad).numpy()
    assert np.array_equal(got.astype(np.float64), ref)


def test_conv_delta_kernel_is_shift():
    """One tap set to 1: the output is the input shifted by (r-pad, s-pad), zero border."""
    g = wl.rng(92)
    x = wl.int8_activations(g, (1, 3, 6, 5))
    for c0, r0, s0 in [(0, 0, 0), (1, 2, 1), (2, 1, 2), (0, 2, 2)]:
        w = np.zeros((1, 3, 3, 3), np.int8)
        w[0, c0, r0, s0] = 1
        y = oracle.conv2d_i8(x, w, (1, 1), (1, 1))
        exp = np.zeros((6, 5), np.int32)
        for p in range(6):
            for q in range(5):
                h, ww = p + r0 - 1, q + s0 - 1
                if 0 <= h < 6 and 0 <= ww < 5:
                    exp[p, q] = x[0, c0, h, ww]
        assert np.array_equal(y[0, 0], exp)


def test_conv_identity_1x1_and_stride2_subsample():
    g = wl.rng(93)
    x = wl.int8_weights(g, (2, 8, 6, 6))
    w = np.zeros((8, 8, 1, 1), np.int8)
    w[np.arange(8), np.arange(8), 0, 0] = 1
    assert np.array_equal(oracle.conv2d_i8(x, w), x.astype(np.int32))
    assert np.array_equal(oracle.conv2d_i8(x, w, (2, 2)), x[:, :, ::2, ::2].astype(np.int32))
    # a channel permutation instead of the identity: catches a transposed weight index
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    w2 = np.zeros((8, 8, 1, 1), np.int8)
    w2[np.arange(8), perm, 0, 0] = 1            # out channel k reads in channel perm[k]
    assert np.array_equal(oracle.conv2d_i8(x, w2), x[:, perm].astype(np.int32))


@pytest.mark.parametrize("H,W,R,S,stride,pad", [
    (7, 9, 3, 3, (1, 1), (1, 1)), (8, 8, 3, 5, (2, 2), (1, 2)), (10, 6, 7, 1, (2, 1), (3, 0)),
])
def test_conv_all_ones_closed_form(H, W, R, S, stride, pad):
    C = 5
    x = np.ones((1, C, H, W), np.int8)
    w = np.ones((2, C, R, S), np.int8)
    y = oracle.conv2d_i8(x, w, stride, pad)
    P, Q = y.shape[2:]
    cnt_h = [sum(1 for r in range(R) if 0 <= p * stride[0] + r - pad[0] < H) for p in range(P)]
    cnt_w = [sum(1 for s in range(S) if 0 <= q * stride[1] + s - pad[1] < W) for q in range(Q)]
    exp = C * np.outer(cnt_h, cnt_w)
    assert np.array_equal(y[0, 0], exp) and np.array_equal(y[0, 1], exp)


def test_conv_extreme_fill_needs_widening_and_int32():
    """x = w = -128: interior outputs are C*R*S*16384; int16 products would wrap."""
    C, R = 64, 3
    x = np.full((1, C, 5, 5), -128, np.int8)
    w = np.full((1, C, R, R), -128, np.int8)
    y = oracle.conv2d_i8(x, w, (1, 1), (1, 1))
    assert y[0, 0, 2, 2] == C * R * R * 16384
    assert y[0, 0, 0, 0] == C * 4 * 16384
    # the largest reduction any benchmark layer has (512*3*3 = 4608) stays below 2^31
    assert 4608 * 16384 < 2 ** 31 and 131071 * 16384 < 2 ** 31 <= 131073 * 16384


def test_conv_linearity_in_weights():
    g = wl.rng(94)
    x = wl.int8_activations(g, (1, 6, 9, 9))
    w1 = g.integers(-60, 60, size=(4, 6, 3, 3), dtype=np.int8)
    w2 = g.integers(-60, 60, size=(4, 6, 3, 3), dtype=np.int8)
    a = oracle.conv2d_i8(x, (w1 + w2).astype(np.int8), (2, 2), (1, 1))
    b = oracle.conv2d_i8(x, w1, (2, 2), (1, 1)) + oracle.conv2d_i8(x, w2, (2, 2), (1, 1))
    assert np.array_equal(a, b)


@pytest.mark.parametrize("shape", [
    (2, 6, 9, 8, 5, 3, 3, (1, 1), (1, 1)), (1, 4, 11, 11, 3, 3, 3, (2, 2), (1, 1)),
    (1, 8, 7, 7, 4, 1, 1, (2, 2), (0, 0)),
])
def test_conv_equals_im2col_matmul(shape):
    N, C, H, W, K, R, S, stride, pad = shape
    g = wl.rng(95, H)
    x = wl.int8_activations(g, (N, C, H, W))
    w = wl.int8_weights(g, (K, C, R, S))
    cols, (n_, P, Q) = im2col_np(x, R, S, stride, pad)
    direct = oracle.conv2d_i8(x, w, stride, pad)
    # through the oracle's own matmul (consistency of the two definitions) ...
    via_mm = oracle.matmul_i8(np.ascontiguousarray(w.reshape(K, -1)), np.ascontiguousarray(cols))
    assert np.array_equal(direct, via_mm.reshape(K, N, P, Q).transpose(1, 0, 2, 3))
    # ... and through numpy's int64 matmul (library)
    via_np = w.reshape(K, -1).astype(np.int64) @ cols.astype(np.int64).T
    assert np.array_equal(direct.astype(np.int64), via_np.reshape(K, N, P, Q).transpose(1, 0, 2, 3))


def test_output_size_matches_table1():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_conv_layers.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 16
    for (idx, C, ihw, K, R, stride, ohw), sh in zip(rows, wl.TABLE1):
        assert oracle.out_dim(int(ihw), int(R), int(stride), 0) == int(ohw)
        assert (sh.c, sh.h, sh.k, sh.r, sh.stride) == (int(C), int(ihw), int(K), int(R), int(stride))
        assert wl.out_hw(sh) == (int(ohw), int(ohw))
    # floor reading when the stride does not divide: the 7x7/2 stem gives 112
    assert oracle.out_dim(224, 7, 2, 3) == 112


def test_workload_tables():
    layers = wl.resnet50_convs()
    assert len(layers) == 53
    assert len(wl.unique_shapes(layers)) == 23
    assert sum(wl.macs(sh) for sh in layers) == 4087136256
    plan = wl.resnet18_plan()
    convs = [plan["stem"]] + [c for blk in plan["blocks"] for c in blk if c is not None]
    assert len(convs) == 20
    assert sum(wl.macs(sh) for sh in convs) == 1813561344
    assert wl.macs(wl.CONFIG1) == 115605504


# ------------------------------------------------------------------ fp16 path

def test_half_decode_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", TINY[:4])
def test_conv_f16_brute_force_order(N, C, H, W, K, R, S, stride, pad):
    """fp32 accumulation in c -> r -> s order, written as a pure-Python gather with
    numpy float32 scalars (products of binary16 values are exact in fp32)."""
    g = wl.rng(96, H)
    x = wl.f16_activations(g, (N, C, H, W))
    w = wl.f16_activations(g, (K, C, R, S))
    got = oracle.conv2d_f16(x, w, stride, pad)
    xf, wf = x.view(np.float16).astype(np.float32), w.view(np.float16).astype(np.float32)
    P, Q = got.shape[2:]
    for n, k, p, q in itertools.product(range(N), range(K), range(P), range(Q)):
        acc = np.float32(0)
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            h, ww = p * stride[0] + r - pad[0], q * stride[1] + s - pad[1]
            if 0 <= h < H and 0 <= ww < W:
                acc = np.float32(acc + np.float32(xf[n, c, h, ww] * wf[k, c, r, s]))
        assert got[n, k, p, q].view(np.uint32) == acc.view(np.uint32)


def test_conv_f16_order_sensitive_case():
    """2048 + 1 + 1 in fp32 is exact, but a case built so that only the c -> r -> s
    order gives the stated answer: 2^24 + 1 - 2^24 + 1."""
    x = wl.f16_bits(np.array([[[[4096.0, 1.0]], [[4096.0, 1.0]]]]))       # [1,2,1,2]
    w = wl.f16_bits(np.array([[[[4096.0, 1.0]], [[-4096.0, 1.0]]]]))      # [1,2,1,2]
    y = oracle.conv2d_f16(x, w)
    # order: c0s0 (+2^24), c0s1 (+1 -> lost: 2^24+1 rounds to 2^24), c1s0 (-2^24), c1s1 (+1) = 1
    assert y.shape == (1, 1, 1, 1) and y[0, 0, 0, 0] == 1.0
    yt, ya = oracle.conv2d_f16_f64(x, w)
    assert yt[0, 0, 0, 0] == 2.0 and ya[0, 0, 0, 0] == 2.0 ** 25 + 2


def test_conv_f16_power_of_two_inputs_are_exact():
    g = wl.rng(97)
    ex = g.integers(-3, 4, size=(1, 8, 7, 7))
    ew = g.integers(-3, 4, size=(4, 8, 3, 3))
    sx = g.choice([-1.0, 1.0], size=ex.shape)
    sw = g.choice([-1.0, 1.0], size=ew.shape)
    x, w = wl.f16_bits(sx * 2.0 ** ex), wl.f16_bits(sw * 2.0 ** ew)
    y32 = oracle.conv2d_f16(x, w, (1, 1), (1, 1))
    y64, _ = oracle.conv2d_f16_f64(x, w, (1, 1), (1, 1))
    assert np.array_equal(y32.astype(np.float64), y64)


def test_conv_f16_within_summation_bound_and_vs_library():
    sh = wl.conv_shape(16, 12, 8, 3, 1, 1)
    x, w = wl.conv_inputs_f16(sh, 2, 98)
    y32 = oracle.conv2d_f16(x, w, (1, 1), (1, 1))
    y64, yabs = oracle.conv2d_f16_f64(x, w, (1, 1), (1, 1))
    kred = sh.c * sh.r * sh.s
    assert np.all(np.abs(y32 - y64) <= kred * 2.0 ** -24 * yabs + 1e-30)
    ref = torch.nn.functional.conv2d(
        torch.from_numpy(x.view(np.float16).astype(np.float64)),
        torch.from_numpy(w.view(np.float16).astype(np.float64)), padding=1).numpy()
    assert np.all(np.abs(ref - y64) <= 1e-13 * yabs + 1e-300)


def test_conv_f16_subnormal_inputs_honoured():
    x = np.full((1, 4, 3, 3), 0x0001, np.uint16)          # 2^-24, smallest subnormal
    w = wl.f16_bits(np.full((1, 4, 1, 1), 1024.0))
    y = oracle.conv2d_f16(x, w)
    assert np.all(y == 4 * 1024.0 * 2.0 ** -24)


# ------------------------------------------------------------------ pooling glue

def test_maxpool_vs_library():
    g = wl.rng(99)
    x = wl.int8_weights(g, (2, 5, 11, 12))
    got = oracle.maxpool_i8(x)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)), 3, 2, 1).numpy()
    assert np.array_equal(got.astype(np.float32), ref)
    # all-negative input: padded positions must not win with an implicit 0
    xn = np.full((1, 1, 4, 4), -7, np.int8)
    assert np.all(oracle.maxpool_i8(xn) == -7)


def test_global_sumpool_requant():
    g = wl.rng(100)
    x = wl.int8_weights(g, (2, 6, 7, 7))
    scale = np.full((6,), 1.0 / 64.0, np.float32)     # power of two: exact product
    got = oracle.global_sumpool_requant_i8(x, scale)
    sums = x.astype(np.int64).sum(axis=(2, 3))
    exp = np.clip(np.array([[round(int(v) / 64) for v in row] for row in sums]), -128, 127)
    assert np.array_equal(got.astype(np.int64), exp)


def test_widen_scale():
    x = np.array([-128, -1, 0, 127], np.int8)
    assert np.array_equal(oracle.widen_scale_i8(x, 256), np.array([-32768, -256, 0, 32512], np.int32))
