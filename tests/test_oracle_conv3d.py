"""Pins for the oracle's conv3d (the paper's extensibility experiment, Section VI-C)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2101_08458_amd import workloads as wl

CASES = [
    # N C D H W K T R S stride pad
    (1, 2, 3, 4, 4, 2, 3, 3, 3, (1, 1, 1), (1, 1, 1)),
    (2, 3, 4, 5, 3, 2, 2, 3, 1, (2, 1, 1), (1, 0, 0)),
    (1, 2, 5, 4, 6, 3, 1, 1, 1, (2, 2, 3), (0, 0, 0)),
    (1, 1, 4, 5, 5, 2, 3, 2, 3, (1, 2, 1), (2, 0, 1)),
]


def scatter3d_py(x, w, stride, pad):
    N, C, D, H, W = x.shape
    K, _, T, R, S = w.shape
    O = (D + 2 * pad[0] - T) // stride[0] + 1
    P = (H + 2 * pad[1] - R) // stride[1] + 1
    Q = (W + 2 * pad[2] - S) // stride[2] + 1
    y = np.zeros((N, K, O, P, Q), dtype=object)
    for n, c, d, h, ww in itertools.product(range(N), range(C), range(D), range(H), range(W)):
        xv = int(x[n, c, d, h, ww])
        for t, r, s in itertools.product(range(T), range(R), range(S)):
            a, b, e = d + pad[0] - t, h + pad[1] - r, ww + pad[2] - s
            if a % stride[0] or b % stride[1] or e % stride[2]:
                continue
            o, p, q = a // stride[0], b // stride[1], e // stride[2]
            if 0 <= o < O and 0 <= p < P and 0 <= q < Q:
                for k in range(K):
                    y[n, k, o, p, q] += xv * int(w[k, c, t, r, s])
    return y.astype(np.int64)


@pytest.mark.parametrize("N,C,D,H,W,K,T,R,S,stride,pad", CASES)
def test_conv3d_i8_brute_force_and_library(N, C, D, H, W, K, T, R, S, stride, pad):
    g = wl.rng(110, D * 10 + H)
    x = wl.int8_weights(g, (N, C, D, H, W))
    w = wl.int8_weights(g, (K, C, T, R, S))
    got = oracle.conv3d_i8(x, w, stride, pad)
    assert np.array_equal(got.astype(np.int64), scatter3d_py(x, w, stride, pad))
    ref = torch.nn.functional.conv3d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                     stride=stride, padding=pad).numpy()
    assert np.array_equal(got.astype(np.float64), ref)


def test_conv3d_depth_one_is_conv2d():
    g = wl.rng(111)
    x = wl.int8_activations(g, (2, 5, 9, 8))
    w = wl.int8_weights(g, (4, 5, 3, 3))
    y2 = oracle.conv2d_i8(x, w, (2, 1), (1, 1))
    y3 = oracle.conv3d_i8(np.ascontiguousarray(x[:, :, None]), np.ascontiguousarray(w[:, :, None]), (1, 2, 1), (0, 1, 1))
    assert np.array_equal(y3[:, :, 0], y2)
    # a kernel that is 1 only at depth tap t0 selects input slice o + t0 - pad
    x3 = wl.int8_activations(g, (1, 3, 6, 5, 5))
    w3 = np.zeros((2, 3, 3, 3, 3), np.int8)
    w2 = wl.int8_weights(g, (2, 3, 3, 3))
    w3[:, :, 2] = w2
    y = oracle.conv3d_i8(x3, w3, (1, 1, 1), (1, 1, 1))
    for o in range(6):
        d = o + 2 - 1
        exp = oracle.conv2d_i8(np.ascontiguousarray(x3[:, :, d]), w2, (1, 1), (1, 1)) if d < 6 else 0
        assert np.array_equal(y[:, :, o], exp if d < 6 else np.zeros_like(y[:, :, o]))


def test_conv3d_f16_order_bound_and_library():
    g = wl.rng(112)
    x = wl.f16_activations(g, (1, 6, 4, 7, 6))
    w = wl.f16_weights(g, (5, 6, 3, 3, 3), 6 * 27)
    y, y64, ya = oracle.conv3d_f16(x, w, (1, 1, 1), (1, 1, 1))
    ref = torch.nn.functional.conv3d(torch.from_numpy(x.view(np.float16).astype(np.float64)),
                                     torch.from_numpy(w.view(np.float16).astype(np.float64)), padding=1).numpy()
    assert np.all(np.abs(ref - y64) <= 1e-13 * ya + 1e-300)
    assert np.all(np.abs(y - y64) <= 6 * 27 * 2.0 ** -24 * ya + 1e-30)
    # sequential fp32 order c -> t -> r -> s, checked on a few outputs with numpy float32 scalars
    xf, wf = x.view(np.float16).astype(np.float32), w.view(np.float16).astype(np.float32)
    for (k, o, p, q) in [(0, 0, 0, 0), (2, 1, 3, 2), (4, 3, 6, 5)]:
        acc = np.float32(0)
        for c, t, r, s in itertools.product(range(6), range(3), range(3), range(3)):
            d, h, ww = o + t - 1, p + r - 1, q + s - 1
            if 0 <= d < 4 and 0 <= h < 7 and 0 <= ww < 6:
                acc = np.float32(acc + np.float32(xf[0, c, d, h, ww] * wf[k, c, t, r, s]))
        assert y[0, k, o, p, q].view(np.uint32) == acc.view(np.uint32)
