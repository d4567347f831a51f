"""GPU parity: libunit (through its C ABI) against the CPU oracle on identical seeded inputs.

int8 paths must be bit-exact; fp16 paths must have max relative error <= 1e-3 (relative to
max(|ref|, 1e-3*rms(ref))) and stay inside the fp32 summation bound 2*K*2^-24*sum|x||w|.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2101_08458_amd import unit, workloads as wl
from gpu_util import announce, dev, host, forced, f16_rel_err, as_accurate_as_oracle, same

pytestmark = pytest.mark.gpu

ALL_TILES = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12]


def ws_bytes(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0")


# ------------------------------------------------------------------ matmul

def run_matmul_i8(A, B, lda=None, ldb=None, ldc=None):
    M, K = A.shape
    N = B.shape[0]
    lda, ldb, ldc = lda or K, ldb or K, ldc or N
    Ap = np.zeros((M, lda), np.int8); Ap[:, :K] = A
    Bp = np.zeros((N, ldb), np.int8); Bp[:, :K] = B
    Ad, Bd = dev(Ap), dev(Bp)
    C = torch.full((M, ldc), -7, dtype=torch.int32, device="cuda:0")
    ws = ws_bytes(unit.unit_matmul_workspace(M, N, K, lda, ldb, unit.UNIT_I8))
    unit.unit_matmul_i8(M, N, K, Ad, lda, Bd, ldb, C, ldc, ws)
    torch.cuda.synchronize()
    return host(C)[:, :N]


def run_matmul_f16(A, B):
    M, K = A.shape
    N = B.shape[0]
    Ad, Bd = dev(A), dev(B)
    C = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    ws = ws_bytes(unit.unit_matmul_workspace(M, N, K, K, K, unit.UNIT_F16))
    unit.unit_matmul_f16(M, N, K, Ad, K, Bd, K, C, N, ws)
    torch.cuda.synchronize()
    return host(C)


def test_mfma_fragment_layout_probe():
    """Index-revealing operands: C[m,n] = 64*m + n needs the lane -> (row, col) mapping of
    the accumulator fragments to be exactly as the epilogue assumes, for every tile shape."""
    for M, N in [(32, 32), (64, 96), (16, 64)]:
        K = 64
        A = np.zeros((M, K), np.int8); A[:, 0] = np.arange(M) % 64; A[:, 1] = 1
        B = np.zeros((N, K), np.int8); B[:, 0] = 64; B[:, 1] = np.arange(N)
        # C[m,n] = 64*(m%64) + n
        exp = 64 * (np.arange(M) % 64)[:, None] + np.arange(N)[None, :]
        for tile in ALL_TILES:
            announce("layout probe", M, N, "tile", tile)
            with forced(tile=tile, split=1):
                got = run_matmul_i8(A, B)
            assert same(got, exp), f"tile {tile} M={M} N={N}"


@pytest.mark.parametrize("M,N,K", [(16, 16, 16), (64, 64, 64), (100, 100, 100), (257, 130, 384),
                                   (1, 1000, 2048), (3, 7, 5), (300, 40, 1040)])
def test_matmul_i8_parity(M, N, K):
    A, B = wl.gemm_inputs_i8(M, N, K, 20, M + K)
    ref = oracle.matmul_i8(A, B)
    announce("matmul_i8", M, N, K, "auto")
    assert same(run_matmul_i8(A, B), ref)
    for tile in ALL_TILES:
        for split in (1, 3):
            announce("matmul_i8", M, N, K, "tile", tile, "split", split)
            with forced(tile=tile, split=split):
                assert same(run_matmul_i8(A, B), ref), (tile, split)


def test_matmul_i8_leading_dimensions():
    A, B = wl.gemm_inputs_i8(70, 50, 96, 21)
    ref = oracle.matmul_i8(A, B)
    announce("matmul_i8 ld aligned")
    assert same(run_matmul_i8(A, B, lda=128, ldb=112, ldc=64), ref)
    announce("matmul_i8 ld unaligned")
    assert same(run_matmul_i8(A, B, lda=101, ldb=97, ldc=51), ref)


def test_matmul_i8_extremes_and_identity():
    K = 4096
    A = np.full((33, K), -128, np.int8)
    B = np.full((17, K), -128, np.int8)
    announce("matmul_i8 extreme fill")
    assert np.all(run_matmul_i8(A, B) == K * 16384)
    g = wl.rng(22)
    Bm = wl.int8_weights(g, (48, 64))
    announce("matmul_i8 identity")
    assert same(run_matmul_i8(np.eye(64, dtype=np.int8), Bm), Bm.T.astype(np.int32))


@pytest.mark.parametrize("M,N,K", [(16, 16, 16), (100, 100, 100), (257, 130, 392), (2, 1000, 512)])
def test_matmul_f16_parity(M, N, K):
    A, B = wl.gemm_inputs_f16(M, N, K, 23, M + K)
    ref = oracle.matmul_f16(A, B)
    truth, mag = oracle.matmul_f16_f64(A, B)
    for tile, split in [(None, None)] + [(t, s) for t in ALL_TILES for s in (1, 2)]:
        announce("matmul_f16", M, N, K, "tile", tile, "split", split)
        with forced(tile=tile, split=split):
            got = run_matmul_f16(A, B)
        assert f16_rel_err(got, ref, K) <= 1e-3, (tile, split)
        assert np.all(np.abs(got - truth) <= 2 * K * 2.0 ** -24 * mag + 1e-30), (tile, split)
        assert as_accurate_as_oracle(got, ref, truth), (tile, split)


def test_matmul_f16_exact_cases():
    """Small integers: every partial sum is exact, so any summation order gives the same bits."""
    g = wl.rng(24)
    Ai = g.integers(-8, 9, size=(70, 200))
    Bi = g.integers(-8, 9, size=(90, 200))
    announce("matmul_f16 exact ints")
    got = run_matmul_f16(wl.f16_bits(Ai), wl.f16_bits(Bi))
    assert same(got.astype(np.int64), Ai @ Bi.T)
    # subnormal inputs must not be flushed: 2^-24 * 1024 * K
    A = np.full((16, 64), 0x0001, np.uint16)
    B = wl.f16_bits(np.full((16, 64), 1024.0))
    announce("matmul_f16 subnormal")
    got = run_matmul_f16(A, B)
    assert np.all(got == 64 * 1024.0 * 2.0 ** -24)


def test_matmul_i8_full_size_sampled():
    """4096^3 in the launch configuration the benchmark times; sampled rows and columns."""
    M = N = K = 4096
    A, B = wl.gemm_inputs_i8(M, N, K)
    announce("matmul_i8 4096^3")
    got = run_matmul_i8(A, B)
    g = wl.rng(25)
    rows = np.unique(np.concatenate([[0, 255, 256, 4095], g.integers(0, M, 12)]))
    cols = np.unique(np.concatenate([[0, 255, 256, 4095], g.integers(0, N, 12)]))
    assert same(got[rows], oracle.matmul_i8(np.ascontiguousarray(A[rows]), B))
    assert same(got[:, cols], oracle.matmul_i8(A, np.ascontiguousarray(B[cols])))
    # property that holds at any size: row sums of C equal A times the column-sum vector of B
    colsum = B.astype(np.int64).sum(axis=0)
    assert same(got.astype(np.int64).sum(axis=1), A.astype(np.int64) @ colsum)


def test_matmul_f16_full_size_sampled():
    M = N = K = 4096
    A, B = wl.gemm_inputs_f16(M, N, K)
    announce("matmul_f16 4096^3")
    got = run_matmul_f16(A, B)
    g = wl.rng(26)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 2047, 4095], g.integers(0, M, 12)]))
    cols = np.unique(np.concatenate([[0, 255, 256, 4095], g.integers(0, N, 12)]))
    for sel, Asel, Bsel in ((np.s_[rows], np.ascontiguousarray(A[rows]), B),
                            (np.s_[:, cols], A, np.ascontiguousarray(B[cols]))):
        ref = oracle.matmul_f16(Asel, Bsel)
        truth, mag = oracle.matmul_f16_f64(Asel, Bsel)
        assert f16_rel_err(got[sel], ref, K) <= 1e-3
        assert np.all(np.abs(got[sel] - truth) <= 2 * K * 2.0 ** -24 * mag)
        assert as_accurate_as_oracle(got[sel], ref, truth)


# ------------------------------------------------------------------ conv2d

def run_conv_i8(sh, n, x, w, rq=None):
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
    p, q = unit.unit_conv2d_out_dims(d)
    ws = ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8))
    xd, wd = dev(x), dev(w)
    y32 = torch.full((n, sh.k, p, q), -7, dtype=torch.int32, device="cuda:0")
    unit.unit_conv2d_i8(d, xd, wd, y32, None, None, ws)
    torch.cuda.synchronize()
    return host(y32)


def run_conv_f16(sh, n, x, w):
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
    p, q = unit.unit_conv2d_out_dims(d)
    ws = ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_F16))
    y = torch.empty((n, sh.k, p, q), dtype=torch.float32, device="cuda:0")
    unit.unit_conv2d_f16(d, dev(x), dev(w), y, ws)
    torch.cuda.synchronize()
    return host(y)


SMALL_CONVS = [
    (wl.ConvShape(2, 4, 4, 2, 3, 3, 1, 1), 1),
    (wl.ConvShape(3, 9, 11, 5, 3, 3, 2, 1), 2),
    (wl.ConvShape(20, 13, 9, 33, 1, 1, 1, 0), 3),
    (wl.ConvShape(16, 14, 14, 8, 1, 1, 2, 0), 1),
    (wl.ConvShape(3, 23, 23, 4, 7, 7, 2, 3), 1),
    (wl.ConvShape(40, 10, 12, 70, 3, 3, 1, 1), 2),
    (wl.ConvShape(70, 17, 17, 130, 3, 3, 2, 1), 1),
]


@pytest.mark.parametrize("sh,n", SMALL_CONVS)
def test_conv_i8_small_all_tiles(sh, n):
    x, w = wl.conv_inputs_i8(sh, n, 30, sh.c)
    ref = oracle.conv2d_i8(x, w, (sh.stride,) * 2, (sh.pad,) * 2)
    announce("conv_i8", sh, n, "auto")
    assert same(run_conv_i8(sh, n, x, w), ref)
    for tile in ALL_TILES:
        for split in (1, 2):
            announce("conv_i8", sh, n, "tile", tile, "split", split)
            with forced(tile=tile, split=split):
                assert same(run_conv_i8(sh, n, x, w), ref), (tile, split)


NCHW_DIRECT = [   # 1x1 / stride 1: read straight from NCHW, whatever the alignment of the channel rows
    (wl.ConvShape(20, 14, 14, 33, 1, 1, 1, 0), 1), (wl.ConvShape(64, 56, 56, 64, 1, 1, 1, 0), 1),
    (wl.ConvShape(70, 10, 10, 130, 1, 1, 1, 0), 1), (wl.ConvShape(256, 6, 6, 40, 1, 1, 1, 0), 1),
    (wl.ConvShape(3, 18, 18, 5, 1, 1, 1, 0), 1),
    (wl.ConvShape(130, 7, 7, 64, 1, 1, 1, 0), 1),      # 49 pixels: channel rows at odd byte offsets
    (wl.ConvShape(37, 3, 5, 20, 1, 1, 1, 0), 1),       # 15 pixels: less than one chunk per row
    (wl.ConvShape(48, 7, 7, 33, 1, 1, 1, 0), 3),       # several images of 49 pixels: per-image tiles, odd offsets
    (wl.ConvShape(24, 8, 8, 40, 1, 1, 1, 0), 3),       # several images, 64 pixels each: direct
    (wl.ConvShape(72, 12, 4, 96, 1, 1, 1, 0), 5),      # 48 pixels per image: direct, tiles straddle images
    (wl.ConvShape(16, 14, 14, 24, 1, 1, 1, 0), 2),     # 196 pixels per image, n > 1: columns tiled per image
    (wl.ConvShape(40, 6, 6, 24, 1, 1, 1, 0), 5),       # 36 pixels per image: per-image tiles, mostly empty
    (wl.ConvShape(256, 14, 14, 70, 1, 1, 1, 0), 3),    # several reduction steps, per-image tiles
    (wl.ConvShape(32, 5, 10, 16, 1, 1, 1, 0), 4),      # 50 pixels per image
    # rows that are not dword-aligned with whole steps of channels: read directly, the chunk that crosses the
    # tensor's end is patched (one-byte types need 128 channels per step, two-byte types 64; the 256-byte-step
    # tile twice as many)
    (wl.ConvShape(128, 7, 7, 40, 1, 1, 1, 0), 1), (wl.ConvShape(256, 5, 5, 33, 1, 1, 1, 0), 3),
    (wl.ConvShape(128, 3, 11, 24, 1, 1, 1, 0), 2), (wl.ConvShape(64, 7, 7, 40, 1, 1, 1, 0), 1),
    (wl.ConvShape(512, 9, 9, 72, 1, 1, 1, 0), 2), (wl.ConvShape(256, 7, 7, 16, 1, 1, 1, 0), 1),
]


@pytest.mark.parametrize("sh,n", NCHW_DIRECT)
def test_conv_wpacked_nchw_direct(sh, n):
    """Pre-packed weights + NCHW activations, the per-layer call the benchmark times."""
    st, pd = (1, 1), (0, 0)
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, 1, 1, 1, 0)
    x, w = wl.conv_inputs_i8(sh, n, 32, sh.c)
    ref = oracle.conv2d_i8(x, w, st, pd)
    xh, wh = wl.conv_inputs_f16(sh, n, 33, sh.c)
    refh = oracle.conv2d_f16(xh, wh, st, pd)
    truth, mag = oracle.conv2d_f16_f64(xh, wh, st, pd)
    xd, xhd = dev(x), dev(xh)
    wp = ws_bytes(unit.unit_packed_weights_bytes(d, unit.UNIT_I8))
    wph = ws_bytes(unit.unit_packed_weights_bytes(d, unit.UNIT_F16))
    unit.unit_pack_weights_i8(d, dev(w), wp)
    unit.unit_pack_weights_f16(d, dev(wh), wph)
    for tile, split in [(None, None)] + [(t, s) for t in ALL_TILES for s in (1, 2)]:
        announce("wpacked", sh, n, "tile", tile, "split", split)
        with forced(tile=tile, split=split):
            y = torch.full((n, sh.k, sh.h, sh.w), -7, dtype=torch.int32, device="cuda:0")
            unit.unit_conv2d_wpacked_i8(d, xd, wp, y, None, None, ws_bytes(unit.unit_conv2d_wpacked_workspace(d, unit.UNIT_I8)))
            yh = torch.empty((n, sh.k, sh.h, sh.w), dtype=torch.float32, device="cuda:0")
            unit.unit_conv2d_wpacked_f16(d, xhd, wph, yh, ws_bytes(unit.unit_conv2d_wpacked_workspace(d, unit.UNIT_F16)))
            torch.cuda.synchronize()
        assert same(host(y), ref, f"i8 tile {tile} split {split}")
        got = host(yh)
        assert f16_rel_err(got, refh, sh.c) <= 1e-3, (tile, split)
        assert np.all(np.abs(got - truth) <= 2 * sh.c * 2.0 ** -24 * mag + 1e-30), (tile, split)
        assert as_accurate_as_oracle(got, refh, truth), (tile, split)


def test_conv_i8_more_than_four_million_columns():
    """Column indices beyond 2^22: the kernels' index divisions (pixel -> image / row / column, tile coordinates)
    must be exact over the whole 31-bit range, not only where a float reciprocal would do.  Two images of
    1450 x 1450 pixels give 4 205 000 output columns; a 1x1 conv reads them directly from NCHW, a 3x3 conv goes
    through pack_act and the gather."""
    g = wl.rng(59)
    n, c, h = 2, 16, 1450
    x = wl.int8_activations(g, (n, c, h, h))
    xd = dev(x)
    for k, r, pad in [(24, 1, 0), (8, 3, 1)]:
        w = wl.int8_weights(g, (k, c, r, r))
        ref = oracle.conv2d_i8(x, w, (1, 1), (pad, pad))
        d = unit.conv_desc(n, c, h, h, k, r, r, 1, pad)
        y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
        announce("conv_i8 4.2M columns", k, r)
        unit.unit_conv2d_i8(d, xd, dev(w), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
        torch.cuda.synchronize()
        assert same(host(y), ref, f"k {k} window {r}")
        del y


def test_conv_i8_asymmetric_geometry():
    """Different stride / pad / window per axis (the C ABI carries them separately)."""
    g = wl.rng(31)
    n, c, h, w_, k, r, s = 2, 12, 11, 9, 20, 3, 2
    x = wl.int8_activations(g, (n, c, h, w_))
    w = wl.int8_weights(g, (k, c, r, s))
    ref = oracle.conv2d_i8(x, w, (2, 1), (1, 0))
    d = unit.unit_conv2d_desc(n, c, h, w_, k, r, s, 2, 1, 1, 0)
    p, q = unit.unit_conv2d_out_dims(d)
    y = torch.empty((n, k, p, q), dtype=torch.int32, device="cuda:0")
    announce("conv_i8 asymmetric")
    unit.unit_conv2d_i8(d, dev(x), dev(w), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
    torch.cuda.synchronize()
    assert same(host(y), ref)


def test_conv_i8_config1_and_determinism():
    sh = wl.CONFIG1
    x, w = wl.conv_inputs_i8(sh, 1, 1)
    ref = oracle.conv2d_i8(x, w, (1, 1), (1, 1))
    announce("conv_i8 config 1")
    first = run_conv_i8(sh, 1, x, w)
    assert same(first, ref)
    for rep in range(20):                      # an LDS double-buffer race would show as a mismatch
        assert same(run_conv_i8(sh, 1, x, w), ref), rep
    x2 = np.full_like(x, -128); w2 = np.full_like(w, -128)
    got = run_conv_i8(sh, 1, x2, w2)
    assert got[0, 0, 5, 5] == 64 * 9 * 16384 and got[0, 0, 0, 0] == 64 * 4 * 16384


def test_conv_i8_resnet50_layers_batch1():
    for idx, (sh, mult) in enumerate(wl.unique_shapes(wl.resnet50_convs())):
        x, w = wl.conv_inputs_i8(sh, 1, 3, idx)
        ref = oracle.conv2d_i8(x, w, (sh.stride,) * 2, (sh.pad,) * 2)
        announce("conv_i8 resnet50", idx, sh)
        assert same(run_conv_i8(sh, 1, x, w), ref), sh


def test_conv_i8_table1_layers():
    for idx, sh in enumerate(wl.TABLE1):
        x, w = wl.conv_inputs_i8(sh, 1, 6, idx)
        ref = oracle.conv2d_i8(x, w, (sh.stride,) * 2, (sh.pad,) * 2)
        announce("conv_i8 table1", idx + 1, sh)
        assert same(run_conv_i8(sh, 1, x, w), ref), sh


def test_conv_f16_table1_layers():
    for idx, sh in enumerate(wl.TABLE1):
        x, w = wl.conv_inputs_f16(sh, 1, 7, idx)
        st, pd = (sh.stride,) * 2, (sh.pad,) * 2
        ref = oracle.conv2d_f16(x, w, st, pd)
        truth, mag = oracle.conv2d_f16_f64(x, w, st, pd)
        kred = sh.c * sh.r * sh.s
        announce("conv_f16 table1", idx + 1, sh)
        got = run_conv_f16(sh, 1, x, w)
        assert f16_rel_err(got, ref, kred) <= 1e-3, sh
        assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), sh
        assert as_accurate_as_oracle(got, ref, truth), sh


@pytest.mark.parametrize("sh,n", SMALL_CONVS[:6])
def test_conv_f16_small_all_tiles(sh, n):
    x, w = wl.conv_inputs_f16(sh, n, 40, sh.c)
    st, pd = (sh.stride,) * 2, (sh.pad,) * 2
    ref = oracle.conv2d_f16(x, w, st, pd)
    truth, mag = oracle.conv2d_f16_f64(x, w, st, pd)
    kred = sh.c * sh.r * sh.s
    for tile, split in [(None, None)] + [(t, s) for t in ALL_TILES for s in (1, 2)]:
        announce("conv_f16", sh, n, "tile", tile, "split", split)
        with forced(tile=tile, split=split):
            got = run_conv_f16(sh, n, x, w)
        assert f16_rel_err(got, ref, kred) <= 1e-3, (tile, split)
        assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), (tile, split)
        assert as_accurate_as_oracle(got, ref, truth), (tile, split)


def test_conv_f16_power_of_two_inputs_bit_exact():
    g = wl.rng(41)
    sh = wl.ConvShape(24, 9, 9, 40, 3, 3, 1, 1)
    x = wl.f16_bits(g.choice([-1.0, 1.0], size=(1, 24, 9, 9)) * 2.0 ** g.integers(-3, 4, size=(1, 24, 9, 9)))
    w = wl.f16_bits(g.choice([-1.0, 1.0], size=(40, 24, 3, 3)) * 2.0 ** g.integers(-3, 4, size=(40, 24, 3, 3)))
    ref = oracle.conv2d_f16(x, w, (1, 1), (1, 1))
    announce("conv_f16 power-of-two")
    got = run_conv_f16(sh, 1, x, w)
    assert same(got.view(np.uint32), ref.view(np.uint32))
    announce("conv_f16 determinism")
    x2, w2 = wl.conv_inputs_f16(sh, 1, 42)
    a = run_conv_f16(sh, 1, x2, w2)
    with forced(split=3):
        b1 = run_conv_f16(sh, 1, x2, w2)
        b2 = run_conv_f16(sh, 1, x2, w2)
    assert same(a.view(np.uint32), run_conv_f16(sh, 1, x2, w2).view(np.uint32))
    assert same(b1.view(np.uint32), b2.view(np.uint32))


def plane_check_f16(sh, n, x, w, got, planes):
    """Whole output planes (one image, one output channel: every pixel, so every column tile, image border and
    ragged tail of that row of the implicit GEMM) against the oracle run on that image and that filter."""
    st, pd = (sh.stride,) * 2, (sh.pad,) * 2
    kred = sh.c * sh.r * sh.s
    refs, gots, truths = [], [], []
    for ni, k in planes:
        xi, wk = np.ascontiguousarray(x[ni:ni + 1]), np.ascontiguousarray(w[k:k + 1])
        ref = oracle.conv2d_f16(xi, wk, st, pd)[0, 0]
        truth, mag = oracle.conv2d_f16_f64(xi, wk, st, pd)
        g_ = got[ni, k]
        assert np.all(np.abs(g_ - truth[0, 0]) <= 2 * kred * 2.0 ** -24 * mag[0, 0] + 1e-30), (sh, ni, k)
        refs.append(ref.ravel()); gots.append(g_.ravel()); truths.append(truth[0, 0].ravel())
    refs, gots, truths = np.concatenate(refs), np.concatenate(gots), np.concatenate(truths)
    assert as_accurate_as_oracle(gots, refs, truths), sh
    return f16_rel_err(gots, refs, kred)


def test_conv_f16_resnet50_layers_batch16_planes():
    """Config 4 at its full size, every one of the 23 unique shapes, in the launch configuration the benchmark
    times.  Six whole (image, channel) planes per layer: first and last image, first and last output channel
    (first and last row tile), and four random pairs."""
    g = wl.rng(43)
    n = 16
    for idx, (sh, mult) in enumerate(wl.unique_shapes(wl.resnet50_convs())):
        x, w = wl.conv_inputs_f16(sh, n, 4, idx)
        announce("conv_f16 resnet50 b16", idx, sh)
        got = run_conv_f16(sh, n, x, w)
        assert np.all(np.isfinite(got))
        planes = [(0, 0), (n - 1, sh.k - 1)] + [(int(g.integers(n)), int(g.integers(sh.k))) for _ in range(4)]
        assert plane_check_f16(sh, n, x, w, got, planes) <= 1e-3, sh


# ------------------------------------------------------------------ fused epilogue / packed path

def test_requant_epilogue_all_paths():
    g = wl.rng(50)
    for sh, n in [(wl.ConvShape(24, 12, 12, 40, 3, 3, 1, 1), 2), (wl.ConvShape(32, 9, 9, 19, 1, 1, 1, 0), 1)]:
        x, w = wl.conv_inputs_i8(sh, n, 50, sh.c)
        st, pd = (sh.stride,) * 2, (sh.pad,) * 2
        acc = oracle.conv2d_i8(x, w, st, pd)
        bias = g.integers(-5000, 5000, size=sh.k).astype(np.int32)
        res = g.integers(-30000, 30000, size=acc.shape).astype(np.int32)
        scale = (120.0 / np.abs(acc).max(axis=(0, 2, 3)).clip(1) * g.uniform(0.5, 1.0, sh.k)).astype(np.float32)
        d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
        p, q = unit.unit_conv2d_out_dims(d)
        xp = ws_bytes(unit.unit_packed_act_bytes(n, sh.c, sh.h, sh.w, unit.UNIT_I8))
        wp = ws_bytes(unit.unit_packed_weights_bytes(d, unit.UNIT_I8))
        unit.unit_pack_act_i8(n, sh.c, sh.h, sh.w, dev(x), xp)
        unit.unit_pack_weights_i8(d, dev(w), wp)
        sd, bd, rd = dev(scale), dev(bias), dev(res)
        kp = (sh.k + 15) // 16 * 16
        # skip connection in the packed int8 form an earlier layer would have written
        skip = wl.int8_weights(g, acc.shape)
        skip_mult = 217
        skp = ws_bytes(unit.unit_packed_act_bytes(n, sh.k, p, q, unit.UNIT_I8))
        unit.unit_pack_act_i8(n, sh.k, p, q, dev(skip), skp)
        for use_bias, use_res, relu, use_skip in [(0, 0, 0, 0), (1, 0, 1, 0), (0, 1, 1, 0), (1, 1, 0, 0), (1, 1, 1, 0),
                                                  (1, 0, 1, 1), (0, 1, 0, 1)]:
            total_res = None
            if use_res or use_skip:
                total_res = (res if use_res else 0) + (skip.astype(np.int32) * skip_mult if use_skip else 0)
                total_res = np.ascontiguousarray(total_res, dtype=np.int32)
            exp = oracle.requant(acc, scale, bias if use_bias else None, total_res, relu)
            rq = unit.make_requant(sd, bd if use_bias else None, rd if use_res else None, relu,
                                   skp if use_skip else None, skip_mult)
            for tile, split in [(None, None), (2, 1), (2, 2), (3, 1), (4, 3), (5, 1), (1, 1), (10, 1), (11, 2)]:
                announce("requant", sh, "bias", use_bias, "res", use_res, "skip", use_skip, "relu", relu,
                         "tile", tile, "split", split)
                y8 = torch.full((n, sh.k, p, q), 99, dtype=torch.int8, device="cuda:0")
                y32 = torch.full((n, sh.k, p, q), -7, dtype=torch.int32, device="cuda:0")
                ypk = torch.full((n, p, q, kp), 99, dtype=torch.int8, device="cuda:0")
                with forced(tile=tile, split=split):
                    ws = ws_bytes(unit.unit_conv2d_packed_workspace(d, unit.UNIT_I8))
                    unit.unit_conv2d_packed_i8(d, xp, wp, y32, rq, y8, ypk, ws)
                torch.cuda.synchronize()
                assert same(host(y8), exp)
                assert same(host(y32), acc)
                pk = host(ypk)
                assert same(pk[..., :sh.k].transpose(0, 3, 1, 2), exp)
                assert np.all(pk[..., sh.k:] == 0)
                # the packed output unpacks to the same NCHW tensor
                back = torch.empty((n, sh.k, p, q), dtype=torch.int8, device="cuda:0")
                unit.unit_unpack_act_i8(n, sh.k, p, q, ypk, back)
                torch.cuda.synchronize()
                assert same(host(back), exp)


def test_requant_epilogue_extreme_accumulators():
    """|acc| up to 4608*2^14 ~ 7.5e7 > 2^24: the int32 -> fp32 conversion rounds, on both sides alike."""
    sh = wl.ConvShape(512, 5, 5, 16, 3, 3, 1, 1)
    g = wl.rng(51)
    x = g.choice(np.array([-128, 127], np.int8), size=(1, 512, 5, 5))
    w = g.choice(np.array([-128, 127], np.int8), size=(16, 512, 3, 3))
    w[0] = -128; x[0, :, 1:4, 1:4] = -128           # one output reaches 4608 * 16384 exactly
    acc = oracle.conv2d_i8(x, w, (1, 1), (1, 1))
    assert acc.max() == 4608 * 16384
    scale = np.full(16, 127.0 / 7.5e7, np.float32)
    scale[1] = 3.3e-6
    exp = oracle.requant(acc, scale)
    d = unit.conv_desc(1, 512, 5, 5, 16, 3, 3, 1, 1)
    y8 = torch.empty((1, 16, 5, 5), dtype=torch.int8, device="cuda:0")
    sd, xd, wd = dev(scale), dev(x), dev(w)          # keep the device tensors alive across the call
    rq = unit.make_requant(sd)
    announce("requant extreme")
    unit.unit_conv2d_i8(d, xd, wd, None, rq, y8, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
    torch.cuda.synchronize()
    assert same(host(y8), exp)


PACK_SHAPES = [   # (n, c, h, w): both pack kernels (rows of pixels on dword boundaries or not), ragged tiles
    (3, 70, 12, 12), (1, 64, 56, 56), (2, 130, 8, 10), (1, 33, 7, 7), (2, 20, 5, 13), (1, 200, 16, 9),
    (4, 17, 4, 4), (1, 96, 3, 44), (2, 64, 1, 128), (1, 257, 2, 2),
]


@pytest.mark.parametrize("n,c,h,w_", PACK_SHAPES)
def test_pack_act_layout(n, c, h, w_):
    """pack_act is a pure permutation with zero fill: xp[n][h*w][cp], cp = channels padded to a 16-byte chunk;
    element (n, c, h, w) lands at xp[n][h*W + w][c].  Checked for one- and two-byte elements."""
    g = wl.rng(58, n * 1000 + c)
    for name, ut, dt, chunk, fn in [("i8", unit.UNIT_I8, np.int8, 16, unit.unit_pack_act_i8),
                                    ("f16", unit.UNIT_F16, np.uint16, 8, unit.unit_pack_act_f16)]:
        x = g.integers(0, 256 if dt == np.int8 else 65536, size=(n, c, h, w_)).astype(np.uint16 if dt == np.uint16 else np.uint8)
        x = x.view(np.int8) if dt == np.int8 else x
        cp = (c + chunk - 1) // chunk * chunk
        xp = torch.full((int(unit.unit_packed_act_bytes(n, c, h, w_, ut)),), 0x5a, dtype=torch.uint8, device="cuda:0")
        announce("pack_act layout", name, n, c, h, w_)
        fn(n, c, h, w_, dev(x.view(np.int16) if dt == np.uint16 else x), xp)
        torch.cuda.synchronize()
        raw = host(xp)[: n * h * w_ * cp * x.itemsize].view(x.dtype).reshape(n, h, w_, cp)
        assert same(raw[..., :c].transpose(0, 3, 1, 2), x), name
        assert np.all(raw[..., c:] == 0), name


def test_pack_roundtrip_and_glue_ops():
    g = wl.rng(52)
    n, c, h, w_ = 2, 37, 13, 11
    x = wl.int8_weights(g, (n, c, h, w_))
    xp = ws_bytes(unit.unit_packed_act_bytes(n, c, h, w_, unit.UNIT_I8))
    announce("pack/unpack")
    unit.unit_pack_act_i8(n, c, h, w_, dev(x), xp)
    back = torch.empty((n, c, h, w_), dtype=torch.int8, device="cuda:0")
    unit.unit_unpack_act_i8(n, c, h, w_, xp, back)
    torch.cuda.synchronize()
    assert same(host(back), x)
    cp = 48
    raw = host(xp)[: n * h * w_ * cp].reshape(n, h, w_, cp)
    assert same(raw[..., :c].view(np.int8).transpose(0, 3, 1, 2), x) and np.all(raw[..., c:] == 0)

    for cs in (1, 3, 4, 5, 8, 9, 16):                # images whose channels fit one chunk: one thread per pixel
        announce("pack small C", cs)
        xs = wl.int8_weights(g, (3, cs, 9, 31))
        xps = ws_bytes(unit.unit_packed_act_bytes(3, cs, 9, 31, unit.UNIT_I8))
        unit.unit_pack_act_i8(3, cs, 9, 31, dev(xs), xps)
        torch.cuda.synchronize()
        raw = host(xps)[: 3 * 9 * 31 * 16].reshape(3, 9, 31, 16)
        assert same(raw[..., :cs].view(np.int8).transpose(0, 3, 1, 2), xs) and np.all(raw[..., cs:] == 0)
        if cs <= 8:
            xh = g.integers(0, 65536, size=(2, cs, 7, 33)).astype(np.uint16)
            xph = ws_bytes(unit.unit_packed_act_bytes(2, cs, 7, 33, unit.UNIT_F16))
            unit.unit_pack_act_f16(2, cs, 7, 33, dev(xh.view(np.int16)), xph)
            torch.cuda.synchronize()
            rawh = host(xph)[: 2 * 7 * 33 * 16].view(np.uint16).reshape(2, 7, 33, 8)
            assert same(rawh[..., :cs].transpose(0, 3, 1, 2), xh) and np.all(rawh[..., cs:] == 0)

    announce("maxpool")
    p, q = oracle.out_dim(h, 3, 2, 1), oracle.out_dim(w_, 3, 2, 1)
    yp = ws_bytes(unit.unit_packed_act_bytes(n, c, p, q, unit.UNIT_I8))
    unit.unit_maxpool_packed_i8(n, c, h, w_, 3, 2, 1, xp, yp)
    mp = torch.empty((n, c, p, q), dtype=torch.int8, device="cuda:0")
    unit.unit_unpack_act_i8(n, c, p, q, yp, mp)
    torch.cuda.synchronize()
    assert same(host(mp), oracle.maxpool_i8(x))
    for win, st, pd in [(2, 2, 0), (3, 1, 1), (3, 2, 0), (5, 2, 2), (2, 1, 1)]:
        announce("maxpool", win, st, pd)             # compile-time windows 2 and 3, and the general walk
        p2, q2 = (h + 2 * pd - win) // st + 1, (w_ + 2 * pd - win) // st + 1
        yp2 = ws_bytes(unit.unit_packed_act_bytes(n, c, p2, q2, unit.UNIT_I8))
        unit.unit_maxpool_packed_i8(n, c, h, w_, win, st, pd, xp, yp2)
        mp2 = torch.empty((n, c, p2, q2), dtype=torch.int8, device="cuda:0")
        unit.unit_unpack_act_i8(n, c, p2, q2, yp2, mp2)
        torch.cuda.synchronize()
        assert same(host(mp2), oracle.maxpool_i8(x, (win, win), (st, st), (pd, pd)))

    announce("avgpool")
    scale = g.uniform(0.002, 0.02, c).astype(np.float32)
    ya = torch.full((n, cp), 99, dtype=torch.int8, device="cuda:0")
    unit.unit_global_avgpool_packed_i8(n, c, h, w_, xp, dev(scale), ya)
    torch.cuda.synchronize()
    assert same(host(ya)[:, :c], oracle.global_sumpool_requant_i8(x, scale))
    assert np.all(host(ya)[:, c:] == 0)

    for n2, c2, h2, w2 in [(3, 150, 7, 7), (1, 512, 7, 7), (2, 70, 1, 1), (1, 16, 20, 21)]:
        announce("avgpool", n2, c2, h2, w2)       # several channel groups, pixel counts around the 16 slices
        x2 = wl.int8_weights(g, (n2, c2, h2, w2))
        xp2 = ws_bytes(unit.unit_packed_act_bytes(n2, c2, h2, w2, unit.UNIT_I8))
        unit.unit_pack_act_i8(n2, c2, h2, w2, dev(x2), xp2)
        cp2 = (c2 + 15) // 16 * 16
        scale2 = g.uniform(0.002, 0.02, c2).astype(np.float32)
        ya2 = torch.full((n2, cp2), 99, dtype=torch.int8, device="cuda:0")
        unit.unit_global_avgpool_packed_i8(n2, c2, h2, w2, xp2, dev(scale2), ya2)
        torch.cuda.synchronize()
        assert same(host(ya2)[:, :c2], oracle.global_sumpool_requant_i8(x2, scale2))
        assert np.all(host(ya2)[:, c2:] == 0)

    announce("widen residual")
    res = torch.empty((n, c, h, w_), dtype=torch.int32, device="cuda:0")
    unit.unit_widen_residual_i8(n, c, h, w_, xp, 64, res)
    torch.cuda.synchronize()
    assert same(host(res), oracle.widen_scale_i8(x, 64))


# ------------------------------------------------------------------ edge and degenerate cases

def test_degenerate_shapes():
    cases = [
        (wl.ConvShape(1, 1, 1, 1, 1, 1, 1, 0), 1),            # one MAC
        (wl.ConvShape(1, 5, 7, 1, 3, 3, 1, 2), 2),            # pad = window - 1: first outputs see one tap
        (wl.ConvShape(5, 9, 9, 3, 1, 1, 3, 0), 1),            # stride larger than the window
        (wl.ConvShape(17, 3, 3, 9, 3, 3, 1, 0), 3),           # output 1x1: a pure dot product per channel
        (wl.ConvShape(33, 6, 5, 65, 3, 3, 1, 1), 5),          # tiles straddle image boundaries (n*p*q = 150)
        (wl.ConvShape(8, 12, 12, 8, 5, 5, 2, 2), 1),
    ]
    for sh, n in cases:
        x, w = wl.conv_inputs_i8(sh, n, 60, sh.c)
        ref = oracle.conv2d_i8(x, w, (sh.stride,) * 2, (sh.pad,) * 2)
        announce("degenerate i8", sh, n)
        assert same(run_conv_i8(sh, n, x, w), ref, str(sh))
        xh, wh = wl.conv_inputs_f16(sh, n, 61, sh.c)
        refh = oracle.conv2d_f16(xh, wh, (sh.stride,) * 2, (sh.pad,) * 2)
        announce("degenerate f16", sh, n)
        assert f16_rel_err(run_conv_f16(sh, n, xh, wh), refh, sh.c * sh.r * sh.s) <= 1e-3, sh
    announce("matmul 1x1x1")
    assert same(run_matmul_i8(np.array([[-128]], np.int8), np.array([[-128]], np.int8)), np.array([[16384]]))


def test_matmul_i8_longest_exact_reduction():
    """k = 131071 with every product at its extreme: the int32 sum is 2147467264 < 2^31."""
    K = unit.UNIT_MAX_REDUCTION_I8
    A = np.full((3, K), -128, np.int8)
    B = np.full((5, K), -128, np.int8)
    B[1] = 127; B[2, ::2] = 127
    announce("matmul_i8 k=131071")
    got = run_matmul_i8(A, B)
    assert same(got, A.astype(np.int64) @ B.astype(np.int64).T, "longest reduction")
    assert got[0, 0] == K * 16384 and got.max() < 2 ** 31


# ------------------------------------------------------------------ two column ranges (whole rounds + narrower tail)

def test_matmul_two_column_ranges():
    """A problem whose 256 x 256 tiles leave a last round of workgroups mostly empty runs as two launches with two
    tile shapes (the selector query reports the second one); rows and columns on both sides of the seam, and the
    tail's own ragged end, against the oracle."""
    M, N, K = 4096, 4352 + 37, 512
    info = unit.unit_select_matmul(M, N, K, unit.UNIT_I8)
    assert (info.block_m, info.block_n) == (256, 256) and info.tail_block_n in (128, 192) and info.tail_first_col == 4096
    g = wl.rng(27)
    A, B = wl.int8_weights(g, (M, K)), wl.int8_weights(g, (N, K))
    announce("matmul_i8 two ranges", M, N, K, "tail", info.tail_block_n)
    got = run_matmul_i8(A, B)
    rows = np.unique(np.concatenate([[0, 255, 256, 4095], g.integers(0, M, 8)]))
    cols = np.unique(np.concatenate([[0, 4095, 4096, 4097, 4223, 4224, 4351, 4352, N - 1], g.integers(4000, N, 8)]))
    assert same(got[rows], oracle.matmul_i8(np.ascontiguousarray(A[rows]), B))
    assert same(got[:, cols], oracle.matmul_i8(A, np.ascontiguousarray(B[cols])))
    colsum = B.astype(np.int64).sum(axis=0)
    assert same(got.astype(np.int64).sum(axis=1), A.astype(np.int64) @ colsum)
    Ah, Bh = wl.f16_activations(g, (M, K)), wl.f16_weights(g, (N, K), K)
    announce("matmul_f16 two ranges")
    goth = run_matmul_f16(Ah, Bh)
    ref = oracle.matmul_f16(Ah, np.ascontiguousarray(Bh[cols]))
    truth, mag = oracle.matmul_f16_f64(Ah, np.ascontiguousarray(Bh[cols]))
    assert f16_rel_err(goth[:, cols], ref, K) <= 1e-3
    assert np.all(np.abs(goth[:, cols] - truth) <= 2 * K * 2.0 ** -24 * mag + 1e-30)
    assert as_accurate_as_oracle(goth[:, cols], ref, truth)


def test_large_conv_two_column_ranges():
    """The compute-bound conv the benchmark times (N=32, C=K=256, 56x56, 3x3): 392 tiles of 256 x 256 = one full
    round plus a tail that runs on a narrower tile.  Whole output planes of the images around the seam (output
    column 65536 lies in image 20), the first and the last image."""
    sh, n = wl.LARGE_CONV, 32
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
    info = unit.unit_select_conv2d(d, unit.UNIT_I8)
    assert info.tail_block_n > 0 and info.tail_first_col == 65536 and info.workgroups == 256
    x, w = wl.conv_inputs_i8(sh, n, 9, 0)
    announce("large conv i8, two ranges: tail", info.tail_block_n, info.tail_workgroups)
    got = run_conv_i8(sh, n, x, w)
    g = wl.rng(28)
    planes = [(0, 0), (20, 255), (20, 17), (21, 100), (31, 255), (19, 3)] + [(int(g.integers(n)), int(g.integers(sh.k))) for _ in range(6)]
    for ni, k in planes:
        ref = oracle.conv2d_i8(np.ascontiguousarray(x[ni:ni + 1]), np.ascontiguousarray(w[k:k + 1]), (1, 1), (1, 1))
        assert same(got[ni, k], ref[0, 0], f"image {ni} channel {k}")
    # a property that holds at any size: summed over output channels, the conv equals the conv with the summed filter
    wsum = w.astype(np.int64).sum(axis=0, keepdims=True)
    for ni in (20, 27):
        xs = x[ni:ni + 1].astype(np.float64)
        import torch.nn.functional as F
        exp = F.conv2d(torch.from_numpy(xs), torch.from_numpy(wsum.astype(np.float64)), padding=1).numpy()[0, 0]
        assert np.array_equal(got[ni].astype(np.int64).sum(axis=0), exp.astype(np.int64)), ni
    xh, wh = wl.conv_inputs_f16(sh, n, 9, 0)
    announce("large conv f16, two ranges")
    goth = run_conv_f16(sh, n, xh, wh)
    assert plane_check_f16(sh, n, xh, wh, goth, planes[:8]) <= 1e-3


# ------------------------------------------------------------------ matmul with very few rows (dot-product path)

@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8])
def test_matmul_few_rows_dot_product_path(M):
    """m <= 4 (int8, fp16) runs one wave per output column on v_dot4 / v_dot2 instead of the matrix units (5 and 8
    rows, which take the 16-row MFMA tile, run through the same cases): the
    FC shape of the benchmark (1 x 1000 x 2048), ragged reductions (tail chunks, fewer chunks than lanes, padded
    copies of misaligned operands), leading dimensions larger than the rows, saturated operands."""
    g = wl.rng(29, M)
    for N, K, lda_extra, ldb_extra, ldc_extra in [(1000, 2048, 0, 0, 0), (37, 16, 0, 0, 0), (130, 1040, 16, 32, 5),
                                                  (9, 3000, 0, 0, 0), (64, 131, 3, 1, 0), (257, 4096 + 16, 0, 0, 3)]:
        info = unit.unit_select_matmul(M, N, K, unit.UNIT_I8)
        assert (info.mfma == 0 and info.workgroups == (N + 3) // 4) if M <= 4 else info.mfma == 16
        A, B = wl.int8_weights(g, (M, K + lda_extra)), wl.int8_weights(g, (N, K + ldb_extra))
        if K == 16:
            A[:], B[:] = -128, -128                                       # 16 * 2^14 per output
        ref = oracle.matmul_i8(np.ascontiguousarray(A[:, :K]), np.ascontiguousarray(B[:, :K]))
        C = torch.full((M, N + ldc_extra), -7, dtype=torch.int32, device="cuda:0")
        ws = ws_bytes(unit.unit_matmul_workspace(M, N, K, K + lda_extra, K + ldb_extra, unit.UNIT_I8))
        announce("matmul_i8 few rows", M, N, K, lda_extra, ldb_extra, ldc_extra)
        unit.unit_matmul_i8(M, N, K, dev(A), K + lda_extra, dev(B), K + ldb_extra, C, N + ldc_extra, ws)
        torch.cuda.synchronize()
        got = host(C)
        assert same(got[:, :N], ref)
        assert np.all(got[:, N:] == -7)                                   # nothing written past a row's n columns
        Ah, Bh = wl.f16_activations(g, (M, K + lda_extra)), wl.f16_weights(g, (N, K + ldb_extra), K)
        Ak, Bk = np.ascontiguousarray(Ah[:, :K]), np.ascontiguousarray(Bh[:, :K])
        refh = oracle.matmul_f16(Ak, Bk)
        truth, mag = oracle.matmul_f16_f64(Ak, Bk)
        Ch = torch.full((M, N + ldc_extra), -7.0, dtype=torch.float32, device="cuda:0")
        ws = ws_bytes(unit.unit_matmul_workspace(M, N, K, K + lda_extra, K + ldb_extra, unit.UNIT_F16))
        announce("matmul_f16 few rows", M, N, K)
        unit.unit_matmul_f16(M, N, K, dev(Ah), K + lda_extra, dev(Bh), K + ldb_extra, Ch, N + ldc_extra, ws)
        torch.cuda.synchronize()
        goth = host(Ch)[:, :N]
        assert f16_rel_err(goth, refh, K) <= 1e-3
        assert np.all(np.abs(goth - truth) <= 2 * K * 2.0 ** -24 * mag + 1e-30)
        assert as_accurate_as_oracle(goth, refh, truth)
    # a forced tile takes the matrix-unit path again (what the tile sweeps of the other tests run)
    with forced(tile=5, split=1):
        assert unit.unit_select_matmul(M, 1000, 2048, unit.UNIT_I8).mfma == 16


def test_direct_1x1_two_column_ranges():
    """Two column ranges in the direct NCHW read of a 1x1 conv (24 images of 56x56, 512 -> 256 channels: 294 tiles of
    256 x 256 = one round + 38 column tiles, which run as 256 x 128 tiles; the 256 x 192 tile has no direct-read
    kernel).  The seam (column 65536) lies inside image 20."""
    sh, n = wl.ConvShape(512, 56, 56, 256, 1, 1, 1, 0), 24
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
    x, w = wl.conv_inputs_i8(sh, n, 9, 5)
    xd = dev(x)
    assert unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd) == unit.UNIT_INPUT_DIRECT
    info = unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_DIRECT)
    assert (info.block_n, info.workgroups, info.tail_block_n, info.tail_first_col) == (256, 256, 128, 65536)
    wp = ws_bytes(unit.unit_packed_weights_bytes(d, unit.UNIT_I8))
    unit.unit_pack_weights_i8(d, dev(w), wp)
    y = torch.full((n, sh.k, 56, 56), -7, dtype=torch.int32, device="cuda:0")
    announce("direct 1x1, two ranges", info.tail_block_n, info.tail_workgroups)
    unit.unit_conv2d_wpacked_i8(d, xd, wp, y, None, None, ws_bytes(unit.unit_conv2d_wpacked_workspace(d, unit.UNIT_I8)))
    torch.cuda.synchronize()
    got = host(y)
    g = wl.rng(30)
    for ni, k in [(0, 0), (20, 255), (20, 1), (21, 77), (23, 255)] + [(int(g.integers(n)), int(g.integers(sh.k))) for _ in range(5)]:
        ref = oracle.conv2d_i8(np.ascontiguousarray(x[ni:ni + 1]), np.ascontiguousarray(w[k:k + 1]))
        assert same(got[ni, k], ref[0, 0], f"image {ni} channel {k}")
    wsum = w.astype(np.int64).sum(axis=0)[:, 0, 0]                    # [c]: the conv summed over output channels
    for ni in (20, 22):
        exp = np.tensordot(wsum, x[ni].astype(np.int64), axes=(0, 0))
        assert np.array_equal(got[ni].astype(np.int64).sum(axis=0), exp), ni


# ------------------------------------------------------------------ random geometries, the selector's own choices

def _random_conv_cases(seed, count):
    """Seeded geometries around the selector's decision boundaries: few to some hundred channels (reductions on both
    sides of 32 / 64 / 160 chunks), 3..30 pixels a side (tile counts on both sides of 64 and 128 tiles of 32x32),
    windows 1..5 with their own stride and padding per axis, one to three images."""
    g = np.random.Generator(np.random.PCG64(seed))
    out = []
    while len(out) < count:
        n = int(g.integers(1, 4))
        c = int(g.choice([1, 3, 8, 16, 24, 32, 48, 64, 96, 128, 160, 256, 288, 512]))
        k = int(g.choice([1, 5, 16, 17, 32, 64, 100, 128, 192, 256, 300]))
        h, w_ = int(g.integers(3, 31)), int(g.integers(3, 31))
        kind = int(g.integers(0, 4))        # half of the cases can take a direct read: 1x1 / "same" 3x3 at stride 1
        if kind == 0:
            r = s = sh_ = sw_ = 1
            ph = pw = 0
        elif kind == 1:
            r = s = 3
            sh_ = sw_ = ph = pw = 1
        else:
            r, s = int(g.choice([1, 1, 3, 3, 5])), int(g.choice([1, 1, 3, 3, 2]))
            sh_, sw_ = int(g.integers(1, 3)), int(g.integers(1, 3))
            ph, pw = int(g.integers(0, (r + 1) // 2 + 1)), int(g.integers(0, (s + 1) // 2 + 1))
        if h + 2 * ph < r or w_ + 2 * pw < s or c * r * s > 6000:
            continue
        out.append((n, c, h, w_, k, r, s, sh_, sw_, ph, pw))
    return out


@pytest.mark.parametrize("seed", [0, 1])
def test_conv_random_geometries_selector_choice(seed):
    """Both entry points that take NCHW activations, with whatever input mode, tile and split the library picks by
    itself: int8 bit-exact, fp16 within tolerance and as accurate as the sequential oracle."""
    for i, (n, c, h, w_, k, r, s, sh_, sw_, ph, pw) in enumerate(_random_conv_cases(9000 + seed, 40)):
        g = wl.rng(70 + seed, i)
        d = unit.unit_conv2d_desc(n, c, h, w_, k, r, s, sh_, sw_, ph, pw)
        p, q = unit.unit_conv2d_out_dims(d)
        x8, w8 = wl.int8_activations(g, (n, c, h, w_)), wl.int8_weights(g, (k, c, r, s))
        ref = oracle.conv2d_i8(x8, w8, (sh_, sw_), (ph, pw))
        xd = dev(x8)
        mode = unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd)
        info = unit.unit_select_conv2d_input(d, unit.UNIT_I8, mode)
        announce("conv random i8", (n, c, h, w_, k, r, s, sh_, sw_, ph, pw), "mode", mode,
                 "tile", info.block_m, info.block_n, info.block_k_bytes, "split", info.split_k)
        y = torch.full((n, k, p, q), -7, dtype=torch.int32, device="cuda:0")
        unit.unit_conv2d_i8(d, xd, dev(w8), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
        torch.cuda.synchronize()
        assert same(host(y), ref, str((n, c, h, w_, k, r, s, sh_, sw_, ph, pw)))
        if i % 2:
            continue
        xf, wf = wl.f16_activations(g, (n, c, h, w_)), wl.f16_weights(g, (k, c, r, s), c * r * s)
        reff = oracle.conv2d_f16(xf, wf, (sh_, sw_), (ph, pw))
        truth, mag = oracle.conv2d_f16_f64(xf, wf, (sh_, sw_), (ph, pw))
        announce("conv random f16", (n, c, h, w_, k, r, s, sh_, sw_, ph, pw))
        yf = torch.empty((n, k, p, q), dtype=torch.float32, device="cuda:0")
        unit.unit_conv2d_f16(d, dev(xf), dev(wf), yf, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_F16)))
        torch.cuda.synchronize()
        got, kred = host(yf), c * r * s
        assert f16_rel_err(got, reff, kred) <= 1e-3, (n, c, h, w_, k, r, s)
        assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), (n, c, h, w_, k, r, s)
        assert as_accurate_as_oracle(got, reff, truth), (n, c, h, w_, k, r, s)


def test_matmul_random_shapes_selector_choice():
    g = np.random.Generator(np.random.PCG64(9100))
    for i in range(40):
        M, N = int(g.integers(1, 300)), int(g.integers(1, 400))
        K = int(g.choice([1, 15, 16, 64, 200, 511, 512, 513, 1024, 1500, 2560, 2561, 4100]))
        gg = wl.rng(72, i)
        A, B = wl.int8_weights(gg, (M, K)), wl.int8_weights(gg, (N, K))
        info = unit.unit_select_matmul(M, N, K, unit.UNIT_I8)
        announce("matmul random i8", M, N, K, "tile", info.block_m, info.block_n, info.block_k_bytes, "split", info.split_k)
        assert same(run_matmul_i8(A, B), oracle.matmul_i8(A, B), str((M, N, K)))
        if i % 2:
            continue
        Af, Bf = wl.f16_activations(gg, (M, K)), wl.f16_weights(gg, (N, K), K)
        ref = oracle.matmul_f16(Af, Bf)
        truth, mag = oracle.matmul_f16_f64(Af, Bf)
        announce("matmul random f16", M, N, K)
        got = run_matmul_f16(Af, Bf)
        assert f16_rel_err(got, ref, K) <= 1e-3, (M, N, K)
        assert np.all(np.abs(got - truth) <= 2 * K * 2.0 ** -24 * mag + 1e-30), (M, N, K)
        assert as_accurate_as_oracle(got, ref, truth), (M, N, K)
