"""GPU parity for the shifted direct read of NCHW activations (stride 1, "same"
padding): the main kernel fetches per-tap shifted windows of the channel rows instead of
running pack_act first.  Every case is compared with the oracle on every tile shape that has
a kernel in this mode and with a forced split; the input mode the library reports is checked
so that the cases really exercise the path they are meant for."""
import numpy as np
import pytest
import torch

import oracle
from paper_2101_08458_amd import unit, workloads as wl
from gpu_util import announce, dev, host, forced, f16_rel_err, as_accurate_as_oracle, fp8_rel_err, fp8_bound, same

pytestmark = pytest.mark.gpu

ALL_TILES = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12]
SHIFTED, DIRECT, PACKED = unit.UNIT_INPUT_DIRECT_SHIFTED, unit.UNIT_INPUT_DIRECT, unit.UNIT_INPUT_PACKED


def ws_bytes(nbytes):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda:0")


# (shape, expected mode at the selector's own choice for int8, for fp16)
CASES = [
    (wl.ConvShape(128, 14, 14, 96, 3, 3, 1, 1), SHIFTED, SHIFTED),     # row pitch 196 bytes: shift differs per channel row
    (wl.ConvShape(256, 28, 28, 40, 3, 3, 1, 1), SHIFTED, SHIFTED),
    (wl.ConvShape(128, 7, 7, 130, 3, 3, 1, 1), SHIFTED, SHIFTED),      # 49-pixel rows, tiles wider than the image
    (wl.ConvShape(128, 9, 13, 40, 3, 3, 1, 1), SHIFTED, SHIFTED),      # odd sizes: every byte shift occurs
    (wl.ConvShape(128, 11, 10, 33, 5, 5, 1, 2), SHIFTED, SHIFTED),     # wider window
    (wl.ConvShape(512, 7, 7, 64, 1, 1, 1, 0), DIRECT, DIRECT),         # 1x1 whose rows are not 4-byte aligned: end chunk patched
    (wl.ConvShape(384, 5, 3, 48, 1, 1, 1, 0), PACKED, DIRECT),         # 15-pixel image: less than a chunk of one-byte elements
    (wl.ConvShape(256, 6, 6, 48, 1, 1, 1, 0), DIRECT, DIRECT),         # 1x1 with dword-aligned rows: the plain direct read
    (wl.ConvShape(64, 12, 12, 64, 3, 3, 1, 1), SHIFTED, SHIFTED),      # 64 channels: one fp16 step; int8 takes the tile with 64-byte steps
    (wl.ConvShape(32, 12, 12, 64, 3, 3, 1, 1), PACKED, SHIFTED),       # 32 channels: 64 bytes of fp16, too few of int8
    (wl.ConvShape(128, 56, 56, 32, 3, 3, 1, 1), SHIFTED, SHIFTED),     # many column tiles
    (wl.ConvShape(128, 12, 12, 16, 3, 3, 1, 1), SHIFTED, SHIFTED),     # 16 output channels: the narrow tile
    (wl.ConvShape(128, 4, 4, 32, 3, 3, 1, 1), PACKED, SHIFTED),        # 16 pixels: too few for 16 one-byte elements per chunk
    (wl.ConvShape(128, 5, 5, 48, 3, 3, 1, 1), SHIFTED, SHIFTED),       # smallest image the one-byte types take
    (wl.ConvShape(128, 7, 7, 48, 5, 5, 1, 2), SHIFTED, SHIFTED),       # largest tap offsets relative to the image
]


def _desc(sh, n=1):
    return unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_shifted_direct_i8(case):
    sh, mode_i8, _ = CASES[case]
    d = _desc(sh)
    x, w = wl.conv_inputs_i8(sh, 1, 61, case)
    ref = oracle.conv2d_i8(x, w, (1, 1), (sh.pad, sh.pad))
    xd = dev(x)
    wp = ws_bytes(unit.unit_packed_weights_bytes(d, unit.UNIT_I8))
    unit.unit_pack_weights_i8(d, dev(w), wp)
    if sh.k > 16:                           # (16 output channels select the 256-byte-step tile)
        assert unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd) == mode_i8
    for tile, split in [(None, None)] + [(t, s) for t in ALL_TILES for s in (1, 3)]:
        with forced(tile=tile, split=split):
            mode = unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd)
            announce("shifted i8", tuple(sh), "tile", tile, "split", split, "mode", mode)
            y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
            unit.unit_conv2d_wpacked_i8(d, xd, wp, y, None, None,
                                        ws_bytes(unit.unit_conv2d_wpacked_workspace(d, unit.UNIT_I8)))
            torch.cuda.synchronize()
        assert same(host(y), ref, f"tile {tile} split {split} mode {mode}")


@pytest.mark.parametrize("case", range(len(CASES)))
def test_shifted_direct_f16_bf16_fp8(case):
    sh, _, mode_f16 = CASES[case]
    d = _desc(sh)
    kred = sh.c * sh.r * sh.s
    pad = (sh.pad, sh.pad)
    kinds = [
        ("f16", unit.UNIT_F16, wl.conv_inputs_f16, lambda x, w: (oracle.conv2d_f16(x, w, (1, 1), pad),) +
         oracle.conv2d_f16_f64(x, w, (1, 1), pad), unit.unit_conv2d_f16),
        ("bf16", unit.UNIT_BF16, wl.conv_inputs_bf16, lambda x, w: oracle.conv2d_bf16(x, w, (1, 1), pad),
         unit.unit_conv2d_bf16),
        ("fp8", unit.UNIT_FP8, wl.conv_inputs_fp8, lambda x, w: oracle.conv2d_fp8(x, w, (1, 1), pad),
         unit.unit_conv2d_fp8),
    ]
    for name, ut, gen, orc, fn in kinds:
        x, w = gen(sh, 1, 62, case)
        ref, truth, mag = orc(x, w)
        xd, wd = dev(x), dev(w)
        if name == "f16" and sh.k > 16:
            assert unit.unit_conv2d_input_mode(d, ut, xd) == mode_f16
        for tile, split in [(None, None)] + [(t, 1) for t in ALL_TILES] + [(3, 2), (4, 3)]:
            if name == "fp8" and tile == 12:
                continue                                    # (the 16x16 tile has no fp8 kernel)
            with forced(tile=tile, split=split):
                mode = unit.unit_conv2d_input_mode(d, ut, xd)
                announce("shifted", name, tuple(sh), "tile", tile, "split", split, "mode", mode)
                y = torch.empty(ref.shape, dtype=torch.float32, device="cuda:0")
                fn(d, xd, wd, y, ws_bytes(unit.unit_conv2d_workspace(d, ut)))
                torch.cuda.synchronize()
            got = host(y)
            if name == "fp8":
                assert fp8_rel_err(got, ref) <= 1e-3, (name, tile, split)
                assert np.all(np.abs(got - truth) <= fp8_bound(kred, mag)), (name, tile, split)
            else:
                assert f16_rel_err(got, ref, kred) <= 1e-3, (name, tile, split)
                assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), (name, tile, split)
                assert as_accurate_as_oracle(got, ref, truth), (name, tile, split)


BATCHES = [   # (n, shape): images of whole 16-byte chunks (tiles span images) and others (tiled per image)
    (3, wl.ConvShape(128, 8, 8, 40, 3, 3, 1, 1)),       # 64 pixels: a 256-wide tile holds four images
    (2, wl.ConvShape(128, 12, 12, 33, 3, 3, 1, 1)),     # 144 pixels: whole chunks for one-byte elements too
    (3, wl.ConvShape(128, 14, 14, 48, 3, 3, 1, 1)),     # 196 pixels: per image for every type
    (5, wl.ConvShape(128, 9, 7, 24, 5, 3, 1, (2, 1))),  # 63 pixels, different window extents
    (2, wl.ConvShape(256, 28, 28, 32, 3, 3, 1, 1)),
]


@pytest.mark.parametrize("case", range(len(BATCHES)))
def test_shifted_direct_batches(case):
    """Several images: every image's border taps are masked on its own, the windows of an image's first
    channel reach back into the previous image (masked), and only the first image's first channel and the
    last image's last channel can touch the tensor's ends."""
    n, sh = BATCHES[case]
    pad = sh.pad if isinstance(sh.pad, tuple) else (sh.pad, sh.pad)
    d = unit.conv_desc(n, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, (1, 1), pad)
    g = wl.rng(66, case)
    x = wl.int8_activations(g, (n, sh.c, sh.h, sh.w))
    w = wl.int8_weights(g, (sh.k, sh.c, sh.r, sh.s))
    ref = oracle.conv2d_i8(x, w, (1, 1), pad)
    xd, wd = dev(x), dev(w)
    for tile, split in [(None, None)] + [(t, 1) for t in ALL_TILES] + [(3, 2), (4, 3)]:
        with forced(tile=tile, split=split):
            mode = unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd)
            announce("shifted batch i8", n, tuple(sh), "tile", tile, "split", split, "mode", mode)
            if tile is None:
                assert mode == SHIFTED
            y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
            unit.unit_conv2d_i8(d, xd, wd, y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
            torch.cuda.synchronize()
        assert same(host(y), ref, f"batch case {case} tile {tile} split {split} mode {mode}")
    kred = sh.c * sh.r * sh.s
    for name, ut, gen, orc, fn in [
        ("f16", unit.UNIT_F16, wl.conv_inputs_f16, lambda a, b: (oracle.conv2d_f16(a, b, (1, 1), pad),) +
         oracle.conv2d_f16_f64(a, b, (1, 1), pad), unit.unit_conv2d_f16),
        ("fp8", unit.UNIT_FP8, wl.conv_inputs_fp8, lambda a, b: oracle.conv2d_fp8(a, b, (1, 1), pad), unit.unit_conv2d_fp8),
    ]:
        xf, wf = gen(wl.ConvShape(sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, 1, 0), n, 67, case)
        reff, truth, mag = orc(xf, wf)
        xfd, wfd = dev(xf), dev(wf)
        for tile in (None, 1, 3, 4):
            with forced(tile=tile):
                mode = unit.unit_conv2d_input_mode(d, ut, xfd)
                announce("shifted batch", name, n, tuple(sh), "tile", tile, "mode", mode)
                if tile is None:
                    assert mode == SHIFTED
                y = torch.empty(reff.shape, dtype=torch.float32, device="cuda:0")
                fn(d, xfd, wfd, y, ws_bytes(unit.unit_conv2d_workspace(d, ut)))
                torch.cuda.synchronize()
            got = host(y)
            if name == "fp8":
                assert fp8_rel_err(got, reff) <= 1e-3, (name, tile)
                assert np.all(np.abs(got - truth) <= fp8_bound(kred, mag)), (name, tile)
            else:
                assert f16_rel_err(got, reff, kred) <= 1e-3, (name, tile)
                assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), (name, tile)
                assert as_accurate_as_oracle(got, reff, truth), (name, tile)


def test_shifted_direct_border_taps_exact():
    """All-ones image and filters: every output equals the number of taps inside the image times
    the channel count, so a wrong border mask or a wrong window shift shows as a wrong count."""
    for h, w, r, pad in [(14, 14, 3, 1), (7, 9, 3, 1), (6, 5, 5, 2), (8, 7, 7, 3)]:
        sh = wl.ConvShape(128, h, w, 32, r, r, 1, pad)
        d = _desc(sh)
        x = np.ones((1, 128, h, w), np.int8)
        wt = np.ones((32, 128, r, r), np.int8)
        rows = np.minimum(np.arange(h) + pad, h - 1) - np.maximum(np.arange(h) - pad, 0) + 1
        cols = np.minimum(np.arange(w) + pad, w - 1) - np.maximum(np.arange(w) - pad, 0) + 1
        exp = np.broadcast_to(128 * rows[:, None] * cols[None, :], (1, 32, h, w))
        xd = dev(x)
        assert unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd) == SHIFTED
        announce("shifted ones", h, w, r)
        y = torch.full((1, 32, h, w), -7, dtype=torch.int32, device="cuda:0")
        unit.unit_conv2d_i8(d, xd, dev(wt), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
        torch.cuda.synchronize()
        assert same(host(y), exp, f"{h}x{w} window {r}")


def test_modes_that_must_not_use_the_shifted_read():
    xd = ws_bytes(1 << 20)
    mode = lambda d, ut=unit.UNIT_I8, x=xd: unit.unit_conv2d_input_mode(d, ut, x)
    assert mode(unit.conv_desc(64, 128, 5, 5, 512, 3, 3, 1, 1)) == PACKED          # small images, one mostly empty 64-wide tile each
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 3, 3, 2, 1)) == PACKED          # stride 2
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 3, 3, 1, 0)) == PACKED          # output grid smaller than input
    assert mode(unit.conv_desc(1, 120, 14, 14, 64, 3, 3, 1, 1)) == PACKED          # channels not a whole step
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 3, 3, 1, 1), unit.UNIT_U8I8) == PACKED
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 1, 1, 1, 0)) == DIRECT          # aligned rows: plain direct read
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 3, 3, 1, 1), x=xd[4:]) == PACKED   # misaligned tensor base
    assert mode(unit.conv_desc(1, 128, 14, 14, 64, 3, 3, 1, 1)) == SHIFTED


def test_shifted_direct_odd_geometries():
    """Windows with different extents per axis, narrow images, and images too small for the shifted read
    (fewer pixels than the largest tap offset plus one 16-byte chunk), which must fall back to packing."""
    geoms = [   # (c, h, w, k, r, s, pad_h, pad_w)
        (128, 6, 9, 24, 1, 3, 0, 1), (128, 9, 6, 24, 3, 1, 1, 0), (128, 1, 17, 40, 3, 3, 1, 1),
        (128, 13, 1, 40, 3, 3, 1, 1), (256, 1, 1, 64, 3, 3, 1, 1), (128, 2, 2, 33, 5, 5, 2, 2),
        (128, 3, 40, 16, 3, 7, 1, 3), (128, 2, 19, 40, 3, 3, 1, 1), (128, 17, 2, 40, 3, 3, 1, 1),
    ]
    for i, (c, h, w, k, r, s, ph, pw) in enumerate(geoms):
        d = unit.conv_desc(1, c, h, w, k, r, s, (1, 1), (ph, pw))
        g = wl.rng(63, i)
        x = wl.int8_activations(g, (1, c, h, w))
        wt = wl.int8_weights(g, (k, c, r, s))
        ref = oracle.conv2d_i8(x, wt, (1, 1), (ph, pw))
        xd = dev(x)
        for tile in (None, 1, 3, 4):
            with forced(tile=tile):
                mode = unit.unit_conv2d_input_mode(d, unit.UNIT_I8, xd)
                announce("shifted odd geometry", (c, h, w, k, r, s, ph, pw), "tile", tile, "mode", mode)
                if tile is None and k > 16:
                    assert mode == (SHIFTED if h * w >= ph * w + pw + 16 else PACKED)
                y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
                unit.unit_conv2d_i8(d, xd, dev(wt), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
                torch.cuda.synchronize()
            assert same(host(y), ref, f"geometry {i} tile {tile}")


def test_strided_1x1_packs_only_the_pixels_it_reads():
    """1x1 convs with stride > 1 run as unit-stride convs on a subsampled packed tensor."""
    geoms = [(3, 70, 13, 9, 40, 2, 2), (2, 24, 8, 11, 17, 2, 3), (1, 130, 7, 7, 64, 3, 1), (4, 16, 5, 6, 8, 1, 2),
             (2, 5, 9, 10, 12, 2, 2)]               # (channels within one chunk: the per-pixel pack kernel)
    for i, (n, c, h, w, k, sh, sw) in enumerate(geoms):
        d = unit.conv_desc(n, c, h, w, k, 1, 1, (sh, sw), (0, 0))
        g = wl.rng(64, i)
        x = wl.int8_activations(g, (n, c, h, w))
        wt = wl.int8_weights(g, (k, c, 1, 1))
        ref = oracle.conv2d_i8(x, wt, (sh, sw), (0, 0))
        xh = wl.f16_activations(g, (n, c, h, w))
        wh = wl.f16_weights(g, (k, c, 1, 1), c)
        refh = oracle.conv2d_f16(xh, wh, (sh, sw), (0, 0))
        for tile, split in [(None, None), (3, 2), (4, 1), (1, 1)]:
            announce("strided 1x1", (n, c, h, w, k, sh, sw), "tile", tile, "split", split)
            with forced(tile=tile, split=split):
                y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
                unit.unit_conv2d_i8(d, dev(x), dev(wt), y, None, None, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_I8)))
                yh = torch.empty(ref.shape, dtype=torch.float32, device="cuda:0")
                unit.unit_conv2d_f16(d, dev(xh), dev(wh), yh, ws_bytes(unit.unit_conv2d_workspace(d, unit.UNIT_F16)))
                torch.cuda.synchronize()
            assert same(host(y), ref, f"geometry {i} tile {tile}")
            assert f16_rel_err(host(yh), refh, c) <= 1e-3, (i, tile)
