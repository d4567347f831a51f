"""conv3d parity (the paper's extensibility experiment: ResNet-18 convolutions lifted to 3-D)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2101_08458_amd import unit, workloads as wl
from gpu_util import announce, dev, host, forced, f16_rel_err, as_accurate_as_oracle, same

pytestmark = pytest.mark.gpu

# (n, c, d, h, w, k, t, r, s, stride, pad): ResNet-18-shaped layers with a depth axis, scaled to test size
CASES = [
    (1, 3, 8, 32, 32, 16, 7, 7, 7, (2, 2, 2), (3, 3, 3)),        # stem-like
    (1, 64, 4, 14, 14, 64, 3, 3, 3, (1, 1, 1), (1, 1, 1)),
    (2, 32, 6, 9, 10, 48, 3, 3, 3, (2, 2, 2), (1, 1, 1)),
    (1, 64, 4, 14, 14, 128, 1, 1, 1, (2, 2, 2), (0, 0, 0)),       # projection
    (1, 40, 3, 8, 8, 24, 1, 1, 1, (1, 1, 1), (0, 0, 0)),          # 1x1x1, one image: read directly from NCDHW
    (1, 20, 5, 7, 6, 33, 2, 3, 1, (1, 2, 1), (1, 0, 0)),          # anisotropic everything
]


def ws(n):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device="cuda:0")


@pytest.mark.parametrize("case", CASES)
def test_conv3d_parity(case):
    n, c, d, h, w_, k, t, r, s, stride, pad = case
    g = wl.rng(120, c * 10 + d)
    x = wl.int8_activations(g, (n, c, d, h, w_))
    w = wl.int8_weights(g, (k, c, t, r, s))
    ref = oracle.conv3d_i8(x, w, stride, pad)
    xh = wl.f16_activations(g, (n, c, d, h, w_))
    wh = wl.f16_weights(g, (k, c, t, r, s), c * t * r * s)
    refh, truth, mag = oracle.conv3d_f16(xh, wh, stride, pad)
    desc = unit.conv3d_desc(n, c, d, h, w_, k, t, r, s, stride, pad)
    assert unit.unit_conv3d_out_dims(desc) == ref.shape[2:]
    xd, wd, xhd, whd = dev(x), dev(w), dev(xh), dev(wh)
    kred = c * t * r * s
    for tile, split in [(None, None), (0, 1), (1, 2), (3, 1), (4, 2), (5, 1), (6, 1), (7, 1), (8, 1), (9, 2), (10, 1), (11, 1), (12, 1), (12, 2)]:
        announce("conv3d", case, "tile", tile, "split", split)
        with forced(tile=tile, split=split):
            y = torch.full(ref.shape, -7, dtype=torch.int32, device="cuda:0")
            unit.unit_conv3d_i8(desc, xd, wd, y, ws(unit.unit_conv3d_workspace(desc, unit.UNIT_I8)))
            yh = torch.empty(ref.shape, dtype=torch.float32, device="cuda:0")
            unit.unit_conv3d_f16(desc, xhd, whd, yh, ws(unit.unit_conv3d_workspace(desc, unit.UNIT_F16)))
            torch.cuda.synchronize()
        assert same(host(y), ref, f"i8 tile {tile} split {split}")
        got = host(yh)
        assert f16_rel_err(got, refh, kred) <= 1e-3, (tile, split)
        assert np.all(np.abs(got - truth) <= 2 * kred * 2.0 ** -24 * mag + 1e-30), (tile, split)
        assert as_accurate_as_oracle(got, refh, truth), (tile, split)


def test_conv3d_depth_one_matches_conv2d_call():
    """The 2-D entry point is the depth-1 case of the same kernel."""
    sh = wl.ConvShape(24, 12, 12, 40, 3, 3, 2, 1)
    x, w = wl.conv_inputs_i8(sh, 2, 121)
    d2 = unit.conv_desc(2, sh.c, sh.h, sh.w, sh.k, 3, 3, 2, 1)
    d3 = unit.conv3d_desc(2, sh.c, 1, sh.h, sh.w, sh.k, 1, 3, 3, (1, 2, 2), (0, 1, 1))
    p, q = unit.unit_conv2d_out_dims(d2)
    xd, wd = dev(x), dev(w)
    y2 = torch.empty((2, sh.k, p, q), dtype=torch.int32, device="cuda:0")
    y3 = torch.empty((2, sh.k, 1, p, q), dtype=torch.int32, device="cuda:0")
    announce("conv3d depth 1")
    unit.unit_conv2d_i8(d2, xd, wd, y2, None, None, ws(unit.unit_conv2d_workspace(d2, unit.UNIT_I8)))
    unit.unit_conv3d_i8(d3, xd, wd, y3, ws(unit.unit_conv3d_workspace(d3, unit.UNIT_I8)))
    torch.cuda.synchronize()
    assert same(host(y3)[:, :, 0], host(y2), "depth 1")
    assert same(host(y2), oracle.conv2d_i8(x, w, (2, 2), (1, 1)), "vs oracle")
