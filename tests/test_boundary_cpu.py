"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
declared symbol, answers the size / selector queries, and rejects bad arguments before
any HIP call (all error paths return ahead of the first launch)."""
import ctypes
import os
import re

import pytest

from paper_2101_08458_amd import unit, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(unit.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return unit.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "unit.h")).read()
    declared = set(re.findall(r"\b(unit_[a-z0-9_]+)\s*\(", header))
    assert declared == set(unit.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert unit.unit_version() >= 100
    assert unit.unit_status_str(unit.UNIT_EOVERFLOW).startswith("byte reduction")


def test_out_dims_and_sizes(lib):
    for sh in wl.resnet50_convs() + wl.TABLE1:
        d = unit.conv_desc(1, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
        assert unit.unit_conv2d_out_dims(d) == wl.out_hw(sh)
    assert unit.unit_packed_act_bytes(1, 3, 224, 224, unit.UNIT_I8) == 224 * 224 * 16
    assert unit.unit_packed_act_bytes(2, 24, 5, 5, unit.UNIT_F16) == (2 * 25 * 24 * 2 + 255) // 256 * 256
    d = unit.conv_desc(1, 64, 56, 56, 64, 3, 3, 1, 1)
    assert unit.unit_packed_weights_bytes(d, unit.UNIT_I8) == 64 * 9 * 64
    assert unit.unit_conv2d_workspace(d, unit.UNIT_I8) >= 56 * 56 * 64 + 64 * 9 * 64
    assert unit.unit_packed_act_bytes(0, 3, 4, 4, unit.UNIT_I8) == 0


def test_selector_answers(lib):
    info = unit.unit_select_matmul(4096, 4096, 4096, unit.UNIT_I8)
    assert info.block_m * info.block_n >= 128 * 128 and info.split_k == 1
    assert info.workgroups == (4096 // info.block_m) * (4096 // info.block_n)
    # the batch-1 fully connected shape runs on the dot-product path (one wave per column), from 5 rows on the MFMA tile
    info = unit.unit_select_matmul(1, 1000, 2048, unit.UNIT_I8)
    assert (info.mfma, info.block_n, info.workgroups, info.split_k) == (0, 4, 250, 1)
    assert unit.unit_select_matmul(4, 1000, 512, unit.UNIT_F16).mfma == 0
    assert unit.unit_select_matmul(8, 1000, 512, unit.UNIT_I8).mfma == 16
    assert unit.unit_select_matmul(1, 1000, 2048, unit.UNIT_FP8).mfma == 16
    assert unit.unit_matmul_workspace(1, 1000, 2048, 2048, 2048, unit.UNIT_I8) == 0
    # a deep, small layer (7x7 output, reduction 4608): split across 32x32 workgroups in the shifted direct read, whole
    # on 16x16 tiles when the activations are packed; the workspace query covers the partial sums of the split
    d = unit.conv_desc(1, 512, 7, 7, 512, 3, 3, 1, 1)
    info = unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_DIRECT_SHIFTED)
    assert info.block_m == 32 and info.split_k > 1 and info.workgroups >= 128
    assert unit.unit_conv2d_wpacked_workspace(d, unit.UNIT_I8) >= info.split_k * 512 * 49 * 4
    info = unit.unit_select_conv2d(d, unit.UNIT_I8)
    assert (info.block_m, info.block_n, info.split_k, info.workgroups) == (16, 16, 1, 32 * 4)
    # ... and a reduction far beyond that is cut into slices of 32 of the tile's steps
    info = unit.unit_select_matmul(64, 64, 32768, unit.UNIT_I8)
    assert (info.block_m, info.block_k_bytes, info.split_k) == (16, 256, 4)
    # per input mode: the packed answer is unit_select_conv2d's; the shifted direct read splits a
    # 14x14 layer of 14 steps that the packed path leaves whole; an unknown mode is an error
    d = unit.conv_desc(1, 192, 14, 14, 192, 3, 3, 1, 1)
    packed = unit.unit_select_conv2d(d, unit.UNIT_I8)
    same = unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_PACKED)
    assert (same.block_m, same.block_n, same.split_k, same.workgroups) == \
           (packed.block_m, packed.block_n, packed.split_k, packed.workgroups)
    shifted = unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_DIRECT_SHIFTED)
    assert packed.split_k == 1 and shifted.split_k > 1
    assert (shifted.block_m, shifted.block_n, shifted.block_k_bytes) == (32, 32, 64)      # 192-byte pixels: 64-byte steps
    assert shifted.workgroups == 6 * 7 * shifted.split_k
    assert (packed.block_m, packed.block_n, packed.workgroups) == (16, 16, 12 * 13)       # packed rows: the 16x16 tile
    # few output elements and a reduction of four to ten 256-byte steps: the 16x16 tile, one workgroup per 16 channels x
    # 16 pixels and no split, in every input mode (the 256-channel 14x14 layers, 1024 -> 256 at 14x14, 2048 -> 512 at 7x7);
    # not for a deeper reduction, for more output elements, or for fp8 (no kernel of that tile)
    for shape, wgs in (((256, 14, 14, 256, 3, 3, 1, 1), 16 * 13), ((1024, 14, 14, 256, 1, 1, 1, 0), 16 * 13),
                       ((2048, 7, 7, 512, 1, 1, 1, 0), 32 * 4)):
        d = unit.conv_desc(1, *shape)
        modes = (unit.UNIT_INPUT_PACKED, unit.UNIT_INPUT_DIRECT_SHIFTED if shape[4] == 3 else unit.UNIT_INPUT_DIRECT)
        for mode in modes:
            info = unit.unit_select_conv2d_input(d, unit.UNIT_I8, mode)
            assert (info.block_m, info.block_n, info.block_k_bytes, info.mfma, info.split_k, info.workgroups) == \
                   (16, 16, 256, 16, 1, wgs), (shape, mode)
        assert unit.unit_select_conv2d_input(d, unit.UNIT_FP8, unit.UNIT_INPUT_PACKED).block_m == 32
    d = unit.conv_desc(1, 256, 14, 14, 1024, 1, 1, 1, 0)        # 224 tiles of 32x32: stays, packed or direct
    assert unit.unit_select_conv2d(d, unit.UNIT_I8).block_m == 32
    assert unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_DIRECT).block_m == 32
    d = unit.conv_desc(1, 1024, 14, 14, 512, 1, 1, 1, 0)        # 112 tiles: 16x16 on packed rows only
    assert unit.unit_select_conv2d(d, unit.UNIT_I8).block_m == 16
    assert unit.unit_select_conv2d_input(d, unit.UNIT_I8, unit.UNIT_INPUT_DIRECT).block_m == 32
    d = unit.conv_desc(1, 64, 56, 56, 128, 1, 1, 2, 0)          # four chunks of reduction: too shallow
    assert unit.unit_select_conv2d(d, unit.UNIT_I8).block_m == 32
    assert unit.unit_select_matmul(256, 196, 2304, unit.UNIT_I8).block_m == 16
    info = unit.unit_tile_info()
    assert lib.unit_select_conv2d_input(ctypes.byref(d), unit.UNIT_I8, 3, ctypes.byref(info)) == unit.UNIT_EINVAL
    assert lib.unit_select_conv2d_input(ctypes.byref(d), unit.UNIT_I8, 0, None) == unit.UNIT_EINVAL


def test_error_paths_return_before_launch(lib):
    d = unit.conv_desc(1, 8, 8, 8, 8, 3, 3, 1, 1)
    null = None
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    st = 0
    f = lib.unit_conv2d_i8
    assert f(None, fake, fake, fake, None, null, fake, 1 << 20, st) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), null, fake, fake, None, null, fake, 1 << 20, st) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), fake, fake, null, None, null, fake, 1 << 20, st) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), fake, fake, fake, None, null, null, 0, st) == unit.UNIT_EWORKSPACE
    assert f(ctypes.byref(d), fake, fake, fake, None, null, fake, 16, st) == unit.UNIT_EWORKSPACE
    # requant without an int8 output / without scale
    rq = unit.unit_requant(None, None, None, 0)
    assert f(ctypes.byref(d), fake, fake, fake, ctypes.byref(rq), fake, fake, 1 << 20, st) == unit.UNIT_EINVAL
    sc = 0x2000
    rq2 = unit.unit_requant(sc, None, None, 1, 3, fake + 4)   # packed residual not 16-byte aligned
    assert lib.unit_conv2d_packed_i8(ctypes.byref(d), fake, fake, None, ctypes.byref(rq2), fake, None, None, 0, st) == unit.UNIT_EINVAL
    rq3 = unit.unit_requant(sc, None, None, 1, 0, None)
    assert lib.unit_conv2d_packed_i8(ctypes.byref(d), fake, fake, None, ctypes.byref(rq3), None, fake + 8, None, 0, st) == unit.UNIT_EINVAL  # packed output misaligned
    bad = unit.conv_desc(1, 8, 2, 2, 8, 3, 3, 1, 0)          # window larger than the image
    assert f(ctypes.byref(bad), fake, fake, fake, None, null, fake, 1 << 20, st) == unit.UNIT_EINVAL
    neg = unit.conv_desc(1, 8, 8, 8, 8, 3, 3, 0, 1)          # stride 0
    assert f(ctypes.byref(neg), fake, fake, fake, None, null, fake, 1 << 20, st) == unit.UNIT_EINVAL
    deep = unit.conv_desc(1, 14564, 8, 8, 8, 3, 3, 1, 1)     # 14564*9 = 131076 > 131071
    assert f(ctypes.byref(deep), fake, fake, fake, None, null, fake, 1 << 30, st) == unit.UNIT_EOVERFLOW
    ok_deep = unit.conv_desc(1, 14563, 8, 8, 8, 3, 3, 1, 1)  # 131067: allowed for int8 ...
    assert unit.unit_conv2d_workspace(ok_deep, unit.UNIT_I8) > 0
    assert unit.unit_conv2d_workspace(deep, unit.UNIT_F16) > 0   # ... and fp16 has no such bound

    g = lib.unit_matmul_i8
    assert g(0, 4, 4, fake, 4, fake, 4, fake, 4, null, 0, st) == unit.UNIT_EINVAL
    assert g(4, 4, 16, fake, 8, fake, 16, fake, 4, null, 0, st) == unit.UNIT_EINVAL      # lda < k
    assert g(4, 4, 16, fake, 16, fake, 16, fake, 2, null, 0, st) == unit.UNIT_EINVAL     # ldc < n
    assert g(4, 4, 131072, fake, 131072, fake, 131072, fake, 4, null, 0, st) == unit.UNIT_EOVERFLOW
    assert g(4, 4, 10, fake, 10, fake, 10, fake, 4, null, 0, st) == unit.UNIT_EWORKSPACE  # needs padding space
    assert g(4, 4, 16, fake + 1, 16, fake, 16, fake, 4, null, 0, st) == unit.UNIT_EINVAL  # misaligned A
    assert lib.unit_matmul_f16(4, 4, 131072, null, 131072, fake, 131072, fake, 4, null, 0, st) == unit.UNIT_EINVAL
    assert lib.unit_pack_act_i8(1, 3, 4, 4, fake, fake, 16, st) == unit.UNIT_EWORKSPACE
    assert lib.unit_maxpool_packed_i8(1, 16, 8, 8, 3, 2, 3, fake, fake, st) == unit.UNIT_EINVAL


def test_size_limits_and_wpacked_errors(lib):
    fake, st = 0x1000, 0
    # every tensor addressed through a buffer descriptor must stay below 2 GiB
    big_act = unit.conv_desc(64, 512, 256, 256, 8, 1, 1, 1, 0)           # 2 GiB of int8 activations
    assert lib.unit_conv2d_packed_i8(ctypes.byref(big_act), fake, fake, fake, None, None, None, None, 0, st) == unit.UNIT_ENOTSUP
    big_out = unit.conv_desc(32, 16, 512, 512, 64, 1, 1, 1, 0)           # 2 GiB of int32 outputs
    assert lib.unit_conv2d_packed_i8(ctypes.byref(big_out), fake, fake, fake, None, None, None, None, 0, st) == unit.UNIT_ENOTSUP
    assert unit.unit_conv2d_workspace(big_act, unit.UNIT_I8) == 0
    assert lib.unit_matmul_i8(4, 4, 16, fake, 1 << 24, fake, 16, fake, 4, None, 0, st) == unit.UNIT_ENOTSUP
    d = unit.conv_desc(1, 64, 8, 8, 32, 1, 1, 1, 0)
    f = lib.unit_conv2d_wpacked_i8
    assert f(ctypes.byref(d), None, fake, fake, None, None, None, 0, st) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), fake, fake, None, None, None, None, 0, st) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), fake, fake + 4, fake, None, None, None, 0, st) == unit.UNIT_EINVAL       # misaligned packed weights
    d3 = unit.conv_desc(1, 64, 8, 8, 32, 3, 3, 2, 1)                      # strided 3x3 needs the pack workspace
    assert f(ctypes.byref(d3), fake, fake, fake, None, None, None, 0, st) == unit.UNIT_EWORKSPACE
    assert unit.unit_conv2d_wpacked_workspace(d3, unit.UNIT_I8) >= 64 * 64
    assert lib.unit_conv2d_wpacked_f16(ctypes.byref(d), fake, fake, None, None, 0, st) == unit.UNIT_EINVAL


def test_column_range_plan(lib):
    """Tile-count-aware selection: whole rounds of 256 x 256 tiles, then a narrower tile for the remaining columns
    when those would otherwise leave a round of workgroups mostly empty."""
    q = lambda m, n, k=4096: unit.unit_select_matmul(m, n, k, unit.UNIT_I8)
    i = q(4096, 4096)
    assert (i.block_n, i.workgroups, i.tail_block_n) == (256, 256, 0)                  # exactly one round
    assert q(8192, 8192).tail_block_n == 0                                             # four whole rounds
    i = q(4096, 6144)                                                                  # 1.5 rounds: tail of 128 tiles -> 256 x 128
    assert (i.workgroups, i.tail_block_n, i.tail_workgroups, i.tail_first_col) == (256, 128, 256, 4096)
    i = q(4096, 4096 + 34 * 256)                                                       # 800 tiles = 3 rounds + 32: those as 64 tiles of 256 x 128
    assert (i.workgroups, i.tail_block_n, i.tail_workgroups, i.tail_first_col) == (768, 128, 64, 48 * 256)
    assert q(2048, 40000).tail_block_n == 0                                            # last round 91 % full: left alone
    assert q(4096, 4096, 256).tail_block_n == 0                                        # short reductions do not use the large tile
    sh = wl.LARGE_CONV                                                                 # the benchmark's large conv: 392 tiles
    d = unit.conv_desc(32, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
    for dt in (unit.UNIT_I8, unit.UNIT_F16, unit.UNIT_FP8):
        i = unit.unit_select_conv2d(d, dt)
        assert (i.block_m, i.block_n, i.workgroups) == (256, 256, 256)
        assert (i.tail_block_n, i.tail_workgroups, i.tail_first_col) == (192, 182, 65536)
    unit.unit_debug_force_tile(8, -1)                                                  # a forced tile is one launch
    try:
        assert unit.unit_select_conv2d(d, unit.UNIT_I8).tail_block_n == 0
    finally:
        unit.unit_debug_force_tile(-1, -1)


def test_input_mode_decisions_are_host_logic(lib):
    """Which layers skip pack_act is decided on the host from the shape and the alignment of
    `x` alone (nothing is dereferenced), so the rule can be checked without a GPU."""
    x = 0x7f0000000000            # 16-byte aligned, never dereferenced
    mode = lambda *a, dtype=unit.UNIT_I8, ptr=x: lib.unit_conv2d_input_mode(
        ctypes.byref(unit.conv_desc(*a)), dtype, ctypes.c_void_p(ptr))
    P, D, S = unit.UNIT_INPUT_PACKED, unit.UNIT_INPUT_DIRECT, unit.UNIT_INPUT_DIRECT_SHIFTED
    assert mode(1, 64, 56, 56, 256, 1, 1, 1, 0) == D              # aligned 1x1
    assert mode(16, 64, 56, 56, 256, 1, 1, 1, 0, dtype=unit.UNIT_F16) == D   # batches: whole chunks per image
    assert mode(16, 256, 14, 14, 1024, 1, 1, 1, 0, dtype=unit.UNIT_F16) == D  # batches: columns tiled per image
    # 49-byte rows: some loads start inside a dword, whose range check would lose the tensor's last bytes; the
    # kernel patches them from a copy of the last 16 bytes, wherever the tensor lies (whole steps of channels only)
    assert mode(16, 512, 7, 7, 2048, 1, 1, 1, 0) == D
    assert mode(16, 512, 7, 7, 2048, 1, 1, 1, 0, ptr=x + 512) == D
    assert mode(1, 512, 7, 7, 2048, 1, 1, 1, 0) == D
    assert mode(1, 512, 7, 7, 2048, 1, 1, 1, 0, dtype=unit.UNIT_F16) == D     # 98-byte rows
    assert mode(1, 520, 7, 7, 2048, 1, 1, 1, 0) == P              # unaligned rows and a partial last step of channels
    assert mode(1, 520, 6, 6, 2048, 1, 1, 1, 0) == D              # 36-byte rows: dword-aligned, any channel count
    assert mode(1, 512, 3, 5, 2048, 1, 1, 1, 0) == P              # 15 pixels: less than one chunk of one-byte elements
    assert mode(1, 256, 14, 14, 256, 3, 3, 1, 1) == S             # 3x3, same padding
    assert mode(1, 128, 11, 10, 33, 5, 5, 1, 2) == S
    assert mode(1, 64, 56, 56, 64, 3, 3, 1, 1) == S               # 64 int8 channels: the small tile with 64-byte steps
    assert mode(1, 32, 56, 56, 64, 3, 3, 1, 1) == P               # 32 int8 channels: less than any tile's step
    assert mode(1, 64, 56, 56, 64, 3, 3, 1, 1, dtype=unit.UNIT_F16) == S
    assert mode(2, 256, 14, 14, 256, 3, 3, 1, 1) == S             # batches: columns tiled per image (196 = 12.25 chunks)
    assert mode(2, 128, 28, 28, 128, 3, 3, 1, 1) == S             # batches: whole chunks per image
    assert mode(16, 128, 28, 28, 128, 3, 3, 1, 1) == P            # large batches: packing first is cheaper than unaligned loads
    assert mode(64, 128, 5, 5, 512, 3, 3, 1, 1) == P              # 25-pixel images would leave 64-wide tiles mostly empty
    assert mode(1, 256, 14, 14, 256, 3, 3, 2, 1) == P             # stride 2
    assert mode(1, 256, 14, 14, 256, 3, 3, 1, 0) == P             # output grid smaller than the input
    assert mode(1, 256, 14, 14, 256, 3, 3, 1, 1, dtype=unit.UNIT_U8I8) == P
    assert mode(1, 256, 14, 14, 256, 3, 3, 1, 1, ptr=x + 8) == P  # misaligned tensor
    assert mode(1, 3, 224, 224, 64, 7, 7, 2, 3) == P              # the stem
    assert lib.unit_conv2d_input_mode(ctypes.byref(unit.conv_desc(1, 8, 8, 8, 8, 3, 3, 1, 1)),
                                      unit.UNIT_I8, None) == unit.UNIT_EINVAL
    assert mode(1, 8, 2, 2, 8, 5, 5, 1, 0) == unit.UNIT_EINVAL    # empty output
    # the ResNet-50-shaped set at batch 1: 46 of the 53 layers read NCHW directly
    direct = sum(mode(1, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad) != P for sh in wl.resnet50_convs())
    assert direct == 46


def test_debug_force_tile_overrides_and_restores_the_rule(lib):
    """The sweep / test hook is a setter, not an environment variable: what it forces shows up in the
    selector queries, a tile without a kernel for an input mode falls back to packed activations,
    and (-1, -1) restores the rule."""
    import os
    d = unit.conv_desc(1, 256, 14, 14, 256, 3, 3, 1, 1)
    rule = unit.unit_select_conv2d(d, unit.UNIT_I8)
    x = ctypes.c_void_p(0x7f0000000000)
    assert lib.unit_conv2d_input_mode(ctypes.byref(d), unit.UNIT_I8, x) == unit.UNIT_INPUT_DIRECT_SHIFTED
    try:
        os.environ["UNIT_TILE"], os.environ["UNIT_SPLITK"] = "1", "5"      # not read any more
        same = unit.unit_select_conv2d(d, unit.UNIT_I8)
        assert (same.block_m, same.split_k) == (rule.block_m, rule.split_k)
        unit.unit_debug_force_tile(3, 2)
        f = unit.unit_select_conv2d(d, unit.UNIT_I8)
        assert (f.block_m, f.block_n, f.waves_k, f.split_k) == (64, 64, 2, 2)
        unit.unit_debug_force_tile(2, -1)                       # tile only: the split is the rule's again
        assert unit.unit_select_conv2d(d, unit.UNIT_I8).waves_k == 4
        # the direct modes' preconditions are re-checked against a forced tile: 64 int8 channels are half
        # a step of the 128x128x128 B tile, so the call would pack first instead of running the shifted read
        d64 = unit.conv_desc(1, 64, 56, 56, 64, 3, 3, 1, 1)
        unit.unit_debug_force_tile(-1, -1)
        assert lib.unit_conv2d_input_mode(ctypes.byref(d64), unit.UNIT_I8, x) == unit.UNIT_INPUT_DIRECT_SHIFTED
        unit.unit_debug_force_tile(1, -1)
        assert lib.unit_conv2d_input_mode(ctypes.byref(d64), unit.UNIT_I8, x) == unit.UNIT_INPUT_PACKED
        # the 256 x 192 tile has no direct-read kernels (a DMA instruction must cover whole channel rows of the
        # column tile): forcing it makes a direct-capable layer pack first
        unit.unit_debug_force_tile(10, -1)
        d1 = unit.conv_desc(1, 256, 56, 56, 64, 1, 1, 1, 0)
        assert lib.unit_conv2d_input_mode(ctypes.byref(d1), unit.UNIT_I8, x) == unit.UNIT_INPUT_PACKED
        assert lib.unit_conv2d_input_mode(ctypes.byref(d), unit.UNIT_I8, x) == unit.UNIT_INPUT_PACKED
        unit.unit_debug_force_tile(-1, -1)
        assert lib.unit_conv2d_input_mode(ctypes.byref(d1), unit.UNIT_I8, x) == unit.UNIT_INPUT_DIRECT
        assert lib.unit_debug_force_tile(99, 1) == unit.UNIT_EINVAL
    finally:
        os.environ.pop("UNIT_TILE", None)
        os.environ.pop("UNIT_SPLITK", None)
        unit.unit_debug_force_tile(-1, -1)
    back = unit.unit_select_conv2d(d, unit.UNIT_I8)
    assert (back.block_m, back.block_n, back.split_k) == (rule.block_m, rule.block_n, rule.split_k)


def test_batch_limit_is_refused_before_launch(lib):
    fake, st = 0x1000, 0
    d = unit.conv_desc(65536, 16, 2, 2, 8, 1, 1, 1, 0)
    assert lib.unit_conv2d_i8(ctypes.byref(d), fake, fake, fake, None, None, fake, 1 << 30, st) == unit.UNIT_ENOTSUP
    assert lib.unit_pack_act_i8(65536, 16, 2, 2, fake, fake, 1 << 30, st) == unit.UNIT_ENOTSUP
    assert unit.unit_conv2d_workspace(d, unit.UNIT_I8) == 0


def test_static_scratch_limit_and_argument_errors(lib):
    """The entry point without a workspace refuses what its static buffer cannot hold, and bad
    arguments, before its first HIP call (no GPU needed to see it)."""
    fake = 0x7f0000000000
    big = unit.conv_desc(64, 3, 224, 224, 64, 7, 7, 2, 3)        # 51 MB of packed activations
    assert unit.unit_conv2d_wpacked_workspace(big, unit.UNIT_I8) > unit.UNIT_STATIC_SCRATCH_BYTES
    f = lib.unit_conv2d_wpacked_i8_static
    assert f(ctypes.byref(big), fake, fake, fake, None, None, 0) == unit.UNIT_ESCRATCH
    d = unit.conv_desc(1, 64, 8, 8, 32, 3, 3, 2, 1)
    assert f(ctypes.byref(d), None, fake, fake, None, None, 0) == unit.UNIT_EINVAL
    assert f(ctypes.byref(d), fake, fake, None, None, None, 0) == unit.UNIT_EINVAL
    assert "static" in unit.unit_status_str(unit.UNIT_ESCRATCH)


def test_build_check_rejects_spills_in_inline_asm_variants(tmp_path):
    """The build fails when a direct-read kernel variant that issues its transposing LDS reads as inline
    assembly has scratch or spilled vector registers (the compiler's resource remarks are parsed by
    csrc/check_resources.py); variants that keep the builtins may spill."""
    import glob
    import subprocess
    import sys
    script = os.path.join(ROOT, "paper_2101_08458_amd", "csrc", "check_resources.py")

    def remark(args, scratch, vspill):
        name = "_ZN4unit12igemm_kernelI" + "".join(f"Li{a}E" for a in args) + "EEvNS_9IgemmArgsE"
        tail = " [-Rpass-analysis=kernel-resource-usage]\n"
        return (f"./igemm.hpp:301:1: remark: Function Name: {name}{tail}"
                f"./igemm.hpp:301:1: remark:     VGPRs: 128{tail}"
                f"./igemm.hpp:301:1: remark:     ScratchSize [bytes/lane]: {scratch}{tail}"
                f"./igemm.hpp:301:1: remark:     SGPRs Spill: 9{tail}"
                f"./igemm.hpp:301:1: remark:     VGPRs Spill: {vspill}{tail}")

    def run(text):
        f = tmp_path / "k.res"
        f.write_text(text)
        return subprocess.run([sys.executable, script, str(f)], capture_output=True, text=True).returncode

    direct_i8 = [0, 32, 32, 128, 1, 1, 4, 32, 4, 2, 3, 0]
    gather_i8 = [0, 32, 32, 128, 1, 1, 4, 32, 4, 2, 1, 0]
    fp8_big = [5, 256, 256, 128, 2, 4, 1, 32, 2, 1, 2, 0]       # 32-byte fragments, 8 MFMA tiles: builtin reads
    assert run(remark(direct_i8, 0, 0) + remark(gather_i8, 64, 12)) == 0     # spills elsewhere do not matter
    assert run(remark(direct_i8, 16, 0)) == 1
    assert run(remark(direct_i8, 0, 3)) == 1
    assert run(remark(fp8_big, 40, 7) + remark(direct_i8, 0, 0)) == 0
    assert run(remark(gather_i8, 0, 0)) == 1                                 # nothing to check: wrong input
    res = sorted(glob.glob(os.path.join(ROOT, "paper_2101_08458_amd", "csrc", "_build", "*.res")))
    if res:                                                                  # the tree's own build, when present
        assert subprocess.run([sys.executable, script] + res, capture_output=True).returncode == 0


def test_column_range_plan_invariants_on_random_shapes(lib):
    """Host logic of the two-launch plan over 3000 seeded random matmul shapes: the first launch covers whole column tiles
    of the large tile from column 0, the second the rest in at most one round of workgroups, and together exactly [0, n)."""
    import numpy as np
    g = wl.rng(77, 1)
    two = 0
    for _ in range(3000):
        m = int(g.integers(1, 9000)); n = int(g.integers(1, 200000)); k = int(g.choice([64, 256, 512, 1024, 4096, 9000]))
        for ut in (unit.UNIT_I8, unit.UNIT_F16, unit.UNIT_FP8):
            i = unit.unit_select_matmul(m, n, k, ut)
            tm = -(-m // i.block_m) if i.mfma else 0
            if not i.tail_block_n:
                assert i.tail_workgroups == 0 and i.tail_first_col == 0
                if i.mfma:
                    assert i.workgroups == tm * -(-n // i.block_n) * i.split_k
                continue
            two += 1
            assert (i.block_m, i.block_n, i.split_k) == (256, 256, 1) and i.tail_block_n in (128, 192)
            assert 0 < i.tail_first_col < n and i.tail_first_col % 256 == 0
            assert i.workgroups == tm * (i.tail_first_col // 256)
            rounds = -(-i.workgroups // 256)                                               # whole rounds, short by less than one column of tiles
            assert 0 <= 256 * rounds - i.workgroups < tm
            assert i.tail_workgroups == tm * -(-(n - i.tail_first_col) // i.tail_block_n) <= 256
    assert two > 50          # the sample does exercise the two-launch branch
