"""Seeded synthetic inputs and layer-shape tables for the benchmark configurations.

This module holds NO arithmetic of the method: only shapes and random draws.
Both the GPU tests and the CPU oracle's tests take their inputs from here, so
the two sides see byte-identical tensors without sharing any compute code.

The paper evaluated model-zoo networks with trained weights (Section V-C); those
are replaced by random tensors of the same shapes, because dense MAC timing and
exactness do not depend on the values.  Shape tables: a ResNet-50-shaped conv
set (53 layers), a ResNet-18-shaped chain, and the 16 layers of Table I.
"""
from collections import namedtuple

import numpy as np

BASE_SEED = 210108458

ConvShape = namedtuple("ConvShape", "c h w k r s stride pad")


def conv_shape(c, hw, k, r, stride, pad):
    return ConvShape(c, hw, hw, k, r, r, stride, pad)


def out_hw(sh):
    p = (sh.h + 2 * sh.pad - sh.r) // sh.stride + 1
    q = (sh.w + 2 * sh.pad - sh.s) // sh.stride + 1
    return p, q


def macs(sh, n=1):
    p, q = out_hw(sh)
    return n * sh.k * p * q * sh.c * sh.r * sh.s


def rng(config_id, layer_id=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + config_id * 1000 + layer_id))


# ----------------------------------------------------------------- generators

def int8_activations(g, shape):
    """int8 uniform in [-64, 63]."""
    return g.integers(-64, 64, size=shape, dtype=np.int8)


def int8_weights(g, shape):
    """int8 uniform in [-128, 127]."""
    return g.integers(-128, 128, size=shape, dtype=np.int8)


def f16_bits(values):
    """float array -> IEEE binary16 bit patterns (round-to-nearest-even) as uint16."""
    return np.ascontiguousarray(np.asarray(values, dtype=np.float64).astype(np.float16)).view(np.uint16)


def f16_activations(g, shape):
    """binary16 bit patterns of N(0,1) draws."""
    return f16_bits(g.standard_normal(size=shape))


def f16_weights(g, shape, fan_in):
    """binary16 bit patterns of N(0, 2/fan_in) draws (He initialisation)."""
    return f16_bits(g.standard_normal(size=shape) * np.sqrt(2.0 / fan_in))


def uint8_activations(g, shape):
    """Unsigned activations over the full byte range (post-ReLU quantised tensors)."""
    return g.integers(0, 256, size=shape, dtype=np.int64).astype(np.uint8)


def bf16_bits(values):
    """float32 array -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(values, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def _fp8_e4m3_magnitudes():
    """The 127 finite non-negative E4M3 values in code order (code 0x7F is NaN)."""
    codes = np.arange(127)
    expo, frac = codes >> 3, codes & 7
    return np.where(expo == 0, frac * 2.0 ** -9, (8 + frac) * 2.0 ** (expo - 10.0))


def fp8_e4m3_bits(values):
    """float array -> OCP E4M3 (finite-only) bit patterns: round to nearest, ties to the even
    code, magnitudes above 448 saturate."""
    v = np.asarray(values, dtype=np.float64)
    mags = _fp8_e4m3_magnitudes()
    a = np.minimum(np.abs(v), mags[-1])
    hi = np.clip(np.searchsorted(mags, a, side="left"), 1, 126)
    lo = hi - 1
    dlo, dhi = a - mags[lo], mags[hi] - a
    code = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo % 2 == 0, lo, hi)))
    return (code | (np.signbit(v).astype(np.int64) << 7)).astype(np.uint8)


def conv_inputs_fp8(sh, n, config_id, layer_id=0):
    g = rng(config_id, layer_id)
    x = fp8_e4m3_bits(g.standard_normal(size=(n, sh.c, sh.h, sh.w)))
    w = fp8_e4m3_bits(g.standard_normal(size=(sh.k, sh.c, sh.r, sh.s)) * np.sqrt(2.0 / (sh.c * sh.r * sh.s)))
    return x, w


def gemm_inputs_fp8(m, n, k, config_id=2, layer_id=4):
    g = rng(config_id, layer_id)
    return (fp8_e4m3_bits(g.standard_normal(size=(m, k))),
            fp8_e4m3_bits(g.standard_normal(size=(n, k)) * np.sqrt(2.0 / k)))


def conv_inputs_i8(sh, n, config_id, layer_id=0):
    g = rng(config_id, layer_id)
    x = int8_activations(g, (n, sh.c, sh.h, sh.w))
    w = int8_weights(g, (sh.k, sh.c, sh.r, sh.s))
    return x, w


def conv_inputs_f16(sh, n, config_id, layer_id=0):
    g = rng(config_id, layer_id)
    x = f16_activations(g, (n, sh.c, sh.h, sh.w))
    w = f16_weights(g, (sh.k, sh.c, sh.r, sh.s), sh.c * sh.r * sh.s)
    return x, w


def conv_inputs_u8i8(sh, n, config_id, layer_id=0):
    g = rng(config_id, layer_id)
    x = uint8_activations(g, (n, sh.c, sh.h, sh.w))
    w = int8_weights(g, (sh.k, sh.c, sh.r, sh.s))
    return x, w


def conv_inputs_bf16(sh, n, config_id, layer_id=0):
    g = rng(config_id, layer_id)
    x = bf16_bits(g.standard_normal(size=(n, sh.c, sh.h, sh.w)))
    w = bf16_bits(g.standard_normal(size=(sh.k, sh.c, sh.r, sh.s)) * np.sqrt(2.0 / (sh.c * sh.r * sh.s)))
    return x, w


def gemm_inputs_u8i8(m, n, k, config_id=2, layer_id=2):
    g = rng(config_id, layer_id)
    return uint8_activations(g, (m, k)), int8_weights(g, (n, k))


def gemm_inputs_bf16(m, n, k, config_id=2, layer_id=3):
    g = rng(config_id, layer_id)
    return (bf16_bits(g.standard_normal(size=(m, k))),
            bf16_bits(g.standard_normal(size=(n, k)) * np.sqrt(2.0 / k)))


def gemm_inputs_i8(m, n, k, config_id=2, layer_id=0):
    """A [m,k] row-major; B as [n,k] (column-major k x n)."""
    g = rng(config_id, layer_id)
    return int8_weights(g, (m, k)), int8_weights(g, (n, k))


def gemm_inputs_f16(m, n, k, config_id=2, layer_id=1):
    g = rng(config_id, layer_id)
    return f16_activations(g, (m, k)), f16_weights(g, (n, k), k)


# ----------------------------------------------------------------- shape tables

CONFIG1 = conv_shape(64, 56, 64, 3, 1, 1)          # single int8 conv, batch 1
LARGE_CONV = conv_shape(256, 56, 256, 3, 1, 1)     # batch 32: compute-bound showcase
GEMM_SQUARE = (4096, 4096, 4096)
GEMM_FC = (1, 1000, 2048)


def resnet50_convs():
    """The 53 conv layers of a ResNet-50-shaped network (stride on the 3x3), in order."""
    layers = [conv_shape(3, 224, 64, 7, 2, 3)]
    hw, cin = 56, 64
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)]):
        out = 4 * mid
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            layers.append(conv_shape(cin, hw, mid, 1, 1, 0))
            layers.append(conv_shape(mid, hw, mid, 3, stride, 1))
            hw_out = hw // stride
            layers.append(conv_shape(mid, hw_out, out, 1, 1, 0))
            if b == 0:
                layers.append(conv_shape(cin, hw, out, 1, stride, 0))
            cin, hw = out, hw_out
    return layers


def unique_shapes(layers):
    """[(shape, multiplicity)] in first-appearance order."""
    seen = {}
    for sh in layers:
        seen[sh] = seen.get(sh, 0) + 1
    return list(seen.items())


# Table I of the paper: 16 selected conv layers; IHW is the already-padded size (pad 0).
TABLE1 = [
    conv_shape(288, 35, 384, 3, 2, 0), conv_shape(160, 9, 224, 3, 1, 0),
    conv_shape(1056, 7, 192, 1, 1, 0), conv_shape(80, 73, 192, 3, 1, 0),
    conv_shape(128, 16, 128, 3, 1, 0), conv_shape(192, 16, 192, 3, 1, 0),
    conv_shape(256, 16, 256, 3, 1, 0), conv_shape(1024, 14, 512, 1, 1, 0),
    conv_shape(128, 16, 160, 3, 1, 0), conv_shape(576, 14, 192, 1, 1, 0),
    conv_shape(96, 16, 128, 3, 1, 0), conv_shape(1024, 14, 256, 1, 1, 0),
    conv_shape(576, 14, 128, 1, 1, 0), conv_shape(64, 29, 96, 3, 1, 0),
    conv_shape(64, 56, 128, 1, 2, 0), conv_shape(608, 14, 192, 1, 1, 0),
]


def resnet18_plan():
    """ResNet-18-shaped chain as a list of stages.

    Each basic block is (conv1, conv2, projection-or-None).  The stem is a 7x7/2
    conv followed by a 3x3/2 max-pool; the tail is a global average pool and a
    512 -> 1000 fully connected layer.
    """
    stem = conv_shape(3, 224, 64, 7, 2, 3)
    blocks = []
    hw, cin = 56, 64
    for stage, width in enumerate([64, 128, 256, 512]):
        for b in range(2):
            stride = 2 if (b == 0 and stage > 0) else 1
            c1 = conv_shape(cin, hw, width, 3, stride, 1)
            hw_out = hw // stride
            c2 = conv_shape(width, hw_out, width, 3, 1, 1)
            proj = conv_shape(cin, hw, width, 1, stride, 0) if (stride != 1 or cin != width) else None
            blocks.append((c1, c2, proj))
            cin, hw = width, hw_out
    return {"stem": stem, "blocks": blocks, "fc": (512, 1000)}
