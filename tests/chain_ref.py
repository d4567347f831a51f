"""CPU reference for the chained ResNet-18-shaped int8 network: composes the oracle's
functions layer by layer and calibrates the per-channel scales on the way (scale[k] =
127 / max|t[.,k,.,.]| times a fixed jitter in [0.5, 1]), so that activations neither
saturate nor vanish.  The scales, biases and residual multipliers it returns are then fed
unchanged to the GPU path.  Chain parity is pinned by composition only: every stage used
here is pinned on its own in tests/test_oracle_*.py."""
import numpy as np

import oracle
from paper_2101_08458_amd import workloads as wl
from paper_2101_08458_amd.resnet18_int8 import layer_list


def _calibrate(t, g):
    k = t.shape[1]
    peak = np.abs(t.astype(np.int64)).max(axis=(0, 2, 3)).clip(1)
    return (127.0 / peak * g.uniform(0.5, 1.0, k)).astype(np.float32)


def build(batch, config_id=5):
    g = wl.rng(config_id, batch)
    plan = wl.resnet18_plan()
    params = {"res_mult": {}}
    x = wl.int8_activations(g, (batch, 3, 224, 224))
    for name, sh in layer_list():
        params[name] = {"w": wl.int8_weights(g, (sh.k, sh.c, sh.r, sh.s)),
                        "bias": g.integers(-2000, 2000, size=sh.k).astype(np.int32), "scale": None}
    params["fc_w"] = wl.int8_weights(g, (1000, 512))
    ref = {}

    def conv(name, inp):
        sh = dict(layer_list())[name]
        return oracle.conv2d_i8(inp, params[name]["w"], (sh.stride,) * 2, (sh.pad,) * 2)

    acc = conv("stem", x)
    t = acc + params["stem"]["bias"][None, :, None, None]
    params["stem"]["scale"] = _calibrate(t, g)
    a = oracle.requant(acc, params["stem"]["scale"], bias=params["stem"]["bias"], relu=True)
    ref["stem"] = a
    cur = oracle.maxpool_i8(a)
    ref["pool"] = cur
    for i, (c1, c2, proj) in enumerate(plan["blocks"]):
        n1, n2 = f"b{i}.c1", f"b{i}.c2"
        acc1 = conv(n1, cur)
        params[n1]["scale"] = _calibrate(acc1 + params[n1]["bias"][None, :, None, None], g)
        a1 = oracle.requant(acc1, params[n1]["scale"], bias=params[n1]["bias"], relu=True)
        acc2 = conv(n2, a1)
        if proj is not None:
            params[f"b{i}.proj"]["bias"] = None
            res = conv(f"b{i}.proj", cur)
        else:
            peak = max(int(np.abs(acc2).max()), 1)
            mult = 1 << max(int(np.round(np.log2(peak / 127.0))) - 1, 0)
            params["res_mult"][i] = mult
            res = oracle.widen_scale_i8(cur, mult)
        t2 = acc2.astype(np.int64) + params[n2]["bias"][None, :, None, None] + res
        assert np.abs(t2).max() < 2 ** 31
        params[n2]["scale"] = _calibrate(t2, g)
        cur = oracle.requant(acc2, params[n2]["scale"], bias=params[n2]["bias"], residual=res, relu=True)
        ref[f"b{i}"] = cur
    sums = np.abs(cur.astype(np.int64).sum(axis=(2, 3))).max(axis=0).clip(1)
    params["pool_scale"] = (127.0 / sums * g.uniform(0.5, 1.0, 512)).astype(np.float32)
    pooled = oracle.global_sumpool_requant_i8(cur, params["pool_scale"])
    ref["pooled"] = pooled
    ref["logits"] = oracle.matmul_i8(pooled, params["fc_w"])
    return x, params, ref
