"""Chained int8 inference of a ResNet-18-shaped network on libunit.

Orchestration only: every operator is one call into the C library (conv with the fused
requantise + ReLU epilogue writing the next layer's packed input, max-pool, global average
pool, and the int8 fully connected layer as a matmul).  The
weights, biases, per-channel scales and residual multipliers are inputs; the harness that
calibrates them is not part of this module.

Block wiring:  a = relu_rq(conv1(x));  y = relu_rq(conv2(a) + residual), where residual is
the raw int32 accumulator of the 1x1 projection, or int32(x) * res_mult for an identity
shortcut (read by conv2's epilogue straight from x's packed int8 form).
"""
import numpy as np

from . import unit
from . import workloads as wl


def layer_list():
    """Conv layers in execution order: [(name, ConvShape)], names 'stem', 'b{i}.c1', 'b{i}.c2', 'b{i}.proj'."""
    plan = wl.resnet18_plan()
    out = [("stem", plan["stem"])]
    for i, (c1, c2, proj) in enumerate(plan["blocks"]):
        out.append((f"b{i}.c1", c1))
        if proj is not None:
            out.append((f"b{i}.proj", proj))
        out.append((f"b{i}.c2", c2))
    return out


def random_params(g):
    """Random weights with uncalibrated but plausible scales (about 3 sigma of the accumulator
    maps to 127): enough for timing runs, where values do not matter."""
    params = {"res_mult": {}}
    for name, sh in layer_list():
        fan_in = sh.c * sh.r * sh.s
        sigma = np.sqrt(fan_in) * 37.0 * 74.0
        params[name] = {"w": wl.int8_weights(g, (sh.k, sh.c, sh.r, sh.s)),
                        "bias": None if name.endswith("proj") else np.zeros(sh.k, np.int32),
                        "scale": np.full(sh.k, 127.0 / (3.0 * sigma), np.float32)}
    for i, (c1, c2, proj) in enumerate(wl.resnet18_plan()["blocks"]):
        if proj is None:
            params["res_mult"][i] = 4096
    params["pool_scale"] = np.full(512, 1.0 / 49.0, np.float32)
    params["fc_w"] = wl.int8_weights(g, (1000, 512))
    return params


class ResNet18Int8:
    def __init__(self, batch, params, device="cuda:0"):
        """params: dict name -> {"w": int8 OIHW, "bias": int32 [k] or None, "scale": float32 [k] or None}
        plus "res_mult" (dict block index -> int), "pool_scale" (float32 [512]), "fc_w" (int8 [1000,512])."""
        import torch
        self.torch = torch
        self.n = batch
        self.dev = device
        self.plan = wl.resnet18_plan()
        self.layers = {}
        ws_need = 256
        for name, sh in layer_list():
            p = params[name]
            d = unit.conv_desc(batch, sh.c, sh.h, sh.w, sh.k, sh.r, sh.s, sh.stride, sh.pad)
            wp = torch.empty(unit.unit_packed_weights_bytes(d, unit.UNIT_I8), dtype=torch.uint8, device=device)
            wdev = torch.from_numpy(np.ascontiguousarray(p["w"])).to(device)
            unit.unit_pack_weights_i8(d, wdev, wp)
            ent = {"d": d, "wp": wp, "sh": sh, "out_hw": wl.out_hw(sh)}
            ent["bias"] = None if p.get("bias") is None else torch.from_numpy(p["bias"]).to(device)
            ent["scale"] = None if p.get("scale") is None else torch.from_numpy(p["scale"]).to(device)
            self.layers[name] = ent
            ws_need = max(ws_need, unit.unit_conv2d_packed_workspace(d, unit.UNIT_I8))
        torch.cuda.synchronize()
        self.res_mult = dict(params["res_mult"])
        self.pool_scale = torch.from_numpy(params["pool_scale"]).to(device)
        self.fc_w = torch.from_numpy(np.ascontiguousarray(params["fc_w"])).to(device)
        ws_need = max(ws_need, unit.unit_matmul_workspace(batch, 1000, 512, 512, 512, unit.UNIT_I8))
        self.ws = torch.empty(ws_need, dtype=torch.uint8, device=device)

        def packed(c, h, w):
            return torch.empty(unit.unit_packed_act_bytes(batch, c, h, w, unit.UNIT_I8), dtype=torch.uint8, device=device)

        stem = self.plan["stem"]
        self.x_packed = packed(stem.c, stem.h, stem.w)
        self.stem_out = packed(64, 112, 112)
        self.pool_out = packed(64, 56, 56)
        self.act_a, self.act_y, self.res = [], [], []
        for i, (c1, c2, proj) in enumerate(self.plan["blocks"]):
            p, q = wl.out_hw(c1)
            self.act_a.append(packed(c1.k, p, q))
            self.act_y.append(packed(c2.k, p, q))
            self.res.append(torch.empty((batch, c2.k, p, q), dtype=torch.int32, device=device)
                            if proj is not None else None)
        self.pooled = torch.empty((batch, 512), dtype=torch.int8, device=device)
        self.logits = torch.empty((batch, 1000), dtype=torch.int32, device=device)

    def _conv(self, name, xin, y_packed, relu, residual=None, y_i32=None, skip=None, skip_mult=0):
        L = self.layers[name]
        rq = None
        if y_packed is not None:
            rq = unit.make_requant(L["scale"], L["bias"], residual, relu, skip, skip_mult)
        unit.unit_conv2d_packed_i8(L["d"], xin, L["wp"], y_i32, rq, None, y_packed, self.ws)

    def forward(self, x_nchw):
        """x_nchw: int8 device tensor [n,3,224,224] -> int32 logits [n,1000] (device tensor, async)."""
        n = self.n
        stem = self.plan["stem"]
        unit.unit_pack_act_i8(n, stem.c, stem.h, stem.w, x_nchw, self.x_packed)
        self._conv("stem", self.x_packed, self.stem_out, relu=True)
        unit.unit_maxpool_packed_i8(n, 64, 112, 112, 3, 2, 1, self.stem_out, self.pool_out)
        x = self.pool_out
        for i, (c1, c2, proj) in enumerate(self.plan["blocks"]):
            self._conv(f"b{i}.c1", x, self.act_a[i], relu=True)
            if proj is not None:
                self._conv(f"b{i}.proj", x, None, relu=False, y_i32=self.res[i])
                self._conv(f"b{i}.c2", self.act_a[i], self.act_y[i], relu=True, residual=self.res[i])
            else:
                self._conv(f"b{i}.c2", self.act_a[i], self.act_y[i], relu=True,
                           skip=x, skip_mult=self.res_mult[i])
            x = self.act_y[i]
        unit.unit_global_avgpool_packed_i8(n, 512, 7, 7, x, self.pool_scale, self.pooled)
        unit.unit_matmul_i8(n, 1000, 512, self.pooled, 512, self.fc_w, 512, self.logits, 1000, self.ws)
        return self.logits
