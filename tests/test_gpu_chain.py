"""End-to-end chained ResNet-18-shaped int8 inference: GPU (libunit calls only) against the
composed CPU oracle, bit-exact at every block boundary and on the final logits."""
import numpy as np
import pytest
import torch

from paper_2101_08458_amd import unit
from paper_2101_08458_amd.resnet18_int8 import ResNet18Int8
from gpu_util import announce, dev, host, same
import chain_ref

pytestmark = pytest.mark.gpu


def unpack(net, buf, c, h, w):
    out = torch.empty((net.n, c, h, w), dtype=torch.int8, device="cuda:0")
    unit.unit_unpack_act_i8(net.n, c, h, w, buf, out)
    torch.cuda.synchronize()
    return host(out)


@pytest.mark.parametrize("batch", [1, 8])
def test_resnet18_chain_bit_exact(batch):
    x, params, ref = chain_ref.build(batch)
    assert ref["logits"].std() > 0 and len(np.unique(ref["pooled"])) > 16      # the chain carries signal
    net = ResNet18Int8(batch, params)
    xd = dev(x)
    announce("resnet18 chain batch", batch)
    logits = net.forward(xd)
    torch.cuda.synchronize()
    assert same(unpack(net, net.stem_out, 64, 112, 112), ref["stem"], "stem")
    assert same(unpack(net, net.pool_out, 64, 56, 56), ref["pool"], "maxpool")
    for i, (c1, c2, proj) in enumerate(net.plan["blocks"]):
        p, q = c2.h, c2.w
        assert same(unpack(net, net.act_y[i], c2.k, p, q), ref[f"b{i}"], f"block {i}")
    assert same(host(net.pooled), ref["pooled"], "avgpool")
    assert same(host(logits), ref["logits"], "logits")
    # run-to-run: a second pass over the same buffers gives the same bytes
    first = host(logits).copy()
    net.forward(xd)
    torch.cuda.synchronize()
    assert same(host(net.logits), first, "second pass")
