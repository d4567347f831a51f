"""Pins for the inspection oracle (Section III-B, Algorithm 1, Section IV-A).

The oracle is checked against (1) the facts the paper states about its worked example,
(2) the definition of a feasible mapping evaluated semantically -- every register lane must
read exactly one memory address -- by brute force over actual index values, and (3) hand-made
cases in which one plausible mistake (ignoring types, opcodes, operand order, annotations,
rebinding, enumeration order) changes the answer.
"""
import itertools
import os
import re

import numpy as np
import pytest

from oracle import inspector as oi
from paper_2101_08458_amd import tensor_programs as tp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "inspector_vnni_conv.txt")


def _golden():
    exp = {"map": {}, "operand": {}}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, _, val = line.partition("=")
        key, val = key.split(), val.strip()
        if key[0] == "applicable":
            exp["applicable"] = bool(int(val))
        elif key[0] == "map":
            exp["map"][key[1]] = val
        else:
            arr, _, bc = val.partition(":")
            exp["operand"][key[1]] = (arr.strip(), bc.split())
    return exp


def test_paper_worked_example_vnni_conv():
    exp = _golden()
    res = oi.inspect(tp.VNNI, tp.paper_conv())
    assert res["applicable"] == exp["applicable"]
    assert res["mapping"] == exp["map"]
    got = {name: (arr, bc) for name, arr, bc in res["operands"]}
    assert got == exp["operand"]


def test_arm_dot_same_mapping_signed_bytes():
    # Section III-A: same form as the x86 instruction, other lanes and types.
    res = oi.inspect(tp.ARM_DOT, tp.paper_conv(act="i8"))
    assert res["applicable"] and res["mapping"] == {"i": "k", "j": "rc"}
    # unsigned activations do not match a signed-byte register: types must agree (Algorithm 1)
    assert oi.inspect(tp.ARM_DOT, tp.paper_conv(act="u8"))["failed_step"] == 1


def test_tensor_core_matmul_identity():
    res = oi.inspect(tp.TENSOR_CORE, tp.matmul(256, 256, 256))
    assert res["applicable"]
    assert res["mapping"] == {"i": "m", "j": "n", "k": "k"}
    assert all(bc == [] for _, _, bc in res["operands"])
    assert res["num_feasible"] == 1


def test_type_mismatch_rejected():
    # signed x signed conv against the unsigned x signed instruction
    res = oi.inspect(tp.VNNI, tp.paper_conv(act="i8", wgt="i8"))
    assert not res["applicable"] and res["failed_step"] == 1
    # accumulator type
    res = oi.inspect(tp.TENSOR_CORE, tp.matmul(16, 16, 16, accum="f16"))
    assert res["failed_step"] == 1


def test_opcode_and_shape_of_tree():
    instr = "loop i 4 dp; loop j 4 red\nout d:i32[i]\nbody (mul a:i32[i,j] b:i32[i,j])"
    ok = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] q:i32[x,r])"
    add = ok.replace("(mul", "(add")
    deeper = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] (cast i32 q:i32[x,r]))"
    assert oi.inspect(instr, ok)["applicable"]
    assert oi.inspect(instr, add)["failed_step"] == 1
    assert oi.inspect(instr, deeper)["failed_step"] == 1     # leaf against arithmetic node


def test_leaf_binding_is_single_valued():
    square = "loop i 4 dp; loop j 4 red\nout d:i32[i]\nbody (mul a:i32[i,j] a:i32[i,j])"
    op_two = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] q:i32[x,r])"
    op_one = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] p:i32[x,r])"
    op_idx = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] p:i32[r,x])"
    assert oi.inspect(square, op_two)["failed_step"] == 1    # one register, two arrays
    assert oi.inspect(square, op_one)["applicable"]
    assert oi.inspect(square, op_idx)["failed_step"] == 1    # one register element, two addresses


def test_operand_order_is_left_to_left():
    # Children are matched lhs-lhs and rhs-rhs, so writing the product the other way round
    # binds the registers the other way round and transposes the loop mapping.
    mfma = "loop i 32 dp; loop j 32 dp; loop kk 32 red\nout d:i32[i,j]\n" \
           "body (mul (cast i32 a:i8[i,kk]) (cast i32 b:i8[j,kk]))"
    loops = "loop n 1 dp; loop k 64 dp; loop p 56 dp; loop q 56 dp; loop r 3 red; loop s 3 red; loop c 64 red\n"
    w_first = loops + "out y:i32[n,k,p,q]\nbody (mul (cast i32 w:i8[k,r,s,c]) (cast i32 x:i8[n,p+r,q+s,c]))"
    x_first = loops + "out y:i32[n,k,p,q]\nbody (mul (cast i32 x:i8[n,p+r,q+s,c]) (cast i32 w:i8[k,r,s,c]))"
    a = oi.inspect(mfma, w_first)
    b = oi.inspect(mfma, x_first)
    assert a["mapping"] == {"i": "k", "j": "q", "kk": "c"}
    assert b["mapping"] == {"i": "q", "j": "k", "kk": "c"}
    assert dict((n, t) for n, t, _ in a["operands"]) == {"d": "y", "a": "w", "b": "x"}
    assert dict((n, t) for n, t, _ in b["operands"]) == {"d": "y", "a": "x", "b": "w"}


def test_annotations_must_agree():
    instr = "loop i 4 dp; loop j 4 red\nout d:i32[i]\nbody (mul a:i32[i,j] b:i32[i,j])"
    no_red = "loop x 8 dp; loop z 8 dp\nout y:i32[x,z]\nbody (mul p:i32[x,z] q:i32[x,z])"
    assert oi.inspect(instr, no_red)["failed_step"] == 2
    # with both loop kinds present, the reduction loop can only take the reduction loop
    op = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[r,x] q:i32[x,r])"
    assert oi.inspect(instr, op)["mapping"] == {"i": "x", "j": "r"}


def test_infeasible_access():
    mfma = "loop i 16 dp; loop j 16 dp; loop kk 64 red\nout d:i32[i,j]\n" \
           "body (mul a:i32[i,kk] b:i32[j,kk])"
    # the first operand depends on both data-parallel loops: a lane of register a would have
    # to hold several addresses whichever way the loops are assigned
    op = "loop x 8 dp; loop y 8 dp; loop r 8 red\nout o:i32[x,y]\nbody (mul p:i32[x,y,r] q:i32[y,r])"
    res = oi.inspect(mfma, op)
    assert not res["applicable"] and res["failed_step"] == 2 and res["num_feasible"] == 0


def test_innermost_first_and_count():
    # For the worked example all 3 x 3 assignments are feasible (any data-parallel loop can
    # take i with a broadcast, any reduction loop can take j); the one returned is the pair
    # of innermost dimensions.
    res = oi.inspect(tp.VNNI, tp.paper_conv())
    assert res["num_feasible"] == 9
    # declaring the channel loops first makes another pair the innermost one
    text = tp.paper_conv()
    text = text.replace("loop x 56 dp; loop y 56 dp; loop k 64 dp", "loop k 64 dp; loop x 56 dp; loop y 56 dp")
    text = text.replace("loop r 3 red; loop s 3 red; loop rc 64 red", "loop rc 64 red; loop r 3 red; loop s 3 red")
    assert oi.inspect(tp.VNNI, text)["mapping"] == {"i": "y", "j": "s"}


def test_constant_operand_is_skipped():
    instr = "loop i 4 dp; loop j 4 red\nout d:i32[i]\nbody (mul a:i32[i,j] b:i32[i,j])"
    op = "loop x 8 dp; loop r 8 red\nout y:i32[x]\nbody (mul p:i32[x,r] const:i32:3)"
    res = oi.inspect(instr, op)
    assert res["applicable"]
    assert ("b", "const", []) in res["operands"]
    bad = op.replace("const:i32:3", "const:f32:3")
    assert oi.inspect(instr, bad)["failed_step"] == 1


# ----------------------------------------------------------------------------------------
# Semantic brute force: a mapping is usable iff, with the unmapped loops held fixed, every lane
# of every instruction register reads one address of the operation's array.  Evaluated with
# actual integers, independent of the set formula.

def _index_value(text, env):
    vals = []
    for dim in text.split(","):
        total = 0
        for sign, term in re.findall(r"([+-]?)([^+-]+)", dim):
            parts = term.split("*")
            v = 1
            for p in parts:
                v *= int(p) if re.fullmatch(r"\d+", p) else env[p]
            total += -v if sign == "-" else v
        vals.append(total)
    return tuple(vals)


def _semantic_feasible(instr, op, pairs, f):
    iloops = instr["loops"]
    inv = {i: o for o, i in f.items()}
    for _, v, u in pairs:
        if u is None:
            continue
        lanes = {}
        for point in itertools.product(*[range(min(e, 3)) for _, e, _ in iloops]):
            ienv = {n: x for (n, _, _), x in zip(iloops, point)}
            oenv = {n: 0 for n, _, _ in op["loops"]}
            for i, x in ienv.items():
                oenv[inv[i]] = x
            lane = _index_value(v["index"], ienv)
            addr = _index_value(u["index"], oenv)
            if lanes.setdefault(lane, addr) != addr:
                return False
    return True


@pytest.mark.parametrize("seed", range(6))
def test_set_criterion_equals_one_address_per_lane(seed):
    g = np.random.default_rng(4200 + seed)
    checked = feasible_seen = 0
    while checked < 60:
        itext, otext = tp.random_program_pair(g)
        instr, op = oi.parse(itext), oi.parse(otext)
        bind = {}
        if instr["out"]["type"] != op["out"]["type"]:
            continue
        if not oi.compute_isomorphism(instr["body"], op["body"], bind):
            continue
        # the register layouts of the generator are injective in their loop variables and all
        # trip counts exceed one, which is what makes the two notions coincide
        pairs = oi._pairs(instr, op, bind)
        inames = [n for n, _, _ in instr["loops"]]
        per_loop = [[n for n, _, a in op["loops"] if a == ann] for _, _, ann in instr["loops"]]
        count = 0
        for choice in itertools.product(*per_loop):
            if len(set(choice)) != len(choice):
                continue
            f = dict(zip(choice, inames))
            sem = _semantic_feasible(instr, op, pairs, f)
            assert oi.feasible(f, pairs) == sem, (itext, otext, f)
            count += sem
        res = oi.inspect(itext, otext)
        if res["failed_step"] != 1:
            assert res["num_feasible"] == count
            assert res["applicable"] == (count > 0)
            feasible_seen += count > 0
        checked += 1
    assert feasible_seen >= 10


def test_parse_errors():
    with pytest.raises(oi.ParseError):
        oi.parse("loop i 4 dp\nout d:i32[z]\nbody a:i32[i]")
    with pytest.raises(oi.ParseError):
        oi.parse("loop i 4 dp\nbody a:i32[i]")
    with pytest.raises(oi.ParseError):
        oi.parse("loop i 0 dp\nout d:i32[i]\nbody a:i32[i]")
