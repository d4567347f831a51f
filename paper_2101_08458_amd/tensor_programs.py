"""Tensor programs in text form for the applicability inspection (Section III-A, III-B).

This module holds descriptions only -- no part of the inspection itself.  The
library's `unit_inspect` and the test oracle both parse these strings.

Text form (statements separated by ';' or newlines):
    loop NAME EXTENT dp|red         data-parallel or reduction loop, outermost first
    out  NAME:DTYPE[INDEX,...]      element written
    acc  NAME:DTYPE[INDEX,...]      optional separate addend register (d = c + sum(...));
                                    without it the program accumulates in place (+=)
    body EXPR                       value reduced into the output
    EXPR  := (OPCODE EXPR EXPR) | (cast DTYPE EXPR) | NAME:DTYPE[INDEX,...] | const:DTYPE:VALUE
    INDEX := terms [COEF*]VAR or integers joined by + or -
"""

# Section III-A: the x86 dot-product instruction as a tensor program.  Registers: 64 lanes of
# unsigned bytes, 64 lanes of signed bytes, 16 lanes of int32; loop i is data parallel over the
# 16 results, loop j reduces 4 byte products into each.
VNNI = """
loop i 16 dp; loop j 4 red
out d:i32[i]
acc c:i32[i]
body (mul (cast i32 a:u8[4*i+j]) (cast i32 b:i8[4*i+j]))
"""

# Section III-A: the Arm dot-product instruction has the same form with other lane counts and
# types (public ISA: 4 int32 results, each the sum of 4 signed-byte products).
ARM_DOT = """
loop i 4 dp; loop j 4 red
out d:i32[i]
acc c:i32[i]
body (mul (cast i32 a:i8[4*i+j]) (cast i32 b:i8[4*i+j]))
"""

# Section III-A: the matrix-multiply unit: a 16x16x16 product accumulated in place.
TENSOR_CORE = """
loop i 16 dp; loop j 16 dp; loop k 16 red
out c:f32[i,j]
body (mul (cast f32 a:f16[i,k]) (cast f32 b:f16[k,j]))
"""


def paper_conv(x=56, y=56, k=64, r=3, s=3, rc=64, act="u8", wgt="i8", accum="i32"):
    """Section III-C.2 index forms: c[x,y,k] += a[x+r,y+s,rc] * b[r,s,k,rc]."""
    return (f"loop x {x} dp; loop y {y} dp; loop k {k} dp; "
            f"loop r {r} red; loop s {s} red; loop rc {rc} red\n"
            f"out c:{accum}[x,y,k]\n"
            f"body (mul (cast {accum} a:{act}[x+r,y+s,rc]) (cast {accum} b:{wgt}[r,s,k,rc]))")


def matmul(m, n, k, a="f16", b="f16", accum="f32", b_transposed=False):
    """c[m,n] += a[m,k] * b[k,n]   (b[n,k] when b_transposed)."""
    bidx = "n,k" if b_transposed else "k,n"
    return (f"loop m {m} dp; loop n {n} dp; loop k {k} red\n"
            f"out c:{accum}[m,n]\n"
            f"body (mul (cast {accum} a:{a}[m,k]) (cast {accum} b:{b}[{bidx}]))")


_DTYPES = ["i8", "u8", "f16", "i32", "f32"]
_OPS = ["mul", "add", "max"]


def random_program_pair(g):
    """A seeded (instruction, operation) pair for parity tests.

    The operation is built around a hidden loop correspondence and then disturbed at random
    (extra loops, coupled indices, swapped operands, other types or opcodes), so that the
    inspection meets applicable and inapplicable cases of every kind."""
    ndp, nred = int(g.integers(1, 3)), int(g.integers(1, 3))
    iloops = [(f"i{t}", int(g.choice([2, 4, 16, 32])), "dp") for t in range(ndp)]
    iloops += [(f"j{t}", int(g.choice([2, 4, 8, 16])), "red") for t in range(nred)]
    inames = [n for n, _, _ in iloops]
    dp_names = inames[:ndp]
    in_t, out_t = str(g.choice(_DTYPES[:3])), str(g.choice(_DTYPES[3:]))
    in_t2 = in_t if g.random() < 0.7 else str(g.choice(_DTYPES[:3]))
    opcode = str(g.choice(_OPS))
    with_cast = g.random() < 0.8
    with_acc = g.random() < 0.4
    if not with_cast:
        in_t = in_t2 = out_t

    def subset(names, keep):
        chosen = [n for n in names if g.random() < keep]
        return chosen or [names[int(g.integers(len(names)))]]

    a_vars, b_vars = subset(inames, 0.8), subset(inames, 0.8)

    def leaf(name, dtype, dims):
        text = f"{name}:{dtype}[{','.join(dims)}]"
        return f"(cast {out_t} {text})" if with_cast else text

    instr = "; ".join(f"loop {n} {e} {a}" for n, e, a in iloops) + "\n"
    instr += f"out d:{out_t}[{','.join(dp_names)}]\n"
    if with_acc:
        instr += f"acc c:{out_t}[{','.join(dp_names)}]\n"
    instr += f"body ({opcode} {leaf('a', in_t, a_vars)} {leaf('b', in_t2, b_vars)})"

    # operation: every instruction loop gets a partner, plus some loops of its own
    xdp, xred = int(g.integers(0, 3)), int(g.integers(0, 2))
    odp = [f"x{t}" for t in range(ndp + xdp)]
    ored = [f"r{t}" for t in range(nred + xred)]
    partner = {}
    for names, pool in ((dp_names, list(g.permutation(odp))), (inames[ndp:], list(g.permutation(ored)))):
        for n, o in zip(names, pool):
            partner[n] = str(o)
    free = [o for o in odp + ored if o not in partner.values()]
    oloops = [(o, int(g.choice([7, 16, 56, 64])), "dp") for o in odp]
    oloops += [(o, int(g.choice([3, 16, 64])), "red") for o in ored]

    def op_dims(ivars, allow_free):
        dims = [partner[v] for v in ivars if g.random() < 0.85]
        for o in allow_free:
            if g.random() < 0.35:
                if dims and g.random() < 0.5:
                    slot = int(g.integers(len(dims)))
                    dims[slot] = f"{dims[slot]}+{o}"
                else:
                    dims.append(o)
        if g.random() < 0.15:                      # an index the hidden correspondence forbids
            dims.append(str(g.choice(odp + ored)))
        if not dims:
            dims = [partner[ivars[0]]]
        order = g.permutation(len(dims))
        return [dims[int(t)] for t in order]

    t_a, t_b, t_o = in_t, in_t2, out_t
    roll = g.random()
    if roll < 0.08:
        t_a = str(g.choice(_DTYPES[:3]))
    elif roll < 0.14:
        t_o = str(g.choice(_DTYPES[3:]))
    op_opcode = opcode if g.random() < 0.92 else str(g.choice(_OPS))
    la = leaf("p", t_a, op_dims(a_vars, free))
    if g.random() < 0.06:
        lb = f"const:{t_b}:3" if not with_cast else f"(cast {out_t} const:{t_b}:3)"
    else:
        lb = leaf("q" if g.random() < 0.9 else "p", t_b, op_dims(b_vars, free))
    if g.random() < 0.08:
        la, lb = lb, la
    out_dims = [partner[v] for v in dp_names] + [o for o in odp if o not in partner.values()]
    out_dims = [out_dims[int(t)] for t in g.permutation(len(out_dims))]
    op = "; ".join(f"loop {n} {e} {a}" for n, e, a in oloops) + "\n"
    op += f"out y:{t_o}[{','.join(out_dims)}]\n"
    op += f"body ({op_opcode} {la} {lb})"
    return instr, op
