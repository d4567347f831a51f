"""CPU oracle for the applicability inspection (Section III-B, Algorithm 1; Section IV-A).

TEST INFRASTRUCTURE ONLY: used by the tests, never by the product package, and it
shares no code with the library's own inspector.

The inspection answers: can a tensorized instruction, written as a small tensor
program, execute (a tile of) a tensor operation, and which loops of the operation
become the instruction's loops?  Two steps, in the paper's order:

  1. compute isomorphism (Algorithm 1): walk both expression trees together;
     node data types must agree; two leaves bind the instruction operand to the
     operation operand (a second visit must find the same binding); two
     arithmetic nodes need the same opcode and matching children, left with
     left and right with right.
  2. array-access isomorphism (Section III-B.2): enumerate f : A -> B, where B
     is the instruction's loops and A the operation loops chosen for them (equal
     annotation only).  With S(u) the loop variables in an index expression and
     S'(u) = { f(x) : x in S(u) & A }, f is feasible iff S'(u) is a subset of
     S(v) for every bound pair (u from the operation, v from the instruction).
     Instruction loops in S(v) but not in S'(u) are broadcast directions.
     Constants on the operation side are skipped.
  3. order (Section IV-A): candidates run from the innermost tensor dimension
     outwards and the first feasible mapping is returned.

Readings where the paper leaves room (also listed in the design notes):
  * a type conversion is a one-child arithmetic node whose opcode is "cast" and
    whose type is the destination type;
  * the output access of the operation pairs with the output access of the
    instruction, and with the instruction's separate addend register if it has
    one (the VNNI / DOT form d = c + sum(...)); an instruction without one
    accumulates in place (the Tensor Core "+=" form);
  * "innermost first" means: loops are declared in tensor-dimension order
    (outermost first), candidates are tried in reverse declaration order, and
    the instruction's loops are assigned in their declaration order, the first
    one varying slowest.

Text form of a tensor program (shared with the library: an interface, no arithmetic):
    loop NAME EXTENT dp|red ; ...          data-parallel or reduction loop
    out  NAME:DTYPE[INDEX,...]             the element written
    acc  NAME:DTYPE[INDEX,...]             optional separate addend register
    body EXPR                              the value reduced into the output
    EXPR  := (OPCODE EXPR EXPR) | (cast DTYPE EXPR) | NAME:DTYPE[INDEX,...] | const:DTYPE:VALUE
    INDEX := sum of terms  [COEF*]VAR  or  integer, joined by + or -
Statements are separated by ';' or newlines.
"""
import itertools
import re


class ParseError(ValueError):
    pass


# ---------------------------------------------------------------- parsing

_TOKEN = re.compile(r"\s*(\(|\)|[^\s()]+)")


def _index_vars(text, loops):
    """S(u): the set of loop variables that occur in one access's index list."""
    found = set()
    for dim in text.split(","):
        for term in re.split(r"[+-]", dim):
            term = term.strip()
            if not term:
                continue
            name = term.split("*")[-1].strip()
            if re.fullmatch(r"\d+", name):
                continue
            if name not in loops:
                raise ParseError(f"unknown loop variable {name!r}")
            found.add(name)
    return frozenset(found)


def _access(text, loops):
    m = re.fullmatch(r"(\w+):(\w+)\[([^\]]*)\]", text)
    if not m:
        raise ParseError(f"bad access {text!r}")
    name, dtype, idx = m.groups()
    canon = re.sub(r"\s+", "", idx)
    return {"kind": "load", "type": dtype, "tensor": name, "index": canon,
            "vars": _index_vars(idx, loops)}


def _expr(tokens, pos, loops):
    tok = tokens[pos]
    if tok == "(":
        op = tokens[pos + 1]
        if op == "cast":
            dtype = tokens[pos + 2]
            child, pos = _expr(tokens, pos + 3, loops)
            if tokens[pos] != ")":
                raise ParseError("cast takes one operand")
            return {"kind": "arith", "opcode": "cast", "type": dtype, "children": [child]}, pos + 1
        lhs, pos = _expr(tokens, pos + 2, loops)
        rhs, pos = _expr(tokens, pos, loops)
        if tokens[pos] != ")":
            raise ParseError("binary node takes two operands")
        return {"kind": "arith", "opcode": op, "type": lhs["type"], "children": [lhs, rhs]}, pos + 1
    if tok.startswith("const:"):
        parts = tok.split(":")
        if len(parts) != 3:
            raise ParseError(f"bad constant {tok!r}")
        return {"kind": "const", "type": parts[1], "value": parts[2]}, pos + 1
    return _access(tok, loops), pos + 1


def parse(text):
    """-> {"loops": [(name, extent, annotation)], "out": access, "acc": access|None, "body": tree}"""
    prog = {"loops": [], "out": None, "acc": None, "body": None}
    names = {}
    for stmt in re.split(r"[;\n]", text):
        stmt = stmt.strip()
        if not stmt:
            continue
        head, _, rest = stmt.partition(" ")
        rest = rest.strip()
        if head == "loop":
            f = rest.split()
            if len(f) != 3 or f[2] not in ("dp", "red") or not f[1].isdigit() or int(f[1]) < 1:
                raise ParseError(f"bad loop {stmt!r}")
            if f[0] in names:
                raise ParseError(f"loop {f[0]!r} declared twice")
            names[f[0]] = f[2]
            prog["loops"].append((f[0], int(f[1]), f[2]))
        elif head in ("out", "acc"):
            prog[head] = _access(re.sub(r"\s+", "", rest), names)
        elif head == "body":
            # keep index lists free of blanks so that they stay one token
            compact = re.sub(r"\[[^\]]*\]", lambda m: re.sub(r"\s+", "", m.group(0)), rest)
            tokens = _TOKEN.findall(compact) + [None]
            tree, pos = _expr(tokens, 0, names)
            if tokens[pos] is not None:
                raise ParseError("trailing text after body")
            prog["body"] = tree
        else:
            raise ParseError(f"unknown statement {stmt!r}")
    if prog["out"] is None or prog["body"] is None or not prog["loops"]:
        raise ParseError("a program needs loops, out and body")
    return prog


# ---------------------------------------------------------------- Algorithm 1

def _leaf(n):
    return n["kind"] in ("load", "const")


def _ident(n):
    if n["kind"] == "const":
        return ("const", n["type"], n["value"])
    return ("load", n["tensor"], n["index"])


def compute_isomorphism(a, b, bind):
    """Algorithm 1.  a: instruction node, b: operation node.  bind maps the identity of an
    instruction leaf to (instruction leaf, operation leaf)."""
    if a["type"] != b["type"]:
        return False
    if _leaf(a) and _leaf(b):
        if a["kind"] != "load":
            return False          # an instruction operand is a register, never a literal
        key = _ident(a)
        if key not in bind:
            bind[key] = (a, b)
        elif _ident(bind[key][1]) != _ident(b):
            return False
        return True
    if a["kind"] == "arith" and b["kind"] == "arith":
        if a["opcode"] != b["opcode"] or len(a["children"]) != len(b["children"]):
            return False
        for ca, cb in zip(a["children"], b["children"]):
            if not compute_isomorphism(ca, cb, bind):
                return False
        return True
    return False


# ---------------------------------------------------------------- Section III-B.2

def _pairs(instr, op, bind):
    """(name of instruction operand, v = its access, u = operation access or None for a constant)"""
    pairs = [(instr["out"]["tensor"], instr["out"], op["out"])]
    if instr["acc"] is not None:
        pairs.append((instr["acc"]["tensor"], instr["acc"], op["out"]))
    for a, b in bind.values():
        pairs.append((a["tensor"], a, b if b["kind"] == "load" else None))
    return pairs


def feasible(f, pairs):
    """f: dict operation loop -> instruction loop."""
    for _, v, u in pairs:
        if u is None:
            continue
        s_prime = {f[x] for x in u["vars"] if x in f}
        if not s_prime <= v["vars"]:
            return False
    return True


def inspect(instruction_text, operation_text):
    instr, op = parse(instruction_text), parse(operation_text)
    result = {"applicable": False, "failed_step": 0, "mapping": {}, "operands": [],
              "num_feasible": 0}
    bind = {}
    same_out_type = instr["out"]["type"] == op["out"]["type"]
    if not same_out_type or not compute_isomorphism(instr["body"], op["body"], bind):
        result["failed_step"] = 1
        return result
    # one register <- one array: all leaves of an instruction tensor must come from one source
    source = {}
    for a, b in bind.values():
        src = b["tensor"] if b["kind"] == "load" else "const"
        if source.setdefault(a["tensor"], src) != src:
            result["failed_step"] = 1
            return result
    pairs = _pairs(instr, op, bind)

    candidates = []
    for _, _, annotation in instr["loops"]:
        inner_first = [n for n, _, ann in reversed(op["loops"]) if ann == annotation]
        candidates.append(inner_first)
    instr_names = [n for n, _, _ in instr["loops"]]
    first = None
    for choice in itertools.product(*candidates):
        if len(set(choice)) != len(choice):
            continue
        f = dict(zip(choice, instr_names))
        if feasible(f, pairs):
            result["num_feasible"] += 1
            if first is None:
                first = f
    if first is None:
        result["failed_step"] = 2
        return result
    result["applicable"] = True
    inv = {i: o for o, i in first.items()}
    result["mapping"] = {i: inv[i] for i in instr_names}
    seen = set()
    for name, v, u in pairs:
        if name in seen:
            continue
        seen.add(name)
        if u is None:
            result["operands"].append((name, "const", []))
            continue
        s_prime = {first[x] for x in u["vars"] if x in first}
        bcast = [i for i in instr_names if i in v["vars"] and i not in s_prime]
        result["operands"].append((name, u["tensor"], bcast))
    return result
