"""Helpers shared by the GPU parity tests: device upload, case announcement, selector
overrides, and the fp16 error metric."""
import contextlib
import sys

import numpy as np


def announce(*what):
    """Name the case before the GPU step so a fault can be attributed."""
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def dev(a):
    import torch
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


_forced_now = [-1, -1]


@contextlib.contextmanager
def forced(tile=None, split=None):
    """Override the selector (unit_debug_force_tile) for the duration of a block."""
    from paper_2101_08458_amd import unit
    old = list(_forced_now)
    _forced_now[:] = [-1 if tile is None else int(tile), -1 if split is None else int(split)]
    unit.unit_debug_force_tile(*_forced_now)
    try:
        yield
    finally:
        _forced_now[:] = old
        unit.unit_debug_force_tile(*old)


def f16_rel_err(got, ref, kred):
    """max |got-ref| / max(|ref|, tau).

    Two fp32 summation orders of the same kred exact products differ by a random-walk
    rounding error of about sqrt(kred) * 2^-24 * rms(ref), whatever the implementation, so a
    relative error is only meaningful for |ref| well above that.  tau puts the floor at
    rms(ref) * max(1e-3, 4000 * sqrt(kred) * 2^-24): below tau the check becomes the
    absolute bound 1e-3 * tau = 4 * sqrt(kred) * 2^-24 * rms(ref).
    """
    ref64 = ref.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref64 ** 2)))
    tau = rms * max(1e-3, 4000.0 * np.sqrt(kred) * 2.0 ** -24) + 1e-30
    return float(np.max(np.abs(got.astype(np.float64) - ref64) / np.maximum(np.abs(ref64), tau)))


def fp8_rel_err(got, ref):
    """max |got-ref| / max(|ref|, rms(ref)) for the fp8 paths.

    The fp8 matrix instruction does not add its products in fp32: it sums them in groups of 8
    inside a fixed-point frame that keeps 13 bits below the group's largest product and drops
    (truncates) what lies beneath; the group sums are then accumulated in fp32.  Each product
    thus carries an error of up to 2^-13 of its group's maximum, about 1.5e-4 of rms(ref) over
    a whole reduction for random operands, whatever its length, so errors are measured against
    the output scale rather than against each (possibly cancelled) element.
    """
    ref64 = ref.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref64 ** 2))) + 1e-30
    return float(np.max(np.abs(got.astype(np.float64) - ref64) / np.maximum(np.abs(ref64), rms)))


def fp8_bound(kred, mag):
    """A-priori bound on |got - exact|: every product loses less than 2^-13 of the largest of
    its group of 8, hence less than 8 * 2^-13 of the group's sum of magnitudes, plus the fp32
    accumulation of the group sums."""
    return (2.0 ** -10 + 2 * kred * 2.0 ** -24) * mag + 1e-30


def same(got, exp, what=""):
    """Exact equality with a short mismatch report (never dumps the arrays)."""
    got, exp = np.asarray(got), np.asarray(exp)
    if got.shape != exp.shape:
        print(f"[mismatch] {what}: shape {got.shape} vs {exp.shape}", flush=True)
        return False
    bad = np.flatnonzero(got.reshape(-1) != exp.reshape(-1))
    if bad.size:
        i = bad[:5]
        print(f"[mismatch] {what}: {bad.size}/{got.size} differ; first at {i.tolist()} "
              f"got {got.reshape(-1)[i].tolist()} exp {exp.reshape(-1)[i].tolist()}", flush=True)
        return False
    return True


def as_accurate_as_oracle(got, ref, truth):
    """Accuracy check that does not depend on the tolerance floor of f16_rel_err: against the float64
    accumulation of the exact products, the kernel's rms error may be at most twice the rms error of
    the sequential fp32 oracle, plus half an fp32 unit in the last place of the rms output (cases
    whose sums are exact on both sides, and tiny samples).  A kernel that loses more precision than
    plain fp32 accumulation in some order can lose, fails this whatever the floor is."""
    t = truth.astype(np.float64)
    e_got = float(np.sqrt(np.mean((got.astype(np.float64) - t) ** 2)))
    e_ref = float(np.sqrt(np.mean((ref.astype(np.float64) - t) ** 2)))
    floor = 2.0 ** -24 * float(np.sqrt(np.mean(t ** 2)))
    return e_got <= 2.0 * e_ref + floor
