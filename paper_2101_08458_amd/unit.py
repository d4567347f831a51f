"""Thin ctypes binding of libunit.so: argument marshalling only.

Every function has the name and argument order of its C entry point (include/unit.h)
and takes torch tensors on the GPU (or raw integer device addresses) where the C
call takes device pointers.  All computation happens inside the library's HIP
kernels; this module fails loudly if the library is missing -- there is no CPU
fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libunit.so")

UNIT_OK, UNIT_EINVAL, UNIT_ENOTSUP, UNIT_EOVERFLOW, UNIT_EWORKSPACE, UNIT_EHIP, UNIT_ESCRATCH = 0, -1, -2, -3, -4, -5, -6
UNIT_STATIC_SCRATCH_BYTES = 16 << 20
UNIT_I8, UNIT_F16, UNIT_BF16, UNIT_U8I8, UNIT_FP8 = 0, 1, 2, 3, 4
UNIT_MAX_REDUCTION_I8 = 131071
UNIT_MAX_REDUCTION_U8I8 = 65793


class unit_conv2d_desc(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in
                ("n", "c", "h", "w", "k", "r", "s", "stride_h", "stride_w", "pad_h", "pad_w")]


class unit_conv3d_desc(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in
                ("n", "c", "d", "h", "w", "k", "t", "r", "s",
                 "stride_d", "stride_h", "stride_w", "pad_d", "pad_h", "pad_w")]


class unit_requant(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("residual", ctypes.c_void_p), ("relu", ctypes.c_int32),
                ("residual_mult", ctypes.c_int32), ("residual_packed", ctypes.c_void_p)]


class unit_tile_info(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in
                ("block_m", "block_n", "block_k_bytes", "waves_m", "waves_n", "waves_k",
                 "mfma", "split_k", "workgroups", "tail_block_n", "tail_workgroups", "tail_first_col")]


UNIT_INSPECT_MAX, UNIT_INSPECT_NAME = 8, 16


class unit_inspect_result(ctypes.Structure):
    _names = (ctypes.c_char * UNIT_INSPECT_NAME) * UNIT_INSPECT_MAX
    _fields_ = [("applicable", ctypes.c_int32), ("failed_step", ctypes.c_int32),
                ("num_loops", ctypes.c_int32), ("instr_loop", _names), ("op_loop", _names),
                ("num_operands", ctypes.c_int32), ("instr_operand", _names), ("op_operand", _names),
                ("broadcast", ctypes.c_uint32 * UNIT_INSPECT_MAX), ("num_feasible", ctypes.c_int32)]


class UnitError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        lib = _lib
        msg = lib.unit_status_str(status).decode() if lib else str(status)
        extra = lib.unit_last_hip_error().decode() if lib and status == UNIT_EHIP else ""
        super().__init__(f"{where}: {msg}" + (f" ({extra})" if extra else ""))


_lib = None

EXPORTS = [
    "unit_version", "unit_status_str", "unit_last_hip_error", "unit_conv2d_out_dims",
    "unit_packed_act_bytes", "unit_packed_weights_bytes", "unit_conv2d_workspace",
    "unit_conv2d_packed_workspace", "unit_matmul_workspace", "unit_select_conv2d", "unit_select_conv2d_input",
    "unit_select_matmul", "unit_conv2d_i8", "unit_conv2d_f16", "unit_matmul_i8", "unit_matmul_f16",
    "unit_pack_act_i8", "unit_pack_act_f16", "unit_pack_weights_i8", "unit_pack_weights_f16",
    "unit_unpack_act_i8", "unit_conv2d_packed_i8", "unit_conv2d_packed_f16",
    "unit_maxpool_packed_i8", "unit_global_avgpool_packed_i8", "unit_widen_residual_i8",
    "unit_conv2d_wpacked_workspace", "unit_conv2d_wpacked_i8", "unit_conv2d_wpacked_f16",
    "unit_conv2d_wpacked_i8_static",
    "unit_conv3d_out_dims", "unit_conv3d_workspace", "unit_conv3d_i8", "unit_conv3d_f16",
    "unit_conv2d_bf16", "unit_matmul_bf16", "unit_conv2d_u8i8", "unit_matmul_u8i8",
    "unit_conv2d_fp8", "unit_matmul_fp8",
    "unit_conv2d_input_mode", "unit_debug_force_tile", "unit_measure_mfma",
    "unit_inspect", "unit_describe_mfma", "unit_describe_conv2d", "unit_describe_matmul",
]


def load():
    """Load libunit.so (built by __graft_entry__.build() / make in csrc/)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; "
                          f"g.build()'` (or make -C paper_2101_08458_amd/csrc)")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, sz, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p
    dp = ctypes.POINTER(unit_conv2d_desc)
    d3 = ctypes.POINTER(unit_conv3d_desc)
    rp = ctypes.POINTER(unit_requant)
    tp = ctypes.POINTER(unit_tile_info)
    ip = ctypes.POINTER(ctypes.c_int32)
    sig = {
        "unit_version": (ctypes.c_int, []),
        "unit_status_str": (ctypes.c_char_p, [ctypes.c_int]),
        "unit_last_hip_error": (ctypes.c_char_p, []),
        "unit_conv2d_out_dims": (ctypes.c_int, [dp, ip, ip]),
        "unit_packed_act_bytes": (sz, [i32, i32, i32, i32, ctypes.c_int]),
        "unit_packed_weights_bytes": (sz, [dp, ctypes.c_int]),
        "unit_conv2d_workspace": (sz, [dp, ctypes.c_int]),
        "unit_conv2d_packed_workspace": (sz, [dp, ctypes.c_int]),
        "unit_matmul_workspace": (sz, [i32, i32, i32, i64, i64, ctypes.c_int]),
        "unit_select_conv2d": (ctypes.c_int, [dp, ctypes.c_int, tp]),
        "unit_select_conv2d_input": (ctypes.c_int, [dp, ctypes.c_int, ctypes.c_int, tp]),
        "unit_select_matmul": (ctypes.c_int, [i32, i32, i32, ctypes.c_int, tp]),
        "unit_conv2d_i8": (ctypes.c_int, [dp, vp, vp, vp, rp, vp, vp, sz, vp]),
        "unit_conv2d_f16": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_matmul_i8": (ctypes.c_int, [i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, sz, vp]),
        "unit_matmul_f16": (ctypes.c_int, [i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, sz, vp]),
        "unit_pack_act_i8": (ctypes.c_int, [i32, i32, i32, i32, vp, vp, sz, vp]),
        "unit_pack_act_f16": (ctypes.c_int, [i32, i32, i32, i32, vp, vp, sz, vp]),
        "unit_pack_weights_i8": (ctypes.c_int, [dp, vp, vp, sz, vp]),
        "unit_pack_weights_f16": (ctypes.c_int, [dp, vp, vp, sz, vp]),
        "unit_unpack_act_i8": (ctypes.c_int, [i32, i32, i32, i32, vp, vp, vp]),
        "unit_conv2d_packed_i8": (ctypes.c_int, [dp, vp, vp, vp, rp, vp, vp, vp, sz, vp]),
        "unit_conv2d_packed_f16": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_conv2d_wpacked_workspace": (sz, [dp, ctypes.c_int]),
        "unit_conv2d_wpacked_i8": (ctypes.c_int, [dp, vp, vp, vp, rp, vp, vp, sz, vp]),
        "unit_conv2d_wpacked_f16": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_conv2d_wpacked_i8_static": (ctypes.c_int, [dp, vp, vp, vp, rp, vp, vp]),
        "unit_conv3d_out_dims": (ctypes.c_int, [d3, ip, ip, ip]),
        "unit_conv3d_workspace": (sz, [d3, ctypes.c_int]),
        "unit_conv3d_i8": (ctypes.c_int, [d3, vp, vp, vp, vp, sz, vp]),
        "unit_conv3d_f16": (ctypes.c_int, [d3, vp, vp, vp, vp, sz, vp]),
        "unit_maxpool_packed_i8": (ctypes.c_int, [i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]),
        "unit_global_avgpool_packed_i8": (ctypes.c_int, [i32, i32, i32, i32, vp, vp, vp, vp]),
        "unit_widen_residual_i8": (ctypes.c_int, [i32, i32, i32, i32, vp, i32, vp, vp]),
        "unit_conv2d_bf16": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_conv2d_u8i8": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_conv2d_fp8": (ctypes.c_int, [dp, vp, vp, vp, vp, sz, vp]),
        "unit_matmul_fp8": (ctypes.c_int, [i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, sz, vp]),
        "unit_matmul_bf16": (ctypes.c_int, [i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, sz, vp]),
        "unit_matmul_u8i8": (ctypes.c_int, [i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, sz, vp]),
        "unit_conv2d_input_mode": (ctypes.c_int, [dp, ctypes.c_int, vp]),
        "unit_debug_force_tile": (ctypes.c_int, [i32, i32]),
        "unit_measure_mfma": (ctypes.c_int, [ctypes.c_int, i32, i32, vp, sz, vp]),
        "unit_inspect": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_char_p, ctypes.POINTER(unit_inspect_result)]),
        "unit_describe_mfma": (ctypes.c_int, [ctypes.c_int, i32, ctypes.c_char_p, sz]),
        "unit_describe_conv2d": (ctypes.c_int, [dp, ctypes.c_int, ctypes.c_char_p, sz]),
        "unit_describe_matmul": (ctypes.c_int, [i32, i32, i32, ctypes.c_int, ctypes.c_char_p, sz]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


# ------------------------------------------------------------------ marshalling helpers

def _p(t):
    """Device address of a tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(status, where):
    if status != UNIT_OK:
        raise UnitError(status, where)


def conv_desc(n, c, h, w, k, r, s, stride=(1, 1), pad=(0, 0)):
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    return unit_conv2d_desc(n, c, h, w, k, r, s, sh, sw, ph, pw)


def make_requant(scale, bias=None, residual=None, relu=False, residual_packed=None, residual_mult=0):
    return unit_requant(_p(scale), _p(bias), _p(residual), int(bool(relu)),
                        int(residual_mult), _p(residual_packed))


# ------------------------------------------------------------------ entry points (same names as the C ABI)

def unit_version():
    return load().unit_version()


def unit_status_str(status):
    return load().unit_status_str(status).decode()


def unit_conv2d_out_dims(d):
    p, q = ctypes.c_int32(), ctypes.c_int32()
    _check(load().unit_conv2d_out_dims(ctypes.byref(d), ctypes.byref(p), ctypes.byref(q)), "unit_conv2d_out_dims")
    return p.value, q.value


def unit_packed_act_bytes(n, c, h, w, dtype):
    return load().unit_packed_act_bytes(n, c, h, w, dtype)


def unit_packed_weights_bytes(d, dtype):
    return load().unit_packed_weights_bytes(ctypes.byref(d), dtype)


def unit_conv2d_workspace(d, dtype):
    return load().unit_conv2d_workspace(ctypes.byref(d), dtype)


def unit_conv2d_packed_workspace(d, dtype):
    return load().unit_conv2d_packed_workspace(ctypes.byref(d), dtype)


def unit_matmul_workspace(m, n, k, lda, ldb, dtype):
    return load().unit_matmul_workspace(m, n, k, lda, ldb, dtype)


def unit_select_conv2d(d, dtype):
    info = unit_tile_info()
    _check(load().unit_select_conv2d(ctypes.byref(d), dtype, ctypes.byref(info)), "unit_select_conv2d")
    return info


def unit_select_conv2d_input(d, dtype, input_mode):
    info = unit_tile_info()
    _check(load().unit_select_conv2d_input(ctypes.byref(d), dtype, input_mode, ctypes.byref(info)),
           "unit_select_conv2d_input")
    return info


def unit_select_matmul(m, n, k, dtype):
    info = unit_tile_info()
    _check(load().unit_select_matmul(m, n, k, dtype, ctypes.byref(info)), "unit_select_matmul")
    return info


def unit_conv2d_i8(d, x, w, y_i32, rq, y_i8, ws, stream=None):
    wp, wb = _ws(ws)
    _check(load().unit_conv2d_i8(ctypes.byref(d), _p(x), _p(w), _p(y_i32),
                                 ctypes.byref(rq) if rq is not None else None, _p(y_i8),
                                 wp, wb, _stream(stream)), "unit_conv2d_i8")


def unit_conv2d_f16(d, x, w, y, ws, stream=None):
    wp, wb = _ws(ws)
    _check(load().unit_conv2d_f16(ctypes.byref(d), _p(x), _p(w), _p(y), wp, wb, _stream(stream)),
           "unit_conv2d_f16")


def unit_matmul_i8(m, n, k, A, lda, B, ldb, C, ldc, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().unit_matmul_i8(m, n, k, _p(A), lda, _p(B), ldb, _p(C), ldc, wp, wb, _stream(stream)),
           "unit_matmul_i8")


def unit_matmul_f16(m, n, k, A, lda, B, ldb, C, ldc, ws=None, stream=None):
    wp, wb = _ws(ws)
    _check(load().unit_matmul_f16(m, n, k, _p(A), lda, _p(B), ldb, _p(C), ldc, wp, wb, _stream(stream)),
           "unit_matmul_f16")


def unit_pack_act_i8(n, c, h, w, x, xp, stream=None):
    _check(load().unit_pack_act_i8(n, c, h, w, _p(x), _p(xp), xp.numel() * xp.element_size(),
                                   _stream(stream)), "unit_pack_act_i8")


def unit_pack_act_f16(n, c, h, w, x, xp, stream=None):
    _check(load().unit_pack_act_f16(n, c, h, w, _p(x), _p(xp), xp.numel() * xp.element_size(),
                                    _stream(stream)), "unit_pack_act_f16")


def unit_pack_weights_i8(d, w, wp, stream=None):
    _check(load().unit_pack_weights_i8(ctypes.byref(d), _p(w), _p(wp), wp.numel() * wp.element_size(),
                                       _stream(stream)), "unit_pack_weights_i8")


def unit_pack_weights_f16(d, w, wp, stream=None):
    _check(load().unit_pack_weights_f16(ctypes.byref(d), _p(w), _p(wp), wp.numel() * wp.element_size(),
                                        _stream(stream)), "unit_pack_weights_f16")


def unit_unpack_act_i8(n, c, h, w, xp, x, stream=None):
    _check(load().unit_unpack_act_i8(n, c, h, w, _p(xp), _p(x), _stream(stream)), "unit_unpack_act_i8")


def unit_conv2d_packed_i8(d, xp, wp, y_i32, rq, y_i8, y_packed, ws=None, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv2d_packed_i8(ctypes.byref(d), _p(xp), _p(wp), _p(y_i32),
                                        ctypes.byref(rq) if rq is not None else None,
                                        _p(y_i8), _p(y_packed), wsp, wsb, _stream(stream)),
           "unit_conv2d_packed_i8")


def unit_conv2d_packed_f16(d, xp, wp, y, ws=None, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv2d_packed_f16(ctypes.byref(d), _p(xp), _p(wp), _p(y), wsp, wsb, _stream(stream)),
           "unit_conv2d_packed_f16")


def unit_conv2d_wpacked_workspace(d, dtype):
    return load().unit_conv2d_wpacked_workspace(ctypes.byref(d), dtype)


def unit_conv2d_wpacked_i8(d, x, wp, y_i32, rq, y_i8, ws=None, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv2d_wpacked_i8(ctypes.byref(d), _p(x), _p(wp), _p(y_i32),
                                         ctypes.byref(rq) if rq is not None else None, _p(y_i8),
                                         wsp, wsb, _stream(stream)), "unit_conv2d_wpacked_i8")


def unit_conv2d_wpacked_i8_static(d, x, wp, y_i32, rq, y_i8, stream=None):
    _check(load().unit_conv2d_wpacked_i8_static(ctypes.byref(d), _p(x), _p(wp), _p(y_i32),
                                                ctypes.byref(rq) if rq is not None else None, _p(y_i8),
                                                _stream(stream)), "unit_conv2d_wpacked_i8_static")


def unit_conv2d_wpacked_f16(d, x, wp, y, ws=None, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv2d_wpacked_f16(ctypes.byref(d), _p(x), _p(wp), _p(y), wsp, wsb, _stream(stream)),
           "unit_conv2d_wpacked_f16")


def conv3d_desc(n, c, d, h, w, k, t, r, s, stride=(1, 1, 1), pad=(0, 0, 0)):
    return unit_conv3d_desc(n, c, d, h, w, k, t, r, s, *stride, *pad)


def unit_conv3d_out_dims(d):
    o, p, q = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(load().unit_conv3d_out_dims(ctypes.byref(d), ctypes.byref(o), ctypes.byref(p), ctypes.byref(q)),
           "unit_conv3d_out_dims")
    return o.value, p.value, q.value


def unit_conv3d_workspace(d, dtype):
    return load().unit_conv3d_workspace(ctypes.byref(d), dtype)


def unit_conv3d_i8(d, x, w, y, ws, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv3d_i8(ctypes.byref(d), _p(x), _p(w), _p(y), wsp, wsb, _stream(stream)), "unit_conv3d_i8")


def unit_conv3d_f16(d, x, w, y, ws, stream=None):
    wsp, wsb = _ws(ws)
    _check(load().unit_conv3d_f16(ctypes.byref(d), _p(x), _p(w), _p(y), wsp, wsb, _stream(stream)), "unit_conv3d_f16")


def unit_maxpool_packed_i8(n, c, h, w, window, stride, pad, xp, yp, stream=None):
    _check(load().unit_maxpool_packed_i8(n, c, h, w, window, stride, pad, _p(xp), _p(yp), _stream(stream)),
           "unit_maxpool_packed_i8")


def unit_global_avgpool_packed_i8(n, c, h, w, xp, scale, y, stream=None):
    _check(load().unit_global_avgpool_packed_i8(n, c, h, w, _p(xp), _p(scale), _p(y), _stream(stream)),
           "unit_global_avgpool_packed_i8")


def unit_widen_residual_i8(n, c, h, w, xp, mult, residual, stream=None):
    _check(load().unit_widen_residual_i8(n, c, h, w, _p(xp), mult, _p(residual), _stream(stream)),
           "unit_widen_residual_i8")


UNIT_INPUT_PACKED, UNIT_INPUT_DIRECT, UNIT_INPUT_DIRECT_SHIFTED = 0, 1, 2


def unit_conv2d_input_mode(d, dtype, x):
    rc = load().unit_conv2d_input_mode(ctypes.byref(d), dtype, _p(x))
    if rc < 0:
        _check(rc, "unit_conv2d_input_mode")
    return rc


UNIT_MEASURE_COUNTERS_BYTES = 256 * 8 * 4 * 8


def unit_measure_mfma(dtype, steps, random_operands, counters, stream=None):
    cp, cb = _ws(counters)
    _check(load().unit_measure_mfma(dtype, int(steps), int(bool(random_operands)), cp, cb, _stream(stream)),
           "unit_measure_mfma")


def unit_debug_force_tile(tile, split_k):
    _check(load().unit_debug_force_tile(int(tile), int(split_k)), "unit_debug_force_tile")


# ------------------------------------------------------------------ further operand types

def _conv_simple(name, d, x, w, y, ws, stream):
    wp, wb = _ws(ws)
    _check(getattr(load(), name)(ctypes.byref(d), _p(x), _p(w), _p(y), wp, wb, _stream(stream)), name)


def _matmul_simple(name, m, n, k, A, lda, B, ldb, C, ldc, ws, stream):
    wp, wb = _ws(ws)
    _check(getattr(load(), name)(m, n, k, _p(A), lda, _p(B), ldb, _p(C), ldc, wp, wb, _stream(stream)), name)


def unit_conv2d_bf16(d, x, w, y, ws, stream=None):
    _conv_simple("unit_conv2d_bf16", d, x, w, y, ws, stream)


def unit_conv2d_u8i8(d, x, w, y, ws, stream=None):
    _conv_simple("unit_conv2d_u8i8", d, x, w, y, ws, stream)


def unit_conv2d_fp8(d, x, w, y, ws, stream=None):
    _conv_simple("unit_conv2d_fp8", d, x, w, y, ws, stream)


def unit_matmul_fp8(m, n, k, A, lda, B, ldb, C, ldc, ws=None, stream=None):
    _matmul_simple("unit_matmul_fp8", m, n, k, A, lda, B, ldb, C, ldc, ws, stream)


def unit_matmul_bf16(m, n, k, A, lda, B, ldb, C, ldc, ws=None, stream=None):
    _matmul_simple("unit_matmul_bf16", m, n, k, A, lda, B, ldb, C, ldc, ws, stream)


def unit_matmul_u8i8(m, n, k, A, lda, B, ldb, C, ldc, ws=None, stream=None):
    _matmul_simple("unit_matmul_u8i8", m, n, k, A, lda, B, ldb, C, ldc, ws, stream)


# ------------------------------------------------------------------ applicability inspection (host only)

def unit_inspect(instruction, operation):
    """-> dict(applicable, failed_step, mapping {instr loop: op loop},
    operands [(instr register, op array, [broadcast loops])], num_feasible)."""
    res = unit_inspect_result()
    _check(load().unit_inspect(instruction.encode(), operation.encode(), ctypes.byref(res)), "unit_inspect")
    loops = [res.instr_loop[i].value.decode() for i in range(res.num_loops)]
    mapping = {loops[i]: res.op_loop[i].value.decode() for i in range(res.num_loops)}
    operands = []
    for i in range(res.num_operands):
        bc = [loops[b] for b in range(res.num_loops) if res.broadcast[i] >> b & 1]
        operands.append((res.instr_operand[i].value.decode(), res.op_operand[i].value.decode(), bc))
    return {"applicable": bool(res.applicable), "failed_step": res.failed_step, "mapping": mapping,
            "operands": operands, "num_feasible": res.num_feasible}


def _describe(fn, name, *args):
    need = fn(*args, None, 0)
    if need < 0:
        _check(need, name)
    buf = ctypes.create_string_buffer(need)
    fn(*args, buf, need)
    return buf.value.decode()


def unit_describe_mfma(dtype, edge):
    return _describe(load().unit_describe_mfma, "unit_describe_mfma", dtype, edge)


def unit_describe_conv2d(d, dtype):
    return _describe(load().unit_describe_conv2d, "unit_describe_conv2d", ctypes.byref(d), dtype)


def unit_describe_matmul(m, n, k, dtype):
    return _describe(load().unit_describe_matmul, "unit_describe_matmul", m, n, k, dtype)
