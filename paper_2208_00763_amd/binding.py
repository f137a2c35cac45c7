"""ctypes binding of libhikonv.so: same names as include/hikonv.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing
else); every function enqueues on torch's current stream unless `stream` is given.  There is
no CPU fallback: if the library is missing or was not built, importing this module fails.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("HIKONV_LIB", os.path.join(HERE, "libhikonv.so"))   # HIKONV_LIB: a tuning variant

OK, EINVAL, EOVERFLOW, ENOPLAN, EHIP, EWORKSPACE, EUNSUPPORTED, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7
NOALLOC_SCRATCH_BYTES = 8 << 20
MODE_SINGLE, MODE_CONV1D, MODE_DNN = 0, 1, 2
A_SIGNED, W_SIGNED, BIPOLAR = 1, 2, 4
FMT_INT8, FMT_BITDENSE, FMT_PACKED = 0, 1, 2
OUT_FULL, OUT_VALID = 0, 1
UB_MAD_U32_U24, UB_MAD_U64_U32, UB_MUL_LO_U32, UB_BFE_U32, UB_LSHR_B64, UB_DPP_MOV, UB_ADD_U32 = range(7)
UB_MAD_I32_I24, UB_MAD_I64_I32, UB_ADD_U64, UB_ALIGNBIT, UB_AND_B32 = range(7, 12)
UB_ASHR_I64, UB_BFE_I32, UB_CHAIN_MAD_I64_I32, UB_CHAIN_MAD_I32_I24 = 12, 13, 14, 15
UB_HBM_WRITE, UB_HBM_COPY, UB_HBM_READ, UB_HBM_WRITE_NT, UB_HBM_WRITE_RUNS, UB_HBM_WRITE_VARIED = 16, 17, 18, 19, 20, 21

OBJ_PAPER_OPS, OBJ_MEASURED_COST = 0, 1
KERNEL_AUTO, KERNEL_LDS, KERNEL_SREG, KERNEL_LANES, KERNEL_WINDOW = 0, 1, 2, 3, 4
F_STORES64 = 1
LAYER_MAX_N = 8

PLAN_FIELDS = ("bits_a bits_w a_signed w_signed bipolar L_A L_B L_acc mode M taps tight objective out_bits max_N "
               "kernel flags N K S G_b chunks ops_per_mul paper_exact stride_elems cost_milli").split()


class Plan(C.Structure):
    """Mirror of hikonv_plan_t."""
    _fields_ = [(name, C.c_int32) for name in PLAN_FIELDS]

    def as_dict(self):
        return {name: getattr(self, name) for name in PLAN_FIELDS}

    def __repr__(self):
        return "Plan(%s)" % ", ".join("%s=%d" % kv for kv in self.as_dict().items())


class HikonvError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s failed: %s (code %d, hip error %d)" % (
            where, lib.hikonv_strerror(code).decode(), code, lib.hikonv_last_hip_error()))


def _load():
    # PyTorch ships its own HIP runtime; it must be the one already loaded when libhikonv.so
    # resolves libamdhip64, otherwise the process ends up with two runtimes and the library's
    # launches see no device.  Importing torch first guarantees that.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        from .build import build
        build(force=True)
    return C.CDLL(LIB_PATH)


lib = _load()

_vp, _i, _i64, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
_pp = C.POINTER(Plan)
SIGNATURES = {
    "hikonv_plan": (_i, [_i, _i, _i, _i, _pp]),
    "hikonv_plan_ex": (_i, [_pp, _pp]),
    "hikonv_plan_check": (_i, [_pp]),
    "hikonv_plan_cost": (_i, [_pp]),
    "hikonv_bitdense_row_bytes": (_i64, [_i64, _i]),
    "hikonv_compact": (_i, [_vp, _i64, _i64, _i, _i, _vp, _vp]),
    "hikonv_check_range": (_i, [_vp, _i64, _i, _i, _i, _vp, _vp]),
    "hikonv_conv1d": (_i, [_pp, _vp, _i, _i64, _i64, _vp, _i, _i, _vp, _vp]),
    "hikonv_conv1d_unpacked": (_i, [_i, _i, _i, _vp, _i, _i64, _i64, _vp, _i, _i, _vp, _vp]),
    "hikonv_conv1d_requant": (_i, [_pp, _vp, _i, _i64, _i64, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_conv1d_requant_unpacked": (_i, [_i, _i, _i, _vp, _i, _i64, _i64, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_packed_weights_bytes": (_sz, [_pp, _i, _i, _i, _i]),
    "hikonv_pack_weights": (_i, [_pp, _vp, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_packed_weights_bytes_ex": (_sz, [_pp, _i, _i, _i, _i, _i, _i]),
    "hikonv_pack_weights_ex": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_conv3d_workspace_bytes": (_sz, [_pp, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i]),
    "hikonv_conv3d": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i, _i, _i, _vp, _sz, _vp, _vp]),
    "hikonv_conv2d_workspace_bytes": (_sz, [_pp, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i]),
    "hikonv_conv2d": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i, _vp, _sz, _vp, _vp]),
    "hikonv_conv2d_prepacked": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i, _vp, _sz, _vp, _vp]),
    "hikonv_conv2d_noalloc": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_conv2d_unpacked": (_i, [_i, _i, _i, _vp, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_epilogue": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i, _i, _i, _vp, _vp]),
    "hikonv_epilogue_pack": (_i, [_vp, _i, _i, _i, _i, _i, _i, _i, _pp, _i, _i, _i, _i, _i, _vp, _sz, _vp]),
    "hikonv_conv2d_fused": (_i, [_pp, _vp, _i, _i, _i, _i, _i, _vp, _i, _i, _i, _i, _vp, _sz, _vp, _i, _i, _i, _pp, _i, _i, _i,
                                 _i, _vp, _sz, _vp]),
    "hikonv_ubench": (_i, [_i, _i, _i, _vp, _sz, _vp]),
    "hikonv_selftest_lane_shift": (_i, [_vp, _vp]),
    "hikonv_strerror": (C.c_char_p, [_i]),
    "hikonv_last_hip_error": (_i, []),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


def _check(code, where):
    if code != OK:
        raise HikonvError(code, where)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _raw_stream_getter():
    """Fastest available way to read the raw handle of torch's current stream."""
    import torch
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is not None:
        return lambda: raw(torch.cuda.current_device())
    return lambda: torch.cuda.current_stream().cuda_stream


_current_raw_stream = None


def _stream(stream):
    """Handle of the stream to launch on: the caller's, else torch's current stream."""
    global _current_raw_stream
    if stream is not None:
        return C.c_void_p(stream)
    if _current_raw_stream is None:
        _current_raw_stream = _raw_stream_getter()
    return C.c_void_p(_current_raw_stream())


def signedness(a_signed=False, w_signed=False, bipolar=False):
    return (A_SIGNED if a_signed else 0) | (W_SIGNED if w_signed else 0) | (BIPOLAR if bipolar else 0)


# ---- host-only entry points ------------------------------------------------------------
def hikonv_plan(bits_a, bits_w, signedness_flags, mult_width):
    out = Plan()
    _check(lib.hikonv_plan(bits_a, bits_w, signedness_flags, mult_width, C.byref(out)), "hikonv_plan")
    return out


def hikonv_plan_ex(**request):
    req = Plan(**request)
    out = Plan()
    _check(lib.hikonv_plan_ex(C.byref(req), C.byref(out)), "hikonv_plan_ex")
    return out


def hikonv_plan_check(plan):
    return lib.hikonv_plan_check(C.byref(plan))


def hikonv_plan_cost(plan):
    """Modelled VALU issue slots per output x 1000 of a fully specified 1-D plan (negative: error code)."""
    return lib.hikonv_plan_cost(C.byref(plan))


def with_fields(plan, **fields):
    """A copy of `plan` with some fields replaced (e.g. kernel=KERNEL_SREG, flags=F_STORES64)."""
    out = Plan(**plan.as_dict())
    for name, value in fields.items():
        setattr(out, name, value)
    return out


def hikonv_bitdense_row_bytes(length, bits):
    return lib.hikonv_bitdense_row_bytes(length, bits)


def hikonv_strerror(code):
    return lib.hikonv_strerror(code).decode()


# ---- device entry points ---------------------------------------------------------------
def hikonv_check_range(x, count, bits, is_signed, bipolar, violations, stream=None):
    _check(lib.hikonv_check_range(_ptr(x), count, bits, int(is_signed), int(bipolar), _ptr(violations), _stream(stream)),
           "hikonv_check_range")


def hikonv_compact(x, rows, length, bits, bipolar, out, stream=None):
    _check(lib.hikonv_compact(_ptr(x), rows, length, bits, int(bipolar), _ptr(out), _stream(stream)), "hikonv_compact")


def hikonv_conv1d(plan, x, x_format, rows, length, g, taps, out_mode, y, stream=None):
    _check(lib.hikonv_conv1d(C.byref(plan), _ptr(x), x_format, rows, length, _ptr(g), taps, out_mode, _ptr(y),
                             _stream(stream)), "hikonv_conv1d")


def hikonv_conv1d_unpacked(bits_a, bits_w, signedness_flags, x, x_format, rows, length, g, taps, out_mode, y,
                           stream=None):
    _check(lib.hikonv_conv1d_unpacked(bits_a, bits_w, signedness_flags, _ptr(x), x_format, rows, length, _ptr(g),
                                      taps, out_mode, _ptr(y), _stream(stream)), "hikonv_conv1d_unpacked")


def hikonv_conv1d_requant(plan, x, x_format, rows, length, g, taps, out_mode, shift, qmax, out_bits, q, stream=None):
    _check(lib.hikonv_conv1d_requant(C.byref(plan), _ptr(x), x_format, rows, length, _ptr(g), taps, out_mode, shift,
                                     qmax, out_bits, _ptr(q), _stream(stream)), "hikonv_conv1d_requant")


def hikonv_conv1d_requant_unpacked(bits_a, bits_w, signedness_flags, x, x_format, rows, length, g, taps, out_mode,
                                   shift, qmax, out_bits, q, stream=None):
    _check(lib.hikonv_conv1d_requant_unpacked(bits_a, bits_w, signedness_flags, _ptr(x), x_format, rows, length,
                                              _ptr(g), taps, out_mode, shift, qmax, out_bits, _ptr(q),
                                              _stream(stream)), "hikonv_conv1d_requant_unpacked")


def hikonv_packed_weights_bytes(plan, co, c, kh, kw):
    return lib.hikonv_packed_weights_bytes(C.byref(plan), co, c, kh, kw)


def hikonv_pack_weights(plan, w, co, c, kh, kw, packed, stream=None):
    _check(lib.hikonv_pack_weights(C.byref(plan), _ptr(w), co, c, kh, kw, _ptr(packed), _stream(stream)),
           "hikonv_pack_weights")


def hikonv_packed_weights_bytes_ex(plan, co, c, kd, kh, kw, stride):
    return lib.hikonv_packed_weights_bytes_ex(C.byref(plan), co, c, kd, kh, kw, stride)


def hikonv_pack_weights_ex(plan, w, co, c, kd, kh, kw, stride, packed, stream=None):
    _check(lib.hikonv_pack_weights_ex(C.byref(plan), _ptr(w), co, c, kd, kh, kw, stride, _ptr(packed),
                                      _stream(stream)), "hikonv_pack_weights_ex")


def hikonv_conv3d_workspace_bytes(plan, n, c, d, h, w, co, kd, kh, kw, stride, pad, prepacked):
    return lib.hikonv_conv3d_workspace_bytes(C.byref(plan), n, c, d, h, w, co, kd, kh, kw, stride, pad,
                                             int(prepacked))


def hikonv_conv3d(plan, x, x_format, n, c, d, h, w, weights, prepacked, co, kd, kh, kw, stride, pad, workspace, y,
                  stream=None):
    _check(lib.hikonv_conv3d(C.byref(plan), _ptr(x), x_format, n, c, d, h, w, _ptr(weights), int(prepacked), co, kd,
                             kh, kw, stride, pad, _ptr(workspace), workspace.numel() * workspace.element_size(),
                             _ptr(y), _stream(stream)), "hikonv_conv3d")


def hikonv_conv2d_workspace_bytes(plan, n, c, h, w, co, kh, kw, stride, pad, prepacked):
    return lib.hikonv_conv2d_workspace_bytes(C.byref(plan), n, c, h, w, co, kh, kw, stride, pad, int(prepacked))


def hikonv_conv2d(plan, x, x_format, n, c, h, w, weights, co, kh, kw, stride, pad, workspace, y, stream=None):
    _check(lib.hikonv_conv2d(C.byref(plan), _ptr(x), x_format, n, c, h, w, _ptr(weights), co, kh, kw, stride, pad,
                             _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(y),
                             _stream(stream)), "hikonv_conv2d")


def hikonv_conv2d_noalloc(plan, x, x_format, n, c, h, w, weights, co, kh, kw, stride, pad, y, stream=None):
    _check(lib.hikonv_conv2d_noalloc(C.byref(plan), _ptr(x), x_format, n, c, h, w, _ptr(weights), co, kh, kw, stride,
                                     pad, _ptr(y), _stream(stream)), "hikonv_conv2d_noalloc")


def hikonv_conv2d_prepacked(plan, x, x_format, n, c, h, w, packed, co, kh, kw, stride, pad, workspace, y,
                            stream=None):
    _check(lib.hikonv_conv2d_prepacked(C.byref(plan), _ptr(x), x_format, n, c, h, w, _ptr(packed), co, kh, kw,
                                       stride, pad, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _ptr(y), _stream(stream)), "hikonv_conv2d_prepacked")


def hikonv_conv2d_unpacked(bits_a, bits_w, signedness_flags, x, n, c, h, w, weights, co, kh, kw, stride, pad, y,
                           stream=None):
    _check(lib.hikonv_conv2d_unpacked(bits_a, bits_w, signedness_flags, _ptr(x), n, c, h, w, _ptr(weights), co, kh,
                                      kw, stride, pad, _ptr(y), _stream(stream)), "hikonv_conv2d_unpacked")


def hikonv_epilogue(acc, n, c, h, w, shift, qmax, pool, out_bits, out_format, out, stream=None):
    _check(lib.hikonv_epilogue(_ptr(acc), n, c, h, w, shift, qmax, int(pool), out_bits, out_format, _ptr(out),
                               _stream(stream)), "hikonv_epilogue")


def hikonv_epilogue_pack(acc, n, c, h, w, shift, qmax, pool, next_plan, next_co, next_kh, next_kw, next_stride,
                         next_pad, next_workspace, stream=None):
    _check(lib.hikonv_epilogue_pack(_ptr(acc), n, c, h, w, shift, qmax, int(pool), C.byref(next_plan), next_co,
                                    next_kh, next_kw, next_stride, next_pad, _ptr(next_workspace),
                                    next_workspace.numel() * next_workspace.element_size(), _stream(stream)),
           "hikonv_epilogue_pack")


def hikonv_conv2d_fused(plan, x, x_format, n, c, h, w, packed, co, kh, kw, pad, workspace, y, shift=0, qmax=0, pool=False,
                        next_plan=None, next_co=0, next_kh=0, next_kw=0, next_pad=0, next_workspace=None, stream=None):
    """y may be None (accumulators not stored); next_plan None: plain layer; workspace may be None
    where the layer packs its own input (see include/hikonv.h)."""
    nws_bytes = next_workspace.numel() * next_workspace.element_size() if next_workspace is not None else 0
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.hikonv_conv2d_fused(C.byref(plan), _ptr(x), x_format, n, c, h, w, _ptr(packed), co, kh, kw, pad,
                                   _ptr(workspace), ws_bytes, _ptr(y), shift, qmax,
                                   int(pool), C.byref(next_plan) if next_plan is not None else None, next_co, next_kh,
                                   next_kw, next_pad, _ptr(next_workspace), nws_bytes, _stream(stream)),
           "hikonv_conv2d_fused")


def hikonv_ubench(kind, iters, blocks, buf, stream=None):
    _check(lib.hikonv_ubench(kind, iters, blocks, _ptr(buf), buf.numel() * buf.element_size(), _stream(stream)),
           "hikonv_ubench")


def hikonv_selftest_lane_shift(out, stream=None):
    _check(lib.hikonv_selftest_lane_shift(_ptr(out), _stream(stream)), "hikonv_selftest_lane_shift")
