"""ctypes binding of libmsgemm.so -- argument marshalling only.

The functions carry the names of the C ABI (``include/msgemm.h``, ``include/msgemm_measure.h``); every step of
the msGeMM path runs in the library's HIP kernels.  Device memory and streams
come from PyTorch: a tensor argument is passed as its ``data_ptr()``, the stream
defaults to torch's current stream.  There is no CPU fallback: if the library
has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmsgemm.so")

F32, F16, BF16, I8, I32 = 0, 1, 2, 3, 4
DTYPES = {"f32": F32, "f16": F16, "bf16": BF16, "i8": I8, "i32": I32}
VARIANT_AUTO, VARIANT_GLOBAL_LUT, VARIANT_FUSED_LDS, VARIANT_FUSED_LDS16, VARIANT_GLOBAL_LUT_HALF = 0, 1, 2, 3, 4
OK, ERR_INVALID_ARG, ERR_ALLOC, ERR_HIP, ERR_UNSUPPORTED, ERR_INCOMPLETE, ERR_RANGE = 0, -1, -2, -3, -4, -5, -6

EXPORTS = (
    "msgemm_plan", "msgemm_plan_with_options", "msgemm_plan_codes8", "msgemm_plan_set_codebook", "msgemm_plan_get_info", "msgemm_lut_bytes", "msgemm_build_lut",
    "msgemm_consume_lut", "msgemm_run", "msgemm_run_static", "msgemm_plan_check", "msgemm_dequant_mfma_run", "msgemm_calib_stream_read", "msgemm_calib_stream_read_shape", "msgemm_calib_lds_read", "msgemm_calib_lookup_add", "msgemm_destroy",
    "msgemm_status_string", "msgemm_last_hip_error", "msgemm_version",
)


class MsgemmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        text = status_string(status)
        extra = f" (hipError {last_hip_error()})" if status == ERR_HIP else ""
        super().__init__(f"{where}: {text}{extra}")


class PlanInfo(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int64), ("k", ctypes.c_int64), ("b", ctypes.c_int64),
        ("x_dtype", ctypes.c_int), ("y_dtype", ctypes.c_int), ("lut_dtype", ctypes.c_int),
        ("d", ctypes.c_int), ("scale_group", ctypes.c_int), ("variant", ctypes.c_int),
        ("lut_groups", ctypes.c_int64),
        ("tile_rows", ctypes.c_int), ("tile_groups", ctypes.c_int),
        ("split_k", ctypes.c_int), ("col_chunk", ctypes.c_int),
        ("workspace_bytes", ctypes.c_int64),
    ]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class PlanOptions(ctypes.Structure):
    """msgemm_plan_options_t: requests for a particular kernel form (tests, measurements); zero = none."""
    _fields_ = [
        ("struct_size", ctypes.c_size_t),
        ("panels_per_workgroup", ctypes.c_int), ("k_tiles_per_workgroup", ctypes.c_int),
        ("reduce_mode", ctypes.c_int), ("rows_per_lane", ctypes.c_int), ("no_xcd_map", ctypes.c_int),
        ("batched_form", ctypes.c_int), ("batched_segments", ctypes.c_int),
        ("global_plain_consumer", ctypes.c_int), ("global_chunk_kib", ctypes.c_int), ("global_segments", ctypes.c_int),
        ("build_on_matrix_cores", ctypes.c_int), ("half_tables_in_lds", ctypes.c_int), ("poll_limit", ctypes.c_int),
        ("skip_publish", ctypes.c_int), ("batched_deal", ctypes.c_int),
    ]


def _options(options):
    """dict of field names -> ctypes structure (None stays None)."""
    if options is None:
        return None
    o = PlanOptions()
    o.struct_size = ctypes.sizeof(PlanOptions)
    names = {n for n, _ in PlanOptions._fields_}
    for key, value in options.items():
        if key not in names or key == "struct_size":
            raise ValueError(f"unknown plan option {key!r}")
        setattr(o, key, int(value))
    return o


_lib = None


def load():
    """Load libmsgemm.so (built by ``python -m paper_2310_06178_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2310_06178_amd.build` "
            "(there is no CPU fallback for the msGeMM path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.msgemm_plan.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci, ci, ci, vp, vp, ci, vp]
    lib.msgemm_plan.restype = ci
    lib.msgemm_plan_with_options.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci, ci, ci, vp, vp, ci,
                                             ctypes.POINTER(PlanOptions), vp]
    lib.msgemm_plan_with_options.restype = ci
    lib.msgemm_plan_codes8.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, ci, ci, vp, vp,
                                       ctypes.POINTER(ctypes.c_float), ctypes.POINTER(PlanOptions), vp]
    lib.msgemm_plan_codes8.restype = ci
    lib.msgemm_plan_set_codebook.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    lib.msgemm_plan_set_codebook.restype = ci
    lib.msgemm_plan_get_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
    lib.msgemm_plan_get_info.restype = ci
    lib.msgemm_lut_bytes.argtypes = [vp]
    lib.msgemm_lut_bytes.restype = ctypes.c_size_t
    lib.msgemm_build_lut.argtypes = [vp, vp, i64, vp, vp]
    lib.msgemm_build_lut.restype = ci
    lib.msgemm_consume_lut.argtypes = [vp, vp, vp, i64, vp]
    lib.msgemm_consume_lut.restype = ci
    lib.msgemm_run.argtypes = [vp, vp, i64, vp, i64, vp]
    lib.msgemm_run.restype = ci
    lib.msgemm_run_static.argtypes = [vp, vp, i64, vp, i64, vp]
    lib.msgemm_run_static.restype = ci
    lib.msgemm_plan_check.argtypes = [vp, vp]
    lib.msgemm_plan_check.restype = ci
    lib.msgemm_dequant_mfma_run.argtypes = [vp, vp, i64, vp, i64, vp]
    lib.msgemm_dequant_mfma_run.restype = ci
    lib.msgemm_calib_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.msgemm_calib_stream_read.restype = ci
    lib.msgemm_calib_stream_read_shape.argtypes = [vp, ctypes.c_size_t, vp, ci, ci, ci, ci, vp]
    lib.msgemm_calib_stream_read_shape.restype = ci
    lib.msgemm_calib_lds_read.argtypes = [ci, ci, vp, ctypes.POINTER(ctypes.c_size_t), vp]
    lib.msgemm_calib_lds_read.restype = ci
    lib.msgemm_calib_lookup_add.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_size_t), vp]
    lib.msgemm_calib_lookup_add.restype = ci
    lib.msgemm_destroy.argtypes = [vp]
    lib.msgemm_destroy.restype = None
    lib.msgemm_status_string.argtypes = [ci]
    lib.msgemm_status_string.restype = ctypes.c_char_p
    lib.msgemm_last_hip_error.argtypes = []
    lib.msgemm_last_hip_error.restype = ci
    lib.msgemm_version.argtypes = []
    lib.msgemm_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _ptr(t):
    """Device address of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def status_string(status: int) -> str:
    return load().msgemm_status_string(int(status)).decode()


def last_hip_error() -> int:
    return int(load().msgemm_last_hip_error())


def version() -> str:
    return load().msgemm_version().decode()


def msgemm_plan(m, k, b, x_dtype, y_dtype, d, scale_group, W_codes, scales=None,
                variant=VARIANT_AUTO, stream=None, check=True, options=None):
    """Returns the plan handle (an int).  With check=False returns (status, handle).
    options: dict of msgemm_plan_options_t fields; given, msgemm_plan_with_options is the call made."""
    if options is not None:
        return msgemm_plan_with_options(m, k, b, x_dtype, y_dtype, d, scale_group, W_codes, scales, variant,
                                        options, stream, check)
    lib = load()
    out = ctypes.c_void_p()
    rc = lib.msgemm_plan(ctypes.byref(out), int(m), int(k), int(b),
                         DTYPES.get(x_dtype, x_dtype), DTYPES.get(y_dtype, y_dtype),
                         int(d), int(scale_group), _ptr(W_codes), _ptr(scales), int(variant),
                         _stream(stream))
    if not check:
        return rc, out.value
    if rc != OK:
        raise MsgemmError(rc, "msgemm_plan")
    return out.value


def msgemm_plan_with_options(m, k, b, x_dtype, y_dtype, d, scale_group, W_codes, scales, variant, options,
                             stream=None, check=True):
    """options: dict of msgemm_plan_options_t fields, a PlanOptions, or None."""
    lib = load()
    out = ctypes.c_void_p()
    opts = options if isinstance(options, PlanOptions) or options is None else _options(options)
    rc = lib.msgemm_plan_with_options(ctypes.byref(out), int(m), int(k), int(b),
                                      DTYPES.get(x_dtype, x_dtype), DTYPES.get(y_dtype, y_dtype),
                                      int(d), int(scale_group), _ptr(W_codes), _ptr(scales), int(variant),
                                      None if opts is None else ctypes.byref(opts), _stream(stream))
    if not check:
        return rc, out.value
    if rc != OK:
        raise MsgemmError(rc, "msgemm_plan_with_options")
    return out.value


def msgemm_plan_codes8(m, k, b, x_dtype, y_dtype, scale_group, W_codes8, scales, values256,
                       stream=None, check=True, options=None):
    """Plan for 8-bit weights; values256: 256 floats (host).  Returns the handle,
    or (status, handle) with check=False."""
    lib = load()
    out = ctypes.c_void_p()
    vals = (ctypes.c_float * 256)(*[float(v) for v in values256])
    rc = lib.msgemm_plan_codes8(ctypes.byref(out), int(m), int(k), int(b),
                                DTYPES.get(x_dtype, x_dtype), DTYPES.get(y_dtype, y_dtype),
                                int(scale_group), _ptr(W_codes8), _ptr(scales), vals,
                                None if options is None else ctypes.byref(_options(options)), _stream(stream))
    if not check:
        return rc, out.value
    if rc != OK:
        raise MsgemmError(rc, "msgemm_plan_codes8")
    return out.value


def msgemm_plan_get_info(plan) -> dict:
    info = PlanInfo()
    rc = load().msgemm_plan_get_info(ctypes.c_void_p(plan), ctypes.byref(info))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_plan_get_info")
    return info.as_dict()


def msgemm_lut_bytes(plan) -> int:
    return int(load().msgemm_lut_bytes(ctypes.c_void_p(plan)))


def msgemm_build_lut(plan, X, ldx, L_out, stream=None):
    rc = load().msgemm_build_lut(ctypes.c_void_p(plan), _ptr(X), int(ldx), _ptr(L_out), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_build_lut")


def msgemm_consume_lut(plan, L, Y, ldy, stream=None):
    rc = load().msgemm_consume_lut(ctypes.c_void_p(plan), _ptr(L), _ptr(Y), int(ldy), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_consume_lut")


def msgemm_run(plan, X, ldx, Y, ldy, stream=None):
    rc = load().msgemm_run(ctypes.c_void_p(plan), _ptr(X), int(ldx), _ptr(Y), int(ldy), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_run")


def msgemm_run_static(plan, X, ldx, Y, ldy, stream=None, check=True):
    rc = load().msgemm_run_static(ctypes.c_void_p(plan), _ptr(X), int(ldx), _ptr(Y), int(ldy), _stream(stream))
    if check and rc != OK:
        raise MsgemmError(rc, "msgemm_run_static")
    return rc


def msgemm_plan_check(plan, stream=None) -> int:
    """OK, or ERR_INCOMPLETE when a reduction inside a launch gave up since the last check (then cleared)."""
    return int(load().msgemm_plan_check(ctypes.c_void_p(plan), _stream(stream)))


def msgemm_dequant_mfma_run(plan, X, ldx, Y, ldy, stream=None):
    rc = load().msgemm_dequant_mfma_run(ctypes.c_void_p(plan), _ptr(X), int(ldx), _ptr(Y), int(ldy),
                                        _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_dequant_mfma_run")


def msgemm_calib_lds_read(width_bytes, reads, sink, stream=None):
    """Returns the bytes one launch reads from LDS."""
    out = ctypes.c_size_t(0)
    rc = load().msgemm_calib_lds_read(int(width_bytes), int(reads), _ptr(sink), ctypes.byref(out), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_calib_lds_read")
    return out.value


def msgemm_calib_lookup_add(tiles, sink, stream=None):
    """Returns the lane look-ups one launch makes."""
    out = ctypes.c_size_t(0)
    rc = load().msgemm_calib_lookup_add(int(tiles), _ptr(sink), ctypes.byref(out), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_calib_lookup_add")
    return out.value


def msgemm_calib_stream_read(src, nbytes, sink, stream=None):
    rc = load().msgemm_calib_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream))
    if rc != OK:
        raise MsgemmError(rc, "msgemm_calib_stream_read")


def msgemm_calib_stream_read_shape(src, nbytes, sink, waves_per_workgroup, workgroups_per_cu, depth, non_temporal,
                                   stream=None, check=True):
    rc = load().msgemm_calib_stream_read_shape(_ptr(src), int(nbytes), _ptr(sink), int(waves_per_workgroup),
                                               int(workgroups_per_cu), int(depth), int(non_temporal), _stream(stream))
    if check and rc != OK:
        raise MsgemmError(rc, "msgemm_calib_stream_read_shape")
    return rc


def msgemm_plan_set_codebook(plan, values16, check: bool = True):
    """values16: 16 floats (value of each bit pattern) or None for the paper's two's complement."""
    arr = None
    if values16 is not None:
        vals = [float(v) for v in values16]
        if len(vals) != 16:
            raise ValueError("a codebook has 16 values")
        arr = (ctypes.c_float * 16)(*vals)
    rc = load().msgemm_plan_set_codebook(ctypes.c_void_p(plan), arr)
    if check and rc != OK:
        raise MsgemmError(rc, "msgemm_plan_set_codebook")
    return rc


def msgemm_destroy(plan) -> None:
    if plan:
        load().msgemm_destroy(ctypes.c_void_p(plan))
