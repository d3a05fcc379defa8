"""ctypes binding of libdwm.so: same names as include/dwm.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  There is no CPU fallback: if
libdwm.so has not been built (python -m paper_2002_00552_amd.build), loading fails loudly.
Device pointers are plain integers (e.g. torch.Tensor.data_ptr()); `stream` is a
hipStream_t handle as an integer (e.g. torch.cuda.current_stream().cuda_stream).
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdwm.so")

DWM_OK, DWM_ERR_INVALID_ARG, DWM_ERR_UNSUPPORTED, DWM_ERR_WORKSPACE, DWM_ERR_ALLOC, DWM_ERR_HIP = range(6)


class DwmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        RuntimeError.__init__(self, "%s: %s (status %d)" % (where, dwm_status_string(status), status))


class dwm_plan_info_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad",
                                            "OH", "OW", "TH", "TW")] + [
        ("T", ctypes.c_longlong), ("n_parts", ctypes.c_int), ("n_classes", ctypes.c_int),
        ("n_planes", ctypes.c_int), ("mults_per_tile", ctypes.c_longlong),
        ("direct_flops", ctypes.c_double), ("winograd_flops", ctypes.c_double),
        ("Kpad", ctypes.c_int), ("Tpad", ctypes.c_longlong), ("Vblock", ctypes.c_longlong),
        ("forward_path", ctypes.c_int)]


class dwm_part_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("phase_h", "off_h", "len_h", "phase_w", "off_w", "len_w",
                                            "cls", "slot")]


class dwm_class_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("len_h", "len_w", "n_parts", "L", "Lpad")] + [
        ("u_offset", ctypes.c_longlong), ("v_offset", ctypes.c_longlong)]


class dwm_fused_class_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("wide_h", "wide_w", "n_freq_h", "n_freq_w", "first_row", "rows")] + [
        ("uf_offset", ctypes.c_longlong)]


class dwm_fused_row_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("part", "channel", "real")]


class dwm_bwd_data_info_t(ctypes.Structure):
    _fields_ = [("n_phases", ctypes.c_int), ("n_subconvs", ctypes.c_int), ("mults_per_input_block", ctypes.c_longlong),
                ("direct_flops", ctypes.c_double), ("winograd_flops", ctypes.c_double), ("single_kernel", ctypes.c_int)]


class dwm_bwd_phase_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("phase_h", "phase_w", "taps_h", "taps_w", "first_h", "first_w",
                                            "count_h", "count_w", "has_subconv")]


class dwm_bwd_filter_info_t(ctypes.Structure):
    _fields_ = [("n_planes", ctypes.c_int), ("n_tiles", ctypes.c_int), ("splits", ctypes.c_int),
                ("direct_flops", ctypes.c_double), ("winograd_flops", ctypes.c_double)]


_P = ctypes.c_void_p
_I = ctypes.c_int
_SIGNATURES = {
    "dwm_plan_create": (_I, [ctypes.POINTER(_P)] + [_I] * 9),
    "dwm_plan_destroy": (_I, [_P]),
    "dwm_plan_info": (_I, [_P, ctypes.POINTER(dwm_plan_info_t)]),
    "dwm_plan_part": (_I, [_P, _I, ctypes.POINTER(dwm_part_t)]),
    "dwm_plan_class": (_I, [_P, _I, ctypes.POINTER(dwm_class_t)]),
    "dwm_plan_fused_info": (_I, [_P] + [ctypes.POINTER(_I)] * 3),
    "dwm_plan_fused_class": (_I, [_P, _I, ctypes.POINTER(dwm_fused_class_t)]),
    "dwm_plan_fused_row": (_I, [_P, _I, ctypes.POINTER(dwm_fused_row_t)]),
    "dwm_plan_filter_bytes": (ctypes.c_size_t, [_P]),
    "dwm_plan_workspace_bytes": (ctypes.c_size_t, [_P]),
    "dwm_plan_set_workspace": (_I, [_P, _P, ctypes.c_size_t]),
    "dwm_plan_set_variant": (_I, [_P, ctypes.c_char_p, _I]),
    "dwm_filter_transform": (_I, [_P, _P, _P, _P]),
    "dwm_conv_forward": (_I, [_P, _P, _P, _P, _P]),
    "dwm_static_scratch_bytes": (ctypes.c_size_t, []),
    "dwm_conv_forward_static": (_I, [_P, _P, _P, _P, _P]),
    "dwm_input_transform": (_I, [_P, _P, _P]),
    "dwm_contract_output": (_I, [_P, _P, _P, _P]),
    "dwm_status_string": (ctypes.c_char_p, [_I]),
    "dwm_bwd_data_plan_create": (_I, [ctypes.POINTER(_P)] + [_I] * 9),
    "dwm_bwd_data_plan_destroy": (_I, [_P]),
    "dwm_bwd_data_plan_info": (_I, [_P, ctypes.POINTER(dwm_bwd_data_info_t)]),
    "dwm_bwd_data_plan_phase": (_I, [_P, _I, ctypes.POINTER(dwm_bwd_phase_t)]),
    "dwm_bwd_data_filter_bytes": (ctypes.c_size_t, [_P]),
    "dwm_bwd_data_workspace_bytes": (ctypes.c_size_t, [_P]),
    "dwm_bwd_data_set_workspace": (_I, [_P, _P, ctypes.c_size_t]),
    "dwm_bwd_data_set_variant": (_I, [_P, ctypes.c_char_p, _I]),
    "dwm_bwd_data_filter_transform": (_I, [_P, _P, _P, _P]),
    "dwm_conv_backward_data": (_I, [_P, _P, _P, _P, _P]),
    "dwm_bwd_filter_plan_create": (_I, [ctypes.POINTER(_P)] + [_I] * 9),
    "dwm_bwd_filter_plan_destroy": (_I, [_P]),
    "dwm_bwd_filter_plan_info": (_I, [_P, ctypes.POINTER(dwm_bwd_filter_info_t)]),
    "dwm_bwd_filter_workspace_bytes": (ctypes.c_size_t, [_P]),
    "dwm_bwd_filter_set_workspace": (_I, [_P, _P, ctypes.c_size_t]),
    "dwm_conv_backward_filter": (_I, [_P, _P, _P, _P, _P]),
    "dwm_f16_plan_create": (_I, [ctypes.POINTER(_P)] + [_I] * 9),
    "dwm_f16_plan_destroy": (_I, [_P]),
    "dwm_f16_plan_info": (_I, [_P, ctypes.POINTER(dwm_plan_info_t)]),
    "dwm_f16_filter_bytes": (ctypes.c_size_t, [_P]),
    "dwm_f16_workspace_bytes": (ctypes.c_size_t, [_P]),
    "dwm_f16_set_workspace": (_I, [_P, _P, ctypes.c_size_t]),
    "dwm_f16_set_variant": (_I, [_P, ctypes.c_char_p, _I]),
    "dwm_f16_filter_transform": (_I, [_P, _P, _P, _P]),
    "dwm_f16_conv_forward": (_I, [_P, _P, _P, _P, _P]),
    "dwm_f16_conv_forward_f32out": (_I, [_P, _P, _P, _P, _P]),
    "dwm_f16_input_transform": (_I, [_P, _P, _P]),
    "dwm_f16_contract_output": (_I, [_P, _P, _P, _P]),
    "dwm_bf16_plan_create": (_I, [ctypes.POINTER(_P)] + [_I] * 9),
    "dwm_bf16_plan_destroy": (_I, [_P]),
    "dwm_bf16_plan_info": (_I, [_P, ctypes.POINTER(dwm_plan_info_t)]),
    "dwm_bf16_filter_bytes": (ctypes.c_size_t, [_P]),
    "dwm_bf16_workspace_bytes": (ctypes.c_size_t, [_P]),
    "dwm_bf16_set_workspace": (_I, [_P, _P, ctypes.c_size_t]),
    "dwm_bf16_set_variant": (_I, [_P, ctypes.c_char_p, _I]),
    "dwm_bf16_filter_transform": (_I, [_P, _P, _P, _P]),
    "dwm_bf16_conv_forward": (_I, [_P, _P, _P, _P, _P]),
    "dwm_bf16_conv_forward_f32out": (_I, [_P, _P, _P, _P, _P]),
    "dwm_bf16_input_transform": (_I, [_P, _P, _P]),
    "dwm_bf16_contract_output": (_I, [_P, _P, _P, _P]),
}
EXPORTS = sorted(_SIGNATURES)

_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libdwm.so is not built: run `python -m paper_2002_00552_amd.build` "
                              "(there is no CPU fallback)")
        _lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(_lib, name)
            fn.restype, fn.argtypes = res, args
    return _lib


def _check(status, where):
    if status != DWM_OK:
        raise DwmError(status, where)


def dwm_status_string(status):
    return lib().dwm_status_string(int(status)).decode()


def dwm_plan_create(N, C, H, W, K, R, S, stride, pad):
    h = _P()
    _check(lib().dwm_plan_create(ctypes.byref(h), N, C, H, W, K, R, S, stride, pad), "dwm_plan_create")
    return h


def dwm_plan_destroy(plan):
    _check(lib().dwm_plan_destroy(plan), "dwm_plan_destroy")


def dwm_plan_info(plan):
    info = dwm_plan_info_t()
    _check(lib().dwm_plan_info(plan, ctypes.byref(info)), "dwm_plan_info")
    return info


def dwm_plan_part(plan, i):
    part = dwm_part_t()
    _check(lib().dwm_plan_part(plan, i, ctypes.byref(part)), "dwm_plan_part")
    return part


def dwm_plan_class(plan, i):
    cls = dwm_class_t()
    _check(lib().dwm_plan_class(plan, i, ctypes.byref(cls)), "dwm_plan_class")
    return cls


def dwm_plan_fused_info(plan):
    """(n_classes, n_rows, n_slices) of the single-kernel path's filter copy; zeros where it does not apply."""
    a, b, c = _I(), _I(), _I()
    _check(lib().dwm_plan_fused_info(plan, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "dwm_plan_fused_info")
    return a.value, b.value, c.value


def dwm_plan_fused_class(plan, i):
    cls = dwm_fused_class_t()
    _check(lib().dwm_plan_fused_class(plan, i, ctypes.byref(cls)), "dwm_plan_fused_class")
    return cls


def dwm_plan_fused_row(plan, row):
    out = dwm_fused_row_t()
    _check(lib().dwm_plan_fused_row(plan, row, ctypes.byref(out)), "dwm_plan_fused_row")
    return out


def dwm_plan_filter_bytes(plan):
    return int(lib().dwm_plan_filter_bytes(plan))


def dwm_plan_workspace_bytes(plan):
    return int(lib().dwm_plan_workspace_bytes(plan))


def dwm_plan_set_workspace(plan, ws_dev, nbytes):
    _check(lib().dwm_plan_set_workspace(plan, ws_dev, nbytes), "dwm_plan_set_workspace")


def dwm_plan_set_variant(plan, stage, variant):
    _check(lib().dwm_plan_set_variant(plan, stage.encode(), variant), "dwm_plan_set_variant")


def dwm_filter_transform(plan, w_dev, Ugw_dev, stream=None):
    _check(lib().dwm_filter_transform(plan, w_dev, Ugw_dev, stream), "dwm_filter_transform")


def dwm_conv_forward(plan, x_dev, Ugw_dev, y_dev, stream=None):
    _check(lib().dwm_conv_forward(plan, x_dev, Ugw_dev, y_dev, stream), "dwm_conv_forward")


def dwm_static_scratch_bytes():
    return int(lib().dwm_static_scratch_bytes())


def dwm_conv_forward_static(plan, x_dev, Ugw_dev, y_dev, stream=None):
    _check(lib().dwm_conv_forward_static(plan, x_dev, Ugw_dev, y_dev, stream), "dwm_conv_forward_static")


def dwm_input_transform(plan, x_dev, stream=None):
    _check(lib().dwm_input_transform(plan, x_dev, stream), "dwm_input_transform")


def dwm_contract_output(plan, Ugw_dev, y_dev, stream=None):
    _check(lib().dwm_contract_output(plan, Ugw_dev, y_dev, stream), "dwm_contract_output")


def dwm_bwd_data_plan_create(N, C, H, W, K, R, S, stride, pad):
    h = _P()
    _check(lib().dwm_bwd_data_plan_create(ctypes.byref(h), N, C, H, W, K, R, S, stride, pad), "dwm_bwd_data_plan_create")
    return h


def dwm_bwd_data_plan_destroy(plan):
    _check(lib().dwm_bwd_data_plan_destroy(plan), "dwm_bwd_data_plan_destroy")


def dwm_bwd_data_plan_info(plan):
    info = dwm_bwd_data_info_t()
    _check(lib().dwm_bwd_data_plan_info(plan, ctypes.byref(info)), "dwm_bwd_data_plan_info")
    return info


def dwm_bwd_data_plan_phase(plan, i):
    out = dwm_bwd_phase_t()
    _check(lib().dwm_bwd_data_plan_phase(plan, i, ctypes.byref(out)), "dwm_bwd_data_plan_phase")
    return out


def dwm_bwd_data_filter_bytes(plan):
    return int(lib().dwm_bwd_data_filter_bytes(plan))


def dwm_bwd_data_workspace_bytes(plan):
    return int(lib().dwm_bwd_data_workspace_bytes(plan))


def dwm_bwd_data_set_workspace(plan, ws_dev, nbytes):
    _check(lib().dwm_bwd_data_set_workspace(plan, ws_dev, nbytes), "dwm_bwd_data_set_workspace")


def dwm_bwd_data_set_variant(plan, stage, variant):
    _check(lib().dwm_bwd_data_set_variant(plan, stage.encode(), variant), "dwm_bwd_data_set_variant")


def dwm_bwd_data_filter_transform(plan, w_dev, Ugw_dev, stream=None):
    _check(lib().dwm_bwd_data_filter_transform(plan, w_dev, Ugw_dev, stream), "dwm_bwd_data_filter_transform")


def dwm_conv_backward_data(plan, dy_dev, Ugw_dev, dx_dev, stream=None):
    _check(lib().dwm_conv_backward_data(plan, dy_dev, Ugw_dev, dx_dev, stream), "dwm_conv_backward_data")


def dwm_bwd_filter_plan_create(N, C, H, W, K, R, S, stride, pad):
    h = _P()
    _check(lib().dwm_bwd_filter_plan_create(ctypes.byref(h), N, C, H, W, K, R, S, stride, pad),
           "dwm_bwd_filter_plan_create")
    return h


def dwm_bwd_filter_plan_destroy(plan):
    _check(lib().dwm_bwd_filter_plan_destroy(plan), "dwm_bwd_filter_plan_destroy")


def dwm_bwd_filter_plan_info(plan):
    info = dwm_bwd_filter_info_t()
    _check(lib().dwm_bwd_filter_plan_info(plan, ctypes.byref(info)), "dwm_bwd_filter_plan_info")
    return info


def dwm_bwd_filter_workspace_bytes(plan):
    return int(lib().dwm_bwd_filter_workspace_bytes(plan))


def dwm_bwd_filter_set_workspace(plan, ws_dev, nbytes):
    _check(lib().dwm_bwd_filter_set_workspace(plan, ws_dev, nbytes), "dwm_bwd_filter_set_workspace")


def dwm_conv_backward_filter(plan, x_dev, dy_dev, dw_dev, stream=None):
    _check(lib().dwm_conv_backward_filter(plan, x_dev, dy_dev, dw_dev, stream), "dwm_conv_backward_filter")


def dwm_f16_plan_create(N, C, H, W, K, R, S, stride, pad):
    h = _P()
    _check(lib().dwm_f16_plan_create(ctypes.byref(h), N, C, H, W, K, R, S, stride, pad), "dwm_f16_plan_create")
    return h


def dwm_f16_plan_destroy(plan):
    _check(lib().dwm_f16_plan_destroy(plan), "dwm_f16_plan_destroy")


def dwm_f16_plan_info(plan):
    info = dwm_plan_info_t()
    _check(lib().dwm_f16_plan_info(plan, ctypes.byref(info)), "dwm_f16_plan_info")
    return info


def dwm_f16_filter_bytes(plan):
    return int(lib().dwm_f16_filter_bytes(plan))


def dwm_f16_workspace_bytes(plan):
    return int(lib().dwm_f16_workspace_bytes(plan))


def dwm_f16_set_workspace(plan, ws_dev, nbytes):
    _check(lib().dwm_f16_set_workspace(plan, ws_dev, nbytes), "dwm_f16_set_workspace")


def dwm_f16_set_variant(plan, stage, variant):
    _check(lib().dwm_f16_set_variant(plan, stage.encode(), variant), "dwm_f16_set_variant")


def dwm_f16_filter_transform(plan, w_dev, U_dev, stream=None):
    _check(lib().dwm_f16_filter_transform(plan, w_dev, U_dev, stream), "dwm_f16_filter_transform")


def dwm_f16_conv_forward(plan, x_dev, U_dev, y_dev, stream=None):
    _check(lib().dwm_f16_conv_forward(plan, x_dev, U_dev, y_dev, stream), "dwm_f16_conv_forward")


def dwm_f16_conv_forward_f32out(plan, x_dev, U_dev, y_dev, stream=None):
    _check(lib().dwm_f16_conv_forward_f32out(plan, x_dev, U_dev, y_dev, stream), "dwm_f16_conv_forward_f32out")


def dwm_f16_input_transform(plan, x_dev, stream=None):
    _check(lib().dwm_f16_input_transform(plan, x_dev, stream), "dwm_f16_input_transform")


def dwm_f16_contract_output(plan, U_dev, y_dev, stream=None):
    _check(lib().dwm_f16_contract_output(plan, U_dev, y_dev, stream), "dwm_f16_contract_output")


def dwm_bf16_plan_create(N, C, H, W, K, R, S, stride, pad):
    h = _P()
    _check(lib().dwm_bf16_plan_create(ctypes.byref(h), N, C, H, W, K, R, S, stride, pad), "dwm_bf16_plan_create")
    return h


def dwm_bf16_plan_destroy(plan):
    _check(lib().dwm_bf16_plan_destroy(plan), "dwm_bf16_plan_destroy")


def dwm_bf16_plan_info(plan):
    info = dwm_plan_info_t()
    _check(lib().dwm_bf16_plan_info(plan, ctypes.byref(info)), "dwm_bf16_plan_info")
    return info


def dwm_bf16_filter_bytes(plan):
    return int(lib().dwm_bf16_filter_bytes(plan))


def dwm_bf16_workspace_bytes(plan):
    return int(lib().dwm_bf16_workspace_bytes(plan))


def dwm_bf16_set_workspace(plan, ws_dev, nbytes):
    _check(lib().dwm_bf16_set_workspace(plan, ws_dev, nbytes), "dwm_bf16_set_workspace")


def dwm_bf16_set_variant(plan, stage, variant):
    _check(lib().dwm_bf16_set_variant(plan, stage.encode(), variant), "dwm_bf16_set_variant")


def dwm_bf16_filter_transform(plan, w_dev, U_dev, stream=None):
    _check(lib().dwm_bf16_filter_transform(plan, w_dev, U_dev, stream), "dwm_bf16_filter_transform")


def dwm_bf16_conv_forward(plan, x_dev, U_dev, y_dev, stream=None):
    _check(lib().dwm_bf16_conv_forward(plan, x_dev, U_dev, y_dev, stream), "dwm_bf16_conv_forward")


def dwm_bf16_conv_forward_f32out(plan, x_dev, U_dev, y_dev, stream=None):
    _check(lib().dwm_bf16_conv_forward_f32out(plan, x_dev, U_dev, y_dev, stream), "dwm_bf16_conv_forward_f32out")


def dwm_bf16_input_transform(plan, x_dev, stream=None):
    _check(lib().dwm_bf16_input_transform(plan, x_dev, stream), "dwm_bf16_input_transform")


def dwm_bf16_contract_output(plan, U_dev, y_dev, stream=None):
    _check(lib().dwm_bf16_contract_output(plan, U_dev, y_dev, stream), "dwm_bf16_contract_output")
