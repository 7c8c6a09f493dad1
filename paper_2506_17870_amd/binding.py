"""ctypes binding of libnq.so -- argument marshalling only.

Every function has the name and the argument order of its C entry point in
include/nq.h; tensors are PyTorch tensors used purely as owners of device (or pinned
host) memory, streams are `torch.cuda.Stream` objects or raw handles.  No step of the
path is computed here.  Importing this module fails if the library has not been built:
there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnq.so")

NQ_OK, NQ_ERR_INVALID_ARG, NQ_ERR_UNSUPPORTED, NQ_ERR_SHAPE, NQ_ERR_ALIGN, NQ_ERR_NOT_RESIDENT, \
    NQ_ERR_RANGE, NQ_ERR_HIP = range(8)
NQ_LOW_UNSIGNED_L, NQ_LOW_SIGNED_L1 = 0, 1
NQ_LAYOUT_DENSE, NQ_LAYOUT_PAPER_U64 = 0, 1
NQ_MAX_K = 65536
NQ_TUNE_KERNEL, NQ_TUNE_BIG_TM, NQ_TUNE_GC_UNITS, NQ_TUNE_STAT_ROWS = 0, 1, 2, 3

EXPORTS = ["nq_version", "nq_status_string", "nq_packed_bytes", "nq_quantize", "nq_tensor_scale", "nq_quantize_tensor", "nq_quantize_decompose_pack",
           "nq_decompose", "nq_pack", "nq_decompose_pack", "nq_decompose_pack_batch",
           "nq_unpack", "nq_weight_init", "nq_weight_destroy", "nq_page_out_low", "nq_page_in_low",
           "nq_weight_init_group", "nq_page_out_low_batch", "nq_page_in_low_batch",
           "nq_gemm_full", "nq_gemm_part", "nq_gemm_batch_workspace_bytes", "nq_gemm_batch", "nq_gemm_batch_static", "nq_conv_full", "nq_conv_part", "nq_gconv_full", "nq_gconv_part",
           "nq_set_tuning", "nq_profile_next_launch", "nq_profile_last_kernel", "nq_event_create", "nq_event_destroy",
           "nq_event_elapsed_ms", "nq_maxpool_i8", "nq_avgpool_i8"]


class nq_cfg(ctypes.Structure):
    _fields_ = [("n_bits", ctypes.c_int32), ("l_bits", ctypes.c_int32), ("low_format", ctypes.c_int32),
                ("layout", ctypes.c_int32)]


class nq_weight(ctypes.Structure):
    _fields_ = [("cfg", nq_cfg), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("d_high", ctypes.c_void_p), ("high_bytes", ctypes.c_uint64),
                ("d_low", ctypes.c_void_p), ("low_bytes", ctypes.c_uint64),
                ("h_low", ctypes.c_void_p), ("d_scale", ctypes.c_void_p),
                ("low_resident", ctypes.c_int32), ("low_event_armed", ctypes.c_int32),
                ("low_event", ctypes.c_void_p), ("free_event", ctypes.c_void_p),
                ("free_event_armed", ctypes.c_int32), ("events_borrowed", ctypes.c_int32),
                ("group_head", ctypes.c_int32), ("reserved_", ctypes.c_int32)]


class nq_pack_job(ctypes.Structure):
    _fields_ = [("d_w_int", ctypes.c_void_p), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("d_packed_high", ctypes.c_void_p), ("d_packed_low", ctypes.c_void_p)]


class nq_epilogue(ctypes.Structure):
    _fields_ = [("act_scale", ctypes.c_float), ("d_bias", ctypes.c_void_p), ("d_residual", ctypes.c_void_p),
                ("residual_scale", ctypes.c_float), ("relu", ctypes.c_int32), ("out_int8", ctypes.c_int32),
                ("inv_out_scale", ctypes.c_float), ("d_acc_dump", ctypes.c_void_p)]


class nq_gemm_job(ctypes.Structure):
    _fields_ = [("d_x", ctypes.c_void_p), ("M", ctypes.c_int64), ("w", ctypes.POINTER(nq_weight)),
                ("epi", nq_epilogue), ("d_y", ctypes.c_void_p)]


NQ_GEMM_BATCH_STATIC_MAX = 2048


class nq_conv_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64), ("Cin", ctypes.c_int64),
                ("Cout", ctypes.c_int64), ("KH", ctypes.c_int32), ("KW", ctypes.c_int32),
                ("stride", ctypes.c_int32), ("pad", ctypes.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_17870_amd.build` "
                      "(there is no CPU or PyTorch fallback for the HIP path)")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i64, _int, _f = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
_cfgp, _wp, _ep, _sp = ctypes.POINTER(nq_cfg), ctypes.POINTER(nq_weight), ctypes.POINTER(nq_epilogue), \
    ctypes.POINTER(nq_conv_shape)
_SIGS = {
    "nq_version": (ctypes.c_int, []),
    "nq_status_string": (ctypes.c_char_p, [_int]),
    "nq_packed_bytes": (ctypes.c_size_t, [_i64, _i64, _int, _int]),
    "nq_quantize": (_int, [_vp, _i64, _i64, _int, _vp, _vp, _vp]),
    "nq_tensor_scale": (_int, [_vp, _i64, _int, _vp, _vp]),
    "nq_quantize_tensor": (_int, [_vp, _i64, _int, _vp, _vp, _vp]),
    "nq_quantize_decompose_pack": (_int, [_vp, _i64, _i64, _cfgp, _vp, _vp, _vp, _vp]),
    "nq_decompose": (_int, [_vp, _i64, _i64, _cfgp, _vp, _vp, _vp]),
    "nq_pack": (_int, [_vp, _vp, _i64, _i64, _cfgp, _vp, _vp, _vp]),
    "nq_decompose_pack": (_int, [_vp, _i64, _i64, _cfgp, _vp, _vp, _vp]),
    "nq_decompose_pack_batch": (_int, [ctypes.POINTER(nq_pack_job), _i64, _cfgp, _vp]),
    "nq_unpack": (_int, [_vp, _vp, _i64, _i64, _cfgp, _vp, _vp, _vp]),
    "nq_weight_init": (_int, [_wp]),
    "nq_weight_destroy": (_int, [_wp]),
    "nq_page_out_low": (_int, [_wp, _vp]),
    "nq_page_in_low": (_int, [_wp, _vp]),
    "nq_weight_init_group": (_int, [ctypes.POINTER(_wp), _i64]),
    "nq_page_out_low_batch": (_int, [ctypes.POINTER(_wp), _i64, _vp]),
    "nq_page_in_low_batch": (_int, [ctypes.POINTER(_wp), _i64, _vp]),
    "nq_gemm_full": (_int, [_vp, _i64, _wp, _ep, _vp, _vp]),
    "nq_gemm_part": (_int, [_vp, _i64, _wp, _ep, _vp, _vp]),
    "nq_gemm_batch_workspace_bytes": (ctypes.c_size_t, [_i64]),
    "nq_gemm_batch": (_int, [ctypes.POINTER(nq_gemm_job), _i64, _int, _vp, ctypes.c_size_t, _vp]),
    "nq_gemm_batch_static": (_int, [ctypes.POINTER(nq_gemm_job), _i64, _int, _vp]),
    "nq_conv_full": (_int, [_vp, _sp, _wp, _ep, _vp, _vp]),
    "nq_conv_part": (_int, [_vp, _sp, _wp, _ep, _vp, _vp]),
    "nq_gconv_full": (_int, [_vp, _sp, _int, _wp, _ep, _vp, _vp]),
    "nq_gconv_part": (_int, [_vp, _sp, _int, _wp, _ep, _vp, _vp]),
    "nq_set_tuning": (_int, [_int, _int]),
    "nq_profile_next_launch": (_int, [_vp, _vp]),
    "nq_profile_last_kernel": (_int, [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "nq_event_create": (_int, [ctypes.POINTER(ctypes.c_void_p)]),
    "nq_event_destroy": (_int, [_vp]),
    "nq_event_elapsed_ms": (_int, [_vp, _vp, ctypes.POINTER(ctypes.c_float)]),
    "nq_maxpool_i8": (_int, [_vp, _i64, _i64, _i64, _i64, _int, _int, _int, _vp, _vp]),
    "nq_avgpool_i8": (_int, [_vp, _i64, _i64, _i64, _f, _f, _vp, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


class NQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.nq_status_string(status).decode()} (status {status})")


def _check(status: int, where: str):
    if status != NQ_OK:
        raise NQError(status, where)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors handed to libnq must be contiguous"
    return t.data_ptr()


def _stream(s):
    if s is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(s, int):
        return s
    return s.cuda_stream


def make_cfg(n_bits=8, l_bits=2, low_format=NQ_LOW_UNSIGNED_L, layout=NQ_LAYOUT_DENSE) -> nq_cfg:
    return nq_cfg(n_bits, l_bits, low_format, layout)


def nq_version() -> int:
    return _lib.nq_version()


def nq_status_string(status: int) -> str:
    return _lib.nq_status_string(status).decode()


def nq_packed_bytes(N, K, field_bits, layout=NQ_LAYOUT_DENSE) -> int:
    return int(_lib.nq_packed_bytes(N, K, field_bits, layout))


def nq_decompose(d_w_int, N, K, cfg, d_high, d_low, stream=None):
    _check(_lib.nq_decompose(_ptr(d_w_int), N, K, ctypes.byref(cfg), _ptr(d_high), _ptr(d_low), _stream(stream)),
           "nq_decompose")


def nq_pack(d_high, d_low, N, K, cfg, d_packed_high, d_packed_low, stream=None):
    _check(_lib.nq_pack(_ptr(d_high), _ptr(d_low), N, K, ctypes.byref(cfg), _ptr(d_packed_high),
                        _ptr(d_packed_low), _stream(stream)), "nq_pack")


def nq_quantize(d_w, N, K, n_bits, d_w_int, d_scale, stream=None):
    _check(_lib.nq_quantize(_ptr(d_w), N, K, n_bits, _ptr(d_w_int), _ptr(d_scale), _stream(stream)), "nq_quantize")


def nq_tensor_scale(d_x, count, n_bits, d_scale, stream=None):
    _check(_lib.nq_tensor_scale(_ptr(d_x), count, n_bits, _ptr(d_scale), _stream(stream)), "nq_tensor_scale")


def nq_quantize_tensor(d_x, count, n_bits, d_codes, d_scale, stream=None):
    _check(_lib.nq_quantize_tensor(_ptr(d_x), count, n_bits, _ptr(d_codes), _ptr(d_scale), _stream(stream)),
           "nq_quantize_tensor")


def nq_quantize_decompose_pack(d_w, N, K, cfg, d_scale, d_packed_high, d_packed_low, stream=None):
    _check(_lib.nq_quantize_decompose_pack(_ptr(d_w), N, K, ctypes.byref(cfg), _ptr(d_scale), _ptr(d_packed_high),
                                           _ptr(d_packed_low), _stream(stream)), "nq_quantize_decompose_pack")


def nq_decompose_pack(d_w_int, N, K, cfg, d_packed_high, d_packed_low, stream=None):
    _check(_lib.nq_decompose_pack(_ptr(d_w_int), N, K, ctypes.byref(cfg), _ptr(d_packed_high),
                                  _ptr(d_packed_low), _stream(stream)), "nq_decompose_pack")


def nq_decompose_pack_batch(jobs, cfg, stream=None):
    """jobs: sequence of (d_w_int, N, K, d_packed_high, d_packed_low)."""
    arr = (nq_pack_job * max(len(jobs), 1))()
    for i, (w, n, k, ph, pl) in enumerate(jobs):
        arr[i] = nq_pack_job(_ptr(w), n, k, _ptr(ph), _ptr(pl))
    _check(_lib.nq_decompose_pack_batch(arr, len(jobs), ctypes.byref(cfg), _stream(stream)), "nq_decompose_pack_batch")


def nq_unpack(d_packed_high, d_packed_low, N, K, cfg, d_high, d_low, stream=None):
    _check(_lib.nq_unpack(_ptr(d_packed_high), _ptr(d_packed_low), N, K, ctypes.byref(cfg), _ptr(d_high),
                          _ptr(d_low), _stream(stream)), "nq_unpack")


def nq_weight_init(w: nq_weight):
    _check(_lib.nq_weight_init(ctypes.byref(w)), "nq_weight_init")


def nq_weight_destroy(w: nq_weight):
    _check(_lib.nq_weight_destroy(ctypes.byref(w)), "nq_weight_destroy")


def nq_page_out_low(w: nq_weight, stream=None):
    _check(_lib.nq_page_out_low(ctypes.byref(w), _stream(stream)), "nq_page_out_low")


def nq_page_in_low(w: nq_weight, copy_stream=None):
    _check(_lib.nq_page_in_low(ctypes.byref(w), _stream(copy_stream)), "nq_page_in_low")


def _wlist(ws):
    arr = (_wp * len(ws))(*[ctypes.pointer(w) for w in ws])
    return arr


def nq_weight_init_group(ws):
    _check(_lib.nq_weight_init_group(_wlist(ws), len(ws)), "nq_weight_init_group")


def nq_page_out_low_batch(ws, stream=None):
    _check(_lib.nq_page_out_low_batch(_wlist(ws), len(ws), _stream(stream)), "nq_page_out_low_batch")


def nq_page_in_low_batch(ws, copy_stream=None):
    _check(_lib.nq_page_in_low_batch(_wlist(ws), len(ws), _stream(copy_stream)), "nq_page_in_low_batch")


def make_epilogue(act_scale=1.0, d_bias=None, d_residual=None, residual_scale=0.0, relu=False, out_int8=False,
                  inv_out_scale=1.0, d_acc_dump=None) -> nq_epilogue:
    return nq_epilogue(act_scale, _ptr(d_bias), _ptr(d_residual), residual_scale, int(relu), int(out_int8),
                       inv_out_scale, _ptr(d_acc_dump))


def nq_gemm_full(d_x, M, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_gemm_full(_ptr(d_x), M, ctypes.byref(w), ctypes.byref(epi), _ptr(d_y), _stream(stream)),
           "nq_gemm_full")


def nq_gemm_part(d_x, M, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_gemm_part(_ptr(d_x), M, ctypes.byref(w), ctypes.byref(epi), _ptr(d_y), _stream(stream)),
           "nq_gemm_part")


def _jobs(jobs):
    """jobs: sequence of (d_x, M, nq_weight, nq_epilogue, d_y)."""
    arr = (nq_gemm_job * max(len(jobs), 1))()
    for i, (x, M, w, epi, y) in enumerate(jobs):
        arr[i] = nq_gemm_job(_ptr(x), M, ctypes.pointer(w), epi, _ptr(y))
    return arr


def nq_gemm_batch_workspace_bytes(count) -> int:
    return int(_lib.nq_gemm_batch_workspace_bytes(count))


def nq_gemm_batch(jobs, full_bit, d_workspace, stream=None):
    _check(_lib.nq_gemm_batch(_jobs(jobs), len(jobs), int(full_bit), _ptr(d_workspace),
                              d_workspace.numel() * d_workspace.element_size() if d_workspace is not None else 0,
                              _stream(stream)), "nq_gemm_batch")


def nq_gemm_batch_static(jobs, full_bit, stream=None):
    _check(_lib.nq_gemm_batch_static(_jobs(jobs), len(jobs), int(full_bit), _stream(stream)), "nq_gemm_batch_static")


def nq_conv_full(d_x, shape: nq_conv_shape, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_conv_full(_ptr(d_x), ctypes.byref(shape), ctypes.byref(w), ctypes.byref(epi), _ptr(d_y),
                             _stream(stream)), "nq_conv_full")


def nq_conv_part(d_x, shape: nq_conv_shape, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_conv_part(_ptr(d_x), ctypes.byref(shape), ctypes.byref(w), ctypes.byref(epi), _ptr(d_y),
                             _stream(stream)), "nq_conv_part")


def nq_gconv_full(d_x, shape: nq_conv_shape, groups: int, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_gconv_full(_ptr(d_x), ctypes.byref(shape), groups, ctypes.byref(w), ctypes.byref(epi), _ptr(d_y),
                              _stream(stream)), "nq_gconv_full")


def nq_gconv_part(d_x, shape: nq_conv_shape, groups: int, w: nq_weight, epi: nq_epilogue, d_y, stream=None):
    _check(_lib.nq_gconv_part(_ptr(d_x), ctypes.byref(shape), groups, ctypes.byref(w), ctypes.byref(epi), _ptr(d_y),
                              _stream(stream)), "nq_gconv_part")


def nq_set_tuning(key: int, value: int):
    _check(_lib.nq_set_tuning(key, value), "nq_set_tuning")


def nq_profile_next_launch(start_event, stop_event):
    """Raw hipEvent_t handles (integers) or None."""
    _check(_lib.nq_profile_next_launch(start_event, stop_event), "nq_profile_next_launch")


def nq_profile_last_kernel():
    """(family, variant) of the last GEMM / convolution launch of this thread."""
    fam, var = ctypes.c_int(), ctypes.c_int()
    _check(_lib.nq_profile_last_kernel(ctypes.byref(fam), ctypes.byref(var)), "nq_profile_last_kernel")
    return fam.value, var.value


def nq_event_create() -> int:
    ev = ctypes.c_void_p()
    _check(_lib.nq_event_create(ctypes.byref(ev)), "nq_event_create")
    return ev.value


def nq_event_destroy(event):
    _check(_lib.nq_event_destroy(event), "nq_event_destroy")


def nq_event_elapsed_ms(start_event, stop_event) -> float:
    ms = ctypes.c_float()
    _check(_lib.nq_event_elapsed_ms(start_event, stop_event, ctypes.byref(ms)), "nq_event_elapsed_ms")
    return ms.value


def nq_maxpool_i8(d_x, B, H, W, C, ksize, stride, pad, d_y, stream=None):
    _check(_lib.nq_maxpool_i8(_ptr(d_x), B, H, W, C, ksize, stride, pad, _ptr(d_y), _stream(stream)),
           "nq_maxpool_i8")


def nq_avgpool_i8(d_x, B, HW, C, in_scale, inv_out_scale, d_y, stream=None):
    _check(_lib.nq_avgpool_i8(_ptr(d_x), B, HW, C, in_scale, inv_out_scale, _ptr(d_y), _stream(stream)),
           "nq_avgpool_i8")


class NestedWeight:
    """Owner of the buffers one nq_weight descriptor points to (memory plumbing only).

    Holds the packed higher-bit page and the device slot of the lower-bit page as torch
    tensors, the pinned host master copy of the lower-bit page and the per-channel scales,
    and fills the descriptor.  `from_int8` runs nq_decompose_pack on the device and copies
    the lower-bit page once to the pinned host buffer (the "storage" it is paged in from).
    """

    def __init__(self, N, K, cfg: nq_cfg, device="cuda", low=None, low_host=None, init=True):
        """low / low_host: optional uint8 views (device / pinned host) to use for the lower-bit page, e.g.
        slices of two arenas so that a whole model can be paged in with few copies."""
        h = cfg.n_bits - cfg.l_bits
        self.cfg, self.N, self.K = cfg, N, K
        low_field = cfg.l_bits + (1 if cfg.low_format == NQ_LOW_SIGNED_L1 else 0)   # compensated part: l + 1 bits
        low_bytes = max(nq_packed_bytes(N, K, low_field, cfg.layout), 16)
        self.high = torch.empty(max(nq_packed_bytes(N, K, h, cfg.layout), 16), dtype=torch.uint8, device=device)
        self.low = low if low is not None else torch.empty(low_bytes, dtype=torch.uint8, device=device)
        self.low_host = low_host if low_host is not None else torch.empty(low_bytes, dtype=torch.uint8,
                                                                          pin_memory=True)
        assert self.low.numel() == low_bytes and self.low_host.numel() == low_bytes
        self.scale = torch.ones(max(N, 1), dtype=torch.float32, device=device)
        self.desc = nq_weight(cfg, N, K, self.high.data_ptr(), self.high.numel(), self.low.data_ptr(),
                              self.low.numel(), self.low_host.data_ptr(), self.scale.data_ptr(), 0, 0, None, None, 0, 0, 0, 0)
        if init:
            nq_weight_init(self.desc)

    def fill_from_int8(self, d_w_int, d_scale, stream=None):
        """nq_decompose_pack on the device, then the master copy of the lower-bit page to the host."""
        nq_decompose_pack(d_w_int, self.N, self.K, self.cfg, self.high, self.low, stream)
        self.scale.copy_(d_scale)
        self.low_host.copy_(self.low)
        torch.cuda.synchronize()
        self.desc.low_resident = 1
        return self

    @classmethod
    def from_int8(cls, d_w_int, d_scale, cfg: nq_cfg, stream=None):
        N, K = d_w_int.shape
        return cls(N, K, cfg, device=d_w_int.device).fill_from_int8(d_w_int, d_scale, stream)

    @classmethod
    def from_float(cls, d_w, cfg: nq_cfg, stream=None):
        """nq_quantize_decompose_pack of fp32 weights [N, K] on the device (dense layout), then the master
        copy of the lower-bit page to the host."""
        N, K = d_w.shape
        self = cls(N, K, cfg, device=d_w.device)
        nq_quantize_decompose_pack(d_w, N, K, cfg, self.scale, self.high, self.low, stream)
        self.low_host.copy_(self.low)
        torch.cuda.synchronize()
        self.desc.low_resident = 1
        return self

    def fill_from_parts(self, d_high, d_low, d_scale, stream=None):
        """nq_pack of separately supplied w_high / w_low (e.g. a w_high rounded by the caller's own rule with
        its signed residual, cfg.low_format = NQ_LOW_SIGNED_L1), then the master copy of the lower-bit page."""
        nq_pack(d_high, d_low, self.N, self.K, self.cfg, self.high, self.low, stream)
        self.scale.copy_(d_scale)
        self.low_host.copy_(self.low)
        torch.cuda.synchronize()
        self.desc.low_resident = 1
        return self

    def fill_from_pages(self, high_page, low_page, d_scale):
        """Takes pages that are packed already in cfg.layout (uint8 tensors or arrays of nq_packed_bytes each),
        e.g. a model file that stores w_high and w_low as the paper's 64-bit words (Sec. 3.3.4)."""
        for dst, src in ((self.high, high_page), (self.low, low_page)):
            src = torch.as_tensor(src).reshape(-1).view(torch.uint8)
            assert src.numel() <= dst.numel()
            dst.zero_()
            dst[:src.numel()].copy_(src)
        self.scale.copy_(torch.as_tensor(d_scale))
        self.low_host.copy_(self.low)
        torch.cuda.synchronize()
        self.desc.low_resident = 1
        return self

    def close(self):
        if self.desc.low_event:
            nq_weight_destroy(self.desc)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
