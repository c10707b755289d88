"""ctypes binding of include/mnn_conv.h.  Argument marshalling only.

PyTorch is used for device memory and streams: tensors are passed as raw
``data_ptr()`` addresses and the current stream as its ``hipStream_t`` handle.
There is no CPU fallback: if libmnnconv.so is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int32, c_size_t, c_void_p
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libmnnconv.so")

SCHEME_AUTO, SCHEME_DIRECT, SCHEME_WINOGRAD, SCHEME_GEMM1X1 = 0, 1, 2, 3
GEMM_FP32, GEMM_BF16, GEMM_BF16X3 = 0, 1, 2
STAGE_FILTER, STAGE_INPUT, STAGE_GEMM, STAGE_OUTPUT, STAGE_COUNT = 0, 1, 2, 3, 4
BUF_U, BUF_V, BUF_M = 0, 1, 2
WINO_UNFUSED, WINO_FUSED_OUT_32, WINO_FUSED_OUT_64 = 0, 1, 2
_KIND_NAMES = {SCHEME_AUTO: "auto", SCHEME_DIRECT: "direct", SCHEME_WINOGRAD: "winograd", SCHEME_GEMM1X1: "gemm1x1"}


class MnnError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"mnn_conv error {code}: {msg}")
        self.code = code


class _Shape(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("n", "c_in", "h", "w", "c_out", "kh", "kw")]


class _Geom(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


class _Scheme(ctypes.Structure):
    _fields_ = [("kind", c_int32), ("tile_n", c_int32), ("prec", c_int32), ("variant", c_int32), ("est_ms", c_float)]


class _Options(ctypes.Structure):
    _fields_ = [("force_kind", c_int32), ("force_tile_n", c_int32), ("force_prec", c_int32),
                ("force_variant", c_int32), ("allow_bf16", c_int32), ("alpha_max", c_int32), ("point_scale_f", c_float),
                ("plan_warmup", c_int32), ("plan_iters", c_int32), ("use_cache", c_int32), ("prune_ratio", c_float)]


class _DevicePeaks(ctypes.Structure):
    _fields_ = [("mfma_f32_flops", c_double), ("copy_bytes_per_s", c_double)]


class _DeviceModel(ctypes.Structure):
    _fields_ = [("flops", c_double), ("bytes_per_s", c_double), ("t_schedule_ms", c_double)]


class _GemmDesc(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("M", "ncols", "R", "batch", "lda", "L", "variant", "prec")] + \
               [(n, ctypes.c_int64) for n in ("strideA_batch", "strideB_batch", "strideB_img", "strideB_row",
                                              "strideD_batch", "strideD_img", "strideD_row")]


class _Info(ctypes.Structure):
    _fields_ = [(n, c_int32) for n in ("alpha", "tile_n", "tiles_h", "tiles_w", "p", "ldp", "ldk", "kg", "pg", "h_out", "w_out",
                                             "alpha_w", "tile_n_w", "tiled", "pb")]


class _ChainLayer(ctypes.Structure):
    _fields_ = [("shape", _Shape), ("geom", _Geom)]


class _ChainInfo(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("kernels_per_run", c_int32), ("graph_nodes", c_int32), ("reserved", c_int32),
                ("arena_bytes", ctypes.c_uint64), ("unshared_bytes", ctypes.c_uint64),
                ("live_peak_bytes", ctypes.c_uint64), ("weight_bytes", ctypes.c_uint64)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        # build once if nothing is built; a missing toolchain is a hard error
        from .build import build_library
        build_library(verbose=False)
    # torch first: its bundled HIP runtime must be the one libmnnconv.so binds to,
    # otherwise device pointers from torch would belong to a different runtime instance.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp = c_void_p
    L.mnn_conv_options_default.argtypes = [POINTER(_Options)]
    L.mnn_conv_plan.argtypes = [POINTER(_Shape), POINTER(_Geom), POINTER(_Options), vp, POINTER(vp)]
    L.mnn_conv_plan_scheme.argtypes = [vp, POINTER(_Scheme)]
    L.mnn_conv_plan_candidates.argtypes = [vp, POINTER(_Scheme), c_int32, POINTER(c_int32)]
    L.mnn_conv_plan_info.argtypes = [vp, POINTER(_Info)]
    L.mnn_conv_plan_describe.argtypes = [vp, ctypes.c_char_p, c_size_t]
    L.mnn_conv_workspace_bytes.argtypes = [vp]
    L.mnn_conv_workspace_bytes.restype = c_size_t
    L.mnn_conv_run.argtypes = [vp, vp, vp, vp, vp, vp]
    L.mnn_conv_run_timed.argtypes = [vp, vp, vp, vp, vp, vp, c_int32, POINTER(c_float)]
    L.mnn_conv_run_stage.argtypes = [vp, c_int32, vp, vp, vp, vp, vp]
    L.mnn_conv_invalidate_weights.argtypes = [vp]
    L.mnn_conv_set_weights.argtypes = [vp, vp, vp]
    L.mnn_conv_run_static.argtypes = [POINTER(_Shape), POINTER(_Geom), c_int32, vp, vp, vp, vp, vp]
    L.mnn_conv_static_scratch_bytes.argtypes = []
    L.mnn_conv_static_scratch_bytes.restype = c_size_t
    L.mnn_conv_plan_buffer.argtypes = [vp, c_int32, POINTER(vp), POINTER(c_size_t)]
    L.mnn_conv_read_buffer.argtypes = [vp, c_int32, vp, c_size_t, vp]
    L.mnn_conv_plan_destroy.argtypes = [vp]
    L.mnn_conv_plan_destroy.restype = None
    L.mnn_conv_get_transforms.argtypes = [c_int32, c_int32, c_float, vp, vp, vp]
    L.mnn_conv_analytic_cost.argtypes = [c_int32] * 6 + [POINTER(c_double)]
    L.mnn_conv_analytic_tile.argtypes = [c_int32] * 6 + [POINTER(c_int32)]
    L.mnn_conv_enumerate.argtypes = [POINTER(_Shape), POINTER(_Geom), POINTER(_Options), POINTER(_Scheme), c_int32,
                                     POINTER(c_int32)]
    L.mnn_conv_select.argtypes = [POINTER(_Scheme), c_int32, c_int32, POINTER(c_int32)]
    L.mnn_gemm_f32.argtypes = [POINTER(_GemmDesc), vp, vp, vp, vp, vp]
    L.mnn_gemm_variant_count.argtypes = [c_int32]
    L.mnn_gemm_variant_name.argtypes = [c_int32, c_int32]
    L.mnn_gemm_variant_name.restype = c_char_p
    L.mnn_chain_create.argtypes = [POINTER(_ChainLayer), c_int32, POINTER(_Options), vp, POINTER(vp)]
    L.mnn_chain_set_weights.argtypes = [vp, c_int32, vp, vp, vp]
    L.mnn_chain_run.argtypes = [vp, vp, vp, vp]
    L.mnn_chain_capture.argtypes = [vp, vp, vp]
    L.mnn_chain_replay.argtypes = [vp, vp]
    L.mnn_chain_info.argtypes = [vp, POINTER(_ChainInfo)]
    L.mnn_chain_layer_scheme.argtypes = [vp, c_int32, POINTER(_Scheme)]
    L.mnn_chain_layer_describe.argtypes = [vp, c_int32, ctypes.c_char_p, c_size_t]
    L.mnn_chain_read_activation.argtypes = [vp, c_int32, vp, c_size_t, vp]
    L.mnn_chain_destroy.argtypes = [vp]
    L.mnn_chain_destroy.restype = None
    L.mnn_arena_plan.argtypes = [POINTER(ctypes.c_int64), POINTER(c_int32), POINTER(c_int32), c_int32, ctypes.c_int64,
                                 POINTER(ctypes.c_int64), POINTER(ctypes.c_int64)]
    L.mnn_strassen_levels_by_rule.argtypes = [c_int32] * 4
    L.mnn_strassen_create.argtypes = [POINTER(_GemmDesc), c_int32, vp, POINTER(vp)]
    L.mnn_strassen_set_left.argtypes = [vp, vp, vp]
    L.mnn_strassen_run.argtypes = [vp, vp, vp, vp, vp]
    L.mnn_strassen_info.argtypes = [vp, POINTER(c_int32), POINTER(c_int32), POINTER(c_size_t)]
    L.mnn_strassen_destroy.argtypes = [vp]
    L.mnn_strassen_destroy.restype = None
    L.mnn_conv_get_device_model.argtypes = [POINTER(_DeviceModel)]
    L.mnn_conv_set_device_model.argtypes = [POINTER(_DeviceModel)]
    L.mnn_conv_calibrate.argtypes = [vp, POINTER(_DeviceModel)]
    L.mnn_measure_device_peaks.argtypes = [vp, POINTER(_DevicePeaks)]
    L.mnn_conv_predict_ms.argtypes = [POINTER(_Shape), POINTER(_Geom), POINTER(_Scheme), POINTER(c_double)]
    L.mnn_conv_cache_size.argtypes = []
    L.mnn_conv_cache_clear.argtypes = []
    L.mnn_conv_cache_clear.restype = None
    L.mnn_conv_cache_save.argtypes = [c_char_p]
    L.mnn_conv_cache_load.argtypes = [c_char_p]
    L.mnn_last_error.restype = c_char_p
    L.mnn_version.argtypes = []
    return L


lib = _load()


def library_path() -> str:
    return _LIB_PATH


def _check(rc: int):
    if rc != 0:
        raise MnnError(rc, (lib.mnn_last_error() or b"").decode("utf-8", "replace"))


def version() -> int:
    return int(lib.mnn_version())


@dataclass
class Scheme:
    kind: int
    tile_n: int = 0
    prec: int = GEMM_FP32
    variant: int = 0
    est_ms: float = -1.0

    def label(self, k: Optional[int] = None) -> str:
        p = {GEMM_FP32: "", GEMM_BF16: "/bf16", GEMM_BF16X3: "/bf16x3"}.get(self.prec, f"/p{self.prec}")
        if self.kind == SCHEME_WINOGRAD:
            v = {WINO_UNFUSED: "", WINO_FUSED_OUT_32: "+fo32", WINO_FUSED_OUT_64: "+fo64"}.get(self.variant, f"+v{self.variant}")
            return f"F({self.tile_n},{k if k is not None else 'k'}){v}{p}"
        st = f"+strassen{self.variant}" if (self.kind == SCHEME_GEMM1X1 and self.variant > 0) else ""
        return _KIND_NAMES.get(self.kind, str(self.kind)) + st + p

    def _c(self) -> _Scheme:
        return _Scheme(self.kind, self.tile_n, self.prec, self.variant, self.est_ms)

    @staticmethod
    def _from(c: _Scheme) -> "Scheme":
        return Scheme(int(c.kind), int(c.tile_n), int(c.prec), int(c.variant), float(c.est_ms))


@dataclass
class Options:
    force_kind: int = SCHEME_AUTO
    force_tile_n: int = 0
    force_prec: int = GEMM_FP32
    force_variant: int = -1
    allow_bf16: int = 0
    alpha_max: int = 10
    point_scale_f: float = 0.0
    plan_warmup: int = 2
    plan_iters: int = 10
    use_cache: int = 1
    prune_ratio: float = 0.0

    def _c(self) -> _Options:
        return _Options(self.force_kind, self.force_tile_n, self.force_prec, self.force_variant, self.allow_bf16, self.alpha_max,
                        self.point_scale_f, self.plan_warmup, self.plan_iters, self.use_cache, self.prune_ratio)

    @staticmethod
    def defaults() -> "Options":
        c = _Options()
        _check(lib.mnn_conv_options_default(byref(c)))
        return Options(*(getattr(c, f) for f, _ in _Options._fields_))


def _pair(v) -> Tuple[int, int]:
    if isinstance(v, (tuple, list)):
        return int(v[0]), int(v[1])
    return int(v), int(v)


def _shape_geom(n, c_in, h, w, c_out, kh, kw, stride, pad, dil):
    sh, sw = _pair(stride)
    ph, pw = _pair(pad)
    dh, dw = _pair(dil)
    return _Shape(n, c_in, h, w, c_out, kh, kw), _Geom(sh, sw, ph, pw, dh, dw)


def get_transforms(n: int, k: int, f: float = 0.5):
    """(A^T [n, alpha], G [alpha, k], B^T [alpha, alpha]) as float32 arrays from the host generator."""
    a = n + k - 1
    AT = np.zeros((max(n, 1), max(a, 1)), np.float32)
    G = np.zeros((max(a, 1), max(k, 1)), np.float32)
    BT = np.zeros((max(a, 1), max(a, 1)), np.float32)
    _check(lib.mnn_conv_get_transforms(n, k, f, AT.ctypes.data, G.ctypes.data, BT.ctypes.data))
    return AT, G, BT


def analytic_cost(k, i_c, o_c, o_h, o_w, n) -> float:
    out = c_double()
    _check(lib.mnn_conv_analytic_cost(k, i_c, o_c, o_h, o_w, n, byref(out)))
    return float(out.value)


def analytic_tile(k, i_c, o_c, o_h, o_w, alpha_max=10) -> int:
    out = c_int32()
    _check(lib.mnn_conv_analytic_tile(k, i_c, o_c, o_h, o_w, alpha_max, byref(out)))
    return int(out.value)


def enumerate_schemes(n, c_in, h, w, c_out, kh, kw, stride=1, pad=0, dil=1, options: Optional[Options] = None) -> List[Scheme]:
    s, g = _shape_geom(n, c_in, h, w, c_out, kh, kw, stride, pad, dil)
    o = options._c() if options else None
    cnt = c_int32()
    buf = (_Scheme * 64)()
    _check(lib.mnn_conv_enumerate(byref(s), byref(g), byref(o) if o else None, buf, 64, byref(cnt)))
    return [Scheme._from(buf[i]) for i in range(min(64, cnt.value))]


def select_scheme(cands: Sequence[Scheme], k: int) -> int:
    arr = (_Scheme * len(cands))(*[c._c() for c in cands])
    out = c_int32()
    _check(lib.mnn_conv_select(arr, len(cands), k, byref(out)))
    return int(out.value)


def gemm_variants(prec: int = GEMM_FP32) -> List[str]:
    return [lib.mnn_gemm_variant_name(prec, i).decode() for i in range(lib.mnn_gemm_variant_count(prec))]


def gemm_f32(At, B, D, bias=None, *, M, ncols, R, batch=1, lda=None, L=None, variant=0, prec=GEMM_FP32,
             strideA_batch=0, strideB_batch=0, strideB_img=0, strideB_row=None,
             strideD_batch=0, strideD_img=0, strideD_row=None, stream=None):
    """mnn_gemm_f32 on device tensors (only their data_ptr() is used)."""
    L = ncols if L is None else L
    d = _GemmDesc(M, ncols, R, batch, M if lda is None else lda, L, variant, prec, strideA_batch, strideB_batch,
                  strideB_img, L if strideB_row is None else strideB_row, strideD_batch, strideD_img,
                  L if strideD_row is None else strideD_row)
    _check(lib.mnn_gemm_f32(byref(d), At.data_ptr(), B.data_ptr(), bias.data_ptr() if bias is not None else None,
                            D.data_ptr(), _stream_handle(stream)))
    return D


def strassen_levels_by_rule(M: int, R: int, ncols: int, max_levels: int) -> int:
    return int(lib.mnn_strassen_levels_by_rule(M, R, ncols, max_levels))


class StrassenGemm:
    """mnn_strassen_*: D[m][col] = sum_r At[r][m] B[r][col] (+ bias[m]) with `levels` levels of Strassen."""

    def __init__(self, M, ncols, R, levels, *, lda=None, L=None, strideB_img=0, strideB_row=None, strideD_img=0,
                 strideD_row=None, stream=None):
        self._h = c_void_p()
        L = ncols if L is None else L
        d = _GemmDesc(M, ncols, R, 1, M if lda is None else lda, L, 0, GEMM_FP32, 0, 0, strideB_img,
                      L if strideB_row is None else strideB_row, 0, strideD_img, L if strideD_row is None else strideD_row)
        _check(lib.mnn_strassen_create(byref(d), levels, _stream_handle(stream), byref(self._h)))
        self._keep = None

    @property
    def info(self) -> dict:
        lv, la, wb = c_int32(), c_int32(), c_size_t()
        _check(lib.mnn_strassen_info(self._h, byref(lv), byref(la), byref(wb)))
        return {"levels": lv.value, "launches": la.value, "workspace_bytes": int(wb.value)}

    def set_left(self, At, stream=None):
        _check(lib.mnn_strassen_set_left(self._h, At.data_ptr(), _stream_handle(stream)))
        self._keep = At

    def run(self, B, D, bias=None, stream=None):
        _check(lib.mnn_strassen_run(self._h, B.data_ptr(), bias.data_ptr() if bias is not None else None, D.data_ptr(),
                                    _stream_handle(stream)))
        return D

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib.mnn_strassen_destroy(self._h)
            self._h = c_void_p()
        self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def get_device_model() -> dict:
    m = _DeviceModel()
    _check(lib.mnn_conv_get_device_model(byref(m)))
    return {"flops": m.flops, "bytes_per_s": m.bytes_per_s, "t_schedule_ms": m.t_schedule_ms}


def set_device_model(flops: float, bytes_per_s: float, t_schedule_ms: float) -> None:
    m = _DeviceModel(flops, bytes_per_s, t_schedule_ms)
    _check(lib.mnn_conv_set_device_model(byref(m)))


def calibrate(stream=None) -> dict:
    m = _DeviceModel()
    _check(lib.mnn_conv_calibrate(_stream_handle(stream), byref(m)))
    return {"flops": m.flops, "bytes_per_s": m.bytes_per_s, "t_schedule_ms": m.t_schedule_ms}


def measure_device_peaks(stream=None) -> dict:
    m = _DevicePeaks()
    _check(lib.mnn_measure_device_peaks(_stream_handle(stream), byref(m)))
    return {"mfma_f32_flops": m.mfma_f32_flops, "copy_bytes_per_s": m.copy_bytes_per_s}


def predict_ms(n, c_in, h, w, c_out, kh, kw, scheme: "Scheme", stride=1, pad=0, dil=1) -> float:
    s, g = _shape_geom(n, c_in, h, w, c_out, kh, kw, stride, pad, dil)
    c = scheme._c()
    ms = c_double()
    _check(lib.mnn_conv_predict_ms(byref(s), byref(g), byref(c), byref(ms)))
    return float(ms.value)


def cache_size() -> int:
    return int(lib.mnn_conv_cache_size())


def cache_clear() -> None:
    lib.mnn_conv_cache_clear()


def cache_save(path: str) -> None:
    _check(lib.mnn_conv_cache_save(os.fsencode(path)))


def cache_load(path: str) -> None:
    _check(lib.mnn_conv_cache_load(os.fsencode(path)))


def _stream_handle(stream) -> int:
    import torch
    if stream is None:
        if not torch.cuda.is_available():
            return 0          # the library itself reports MNN_E_NO_DEVICE
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


class ConvPlan:
    """mnn_conv_plan / mnn_conv_run for one layer shape."""

    def __init__(self, n, c_in, h, w, c_out, kh, kw, stride=1, pad=0, dil=1,
                 options: Optional[Options] = None, stream=None):
        self._h = c_void_p()
        self.shape = (n, c_in, h, w, c_out, kh, kw)
        s, g = _shape_geom(n, c_in, h, w, c_out, kh, kw, stride, pad, dil)
        o = options._c() if options else None
        _check(lib.mnn_conv_plan(byref(s), byref(g), byref(o) if o else None, _stream_handle(stream), byref(self._h)))
        info = _Info()
        _check(lib.mnn_conv_plan_info(self._h, byref(info)))
        self.info = {f: int(getattr(info, f)) for f, _ in _Info._fields_}
        self.out_shape = (n, c_out, self.info["h_out"], self.info["w_out"])
        self._w_seen = None          # (address, torch version counter) of the weight tensor last handed to the library

    @classmethod
    def for_layer(cls, layer, options: Optional[Options] = None, stream=None) -> "ConvPlan":
        return cls(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                   stride=layer.stride, pad=layer.pad, dil=layer.dil, options=options, stream=stream)

    @property
    def scheme(self) -> Scheme:
        c = _Scheme()
        _check(lib.mnn_conv_plan_scheme(self._h, byref(c)))
        return Scheme._from(c)

    @property
    def candidates(self) -> List[Scheme]:
        cnt = c_int32()
        buf = (_Scheme * 64)()
        _check(lib.mnn_conv_plan_candidates(self._h, buf, 64, byref(cnt)))
        return [Scheme._from(buf[i]) for i in range(min(64, cnt.value))]

    def describe(self) -> str:
        buf = ctypes.create_string_buffer(256)
        _check(lib.mnn_conv_plan_describe(self._h, buf, 256))
        return buf.value.decode()

    @property
    def workspace_bytes(self) -> int:
        return int(lib.mnn_conv_workspace_bytes(self._h))

    def _check_tensors(self, x, w, b, y):
        import torch
        n, c_in, h, wd, c_out, kh, kw = self.shape
        for t, shp, name in ((x, (n, c_in, h, wd), "input"), (w, (c_out, c_in, kh, kw), "weight"),
                             (y, self.out_shape, "output")):
            if tuple(t.shape) != tuple(shp) or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
                raise ValueError(f"{name}: expected contiguous float32 device tensor of shape {shp}, got {tuple(t.shape)} {t.dtype}")
        if b is not None and (tuple(b.shape) != (c_out,) or b.dtype != torch.float32 or not b.is_cuda or not b.is_contiguous()):
            raise ValueError("bias: expected contiguous float32 device tensor of shape (c_out,)")

    def run(self, x, w, b, y=None, stream=None):
        import torch
        if y is None:
            y = torch.empty(self.out_shape, dtype=torch.float32, device=x.device)
        self._check_tensors(x, w, b, y)
        self._note_weight(w)
        _check(lib.mnn_conv_run(self._h, x.data_ptr(), w.data_ptr(), b.data_ptr() if b is not None else None,
                                y.data_ptr(), _stream_handle(stream)))
        return y

    def _note_weight(self, w):
        # The library re-prepares the weights when the pointer changes; it cannot see new values behind the same
        # pointer (an in-place update, or a new tensor the allocator put at the old address).  torch counts in-place
        # writes per tensor, and the tensor object is kept alive here so that its address cannot be reused.
        seen = (w.data_ptr(), w._version, id(w))
        if self._w_seen is not None and self._w_seen[0][0] == seen[0] and self._w_seen[0] != seen:
            _check(lib.mnn_conv_invalidate_weights(self._h))
        self._w_seen = (seen, w)

    def set_weights(self, w, stream=None):
        """mnn_conv_set_weights: prepare the weights now (after new values were written behind the same pointer by
        something torch's version counter does not see, e.g. another library)."""
        import torch
        n, c_in, h, wd, c_out, kh, kw = self.shape
        if tuple(w.shape) != (c_out, c_in, kh, kw) or w.dtype != torch.float32 or not w.is_contiguous() or not w.is_cuda:
            raise ValueError("weight: expected contiguous float32 device tensor of shape (c_out, c_in, kh, kw)")
        _check(lib.mnn_conv_set_weights(self._h, w.data_ptr(), _stream_handle(stream)))
        self._w_seen = ((w.data_ptr(), w._version, id(w)), w)

    def run_stage(self, stage: int, x, w, b, y, stream=None):
        self._check_tensors(x, w, b, y)
        _check(lib.mnn_conv_run_stage(self._h, stage, x.data_ptr(), w.data_ptr(),
                                      b.data_ptr() if b is not None else None, y.data_ptr(), _stream_handle(stream)))

    def run_timed(self, x, w, b, y, iters: int = 10, stream=None) -> List[float]:
        self._check_tensors(x, w, b, y)
        ms = (c_float * STAGE_COUNT)()
        _check(lib.mnn_conv_run_timed(self._h, x.data_ptr(), w.data_ptr(), b.data_ptr() if b is not None else None,
                                      y.data_ptr(), _stream_handle(stream), iters, ms))
        return [float(v) for v in ms]

    def invalidate_weights(self):
        _check(lib.mnn_conv_invalidate_weights(self._h))

    def buffer(self, which: int) -> Tuple[int, int]:
        p, nbytes = c_void_p(), c_size_t()
        _check(lib.mnn_conv_plan_buffer(self._h, which, byref(p), byref(nbytes)))
        return (p.value or 0), int(nbytes.value)

    def buffer_to_numpy(self, which: int, stream=None) -> Optional[np.ndarray]:
        """Copy one of the plan's device buffers to the host as a flat float32 array (test helper)."""
        ptr, nbytes = self.buffer(which)
        if not ptr:
            return None
        out = np.empty(nbytes // 4, dtype=np.float32)
        _check(lib.mnn_conv_read_buffer(self._h, which, out.ctypes.data, nbytes, _stream_handle(stream)))
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib.mnn_conv_plan_destroy(self._h)
            self._h = c_void_p()
        self._w_seen = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def static_scratch_bytes() -> int:
    return int(lib.mnn_conv_static_scratch_bytes())


def conv_run_static(layer, tile_n: int, x, w, b, y, stream=None):
    """mnn_conv_run_static: one convolution with no device allocation (scratch in the library's fixed array)."""
    s, g = _shape_geom(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw, layer.stride, layer.pad, layer.dil)
    _check(lib.mnn_conv_run_static(byref(s), byref(g), tile_n, x.data_ptr(), w.data_ptr(),
                                   b.data_ptr() if b is not None else None, y.data_ptr(), _stream_handle(stream)))
    return y


def arena_plan(sizes: Sequence[int], first: Sequence[int], last: Sequence[int], align: int = 256):
    """mnn_arena_plan: (offsets, total) for buffers alive over operators first[i]..last[i]."""
    n = len(sizes)
    if len(first) != n or len(last) != n:
        raise ValueError("sizes, first and last must have the same length")
    sz = (ctypes.c_int64 * max(n, 1))(*sizes)
    fi = (c_int32 * max(n, 1))(*first)
    la = (c_int32 * max(n, 1))(*last)
    off = (ctypes.c_int64 * max(n, 1))()
    tot = ctypes.c_int64()
    _check(lib.mnn_arena_plan(sz, fi, la, n, align, off, byref(tot)))
    return [int(off[i]) for i in range(n)], int(tot.value)


class ConvChain:
    """mnn_chain_*: a chain of layers planned once, one arena, eager run or HIP-graph replay."""

    def __init__(self, layers, options: Optional[Options] = None, stream=None):
        self._h = c_void_p()
        self.layers = list(layers)
        arr = (_ChainLayer * max(len(self.layers), 1))()
        for i, l in enumerate(self.layers):
            s, g = _shape_geom(l.n, l.c_in, l.h, l.w, l.c_out, l.kh, l.kw, l.stride, l.pad, l.dil)
            arr[i].shape, arr[i].geom = s, g
        o = options._c() if options else None
        _check(lib.mnn_chain_create(arr, len(self.layers), byref(o) if o else None, _stream_handle(stream),
                                    byref(self._h)))
        self._keep = None

    @property
    def info(self) -> dict:
        c = _ChainInfo()
        _check(lib.mnn_chain_info(self._h, byref(c)))
        return {f: int(getattr(c, f)) for f, _ in _ChainInfo._fields_ if f != "reserved"}

    def scheme(self, layer: int) -> Scheme:
        c = _Scheme()
        _check(lib.mnn_chain_layer_scheme(self._h, layer, byref(c)))
        return Scheme._from(c)

    def describe(self, layer: int) -> str:
        buf = ctypes.create_string_buffer(256)
        _check(lib.mnn_chain_layer_describe(self._h, layer, buf, 256))
        return buf.value.decode()

    @staticmethod
    def _dev_f32(t, shape, name):
        import torch
        if tuple(t.shape) != tuple(shape) or t.dtype != torch.float32 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"{name}: expected contiguous float32 device tensor of shape {tuple(shape)}, got {tuple(t.shape)} {t.dtype}")

    def set_weights(self, layer: int, w, b=None, stream=None):
        l = self.layers[layer]
        self._dev_f32(w, (l.c_out, l.c_in, l.kh, l.kw), "weight")
        if b is not None:
            self._dev_f32(b, (l.c_out,), "bias")
        _check(lib.mnn_chain_set_weights(self._h, layer, w.data_ptr(), b.data_ptr() if b is not None else None,
                                         _stream_handle(stream)))

    def _io(self, x, y):
        import torch
        l0, ln = self.layers[0], self.layers[-1]
        self._dev_f32(x, (l0.n, l0.c_in, l0.h, l0.w), "input")
        if y is None:
            y = torch.empty(ln.out_shape, dtype=torch.float32, device=x.device)
        self._dev_f32(y, ln.out_shape, "output")
        return y

    def run(self, x, y=None, stream=None):
        y = self._io(x, y)
        _check(lib.mnn_chain_run(self._h, x.data_ptr(), y.data_ptr(), _stream_handle(stream)))
        return y

    def capture(self, x, y=None):
        y = self._io(x, y)
        _check(lib.mnn_chain_capture(self._h, x.data_ptr(), y.data_ptr()))
        self._keep = (x, y)          # the graph holds these addresses
        return y

    def replay(self, stream=None):
        _check(lib.mnn_chain_replay(self._h, _stream_handle(stream)))

    def activation_to_numpy(self, layer: int, stream=None) -> np.ndarray:
        l = self.layers[layer]
        out = np.empty(l.out_shape, dtype=np.float32)
        _check(lib.mnn_chain_read_activation(self._h, layer, out.ctypes.data, out.nbytes, _stream_handle(stream)))
        return out

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib.mnn_chain_destroy(self._h)
            self._h = c_void_p()
        self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
