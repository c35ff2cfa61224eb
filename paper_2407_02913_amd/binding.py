"""ctypes binding of ``libsfc_hip.so`` (declared in ``include/sfc.h``).

Argument marshalling only: every numeric step runs in the HIP kernels.  PyTorch
is used for device memory and streams.  There is no CPU fallback -- if the
library has not been built (``python __graft_entry__.py``) loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsfc_hip.so")

SFC_OK = 0
STATUS_NAMES = {0: "SFC_OK", 1: "SFC_EINVAL", 2: "SFC_EUNSUPPORTED", 3: "SFC_ENOMEM",
                4: "SFC_ENOTREADY", 5: "SFC_EHIP", 6: "SFC_EWORKSPACE"}
ALG = {"auto": -1, "6x6_p88": 0, "6x6_p100": 1, "7x7_p132": 2, "7x7_p144": 3, "4x4_p46": 4, "4x4_p49": 5,
       "6x6_5x5_p184": 6, "6x6_5x5_p196": 7, "4x4_7x7_p184": 8, "4x4_7x7_p196": 9}
ACT_GRANULARITY = {"tensor": 0, "point": 1}
FILTER_GRANULARITY = {"channel": 0, "point": 1, "channel_point": 2}
ALG_NAME = {v: k for k, v in ALG.items()}
KERNEL_SIZE = {name: 7 if name.startswith("4x4_7x7") else 5 if "5x5" in name else 3
               for name in ALG}  # filter edge R
MODE = {"exact": 0, "requant": 1}
OUT = {"f32": 0, "i32": 1, "i8": 2}
PATH = {"auto": -1, "staged": 0, "fused": 1, "single": 2}
PATH_NAME = {v: k for k, v in PATH.items()}
FLAG_EXACT_WIDE = 1
#: what alg="auto" resolves to for 3x3 filters in requantized mode, and the widest layer
#: path="auto" runs in one kernel (mirrors of the library's rule, for tests and reports)
AUTO_ALG_3X3 = "4x4_p46"
SINGLE_MAX_CIN = 128
STATIC_WORKSPACE_BYTES = 32 << 20  # SFC_STATIC_WORKSPACE_BYTES
STAGE_INPUT, STAGE_PRODUCT, STAGE_OUTPUT, STAGE_ALL = 1, 2, 4, 7
#: every symbol include/sfc.h declares
EXPORTS = (
    "sfc_plan", "sfc_plan_destroy", "sfc_plan_choice", "sfc_plan_sizes", "sfc_set_point_scales",
    "sfc_set_output_scale",
    "sfc_group_scales",
    "sfc_calibrate_act_scales", "sfc_calibrate_filter_scales", "sfc_transform_filter",
    "sfc_conv2d_nchw", "sfc_conv2d_nchw_static", "sfc_conv2d_stages", "sfc_tap_info", "sfc_stream_copy", "sfc_status_string",
)


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("N", "Cin", "Cout", "H", "W", "alg", "mode", "out", "path", "per_channel_wscale",
                 "transform_bits", "flags")]


class SfcError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _lib.sfc_status_string(code).decode() if _lib is not None else "?"
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)} ({msg})")


_lib = None


def load(force: bool = False):
    """Load the shared library; raises if it is missing (there is no fallback)."""
    global _lib
    if _lib is not None and not force:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python __graft_entry__.py` "
            "(hipcc --offload-arch=gfx950); this package has no CPU fallback")
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    lib.sfc_plan.argtypes = [C.POINTER(ConvDesc), C.POINTER(vp)]
    lib.sfc_plan.restype = i32
    lib.sfc_plan_destroy.argtypes = [vp]
    lib.sfc_plan_destroy.restype = None
    lib.sfc_plan_choice.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
    lib.sfc_plan_choice.restype = i32
    lib.sfc_plan_sizes.argtypes = [vp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t),
                                   C.POINTER(i32), C.POINTER(C.c_int64)]
    lib.sfc_plan_sizes.restype = i32
    lib.sfc_set_point_scales.argtypes = [vp, C.POINTER(f32), C.POINTER(f32)]
    lib.sfc_set_point_scales.restype = i32
    lib.sfc_group_scales.argtypes = [vp, i32, i32, C.POINTER(f32), C.POINTER(f32)]
    lib.sfc_group_scales.restype = i32
    lib.sfc_set_output_scale.argtypes = [vp, f32]
    lib.sfc_set_output_scale.restype = i32
    lib.sfc_calibrate_act_scales.argtypes = [vp, vp, i32, vp, C.c_size_t, vp, C.POINTER(f32)]
    lib.sfc_calibrate_act_scales.restype = i32
    lib.sfc_calibrate_filter_scales.argtypes = [vp, vp, vp, C.c_size_t, vp, C.POINTER(f32)]
    lib.sfc_calibrate_filter_scales.restype = i32
    lib.sfc_transform_filter.argtypes = [vp, vp, C.POINTER(f32), vp, C.c_size_t, vp]
    lib.sfc_transform_filter.restype = i32
    lib.sfc_conv2d_nchw.argtypes = [vp, vp, f32, vp, vp, C.c_size_t, vp]
    lib.sfc_conv2d_nchw.restype = i32
    lib.sfc_conv2d_nchw_static.argtypes = [vp, vp, f32, vp, vp]
    lib.sfc_conv2d_nchw_static.restype = i32
    lib.sfc_conv2d_stages.argtypes = [vp, vp, f32, vp, vp, C.c_size_t, vp, i32]
    lib.sfc_conv2d_stages.restype = i32
    lib.sfc_tap_info.argtypes = [vp, vp, i32, C.POINTER(vp), C.POINTER(i32),
                                 C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.sfc_tap_info.restype = i32
    lib.sfc_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
    lib.sfc_stream_copy.restype = i32
    lib.sfc_status_string.argtypes = [i32]
    lib.sfc_status_string.restype = C.c_char_p
    _lib = lib
    return lib


def _check(code, where):
    if code != SFC_OK:
        raise SfcError(code, where)


def _f32_ptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _nbytes(t) -> int:
    return int(t.numel() * t.element_size())


def _stream_ptr(stream):
    import torch

    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


class Plan:
    """Owns one sfc_plan_t.  Tensors passed in are torch CUDA tensors."""

    def __init__(self, N, Cin, Cout, H, W, alg="6x6_p88", mode="requant", out="f32",
                 path="staged", per_channel_wscale=True, transform_bits=0, flags=0):
        lib = load()
        self.desc = ConvDesc(N, Cin, Cout, H, W, ALG[alg], MODE[mode], OUT[out], PATH[path],
                             1 if per_channel_wscale else 0, int(transform_bits), int(flags))
        self._h = C.c_void_p()
        _check(lib.sfc_plan(C.byref(self.desc), C.byref(self._h)), "sfc_plan")
        a, pth = C.c_int32(), C.c_int32()
        _check(lib.sfc_plan_choice(self._h, C.byref(a), C.byref(pth)), "sfc_plan_choice")
        #: what the plan runs ("auto" resolved by the library)
        self.alg, self.path = ALG_NAME[a.value], PATH_NAME[pth.value]
        fb, wb, p, t = C.c_size_t(), C.c_size_t(), C.c_int32(), C.c_int64()
        _check(lib.sfc_plan_sizes(self._h, C.byref(fb), C.byref(wb), C.byref(p), C.byref(t)),
               "sfc_plan_sizes")
        self.filter_bytes, self.workspace_bytes, self.P, self.tiles = fb.value, wb.value, p.value, t.value
        self.mode, self.out = mode, out
        self.kernel_size = KERNEL_SIZE[self.alg]
        self._keep = []

    def close(self):
        if self._h:
            load().sfc_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_point_scales(self, sx: np.ndarray, sw: np.ndarray):
        sx = np.ascontiguousarray(sx, dtype=np.float32)
        sw = np.ascontiguousarray(sw, dtype=np.float32)
        assert sx.shape == (self.P,) and sw.shape == (self.P, self.desc.Cout), (sx.shape, sw.shape)
        _check(load().sfc_set_point_scales(self._h, _f32_ptr(sx), _f32_ptr(sw)),
               "sfc_set_point_scales")

    def group_scales(self, sx: np.ndarray, sw: np.ndarray, act="point", filt="channel_point"):
        """Copies of the finest-granularity scales coarsened to the ablation's groupings."""
        sx = np.array(sx, dtype=np.float32, order="C")
        sw = np.array(sw, dtype=np.float32, order="C")
        assert sx.shape == (self.P,) and sw.shape == (self.P, self.desc.Cout), (sx.shape, sw.shape)
        _check(load().sfc_group_scales(self._h, ACT_GRANULARITY[act], FILTER_GRANULARITY[filt],
                                       _f32_ptr(sx), _f32_ptr(sw)), "sfc_group_scales")
        return sx, sw

    def set_output_scale(self, y_scale: float):
        _check(load().sfc_set_output_scale(self._h, C.c_float(y_scale)), "sfc_set_output_scale")

    def calibrate_act_scales(self, x_dev, workspace, stream=None) -> np.ndarray:
        out = np.empty(self.P, dtype=np.float32)
        _check(load().sfc_calibrate_act_scales(self._h, C.c_void_p(x_dev.data_ptr()),
                                               int(x_dev.shape[0]), C.c_void_p(workspace.data_ptr()),
                                               _nbytes(workspace), _stream_ptr(stream), _f32_ptr(out)),
               "sfc_calibrate_act_scales")
        return out

    def _check_weights(self, w_dev):
        d, r = self.desc, self.kernel_size
        assert w_dev.element_size() == 1 and w_dev.numel() == d.Cout * d.Cin * r * r, \
            (tuple(w_dev.shape), (d.Cout, d.Cin, r, r))

    def calibrate_filter_scales(self, w_dev, workspace, stream=None) -> np.ndarray:
        self._check_weights(w_dev)
        out = np.empty((self.P, self.desc.Cout), dtype=np.float32)
        _check(load().sfc_calibrate_filter_scales(self._h, C.c_void_p(w_dev.data_ptr()),
                                                  C.c_void_p(workspace.data_ptr()), _nbytes(workspace),
                                                  _stream_ptr(stream), _f32_ptr(out)),
               "sfc_calibrate_filter_scales")
        return out

    def transform_filter(self, w_dev, w_scale: np.ndarray, filter_buf, stream=None):
        ws = np.ascontiguousarray(np.asarray(w_scale, dtype=np.float32).reshape(-1))
        need = self.desc.Cout if self.desc.per_channel_wscale else 1
        assert ws.size == need, (ws.size, need)
        self._check_weights(w_dev)
        _check(load().sfc_transform_filter(self._h, C.c_void_p(w_dev.data_ptr()), _f32_ptr(ws),
                                           C.c_void_p(filter_buf.data_ptr()), _nbytes(filter_buf),
                                           _stream_ptr(stream)),
               "sfc_transform_filter")
        self._keep = [filter_buf]

    def conv2d(self, x_dev, x_scale: float, y_dev, workspace, stream=None):
        _check(load().sfc_conv2d_nchw(self._h, C.c_void_p(x_dev.data_ptr()), C.c_float(x_scale),
                                      C.c_void_p(y_dev.data_ptr()), C.c_void_p(workspace.data_ptr()),
                                      _nbytes(workspace), _stream_ptr(stream)),
               "sfc_conv2d_nchw")

    def conv2d_static(self, x_dev, x_scale: float, y_dev, stream=None):
        """sfc_conv2d_nchw with the library's built-in workspace (nothing is allocated)."""
        _check(load().sfc_conv2d_nchw_static(self._h, C.c_void_p(x_dev.data_ptr()), C.c_float(x_scale),
                                             C.c_void_p(y_dev.data_ptr()), _stream_ptr(stream)),
               "sfc_conv2d_nchw_static")

    def conv2d_stages(self, x_dev, x_scale: float, y_dev, workspace, mask: int, stream=None):
        _check(load().sfc_conv2d_stages(self._h, C.c_void_p(x_dev.data_ptr()), C.c_float(x_scale),
                                        C.c_void_p(y_dev.data_ptr()),
                                        C.c_void_p(workspace.data_ptr()), _nbytes(workspace),
                                        _stream_ptr(stream), int(mask)), "sfc_conv2d_stages")

    def tap(self, which: str, workspace) -> np.ndarray:
        """Copy of V, U or M in canonical [P][tiles|Cout][Cin|Cout] order (synchronizes)."""
        # sfc_tap_info describes the tensor as a five-axis strided view; padding is cut off
        import torch

        idx = {"V": 0, "U": 1, "M": 2}[which]
        ptr, esz = C.c_void_p(), C.c_int32()
        dims, strides = (C.c_int64 * 5)(), (C.c_int64 * 5)()
        _check(load().sfc_tap_info(self._h, C.c_void_p(workspace.data_ptr()), idx, C.byref(ptr),
                                   C.byref(esz), dims, strides), "sfc_tap_info")
        base = self._keep[0] if which == "U" else workspace
        off = ptr.value - base.data_ptr()
        nbytes = base.numel() * base.element_size()
        assert 0 <= off < nbytes
        torch.cuda.synchronize()
        if esz.value == 3:  # 24-bit sums: three bytes per element, little-endian, two's complement
            flat = base.view(torch.uint8)[off:]
            view = torch.as_strided(flat, tuple(dims) + (3,), tuple(3 * s for s in strides) + (1,))
            b = view.cpu().numpy().astype(np.int32)
            full = (b[..., 0] | (b[..., 1] << 8) | (b[..., 2] << 16))
            full = (full ^ 0x800000) - 0x800000
        else:
            dtype = {1: torch.int8, 2: torch.int16, 4: torch.int32}[esz.value]
            flat = base.view(torch.uint8)[off:].view(dtype)
            full = torch.as_strided(flat, tuple(dims), tuple(strides)).cpu().numpy()
        full = full.reshape(dims[0], dims[1] * dims[2], dims[3] * dims[4])
        d = self.desc
        rows, cols = {"V": (self.tiles, d.Cin), "U": (d.Cout, d.Cin), "M": (self.tiles, d.Cout)}[which]
        return full[:, :rows, :cols].copy()


def stream_copy(dst, src, stream=None):
    """Plain streaming copy kernel of the library (bandwidth / counter calibration)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes and nbytes % 16 == 0
    _check(load().sfc_stream_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes,
                                  _stream_ptr(stream)), "sfc_stream_copy")


def device_buffer(nbytes: int):
    """A 256-byte-aligned byte buffer on the current CUDA (HIP) device."""
    import torch

    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device="cuda")


def conv2d(x: np.ndarray, w: np.ndarray, x_scale: float, w_scale, mode="requant", alg="6x6_p88",
           out="f32", path="staged", sx=None, sw=None, return_taps=False, y_scale=None,
           transform_bits=0, flags=0):
    """Convenience wrapper: numpy in, numpy out, one layer through the C ABI."""
    import torch

    n, cin, h, wd = x.shape
    cout = w.shape[0]
    ws_arr = np.asarray(w_scale, dtype=np.float32).reshape(-1)
    plan = Plan(n, cin, cout, h, wd, alg=alg, mode=mode, out=out, path=path,
                per_channel_wscale=ws_arr.size != 1, transform_bits=transform_bits, flags=flags)
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    wdv = torch.from_numpy(np.ascontiguousarray(w)).cuda()
    fbuf = device_buffer(plan.filter_bytes)
    wbuf = device_buffer(plan.workspace_bytes)
    if mode == "requant":
        plan.set_point_scales(sx, sw)
    if out == "i8":
        plan.set_output_scale(float(y_scale))
    plan.transform_filter(wdv, ws_arr, fbuf)
    ydt = {"i32": torch.int32, "f32": torch.float32, "i8": torch.int8}[out]
    y = torch.empty((n, cout, h, wd), dtype=ydt, device="cuda")
    plan.conv2d(xd, float(x_scale), y, wbuf)
    torch.cuda.synchronize()
    res = y.cpu().numpy()
    if return_taps:
        names = {"staged": ("V", "U", "M"), "fused": ("V", "U"), "single": ("U",)}[plan.path]
        taps = {k: plan.tap(k, wbuf) for k in names}
        plan.close()
        return res, taps
    plan.close()
    return res
