"""ctypes marshalling for libcadnn.so.  No arithmetic happens in this file."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = 0
F16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
# CADNN_LIB_PATH: another build of the same library (the host-sanitizer build); never a fallback
_LIB_PATH = os.environ.get("CADNN_LIB_PATH") or os.path.join(_HERE, "libcadnn.so")
_lib = None

_vp = ctypes.c_void_p
_i = ctypes.c_int
_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)

_STATUS = {0: "CADNN_OK", 1: "CADNN_EINVAL", 2: "CADNN_EUNSUPPORTED", 3: "CADNN_ENOMEM", 4: "CADNN_EHIP"}


class CadnnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{_STATUS.get(code, code)}: {text}")
        self.code = code
        self.text = text


class OpInfo(ctypes.Structure):
    """Mirror of cadnn_op_info."""
    _fields_ = [("halo_h", ctypes.c_int), ("halo_w", ctypes.c_int), ("pitch", ctypes.c_int),
                ("plane", ctypes.c_int64), ("image", ctypes.c_int64), ("deinterleaved", ctypes.c_int),
                ("offset", ctypes.c_int64), ("fused_into", ctypes.c_int), ("slice_of", ctypes.c_int),
                ("slice_channel", ctypes.c_int), ("launched_with", ctypes.c_int), ("launched_after", ctypes.c_int),
                ("input_copy", ctypes.c_int64)]


class PlanInfo(ctypes.Structure):
    """Mirror of cadnn_plan_info."""
    _fields_ = [("entries", ctypes.c_int64), ("stream_bytes", ctypes.c_int64), ("alloc_bytes", ctypes.c_int64), ("table_bytes", ctypes.c_int64),
                ("bytes_per_nonzero", ctypes.c_double), ("chunks", ctypes.c_int), ("lds_bytes", ctypes.c_int)]


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Loads libcadnn.so (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_1905_00571_amd.build` "
            "(there is no fallback path)")
    try:
        import torch  # noqa: F401  (loads the HIP runtime the process will use)
    except Exception:  # pragma: no cover - torch is optional for symbol checks only
        pass
    L = ctypes.CDLL(_LIB_PATH)
    sig = {
        "cadnn_last_error": (ctypes.c_char_p, []),
        "cadnn_pack_weights": (_i, [_f32p, _i, _i, _i, _i, _i, ctypes.POINTER(_vp)]),
        "cadnn_free_weights": (_i, [_vp]),
        "cadnn_packed_nnz": (_i, [_vp, ctypes.POINTER(ctypes.c_int64)]),
        "cadnn_packed_export": (_i, [_vp, _i32p, _i32p, _i32p, _vp]),
        "cadnn_unpack_weights": (_i, [_vp, _f32p]),
        "cadnn_sparse_conv2d": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp]),
        "cadnn_conv2d_prepare": (_i, [_vp, _i, _i, _i, _i, _i]),
        "cadnn_conv2d_variant_name": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_char_p, ctypes.c_size_t]),
        "cadnn_conv2d_tune": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _i, _vp, _i, _f32p]),
        "cadnn_conv2d_list_variants": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_char_p, ctypes.c_size_t]),
        "cadnn_conv2d_set_variant": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_char_p]),
        "cadnn_conv2d_plan_info": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_char_p, ctypes.POINTER(PlanInfo)]),
        "cadnn_conv2d_plan_unpack": (_i, [_vp, _i, _i, _i, _i, _i, ctypes.c_char_p, _f32p]),
        "cadnn_sparse_fc": (_i, [_vp, _vp, _vp, _i, _vp, _i, _vp]),
        "cadnn_fc_prepare": (_i, [_vp]),
        "cadnn_depthwise_conv2d": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _i, _vp]),
        "cadnn_depthwise_prepare": (_i, [_vp]),
        "cadnn_device_copy": (_i, [_vp, _vp, ctypes.c_size_t, _vp]),
        "cadnn_maxpool2d": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i, _vp]),
        "cadnn_avgpool2d": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _i, _i, _i, _vp]),
        "cadnn_global_avgpool": (_i, [_vp, _vp, _i, _i, _i, _i, _i, _vp]),
        "cadnn_dense_conv2d": (_i, [_vp, _vp, _vp] + [_i] * 9 + [_vp, _vp, _i, _i, _vp]),
        "cadnn_net_create": (_i, [_i, _i, _i, _i, _i, ctypes.POINTER(_vp)]),
        "cadnn_net_add_conv": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i]),
        "cadnn_net_add_depthwise": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i]),
        "cadnn_net_add_maxpool": (_i, [_vp, _i, _i, _i, _i, _i]),
        "cadnn_net_add_global_avgpool": (_i, [_vp, _i, _i]),
        "cadnn_net_add_avgpool": (_i, [_vp, _i, _i, _i, _i, _i]),
        "cadnn_net_add_concat": (_i, [_vp, ctypes.POINTER(_i), _i, _i]),
        "cadnn_net_add_fc": (_i, [_vp, _vp, _vp, _i, _i, _i]),
        "cadnn_net_workspace_bytes": (_i, [_vp, ctypes.POINTER(ctypes.c_size_t)]),
        "cadnn_net_finalize": (_i, [_vp, _vp, ctypes.c_size_t, _i]),
        "cadnn_net_op_info": (_i, [_vp, _i, _i, ctypes.POINTER(OpInfo)]),
        "cadnn_run_net": (_i, [_vp, _vp, _vp, _vp]),
        "cadnn_net_num_ops": (_i, [_vp, ctypes.POINTER(_i)]),
        "cadnn_graph_launch_floor": (_i, [_vp, _i, _i, _vp, _f32p]),
        "cadnn_run_net_noalloc": (_i, [_vp, _vp, _vp, _vp]),
        "cadnn_net_profile": (_i, [_vp, _vp, _vp, _vp, _i, _f32p]),
        "cadnn_net_profile_in_order": (_i, [_vp, _vp, _vp, _vp, _i, _f32p]),
        "cadnn_net_op_variant": (_i, [_vp, _i, ctypes.c_char_p, ctypes.c_size_t]),
        "cadnn_net_op_candidates": (_i, [_vp, _i, ctypes.c_char_p, ctypes.c_size_t]),
        "cadnn_net_set_op_variant": (_i, [_vp, _i, ctypes.c_char_p]),
        "cadnn_net_read_buffer": (_i, [_vp, _i, _vp, ctypes.c_size_t, _vp]),
        "cadnn_net_free": (_i, [_vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTED = None  # filled lazily by tests from include/cadnn.h


def _check(rc: int) -> None:
    if rc != 0:
        raise CadnnError(rc, lib().cadnn_last_error().decode("utf-8", "replace"))


def _stream_ptr(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _torch_dtype(dtype: int):
    import torch
    return torch.float16 if dtype == F16 else torch.float32


class Weights:
    """Owner of a cadnn_weights handle."""

    def __init__(self, handle: int, cout: int, cin: int, kh: int, kw: int, dtype: int):
        self.handle = handle
        self.cout, self.cin, self.kh, self.kw, self.dtype = cout, cin, kh, kw, dtype

    def free(self) -> None:
        if self.handle:
            lib().cadnn_free_weights(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def cadnn_pack_weights(w: np.ndarray, dtype: int = F32) -> Weights:
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim == 2:
        w = w.reshape(w.shape[0], w.shape[1], 1, 1)
    cout, cin, kh, kw = w.shape
    out = _vp()
    _check(lib().cadnn_pack_weights(w.ctypes.data_as(_f32p), cout, cin, kh, kw, dtype, ctypes.byref(out)))
    return Weights(out.value, cout, cin, kh, kw, dtype)


def cadnn_free_weights(w: Weights) -> None:
    w.free()


def cadnn_packed_nnz(w: Weights) -> int:
    n = ctypes.c_int64()
    _check(lib().cadnn_packed_nnz(w.handle, ctypes.byref(n)))
    return int(n.value)


def cadnn_packed_export(w: Weights):
    nnz = cadnn_packed_nnz(w)
    perm = np.empty(w.cout, np.int32)
    row_ptr = np.empty(w.cout + 1, np.int32)
    col = np.empty(nnz, np.int32)
    vals = np.empty(nnz, np.float16 if w.dtype == F16 else np.float32)
    _check(lib().cadnn_packed_export(w.handle, perm.ctypes.data_as(_i32p), row_ptr.ctypes.data_as(_i32p),
                                     col.ctypes.data_as(_i32p), vals.ctypes.data_as(_vp)))
    return {"perm": perm, "row_ptr": row_ptr, "col_idx": col, "vals": vals}


def cadnn_unpack_weights(w: Weights) -> np.ndarray:
    out = np.empty((w.cout, w.cin, w.kh, w.kw), np.float32)
    _check(lib().cadnn_unpack_weights(w.handle, out.ctypes.data_as(_f32p)))
    return out


def cadnn_conv2d_prepare(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int) -> None:
    _check(lib().cadnn_conv2d_prepare(w.handle, n, h, wdt, stride, pad))


def cadnn_conv2d_variant_name(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int) -> str:
    buf = ctypes.create_string_buffer(256)
    _check(lib().cadnn_conv2d_variant_name(w.handle, n, h, wdt, stride, pad, buf, 256))
    return buf.value.decode()


def cadnn_conv2d_list_variants(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int) -> List[str]:
    buf = ctypes.create_string_buffer(1 << 16)
    _check(lib().cadnn_conv2d_list_variants(w.handle, n, h, wdt, stride, pad, buf, 1 << 16))
    text = buf.value.decode()
    return text.split("\n") if text else []


def cadnn_graph_launch_floor(scratch, launches: int = 64, reps: int = 20, stream=None) -> float:
    """Microseconds per kernel boundary inside a replayed graph (scratch: >= 32 bytes on the device)."""
    us = ctypes.c_float(0.0)
    _check(lib().cadnn_graph_launch_floor(_dptr(scratch), launches, reps, _stream_ptr(stream), ctypes.byref(us)))
    return float(us.value)


def cadnn_conv2d_plan_info(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int,
                           variant: Optional[str] = None) -> dict:
    info = PlanInfo()
    _check(lib().cadnn_conv2d_plan_info(w.handle, n, h, wdt, stride, pad, None if not variant else variant.encode(),
                                        ctypes.byref(info)))
    return {k: getattr(info, k) for k, _ in PlanInfo._fields_}


def cadnn_conv2d_plan_unpack(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int,
                             variant: Optional[str] = None) -> np.ndarray:
    out = np.empty((w.cout, w.cin, w.kh, w.kw), np.float32)
    _check(lib().cadnn_conv2d_plan_unpack(w.handle, n, h, wdt, stride, pad, None if not variant else variant.encode(),
                                          out.ctypes.data_as(_f32p)))
    return out


def cadnn_conv2d_set_variant(w: Weights, n: int, h: int, wdt: int, stride: int, pad: int,
                             name: Optional[str]) -> None:
    _check(lib().cadnn_conv2d_set_variant(w.handle, n, h, wdt, stride, pad,
                                          None if not name else name.encode()))


def cadnn_conv2d_tune(w: Weights, x, y, stride: int = 1, pad: int = 0, bias=None, residual=None,
                      relu: bool = False, reps: int = 20, stream=None) -> float:
    """Times every variant on (x, y) and pins the fastest; returns its microseconds per launch."""
    n, _, h, wdt = x.shape
    us = ctypes.c_float()
    _check(lib().cadnn_conv2d_tune(w.handle, _dptr(x), _dptr(y), n, h, wdt, stride, pad, _dptr(bias),
                                   _dptr(residual), int(bool(relu)), _stream_ptr(stream), reps,
                                   ctypes.byref(us)))
    return float(us.value)


def _out_size(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def cadnn_sparse_conv2d(w: Weights, x, stride: int = 1, pad: int = 0, bias=None, residual=None,
                        relu: bool = False, out=None, stream=None):
    """x: contiguous CUDA tensor [n][cin][h][w]; returns (or fills) y."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dtype == _torch_dtype(w.dtype)
    n, cin, h, wdt = x.shape
    if cin != w.cin:
        raise ValueError("channel mismatch")
    hout, wout = _out_size(h, w.kh, stride, pad), _out_size(wdt, w.kw, stride, pad)
    if out is None:
        if hout <= 0 or wout <= 0:
            raise CadnnError(1, "empty output")
        out = torch.empty((n, w.cout, hout, wout), dtype=x.dtype, device=x.device)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float32 and bias.numel() == w.cout
    if residual is not None:
        assert residual.is_cuda and residual.is_contiguous() and residual.shape == out.shape
    _check(lib().cadnn_sparse_conv2d(w.handle, _dptr(x), _dptr(out), n, h, wdt, stride, pad, _dptr(bias),
                                     _dptr(residual), int(bool(relu)), _stream_ptr(stream)))
    return out


def cadnn_depthwise_conv2d(w: Weights, x, stride: int = 1, pad: int = 0, bias=None, relu: bool = False,
                           out=None, stream=None):
    """w packed from [channels][1][kh][kw]; x: contiguous CUDA tensor [n][channels][h][w]."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dtype == _torch_dtype(w.dtype)
    n, ch, h, wdt = x.shape
    if ch != w.cout:
        raise ValueError("channel mismatch")
    hout, wout = _out_size(h, w.kh, stride, pad), _out_size(wdt, w.kw, stride, pad)
    if out is None:
        if hout <= 0 or wout <= 0:
            raise CadnnError(1, "empty output")
        out = torch.empty((n, ch, hout, wout), dtype=x.dtype, device=x.device)
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.float32 and bias.numel() == ch
    _check(lib().cadnn_depthwise_conv2d(w.handle, _dptr(x), _dptr(out), n, h, wdt, stride, pad, _dptr(bias),
                                        int(bool(relu)), _stream_ptr(stream)))
    return out


def cadnn_depthwise_prepare(w: Weights) -> None:
    _check(lib().cadnn_depthwise_prepare(w.handle))


def cadnn_sparse_fc(w: Weights, x, bias=None, relu: bool = False, out=None, stream=None):
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dtype == _torch_dtype(w.dtype)
    n = x.shape[0]
    if x.numel() != n * w.cin:
        raise ValueError("feature mismatch")
    if out is None:
        out = torch.empty((n, w.cout), dtype=x.dtype, device=x.device)
    _check(lib().cadnn_sparse_fc(w.handle, _dptr(x), _dptr(out), n, _dptr(bias), int(bool(relu)),
                                 _stream_ptr(stream)))
    return out


def cadnn_fc_prepare(w: Weights) -> None:
    _check(lib().cadnn_fc_prepare(w.handle))


def cadnn_device_copy(src, dst, stream=None) -> None:
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(lib().cadnn_device_copy(_dptr(src), _dptr(dst), nbytes, _stream_ptr(stream)))


def cadnn_maxpool2d(x, k: int, stride: int, pad: int, stream=None):
    import torch
    assert x.is_cuda and x.is_contiguous()
    dtype = F16 if x.dtype == torch.float16 else F32
    n, c, h, wdt = x.shape
    out = torch.empty((n, c, _out_size(h, k, stride, pad), _out_size(wdt, k, stride, pad)),
                      dtype=x.dtype, device=x.device)
    _check(lib().cadnn_maxpool2d(_dptr(x), _dptr(out), n, c, h, wdt, k, stride, pad, dtype, _stream_ptr(stream)))
    return out


def cadnn_avgpool2d(x, k: int, stride: int, pad: int, stream=None):
    import torch
    assert x.is_cuda and x.is_contiguous()
    dtype = F16 if x.dtype == torch.float16 else F32
    n, c, h, wdt = x.shape
    out = torch.empty((n, c, _out_size(h, k, stride, pad), _out_size(wdt, k, stride, pad)),
                      dtype=x.dtype, device=x.device)
    _check(lib().cadnn_avgpool2d(_dptr(x), _dptr(out), n, c, h, wdt, k, stride, pad, dtype, _stream_ptr(stream)))
    return out


def cadnn_global_avgpool(x, stream=None):
    import torch
    assert x.is_cuda and x.is_contiguous()
    dtype = F16 if x.dtype == torch.float16 else F32
    n, c, h, wdt = x.shape
    out = torch.empty((n, c, 1, 1), dtype=x.dtype, device=x.device)
    _check(lib().cadnn_global_avgpool(_dptr(x), _dptr(out), n, c, h, wdt, dtype, _stream_ptr(stream)))
    return out


def cadnn_dense_conv2d(w_dev, x, stride: int = 1, pad: int = 0, bias=None, residual=None,
                       relu: bool = False, out=None, stream=None):
    import torch
    assert x.is_cuda and x.is_contiguous() and w_dev.is_cuda and w_dev.is_contiguous()
    assert w_dev.dtype == x.dtype
    dtype = F16 if x.dtype == torch.float16 else F32
    n, cin, h, wdt = x.shape
    cout, cin2, kh, kw = w_dev.shape
    if cin2 != cin:
        raise ValueError("channel mismatch")
    if out is None:
        out = torch.empty((n, cout, _out_size(h, kh, stride, pad), _out_size(wdt, kw, stride, pad)),
                          dtype=x.dtype, device=x.device)
    _check(lib().cadnn_dense_conv2d(_dptr(w_dev), _dptr(x), _dptr(out), n, cin, h, wdt, cout, kh, kw,
                                    stride, pad, _dptr(bias), _dptr(residual), int(bool(relu)), dtype,
                                    _stream_ptr(stream)))
    return out


class Net:
    """Owner of a cadnn_net handle plus the tensors it points into."""

    def __init__(self, handle: int, dtype: int, in_shape, out_shape, keep: list, ops: Sequence, flags: int = 0):
        self.handle = handle
        self.flags = flags
        self.dtype = dtype
        self.in_shape = tuple(in_shape)
        self.out_shape = tuple(out_shape)
        self._keep = keep
        self.ops = list(ops)

    def op_info(self, op_index: int) -> dict:
        """Where op `op_index` puts its output and whether it launches (cadnn_net_op_info, for the
        flags the net was finalized with; after live tuning it shows the groups that were kept)."""
        info = OpInfo()
        _check(lib().cadnn_net_op_info(self.handle, op_index, self.flags, ctypes.byref(info)))
        return {name: getattr(info, name) for name, _ in OpInfo._fields_}

    def num_ops(self) -> int:
        n = _i()
        _check(lib().cadnn_net_num_ops(self.handle, ctypes.byref(n)))
        return int(n.value)

    def run(self, x, y=None, stream=None):
        import torch
        assert x.is_cuda and x.is_contiguous() and tuple(x.shape) == self.in_shape
        if y is None:
            y = torch.empty(self.out_shape, dtype=x.dtype, device=x.device)
        _check(lib().cadnn_run_net(self.handle, _dptr(x), _dptr(y), _stream_ptr(stream)))
        return y

    def run_noalloc(self, x, y, stream=None):
        """cadnn_run_net_noalloc: y is the caller's (nothing is allocated, here or in the library)."""
        assert x.is_cuda and x.is_contiguous() and tuple(x.shape) == self.in_shape
        assert y.is_cuda and y.is_contiguous() and tuple(y.shape) == self.out_shape
        _check(lib().cadnn_run_net_noalloc(self.handle, _dptr(x), _dptr(y), _stream_ptr(stream)))
        return y

    def profile(self, x, y, repeats: int = 10, stream=None) -> np.ndarray:
        ms = np.zeros(self.num_ops(), np.float32)
        _check(lib().cadnn_net_profile(self.handle, _dptr(x), _dptr(y), _stream_ptr(stream), repeats,
                                       ms.ctypes.data_as(_f32p)))
        return ms

    def profile_in_order(self, x, y, repeats: int = 10, stream=None) -> np.ndarray:
        """ms per op with the ops in launch order (each kernel's own device time)."""
        ms = np.zeros(self.num_ops(), np.float32)
        _check(lib().cadnn_net_profile_in_order(self.handle, _dptr(x), _dptr(y), _stream_ptr(stream), repeats,
                                                ms.ctypes.data_as(_f32p)))
        return ms

    def op_variant(self, op_index: int) -> str:
        buf = ctypes.create_string_buffer(256)
        _check(lib().cadnn_net_op_variant(self.handle, op_index, buf, 256))
        return buf.value.decode()

    def op_candidates(self, op_index: int) -> List[str]:
        buf = ctypes.create_string_buffer(1 << 16)
        _check(lib().cadnn_net_op_candidates(self.handle, op_index, buf, 1 << 16))
        text = buf.value.decode()
        return text.split("\n") if text else []

    def set_op_variant(self, op_index: int, name: Optional[str]) -> None:
        _check(lib().cadnn_net_set_op_variant(self.handle, op_index, None if not name else name.encode()))

    def variants(self) -> List[str]:
        return [self.op_variant(i) for i in range(self.num_ops())]

    def set_variants(self, names: Sequence[str]) -> None:
        """Pins every convolution op to the named variant (a saved tuning result: the list
        `variants()` returned).  An op that shares another op's launch here but had a launch of
        its own when the list was saved belongs to a group that tuning took apart: the group
        is taken apart first."""
        infos = [self.op_info(i) for i in range(len(self.ops))]
        apart = sorted({infos[i]["fused_into"] for i, name in enumerate(names)
                        if infos[i]["launched_with"] and name != "fused"})
        for lead in apart:
            self.set_op_variant(lead, "apart")
        for i, (op, name) in enumerate(zip(self.ops, names)):
            if op.kind == "conv" and name != "fused":
                self.set_op_variant(i, name)

    def read_buffer(self, buf: int, shape, stream=None) -> np.ndarray:
        out = np.empty(shape, np.float16 if self.dtype == F16 else np.float32)
        _check(lib().cadnn_net_read_buffer(self.handle, buf, out.ctypes.data_as(_vp), out.nbytes,
                                           _stream_ptr(stream)))
        return out

    def free(self) -> None:
        if self.handle:
            lib().cadnn_net_free(self.handle)
            self.handle = None
        self._keep = []

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def cadnn_run_net(net: Net, x, y=None, stream=None):
    return net.run(x, y, stream)


def cadnn_run_net_noalloc(net: Net, x, y, stream=None):
    return net.run_noalloc(x, y, stream)


def _add_ops(L, handle, ops, weights, biases, input_shape, dtype, keep, to_device):
    """Packs the weights and adds every op of the table to the net; returns the buffer shapes.
    `to_device` turns a host bias vector into a device tensor (None: the ops get no bias, which
    is enough for calls that only look at shapes and layouts)."""
    shapes = {0: tuple(input_shape)}
    for i, op in enumerate(ops):
        if op.kind in ("conv", "fc", "dwconv"):
            pw = cadnn_pack_weights(np.asarray(weights[i], dtype=np.float32), dtype)
            b = None
            if to_device is not None and biases[i] is not None:
                b = to_device(biases[i])
            keep += [pw, b]
            if op.kind == "conv":
                _check(L.cadnn_net_add_conv(handle, pw.handle, _dptr(b), op.stride, op.pad,
                                            int(bool(op.relu)), op.src, op.dst, op.res))
                s = shapes[op.src]
                shapes[op.dst] = (s[0], pw.cout, _out_size(s[2], pw.kh, op.stride, op.pad),
                                  _out_size(s[3], pw.kw, op.stride, op.pad))
            elif op.kind == "dwconv":
                _check(L.cadnn_net_add_depthwise(handle, pw.handle, _dptr(b), op.stride, op.pad,
                                                 int(bool(op.relu)), op.src, op.dst))
                s = shapes[op.src]
                shapes[op.dst] = (s[0], s[1], _out_size(s[2], pw.kh, op.stride, op.pad),
                                  _out_size(s[3], pw.kw, op.stride, op.pad))
            else:
                _check(L.cadnn_net_add_fc(handle, pw.handle, _dptr(b), int(bool(op.relu)), op.src, op.dst))
                shapes[op.dst] = (shapes[op.src][0], pw.cout, 1, 1)
        elif op.kind == "maxpool":
            _check(L.cadnn_net_add_maxpool(handle, op.k, op.stride, op.pad, op.src, op.dst))
            s = shapes[op.src]
            shapes[op.dst] = (s[0], s[1], _out_size(s[2], op.k, op.stride, op.pad),
                              _out_size(s[3], op.k, op.stride, op.pad))
        elif op.kind == "avgpool2d":
            _check(L.cadnn_net_add_avgpool(handle, op.k, op.stride, op.pad, op.src, op.dst))
            s = shapes[op.src]
            shapes[op.dst] = (s[0], s[1], _out_size(s[2], op.k, op.stride, op.pad),
                              _out_size(s[3], op.k, op.stride, op.pad))
        elif op.kind == "concat":
            arr = (ctypes.c_int * len(op.srcs))(*op.srcs)
            _check(L.cadnn_net_add_concat(handle, arr, len(op.srcs), op.dst))
            s = shapes[op.srcs[0]]
            shapes[op.dst] = (s[0], sum(shapes[b][1] for b in op.srcs), s[2], s[3])
        elif op.kind == "avgpool":
            _check(L.cadnn_net_add_global_avgpool(handle, op.src, op.dst))
            s = shapes[op.src]
            shapes[op.dst] = (s[0], s[1], 1, 1)
        else:
            raise ValueError(op.kind)
    return shapes


def plan_net(ops: Sequence, weights: Sequence, input_shape, dtype: int = F32, plain_layout: bool = False,
             fuse: bool = True):
    """Host-only: wires the op list into a cadnn_net and returns (per-op cadnn_op_info records as
    dicts, workspace bytes) for the given layout flags.  Needs no GPU and runs nothing."""
    L = lib()
    n, c, h, w = input_shape
    handle = _vp()
    _check(L.cadnn_net_create(dtype, n, c, h, w, ctypes.byref(handle)))
    keep: list = []
    try:
        _add_ops(L, handle, ops, weights, [None] * len(ops), input_shape, dtype, keep, None)
        flags = (4 if plain_layout else 0) | (0 if fuse else 8)
        infos = []
        for i in range(len(ops)):
            info = OpInfo()
            _check(L.cadnn_net_op_info(handle, i, flags, ctypes.byref(info)))
            infos.append({name: getattr(info, name) for name, _ in OpInfo._fields_})
        nbytes = ctypes.c_size_t()
        _check(L.cadnn_net_workspace_bytes(handle, ctypes.byref(nbytes)))
    finally:
        L.cadnn_net_free(handle)
        for k in keep:
            if isinstance(k, Weights):
                k.free()
    return infos, int(nbytes.value)


def build_net(ops: Sequence, weights: Sequence, biases: Sequence, input_shape, dtype: int = F32,
              use_graph: bool = True, tune: bool = False, device: str = "cuda:0",
              plain_layout: bool = False, fuse: bool = True, static_workspace: bool = False) -> Net:
    """Packs every layer's weights and wires the op list into a cadnn_net.
    static_workspace: the net's intermediate tensors live in the library's static device array
    (CADNN_NET_STATIC_WORKSPACE), which is what Net.run_noalloc needs.

    `ops` are records with .kind in {"conv", "dwconv", "fc", "maxpool", "avgpool2d", "avgpool", "concat"} and
    .src/.dst/.res/.k/.stride/.pad/.relu fields (see workloads.nets.Op).
    """
    import torch
    L = lib()
    n, c, h, w = input_shape
    handle = _vp()
    _check(L.cadnn_net_create(dtype, n, c, h, w, ctypes.byref(handle)))
    keep: list = []
    try:
        shapes = _add_ops(L, handle, ops, weights, biases, input_shape, dtype, keep,
                          lambda b: torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(device))
        flags = (1 if use_graph else 0) | (2 if tune else 0) | (4 if plain_layout else 0) | (0 if fuse else 8)
        # the workspace size depends on the layout flags: have the library lay the net out for them first
        _check(L.cadnn_net_op_info(handle, 0, flags, ctypes.byref(OpInfo())))
        nbytes = ctypes.c_size_t()
        _check(L.cadnn_net_workspace_bytes(handle, ctypes.byref(nbytes)))
        if static_workspace:
            flags |= 16
            _check(L.cadnn_net_finalize(handle, None, 0, flags))
        else:
            ws = torch.empty(max(int(nbytes.value), 256), dtype=torch.uint8, device=device)
            keep.append(ws)
            _check(L.cadnn_net_finalize(handle, _dptr(ws), int(nbytes.value), flags))
    except Exception:
        L.cadnn_net_free(handle)
        raise
    return Net(handle.value, dtype, input_shape, shapes[ops[-1].dst], keep, ops, flags)
