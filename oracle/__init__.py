"""CPU oracle: TEST INFRASTRUCTURE ONLY.

Plain, slow and obviously correct reference for what the sparse-inference path
computes.  Only tests/, `__graft_entry__.smoke()` and bench.py's cpu_baseline
leg may import this package; the product package never does, and the two share
no code.

Layers (conv / fc / pools) are the C functions in cadnn_oracle.c, which are the
definition of a fused convolution layer written out (paper Section 4: conv +
batch-norm + activation fused; 1x1 convolution == matrix multiply).  Sums are
taken in double and rounded ONCE to the storage dtype here.

The reference packer below fixes the canonical compact weight format.  The
paper only says that pruned filters are stored compactly with accompanying
indices and that the filter layout is transformed (tiling, alignment, padding;
Sections 3 and 4) without giving a format, so the canonical form is this
build's reading:

  * row `co` is the filter of output channel co flattened over
    k = (ci*Kh + kh)*Kw + kw;
  * an entry is kept iff its fp32 value != 0 (drops +0/-0, keeps denormals);
  * inside a row entries are in ascending k;
  * rows are ordered by nonzero count, descending, ties by ascending channel
    index (`perm[i]` = original channel of packed row i);
  * `row_ptr` (over the permuted order), `col_idx` (int32 k) and `vals`
    (fp32 bit copies, or round-to-nearest-even fp16 for the fp16 variant) are
    the concatenation in that order.

Whole-network outputs: parity unpinned by the paper (it prints no logits or
weights); they are pinned only through the per-layer pins.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.oracle_conv2d.argtypes = [fp, fp, fp, fp, dp] + [i] * 10
        lib.oracle_conv2d.restype = i
        lib.oracle_depthwise_conv2d.argtypes = [fp, fp, fp, dp] + [i] * 9
        lib.oracle_depthwise_conv2d.restype = i
        lib.oracle_fc.argtypes = [fp, fp, fp, dp, i, i, i, i]
        lib.oracle_fc.restype = i
        lib.oracle_maxpool.argtypes = [fp, dp] + [i] * 7
        lib.oracle_maxpool.restype = i
        lib.oracle_avgpool.argtypes = [fp, dp] + [i] * 7
        lib.oracle_avgpool.restype = i
        lib.oracle_global_avgpool.argtypes = [fp, dp] + [i] * 4
        lib.oracle_global_avgpool.restype = i
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = i
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a) -> np.ndarray:
    """Exact widening of an fp32/fp16 array to contiguous fp32."""
    a = np.asarray(a)
    if a.dtype not in (np.float32, np.float16):
        raise TypeError(f"oracle takes float32 or float16 storage, got {a.dtype}")
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray], ct):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ct))


def out_size(size: int, k: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - k) // stride + 1


def conv2d_f64(x, w, bias=None, residual=None, stride=1, pad=0, relu=False) -> np.ndarray:
    """Fused conv layer, result in float64 (before the single rounding)."""
    xf, wf = _f32(x), _f32(w)
    n, cin, h, wd = xf.shape
    cout, cin2, kh, kw = wf.shape
    if cin2 != cin:
        raise ValueError("channel mismatch")
    hout, wout = out_size(h, kh, stride, pad), out_size(wd, kw, stride, pad)
    if hout <= 0 or wout <= 0:
        raise ValueError("empty output")
    bf = None if bias is None else _f32(bias)
    rf = None if residual is None else _f32(residual)
    if bf is not None and bf.shape != (cout,):
        raise ValueError("bias shape")
    if rf is not None and rf.shape != (n, cout, hout, wout):
        raise ValueError("residual shape")
    y = np.empty((n, cout, hout, wout), dtype=np.float64)
    rc = _load().oracle_conv2d(_ptr(xf, ctypes.c_float), _ptr(wf, ctypes.c_float),
                               _ptr(bf, ctypes.c_float), _ptr(rf, ctypes.c_float),
                               _ptr(y, ctypes.c_double), n, cin, h, wd, cout, kh, kw,
                               stride, pad, int(bool(relu)))
    if rc != 0:
        raise RuntimeError("oracle_conv2d failed")
    return y


def conv2d(x, w, bias=None, residual=None, stride=1, pad=0, relu=False, dtype=np.float32):
    """Fused conv layer rounded once to `dtype` (float32 or float16)."""
    return conv2d_f64(x, w, bias, residual, stride, pad, relu).astype(dtype)


def depthwise_conv2d_f64(x, w, bias=None, stride=1, pad=0, relu=False) -> np.ndarray:
    """Fused depthwise layer (paper Section 4), w of shape [c][1][kh][kw]; result in float64."""
    xf, wf = _f32(x), _f32(w)
    n, ch, h, wd = xf.shape
    if wf.ndim != 4 or wf.shape[0] != ch or wf.shape[1] != 1:
        raise ValueError("depthwise weights must be [channels][1][kh][kw]")
    kh, kw = wf.shape[2], wf.shape[3]
    hout, wout = out_size(h, kh, stride, pad), out_size(wd, kw, stride, pad)
    if hout <= 0 or wout <= 0:
        raise ValueError("empty output")
    bf = None if bias is None else _f32(bias)
    if bf is not None and bf.shape != (ch,):
        raise ValueError("bias shape")
    y = np.empty((n, ch, hout, wout), dtype=np.float64)
    rc = _load().oracle_depthwise_conv2d(_ptr(xf, ctypes.c_float), _ptr(wf, ctypes.c_float),
                                         _ptr(bf, ctypes.c_float), _ptr(y, ctypes.c_double), n, ch, h, wd,
                                         kh, kw, stride, pad, int(bool(relu)))
    if rc != 0:
        raise RuntimeError("oracle_depthwise_conv2d failed")
    return y


def depthwise_conv2d(x, w, bias=None, stride=1, pad=0, relu=False, dtype=np.float32):
    """Fused depthwise layer rounded once to `dtype` (float32 or float16)."""
    return depthwise_conv2d_f64(x, w, bias, stride, pad, relu).astype(dtype)


def fc_f64(x, w, bias=None, relu=False) -> np.ndarray:
    xf, wf = _f32(x), _f32(w)
    xf = np.ascontiguousarray(xf.reshape(xf.shape[0], -1))
    wf = np.ascontiguousarray(wf.reshape(wf.shape[0], -1))
    n, cin = xf.shape
    cout, cin2 = wf.shape
    if cin2 != cin:
        raise ValueError("feature mismatch")
    bf = None if bias is None else _f32(bias)
    y = np.empty((n, cout), dtype=np.float64)
    rc = _load().oracle_fc(_ptr(xf, ctypes.c_float), _ptr(wf, ctypes.c_float),
                           _ptr(bf, ctypes.c_float), _ptr(y, ctypes.c_double), n, cin, cout,
                           int(bool(relu)))
    if rc != 0:
        raise RuntimeError("oracle_fc failed")
    return y


def fc(x, w, bias=None, relu=False, dtype=np.float32):
    return fc_f64(x, w, bias, relu).astype(dtype)


def maxpool(x, k, stride, pad, dtype=None):
    xf = _f32(x)
    n, c, h, wd = xf.shape
    hout, wout = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    y = np.empty((n, c, hout, wout), dtype=np.float64)
    rc = _load().oracle_maxpool(_ptr(xf, ctypes.c_float), _ptr(y, ctypes.c_double), n, c, h, wd,
                                k, stride, pad)
    if rc != 0:
        raise RuntimeError("oracle_maxpool failed")
    return y.astype(dtype or np.asarray(x).dtype)


def avgpool(x, k, stride, pad, dtype=None):
    """Mean over the in-image part of each k x k window (padding neither summed nor counted)."""
    xf = _f32(x)
    n, c, h, wd = xf.shape
    hout, wout = out_size(h, k, stride, pad), out_size(wd, k, stride, pad)
    y = np.empty((n, c, hout, wout), dtype=np.float64)
    rc = _load().oracle_avgpool(_ptr(xf, ctypes.c_float), _ptr(y, ctypes.c_double), n, c, h, wd,
                                k, stride, pad)
    if rc != 0:
        raise RuntimeError("oracle_avgpool failed")
    return y.astype(dtype or np.asarray(x).dtype)


def global_avgpool(x, dtype=None):
    xf = _f32(x)
    n, c, h, wd = xf.shape
    y = np.empty((n, c, 1, 1), dtype=np.float64)
    rc = _load().oracle_global_avgpool(_ptr(xf, ctypes.c_float), _ptr(y, ctypes.c_double), n, c,
                                       h, wd)
    if rc != 0:
        raise RuntimeError("oracle_global_avgpool failed")
    return y.astype(dtype or np.asarray(x).dtype)


# ----------------------------------------------------------------------------
# Reference packer (canonical compact format, see module docstring)
# ----------------------------------------------------------------------------

def pack(w, dtype=np.float32) -> Dict[str, np.ndarray]:
    w = np.asarray(w)
    if w.dtype != np.float32:
        raise TypeError("pack takes the fp32 pruned tensor")
    cout = w.shape[0]
    flat = w.reshape(cout, -1)
    nz = flat != np.float32(0.0)
    counts = nz.sum(axis=1).astype(np.int64)
    perm = np.argsort(-counts, kind="stable").astype(np.int32)
    row_ptr = np.zeros(cout + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(counts[perm])
    cols: List[np.ndarray] = []
    vals: List[np.ndarray] = []
    for r in perm:
        k = np.flatnonzero(nz[r])
        cols.append(k.astype(np.int32))
        vals.append(flat[r, k].astype(dtype))
    col_idx = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    v = np.concatenate(vals) if vals else np.zeros(0, dtype)
    return {"perm": perm, "row_ptr": row_ptr, "col_idx": col_idx.astype(np.int32),
            "vals": v.astype(dtype), "shape": tuple(w.shape)}


def unpack(packed: Dict[str, np.ndarray]) -> np.ndarray:
    shape = packed["shape"]
    cout = shape[0]
    k_total = int(np.prod(shape[1:]))
    out = np.zeros((cout, k_total), dtype=packed["vals"].dtype)
    rp = packed["row_ptr"]
    for i, r in enumerate(packed["perm"]):
        s, e = int(rp[i]), int(rp[i + 1])
        out[r, packed["col_idx"][s:e]] = packed["vals"][s:e]
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# Whole-net interpreter over a layer table (objects with .kind/.src/.dst/...)
# ----------------------------------------------------------------------------

def run_net(ops: Sequence, x, weights: Sequence, biases: Sequence, dtype=np.float32
            ) -> Tuple[np.ndarray, List[np.ndarray], List[np.ndarray]]:
    """Runs the op list layer by layer.

    Returns (output, ins, outs) where ins[i]/outs[i] are the storage-dtype input
    and output of op i (so each layer can also be checked in isolation on the
    oracle's own input).  In the fp16 variant weights and every activation are
    held in IEEE fp16, bias in fp32, and each layer is rounded once to fp16.
    """
    bufs: Dict[int, np.ndarray] = {0: np.asarray(x).astype(dtype)}
    ins: List[np.ndarray] = []
    outs: List[np.ndarray] = []
    for i, op in enumerate(ops):
        src = bufs[op.src]
        if op.kind == "conv":
            res = bufs[op.res] if op.res >= 0 else None
            w = np.asarray(weights[i]).astype(dtype)
            y = conv2d(src, w, biases[i], res, op.stride, op.pad, op.relu, dtype)
        elif op.kind == "dwconv":
            w = np.asarray(weights[i]).astype(dtype)
            y = depthwise_conv2d(src, w, biases[i], op.stride, op.pad, op.relu, dtype)
        elif op.kind == "fc":
            w = np.asarray(weights[i]).astype(dtype)
            y = fc(src, w, biases[i], op.relu, dtype)
            y = y.reshape(y.shape[0], y.shape[1], 1, 1)
        elif op.kind == "maxpool":
            y = maxpool(src, op.k, op.stride, op.pad, dtype)
        elif op.kind == "avgpool":
            y = global_avgpool(src, dtype)
        elif op.kind == "avgpool2d":
            y = avgpool(src, op.k, op.stride, op.pad, dtype)
        elif op.kind == "concat":
            y = np.concatenate([bufs[b] for b in op.srcs], axis=1)
        else:
            raise ValueError(op.kind)
        ins.append(src)
        outs.append(y)
        bufs[op.dst] = y
    return outs[-1], ins, outs
