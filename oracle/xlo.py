"""ctypes front end of the CPU oracle (oracle/xlo.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module; the product path never does.  It imports nothing from the HIP
package.

`forward` walks a layer graph in topological (list) order and evaluates every
layer unfused with full intermediates held in host memory -- the plain
definition that any fused execution (paper section 3.1, straight / split /
merge) has to reproduce.  The graph is any object with `.layers` (each with
op, inputs, out, cin, cout, k, stride, pad, groups, relu) and `.shapes`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xlo.c")
_LIB = os.path.join(_HERE, "libxlo.so")
_lib = None

_F = ctypes.POINTER(ctypes.c_float)


def build(force: bool = False) -> str:
    """Compile oracle/xlo.c with gcc (-O2, OpenMP over outer loops only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i, ll = ctypes.c_int, ctypes.c_longlong
        L.xlo_num_threads.restype = i
        L.xlo_set_num_threads.argtypes = [i]
        L.xlo_conv2d.argtypes = [_F, i, i, i, i, _F, i, i, i, i, i, i, _F, _F, i, _F]
        L.xlo_conv2d.restype = i
        L.xlo_maxpool2d.argtypes = [_F, i, i, i, i, i, i, i, _F]
        L.xlo_maxpool2d.restype = i
        L.xlo_global_avgpool.argtypes = [_F, i, i, i, i, _F]
        L.xlo_global_avgpool.restype = i
        L.xlo_add.argtypes = [_F, _F, ll, i, _F]
        L.xlo_add.restype = i
        L.xlo_concat_channels.argtypes = [_F, i, _F, i, i, ll, _F]
        L.xlo_concat_channels.restype = i
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.cast(None, _F)
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_F)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(lib().xlo_num_threads())


def set_num_threads(n: int) -> None:
    lib().xlo_set_num_threads(int(n))


def conv2d(x, w, stride=1, pad=0, groups=1, scale=None, shift=None, relu=False) -> np.ndarray:
    x, w = _f32(x), _f32(w)
    n, c, h, wd = x.shape
    o, cg, kh, kw = w.shape
    if cg * groups != c:
        raise ValueError("filter/input channel mismatch")
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.empty((n, o, ho, wo), dtype=np.float32)
    scale = None if scale is None else _f32(scale)
    shift = None if shift is None else _f32(shift)
    rc = lib().xlo_conv2d(_p(x), n, c, h, wd, _p(w), o, kh, kw, stride, pad, groups,
                          _p(scale), _p(shift), int(bool(relu)), _p(y))
    if rc != 0:
        raise ValueError("xlo_conv2d rejected the sizes")
    return y


def maxpool2d(x, k, stride, pad=0) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, ho, wo), dtype=np.float32)
    if lib().xlo_maxpool2d(_p(x), n, c, h, w, k, stride, pad, _p(y)) != 0:
        raise ValueError("xlo_maxpool2d rejected the sizes")
    return y


def global_avgpool(x) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = x.shape
    y = np.empty((n, c, 1, 1), dtype=np.float32)
    if lib().xlo_global_avgpool(_p(x), n, c, h, w, _p(y)) != 0:
        raise ValueError("xlo_global_avgpool rejected the sizes")
    return y


def add(a, b, relu=False) -> np.ndarray:
    a, b = _f32(a), _f32(b)
    if a.shape != b.shape:
        raise ValueError("add: shape mismatch")
    y = np.empty_like(a)
    lib().xlo_add(_p(a), _p(b), a.size, int(bool(relu)), _p(y))
    return y


def concat_channels(a, b) -> np.ndarray:
    a, b = _f32(a), _f32(b)
    n, ca, h, w = a.shape
    nb, cb, hb, wb = b.shape
    if (n, h, w) != (nb, hb, wb):
        raise ValueError("concat: shape mismatch")
    y = np.empty((n, ca + cb, h, w), dtype=np.float32)
    lib().xlo_concat_channels(_p(a), ca, _p(b), cb, n, h * w, _p(y))
    return y


def forward(graph, x: np.ndarray, params: Dict[int, dict], keep_all: bool = False):
    """Evaluate `graph` layer by layer.  Returns the output tensor, or the dict
    of every tensor by id when keep_all is set."""
    t: Dict[int, np.ndarray] = {graph.input_id: _f32(x)}
    for li, L in enumerate(graph.layers):
        if L.op == "conv":
            p = params[li]
            t[L.out] = conv2d(t[L.inputs[0]], p["w"], L.stride, L.pad, L.groups,
                              p.get("scale"), p.get("shift"), L.relu)
        elif L.op == "maxpool":
            t[L.out] = maxpool2d(t[L.inputs[0]], L.k, L.stride, L.pad)
        elif L.op == "gap":
            t[L.out] = global_avgpool(t[L.inputs[0]])
        elif L.op == "add":
            t[L.out] = add(t[L.inputs[0]], t[L.inputs[1]], L.relu)
        elif L.op == "concat":
            t[L.out] = concat_channels(t[L.inputs[0]], t[L.inputs[1]])
        else:
            raise ValueError(f"unknown op {L.op}")
        if tuple(t[L.out].shape) != tuple(graph.shapes[L.out]):
            raise ValueError(f"layer {li}: shape {t[L.out].shape} != declared {graph.shapes[L.out]}")
    return t if keep_all else t[graph.output_id]
