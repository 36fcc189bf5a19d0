"""ctypes access to the fp64 C operators of the oracle (test infrastructure only)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vpe_oracle.c")
_LIB = os.path.join(_HERE, "libvpe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile vpe_oracle.c with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.vo_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().vo_num_threads())


def set_num_threads(n: int) -> None:
    lib().vo_set_num_threads(C.c_int(n))


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def patch_embed(img, w, b, ps: int = 14):
    img, w, b = _d(img), _d(w), _d(b)
    _, H, W = img.shape
    D = w.shape[0]
    out = np.empty(((H // ps) * (W // ps), D))
    lib().vo_patch_embed(_p(img), H, W, ps, _p(w), _p(b), D, _p(out))
    return out


def layernorm(x, g, b, eps: float):
    x, g, b = _d(x), _d(g), _d(b)
    T, D = x.shape
    y = np.empty_like(x)
    lib().vo_layernorm(_p(x), T, D, _p(g), _p(b), C.c_double(eps), _p(y))
    return y


def linear(x, w, b=None):
    x, w = _d(x), _d(w)
    b = None if b is None else _d(b)
    T, K = x.shape
    K2, N = w.shape
    assert K == K2
    y = np.empty((T, N))
    lib().vo_linear(_p(x), T, K, _p(w), _p(b), N, _p(y))
    return y


def attention(qkv, nh: int, dh: int, return_probs: bool = False):
    qkv = _d(qkv)
    N = qkv.shape[0]
    assert qkv.shape[1] == 3 * nh * dh
    out = np.empty((N, nh * dh))
    probs = np.empty((nh, N, N)) if return_probs else None
    lib().vo_attention(_p(qkv), N, nh, dh, _p(out), _p(probs))
    return (out, probs) if return_probs else out


def gelu(x):
    y = _d(x).copy()
    lib().vo_gelu(_p(y), C.c_int64(y.size))
    return y


def swiglu(h):
    h = _d(h)
    T, M2 = h.shape
    out = np.empty((T, M2 // 2))
    lib().vo_swiglu(_p(h), T, M2 // 2, _p(out))
    return out


def scale_residual(x, m, gamma):
    x = _d(x).copy()
    m, gamma = _d(m), _d(gamma)
    T, D = x.shape
    lib().vo_scale_residual(_p(x), _p(m), _p(gamma), T, D)
    return x


def conv3x3(inp, w, b, relu: bool = False):
    inp, w = _d(inp), _d(w)
    b = None if b is None else _d(b)
    Cin, H, W = inp.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin, 3, 3)
    out = np.empty((Cout, H, W))
    lib().vo_conv3x3(_p(inp), Cin, H, W, _p(w), _p(b), Cout, int(relu), _p(out))
    return out


def conv1x1(inp, w, b):
    inp, w = _d(inp), _d(w)
    b = None if b is None else _d(b)
    Cin = inp.shape[0]
    HW = int(np.prod(inp.shape[1:]))
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin)
    out = np.empty((Cout,) + inp.shape[1:])
    lib().vo_conv1x1(_p(inp), Cin, C.c_int64(HW), _p(w), _p(b), Cout, _p(out))
    return out


def bilinear(inp, H: int, W: int):
    inp = _d(inp)
    Cc, h, w = inp.shape
    out = np.empty((Cc, H, W))
    lib().vo_bilinear(_p(inp), Cc, h, w, H, W, _p(out))
    return out


def conv3x3_s2(inp, w, b):
    inp, w = _d(inp), _d(w)
    b = None if b is None else _d(b)
    Cin, H, W = inp.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin, 3, 3)
    out = np.empty((Cout, (H - 1) // 2 + 1, (W - 1) // 2 + 1))
    lib().vo_conv3x3_s2(_p(inp), Cin, H, W, _p(w), _p(b), Cout, _p(out))
    return out


def conv_transpose(inp, w, b, stride: int):
    inp, w = _d(inp), _d(w)
    b = None if b is None else _d(b)
    Cin, H, W = inp.shape
    Cout = w.shape[1]
    assert w.shape == (Cin, Cout, stride, stride)
    out = np.empty((Cout, stride * H, stride * W))
    lib().vo_conv_transpose(_p(inp), Cin, H, W, _p(w), _p(b), Cout, stride, _p(out))
    return out


def bilinear_ac(inp, H: int, W: int):
    inp = _d(inp)
    Cc, h, w = inp.shape
    out = np.empty((Cc, H, W))
    lib().vo_bilinear_ac(_p(inp), Cc, h, w, H, W, _p(out))
    return out


def argmax_channels(inp):
    inp = _d(inp)
    Cc = inp.shape[0]
    HW = int(np.prod(inp.shape[1:]))
    out = np.empty(inp.shape[1:], dtype=np.int32)
    lib().vo_argmax_channels(_p(inp), Cc, C.c_int64(HW), _p(out))
    return out
