"""CPU oracle for the memory-bound CNN layers: numpy front end.

TEST INFRASTRUCTURE ONLY.  This package wraps ``cnnmem_ref.c`` (plain C, host
pointers) with ctypes so that tests, the smoke check and the benchmark's
``cpu_baseline`` leg can call it on numpy arrays.  It imports nothing from the
GPU package and the GPU package imports nothing from here.

Functions mirror the C ones: ``transform`` (Section IV.C), ``pool``
(Equation 2 / Section II.A) and ``softmax`` (Section II.A, steps 1-5).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

NCHW, CHWN = 0, 1
POOL_MAX, POOL_AVG = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cnnmem_ref.c")
_LIB = os.path.join(_HERE, "libcnnmem_ref.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc into ``oracle/libcnnmem_ref.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.c_void_p
        i = ctypes.c_int
        lib.cnnmem_ref_transform.argtypes = [fp, fp, i, i, i, i, i, i]
        lib.cnnmem_ref_pool_out_dims.argtypes = [i] * 8 + [ctypes.POINTER(i)] * 2
        lib.cnnmem_ref_pool.argtypes = [fp, fp] + [i] * 12
        lib.cnnmem_ref_softmax.argtypes = [fp, fp, i, i]
        lib.cnnmem_ref_naive_pool_loads_1d.argtypes = [i, i, i]
        lib.cnnmem_ref_choose_layout.argtypes = [i] * 5
        lib.cnnmem_ref_choose_layout.restype = i
        ip = ctypes.POINTER(i)
        lib.cnnmem_ref_plan_layouts.argtypes = [ip, ip, ip, i, i, i, i, i, ip, ip]
        lib.cnnmem_ref_plan_layouts.restype = i
        lib.cnnmem_ref_permute.argtypes = [fp, fp, ip, ip]
        lib.cnnmem_ref_permute.restype = i
        lib.cnnmem_ref_relayout.argtypes = [fp, fp, i, i, i, i, ctypes.c_char_p, ctypes.c_char_p]
        lib.cnnmem_ref_relayout.restype = i
        lib.cnnmem_ref_widen16.argtypes = [ctypes.c_uint, i]
        lib.cnnmem_ref_widen16.restype = ctypes.c_double
        lib.cnnmem_ref_narrow16.argtypes = [ctypes.c_double, i]
        lib.cnnmem_ref_narrow16.restype = ctypes.c_uint
        lib.cnnmem_ref_transform16.argtypes = [fp, fp, i, i, i, i, i, i]
        lib.cnnmem_ref_transform16.restype = i
        lib.cnnmem_ref_pool16.argtypes = [fp, fp] + [i] * 13
        lib.cnnmem_ref_pool16.restype = i
        lib.cnnmem_ref_softmax16.argtypes = [fp, fp, i, i, i]
        lib.cnnmem_ref_softmax16.restype = i
        lib.cnnmem_ref_pool_backward.argtypes = [fp, fp, fp] + [i] * 12
        lib.cnnmem_ref_pool_backward.restype = i
        lib.cnnmem_ref_softmax_backward.argtypes = [fp, fp, fp, i, i]
        lib.cnnmem_ref_softmax_backward.restype = i
        lib.cnnmem_ref_permute16.argtypes = [fp, fp, ip, ip]
        lib.cnnmem_ref_permute16.restype = i
        lib.cnnmem_ref_index.argtypes = [i] * 9
        lib.cnnmem_ref_index.restype = ctypes.c_ulonglong
        for name in ("cnnmem_ref_transform", "cnnmem_ref_pool_out_dims", "cnnmem_ref_pool",
                     "cnnmem_ref_softmax", "cnnmem_ref_naive_pool_loads_1d", "cnnmem_ref_threads",
                     "cnnmem_ref_set_threads"):
            getattr(lib, name).restype = i
        _lib = lib
    return _lib


def _check(status: int, what: str) -> None:
    if status != 0:
        raise ValueError(f"oracle {what} failed with status {status}")


def _f32(a: np.ndarray) -> np.ndarray:
    if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("oracle takes C-contiguous float32 arrays")
    return a


def threads() -> int:
    """Threads the oracle's OpenMP loops will use."""
    return int(_load().cnnmem_ref_threads())


def set_threads(n: int) -> None:
    """Caps the threads of the oracle's loops (timing aid; results do not depend on it)."""
    _load().cnnmem_ref_set_threads.argtypes = [ctypes.c_int]
    _load().cnnmem_ref_set_threads(int(n))


def shape_of(layout: int, N: int, C: int, H: int, W: int):
    """numpy shape of an N x C x H x W tensor stored in ``layout``."""
    return (N, C, H, W) if layout == NCHW else (C, H, W, N)


def transform(src: np.ndarray, N: int, C: int, H: int, W: int,
              src_layout: int, dst_layout: int) -> np.ndarray:
    src = _f32(src)
    assert src.size == N * C * H * W
    dst = np.empty(shape_of(dst_layout, N, C, H, W), dtype=np.float32)
    _check(_load().cnnmem_ref_transform(src.ctypes.data, dst.ctypes.data, N, C, H, W,
                                        src_layout, dst_layout), "transform")
    return dst


def permute(src: np.ndarray, dims, perm) -> np.ndarray:
    """Axis permutation of a 4-D tensor: destination axis i is source axis ``perm[i]`` (Section I)."""
    src = _f32(src)
    assert src.size == int(np.prod(dims)) and len(dims) == 4 and len(perm) == 4
    dst = np.empty(tuple(dims[p] for p in perm), dtype=np.float32)
    _check(_load().cnnmem_ref_permute(src.ctypes.data, dst.ctypes.data, (ctypes.c_int * 4)(*dims),
                                      (ctypes.c_int * 4)(*perm)), "permute")
    return dst


def relayout(src: np.ndarray, N: int, C: int, H: int, W: int, src_layout: str, dst_layout: str) -> np.ndarray:
    """Storage-order change between two spelled layouts such as "NCHW" -> "NHWC" (Section I, IV.A)."""
    src = _f32(src)
    assert src.size == N * C * H * W
    ext = dict(N=N, C=C, H=H, W=W)
    dst = np.empty(tuple(ext[l] for l in dst_layout) if len(dst_layout) == 4 else (N * C * H * W,), dtype=np.float32)
    _check(_load().cnnmem_ref_relayout(src.ctypes.data, dst.ctypes.data, N, C, H, W,
                                       src_layout.encode(), dst_layout.encode()), "relayout")
    return dst


def pool_out_dims(H, W, kh, kw, sh, sw, ph, pw):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    _check(_load().cnnmem_ref_pool_out_dims(H, W, kh, kw, sh, sw, ph, pw,
                                            ctypes.byref(ho), ctypes.byref(wo)), "pool_out_dims")
    return ho.value, wo.value


def pool(src: np.ndarray, N: int, C: int, H: int, W: int, layout: int, mode: int,
         kh: int, kw: int, sh: int, sw: int, ph: int = 0, pw: int = 0) -> np.ndarray:
    src = _f32(src)
    assert src.size == N * C * H * W
    Ho, Wo = pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
    dst = np.empty(shape_of(layout, N, C, Ho, Wo), dtype=np.float32)
    _check(_load().cnnmem_ref_pool(src.ctypes.data, dst.ctypes.data, N, C, H, W, layout, mode,
                                   kh, kw, sh, sw, ph, pw), "pool")
    return dst


def pool_backward(src, ddst: np.ndarray, N: int, C: int, H: int, W: int, layout: int, mode: int,
                  kh: int, kw: int, sh: int, sw: int, ph: int = 0, pw: int = 0) -> np.ndarray:
    """Gradient of ``pool`` with respect to its input; ``src`` may be None for the average."""
    ddst = _f32(ddst)
    Ho, Wo = pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
    assert ddst.size == N * C * Ho * Wo
    if src is not None:
        src = _f32(src)
        assert src.size == N * C * H * W
    dsrc = np.empty(shape_of(layout, N, C, H, W), dtype=np.float32)
    _check(_load().cnnmem_ref_pool_backward(src.ctypes.data if src is not None else None, ddst.ctypes.data,
                                            dsrc.ctypes.data, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw),
           "pool_backward")
    return dsrc


def softmax_backward(probs: np.ndarray, dprobs: np.ndarray) -> np.ndarray:
    """Gradient with respect to the logits, given the softmax output and the gradient arriving at it."""
    probs, dprobs = _f32(probs), _f32(dprobs)
    assert probs.ndim == 2 and probs.shape == dprobs.shape
    N, classes = probs.shape
    out = np.empty_like(probs)
    _check(_load().cnnmem_ref_softmax_backward(probs.ctypes.data, dprobs.ctypes.data, out.ctypes.data, N, classes),
           "softmax_backward")
    return out


def softmax(logits: np.ndarray) -> np.ndarray:
    logits = _f32(logits)
    assert logits.ndim == 2
    N, classes = logits.shape
    probs = np.empty_like(logits)
    _check(_load().cnnmem_ref_softmax(logits.ctypes.data, probs.ctypes.data, N, classes), "softmax")
    return probs


def index(layout: int, N: int, C: int, H: int, W: int, n: int, c: int, h: int, w: int) -> int:
    """Linear index of element (n, c, h, w) of an N x C x H x W tensor stored in ``layout``."""
    return int(_load().cnnmem_ref_index(layout, N, C, H, W, n, c, h, w))


LAYER_CONV, LAYER_POOL, LAYER_OTHER = 0, 1, 2


def choose_layout(kind: int, N: int, C: int, Ct: int, Nt: int) -> int:
    """Preferred layout of one layer (Section IV.A / IV.B); -1 = no preference."""
    return int(_load().cnnmem_ref_choose_layout(kind, N, C, Ct, Nt))


def plan_layouts(layers, Ct: int, Nt: int, input_layout: int, pool_keeps_layout: bool = False):
    """Layout plan for ``layers`` = [(kind, N, C), ...] (Section IV.D).

    Returns (layouts, transform_before, n_transforms)."""
    n = len(layers)
    arr = lambda vals: (ctypes.c_int * n)(*vals)
    kinds, Ns, Cs = arr([l[0] for l in layers]), arr([l[1] for l in layers]), arr([l[2] for l in layers])
    layouts, tb = (ctypes.c_int * n)(), (ctypes.c_int * n)()
    count = _load().cnnmem_ref_plan_layouts(kinds, Ns, Cs, n, Ct, Nt, input_layout, int(pool_keeps_layout),
                                            layouts, tb)
    return list(layouts), list(tb), int(count)


def naive_pool_loads_1d(L: int, k: int, s: int) -> int:
    return int(_load().cnnmem_ref_naive_pool_loads_1d(L, k, s))


# ---- 16-bit storage: arrays of uint16 bit patterns; F16 = IEEE binary16, BF16 = upper half of binary32 ----
F32, F16, BF16 = 0, 1, 2


def _u16(a: np.ndarray) -> np.ndarray:
    if a.dtype != np.uint16 or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("the 16-bit oracle takes C-contiguous uint16 arrays of bit patterns")
    return a


def widen16(bits: int, dtype: int) -> float:
    """Exact value of one 16-bit pattern."""
    return float(_load().cnnmem_ref_widen16(int(bits), dtype))


def narrow16(x: float, dtype: int) -> int:
    """Nearest 16-bit pattern (ties to even) to a double."""
    return int(_load().cnnmem_ref_narrow16(float(x), dtype))


def transform16(src: np.ndarray, N, C, H, W, src_layout, dst_layout) -> np.ndarray:
    src = _u16(src)
    assert src.size == N * C * H * W
    dst = np.empty(shape_of(dst_layout, N, C, H, W), dtype=np.uint16)
    _check(_load().cnnmem_ref_transform16(src.ctypes.data, dst.ctypes.data, N, C, H, W, src_layout, dst_layout),
           "transform16")
    return dst


def pool16(src: np.ndarray, N, C, H, W, layout, mode, kh, kw, sh, sw, ph=0, pw=0, dtype=F16) -> np.ndarray:
    src = _u16(src)
    assert src.size == N * C * H * W
    Ho, Wo = pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
    dst = np.empty(shape_of(layout, N, C, Ho, Wo), dtype=np.uint16)
    _check(_load().cnnmem_ref_pool16(src.ctypes.data, dst.ctypes.data, N, C, H, W, layout, mode,
                                     kh, kw, sh, sw, ph, pw, dtype), "pool16")
    return dst


def softmax16(logits: np.ndarray, dtype=F16) -> np.ndarray:
    logits = _u16(logits)
    assert logits.ndim == 2
    N, classes = logits.shape
    probs = np.empty_like(logits)
    _check(_load().cnnmem_ref_softmax16(logits.ctypes.data, probs.ctypes.data, N, classes, dtype), "softmax16")
    return probs


def permute16(src: np.ndarray, dims, perm) -> np.ndarray:
    """Axis permutation of a tensor of 16-bit words (bit patterns move untouched)."""
    src = _u16(src)
    assert src.size == int(np.prod(dims)) and len(dims) == 4 and len(perm) == 4
    dst = np.empty(tuple(dims[p] for p in perm), dtype=np.uint16)
    _check(_load().cnnmem_ref_permute16(src.ctypes.data, dst.ctypes.data, (ctypes.c_int * 4)(*dims),
                                        (ctypes.c_int * 4)(*perm)), "permute16")
    return dst
