"""ctypes binding of libcnnmem.so: argument marshalling only.

``cnnmem_*`` mirror the C entry points one to one and return the status code.
``transform`` / ``pool`` / ``softmax`` allocate the output with torch (device
memory is torch's job here), call the entry point on torch's current stream
and raise :class:`CnnmemError` on a non-zero status.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

NCHW, CHWN = 0, 1
POOL_MAX, POOL_AVG = 0, 1
LAYER_CONV, LAYER_POOL, LAYER_OTHER = 0, 1, 2
POOL_PREFERS_CHWN, POOL_KEEPS_LAYOUT = 0, 1
F32, F16, BF16 = 0, 1, 2                       # storage formats (cnnmem.h: CNNMEM_F32 / _F16 / _BF16)
_DTYPE_OF = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}


class PoolTuning(ctypes.Structure):
    """Launch-shape choices of a pooling call (``cnnmem_pool_tuning``); zeros = library defaults."""
    _fields_ = [("rows_per_lane", ctypes.c_int), ("cols_per_lane", ctypes.c_int),
                ("workgroups_per_cu", ctypes.c_int), ("nchw_kernel", ctypes.c_int), ("slab_lanes", ctypes.c_int)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class _Layer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("N", ctypes.c_int), ("C", ctypes.c_int)]

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcnnmem.so")
_lib = None


class CnnmemError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {cnnmem_status_string(status)} (status {status})")
        self.status = status


def library() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_1610_03618_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(_LIB_PATH)
        i, p = ctypes.c_int, ctypes.c_void_p
        lib.cnnmem_transform.argtypes = [p, p, i, i, i, i, i, i, p]
        lib.cnnmem_permute.argtypes = [p, p, ctypes.POINTER(i), ctypes.POINTER(i), p]
        lib.cnnmem_permute.restype = i
        lib.cnnmem_relayout.argtypes = [p, p, i, i, i, i, ctypes.c_char_p, ctypes.c_char_p, p]
        lib.cnnmem_relayout.restype = i
        lib.cnnmem_permute_dtype.argtypes = [p, p, ctypes.POINTER(i), ctypes.POINTER(i), i, p]
        lib.cnnmem_permute_dtype.restype = i
        lib.cnnmem_relayout_dtype.argtypes = [p, p, i, i, i, i, ctypes.c_char_p, ctypes.c_char_p, i, p]
        lib.cnnmem_relayout_dtype.restype = i
        lib.cnnmem_pool_backward.argtypes = [p, p, p] + [i] * 12 + [p]
        lib.cnnmem_pool_backward.restype = i
        lib.cnnmem_softmax_backward.argtypes = [p, p, p, i, i, p]
        lib.cnnmem_softmax_backward.restype = i
        lib.cnnmem_transform_dtype.argtypes = [p, p, i, i, i, i, i, i, i, p]
        lib.cnnmem_pool_dtype.argtypes = [p, p] + [i] * 13 + [p]
        lib.cnnmem_softmax_dtype.argtypes = [p, p, i, i, i, p]
        for name in ("cnnmem_transform_dtype", "cnnmem_pool_dtype", "cnnmem_softmax_dtype"):
            getattr(lib, name).restype = i
        lib.cnnmem_pool_out_dims.argtypes = [i] * 8 + [ctypes.POINTER(i)] * 2
        lib.cnnmem_pool.argtypes = [p, p] + [i] * 12 + [p]
        lib.cnnmem_pool_tuned.argtypes = [p, p] + [i] * 12 + [ctypes.POINTER(PoolTuning), p]
        lib.cnnmem_pool_tuned.restype = i
        lib.cnnmem_softmax.argtypes = [p, p, i, i, p]
        ip = ctypes.POINTER(i)
        lib.cnnmem_choose_layout.argtypes = [i, i, i, i, i, ip]
        lib.cnnmem_choose_layout.restype = i
        lib.cnnmem_plan_layouts.argtypes = [ctypes.POINTER(_Layer), i, i, i, i, i, ip, ip, ip]
        lib.cnnmem_plan_layouts.restype = i
        lib.cnnmem_status_string.argtypes = [i]
        lib.cnnmem_status_string.restype = ctypes.c_char_p
        lib.cnnmem_version.argtypes = []
        for name in ("cnnmem_transform", "cnnmem_pool_out_dims", "cnnmem_pool", "cnnmem_softmax",
                     "cnnmem_version"):
            getattr(lib, name).restype = i
        _lib = lib
    return _lib


_HOOKS_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcnnmem_testhooks.so")
_hooks = None


def test_hooks() -> ctypes.CDLL:
    """The host-only hooks of the CPU test-suite (include/cnnmem_debug.h), a library of their own."""
    global _hooks
    if _hooks is None:
        if not os.path.exists(_HOOKS_PATH):
            raise RuntimeError(f"{_HOOKS_PATH} is missing: build it with `python -m paper_1610_03618_amd.build`")
        lib = ctypes.CDLL(_HOOKS_PATH)
        i = ctypes.c_int
        lib.cnnmem_debug_canonical_permutation.argtypes = [ctypes.POINTER(i), ctypes.POINTER(i), ctypes.POINTER(i),
                                                           ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(i)]
        lib.cnnmem_debug_canonical_permutation.restype = i
        lib.cnnmem_debug_fastdiv.argtypes = [ctypes.c_uint, ctypes.c_uint]
        lib.cnnmem_debug_fastdiv.restype = ctypes.c_uint
        lib.cnnmem_debug_smalldiv_mismatches.argtypes = [ctypes.c_uint, ctypes.c_uint]
        lib.cnnmem_debug_smalldiv_mismatches.restype = ctypes.c_longlong
        lib.cnnmem_debug_xcd_tile.argtypes = [ctypes.c_uint, ctypes.c_uint]
        lib.cnnmem_debug_xcd_tile.restype = ctypes.c_uint
        _hooks = lib
    return _hooks


def _ptr(t, dtype: int = F32, numel: Optional[int] = None) -> Optional[int]:
    """Device address of a torch tensor (or a raw integer address / None).

    ``numel``: the elements the call will read or write there.  The C ABI takes bare pointers and cannot know
    a buffer's size, so this is the one place a tensor that is too small can be refused before a kernel runs
    past its end."""
    if t is None or isinstance(t, int):
        return t
    if not isinstance(t, torch.Tensor):
        raise TypeError("expected a torch tensor or an integer address")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"tensor of {t.numel()} elements where the call needs {numel}")
    if t.device.type != "cuda":
        raise ValueError("cnnmem works on GPU memory only (got a CPU tensor)")
    if _DTYPE_OF.get(t.dtype) != dtype or not t.is_contiguous():
        raise ValueError("cnnmem takes contiguous tensors of the stated storage format "
                         "(float32 unless a dtype is given)")
    return t.data_ptr()


def _prod(*extents) -> Optional[int]:
    """Element count of a tensor with these extents; None when an extent is not positive (the library then
    rejects the call itself)."""
    n = 1
    for e in extents:
        if e <= 0:
            return None
        n *= e
    return n


def _pooled(N, C, H, W, kh, kw, sh, sw, ph, pw) -> Optional[int]:
    if min(N, C, H, W, kh, kw, sh, sw) <= 0 or ph < 0 or pw < 0 or H + 2 * ph < kh or W + 2 * pw < kw:
        return None
    return N * C * ((H + 2 * ph - kh) // sh + 1) * ((W + 2 * pw - kw) // sw + 1)


def dtype_of(t: torch.Tensor) -> int:
    """Storage-format tag of a torch tensor (float32 / float16 / bfloat16)."""
    try:
        return _DTYPE_OF[t.dtype]
    except KeyError:
        raise ValueError("cnnmem stores float32, float16 or bfloat16") from None


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return stream or None


# ---- one-to-one mirrors of the C entry points (return the status code) ----

def cnnmem_transform(src, dst, N, C, H, W, src_layout, dst_layout, stream=None) -> int:
    n = _prod(N, C, H, W)
    return library().cnnmem_transform(_ptr(src, F32, n), _ptr(dst, F32, n), N, C, H, W, src_layout, dst_layout,
                                      _stream(stream))


def cnnmem_permute(src, dst, dims, perm, stream=None) -> int:
    n = _prod(*dims)
    return library().cnnmem_permute(_ptr(src, F32, n), _ptr(dst, F32, n), (ctypes.c_int * 4)(*dims),
                                    (ctypes.c_int * 4)(*perm), _stream(stream))


def cnnmem_relayout(src, dst, N, C, H, W, src_layout: str, dst_layout: str, stream=None) -> int:
    n = _prod(N, C, H, W)
    return library().cnnmem_relayout(_ptr(src, F32, n), _ptr(dst, F32, n), N, C, H, W, src_layout.encode(),
                                     dst_layout.encode(), _stream(stream))


def cnnmem_permute_dtype(src, dst, dims, perm, dtype, stream=None) -> int:
    n = _prod(*dims)
    return library().cnnmem_permute_dtype(_ptr(src, dtype, n), _ptr(dst, dtype, n), (ctypes.c_int * 4)(*dims),
                                          (ctypes.c_int * 4)(*perm), dtype, _stream(stream))


def cnnmem_relayout_dtype(src, dst, N, C, H, W, src_layout: str, dst_layout: str, dtype, stream=None) -> int:
    n = _prod(N, C, H, W)
    return library().cnnmem_relayout_dtype(_ptr(src, dtype, n), _ptr(dst, dtype, n), N, C, H, W, src_layout.encode(),
                                           dst_layout.encode(), dtype, _stream(stream))


def cnnmem_debug_canonical_permutation(dims, perm):
    """(status, rank, merged source extents, permutation over them): host-only debug hook."""
    rank = ctypes.c_int(0)
    cd, cp = (ctypes.c_longlong * 4)(), (ctypes.c_int * 4)()
    st = test_hooks().cnnmem_debug_canonical_permutation((ctypes.c_int * 4)(*dims), (ctypes.c_int * 4)(*perm),
                                                      ctypes.byref(rank), cd, cp)
    return st, rank.value, list(cd)[:rank.value], list(cp)[:rank.value]


def cnnmem_pool_backward(src, ddst, dsrc, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, stream=None) -> int:
    n, no = _prod(N, C, H, W), _pooled(N, C, H, W, kh, kw, sh, sw, ph, pw)
    return library().cnnmem_pool_backward(_ptr(src, F32, n), _ptr(ddst, F32, no), _ptr(dsrc, F32, n), N, C, H, W, layout,
                                          mode, kh, kw, sh, sw, ph, pw, _stream(stream))


def cnnmem_softmax_backward(probs, dprobs, dlogits, N, classes, stream=None) -> int:
    n = _prod(N, classes)
    return library().cnnmem_softmax_backward(_ptr(probs, F32, n), _ptr(dprobs, F32, n), _ptr(dlogits, F32, n), N, classes,
                                             _stream(stream))


def cnnmem_transform_dtype(src, dst, N, C, H, W, src_layout, dst_layout, dtype, stream=None) -> int:
    n = _prod(N, C, H, W)
    return library().cnnmem_transform_dtype(_ptr(src, dtype, n), _ptr(dst, dtype, n), N, C, H, W, src_layout, dst_layout,
                                            dtype, _stream(stream))


def cnnmem_pool_dtype(src, dst, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, dtype, stream=None) -> int:
    n, no = _prod(N, C, H, W), _pooled(N, C, H, W, kh, kw, sh, sw, ph, pw)
    return library().cnnmem_pool_dtype(_ptr(src, dtype, n), _ptr(dst, dtype, no), N, C, H, W, layout, mode, kh, kw, sh, sw,
                                       ph, pw, dtype, _stream(stream))


def cnnmem_softmax_dtype(logits, probs, N, classes, dtype, stream=None) -> int:
    n = _prod(N, classes)
    return library().cnnmem_softmax_dtype(_ptr(logits, dtype, n), _ptr(probs, dtype, n), N, classes, dtype,
                                          _stream(stream))


def cnnmem_pool_out_dims(H, W, kh, kw, sh, sw, ph, pw) -> Tuple[int, int, int]:
    ho, wo = ctypes.c_int(0), ctypes.c_int(0)
    st = library().cnnmem_pool_out_dims(H, W, kh, kw, sh, sw, ph, pw, ctypes.byref(ho), ctypes.byref(wo))
    return st, ho.value, wo.value


def cnnmem_pool(src, dst, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, stream=None) -> int:
    n, no = _prod(N, C, H, W), _pooled(N, C, H, W, kh, kw, sh, sw, ph, pw)
    return library().cnnmem_pool(_ptr(src, F32, n), _ptr(dst, F32, no), N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw,
                                 _stream(stream))


def _tuning(tuning):
    if tuning is None or isinstance(tuning, PoolTuning):
        return tuning
    return PoolTuning(**tuning)


def cnnmem_pool_tuned(src, dst, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, tuning=None, stream=None) -> int:
    """``tuning``: a :class:`PoolTuning`, a dict of its fields, or None."""
    t = _tuning(tuning)
    n, no = _prod(N, C, H, W), _pooled(N, C, H, W, kh, kw, sh, sw, ph, pw)
    return library().cnnmem_pool_tuned(_ptr(src, F32, n), _ptr(dst, F32, no), N, C, H, W, layout, mode, kh, kw, sh, sw,
                                       ph, pw, ctypes.byref(t) if t is not None else None, _stream(stream))


def cnnmem_softmax(logits, probs, N, classes, stream=None) -> int:
    n = _prod(N, classes)
    return library().cnnmem_softmax(_ptr(logits, F32, n), _ptr(probs, F32, n), N, classes, _stream(stream))


def cnnmem_choose_layout(kind: int, N: int, C: int, Ct: int, Nt: int, default: int = NCHW) -> Tuple[int, int]:
    """(status, layout); ``default`` is what a layer without a preference reports."""
    out = ctypes.c_int(default)
    st = library().cnnmem_choose_layout(kind, N, C, Ct, Nt, ctypes.byref(out))
    return st, out.value


def cnnmem_plan_layouts(layers, Ct: int, Nt: int, input_layout: int, pool_policy: int = POOL_PREFERS_CHWN):
    """(status, layouts, transform_before, n_transforms) for ``layers`` = [(kind, N, C), ...]."""
    n = len(layers)
    arr = (_Layer * max(n, 1))(*[_Layer(*l) for l in layers])
    layouts, tb, cnt = (ctypes.c_int * max(n, 1))(), (ctypes.c_int * max(n, 1))(), ctypes.c_int(0)
    st = library().cnnmem_plan_layouts(arr, n, Ct, Nt, input_layout, pool_policy, layouts, tb, ctypes.byref(cnt))
    return st, list(layouts)[:n], list(tb)[:n], cnt.value


def cnnmem_status_string(status: int) -> str:
    return library().cnnmem_status_string(status).decode()


def cnnmem_version() -> int:
    return library().cnnmem_version()


# ---- conveniences: allocate the output, raise on error ----

def _shape(layout, N, C, H, W):
    return (N, C, H, W) if layout == NCHW else (C, H, W, N)


def transform(src: torch.Tensor, N, C, H, W, src_layout, dst_layout, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty(_shape(dst_layout, N, C, H, W), dtype=src.dtype, device=src.device)
    st = cnnmem_transform_dtype(src, out, N, C, H, W, src_layout, dst_layout, dtype_of(src), stream)
    if st:
        raise CnnmemError(st, "cnnmem_transform")
    return out


def permute(src: torch.Tensor, dims, perm, out=None, stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty(tuple(dims[a] for a in perm), dtype=src.dtype, device=src.device)
    st = cnnmem_permute_dtype(src, out, dims, perm, dtype_of(src), stream)
    if st:
        raise CnnmemError(st, "cnnmem_permute")
    return out


def relayout(src: torch.Tensor, N, C, H, W, src_layout: str, dst_layout: str, out=None, stream=None) -> torch.Tensor:
    if out is None:
        ext = dict(N=N, C=C, H=H, W=W)
        shape = tuple(ext.get(l, 0) for l in dst_layout) if len(dst_layout) == 4 else (N * C * H * W,)
        out = torch.empty(shape if all(shape) else (N * C * H * W,), dtype=src.dtype, device=src.device)
    st = cnnmem_relayout_dtype(src, out, N, C, H, W, src_layout, dst_layout, dtype_of(src), stream)
    if st:
        raise CnnmemError(st, "cnnmem_relayout")
    return out


def pool(src: torch.Tensor, N, C, H, W, layout, mode, kh, kw, sh, sw, ph=0, pw=0, out=None,
         stream=None, tuning=None) -> torch.Tensor:
    st, Ho, Wo = cnnmem_pool_out_dims(H, W, kh, kw, sh, sw, ph, pw)
    if st:
        raise CnnmemError(st, "cnnmem_pool_out_dims")
    if out is None:
        out = torch.empty(_shape(layout, N, C, Ho, Wo), dtype=src.dtype, device=src.device)
    if dtype_of(src) != F32:
        st = cnnmem_pool_dtype(src, out, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, dtype_of(src), stream)
    else:
        st = cnnmem_pool_tuned(src, out, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, tuning, stream)
    if st:
        raise CnnmemError(st, "cnnmem_pool")
    return out


def pool_backward(src, ddst: torch.Tensor, N, C, H, W, layout, mode, kh, kw, sh, sw, ph=0, pw=0, out=None,
                  stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty(_shape(layout, N, C, H, W), dtype=torch.float32, device=ddst.device)
    st = cnnmem_pool_backward(src, ddst, out, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, stream)
    if st:
        raise CnnmemError(st, "cnnmem_pool_backward")
    return out


def softmax_backward(probs: torch.Tensor, dprobs: torch.Tensor, out=None, stream=None) -> torch.Tensor:
    N, classes = probs.shape
    if out is None:
        out = torch.empty_like(probs)
    st = cnnmem_softmax_backward(probs, dprobs, out, N, classes, stream)
    if st:
        raise CnnmemError(st, "cnnmem_softmax_backward")
    return out


def softmax(logits: torch.Tensor, out=None, stream=None) -> torch.Tensor:
    N, classes = logits.shape
    if out is None:
        out = torch.empty_like(logits)
    st = cnnmem_softmax_dtype(logits, out, N, classes, dtype_of(logits), stream)
    if st:
        raise CnnmemError(st, "cnnmem_softmax")
    return out
