"""ctypes binding of libinfinipot (include/infinipot.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  Tensors are
torch CUDA tensors (torch owns device memory and streams); bf16 caches may be passed as torch.bfloat16
or as int16/uint16 bit patterns.  There is no CPU fallback: if the shared library is missing the import
of any entry point raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libinfinipot.so")

CCD_OK, CCD_NOOP = 0, 1
CCD_EINVAL, CCD_EUNSUPPORTED, CCD_EALIGN, CCD_EWORKSPACE, CCD_ELAUNCH = -1, -2, -3, -4, -5
CCD_FP32, CCD_BF16 = 0, 1
CCD_POOL_NONE, CCD_POOL_MAX, CCD_POOL_AVG = 0, 1, 2
CCD_PATH_AUTO, CCD_PATH_VALU, CCD_PATH_MFMA_SLICES, CCD_PATH_MFMA_UNIT = 0, 1, 2, 3

EXPORTS = ("ccd_workspace_bytes", "ccd_score", "ccd_select", "ccd_compact", "ccd_compress", "ccd_append", "ccd_cr_rope",
           "ccd_compress_rope", "ccd_score_kcat", "ccd_compress_kcat", "ccd_score_lse", "ccd_compress_lse",
           "ccd_nuc_from_logits", "ccd_compress_noalloc", "ccd_profile_enable", "ccd_profile_stages", "ccd_profile_stage_name",
           "ccd_profile_collect", "ccd_strerror")


class ccd_shape_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "L", "Hq", "Hkv", "d", "n_valid", "n_cap", "k", "P", "T", "pool_w", "pool_mode", "dtype")]
    _fields_ += [("scale", ctypes.c_float), ("window", ctypes.c_int32), ("score_path", ctypes.c_int32)]
    _fields_ += [(n, ctypes.c_int64) for n in
                 ("kv_stride_b", "kv_stride_l", "kv_stride_h", "q_stride_b", "q_stride_l", "q_stride_h",
                  "nov_stride_b", "nov_stride_l", "nov_stride_h")]


class CCDError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libinfinipot: {text} (code {code})")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_01518_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sp = ctypes.c_void_p, ctypes.POINTER(ccd_shape_t)
        L.ccd_workspace_bytes.restype = ctypes.c_size_t
        L.ccd_workspace_bytes.argtypes = [sp]
        L.ccd_score.restype = ctypes.c_int
        L.ccd_score.argtypes = [sp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_select.restype = ctypes.c_int
        L.ccd_select.argtypes = [sp, vp, vp, vp]
        L.ccd_compact.restype = ctypes.c_int
        L.ccd_compact.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
        L.ccd_compress.restype = ctypes.c_int
        L.ccd_compress.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_append.restype = ctypes.c_int
        L.ccd_append.argtypes = [sp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp]
        L.ccd_compress_noalloc.restype = ctypes.c_int
        L.ccd_compress_noalloc.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
        L.ccd_cr_rope.restype = ctypes.c_int
        L.ccd_cr_rope.argtypes = [sp, vp, vp, vp, ctypes.c_int32, vp, vp]
        L.ccd_compress_rope.restype = ctypes.c_int
        L.ccd_compress_rope.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_score_lse.restype = ctypes.c_int
        L.ccd_score_lse.argtypes = [sp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_compress_lse.restype = ctypes.c_int
        L.ccd_compress_lse.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_score_kcat.restype = ctypes.c_int
        L.ccd_score_kcat.argtypes = [sp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_compress_kcat.restype = ctypes.c_int
        L.ccd_compress_kcat.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.ccd_nuc_from_logits.restype = ctypes.c_int
        L.ccd_nuc_from_logits.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, vp]
        L.ccd_profile_enable.restype = ctypes.c_int
        L.ccd_profile_enable.argtypes = [ctypes.c_int]
        L.ccd_profile_stages.restype = ctypes.c_int
        L.ccd_profile_stages.argtypes = []
        L.ccd_profile_stage_name.restype = ctypes.c_char_p
        L.ccd_profile_stage_name.argtypes = [ctypes.c_int]
        L.ccd_profile_collect.restype = ctypes.c_int
        L.ccd_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.ccd_strerror.restype = ctypes.c_char_p
        L.ccd_strerror.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def ccd_strerror(code: int) -> str:
    return lib().ccd_strerror(code).decode()


def _check(code: int) -> int:
    if code < 0:
        raise CCDError(code, ccd_strerror(code))
    return code


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CCD_FP32
    if t.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        return CCD_BF16
    raise TypeError(f"unsupported cache dtype {t.dtype}")


def make_shape(Q_cat, K, novelty, *, k, T=0, pool_w=1, pool_mode=CCD_POOL_MAX, scale=0.0, n_valid=None,
               window=0, score_path=CCD_PATH_AUTO) -> ccd_shape_t:
    """Shape descriptor from tensor geometry: Q_cat [B,L,Hq,P,d], K [B,L,Hkv,n_cap,d], novelty [B,n] or
    [B,L,Hkv,n_cap] (may be None when T == 0).  Q_cat may be None for calls that do not read it."""
    B, L, Hkv, n_cap, d = K.shape
    s = ccd_shape_t()
    s.B, s.L, s.Hkv, s.d, s.n_cap = B, L, Hkv, d, n_cap
    s.n_valid = n_cap if n_valid is None else n_valid
    s.k, s.T, s.pool_w, s.pool_mode, s.scale = k, T, pool_w, pool_mode, scale
    s.window = window
    s.score_path = score_path
    s.dtype = _dtype_code(K)
    assert K.stride(4) == 1 and K.stride(3) == d, "K rows must be contiguous with stride d"
    s.kv_stride_b, s.kv_stride_l, s.kv_stride_h = K.stride(0), K.stride(1), K.stride(2)
    if Q_cat is not None:
        assert Q_cat.stride(4) == 1 and Q_cat.stride(3) == d
        s.Hq, s.P = Q_cat.shape[2], Q_cat.shape[3]
        s.q_stride_b, s.q_stride_l, s.q_stride_h = Q_cat.stride(0), Q_cat.stride(1), Q_cat.stride(2)
    else:
        s.Hq, s.P = Hkv, 1
        s.q_stride_h = d
    if novelty is not None:
        assert novelty.dtype == torch.float32 and novelty.stride(-1) == 1
        if novelty.dim() == 2:
            s.nov_stride_b = novelty.stride(0)
        else:
            s.nov_stride_b, s.nov_stride_l, s.nov_stride_h = novelty.stride(0), novelty.stride(1), novelty.stride(2)
    return s


def ccd_workspace_bytes(shape: ccd_shape_t) -> int:
    return int(lib().ccd_workspace_bytes(ctypes.byref(shape)))


def alloc_workspace(shape: ccd_shape_t, device="cuda") -> torch.Tensor:
    nbytes = ccd_workspace_bytes(shape)
    if nbytes == 0:
        raise CCDError(CCD_EINVAL, "invalid shape")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def ccd_score(shape, Q_cat, K, novelty, scores, workspace, stream=None) -> int:
    return _check(lib().ccd_score(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(novelty), _ptr(scores),
                                  _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))


def ccd_select(shape, scores, keep_idx, stream=None) -> int:
    return _check(lib().ccd_select(ctypes.byref(shape), _ptr(scores), _ptr(keep_idx), _stream(stream)))


def ccd_append(shape, K, V, novelty, K_new, V_new, novelty_new, stream=None) -> int:
    """Rows shape.n_valid .. + count - 1 of every unit of K, V (and novelty) <- the chunk K_new, V_new [B,L,Hkv,count,d]
    (dense) and novelty_new [B,count]; the caller raises n_valid afterwards."""
    assert K_new.is_contiguous() and V_new.is_contiguous() and (novelty_new is None or novelty_new.is_contiguous())
    return _check(lib().ccd_append(ctypes.byref(shape), _ptr(K), _ptr(V), _ptr(novelty), _ptr(K_new), _ptr(V_new),
                                   _ptr(novelty_new), int(K_new.shape[3]), _stream(stream)))


def ccd_compact(shape, K_src, V_src, keep_idx, K_dst, V_dst, novelty_inout=None, stream=None) -> int:
    return _check(lib().ccd_compact(ctypes.byref(shape), _ptr(K_src), _ptr(V_src), _ptr(keep_idx), _ptr(K_dst),
                                    _ptr(V_dst), _ptr(novelty_inout), _stream(stream)))


def ccd_compress(shape, Q_cat, K, V, novelty, keep_idx, workspace, scores=None, stream=None) -> int:
    return _check(lib().ccd_compress(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(V), _ptr(novelty), _ptr(scores),
                                     _ptr(keep_idx), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                     _stream(stream)))


NOALLOC_WORKSPACE_BYTES = 16 << 20


def ccd_compress_noalloc(shape, Q_cat, K, V, novelty, keep_idx, scores=None, stream=None) -> int:
    """ccd_compress on the workspace the library holds itself (no allocation anywhere in the call)."""
    return _check(lib().ccd_compress_noalloc(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(V), _ptr(novelty), _ptr(scores),
                                             _ptr(keep_idx), _stream(stream)))


def ccd_nuc_from_logits(logits, labels, novelty, stream=None) -> int:
    """novelty[r] = cross entropy of labels[r] under logits[r, :]; logits [..., V] with a dense last axis and equally
    spaced rows, labels and novelty with the same leading shape (flattened row-major)."""
    V = logits.shape[-1]
    assert logits.stride(-1) == 1 and labels.dtype == torch.int32 and novelty.dtype == torch.float32
    assert labels.is_contiguous() and novelty.is_contiguous() and labels.numel() == novelty.numel()
    lead = logits.shape[:-1]
    rows = int(np.prod(lead)) if len(lead) else 1
    flat = logits.reshape(rows, V) if rows else logits
    assert rows == 0 or flat.data_ptr() == logits.data_ptr(), "rows must be equally spaced"
    esz = logits.element_size()
    stride = flat.stride(0) if rows > 1 else (V * esz + 15) // 16 * 16 // esz   # a single row: any legal stride
    return _check(lib().ccd_nuc_from_logits(_ptr(logits), _ptr(labels), _ptr(novelty), rows, V, stride,
                                            _dtype_code(logits), _stream(stream)))


def ccd_cr_rope(shape, K, rope_cos, rope_sin, count, K_rot, stream=None) -> int:
    return _check(lib().ccd_cr_rope(ctypes.byref(shape), _ptr(K), _ptr(rope_cos), _ptr(rope_sin), int(count), _ptr(K_rot),
                                    _stream(stream)))


def ccd_compress_rope(shape, Q_cat, K, V, novelty, keep_idx, rope_cos, rope_sin, K_rot, workspace, scores=None,
                      K_score=None, K_cap=None, lse=None, stream=None) -> int:
    assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32)
    return _check(lib().ccd_compress_rope(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(V), _ptr(novelty), _ptr(scores),
                                          _ptr(keep_idx), _ptr(K_score), _ptr(K_cap), _ptr(lse), _ptr(rope_cos), _ptr(rope_sin),
                                          _ptr(K_rot), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                          _stream(stream)))


def ccd_score_kcat(shape, Q_cat, K, K_cap, novelty, scores, workspace, stream=None) -> int:
    """K_cap [B, L, Hkv, P, d], contiguous."""
    assert K_cap is None or K_cap.is_contiguous()
    return _check(lib().ccd_score_kcat(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(K_cap), _ptr(novelty), _ptr(scores),
                                       _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))


def ccd_score_lse(shape, Q_cat, K, lse, novelty, scores, workspace, stream=None) -> int:
    """lse [B, L, Hq, P] fp32, contiguous: the natural-log-sum-exp of every CaP query's attention row."""
    assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32)
    return _check(lib().ccd_score_lse(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(lse), _ptr(novelty), _ptr(scores),
                                      _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(stream)))


def ccd_compress_lse(shape, Q_cat, K, V, lse, novelty, keep_idx, workspace, scores=None, stream=None) -> int:
    assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32)
    return _check(lib().ccd_compress_lse(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(V), _ptr(lse), _ptr(novelty),
                                         _ptr(scores), _ptr(keep_idx), _ptr(workspace),
                                         0 if workspace is None else workspace.numel(), _stream(stream)))


def ccd_compress_kcat(shape, Q_cat, K, V, K_cap, novelty, keep_idx, workspace, scores=None, stream=None) -> int:
    assert K_cap is None or K_cap.is_contiguous()
    return _check(lib().ccd_compress_kcat(ctypes.byref(shape), _ptr(Q_cat), _ptr(K), _ptr(V), _ptr(K_cap), _ptr(novelty),
                                          _ptr(scores), _ptr(keep_idx), _ptr(workspace),
                                          0 if workspace is None else workspace.numel(), _stream(stream)))


def ccd_profile_enable(on: bool) -> int:
    return _check(lib().ccd_profile_enable(1 if on else 0))


def ccd_profile_collect():
    """(dict stage name -> total ms, number of ccd_compress calls covered) since profiling was enabled."""
    n = lib().ccd_profile_stages()
    ms = (ctypes.c_double * n)()
    calls = ctypes.c_int64(0)
    _check(lib().ccd_profile_collect(ms, ctypes.byref(calls)))
    return {lib().ccd_profile_stage_name(i).decode(): ms[i] for i in range(n)}, calls.value
