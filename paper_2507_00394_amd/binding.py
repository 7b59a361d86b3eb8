"""Thin ctypes binding of ``libhelix_attn.so``: argument marshalling only.

Every function has the name and argument order of its C entry point (see
``include/helix_attn.h``); tensors are torch device tensors whose ``data_ptr()`` is
handed over, and work is enqueued on torch's current stream.  There is no fallback: a
missing library raises ``HelixLibraryError`` on first use.
"""
from __future__ import annotations

import ctypes
import pathlib

import torch

LIB_PATH = pathlib.Path(__file__).resolve().parent / "csrc" / "libhelix_attn.so"
EXPORTS = ("helix_attn_fwd", "helix_attn_bwd", "helix_attn_bwd_static", "helix_attn_fwd_strided", "helix_attn_bwd_strided",
           "helix_attn_check_strides", "helix_qkv_linear_fwd", "helix_qkv_linear_bwd", "helix_qkv_linear_bwd_workspace_bytes",
           "helix_attn_bwd_workspace_bytes",
           "helix_attn_bwd_preprocess", "helix_attn_bwd_delta_head", "helix_attn_bwd_dkdv", "helix_attn_bwd_dq",
           "helix_attn_device_info", "helix_mfma_probe", "helix_mfma_mix_probe", "helix_status_string", "helix_attn_version")
HELIX_OK = 0
_lib = None


class helix_strides(ctypes.Structure):
    """Element strides (batch, head, row) of a logical [B, H, S, D] view; see the header."""
    _fields_ = [("batch", ctypes.c_longlong), ("head", ctypes.c_longlong), ("row", ctypes.c_longlong)]


class HelixLibraryError(RuntimeError):
    pass


class HelixStatusError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise HelixLibraryError(f"{LIB_PATH} is not built; run `python -m paper_2507_00394_amd.build`")
        L = ctypes.CDLL(str(LIB_PATH))
        vp, fp, i, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.helix_attn_fwd.argtypes = [vp, vp, vp, vp, fp, i, i, i, i, f, i, vp]
        L.helix_attn_bwd.argtypes = [vp, vp, vp, vp, fp, vp, vp, vp, vp, vp, sz, i, i, i, i, f, i, vp]
        L.helix_attn_bwd_static.argtypes = [vp, vp, vp, vp, fp, vp, vp, vp, vp, i, i, i, i, f, i, vp]
        L.helix_attn_bwd_static.restype = i
        sp = ctypes.POINTER(helix_strides)
        L.helix_attn_fwd_strided.argtypes = [vp, sp, vp, sp, vp, sp, vp, sp, fp, i, i, i, i, f, i, vp]
        L.helix_attn_bwd_strided.argtypes = [vp, sp, vp, sp, vp, sp, vp, sp, fp, vp, sp, vp, sp, vp, sp, vp, sp,
                                             vp, sz, i, i, i, i, f, i, vp]
        L.helix_attn_check_strides.argtypes = [sp, i, i, i, i]
        L.helix_attn_check_strides.restype = i
        ll = ctypes.c_longlong
        L.helix_qkv_linear_fwd.argtypes = [vp, ll, vp, ll, vp, ll, i, i, i, vp]
        L.helix_qkv_linear_bwd.argtypes = [vp, ll, vp, ll, vp, ll, vp, ll, fp, ll, vp, sz, i, i, i, vp]
        L.helix_qkv_linear_bwd_workspace_bytes.argtypes = [i, i, i]
        L.helix_qkv_linear_bwd_workspace_bytes.restype = sz
        L.helix_qkv_linear_fwd.restype = i
        L.helix_qkv_linear_bwd.restype = i
        L.helix_attn_bwd_workspace_bytes.argtypes = [i, i, i, i]
        L.helix_attn_bwd_workspace_bytes.restype = sz
        L.helix_attn_bwd_preprocess.argtypes = [vp, vp, fp, vp, i, i, i, i, vp]
        L.helix_attn_bwd_delta_head.argtypes = [vp, vp, vp, vp, fp, vp, i, i, i, i, i, f, i, vp]
        L.helix_attn_bwd_dkdv.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, f, i, vp]
        L.helix_attn_bwd_dq.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, f, i, vp]
        L.helix_status_string.argtypes = [i]
        L.helix_status_string.restype = ctypes.c_char_p
        L.helix_attn_version.argtypes = []
        L.helix_attn_device_info.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.helix_attn_device_info.restype = i
        L.helix_mfma_probe.argtypes = [fp, i, i, i, ctypes.POINTER(ctypes.c_longlong), vp]
        L.helix_mfma_probe.restype = i
        L.helix_mfma_mix_probe.argtypes = [fp, i, i, i, ctypes.POINTER(ctypes.c_longlong), vp]
        L.helix_mfma_mix_probe.restype = i
        for name in ("helix_attn_fwd", "helix_attn_bwd", "helix_attn_fwd_strided", "helix_attn_bwd_strided",
                     "helix_attn_bwd_preprocess", "helix_attn_bwd_delta_head",
                     "helix_attn_bwd_dkdv",
                     "helix_attn_bwd_dq", "helix_attn_version"):
            getattr(L, name).restype = i
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().helix_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check_bf16(name, t, shape):
    if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: need a contiguous CUDA bfloat16 tensor of shape {tuple(shape)}")


def _check_f32(name, t, shape):
    if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: need a contiguous CUDA float32 tensor of shape {tuple(shape)}")


def _raise(status, where):
    if status != HELIX_OK:
        raise HelixStatusError(status, where)


def helix_attn_version() -> int:
    return lib().helix_attn_version()


def helix_attn_device_info():
    """(compute units, peak engine clock in kHz) of the current device."""
    cu, khz = ctypes.c_int(0), ctypes.c_int(0)
    _raise(lib().helix_attn_device_info(ctypes.byref(cu), ctypes.byref(khz)), "helix_attn_device_info")
    return cu.value, khz.value


def helix_mfma_probe(sink, workgroups, iters, random_operands, stream=None) -> int:
    """Enqueues the pure MFMA loop; returns the FLOPs it performs.  `sink`: a CUDA float32 tensor with one element."""
    _check_f32("sink", sink, (1,))
    flops = ctypes.c_longlong(0)
    _raise(lib().helix_mfma_probe(_ptr(sink), int(workgroups), int(iters), int(bool(random_operands)), ctypes.byref(flops),
                                  _stream(stream)), "helix_mfma_probe")
    return flops.value


def helix_mfma_mix_probe(sink, workgroups, iters, forward_mix, stream=None) -> int:
    """Enqueues the MFMA loop with LDS reads and vector work beside it; returns the FLOPs it performs."""
    _check_f32("sink", sink, (1,))
    flops = ctypes.c_longlong(0)
    _raise(lib().helix_mfma_mix_probe(_ptr(sink), int(workgroups), int(iters), int(bool(forward_mix)), ctypes.byref(flops),
                                      _stream(stream)), "helix_mfma_mix_probe")
    return flops.value


def helix_attn_bwd_workspace_bytes(B, H, S, D) -> int:
    return int(lib().helix_attn_bwd_workspace_bytes(B, H, S, D))


def helix_attn_fwd(q, k, v, o, lse, scale, causal=True, stream=None):
    """o, lse <- attention forward of q, k, v ([B,H,S,D] bf16); lse is [B,H,S] fp32."""
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("o", o)):
        _check_bf16(n, t, (B, H, S, D))
    _check_f32("lse", lse, (B, H, S))
    _raise(lib().helix_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, H, S, D, float(scale), int(causal),
                                _stream(stream)), "helix_attn_fwd")


def helix_attn_bwd(q, k, v, o, lse, dO, dq, dk, dv, workspace, scale, causal=True, stream=None):
    """dq, dk, dv <- attention backward; workspace is a uint8 CUDA tensor of the required size."""
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("o", o), ("dO", dO), ("dq", dq), ("dk", dk), ("dv", dv)):
        _check_bf16(n, t, (B, H, S, D))
    _check_f32("lse", lse, (B, H, S))
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace: need a contiguous CUDA uint8 tensor")
    _raise(lib().helix_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq), _ptr(dk), _ptr(dv),
                                _ptr(workspace), workspace.numel(), B, H, S, D, float(scale), int(causal),
                                _stream(stream)), "helix_attn_bwd")


def helix_attn_bwd_static(q, k, v, o, lse, dO, dq, dk, dv, scale, causal=True, stream=None):
    """helix_attn_bwd without a workspace argument: the statistics live in the library's built-in device array."""
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("o", o), ("dO", dO), ("dq", dq), ("dk", dk), ("dv", dv)):
        _check_bf16(n, t, (B, H, S, D))
    _check_f32("lse", lse, (B, H, S))
    _raise(lib().helix_attn_bwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), _ptr(dq), _ptr(dk), _ptr(dv),
                                       B, H, S, D, float(scale), int(causal), _stream(stream)), "helix_attn_bwd_static")


def _view(name, t, shape):
    """(pointer, strides) of a logical [B, H, S, D] bf16 view whose last dimension is contiguous."""
    if t.dtype != torch.bfloat16 or not t.is_cuda or tuple(t.shape) != tuple(shape) or t.stride(3) != 1:
        raise ValueError(f"{name}: need a CUDA bfloat16 view of shape {tuple(shape)} with unit stride in D")
    sb, sh, ss, _ = t.stride()
    return _ptr(t), ctypes.byref(helix_strides(sb, sh, ss))


def helix_attn_check_strides(strides, B, H, S, D) -> int:
    """Status for element strides (batch, head, row), or None for contiguous."""
    arg = None if strides is None else ctypes.byref(helix_strides(*strides))
    return int(lib().helix_attn_check_strides(arg, B, H, S, D))


def helix_attn_fwd_strided(q, k, v, o, lse, scale, causal=True, stream=None):
    """helix_attn_fwd on views: each of q, k, v, o has logical shape [B,H,S,D] and any strides the
    library accepts (for example ``x.permute(1, 2, 0, 3)`` of an [S,B,H,D] activation)."""
    B, H, S, D = q.shape
    (pq, sq), (pk, sk), (pv, sv), (po, so) = (_view(n, t, (B, H, S, D)) for n, t in
                                              (("q", q), ("k", k), ("v", v), ("o", o)))
    _check_f32("lse", lse, (B, H, S))
    _raise(lib().helix_attn_fwd_strided(pq, sq, pk, sk, pv, sv, po, so, _ptr(lse), B, H, S, D, float(scale),
                                        int(causal), _stream(stream)), "helix_attn_fwd_strided")


def helix_attn_bwd_strided(q, k, v, o, lse, dO, dq, dk, dv, workspace, scale, causal=True, stream=None):
    """helix_attn_bwd on views (see helix_attn_fwd_strided)."""
    B, H, S, D = q.shape
    views = [_view(n, t, (B, H, S, D)) for n, t in (("q", q), ("k", k), ("v", v), ("o", o), ("dO", dO),
                                                    ("dq", dq), ("dk", dk), ("dv", dv))]
    _check_f32("lse", lse, (B, H, S))
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace: need a contiguous CUDA uint8 tensor")
    (pq, sq), (pk, sk), (pv, sv), (po, so), (pg, sg), (pdq, sdq), (pdk, sdk), (pdv, sdv) = views
    _raise(lib().helix_attn_bwd_strided(pq, sq, pk, sk, pv, sv, po, so, _ptr(lse), pg, sg, pdq, sdq, pdk, sdk,
                                        pdv, sdv, _ptr(workspace), workspace.numel(), B, H, S, D, float(scale),
                                        int(causal), _stream(stream)), "helix_attn_bwd_strided")


def _check_stats(stats, B, H, S, D):
    """The backward's workspace as the stage calls see it: a uint8 CUDA tensor of at least
    helix_attn_bwd_workspace_bytes bytes (plane 0: -delta, plane 1: lse * log2(e))."""
    if stats.dtype != torch.uint8 or not stats.is_cuda or not stats.is_contiguous() or \
            stats.numel() < helix_attn_bwd_workspace_bytes(B, H, S, D):
        raise ValueError("stats: need a contiguous CUDA uint8 tensor of helix_attn_bwd_workspace_bytes(B, H, S, D) bytes")


def helix_attn_bwd_preprocess(o, dO, lse, stats, stream=None):
    B, H, S, D = o.shape
    _check_bf16("o", o, (B, H, S, D)); _check_bf16("dO", dO, (B, H, S, D)); _check_f32("lse", lse, (B, H, S))
    _check_stats(stats, B, H, S, D)
    _raise(lib().helix_attn_bwd_preprocess(_ptr(o), _ptr(dO), _ptr(lse), _ptr(stats), B, H, S, D, _stream(stream)),
           "helix_attn_bwd_preprocess")


DELTA_HEAD_ROWS = 2048


def helix_attn_bwd_delta_head(q, k, v, dO, lse, stats, rows, scale, causal=True, stream=None):
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("dO", dO)):
        _check_bf16(n, t, (B, H, S, D))
    _check_f32("lse", lse, (B, H, S)); _check_stats(stats, B, H, S, D)
    _raise(lib().helix_attn_bwd_delta_head(_ptr(q), _ptr(k), _ptr(v), _ptr(dO), _ptr(lse), _ptr(stats), int(rows),
                                           B, H, S, D, float(scale), int(causal), _stream(stream)),
           "helix_attn_bwd_delta_head")


def helix_attn_bwd_dkdv(q, k, v, dO, stats, dk, dv, scale, causal=True, stream=None):
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("dO", dO), ("dk", dk), ("dv", dv)):
        _check_bf16(n, t, (B, H, S, D))
    _check_stats(stats, B, H, S, D)
    _raise(lib().helix_attn_bwd_dkdv(_ptr(q), _ptr(k), _ptr(v), _ptr(dO), _ptr(stats), _ptr(dk), _ptr(dv),
                                     B, H, S, D, float(scale), int(causal), _stream(stream)), "helix_attn_bwd_dkdv")


def helix_attn_bwd_dq(q, k, v, dO, stats, dq, scale, causal=True, stream=None):
    B, H, S, D = q.shape
    for n, t in (("q", q), ("k", k), ("v", v), ("dO", dO), ("dq", dq)):
        _check_bf16(n, t, (B, H, S, D))
    _check_stats(stats, B, H, S, D)
    _raise(lib().helix_attn_bwd_dq(_ptr(q), _ptr(k), _ptr(v), _ptr(dO), _ptr(stats), _ptr(dq),
                                   B, H, S, D, float(scale), int(causal), _stream(stream)), "helix_attn_bwd_dq")


def _matrix(name, t, rows, cols, dtype=torch.bfloat16):
    """(pointer, leading dimension) of a 2-D device matrix whose rows are contiguous."""
    if t.dtype != dtype or not t.is_cuda or tuple(t.shape) != (rows, cols) or t.stride(1) != 1:
        raise ValueError(f"{name}: need a CUDA {dtype} matrix of shape ({rows}, {cols}) with contiguous rows")
    return _ptr(t), t.stride(0)


def helix_qkv_linear_fwd(a, w, qkv, stream=None):
    """qkv[M,N] <- a[M,K] @ w[K,N]; 2-D views with contiguous rows (qkv may be the [S*B, 3*H*D] view of a fused buffer)."""
    M, K = a.shape
    N = w.shape[1]
    (pa, lda), (pw, ldw), (pq, ldq) = _matrix("a", a, M, K), _matrix("w", w, K, N), _matrix("qkv", qkv, M, N)
    _raise(lib().helix_qkv_linear_fwd(pa, lda, pw, ldw, pq, ldq, M, K, N, _stream(stream)), "helix_qkv_linear_fwd")


def helix_qkv_linear_bwd_workspace_bytes(M, K, N) -> int:
    return int(lib().helix_qkv_linear_bwd_workspace_bytes(M, K, N))


def helix_qkv_linear_bwd(a, w, dqkv, da, dw, workspace=None, stream=None):
    """da[M,K] <- dqkv @ w^T (bf16), dw[K,N] <- a^T @ dqkv (fp32); workspace: uint8 CUDA tensor of
    helix_qkv_linear_bwd_workspace_bytes(M, K, N) bytes."""
    M, K = a.shape
    N = w.shape[1]
    (pa, lda), (pw, ldw), (pg, ldg) = _matrix("a", a, M, K), _matrix("w", w, K, N), _matrix("dqkv", dqkv, M, N)
    (pda, ldda), (pdw, lddw) = _matrix("da", da, M, K), _matrix("dw", dw, K, N, torch.float32)
    if workspace is not None and (workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous()):
        raise ValueError("workspace: need a contiguous CUDA uint8 tensor")
    _raise(lib().helix_qkv_linear_bwd(pa, lda, pw, ldw, pg, ldg, pda, ldda, pdw, lddw, _ptr(workspace),
                                      0 if workspace is None else workspace.numel(), M, K, N, _stream(stream)),
           "helix_qkv_linear_bwd")
