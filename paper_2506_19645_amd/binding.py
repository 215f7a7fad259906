"""Thin ctypes binding of libcaat.so: argument marshalling only -- every step of the path runs in the HIP
kernels behind the C ABI declared in include/caat.h.  PyTorch is used for device memory and streams.

The library must have been built (python -m paper_2506_19645_amd.build, or __graft_entry__.build());
loading fails loudly otherwise -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcaat.so")

OK, EINVAL, ESHAPE, EALIGN, EWORKSPACE, EHIP, EUNSUPPORTED, ESCRATCH = range(8)
MLP_GELU, MLP_SWIGLU, ATTN, ATTN_DECODE, LAYER_PREFILL = range(5)
LAYERNORM, RMSNORM = 0, 1
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2


class CaatError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: caat status %d (%s)" % (where, status, status_string(status)))


class caat_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("norm", C.c_int), ("h", C.c_int), ("ffn", C.c_int), ("T", C.c_int),
                ("hs", C.c_int), ("tokens", C.c_longlong), ("batch", C.c_int), ("seq", C.c_int),
                ("n_heads", C.c_int), ("head_dim", C.c_int), ("kv_len", C.c_longlong), ("kv_cap", C.c_longlong),
                ("eps", C.c_float), ("private_scale", C.c_float), ("rope_base", C.c_float), ("n_kv_heads", C.c_int),
                ("reduce_in_gemm", C.c_int), ("dedup_shared", C.c_int), ("separate_reduce", C.c_int)]


class caat_ws_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in (
        "total_bytes", "off_P", "bytes_P", "off_Y", "bytes_Y", "off_mean", "bytes_mean", "off_rstd", "bytes_rstd",
        "off_dZt", "bytes_dZt", "off_dP", "bytes_dP", "off_Q", "bytes_Q", "off_scratch", "bytes_scratch", "off_H", "bytes_H",
        "off_X1", "bytes_X1", "off_R1", "bytes_R1", "off_X2", "bytes_X2", "off_stats", "bytes_stats", "off_dH", "bytes_dH")]


# the method's C ABI (include/caat.h) and the measuring tools the library exports beside it (csrc/caat_tools.h)
EXPORTS = ["caat_shared_channels", "caat_status_string", "caat_workspace_bytes", "caat_workspace_layout",
           "caat_partial_sync", "caat_norm_fwd", "caat_partial_sync_norm_fwd", "caat_norm_bwd_workspace_bytes",
           "caat_norm_bwd", "caat_norm_bwd_static", "caat_gemm_bf16", "caat_block_fwd", "caat_block_bwd"]
TOOL_EXPORTS = ["caat_profile_enable", "caat_profile_reset", "caat_profile_count", "caat_profile_get", "caat_hbm_probe"]

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libcaat.so is not built: run `python -m paper_2506_19645_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, ll, i, f, sz = C.c_void_p, C.c_longlong, C.c_int, C.c_float, C.c_size_t
        L.caat_shared_channels.argtypes = [i, C.c_double]
        L.caat_shared_channels.restype = i
        L.caat_status_string.argtypes = [i]
        L.caat_status_string.restype = C.c_char_p
        L.caat_workspace_bytes.argtypes = [C.POINTER(caat_desc)]
        L.caat_workspace_bytes.restype = sz
        L.caat_workspace_layout.argtypes = [C.POINTER(caat_desc), C.POINTER(caat_ws_layout)]
        L.caat_workspace_layout.restype = i
        L.caat_partial_sync.argtypes = [vp, vp, vp, i, ll, i, i, f, vp]
        L.caat_partial_sync.restype = i
        L.caat_norm_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, ll, i, f, vp]
        L.caat_norm_fwd.restype = i
        L.caat_partial_sync_norm_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, ll, i, i, f, vp]
        L.caat_partial_sync_norm_fwd.restype = i
        L.caat_norm_bwd_workspace_bytes.argtypes = [i, ll, i]
        L.caat_norm_bwd_workspace_bytes.restype = sz
        L.caat_norm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, ll, i, i, f, vp, sz, vp]
        L.caat_norm_bwd.restype = i
        L.caat_norm_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i, i, ll, i, i, f, vp]
        L.caat_norm_bwd_static.restype = i
        L.caat_gemm_bf16.argtypes = [vp, vp, vp, i, i, ll, ll, ll, ll, ll, ll, ll, ll, ll, vp]
        L.caat_gemm_bf16.restype = i
        L.caat_block_fwd.argtypes = [C.POINTER(caat_desc), C.POINTER(vp), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.caat_block_fwd.restype = i
        L.caat_block_bwd.argtypes = [C.POINTER(caat_desc), C.POINTER(vp), vp, vp, vp, sz, vp, vp, vp, vp,
                                     C.POINTER(vp), vp, vp, vp]
        L.caat_block_bwd.restype = i
        L.caat_profile_enable.argtypes = [i]
        L.caat_profile_enable.restype = i
        L.caat_profile_reset.argtypes = []
        L.caat_profile_reset.restype = i
        L.caat_profile_count.argtypes = []
        L.caat_profile_count.restype = i
        L.caat_profile_get.argtypes = [i, C.POINTER(C.c_char_p), C.POINTER(f)]
        L.caat_profile_get.restype = i
        L.caat_hbm_probe.argtypes = [vp, vp, C.c_size_t, i, vp]
        L.caat_hbm_probe.restype = i
        _lib = L
    return _lib


# ------------------------------------------------------------------ marshalling helpers
def _ptr(t) -> Optional[int]:
    """Device pointer of a torch tensor (or pass an int / None through)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(st: int, where: str) -> None:
    if st != OK:
        raise CaatError(st, where)


def to_device(bits: np.ndarray):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on cuda:0 (no value conversion)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.bfloat16)


def to_host_bits(t) -> np.ndarray:
    """torch.bfloat16 CUDA tensor -> numpy uint16 bit patterns."""
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def make_desc(cfg, hs: Optional[int] = None, kv_cap: Optional[int] = None, reduce_in_gemm: bool = False,
              dedup_shared: bool = False, separate_reduce: bool = False) -> caat_desc:
    """caat_desc from a paper_2506_19645_amd.inputs.BlockConfig (cache capacity: one position more than what the
    call fills, unless given; shared-channel count from caat_shared_channels(h, p), unless given)."""
    if kv_cap is None:
        kv_cap = cfg.seq + 1 if cfg.kind == LAYER_PREFILL else cfg.kv_len + 1
    if hs is None:
        hs = shared_channels(cfg.h, float(cfg.p))     # the library's own floor(h*p), Eq. A3
    return caat_desc(kind=cfg.kind, norm=cfg.norm, h=cfg.h, ffn=cfg.ffn, T=cfg.T,
                     hs=hs, tokens=cfg.tokens, batch=cfg.batch, seq=cfg.seq,
                     n_heads=cfg.n_heads, head_dim=cfg.head_dim, kv_len=cfg.kv_len, kv_cap=kv_cap,
                     eps=cfg.eps, private_scale=cfg.private_scale, rope_base=cfg.rope_base,
                     n_kv_heads=getattr(cfg, "n_kv_heads", 0), reduce_in_gemm=1 if reduce_in_gemm else 0,
                     dedup_shared=1 if dedup_shared else 0, separate_reduce=1 if separate_reduce else 0)


# ------------------------------------------------------------------ entry points (same names as the C ABI)
def shared_channels(h: int, p: float) -> int:
    return lib().caat_shared_channels(h, p)


def status_string(status: int) -> str:
    return lib().caat_status_string(status).decode()


def workspace_bytes(desc: caat_desc) -> int:
    return lib().caat_workspace_bytes(C.byref(desc))


def workspace_layout(desc: caat_desc) -> caat_ws_layout:
    out = caat_ws_layout()
    _check(lib().caat_workspace_layout(C.byref(desc), C.byref(out)), "caat_workspace_layout")
    return out


def partial_sync(y, resid, out, T: int, tokens: int, h: int, hs: int, private_scale: float = 1.0, stream=None,
                 check: bool = True) -> int:
    st = lib().caat_partial_sync(_ptr(y), _ptr(resid), _ptr(out), T, tokens, h, hs, private_scale, _stream(stream))
    if check:
        _check(st, "caat_partial_sync")
    return st


def norm_fwd(x, gamma, beta, y, mean, rstd, norm: int, T: int, tokens: int, h: int, eps: float, stream=None,
             check: bool = True) -> int:
    st = lib().caat_norm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean), _ptr(rstd), norm, T, tokens, h,
                             eps, _stream(stream))
    if check:
        _check(st, "caat_norm_fwd")
    return st


def partial_sync_norm_fwd(io, resid, gamma, beta, x_out, mean, rstd, norm: int, T: int, tokens: int, h: int, hs: int,
                          eps: float, stream=None, check: bool = True) -> int:
    st = lib().caat_partial_sync_norm_fwd(_ptr(io), _ptr(resid), _ptr(gamma), _ptr(beta), _ptr(x_out), _ptr(mean),
                                          _ptr(rstd), norm, T, tokens, h, hs, eps, _stream(stream))
    if check:
        _check(st, "caat_partial_sync_norm_fwd")
    return st


def norm_bwd_workspace_bytes(T: int, tokens: int, h: int) -> int:
    return lib().caat_norm_bwd_workspace_bytes(T, tokens, h)


def norm_bwd(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, dgamma, dbeta, norm: int, T: int, tokens: int, h: int,
             hs: int, private_scale: float, workspace, stream=None, check: bool = True) -> int:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = lib().caat_norm_bwd(_ptr(dy), _ptr(dres), _ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(g_out),
                             _ptr(g_scaled), _ptr(dgamma), _ptr(dbeta), norm, T, tokens, h, hs, private_scale,
                             _ptr(workspace), ws_bytes, _stream(stream))
    if check:
        _check(st, "caat_norm_bwd")
    return st


def norm_bwd_static(dy, dres, x, gamma, mean, rstd, g_out, g_scaled, dgamma, dbeta, norm: int, T: int, tokens: int,
                    h: int, hs: int, private_scale: float, stream=None, check: bool = True) -> int:
    st = lib().caat_norm_bwd_static(_ptr(dy), _ptr(dres), _ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(g_out),
                                    _ptr(g_scaled), _ptr(dgamma), _ptr(dbeta), norm, T, tokens, h, hs, private_scale,
                                    _stream(stream))
    if check:
        _check(st, "caat_norm_bwd_static")
    return st


def gemm_bf16(a, b, c, layout: int, G: int, M: int, N: int, K: int, lda: int, ldb: int, ldc: int, stride_a: int,
              stride_b: int, stride_c: int, stream=None, check: bool = True) -> int:
    st = lib().caat_gemm_bf16(_ptr(a), _ptr(b), _ptr(c), layout, G, M, N, K, lda, ldb, ldc, stride_a, stride_b,
                              stride_c, _stream(stream))
    if check:
        _check(st, "caat_gemm_bf16")
    return st


def _ptr_array(ts: Sequence) -> "C.Array":
    arr = (C.c_void_p * len(ts))()
    for k, t in enumerate(ts):
        arr[k] = _ptr(t)
    return arr


def block_fwd(desc: caat_desc, weights: Sequence, x, r, r_out, x_out, workspace, kv_k=None, kv_v=None, stream=None,
              check: bool = True) -> int:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = lib().caat_block_fwd(C.byref(desc), _ptr_array(weights), _ptr(x), _ptr(r), _ptr(r_out), _ptr(x_out),
                              _ptr(kv_k), _ptr(kv_v), _ptr(workspace), ws_bytes, _stream(stream))
    if check:
        _check(st, "caat_block_fwd")
    return st


def block_bwd(desc: caat_desc, weights: Sequence, x, r_out, workspace, dx_out, dr_out, dx, dr, dweights: Sequence,
              dgamma, dbeta, stream=None, check: bool = True) -> int:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = lib().caat_block_bwd(C.byref(desc), _ptr_array(weights), _ptr(x), _ptr(r_out), _ptr(workspace), ws_bytes,
                              _ptr(dx_out), _ptr(dr_out), _ptr(dx), _ptr(dr), _ptr_array(dweights), _ptr(dgamma),
                              _ptr(dbeta), _stream(stream))
    if check:
        _check(st, "caat_block_bwd")
    return st


def hbm_probe(src, dst, nbytes: int, mode: int, stream=None) -> None:
    _check(lib().caat_hbm_probe(_ptr(src), _ptr(dst), nbytes, mode, _stream(stream)), "caat_hbm_probe")


def profile_enable(on: bool) -> None:
    _check(lib().caat_profile_enable(1 if on else 0), "caat_profile_enable")


def profile_reset() -> None:
    _check(lib().caat_profile_reset(), "caat_profile_reset")


def profile_records():
    """[(kernel family name, milliseconds)] in launch order since the last reset (waits for completion)."""
    L = lib()
    out = []
    for k in range(L.caat_profile_count()):
        name, ms = C.c_char_p(), C.c_float()
        _check(L.caat_profile_get(k, C.byref(name), C.byref(ms)), "caat_profile_get")
        out.append((name.value.decode(), float(ms.value)))
    return out
