"""ctypes binding of libserq.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/serq.h).
PyTorch supplies device memory and the current stream; no arithmetic of the
method happens in Python.  If the shared library is missing the import of
this module's `lib()` raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libserq.so")

F32, F16, BF16, I4 = 0, 1, 2, 3
PATH_AUTO, PATH_SKINNY, PATH_MFMA = 0, 1, 2

_DT = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}

# name -> (restype, argtypes): mirrors include/serq.h declaration by declaration
_vp, _i, _i64, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
SIGNATURES = {
    "serq_version": (_i, []),
    "serq_strerror": (C.c_char_p, [_i]),
    "serq_packed_act_bytes": (_sz, [_i64, _i64, _i]),
    "serq_packed_weight_bytes": (_sz, [_i64, _i64]),
    "serq_packed_lowrank_bytes": (_sz, [_i64, _i]),
    "serq_packed_lowrank_q4_bytes": (_sz, [_i64, _i]),
    "serq_workspace_bytes": (_sz, [_i64, _i64, _i64, _i, _i]),
    "serq_workspace_init": (_i, [_vp, _sz, _vp]),
    "serq_pack_weights": (_i, [_vp, _i, _vp, _vp, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp]),
    "serq_pack_lowrank": (_i, [_vp, _i, _i64, _i, _vp, _vp]),
    "serq_unpack_lowrank": (_i, [_vp, _i64, _i, _vp, _vp]),
    "serq_pack_lowrank_q4": (_i, [_vp, _i, _i64, _i, _vp, _vp]),
    "serq_unpack_lowrank_q4": (_i, [_vp, _i64, _i, _vp, _vp, _vp]),
    "serq_unpack_weights": (_i, [_vp, _i64, _i64, _vp, _vp]),
    "serq_unpack_act": (_i, [_vp, _i, _i64, _i64, _vp, _vp]),
    "serq_quantize_act": (_i, [_vp, _i, _vp, _i64, _i64, _i64, _i, _vp, _vp, _vp]),
    "serq_swiglu_quantize_act": (_i, [_vp, _vp, _i, _vp, _i64, _i64, _i64, _i64, _i, _vp, _vp, _vp]),
    "serq_mx_swiglu_quantize_act": (_i, [_vp, _vp, _i, _vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp]),
    "serq_linear": (_i, [_vp, _vp, _i, _vp, _vp, _i, _i, _vp, _i, _i64, _i64, _i64, _vp, _i, _i64,
                         _vp, _sz, _i, _vp]),
    "serq_linear_noalloc": (_i, [_vp, _vp, _i, _vp, _vp, _i, _i, _vp, _i, _i64, _i64, _i64, _vp, _i, _i64, _i, _vp]),
    "serq_gemm_i32": (_i, [_vp, _i, _vp, _i64, _i64, _i64, _vp, _i64, _vp, _sz, _i, _vp]),
    "serq_mx_act_scale_bytes": (_sz, [_i64, _i64]),
    "serq_mx_weight_scale_bytes": (_sz, [_i64, _i64]),
    "serq_mx_quantize_act": (_i, [_vp, _i, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "serq_mx_pack_weights": (_i, [_vp, _i, _vp, _vp, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "serq_mx_unpack_weights": (_i, [_vp, _vp, _i64, _i64, _vp, _vp, _vp]),
    "serq_mx_unpack_act": (_i, [_vp, _vp, _i64, _i64, _vp, _vp, _vp]),
    "serq_mx_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "serq_mx_linear": (_i, [_vp, _vp, _vp, _vp, _i, _i, _vp, _vp, _i64, _i64, _i64, _vp, _i, _i64, _vp, _sz, _i, _vp]),
    "serq_g128_scale_bytes": (_sz, [_i64, _i64]),
    "serq_quantize_act_asym": (_i, [_vp, _i, _vp, _i64, _i64, _i64, _i, _vp, _vp, _vp, _vp]),
    "serq_g128_pack_weights": (_i, [_vp, _i, _vp, _vp, _i64, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _vp]),
    "serq_g128_unpack_scales": (_i, [_vp, _i64, _i64, _vp, _vp]),
    "serq_g128_linear": (_i, [_vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _i, _vp, _i, _i64, _i64, _i64, _vp, _i, _i64, _i, _vp]),
    "serq_fp6_weight_bytes": (_sz, [_i64, _i64]),
    "serq_fp6_act_bytes": (_sz, [_i64, _i64]),
    "serq_fp6_pack_weights": (_i, [_vp, _i64, _i64, _vp, _vp]),
    "serq_fp6_pack_act": (_i, [_vp, _i64, _i64, _vp, _vp]),
    "serq_proto_gemm_i32": (_i, [_vp, _vp, _i, _i64, _i64, _i64, _vp, _i64, _vp]),
    "serq_bench_mfma_peak": (_i, [_vp, _i, _i, _vp, _vp]),
    "serq_bench_mfma_fp4_peak": (_i, [_vp, _i, _i, _vp, _vp]),
    "serq_bench_read": (_i, [_vp, _sz, _i, _vp, _vp]),
}

_lib = None


class SerqError(RuntimeError):
    def __init__(self, fn: str, code: int):
        msg = lib().serq_strerror(code).decode()
        super().__init__(f"{fn} failed: {msg} ({code})")
        self.code = code


def lib() -> C.CDLL:
    """Load libserq.so (built by paper_2603_08185_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} not found: build it with `python -m paper_2603_08185_amd.build` "
                "(the SERQ kernels have no fallback implementation)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(fn: str, rc: int):
    if rc != 0:
        raise SerqError(fn, rc)


def _dev(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def flags(path: int = PATH_AUTO, splitk: int = 0, groupm: int = 0, coltiles: int = 0) -> int:
    return (path & 0xff) | ((splitk & 0xff) << 8) | ((groupm & 0xf) << 16) | ((coltiles & 0x7ff) << 20)


def workspace(M: int, N: int, K: int, r: int, abits: int, device) -> torch.Tensor:
    n = lib().serq_workspace_bytes(M, N, K, r, abits)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=device)
    _check("serq_workspace_init", lib().serq_workspace_init(_ptr(ws), ws.numel(), _stream()))
    return ws


@dataclass
class PackedLayer:
    """Device-resident artefacts of serq_pack_weights for one layer."""
    N: int
    K: int
    r: int
    Wq: torch.Tensor        # uint8 blob
    wscale: torch.Tensor    # fp32 [N]
    perm: torch.Tensor      # int32 [K]
    s_inv: torch.Tensor     # fp32 [K]
    R: Optional[torch.Tensor]    # [r,N] canonical residual (r_dtype) or None
    Rp: Optional[torch.Tensor]   # packed residual or None


def pack_weights(W: torch.Tensor, s: Optional[torch.Tensor], r: int, perm_in: Optional[torch.Tensor] = None,
                 r_dtype: torch.dtype = torch.bfloat16, want_R: bool = True, want_Rp: bool = True) -> PackedLayer:
    _dev(W, "W")
    N, K = W.shape
    L = lib()
    nbytes = L.serq_packed_weight_bytes(N, K)
    if nbytes == 0:
        raise SerqError("serq_packed_weight_bytes", -3)
    dev = W.device
    Wq = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    wscale = torch.empty(N, dtype=torch.float32, device=dev)
    perm = torch.empty(K, dtype=torch.int32, device=dev)
    s_inv = torch.empty(K, dtype=torch.float32, device=dev)
    R = torch.empty((r, N), dtype=r_dtype, device=dev) if (r > 0 and want_R) else None
    Rp = None
    if r > 0 and want_Rp and r_dtype in (torch.float16, torch.bfloat16):
        Rp = torch.empty(L.serq_packed_lowrank_bytes(N, r), dtype=torch.uint8, device=dev)
    if s is not None:
        _dev(s, "s")
    if perm_in is not None:
        _dev(perm_in, "perm_in")
    rc = L.serq_pack_weights(_ptr(W), _DT[W.dtype], _ptr(s), _ptr(perm_in), N, K, r, _ptr(Wq), _ptr(wscale),
                             _ptr(perm), _ptr(s_inv), _ptr(R), _DT[r_dtype], _ptr(Rp), _stream())
    _check("serq_pack_weights", rc)
    return PackedLayer(N, K, r, Wq, wscale, perm, s_inv, R, Rp)


def pack_lowrank(R: torch.Tensor) -> torch.Tensor:
    _dev(R, "R")
    r, N = R.shape
    L = lib()
    Rp = torch.empty(max(L.serq_packed_lowrank_bytes(N, r), 16), dtype=torch.uint8, device=R.device)
    _check("serq_pack_lowrank", L.serq_pack_lowrank(_ptr(R), _DT[R.dtype], N, r, _ptr(Rp), _stream()))
    return Rp


def unpack_lowrank(Rp: torch.Tensor, N: int, r: int, dtype: torch.dtype) -> torch.Tensor:
    out = torch.empty((r, N), dtype=dtype, device=Rp.device)
    _check("serq_unpack_lowrank", lib().serq_unpack_lowrank(_ptr(Rp), N, r, _ptr(out), _stream()))
    return out


def pack_lowrank_q4(R: torch.Tensor) -> torch.Tensor:
    """serq_pack_lowrank_q4: the compensation matrix [r,N] as 4-bit codes + per-channel scales."""
    _dev(R, "R")
    r, N = R.shape
    L = lib()
    Rq = torch.empty(max(L.serq_packed_lowrank_q4_bytes(N, r), 16), dtype=torch.uint8, device=R.device)
    _check("serq_pack_lowrank_q4", L.serq_pack_lowrank_q4(_ptr(R), _DT[R.dtype], N, r, _ptr(Rq), _stream()))
    return Rq


def unpack_lowrank_q4(Rq: torch.Tensor, N: int, r: int):
    codes = torch.empty((r, N), dtype=torch.int8, device=Rq.device)
    rscale = torch.empty(N, dtype=torch.float32, device=Rq.device)
    _check("serq_unpack_lowrank_q4",
           lib().serq_unpack_lowrank_q4(_ptr(Rq), N, r, _ptr(codes), _ptr(rscale), _stream()))
    return codes, rscale


def unpack_weights(Wq: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K), dtype=torch.int8, device=Wq.device)
    _check("serq_unpack_weights", lib().serq_unpack_weights(_ptr(Wq), N, K, _ptr(out), _stream()))
    return out


def unpack_act(Xq: torch.Tensor, abits: int, M: int, K: int) -> torch.Tensor:
    out = torch.empty((M, K), dtype=torch.int8, device=Xq.device)
    _check("serq_unpack_act", lib().serq_unpack_act(_ptr(Xq), abits, M, K, _ptr(out), _stream()))
    return out


def quantize_act(X: torch.Tensor, s_inv: Optional[torch.Tensor], abits: int,
                 Xq: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None):
    """serq_quantize_act: returns (Xq packed uint8 blob, scale fp32 [M])."""
    if not X.is_cuda:
        raise ValueError("X must live in device memory")
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be [M,K] with unit inner stride")
    M, K = X.shape
    L = lib()
    if Xq is None:
        Xq = torch.empty(max(L.serq_packed_act_bytes(M, K, abits), 16), dtype=torch.uint8, device=X.device)
    if scale is None:
        scale = torch.empty(max(M, 1), dtype=torch.float32, device=X.device)[:M]
    ldx = X.stride(0) if M > 0 else K
    rc = L.serq_quantize_act(_ptr(X), _DT[X.dtype], _ptr(s_inv), M, K, ldx, abits, _ptr(Xq), _ptr(scale), _stream())
    _check("serq_quantize_act", rc)
    return Xq, scale


def _rows(T: torch.Tensor, what: str):
    if not T.is_cuda:
        raise ValueError(f"{what} must live in device memory")
    if T.dim() != 2 or T.stride(1) != 1:
        raise ValueError(f"{what} must be [M,K] with unit inner stride")


def swiglu_quantize_act(G: torch.Tensor, U: torch.Tensor, s_inv: Optional[torch.Tensor], abits: int,
                        Xq: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None):
    """serq_swiglu_quantize_act: quantize_act of silu(G) * U; returns (Xq packed uint8 blob, scale fp32 [M])."""
    _rows(G, "G")
    _rows(U, "U")
    if G.shape != U.shape or G.dtype != U.dtype:
        raise ValueError("G and U must agree in shape and dtype")
    M, K = G.shape
    L = lib()
    if Xq is None:
        Xq = torch.empty(max(L.serq_packed_act_bytes(M, K, abits), 16), dtype=torch.uint8, device=G.device)
    if scale is None:
        scale = torch.empty(max(M, 1), dtype=torch.float32, device=G.device)[:M]
    rc = L.serq_swiglu_quantize_act(_ptr(G), _ptr(U), _DT[G.dtype], _ptr(s_inv), M, K, G.stride(0) if M > 0 else K,
                                    U.stride(0) if M > 0 else K, abits, _ptr(Xq), _ptr(scale), _stream())
    _check("serq_swiglu_quantize_act", rc)
    return Xq, scale


def mx_swiglu_quantize_act(G: torch.Tensor, U: torch.Tensor, s_inv: Optional[torch.Tensor],
                           Xq: Optional[torch.Tensor] = None, xsc: Optional[torch.Tensor] = None):
    """serq_mx_swiglu_quantize_act: mx_quantize_act of silu(G) * U; returns (codes blob, block-scale blob)."""
    _rows(G, "G")
    _rows(U, "U")
    if G.shape != U.shape or G.dtype != U.dtype:
        raise ValueError("G and U must agree in shape and dtype")
    M, K = G.shape
    L = lib()
    if Xq is None:
        Xq = torch.empty(max(L.serq_packed_act_bytes(M, K, 4), 16), dtype=torch.uint8, device=G.device)
    if xsc is None:
        xsc = torch.empty(max(L.serq_mx_act_scale_bytes(M, K), 16), dtype=torch.uint8, device=G.device)
    rc = L.serq_mx_swiglu_quantize_act(_ptr(G), _ptr(U), _DT[G.dtype], _ptr(s_inv), M, K, G.stride(0) if M > 0 else K,
                                       U.stride(0) if M > 0 else K, _ptr(Xq), _ptr(xsc), _stream())
    _check("serq_mx_swiglu_quantize_act", rc)
    return Xq, xsc


def linear(Xq: torch.Tensor, scale: torch.Tensor, abits: int, Wq: torch.Tensor, wscale: torch.Tensor,
           M: int, N: int, K: int, Rp: Optional[torch.Tensor] = None, r: int = 0,
           r_dtype=torch.bfloat16, s_begin: int = 0,
           out_dtype: torch.dtype = torch.bfloat16, Y: Optional[torch.Tensor] = None,
           ws: Optional[torch.Tensor] = None, flags_: int = 0) -> torch.Tensor:
    """serq_linear: Y = scale * (wscale * (Xq . Wq^T) + Xq[:, S] . R).  r_dtype is the 16-bit dtype of the
    packed R, or the constant I4 when Rp is the blob of pack_lowrank_q4."""
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    rc = lib().serq_linear(_ptr(Xq), _ptr(scale), abits, _ptr(Wq), _ptr(wscale), s_begin, r, _ptr(Rp),
                           r_dtype if isinstance(r_dtype, int) else _DT[r_dtype], M, N, K, _ptr(Y), _DT[Y.dtype],
                           Y.stride(0),
                           _ptr(ws), 0 if ws is None else ws.numel(), flags_, _stream())
    _check("serq_linear", rc)
    return Y


def linear_noalloc(Xq: torch.Tensor, scale: torch.Tensor, abits: int, Wq: torch.Tensor, wscale: torch.Tensor,
                   M: int, N: int, K: int, Y: torch.Tensor, Rp: Optional[torch.Tensor] = None, r: int = 0,
                   r_dtype=torch.bfloat16, s_begin: int = 0, flags_: int = 0) -> torch.Tensor:
    """serq_linear_noalloc: serq_linear on the library's built-in scratch buffer; the caller passes Y."""
    rc = lib().serq_linear_noalloc(_ptr(Xq), _ptr(scale), abits, _ptr(Wq), _ptr(wscale), s_begin, r, _ptr(Rp),
                                   r_dtype if isinstance(r_dtype, int) else _DT[r_dtype], M, N, K, _ptr(Y),
                                   _DT[Y.dtype], Y.stride(0), flags_, _stream())
    _check("serq_linear_noalloc", rc)
    return Y


def gemm_i32(Xq: torch.Tensor, abits: int, Wq: torch.Tensor, M: int, N: int, K: int,
             ws: Optional[torch.Tensor] = None, flags_: int = 0) -> torch.Tensor:
    """serq_gemm_i32: the raw INT32 accumulators [M,N]."""
    acc = torch.empty((M, N), dtype=torch.int32, device=Xq.device)
    rc = lib().serq_gemm_i32(_ptr(Xq), abits, _ptr(Wq), M, N, K, _ptr(acc), N,
                             _ptr(ws), 0 if ws is None else ws.numel(), flags_, _stream())
    _check("serq_gemm_i32", rc)
    return acc


# ---- MXFP4 variant ---------------------------------------------------------------------------------
@dataclass
class MxPackedLayer:
    """Device-resident artefacts of serq_mx_pack_weights for one layer."""
    N: int
    K: int
    r: int
    Wq: torch.Tensor        # uint8 blob: E2M1 codes
    wsc: torch.Tensor       # uint8 blob: E8M0 block scales
    perm: torch.Tensor      # int32 [K]
    s_inv: torch.Tensor     # fp32 [K]
    Rq: Optional[torch.Tensor]
    rsc: Optional[torch.Tensor]


def mx_pack_weights(W: torch.Tensor, s: Optional[torch.Tensor], r: int,
                    perm_in: Optional[torch.Tensor] = None) -> MxPackedLayer:
    _dev(W, "W")
    N, K = W.shape
    L = lib()
    nbytes = L.serq_packed_weight_bytes(N, K)
    if nbytes == 0:
        raise SerqError("serq_packed_weight_bytes", -3)
    dev = W.device
    Wq = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    wsc = torch.empty(L.serq_mx_weight_scale_bytes(N, K), dtype=torch.uint8, device=dev)
    perm = torch.empty(K, dtype=torch.int32, device=dev)
    s_inv = torch.empty(K, dtype=torch.float32, device=dev)
    Rq = rsc = None
    if r > 0:
        rk = 64 * ((r + 63) // 64)
        Rq = torch.empty(max(L.serq_packed_weight_bytes(N, rk), 16), dtype=torch.uint8, device=dev)
        rsc = torch.empty(max(L.serq_mx_weight_scale_bytes(N, rk), 16), dtype=torch.uint8, device=dev)
    if s is not None:
        _dev(s, "s")
    if perm_in is not None:
        _dev(perm_in, "perm_in")
    rc = L.serq_mx_pack_weights(_ptr(W), _DT[W.dtype], _ptr(s), _ptr(perm_in), N, K, r, _ptr(Wq), _ptr(wsc),
                                _ptr(perm), _ptr(s_inv), _ptr(Rq), _ptr(rsc), _stream())
    _check("serq_mx_pack_weights", rc)
    return MxPackedLayer(N, K, r, Wq, wsc, perm, s_inv, Rq, rsc)


def mx_unpack_weights(Wq: torch.Tensor, wsc: torch.Tensor, N: int, K: int):
    """Canonical view: (codes uint8 [N,K], exponent bytes uint8 [N,K/32])."""
    codes = torch.empty((N, K), dtype=torch.uint8, device=Wq.device)
    exps = torch.empty((N, K // 32), dtype=torch.uint8, device=Wq.device)
    _check("serq_mx_unpack_weights",
           lib().serq_mx_unpack_weights(_ptr(Wq), _ptr(wsc), N, K, _ptr(codes), _ptr(exps), _stream()))
    return codes, exps


def mx_quantize_act(X: torch.Tensor, s_inv: Optional[torch.Tensor],
                    Xq: Optional[torch.Tensor] = None, xsc: Optional[torch.Tensor] = None):
    """serq_mx_quantize_act: returns (E2M1 codes blob, E8M0 block-scale blob)."""
    if not X.is_cuda:
        raise ValueError("X must live in device memory")
    if X.dim() != 2 or X.stride(1) != 1:
        raise ValueError("X must be [M,K] with unit inner stride")
    M, K = X.shape
    L = lib()
    if Xq is None:
        Xq = torch.empty(max(L.serq_packed_act_bytes(M, K, 4), 16), dtype=torch.uint8, device=X.device)
    if xsc is None:
        xsc = torch.empty(max(L.serq_mx_act_scale_bytes(M, K), 16), dtype=torch.uint8, device=X.device)
    ldx = X.stride(0) if M > 0 else K
    rc = L.serq_mx_quantize_act(_ptr(X), _DT[X.dtype], _ptr(s_inv), M, K, ldx, _ptr(Xq), _ptr(xsc), _stream())
    _check("serq_mx_quantize_act", rc)
    return Xq, xsc


def mx_workspace(M: int, N: int, K: int, device) -> torch.Tensor:
    """A zeroed workspace for serq_mx_linear (K slicing of the decode kernel)."""
    n = lib().serq_mx_workspace_bytes(M, N, K)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device=device)
    _check("serq_workspace_init", lib().serq_workspace_init(_ptr(ws), ws.numel(), _stream()))
    return ws


def mx_unpack_act(Xq: torch.Tensor, xsc: torch.Tensor, M: int, K: int):
    codes = torch.empty((M, K), dtype=torch.uint8, device=Xq.device)
    exps = torch.empty((M, K // 32), dtype=torch.uint8, device=Xq.device)
    _check("serq_mx_unpack_act",
           lib().serq_mx_unpack_act(_ptr(Xq), _ptr(xsc), M, K, _ptr(codes), _ptr(exps), _stream()))
    return codes, exps


def mx_linear(Xq: torch.Tensor, xsc: torch.Tensor, Wq: torch.Tensor, wsc: torch.Tensor, M: int, N: int, K: int,
              Rq: Optional[torch.Tensor] = None, rsc: Optional[torch.Tensor] = None, r: int = 0, s_begin: int = 0,
              out_dtype: torch.dtype = torch.bfloat16, Y: Optional[torch.Tensor] = None,
              ws: Optional[torch.Tensor] = None, flags_: int = 0) -> torch.Tensor:
    """serq_mx_linear: Y = deq(X) . deq(W)^T + deq(X)[:, S] . deq(R)^T on the block-scaled FP4 units."""
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    rc = lib().serq_mx_linear(_ptr(Xq), _ptr(xsc), _ptr(Wq), _ptr(wsc), s_begin, r, _ptr(Rq), _ptr(rsc), M, N, K,
                              _ptr(Y), _DT[Y.dtype], Y.stride(0) if M > 0 else N,
                              _ptr(ws), 0 if ws is None else ws.numel(), flags_, _stream())
    _check("serq_mx_linear", rc)
    return Y


def bench_mfma_peak(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor) -> None:
    """serq_bench_mfma_peak: nothing but int8 MFMAs on the given 32 KiB of operand bytes."""
    assert operands.numel() * operands.element_size() >= 32768
    _check("serq_bench_mfma_peak", lib().serq_bench_mfma_peak(_ptr(operands), iters, workgroups, _ptr(sink), _stream()))


def bench_mfma_fp4_peak(operands: torch.Tensor, iters: int, workgroups: int, sink: torch.Tensor) -> None:
    """serq_bench_mfma_fp4_peak: nothing but block-scaled FP4 MFMAs on the given 32 KiB of operand bytes."""
    assert operands.numel() * operands.element_size() >= 32768
    _check("serq_bench_mfma_fp4_peak",
           lib().serq_bench_mfma_fp4_peak(_ptr(operands), iters, workgroups, _ptr(sink), _stream()))


def bench_read(src: torch.Tensor, nbytes: int, workgroups: int, sink: torch.Tensor) -> None:
    """serq_bench_read: nothing but one read of the first nbytes of src."""
    _check("serq_bench_read", lib().serq_bench_read(_ptr(src), nbytes, workgroups, _ptr(sink), _stream()))


# ---- group-128 weight scales + asymmetric activations -------------------------------------------------
@dataclass
class G128PackedLayer:
    """Device-resident artefacts of serq_g128_pack_weights for one layer."""
    N: int
    K: int
    r: int
    Wq: torch.Tensor        # uint8 blob (the layout of serq_pack_weights)
    gscale: torch.Tensor    # uint8 blob: fp16 group scales
    wsum: torch.Tensor      # fp32 [N]
    perm: torch.Tensor
    s_inv: torch.Tensor
    R: Optional[torch.Tensor]
    Rp: Optional[torch.Tensor]


def g128_pack_weights(W: torch.Tensor, s: Optional[torch.Tensor], r: int, perm_in: Optional[torch.Tensor] = None,
                      r_dtype: torch.dtype = torch.bfloat16) -> G128PackedLayer:
    _dev(W, "W")
    N, K = W.shape
    L = lib()
    nb = L.serq_g128_scale_bytes(N, K)
    if nb == 0:
        raise SerqError("serq_g128_scale_bytes", -3)
    dev = W.device
    Wq = torch.empty(N * K // 2, dtype=torch.uint8, device=dev)
    gsc = torch.empty(nb, dtype=torch.uint8, device=dev)
    wsum = torch.empty(N, dtype=torch.float32, device=dev)
    perm = torch.empty(K, dtype=torch.int32, device=dev)
    s_inv = torch.empty(K, dtype=torch.float32, device=dev)
    R = torch.empty((r, N), dtype=r_dtype, device=dev) if r > 0 else None
    Rp = torch.empty(L.serq_packed_lowrank_bytes(N, r), dtype=torch.uint8, device=dev) \
        if r > 0 and r_dtype in (torch.float16, torch.bfloat16) else None
    rc = L.serq_g128_pack_weights(_ptr(W), _DT[W.dtype], _ptr(s), _ptr(perm_in), N, K, r, _ptr(Wq), _ptr(gsc), _ptr(wsum),
                                  _ptr(perm), _ptr(s_inv), _ptr(R), _DT[r_dtype], _ptr(Rp), _stream())
    _check("serq_g128_pack_weights", rc)
    return G128PackedLayer(N, K, r, Wq, gsc, wsum, perm, s_inv, R, Rp)


def g128_unpack_scales(gscale: torch.Tensor, N: int, K: int) -> torch.Tensor:
    out = torch.empty((N, K // 128), dtype=torch.float32, device=gscale.device)
    _check("serq_g128_unpack_scales", lib().serq_g128_unpack_scales(_ptr(gscale), N, K, _ptr(out), _stream()))
    return out


def quantize_act_asym(X: torch.Tensor, s_inv: Optional[torch.Tensor], abits: int, Xq: Optional[torch.Tensor] = None,
                      scale: Optional[torch.Tensor] = None, zero: Optional[torch.Tensor] = None):
    """serq_quantize_act_asym: returns (Xq packed uint8 blob, scale fp32 [M], zero int32 [M])."""
    _rows(X, "X")
    M, K = X.shape
    L = lib()
    if Xq is None:
        Xq = torch.empty(max(L.serq_packed_act_bytes(M, K, abits), 16), dtype=torch.uint8, device=X.device)
    if scale is None:
        scale = torch.empty(max(M, 1), dtype=torch.float32, device=X.device)[:M]
    if zero is None:
        zero = torch.empty(max(M, 1), dtype=torch.int32, device=X.device)[:M]
    rc = L.serq_quantize_act_asym(_ptr(X), _DT[X.dtype], _ptr(s_inv), M, K, X.stride(0) if M > 0 else K, abits,
                                  _ptr(Xq), _ptr(scale), _ptr(zero), _stream())
    _check("serq_quantize_act_asym", rc)
    return Xq, scale, zero


def g128_linear(Xq: torch.Tensor, scale: torch.Tensor, zero: Optional[torch.Tensor], abits: int, Wq: torch.Tensor,
                gscale: torch.Tensor, wsum: torch.Tensor, M: int, N: int, K: int, Rp: Optional[torch.Tensor] = None,
                r: int = 0, r_dtype: torch.dtype = torch.bfloat16, s_begin: int = 0,
                out_dtype: torch.dtype = torch.bfloat16, Y: Optional[torch.Tensor] = None, flags_: int = 0) -> torch.Tensor:
    """serq_g128_linear: the layer with group-128 weight scales and (optionally) per-token zero points."""
    if Y is None:
        Y = torch.empty((M, N), dtype=out_dtype, device=Xq.device)
    rc = lib().serq_g128_linear(_ptr(Xq), _ptr(scale), _ptr(zero), abits, _ptr(Wq), _ptr(gscale), _ptr(wsum), s_begin, r,
                                _ptr(Rp), _DT[r_dtype], M, N, K, _ptr(Y), _DT[Y.dtype], Y.stride(0), flags_, _stream())
    _check("serq_g128_linear", rc)
    return Y


# ---- experiment: W4A4 integer sums on the FP6 form of the scaled matrix instruction -----------------------
def fp6_pack_weights(codes: torch.Tensor) -> torch.Tensor:
    """serq_fp6_pack_weights: canonical int8 codes [N,K] -> FP6 weight fragments."""
    _dev(codes, "codes")
    N, K = codes.shape
    out = torch.empty(max(lib().serq_fp6_weight_bytes(N, K), 16), dtype=torch.uint8, device=codes.device)
    _check("serq_fp6_pack_weights", lib().serq_fp6_pack_weights(_ptr(codes), N, K, _ptr(out), _stream()))
    return out


def fp6_pack_act(codes: torch.Tensor) -> torch.Tensor:
    """serq_fp6_pack_act: canonical int8 codes [M,K] -> FP6 rows."""
    _dev(codes, "codes")
    M, K = codes.shape
    out = torch.empty(max(lib().serq_fp6_act_bytes(M, K), 16), dtype=torch.uint8, device=codes.device)
    _check("serq_fp6_pack_act", lib().serq_fp6_pack_act(_ptr(codes), M, K, _ptr(out), _stream()))
    return out


def proto_gemm_i32(X: torch.Tensor, W: torch.Tensor, fp6: bool, M: int, N: int, K: int,
                   acc: Optional[torch.Tensor] = None) -> torch.Tensor:
    """serq_proto_gemm_i32: the INT32 sums from the plain tiled kernel, int8 route (fp6 = False) or FP6 route."""
    if acc is None:
        acc = torch.empty((M, N), dtype=torch.int32, device=X.device)
    _check("serq_proto_gemm_i32", lib().serq_proto_gemm_i32(_ptr(X), _ptr(W), 1 if fp6 else 0, M, N, K, _ptr(acc),
                                                            acc.stride(0) if M > 0 else N, _stream()))
    return acc
