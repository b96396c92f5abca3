"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and
rejects bad arguments before any GPU work (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2603_08185_amd import binding as serq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not h.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(serq_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_exported_and_bound():
    names = _declared()
    assert len(names) >= 14
    L = serq.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/*.h but not exported"
        assert n in serq.SIGNATURES, f"{n} has no Python binding signature"
    assert sorted(serq.SIGNATURES) == names


def test_version_and_messages():
    L = serq.lib()
    assert L.serq_version() >= 100
    for code in range(0, -9, -1):
        assert len(L.serq_strerror(code)) > 0
    assert b"unknown" in L.serq_strerror(-99)


def test_size_queries():
    L = serq.lib()
    assert L.serq_packed_act_bytes(4096, 4096, 8) == 4096 * 4096
    assert L.serq_packed_act_bytes(4096, 4096, 4) == 4096 * 2048
    assert L.serq_packed_act_bytes(1, 100, 4) == 0          # K not a multiple of 64
    assert L.serq_packed_act_bytes(1, 64, 3) == 0
    assert L.serq_packed_weight_bytes(11008, 4096) == 11008 * 4096 // 2
    assert L.serq_packed_weight_bytes(11000, 4096) == 0     # N not a multiple of 32
    assert L.serq_packed_lowrank_bytes(11008, 128) == 11008 * 128 * 2
    assert L.serq_packed_lowrank_bytes(11008, 100) == 0
    assert L.serq_workspace_bytes(1, 11008, 4096, 128, 8) > 0
    assert L.serq_workspace_bytes(1, 11008, 100, 128, 8) == 0


def test_argument_validation_precedes_any_launch():
    L = serq.lib()
    buf = (ctypes.c_char * 4096)()
    a = ctypes.cast(buf, ctypes.c_void_p).value
    a = (a + 15) & ~15
    p = ctypes.c_void_p(a)
    # quantize_act
    assert L.serq_quantize_act(p, 7, None, 1, 64, 64, 4, p, p, None) == -2      # dtype
    assert L.serq_quantize_act(p, 2, None, 1, 64, 64, 5, p, p, None) == -2      # abits
    assert L.serq_quantize_act(p, 2, None, 1, 100, 104, 4, p, p, None) == -3    # K
    assert L.serq_quantize_act(p, 2, None, 1, 128, 64, 4, p, p, None) == -3     # ldx < K
    assert L.serq_quantize_act(p, 2, None, 1, 64, 68, 4, p, p, None) == -4      # ldx alignment
    assert L.serq_quantize_act(None, 2, None, 1, 64, 64, 4, p, p, None) == -1
    assert L.serq_quantize_act(ctypes.c_void_p(a + 2), 2, None, 1, 64, 64, 4, p, p, None) == -4
    assert L.serq_quantize_act(None, 2, None, 0, 64, 64, 4, None, None, None) == 0   # M = 0: nothing to do
    # linear
    args = dict(M=1, N=64, K=64)
    def lin(Xq=p, scale=p, abits=4, Wq=p, wscale=p, s_begin=0, r=0, Rp=None, rdt=2, M=1, N=64, K=64, Y=p, ydt=2,
            ldy=64, ws=None, wsb=0, fl=0):
        return L.serq_linear(Xq, scale, abits, Wq, wscale, s_begin, r, Rp, rdt, M, N, K, Y, ydt, ldy, ws, wsb, fl, None)
    assert lin(abits=6) == -2
    assert lin(ydt=9) == -2
    assert lin(N=48) == -3
    assert lin(K=96) == -3
    assert lin(K=262144) == -3
    assert lin(r=24, Rp=p) == -3
    assert lin(r=128, Rp=p) == -3            # s_begin + r > K
    assert lin(s_begin=16, r=16, Rp=p) == -3    # the salient block starts at a multiple of 32
    assert lin(r=16, Rp=p, rdt=0) == -2      # R must be a 16-bit type
    assert lin(ldy=32) == -3
    assert lin(ldy=68) == -4
    assert lin(Y=None) == -1
    assert lin(Wq=None) == -1
    assert lin(M=64, fl=1) == -3             # skinny path forced with M > 32
    assert lin(fl=9) == -7
    assert lin(M=0) == 0
    # gemm_i32
    assert L.serq_gemm_i32(p, 4, p, 1, 64, 64, None, 64, None, 0, 0, None) == -1
    assert L.serq_gemm_i32(p, 4, p, 1, 64, 64, p, 32, None, 0, 0, None) == -3
    # pack
    assert L.serq_pack_weights(None, 2, None, None, 64, 64, 0, p, p, p, p, None, 2, None, None) == -1
    assert L.serq_pack_weights(p, 2, None, None, 64, 64, 8, p, p, p, p, None, 2, None, None) == -3
    assert L.serq_pack_weights(p, 2, None, None, 64, 64, 16, p, p, p, p, None, 0, p, None) == -2
    assert L.serq_pack_lowrank(p, 0, 64, 16, p, None) == -2
    assert L.serq_unpack_weights(p, 60, 64, p, None) == -3
    assert L.serq_unpack_act(p, 4, 1, 60, p, None) == -3
    assert L.serq_workspace_init(None, 16, None) == -1
    assert L.serq_workspace_init(None, 0, None) == 0


def test_mx_and_fused_entry_points_validate_before_any_launch():
    L = serq.lib()
    buf = (ctypes.c_char * 4096)()
    a = (ctypes.cast(buf, ctypes.c_void_p).value + 15) & ~15
    p = ctypes.c_void_p(a)
    odd = ctypes.c_void_p(a + 4)
    # size queries
    assert L.serq_mx_act_scale_bytes(4096, 4096) == 16 * 4096 * 8
    assert L.serq_mx_act_scale_bytes(3, 320) == 2 * 4 * 8             # two 256-channel tiles, M rounded up to even
    assert L.serq_mx_act_scale_bytes(1, 100) == 0
    assert L.serq_mx_weight_scale_bytes(11008, 4096) == 344 * 16 * 256
    assert L.serq_mx_weight_scale_bytes(48, 4096) == 0
    assert L.serq_mx_workspace_bytes(1, 4096, 4096) == 128 * 1024 * 4 * 17
    assert L.serq_mx_workspace_bytes(4096, 4096, 4096) == 128 * 1024 * 4 * 17   # enough tiles: the tiled kernel never cuts K
    assert L.serq_mx_workspace_bytes(64, 4096, 4096) >= 128 * 1024 * 4 * 17     # few tokens: room for parked tiles behind it
    # mx_quantize_act / the fused quantisers
    assert L.serq_mx_quantize_act(p, 7, None, 1, 64, 64, p, p, None) == -2
    assert L.serq_mx_quantize_act(p, 2, None, 1, 96, 96, p, p, None) == -3
    assert L.serq_mx_quantize_act(p, 2, None, 1, 128, 64, p, p, None) == -3       # ldx < K
    assert L.serq_mx_quantize_act(p, 2, None, 1, 64, 68, p, p, None) == -4
    assert L.serq_mx_quantize_act(None, 2, None, 1, 64, 64, p, p, None) == -1
    assert L.serq_mx_quantize_act(p, 2, None, 1, 64, 64, p, odd, None) == -4
    assert L.serq_mx_quantize_act(None, 2, None, 0, 64, 64, None, None, None) == 0
    assert L.serq_swiglu_quantize_act(p, None, 2, None, 1, 64, 64, 64, 8, p, p, None) == -1
    assert L.serq_swiglu_quantize_act(p, p, 2, None, 1, 64, 64, 32, 8, p, p, None) == -3   # ldu < K
    assert L.serq_swiglu_quantize_act(p, p, 2, None, 1, 64, 64, 64, 3, p, p, None) == -2
    assert L.serq_swiglu_quantize_act(None, None, 2, None, 0, 64, 64, 64, 8, None, None, None) == 0
    assert L.serq_mx_swiglu_quantize_act(p, None, 2, None, 1, 64, 64, 64, p, p, None) == -1
    assert L.serq_mx_swiglu_quantize_act(p, p, 9, None, 1, 64, 64, 64, p, p, None) == -2
    # mx_pack_weights
    assert L.serq_mx_pack_weights(None, 2, None, None, 64, 64, 0, p, p, p, p, None, None, None) == -1
    assert L.serq_mx_pack_weights(p, 2, None, None, 64, 64, 16, p, p, p, p, p, p, None) == -3      # r not a multiple of 32
    assert L.serq_mx_pack_weights(p, 2, None, None, 64, 64, 32, p, p, p, p, None, None, None) == -1  # r > 0 needs Rq / rscale
    assert L.serq_mx_pack_weights(p, 2, None, None, 60, 64, 0, p, p, p, p, None, None, None) == -3
    assert L.serq_mx_unpack_weights(p, p, 64, 60, p, p, None) == -3
    assert L.serq_mx_unpack_act(p, p, 1, 60, p, p, None) == -3
    # mx_linear
    def lin(Xq=p, xs=p, Wq=p, ws_=p, s_begin=0, r=0, Rq=None, rs=None, M=1, N=64, K=512, Y=p, ydt=2, ldy=64, wsp=None,
            wsb=0, fl=0):
        return L.serq_mx_linear(Xq, xs, Wq, ws_, s_begin, r, Rq, rs, M, N, K, Y, ydt, ldy, wsp, wsb, fl, None)
    assert lin(N=48) == -3
    assert lin(K=96) == -3
    assert lin(ydt=9) == -2
    assert lin(r=48, Rq=p, rs=p) == -3                 # rank not a multiple of the block
    assert lin(s_begin=128, r=32, Rq=p, rs=p) == -3    # salient block off the 256-channel tiles
    assert lin(s_begin=256, r=320, Rq=p, rs=p) == -3   # past K
    assert lin(r=32, Rq=p, rs=None) == -1
    assert lin(ws_=None) == -1
    assert lin(ldy=32) == -3
    assert lin(ldy=68) == -4
    assert lin(Y=odd) == -4
    assert lin(M=64, fl=1) == -3                       # streaming kernel forced with M > 32
    assert lin(fl=9) == -7
    assert lin(M=0) == 0


def test_grouped_fp6_and_noalloc_entry_points_validate_before_any_launch():
    L = serq.lib()
    buf = (ctypes.c_char * 4096)()
    a = (ctypes.cast(buf, ctypes.c_void_p).value + 15) & ~15
    p = ctypes.c_void_p(a)
    odd = ctypes.c_void_p(a + 4)
    # group-128 / asymmetric variant
    assert L.serq_g128_scale_bytes(11008, 4096) == 11008 * 32 * 2
    assert L.serq_g128_scale_bytes(64, 192) == 0 and L.serq_g128_scale_bytes(48, 256) == 0
    assert L.serq_quantize_act_asym(p, 7, None, 1, 64, 64, 4, p, p, p, None) == -2
    assert L.serq_quantize_act_asym(p, 2, None, 1, 64, 64, 6, p, p, p, None) == -2
    assert L.serq_quantize_act_asym(p, 2, None, 1, 100, 100, 4, p, p, p, None) == -3
    assert L.serq_quantize_act_asym(p, 2, None, 1, 128, 64, 4, p, p, p, None) == -3      # ldx < K
    assert L.serq_quantize_act_asym(p, 2, None, 1, 64, 68, 4, p, p, p, None) == -4
    assert L.serq_quantize_act_asym(p, 2, None, 1, 64, 64, 4, p, p, None, None) == -1    # zero_out required
    assert L.serq_quantize_act_asym(None, 2, None, 0, 64, 64, 4, None, None, None, None) == 0
    def gpack(W=p, wdt=2, N=64, K=128, r=0, Wq=p, gs=p, ws_=p, perm=p, sinv=p, R=None, rdt=2, Rp=None):
        return L.serq_g128_pack_weights(W, wdt, None, None, N, K, r, Wq, gs, ws_, perm, sinv, R, rdt, Rp, None)
    assert gpack(W=None) == -1 and gpack(gs=None) == -1 and gpack(ws_=None) == -1
    assert gpack(wdt=5) == -2
    assert gpack(K=192) == -3 and gpack(N=48) == -3 and gpack(r=24) == -3 and gpack(r=256) == -3
    assert gpack(r=16, Rp=p, rdt=0) == -2                # a packed R is 16-bit
    assert gpack(Wq=odd) == -4
    assert L.serq_g128_unpack_scales(None, 64, 128, p, None) == -1
    assert L.serq_g128_unpack_scales(p, 64, 100, p, None) == -3
    def glin(Xq=p, sc=p, z=p, ab=8, Wq=p, gs=p, ws_=p, s_begin=0, r=0, Rp=None, rdt=2, M=1, N=64, K=128, Y=p, ydt=2,
             ldy=64, fl=0):
        return L.serq_g128_linear(Xq, sc, z, ab, Wq, gs, ws_, s_begin, r, Rp, rdt, M, N, K, Y, ydt, ldy, fl, None)
    assert glin(ab=5) == -2 and glin(ydt=7) == -2
    assert glin(K=192) == -3 and glin(N=48) == -3 and glin(ldy=32) == -3
    assert glin(r=24, Rp=p) == -3 and glin(s_begin=16, r=16, Rp=p) == -3 and glin(s_begin=96, r=64, Rp=p) == -3
    assert glin(r=16, Rp=p, rdt=0) == -2
    assert glin(gs=None) == -1 and glin(ws_=None) == -1 and glin(sc=None) == -1
    assert glin(ldy=68) == -4 and glin(Y=odd) == -4 and glin(z=ctypes.c_void_p(a + 2)) == -4
    assert glin(M=40, fl=1) == -3 and glin(fl=9) == -7
    assert glin(M=0) == 0
    # FP6 experiment
    assert L.serq_fp6_weight_bytes(4096, 4096) == 4096 * 4096 * 3 // 4
    assert L.serq_fp6_weight_bytes(4096, 192) == 0 and L.serq_fp6_act_bytes(5, 256) == 5 * 192
    assert L.serq_fp6_pack_weights(None, 64, 128, p, None) == -1
    assert L.serq_fp6_pack_weights(p, 64, 192, p, None) == -3
    assert L.serq_fp6_pack_act(p, 1, 192, p, None) == -3
    assert L.serq_fp6_pack_act(None, 0, 128, None, None) == 0
    assert L.serq_proto_gemm_i32(p, p, 1, 1, 64, 192, p, 64, None) == -3
    assert L.serq_proto_gemm_i32(p, p, 1, 1, 64, 128, p, 32, None) == -3          # ldacc < N
    assert L.serq_proto_gemm_i32(p, None, 0, 1, 64, 128, p, 64, None) == -1
    assert L.serq_proto_gemm_i32(p, p, 0, 1, 64, 128, odd, 64, None) == -4
    assert L.serq_proto_gemm_i32(None, None, 0, 0, 64, 128, None, 64, None) == 0
    # the allocation-free entry point refuses layers wider than its built-in scratch before it touches the device
    assert L.serq_linear_noalloc(p, p, 4, p, p, 0, 0, None, 2, 1, 32768 + 32, 64, p, 2, 32768 + 32, 0, None) == -8
    assert b"scratch" in L.serq_strerror(-8)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(serq, "_lib", None)
    monkeypatch.setattr(serq, "LIB_PATH", "/nonexistent/libserq.so")
    with pytest.raises(ImportError):
        serq.lib()
