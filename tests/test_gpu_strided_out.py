"""Outputs with a row stride larger than N (a column slice of a wider buffer): every layer entry point, both kernels.

The result must equal the contiguous call's bit for bit, and the columns of the wider buffer that lie outside the
slice must keep their contents (the tiled kernels store whole row segments: none may reach past column N).
"""
import pytest
import torch

import workloads
from paper_2603_08185_amd import binding as serq

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SENTINEL = -12345.0


def _wide(M, N, pad, dtype):
    big = torch.full((M, N + pad), SENTINEL, dtype=dtype, device=DEV)
    return big, big[:, :N]


def _check(big, view, ref, N):
    assert torch.equal(view, ref)
    assert bool((big[:, N:] == SENTINEL).all()), "the call wrote outside its N columns"


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("abits,M,K,N,r", [(8, 5, 512, 96, 32), (4, 32, 1024, 160, 64), (8, 300, 640, 288, 48), (4, 513, 512, 800, 32)])
def test_integer_layer_strided_output(out_dtype, abits, M, K, N, r):
    spec = workloads.LayerSpec("strided", 9, abits, M, K, N, r, "bf16", "bf16", 3, 20.0, 60.0)
    L = workloads.make_layer(spec)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    Xq, scale = serq.quantize_act(L["X"].to(DEV), pk.s_inv, abits)
    ws = serq.workspace(M, N, K, r, abits, DEV)
    for Rp, rdt in ((serq.pack_lowrank(L["R"].to(DEV)), torch.bfloat16), (serq.pack_lowrank_q4(L["R"].to(DEV)), serq.I4)):
        ref = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=r, r_dtype=rdt, out_dtype=out_dtype, ws=ws)
        for pad in (8, 104):
            big, view = _wide(M, N, pad, out_dtype)
            serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=r, r_dtype=rdt, Y=view, ws=ws)
            _check(big, view, ref, N)


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("M,K,N,r", [(5, 512, 96, 32), (300, 768, 288, 64), (257, 512, 800, 32)])
def test_mxfp4_layer_strided_output(out_dtype, M, K, N, r):
    spec = workloads.LayerSpec("strided_mx", 9, 4, M, K, N, r, "bf16", "bf16", 3, 20.0, 60.0)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk = serq.mx_pack_weights(L["W"].to(DEV), L["s"].to(DEV), r)
    Xq, xsc = serq.mx_quantize_act(L["X"].to(DEV), pk.s_inv)
    kw = dict(Rq=pk.Rq, rsc=pk.rsc, r=r)
    ref = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, out_dtype=out_dtype, **kw)
    for pad in (8, 104):
        big, view = _wide(M, N, pad, out_dtype)
        serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, Y=view, **kw)
        _check(big, view, ref, N)


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("abits,M,K,N,r", [(8, 5, 512, 96, 32), (4, 300, 768, 288, 64), (8, 257, 512, 800, 32)])
def test_group128_layer_strided_output(out_dtype, abits, M, K, N, r):
    spec = workloads.LayerSpec("strided_g128", 9, abits, M, K, N, r, "bf16", "bf16", 3, 20.0, 60.0)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk = serq.g128_pack_weights(L["W"].to(DEV), L["s"].to(DEV), r)
    Xq, scale, zero = serq.quantize_act_asym(L["X"].to(DEV), pk.s_inv, abits)
    kw = dict(Rp=pk.Rp, r=r)
    ref = serq.g128_linear(Xq, scale, zero, abits, pk.Wq, pk.gscale, pk.wsum, M, N, K, out_dtype=out_dtype, **kw)
    for pad in (8, 104):
        big, view = _wide(M, N, pad, out_dtype)
        serq.g128_linear(Xq, scale, zero, abits, pk.Wq, pk.gscale, pk.wsum, M, N, K, Y=view, **kw)
        _check(big, view, ref, N)
