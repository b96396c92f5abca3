"""The quantisers fused into the producer of the down projection's input: silu(G) * U -> codes.

The product goes through an exponential, so the two sides cannot agree bit for bit: the HIP path forms
it in fp32 (good to a few ulps), the oracle in fp64 rounded once.  What is unique is compared exactly
(zero rows, the code of every value that is not within the fp32 error of a rounding boundary -- counted
and bounded), and the rest is checked for validity against the fp64 product: every code is a nearest
grid point of v / scale up to the fp32 error budget written below, every scale / block exponent the one
the row / block maximum gives.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import serq_oracle as orc
from paper_2603_08185_amd import binding as serq
from tests._util import DT, f64

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
REL = 4e-6          # fp32 error budget of silu(g) * u * s_inv: a handful of roundings at 6e-8 each, with margin


def _inputs(M, K, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    G = (torch.randn((M, K), generator=g) * 2.5).to(DT[dtype])
    U = (torch.randn((M, K), generator=g) * 1.5).to(DT[dtype])
    U[:, ::97] *= 30.0                                   # a few outlier channels
    s_inv = (1.0 / (0.5 + 1.5 * torch.rand(K, generator=g))).float()
    return G, U, s_inv


def _check_int(G, U, s_inv, abits, codes, scale):
    qmax = float(orc.qmax(abits))
    sv = np.ones(G.shape[1]) if s_inv is None else s_inv.double().numpy()
    v = orc.silu(f64(G)) * f64(U) * sv[None, :]
    amax = np.max(np.abs(v), axis=1)
    tiny = amax < 1e-30                                   # below fp32's normal range the product underflows (to zero: scale 1)
    want = np.where(tiny, 1.0, amax / qmax)
    assert np.all((np.abs(scale - want) <= REL * want) | (tiny & (scale <= 1e-30))), "per-token scale"
    t = np.clip(v / scale.astype(np.float64)[:, None], -qmax, qmax)
    t[tiny] = 0.0
    err = np.abs(codes.astype(np.float64) - t)
    assert np.all(err <= 0.5 + REL * np.maximum(1.0, np.abs(t)) * 2), "a code is not a nearest integer of v / scale"
    # against the oracle's own codes: equal except in the tie zones, and never more than one step apart
    c_o, s_o = orc.swiglu_quantize_act(G.float().numpy(), U.float().numpy(), None if s_inv is None else s_inv.numpy(), abits)
    diff = np.abs(codes.astype(np.int32) - c_o.astype(np.int32))
    assert diff.max(initial=0) <= 1
    assert np.count_nonzero(diff) <= 1e-3 * diff.size + 2
    assert np.all(np.abs(scale - s_o) <= REL * s_o)


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("M,K", [(1, 64), (7, 192), (33, 2048), (5, 11008), (2, 16448)])
def test_swiglu_quantize_act(abits, dtype, M, K):
    G, U, s_inv = _inputs(M, K, dtype, 100 * M + K % 97)
    for sv in (s_inv, None):
        Xq, scale = serq.swiglu_quantize_act(G.to(DEV), U.to(DEV), None if sv is None else sv.to(DEV), abits)
        codes = serq.unpack_act(Xq, abits, M, K).cpu().numpy()
        _check_int(G, U, sv, abits, codes, scale.cpu().numpy())


def test_swiglu_quantize_act_edges():
    K = 256
    G, U, s_inv = _inputs(6, K, "bf16", 3)
    G[1] = -200.0                                        # a closed gate: an all-zero token
    G[2] = 60.0                                          # far in the linear region: silu(g) = g exactly
    U[3] = 0.0
    for abits in (4, 8):
        Xq, scale = serq.swiglu_quantize_act(G.to(DEV), U.to(DEV), None, abits)
        codes = serq.unpack_act(Xq, abits, 6, K).cpu().numpy()
        sc = scale.cpu().numpy()
        assert not codes[1].any() and sc[1] == 1.0 and not codes[3].any() and sc[3] == 1.0
        # row 2 is 60 * U exactly on both sides: bit-exact against the plain quantiser
        c_o, s_o = orc.quantize_act((60.0 * U[2:3].double()).float().numpy(), None, abits)
        assert np.array_equal(codes[2:3], c_o) and sc[2] == s_o[0]
        _check_int(G, U, None, abits, codes, sc)
    # the two inputs as halves of one [M, 2K] buffer (row stride 2K)
    both = torch.cat([G, U], dim=1).to(DEV)
    Xq, scale = serq.swiglu_quantize_act(both[:, :K], both[:, K:], s_inv.to(DEV), 8)
    _check_int(G, U, s_inv, 8, serq.unpack_act(Xq, 8, 6, K).cpu().numpy(), scale.cpu().numpy())
    e = torch.empty((0, K), dtype=torch.bfloat16, device=DEV)
    Xq, scale = serq.swiglu_quantize_act(e, e, None, 4)
    assert scale.numel() == 0
    with pytest.raises(serq.SerqError) as ex:
        serq.swiglu_quantize_act(G.to(DEV)[:, :72], U.to(DEV)[:, :72], None, 8)       # K not a multiple of 64
    assert ex.value.code == -3


def _check_mx(G, U, s_inv, codes, exps):
    sv = np.ones(G.shape[1]) if s_inv is None else s_inv.double().numpy()
    v = orc.silu(f64(G)) * f64(U) * sv[None, :]
    M, K = v.shape
    B = v.reshape(M, K // 32, 32)
    amax = np.max(np.abs(B), axis=2)
    _, ex = np.frexp(amax)
    tiny = amax < 1e-44                                    # underflows to zero in fp32: an all-zero block
    want = np.where(tiny, 0, np.maximum(ex - 1 - 2, -127)) + 127
    near_pow2 = np.abs(amax / np.ldexp(1.0, ex) - 0.5) <= REL      # maximum within the error of a power of two
    near_pow2 |= np.abs(amax / np.ldexp(1.0, ex) - 1.0) <= REL
    dE = exps.astype(np.int32) - want
    assert np.all((dE == 0) | (near_pow2 & (np.abs(dE) <= 1))), "block exponent"
    # every code is a nearest grid point of v / 2^(E-127) (with the HIP side's own exponent), up to the budget
    t = np.ldexp(B, -(exps.astype(np.int32) - 127)[..., None])
    t[tiny] = 0.0
    grid = orc.E2M1_VALUES.astype(np.float64)
    best = np.min(np.abs(np.abs(t)[..., None] - grid), axis=-1)
    mag = grid[codes.reshape(B.shape) & 7]
    val = np.where(codes.reshape(B.shape) & 8, -mag, mag)
    assert np.all(np.abs(np.abs(val - t) - best) <= 2 * REL * np.maximum(1.0, np.abs(t))), "a code is not a nearest grid value"
    assert np.all((val == 0) | (np.sign(val) == np.sign(t)))
    # against the oracle's own output: equal except in the tie zones
    c_o, e_o = orc.mx_swiglu_quantize_act(G.float().numpy(), U.float().numpy(), None if s_inv is None else s_inv.numpy())
    same_e = exps == e_o
    assert np.count_nonzero(~same_e) <= 1e-3 * same_e.size + 1
    neq = (codes != c_o) & np.repeat(same_e, 32, axis=1)
    assert np.count_nonzero(neq) <= 1e-3 * neq.size + 2


@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("M,K", [(1, 64), (7, 192), (33, 2048), (5, 11008), (3, 16448)])
def test_mx_swiglu_quantize_act(dtype, M, K):
    G, U, s_inv = _inputs(M, K, dtype, 200 * M + K % 89)
    for sv in (s_inv, None):
        Xq, xsc = serq.mx_swiglu_quantize_act(G.to(DEV), U.to(DEV), None if sv is None else sv.to(DEV))
        codes, exps = serq.mx_unpack_act(Xq, xsc, M, K)
        _check_mx(G, U, sv, codes.cpu().numpy(), exps.cpu().numpy())


def test_mx_swiglu_edges():
    K = 256
    G, U, s_inv = _inputs(5, K, "fp16", 9)
    G[1] = -200.0
    G[2] = 60.0
    both = torch.cat([G, U], dim=1).to(DEV)
    Xq, xsc = serq.mx_swiglu_quantize_act(both[:, :K], both[:, K:], None)
    codes, exps = serq.mx_unpack_act(Xq, xsc, 5, K)
    codes, exps = codes.cpu().numpy(), exps.cpu().numpy()
    assert not codes[1].any() and np.all(exps[1] == 127)
    c_o, e_o = orc.mx_quantize_act((60.0 * U[2:3].double()).float().numpy(), None)
    assert np.array_equal(codes[2:3], c_o) and np.array_equal(exps[2:3], e_o)
    _check_mx(G, U, None, codes, exps)
    e = torch.empty((0, K), dtype=torch.bfloat16, device=DEV)
    serq.mx_swiglu_quantize_act(e, e, None)


def test_swiglu_feeds_the_down_projection_sampled_rows():
    # configuration 3's down projection at its full width, tokens sampled: fused quantiser -> serq_linear against
    # the oracle's layer on the oracle's own codes (Y within the layer tolerance; the codes differ only in tie zones)
    spec = workloads.config3("down", 64)
    L = workloads.make_layer(spec, want=("s", "W", "R"))
    G, U, _ = _inputs(spec.M, spec.K, "bf16", 77)
    pk_o = orc.pack_weights(L["W"].float().numpy(), L["s"].numpy(), spec.r)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r, r_dtype=torch.bfloat16)
    Xq, scale = serq.swiglu_quantize_act(G.to(DEV), U.to(DEV), pk.s_inv, spec.abits)
    codes = serq.unpack_act(Xq, spec.abits, spec.M, spec.K).cpu().numpy()
    s_inv = pk.s_inv.cpu()
    _check_int(G, U, s_inv, spec.abits, codes, scale.cpu().numpy())
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    ws = serq.workspace(spec.M, spec.N, spec.K, spec.r, spec.abits, DEV)
    Y = serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=Rp, r=spec.r,
                    r_dtype=torch.bfloat16, out_dtype=torch.float32, ws=ws)
    # the layer evaluated by the oracle on the HIP side's codes (they are valid codes, checked above)
    Y64 = orc.linear(codes, scale.cpu().numpy(), pk_o["Wq"], pk_o["wscale"], f64(L["R"]))
    g, mix = orc.rel_errors(f64(Y), Y64)
    assert g <= 1e-3 and mix <= 1e-3
