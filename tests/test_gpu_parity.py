"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bit-exact: packed weights, scales, permutation, activation codes, INT32
accumulators.  Tolerance (max relative error, written below): Y within 1e-3 for
fp32 output and 1e-2 for bf16 / fp16 output.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import serq_oracle as orc
from paper_2603_08185_amd import binding as serq
from tests._util import DT, assert_y_close, f32, f64, oracle_layer, ulp_close

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _small_spec(abits, M, K, N, r, in_dtype="bf16", out_dtype="bf16", n_outlier=3, seed_index=0):
    return workloads.LayerSpec(f"t_a{abits}_M{M}_K{K}_N{N}_r{r}", 9, abits, M, K, N, r, in_dtype, out_dtype,
                               n_outlier, 20.0, 60.0, seed_index=seed_index)


# ---------------------------------------------------------------------------
# quantize_act
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("M,K", [(1, 64), (7, 192), (33, 2048), (5, 4096), (3, 11008), (2, 14336), (2, 16448)])
def test_quantize_act_bit_exact(abits, dtype, M, K):
    spec = _small_spec(abits, M, K, 32, 0, in_dtype=dtype)
    L = workloads.make_layer(spec, want=("X", "s"))
    X = L["X"] if dtype != "fp32" else L["X"].float()
    s_inv = (np.float32(1.0) / L["s"].numpy()).astype(np.float32)
    Xq_o, scale_o = orc.quantize_act(f32(X), s_inv, abits)
    Xq, scale = serq.quantize_act(X.to(DEV), torch.from_numpy(s_inv).to(DEV), abits)
    got = serq.unpack_act(Xq, abits, M, K).cpu().numpy()
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), scale_o.view(np.uint32))
    assert np.array_equal(got, Xq_o)
    # already-flattened input: s_inv = NULL skips the multiply
    Xq2, scale2 = serq.quantize_act(X.to(DEV), None, abits)
    Xq_o2, scale_o2 = orc.quantize_act(f32(X), None, abits)
    assert np.array_equal(scale2.cpu().numpy().view(np.uint32), scale_o2.view(np.uint32))
    assert np.array_equal(serq.unpack_act(Xq2, abits, M, K).cpu().numpy(), Xq_o2)


def test_quantize_act_edges():
    # zero token, a tie-heavy integer row, strided rows, and M = 0
    K = 128
    X = torch.zeros((4, K), dtype=torch.float32)
    X[1] = torch.arange(K, dtype=torch.float32) % 15 - 7          # integers -7..7: scale exactly 1
    X[2] = (torch.arange(K, dtype=torch.float32) % 29 - 14) * 0.5  # halves: ties at scale 1
    X[2, 0] = 7.0
    X[3, 5] = -3.25
    for abits in (4, 8):
        Xq_o, scale_o = orc.quantize_act(X.numpy(), None, abits)
        Xq, scale = serq.quantize_act(X.to(DEV), None, abits)
        assert np.array_equal(scale.cpu().numpy(), scale_o)
        assert np.array_equal(serq.unpack_act(Xq, abits, 4, K).cpu().numpy(), Xq_o)
        assert scale_o[0] == 1.0
    big = torch.randn((6, 2 * K), dtype=torch.bfloat16, generator=torch.Generator().manual_seed(3))
    view = big.to(DEV)[:, :K]                                       # row stride 2K
    Xq, scale = serq.quantize_act(view, None, 4)
    Xq_o, scale_o = orc.quantize_act(f32(big[:, :K]), None, 4)
    assert np.array_equal(serq.unpack_act(Xq, 4, 6, K).cpu().numpy(), Xq_o)
    assert np.array_equal(scale.cpu().numpy(), scale_o)
    e = torch.empty((0, K), dtype=torch.bfloat16, device=DEV)
    Xq, scale = serq.quantize_act(e, None, 4)
    assert scale.numel() == 0


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_quantize_act_tiny_scales(abits, dtype):
    # tokens at the bottom of the exponent range: scales that are subnormal (the reciprocal of such a
    # scale is not finite), barely normal, and ordinary ones in between; zeros inside every row
    K = 256
    g = torch.Generator().manual_seed(17)
    base = torch.randn((8, K), generator=g)
    base[:, ::7] = 0.0
    mags = torch.tensor([1e-38, 3e-39, 2e-37, 1e-36, 1e-33, 1e-30, 1e-25, 1.0]).reshape(8, 1)
    X = (base.double() * mags.double()).to(torch.float32).to(dtype)
    s_inv = torch.ones(K)
    s_inv[::2] = 0.5
    for sv in (None, s_inv):
        Xq_o, scale_o = orc.quantize_act(f32(X), None if sv is None else sv.numpy(), abits)
        Xq, scale = serq.quantize_act(X.to(DEV), None if sv is None else sv.to(DEV), abits)
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), scale_o.view(np.uint32))
        assert np.array_equal(serq.unpack_act(Xq, abits, 8, K).cpu().numpy(), Xq_o)
        assert scale_o[0] < 2.0 ** -126 and np.abs(Xq_o[0]).max() == orc.qmax(abits)
        assert len(np.unique(Xq_o[0])) > 4                                     # not collapsed onto +-qmax


# ---------------------------------------------------------------------------
# offline pack
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["fp16", "bf16", "fp32"])
@pytest.mark.parametrize("N,K,r", [(32, 64, 16), (96, 320, 32), (256, 256, 16), (288, 1088, 128)])
def test_pack_weights_parity(dtype, N, K, r):
    spec = _small_spec(4, 4, K, N, r, in_dtype=dtype)
    L = workloads.make_layer(spec, want=("W", "s"))
    W = L["W"] if dtype != "fp32" else L["W"].float()
    pk_o = orc.pack_weights(f32(W), L["s"].numpy(), r)
    rdt = DT[dtype] if dtype != "fp32" else torch.bfloat16
    pk = serq.pack_weights(W.to(DEV), L["s"].to(DEV), r, r_dtype=rdt)
    assert np.array_equal(pk.perm.cpu().numpy(), pk_o["perm"])
    assert np.array_equal(pk.wscale.cpu().numpy().view(np.uint32), pk_o["wscale"].view(np.uint32))
    assert np.array_equal(pk.s_inv.cpu().numpy().view(np.uint32), pk_o["s_inv"].view(np.uint32))
    assert np.array_equal(serq.unpack_weights(pk.Wq, N, K).cpu().numpy(), pk_o["Wq"])
    # residual: fp32 fused multiply-add then one rounding to the storage type, against the fp64 value
    assert ulp_close(f64(pk.R), pk_o["R"], rdt, ulps=1.0)
    assert np.max(np.abs(f64(pk.R))) > 0
    back = serq.unpack_lowrank(pk.Rp, N, r, rdt)
    assert torch.equal(back.view(torch.int16), pk.R.view(torch.int16))
    # caller-supplied order and no flattening vector
    rng = np.random.default_rng(1)
    perm = rng.permutation(K).astype(np.int32)
    pk_o2 = orc.pack_weights(f32(W), None, r, perm=perm)
    pk2 = serq.pack_weights(W.to(DEV), None, r, perm_in=torch.from_numpy(perm).to(DEV), r_dtype=rdt)
    assert np.array_equal(pk2.perm.cpu().numpy(), perm)
    assert np.all(pk2.s_inv.cpu().numpy() == 1.0)
    assert np.array_equal(serq.unpack_weights(pk2.Wq, N, K).cpu().numpy(), pk_o2["Wq"])
    assert np.array_equal(pk2.wscale.cpu().numpy(), pk_o2["wscale"])


def test_pack_saliency_ties_and_zero_rows():
    N, K = 32, 64
    W = torch.zeros((N, K), dtype=torch.float32)
    W[:, 5] = 1.0
    W[:, 9] = 1.0          # ties with channel 5: lower index first
    W[:, 60] = 2.0
    W[3, :] = 0.0          # an all-zero output channel
    pk_o = orc.pack_weights(W.numpy(), None, 16)
    pk = serq.pack_weights(W.to(DEV), None, 16, r_dtype=torch.float16)
    assert pk_o["perm"][:3].tolist() == [60, 5, 9]
    assert np.array_equal(pk.perm.cpu().numpy(), pk_o["perm"])
    assert np.array_equal(pk.wscale.cpu().numpy(), pk_o["wscale"]) and pk_o["wscale"][3] == 1.0
    assert np.array_equal(serq.unpack_weights(pk.Wq, N, K).cpu().numpy(), pk_o["Wq"])


def test_pack_clamps_a_bad_caller_order():
    # perm_in is trusted input, but indices are clamped into range before anything is read through them
    N, K = 32, 128
    W = torch.randn((N, K), generator=torch.Generator().manual_seed(9)).to(DEV)
    perm = torch.arange(K, dtype=torch.int32)
    perm[3], perm[7] = -5, K + 10
    pk = serq.pack_weights(W, None, 16, perm_in=perm.to(DEV))
    got = pk.perm.cpu()
    assert got[3] == 0 and got[7] == K - 1 and torch.equal(got[8:], perm[8:])
    want = orc.pack_weights(W.cpu().numpy(), None, 16, perm=None)   # (only to show the call returned a layer at all)
    assert serq.unpack_weights(pk.Wq, N, K).shape == want["Wq"].shape


def test_pack_lowrank_roundtrip():
    for dt in (torch.float16, torch.bfloat16):
        R = torch.randn((48, 96), generator=torch.Generator().manual_seed(5)).to(dt).to(DEV)
        Rp = serq.pack_lowrank(R)
        assert torch.equal(serq.unpack_lowrank(Rp, 96, 48, dt).view(torch.int16), R.view(torch.int16))


# ---------------------------------------------------------------------------
# integer GEMM: bit-exact accumulators on both kernels, tiles + ragged tails
# ---------------------------------------------------------------------------
def _codes(M, K, N, abits, seed):
    rng = np.random.default_rng(seed)
    q = orc.qmax(abits)
    Xq = rng.integers(-q, q + 1, size=(M, K)).astype(np.int8)
    Wq = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    # integer-valued fp32 inputs whose quantisation is the identity (row extremes present)
    Xq[:, 0] = q
    Wq[:, 1] = -7
    return Xq, Wq


def _device_codes(Xq, Wq, abits):
    M, K = Xq.shape
    N = Wq.shape[0]
    pk = serq.pack_weights(torch.from_numpy(Wq.astype(np.float32)).to(DEV), None, 0,
                           perm_in=torch.arange(K, dtype=torch.int32, device=DEV))
    xq, scale = serq.quantize_act(torch.from_numpy(Xq.astype(np.float32)).to(DEV), None, abits)
    assert torch.all(scale == 1.0) and torch.all(pk.wscale == 1.0)
    return pk, xq, scale


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (5, 96, 192), (16, 288, 448), (32, 1024, 2048), (17, 64, 8192)])
@pytest.mark.parametrize("splitk", [0, 1, 2, 3, 7])
def test_gemm_i32_skinny(abits, M, N, K, splitk):
    Xq, Wq = _codes(M, K, N, abits, seed=M + N + K)
    pk, xq, _ = _device_codes(Xq, Wq, abits)
    want = orc.gemm_i32(Xq, Wq)
    ws = serq.workspace(M, N, K, 0, abits, DEV)
    if splitk > K // 64:
        pytest.skip("split factor exceeds the number of K fragments")
    fl = serq.flags(serq.PATH_SKINNY, splitk=splitk)
    got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, ws=ws, flags_=fl)
    assert np.array_equal(got.cpu().numpy(), want)
    again = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, ws=ws, flags_=fl)   # workspace left clean, result repeatable
    assert torch.equal(got, again)


# Decode kernel variants: 4 or 8 waves per workgroup (0 = the library's choice), groups of 4 or 8 fragments,
# slices longer than one group per wave (K = 13312).
@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("waves", [0, 4, 8])
@pytest.mark.parametrize("M,N,K", [(1, 64, 4096), (4, 64, 13312), (16, 96, 4096), (32, 64, 2048), (32, 64, 8192),
                                   (7, 32, 832), (2, 32, 64)])
def test_gemm_i32_skinny_wave_counts(abits, waves, M, N, K):
    Xq, Wq = _codes(M, K, N, abits, seed=M + N + K + waves)
    pk, xq, _ = _device_codes(Xq, Wq, abits)
    want = orc.gemm_i32(Xq, Wq)
    ws = serq.workspace(M, N, K, 0, abits, DEV)
    for splitk in (1, 2):
        if splitk > K // 64:
            continue
        fl = serq.flags(serq.PATH_SKINNY, splitk=splitk, groupm=waves // 4)
        got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, ws=ws, flags_=fl)
        assert np.array_equal(got.cpu().numpy(), want), f"splitk={splitk}"


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("waves", [0, 4, 8])
@pytest.mark.parametrize("M,K,N,r", [(1, 4096, 64, 128), (16, 2048, 96, 256), (32, 2048, 64, 128), (32, 8192, 64, 32),
                                     (3, 832, 32, 16)])
def test_layer_skinny_wave_counts(abits, waves, M, K, N, r):
    # rank-r partials parked in LDS after the integer partials (M rows further), for every workgroup size
    spec = _small_spec(abits, M, K, N, r)
    _run_layer(spec, R_mode="random", path=serq.PATH_SKINNY, groupm=waves // 4, check_pack=False)
    _run_layer(spec, R_mode="random", path=serq.PATH_SKINNY, groupm=waves // 4, splitk=2, check_pack=False)


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("M,N,K", [(1, 32, 64), (40, 96, 192), (256, 256, 512), (300, 288, 448), (513, 544, 1088),
                                   (700, 320, 1024), (257, 32, 256), (64, 800, 2560), (33, 64, 128), (90, 160, 832)])
def test_gemm_i32_mfma(abits, M, N, K):
    Xq, Wq = _codes(M, K, N, abits, seed=M + N + K + 1)
    pk, xq, _ = _device_codes(Xq, Wq, abits)
    want = orc.gemm_i32(Xq, Wq)
    got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, flags_=serq.flags(serq.PATH_MFMA))
    assert np.array_equal(got.cpu().numpy(), want)
    if M <= 32:
        sk = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, ws=serq.workspace(M, N, K, 0, abits, DEV),
                           flags_=serq.flags(serq.PATH_SKINNY))
        assert torch.equal(sk, got)


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("coltiles", [1, 2, 3, 5, 7, 13, 25, 2047])
def test_gemm_i32_mfma_column_tiling_override(abits, coltiles):
    # N = 25 blocks of 32 channels: every way of cutting them into column tiles (clamped to 4 .. 25 tiles of at
    # most 8 blocks) and every group height must give the same exact accumulators
    M, N, K = 300, 800, 640
    Xq, Wq = _codes(M, K, N, abits, seed=coltiles)
    pk, xq, _ = _device_codes(Xq, Wq, abits)
    want = orc.gemm_i32(Xq, Wq)
    for groupm in (0, 1, 3):
        fl = serq.flags(serq.PATH_MFMA, groupm=groupm, coltiles=coltiles)
        got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, flags_=fl)
        assert np.array_equal(got.cpu().numpy(), want), f"groupm={groupm}"


def _split_ws(M, N, S):
    # the decode path's words, then room for S parked INT32 tiles of 256 x 256 per output tile
    n = serq.lib().serq_workspace_bytes(1, N, 64, 0, 8) + S * ((M + 255) // 256) * (N // 32) * 256 * 1024
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    serq._check("serq_workspace_init", serq.lib().serq_workspace_init(serq._ptr(ws), ws.numel(), serq._stream()))
    return ws


# K slices of the tiled kernel (two launches: the slices park their INT32 tiles, a second pass adds them up):
# forced through the flags on shapes with ragged K tiles, several token tiles and every column tiling
@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("S", [2, 3, 5])
@pytest.mark.parametrize("M,N,K", [(40, 96, 704), (256, 256, 1024), (300, 288, 1088), (64, 800, 2560), (513, 64, 1344),
                                   (90, 160, 832)])
def test_gemm_i32_mfma_k_slices(abits, S, M, N, K):
    Xq, Wq = _codes(M, K, N, abits, seed=M + N + K + S)
    pk, xq, _ = _device_codes(Xq, Wq, abits)
    want = orc.gemm_i32(Xq, Wq)
    ws = _split_ws(M, N, S)
    for coltiles in (0, 3, 2047):
        got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, ws=ws, flags_=serq.flags(serq.PATH_MFMA, splitk=S, coltiles=coltiles))
        assert np.array_equal(got.cpu().numpy(), want), coltiles
    assert not ws[:serq.lib().serq_workspace_bytes(1, N, 64, 0, 8)].any()      # the decode path's words stay clean


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("out_dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("M,K,N,r,S", [(70, 832, 64, 48, 2), (300, 1088, 288, 128, 4), (256, 2048, 96, 640, 3)])
def test_layer_mfma_k_slices(abits, out_dtype, M, K, N, r, S):
    # the sliced layer gives the bits of the unsliced one (integer sums), with every form of the compensation matrix
    spec = _small_spec(abits, M, K, N, r, out_dtype=out_dtype)
    L = workloads.make_layer(spec)
    O = oracle_layer(spec, L)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, abits)
    ws = _split_ws(M, N, S)
    Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], f64(L["R"]))
    for Rp, rdt in ((serq.pack_lowrank(L["R"].to(DEV)), torch.bfloat16), (serq.pack_lowrank_q4(L["R"].to(DEV)), serq.I4),
                    (None, torch.bfloat16)):
        kw = dict(Rp=Rp, r=r if Rp is not None else 0, r_dtype=rdt, out_dtype=DT[out_dtype])
        Y1 = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, flags_=serq.flags(serq.PATH_MFMA, splitk=1), **kw)
        Ys = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, ws=ws, flags_=serq.flags(serq.PATH_MFMA, splitk=S), **kw)
        assert torch.equal(Y1, Ys)
        if rdt == torch.bfloat16 and Rp is not None:
            assert_y_close(Ys, Y64, spec.name)
    with pytest.raises(serq.SerqError) as e:           # slices asked for without the room to park them
        serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, N, K, flags_=serq.flags(serq.PATH_MFMA, splitk=S))
    assert e.value.code == -5


def test_gemm_extreme_codes_no_overflow():
    # every product at its maximum magnitude over a long K
    for abits in (4, 8):
        q = orc.qmax(abits)
        M, N, K = 33, 64, 14336
        Xq = np.full((M, K), -q, np.int8)
        Wq = np.full((N, K), 7, np.int8)
        Wq[::2] = -7
        pk, xq, _ = _device_codes(Xq, Wq, abits)
        got = serq.gemm_i32(xq, abits, pk.Wq, M, N, K, flags_=serq.flags(serq.PATH_MFMA))
        assert np.array_equal(got.cpu().numpy(), orc.gemm_i32(Xq, Wq))


# ---------------------------------------------------------------------------
# the fused layer
# ---------------------------------------------------------------------------
def _run_layer(spec, R_mode="random", path=serq.PATH_AUTO, rows=None, splitk=0, check_pack=True, groupm=0):
    want = ("X", "s", "W", "R") if R_mode == "random" else ("X", "s", "W")
    L = workloads.make_layer(spec, want=want)
    O = oracle_layer(spec, L, R_mode=R_mode, rows=rows)
    rdt = DT[spec.in_dtype]
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r, r_dtype=rdt)
    assert np.array_equal(pk.perm.cpu().numpy(), O.pk["perm"])
    if check_pack:
        assert np.array_equal(pk.wscale.cpu().numpy(), O.pk["wscale"])
        assert np.array_equal(serq.unpack_weights(pk.Wq, spec.N, spec.K).cpu().numpy(), O.pk["Wq"])
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, spec.abits)
    codes = serq.unpack_act(Xq, spec.abits, spec.M, spec.K).cpu().numpy()
    sc = scale.cpu().numpy()
    sel = slice(None) if rows is None else O.rows
    assert np.array_equal(codes[sel], O.Xq)
    assert np.array_equal(sc[sel].view(np.uint32), O.scale.view(np.uint32))
    if R_mode == "random":
        Rp = serq.pack_lowrank(L["R"].to(DEV))
    elif R_mode == "residual":
        Rp = pk.Rp
        assert ulp_close(f64(pk.R), O.pk["R"], rdt)
    else:
        Rp = None
    ws = serq.workspace(spec.M, spec.N, spec.K, spec.r, spec.abits, DEV)
    fl = serq.flags(path, splitk=splitk, groupm=groupm)
    acc = serq.gemm_i32(Xq, spec.abits, pk.Wq, spec.M, spec.N, spec.K, ws=ws, flags_=fl).cpu().numpy()
    acc_o = orc.gemm_i32(O.Xq, O.pk["Wq"])
    assert np.array_equal(acc[sel], acc_o)
    Y = serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=Rp,
                    r=spec.r if Rp is not None else 0, r_dtype=rdt, out_dtype=DT[spec.out_dtype], ws=ws, flags_=fl)
    Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], O.R, acc=acc_o)
    Ysel = Y if rows is None else Y[torch.as_tensor(O.rows, device=Y.device)]
    errs = assert_y_close(Ysel, Y64, spec.name)
    return Y, Y64, errs


@pytest.mark.parametrize("R_mode", ["random", "residual", "none"])
def test_config1_tiny(R_mode):
    _run_layer(workloads.config1(), R_mode=R_mode)
    _run_layer(workloads.config1(), R_mode=R_mode, path=serq.PATH_MFMA)


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("in_dtype,out_dtype", [("bf16", "bf16"), ("fp16", "fp32"), ("fp16", "fp16")])
@pytest.mark.parametrize("M,K,N,r,path", [
    (3, 192, 96, 16, serq.PATH_SKINNY),
    (32, 1088, 288, 128, serq.PATH_SKINNY),
    (40, 192, 96, 32, serq.PATH_MFMA),
    (300, 1088, 288, 128, serq.PATH_MFMA),
    (257, 512, 544, 64, serq.PATH_MFMA),
    (70, 320, 64, 48, serq.PATH_MFMA),
    (130, 256, 96, 80, serq.PATH_MFMA),
    (64, 832, 32, 16, serq.PATH_MFMA),
    (5, 320, 64, 144, serq.PATH_SKINNY),
])
def test_layer_small_shapes(abits, in_dtype, out_dtype, M, K, N, r, path):
    spec = _small_spec(abits, M, K, N, r, in_dtype=in_dtype, out_dtype=out_dtype)
    _run_layer(spec, R_mode="random", path=path)
    _run_layer(spec, R_mode="residual", path=path)


def test_salient_block_offset_and_rank_zero():
    spec = _small_spec(4, 9, 256, 64, 32)
    L = workloads.make_layer(spec)
    O = oracle_layer(spec, L)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, 4)
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    for path in (serq.PATH_SKINNY, serq.PATH_MFMA):
        fl = serq.flags(path, splitk=1)
        Y = serq.linear(Xq, scale, 4, pk.Wq, pk.wscale, 9, 64, 256, Rp=Rp, r=32, s_begin=96, flags_=fl)
        Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], f64(L["R"]), s_begin=96)
        assert_y_close(Y, Y64, "s_begin=96")
        Y0 = serq.linear(Xq, scale, 4, pk.Wq, pk.wscale, 9, 64, 256, Rp=Rp, r=0, flags_=fl)
        Yn = serq.linear(Xq, scale, 4, pk.Wq, pk.wscale, 9, 64, 256, Rp=None, r=32, flags_=fl)
        plain = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], None)
        assert_y_close(Y0, plain, "r=0")
        assert torch.equal(Y0, Yn)


# ---------------------------------------------------------------------------
# the 4-bit compensation matrix Q(R) (Eq. 7, second line)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16, torch.float32])
@pytest.mark.parametrize("N,r", [(32, 16), (96, 48), (288, 64), (1024, 128), (64, 208)])
def test_pack_lowrank_q4_matches_oracle(dtype, N, r):
    g = torch.Generator().manual_seed(N + r)
    R = (torch.randn((r, N), generator=g) * 0.01).to(dtype)
    R[:, 5] = 0                                        # a zero column: scale 1, codes 0
    R[3, 7] = R[:, 7].abs().max() * 2                  # and a column whose extreme is unique
    Rq, rscale = orc.quantize_lowrank(R.float().numpy())
    blob = serq.pack_lowrank_q4(R.to(DEV))
    codes, rs = serq.unpack_lowrank_q4(blob, N, r)
    assert np.array_equal(rs.cpu().numpy().view(np.uint32), rscale.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), Rq)


def _run_layer_q4r(spec, path=serq.PATH_AUTO, splitk=0, groupm=0, rows=None, s_begin=0):
    L = workloads.make_layer(spec)
    O = oracle_layer(spec, L, rows=rows)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, spec.abits)
    Rq, rscale = orc.quantize_lowrank(L["R"].float().numpy())
    blob = serq.pack_lowrank_q4(L["R"].to(DEV))
    ws = serq.workspace(spec.M, spec.N, spec.K, spec.r, spec.abits, DEV)
    Y = serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=blob, r=spec.r,
                    r_dtype=serq.I4, s_begin=s_begin, out_dtype=DT[spec.out_dtype], ws=ws,
                    flags_=serq.flags(path, splitk=splitk, groupm=groupm))
    Y64 = orc.linear_q4r(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], Rq, rscale, s_begin=s_begin)
    Ysel = Y if rows is None else Y[torch.as_tensor(O.rows, device=Y.device)]
    return assert_y_close(Ysel, Y64, spec.name + " q4r")


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("out_dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("M,K,N,r,path", [
    (3, 192, 96, 16, serq.PATH_SKINNY),
    (32, 1088, 288, 128, serq.PATH_SKINNY),
    (1, 4096, 64, 256, serq.PATH_SKINNY),
    (5, 1024, 64, 144, serq.PATH_SKINNY),
    (40, 192, 96, 32, serq.PATH_MFMA),
    (300, 1088, 288, 128, serq.PATH_MFMA),
    (257, 512, 544, 64, serq.PATH_MFMA),
    (70, 320, 64, 48, serq.PATH_MFMA),
    (130, 256, 96, 80, serq.PATH_MFMA),
    (64, 832, 32, 16, serq.PATH_MFMA),
    (513, 640, 800, 256, serq.PATH_MFMA),
])
def test_layer_q4r_small_shapes(abits, out_dtype, M, K, N, r, path):
    spec = _small_spec(abits, M, K, N, r, out_dtype=out_dtype)
    _run_layer_q4r(spec, path=path)
    if path == serq.PATH_SKINNY:
        _run_layer_q4r(spec, path=path, splitk=2)
        _run_layer_q4r(spec, path=path, groupm=1)


@pytest.mark.parametrize("abits", [4, 8])
@pytest.mark.parametrize("M,path,groupm", [(2, serq.PATH_SKINNY, 1), (32, serq.PATH_SKINNY, 2), (70, serq.PATH_MFMA, 0)])
def test_layer_large_rank(abits, M, path, groupm):
    # more rank fragments than a workgroup has waves (decode kernel) / ten rank-r tiles (GEMM kernel)
    spec = _small_spec(abits, M, 1024, 96, 640)
    _run_layer(spec, R_mode="random", path=path, groupm=groupm, check_pack=False)
    _run_layer_q4r(spec, path=path, groupm=groupm)


@pytest.mark.parametrize("path", [serq.PATH_SKINNY, serq.PATH_MFMA])
def test_layer_q4r_salient_block_offset(path):
    spec = _small_spec(8, 9, 512, 64, 80)
    _run_layer_q4r(spec, path=path, s_begin=96)


@pytest.mark.parametrize("which,M", [("up", 1), ("up", 16), ("down", 1), ("down", 256)])
def test_config3_q4r(which, M):
    _run_layer_q4r(workloads.config3(which, M))


@pytest.mark.parametrize("which", ["up", "down"])
def test_config3_q4r_M4096(which):
    # the benchmark's launch with the 4-bit compensation matrix: every token row against the oracle
    _run_layer_q4r(workloads.config3(which, 4096))


@pytest.mark.parametrize("M", [1, 32])
def test_config4_q4r(M):
    _run_layer_q4r(workloads.config4(M))


def test_q4r_error_codes():
    x = torch.zeros(64 * 64, dtype=torch.uint8, device=DEV)
    sc = torch.ones(64, dtype=torch.float32, device=DEV)
    y = torch.empty((1, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(serq.SerqError) as e:           # the 64-rank fragment would read past K
        serq.linear(x, sc, 8, x, sc, 1, 64, 64, Rp=x, r=16, r_dtype=serq.I4, s_begin=32, Y=y)
    assert e.value.code == -3


def test_config2_attention_projection():
    _run_layer(workloads.config2())


@pytest.mark.parametrize("which,M", [("up", 1), ("up", 16), ("down", 1), ("down", 16), ("up", 256), ("down", 256)])
def test_config3_mlp_pair(which, M):
    _run_layer(workloads.config3(which, M))


@pytest.mark.parametrize("which", ["up", "down"])
def test_config3_mlp_pair_M4096(which):
    # the launch the benchmark times: codes, scales, every INT32 accumulator and every output against the oracle
    _run_layer(workloads.config3(which, 4096))


@pytest.mark.parametrize("M", [1, 4, 32])
def test_config4_wide_decode(M):
    _run_layer(workloads.config4(M), check_pack=(M == 1))


@pytest.mark.parametrize("layer", workloads.config5_layers())
def test_config5_block_stack(layer):
    # every (layer, rank) cell of the block stack, all 4096 token rows.  The weights, the activations and hence
    # the codes and the INT32 sums do not depend on the rank: they are computed once per layer on both sides
    # and reused across the rank sweep; the compensation matrix is drawn per rank.
    spec0 = workloads.config5(layer, 0)
    L = workloads.make_layer(spec0, want=("X", "s", "W"))
    O = oracle_layer(spec0, L, R_mode="none")
    M, N, K = spec0.M, spec0.N, spec0.K
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    assert np.array_equal(pk.perm.cpu().numpy(), O.pk["perm"])
    assert np.array_equal(pk.wscale.cpu().numpy(), O.pk["wscale"])
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, spec0.abits)
    assert np.array_equal(serq.unpack_act(Xq, spec0.abits, M, K).cpu().numpy(), O.Xq)
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), O.scale.view(np.uint32))
    acc_o = orc.gemm_i32(O.Xq, O.pk["Wq"])
    acc = serq.gemm_i32(Xq, spec0.abits, pk.Wq, M, N, K)
    assert torch.equal(acc.cpu(), torch.from_numpy(acc_o))
    del acc
    for r in (0, 32, 64, 128, 256):
        print(f"  [cfg5] {layer} r={r}", flush=True)
        spec = workloads.config5(layer, r)
        R = workloads.make_layer(spec, want=("R",)).get("R")
        Rp = serq.pack_lowrank(R.to(DEV)) if r else None
        Y = serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=r, out_dtype=DT[spec.out_dtype])
        Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], f64(R) if r else None, acc=acc_o)
        assert_y_close(Y, Y64, spec.name)
        del Y, Y64


def test_lowrank_term_alone_at_its_own_magnitude():
    # Y(r) - Y(r = 0) in fp32 is the compensation term by itself: compared with the oracle's
    # scale[m] * sum_j Xq[m,S_j] R[j,n] relative to THAT term's size, so a wrong rank-r product cannot hide
    # behind the much larger main product.  Both kernels, both activation widths, an offset salient block.
    for abits, M, path in ((4, 9, serq.PATH_SKINNY), (8, 32, serq.PATH_SKINNY), (4, 300, serq.PATH_MFMA),
                           (8, 130, serq.PATH_MFMA)):
        spec = _small_spec(abits, M, 1088, 288, 128, out_dtype="fp32")
        L = workloads.make_layer(spec)
        O = oracle_layer(spec, L)
        pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
        Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, abits)
        Rp = serq.pack_lowrank(L["R"].to(DEV))
        fl = serq.flags(path, splitk=1)
        for s_begin in (0, 64):
            Yr = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, spec.N, spec.K, Rp=Rp, r=spec.r, s_begin=s_begin,
                             out_dtype=torch.float32, flags_=fl)
            Y0 = serq.linear(Xq, scale, abits, pk.Wq, pk.wscale, M, spec.N, spec.K, Rp=None, r=0,
                             out_dtype=torch.float32, flags_=fl)
            term = (Yr.double() - Y0.double()).cpu().numpy()
            want = O.scale.astype(np.float64)[:, None] * orc.lowrank(O.Xq, f64(L["R"]), s_begin)
            main = np.max(np.abs(f64(Y0)))
            # the difference of two fp32 outputs carries their rounding: a few ulps of the main product
            assert np.max(np.abs(term - want)) <= 1e-3 * np.max(np.abs(want)) + 4 * 2.0 ** -24 * main, (abits, M, s_begin)
            assert np.max(np.abs(want)) > 0


def test_split_k_is_deterministic_and_matches_unsplit():
    spec = workloads.config3("down", 16)
    L = workloads.make_layer(spec)
    O = oracle_layer(spec, L)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, spec.abits)
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    ws = serq.workspace(spec.M, spec.N, spec.K, spec.r, spec.abits, DEV)
    outs = []
    for splitk in (1, 4, 8, 8, 8):
        outs.append(serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=Rp, r=spec.r,
                                ws=ws, flags_=serq.flags(serq.PATH_SKINNY, splitk=splitk)))
    assert torch.equal(outs[2], outs[3]) and torch.equal(outs[3], outs[4])
    Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], f64(L["R"]))
    for y in outs:
        assert_y_close(y, Y64)


def test_error_codes():
    L = serq.lib()
    x = torch.zeros(64 * 64, dtype=torch.uint8, device=DEV)
    sc = torch.ones(64, dtype=torch.float32, device=DEV)
    y = torch.empty((64, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 5, x, sc, 1, 64, 64, Y=y)
    assert e.value.code == -2
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 4, x, sc, 1, 48, 64, Y=y)          # N not a multiple of 32
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 4, x, sc, 1, 64, 96, Y=y)          # K not a multiple of 64
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 4, x, sc, 1, 64, 64, Rp=x, r=24, Y=y)   # r not a multiple of 16
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 4, x, sc, 40, 64, 64, Y=y, flags_=serq.flags(serq.PATH_SKINNY))  # M > 32
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x[1:], sc, 4, x, sc, 1, 64, 64, Y=y)      # misaligned
    assert e.value.code == -4
    with pytest.raises(serq.SerqError) as e:
        serq.linear(x, sc, 4, x, sc, 1, 64, 128, Y=y, flags_=serq.flags(serq.PATH_SKINNY, splitk=2))  # no workspace
    assert e.value.code == -5
    assert L.serq_linear(None, None, 4, None, None, 0, 0, None, 2, 1, 64, 64, None, 2, 64, None, 0, 0, None) == -1
