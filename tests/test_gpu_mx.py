"""Parity of the MXFP4 variant of the layer (through the C ABI) with the CPU oracle.

Bit-exact: E2M1 codes and E8M0 exponent bytes of activations, weights and the
compensation matrix, the permutation and 1/s.  Tolerance (max relative error,
from tests/_util.TOL): Y within 1e-3 for fp32 output and 1e-2 for bf16 / fp16
output -- the products are exact, the sums are accumulated in fp32.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import serq_oracle as orc
from paper_2603_08185_amd import binding as serq
from tests._util import DT, assert_y_close, f32, f64, oracle_pack

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _spec(M, K, N, r, in_dtype="bf16", out_dtype="bf16", seed_index=0):
    return workloads.LayerSpec(f"mx_M{M}_K{K}_N{N}_r{r}", 9, 4, M, K, N, r, in_dtype, out_dtype, 3, 20.0, 60.0,
                               seed_index=seed_index)


# ---------------------------------------------------------------------------
# activations
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "fp16", "fp32"])
@pytest.mark.parametrize("M,K", [(1, 64), (7, 192), (33, 2048), (5, 4096), (3, 11008), (2, 14336), (2, 16448)])
def test_mx_quantize_act_bit_exact(dtype, M, K):
    L = workloads.make_layer(_spec(M, K, 32, 0, in_dtype=dtype), want=("X", "s"))
    X = L["X"] if dtype != "fp32" else L["X"].float()
    s_inv = (np.float32(1.0) / L["s"].numpy()).astype(np.float32)
    for sv in (s_inv, None):
        Xc_o, Xe_o = orc.mx_quantize_act(f32(X), sv)
        Xq, xsc = serq.mx_quantize_act(X.to(DEV), None if sv is None else torch.from_numpy(sv).to(DEV))
        codes, exps = serq.mx_unpack_act(Xq, xsc, M, K)
        assert np.array_equal(exps.cpu().numpy(), Xe_o)
        assert np.array_equal(codes.cpu().numpy(), Xc_o)


def test_mx_quantize_act_edges():
    # zero blocks, exact grid values and every tie, saturation, tiny and huge magnitudes, strided rows, M = 0
    K = 128
    X = torch.zeros((6, K), dtype=torch.float32)
    grid = torch.tensor([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    mids = torch.tensor([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    X[1, :8] = grid
    X[1, 8:16] = -grid
    X[1, 16:23] = mids
    X[1, 23:30] = -mids
    X[1, 32:39] = mids * 4.0              # block maximum 20 -> scale 4: the same ties, scaled
    X[1, 40] = 24.0
    X[1, 64:71] = mids * 0.125
    X[1, 71] = 0.75                       # block maximum 0.75 -> scale 1/8
    X[2, 0] = 7.9                         # above 6 * scale: saturates
    X[2, 1] = -7.9
    X[2, 2] = 4.0
    X[2, 33] = 1e-40                      # subnormal block maximum: exponent clipped at -127
    X[2, 34] = -3e-39
    X[2, 64] = 3e38                       # near the top of fp32
    X[2, 65] = -1e38
    X[2, 96] = 2.0 ** -120
    X[2, 97] = 2.0 ** -121 * 1.25
    X[3] = torch.randn(K, generator=torch.Generator().manual_seed(1)) * 1e-3
    X[4] = torch.randn(K, generator=torch.Generator().manual_seed(2)) * 1e4
    X[5, 5] = -3.25
    Xc_o, Xe_o = orc.mx_quantize_act(X.numpy(), None)
    Xq, xsc = serq.mx_quantize_act(X.to(DEV), None)
    codes, exps = serq.mx_unpack_act(Xq, xsc, 6, K)
    assert np.array_equal(exps.cpu().numpy(), Xe_o)
    assert np.array_equal(codes.cpu().numpy(), Xc_o)
    assert Xe_o[0].tolist() == [127] * 4 and not Xc_o[0].any()
    assert Xe_o[2, 1] == 0                                           # the clipped exponent
    big = torch.randn((5, 2 * K), dtype=torch.bfloat16, generator=torch.Generator().manual_seed(3))
    view = big.to(DEV)[:, :K]                                        # row stride 2K
    Xq, xsc = serq.mx_quantize_act(view, None)
    Xc_o, Xe_o = orc.mx_quantize_act(f32(big[:, :K]), None)
    codes, exps = serq.mx_unpack_act(Xq, xsc, 5, K)
    assert np.array_equal(codes.cpu().numpy(), Xc_o) and np.array_equal(exps.cpu().numpy(), Xe_o)
    e = torch.empty((0, K), dtype=torch.bfloat16, device=DEV)
    serq.mx_quantize_act(e, None)


# ---------------------------------------------------------------------------
# offline pack
# ---------------------------------------------------------------------------
def _check_pack(pk, pk_o, N, K, r):
    assert np.array_equal(pk.perm.cpu().numpy(), pk_o["perm"])
    assert np.array_equal(pk.s_inv.cpu().numpy().view(np.uint32), pk_o["s_inv"].view(np.uint32))
    codes, exps = serq.mx_unpack_weights(pk.Wq, pk.wsc, N, K)
    assert np.array_equal(exps.cpu().numpy(), pk_o["We"])
    assert np.array_equal(codes.cpu().numpy(), pk_o["Wc"])
    if r > 0:
        rk = 64 * ((r + 63) // 64)
        codes, exps = serq.mx_unpack_weights(pk.Rq, pk.rsc, N, rk)
        codes, exps = codes.cpu().numpy(), exps.cpu().numpy()
        assert np.array_equal(exps[:, :r // 32], pk_o["Re"])
        assert np.array_equal(codes[:, :r], pk_o["Rc"])
        assert not codes[:, r:].any() and np.all(exps[:, r // 32:] == 127)   # ranks past r: zero blocks


@pytest.mark.parametrize("dtype", ["fp16", "bf16", "fp32"])
@pytest.mark.parametrize("N,K,r", [(32, 64, 32), (96, 320, 32), (256, 256, 64), (288, 1088, 128), (64, 576, 96)])
def test_mx_pack_weights_parity(dtype, N, K, r):
    L = workloads.make_layer(_spec(4, K, N, r, in_dtype=dtype), want=("W", "s"))
    W = L["W"] if dtype != "fp32" else L["W"].float()
    pk_o = orc.mx_pack_weights(f32(W), L["s"].numpy(), r)
    pk = serq.mx_pack_weights(W.to(DEV), L["s"].to(DEV), r)
    _check_pack(pk, pk_o, N, K, r)
    assert pk_o["Rc"].any()
    # caller-supplied order, no flattening vector, no compensation matrix
    perm = np.random.default_rng(1).permutation(K).astype(np.int32)
    pk_o2 = orc.mx_pack_weights(f32(W), None, 0, perm=perm)
    pk2 = serq.mx_pack_weights(W.to(DEV), None, 0, perm_in=torch.from_numpy(perm).to(DEV))
    _check_pack(pk2, pk_o2, N, K, 0)
    assert np.all(pk2.s_inv.cpu().numpy() == 1.0)


def test_mx_pack_zero_rows_and_blocks():
    N, K = 32, 128
    W = torch.randn((N, K), generator=torch.Generator().manual_seed(4))
    W[3, :] = 0.0
    W[5, 32:64] = 0.0
    perm = np.arange(K, dtype=np.int32)
    pk_o = orc.mx_pack_weights(W.numpy(), None, 32, perm=perm)
    pk = serq.mx_pack_weights(W.to(DEV), None, 32, perm_in=torch.from_numpy(perm).to(DEV))
    _check_pack(pk, pk_o, N, K, 32)
    assert pk_o["We"][3].tolist() == [127] * 4 and pk_o["We"][5, 1] == 127


# ---------------------------------------------------------------------------
# the layer
# ---------------------------------------------------------------------------
def _run_mx(spec, rows=None, s_begin=0, with_R=True, coltiles=0, path=serq.PATH_AUTO, cols=None, ws=False, splitk=0):
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk_o = oracle_pack("mx", spec, L)
    pk = serq.mx_pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    _check_pack(pk, pk_o, spec.N, spec.K, spec.r)
    Xhat = workloads.permute_channels(L["X"], pk_o["perm"])
    Xs = Xhat if rows is None else Xhat[torch.as_tensor(rows)]
    Xc_o, Xe_o = orc.mx_quantize_act(f32(Xs), pk_o["s_inv"])
    Xq, xsc = serq.mx_quantize_act(Xhat.to(DEV), pk.s_inv)
    codes, exps = serq.mx_unpack_act(Xq, xsc, spec.M, spec.K)
    sel = slice(None) if rows is None else np.asarray(rows)
    assert np.array_equal(codes.cpu().numpy()[sel], Xc_o)
    assert np.array_equal(exps.cpu().numpy()[sel], Xe_o)
    use_R = with_R and spec.r > 0
    Y = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, spec.M, spec.N, spec.K, Rq=pk.Rq if use_R else None,
                       rsc=pk.rsc if use_R else None, r=spec.r if use_R else 0, s_begin=s_begin,
                       out_dtype=DT[spec.out_dtype],
                       ws=serq.mx_workspace(spec.M, spec.N, spec.K, DEV) if ws else None,
                       flags_=serq.flags(path, splitk=splitk, coltiles=coltiles))
    csel = slice(None) if cols is None else np.asarray(cols)         # oracle on a sample of the output channels
    Y64 = orc.mx_linear(Xc_o, Xe_o, pk_o["Wc"][csel], pk_o["We"][csel], pk_o["Rc"][csel] if use_R else None,
                        pk_o["Re"][csel] if use_R else None, s_begin=s_begin)
    Ysel = Y if rows is None else Y[torch.as_tensor(np.asarray(rows), device=Y.device)]
    if cols is not None:
        Ysel = Ysel[:, torch.as_tensor(np.asarray(cols), device=Y.device)]
    errs = assert_y_close(Ysel, Y64, spec.name)
    return Y, Y64, errs


@pytest.mark.parametrize("in_dtype,out_dtype", [("bf16", "bf16"), ("fp16", "fp32"), ("fp16", "fp16")])
@pytest.mark.parametrize("M,K,N,r", [
    (1, 64, 32, 32),        # one fragment, one block
    (40, 192, 96, 32),      # a partial tile only
    (300, 1088, 288, 128),  # 4 full tiles + 1 fragment; two token tiles, ragged; 9 channel blocks
    (257, 512, 544, 64),    # 17 channel blocks
    (70, 320, 64, 96),      # odd fragment counts in both sequences
    (130, 256, 96, 0),      # no compensation matrix
    (64, 832, 32, 256),     # a full low-rank tile
    (33, 1280, 64, 320),    # two low-rank tiles
    (512, 2048, 256, 128),  # the steady-state loop (8 full tiles)
    (777, 2304, 1056, 96),  # four token tiles (ragged), 33 channel blocks over several column tiles, 9 K tiles
])
def test_mx_layer_small_shapes(in_dtype, out_dtype, M, K, N, r):
    _run_mx(_spec(M, K, N, r, in_dtype=in_dtype, out_dtype=out_dtype))


@pytest.mark.parametrize("in_dtype,out_dtype", [("bf16", "bf16"), ("fp16", "fp32")])
@pytest.mark.parametrize("M,K,N,r", [
    (1, 64, 32, 32),        # one fragment
    (3, 192, 96, 32),       # a partial scale tile
    (32, 1088, 288, 128),   # 17 fragments: ragged last group
    (5, 320, 64, 96),       # odd fragment counts in both sequences
    (17, 2048, 64, 256),    # 8 waves, groups of 4
    (8, 4096, 128, 128),    # 8 waves, groups of 8
    (32, 2560, 96, 320),    # 5 compensation fragments on 8 waves
    (2, 8192, 64, 0),       # no compensation matrix
])
def test_mx_layer_decode_kernel(in_dtype, out_dtype, M, K, N, r):
    _run_mx(_spec(M, K, N, r, in_dtype=in_dtype, out_dtype=out_dtype), path=serq.PATH_SKINNY)


def test_mx_decode_kernel_offset_and_paths_agree():
    _run_mx(_spec(7, 1024, 96, 64, out_dtype="fp32"), s_begin=512, path=serq.PATH_SKINNY)
    # the two kernels on the same decode-sized call: same sums up to fp32 reordering
    spec = _spec(20, 1536, 160, 128, out_dtype="fp32")
    Ya, Y64, _ = _run_mx(spec, path=serq.PATH_SKINNY)
    Yb, _, _ = _run_mx(spec, path=serq.PATH_MFMA)
    assert np.max(np.abs(Ya.cpu().numpy() - Yb.cpu().numpy())) <= 1e-5 * np.max(np.abs(Y64))
    # run-to-run identical
    Yc, _, _ = _run_mx(spec, path=serq.PATH_SKINNY)
    assert torch.equal(Ya, Yc)


@pytest.mark.parametrize("which,M,ws", [("up", 1, False), ("up", 16, True), ("down", 1, True), ("down", 16, True),
                                        ("down", 1, False)])
def test_mx_config3_decode(which, M, ws):
    # (a workspace may be given; these layers have too many channel blocks for K slicing to pay, so none happens)
    _run_mx(workloads.config3(which, M), ws=ws)


@pytest.mark.parametrize("M,K,N,r,splitk", [
    (1, 512, 32, 32, 2),        # two slices of one scale tile each
    (5, 1088, 96, 128, 3),      # 5 scale tiles over 3 slices (2, 2, 1), the last one partial
    (32, 4096, 64, 128, 16),    # the most slices
    (17, 2048, 160, 64, 5),     # 8 scale tiles over 5 slices
    (8, 8192, 64, 256, 0),      # chosen by the library: 2 blocks on 256 CUs, 32 scale tiles -> 4 slices
])
def test_mx_decode_kernel_k_slices(M, K, N, r, splitk):
    spec = _spec(M, K, N, r, out_dtype="fp32")
    Ya, Y64, _ = _run_mx(spec, path=serq.PATH_SKINNY, ws=True, splitk=splitk)
    Yb, _, _ = _run_mx(spec, path=serq.PATH_SKINNY, ws=True, splitk=splitk)
    assert torch.equal(Ya, Yb)                                      # the slices are added in a fixed order
    Y1, _, _ = _run_mx(spec, path=serq.PATH_SKINNY, ws=False)      # one slice: same sums up to fp32 reordering
    assert np.max(np.abs(Ya.cpu().numpy() - Y1.cpu().numpy())) <= 1e-5 * np.max(np.abs(Y64))


def test_mx_decode_workspace_is_left_clean():
    spec = _spec(9, 2048, 96, 64, out_dtype="fp32")
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk = serq.mx_pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    Xq, xsc = serq.mx_quantize_act(L["X"].to(DEV), pk.s_inv)
    ws = serq.mx_workspace(spec.M, spec.N, spec.K, DEV)
    outs = []
    for _ in range(3):                                              # the same workspace, call after call
        outs.append(serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, spec.M, spec.N, spec.K, Rq=pk.Rq, rsc=pk.rsc, r=spec.r,
                                   out_dtype=torch.float32, ws=ws, flags_=serq.flags(serq.PATH_SKINNY, splitk=4)))
        assert not ws.any()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("M", [1, 4, 32])
def test_mx_config4_decode(M):
    # every output channel of the wide decode layer against the oracle
    _run_mx(workloads.config4(M))


def test_mx_layer_compensation_matters_and_can_be_left_out():
    spec = _spec(96, 512, 128, 128, out_dtype="fp32")
    Y, Y64, _ = _run_mx(spec)
    Y0, Y064, _ = _run_mx(spec, with_R=False)
    assert np.max(np.abs(Y64 - Y064)) > 1e-3 * np.max(np.abs(Y64))


def test_mx_layer_salient_block_offset():
    _run_mx(_spec(70, 1024, 96, 64, out_dtype="fp32"), s_begin=256)
    _run_mx(_spec(70, 1024, 96, 256, out_dtype="fp32"), s_begin=768)


@pytest.mark.parametrize("coltiles", [1, 3, 5, 9])
def test_mx_layer_column_tiling_override(coltiles):
    _run_mx(_spec(260, 768, 288, 64, out_dtype="fp32"), coltiles=coltiles)


def test_mx_layer_extreme_scales():
    # blocks whose scales differ by many binades, zero blocks and saturated codes, straight from codes
    M, K, N = 64, 512, 64
    rng = np.random.default_rng(7)
    X = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-30, 30, size=(M, K // 32)).repeat(32, axis=1))).astype(np.float32)
    W = (rng.standard_normal((N, K)) * np.exp2(rng.integers(-30, 30, size=(N, K // 32)).repeat(32, axis=1))).astype(np.float32)
    X[3, 64:96] = 0.0
    W[5, :] = 0.0
    perm = np.arange(K, dtype=np.int32)
    pk_o = orc.mx_pack_weights(W, None, 64, perm=perm)
    pk = serq.mx_pack_weights(torch.from_numpy(W).to(DEV), None, 64, perm_in=torch.from_numpy(perm).to(DEV))
    _check_pack(pk, pk_o, N, K, 64)
    Xc_o, Xe_o = orc.mx_quantize_act(X, None)
    Xq, xsc = serq.mx_quantize_act(torch.from_numpy(X).to(DEV), None)
    Y = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, Rq=pk.Rq, rsc=pk.rsc, r=64, out_dtype=torch.float32)
    Y64 = orc.mx_linear(Xc_o, Xe_o, pk_o["Wc"], pk_o["We"], pk_o["Rc"], pk_o["Re"])
    assert_y_close(Y, Y64, "extreme scales")
    assert np.all(Y.cpu().numpy()[:, 5] == 0.0)


@pytest.mark.parametrize("M,path", [(8, serq.PATH_SKINNY), (64, serq.PATH_MFMA)])
@pytest.mark.parametrize("ex,ew", [(-125, 100), (-110, -16), (100, 20), (-60, 60)])
def test_mx_layer_ends_of_the_exponent_range(M, path, ex, ew):
    # block exponents at and near both ends of E8M0 (E = 0 .. 2 and E around 225) through the matrix unit
    K, N = 512, 64
    rng = np.random.default_rng(21)
    X = np.ldexp(rng.standard_normal((M, K)), ex).astype(np.float32)
    W = np.ldexp(rng.standard_normal((N, K)), ew).astype(np.float32)
    perm = np.arange(K, dtype=np.int32)
    pk_o = orc.mx_pack_weights(W, None, 64, perm=perm)
    pk = serq.mx_pack_weights(torch.from_numpy(W).to(DEV), None, 64, perm_in=torch.from_numpy(perm).to(DEV))
    _check_pack(pk, pk_o, N, K, 64)
    Xc_o, Xe_o = orc.mx_quantize_act(X, None)
    Xq, xsc = serq.mx_quantize_act(torch.from_numpy(X).to(DEV), None)
    codes, exps = serq.mx_unpack_act(Xq, xsc, M, K)
    assert np.array_equal(codes.cpu().numpy(), Xc_o) and np.array_equal(exps.cpu().numpy(), Xe_o)
    if ex == -125:
        assert Xe_o.min() <= 1                                       # the clipped end of the range is exercised
    Y = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, Rq=pk.Rq, rsc=pk.rsc, r=64, out_dtype=torch.float32,
                       flags_=serq.flags(path))
    Y64 = orc.mx_linear(Xc_o, Xe_o, pk_o["Wc"], pk_o["We"], pk_o["Rc"], pk_o["Re"])
    assert np.max(np.abs(Y64)) > 0 and np.all(np.isfinite(Y.cpu().numpy()))
    assert_y_close(Y, Y64, f"exponents {ex} {ew}")


@pytest.mark.parametrize("which", ["up", "down"])
def test_mx_config3_M4096(which):
    # the shapes `bench.py --mx` times, in the launch configuration it times: every token row and
    # every output channel against the oracle
    _run_mx(workloads.config3(which, 4096))


@pytest.mark.parametrize("which", ["up", "down"])
def test_mx_config3_M256(which):
    _run_mx(workloads.config3(which, 256))


def _mx_split_ws(M, N, K, S):
    # the decode kernel's words, then room for S parked fp32 tiles of 256 x 256 per output tile
    n = serq.lib().serq_mx_workspace_bytes(1, N, K) + S * ((M + 255) // 256) * (N // 32) * 256 * 1024
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    serq._check("serq_workspace_init", serq.lib().serq_workspace_init(serq._ptr(ws), ws.numel(), serq._stream()))
    return ws


# K slices of the tiled kernel (two launches: the slices park their fp32 tiles, a second pass adds them up in
# slice order and runs the compensation tiles): forced through the flags on shapes with a partial last
# 256-channel tile, several token tiles and several column tilings
@pytest.mark.parametrize("out_dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("M,K,N,r,S", [(70, 832, 64, 64, 2), (300, 1088, 288, 128, 4), (256, 2048, 96, 256, 3),
                                       (33, 4352, 544, 0, 7)])
def test_mx_tiled_kernel_k_slices(out_dtype, M, K, N, r, S):
    spec = _spec(M, K, N, r, out_dtype=out_dtype)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk_o = orc.mx_pack_weights(f32(L["W"]), L["s"].numpy(), r)
    pk = serq.mx_pack_weights(L["W"].to(DEV), L["s"].to(DEV), r)
    Xhat = workloads.permute_channels(L["X"], pk_o["perm"])
    Xc_o, Xe_o = orc.mx_quantize_act(f32(Xhat), pk_o["s_inv"])
    Xq, xsc = serq.mx_quantize_act(Xhat.to(DEV), pk.s_inv)
    Y64 = orc.mx_linear(Xc_o, Xe_o, pk_o["Wc"], pk_o["We"], pk_o["Rc"] if r else None, pk_o["Re"] if r else None)
    ws = _mx_split_ws(M, N, K, S)
    kw = dict(Rq=pk.Rq if r else None, rsc=pk.rsc if r else None, r=r, out_dtype=DT[out_dtype])
    Y1 = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, flags_=serq.flags(serq.PATH_MFMA, splitk=1), **kw)
    for coltiles in (0, 3, 2047):
        fl = serq.flags(serq.PATH_MFMA, splitk=S, coltiles=coltiles)
        Ya = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, ws=ws, flags_=fl, **kw)
        Yb = serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, ws=ws, flags_=fl, **kw)
        assert torch.equal(Ya, Yb), coltiles                       # fixed order of addition
        assert_y_close(Ya, Y64, f"{spec.name} S={S} coltiles={coltiles}")
        # against the unsliced kernel: the same sums up to fp32 reordering (and one rounding of a 16-bit output)
        tol = 1e-5 if out_dtype == "fp32" else 2.0 ** -7
        assert np.max(np.abs(f64(Ya) - f64(Y1))) <= tol * np.max(np.abs(Y64)), coltiles
    assert not ws[:serq.lib().serq_mx_workspace_bytes(1, N, K)].any()     # the decode kernel's words stay clean
    with pytest.raises(serq.SerqError) as e:                       # an explicit request without room for it
        serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, N, K, ws=None, flags_=serq.flags(serq.PATH_MFMA, splitk=S), **kw)
    assert e.value.code == -5


def test_mx_config3_down_M256_sliced_by_the_library():
    # K = 11008 over 43 tiles of 256 channels, one token tile: the library cuts K when it is given the workspace
    spec = workloads.config3("down", 256)
    assert serq.lib().serq_mx_workspace_bytes(spec.M, spec.N, spec.K) > serq.lib().serq_mx_workspace_bytes(1, spec.N, spec.K)
    Ya, Y64, _ = _run_mx(spec, ws=True)
    Yb, _, _ = _run_mx(spec, ws=False)
    assert np.max(np.abs(f64(Ya) - f64(Yb))) <= 2.0 ** -7 * np.max(np.abs(Y64))


def test_mx_error_codes():
    Xq = torch.zeros(64 * 512 // 2, dtype=torch.uint8, device=DEV)
    xsc = torch.zeros(serq.lib().serq_mx_act_scale_bytes(64, 512), dtype=torch.uint8, device=DEV)
    Wq = torch.zeros(64 * 512 // 2, dtype=torch.uint8, device=DEV)
    wsc = torch.zeros(serq.lib().serq_mx_weight_scale_bytes(64, 512), dtype=torch.uint8, device=DEV)
    with pytest.raises(serq.SerqError) as e:                       # s_begin not on a 256-channel tile
        serq.mx_linear(Xq, xsc, Wq, wsc, 64, 64, 512, Rq=Wq, rsc=wsc, r=64, s_begin=128)
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:                       # rank not a multiple of the block
        serq.mx_linear(Xq, xsc, Wq, wsc, 64, 64, 512, Rq=Wq, rsc=wsc, r=48)
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:                       # salient block past K
        serq.mx_linear(Xq, xsc, Wq, wsc, 64, 64, 512, Rq=Wq, rsc=wsc, r=320, s_begin=256)
    assert e.value.code == -3
    with pytest.raises(serq.SerqError) as e:                       # missing scales
        serq.mx_linear(Xq, xsc, Wq, None, 64, 64, 512)
    assert e.value.code == -1
    with pytest.raises(serq.SerqError) as e:                       # K slices asked for without a workspace
        serq.mx_linear(Xq[:8 * 256], xsc, Wq, wsc, 8, 64, 512, flags_=serq.flags(serq.PATH_SKINNY, splitk=2))
    assert e.value.code == -5
    with pytest.raises(serq.SerqError) as e:                       # the streaming kernel takes at most 32 tokens
        serq.mx_linear(Xq, xsc, Wq, wsc, 64, 64, 512, flags_=serq.flags(serq.PATH_SKINNY))
    assert e.value.code == -3
    assert serq.lib().serq_mx_act_scale_bytes(3, 320) == 2 * 4 * 8
    assert serq.lib().serq_mx_weight_scale_bytes(64, 320) == 2 * 2 * 256
    assert serq.lib().serq_mx_weight_scale_bytes(48, 320) == 0
    Y = serq.mx_linear(Xq, xsc, Wq, wsc, 0, 64, 512)               # M = 0: no-op
    assert Y.shape == (0, 64)
