"""The W4A4 integer sums on the FP6 (E2M3) form of the block-scaled matrix instruction, against the oracle.

Both routes of serq_proto_gemm_i32 (4-bit operands widened for the int8 instruction; FP6 operands at unit
scale) must give exactly the oracle's INT32 sums: integer work, bit-exact.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import serq_oracle as orc
from paper_2603_08185_amd import binding as serq
from tests._util import f32

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _both_routes(Xq_o, Wq_o):
    M, K = Xq_o.shape
    N = Wq_o.shape[0]
    want = orc.gemm_i32(Xq_o, Wq_o)
    pk = serq.pack_weights(torch.from_numpy(Wq_o.astype(np.float32)).to(DEV), None, 0,
                           perm_in=torch.arange(K, dtype=torch.int32, device=DEV), want_R=False, want_Rp=False)
    xq, scale = serq.quantize_act(torch.from_numpy(Xq_o.astype(np.float32)).to(DEV), None, 4)
    assert torch.all(scale == 1.0) and torch.all(pk.wscale == 1.0)
    a0 = serq.proto_gemm_i32(xq, pk.Wq, False, M, N, K)
    assert np.array_equal(a0.cpu().numpy(), want)
    W6 = serq.fp6_pack_weights(torch.from_numpy(Wq_o).to(DEV))
    X6 = serq.fp6_pack_act(torch.from_numpy(Xq_o).to(DEV))
    a1 = serq.proto_gemm_i32(X6, W6, True, M, N, K)
    assert np.array_equal(a1.cpu().numpy(), want)


@pytest.mark.parametrize("M,N,K", [(1, 32, 128), (40, 96, 384), (128, 128, 256), (300, 288, 1152), (513, 544, 1024),
                                   (33, 64, 14336)])
def test_fp6_route_is_exact_on_random_codes(M, N, K):
    rng = np.random.default_rng(M + N + K)
    Xq = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    Wq = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    Xq[:, 0] = 7
    Wq[:, 1] = -7
    _both_routes(Xq, Wq)


def test_fp6_route_every_code_pair_and_extremes():
    # every product of two codes appears; then every product at its extreme over the longest K of the configs
    M, N, K = 15, 32, 256
    Xq = np.zeros((M, K), np.int8)
    Wq = np.zeros((N, K), np.int8)
    for a in range(15):
        Xq[a, :128] = a - 7
    for b in range(15):
        Wq[b, b:128:15] = b - 7
    Xq[:, 255] = 7                      # every row holds its extreme, so the quantisers are the identity
    Wq[:, 254] = 7
    _both_routes(Xq, Wq)
    M, N, K = 33, 64, 14336
    Xq = np.full((M, K), -7, np.int8)
    Wq = np.full((N, K), 7, np.int8)
    Wq[::2] = -7
    _both_routes(Xq, Wq)


@pytest.mark.parametrize("layer", ["o", "down"])
def test_fp6_route_config5_full_size(layer):
    # the two layers of the block stack the comparison is timed on, every INT32 sum against the oracle
    spec = workloads.config5(layer, 0)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk_o = orc.pack_weights(f32(L["W"]), L["s"].numpy(), 0)
    Xhat = workloads.permute_channels(L["X"], pk_o["perm"])
    Xq_o, _ = orc.quantize_act(f32(Xhat), pk_o["s_inv"], 4)
    want = torch.from_numpy(orc.gemm_i32(Xq_o, pk_o["Wq"]))
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    xq, _ = serq.quantize_act(Xhat.to(DEV), pk.s_inv, 4)
    codes_w = serq.unpack_weights(pk.Wq, spec.N, spec.K)
    codes_x = serq.unpack_act(xq, 4, spec.M, spec.K)
    assert np.array_equal(codes_w.cpu().numpy(), pk_o["Wq"]) and np.array_equal(codes_x.cpu().numpy(), Xq_o)
    a0 = serq.proto_gemm_i32(xq, pk.Wq, False, spec.M, spec.N, spec.K)
    assert torch.equal(a0.cpu(), want)
    a1 = serq.proto_gemm_i32(serq.fp6_pack_act(codes_x), serq.fp6_pack_weights(codes_w), True, spec.M, spec.N, spec.K)
    assert torch.equal(a1.cpu(), want)
