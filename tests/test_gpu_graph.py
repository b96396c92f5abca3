"""The layer's calls recorded into a HIP graph and replayed: every replay must reproduce the eager result.

The library only launches kernels on the caller's stream (no allocation, no memset nodes, no host
synchronisation), so a capture holds nothing but kernel nodes; the split-K workspace is left zeroed by
the kernel itself.  Replays are interleaved with eager work and synchronisations of the program's own.
"""
import pytest
import torch

import workloads
from paper_2603_08185_amd import binding as serq
from tests._util import replay_check as _replay_check

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.mark.parametrize("M,which", [(4, "down"), (16, "up"), (300, "up")])
def test_integer_layer_replays(M, which):
    base = workloads.config3(which, M)
    spec = base.with_(K=1024, N=512 if which == "down" else 1376, r=64)
    L = workloads.make_layer(spec)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r, r_dtype=torch.bfloat16)
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    X = L["X"].to(DEV).clone()
    X0 = X.clone()
    Xq = torch.empty(M * spec.K * spec.abits // 8, dtype=torch.uint8, device=DEV)
    scale = torch.empty(M, dtype=torch.float32, device=DEV)
    Y = torch.empty((M, spec.N), dtype=torch.bfloat16, device=DEV)
    ws = serq.workspace(M, spec.N, spec.K, spec.r, spec.abits, DEV)      # K is sliced for M <= 32 here (16 / 43 blocks)

    def step():
        serq.quantize_act(X, pk.s_inv, spec.abits, Xq=Xq, scale=scale)
        serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, spec.N, spec.K, Rp=Rp, r=spec.r, Y=Y, ws=ws)

    def mutate(it):
        X.copy_(X0 * (1.0 + 0.25 * it))
        X[:, it] += 3.0

    _replay_check(step, [Y, Xq, scale], mutate)


@pytest.mark.parametrize("M", [8, 300])
def test_mxfp4_layer_replays(M):
    spec = workloads.config3("up", M).with_(K=1024, N=1376, r=64, abits=4)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk = serq.mx_pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    X = L["X"].to(DEV).clone()
    X0 = X.clone()
    Xq = torch.empty(M * spec.K // 2, dtype=torch.uint8, device=DEV)
    xsc = torch.empty(serq.lib().serq_mx_act_scale_bytes(M, spec.K), dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, spec.N), dtype=torch.bfloat16, device=DEV)

    def step():
        serq.mx_quantize_act(X, pk.s_inv, Xq=Xq, xsc=xsc)
        serq.mx_linear(Xq, xsc, pk.Wq, pk.wsc, M, spec.N, spec.K, Rq=pk.Rq, rsc=pk.rsc, r=spec.r, Y=Y)

    def mutate(it):
        X.copy_(X0 * (1.0 + 0.25 * it))
        X[:, it] += 3.0

    _replay_check(step, [Y, Xq, xsc], mutate)


@pytest.mark.parametrize("abits,M", [(4, 8), (8, 16), (8, 300)])
def test_group128_layer_replays(abits, M):
    spec = workloads.config3("up", M).with_(K=1024, N=1376, r=64, abits=abits)
    L = workloads.make_layer(spec, want=("X", "s", "W"))
    pk = serq.g128_pack_weights(L["W"].to(DEV), L["s"].to(DEV), spec.r)
    X = L["X"].to(DEV).clone()
    X0 = X.clone()
    Xq = torch.empty(M * spec.K * abits // 8, dtype=torch.uint8, device=DEV)
    scale = torch.empty(M, dtype=torch.float32, device=DEV)
    zero = torch.empty(M, dtype=torch.int32, device=DEV)
    Y = torch.empty((M, spec.N), dtype=torch.bfloat16, device=DEV)

    def step():
        serq.quantize_act_asym(X, pk.s_inv, abits, Xq=Xq, scale=scale, zero=zero)
        serq.g128_linear(Xq, scale, zero, abits, pk.Wq, pk.gscale, pk.wsum, M, spec.N, spec.K, Rp=pk.Rp, r=spec.r, Y=Y)

    def mutate(it):
        X.copy_(X0 * (1.0 + 0.25 * it))
        X[:, it] += 3.0

    _replay_check(step, [Y, Xq, scale, zero], mutate)
