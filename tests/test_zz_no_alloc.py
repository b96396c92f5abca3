"""serq_linear_noalloc (the entry point for callers that cannot allocate) against serq_linear.

Two calls in a row on the library's built-in scratch buffer, the second with a smaller input; shapes whose
decode path cuts K into slices (fewer channel blocks than compute units), so the scratch words are really
used.  The results must equal serq_linear's with a caller's workspace bit for bit, and the oracle's within
the tolerance of the output type.
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import serq_oracle as orc
from paper_2603_08185_amd import binding as serq
from tests._util import DT, assert_y_close, f64, oracle_layer, replay_check

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _prepare(spec):
    L = workloads.make_layer(spec)
    O = oracle_layer(spec, L)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    Xq, scale = serq.quantize_act(O.Xhat.to(DEV), pk.s_inv, spec.abits)
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    Y64 = orc.linear(O.Xq, O.scale, O.pk["Wq"], O.pk["wscale"], f64(L["R"]))
    return pk, Xq, scale, Rp, Y64


def test_noalloc_matches_linear_two_calls_second_smaller():
    big = workloads.LayerSpec("noalloc_big", 9, 8, 16, 11008, 4096, 128, "bf16", "bf16", 5, 20.0, 60.0)
    small = workloads.LayerSpec("noalloc_small", 9, 4, 3, 2048, 1056, 32, "bf16", "fp32", 3, 20.0, 60.0, seed_index=1)
    prepared = [(_spec, _prepare(_spec)) for _spec in (big, small)]
    for rep in range(2):                                    # the whole sequence twice: the array stays clean
        for spec, (pk, Xq, scale, Rp, Y64) in prepared:
            M, N, K = spec.M, spec.N, spec.K
            for splitk in (0, 4):
                fl = serq.flags(serq.PATH_SKINNY, splitk=splitk)
                Y = torch.full((M, N), float("nan"), dtype=DT[spec.out_dtype], device=DEV)
                serq.linear_noalloc(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, N, K, Y, Rp=Rp, r=spec.r, flags_=fl)
                ws = serq.workspace(M, N, K, spec.r, spec.abits, DEV)
                Yref = serq.linear(Xq, scale, spec.abits, pk.Wq, pk.wscale, M, N, K, Rp=Rp, r=spec.r,
                                   out_dtype=DT[spec.out_dtype], ws=ws, flags_=fl)
                assert torch.equal(Y, Yref), (spec.name, rep, splitk)
                assert_y_close(Y, Y64, spec.name)


def test_noalloc_tiled_path_and_limit():
    # M > 32 runs the tiled kernel (no scratch needed); a layer wider than the built-in buffer is refused
    spec = workloads.LayerSpec("noalloc_tiled", 9, 4, 70, 320, 96, 32, "bf16", "bf16", 3, 20.0, 60.0)
    pk, Xq, scale, Rp, Y64 = _prepare(spec)
    Y = torch.empty((spec.M, spec.N), dtype=torch.bfloat16, device=DEV)
    serq.linear_noalloc(Xq, scale, 4, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Y, Rp=Rp, r=spec.r)
    assert torch.equal(Y, serq.linear(Xq, scale, 4, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=Rp, r=spec.r))
    assert_y_close(Y, Y64, spec.name)
    with pytest.raises(serq.SerqError) as e:
        serq.linear_noalloc(Xq, scale, 4, pk.Wq, pk.wscale, 1, 32768 + 32, 64, Y)
    assert e.value.code == -8


def test_noalloc_under_graph_capture():
    # the caller this entry point is for: one eager call first (it looks up and clears the built-in array),
    # then the call recorded into a HIP graph and replayed on changed inputs
    spec = workloads.LayerSpec("noalloc_graph", 9, 8, 8, 1024, 1376, 64, "bf16", "bf16", 3, 20.0, 60.0)
    L = workloads.make_layer(spec)
    pk = serq.pack_weights(L["W"].to(DEV), L["s"].to(DEV), 0, want_R=False, want_Rp=False)
    Rp = serq.pack_lowrank(L["R"].to(DEV))
    X = L["X"].to(DEV).clone()
    X0 = X.clone()
    Xq = torch.empty(spec.M * spec.K, dtype=torch.uint8, device=DEV)
    scale = torch.empty(spec.M, dtype=torch.float32, device=DEV)
    Y = torch.empty((spec.M, spec.N), dtype=torch.bfloat16, device=DEV)

    def step():
        serq.quantize_act(X, pk.s_inv, 8, Xq=Xq, scale=scale)
        serq.linear_noalloc(Xq, scale, 8, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Y, Rp=Rp, r=spec.r)

    def mutate(it):
        X.copy_(X0 * (1.0 + 0.25 * it))
        X[:, it] += 3.0

    replay_check(step, [Y, Xq, scale], mutate)
    ws = serq.workspace(spec.M, spec.N, spec.K, spec.r, 8, DEV)
    assert torch.equal(Y, serq.linear(Xq, scale, 8, pk.Wq, pk.wscale, spec.M, spec.N, spec.K, Rp=Rp, r=spec.r, ws=ws))
