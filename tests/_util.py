"""Shared plumbing of the parity tests: run both sides on the same seeded inputs.

The oracle side and the HIP side never exchange intermediate values: each
starts from the tensors `workloads.make_layer` drew.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

import workloads
from oracle import serq_oracle as orc

TOL = {torch.float32: 1e-3, torch.bfloat16: 1e-2, torch.float16: 1e-2}
DT = {"fp16": torch.float16, "bf16": torch.bfloat16, "fp32": torch.float32}


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().double().cpu().numpy()


@dataclass
class OracleLayer:
    spec: workloads.LayerSpec
    pk: dict
    Xhat: torch.Tensor        # permuted activations, storage dtype, host
    Xq: np.ndarray
    scale: np.ndarray
    R: Optional[np.ndarray]   # the R actually used (fp64 view of stored values) or None
    rows: Optional[np.ndarray]  # sampled token rows (None = all)


_PACK_CACHE: dict = {}


def oracle_pack(kind: str, spec, L) -> dict:
    """The oracle's offline pack of a layer ('int', 'mx' or 'g128'), kept for the next test that asks for the same
    layer: the wide decode layers are packed once for all their token counts (one entry per kind; the key holds
    the layer's identity and a sample of its values).  Callers read the result, they do not change it."""
    s_t = L.get("s")
    key = (spec.cfg, spec.seed_index, spec.N, spec.K, spec.r, spec.in_dtype,
           L["W"][0, :64].double().sum().item(), L["W"][-1, -64:].double().sum().item(),
           None if s_t is None else s_t[:64].double().sum().item())
    hit = _PACK_CACHE.get(kind)
    if hit is not None and hit[0] == key:
        return hit[1]
    fn = {"int": orc.pack_weights, "mx": orc.mx_pack_weights, "g128": orc.pack_weights_grouped}[kind]
    pk = fn(f32(L["W"]), s_t.numpy() if s_t is not None else None, spec.r)
    _PACK_CACHE[kind] = (key, pk)
    return pk


def oracle_layer(spec, L, R_mode: str = "random", rows=None) -> OracleLayer:
    """Oracle-side preparation.  R_mode: 'random' (the drawn R), 'residual' (Eq. 5), 'none'."""
    pk = oracle_pack("int", spec, L)
    Xhat = workloads.permute_channels(L["X"], pk["perm"])
    Xs = Xhat if rows is None else Xhat[torch.as_tensor(rows)]
    Xq, scale = orc.quantize_act(f32(Xs), pk["s_inv"], spec.abits)
    if spec.r == 0 or R_mode == "none":
        R = None
    elif R_mode == "random":
        R = f64(L["R"])
    else:
        R = f64(torch.from_numpy(pk["R"]).to(DT[spec.in_dtype]))   # the residual as it is stored
    return OracleLayer(spec, pk, Xhat, Xq, scale, R, None if rows is None else np.asarray(rows))


def assert_y_close(Y: torch.Tensor, Y64: np.ndarray, what: str = ""):
    tol = TOL[Y.dtype]
    g, mix = orc.rel_errors(f64(Y), Y64)
    assert g <= tol and mix <= tol, f"{what}: max|dY|/max|Y| = {g:.3e}, mixed = {mix:.3e}, tol = {tol}"
    return g, mix


def ulp_close(a: np.ndarray, ref64: np.ndarray, dtype: torch.dtype, ulps: float = 1.0) -> bool:
    """|a - ref| within `ulps` units in the last place of `dtype` at ref's magnitude (plus its subnormal step)."""
    mant = {torch.float32: 24, torch.float16: 11, torch.bfloat16: 8}[dtype]
    tiny = {torch.float32: 2.0 ** -149, torch.float16: 2.0 ** -24, torch.bfloat16: 2.0 ** -133}[dtype]
    step = np.maximum(np.abs(ref64) * 2.0 ** (1 - mant), tiny)
    return bool(np.all(np.abs(a.astype(np.float64) - ref64) <= ulps * step))


def replay_check(step, outputs, inputs_mutator):
    """Run `step` eagerly, capture it, replay it three times (with eager work in between) on changed inputs."""
    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for it in range(3):
        inputs_mutator(it)
        step()                                           # eager reference on the new inputs
        torch.cuda.synchronize()
        want = [o.clone() for o in outputs]
        for o in outputs:
            o.zero_()                                    # eager work of the program's own between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, w in zip(outputs, want):
            assert torch.equal(o, w), f"replay {it} differs from the eager result"
