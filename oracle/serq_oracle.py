"""CPU oracle for the SERQ online linear layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this file: it exists so that the tests,
the smoke check and the benchmark's CPU-baseline leg have an independent, slow,
obviously-correct statement of what the HIP kernels must compute.  It shares no
code, table or helper with the HIP path.

Everything here is the plain definition written out with NumPy:

  * quantisation scale and integer codes are taken in IEEE fp32 (the precision
    the kernels use for the same decision), with round-half-to-even;
  * the integer GEMM is exact;
  * the dequantising epilogue and the rank-r compensation are evaluated in fp64.

Notation follows the paper: X activations [tokens M, input channels K],
W weights stored [output channels N, input channels K] (so a "weight row" of
the paper, one input channel, is a column here), s the static flattening
vector, P the saliency permutation, R the single compensation matrix [r, N].

Pins (tests/test_oracle_*.py): hand-worked tiny layer, the integer-layer
reduction to a textbook matmul, the scale/2 rounding bound, permutation and
flattening invariances, the r = 0 reduction, and the exact-residual identity
main + compensation == Q(X) . [W_s ; deq(Q(W_r))]; for the 4-bit compensation
matrix a hand-worked example, the integer-matrix reduction, the scale/2 bound
and the reduction to `linear` with the dequantised matrix; for MXFP4 the value
table and tie cases of the format, hand-worked blocks, the power-of-two
invariance, the error bound of the grid, brute force and a hand-worked offline
preparation; for the gated product a library routine, the odd-part identity,
limits and the reductions to the plain quantisers; for the group-128 / asymmetric
setting a hand-worked row, the reductions to the per-channel symmetric path, the
dense matmul of the dequantised operands and the half-step bounds; for the comparator
`rel_errors` hand-made pairs with known values.  No function is unpinned.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def qmax(bits: int) -> int:
    """Largest code of a symmetric n-bit grid, 2^(n-1) - 1 (Sec. 2.1, Eq. 1).

    The printed clip range "[-2^(n-1)-1, 2^(n-1)-1]" is read as the symmetric
    range [-(2^(n-1)-1), +(2^(n-1)-1)], the one consistent with the scale
    max|X| / (2^(n-1)-1) given in the same equation.
    """
    return (1 << (bits - 1)) - 1


def flatten(X: np.ndarray, s_inv) -> np.ndarray:
    """X~ = X . diag(s^-1), one fp32 multiply per element (Sec. 3.2, Eq. 4).

    `s_inv` is the reciprocal vector prepared offline (see pack_weights);
    None means the activations arrive already flattened.
    """
    X = np.asarray(X, dtype=F32)
    if s_inv is None:
        return X
    return X * np.asarray(s_inv, dtype=F32)[None, :]


def quantize_act(X: np.ndarray, s_inv, abits: int):
    """Per-token symmetric max-scaled quantisation of the flattened activations (Eq. 1).

    scale[m] = max_k |v[m,k]| / qmax   (fp32 division; 1.0 for an all-zero token)
    Xq[m,k]  = clip(rne(v[m,k] / scale[m]), -qmax, +qmax)
    Returns (Xq int8 [M,K], scale fp32 [M]).
    """
    v = flatten(X, s_inv)
    q = F32(qmax(abits))
    amax = np.max(np.abs(v), axis=1).astype(F32) if v.shape[1] else np.zeros(v.shape[0], F32)
    scale = np.where(amax > 0, amax / q, F32(1.0)).astype(F32)
    t = (v / scale[:, None]).astype(F32)
    Xq = np.clip(np.rint(t), -q, q).astype(np.int8)
    return Xq, scale


def saliency_permutation(Wt: np.ndarray) -> np.ndarray:
    """Descending-saliency order P of the input channels (Sec. 3.2, text before Eq. 5).

    After flattening, the salient weight rows (input channels) are recognised
    by their scale; the scale of channel k is taken as max_n |W~[n,k]|.  Ties
    keep the lower original index first.  perm[kp] = original channel at
    permuted position kp.
    """
    sal = np.max(np.abs(Wt), axis=0) if Wt.shape[0] else np.zeros(Wt.shape[1], F32)
    return np.argsort(-sal.astype(F32), kind="stable").astype(np.int32)


def pack_weights(W: np.ndarray, s, r: int, perm=None):
    """Offline preparation of one layer (Eq. 4, Eq. 5; per-output-channel Eq. 1).

    W [N,K] fp32 (exactly widened storage values), s [K] fp32 or None.
      W~[n,k]   = W[n,k] * s[k]                       (fp32)
      W^        = W~[:, perm]                         (salient channels lead)
      wscale[n] = max_k |W^[n,k]| / 7                 (fp32; 1.0 for a zero row)
      Wq[n,k]   = clip(rne(W^[n,k] / wscale[n]), -7, 7)
      R[j,n]    = W^[n,j] - wscale[n] * Wq[n,j],  j < r   (fp64, exact residual)
      s_inv[kp] = 1 / s[perm[kp]]                     (fp32; what quantize_act multiplies by)
    Returns dict(Wq int8 [N,K], wscale fp32 [N], perm int32 [K], s_inv fp32 [K], R fp64 [r,N]).
    """
    W = np.asarray(W, dtype=F32)
    N, K = W.shape
    s = np.ones(K, F32) if s is None else np.asarray(s, dtype=F32)
    Wt = W * s[None, :]
    perm = saliency_permutation(Wt) if perm is None else np.asarray(perm, dtype=np.int32)
    assert sorted(perm.tolist()) == list(range(K)), "perm must be a permutation of the channels"
    Wp = Wt[:, perm]
    amax = np.max(np.abs(Wp), axis=1).astype(F32)
    wscale = np.where(amax > 0, amax / F32(7), F32(1.0)).astype(F32)
    Wq = np.clip(np.rint((Wp / wscale[:, None]).astype(F32)), -7, 7).astype(np.int8)
    R = (Wp[:, :r].astype(np.float64)
         - wscale.astype(np.float64)[:, None] * Wq[:, :r].astype(np.float64)).T.copy()
    s_inv = (F32(1.0) / s)[perm].astype(F32)
    return {"Wq": Wq, "wscale": wscale, "perm": perm, "s_inv": s_inv, "R": R}


def gemm_i32(Xq: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    """acc[m,n] = sum_k Xq[m,k] * Wq[n,k], exact (Eq. 2; first term of Eq. 7).

    The contraction is done by a float64 matrix product: every operand is an
    integer of at most 8 bits and every partial sum stays far below 2^53, so
    the result is the exact integer whatever the summation order.
    """
    M, K = Xq.shape
    bound = 128.0 * 128.0 * max(K, 1)
    assert bound < 2.0 ** 31
    acc = Xq.astype(np.float64) @ Wq.astype(np.float64).T
    return acc.astype(np.int64).astype(np.int32)


def gemm_i32_loops(Xq: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    """The same sum as gemm_i32 as three nested Python loops (tiny inputs only)."""
    M, K = Xq.shape
    N = Wq.shape[0]
    acc = np.zeros((M, N), dtype=np.int64)
    for m in range(M):
        for n in range(N):
            t = 0
            for k in range(K):
                t += int(Xq[m, k]) * int(Wq[n, k])
            acc[m, n] = t
    return acc.astype(np.int32)


def lowrank(Xq: np.ndarray, R: np.ndarray, s_begin: int = 0) -> np.ndarray:
    """lr[m,n] = sum_{j<r} Xq[m, s_begin+j] * R[j,n]  in fp64 (second term of Eq. 7).

    Only the salient channel block S = [s_begin, s_begin+r) of the *quantised*
    activations takes part; the common factor scale[m] is applied in `linear`.
    """
    r = 0 if R is None else R.shape[0]
    if r == 0:
        return np.zeros((Xq.shape[0], 0 if R is None else R.shape[1]), np.float64)
    return Xq[:, s_begin:s_begin + r].astype(np.float64) @ np.asarray(R, dtype=np.float64)


def linear(Xq, scale, Wq, wscale, R=None, s_begin: int = 0, acc=None) -> np.ndarray:
    """Y[m,n] = scale[m] * ( wscale[n] * acc[m,n] + lr[m,n] )  in fp64 (Eq. 2 + Eq. 7).

    `R` holds the values actually stored (fp16/bf16 widened exactly) or None / r = 0
    for the plain W4A4 / W4A8 GEMM.  `acc` may be passed in to reuse a GEMM.
    """
    if acc is None:
        acc = gemm_i32(Xq, Wq)
    y = np.asarray(wscale, np.float64)[None, :] * acc.astype(np.float64)
    if R is not None and R.shape[0] > 0:
        y = y + lowrank(Xq, R, s_begin)
    return np.asarray(scale, np.float64)[:, None] * y


def quantize_lowrank(R: np.ndarray):
    """Q(R): the compensation matrix itself on the INT4 grid (Sec. 3.2, second line of Eq. 7).

    R [r, N] holds the values actually stored (fp16/bf16 widened exactly).  The
    grid is the weights' one, Eq. 1 per output channel n (a column of R here):
      rscale[n] = max_j |R[j,n]| / 7              (fp32 division; 1.0 for a zero column)
      Rq[j,n]   = clip(rne(R[j,n] / rscale[n]), -7, 7)
    Returns (Rq int8 [r, N], rscale fp32 [N]).
    """
    R = np.asarray(R, dtype=F32)
    r, N = R.shape
    amax = np.max(np.abs(R), axis=0).astype(F32) if r else np.zeros(N, F32)
    rscale = np.where(amax > 0, amax / F32(7), F32(1.0)).astype(F32)
    Rq = np.clip(np.rint((R / rscale[None, :]).astype(F32)), -7, 7).astype(np.int8)
    return Rq, rscale


def lowrank_i32(Xq: np.ndarray, Rq: np.ndarray, s_begin: int = 0) -> np.ndarray:
    """acc_r[m,n] = sum_{j<r} Xq[m, s_begin+j] * Rq[j,n], exact (integer form of the second term of Eq. 7)."""
    r = Rq.shape[0]
    a = Xq[:, s_begin:s_begin + r].astype(np.int64) @ Rq.astype(np.int64)
    assert r * 128 * 8 < 2 ** 31
    return a.astype(np.int32)


def linear_q4r(Xq, scale, Wq, wscale, Rq, rscale, s_begin: int = 0, acc=None) -> np.ndarray:
    """Y[m,n] = scale[m] * ( wscale[n] * acc[m,n] + rscale[n] * acc_r[m,n] )  in fp64.

    The all-low-precision form of Eq. 7 (second line): both products are integer
    GEMMs and each is dequantised by its own per-output-channel scale.
    """
    if acc is None:
        acc = gemm_i32(Xq, Wq)
    acc_r = lowrank_i32(Xq, Rq, s_begin)
    y = (np.asarray(wscale, np.float64)[None, :] * acc.astype(np.float64)
         + np.asarray(rscale, np.float64)[None, :] * acc_r.astype(np.float64))
    return np.asarray(scale, np.float64)[:, None] * y


# ---------------------------------------------------------------------------
# The accuracy-table setting (Sec. 4.1, implementation details): weights quantised in
# groups of 128 input channels (round-to-nearest, symmetric), activations per token with
# round-to-nearest ASYMMETRIC integer quantisation.  The paper names the scheme and gives
# no formulas; the arithmetic below is the usual min-max affine quantiser:
#   range [lo, hi] widened to contain 0, scale = (hi - lo) / (2^n - 1),
#   zero = rne(-lo / scale), code = clip(rne(v / scale) + zero, 0, 2^n - 1),
#   v^ = scale * (code - zero).
# Codes are returned re-centred (code - 2^(n-1), zero - 2^(n-1)) so that they fit the signed
# containers of the symmetric path; the dequantised values are the same.
# ---------------------------------------------------------------------------
GROUP = 128


def quantize_act_asym(X: np.ndarray, s_inv, abits: int):
    """Per-token asymmetric quantisation of the flattened activations (Eq. 4, then Sec. 4.1).

    All decisions in IEEE fp32, as for the symmetric quantiser:
      lo = min(0, min_k v), hi = max(0, max_k v)
      scale[m] = (hi - lo) / (2^n - 1)            (1.0 for an all-zero token)
      z[m]     = rne(-lo / scale)                 (0 .. 2^n - 1)
      c[m,k]   = clip(rne(v / scale) + z, 0, 2^n - 1)
    Returns (Xq int8 [M,K] = c - 2^(n-1), scale fp32 [M], zero int32 [M] = z - 2^(n-1));
    the token stands for scale * (Xq - zero).
    """
    v = flatten(X, s_inv)
    M, K = v.shape
    top = F32((1 << abits) - 1)
    half = 1 << (abits - 1)
    lo = np.minimum(np.min(v, axis=1), F32(0)).astype(F32) if K else np.zeros(M, F32)
    hi = np.maximum(np.max(v, axis=1), F32(0)).astype(F32) if K else np.zeros(M, F32)
    span = (hi - lo).astype(F32)
    scale = np.where(span > 0, span / top, F32(1.0)).astype(F32)
    z = np.rint((-lo / scale).astype(F32)).astype(F32)
    t = np.rint((v / scale[:, None]).astype(F32)).astype(F32)
    c = np.clip((t + z[:, None]).astype(F32), F32(0), top)
    return (c - F32(half)).astype(np.int8), scale, (z - F32(half)).astype(np.int32)


def group_scales(Wp: np.ndarray, group: int = GROUP) -> np.ndarray:
    """One symmetric INT4 scale per output channel and group of `group` input channels (Eq. 1 per group),
    stored in 16 bits as the paper's effective-bit-width accounting assumes (4 + 16/128 = 4.125 bits):
      gscale[n,g] = fp16_rne(max_{k in g} |W^[n,k]| / 7), kept inside fp16's positive range
      [2^-24, 65504]; 1.0 for an all-zero group.  Returned widened to fp32 [N, K/group].
    """
    Wp = np.asarray(Wp, dtype=F32)
    N, K = Wp.shape
    assert K % group == 0
    amax = np.max(np.abs(Wp.reshape(N, K // group, group)), axis=2).astype(F32)
    with np.errstate(over="ignore"):
        g16 = (amax / F32(7)).astype(F32).astype(np.float16)
    g = g16.astype(F32)
    g = np.clip(g, F32(2.0 ** -24), F32(65504.0)).astype(F32)
    return np.where(amax > 0, g, F32(1.0)).astype(F32)


def pack_weights_grouped(W: np.ndarray, s, r: int, perm=None, group: int = GROUP):
    """Offline preparation with group-wise weight scales (Eq. 4, Eq. 5; Eq. 1 per group of 128 channels).

      W^        = (W * s)[:, perm]                         fp32, salient channels lead
      gscale    = group_scales(W^)                         [N, K/128]
      Wq[n,k]   = clip(rne(W^[n,k] / gscale[n, k//128]), -7, 7)
      R[j,n]    = W^[n,j] - gscale[n, j//128] * Wq[n,j],  j < r   (fp64, exact residual)
      wsum[n]   = sum_k gscale[n, k//128] * Wq[n,k]        (fp64; what a zero point multiplies)
    Returns dict(Wq, gscale, wsum, perm, s_inv, R).
    """
    W = np.asarray(W, dtype=F32)
    N, K = W.shape
    s = np.ones(K, F32) if s is None else np.asarray(s, dtype=F32)
    Wt = W * s[None, :]
    perm = saliency_permutation(Wt) if perm is None else np.asarray(perm, dtype=np.int32)
    assert sorted(perm.tolist()) == list(range(K)), "perm must be a permutation of the channels"
    Wp = Wt[:, perm]
    gs = group_scales(Wp, group)
    gfull = np.repeat(gs, group, axis=1)
    Wq = np.clip(np.rint((Wp / gfull).astype(F32)), -7, 7).astype(np.int8)
    deq = gfull.astype(np.float64) * Wq.astype(np.float64)
    R = (Wp[:, :r].astype(np.float64) - deq[:, :r]).T.copy()
    return {"Wq": Wq, "gscale": gs, "wsum": deq.sum(axis=1), "perm": perm,
            "s_inv": (F32(1.0) / s)[perm].astype(F32), "R": R}


def gemm_i32_grouped(Xq: np.ndarray, Wq: np.ndarray, group: int = GROUP) -> np.ndarray:
    """acc[g,m,n] = sum_{k in group g} Xq[m,k] * Wq[n,k], exact: the integer GEMM of Eq. 2 cut at the
    group boundaries, because every group is dequantised with its own scale."""
    M, K = Xq.shape
    N = Wq.shape[0]
    G = K // group
    out = np.empty((G, M, N), dtype=np.int32)
    for g in range(G):
        out[g] = gemm_i32(Xq[:, g * group:(g + 1) * group], Wq[:, g * group:(g + 1) * group])
    return out


def linear_grouped(Xq, scale, zero, Wq, gscale, R=None, s_begin: int = 0, group: int = GROUP) -> np.ndarray:
    """The layer with group-wise weight scales and asymmetric activations, in fp64 (Eq. 2 + Eq. 7, first line):

      Y[m,n] = sum_k x^[m,k] w^[n,k] + sum_{j<r} x^[m,S_j] R[j,n],
      x^[m,k] = scale[m] (Xq[m,k] - zero[m]),  w^[n,k] = gscale[n, k//128] Wq[n,k],

    evaluated as the definition says: group by group for the integer part, the zero point as its own term.
    `zero` may be None (symmetric codes)."""
    M, K = Xq.shape
    N = Wq.shape[0]
    z = np.zeros(M, np.float64) if zero is None else np.asarray(zero, np.float64)
    gs = np.asarray(gscale, np.float64)                                      # [N, G]
    y = np.zeros((M, N), np.float64)
    wsum = np.zeros(N, np.float64)
    for g in range(K // group):                                              # one exact integer GEMM per group
        sl = slice(g * group, (g + 1) * group)
        y += gemm_i32(Xq[:, sl], Wq[:, sl]).astype(np.float64) * gs[None, :, g]
        wsum += gs[:, g] * Wq[:, sl].astype(np.float64).sum(axis=1)
    y -= z[:, None] * wsum[None, :]
    if R is not None and R.shape[0] > 0:
        r = R.shape[0]
        xs = Xq[:, s_begin:s_begin + r].astype(np.float64) - z[:, None]
        y = y + xs @ np.asarray(R, np.float64)
    return np.asarray(scale, np.float64)[:, None] * y


# ---------------------------------------------------------------------------
# MXFP4: the 4-bit Microscaling format the paper's W4A4 latency runs use
# (Sec. 4.1; appendix on the MX format: blocks of 32 elements sharing one
# 8-bit power-of-two scale taken from the block's maximum, elements in a 4-bit
# floating-point format).  The arithmetic below follows the published OCP
# Microscaling specification for MXFP4: element format E2M1 (values
# +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}), scale format E8M0.
# ---------------------------------------------------------------------------
MX_BLOCK = 32
E2M1_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=F32)
_E2M1_MID = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], dtype=F32)   # midpoints of neighbouring values


def e2m1_round(t: np.ndarray) -> np.ndarray:
    """Nearest E2M1 code (0..15: sign bit 8, magnitude index 0..7) of each element of t.

    Round to nearest, ties to the code with an even mantissa bit (index 0, 2, 4, 6:
    values 0, 1, 2, 4), magnitudes above 6 saturate to 6; zero keeps sign 0.
    """
    t = np.asarray(t, dtype=F32)
    a = np.abs(t)
    idx = np.searchsorted(_E2M1_MID, a, side="left")               # midpoints strictly below |t|
    tie = (idx < 7) & (a == _E2M1_MID[np.minimum(idx, 6)])
    idx = np.where(tie & (idx % 2 == 1), idx + 1, idx)             # at a tie idx is the lower neighbour
    idx = np.minimum(idx, 7)
    sign = (t < 0) & (idx > 0)
    return (idx + 8 * sign).astype(np.uint8)


def mx_quantize(V: np.ndarray):
    """MXFP4 quantisation of the last axis in blocks of 32.

    Per block: shared exponent se = max(floor(log2(max|v|)) - 2, -127) (2 = exponent of
    the largest E2M1 value; 0 for an all-zero block), stored biased as E = se + 127;
    elements e2m1_round(v / 2^se).  Division by a power of two is exact in fp32.
    Returns (codes uint8 [..., K] with values 0..15, E uint8 [..., K/32]).
    """
    V = np.asarray(V, dtype=F32)
    K = V.shape[-1]
    assert K % MX_BLOCK == 0
    B = V.reshape(V.shape[:-1] + (K // MX_BLOCK, MX_BLOCK))
    amax = np.max(np.abs(B), axis=-1)
    _, ex = np.frexp(amax)                                          # amax = m * 2^ex, m in [0.5, 1)
    se = np.where(amax > 0, np.maximum(ex.astype(np.int32) - 1 - 2, -127), 0).astype(np.int32)
    t = np.ldexp(B, -se[..., None]).astype(F32)
    codes = e2m1_round(t).reshape(V.shape)
    return codes, (se + 127).astype(np.uint8)


def mx_dequantize(codes: np.ndarray, E: np.ndarray) -> np.ndarray:
    """The fp64 values an MXFP4 tensor stands for: +-E2M1 value * 2^(E - 127) per block of 32."""
    codes = np.asarray(codes)
    mag = E2M1_VALUES.astype(np.float64)[codes & 7]
    val = np.where(codes & 8, -mag, mag)
    scale = np.ldexp(1.0, np.asarray(E, dtype=np.int32) - 127)
    return val * np.repeat(scale, MX_BLOCK, axis=-1)


def mx_pack_weights(W: np.ndarray, s, r: int, perm=None):
    """Offline preparation for the MXFP4 path (Eq. 4, Eq. 5 with Q = MXFP4 along the input channels).

      W^ = (W * s)[:, perm]                    fp32, salient channels lead
      Wc, We = mx_quantize(W^)                 per output channel, blocks of 32 input channels
      R[n, j] = W^[n, j] - deq(Wc, We)[n, j]   j < r, one fp32 subtraction
      Rc, Re = mx_quantize(R)                  the compensation matrix in MXFP4 as well (Eq. 7, second line)
    Returns dict(Wc, We, Rc, Re, perm, s_inv); Rc is [N, r] (output channel major, like Wc).
    """
    W = np.asarray(W, dtype=F32)
    N, K = W.shape
    s = np.ones(K, F32) if s is None else np.asarray(s, dtype=F32)
    Wt = W * s[None, :]
    perm = saliency_permutation(Wt) if perm is None else np.asarray(perm, dtype=np.int32)
    Wp = Wt[:, perm]
    Wc, We = mx_quantize(Wp)
    out = {"Wc": Wc, "We": We, "perm": perm, "s_inv": (F32(1.0) / s)[perm].astype(F32)}
    if r > 0:
        R = (Wp[:, :r] - mx_dequantize(Wc[:, :r], We[:, :r // MX_BLOCK]).astype(F32)).astype(F32)
        out["Rc"], out["Re"] = mx_quantize(R)
    return out


def mx_quantize_act(X: np.ndarray, s_inv):
    """Online step for the MXFP4 path: flatten (Eq. 4), then MXFP4 per token in blocks of 32 channels."""
    return mx_quantize(flatten(X, s_inv))


def mx_linear(Xc, Xe, Wc, We, Rc=None, Re=None, s_begin: int = 0) -> np.ndarray:
    """Y = deq(X) . deq(W)^T + deq(X)[:, S] . deq(R)^T in fp64 (Eq. 7, second line, with Q = MXFP4)."""
    Xd = mx_dequantize(Xc, Xe)
    Y = Xd @ mx_dequantize(Wc, We).T
    if Rc is not None and Rc.shape[1] > 0:
        r = Rc.shape[1]
        Y = Y + Xd[:, s_begin:s_begin + r] @ mx_dequantize(Rc, Re).T
    return Y


# ---------------------------------------------------------------------------
# Producer side of the down projection: the gated product, quantised where it is made
# (Sec. 3.2, "Offline Weight Permutation" / the decoder-layer flow of Fig. 2(b): the
# input of the down projection is act(gate) * up in the permuted channel order, and the
# flattening is merged into the adjacent step)
# ---------------------------------------------------------------------------
def silu(x: np.ndarray) -> np.ndarray:
    """x * sigmoid(x) in fp64."""
    x = np.asarray(x, dtype=np.float64)
    with np.errstate(over="ignore"):
        return x / (1.0 + np.exp(-x))


def swiglu(gate: np.ndarray, up: np.ndarray) -> np.ndarray:
    """silu(gate) * up, evaluated in fp64 and rounded once to fp32: the activations the
    down projection would receive if the product were stored unrounded."""
    return (silu(gate) * np.asarray(up, dtype=np.float64)).astype(F32)


def swiglu_quantize_act(gate, up, s_inv, abits: int):
    """quantize_act (Eq. 4 + Eq. 1) of the gated product."""
    return quantize_act(swiglu(gate, up), s_inv, abits)


def mx_swiglu_quantize_act(gate, up, s_inv):
    """mx_quantize_act of the gated product."""
    return mx_quantize_act(swiglu(gate, up), s_inv)


def linear_f32(Xq, scale, Wq, wscale, R=None, s_begin: int = 0, acc=None) -> np.ndarray:
    """The same formula evaluated in fp32 in the stated order (documents fp32's share of the tolerance)."""
    if acc is None:
        acc = gemm_i32(Xq, Wq)
    y = np.asarray(wscale, F32)[None, :] * acc.astype(F32)
    if R is not None and R.shape[0] > 0:
        r = R.shape[0]
        y = y + (Xq[:, s_begin:s_begin + r].astype(F32) @ np.asarray(R, dtype=F32)).astype(F32)
    return (np.asarray(scale, F32)[:, None] * y).astype(F32)


def dequant_reference(X, s, W, r: int, abits: int, perm=None):
    """Convenience: the whole layer from unquantised inputs, with the exact residual R.

    Returns (Y fp64, pieces dict).  Used by the tests that check the
    compensation really reduces the error of the salient channels.
    """
    pk = pack_weights(W, s, r, perm)
    Xp = np.asarray(X, dtype=F32)[:, pk["perm"]]
    Xq, scale = quantize_act(Xp, pk["s_inv"], abits)
    Y = linear(Xq, scale, pk["Wq"], pk["wscale"], pk["R"] if r > 0 else None)
    pk.update({"Xq": Xq, "scale": scale})
    return Y, pk


def rel_errors(Y, Y64):
    """The two error measures the parity tests use for Y (the reading of "max relative error").

    global : max |Y - Y64| / max |Y64|
    mixed  : max over elements of |Y - Y64| / (|Y64| + rms(Y64))
    Both are 0 for empty inputs.  Against an all-zero reference any non-zero difference is an
    infinite relative error (and an exact match is 0).
    """
    Y = np.asarray(Y, np.float64)
    Y64 = np.asarray(Y64, np.float64)
    if Y64.size == 0:
        return 0.0, 0.0
    d = np.abs(Y - Y64)
    dmax = float(np.max(d))
    denom = float(np.max(np.abs(Y64)))
    rms = float(np.sqrt(np.mean(Y64 * Y64)))
    if denom == 0.0:
        e = 0.0 if dmax == 0.0 else float("inf")
        return e, e
    return dmax / denom, float(np.max(d / (np.abs(Y64) + rms)))


def effective_weight_bits(K: int, N: int, r: int, group: int = 0, scale_bits: int = 16,
                          r_bits: int = 4) -> float:
    """Stored bits per main-weight element for one layer (Tables 1-2, effective bit-width).

    4-bit codes, one `scale_bits` scale per group of `group` input channels
    (group = 0: one per output channel), plus an r x N compensation matrix of
    `r_bits`-bit codes.
    """
    n_w = K * N
    bits = 4.0 * n_w
    bits += scale_bits * (N * (K // group) if group else N)
    bits += r_bits * r * N
    return bits / n_w
