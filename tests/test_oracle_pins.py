"""Pins for the CPU oracle: every check here compares it with something other than itself.

Hand-worked numbers (tests/golden/tiny_layer.txt), textbook integer matmul,
the rounding bound of Eq. 1, the exact identities of Eq. 4 / Eq. 6, the r = 0
reduction (Eq. 2), and the exact-residual identity behind Eq. 5 + Eq. 7.
"""
import os

import numpy as np
import pytest

import workloads
from oracle import serq_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _read_golden(path):
    out = {}
    with open(path) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        name, rows, cols = lines[i].split()
        rows, cols = int(rows), int(cols)
        data = [[float(t) for t in lines[i + 1 + r].split()] for r in range(rows)]
        arr = np.array(data, dtype=np.float64)
        assert arr.shape == (rows, cols)
        out[name] = arr
        i += 1 + rows
    return out


def test_T1_hand_worked_tiny_layer():
    g = _read_golden(os.path.join(HERE, "golden", "tiny_layer.txt"))
    X, W, s = g["X"].astype(np.float32), g["W"].astype(np.float32), g["s"][0].astype(np.float32)
    pk = orc.pack_weights(W, s, r=2)
    assert pk["perm"].tolist() == g["perm"][0].astype(int).tolist()
    assert np.array_equal(pk["s_inv"], g["s_inv"][0].astype(np.float32))
    assert np.array_equal(pk["wscale"], g["wscale"][0].astype(np.float32))
    assert np.array_equal(pk["Wq"], g["Wq"].astype(np.int8))
    assert np.array_equal(pk["R"], g["R"])
    Xp = X[:, pk["perm"]]
    Xq, scale = orc.quantize_act(Xp, pk["s_inv"], 4)
    assert np.array_equal(scale, g["scale"][0].astype(np.float32))
    assert np.array_equal(Xq, g["Xq"].astype(np.int8))
    acc = orc.gemm_i32(Xq, pk["Wq"])
    assert np.array_equal(acc, g["acc"].astype(np.int32))
    assert np.array_equal(orc.gemm_i32_loops(Xq, pk["Wq"]), g["acc"].astype(np.int32))
    Y = orc.linear(Xq, scale, pk["Wq"], pk["wscale"], pk["R"])
    assert np.array_equal(Y, g["Y"])
    Yf = orc.linear_f32(Xq, scale, pk["Wq"], pk["wscale"], pk["R"])
    assert np.array_equal(Yf.astype(np.float64), g["Y"])
    # the one-call convenience path gives the same answer
    Y2, _ = orc.dequant_reference(X, s, W, 2, 4)
    assert np.array_equal(Y2, g["Y"])


@pytest.mark.parametrize("abits", [4, 8])
def test_T2_integer_layer_is_textbook_matmul(abits):
    q = orc.qmax(abits)
    X, W = workloads.integer_layer(M=9, K=64, N=13, qx=q, seed=7 + abits)
    pk = orc.pack_weights(W, None, r=0, perm=np.arange(64))
    Xq, scale = orc.quantize_act(X, None, abits)
    assert np.all(scale == 1.0) and np.all(pk["wscale"] == 1.0)
    assert np.array_equal(Xq.astype(np.float32), X)
    assert np.array_equal(pk["Wq"].astype(np.float32), W)
    want = X.astype(np.int64) @ W.astype(np.int64).T
    assert np.array_equal(orc.gemm_i32(Xq, pk["Wq"]).astype(np.int64), want)
    Y = orc.linear(Xq, scale, pk["Wq"], pk["wscale"])
    assert np.array_equal(Y, want.astype(np.float64))


def test_rounding_is_half_to_even():
    # scale is exactly 1 (row maximum 7): codes are rne of the values themselves
    X = np.array([[7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 4.5, -6.5, 6.49, -3.51]], np.float32)
    Xq, scale = orc.quantize_act(X, None, 4)
    assert scale[0] == 1.0
    assert Xq[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 4, 4, -6, 6, -4]


@pytest.mark.parametrize("abits", [4, 8])
def test_quantiser_at_the_bottom_of_the_exponent_range(abits):
    # a token whose values are k * 2^-140 (exact subnormals): the scale is itself subnormal and the codes
    # follow from exact rational arithmetic
    from fractions import Fraction
    q = orc.qmax(abits)
    ks = np.array([100, -100, 37, -1, 0, 64, 99, -50, 13, 7, 3, 51], dtype=np.int64)
    X = np.ldexp(ks.astype(np.float64), -140).astype(np.float32)[None, :]
    assert np.array_equal(np.ldexp(X.astype(np.float64), 140)[0], ks)          # nothing was lost
    Xq, scale = orc.quantize_act(X, None, abits)
    # scale = rne(100 * 2^-140 / q) to a multiple of 2^-149 = rne(51200 / q) * 2^-149
    num = Fraction(100 * 512, q)
    sc_int = int(num) + (1 if (num - int(num) > Fraction(1, 2) or (num - int(num) == Fraction(1, 2) and int(num) % 2)) else 0)
    assert float(scale[0]) == float(np.ldexp(float(sc_int), -149))
    want = []
    for k in ks.tolist():
        t = Fraction(k * 512, sc_int)                     # exact quotient; fp32 rounds it to 24 bits, far from any tie here
        n = int(t + Fraction(1, 2)) if t >= 0 else -int(-t + Fraction(1, 2))
        assert abs(abs(t - int(t)) - Fraction(1, 2)) > Fraction(1, 100000)      # fp32 resolves 2^-22 here
        want.append(max(-q, min(q, n)))
    assert Xq[0].tolist() == want
    assert abs(int(Xq[0, 0])) == q


def test_zero_token_and_zero_weight_row():
    X = np.zeros((2, 16), np.float32)
    X[1, 3] = -2.0
    Xq, scale = orc.quantize_act(X, None, 8)
    assert scale[0] == 1.0 and not Xq[0].any()
    assert Xq[1, 3] == -127 and scale[1] == np.float32(2.0) / np.float32(127)
    W = np.zeros((2, 16), np.float32)
    W[0, 1] = 1.0
    pk = orc.pack_weights(W, None, 0)
    assert pk["wscale"][1] == 1.0 and not pk["Wq"][1].any()


@pytest.mark.parametrize("abits", [4, 8])
def test_T3_rounding_bound_and_extremes(abits):
    spec = workloads.config1().with_(M=33, K=512, abits=abits)
    L = workloads.make_layer(spec, want=("X", "s"))
    X = L["X"].float().numpy()
    s_inv = (np.float32(1) / L["s"].numpy()).astype(np.float32)
    Xq, scale = orc.quantize_act(X, s_inv, abits)
    q = orc.qmax(abits)
    v = X.astype(np.float64) * s_inv.astype(np.float64)  # the exact product
    v32 = (X * s_inv[None, :]).astype(np.float64)
    assert np.max(np.abs(Xq)) <= q
    err = np.abs(v32 - scale.astype(np.float64)[:, None] * Xq)
    assert np.all(err <= 0.5 * scale[:, None] * (1 + 1e-6))
    # fp32 flattening is within one rounding of the exact product
    assert np.all(np.abs(v - v32) <= np.abs(v) * 2.0 ** -24 + 1e-300)
    am = np.argmax(np.abs(v32), axis=1)
    rows = np.arange(X.shape[0])
    assert np.all(np.abs(Xq[rows, am]) == q)
    assert np.all(np.sign(Xq[rows, am]) == np.sign(v32[rows, am]))
    assert np.allclose(scale, np.max(np.abs(v32), axis=1) / q, rtol=1e-7)


def test_T4_permutation_invariance():
    spec = workloads.config1().with_(M=5, K=128, N=24, r=16)
    L = workloads.make_layer(spec)
    X, W, s = L["X"].float().numpy(), L["W"].float().numpy(), L["s"].numpy()
    Y0, p0 = orc.dequant_reference(X, s, W, 16, 4)
    rng = np.random.default_rng(5)
    pi = rng.permutation(128)
    # the same layer with its input channels presented in another order
    Y1, p1 = orc.dequant_reference(X[:, pi], s[pi], W[:, pi], 16, 4)
    assert np.array_equal(p0["scale"], p1["scale"])
    assert np.array_equal(p0["wscale"], p1["wscale"])
    assert np.array_equal(orc.gemm_i32(p0["Xq"], p0["Wq"]), orc.gemm_i32(p1["Xq"], p1["Wq"]))
    # the saliency order picks the same physical channels, so S maps to itself
    assert np.array_equal(pi[p1["perm"]][:16], p0["perm"][:16])
    assert np.allclose(Y0, Y1, rtol=1e-12, atol=1e-12)
    # an arbitrary (non-saliency) order of the non-salient channels changes nothing either
    perm2 = np.concatenate([p0["perm"][:16], rng.permutation(p0["perm"][16:])])
    Y2, p2 = orc.dequant_reference(X, s, W, 16, 4, perm=perm2)
    assert np.array_equal(orc.gemm_i32(p0["Xq"], p0["Wq"]), orc.gemm_i32(p2["Xq"], p2["Wq"]))
    assert np.allclose(Y0, Y2, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("abits", [4, 8])
def test_T5_rank_zero_is_plain_quantised_gemm(abits):
    spec = workloads.config1().with_(M=6, K=64, N=20, r=16, abits=abits)
    L = workloads.make_layer(spec)
    X, W, s = L["X"].float().numpy(), L["W"].float().numpy(), L["s"].numpy()
    pk = orc.pack_weights(W, s, 16)
    Xq, scale = orc.quantize_act(X[:, pk["perm"]], pk["s_inv"], abits)
    acc = orc.gemm_i32_loops(Xq, pk["Wq"]).astype(np.float64)
    plain = scale.astype(np.float64)[:, None] * pk["wscale"].astype(np.float64)[None, :] * acc
    assert np.allclose(orc.linear(Xq, scale, pk["Wq"], pk["wscale"], None), plain, rtol=1e-15)
    assert np.allclose(orc.linear(Xq, scale, pk["Wq"], pk["wscale"], np.zeros((16, 20))), plain, rtol=1e-15)
    assert np.allclose(orc.linear(Xq, scale, pk["Wq"], pk["wscale"], np.zeros((0, 20))), plain, rtol=1e-15)


@pytest.mark.parametrize("abits,r", [(4, 16), (8, 32)])
def test_T6_exact_residual_identity(abits, r):
    """main + compensation == deq(Xq) . [W~_s ; deq(Wq_r)]^T with the unrounded residual (Eq. 5 + Eq. 7)."""
    spec = workloads.config1().with_(M=7, K=96, N=40, r=r, abits=abits)
    L = workloads.make_layer(spec)
    X, W, s = L["X"].float().numpy(), L["W"].float().numpy(), L["s"].numpy()
    Y, pk = orc.dequant_reference(X, s, W, r, abits)
    Wt = (W * s[None, :])[:, pk["perm"]].astype(np.float64)          # folded, permuted, unquantised
    Wmix = pk["wscale"].astype(np.float64)[:, None] * pk["Wq"].astype(np.float64)
    Wmix[:, :r] = Wt[:, :r]                                           # salient channels exact
    Xdq = pk["scale"].astype(np.float64)[:, None] * pk["Xq"].astype(np.float64)
    want = Xdq @ Wmix.T
    assert np.allclose(Y, want, rtol=1e-12, atol=1e-12 * np.max(np.abs(want)))
    # a transposed / shifted use of R would not satisfy it
    Rbad = np.roll(pk["R"], 1, axis=0)
    Ybad = orc.linear(pk["Xq"], pk["scale"], pk["Wq"], pk["wscale"], Rbad)
    assert not np.allclose(Ybad, want, rtol=1e-6, atol=1e-9)


def test_T7_residual_is_at_most_half_a_step():
    spec = workloads.config1().with_(K=128, N=64, r=32)
    L = workloads.make_layer(spec, want=("W", "s"))
    pk = orc.pack_weights(L["W"].float().numpy(), L["s"].numpy(), 32)
    assert np.all(np.abs(pk["R"]) <= 0.5 * pk["wscale"].astype(np.float64)[None, :] * (1 + 1e-6))
    assert np.max(np.abs(pk["R"])) > 0


@pytest.mark.parametrize("abits", [4, 8])
def test_T8_flattening_identity_power_of_two(abits):
    """(X, W, s) and (X/s, W*s, 1) give bit-identical results when s is exact (Eq. 4)."""
    spec = workloads.config1().with_(M=6, K=64, N=24, r=16, abits=abits)
    L = workloads.make_layer(spec)
    X, W = L["X"].float().numpy(), L["W"].float().numpy()
    rng = np.random.default_rng(11)
    s = (2.0 ** rng.integers(-3, 4, size=64)).astype(np.float32)
    Ya, pa = orc.dequant_reference(X, s, W, 16, abits)
    Yb, pb = orc.dequant_reference(X / s[None, :], None, W * s[None, :], 16, abits)
    assert np.array_equal(pa["perm"], pb["perm"])
    assert np.array_equal(pa["Xq"], pb["Xq"]) and np.array_equal(pa["scale"], pb["scale"])
    assert np.array_equal(pa["Wq"], pb["Wq"]) and np.array_equal(pa["wscale"], pb["wscale"])
    assert np.array_equal(Ya, Yb)


def test_T9_compensation_reduces_output_error():
    spec = workloads.config2().with_(M=64, K=512, N=256, r=32, n_outlier=5)
    L = workloads.make_layer(spec)
    X, W, s = L["X"].float().numpy(), L["W"].float().numpy(), L["s"].numpy()
    exact = X.astype(np.float64) @ W.astype(np.float64).T
    errs = []
    for r in (0, 8, 32):
        Y, pk = orc.dequant_reference(X, s, W, r, 4)
        errs.append(np.linalg.norm(Y - exact))
        if r:
            assert set(L["outliers"].tolist()) <= set(pk["perm"][:8].tolist())
    assert errs[2] < errs[1] < errs[0]


def test_gemm_matches_loops_and_int64():
    rng = np.random.default_rng(3)
    Xq = rng.integers(-127, 128, size=(5, 40)).astype(np.int8)
    Wq = rng.integers(-7, 8, size=(9, 40)).astype(np.int8)
    a = orc.gemm_i32(Xq, Wq)
    assert a.dtype == np.int32
    assert np.array_equal(a, orc.gemm_i32_loops(Xq, Wq))
    assert np.array_equal(a.astype(np.int64), Xq.astype(np.int64) @ Wq.astype(np.int64).T)
    # extreme magnitudes at a large K stay exact
    Xq = np.full((2, 16384), -127, np.int8)
    Wq = np.full((3, 16384), 7, np.int8)
    assert np.all(orc.gemm_i32(Xq, Wq) == -127 * 7 * 16384)


def test_lowrank_uses_the_salient_block_only():
    rng = np.random.default_rng(9)
    Xq = rng.integers(-7, 8, size=(4, 64)).astype(np.int8)
    R = rng.standard_normal((16, 6))
    want = np.zeros((4, 6))
    for m in range(4):
        for n in range(6):
            want[m, n] = sum(float(Xq[m, 16 + j]) * R[j, n] for j in range(16))
    assert np.allclose(orc.lowrank(Xq, R, s_begin=16), want, rtol=1e-14, atol=1e-14)


def test_T11_effective_weight_bits():
    # group-128 scales alone: 4 + 16/128 (Table 2, "4.13")
    assert orc.effective_weight_bits(4096, 4096, 0, group=128) == pytest.approx(4.125)
    # LLaMA-2-7B decoder layer mix with r = 128, 4-bit R (Table 1, "4.24")
    layers = [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)]
    tot = sum(k * n for k, n in layers)
    eff = sum(orc.effective_weight_bits(k, n, 128, group=128) * k * n for k, n in layers) / tot
    assert 4.225 <= eff <= 4.245
    # 8-bit low-rank factors of the same parameter count (Table 1, "4.35" for the two-factor baseline)
    eff8 = sum(orc.effective_weight_bits(k, n, 128, group=128, r_bits=8) * k * n for k, n in layers) / tot
    assert 4.33 <= eff8 <= 4.355


# ---------------------------------------------------------------------------
# the 4-bit compensation matrix Q(R) (Eq. 7, second line)
# ---------------------------------------------------------------------------
def test_q4r_hand_worked_example():
    g = _read_golden(os.path.join(HERE, "golden", "tiny_lowrank_q4.txt"))
    Rq, rscale = orc.quantize_lowrank(g["R"])
    assert np.array_equal(rscale, g["rscale"][0].astype(np.float32))
    assert np.array_equal(Rq, g["Rq"].astype(np.int8))
    Xq = g["Xq"].astype(np.int8)
    assert np.array_equal(orc.lowrank_i32(Xq, Rq), g["acc_r"].astype(np.int32))
    Y = orc.linear_q4r(Xq, g["scale"][0], None, g["wscale"][0], Rq, rscale, acc=g["acc"].astype(np.int32))
    assert np.array_equal(Y, g["Y"])


def test_q4r_integer_matrix_is_textbook_matmul():
    # R integer-valued in [-7, 7] with a +-7 in every column: rscale = 1, codes = R, and the whole
    # layer is two textbook integer matrix products
    rng = np.random.default_rng(5)
    M, K, N, r, s_begin = 5, 96, 7, 48, 32
    R = rng.integers(-7, 8, size=(r, N))
    R[rng.integers(0, r, size=N), np.arange(N)] = rng.choice([-7, 7], size=N)
    Rq, rscale = orc.quantize_lowrank(R.astype(np.float32))
    assert np.all(rscale == 1.0) and np.array_equal(Rq, R.astype(np.int8))
    Xq = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    Wq = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    Y = orc.linear_q4r(Xq, np.ones(M, np.float32), Wq, np.ones(N, np.float32), Rq, rscale, s_begin=s_begin)
    want = Xq.astype(np.int64) @ Wq.astype(np.int64).T + Xq[:, s_begin:s_begin + r].astype(np.int64) @ R
    assert np.array_equal(Y, want.astype(np.float64))
    # brute force over the definition
    acc_r = orc.lowrank_i32(Xq, Rq, s_begin)
    for m in range(M):
        for n in range(N):
            assert acc_r[m, n] == sum(int(Xq[m, s_begin + j]) * int(R[j, n]) for j in range(r))


def test_q4r_rounding_bound_and_extremes():
    rng = np.random.default_rng(6)
    R = (rng.standard_normal((64, 40)) * 0.01).astype(np.float32)
    R[:, 3] = 0.0
    Rq, rscale = orc.quantize_lowrank(R)
    assert rscale[3] == 1.0 and not Rq[:, 3].any()
    assert np.max(np.abs(Rq)) <= 7
    err = np.abs(R.astype(np.float64) - rscale.astype(np.float64)[None, :] * Rq)
    assert np.all(err <= rscale.astype(np.float64)[None, :] * (0.5 + 1e-6))
    cols = np.arange(40) != 3
    jmax = np.argmax(np.abs(R), axis=0)
    assert np.all(np.abs(Rq[jmax, np.arange(40)])[cols] == 7)


def test_q4r_reduces_to_linear_with_the_dequantised_matrix():
    # rscale * Rq is a matrix like any other: the 16-bit-R routine fed with it must agree up to fp64 rounding
    spec = workloads.LayerSpec("pin", 1, 8, 6, 128, 24, 32, "bf16", "bf16", 2, 20.0, 20.0)
    L = workloads.make_layer(spec)
    pk = orc.pack_weights(L["W"].float().numpy(), L["s"].numpy(), spec.r)
    Xq, scale = orc.quantize_act(L["X"].float().numpy()[:, pk["perm"]], pk["s_inv"], spec.abits)
    Rq, rscale = orc.quantize_lowrank(L["R"].float().numpy())
    Ya = orc.linear_q4r(Xq, scale, pk["Wq"], pk["wscale"], Rq, rscale)
    Yb = orc.linear(Xq, scale, pk["Wq"], pk["wscale"], rscale.astype(np.float64)[None, :] * Rq)
    assert np.allclose(Ya, Yb, rtol=1e-12, atol=0.0)
    # and quantising the compensation matrix moves the output by at most what the half-step bound allows
    Y16 = orc.linear(Xq, scale, pk["Wq"], pk["wscale"], L["R"].double().numpy())
    bound = scale.astype(np.float64)[:, None] * (np.abs(Xq[:, :spec.r]).sum(axis=1)[:, None]
                                                 * rscale.astype(np.float64)[None, :] * 0.5)
    assert np.all(np.abs(Ya - Y16) <= bound * (1 + 1e-6) + 1e-12)


# ---------------------------------------------------------------------------
# MXFP4 (OCP Microscaling: E2M1 elements, E8M0 scale per block of 32)
# ---------------------------------------------------------------------------
def test_mx_e2m1_value_table_and_ties():
    # the eight magnitudes of the format and every tie between neighbours (to the even mantissa bit)
    assert orc.E2M1_VALUES.tolist() == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    cases = {0.0: 0, 0.24: 0, 0.25: 0, 0.26: 1, 0.5: 1, 0.75: 2, 1.0: 2, 1.25: 2, 1.26: 3, 1.5: 3, 1.75: 4,
             2.0: 4, 2.5: 4, 2.51: 5, 3.0: 5, 3.5: 6, 4.0: 6, 4.99: 6, 5.0: 6, 5.01: 7, 6.0: 7, 7.9: 7, 100.0: 7}
    for v, code in cases.items():
        assert orc.e2m1_round(np.float32(v)) == code, v
        assert orc.e2m1_round(np.float32(-v)) == (code + 8 if code else 0), -v


def test_mx_hand_worked_blocks():
    # block 1: max 6 -> floor(log2 6) = 2 -> shared exponent 0 (E = 127); values are their own codes
    b1 = np.array([6, -3, 1.5, 0.5, 0, 0.25, -0.75, 2.5] + [0] * 24, np.float32)
    # block 2: max 7 -> still exponent 0; 7 saturates to 6, 5 is the tie between 4 and 6 (-> 4)
    b2 = np.array([7, 5, -1.25] + [0] * 29, np.float32)
    # block 3: max 0.1875 = 1.5 * 2^-3 -> floor(log2) = -3 -> exponent -5 (E = 122); 0.1875 / 2^-5 = 6
    b3 = np.array([0.1875, -0.0625, 0.015625] + [0] * 29, np.float32)
    # block 4: all zero -> E = 127, codes 0
    b4 = np.zeros(32, np.float32)
    codes, E = orc.mx_quantize(np.concatenate([b1, b2, b3, b4])[None, :])
    assert E[0].tolist() == [127, 127, 122, 127]
    assert codes[0, :8].tolist() == [7, 8 + 5, 3, 1, 0, 0, 8 + 2, 4]
    assert codes[0, 32:35].tolist() == [7, 6, 8 + 2]
    assert codes[0, 64:67].tolist() == [7, 8 + 4, 1]            # -0.0625 * 32 = -2 ; 0.015625 * 32 = 0.5
    assert not codes[0, 96:].any()
    d = orc.mx_dequantize(codes, E)
    assert d[0, :8].tolist() == [6, -3, 1.5, 0.5, 0, 0, -1, 2]
    assert d[0, 32:35].tolist() == [6, 4, -1]
    assert d[0, 64:67].tolist() == [0.1875, -0.0625, 0.015625]


def test_mx_power_of_two_invariance_and_error_bound():
    rng = np.random.default_rng(11)
    V = (rng.standard_normal((5, 256)) * np.exp(rng.standard_normal((5, 256)))).astype(np.float32)
    codes, E = orc.mx_quantize(V)
    for k in (-9, 3, 20):
        c2, E2 = orc.mx_quantize(np.ldexp(V, k))
        assert np.array_equal(c2, codes) and np.array_equal(E2.astype(int), E.astype(int) + k)
    # inside the grid the error is at most half the local step; the block maximum may saturate (6 <- up to 8)
    d = orc.mx_dequantize(codes, E)
    scale = np.repeat(np.ldexp(1.0, E.astype(int) - 127), 32, axis=-1)
    t = np.abs(V.astype(np.float64)) / scale
    step = np.select([t < 2, t < 4, t <= 6], [0.5, 1.0, 2.0], default=4.0)
    assert np.all(np.abs(V - d) <= 0.5 * step * scale * (1 + 1e-12))
    assert np.all(t < 8) and np.all(np.max(t.reshape(5, 8, 32), axis=-1) >= 4)


def test_mx_linear_is_the_matmul_of_what_the_codes_stand_for():
    rng = np.random.default_rng(12)
    M, K, N, r, s_begin = 3, 128, 5, 64, 32
    # operands that are exactly representable: codes and exponents drawn directly
    Xc, Wc, Rc = (rng.integers(0, 16, size=sh).astype(np.uint8) for sh in ((M, K), (N, K), (N, r)))
    Xe, We, Re = (rng.integers(120, 134, size=sh).astype(np.uint8) for sh in ((M, K // 32), (N, K // 32), (N, r // 32)))
    Y = orc.mx_linear(Xc, Xe, Wc, We, Rc, Re, s_begin=s_begin)
    val = lambda c: (-1.0 if c & 8 else 1.0) * [0, .5, 1, 1.5, 2, 3, 4, 6][c & 7]
    for m in range(M):
        for n in range(N):
            t = 0.0
            for k in range(K):
                t += val(Xc[m, k]) * 2.0 ** (int(Xe[m, k // 32]) - 127) * val(Wc[n, k]) * 2.0 ** (int(We[n, k // 32]) - 127)
            for j in range(r):
                k = s_begin + j
                t += val(Xc[m, k]) * 2.0 ** (int(Xe[m, k // 32]) - 127) * val(Rc[n, j]) * 2.0 ** (int(Re[n, j // 32]) - 127)
            assert abs(Y[m, n] - t) <= 1e-12 * max(1.0, abs(t))
    # a tensor that is already on the grid survives quantisation unchanged
    Xd = orc.mx_dequantize(Xc, Xe).astype(np.float32)
    c2, e2 = orc.mx_quantize(Xd)
    assert np.array_equal(orc.mx_dequantize(c2, e2), Xd.astype(np.float64))


def test_mx_pack_residual_and_compensation():
    spec = workloads.LayerSpec("pin", 1, 4, 6, 128, 24, 64, "bf16", "bf16", 2, 20.0, 20.0)
    L = workloads.make_layer(spec)
    W, s = L["W"].float().numpy(), L["s"].numpy()
    pk = orc.mx_pack_weights(W, s, spec.r)
    Wp = (W * s[None, :])[:, pk["perm"]]
    Wd = orc.mx_dequantize(pk["Wc"], pk["We"])
    Rd = orc.mx_dequantize(pk["Rc"], pk["Re"])
    # the compensated salient rows are closer to the folded weights than the quantised ones alone
    e0 = np.linalg.norm(Wp[:, :spec.r] - Wd[:, :spec.r])
    e1 = np.linalg.norm(Wp[:, :spec.r] - (Wd[:, :spec.r] + Rd))
    assert e1 < 0.5 * e0
    # and the layer with it is closer to the unquantised product over the salient block
    Xc, Xe = orc.mx_quantize_act(L["X"].float().numpy()[:, pk["perm"]], pk["s_inv"])
    Xd = orc.mx_dequantize(Xc, Xe)
    ref = Xd[:, :spec.r] @ Wp[:, :spec.r].T.astype(np.float64)
    y0 = Xd[:, :spec.r] @ Wd[:, :spec.r].T
    y1 = y0 + Xd[:, :spec.r] @ Rd.T
    assert np.linalg.norm(y1 - ref) < np.linalg.norm(y0 - ref)
    full = orc.mx_linear(Xc, Xe, pk["Wc"], pk["We"], pk["Rc"], pk["Re"])
    assert np.allclose(full, Xd @ Wd.T + Xd[:, :spec.r] @ Rd.T, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------
# gated product (producer side of the down projection)
# ---------------------------------------------------------------------------
def test_silu_against_library_identity_and_limits():
    import torch
    x = np.concatenate([np.linspace(-30, 30, 2001), [0.0, 1.0, -1.0, 1e-8, -1e-8, 700.0, -700.0, 1e4, -1e4]])
    y = orc.silu(x)
    ref = torch.nn.functional.silu(torch.from_numpy(x)).numpy()          # library routine, fp64
    assert np.allclose(y, ref, rtol=1e-14, atol=1e-300)
    assert y[x == 0.0][0] == 0.0
    assert abs(orc.silu(np.array([1.0]))[0] - 0.7310585786300049) < 1e-16   # 1 / (1 + e^-1)
    # odd part: silu(x) - silu(-x) = x (sigmoid(x) + sigmoid(-x) = 1)
    assert np.allclose(y - orc.silu(-x), x, rtol=1e-14, atol=1e-14)
    assert orc.silu(np.array([700.0]))[0] == 700.0 and orc.silu(np.array([-1e4]))[0] == 0.0
    assert np.all(np.isfinite(y))
    # minimum of silu is about -0.2785 at x about -1.2785
    assert abs(y.min() + 0.27846) < 1e-4


def test_swiglu_reductions_to_the_plain_quantisers():
    rng = np.random.default_rng(5)
    M, K = 6, 128
    g = rng.standard_normal((M, K)).astype(np.float32) * 3
    u = rng.standard_normal((M, K)).astype(np.float32)
    s_inv = rng.uniform(0.5, 2.0, K).astype(np.float32)
    # up = 1: the product is silu itself
    assert np.array_equal(orc.swiglu(g, np.ones_like(g)), orc.silu(g).astype(np.float32))
    # a gate far in the linear region: silu(g) = g to the last bit, so the product is g * u rounded once
    big = (np.abs(g) + 50).astype(np.float32)
    assert np.array_equal(orc.swiglu(big, u), (big.astype(np.float64) * u).astype(np.float32))
    for abits in (4, 8):
        a = orc.swiglu_quantize_act(big, u, s_inv, abits)
        b = orc.quantize_act((big.astype(np.float64) * u).astype(np.float32), s_inv, abits)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    a = orc.mx_swiglu_quantize_act(big, u, s_inv)
    b = orc.mx_quantize_act((big.astype(np.float64) * u).astype(np.float32), s_inv)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # a gate far in the negative region closes the gate: all-zero tokens, scale 1 / exponent byte 127
    shut = np.full_like(g, -800.0)
    codes, scale = orc.swiglu_quantize_act(shut, u, None, 8)
    assert not codes.any() and np.all(scale == 1.0)
    codes, E = orc.mx_swiglu_quantize_act(shut, u, None)
    assert not codes.any() and np.all(E == 127)
    # sign: a negative `up` flips every code (both grids are symmetric)
    c1, s1 = orc.swiglu_quantize_act(g, u, s_inv, 8)
    c2, s2 = orc.swiglu_quantize_act(g, -u, s_inv, 8)
    assert np.array_equal(c1, -c2) and np.array_equal(s1, s2)


def test_mx_pack_hand_worked_blocks():
    # tests/golden/tiny_mx_pack.txt: two output channels, three blocks of 32 input channels, two of them
    # salient, every code and exponent byte derived by hand; a wrong block offset between the weights'
    # exponents and the residual, a swapped block or a dropped tie rule changes Rc / Re
    g = _read_golden(os.path.join(HERE, "golden", "tiny_mx_pack.txt"))
    W = g["W"].astype(np.float32)
    pk = orc.mx_pack_weights(W, None, 64, perm=np.arange(96, dtype=np.int32))
    assert np.array_equal(pk["Wc"], g["Wc"].astype(np.uint8))
    assert np.array_equal(pk["We"], g["We"].astype(np.uint8))
    assert np.array_equal(pk["Rc"], g["Rc"].astype(np.uint8))
    assert np.array_equal(pk["Re"], g["Re"].astype(np.uint8))
    assert np.all(pk["s_inv"] == 1.0)
    # with one salient block only, the compensation matrix is the first block of the one above
    pk1 = orc.mx_pack_weights(W, None, 32, perm=np.arange(96, dtype=np.int32))
    assert np.array_equal(pk1["Rc"], g["Rc"].astype(np.uint8)[:, :32])
    assert np.array_equal(pk1["Re"], g["Re"].astype(np.uint8)[:, :1])
    # the residual the codes stand for, by hand: row 0 block 0 = (0 1 .5 -.25 -.1875 .25 -.25 0) rounded to
    # the grid at exponent -2, i.e. 0 1 .5 -.25 -.25 .25 -.25 0
    Rd = orc.mx_dequantize(pk["Rc"], pk["Re"])
    assert np.array_equal(Rd[0, :8], [0, 1, 0.5, -0.25, -0.25, 0.25, -0.25, 0])
    assert np.array_equal(Rd[1, :8] * 32, Rd[0, :8])
    assert np.array_equal(Rd[0, 32:40] * 4, Rd[0, :8][::-1])


def test_rel_errors_hand_made_pairs():
    # reference 3 4 0 0: max 4, rms sqrt(25/4) = 2.5
    Y64 = np.array([[3.0, 4.0], [0.0, 0.0]])
    Y = np.array([[3.5, 4.0], [0.25, 0.0]])
    g, mix = orc.rel_errors(Y, Y64)
    assert g == 0.5 / 4.0                                    # largest difference over the largest reference
    assert mix == max(0.5 / (3.0 + 2.5), 0.25 / (0.0 + 2.5))  # a near-zero output is held to the rms
    assert orc.rel_errors(Y64, Y64) == (0.0, 0.0)
    # a sign error on the largest element: twice its magnitude
    g, mix = orc.rel_errors(np.array([[3.0, -4.0], [0.0, 0.0]]), Y64)
    assert g == 2.0 and mix == 8.0 / 6.5
    # the two measures disagree where they should: a small error on a small element of a wide-range row
    ref = np.array([[1000.0, 1.0]])
    g, mix = orc.rel_errors(np.array([[1000.0, 2.0]]), ref)
    assert g == 1e-3 and abs(mix - 1.0 / (1.0 + np.sqrt(1000001.0 / 2))) < 1e-15
    # empty and all-zero references
    assert orc.rel_errors(np.zeros((0, 4)), np.zeros((0, 4))) == (0.0, 0.0)
    assert orc.rel_errors(np.zeros((2, 2)), np.zeros((2, 2))) == (0.0, 0.0)
    g, mix = orc.rel_errors(np.full((2, 2), 1e-30), np.zeros((2, 2)))
    assert g == float("inf") and mix == float("inf")
    # any float type in, same numbers out
    g32, m32 = orc.rel_errors(Y.astype(np.float32), Y64)
    assert (g32, m32) == orc.rel_errors(Y, Y64)


# ---------------------------------------------------------------------------
# group-128 weight scales + asymmetric activations (the accuracy-table setting, Sec. 4.1)
# ---------------------------------------------------------------------------
def test_grouped_asym_hand_worked_layer():
    g = _read_golden(os.path.join(HERE, "golden", "tiny_grouped_asym.txt"))
    X, W = g["X"].astype(np.float32), g["W"].astype(np.float32)
    Xq, scale, zero = orc.quantize_act_asym(X, None, 4)
    assert np.array_equal(scale, g["scale"][0].astype(np.float32))
    assert np.array_equal(zero, g["zero"][0].astype(np.int32))
    assert np.array_equal(Xq, g["Xq"].astype(np.int8))
    pk = orc.pack_weights_grouped(W, None, 2, perm=np.arange(256, dtype=np.int32))
    assert np.array_equal(pk["gscale"], g["gscale"].astype(np.float32))
    assert np.array_equal(pk["Wq"], g["Wq"].astype(np.int8))
    assert np.array_equal(pk["R"], g["R"])
    assert np.array_equal(pk["wsum"], g["wsum"][0])
    assert np.array_equal(orc.linear_grouped(Xq, scale, zero, pk["Wq"], pk["gscale"], None), g["Y0"])
    assert np.array_equal(orc.linear_grouped(Xq, scale, zero, pk["Wq"], pk["gscale"], pk["R"]), g["Y"])


@pytest.mark.parametrize("abits", [4, 8])
def test_asym_quantiser_bounds_and_nearest_grid_point(abits):
    rng = np.random.default_rng(abits)
    M, K = 12, 256
    X = rng.standard_normal((M, K)).astype(np.float32)
    X[0] += 3.0                      # mostly positive
    X[1] = np.abs(X[1]) + 0.5        # strictly positive: the range is widened down to 0
    X[2] = -np.abs(X[2]) - 0.5       # strictly negative: widened up to 0
    X[3] = 0.0                       # zero token
    X[4, :] = 2.5                    # constant token
    s_inv = rng.uniform(0.5, 2.0, K).astype(np.float32)
    v = orc.flatten(X, s_inv).astype(np.float64)
    Xq, scale, zero = orc.quantize_act_asym(X, s_inv, abits)
    top, half = (1 << abits) - 1, 1 << (abits - 1)
    c = Xq.astype(np.int64) + half
    z = zero.astype(np.int64) + half
    assert c.min() >= 0 and c.max() <= top and z.min() >= 0 and z.max() <= top
    assert scale[3] == 1.0 and not (c[3] - z[3]).any()
    lo, hi = np.minimum(v.min(axis=1), 0), np.maximum(v.max(axis=1), 0)
    ok = hi > lo
    assert np.allclose(scale[ok], ((hi - lo) / top)[ok], rtol=1e-6)
    assert z[1] == 0 and z[2] == top                     # one-sided tokens: zero point at an end of the grid
    xh = scale.astype(np.float64)[:, None] * (c - z[:, None])
    # half a step everywhere, plus the half step the zero point's own rounding can shift the grid by at the ends
    assert np.all(np.abs(xh - v) <= scale[:, None] * (1.0 + 1e-5))
    inner = (c > 0) & (c < top)
    assert np.all(np.abs(xh - v)[inner] <= (0.5 + 1e-5) * np.broadcast_to(scale[:, None], v.shape)[inner])
    # brute force: no other code of the grid is closer (beyond fp32 rounding of the quotient)
    grid = scale.astype(np.float64)[:, None, None] * (np.arange(top + 1)[None, None, :] - z[:, None, None])
    best = np.min(np.abs(grid - v[:, :, None]), axis=2)
    assert np.all(np.abs(xh - v) <= best + 1e-5 * scale[:, None])
    # zero is on the grid
    assert np.all(np.min(np.abs(grid), axis=2) == 0)


def test_grouped_weights_bounds_and_16_bit_scales():
    rng = np.random.default_rng(3)
    N, K, r = 24, 512, 32
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    s = rng.uniform(0.5, 2.0, K).astype(np.float32)
    pk = orc.pack_weights_grouped(W, s, r)
    gs = pk["gscale"]
    assert gs.shape == (N, K // 128)
    assert np.array_equal(gs.astype(np.float16).astype(np.float32), gs)       # representable in 16 bits
    Wp = (W * s[None, :])[:, pk["perm"]]
    amax = np.abs(Wp.reshape(N, K // 128, 128)).max(axis=2)
    assert np.allclose(gs[amax > 0], (amax / 7)[amax > 0], rtol=2.0 ** -11)
    deq = np.repeat(gs, 128, axis=1).astype(np.float64) * pk["Wq"]
    # half a step, except where the 16-bit scale came out below max/7 and the extreme value clips at 7
    assert np.all(np.abs(deq - Wp) <= np.repeat(gs, 128, axis=1) * (0.5 + 2.0 ** -9))
    assert np.abs(pk["Wq"]).max() == 7
    assert np.allclose(pk["R"], (Wp[:, :r] - deq[:, :r]).T, rtol=0, atol=0)
    assert np.allclose(pk["wsum"], deq.sum(axis=1), rtol=1e-15)
    # a zero group has scale 1 and zero codes
    Wz = np.zeros((2, 256), np.float32)
    Wz[0, 5] = 1.0
    pz = orc.pack_weights_grouped(Wz, None, 0, perm=np.arange(256))
    assert pz["gscale"].tolist() == [[np.float32(np.float16(1.0 / 7)), 1.0], [1.0, 1.0]] and not pz["Wq"][1].any()


@pytest.mark.parametrize("abits", [4, 8])
def test_grouped_reduces_to_the_per_channel_symmetric_path(abits):
    # (a) equal group scales and no zero point: the grouped layer is the per-channel layer
    rng = np.random.default_rng(11 + abits)
    M, K, N, r = 5, 384, 6, 16
    q = orc.qmax(abits)
    Xq = rng.integers(-q, q + 1, size=(M, K)).astype(np.int8)
    Wq = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    scale = rng.uniform(0.01, 0.1, M).astype(np.float32)
    wscale = rng.uniform(0.001, 0.01, N).astype(np.float32)
    R = rng.standard_normal((r, N)) * 0.01
    a = orc.linear_grouped(Xq, scale, None, Wq, np.repeat(wscale[:, None], K // 128, axis=1), R)
    b = orc.linear(Xq, scale, Wq, wscale, R)
    assert np.allclose(a, b, rtol=1e-13, atol=1e-13)
    assert np.array_equal(orc.gemm_i32_grouped(Xq, Wq).sum(axis=0), orc.gemm_i32(Xq, Wq))
    # (b) the dense product of what the codes stand for, zero point included, salient block offset
    zero = rng.integers(-q - 1, q + 1, size=M).astype(np.int32)
    gs = rng.uniform(0.001, 0.01, (N, K // 128)).astype(np.float32)
    xh = scale.astype(np.float64)[:, None] * (Xq.astype(np.float64) - zero[:, None])
    wh = np.repeat(gs, 128, axis=1).astype(np.float64) * Wq
    want = xh @ wh.T + xh[:, 128:128 + r] @ R
    got = orc.linear_grouped(Xq, scale, zero, Wq, gs, R, s_begin=128)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    # (c) one group spanning all of K with a scale that 16 bits hold exactly: the per-channel pack
    W = rng.integers(-7, 8, size=(N, 128)).astype(np.float32) * np.float32(2.0 ** -6)
    W[np.arange(N), rng.integers(0, 128, N)] = 7 * 2.0 ** -6
    pg = orc.pack_weights_grouped(W, None, 16, perm=np.arange(128))
    pc = orc.pack_weights(W, None, 16, perm=np.arange(128))
    assert np.array_equal(pg["Wq"], pc["Wq"]) and np.array_equal(pg["gscale"][:, 0], pc["wscale"])
    assert np.array_equal(pg["R"], pc["R"])
    # (d) a symmetric token (lo = -hi) whose step is a power of two: the zero point sits at the exact tie
    # (2^n - 1) / 2 -> 2^(n-1) by round-half-to-even, and the codes are the plain rounding on that step
    top = (1 << abits) - 1
    X = (rng.standard_normal((3, 256)) * 0.3).astype(np.float32)
    X[:, 0] = top / 8.0
    X[:, 1] = -top / 8.0
    Xa, sa, za = orc.quantize_act_asym(X, None, abits)
    assert np.all(za == 0) and np.all(sa == 0.25)
    assert np.array_equal(Xa, np.clip(np.rint(X / np.float32(0.25)), -(top + 1) // 2, top // 2).astype(np.int8))
