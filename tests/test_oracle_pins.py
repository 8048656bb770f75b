"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things that are not the oracle: hand-worked
numbers (tests/golden), brute force in Python integers / exact rationals,
closed forms, invariants the paper states, reduction to textbook W8A8, and the
analytic quantization-error bound.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2507_14811_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# hand-worked example (tests/golden/handworked_2x4x2.json)
# ----------------------------------------------------------------------------
@pytest.fixture(scope="module")
def gold():
    with open(os.path.join(GOLD, "handworked_2x4x2.json")) as f:
        return json.load(f)


def test_handworked_codes_and_accumulators(oracle, gold):
    g, e = gold, gold["expect"]
    x = np.array(g["x"], np.float32)
    w = np.array(g["w"], np.float32)
    wq, ws = oracle.quantize_weight(w, g["kseg_off"])
    xp, xn = oracle.quantize_act(x, g["kseg_off"], g["dual"], g["s_pos"], g["s_neg"])
    ap, an = oracle.int_gemm(xp, xn, wq, g["kseg_off"], g["dual"])
    assert wq.tolist() == e["wq"]
    assert ws.tolist() == e["wscale"]
    assert xp.tolist() == e["xq_pos"]
    assert xn.tolist() == e["xq_neg"]
    assert ap.tolist() == e["acc_pos"]
    assert an.tolist() == e["acc_neg"]


@pytest.mark.parametrize("case", ["case_plain", "case_segscale_bias"])
def test_handworked_output(oracle, gold, case):
    g, c = gold, gold[case]
    r = oracle.seglinear(np.array(g["x"], np.float32), np.array(g["w"], np.float32), g["kseg_off"], c["nseg_off"],
                         g["dual"], g["s_pos"], g["s_neg"],
                         None if c["seg_scale"] is None else np.array(c["seg_scale"], np.float32),
                         None if c["bias"] is None else np.array(c["bias"], np.float32))
    assert r.y32.tolist() == c["y"]          # exact: every operand is a dyadic rational
    assert r.y64.tolist() == c["y"]


def test_bf16_cast_ties(oracle, gold):
    b = gold["bf16_cast"]
    f = np.array([int(h, 16) for h in b["f32_hex"]], np.uint32).view(np.float32)
    got = oracle.cast_bf16(f)
    assert [f"{v:04X}" for v in got.tolist()] == b["bf16_hex"]
    # widening is the exact inverse on bf16 values
    assert np.array_equal(oracle.cast_bf16(oracle.widen_bf16(got)), got)
    # and agrees with the (independent) data-preparation helper on random values
    r = np.random.default_rng(1).standard_normal(10000).astype(np.float32) * 37
    assert np.array_equal(oracle.cast_bf16(r), wl.f32_to_bf16_bits(r))


# ----------------------------------------------------------------------------
# brute force on tiny inputs: Python ints and exact rationals
# ----------------------------------------------------------------------------
def _rne_fraction(q: Fraction) -> int:
    fl = math.floor(q)
    d = q - fl
    if d > Fraction(1, 2):
        return fl + 1
    if d < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def _clip(v, lo=-127, hi=127):
    return max(lo, min(hi, v))


def _brute(x, w, kseg, nseg, dual, s_pos, s_neg, seg_scale, bias):
    """Independent evaluation with exact rationals.  Scales must be powers of two times small
    integers so that fp32 x / s is exact and the rational rounding equals the fp32 one."""
    M, K = x.shape
    N = w.shape[0]
    S, T = len(kseg) - 1, len(nseg) - 1
    F = lambda v: Fraction(float(v))
    wq = [[0] * K for _ in range(N)]
    wsc = [[Fraction(1)] * N for _ in range(S)]
    for n in range(N):
        for ks in range(S):
            a = max(abs(F(w[n, k])) for k in range(kseg[ks], kseg[ks + 1]))
            sw = a / 127 if a != 0 else Fraction(1)
            wsc[ks][n] = sw
            for k in range(kseg[ks], kseg[ks + 1]):
                wq[n][k] = _clip(_rne_fraction(F(w[n, k]) / sw))
    xp = [[0] * K for _ in range(M)]
    xn = [[0] * K for _ in range(M)]
    for m in range(M):
        for ks in range(S):
            for k in range(kseg[ks], kseg[ks + 1]):
                v = F(x[m, k])
                if dual[ks]:
                    if v < 0:
                        xn[m][k] = _clip(_rne_fraction(v / F(s_neg[ks])))
                    else:
                        xp[m][k] = _clip(_rne_fraction(v / F(s_pos[ks])))
                else:
                    xp[m][k] = _clip(_rne_fraction(v / F(s_pos[ks])))
    y = [[Fraction(0)] * N for _ in range(M)]
    accp = [[[0] * N for _ in range(M)] for _ in range(S)]
    accn = [[[0] * N for _ in range(M)] for _ in range(S)]
    for m in range(M):
        for n in range(N):
            t = next(j for j in range(T) if nseg[j] <= n < nseg[j + 1])
            for ks in range(S):
                ap = sum(xp[m][k] * wq[n][k] for k in range(kseg[ks], kseg[ks + 1]))
                an = sum(xn[m][k] * wq[n][k] for k in range(kseg[ks], kseg[ks + 1])) if dual[ks] else 0
                accp[ks][m][n], accn[ks][m][n] = ap, an
                g = F(seg_scale[ks][t]) if seg_scale is not None else Fraction(1)
                y[m][n] += g * wsc[ks][n] * (F(s_pos[ks]) * ap + (F(s_neg[ks]) * an if dual[ks] else 0))
            if bias is not None:
                y[m][n] += F(bias[n])
    return wq, wsc, xp, xn, accp, accn, y


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_tiny(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    M, K, N = int(rng.integers(1, 7)), int(rng.integers(2, 9)), int(rng.integers(1, 8))
    S = 2 if K >= 2 and seed % 2 else 1
    T = 2 if N >= 2 and seed % 3 else 1
    kseg = [0, K] if S == 1 else [0, int(rng.integers(1, K)), K]
    nseg = [0, N] if T == 1 else [0, int(rng.integers(1, N)), N]
    dual = [int(rng.integers(0, 2)) for _ in range(S)]
    if seed == 0:
        dual = [1] * S
    # dyadic data: x multiples of 1/64, scales powers of two => fp32 x/s exact, ties occur often.
    # weights: integers i/2^j with the per-(row, segment) absmax forced to 127/2^j => step exactly 2^-j.
    x = (rng.integers(-300, 301, size=(M, K)) / 64.0).astype(np.float32)
    s_pos = np.array([2.0 ** int(rng.integers(-6, 1)) for _ in range(S)], np.float32)
    s_neg = np.array([2.0 ** int(rng.integers(-8, -2)) for _ in range(S)], np.float32)
    w = np.zeros((N, K), np.float32)
    for n in range(N):
        for ks in range(S):
            j = int(rng.integers(3, 9))
            seg = rng.integers(-2 * 127, 2 * 127 + 1, size=kseg[ks + 1] - kseg[ks]) / 2.0   # half-integers: ties
            seg[int(rng.integers(0, len(seg)))] = 127.0 * (1 if rng.integers(0, 2) else -1)
            w[n, kseg[ks]:kseg[ks + 1]] = seg / 2.0 ** j
    seg_scale = rng.choice([0.5, 1.0, 2.0, 4.0], size=(S, T)).astype(np.float32) if seed % 2 else None
    bias = (rng.integers(-8, 9, size=N) / 4.0).astype(np.float32) if seed % 3 == 0 else None

    r = oracle.seglinear(x, w, kseg, nseg, dual, s_pos, s_neg, seg_scale, bias)
    wq, wsc, xp, xn, accp, accn, y = _brute(x, w, kseg, nseg, dual, s_pos, s_neg, seg_scale, bias)
    assert r.wq.tolist() == wq
    assert [[Fraction(float(v)) for v in row] for row in r.wscale] == wsc
    assert r.xq_pos.tolist() == xp and r.xq_neg.tolist() == xn
    assert r.acc_pos.tolist() == accp and r.acc_neg.tolist() == accn
    yb = np.array([[float(v) for v in row] for row in y])
    assert np.allclose(r.y64, yb, rtol=1e-13, atol=1e-13)
    scale = max(1.0, float(np.abs(yb).max()))
    assert np.abs(r.y32 - yb).max() <= 1e-6 * scale


def test_general_scales_nearest_code_property(oracle):
    """For arbitrary (non-dyadic) steps the code is the nearest integer to x/s, clipped (Sec. 3)."""
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((5, 64)) * 3).astype(np.float32)
    s_pos, s_neg = np.array([0.0123], np.float32), np.array([0.00457], np.float32)
    xp, xn = oracle.quantize_act(x, [0, 64], [1], s_pos, s_neg)
    for v, p, n in zip(x.ravel().tolist(), xp.ravel().tolist(), xn.ravel().tolist()):
        q = Fraction(v) / Fraction(float(s_neg[0] if v < 0 else s_pos[0]))
        want = _clip(_rne_fraction(q))
        got = n if v < 0 else p
        assert abs(got - want) <= (1 if abs(abs(q - math.floor(q)) - Fraction(1, 2)) < Fraction(1, 10 ** 5) else 0)
        assert (p == 0) if v < 0 else (n == 0)
    assert np.any(xp == 127) and np.any(xn == -127)      # clipping exercised


# ----------------------------------------------------------------------------
# invariants stated by the paper
# ----------------------------------------------------------------------------
def test_polarity_split_is_exact(oracle):
    """X = X_+ + X_- (Sec. 4.3.2) and the two code tensors have disjoint support and fixed signs."""
    w_ = wl.cfg1_tiny()
    xpos, xneg = np.maximum(w_.x, 0), np.minimum(w_.x, 0)
    assert np.array_equal((xpos + xneg).view(np.uint32), w_.x.view(np.uint32))
    xp, xn = oracle.quantize_act(w_.x, w_.kseg_off, w_.dual, w_.s_pos, w_.s_neg)
    assert (xp >= 0).all() and (xn <= 0).all()
    assert not np.any((xp != 0) & (xn != 0))
    assert xp.max() == 127 and xn.min() == -127            # steps = extreme / 127 reach the range ends
    # quantizing the two halves separately gives the same codes as Q_dual on X
    zp, _ = oracle.quantize_act(xpos, w_.kseg_off, w_.dual, w_.s_pos, w_.s_neg)
    _, zn = oracle.quantize_act(xneg, w_.kseg_off, w_.dual, w_.s_pos, w_.s_neg)
    assert np.array_equal(zp, xp) and np.array_equal(zn, xn)


def test_reduces_to_textbook_w8a8(oracle):
    """x >= 0, one segment, per-tensor weight step: DualScale == plain symmetric W8A8 (App. A)."""
    rng = np.random.default_rng(11)
    M, K, N = 9, 40, 7
    x = np.maximum(rng.standard_normal((M, K)), 0).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    w[:, 0] = np.abs(w).max() * np.sign(w[:, 0] + 1e-9)        # every row reaches the same absmax
    s_x = np.float32(x.max()) / np.float32(127)
    r = oracle.seglinear(x, w, [0, K], [0, N], [1], [s_x], [np.float32(1.0)])
    assert not r.acc_neg.any()
    s_w = np.float32(np.abs(w).max()) / np.float32(127)
    assert np.all(r.wscale == s_w)
    # textbook routine: numpy rint (half-even) + int64 matmul + one product of scales
    xq = np.clip(np.rint(x / s_x), -127, 127).astype(np.int64)
    wq = np.clip(np.rint(w / s_w), -127, 127).astype(np.int64)
    yhat = xq @ wq.T
    assert np.array_equal(r.acc_pos[0], yhat)
    y = np.float64(s_x) * np.float64(s_w) * yhat
    assert np.abs(r.y64 - y).max() <= 1e-12 * np.abs(y).max()
    assert np.abs(r.y32 - y).max() <= 2e-7 * np.abs(y).max()


def test_grid_values_round_trip(oracle):
    """Values on the quantization grid come back as their own codes; small-K product is exact."""
    rng = np.random.default_rng(5)
    M, K, N = 6, 16, 5
    s_p, s_n, s_w = np.float32(2.0 ** -4), np.float32(2.0 ** -7), 2.0 ** -6
    j = rng.integers(-127, 128, size=(M, K))
    j[0, 0], j[0, 1] = 127, -127
    x = np.where(j >= 0, j * float(s_p), j * float(s_n)).astype(np.float32)
    i = rng.integers(-127, 128, size=(N, K))
    i[:, 3] = 127
    w = (i * s_w).astype(np.float32)
    r = oracle.seglinear(x, w, [0, K], [0, N], [1], [s_p], [s_n])
    assert np.array_equal(r.xq_pos, np.where(j >= 0, j, 0))
    assert np.array_equal(r.xq_neg, np.where(j < 0, j, 0))
    assert np.array_equal(r.wq, i)
    assert np.all(r.wscale == np.float32(s_w))
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.array_equal(r.y64, exact)
    assert np.array_equal(r.y32.astype(np.float64), exact)   # all partial sums fit 24 bits here


def test_equal_scales_collapse_to_single_path(oracle):
    """s_+ = s_- makes Q_dual the plain symmetric quantizer: codes and accumulators add up exactly."""
    w_ = wl.random_layer(13, 96, 21, [0, 32, 96], [0, 21], [1, 1], seed=3, x_dtype="f32", act="normal")
    s = np.maximum(w_.s_pos, w_.s_neg)
    wq, _ = oracle.quantize_weight(w_.w, w_.kseg_off)
    xp, xn = oracle.quantize_act(w_.x, w_.kseg_off, [1, 1], s, s)
    x1, z1 = oracle.quantize_act(w_.x, w_.kseg_off, [0, 0], s, s)
    assert np.array_equal(xp.astype(np.int32) + xn, x1) and not z1.any()
    ap, an = oracle.int_gemm(xp, xn, wq, w_.kseg_off, [1, 1])
    a1, _ = oracle.int_gemm(x1, z1, wq, w_.kseg_off, [0, 0])
    assert np.array_equal(ap + an, a1)


def test_segmentation_bookkeeping(oracle):
    """SegLinear invariances (Sec. 4.2.2): splitting a K-segment with equal steps keeps the integer sum;
    permuting whole N-segments permutes output columns; N-segment boundaries do not matter when seg_scale = 1."""
    w_ = wl.random_layer(7, 64, 24, [0, 64], [0, 8, 24], [1], seed=9, x_dtype="f32", act="gelu")
    wq, ws = oracle.quantize_weight(w_.w, [0, 64])
    xp, xn = oracle.quantize_act(w_.x, [0, 64], [1], w_.s_pos, w_.s_neg)
    a1p, a1n = oracle.int_gemm(xp, xn, wq, [0, 64], [1])
    a2p, a2n = oracle.int_gemm(xp, xn, wq, [0, 24, 64], [1, 1])
    assert np.array_equal(a2p.sum(0), a1p[0]) and np.array_equal(a2n.sum(0), a1n[0])
    # K-segment slices really are the column ranges kseg_off names
    a_first, _ = oracle.int_gemm(xp[:, :24].copy(), xn[:, :24].copy(), wq[:, :24].copy(), [0, 24], [1])
    assert np.array_equal(a2p[0], a_first[0])
    y_a, _ = oracle.dequant(a1p, a1n, [0, 8, 24], [1], w_.s_pos, w_.s_neg, ws)
    y_b, _ = oracle.dequant(a1p, a1n, [0, 24], [1], w_.s_pos, w_.s_neg, ws)
    assert np.array_equal(y_a, y_b)
    perm = np.r_[8:24, 0:8]
    r_p = oracle.seglinear(w_.x, w_.w[perm], [0, 64], [0, 16, 24], [1], w_.s_pos, w_.s_neg)
    assert np.array_equal(r_p.y32, y_a[:, perm])
    # seg_scale multiplies exactly its own (K-segment, N-segment) block
    g = np.array([[2.0, 0.5]], np.float32)
    y_g, _ = oracle.dequant(a1p, a1n, [0, 8, 24], [1], w_.s_pos, w_.s_neg, ws, g)
    assert np.array_equal(y_g[:, :8], 2 * y_a[:, :8]) and np.array_equal(y_g[:, 8:], 0.5 * y_a[:, 8:])


def test_int32_guard(oracle):
    """127 * 127 * K_ks must fit int32: the oracle refuses a segment whose worst case does not."""
    K = 133200                                   # 127^2 * K > 2^31 - 1
    xp = np.full((1, K), 127, np.int8)
    wq = np.full((1, K), 127, np.int8)
    with pytest.raises(RuntimeError):
        oracle.int_gemm(xp, np.zeros_like(xp), wq, [0, K], [0])
    ap, _ = oracle.int_gemm(xp[:, :133143].copy(), xp[:, :133143].copy() * 0, wq[:, :133143].copy(), [0, 133143], [0])
    assert int(ap[0, 0, 0]) == 127 * 127 * 133143


# ----------------------------------------------------------------------------
# accuracy: analytic bound and the paper's qualitative claims
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["cfg1", "rand"])
def test_analytic_error_bound(oracle, name):
    w_ = wl.cfg1_tiny() if name == "cfg1" else wl.random_layer(11, 192, 37, [0, 64, 192], [0, 37], [0, 1], seed=21,
                                                               x_dtype="bf16", act="gelu")
    r = oracle.seglinear(w_.x, w_.w, w_.kseg_off, w_.nseg_off, w_.dual, w_.s_pos, w_.s_neg)
    yfp = oracle.fp_reference(w_.x, w_.w)
    bound = oracle.error_bound(w_.x, w_.w, w_.kseg_off, w_.dual, w_.s_pos, w_.s_neg, r.wscale)
    err = np.abs(r.y64 - yfp)
    assert (err <= bound * (1 + 1e-6) + 1e-9).all()
    assert err.max() > 1e-3 * bound.max()          # the bound is not vacuous: real error is within 3 decades of it
    assert np.abs(r.y32 - r.y64).max() <= 1e-6 * np.abs(r.y64).max()


def test_silu_gelu_negative_range_anchors():
    """Closed forms behind the narrow negative range (Sec. 4.3.1): min SiLU = -0.27846, min GELU = -0.16997."""
    z = np.linspace(-6, 0, 600001)
    assert abs(wl._silu(z).min() + 0.278464542761) < 1e-9
    assert abs(wl._gelu(z).min() + 0.169971) < 1e-6
    w_ = wl.cfg1_tiny()
    assert (w_.s_neg <= np.float32(0.2785 / 127)).all() and (w_.s_pos > 5 * w_.s_neg).all()


def test_dual_scale_beats_single_scale_on_silu(oracle):
    """Direction of the sensitivity table in App. B: lower relative F-norm error with DualScale."""
    w_ = wl.random_layer(64, 256, 96, [0, 256], [0, 96], [1], seed=2, x_dtype="f32", act="silu")
    yfp = oracle.fp_reference(w_.x, w_.w)
    rd = oracle.seglinear(w_.x, w_.w, w_.kseg_off, w_.nseg_off, [1], w_.s_pos, w_.s_neg)
    s1 = np.float32(np.abs(w_.x).max()) / np.float32(127)
    rs = oracle.seglinear(w_.x, w_.w, w_.kseg_off, w_.nseg_off, [0], [s1], [s1])
    fd = np.linalg.norm(rd.y64 - yfp) / np.linalg.norm(yfp)
    fs = np.linalg.norm(rs.y64 - yfp) / np.linalg.norm(yfp)
    assert fd < fs


def test_workload_recipes():
    """Shapes, segment tables and op counts of the named configurations."""
    c1 = wl.cfg1_tiny()
    assert (c1.M, c1.K, c1.N, c1.S, c1.T) == (64, 256, 384, 2, 3) and c1.int8_ops == 2 * 64 * 384 * 512
    c3 = wl.cfg3_adaln()
    assert (c3.M, c3.K, c3.N, c3.T) == (16, 1152, 6912, 6) and sorted(c3.extra["sigma"]) == [0.01, 0.02, 0.05, 0.1, 0.2, 0.5]
    assert c3.x_dtype == "bf16" and np.array_equal(wl.bf16_bits_to_f32(c3.x_bf16_bits()), c3.x)
    stds = [c3.w[j * 1152:(j + 1) * 1152].std() for j in range(6)]
    assert np.allclose(stds, c3.extra["sigma"], rtol=0.02)
    assert c3.seglinear_bytes() == 16 * 1152 + 6912 * 1152 + 4 * 6912 + 16 * 6912 * 2   # merged codes: X^ once


# ----------------------------------------------------------------------------------------------------
# calibration of the activation steps (Sec. 4.3.2 step definitions, min/max rule) and the block-granular
# weight quantizer (App. B: per-tensor 8-bit granularity, i.e. one step per weight segment)
# ----------------------------------------------------------------------------------------------------
def test_calibrate_act_handworked(oracle):
    x = np.array([[-2.0, 0.5, 3.0, -0.25], [1.0, -4.0, 0.0, 2.0]], np.float32)
    sp, sn, ap, an = oracle.calibrate_act(x, [0, 2, 4], [1, 0])
    # segment 0 is dual: max x = 1, min x = -4; segment 1 is single-scale: max |x| = 3, no second step
    assert ap.tolist() == [1.0, 3.0] and an.tolist() == [4.0, 0.0]
    q = np.float32(127.0)
    assert sp[0] == np.float32(1.0) / q and sn[0] == np.float32(4.0) / q and sp[1] == np.float32(3.0) / q
    assert sn[1] == np.float32(1.0)               # a polarity that never occurs gets the neutral step
    # a dual segment without negative values
    sp, sn, _, an = oracle.calibrate_act(np.array([[0.5, 2.0]], np.float32), [0, 2], [1])
    assert an[0] == 0.0 and sn[0] == 1.0 and sp[0] == np.float32(2.0) / q


def test_calibrate_act_batches_and_extremes(oracle):
    rng = np.random.default_rng(9)
    x = (rng.standard_normal((60, 96)) * 3).astype(np.float32)
    x[:, 32:64] = np.maximum(x[:, 32:64], -0.2)                      # a skewed (activation-like) segment
    kseg, dual = [0, 32, 64, 96], [0, 1, 1]
    whole = oracle.calibrate_act(x, kseg, dual)
    first = oracle.calibrate_act(x[:25], kseg, dual)
    both = oracle.calibrate_act(x[25:], kseg, dual, running=(first[2], first[3]))
    for a, b in zip(whole, both):                                    # running maxima over batches = one pass over all
        assert np.array_equal(a, b)
    # the independent numpy recipe of the workload generators gives the same steps
    sp2, sn2 = wl.amax_scales(x, kseg, dual)
    assert np.array_equal(whole[0], sp2)
    assert all(whole[1][ks] == sn2[ks] for ks in range(3) if dual[ks])
    # with these steps the extreme values land exactly on the ends of the code range
    xp, xn = oracle.quantize_act(x, kseg, dual, whole[0], whole[1])
    for ks in range(3):
        blk_p, blk_n = xp[:, kseg[ks]:kseg[ks + 1]], xn[:, kseg[ks]:kseg[ks + 1]]
        if dual[ks]:
            assert blk_p.max() == 127 and blk_n.min() == -127
        else:
            assert max(blk_p.max(), -blk_p.min()) == 127


# the activation in front of a DualScale layer, specified to the bit in fp32 and fused with the quantizer
# (Sec. 4.3.1: SiLU and GELU are the polarity-asymmetric activations the scheme is built for)
def _act_inputs():
    rng = np.random.default_rng(33)
    grid = np.linspace(-20.0, 20.0, 8001)
    rnd = rng.standard_normal(20000) * 3
    edge = np.array([0.0, -0.0, 1e-30, -1e-30, 1e-6, -1e-6, 0.5, -0.5, 86.9, -86.9, 87.5, -87.5, 88.5, -88.5, 100.0, -100.0,
                     1e4, -1e4, 3e19, -3e19, 1e38, -1e38, -0.7517916, -1.2784645])        # incl. the two minima
    return np.concatenate([grid, rnd, edge]).astype(np.float32)


def test_activation_against_closed_forms(oracle):
    """The fp32 activation against the closed forms in fp64 and against torch's own routines."""
    import torch

    x = _act_inputs()
    x64 = x.astype(np.float64)
    one = np.zeros((1, x.size), np.float32)
    one[0] = x
    silu = oracle.activation(one, [0, x.size], [oracle.ACT_SILU])[0].astype(np.float64)
    gelu = oracle.activation(one, [0, x.size], [oracle.ACT_GELU])[0].astype(np.float64)
    same = oracle.activation(one, [0, x.size], [oracle.ACT_NONE])[0]
    assert np.array_equal(same.view(np.uint32), x.view(np.uint32))
    with np.errstate(over="ignore"):
        silu_ref = x64 / (1.0 + np.exp(-x64))
        u = np.sqrt(2.0 / np.pi) * (x64 + 0.044715 * x64 ** 3)
        gelu_tanh_form = 0.5 * x64 * (1.0 + np.tanh(u))          # the textbook form; cancels in the negative tail
        gelu_ref = x64 / (1.0 + np.exp(-2.0 * u))                # the same function without the cancellation
    t = torch.from_numpy(x64)
    assert np.allclose(silu_ref, torch.nn.functional.silu(t).numpy(), rtol=1e-12, atol=1e-300)
    mid = np.abs(x64) < 1e3
    assert np.allclose(gelu_ref[mid], gelu_tanh_form[mid], rtol=0, atol=2e-15 * (1 + np.abs(x64[mid]).max()))
    assert np.allclose(gelu_tanh_form[mid], torch.nn.functional.gelu(t, approximate="tanh").numpy()[mid], rtol=0, atol=1e-12)
    with np.errstate(over="ignore", invalid="ignore"):
        zarg = np.nan_to_num(np.minimum(np.abs(2.0 * u), 90.0), nan=90.0)
    for got, ref, cond, name in ((silu, silu_ref, 0.0 * zarg, "silu"), (gelu, gelu_ref, zarg, "gelu")):
        assert np.all(np.isfinite(got)), name
        # a few fp32 roundings (exp32 is good to ~1.5 ulp, then an add, a division): 6e-7 relative.  GELU's exponent
        # z is itself a rounded fp32 number (three roundings, 2e-7 relative), which e^z turns into 2e-7 |z| relative.
        # Deep in the negative tail the result underflows towards -0 and only an absolute bound is meaningful.
        err = np.abs(got - ref)
        tol = (6e-7 + 2e-7 * cond) * np.abs(ref) + 1e-30
        assert np.all(err <= tol), (name, float(np.max(err / tol)))
    # landmarks: fixed points and the sign structure the DualScale split relies on
    assert np.all(silu[x == 0.0] == 0.0) and np.all(gelu[x == 0.0] == 0.0) and np.count_nonzero(x == 0.0) >= 2
    assert np.all(silu[x > 0] > 0) and np.all(silu[(x < 0) & (x > -80)] < 0)
    assert silu.min() > -0.27847 and silu.min() < -0.27845            # min of SiLU = -0.278465 at x = -1.27846
    assert gelu.min() > -0.17005 and gelu.min() < -0.17003            # min of tanh-GELU = -0.170041 at x = -0.75179
    big = x > 30
    assert np.array_equal(silu[big], x64[big]) and np.array_equal(gelu[big], x64[big])   # identity for large x


def test_fused_quantizer_is_activation_then_quantizer(oracle):
    rng = np.random.default_rng(5)
    h = (rng.standard_normal((9, 48)) * 2).astype(np.float32)
    kseg, dual, act = [0, 16, 32, 48], [0, 1, 1], [oracle.ACT_NONE, oracle.ACT_GELU, oracle.ACT_SILU]
    a = oracle.activation(h, kseg, act)
    assert np.array_equal(a[:, :16], h[:, :16])
    assert np.array_equal(a[:, 16:32], oracle.activation(h[:, 16:32], [0, 16], [oracle.ACT_GELU]))
    assert np.array_equal(a[:, 32:], oracle.activation(h[:, 32:], [0, 16], [oracle.ACT_SILU]))
    sp, sn, _, _ = oracle.calibrate_act(a, kseg, dual)
    xp, xn = oracle.quantize_act_fused(h, kseg, dual, act, sp, sn)
    xp2, xn2 = oracle.quantize_act(a, kseg, dual, sp, sn)
    assert np.array_equal(xp, xp2) and np.array_equal(xn, xn2)
    # the negative lobe of the activation fills the negative code range: that is what the second step is for
    assert xn[:, 16:32].min() == -127 and xp[:, 16:32].max() == 127
    # hand-worked: SiLU(1) = 0.7310586, SiLU(-1) = -0.2689414 ; steps 0.01 and 0.005 -> codes 73 and -54
    xp, xn = oracle.quantize_act_fused(np.array([[1.0, -1.0]], np.float32), [0, 2], [1], [oracle.ACT_SILU], [0.01], [0.005])
    assert xp.tolist() == [[73, 0]] and xn.tolist() == [[0, -54]]
    # GELU(1) = 0.841192, GELU(-1) = -0.158808 -> 84 and -32
    xp, xn = oracle.quantize_act_fused(np.array([[1.0, -1.0]], np.float32), [0, 2], [1], [oracle.ACT_GELU], [0.01], [0.005])
    assert xp.tolist() == [[84, 0]] and xn.tolist() == [[0, -32]]
    with pytest.raises(Exception):
        oracle.quantize_act_fused(h, kseg, dual, [0, 3, 1], sp, sn)


# percentile-clipping calibration (App. B, dual-scale sensitivity study: p = 1.0 against p <= 0.9999)
def test_calibrate_percentile_handworked(oracle):
    q = np.float32(127.0)
    x = np.array([[-4.0, -3.0, -2.0, -1.0, 0.5, 1.0, 2.0, 3.0, 5.0, 100.0]], np.float32)
    # dual: max(x,0) sorted = 0,0,0,0,.5,1,2,3,5,100 ; max(-x,0) sorted = 0,0,0,0,0,0,1,2,3,4 ; n = 10
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [1], 0.9)        # k = ceil(9.0) = 9
    assert ap[0] == 5.0 and an[0] == 3.0 and sp[0] == np.float32(5.0) / q and sn[0] == np.float32(3.0) / q
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [1], 0.91)       # k = ceil(9.1) = 10: the maxima
    assert ap[0] == 100.0 and an[0] == 4.0
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [1], 0.5)        # k = 5: 0.5 and a zero
    assert ap[0] == 0.5 and an[0] == 0.0 and sn[0] == 1.0                         # zero threshold: neutral step
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [1], 0.05)       # k = 1: the minima, both zero
    assert ap[0] == 0.0 and an[0] == 0.0 and sp[0] == 1.0
    # single-scale: |x| sorted = .5,1,1,2,2,3,3,4,5,100 ; no second step
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [0], 0.9)
    assert ap[0] == 5.0 and an[0] == 0.0 and sn[0] == 1.0
    sp, sn, ap, an = oracle.calibrate_act_percentile(x, [0, 10], [0], 0.8)        # k = 8
    assert ap[0] == 4.0
    # two K-segments, two rows: each segment ranks its own 2 x 2 values; k = ceil(0.75 * 4) = 3
    x2 = np.array([[1.0, 8.0, -1.0, 7.0], [2.0, 9.0, -2.0, -6.0]], np.float32)
    sp, sn, ap, an = oracle.calibrate_act_percentile(x2, [0, 2, 4], [0, 1], 0.75)
    assert ap.tolist() == [8.0, 0.0] and an.tolist() == [0.0, 2.0]                # seg 1: V+ = 0,7,0,0 ; V- = 1,0,2,6
    # batches: the running maximum of the per-batch thresholds, not the quantile of the union
    a = np.array([[1.0, 2.0, 3.0, 4.0]], np.float32)
    b = np.array([[10.0, 0.1, 0.2, 0.3]], np.float32)
    r1 = oracle.calibrate_act_percentile(a, [0, 4], [0], 0.75)                    # k = 3 -> 3.0
    r2 = oracle.calibrate_act_percentile(b, [0, 4], [0], 0.75, running=(r1[2], r1[3]))   # batch: 0.3
    assert r1[2][0] == 3.0 and r2[2][0] == 3.0
    r3 = oracle.calibrate_act_percentile(b, [0, 4], [0], 1.0, running=(r1[2], r1[3]))
    assert r3[2][0] == 10.0
    for bad in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(Exception):
            oracle.calibrate_act_percentile(a, [0, 4], [0], bad)


def test_calibrate_percentile_definition(oracle):
    """The threshold against what defines a nearest-rank quantile (a count, no sort), against numpy's own quantile
    routine, and against the min/max rule at p = 1."""
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((37, 160)) * 2).astype(np.float32)
    x[:, 64:] = np.where(x[:, 64:] > 0, x[:, 64:], 0.1 * x[:, 64:])          # an activation-like skewed segment
    x[3, 70] = 55.0                                                          # outliers that clipping removes
    x[9, 10] = -80.0
    kseg, dual = [0, 64, 160], [0, 1]
    mm = oracle.calibrate_act(x, kseg, dual)
    one = oracle.calibrate_act_percentile(x, kseg, dual, 1.0)
    for a, b in zip(mm, one):
        assert np.array_equal(a, b)
    prev = None
    for p in (0.37, 0.9, 0.99, 0.999, 0.9999):
        sp, sn, ap, an = oracle.calibrate_act_percentile(x, kseg, dual, p)
        for ks in range(2):
            blk = x[:, kseg[ks]:kseg[ks + 1]].astype(np.float64).ravel()
            n = blk.size
            k = int(np.ceil(p * n))
            assert abs(p * n - round(p * n)) > 1e-6                           # the cases sit away from rank boundaries
            pops = [(np.maximum(blk, 0), ap[ks]), (np.maximum(-blk, 0), an[ks])] if dual[ks] else [(np.abs(blk), ap[ks])]
            for v, t in pops:
                t = float(t)
                assert np.count_nonzero(v <= t) >= k and np.count_nonzero(v < t) < k
                assert t == np.quantile(v, p, method="inverted_cdf")
            if not dual[ks]:
                assert an[ks] == 0.0
        if prev is not None:                                                  # monotone in p
            assert np.all(ap >= prev[0]) and np.all(an >= prev[1])
        prev = (ap, an)
    # the outliers are what p = 0.9999 still keeps and p = 0.999 clips (n = 2368 and 3552: k = n at 0.9999)
    assert oracle.calibrate_act_percentile(x, kseg, dual, 0.9999)[2][1] == 55.0
    assert oracle.calibrate_act_percentile(x, kseg, dual, 0.999)[2][1] < 10.0
    assert oracle.calibrate_act_percentile(x, kseg, dual, 0.999)[2][0] < 80.0


def test_block_weight_quantizer(oracle):
    rng = np.random.default_rng(4)
    w = (rng.standard_normal((12, 40)) * 0.05).astype(np.float32)
    kseg, nseg = [0, 16, 40], [0, 5, 12]
    wq, ws = oracle.quantize_weight_block(w, kseg, nseg)
    for ks in range(2):
        for ns in range(2):
            blk = w[nseg[ns]:nseg[ns + 1], kseg[ks]:kseg[ks + 1]]
            s = ws[ks, nseg[ns]:nseg[ns + 1]]
            assert (s == s[0]).all()                                  # one step per block
            a = Fraction(float(np.abs(blk).max()))
            assert Fraction(float(s[0])) == Fraction(float(np.float32(float(a)) / np.float32(127.0)))
            codes = wq[nseg[ns]:nseg[ns + 1], kseg[ks]:kseg[ks + 1]]
            assert np.abs(codes).max() == 127                         # the block's largest weight sits on the grid end
            for (i, j), v in np.ndenumerate(blk):                     # every code is the nearest grid point (exact rationals)
                q = Fraction(float(v)) / Fraction(float(s[0]))
                want = _clip(_rne_fraction(Fraction(float(np.float32(v) / s[0]))))
                assert int(codes[i, j]) == want and abs(Fraction(int(codes[i, j])) - q) <= Fraction(1, 2) + Fraction(1, 10 ** 6)
    # one block = per-tensor; rows with equal maxima: identical to the per-channel quantizer (pinned above)
    w2 = w.copy()
    w2[:, 0] = 0.3
    w2[:, 20] = -0.3
    a, sa = oracle.quantize_weight_block(w2, kseg, [0, 12])
    b, sb = oracle.quantize_weight(w2, kseg)
    assert np.array_equal(a, b) and np.array_equal(sa, sb)
    # an all-zero block gets the neutral step
    w3 = w.copy()
    w3[0:5, 0:16] = 0.0
    _, s3 = oracle.quantize_weight_block(w3, kseg, nseg)
    assert (s3[0, 0:5] == 1.0).all()


# 4-bit weights (App. B: per-channel weights in the 4-bit settings) and their packed storage format
def test_w4_quantizer_and_packing(oracle):
    from fractions import Fraction

    rng = np.random.default_rng(12)
    w = (rng.standard_normal((6, 256)) * 0.05).astype(np.float32)
    w[2, :128] = 0.0                                              # an all-zero row segment: neutral step
    kseg = [0, 128, 256]
    wq, ws = oracle.quantize_weight_w4(w, kseg)
    assert wq.min() >= -7 and wq.max() <= 7
    for n in range(6):
        for ks in range(2):
            seg = w[n, kseg[ks]:kseg[ks + 1]]
            a = np.abs(seg).max()
            step = np.float32(1.0) if a == 0 else np.float32(a) / np.float32(7.0)
            assert ws[ks, n] == step
            # nearest code in exact rational arithmetic (ties do not occur in this sample)
            for k in range(0, 128, 7):
                q = Fraction(float(seg[k])) / Fraction(float(step))
                near = int(np.floor(q + Fraction(1, 2)))
                assert abs(q - near) != Fraction(1, 2)
                assert wq[n, kseg[ks] + k] == max(-7, min(7, near))
            if a > 0:                                             # the extreme value takes the end of the code range
                assert np.abs(wq[n, kseg[ks]:kseg[ks + 1]]).max() == 7
    assert np.all(wq[2, :128] == 0) and ws[0, 2] == 1.0
    # hand-worked: step 0.7 / 7 = 0.1 ; 0.25 / 0.1 = 2.5 -> 2 (ties to even), 0.35 -> 3.5 -> 4, -0.7 -> -7
    row = np.zeros((1, 128), np.float32)
    row[0, :4] = [0.25, 0.35, -0.7, 0.04]
    q1, s1 = oracle.quantize_weight_w4(row, [0, 128])
    assert s1[0, 0] == np.float32(0.7) / np.float32(7.0)
    expect = [int(np.rint(np.float32(v) / s1[0, 0])) for v in (0.25, 0.35, -0.7, 0.04)]
    assert q1[0, :4].tolist() == expect and expect[2] == -7 and expect[3] == 0
    # packing: groups of 16 rows, steps of 128 codes, one KiB per (group, step):
    #   packed[((g T + t) 16 + r) 64 + j] = code(16 g + r, 128 t + j) | code(16 g + r, 128 t + 64 + j) << 4
    codes = np.zeros((18, 256), np.int8)                          # two row groups (the second one padded), T = 2
    codes[0, 0], codes[0, 64], codes[0, 1], codes[0, 65] = 3, -2, -8, 7
    codes[5, 128 + 63], codes[5, 128 + 127] = -1, 5
    codes[17, 2], codes[17, 66] = 4, -4
    pk = oracle.pack_w4(codes)
    assert pk.shape == (2 * 16 * 128,)
    assert pk[0] == (3 | (0xE << 4)) and pk[1] == (0x8 | (7 << 4))
    assert pk[((0 * 2 + 1) * 16 + 5) * 64 + 63] == (0xF | (5 << 4))
    assert pk[((1 * 2 + 0) * 16 + 1) * 64 + 2] == (4 | (0xC << 4))
    assert np.count_nonzero(pk) == 4                              # padding rows and everything else are zero
    # round trip through an independent unpacker
    pk = oracle.pack_w4(wq).reshape(1, 2, 16, 64)                 # [group][step][row][byte]; 6 rows -> one group
    lo = (pk & 0xF).astype(np.int8)
    hi = (pk >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo)
    hi = np.where(hi > 7, hi - 16, hi)
    back = np.zeros((16, 256), np.int8)
    for t in range(2):
        back[:, 128 * t:128 * t + 64] = lo[0, t]
        back[:, 128 * t + 64:128 * t + 128] = hi[0, t]
    assert np.array_equal(back[:6], wq) and not back[6:].any()
    with pytest.raises(Exception):
        oracle.pack_w4(np.zeros((2, 100), np.int8))               # K must be a multiple of 128
    with pytest.raises(Exception):
        oracle.pack_w4(np.full((1, 128), 9, np.int8))             # not a 4-bit code
    # the layer with 4-bit weights is the same integer GEMM and DeQuant on these codes: against a float64 matmul
    x = (rng.standard_normal((5, 256))).astype(np.float32)
    sp, sn, _, _ = oracle.calibrate_act(x, kseg, [1, 0])
    r = oracle.seglinear(x, w, kseg, [0, 6], [1, 0], sp, sn, wbits=4)
    assert np.array_equal(r.wq, wq)
    xq = r.xq_pos.astype(np.float64) * np.repeat(sp, 128)[None, :] + r.xq_neg.astype(np.float64) * np.repeat(sn, 128)[None, :]
    wd = wq.astype(np.float64) * np.repeat(ws.T, 128, axis=1)
    assert np.allclose(r.y64, xq @ wd.T, rtol=1e-12, atol=1e-12)


# dynamic per-token activation steps (App. B: activations of the 4-bit settings)
def test_dynamic_per_token_steps(oracle):
    rng = np.random.default_rng(8)
    kseg, dual = [0, 128, 256], [0, 1]
    x = (rng.standard_normal((6, 256)) * rng.uniform(0.2, 5.0, size=(6, 1))).astype(np.float32)   # rows of different scale
    x[:, 128:] = np.where(x[:, 128:] > 0, x[:, 128:], 0.1 * x[:, 128:])
    w = (rng.standard_normal((10, 256)) * 0.05).astype(np.float32)
    xp, xn, sp, sn = oracle.quantize_act_dynamic(x, kseg, dual)
    q = np.float32(127.0)
    for m in range(6):
        assert sp[m, 0] == np.abs(x[m, :128]).max() / q and sn[m, 0] == 1.0          # single-scale segment
        assert sp[m, 1] == x[m, 128:].max() / q and sn[m, 1] == (-x[m, 128:].min()) / q
        # every token uses its whole code range
        assert max(xp[m, :128].max(), -xp[m, :128].min()) == 127
        assert xp[m, 128:].max() == 127 and xn[m, 128:].min() == -127
    # a row on its own gives the same codes: tokens do not interact
    a, b, c, d = oracle.quantize_act_dynamic(x[3:4], kseg, dual)
    assert np.array_equal(a[0], xp[3]) and np.array_equal(b[0], xn[3]) and np.array_equal(c[0], sp[3])
    r = oracle.seglinear_dynamic(x, w, kseg, [0, 10], dual)
    # rows that share their extremes with the whole batch: static calibration of that batch is the same layer
    same = np.tile(x[2:3], (3, 1))
    rs = oracle.seglinear_dynamic(same, w, kseg, [0, 10], dual)
    s_sp, s_sn, _, _ = oracle.calibrate_act(same, kseg, dual)
    st = oracle.seglinear(same, w, kseg, [0, 10], dual, s_sp, s_sn)
    assert np.array_equal(rs.y32, st.y32) and np.array_equal(rs.acc_pos, st.acc_pos)
    assert np.array_equal(rs.y32[0], r.y32[2])
    # against a float64 evaluation with every token's own steps
    xd = (r.xq_pos.astype(np.float64) * np.repeat(sp.astype(np.float64), 128, axis=1)
          + r.xq_neg.astype(np.float64) * np.repeat(sn.astype(np.float64), 128, axis=1))
    wd = r.wq.astype(np.float64) * np.repeat(r.wscale.T.astype(np.float64), 128, axis=1)
    assert np.allclose(r.y64, xd @ wd.T, rtol=1e-12, atol=1e-12)
    # dynamic steps are never worse than static ones of the batch, and better for the small-scale tokens
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    g_sp, g_sn, _, _ = oracle.calibrate_act(x, kseg, dual)
    stat = oracle.seglinear(x, w, kseg, [0, 10], dual, g_sp, g_sn)
    small = int(np.argmin(np.abs(x).max(axis=1)))
    assert np.abs(r.y64[small] - ref[small]).max() < np.abs(stat.y64[small] - ref[small]).max()


def test_geglu_against_closed_form_and_landmarks(oracle):
    """GEGLU (App. B lists it with SiLU and GELU): value * GELU(gate) with [value | gate] the two halves of a row.
    Closed form in fp64, torch's own routines, which half is gated, exact landmarks, and the composed quantizer."""
    import torch

    rng = np.random.default_rng(77)
    M, K = 9, 40
    h = (rng.standard_normal((M, 2 * K)) * 2.5).astype(np.float32)
    h[0, :6] = [2.0, -3.0, 0.5, 7.0, -1.0, 4.0]              # values
    h[0, K:K + 6] = [0.0, -0.0, 40.0, -40.0, 35.0, 1.0]      # their gates
    out = oracle.geglu(h)
    assert out.shape == (M, K) and out.dtype == np.float32
    v, g = h[:, :K].astype(np.float64), h[:, K:].astype(np.float64)
    u = np.sqrt(2.0 / np.pi) * (g + 0.044715 * g ** 3)
    with np.errstate(over="ignore"):
        ref = v * (g / (1.0 + np.exp(-2.0 * u)))
    tref = (torch.from_numpy(v) * torch.nn.functional.gelu(torch.from_numpy(g), approximate="tanh")).numpy()
    assert np.allclose(ref, tref, rtol=0, atol=1e-12 * (1 + np.abs(ref).max()))
    cond = np.minimum(np.abs(2.0 * u), 90.0)
    tol = (7e-7 + 2e-7 * cond) * np.abs(ref) + 1e-30          # the GELU's few roundings plus one product
    assert np.all(np.abs(out - ref) <= tol)
    # landmarks: GELU(0) = 0, GELU(g) = g for large g, GELU(g) = -0 for very negative g
    assert out[0, 0] == 0.0 and out[0, 1] == 0.0
    assert out[0, 2] == np.float32(0.5) * np.float32(40.0) and out[0, 4] == np.float32(-35.0)
    assert out[0, 3] == 0.0
    # which half is gated: swapping the halves is a different function (value * GELU(gate) is not symmetric)
    swapped = oracle.geglu(np.concatenate([h[:, K:], h[:, :K]], axis=1))
    assert not np.allclose(swapped, out, atol=1e-3)
    assert swapped[0, 5] == np.float32(1.0) * oracle.activation(np.array([[4.0]], np.float32), [0, 1], [oracle.ACT_GELU])[0, 0]
    # the product is a single fp32 rounding of the exact product of the two fp32 factors
    gl = oracle.activation(np.ascontiguousarray(h[:, K:]), [0, K], [oracle.ACT_GELU])
    exact = h[:, :K].astype(np.float64) * gl.astype(np.float64)
    assert np.array_equal(out, exact.astype(np.float32))
    # composed quantizer: the codes are those of the plain quantizer applied to GEGLU(h), K-segments over the output
    kseg, dual = [0, 16, K], [1, 0]
    sp, sn, _, _ = oracle.calibrate_act(out, kseg, dual)
    xp, xn = oracle.quantize_act_geglu(h, kseg, dual, sp, sn)
    rp, rn = oracle.quantize_act(out, kseg, dual, sp, sn)
    assert np.array_equal(xp, rp) and np.array_equal(xn, rn) and xp.max() == 127 and xn[:, :16].min() == -127
    with pytest.raises(ValueError):
        oracle.geglu(np.zeros((2, 5), np.float32))


def test_dynamic_steps_with_4bit_activation_codes(oracle):
    """a_bits = 4 (the W4A4 setting): q_max = 2^3 - 1 = 7 (Sec. 3), steps = row extreme / 7, the extreme itself gets code
    +-7, nothing leaves [-7, 7], the dequantized value is within half a step, and 8 bits is the default unchanged."""
    rng = np.random.default_rng(4)
    x = (rng.standard_normal((6, 96)) * rng.uniform(0.5, 4.0, size=(6, 1))).astype(np.float32)
    kseg, dual = [0, 32, 96], [1, 0]
    xp, xn, sp, sn = oracle.quantize_act_dynamic(x, kseg, dual, abits=4)
    xp8, xn8, sp8, sn8 = oracle.quantize_act_dynamic(x, kseg, dual)
    d8 = oracle.quantize_act_dynamic(x, kseg, dual, abits=8)
    assert all(np.array_equal(a, b) for a, b in zip((xp8, xn8, sp8, sn8), d8))
    assert xp.max() == 7 and xp[:, :32].min() >= 0 and xn.min() == -7 and xn.max() <= 0 and not xn[:, 32:].any()
    assert np.abs(xp[:, 32:].astype(int) + xn[:, 32:].astype(int)).max() == 7          # single-scale segment: |code| <= 7
    q7, q127 = np.float32(7), np.float32(127)
    for m in range(6):
        assert sp[m, 0] == x[m, :32].max() / q7 and sn[m, 0] == (-x[m, :32].min()) / q7
        assert sp[m, 1] == np.abs(x[m, 32:]).max() / q7 and sn[m, 1] == 1.0
        assert sp8[m, 0] == x[m, :32].max() / q127
        k = int(np.argmax(x[m, :32]))
        assert xp[m, k] == 7 and xn[m, int(np.argmin(x[m, :32]))] == -7
        deq = xp[m, :32] * np.float64(sp[m, 0]) + xn[m, :32] * np.float64(sn[m, 0])
        half = np.where(x[m, :32] >= 0, sp[m, 0], sn[m, 0]) / 2
        assert np.all(np.abs(deq - x[m, :32]) <= half * (1 + 1e-6))
    # the layer: with 4-bit codes the error grows (coarser steps) but stays inside its bound direction
    w = (rng.standard_normal((40, 96)) * 0.05).astype(np.float32)
    r4 = oracle.seglinear_dynamic(x, w, kseg, [0, 40], dual, abits=4)
    r8 = oracle.seglinear_dynamic(x, w, kseg, [0, 40], dual, abits=8)
    yfp = oracle.fp_reference(x, w)
    e4, e8 = np.linalg.norm(r4.y64 - yfp), np.linalg.norm(r8.y64 - yfp)
    assert e8 < e4 < 40 * e8


# ----------------------------------------------------------------------------------------------------
# SmoothQuant factors with one migration strength per K-segment (Sec. 4.2.2 last paragraph; App. B)
# ----------------------------------------------------------------------------------------------------
def test_smooth_factors_closed_forms(oracle):
    """s = a_x^alpha / a_w^(1 - alpha): hand-worked values, the two ends of alpha, the geometric mean in the middle,
    the neutral factor for a dead channel, one alpha per K-segment."""
    ax = np.array([16.0, 16.0, 9.0, 0.0, 2.0, 5.0], np.float32)
    aw = np.array([4.0, 4.0, 0.25, 3.0, 0.0, 0.125], np.float32)
    s, r = oracle.smooth_factors(ax, aw, [0, 6], [0.5])
    assert s[0] == 2.0 and s[2] == 6.0                       # sqrt(16)/sqrt(4), sqrt(9)/sqrt(0.25)
    assert s[3] == 1.0 and s[4] == 1.0                       # a_x = 0 or a_w = 0: the channel is left alone
    assert np.array_equal(r, (np.float32(1.0) / s).astype(np.float32))
    s0, _ = oracle.smooth_factors(ax, aw, [0, 6], [0.0])     # alpha = 0: everything migrates to the activation side
    assert s0[0] == 0.25 and s0[5] == 8.0
    s1, _ = oracle.smooth_factors(ax, aw, [0, 6], [1.0])     # alpha = 1: s = a_x
    assert s1[0] == 16.0 and s1[5] == 5.0
    sq, _ = oracle.smooth_factors(ax, aw, [0, 6], [0.25])    # 16^0.25 / 4^0.75 = 2 / 2^1.5 = 2^-0.5
    assert abs(float(sq[0]) - 2.0 ** -0.5) <= 2.0 ** -25
    # one alpha per K-segment: each segment is the single-segment rule with its own alpha
    s2, _ = oracle.smooth_factors(ax, aw, [0, 2, 6], [0.0, 1.0])
    assert np.array_equal(s2[:2], s0[:2]) and np.array_equal(s2[2:], s1[2:])
    rng = np.random.default_rng(0)
    ax = rng.uniform(0.01, 50, 300).astype(np.float32)
    aw = rng.uniform(0.001, 2, 300).astype(np.float32)
    for a in (0.1, 0.3, 0.5, 0.8):
        s, r = oracle.smooth_factors(ax, aw, [0, 300], [a])
        want = ax.astype(np.float64) ** np.float64(np.float32(a)) / aw.astype(np.float64) ** (1 - np.float64(np.float32(a)))
        assert np.all(np.abs(s - want) <= np.abs(want) * 2.0 ** -23)
        assert np.all(np.abs(r.astype(np.float64) * s - 1) <= 2.0 ** -22)
    with pytest.raises(RuntimeError):
        oracle.smooth_factors(ax, aw, [0, 300], [1.5])


def test_channel_amax(oracle):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((37, 50)).astype(np.float32)
    a = oracle.channel_amax(x)
    assert np.array_equal(a, np.abs(x).max(axis=0))
    x2 = (3 * rng.standard_normal((5, 50))).astype(np.float32)
    b = oracle.channel_amax(x2, running=a)
    assert np.array_equal(b, np.maximum(np.abs(x).max(axis=0), np.abs(x2).max(axis=0)))
    z = np.zeros((4, 3), np.float32)
    assert np.array_equal(oracle.channel_amax(z), np.zeros(3, np.float32))


def test_smoothing_migrates_range_between_the_operands(oracle):
    """Which operand is divided and which is multiplied: alpha = 1 normalises every activation channel to a maximum of
    1 (and gives the weights the activation's range), alpha = 0 normalises every weight channel; the product of the two
    smoothed operands is the product of the original ones."""
    rng = np.random.default_rng(2)
    M, K, N = 40, 24, 9
    x = (rng.standard_normal((M, K)) * rng.uniform(0.1, 30, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    ax, aw = oracle.channel_amax(x), oracle.channel_amax(w)
    s, r = oracle.smooth_factors(ax, aw, [0, K], [1.0])
    xs = oracle.smooth_act(x, r)
    assert np.all(np.abs(np.abs(xs).max(axis=0) - 1.0) <= 2.0 ** -22)
    s, r = oracle.smooth_factors(ax, aw, [0, K], [0.0])
    assert np.all(np.abs(np.abs(w * s).max(axis=0) - 1.0) <= 2.0 ** -22)
    s, r = oracle.smooth_factors(ax, aw, [0, K], [0.5])
    xs = oracle.smooth_act(x, r)
    assert np.array_equal(xs, (x * r).astype(np.float32))                   # one fp32 multiplication per element
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    got = xs.astype(np.float64) @ (w * s).astype(np.float64).T
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()


def test_power_of_two_smoothing_changes_nothing(oracle):
    """A smoothing factor that is the same power of two for every channel of a K-segment only moves exponents: the
    weight codes are those of the plain quantizer, the weight steps are multiplied by it, the activation codes are
    unchanged when the activation steps are divided by it, and the layer's output is bit-identical."""
    rng = np.random.default_rng(3)
    M, K, N = 11, 64, 13
    kseg, dual = [0, 24, 64], [1, 0]
    w_ = wl.random_layer(M, K, N, kseg, [0, N], dual, seed=7, x_dtype="f32", act="gelu")
    smooth = np.concatenate([np.full(24, 4.0, np.float32), np.full(40, 0.125, np.float32)])
    inv = (np.float32(1.0) / smooth).astype(np.float32)
    wq0, ws0 = oracle.quantize_weight(w_.w, kseg)
    wq1, ws1 = oracle.quantize_weight_smoothed(w_.w, kseg, smooth)
    assert np.array_equal(wq0, wq1)
    assert np.array_equal(ws1[0], ws0[0] * np.float32(4.0)) and np.array_equal(ws1[1], ws0[1] * np.float32(0.125))
    xs = oracle.smooth_act(w_.x, inv)
    seg_s = np.array([4.0, 0.125], np.float32)
    sp, sn = (w_.s_pos / seg_s).astype(np.float32), (w_.s_neg / seg_s).astype(np.float32)
    xp0, xn0 = oracle.quantize_act(w_.x, kseg, dual, w_.s_pos, w_.s_neg)
    xp1, xn1 = oracle.quantize_act(xs, kseg, dual, sp, sn)
    assert np.array_equal(xp0, xp1) and np.array_equal(xn0, xn1)
    ap, an = oracle.int_gemm(xp1, xn1, wq1, kseg, dual)
    y0, _ = oracle.dequant(ap, an, [0, N], dual, w_.s_pos, w_.s_neg, ws0)
    y1, _ = oracle.dequant(ap, an, [0, N], dual, sp, sn, ws1)
    assert np.array_equal(y0.view(np.uint32), y1.view(np.uint32))


def test_smoothed_weight_quantizer_is_the_quantizer_of_the_smoothed_weight(oracle):
    rng = np.random.default_rng(4)
    N, K = 17, 96
    kseg = [0, 32, 96]
    w = (rng.standard_normal((N, K)) * 0.03).astype(np.float32)
    s = rng.uniform(0.2, 7.0, K).astype(np.float32)
    a, b = oracle.quantize_weight_smoothed(w, kseg, s)
    c, d = oracle.quantize_weight((w * s).astype(np.float32), kseg)
    assert np.array_equal(a, c) and np.array_equal(b.view(np.uint32), d.view(np.uint32))
    # exact-rational nearest code for a few entries
    for (n, k) in [(0, 0), (3, 40), (16, 95)]:
        ks = 0 if k < 32 else 1
        v = Fraction(float(np.float32(w[n, k] * s[k]))) / Fraction(float(b[ks, n]))
        assert abs(Fraction(int(a[n, k])) - v) <= Fraction(1, 2) + Fraction(1, 10 ** 6)


def test_smoothing_lowers_the_error_on_outlier_channels(oracle):
    """The purpose of the optimizer (App. B, Frobenius-norm table of single layers): with a few activation channels
    20 times larger than the rest, migrating range to the weights (alpha = 0.5) lowers the layer's quantization error."""
    rng = np.random.default_rng(5)
    M, K, N = 64, 256, 48
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.permutation(K)[:3]] *= 20.0
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    kseg, nseg, dual = [0, K], [0, N], [0]
    ref = x.astype(np.float64) @ w.astype(np.float64).T

    def err(xx, ww_codes, ww_scales):
        sp = np.array([np.abs(xx).max() / 127], np.float32)
        xp, xn = oracle.quantize_act(xx, kseg, dual, sp, sp)
        ap, an = oracle.int_gemm(xp, xn, ww_codes, kseg, dual)
        y, _ = oracle.dequant(ap, an, nseg, dual, sp, sp, ww_scales)
        return float(np.linalg.norm(y - ref))

    plain = err(x, *oracle.quantize_weight(w, kseg))
    s, r = oracle.smooth_factors(oracle.channel_amax(x), oracle.channel_amax(w), kseg, [0.5])
    smoothed = err(oracle.smooth_act(x, r), *oracle.quantize_weight_smoothed(w, kseg, s))
    assert smoothed < 0.6 * plain, (smoothed, plain)


# ----------------------------------------------------------------------------------------------------
# low-rank side branch of the 4-bit settings (App. B: SVDQuant, rank 64)
# ----------------------------------------------------------------------------------------------------
def test_lowrank_branch_handworked_and_orientation(oracle):
    """y = y_q + (X Ld^T) Lu^T: integers by hand, a rank-1 outer product in closed form, and the orientation of the
    two factors (Ld [r][K] multiplies the input features, Lu [N][r] makes the output features)."""
    x = np.array([[1, 2, 3], [0, -1, 4]], np.float32)                       # M = 2, K = 3
    ld = np.array([[1, 0, 2], [0, 1, -1]], np.float32)                      # r = 2
    lu = np.array([[1, 1], [2, 0], [0, -3], [1, -1]], np.float32)           # N = 4
    t, y = oracle.lowrank(x, ld, lu)
    assert t.tolist() == [[7.0, -1.0], [8.0, -5.0]]
    assert y.tolist() == [[6.0, 14.0, 3.0, 8.0], [3.0, 16.0, 15.0, 13.0]]
    yq = np.arange(8, dtype=np.float32).reshape(2, 4)
    _, y2 = oracle.lowrank(x, ld, lu, yq)
    assert np.array_equal(y2, y + yq)
    rng = np.random.default_rng(0)
    u, v, xx = rng.standard_normal(7), rng.standard_normal(5), rng.standard_normal((3, 5))
    u, v, xx = u.astype(np.float32), v.astype(np.float32), xx.astype(np.float32)
    _, y = oracle.lowrank(xx, v[None, :], u[:, None])                       # W = u v^T
    want = (xx.astype(np.float64) @ v.astype(np.float64))[:, None] * u.astype(np.float64)[None, :]
    assert np.abs(y - want).max() <= 1e-14 * np.abs(want).max()


def test_lowrank_branch_reproduces_a_low_rank_weight(oracle):
    """A weight of rank <= r is reproduced by its factors: X W^T == (X Ld^T) Lu^T to double precision (numpy's SVD as
    the independent factorisation), and the branch plus the quantized residual is closer to the unquantized layer than
    the 4-bit quantizer alone when the weight has a strong low-rank part (the purpose of the optimizer)."""
    rng = np.random.default_rng(1)
    M, K, N, r = 24, 256, 40, 8
    a, b = rng.standard_normal((N, r)), rng.standard_normal((r, K))
    x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32)))
    w_low = (a @ b).astype(np.float32)
    uu, ss, vt = np.linalg.svd(w_low.astype(np.float64), full_matrices=False)
    lu = (uu[:, :r] * ss[:r]).astype(np.float32)
    ld = vt[:r].astype(np.float32)
    _, y = oracle.lowrank(x, ld, lu)
    ref = x.astype(np.float64) @ w_low.astype(np.float64).T
    assert np.abs(y - ref).max() <= 1e-5 * np.abs(ref).max()             # fp32 factors of an fp32 matrix
    # weight = strong low-rank part + small dense part, 4-bit residual
    w = (w_low * 0.05 + 0.02 * rng.standard_normal((N, K))).astype(np.float32)
    uu, ss, vt = np.linalg.svd(w.astype(np.float64), full_matrices=False)
    lu = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((uu[:, :r] * ss[:r]).astype(np.float32)))
    ld = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(vt[:r].astype(np.float32)))
    resid = (w.astype(np.float64) - lu.astype(np.float64) @ ld.astype(np.float64)).astype(np.float32)
    kseg, nseg, dual = [0, K], [0, N], [0]
    sp = np.array([np.abs(x).max() / 127], np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    plain = oracle.seglinear(x, w, kseg, nseg, dual, sp, sp, wbits=4)
    res = oracle.seglinear(x, resid, kseg, nseg, dual, sp, sp, wbits=4)
    _, y = oracle.lowrank(x, ld, lu, res.y32)
    assert np.linalg.norm(y - ref) < 0.5 * np.linalg.norm(plain.y32 - ref)


# ----------------------------------------------------------------------------------------------------
# fp8 variant (the 8/8 floating-point rows of the main results): OCP E4M3 codes in place of int8 ones
# ----------------------------------------------------------------------------------------------------
def test_fp8_format_against_the_published_table_and_torch(oracle):
    """E4M3: landmark values of the published format, every code against torch's float8_e4m3fn (an independent
    implementation), round trip of every finite code, ties to even, saturation at 448."""
    torch = pytest.importorskip("torch")
    codes = np.arange(256, dtype=np.uint8)
    v = oracle.fp8_decode(codes)
    assert v[0x00] == 0.0 and v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6      # subnormals, first normal
    assert v[0x38] == 1.0 and v[0x3C] == 1.5 and v[0x7E] == 448.0 and np.isnan(v[0x7F]) and np.isnan(v[0xFF])
    assert v[0xB8] == -1.0 and v[0xFE] == -448.0
    t = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    assert np.array_equal(np.nan_to_num(v, nan=-1e9), np.nan_to_num(t, nan=-1e9))
    fin = (codes & 0x7F) != 0x7F
    back = oracle.fp8_encode(v[fin])
    want = codes[fin].copy()
    assert np.array_equal(back & 0x7F, want & 0x7F) and np.array_equal(back[want != 0x80], want[want != 0x80])
    # ties: halfway between neighbours goes to the even mantissa; just off the tie goes to the nearer one
    assert oracle.fp8_encode(np.array([1.0625, 1.1875, 1.0626, 1.0624], np.float32)).tolist() == [0x38, 0x3A, 0x39, 0x38]
    assert oracle.fp8_encode(np.array([2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -11], np.float32)).tolist() == [0x00, 0x02, 0x00]
    assert oracle.fp8_encode(np.array([448.0, 449.0, 1e9, -1e9, 464.0], np.float32)).tolist() == [0x7E, 0x7E, 0x7E, 0xFE, 0x7E]
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * rng.choice([1e-3, 0.05, 1, 30, 200], 100000)).astype(np.float32)
    x = np.clip(x, -448, 448)
    te = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.fp8_encode(x), te)
    # nearest: no other code is closer
    grid = v[:0x7F].astype(np.float64)
    xa = np.abs(x[:2000]).astype(np.float64)
    got = oracle.fp8_decode(oracle.fp8_encode(np.abs(x[:2000]))).astype(np.float64)
    assert np.all(np.abs(got - xa) <= np.abs(grid[None, :] - xa[:, None]).min(axis=1) + 1e-300)


def test_fp8_quantizers_and_layer(oracle):
    """Steps = range / 448; the extreme gets +-448; values on the code grid with power-of-two steps round-trip and the
    layer is then exact; Q_dual keeps the two polarity matrices disjoint; the layer in double agrees with a float64
    matmul of the decoded operands; the error against the unquantized layer stays inside the format's bound."""
    rng = np.random.default_rng(1)
    M, K, N = 9, 64, 7
    kseg, nseg, dual = [0, 24, 64], [0, 3, 7], [1, 0]
    w_ = wl.random_layer(M, K, N, kseg, nseg, dual, seed=3, x_dtype="f32", act="gelu", with_seg_scale=True, with_bias=True)
    wq, ws = oracle.quantize_weight_fp8(w_.w, kseg)
    for ks in range(2):
        blk = np.abs(w_.w[:, kseg[ks]:kseg[ks + 1]]).max(axis=1)
        assert np.array_equal(ws[ks], (blk / np.float32(448)).astype(np.float32))
        assert np.all((wq[:, kseg[ks]:kseg[ks + 1]] & 0x7F).max(axis=1) == 0x7E)
    sp, sn, ap, an = oracle.calibrate_act(w_.x, kseg, dual)
    sp8 = np.where(ap == 0, np.float32(1), ap / np.float32(448)).astype(np.float32)
    sn8 = np.where(an == 0, np.float32(1), an / np.float32(448)).astype(np.float32)
    xp, xn = oracle.quantize_act_fp8(w_.x, kseg, dual, sp8, sn8)
    assert not np.logical_and((xp & 0x7F) != 0, (xn & 0x7F) != 0).any()
    assert np.all(xn[:, 24:] == 0) and np.all((xn & 0x80)[(xn & 0x7F) != 0] == 0x80) and np.all((xp[:, :24] & 0x80) == 0)
    y, mag = oracle.seglinear_fp8(xp, xn, wq, kseg, nseg, dual, sp8, sn8, ws, w_.seg_scale, w_.bias)
    # independent evaluation: decode, scale, float64 matmul per K-segment
    ref = np.zeros((M, N))
    nsof = np.searchsorted(np.asarray(nseg), np.arange(N), side="right") - 1
    for ks in range(2):
        sl = slice(kseg[ks], kseg[ks + 1])
        xv = oracle.fp8_decode(xp[:, sl]).astype(np.float64) * sp8[ks] + oracle.fp8_decode(xn[:, sl]).astype(np.float64) * sn8[ks]
        wv = oracle.fp8_decode(wq[:, sl]).astype(np.float64) * ws[ks][:, None].astype(np.float64)
        ref += (xv @ wv.T) * w_.seg_scale.reshape(2, -1)[ks][nsof][None, :]
    ref += w_.bias
    assert np.abs(y - ref).max() <= 1e-12 * np.abs(mag).max()
    assert np.all(mag + 1e-300 >= np.abs(y) - 1e-12 * np.abs(mag).max())
    # grid values, power-of-two steps: exact
    gx = oracle.fp8_decode(rng.integers(0, 0x7F, size=(4, 16)).astype(np.uint8)) * np.float32(0.25)
    gx[0, 0] = 448 * 0.25
    gw = oracle.fp8_decode(rng.integers(0x80, 0xFF, size=(3, 16)).astype(np.uint8)) * np.float32(2.0)
    gw[:, 0] = -448 * 2.0                                  # every output channel holds the extreme: its step is exactly 2
    q, s = oracle.quantize_weight_fp8(gw, [0, 16])
    assert np.all(s == 2.0) and np.array_equal(oracle.fp8_decode(q) * 2.0, gw)
    p, n_ = oracle.quantize_act_fp8(gx, [0, 16], [0], [0.25], [0.25])
    yy, _ = oracle.seglinear_fp8(p, n_, q, [0, 16], [0, 3], [0], [0.25], [0.25], s)
    assert np.array_equal(yy, gx.astype(np.float64) @ gw.astype(np.float64).T)
    # error against the unquantized layer: relative 2^-4 per operand (3 mantissa bits), subnormal codes aside
    full = w_.x.astype(np.float64) @ w_.w.astype(np.float64).T
    plain, _ = oracle.seglinear_fp8(xp, xn, wq, kseg, nseg, dual, sp8, sn8, ws)
    bound = (np.abs(w_.x).astype(np.float64) @ np.abs(w_.w).astype(np.float64).T) * (2 * 2.0 ** -4 + 2.0 ** -8) + 1e-3
    assert np.all(np.abs(plain - full) <= bound)


def test_fp8_quantizer_behind_the_activation(oracle):
    """Q_dual(act(h)) on the fp8 grid: hand-worked landmarks (SiLU(0) = 0, GELU of a large argument is the argument, both
    activations' minima are negative and small, so with a dual K-segment they take the s_- step), the single-scale
    K-segment passes h through unchanged, and the code of every element is the nearest E4M3 value of act(h) / s computed in
    double from the closed forms."""
    kseg, dual, act = [0, 4, 8, 12], [1, 1, 0], [1, 2, 0]           # SiLU | GELU | none
    s_pos, s_neg = np.float32([0.25, 0.125, 0.5]), np.float32([2.0 ** -9, 2.0 ** -9, 1.0])
    h = np.float32([[0.0, 8.0, -1.0, 30.0, 0.0, 8.0, -0.75, 30.0, 3.0, -3.0, 0.0, 224.0]])
    xp, xn = oracle.quantize_act_fp8_fused(h, kseg, dual, act, s_pos, s_neg)
    vp, vn = oracle.fp8_decode(xp)[0], oracle.fp8_decode(xn)[0]
    assert vp[0] == 0 and vn[0] == 0 and vp[4] == 0 and vn[4] == 0
    assert vp[3] == 120.0 and vp[7] == 240.0                        # 30 / 0.25, 30 / 0.125: exact grid values
    assert vp[1] == 32.0 and vn[1] == 0                             # SiLU(8) = 7.997 -> 31.99 -> 32
    assert vp[2] == 0 and vn[2] == -144.0                           # SiLU(-1) = -0.26894 / 2^-9 = -137.7 -> -144 (step 16 there)
    assert vp[6] == 0 and vn[6] == -88.0                            # GELU(-0.75) = -0.17004 / 2^-9 = -87.06 -> -88 (step 8 there)
    assert list(vp[8:]) == [6.0, -6.0, 0.0, 448.0] and not vn[8:].any()
    rng = np.random.default_rng(11)
    h = (rng.standard_normal((64, 12)) * 2.5).astype(np.float32)
    xp, xn = oracle.quantize_act_fp8_fused(h, kseg, dual, act, s_pos, s_neg)
    z = h.astype(np.float64)
    a = np.where(np.arange(12) < 4, z / (1 + np.exp(-z)),
                 np.where(np.arange(12) < 8, 0.5 * z * (1 + np.tanh(np.sqrt(2 / np.pi) * (z + 0.044715 * z ** 3))), z))
    step = np.where(a < 0, np.repeat(s_neg, 4).astype(np.float64), np.repeat(s_pos, 4).astype(np.float64))
    step[:, 8:] = s_pos[2]
    q = np.clip(a / step, -448, 448)
    grid = np.unique(oracle.fp8_decode(np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)).astype(np.float64))
    got = (oracle.fp8_decode(xp).astype(np.float64) + oracle.fp8_decode(xn).astype(np.float64))
    nearest = np.abs(q[..., None] - grid).min(axis=-1)
    assert (np.abs(got - q) <= nearest * (1 + 1e-5) + 1e-6 * np.abs(q) + 1e-12).all()
    assert (oracle.fp8_decode(xp)[:, :8] >= 0).all() and (oracle.fp8_decode(xn)[:, :8] <= 0).all()
