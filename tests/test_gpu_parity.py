"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: int8 codes, weight steps and int32 accumulators bit-exact; fp32 outputs within 1e-5 * max|y|;
bf16 outputs equal to bf16(oracle) up to one ulp where the fp32 tolerance straddles a rounding boundary.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

import paper_2507_14811_amd as sq  # noqa: E402
from paper_2507_14811_amd import workloads as wl  # noqa: E402

RTOL = 1e-5


def _gpu():
    from tests import gpu_util

    return gpu_util


@pytest.fixture(autouse=True)
def _reset_tuning():
    sq.sq_tuning_set("gemm_variant", -1)
    sq.sq_tuning_set("force_path", -1)
    yield
    sq.sq_tuning_set("gemm_variant", -1)
    sq.sq_tuning_set("force_path", -1)


# ----------------------------------------------------------------------------------------------------
# quantizers
# ----------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(5, 24, 7, [0, 24]), (33, 256, 70, [0, 64, 256]), (17, 100, 9, [0, 3, 100]),
                                   (8, 4096, 130, [0, 1024, 4096]), (3, 7, 2, [0, 7])])
@pytest.mark.parametrize("w_dtype", ["f32", "bf16"])
def test_quantize_weight(oracle, shape, w_dtype):
    g = _gpu()
    M, K, N, kseg = shape
    w = wl.random_layer(M, K, N, kseg, [0, N], [1] * (len(kseg) - 1), seed=K + N, w_std=0.05)
    w.w[1 % N, :] = 0.0                                     # an all-zero row: step 1.0, codes 0
    if w_dtype == "bf16":
        w.w = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.w))
    gl = g.GpuLayer(w, w_dtype=w_dtype)
    wq, ws = gl.quantize_weight()
    rq, rs = oracle.quantize_weight(w.w, kseg)
    assert np.array_equal(ws.view(np.uint32), rs.view(np.uint32))
    assert np.array_equal(wq, rq)


@pytest.mark.parametrize("case", [
    dict(M=9, K=64, kseg=[0, 64], dual=[1], x_dtype="bf16"),
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[0, 1], x_dtype="bf16"),
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[1, 0], x_dtype="f32"),
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 1], x_dtype="bf16"),        # unaligned: generic kernel
    dict(M=1, K=8, kseg=[0, 8], dual=[1], x_dtype="f32"),
    dict(M=300, K=2048, kseg=[0, 2048], dual=[0], x_dtype="bf16"),
    dict(M=129, K=1024, kseg=[0, 8, 16, 24, 1024], dual=[1, 0, 1, 1], x_dtype="bf16"),
])
@pytest.mark.parametrize("scales", ["amax", "pow2", "tiny", "clip"])
def test_quantize_act(oracle, case, scales):
    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], 4, case["kseg"], [0, 4], case["dual"], seed=case["K"] + case["M"],
                        x_dtype=case["x_dtype"], act="gelu")
    S = w.S
    if scales == "pow2":      # x / s exact, many exact ties
        w.x = np.round(w.x * 64).astype(np.float32) / 64
        w.s_pos = np.full(S, 2.0 ** -5, np.float32)
        w.s_neg = np.full(S, 2.0 ** -8, np.float32)
    elif scales == "tiny":    # reciprocal unusable: always the true division
        w.s_pos = np.full(S, 1e-35, np.float32)
        w.s_neg = np.full(S, 3e-36, np.float32)
        w.x = (w.x * 1e-33).astype(np.float32)
        if case["x_dtype"] == "bf16":
            w.x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.x))
    elif scales == "clip":    # steps far too small: everything saturates at +-127
        w.s_pos = (w.s_pos / 50).astype(np.float32)
        w.s_neg = (w.s_neg / 50).astype(np.float32)
    gl = g.GpuLayer(w)
    xp, xn, xq = gl.quantize_act()
    rp, rn = oracle.quantize_act(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    assert np.array_equal(xp, rp) and np.array_equal(xn, rn)
    # the merged array is the sum of the two polarity matrices, which never overlap
    assert not np.logical_and(rp != 0, rn != 0).any()
    assert np.array_equal(xq.astype(np.int16), rp.astype(np.int16) + rn.astype(np.int16))


def test_quantize_act_near_ties(oracle):
    """Quotients within a few ulp of k + 0.5: the reciprocal fast path must defer to the true division."""
    g = _gpu()
    rng = np.random.default_rng(3)
    s = np.float32(0.0123456)
    k = rng.integers(-126, 126, size=(64, 512)).astype(np.float32) + np.float32(0.5)
    x = (k * s).astype(np.float32)
    x = np.nextafter(x, np.where(rng.integers(0, 2, size=x.shape) == 0, -np.inf, np.inf).astype(np.float32))
    x[::3] = (k[::3] * s).astype(np.float32)
    w = wl.random_layer(64, 512, 4, [0, 512], [0, 4], [1], seed=1, x_dtype="f32")
    w.x = x
    w.s_pos = np.array([s], np.float32)
    w.s_neg = np.array([s * np.float32(0.37)], np.float32)
    gl = g.GpuLayer(w)
    xp, xn, _ = gl.quantize_act()
    rp, rn = oracle.quantize_act(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    assert np.array_equal(xp, rp) and np.array_equal(xn, rn)


FUSED = [
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[0, 1], act=[0, 2], h_dtype="bf16"),          # concat(plain, GELU(.))
    dict(M=1100, K=3072, kseg=[0, 512, 3072], dual=[0, 1], act=[0, 2], h_dtype="bf16"),       # many chunks per workgroup
    dict(M=3, K=1040, kseg=[0, 16, 1040], dual=[1, 1], act=[2, 1], h_dtype="bf16"),           # fewer chunks than threads
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[1, 1], act=[1, 2], h_dtype="f32"),
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 1], act=[2, 1], h_dtype="bf16"),           # unaligned: generic kernel
    dict(M=300, K=2048, kseg=[0, 2048], dual=[1], act=[1], h_dtype="bf16"),
    dict(M=129, K=1024, kseg=[0, 16, 32, 48, 1024], dual=[1, 0, 1, 1], act=[1, 0, 2, 1], h_dtype="f32"),
    dict(M=64, K=256, kseg=[0, 256], dual=[0], act=[2], h_dtype="f32"),                      # single-scale after an activation
]


@pytest.mark.parametrize("case", FUSED)
@pytest.mark.parametrize("spread", ["unit", "wide"])
def test_quantize_act_fused(oracle, case, spread):
    """xq = Q_dual(act(h)) with the bit-specified fp32 SiLU / GELU: codes bit-exact against the oracle."""
    import torch

    g = _gpu()
    M, K = case["M"], case["K"]
    rng = np.random.default_rng(M * 31 + K)
    h = rng.standard_normal((M, K)) * (1.0 if spread == "unit" else 12.0)
    h = h.astype(np.float32)
    if spread == "wide":                      # exercise the clamps of the exponential and exact zeros
        h[0, :8] = [0.0, -0.0, 95.0, -95.0, 1e4, -1e4, 88.25, -88.25]
    if case["h_dtype"] == "bf16":
        h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(h))
        hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        hd = torch.from_numpy(h).to(g.DEV)
    a = oracle.activation(h, case["kseg"], case["act"])
    sp, sn, _, _ = oracle.calibrate_act(a, case["kseg"], case["dual"])
    layer = sq.Layer(M, K, 4, case["kseg"], [0, 4], case["dual"], sp, sn)
    xq = torch.full((M, K), 99, dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_fused(layer, hd, case["act"], xq)
    torch.cuda.synchronize()
    rp, rn = oracle.quantize_act_fused(h, case["kseg"], case["dual"], case["act"], sp, sn)
    got = xq.cpu().numpy()
    want = (rp.astype(np.int16) + rn.astype(np.int16)).astype(np.int8)
    bad = np.argwhere(got != want)
    assert bad.size == 0, (len(bad), bad[:5], h[tuple(bad[0])], got[tuple(bad[0])], want[tuple(bad[0])])
    # with a workspace (bf16 inputs with aligned segments go through the code tables): the same codes
    ws = torch.full((sq.sq_quantize_act_fused_workspace_bytes(layer),), 0x33, dtype=torch.uint8, device=g.DEV)
    xq_t = torch.full((M, K), 99, dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_fused(layer, hd, case["act"], xq_t, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(xq_t, xq)
    # all-none codes: the plain quantizer
    sq.sq_quantize_act_fused(layer, hd, [0] * len(case["act"]), xq)
    xq2 = torch.empty_like(xq)
    sq.sq_quantize_act(layer, hd, xq2)
    torch.cuda.synchronize()
    assert torch.equal(xq, xq2)


@pytest.mark.parametrize("act", [1, 2])
def test_quantize_act_fused_exhaustive_bf16_and_dense_f32(oracle, act):
    """Every finite bf16 value, and 4 M fp32 values spread over the magnitudes that matter, through the fused pass."""
    import torch

    g = _gpu()
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = wl.bf16_bits_to_f32(bits)
    vals = vals[np.isfinite(vals)]
    vals = np.concatenate([vals, np.zeros(65536 - vals.size, np.float32)]).reshape(64, 1024)
    rng = np.random.default_rng(act)
    mag = np.exp(rng.uniform(np.log(1e-4), np.log(120.0), size=(2048, 2048)))
    dense = (mag * rng.choice([-1.0, 1.0], size=mag.shape)).astype(np.float32)
    for h, dt in ((vals, "bf16"), (dense, "f32")):
        M, K = h.shape
        if dt == "bf16":
            hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
        else:
            hd = torch.from_numpy(h).to(g.DEV)
        sp, sn = np.array([0.011], np.float32), np.array([0.0021], np.float32)
        layer = sq.Layer(M, K, 4, [0, K], [0, 4], [1], sp, sn)
        xq = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
        ws = torch.empty((sq.sq_quantize_act_fused_workspace_bytes(layer),), dtype=torch.uint8, device=g.DEV) if dt == "bf16" else None
        sq.sq_quantize_act_fused(layer, hd, [act], xq, workspace=ws)     # bf16: by table; fp32: arithmetic per element
        torch.cuda.synchronize()
        rp, rn = oracle.quantize_act_fused(h, [0, K], [1], [act], sp, sn)
        want = (rp.astype(np.int16) + rn.astype(np.int16)).astype(np.int8)
        got = xq.cpu().numpy()
        bad = np.argwhere(got != want)
        assert bad.size == 0, (dt, len(bad), h[tuple(bad[0])], got[tuple(bad[0])], want[tuple(bad[0])])
        assert len(np.unique(want)) > 200                 # the sample really spans the code range


# ----------------------------------------------------------------------------------------------------
# SegLinear GEMM on small / ragged shapes, every kernel path
# ----------------------------------------------------------------------------------------------------
def _check_layer(oracle, g, w, path, variant=-1, rows=None, y_dtypes=("f32", "bf16")):
    gl = g.GpuLayer(w)
    wq, ws = gl.quantize_weight()
    xp, xn, _ = gl.quantize_act()
    r = oracle.seglinear(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, w.seg_scale, w.bias, rows)
    assert np.array_equal(wq, r.wq) and np.array_equal(ws.view(np.uint32), r.wscale.view(np.uint32))
    assert np.array_equal(xp, r.xq_pos) and np.array_equal(xn, r.xq_neg)
    sq.sq_tuning_set("force_path", path)
    sq.sq_tuning_set("gemm_variant", variant)
    sel = slice(None) if rows is None else np.asarray(rows)
    ap, an = gl.debug_acc()
    assert np.array_equal(ap[:, sel], r.acc_pos), "acc_pos differs"
    assert np.array_equal(an[:, sel], r.acc_neg), "acc_neg differs"
    ymax = float(np.abs(r.y32).max())
    out = {}
    if "f32" in y_dtypes:
        y = gl.seglinear("f32")
        assert not np.isnan(y).any()
        err = float(np.abs(y[sel].astype(np.float64) - r.y32.astype(np.float64)).max())
        assert err <= RTOL * ymax, f"fp32 output error {err} > {RTOL} * {ymax}"
        out["err_rel"] = err / ymax if ymax > 0 else 0.0
    if "bf16" in y_dtypes:
        yb = gl.seglinear("bf16")
        out["bf16_mismatch"] = g.check_bf16_against(yb[sel], r.y32, r.y_bf16_bits, RTOL * ymax)
    # run-to-run determinism into freshly poisoned buffers
    ap2, an2 = gl.debug_acc()
    assert np.array_equal(ap, ap2) and np.array_equal(an, an2)
    return out


SMALL = [
    dict(M=64, K=256, N=384, kseg=[0, 128, 256], nseg=[0, 128, 256, 384], dual=[1, 1]),
    dict(M=130, K=384, N=70, kseg=[0, 384], nseg=[0, 70], dual=[1]),
    dict(M=257, K=640, N=300, kseg=[0, 128, 640], nseg=[0, 100, 300], dual=[0, 1]),
    dict(M=1, K=128, N=1, kseg=[0, 128], nseg=[0, 1], dual=[0]),
    dict(M=200, K=512, N=520, kseg=[0, 128, 256, 512], nseg=[0, 520], dual=[1, 0, 1]),
    dict(M=300, K=128, N=40, kseg=[0, 128], nseg=[0, 40], dual=[0]),
    dict(M=257, K=320, N=300, kseg=[0, 64, 320], nseg=[0, 100, 300], dual=[0, 1]),     # 64-aligned: 64-byte stages
    dict(M=97, K=192, N=264, kseg=[0, 192], nseg=[0, 264], dual=[1]),                  # 64-aligned
    dict(M=140, K=768, N=272, kseg=[0, 256, 384, 768], nseg=[0, 272], dual=[0, 1, 0]),   # one dual segment, in the middle
    dict(M=70, K=512, N=136, kseg=[0, 128, 512], nseg=[0, 136], dual=[1, 0]),           # one dual segment, first
]

# what each tile variant can hold: (K bytes per stage, two accumulator sets, fp32 running sum, both,
# both when exactly one K-segment is dual: its X^_- registers then double as the running sum)
VARIANT_CAPS = {0: (128, True, True, False, True), 1: (128, True, True, True, True), 2: (128, True, True, True, True),
                3: (128, True, True, True, True), 4: (128, False, False, False, False), 5: (128, True, True, True, True),
                6: (64, True, True, True, True), 7: (128, True, True, True, True), 8: (128, True, True, True, True)}


@pytest.mark.parametrize("case", SMALL)
@pytest.mark.parametrize("variant", sorted(VARIANT_CAPS))
def test_seglinear_mfma_small(oracle, case, variant):
    g = _gpu()
    any_dual, multi = any(case["dual"]), len(case["dual"]) > 1
    sk, dual_ok, multi_ok, multi_dual_ok, share_ok = VARIANT_CAPS[variant]
    kalign = 128 if all(k % 128 == 0 for k in case["kseg"]) else 64
    share = multi and sum(case["dual"]) == 1
    supported = sk <= kalign and (dual_ok or not any_dual) and (multi_ok or not multi or any_dual) and \
        (multi_dual_ok or (share and share_ok) or not (multi and any_dual))
    w = wl.random_layer(case["M"], case["K"], case["N"], case["kseg"], case["nseg"], case["dual"],
                        seed=case["M"] * 7 + variant, x_dtype="bf16", act="gelu", with_seg_scale=True, with_bias=True)
    if not supported:
        gl = g.GpuLayer(w)
        gl.quantize_weight()
        gl.quantize_act()
        sq.sq_tuning_set("force_path", 1)
        sq.sq_tuning_set("gemm_variant", variant)
        with pytest.raises(sq.SqError) as e:
            gl.seglinear("f32")
        assert e.value.status == 2          # SQ_ERR_UNSUPPORTED, nothing launched
        return
    _check_layer(oracle, g, w, path=1, variant=variant)


SKINNY = [
    dict(M=16, K=1152, N=176, kseg=[0, 1152], nseg=[0, 16, 176], dual=[1]),
    dict(M=5, K=256, N=33, kseg=[0, 64, 256], nseg=[0, 33], dual=[1, 0]),
    dict(M=33, K=320, N=100, kseg=[0, 320], nseg=[0, 100], dual=[0]),
    dict(M=64, K=640, N=48, kseg=[0, 128, 192, 640], nseg=[0, 48], dual=[1, 1, 0]),
    dict(M=48, K=64, N=17, kseg=[0, 64], nseg=[0, 17], dual=[1]),
    dict(M=1, K=128, N=16, kseg=[0, 128], nseg=[0, 16], dual=[1]),
]


@pytest.mark.parametrize("case", SKINNY)
def test_seglinear_skinny_small(oracle, case):
    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], case["N"], case["kseg"], case["nseg"], case["dual"],
                        seed=case["K"] + 1, x_dtype="bf16", act="silu", with_seg_scale=True, with_bias=True)
    _check_layer(oracle, g, w, path=2)


STREAM = [
    dict(M=16, K=1152, N=6912, kseg=[0, 1152], nseg=[0, 1152, 2304, 3456, 4608, 5760, 6912], dual=[1]),
    dict(M=5, K=256, N=33, kseg=[0, 128, 256], nseg=[0, 33], dual=[1, 0]),          # ragged N, two K-segments
    dict(M=33, K=384, N=100, kseg=[0, 384], nseg=[0, 100], dual=[0]),                # single path, three row tiles
    dict(M=64, K=640, N=4100, kseg=[0, 128, 256, 640], nseg=[0, 4100], dual=[1, 1, 0]),
    dict(M=1, K=128, N=16, kseg=[0, 128], nseg=[0, 16], dual=[1]),
    dict(M=48, K=1280, N=18000, kseg=[0, 1280], nseg=[0, 9000, 18000], dual=[1]),   # several groups per wave, 80 KB slab
    dict(M=16, K=1152, N=16 * 2100, kseg=[0, 1152], nseg=[0, 16 * 2100], dual=[1]),  # runs of groups, ring wraps
]


@pytest.mark.parametrize("case", STREAM)
def test_seglinear_stream_small(oracle, case):
    """Persistent weight-stream kernel of wide skinny layers (forced; automatic only for very wide N)."""
    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], case["N"], case["kseg"], case["nseg"], case["dual"],
                        seed=case["K"] + 11, x_dtype="bf16", act="silu", with_seg_scale=True, with_bias=True)
    _check_layer(oracle, g, w, path=3)


def test_stream_rejects_unaligned_k(oracle):
    g = _gpu()
    w = wl.random_layer(8, 192, 64, [0, 192], [0, 64], [1], seed=1, x_dtype="bf16", act="silu")
    gl = g.GpuLayer(w)
    gl.quantize_weight()
    gl.quantize_act()
    sq.sq_tuning_set("force_path", 3)
    with pytest.raises(sq.SqError) as e:
        gl.seglinear("f32")
    assert e.value.status == 2
    sq.sq_tuning_set("force_path", -1)


GROUPED = [
    dict(M=16, K=1152, N=1152, L=5, kseg=[0, 1152], dual=[1], ydt="bf16"),
    dict(M=7, K=256, N=100, L=3, kseg=[0, 128, 256], dual=[1, 0], ydt="f32"),        # ragged N, two K-segments
    dict(M=32, K=384, N=528, L=64, kseg=[0, 384], dual=[0], ydt="bf16"),              # the maximum group, single path
    dict(M=1, K=128, N=16, L=1, kseg=[0, 128], dual=[1], ydt="f32"),
    dict(M=16, K=640, N=4240, L=9, kseg=[0, 256, 640], dual=[0, 1], ydt="bf16"),     # runs of groups cross layer boundaries
]


@pytest.mark.parametrize("case", GROUPED)
def test_seglinear_grouped(oracle, case):
    """L layers that share the quantized input, one launch: every layer's output against the oracle's, layer by layer."""
    import torch

    g = _gpu()
    M, K, N, L = case["M"], case["K"], case["N"], case["L"]
    base = wl.random_layer(M, K, N, case["kseg"], [0, N], case["dual"], seed=K + L, x_dtype="bf16", act="silu", with_bias=True)
    gl = g.GpuLayer(base)
    gl.quantize_act()
    rng = np.random.default_rng(L * 1000 + N)
    tdt = torch.bfloat16 if case["ydt"] == "bf16" else torch.float32
    items, hosts = [], []
    for l in range(L):
        wl_l = (rng.standard_normal((N, K)) * (0.01 * (1 + l % 5))).astype(np.float32)
        bias_l = None if l % 3 == 2 else rng.standard_normal(N).astype(np.float32)
        wt = torch.from_numpy(wl_l).to(g.DEV)
        wq = torch.empty((N, K), dtype=torch.int8, device=g.DEV)
        ws = torch.empty((base.S, N), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_weight(gl.layer, wt, wq, ws)
        y = torch.full((M, N), float("nan"), dtype=tdt, device=g.DEV)
        items.append((wq, ws, None if bias_l is None else torch.from_numpy(bias_l).to(g.DEV), y))
        hosts.append((wl_l, bias_l))
    sq.sq_seglinear_grouped(gl.layer, gl.xq, items)
    torch.cuda.synchronize()
    for l in range(L):
        wl_l, bias_l = hosts[l]
        r = oracle.seglinear(base.x, wl_l, base.kseg_off, base.nseg_off, base.dual, base.s_pos, base.s_neg, None, bias_l)
        assert np.array_equal(items[l][0].cpu().numpy(), r.wq)
        ymax = float(np.abs(r.y32).max())
        if case["ydt"] == "f32":
            y = items[l][3].cpu().numpy()
            assert not np.isnan(y).any()
            err = float(np.abs(y.astype(np.float64) - r.y32.astype(np.float64)).max())
            assert err <= RTOL * ymax, f"layer {l}: fp32 output error {err} > {RTOL} * {ymax}"
        else:
            g.check_bf16_against(g.bf16_tensor_bits(items[l][3]), r.y32, r.y_bf16_bits, RTOL * ymax)


@pytest.mark.parametrize("case", [
    dict(M=16, K=1152, N=576, L=5, kseg=[0, 1152], dual=[1], ydt="f32"),              # two slab planes
    dict(M=32, K=512, N=200, L=3, kseg=[0, 128, 512], dual=[0, 1], ydt="bf16"),
    dict(M=7, K=256, N=1000, L=28, kseg=[0, 256], dual=[0], ydt="f32"),                # more groups than waves
])
def test_seglinear_grouped_fp8(oracle, case):
    """L layers on fp8 codes that share the quantized input, one launch: every layer against the oracle, layer by layer, and
    bit-identical to the single-layer call."""
    import torch

    g = _gpu()
    M, K, N, L = case["M"], case["K"], case["N"], case["L"]
    base = wl.random_layer(M, K, N, case["kseg"], [0, N], case["dual"], seed=K + L, x_dtype="bf16", act="silu", with_bias=True)
    base.s_pos = (base.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)
    base.s_neg = (base.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
    gl = g.GpuLayer(base)
    xq = torch.empty((M, K), dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
    r_xp, r_xn = oracle.quantize_act_fp8(base.x, base.kseg_off, base.dual, base.s_pos, base.s_neg)
    rng = np.random.default_rng(L * 1000 + N)
    tdt = torch.bfloat16 if case["ydt"] == "bf16" else torch.float32
    items, hosts = [], []
    for l in range(L):
        wl_l = (rng.standard_normal((N, K)) * (0.01 * (1 + l % 5))).astype(np.float32)
        bias_l = None if l % 3 == 2 else rng.standard_normal(N).astype(np.float32)
        wq = torch.empty((N, K), dtype=torch.uint8, device=g.DEV)
        ws = torch.empty((base.S, N), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_weight_fp8(gl.layer, torch.from_numpy(wl_l).to(g.DEV), wq, ws)
        y = torch.full((M, N), float("nan"), dtype=tdt, device=g.DEV)
        items.append((wq, ws, None if bias_l is None else torch.from_numpy(bias_l).to(g.DEV), y))
        hosts.append((wl_l, bias_l))
    sq.sq_seglinear_grouped_fp8(gl.layer, xq, items)
    torch.cuda.synchronize()
    for l in range(L):
        wl_l, bias_l = hosts[l]
        r_wq, r_ws = oracle.quantize_weight_fp8(wl_l, base.kseg_off)
        assert np.array_equal(items[l][0].cpu().numpy(), _plus_zero(r_wq))
        ref, mag = oracle.seglinear_fp8(r_xp, r_xn, r_wq, base.kseg_off, base.nseg_off, base.dual, base.s_pos, base.s_neg, r_ws,
                                        None, bias_l)
        got = items[l][3].float().cpu().numpy().astype(np.float64)
        assert not np.isnan(got).any()
        assert (np.abs(got - ref) <= _fp8_tol(K, mag, ref, case["ydt"])).all(), l
        single = torch.empty_like(items[l][3])
        sq.sq_tuning_set("force_path", 3)
        sq.sq_seglinear_fp8(gl.layer, xq, items[l][0], items[l][1], items[l][2], single)
        torch.cuda.synchronize()
        assert torch.equal(single, items[l][3])


def test_grouped_rejects_what_it_cannot_run(oracle):
    import torch

    g = _gpu()
    w = wl.random_layer(40, 256, 64, [0, 256], [0, 64], [1], seed=1, x_dtype="bf16", act="silu")   # M > 32
    gl = g.GpuLayer(w)
    gl.quantize_weight()
    gl.quantize_act()
    y = torch.empty((40, 64), dtype=torch.float32, device=g.DEV)
    with pytest.raises(sq.SqError) as e:
        sq.sq_seglinear_grouped(gl.layer, gl.xq, [(gl.wq, gl.wscale, None, y)])
    assert e.value.status == 2


def test_graph_capture_and_replay(oracle):
    """The calls allocate nothing and take their tables by value, so a step can be captured in a HIP graph.  Replay it
    several times with eager work and synchronisations in between, on fresh inputs, and check every replay."""
    import torch

    g = _gpu()
    w = wl.random_layer(300, 1024, 520, [0, 256, 1024], [0, 520], [0, 1], seed=21, x_dtype="bf16", act="gelu", with_bias=True)
    gl = g.GpuLayer(w)
    gl.quantize_weight()
    sq.sq_tuning_set("force_path", -1)
    sq.sq_tuning_set("gemm_variant", -1)
    y = torch.zeros((w.M, w.N), dtype=torch.float32, device=g.DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up outside the capture
        sq.sq_quantize_act(gl.layer, gl.x, gl.xq)
        sq.sq_seglinear(gl.layer, gl.xq, gl.wq, gl.wscale, gl.bias, y)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sq.sq_quantize_act(gl.layer, gl.x, gl.xq)
        sq.sq_seglinear(gl.layer, gl.xq, gl.wq, gl.wscale, gl.bias, y)
    rng = np.random.default_rng(5)
    for rep in range(3):
        xs = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((w.x * (1.0 + 0.1 * rep) + 0.01 * rng.standard_normal(w.x.shape)).astype(np.float32)))
        xs = np.clip(xs, w.x.min(), w.x.max()).astype(np.float32)       # stay inside the calibrated range: same steps
        gl.x.copy_(torch.from_numpy(wl.f32_to_bf16_bits(xs).view(np.int16)).view(torch.bfloat16).to(g.DEV))
        y.fill_(float("nan"))                                           # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        r = oracle.seglinear(xs, w.w, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, None, w.bias)
        xq = gl.xq.cpu().numpy()
        assert np.array_equal(xq.astype(np.int16), r.xq_pos.astype(np.int16) + r.xq_neg.astype(np.int16)), f"replay {rep}"
        err = float(np.abs(y.cpu().numpy().astype(np.float64) - r.y32).max())
        assert err <= RTOL * float(np.abs(r.y32).max()), f"replay {rep}: {err}"


CALIB = [
    dict(M=300, K=1024, kseg=[0, 256, 1024], dual=[0, 1], x_dtype="bf16"),
    dict(M=37, K=100, kseg=[0, 37, 100], dual=[1, 0], x_dtype="f32"),            # unaligned: scalar path
    dict(M=64, K=256, kseg=[0, 128, 256], dual=[1, 1], x_dtype="f32"),
    dict(M=5, K=64, kseg=[0, 64], dual=[1], x_dtype="bf16"),
]


@pytest.mark.parametrize("case", CALIB)
def test_calibrate_act(oracle, case):
    """Device min/max calibration: running maxima over two batches and the steps, bit-exact against the oracle."""
    import torch

    g = _gpu()
    M, K = case["M"], case["K"]
    w = wl.random_layer(M, K, 16, case["kseg"], [0, 16], case["dual"], seed=M + K, x_dtype=case["x_dtype"], act="gelu")
    S = w.S
    gl = g.GpuLayer(w)
    amax = torch.full((2, S), float("nan"), dtype=torch.float32, device=g.DEV)      # poisoned: the call must initialise it
    steps = torch.full((2, S), float("nan"), dtype=torch.float32, device=g.DEV)
    half = max(1, M // 2)
    lay_a = sq.Layer(half, K, 16, w.kseg_off, [0, 16], w.dual)
    lay_b = sq.Layer(M - half, K, 16, w.kseg_off, [0, 16], w.dual) if M > half else None
    sq.sq_calibrate_act(lay_a, gl.x[:half].contiguous(), amax, steps, accumulate=False)
    r1 = oracle.calibrate_act(w.x[:half], w.kseg_off, w.dual)
    torch.cuda.synchronize()
    assert np.array_equal(amax.cpu().numpy().view(np.uint32), np.stack([r1[2], r1[3]]).view(np.uint32))
    assert np.array_equal(steps.cpu().numpy().view(np.uint32), np.stack([r1[0], r1[1]]).view(np.uint32))
    if lay_b is not None:
        sq.sq_calibrate_act(lay_b, gl.x[half:].contiguous(), amax, steps, accumulate=True)
        r2 = oracle.calibrate_act(w.x[half:], w.kseg_off, w.dual, running=(r1[2], r1[3]))
        torch.cuda.synchronize()
        assert np.array_equal(amax.cpu().numpy().view(np.uint32), np.stack([r2[2], r2[3]]).view(np.uint32))
        assert np.array_equal(steps.cpu().numpy().view(np.uint32), np.stack([r2[0], r2[1]]).view(np.uint32))
        whole = oracle.calibrate_act(w.x, w.kseg_off, w.dual)
        assert np.array_equal(steps.cpu().numpy()[0], whole[0])


PCTL = [
    dict(M=300, K=1024, kseg=[0, 256, 1024], dual=[0, 1], x_dtype="bf16", ps=(0.9999, 0.999, 0.5)),
    dict(M=37, K=100, kseg=[0, 37, 100], dual=[1, 0], x_dtype="f32", ps=(0.99, 0.03)),         # unaligned: scalar path
    dict(M=67, K=256, kseg=[0, 128, 256], dual=[1, 1], x_dtype="f32", ps=(0.9999, 0.9, 1.0)),   # ragged row block
    dict(M=5, K=64, kseg=[0, 64], dual=[1], x_dtype="bf16", ps=(0.75, 1.0)),
    dict(M=1500, K=3072, kseg=[0, 1024, 3072], dual=[1, 0], x_dtype="bf16", ps=(0.9999, 0.99)),  # many workgroups
]


@pytest.mark.parametrize("case", PCTL)
def test_calibrate_act_percentile(oracle, case):
    """Device percentile-clipping calibration (exact radix select): thresholds, running maxima over two batches and
    the steps, bit-exact against the oracle's sort-and-index definition."""
    import torch

    g = _gpu()
    M, K = case["M"], case["K"]
    w = wl.random_layer(M, K, 16, case["kseg"], [0, 16], case["dual"], seed=7 * M + K, x_dtype=case["x_dtype"], act="gelu")
    x = w.x.copy()
    x[0, 0], x[M - 1, K - 1] = 77.0, -91.0                                         # outliers for the clipping to act on
    if case["x_dtype"] == "bf16":
        xd = torch.from_numpy(wl.f32_to_bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        xd = torch.from_numpy(x).to(g.DEV)
    S = w.S
    ws = torch.full((sq.sq_calibrate_workspace_bytes(),), 0x5A, dtype=torch.uint8, device=g.DEV)   # dirty on entry
    half = max(1, M // 2)
    lay_a = sq.Layer(half, K, 16, w.kseg_off, [0, 16], w.dual)
    lay_b = sq.Layer(M - half, K, 16, w.kseg_off, [0, 16], w.dual)
    for p in case["ps"]:
        amax = torch.full((2, S), float("nan"), dtype=torch.float32, device=g.DEV)  # poisoned: the call must initialise it
        steps = torch.full((2, S), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_calibrate_act_percentile(lay_a, xd[:half].contiguous(), p, amax, steps, ws, accumulate=False)
        r1 = oracle.calibrate_act_percentile(x[:half], w.kseg_off, w.dual, p)
        torch.cuda.synchronize()
        assert np.array_equal(amax.cpu().numpy().view(np.uint32), np.stack([r1[2], r1[3]]).view(np.uint32)), (p, "first batch")
        assert np.array_equal(steps.cpu().numpy().view(np.uint32), np.stack([r1[0], r1[1]]).view(np.uint32))
        sq.sq_calibrate_act_percentile(lay_b, xd[half:].contiguous(), p, amax, steps, ws, accumulate=True)
        r2 = oracle.calibrate_act_percentile(x[half:], w.kseg_off, w.dual, p, running=(r1[2], r1[3]))
        torch.cuda.synchronize()
        assert np.array_equal(amax.cpu().numpy().view(np.uint32), np.stack([r2[2], r2[3]]).view(np.uint32)), (p, "second batch")
        assert np.array_equal(steps.cpu().numpy().view(np.uint32), np.stack([r2[0], r2[1]]).view(np.uint32))


WBLOCK = [
    dict(N=384, K=256, kseg=[0, 128, 256], nseg=[0, 128, 256, 384], w_dtype="f32"),
    dict(N=70, K=100, kseg=[0, 37, 100], nseg=[0, 5, 70], w_dtype="f32"),           # unaligned
    dict(N=1152, K=1152, kseg=[0, 1152], nseg=[0, 1152], w_dtype="bf16"),            # one block: per tensor
    dict(N=600, K=512, kseg=[0, 512], nseg=[0, 100, 300, 600], w_dtype="bf16"),      # segments longer than a workgroup
]


@pytest.mark.parametrize("case", WBLOCK)
def test_quantize_weight_block(oracle, case):
    import torch

    g = _gpu()
    N, K = case["N"], case["K"]
    S = len(case["kseg"]) - 1
    w = wl.random_layer(4, K, N, case["kseg"], case["nseg"], [0] * S, seed=N + K, x_dtype="f32")
    ww = w.w.copy()
    ww[case["nseg"][0]:case["nseg"][1], case["kseg"][0]:case["kseg"][1]] *= 3.0          # blocks with different ranges
    if case["w_dtype"] == "bf16":
        ww = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(ww))
    w.w = ww
    gl = g.GpuLayer(w, w_dtype=case["w_dtype"])
    sq.sq_quantize_weight_block(gl.layer, gl.wt, gl.wq, gl.wscale)
    torch.cuda.synchronize()
    rq, rs = oracle.quantize_weight_block(ww, case["kseg"], case["nseg"])
    assert np.array_equal(gl.wscale.cpu().numpy().view(np.uint32), rs.view(np.uint32))
    assert np.array_equal(gl.wq.cpu().numpy(), rq)


SMOOTH = [
    dict(M=300, K=1536, N=200, kseg=[0, 1536], dual=[0], alpha=[0.5], x_dtype="bf16", w_dtype="f32", outliers=15),      # fused QKV with outlier channels
    dict(M=130, K=640, N=70, kseg=[0, 128, 640], dual=[0, 1], alpha=[0.3, 0.8], x_dtype="bf16", w_dtype="bf16", outliers=4),
    dict(M=64, K=256, N=33, kseg=[0, 64, 128, 256], dual=[1, 1, 0], alpha=[0.0, 1.0, 0.5], x_dtype="f32", w_dtype="f32", outliers=2),
    dict(M=13, K=100, N=9, kseg=[0, 37, 100], dual=[1, 0], alpha=[0.6, 0.4], x_dtype="f32", w_dtype="bf16", outliers=1),  # unaligned: one element per thread
    dict(M=1, K=16, N=1, kseg=[0, 16], dual=[1], alpha=[0.5], x_dtype="bf16", w_dtype="f32", outliers=0),
]


@pytest.mark.parametrize("case", SMOOTH)
def test_smoothed_layer(oracle, case):
    """SmoothQuant factors with one alpha per K-segment in front of the quantizers: per-channel maxima over two
    calibration batches, factors, smoothed weight codes and steps, smoothed activation codes: all bit-exact against the
    oracle; the layer's accumulators bit-exact and its output within the fp32 tolerance, every element."""
    import torch

    g = _gpu()
    M, K, N, kseg, dual = case["M"], case["K"], case["N"], case["kseg"], case["dual"]
    w = wl.random_layer(M, K, N, kseg, [0, N], dual, seed=M + K, x_dtype=case["x_dtype"], act="gelu", with_bias=True)
    rng = np.random.default_rng(K)
    if case["outliers"]:
        w.x[:, rng.permutation(K)[:case["outliers"]]] *= 20.0
        if case["x_dtype"] == "bf16":
            w.x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.x))
    if case["w_dtype"] == "bf16":
        w.w = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.w))
    w.w[:, 0] = 0.0                                            # a dead weight channel keeps the neutral factor
    gl = g.GpuLayer(w, w_dtype=case["w_dtype"])
    # calibration: two batches of activations (the second is the first, scaled), the weight
    x2 = (w.x * np.float32(0.5)).astype(np.float32)
    x2[:, 1] *= 7.0
    if case["x_dtype"] == "bf16":
        x2 = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x2))
        x2d = torch.from_numpy(wl.f32_to_bf16_bits(x2).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        x2d = torch.from_numpy(x2).to(g.DEV)
    ax = torch.full((K,), float("nan"), dtype=torch.float32, device=g.DEV)
    aw = torch.full((K,), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_calibrate_channel_amax(gl.layer, gl.x, ax)
    sq.sq_calibrate_channel_amax(gl.layer, x2d, ax, accumulate=True)
    sq.sq_weight_channel_amax(gl.layer, gl.wt, aw)
    torch.cuda.synchronize()
    r_ax = oracle.channel_amax(x2, running=oracle.channel_amax(w.x))
    r_aw = oracle.channel_amax(w.w)
    assert np.array_equal(ax.cpu().numpy().view(np.uint32), r_ax.view(np.uint32))
    assert np.array_equal(aw.cpu().numpy().view(np.uint32), r_aw.view(np.uint32))
    smooth, inv = sq.sq_smooth_factors(gl.layer, ax.cpu().numpy(), aw.cpu().numpy(), case["alpha"])
    r_s, r_inv = oracle.smooth_factors(r_ax, r_aw, kseg, case["alpha"])
    assert np.array_equal(smooth.view(np.uint32), r_s.view(np.uint32)) and np.array_equal(inv.view(np.uint32), r_inv.view(np.uint32))
    assert smooth[0] == 1.0
    # weights
    sq.sq_quantize_weight_smoothed(gl.layer, gl.wt, torch.from_numpy(smooth).to(g.DEV), gl.wq, gl.wscale)
    torch.cuda.synchronize()
    r_wq, r_ws = oracle.quantize_weight_smoothed(w.w, kseg, r_s)
    assert np.array_equal(gl.wq.cpu().numpy(), r_wq)
    assert np.array_equal(gl.wscale.cpu().numpy().view(np.uint32), r_ws.view(np.uint32))
    # activations: steps calibrated on the smoothed tensor (oracle side: no device value enters the oracle)
    xs = oracle.smooth_act(w.x, r_inv)
    sp, sn, _, _ = oracle.calibrate_act(xs, kseg, dual)
    lay = sq.Layer(M, K, N, kseg, [0, N], dual, sp, sn)
    sq.sq_quantize_act_smoothed(lay, gl.x, torch.from_numpy(inv).to(g.DEV), gl.xq)
    torch.cuda.synchronize()
    r_xp, r_xn = oracle.quantize_act(xs, kseg, dual, sp, sn)
    xp, xn = g.split_codes(w, gl.xq.cpu().numpy())
    assert np.array_equal(xp, r_xp) and np.array_equal(xn, r_xn)
    # the layer on the smoothed operands
    r_ap, r_an = oracle.int_gemm(r_xp, r_xn, r_wq, kseg, dual)
    r_y, _ = oracle.dequant(r_ap, r_an, [0, N], dual, sp, sn, r_ws, None, w.bias)
    ap = torch.empty((w.S, M, N), dtype=torch.int32, device=g.DEV)
    an = torch.empty((w.S, M, N), dtype=torch.int32, device=g.DEV)
    sq.sq_seglinear_debug_acc(lay, gl.xq, gl.wq, ap, an)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_seglinear(lay, gl.xq, gl.wq, gl.wscale, gl.bias, y)
    torch.cuda.synchronize()
    assert np.array_equal(ap.cpu().numpy(), r_ap) and np.array_equal(an.cpu().numpy(), r_an)
    ymax = float(np.abs(r_y).max())
    assert float(np.abs(y.cpu().numpy().astype(np.float64) - r_y).max()) <= RTOL * ymax
    # and it serves its purpose: closer to the unquantized layer than the plain quantizers on the outlier case
    if case["outliers"] >= 15:
        ref = w.x.astype(np.float64) @ w.w.astype(np.float64).T + w.bias
        plain = oracle.seglinear(w.x, w.w, kseg, [0, N], dual, w.s_pos, w.s_neg, None, w.bias)
        assert np.linalg.norm(r_y - ref) < np.linalg.norm(plain.y32 - ref)


LOWRANK = [
    dict(M=300, K=512, N=200, rank=64, x_dtype="bf16", yq=True),
    dict(M=33, K=48, N=7, rank=32, x_dtype="f32", yq=False),             # shorter than one group of four steps, ragged everywhere
    dict(M=129, K=1040, N=257, rank=64, x_dtype="f32", yq=True),         # K = 16 * 65: groups of four steps and a tail
    dict(M=2048, K=4608, N=1152, rank=64, x_dtype="bf16", yq=True),      # several K slices, many row blocks
    dict(M=16, K=1152, N=6912, rank=64, x_dtype="bf16", yq=False),
    dict(M=257, K=64, N=40, rank=32, x_dtype="bf16", yq=True),           # LDS-staged down projection: a single stage
    dict(M=1000, K=1088, N=96, rank=32, x_dtype="bf16", yq=False),       # 17 stages dealt unevenly over the K slices
    dict(M=515, K=8192, N=64, rank=64, x_dtype="bf16", yq=True),         # long slices: the ring wraps many times
]


def _bf16_round(a):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.ascontiguousarray(a, dtype=np.float32)))


def _bf16_dev(g, a):
    import torch

    return torch.from_numpy(wl.f32_to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(g.DEV)


def _lowrank_bound(x, ld, lu, K):
    """fp32 evaluation of the two products against the double-precision oracle: both sums run in fp32 (matrix cores over
    K, FMAs over the rank), so the error of an output is bounded by the rounding unit times the sum of the magnitudes of
    its terms, times a factor that grows like the square root of the number of terms (with a wide safety margin)."""
    b = np.abs(x).astype(np.float64) @ np.abs(ld).astype(np.float64).T @ np.abs(lu).astype(np.float64).T
    return (8.0 * np.sqrt(K) + 64.0) * 2.0 ** -24 * b


@pytest.mark.parametrize("case", LOWRANK)
def test_lowrank_add(oracle, case):
    """y = y_q + (X Ld^T) Lu^T: the 16-bit side branch of the 4-bit settings against the double-precision oracle on every
    element, fp32 and bf16 outputs, with and without a quantized-layer output to add to."""
    import torch

    g = _gpu()
    M, K, N, r = case["M"], case["K"], case["N"], case["rank"]
    rng = np.random.default_rng(M + K + r)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, :3] *= 15.0
    ld = _bf16_round(rng.standard_normal((r, K)) / np.sqrt(K))
    lu = _bf16_round(rng.standard_normal((N, r)) * 0.1)
    yq = (rng.standard_normal((M, N)) * 0.3).astype(np.float32) if case["yq"] else None
    xb = _bf16_round(x)                                   # what the 16-bit branch multiplies
    if case["x_dtype"] == "bf16":
        x = xb
        xd = _bf16_dev(g, x)
    else:
        xd = torch.from_numpy(x).to(g.DEV)
    layer = sq.Layer(M, K, N, [0, K], [0, N], [0])
    ws = torch.full((sq.sq_lowrank_workspace_bytes(layer, r),), 0xFF, dtype=torch.uint8, device=g.DEV)
    yqd = None if yq is None else torch.from_numpy(yq).to(g.DEV)
    _, ref = oracle.lowrank(xb, ld, lu, yq)
    bound = _lowrank_bound(xb, ld, lu, K) + (0 if yq is None else np.abs(yq) * 2.0 ** -23)
    for ydt in ("f32", "bf16"):
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16 if ydt == "bf16" else torch.float32, device=g.DEV)
        sq.sq_lowrank_add(layer, xd, _bf16_dev(g, ld), _bf16_dev(g, lu), yqd, y, ws)
        torch.cuda.synchronize()
        got = y.float().cpu().numpy().astype(np.float64)
        assert not np.isnan(got).any()
        tol = bound + (np.abs(ref) * 2.0 ** -8 if ydt == "bf16" else np.abs(ref) * 2.0 ** -23)
        assert (np.abs(got - ref) <= tol + 1e-30).all(), float((np.abs(got - ref) / (tol + 1e-30)).max())
        if ydt == "f32":      # the typical error is far inside the bound
            assert np.abs(got - ref).max() <= 2e-5 * np.abs(ref).max()
    # run-to-run determinism and in-place use (y is y_q)
    if yq is not None:
        y1 = yqd.clone()
        sq.sq_lowrank_add(layer, xd, _bf16_dev(g, ld), _bf16_dev(g, lu), y1, y1, ws)
        y2 = torch.empty_like(yqd)
        sq.sq_lowrank_add(layer, xd, _bf16_dev(g, ld), _bf16_dev(g, lu), yqd, y2, ws)
        torch.cuda.synchronize()
        assert torch.equal(y1, y2)


@pytest.mark.parametrize("M", [16, 300])
def test_w4_layer_with_lowrank_branch(oracle, M):
    """The 4-bit setting end to end: W = Lu Ld + R (numpy's SVD, rank 64), R through the 4-bit weight quantizer and the
    SegLinear kernels (weight stream for a few token rows; unpacked into the tile kernel for many), the rank-64 part
    through sq_lowrank_add: against the oracle's composition of the same steps on every element, and closer to the
    unquantized layer than the 4-bit quantizer alone."""
    import torch

    g = _gpu()
    K, N, r = 1152, 640, 64
    w = wl.random_layer(M, K, N, [0, K], [0, N], [1], seed=31 + M, x_dtype="bf16", act="silu")
    rng = np.random.default_rng(M)
    low = (rng.standard_normal((N, 12)) @ rng.standard_normal((12, K))).astype(np.float32) * 0.02
    wt = (w.w + low).astype(np.float32)
    uu, ss, vt = np.linalg.svd(wt.astype(np.float64), full_matrices=False)
    lu, ld = _bf16_round(uu[:, :r] * ss[:r]), _bf16_round(vt[:r])
    resid = (wt.astype(np.float64) - lu.astype(np.float64) @ ld.astype(np.float64)).astype(np.float32)
    w.w = resid
    gl = g.GpuLayer(w)
    wq4 = torch.empty((((N + 15) // 16) * 16 * (K // 2),), dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_weight_w4(gl.layer, gl.wt, wq4, gl.wscale)
    gl.quantize_act()
    yq = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    if M <= 64:
        sq.sq_seglinear_w4(gl.layer, gl.xq, wq4, gl.wscale, None, yq)
    else:
        sq.sq_unpack_w4(gl.layer, wq4, gl.wq)
        sq.sq_seglinear(gl.layer, gl.xq, gl.wq, gl.wscale, None, yq)
    ws = torch.empty((sq.sq_lowrank_workspace_bytes(gl.layer, r),), dtype=torch.uint8, device=g.DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_lowrank_add(gl.layer, gl.x, _bf16_dev(g, ld), _bf16_dev(g, lu), yq, y, ws)
    torch.cuda.synchronize()
    r_q = oracle.seglinear(w.x, resid, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, wbits=4)
    ymax = float(np.abs(r_q.y32).max())
    assert float(np.abs(yq.cpu().numpy().astype(np.float64) - r_q.y32).max()) <= RTOL * ymax
    _, ref = oracle.lowrank(w.x, ld, lu, r_q.y32)
    tol = _lowrank_bound(w.x, ld, lu, K) + RTOL * ymax + np.abs(ref) * 2.0 ** -23
    got = y.cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= tol).all()
    full = w.x.astype(np.float64) @ wt.astype(np.float64).T
    plain = oracle.seglinear(w.x, wt, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, wbits=4)
    assert np.linalg.norm(got - full) < np.linalg.norm(plain.y32 - full)


# ----------------------------------------------------------------------------------------------------
# the 8-bit floating-point variant (OCP E4M3 codes)
# ----------------------------------------------------------------------------------------------------
def _plus_zero(c):
    """The library stores every zero as +0; the format's -0 is the same value."""
    c = c.copy()
    c[c == 0x80] = 0
    return c


def _split_fp8(w, xq):
    """Documented decoding of the merged fp8 activation codes: in a dual K-segment X^_- holds the codes with the sign bit
    set and X^_+ the others, the rest +0; elsewhere X^_+ = xq (index work only)."""
    mask = _gpu().dual_col_mask(w)
    xp, xn = xq.copy(), np.zeros_like(xq)
    neg = (xq & 0x80) != 0
    neg[:, ~mask] = False
    xn[neg] = xq[neg]
    xp[neg] = 0
    return xp, xn


@pytest.mark.parametrize("w_dtype", ["f32", "bf16"])
def test_fp8_encoding_through_the_weight_quantizer(oracle, w_dtype):
    """Rows whose largest magnitude is 448 have step 1, so their codes are the bare fp32 -> E4M3 conversion: every finite
    code's value, every midpoint between neighbours (ties), the fp32 neighbours of those midpoints, the subnormal range,
    zeros of both signs and values that underflow.  Other rows: random steps."""
    import torch

    g = _gpu()
    vals = oracle.fp8_decode(np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8))
    pos = np.sort(np.unique(np.abs(vals)))
    mid = ((pos[:-1].astype(np.float64) + pos[1:].astype(np.float64)) / 2).astype(np.float32)
    probe = np.concatenate([vals, mid, -mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)),
                            -np.nextafter(mid, np.float32(0)), np.float32([0.0, -0.0, 1e-6, -1e-6, 2.0 ** -10, -2.0 ** -10, 447.9, 448.0])])
    if w_dtype == "bf16":
        probe = _bf16_round(probe)
    K = 1024
    assert probe.size <= K - 1
    rng = np.random.default_rng(5)
    N = 37
    wm = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    wm[0, :probe.size] = probe
    wm[0, probe.size:] = 0.0
    wm[0, K - 1] = -448.0
    wm[1] = 0.0                                                   # dead channel: step 1, codes +0
    wm[2] = np.float32(1e-30) * rng.standard_normal(K).astype(np.float32)
    if w_dtype == "bf16":
        wm = _bf16_round(wm)
    for kseg in ([0, K], [0, 100, 612, K]):
        S = len(kseg) - 1
        layer = sq.Layer(4, K, N, kseg, [0, N], [0] * S)
        wd = _bf16_dev(g, wm) if w_dtype == "bf16" else torch.from_numpy(wm).to(g.DEV)
        wq = torch.full((N, K), 0x7F, dtype=torch.uint8, device=g.DEV)
        ws = torch.full((S, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_weight_fp8(layer, wd, wq, ws)
        torch.cuda.synchronize()
        r_wq, r_ws = oracle.quantize_weight_fp8(wm, kseg)
        assert np.array_equal(ws.cpu().numpy().view(np.uint32), r_ws.view(np.uint32))
        assert np.array_equal(wq.cpu().numpy(), _plus_zero(r_wq))
    assert r_ws[0, 1] == 1.0


@pytest.mark.parametrize("case", [
    dict(M=9, K=64, kseg=[0, 64], dual=[1], x_dtype="bf16"),
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[0, 1], x_dtype="f32"),
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 1], x_dtype="bf16"),        # unaligned: element-wise kernel
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 0], x_dtype="f32"),
    dict(M=300, K=2048, kseg=[0, 2048], dual=[0], x_dtype="bf16"),
    dict(M=129, K=1024, kseg=[0, 16, 32, 48, 1024], dual=[1, 0, 1, 1], x_dtype="bf16"),
])
@pytest.mark.parametrize("scales", ["amax", "pow2", "clip"])
def test_quantize_act_fp8(oracle, case, scales):
    import torch

    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], 4, case["kseg"], [0, 4], case["dual"], seed=case["K"] + case["M"],
                        x_dtype=case["x_dtype"], act="gelu")
    S = w.S
    w.s_pos = (w.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)      # the calibrated ranges over 448
    w.s_neg = (w.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
    if scales == "pow2":      # exact quotients, many of them ties of the 3-bit mantissa
        w.x = np.round(w.x * 64).astype(np.float32) / 64
        w.s_pos = np.full(S, 2.0 ** -5, np.float32)
        w.s_neg = np.full(S, 2.0 ** -8, np.float32)
    elif scales == "clip":    # steps far too small: saturation at +-448
        w.s_pos = (w.s_pos / 50).astype(np.float32)
        w.s_neg = (w.s_neg / 50).astype(np.float32)
    w.x[0, 0] = -0.0
    gl = g.GpuLayer(w)
    xq = torch.full((w.M, w.K), 0x7F, dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
    torch.cuda.synchronize()
    r_xp, r_xn = oracle.quantize_act_fp8(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    xp, xn = _split_fp8(w, xq.cpu().numpy())
    assert np.array_equal(xp, _plus_zero(r_xp)) and np.array_equal(xn, _plus_zero(r_xn))
    if scales == "clip":
        assert (xp == 0x7E).any()


@pytest.mark.parametrize("case", [
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[0, 1], act=[0, 2], x_dtype="bf16"),
    dict(M=33, K=1024, kseg=[0, 1024], dual=[1], act=[1], x_dtype="f32"),
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 1], act=[2, 1], x_dtype="bf16"),      # unaligned: element-wise kernel
    dict(M=300, K=2048, kseg=[0, 512, 2048], dual=[1, 0], act=[1, 0], x_dtype="bf16"),
])
def test_quantize_act_fp8_fused(oracle, case):
    """Q_dual(act(h)) with fp8 codes in one pass: bit-exact against the oracle's activation followed by its fp8 quantizer."""
    import torch

    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], 4, case["kseg"], [0, 4], case["dual"], seed=case["K"] + case["M"],
                        x_dtype=case["x_dtype"], act="normal")
    w.x = (w.x * np.float32(2.0)).astype(np.float32)
    if case["x_dtype"] == "bf16":
        w.x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.x))
    a = oracle.activation(w.x, case["kseg"], case["act"])
    sp, sn, _, _ = oracle.calibrate_act(a, case["kseg"], case["dual"])
    w.s_pos = (sp * np.float32(127.0 / 448.0)).astype(np.float32)
    w.s_neg = (sn * np.float32(127.0 / 448.0)).astype(np.float32)
    gl = g.GpuLayer(w)
    xq = torch.full((w.M, w.K), 0x7F, dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_act_fp8_fused(gl.layer, gl.x, case["act"], xq)
    torch.cuda.synchronize()
    r_xp, r_xn = oracle.quantize_act_fp8_fused(w.x, w.kseg_off, w.dual, case["act"], w.s_pos, w.s_neg)
    xp, xn = _split_fp8(w, xq.cpu().numpy())
    assert np.array_equal(xp, _plus_zero(r_xp)) and np.array_equal(xn, _plus_zero(r_xn))
    # with a workspace (bf16 inputs: code tables in LDS): the same codes
    ws = torch.full((sq.sq_quantize_act_fused_workspace_bytes(gl.layer),), 0xA5, dtype=torch.uint8, device=g.DEV)
    xq_t = torch.full_like(xq, 0x7F)
    sq.sq_quantize_act_fp8_fused(gl.layer, gl.x, case["act"], xq_t, ws)
    torch.cuda.synchronize()
    assert torch.equal(xq_t, xq)
    # all-none codes: the plain quantizer
    xq2 = torch.empty_like(xq)
    xq3 = torch.empty_like(xq)
    sq.sq_quantize_act_fp8_fused(gl.layer, gl.x, [0] * w.S, xq2)
    sq.sq_quantize_act_fp8(gl.layer, gl.x, xq3)
    torch.cuda.synchronize()
    assert torch.equal(xq2, xq3)


FP8GEMM = [
    dict(M=300, K=512, N=200, kseg=[0, 128, 512], nseg=[0, 200], dual=[1, 0], bias=True),
    dict(M=128, K=1152, N=256, kseg=[0, 1152], nseg=[0, 256], dual=[1], bias=False),
    dict(M=5, K=128, N=3, kseg=[0, 128], nseg=[0, 3], dual=[0], bias=True),              # one stage, mostly masked tile
    dict(M=257, K=1536, N=385, kseg=[0, 256, 384, 1536], nseg=[0, 129, 385], dual=[0, 1, 1], bias=True, seg_scale=True),
    dict(M=1024, K=4608, N=1152, kseg=[0, 1536, 4608], nseg=[0, 1152], dual=[0, 1], bias=True),
    # skinny layers: the weight-stream kernel on fp8 codes (two slab planes / one plane, one to four 16-row tiles)
    dict(M=16, K=1152, N=640, kseg=[0, 1152], nseg=[0, 640], dual=[1], bias=True),
    dict(M=40, K=512, N=200, kseg=[0, 128, 512], nseg=[0, 200], dual=[1, 0], bias=False),
    dict(M=64, K=2304, N=1157, kseg=[0, 1024, 1152, 2304], nseg=[0, 500, 1157], dual=[0, 1, 1], bias=True, seg_scale=True),
    dict(M=31, K=256, N=7000, kseg=[0, 256], nseg=[0, 7000], dual=[0], bias=True),      # more column groups than waves
]


def _fp8_tol(K, mag, ref, ydt):
    """Error of the device's evaluation around the double-precision oracle.  The fp8 matrix instruction adds the eight
    products of every aligned group of eight k after aligning them to the group's largest exponent sum E and dropping
    the bits below 2^(E - 13) (measured: a product 2^14 below the largest one of its group vanishes, one in another group
    of the same instruction does not), so a group loses less than 8 * 2^(E - 13) <= 2^-10 of its largest product and an
    output less than 2^-10 of the sum of its terms' magnitudes, `mag`; the sums across groups, K-segments and the
    dequantization are fp32 (second term); then the output rounding."""
    return (2.0 ** -10 + (8.0 * np.sqrt(K) + 64.0) * 2.0 ** -24) * mag + np.abs(ref) * (2.0 ** -8 if ydt == "bf16" else 2.0 ** -23) + 1e-30


@pytest.mark.parametrize("case", FP8GEMM)
def test_seglinear_fp8(oracle, case):
    """The fp8 layer end to end on every element: codes and steps bit-exact, outputs within the bound of an fp32
    evaluation around the double-precision oracle, fp32 and bf16 outputs."""
    import torch

    g = _gpu()
    M, K, N = case["M"], case["K"], case["N"]
    w = wl.random_layer(M, K, N, case["kseg"], case["nseg"], case["dual"], seed=M + K + N, x_dtype="bf16", act="silu",
                        with_bias=case["bias"], with_seg_scale=case.get("seg_scale", False))
    w.s_pos = (w.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)
    w.s_neg = (w.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
    gl = g.GpuLayer(w)
    wq = torch.full((N, K), 0x7F, dtype=torch.uint8, device=g.DEV)
    xq = torch.full((M, K), 0x7F, dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_weight_fp8(gl.layer, gl.wt, wq, gl.wscale)
    sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
    torch.cuda.synchronize()
    r_wq, r_ws = oracle.quantize_weight_fp8(w.w, w.kseg_off)
    r_xp, r_xn = oracle.quantize_act_fp8(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    assert np.array_equal(wq.cpu().numpy(), _plus_zero(r_wq))
    assert np.array_equal(gl.wscale.cpu().numpy().view(np.uint32), r_ws.view(np.uint32))
    xp, xn = _split_fp8(w, xq.cpu().numpy())
    assert np.array_equal(xp, _plus_zero(r_xp)) and np.array_equal(xn, _plus_zero(r_xn))
    ref, mag = oracle.seglinear_fp8(r_xp, r_xn, r_wq, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, r_ws, w.seg_scale, w.bias)
    # automatic choice, the plain tile kernel, and every tile configuration of the pipelined kernel built for fp8 codes
    ran = 0
    for path, variant in [(-1, -1), (0, -1), (3, -1)] + [(1, v) for v in range(9)]:
        sq.sq_tuning_set("force_path", path)
        sq.sq_tuning_set("gemm_variant", variant)
        for ydt in ("f32", "bf16"):
            y = torch.full((M, N), float("nan"), dtype=torch.bfloat16 if ydt == "bf16" else torch.float32, device=g.DEV)
            try:
                sq.sq_seglinear_fp8(gl.layer, xq, wq, gl.wscale, gl.bias, y)
            except sq.SqError:
                assert variant >= 0 or path == 3   # a tile configuration that does not serve this layer class; no room for the X^ slab
                continue
            torch.cuda.synchronize()
            ran += 1
            got = y.float().cpu().numpy().astype(np.float64)
            assert not np.isnan(got).any(), (path, variant)
            tol = _fp8_tol(K, mag, ref, ydt)
            assert (np.abs(got - ref) <= tol).all(), (path, variant, float((np.abs(got - ref) / tol).max()))
            if ydt == "f32":          # the typical error is far inside the bound
                assert np.abs(got - ref).max() <= 5e-5 * np.abs(ref).max(), (path, variant)
    assert ran >= 8
    # the variant does its job: close to the unquantized layer (3 mantissa bits: a few percent)
    if w.seg_scale is None:
        full = w.x.astype(np.float64) @ w.w.astype(np.float64).T + (0.0 if w.bias is None else w.bias)
        assert np.linalg.norm(ref - full) < 0.06 * np.linalg.norm(full)


def test_seglinear_fp8_exact_sums_and_polarity(oracle):
    """Codes of small integers and steps that are powers of two: every product is an integer within 2^13 of the largest
    one (the window the matrix instruction keeps inside a group of eight) and every partial sum an integer below 2^24, so
    the device's evaluation is exact in any order and the output must equal the oracle's to the bit; the dual K-segment has
    both polarities in every row."""
    import torch

    g = _gpu()
    M, K, N = 200, 640, 136
    kseg, dual = [0, 256, 640], [1, 0]
    rng = np.random.default_rng(9)
    xi = rng.integers(-8, 9, size=(M, K)).astype(np.float32)
    wi = rng.integers(-8, 9, size=(N, K)).astype(np.float32)
    wi[:, 0] = 448.0                                        # weight steps of exactly 1 in the first K-segment
    wi[:, 300] = -448.0
    s_pos, s_neg = np.float32([0.5, 2.0]), np.float32([0.25, 1.0])
    x = xi.copy()
    x[:, :256] *= np.where(xi[:, :256] < 0, s_neg[0], s_pos[0])
    x[:, 256:] *= s_pos[1]
    layer = sq.Layer(M, K, N, kseg, [0, N], dual, s_pos, s_neg)
    xq = torch.empty((M, K), dtype=torch.uint8, device=g.DEV)
    wq = torch.empty((N, K), dtype=torch.uint8, device=g.DEV)
    ws = torch.empty((2, N), dtype=torch.float32, device=g.DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight_fp8(layer, torch.from_numpy(wi).to(g.DEV), wq, ws)
    sq.sq_quantize_act_fp8(layer, torch.from_numpy(x).to(g.DEV), xq)
    sq.sq_seglinear_fp8(layer, xq, wq, ws, None, y)
    torch.cuda.synchronize()
    r_wq, r_ws = oracle.quantize_weight_fp8(wi, kseg)
    r_xp, r_xn = oracle.quantize_act_fp8(x, kseg, dual, s_pos, s_neg)
    assert (r_ws == 1.0).all()
    ref, _ = oracle.seglinear_fp8(r_xp, r_xn, r_wq, kseg, [0, N], dual, s_pos, s_neg, r_ws)
    assert np.array_equal(y.cpu().numpy().astype(np.float64), ref)
    # and the plain definition on the integers themselves
    plain = (x.astype(np.float64) @ wi.astype(np.float64).T)
    assert np.array_equal(ref, plain)


def test_fp8_products_far_below_the_largest_of_their_group(oracle):
    """The case the tolerance is derived from: one product of 2^17.6 next to 127 products of 2^-j.  Inside its group of
    eight the matrix instruction drops what lies 2^14 below the largest product, elsewhere the sum is fp32: the output
    stays within the derived bound of the double-precision value, and the plain and the pipelined kernel (same
    instruction, same groups) agree to the bit."""
    import torch

    g = _gpu()
    M, K, N = 32, 128, 32
    one = np.ones(1, np.float32)
    layer = sq.Layer(M, K, N, [0, K], [0, N], [0], one, one)
    for j in range(10):
        t = np.float32(2.0 ** -j)
        xv = np.full((M, K), t, np.float32)
        wv = np.ones((N, K), np.float32)
        xv[:, 0] = 448.0
        wv[:, 0] = 448.0
        xq, wq = oracle.fp8_encode(xv), oracle.fp8_encode(wv)
        ref, mag = oracle.seglinear_fp8(xq, np.zeros_like(xq), wq, [0, K], [0, N], [0], one, one, np.ones((1, N), np.float32))
        assert ref[0, 0] == 448.0 * 448.0 + 127 * float(t)
        outs = []
        for path in (0, -1):
            sq.sq_tuning_set("force_path", path)
            y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
            sq.sq_seglinear_fp8(layer, torch.from_numpy(xq).to(g.DEV), torch.from_numpy(wq).to(g.DEV),
                                torch.ones((1, N), dtype=torch.float32, device=g.DEV), None, y)
            torch.cuda.synchronize()
            outs.append(y.cpu().numpy())
        assert np.array_equal(outs[0], outs[1])
        err = np.abs(outs[0].astype(np.float64) - ref)
        assert (err <= _fp8_tol(K, mag, ref, "f32")).all()
        assert (err <= 8 * float(t)).all()          # at most the seven neighbours of the large product (and fp32 rounding)


def test_seglinear_fp8_rejects_unaligned_layouts():
    import torch

    g = _gpu()
    for K, kseg in ((192, [0, 192]), (256, [0, 64, 256])):
        layer = sq.Layer(4, K, 8, kseg, [0, 8], [0] * (len(kseg) - 1), np.ones(len(kseg) - 1, np.float32), np.ones(len(kseg) - 1, np.float32))
        xq = torch.zeros((4, K), dtype=torch.uint8, device=g.DEV)
        wq = torch.zeros((8, K), dtype=torch.uint8, device=g.DEV)
        ws = torch.ones((len(kseg) - 1, 8), dtype=torch.float32, device=g.DEV)
        y = torch.zeros((4, 8), dtype=torch.float32, device=g.DEV)
        with pytest.raises(sq.SqError):
            sq.sq_seglinear_fp8(layer, xq, wq, ws, None, y)


GENERIC = [
    dict(M=7, K=100, N=13, kseg=[0, 37, 100], nseg=[0, 5, 13], dual=[1, 0]),
    dict(M=70, K=96, N=65, kseg=[0, 96], nseg=[0, 65], dual=[1]),
    dict(M=3, K=1, N=2, kseg=[0, 1], nseg=[0, 2], dual=[1]),
]


@pytest.mark.parametrize("case", GENERIC)
def test_seglinear_generic_small(oracle, case):
    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], case["N"], case["kseg"], case["nseg"], case["dual"],
                        seed=case["K"] + 5, x_dtype="f32", act="silu", with_seg_scale=True, with_bias=True)
    _check_layer(oracle, g, w, path=-1)


def test_many_segments(oracle):
    """Head-merge style input segmentation: 24 K-segments of 64, alternating dual flags; 6 N-segments."""
    g = _gpu()
    kseg = [64 * i for i in range(25)]
    w = wl.random_layer(150, 1536, 192, kseg, [32 * i for i in range(7)], [i % 2 for i in range(24)], seed=77,
                        x_dtype="bf16", act="silu", with_seg_scale=True)
    _check_layer(oracle, g, w, path=1, variant=6)
    _check_layer(oracle, g, w, path=-1)
    w2 = wl.random_layer(150, 3072, 192, [128 * i for i in range(25)], [32 * i for i in range(7)],
                         [i % 2 for i in range(24)], seed=78, x_dtype="bf16", act="silu", with_seg_scale=True)
    _check_layer(oracle, g, w2, path=1, variant=1)
    _check_layer(oracle, g, w2, path=1, variant=5)


def test_saturated_accumulators(oracle):
    """All codes at +-127 over a 4096-long segment: |acc| = 127*127*4096 = 6.6e7, well inside int32."""
    g = _gpu()
    w = wl.random_layer(40, 4096, 64, [0, 4096], [0, 64], [1], seed=5, x_dtype="bf16", act="normal")
    w.x = np.where(w.x >= 0, 8.0, -8.0).astype(np.float32)
    w.w = np.where(w.w >= 0, 1.0, -1.0).astype(np.float32)
    w.s_pos = np.array([8.0 / 127], np.float32)
    w.s_neg = np.array([8.0 / 127], np.float32)
    # outputs are multiples of one constant here, so a large share sits exactly on bf16 rounding ties:
    # the "rare mismatch" rule for bf16 does not apply; fp32 and the integers are checked.
    out = _check_layer(oracle, g, w, path=1, variant=0, y_dtypes=("f32",))
    assert out is not None


# ----------------------------------------------------------------------------------------------------
# the five named configurations at full size, in the launch configuration the benchmark times
# ----------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg4d", "cfg5"])
def test_named_configs(oracle, name):
    """Every element of every named configuration: codes, weight steps, both int32 accumulator sets of every K-segment,
    fp32 and bf16 outputs, against the oracle's full matrices."""
    g = _gpu()
    w = wl.make(name)
    out = _check_layer(oracle, g, w, path=-1)
    print(name, out)


@pytest.mark.parametrize("name", ["cfg2", "cfg4d", "cfg5"])
def test_named_configs_per_token_steps(oracle, name):
    """The same layers with dynamic per-token activation steps (App. B, 4-bit settings), every element: codes and
    steps bit-exact, outputs of the tile kernel's per-token instantiation within the fp32 tolerance."""
    import torch

    g = _gpu()
    w = wl.make(name)
    gl = g.GpuLayer(w)
    gl.quantize_weight()
    tok = torch.full((2, w.M, w.S), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_act_dynamic(gl.layer, gl.x, gl.xq, tok)
    torch.cuda.synchronize()
    r = oracle.seglinear_dynamic(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.seg_scale, w.bias, wbits=8)
    xp, xn = g.split_codes(w, gl.xq.cpu().numpy())
    assert np.array_equal(xp, r.xq_pos) and np.array_equal(xn, r.xq_neg)
    assert np.array_equal(tok.cpu().numpy().view(np.uint32), r.tok_steps.view(np.uint32))
    ymax = float(np.abs(r.y32).max())
    y = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_seglinear_dynamic(gl.layer, gl.xq, tok, gl.wq, 8, gl.wscale, gl.bias, y)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert not np.isnan(y).any()
    assert float(np.abs(y.astype(np.float64) - r.y32.astype(np.float64)).max()) <= RTOL * ymax
    yb = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=g.DEV)
    sq.sq_seglinear_dynamic(gl.layer, gl.xq, tok, gl.wq, 8, gl.wscale, gl.bias, yb)
    torch.cuda.synchronize()
    g.check_bf16_against(g.bf16_tensor_bits(yb), r.y32, wl.f32_to_bf16_bits(r.y32), RTOL * ymax)


# Several rounds of tiles per persistent workgroup (more tiles than the chip has compute units), every element:
# the load pipeline then runs across tile boundaries.  Two K-segments; `dual` picks the register-sharing
# instantiation (one dual segment) or the one with a separate fp32 running sum (two dual segments).
MULTIROUND = [
    dict(M=4096, K=512, N=2560, kseg=[0, 256, 512], dual=[0, 1], variant=1),     # 640 tiles of 128 x 128, shared registers
    dict(M=4096, K=512, N=2560, kseg=[0, 256, 512], dual=[1, 1], variant=1),     # separate running sum
    dict(M=4100, K=384, N=2570, kseg=[0, 128, 384], dual=[1, 0], variant=0),     # 128 x 256 tiles, ragged edges, shared registers
    dict(M=4100, K=384, N=2570, kseg=[0, 384], dual=[1], variant=3),             # 64 x 128 tiles: 1365 tiles, five rounds
    dict(M=4100, K=256, N=2570, kseg=[0, 256], dual=[0], variant=4),             # 256 x 256 single path
]


@pytest.mark.parametrize("case", MULTIROUND)
def test_seglinear_mfma_many_tiles(oracle, case):
    g = _gpu()
    w = wl.random_layer(case["M"], case["K"], case["N"], case["kseg"], [0, case["N"] // 2, case["N"]], case["dual"],
                        seed=case["M"] + case["K"] + 3 * case["variant"], x_dtype="bf16", act="gelu", with_seg_scale=True,
                        with_bias=True)
    _check_layer(oracle, g, w, path=1, variant=case["variant"])


def test_headline_config_calibration_and_fused_quantizer(oracle):
    """The entry points beyond the hot path, at the headline layer's full size (cfg5: 4608 x 15360 bf16, a plain
    K-segment and a dual one), in the launch configuration the benchmark times: min/max steps against the oracle,
    percentile thresholds through the counting definition of a quantile (valid at any size), and the fused
    GELU + quantizer (table path and per-element path) against the oracle on sampled token rows."""
    import torch

    g = _gpu()
    w = wl.make("cfg5")
    M, K, S = w.M, w.K, w.S
    xd = torch.from_numpy(wl.f32_to_bf16_bits(w.x).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    layer = sq.Layer.from_workload(w)
    amax = torch.empty((2, S), dtype=torch.float32, device=g.DEV)
    steps = torch.empty((2, S), dtype=torch.float32, device=g.DEV)
    sq.sq_calibrate_act(layer, xd, amax, steps)
    r = oracle.calibrate_act(w.x, w.kseg_off, w.dual)
    torch.cuda.synchronize()
    assert np.array_equal(steps.cpu().numpy().view(np.uint32), np.stack([r[0], r[1]]).view(np.uint32))
    # percentile clipping
    ws = torch.empty((sq.sq_calibrate_workspace_bytes(),), dtype=torch.uint8, device=g.DEV)
    p = 0.9999
    sq.sq_calibrate_act_percentile(layer, xd, p, amax, steps, ws)
    torch.cuda.synchronize()
    thr = amax.cpu().numpy()
    for ks in range(S):
        blk = w.x[:, w.kseg_off[ks]:w.kseg_off[ks + 1]]
        n = blk.size
        k = min(max(int(np.ceil(p * n)), 1), n)
        pops = [(np.maximum(blk, 0), thr[0, ks]), (np.maximum(-blk, 0), thr[1, ks])] if w.dual[ks] else [(np.abs(blk), thr[0, ks])]
        for v, t in pops:
            assert np.count_nonzero(v <= t) >= k and np.count_nonzero(v < t) < k, (ks, float(t))
        if not w.dual[ks]:
            assert thr[1, ks] == 0.0
    # fused GELU + quantizer on the dual segment, steps from the activation's own range
    rng = np.random.default_rng(11)
    h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((rng.standard_normal((M, K)) * 1.5).astype(np.float32)))
    hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    act = [sq.SQ_ACT_GELU if d else sq.SQ_ACT_NONE for d in w.dual]
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(M - 4, M), rng.integers(0, M, 24)]))
    a_s = oracle.activation(h[rows], w.kseg_off, act)
    sp, sn, _, _ = oracle.calibrate_act(a_s, w.kseg_off, w.dual)
    lay = sq.Layer(M, K, w.N, w.kseg_off, w.nseg_off, w.dual, sp, sn)
    rp, rn = oracle.quantize_act_fused(h[rows], w.kseg_off, w.dual, act, sp, sn)
    want = (rp.astype(np.int16) + rn.astype(np.int16)).astype(np.int8)
    fws = torch.empty((sq.sq_quantize_act_fused_workspace_bytes(lay),), dtype=torch.uint8, device=g.DEV)
    xq_t = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
    xq_e = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_fused(lay, hd, act, xq_t, workspace=fws)
    sq.sq_quantize_act_fused(lay, hd, act, xq_e)
    torch.cuda.synchronize()
    assert torch.equal(xq_t, xq_e)                                   # the two device paths agree everywhere
    assert np.array_equal(xq_t.cpu().numpy()[rows], want)            # and with the oracle on the sampled rows


# ----------------------------------------------------------------------------------------------------
# 4-bit packed weights (skinny layers)
# ----------------------------------------------------------------------------------------------------
W4CASES = [
    dict(M=16, K=1152, N=6912, kseg=[0, 1152], dual=[1], nseg=None),                       # cfg3's shape
    dict(M=5, K=256, N=70, kseg=[0, 128, 256], dual=[0, 1], nseg=None, bias=True),         # ragged N, mixed segments
    dict(M=40, K=512, N=200, kseg=[0, 384, 512], dual=[1, 1], nseg=[0, 64, 200], seg_scale=True),   # three row tiles
    dict(M=64, K=1152, N=1000, kseg=[0, 1152], dual=[1], nseg=None),                       # the large activation slab
    dict(M=100, K=256, N=96, kseg=[0, 256], dual=[1], nseg=None),                          # M > 64: plain kernel
    dict(M=1, K=128, N=16, kseg=[0, 128], dual=[0], nseg=None),
    dict(M=300, K=640, N=330, kseg=[0, 256, 640], dual=[1, 0], nseg=None, bias=True),      # many token rows, ragged last group
]


@pytest.mark.parametrize("case", W4CASES)
@pytest.mark.parametrize("force_plain", [False, True])
def test_seglinear_w4(oracle, case, force_plain):
    """4-bit weight quantizer + packed storage bit-exact; integer sums bit-exact; output within the fp32 tolerance."""
    import torch

    g = _gpu()
    M, K, N = case["M"], case["K"], case["N"]
    nseg = case["nseg"] or [0, N]
    w = wl.random_layer(M, K, N, case["kseg"], nseg, case["dual"], seed=3 * M + K + N, x_dtype="bf16", act="silu",
                        with_seg_scale=bool(case.get("seg_scale")), with_bias=bool(case.get("bias")))
    gl = g.GpuLayer(w)
    wq4 = torch.full((((N + 15) // 16) * 16 * (K // 2),), 0xAB, dtype=torch.uint8, device=g.DEV)
    sq.sq_quantize_weight_w4(gl.layer, gl.wt, wq4, gl.wscale)
    rq, rs = oracle.quantize_weight_w4(w.w, w.kseg_off)
    torch.cuda.synchronize()
    assert np.array_equal(wq4.cpu().numpy(), oracle.pack_w4(rq))
    assert np.array_equal(gl.wscale.cpu().numpy().view(np.uint32), rs.view(np.uint32))
    xp, xn, _ = gl.quantize_act()
    r = oracle.seglinear(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, w.seg_scale, w.bias, wbits=4)
    assert np.array_equal(xp, r.xq_pos) and np.array_equal(xn, r.xq_neg)
    sq.sq_tuning_set("force_path", 0 if force_plain else -1)
    try:
        ap = torch.full((w.S, M, N), 0x5A5A5A5A, dtype=torch.int32, device=g.DEV)
        an = torch.full((w.S, M, N), 0x5A5A5A5A, dtype=torch.int32, device=g.DEV)
        sq.sq_seglinear_w4_debug_acc(gl.layer, gl.xq, wq4, ap, an)
        torch.cuda.synchronize()
        assert np.array_equal(ap.cpu().numpy(), r.acc_pos), "acc_pos differs"
        assert np.array_equal(an.cpu().numpy(), r.acc_neg), "acc_neg differs"
        ymax = float(np.abs(r.y32).max())
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_seglinear_w4(gl.layer, gl.xq, wq4, gl.wscale, gl.bias, y)
        torch.cuda.synchronize()
        y = y.cpu().numpy()
        assert not np.isnan(y).any()
        assert float(np.abs(y.astype(np.float64) - r.y32.astype(np.float64)).max()) <= 1e-5 * ymax
        assert float(np.abs(y.astype(np.float64) - r.y64).max()) <= 2e-5 * ymax
        yb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=g.DEV)
        sq.sq_seglinear_w4(gl.layer, gl.xq, wq4, gl.wscale, gl.bias, yb)
        torch.cuda.synchronize()
        g.check_bf16_against(g.bf16_tensor_bits(yb), r.y32, wl.f32_to_bf16_bits(r.y32), 1e-5 * ymax)
        # unpacked to one code per byte: the oracle's 4-bit codes exactly, and the int8 entry point (whatever kernel it
        # picks for this shape) gives the 4-bit layer's output with the same scales
        wq8 = torch.full((N, K), 99, dtype=torch.int8, device=g.DEV)
        sq.sq_unpack_w4(gl.layer, wq4, wq8)
        torch.cuda.synchronize()
        assert np.array_equal(wq8.cpu().numpy(), rq)
        y8 = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_seglinear(gl.layer, gl.xq, wq8, gl.wscale, gl.bias, y8)
        torch.cuda.synchronize()
        assert float(np.abs(y8.cpu().numpy().astype(np.float64) - r.y32.astype(np.float64)).max()) <= 1e-5 * ymax
    finally:
        sq.sq_tuning_set("force_path", -1)


def test_w4_rejects_unaligned_layouts():
    import torch

    g = _gpu()
    lay = sq.Layer(4, 192, 16, [0, 192], [0, 16], [1], [0.01], [0.01])      # K not a multiple of 128
    t = torch.zeros(4096, dtype=torch.uint8, device=g.DEV)
    f = torch.zeros(4096, dtype=torch.float32, device=g.DEV)
    with pytest.raises(sq.SqError):
        sq.sq_quantize_weight_w4(lay, f, t, f)
    lay2 = sq.Layer(4, 256, 16, [0, 64, 256], [0, 16], [1, 0], [0.01, 0.01], [0.01, 0.01])   # boundary at 64
    with pytest.raises(sq.SqError):
        sq.sq_seglinear_w4(lay2, t.view(torch.int8), t, f, None, f)


# ----------------------------------------------------------------------------------------------------
# dynamic per-token activation steps
# ----------------------------------------------------------------------------------------------------
DYNCASES = [
    dict(M=16, K=1152, N=6912, kseg=[0, 1152], dual=[1], x_dtype="bf16"),
    dict(M=5, K=256, N=70, kseg=[0, 128, 256], dual=[0, 1], x_dtype="f32", bias=True),
    dict(M=40, K=512, N=200, kseg=[0, 384, 512], dual=[1, 1], nseg=[0, 64, 200], seg_scale=True, x_dtype="bf16"),
    dict(M=100, K=256, N=96, kseg=[0, 256], dual=[1], x_dtype="bf16"),                      # M > 64: plain kernel
    dict(M=7, K=100, N=33, kseg=[0, 37, 100], dual=[1, 0], x_dtype="f32", bits=(8,)),       # unaligned: plain kernel, 8-bit only
    # large M, 8-bit weights: the MFMA tile kernel with per-row steps (4-bit weights: plain kernel)
    dict(M=300, K=512, N=520, kseg=[0, 256, 512], dual=[0, 1], x_dtype="bf16", bias=True),  # one dual segment: shared registers
    dict(M=257, K=384, N=130, kseg=[0, 128, 384], dual=[1, 1], x_dtype="f32", bits=(8,)),   # two dual segments, ragged tiles
    dict(M=200, K=256, N=256, kseg=[0, 256], dual=[0], x_dtype="bf16", bits=(8,)),          # single path
    dict(M=150, K=256, N=192, kseg=[0, 128, 256], dual=[0, 0], nseg=[0, 64, 192], seg_scale=True, x_dtype="bf16", bits=(8,)),
    # long rows: two, four and eight chunks per thread in the row-resident quantizer
    dict(M=3, K=4608, N=16, kseg=[0, 4608], dual=[1], x_dtype="f32", bits=(8,)),
    dict(M=5, K=9216, N=16, kseg=[0, 1024, 9216], dual=[1, 0], x_dtype="bf16", bits=(8,)),
    dict(M=2, K=20480, N=16, kseg=[0, 4096, 20480], dual=[0, 1], x_dtype="bf16", bits=(8,)),
    dict(M=2, K=17408, N=16, kseg=[0, 17408], dual=[1], x_dtype="f32", bits=(8,)),
]


@pytest.mark.parametrize("case", DYNCASES)
def test_seglinear_dynamic(oracle, case):
    """Per-token steps: codes and steps bit-exact against the oracle, outputs within the fp32 tolerance, for 8-bit and
    4-bit weights."""
    import torch

    g = _gpu()
    M, K, N = case["M"], case["K"], case["N"]
    nseg = case.get("nseg") or [0, N]
    w = wl.random_layer(M, K, N, case["kseg"], nseg, case["dual"], seed=5 * M + K + N, x_dtype=case["x_dtype"], act="gelu",
                        with_seg_scale=bool(case.get("seg_scale")), with_bias=bool(case.get("bias")))
    w.x = (w.x * np.random.default_rng(M).uniform(0.1, 8.0, size=(M, 1))).astype(np.float32)   # tokens of different scale
    if case["x_dtype"] == "bf16":
        w.x = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(w.x))
    gl = g.GpuLayer(w)
    S = w.S
    tok = torch.full((2, M, S), float("nan"), dtype=torch.float32, device=g.DEV)
    # 4-bit activation codes first (the W4A4 setting): codes and steps bit-exact, the layer through the same GEMM
    xq4 = torch.full((M, K), 99, dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_dynamic_bits(gl.layer, gl.x, 4, xq4, tok)
    torch.cuda.synchronize()
    r4 = oracle.seglinear_dynamic(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.seg_scale, w.bias, wbits=8, abits=4)
    xp4, xn4 = g.split_codes(w, xq4.cpu().numpy())
    assert np.array_equal(xp4, r4.xq_pos) and np.array_equal(xn4, r4.xq_neg) and np.abs(xq4.cpu().numpy()).max() == 7
    assert np.array_equal(tok.cpu().numpy().view(np.uint32), r4.tok_steps.view(np.uint32))
    gl.quantize_weight()
    y4 = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_seglinear_dynamic(gl.layer, xq4, tok, gl.wq, 8, gl.wscale, gl.bias, y4)
    torch.cuda.synchronize()
    assert float(np.abs(y4.cpu().numpy().astype(np.float64) - r4.y32.astype(np.float64)).max()) <= 1e-5 * float(np.abs(r4.y32).max())
    sq.sq_quantize_act_dynamic(gl.layer, gl.x, gl.xq, tok)
    torch.cuda.synchronize()
    for bits in case.get("bits", (8, 4)):
        r = oracle.seglinear_dynamic(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.seg_scale, w.bias, wbits=bits)
        xp, xn = g.split_codes(w, gl.xq.cpu().numpy())
        assert np.array_equal(xp, r.xq_pos) and np.array_equal(xn, r.xq_neg)
        assert np.array_equal(tok.cpu().numpy().view(np.uint32), r.tok_steps.view(np.uint32))
        if bits == 8:
            wq, _ = gl.quantize_weight()
            wdev = gl.wq
        else:
            wdev = torch.empty((((N + 15) // 16) * 16 * (K // 2),), dtype=torch.uint8, device=g.DEV)
            sq.sq_quantize_weight_w4(gl.layer, gl.wt, wdev, gl.wscale)
        ymax = float(np.abs(r.y32).max())
        runs = [(-1, -1), (0, -1)] + ([(1, v) for v in (0, 1, 3, 7, 8)] if bits == 8 and M > 64 else [])
        for forced, variant in runs:
            sq.sq_tuning_set("force_path", forced)
            sq.sq_tuning_set("gemm_variant", variant)
            try:
                y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
                try:
                    sq.sq_seglinear_dynamic(gl.layer, gl.xq, tok, wdev, bits, gl.wscale, gl.bias, y)
                except sq.SqError as e:
                    assert e.status == 2 and variant >= 0          # a tile shape that does not take this layer class
                    continue
                torch.cuda.synchronize()
                y = y.cpu().numpy()
                assert not np.isnan(y).any()
                assert float(np.abs(y.astype(np.float64) - r.y32.astype(np.float64)).max()) <= 1e-5 * ymax, (bits, forced)
                yb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=g.DEV)
                sq.sq_seglinear_dynamic(gl.layer, gl.xq, tok, wdev, bits, gl.wscale, gl.bias, yb)
                torch.cuda.synchronize()
                g.check_bf16_against(g.bf16_tensor_bits(yb), r.y32, wl.f32_to_bf16_bits(r.y32), 1e-5 * ymax)
            finally:
                sq.sq_tuning_set("force_path", -1)
                sq.sq_tuning_set("gemm_variant", -1)


FUSEDGEMM = [
    dict(M=16, K=1152, N=6912, kseg=[0, 1152], dual=[1], act=[1], h_dtype="bf16", L=3),       # adaLN: Linear(SiLU(c))
    dict(M=5, K=256, N=33, kseg=[0, 128, 256], dual=[1, 0], act=[2, 0], h_dtype="f32", L=2),    # ragged N, mixed segments
    dict(M=33, K=384, N=100, kseg=[0, 384], dual=[0], act=[2], h_dtype="bf16", L=0),           # three row tiles: single only
    dict(M=1, K=128, N=16, kseg=[0, 128], dual=[1], act=[0], h_dtype="f32", L=1),               # no activation
    dict(M=32, K=640, N=4240, kseg=[0, 256, 640], dual=[1, 1], act=[1, 2], h_dtype="bf16", L=9),
    dict(M=64, K=1152, N=520, kseg=[0, 1152], dual=[1], act=[1], h_dtype="f32", L=0),          # four row tiles
]


@pytest.mark.parametrize("case", FUSEDGEMM)
def test_seglinear_fused(oracle, case):
    """Raw activations in, y out, one launch: activation, polarity split and quantizers inside the weight-stream kernel.
    Against the oracle (activation -> Q_dual -> SegLinear) to the fp32 bar, and bit for bit against the two-launch path."""
    import torch

    g = _gpu()
    M, K, N = case["M"], case["K"], case["N"]
    rng = np.random.default_rng(M * 7 + K + N)
    h = (rng.standard_normal((M, K)) * 3.0).astype(np.float32)
    h[0, :4] = [0.0, -0.0, 95.0, -95.0]
    if case["h_dtype"] == "bf16":
        h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(h))
        hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        hd = torch.from_numpy(h).to(g.DEV)
    a = oracle.activation(h, case["kseg"], case["act"])
    sp, sn, _, _ = oracle.calibrate_act(a, case["kseg"], case["dual"])
    layer = sq.Layer(M, K, N, case["kseg"], [0, N], case["dual"], sp, sn)
    S = len(case["dual"])

    def make(l):
        w = (rng.standard_normal((N, K)) * (0.02 * (1 + l % 3))).astype(np.float32)
        b = None if l % 2 else rng.standard_normal(N).astype(np.float32)
        wq = torch.empty((N, K), dtype=torch.int8, device=g.DEV)
        ws = torch.empty((S, N), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_weight(layer, torch.from_numpy(w).to(g.DEV), wq, ws)
        return w, b, wq, ws, None if b is None else torch.from_numpy(b).to(g.DEV)

    def compare(y, w, b, what):
        r = oracle.seglinear(a, w, case["kseg"], [0, N], case["dual"], sp, sn, None, b)
        ymax = float(np.abs(r.y32).max())
        yh = y.cpu().numpy()
        assert not np.isnan(yh).any(), what
        err = float(np.abs(yh.astype(np.float64) - r.y32.astype(np.float64)).max())
        assert err <= RTOL * ymax, f"{what}: fp32 output error {err} > {RTOL} * {ymax}"

    w, b, wq, ws, bd = make(0)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_seglinear_fused(layer, hd, case["act"], wq, ws, bd, y)
    torch.cuda.synchronize()
    compare(y, w, b, "single")
    # the two-launch path gives the same bits (same codes, same kernel)
    xq = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_fused(layer, hd, case["act"], xq)
    y2 = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_tuning_set("force_path", 3)
    sq.sq_seglinear(layer, xq, wq, ws, bd, y2)
    sq.sq_tuning_set("force_path", -1)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int32), y2.view(torch.int32))
    # bf16 output
    yb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=g.DEV)
    sq.sq_seglinear_fused(layer, hd, case["act"], wq, ws, bd, yb)
    torch.cuda.synchronize()
    r = oracle.seglinear(a, w, case["kseg"], [0, N], case["dual"], sp, sn, None, b)
    g.check_bf16_against(g.bf16_tensor_bits(yb), r.y32, r.y_bf16_bits, RTOL * float(np.abs(r.y32).max()))
    if case["L"] == 0:
        with pytest.raises(sq.SqError) as e:                 # the grouped call stops at 32 tokens
            sq.sq_seglinear_grouped_fused(layer, hd, case["act"], [(wq, ws, bd, y)])
        assert e.value.status == 2
        return
    items, hosts = [], []
    for l in range(case["L"]):
        w, b, wq, ws, bd = make(l + 1)
        items.append((wq, ws, bd, torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)))
        hosts.append((w, b))
    sq.sq_seglinear_grouped_fused(layer, hd, case["act"], items)
    torch.cuda.synchronize()
    for l, (w, b) in enumerate(hosts):
        compare(items[l][3], w, b, f"grouped layer {l}")


def test_seglinear_fused_rejects_what_the_stream_kernel_cannot_run():
    import torch

    g = _gpu()
    for (M, K, kseg) in [(65, 256, [0, 256]), (8, 192, [0, 192]), (8, 256, [0, 64, 256])]:
        layer = sq.Layer(M, K, 64, kseg, [0, 64], [1] * (len(kseg) - 1), [0.1] * (len(kseg) - 1), [0.1] * (len(kseg) - 1))
        x = torch.zeros((M, K), dtype=torch.float32, device=g.DEV)
        wq = torch.zeros((64, K), dtype=torch.int8, device=g.DEV)
        ws = torch.ones((len(kseg) - 1, 64), dtype=torch.float32, device=g.DEV)
        y = torch.empty((M, 64), dtype=torch.float32, device=g.DEV)
        with pytest.raises(sq.SqError) as e:
            sq.sq_seglinear_fused(layer, x, None, wq, ws, None, y)
        assert e.value.status == 2


GEGLU = [
    dict(M=70, K=512, kseg=[0, 128, 512], dual=[0, 1], h_dtype="bf16"),
    dict(M=1100, K=1280, kseg=[0, 1280], dual=[1], h_dtype="bf16"),            # many chunks per workgroup
    dict(M=129, K=1024, kseg=[0, 16, 48, 1024], dual=[1, 0, 1], h_dtype="f32"),
    dict(M=13, K=100, kseg=[0, 37, 100], dual=[1, 1], h_dtype="bf16"),         # unaligned: one output per thread
    dict(M=5, K=24, kseg=[0, 24], dual=[1], h_dtype="f32"),
    dict(M=1, K=16, kseg=[0, 16], dual=[0], h_dtype="bf16"),
    dict(M=2100, K=2560, kseg=[0, 512, 2560], dual=[1, 0], h_dtype="bf16"),    # more chunks than threads in flight
    dict(M=4096, K=1024, kseg=[0, 1024], dual=[1], h_dtype="bf16"),
]


@pytest.mark.parametrize("case", GEGLU)
@pytest.mark.parametrize("spread", ["unit", "wide"])
def test_quantize_act_geglu(oracle, case, spread):
    """xq = Q_dual(value * GELU(gate)) over the two halves of every row: codes bit-exact against the oracle."""
    import torch

    g = _gpu()
    M, K = case["M"], case["K"]
    rng = np.random.default_rng(M * 13 + K)
    h = (rng.standard_normal((M, 2 * K)) * (1.0 if spread == "unit" else 9.0)).astype(np.float32)
    if spread == "wide" and K >= 8:
        h[0, K:K + 8] = [0.0, -0.0, 95.0, -95.0, 1e4, -1e4, 30.0, -9.0]
    if K >= 16:                               # tiny and large gates next to ordinary ones
        h[M - 1, K:K + 8] = [2.0 ** -14, -(2.0 ** -14), 2.0 ** -15, -3e-5, 7.96875, -7.96875, 8.0, -8.0]
        h[M - 1, :8] = [3.0, -2.0, 1e3, 5.0, 1.5, -1.5, 0.25, 4.0]
    if case["h_dtype"] == "bf16":
        h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(h))
        hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        hd = torch.from_numpy(h).to(g.DEV)
    a = oracle.geglu(h)
    sp, sn, _, _ = oracle.calibrate_act(a, case["kseg"], case["dual"])
    layer = sq.Layer(M, K, 4, case["kseg"], [0, 4], case["dual"], sp, sn)
    xq = torch.full((M, K), 99, dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act_geglu(layer, hd, xq)
    torch.cuda.synchronize()
    rp, rn = oracle.quantize_act_geglu(h, case["kseg"], case["dual"], sp, sn)
    got = xq.cpu().numpy()
    want = (rp.astype(np.int16) + rn.astype(np.int16)).astype(np.int8)
    bad = np.argwhere(got != want)
    assert bad.size == 0, (len(bad), bad[:5], got[tuple(bad[0])], want[tuple(bad[0])])
    assert np.abs(want).max() == 127


FUSEDDYN = [
    dict(M=16, K=1152, N=6912, kseg=[0, 1152], dual=[1], act=[1], h_dtype="bf16"),                 # adaLN in the 4-bit setting
    dict(M=5, K=256, N=70, kseg=[0, 128, 256], dual=[0, 1], act=[0, 2], h_dtype="f32", bias=True),
    dict(M=40, K=512, N=200, kseg=[0, 384, 512], dual=[1, 1], act=[1, 1], h_dtype="bf16"),          # three row tiles
    dict(M=1, K=128, N=16, kseg=[0, 128], dual=[1], act=[0], h_dtype="f32"),
    dict(M=9, K=3072, N=48, kseg=[0, 1024, 3072], dual=[1, 0], act=[2, 0], h_dtype="bf16"),         # more items than preloaded
]


@pytest.mark.parametrize("case", FUSEDDYN)
def test_seglinear_fused_dynamic(oracle, case):
    """Raw activations in, per-token steps found inside the launch (4-bit settings): against the oracle's
    activation -> dynamic Q_dual -> SegLinear, and bit for bit against quantize_act_dynamic + seglinear_dynamic."""
    import torch

    g = _gpu()
    M, K, N = case["M"], case["K"], case["N"]
    rng = np.random.default_rng(M * 3 + K + N)
    h = (rng.standard_normal((M, K)) * rng.uniform(0.2, 6.0, size=(M, 1))).astype(np.float32)   # tokens of different scale
    h[0, :4] = [0.0, -0.0, 50.0, -50.0]
    if case["h_dtype"] == "bf16":
        h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(h))
        hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    else:
        hd = torch.from_numpy(h).to(g.DEV)
    a = oracle.activation(h, case["kseg"], case["act"])
    S = len(case["dual"])
    layer = sq.Layer(M, K, N, case["kseg"], [0, N], case["dual"], [1.0] * S, [1.0] * S)
    w = (rng.standard_normal((N, K)) * 0.03).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32) if case.get("bias") else None
    bd = None if b is None else torch.from_numpy(b).to(g.DEV)
    wt = torch.from_numpy(w).to(g.DEV)
    ad = torch.from_numpy(a).to(g.DEV)                         # the activation's fp32 result, for the two-launch path
    for bits in (8, 4):
        ws = torch.empty((S, N), dtype=torch.float32, device=g.DEV)
        if bits == 8:
            wq = torch.empty((N, K), dtype=torch.int8, device=g.DEV)
            sq.sq_quantize_weight(layer, wt, wq, ws)
        else:
            wq = torch.empty((((N + 15) // 16) * 16 * (K // 2),), dtype=torch.uint8, device=g.DEV)
            sq.sq_quantize_weight_w4(layer, wt, wq, ws)
        r4 = oracle.seglinear_dynamic(a, w, case["kseg"], [0, N], case["dual"], None, b, wbits=bits, abits=4)
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_seglinear_fused_dynamic(layer, hd, case["act"], wq, bits, ws, bd, y, a_bits=4)      # the W4A4 / W8A4 settings
        torch.cuda.synchronize()
        err4 = float(np.abs(y.cpu().numpy().astype(np.float64) - r4.y32.astype(np.float64)).max())
        assert err4 <= RTOL * float(np.abs(r4.y32).max()), (bits, err4)
        r = oracle.seglinear_dynamic(a, w, case["kseg"], [0, N], case["dual"], None, b, wbits=bits)
        ymax = float(np.abs(r.y32).max())
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_seglinear_fused_dynamic(layer, hd, case["act"], wq, bits, ws, bd, y)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        assert not np.isnan(yh).any()
        err = float(np.abs(yh.astype(np.float64) - r.y32.astype(np.float64)).max())
        assert err <= RTOL * ymax, (bits, err, ymax)
        # two launches on the activated values: same steps, same codes, same kernel -> same bits
        xq = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
        tok = torch.empty((2, M, S), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_act_dynamic(layer, ad, xq, tok)
        y2 = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
        sq.sq_seglinear_dynamic(layer, xq, tok, wq, bits, ws, bd, y2)
        torch.cuda.synchronize()
        assert np.array_equal(tok.cpu().numpy().view(np.uint32), r.tok_steps.view(np.uint32))
        if M <= 32:                                            # above, the two-launch path takes another kernel
            assert torch.equal(y.view(torch.int32), y2.view(torch.int32)), bits
        yb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=g.DEV)
        sq.sq_seglinear_fused_dynamic(layer, hd, case["act"], wq, bits, ws, bd, yb)
        torch.cuda.synchronize()
        g.check_bf16_against(g.bf16_tensor_bits(yb), r.y32, wl.f32_to_bf16_bits(r.y32), RTOL * ymax)


GROUPEDW4 = [
    dict(M=16, K=1152, N=1152, L=4, kseg=[0, 1152], dual=[1], ydt="bf16"),
    dict(M=7, K=256, N=100, L=3, kseg=[0, 128, 256], dual=[1, 0], ydt="f32"),          # ragged N (padded last group)
    dict(M=32, K=384, N=528, L=6, kseg=[0, 384], dual=[0], ydt="f32"),
    dict(M=1, K=128, N=16, L=1, kseg=[0, 128], dual=[1], ydt="f32"),
]


@pytest.mark.parametrize("case", GROUPEDW4)
@pytest.mark.parametrize("dynamic", [False, True])
def test_seglinear_grouped_w4(oracle, case, dynamic):
    """L layers with packed 4-bit weights that share the quantized input, one launch, static or per-token steps
    (8- and 4-bit activation codes): every layer against the oracle."""
    import torch

    g = _gpu()
    M, K, N, L = case["M"], case["K"], case["N"], case["L"]
    base = wl.random_layer(M, K, N, case["kseg"], [0, N], case["dual"], seed=K + L + 1, x_dtype="bf16", act="silu", with_bias=True)
    gl = g.GpuLayer(base)
    rng = np.random.default_rng(L * 77 + N)
    tdt = torch.bfloat16 if case["ydt"] == "bf16" else torch.float32
    items, hosts = [], []
    for l in range(L):
        wl_l = (rng.standard_normal((N, K)) * (0.01 * (1 + l % 4))).astype(np.float32)
        bias_l = None if l % 2 else rng.standard_normal(N).astype(np.float32)
        wq4 = torch.empty((((N + 15) // 16) * 16 * (K // 2),), dtype=torch.uint8, device=g.DEV)
        ws = torch.empty((base.S, N), dtype=torch.float32, device=g.DEV)
        sq.sq_quantize_weight_w4(gl.layer, torch.from_numpy(wl_l).to(g.DEV), wq4, ws)
        y = torch.full((M, N), float("nan"), dtype=tdt, device=g.DEV)
        items.append((wq4, ws, None if bias_l is None else torch.from_numpy(bias_l).to(g.DEV), y))
        hosts.append((wl_l, bias_l))
    for abits in ((8, 4) if dynamic else (None,)):
        if dynamic:
            tok = torch.empty((2, M, base.S), dtype=torch.float32, device=g.DEV)
            sq.sq_quantize_act_dynamic_bits(gl.layer, gl.x, abits, gl.xq, tok)
            sq.sq_seglinear_grouped_w4(gl.layer, gl.xq, items, tok_steps=tok)
        else:
            gl.quantize_act()
            sq.sq_seglinear_grouped_w4(gl.layer, gl.xq, items)
        torch.cuda.synchronize()
        for l, (wl_l, bias_l) in enumerate(hosts):
            if dynamic:
                r = oracle.seglinear_dynamic(base.x, wl_l, base.kseg_off, base.nseg_off, base.dual, None, bias_l, wbits=4, abits=abits)
            else:
                r = oracle.seglinear(base.x, wl_l, base.kseg_off, base.nseg_off, base.dual, base.s_pos, base.s_neg, None, bias_l, wbits=4)
            ymax = float(np.abs(r.y32).max())
            if case["ydt"] == "f32":
                y = items[l][3].cpu().numpy()
                assert not np.isnan(y).any()
                err = float(np.abs(y.astype(np.float64) - r.y32.astype(np.float64)).max())
                assert err <= RTOL * ymax, f"layer {l} (a_bits {abits}): fp32 output error {err} > {RTOL} * {ymax}"
            else:
                g.check_bf16_against(g.bf16_tensor_bits(items[l][3]), r.y32, r.y_bf16_bits, RTOL * ymax)


def test_graph_capture_dynamic_and_fused_paths(oracle):
    """The entry points with per-token steps keep nothing between calls either: a skinny layer fed with raw activations
    (SiLU, per-token steps, packed 4-bit weights: one launch) and a layer with many token rows (dynamic quantizer + tile
    kernel) captured in one HIP graph, replayed on fresh inputs with eager work in between, every replay checked."""
    import torch

    g = _gpu()
    rng = np.random.default_rng(31)
    # skinny layer
    M1, K1, N1 = 16, 512, 330
    h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((rng.standard_normal((M1, K1)) * 2).astype(np.float32)))
    w1 = (rng.standard_normal((N1, K1)) * 0.03).astype(np.float32)
    l1 = sq.Layer(M1, K1, N1, [0, K1], [0, N1], [1], [1.0], [1.0])
    hd = torch.from_numpy(wl.f32_to_bf16_bits(h).view(np.int16)).view(torch.bfloat16).to(g.DEV)
    wq4 = torch.empty((((N1 + 15) // 16) * 16 * (K1 // 2),), dtype=torch.uint8, device=g.DEV)
    ws1 = torch.empty((1, N1), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight_w4(l1, torch.from_numpy(w1).to(g.DEV), wq4, ws1)
    y1 = torch.zeros((M1, N1), dtype=torch.float32, device=g.DEV)
    # layer with many token rows
    w2 = wl.random_layer(300, 512, 260, [0, 256, 512], [0, 260], [0, 1], seed=23, x_dtype="bf16", act="gelu", with_bias=True)
    gl = g.GpuLayer(w2)
    gl.quantize_weight()
    tok = torch.zeros((2, w2.M, w2.S), dtype=torch.float32, device=g.DEV)
    y2 = torch.zeros((w2.M, w2.N), dtype=torch.float32, device=g.DEV)

    def step():
        sq.sq_seglinear_fused_dynamic(l1, hd, [sq.SQ_ACT_SILU], wq4, 4, ws1, None, y1)
        sq.sq_quantize_act_dynamic(gl.layer, gl.x, gl.xq, tok)
        sq.sq_seglinear_dynamic(gl.layer, gl.xq, tok, gl.wq, 8, gl.wscale, gl.bias, y2)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up outside the capture
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        hs = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((h * (1.0 + 0.3 * rep) + 0.05 * rng.standard_normal(h.shape)).astype(np.float32)))
        xs = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits((w2.x * (1.0 + 0.2 * rep) + 0.02 * rng.standard_normal(w2.x.shape)).astype(np.float32)))
        hd.copy_(torch.from_numpy(wl.f32_to_bf16_bits(hs).view(np.int16)).view(torch.bfloat16).to(g.DEV))
        gl.x.copy_(torch.from_numpy(wl.f32_to_bf16_bits(xs).view(np.int16)).view(torch.bfloat16).to(g.DEV))
        y1.fill_(float("nan"))                                          # eager work between replays
        y2.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        r1 = oracle.seglinear_dynamic(oracle.activation(hs, [0, K1], [oracle.ACT_SILU]), w1, [0, K1], [0, N1], [1], None, None, wbits=4)
        e1 = float(np.abs(y1.cpu().numpy().astype(np.float64) - r1.y32).max())
        assert e1 <= RTOL * float(np.abs(r1.y32).max()), f"replay {rep}: skinny layer {e1}"
        r2 = oracle.seglinear_dynamic(xs, w2.w, w2.kseg_off, w2.nseg_off, w2.dual, None, w2.bias)
        assert np.array_equal(tok.cpu().numpy().view(np.uint32), r2.tok_steps.view(np.uint32)), f"replay {rep}"
        e2 = float(np.abs(y2.cpu().numpy().astype(np.float64) - r2.y32).max())
        assert e2 <= RTOL * float(np.abs(r2.y32).max()), f"replay {rep}: large layer {e2}"


def test_near_the_size_limit(oracle):
    """M*K just below 2^31 (the documented limit): static and per-token quantizer and GEMM on sampled rows, which the
    oracle computes one by one.  Inputs are drawn on the device (the oracle only ever sees the sampled rows)."""
    import torch

    g = _gpu()
    M, K, N = 32768, 65408, 64
    assert 0 < 2 ** 31 - M * K <= 2 ** 22
    kseg, dual = [0, 16384, K], [0, 1]
    gen = torch.Generator(device=g.DEV).manual_seed(1)
    x = torch.empty((M, K), dtype=torch.bfloat16, device=g.DEV)
    for i in range(0, M, 4096):
        x[i:i + 4096] = (torch.randn((4096, K), device=g.DEV, generator=gen) * 1.5).to(torch.bfloat16)
    x[:, 16384:] = torch.nn.functional.gelu(x[:, 16384:].float(), approximate="tanh").to(torch.bfloat16)
    w = (np.random.default_rng(2).standard_normal((N, K)) * 0.02).astype(np.float32)
    sp, sn = [6.0 / 127, 7.0 / 127], [1.0, 0.17 / 127]
    layer = sq.Layer(M, K, N, kseg, [0, N], dual, sp, sn)
    wq = torch.empty((N, K), dtype=torch.int8, device=g.DEV)
    ws = torch.empty((2, N), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight(layer, torch.from_numpy(w).to(g.DEV), wq, ws)
    xq = torch.full((M, K), 99, dtype=torch.int8, device=g.DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_act(layer, x, xq)
    sq.sq_seglinear(layer, xq, wq, ws, None, y)
    torch.cuda.synchronize()
    rows = [0, 1, 127, 128, 4095, 16384, 20000, M - 129, M - 2, M - 1]
    xs = x[rows].float().cpu().numpy()
    r = oracle.seglinear(xs, w, kseg, [0, N], dual, layer.s_pos, layer.s_neg)
    want = (r.xq_pos.astype(np.int16) + r.xq_neg.astype(np.int16)).astype(np.int8)
    assert np.array_equal(xq[rows].cpu().numpy(), want)
    assert not torch.isnan(y).any()
    err = float(np.abs(y[rows].cpu().numpy().astype(np.float64) - r.y32.astype(np.float64)).max())
    assert err <= RTOL * float(np.abs(r.y32).max())
    tok = torch.empty((2, M, 2), dtype=torch.float32, device=g.DEV)
    y.fill_(float("nan"))
    sq.sq_quantize_act_dynamic(layer, x, xq, tok)
    sq.sq_seglinear_dynamic(layer, xq, tok, wq, 8, ws, None, y)
    torch.cuda.synchronize()
    rd = oracle.seglinear_dynamic(xs, w, kseg, [0, N], dual)
    assert np.array_equal(tok[:, rows].cpu().numpy().view(np.uint32), rd.tok_steps.view(np.uint32))
    assert not torch.isnan(y).any()
    err = float(np.abs(y[rows].cpu().numpy().astype(np.float64) - rd.y32.astype(np.float64)).max())
    assert err <= RTOL * float(np.abs(rd.y32).max())


@pytest.mark.parametrize("shape", [(16, 1152, 1864000), (16, 65408, 32768), (40, 65408, 32768)])
def test_weights_near_the_size_limit(oracle, shape):
    """N*K just below 2^31: weight quantizer and GEMM (weight-stream kernel for the first shape, tile kernel for the long
    rows) on sampled output channels, whose weight rows the oracle gets one by one.  Weights are drawn on the device."""
    import torch

    g = _gpu()
    M, K, N = shape
    assert 0 < 2 ** 31 - N * K <= 2 ** 23
    kseg, dual = [0, K], [1]
    base = wl.random_layer(M, K, 8, kseg, [0, 8], dual, seed=K + M, x_dtype="bf16", act="silu")
    layer = sq.Layer(M, K, N, kseg, [0, N], dual, base.s_pos, base.s_neg)
    gen = torch.Generator(device=g.DEV).manual_seed(3)
    wt = torch.empty((N, K), dtype=torch.float32, device=g.DEV)
    step = max(1, (1 << 28) // K)
    for i in range(0, N, step):
        n = min(step, N - i)
        wt[i:i + n] = torch.randn((n, K), device=g.DEV, generator=gen) * 0.02
    wq = torch.full((N, K), 99, dtype=torch.int8, device=g.DEV)
    ws = torch.full((1, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight(layer, wt, wq, ws)
    xd = g.to_dev_x(base)
    xq = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act(layer, xd, xq)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_seglinear(layer, xq, wq, ws, None, y)
    torch.cuda.synchronize()
    cols = [0, 1, 15, 16, 255, N // 3, N // 2 + 7, N - 17, N - 2, N - 1]
    wc = wt[cols].cpu().numpy()
    del wt
    r = oracle.seglinear(base.x, wc, kseg, [0, len(cols)], dual, base.s_pos, base.s_neg)
    assert np.array_equal(wq[cols].cpu().numpy(), r.wq)
    assert np.array_equal(ws[:, cols].cpu().numpy().view(np.uint32), r.wscale.view(np.uint32))
    assert not torch.isnan(y).any()
    yc = y[:, cols].cpu().numpy().astype(np.float64)
    err = float(np.abs(yc - r.y32.astype(np.float64)).max())
    assert err <= RTOL * float(np.abs(r.y32).max())


@pytest.mark.parametrize("ydt", ["f32", "bf16"])
def test_output_near_the_size_limit(oracle, ydt):
    """M*N just below 2^31 (a short K): the store epilogue's offsets, on sampled token rows."""
    import torch

    g = _gpu()
    M, K, N = 32768, 128, 65504
    assert 0 < 2 ** 31 - M * N <= 2 ** 21
    kseg, dual = [0, K], [1]
    rng = np.random.default_rng(8)
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    gen = torch.Generator(device=g.DEV).manual_seed(4)
    x = torch.nn.functional.silu(torch.randn((M, K), device=g.DEV, generator=gen) * 1.5).to(torch.bfloat16)
    sp, sn = [6.5 / 127], [0.279 / 127]
    layer = sq.Layer(M, K, N, kseg, [0, N], dual, sp, sn)
    wq = torch.empty((N, K), dtype=torch.int8, device=g.DEV)
    ws = torch.empty((1, N), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight(layer, torch.from_numpy(w).to(g.DEV), wq, ws)
    xq = torch.empty((M, K), dtype=torch.int8, device=g.DEV)
    sq.sq_quantize_act(layer, x, xq)
    y = torch.full((M, N), float("nan"), dtype=torch.float32 if ydt == "f32" else torch.bfloat16, device=g.DEV)
    sq.sq_seglinear(layer, xq, wq, ws, None, y)
    torch.cuda.synchronize()
    rows = [0, 1, 127, 128, 9999, 16384, M - 129, M - 2, M - 1]
    r = oracle.seglinear(x[rows].float().cpu().numpy(), w, kseg, [0, N], dual, layer.s_pos, layer.s_neg)
    assert not torch.isnan(y.float().sum(dim=1)).any()
    ymax = float(np.abs(r.y32).max())
    if ydt == "f32":
        err = float(np.abs(y[rows].cpu().numpy().astype(np.float64) - r.y32.astype(np.float64)).max())
        assert err <= RTOL * ymax
    else:
        g.check_bf16_against(g.bf16_tensor_bits(y[rows]), r.y32, r.y_bf16_bits, RTOL * ymax)


def _random_segments(rng, total, align, maxs):
    units = total // align
    n = int(rng.integers(1, min(maxs, units) + 1))
    cuts = sorted(rng.choice(np.arange(1, units), size=n - 1, replace=False).tolist()) if n > 1 else []
    return [0] + [c * align for c in cuts] + [total]


def test_fp8_random_shapes_against_oracle(oracle):
    """A seeded walk over shapes, K / N segmentations, input types, tile configurations and the plain kernel for the fp8
    variant: codes and weight steps bit-exact, outputs within the bound of an fp32 evaluation."""
    import torch

    g = _gpu()
    rng = np.random.default_rng(20250715)
    ran = 0
    for n in range(60):
        M = int(rng.choice([1, 17, 64, 100, 129, 257, 300, 385, 700]))
        K = 128 * int(rng.integers(1, 13))
        N = int(rng.choice([7, 33, 64, 100, 128, 130, 192, 256, 300, 520]))
        kseg = _random_segments(rng, K, 128, 4)
        nseg = _random_segments(rng, N, 1, 3)
        dual = [int(rng.integers(0, 2)) for _ in kseg[:-1]]
        xdt = str(rng.choice(["bf16", "f32"]))
        act = str(rng.choice(["silu", "gelu", "normal", "relu", "neg"]))
        pick = int(rng.integers(0, 8))
        path, variant = (0, -1) if pick < 2 else (3, -1) if pick == 2 else (-1, int(rng.choice([-1, -1, 0, 1, 3, 4, 5, 8])))
        what = dict(case=n, M=M, K=K, N=N, kseg=kseg, nseg=nseg, dual=dual, xdt=xdt, act=act, path=path, variant=variant)
        w = wl.random_layer(M, K, N, kseg, nseg, dual, seed=9000 + n, x_dtype=xdt, act=act,
                            with_seg_scale=bool(rng.integers(0, 2)), with_bias=bool(rng.integers(0, 2)))
        w.s_pos = (w.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)
        w.s_neg = (w.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
        gl = g.GpuLayer(w)
        wq = torch.full((N, K), 0x7F, dtype=torch.uint8, device=g.DEV)
        xq = torch.full((M, K), 0x7F, dtype=torch.uint8, device=g.DEV)
        sq.sq_quantize_weight_fp8(gl.layer, gl.wt, wq, gl.wscale)
        sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
        ydt = str(rng.choice(["f32", "bf16"]))
        y = torch.full((M, N), float("nan"), dtype=torch.bfloat16 if ydt == "bf16" else torch.float32, device=g.DEV)
        sq.sq_tuning_set("force_path", path)
        sq.sq_tuning_set("gemm_variant", variant)
        try:
            sq.sq_seglinear_fp8(gl.layer, xq, wq, gl.wscale, gl.bias, y)
        except sq.SqError as e:
            assert e.status == 2 and (variant >= 0 or path == 3), what     # a tile configuration / kernel that does not serve this layer
            continue
        torch.cuda.synchronize()
        r_wq, r_ws = oracle.quantize_weight_fp8(w.w, w.kseg_off)
        r_xp, r_xn = oracle.quantize_act_fp8(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
        assert np.array_equal(wq.cpu().numpy(), _plus_zero(r_wq)), what
        assert np.array_equal(gl.wscale.cpu().numpy().view(np.uint32), r_ws.view(np.uint32)), what
        xp, xn = _split_fp8(w, xq.cpu().numpy())
        assert np.array_equal(xp, _plus_zero(r_xp)) and np.array_equal(xn, _plus_zero(r_xn)), what
        ref, mag = oracle.seglinear_fp8(r_xp, r_xn, r_wq, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, r_ws, w.seg_scale, w.bias)
        got = y.float().cpu().numpy().astype(np.float64)
        tol = _fp8_tol(K, mag, ref, ydt)
        assert not np.isnan(got).any() and (np.abs(got - ref) <= tol).all(), (what, float((np.abs(got - ref) / tol).max()))
        ran += 1
    assert ran >= 45


def test_fp8_many_tiles_and_graph_replay(oracle):
    """More tiles than compute units (the persistent workgroups walk several tiles and prefetch across their boundaries), dual
    with several K-segments, ragged edges; then the quantizer and the product captured into a HIP graph and replayed with
    eager work in between: every replay must reproduce the eager result to the bit."""
    import torch

    g = _gpu()
    M, K, N = 3000, 768, 2500
    w = wl.random_layer(M, K, N, [0, 256, 768], [0, 1000, N], [1, 0], seed=77, x_dtype="bf16", act="gelu",
                        with_seg_scale=True, with_bias=True)
    w.s_pos = (w.s_pos * np.float32(127.0 / 448.0)).astype(np.float32)
    w.s_neg = (w.s_neg * np.float32(127.0 / 448.0)).astype(np.float32)
    gl = g.GpuLayer(w)
    wq = torch.empty((N, K), dtype=torch.uint8, device=g.DEV)
    xq = torch.empty((M, K), dtype=torch.uint8, device=g.DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
    sq.sq_quantize_weight_fp8(gl.layer, gl.wt, wq, gl.wscale)
    sq.sq_tuning_set("gemm_variant", 3)                          # 64 x 128 tiles: 47 x 20 = 940 of them
    sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
    sq.sq_seglinear_fp8(gl.layer, xq, wq, gl.wscale, gl.bias, y)
    torch.cuda.synchronize()
    r_wq, r_ws = oracle.quantize_weight_fp8(w.w, w.kseg_off)
    r_xp, r_xn = oracle.quantize_act_fp8(w.x, w.kseg_off, w.dual, w.s_pos, w.s_neg)
    ref, mag = oracle.seglinear_fp8(r_xp, r_xn, r_wq, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, r_ws, w.seg_scale, w.bias)
    got = y.cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= _fp8_tol(K, mag, ref, "f32")).all()
    eager = y.clone()
    st = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=st):
        sq.sq_quantize_act_fp8(gl.layer, gl.x, xq)
        sq.sq_seglinear_fp8(gl.layer, xq, wq, gl.wscale, gl.bias, y)
    for _ in range(3):
        y.fill_(float("nan"))
        xq.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager)


def test_random_shapes_against_oracle(oracle):
    """A seeded walk over legal shapes, segmentations, input types and forced kernels (the committed slice of a much longer
    one-off sweep): quantizers bit-exact, integer sums bit-exact, outputs within the fp32 tolerance, static and per-token."""
    import torch

    g = _gpu()
    rng = np.random.default_rng(20250714)
    ran = 0
    for n in range(160):
        align = int(rng.choice([128, 128, 64, 16, 1]))
        M = int(rng.choice([1, 3, 16, 17, 31, 33, 64, 65, 100, 129, 200, 300, 385]))
        K = align * int(rng.integers(1, max(2, 1536 // align))) if align > 1 else int(rng.integers(5, 700))
        N = int(rng.choice([7, 16, 33, 64, 100, 128, 130, 192, 256, 300, 520]))
        kseg = _random_segments(rng, K, align, 4)
        nseg = _random_segments(rng, N, 1, 3)
        dual = [int(rng.integers(0, 2)) for _ in kseg[:-1]]
        xdt = str(rng.choice(["bf16", "f32"]))
        act = str(rng.choice(["silu", "gelu", "normal", "relu", "neg"]))
        path = int(rng.choice([-1, -1, 0, 1, 2, 3]))
        what = dict(case=n, M=M, K=K, N=N, kseg=kseg, nseg=nseg, dual=dual, xdt=xdt, act=act, path=path)
        w = wl.random_layer(M, K, N, kseg, nseg, dual, seed=7000 + n, x_dtype=xdt, act=act,
                            with_seg_scale=bool(rng.integers(0, 2)), with_bias=bool(rng.integers(0, 2)))
        gl = g.GpuLayer(w)
        wq, ws = gl.quantize_weight()
        xp, xn, _ = gl.quantize_act()
        r = oracle.seglinear(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.s_pos, w.s_neg, w.seg_scale, w.bias)
        assert np.array_equal(wq, r.wq) and np.array_equal(ws.view(np.uint32), r.wscale.view(np.uint32)), what
        assert np.array_equal(xp, r.xq_pos) and np.array_equal(xn, r.xq_neg), what
        sq.sq_tuning_set("force_path", path)
        try:
            ap = torch.full((w.S, M, N), 0x5A5A5A5A, dtype=torch.int32, device=g.DEV)
            an = torch.full_like(ap, 0x5A5A5A5A)
            try:
                sq.sq_seglinear_debug_acc(gl.layer, gl.xq, gl.wq, ap, an)
            except sq.SqError as e:
                assert e.status == 2 and path > 0, what           # a forced kernel that does not take this shape
                continue
            y = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
            sq.sq_seglinear(gl.layer, gl.xq, gl.wq, gl.wscale, gl.bias, y)
            tok = torch.empty((2, M, w.S), dtype=torch.float32, device=g.DEV)
            xqd = torch.empty_like(gl.xq)
            sq.sq_quantize_act_dynamic(gl.layer, gl.x, xqd, tok)
            yd = torch.full((M, N), float("nan"), dtype=torch.float32, device=g.DEV)
            dyn = True
            try:
                sq.sq_seglinear_dynamic(gl.layer, xqd, tok, gl.wq, 8, gl.wscale, gl.bias, yd)
            except sq.SqError as e:
                assert e.status == 2 and path > 0, what           # the forced kernel has no per-token form for this layer
                dyn = False
            torch.cuda.synchronize()
            assert np.array_equal(ap.cpu().numpy(), r.acc_pos) and np.array_equal(an.cpu().numpy(), r.acc_neg), what
            err = float(np.abs(y.cpu().numpy().astype(np.float64) - r.y32.astype(np.float64)).max())
            assert err <= RTOL * float(np.abs(r.y32).max()), (what, err)
            ran += 1
            if not dyn:
                continue
            rd = oracle.seglinear_dynamic(w.x, w.w, w.kseg_off, w.nseg_off, w.dual, w.seg_scale, w.bias)
            xpd, xnd = g.split_codes(w, xqd.cpu().numpy())
            assert np.array_equal(xpd, rd.xq_pos) and np.array_equal(xnd, rd.xq_neg), what
            assert np.array_equal(tok.cpu().numpy().view(np.uint32), rd.tok_steps.view(np.uint32)), what
            errd = float(np.abs(yd.cpu().numpy().astype(np.float64) - rd.y32.astype(np.float64)).max())
            assert errd <= RTOL * float(np.abs(rd.y32).max()), (what, errd)
        finally:
            sq.sq_tuning_set("force_path", -1)
    assert ran >= 100
