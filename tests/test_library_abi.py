"""Host-side checks that need no GPU: the C-ABI library loads, exports every declared symbol, and its
argument validation returns the documented status codes before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sq():
    import paper_2507_14811_amd as m
    from paper_2507_14811_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):          # tests load what is built; build only if nothing is
        build.build_library(verbose=False)
    m.load_library()
    return m


def test_every_declared_symbol_is_exported(sq):
    with open(os.path.join(ROOT, "include", "segquant.h")) as f:
        header = f.read()
    declared = set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", header))
    assert {"sq_quantize_weight", "sq_quantize_act", "sq_seglinear", "sq_seglinear_debug_acc", "sq_status_string",
            "sq_version", "sq_tuning_set"} <= declared
    lib = sq.load_library()
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in segquant.h but not exported"
    from paper_2507_14811_amd import binding

    assert set(binding.EXPORTS) == declared


def test_probe_library_exports_its_header(sq):
    """libsegquant_probes.so (benchmark probes, loaded by bench.py only) exports what include/segquant_probes.h declares,
    and the product library exports none of it."""
    import ctypes

    from paper_2507_14811_amd import build, probes

    if not os.path.exists(probes.LIB_PATH):
        build.build_library(verbose=False)
    with open(os.path.join(ROOT, "include", "segquant_probes.h")) as f:
        declared = set(re.findall(r"\b(sqp_[a-z0-9_]+)\s*\(", f.read()))
    assert declared == set(probes.EXPORTS)
    lib = ctypes.CDLL(probes.LIB_PATH)
    main = sq.load_library()
    for name in declared:
        assert hasattr(lib, name), name
        assert not hasattr(main, name), name
    # argument checks run on the host, before anything is launched
    assert lib.sqp_launch(0, 64, 0, None) == 1 and lib.sqp_launch(1, 100, 0, None) == 1
    assert lib.sqp_copy(None, None, ctypes.c_size_t(16), None) == 1


def test_smooth_factors_on_the_host_match_the_oracle(sq, oracle):
    """sq_smooth_factors is a host computation (it launches nothing): bit-equal to the oracle's, dead channels and the
    ends of alpha included; alpha outside [0, 1] and negative maxima are rejected."""
    rng = np.random.default_rng(12)
    K, kseg = 300, [0, 100, 180, 300]
    layer = sq.Layer(4, K, 8, kseg, [0, 8], [1, 0, 1])
    ax = rng.uniform(0.0, 40.0, K).astype(np.float32)
    aw = rng.uniform(0.0, 1.5, K).astype(np.float32)
    ax[[3, 150]] = 0.0
    aw[[7, 299]] = 0.0
    ax[10], aw[10] = 1e30, 1e-30                     # the factor overflows fp32: the channel keeps 1
    for alpha in ([0.5, 0.5, 0.5], [0.0, 1.0, 0.3], [0.1, 0.9, 0.7]):
        s, r = sq.sq_smooth_factors(layer, ax, aw, alpha)
        os_, or_ = oracle.smooth_factors(ax, aw, kseg, alpha)
        assert np.array_equal(s.view(np.uint32), os_.view(np.uint32)) and np.array_equal(r.view(np.uint32), or_.view(np.uint32))
        assert s[3] == 1.0 and s[7] == 1.0
    with pytest.raises(sq.SqError):
        sq.sq_smooth_factors(layer, ax, aw, [0.5, 1.2, 0.5])
    with pytest.raises(sq.SqError):
        sq.sq_smooth_factors(layer, -ax - 1, aw, [0.5, 0.5, 0.5])


def test_status_strings_and_version(sq):
    assert sq.sq_version() >= 100
    assert [sq.status_string(i) for i in range(4)] == ["SQ_OK", "SQ_ERR_INVALID_ARG", "SQ_ERR_UNSUPPORTED", "SQ_ERR_LAUNCH"]


def test_tuning_hook_validation(sq):
    sq.sq_tuning_set("gemm_variant", -1)
    sq.sq_tuning_set("force_path", -1)
    for key, val in (("gemm_variant", 99), ("force_path", 7), ("no_such_key", 0)):
        with pytest.raises(sq.SqError) as e:
            sq.sq_tuning_set(key, val)
        assert e.value.status == 1


def _layer(sq, **kw):
    d = dict(M=8, K=128, N=16, kseg_off=[0, 128], nseg_off=[0, 16], dual=[1], s_pos=[0.5], s_neg=[0.25], seg_scale=None)
    d.update(kw)
    return sq.Layer(d["M"], d["K"], d["N"], d["kseg_off"], d["nseg_off"], d["dual"], d["s_pos"], d["s_neg"], d["seg_scale"])


FAKE = C.c_void_p(0x1000)      # never dereferenced: every case below is rejected on the host


def _act(sq, layer, x=FAKE, dt=1, xq=FAKE):
    return sq.load_library().sq_quantize_act(C.byref(layer.c), x, dt, xq, None)


def _gemm(sq, layer, xq=FAKE, wq=FAKE, ws=FAKE, y=FAKE, dt=0):
    return sq.load_library().sq_seglinear(C.byref(layer.c), xq, wq, ws, None, y, dt, None)


def test_invalid_arguments_are_rejected_on_the_host(sq):
    INVALID, UNSUPPORTED = 1, 2
    lib = sq.load_library()
    ok = _layer(sq)
    assert _act(sq, ok, x=None) == INVALID
    assert _act(sq, ok, xq=None) == INVALID
    assert _act(sq, ok, dt=5) == INVALID
    assert lib.sq_quantize_act(None, FAKE, 1, FAKE, None) == INVALID
    assert _act(sq, _layer(sq, kseg_off=[0, 64])) == INVALID      # off[S] != K
    assert _act(sq, _layer(sq, kseg_off=[0, 64, 64, 128], dual=[1, 1, 1], s_pos=[1, 1, 1], s_neg=[1, 1, 1])) == INVALID
    assert _act(sq, _layer(sq, nseg_off=[0, 8, 4, 16])) == INVALID
    assert _act(sq, _layer(sq, kseg_off=[1, 128])) == INVALID
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        assert _act(sq, _layer(sq, s_pos=[bad])) == INVALID
        assert _act(sq, _layer(sq, s_neg=[bad])) == INVALID
    assert _act(sq, _layer(sq, M=0)) == INVALID
    assert _gemm(sq, ok, wq=None) == INVALID
    assert _gemm(sq, ok, y=None) == INVALID
    assert _gemm(sq, ok, dt=9) == INVALID
    assert _gemm(sq, _layer(sq, seg_scale=[[float("nan")]])) == INVALID
    # legal but outside the documented limits
    n = 65
    many = _layer(sq, K=64 * n, kseg_off=[64 * i for i in range(n + 1)], dual=[0] * n, s_pos=[1.0] * n, s_neg=[1.0] * n)
    assert _act(sq, many) == UNSUPPORTED
    long_seg = _layer(sq, K=133144, kseg_off=[0, 133144])
    assert _gemm(sq, long_seg) == UNSUPPORTED                     # 127*127*K_ks would not fit int32
    big = _layer(sq, M=70000, K=40000, N=16, kseg_off=[0, 40000])
    assert _act(sq, big) == UNSUPPORTED                           # M*K >= 2^31
    s, t = 32, 32
    blocks = _layer(sq, K=64 * s, N=t, kseg_off=[64 * i for i in range(s + 1)], nseg_off=list(range(t + 1)), dual=[0] * s,
                    s_pos=[1.0] * s, s_neg=[1.0] * s, seg_scale=np.ones((s, t), np.float32))
    assert _gemm(sq, blocks) == UNSUPPORTED                       # S*T > SQ_MAX_SEG_SCALE
    w = _layer(sq)
    assert lib.sq_quantize_weight(C.byref(w.c), None, 0, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_weight(C.byref(w.c), FAKE, 3, FAKE, FAKE, None) == INVALID
    assert lib.sq_seglinear_debug_acc(C.byref(w.c), FAKE, FAKE, FAKE, None, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_block(C.byref(w.c), None, 0, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_block(C.byref(w.c), FAKE, 0, FAKE, None, None) == INVALID
    assert lib.sq_calibrate_act(C.byref(ok.c), None, 1, FAKE, FAKE, 0, None) == INVALID
    assert lib.sq_calibrate_act(C.byref(ok.c), FAKE, 1, None, FAKE, 0, None) == INVALID
    assert lib.sq_calibrate_act(C.byref(ok.c), FAKE, 4, FAKE, FAKE, 0, None) == INVALID
    codes = (C.c_int32 * 1)(1)
    fused = lambda h=FAKE, act=codes, ws=None, nbytes=0: lib.sq_quantize_act_fused(C.byref(ok.c), h, 1, act, FAKE, ws, nbytes, None)
    assert fused(act=None) == INVALID and fused(h=None) == INVALID
    assert fused(act=(C.c_int32 * 1)(3)) == INVALID and fused(act=(C.c_int32 * 1)(-1)) == INVALID
    wneed = lib.sq_quantize_act_fused_workspace_bytes(C.byref(ok.c))
    assert wneed == 65536 * ok.c.S and lib.sq_quantize_act_fused_workspace_bytes(None) == 0
    assert fused(ws=FAKE, nbytes=wneed - 1) == INVALID and fused(ws=C.c_void_p(0x1008), nbytes=wneed) == INVALID
    w4 = _layer(sq, K=256, kseg_off=[0, 256])
    assert lib.sq_quantize_weight_w4(C.byref(w4.c), None, 0, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_w4(C.byref(w4.c), FAKE, 0, FAKE, None, None) == INVALID
    assert lib.sq_seglinear_w4(C.byref(w4.c), FAKE, None, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_w4(C.byref(w4.c), FAKE, FAKE, FAKE, None, FAKE, 9, None) == INVALID
    assert lib.sq_seglinear_w4_debug_acc(C.byref(w4.c), FAKE, FAKE, None, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_w4(C.byref(ok.c), FAKE, 0, FAKE, FAKE, None) in (UNSUPPORTED, INVALID) or ok.c.K % 128 == 0
    assert lib.sq_quantize_act_dynamic(C.byref(ok.c), FAKE, 1, FAKE, None, None) == INVALID
    assert lib.sq_quantize_act_dynamic(C.byref(ok.c), None, 1, FAKE, FAKE, None) == INVALID
    assert lib.sq_seglinear_dynamic(C.byref(ok.c), FAKE, None, FAKE, 8, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_dynamic(C.byref(ok.c), FAKE, FAKE, FAKE, 5, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_dynamic(C.byref(_layer(sq, K=192, kseg_off=[0, 192]).c), FAKE, FAKE, FAKE, 4, FAKE, None, FAKE, 0, None) == UNSUPPORTED
    need = lib.sq_calibrate_workspace_bytes()
    assert 0 < need < (1 << 20)
    pct = lambda p, ws=FAKE, nbytes=need, x=FAKE: lib.sq_calibrate_act_percentile(C.byref(ok.c), x, 1, p, FAKE, FAKE, ws, nbytes, 0, None)
    assert pct(0.0) == INVALID and pct(1.5) == INVALID and pct(float("nan")) == INVALID and pct(-0.5) == INVALID
    assert pct(0.999, ws=None) == INVALID and pct(0.999, nbytes=need - 1) == INVALID and pct(0.999, x=None) == INVALID
    # grouped call: NULL item table, empty group, oversized group, NULL member, per-block multiplier
    from paper_2507_14811_amd.binding import sq_group_item
    one = (sq_group_item * 1)(sq_group_item(0x1000, 0x1000, None, 0x1000))
    assert lib.sq_seglinear_grouped(C.byref(ok.c), FAKE, 1, None, 0, None) == INVALID
    assert lib.sq_seglinear_grouped(C.byref(ok.c), FAKE, 0, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped(C.byref(ok.c), FAKE, 65, one, 0, None) == UNSUPPORTED
    bad = (sq_group_item * 1)(sq_group_item(0x1000, None, None, 0x1000))
    assert lib.sq_seglinear_grouped(C.byref(ok.c), FAKE, 1, bad, 0, None) == INVALID
    assert lib.sq_seglinear_grouped(C.byref(_layer(sq, seg_scale=[[1.0]]).c), FAKE, 1, one, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_grouped(C.byref(ok.c), FAKE, 1, one, 7, None) == INVALID
    assert lib.sq_quantize_act_geglu(C.byref(ok.c), None, 1, FAKE, None) == INVALID
    assert lib.sq_quantize_act_geglu(C.byref(ok.c), FAKE, 1, None, None) == INVALID
    assert lib.sq_quantize_act_geglu(C.byref(ok.c), FAKE, 9, FAKE, None) == INVALID
    assert lib.sq_quantize_act_geglu(C.byref(_layer(sq, s_pos=[0.0]).c), FAKE, 1, FAKE, None) == INVALID
    # raw-activation entry points: NULL input, unknown dtype, unknown activation code, shapes the stream kernel cannot run
    codes = lambda *a: (C.c_int32 * len(a))(*a)
    assert lib.sq_seglinear_fused(C.byref(ok.c), None, 1, None, FAKE, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_fused(C.byref(ok.c), FAKE, 5, None, FAKE, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_fused(C.byref(ok.c), FAKE, 1, codes(3), FAKE, FAKE, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_fused(C.byref(ok.c), FAKE, 1, codes(1), FAKE, None, None, FAKE, 0, None) == INVALID
    assert lib.sq_seglinear_fused(C.byref(_layer(sq, K=192, kseg_off=[0, 192]).c), FAKE, 1, codes(1), FAKE, FAKE, None, FAKE, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_fused(C.byref(_layer(sq, M=65).c), FAKE, 1, codes(1), FAKE, FAKE, None, FAKE, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_fused(C.byref(ok.c), C.c_void_p(0x1004), 0, None, FAKE, FAKE, None, FAKE, 0, None) == UNSUPPORTED
    assert lib.sq_unpack_w4(C.byref(w4.c), None, FAKE, None) == INVALID and lib.sq_unpack_w4(C.byref(w4.c), FAKE, None, None) == INVALID
    assert lib.sq_unpack_w4(C.byref(_layer(sq, K=192, kseg_off=[0, 192]).c), FAKE, FAKE, None) == UNSUPPORTED
    assert lib.sq_unpack_w4(C.byref(w4.c), C.c_void_p(0x1008), FAKE, None) == UNSUPPORTED
    assert lib.sq_seglinear_grouped_w4(C.byref(w4.c), None, None, 1, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_w4(C.byref(w4.c), FAKE, None, 1, None, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_w4(C.byref(_layer(sq, K=192, kseg_off=[0, 192]).c), FAKE, None, 1, one, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_grouped_w4(C.byref(w4.c), FAKE, None, 65, one, 0, None) == UNSUPPORTED
    fd = lambda layer=ok, x=FAKE, dt=1, act=None, abits=8, wq=FAKE, bits=8, ws=FAKE, y=FAKE: lib.sq_seglinear_fused_dynamic(
        C.byref(layer.c), x, dt, act, abits, wq, bits, ws, None, y, 0, None)
    assert fd(x=None) == INVALID and fd(wq=None) == INVALID and fd(ws=None) == INVALID and fd(y=None) == INVALID
    assert fd(dt=7) == INVALID and fd(bits=5) == INVALID and fd(act=codes(9)) == INVALID and fd(abits=6) == INVALID
    assert lib.sq_quantize_act_dynamic_bits(C.byref(ok.c), FAKE, 1, 5, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_act_dynamic_bits(C.byref(ok.c), FAKE, 1, 4, FAKE, None, None) == INVALID
    assert fd(layer=_layer(sq, K=192, kseg_off=[0, 192])) == UNSUPPORTED and fd(layer=_layer(sq, M=65)) == UNSUPPORTED
    assert fd(layer=_layer(sq, K=192, kseg_off=[0, 192]), bits=4) == UNSUPPORTED
    nine = _layer(sq, K=128 * 9, kseg_off=[128 * i for i in range(10)], dual=[1] * 9, s_pos=[0.5] * 9, s_neg=[0.5] * 9)
    assert fd(layer=nine) == UNSUPPORTED
    assert lib.sq_seglinear_grouped_fused(C.byref(ok.c), None, 1, None, 1, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_fused(C.byref(ok.c), FAKE, 7, None, 1, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_fused(C.byref(ok.c), FAKE, 1, codes(-1), 1, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_fused(C.byref(ok.c), FAKE, 1, None, 65, one, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_grouped_fused(C.byref(_layer(sq, M=40).c), FAKE, 1, None, 1, one, 0, None) == UNSUPPORTED


def test_invalid_arguments_of_the_optimizer_side_and_fp8_entry_points(sq):
    """Smoothing, low-rank branch, fp8 variant, allocation-free calibration: rejected on the host before anything is
    launched (no GPU needed)."""
    INVALID, UNSUPPORTED = 1, 2
    lib = sq.load_library()
    ok = _layer(sq)                                               # K = 128
    c = lambda l: C.byref(l.c)
    # per-channel maxima and smoothed quantizers
    assert lib.sq_calibrate_channel_amax(c(ok), None, 1, FAKE, 0, None) == INVALID
    assert lib.sq_calibrate_channel_amax(c(ok), FAKE, 1, None, 0, None) == INVALID
    assert lib.sq_calibrate_channel_amax(c(ok), FAKE, 6, FAKE, 0, None) == INVALID
    assert lib.sq_weight_channel_amax(c(ok), None, 0, FAKE, None) == INVALID
    assert lib.sq_weight_channel_amax(c(ok), FAKE, 0, None, None) == INVALID
    assert lib.sq_smooth_factors(c(ok), None, FAKE, FAKE, FAKE, FAKE) == INVALID
    assert lib.sq_smooth_factors(c(ok), FAKE, FAKE, None, FAKE, FAKE) == INVALID
    assert lib.sq_quantize_weight_smoothed(c(ok), FAKE, 0, None, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_smoothed(c(ok), FAKE, 4, FAKE, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_act_smoothed(c(ok), FAKE, 1, None, FAKE, None) == INVALID
    assert lib.sq_quantize_act_smoothed(c(ok), None, 1, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_act_smoothed(c(_layer(sq, s_pos=[0.0])), FAKE, 1, FAKE, FAKE, None) == INVALID
    # low-rank side branch
    lr = lambda layer=ok, x=FAKE, dt=1, ld=FAKE, lu=FAKE, rank=64, y=FAKE, ydt=1, ws=FAKE, nbytes=1 << 30: lib.sq_lowrank_add(
        c(layer), x, dt, ld, lu, rank, None, y, ydt, ws, nbytes, None)
    assert lr(x=None) == INVALID and lr(ld=None) == INVALID and lr(lu=None) == INVALID and lr(y=None) == INVALID
    assert lr(ws=None) == INVALID and lr(dt=3) == INVALID and lr(ydt=7) == INVALID
    assert lr(rank=48) == UNSUPPORTED and lr(rank=0) == UNSUPPORTED
    assert lr(layer=_layer(sq, K=72, kseg_off=[0, 72])) == UNSUPPORTED                 # K not a multiple of 16
    assert lr(x=C.c_void_p(0x1004)) == INVALID                                       # 16-byte alignment
    need = lib.sq_lowrank_workspace_bytes(c(ok), 64)
    assert need > 0 and lr(nbytes=need - 1) == INVALID
    assert lib.sq_lowrank_workspace_bytes(c(ok), 48) == 0 and lib.sq_lowrank_workspace_bytes(None, 64) == 0
    # fp8 variant
    assert lib.sq_quantize_weight_fp8(c(ok), None, 0, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_weight_fp8(c(ok), FAKE, 0, FAKE, None, None) == INVALID
    assert lib.sq_quantize_weight_fp8(c(ok), FAKE, 2, FAKE, FAKE, None) == INVALID
    assert lib.sq_quantize_act_fp8(c(ok), None, 1, FAKE, None) == INVALID
    assert lib.sq_quantize_act_fp8(c(ok), FAKE, 1, None, None) == INVALID
    assert lib.sq_quantize_act_fp8(c(_layer(sq, s_neg=[float("nan")])), FAKE, 1, FAKE, None) == INVALID
    one_code = (C.c_int32 * 1)(1)
    assert lib.sq_quantize_act_fp8_fused(c(ok), FAKE, 1, None, FAKE, None, 0, None) == INVALID
    assert lib.sq_quantize_act_fp8_fused(c(ok), None, 1, one_code, FAKE, None, 0, None) == INVALID
    assert lib.sq_quantize_act_fp8_fused(c(ok), FAKE, 1, (C.c_int32 * 1)(3), FAKE, None, 0, None) == INVALID
    assert lib.sq_quantize_act_fp8_fused(c(ok), FAKE, 1, one_code, FAKE, FAKE, 65535, None) == INVALID
    assert lib.sq_quantize_act_fp8_fused(c(ok), FAKE, 1, one_code, FAKE, C.c_void_p(0x1008), 65536, None) == INVALID
    f8 = lambda layer=ok, xq=FAKE, wq=FAKE, ws=FAKE, y=FAKE, ydt=1: lib.sq_seglinear_fp8(c(layer), xq, wq, ws, None, y, ydt, None)
    assert f8(xq=None) == INVALID and f8(wq=None) == INVALID and f8(ws=None) == INVALID and f8(y=None) == INVALID
    assert f8(ydt=5) == INVALID
    assert f8(layer=_layer(sq, K=192, kseg_off=[0, 192])) == UNSUPPORTED             # K not a multiple of 128
    assert f8(layer=_layer(sq, K=256, kseg_off=[0, 64, 256], dual=[1, 0], s_pos=[1, 1], s_neg=[1, 1])) == UNSUPPORTED
    assert f8(xq=C.c_void_p(0x1008)) == UNSUPPORTED                                  # 16-byte alignment of the code matrices
    from paper_2507_14811_amd.binding import sq_group_item
    one = (sq_group_item * 1)(sq_group_item(0x1000, 0x1000, None, 0x1000))
    assert lib.sq_seglinear_grouped_fp8(c(ok), None, 1, one, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_fp8(c(ok), FAKE, 1, None, 0, None) == INVALID
    assert lib.sq_seglinear_grouped_fp8(c(ok), FAKE, 65, one, 0, None) == UNSUPPORTED
    assert lib.sq_seglinear_grouped_fp8(c(_layer(sq, M=40)), FAKE, 1, one, 0, None) == UNSUPPORTED
    # percentile calibration on the library's own scratch array
    assert 0 < lib.sq_calibrate_static_scratch_bytes() < (1 << 20)
    st = lambda p, x=FAKE, amax=FAKE, steps=FAKE: lib.sq_calibrate_act_percentile_static(c(ok), x, 1, p, amax, steps, 0, None)
    assert st(0.0) == INVALID and st(1.5) == INVALID and st(0.99, x=None) == INVALID and st(0.99, amax=None) == INVALID


def test_missing_library_fails_loudly(monkeypatch, sq):
    from paper_2507_14811_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libsegquant.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_binding_wrappers_are_well_formed():
    """Every wrapper of the binding passes exactly (status, its own name) to _check, names a function the header declares,
    and every declared entry point has a wrapper or is listed in EXPORTS."""
    import ast
    import re

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = open(os.path.join(root, "paper_2507_14811_amd", "binding.py")).read()
    header = open(os.path.join(root, "include", "segquant.h")).read()
    declared = set(re.findall(r"\b(sq_[a-z0-9_]+)\s*\(", header))
    tree = ast.parse(src)
    seen = 0
    for fn in [n for n in ast.walk(tree) if isinstance(n, ast.FunctionDef)]:
        for call in [n for n in ast.walk(fn) if isinstance(n, ast.Call) and getattr(n.func, "id", None) == "_check"]:
            if fn.name in ("_check",):
                continue
            seen += 1
            assert len(call.args) == 2 and not call.keywords, fn.name
            name = call.args[1]
            assert isinstance(name, ast.Constant) and name.value == fn.name, (fn.name, ast.dump(name))
            assert fn.name in declared, fn.name
    assert seen >= 20
