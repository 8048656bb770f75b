"""numpy front-end of the plain-C CPU oracle (test infrastructure only).

Argument marshalling, with two exceptions that are plain numpy here and say so where they stand: the GEGLU product
(one fp32 multiplication per element) and the per-token steps of the dynamic rule with 4-bit activation codes (row
extremes divided by q_max = 7).  Every other arithmetic step is in ``segquant_oracle.c`` next to this file.  ``build()`` compiles it with gcc; the shared object is
loaded lazily and rebuilt when the source is newer.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "segquant_oracle.c")
_SO = os.path.join(_HERE, "libsegquant_oracle.so")
_lib = None

_CFLAGS = ["-O3", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-frounding-math",
           "-fPIC", "-shared", "-Wall"]


def build(force: bool = False) -> str:
    """Compile the oracle (gcc).  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        _lib.sqo_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return int(_load().sqo_num_threads())


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    _load().sqo_widen_bf16(_p(bits), C.c_int64(bits.size), _p(out))
    return out


def cast_bf16(y: np.ndarray) -> np.ndarray:
    y = _f32(y)
    out = np.empty(y.shape, dtype=np.uint16)
    _load().sqo_cast_bf16(_p(y), C.c_int64(y.size), _p(out))
    return out


def quantize_weight(w: np.ndarray, kseg_off):
    """-> (wq int8 [N][K], wscale fp32 [S][N])"""
    w = _f32(w)
    N, K = w.shape
    off = _i32(kseg_off)
    S = len(off) - 1
    wq = np.empty((N, K), dtype=np.int8)
    ws = np.empty((S, N), dtype=np.float32)
    _check(_load().sqo_quantize_weight(_p(w), N, K, S, _p(off), _p(wq), _p(ws)), "quantize_weight")
    return wq, ws


def quantize_weight_w4(w: np.ndarray, kseg_off):
    """4-bit weights per output channel and K-segment (q_max = 7) -> (wq int8 [N][K] in [-7, 7], wscale fp32 [S][N])"""
    w = _f32(w)
    N, K = w.shape
    off = _i32(kseg_off)
    S = len(off) - 1
    wq = np.empty((N, K), dtype=np.int8)
    ws = np.empty((S, N), dtype=np.float32)
    _check(_load().sqo_quantize_weight_w4(_p(w), N, K, S, _p(off), _p(wq), _p(ws)), "quantize_weight_w4")
    return wq, ws


def pack_w4(wq: np.ndarray):
    """int8 codes [N][K] in [-8, 7] -> the packed storage format, uint8 [ceil(N/16) * 16 * K/2] (16-row groups,
    128-code steps, one KiB per (group, step))"""
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    N, K = wq.shape
    out = np.empty((((N + 15) // 16) * 16 * (K // 2),), dtype=np.uint8)
    _check(_load().sqo_pack_w4(_p(wq), N, K, _p(out)), "pack_w4")
    return out


def quantize_weight_block(w: np.ndarray, kseg_off, nseg_off):
    """One step per (K-segment, N-segment) block -> (wq int8 [N][K], wscale fp32 [S][N], constant inside a block)"""
    w = _f32(w)
    N, K = w.shape
    koff, noff = _i32(kseg_off), _i32(nseg_off)
    S, T = len(koff) - 1, len(noff) - 1
    wq = np.empty((N, K), dtype=np.int8)
    ws = np.empty((S, N), dtype=np.float32)
    _check(_load().sqo_quantize_weight_block(_p(w), N, K, S, _p(koff), T, _p(noff), _p(wq), _p(ws)),
           "quantize_weight_block")
    return wq, ws


def calibrate_act(x: np.ndarray, kseg_off, dual, running=None):
    """Min/max calibration of the activation steps.  running: (amax_pos, amax_neg) of earlier batches or None.
    -> (s_pos, s_neg, amax_pos, amax_neg), fp32 [S] each."""
    x = _f32(x)
    M, K = x.shape
    off, dual = _i32(kseg_off), _u8(dual)
    S = len(off) - 1
    if running is None:
        ap, an, acc = np.zeros(S, np.float32), np.zeros(S, np.float32), 0
    else:
        ap, an, acc = _f32(running[0]).copy(), _f32(running[1]).copy(), 1
    sp, sn = np.empty(S, np.float32), np.empty(S, np.float32)
    _check(_load().sqo_calibrate_act(_p(x), M, K, S, _p(off), _p(dual), acc, _p(ap), _p(an), _p(sp), _p(sn)),
           "calibrate_act")
    return sp, sn, ap, an


def calibrate_act_percentile(x: np.ndarray, kseg_off, dual, p: float, running=None):
    """Percentile-clipping calibration of the activation steps (nearest-rank p-quantile of max(X,0), max(-X,0) or |X|
    per K-segment and batch, running maximum over batches).  -> (s_pos, s_neg, amax_pos, amax_neg), fp32 [S] each."""
    x = _f32(x)
    M, K = x.shape
    off, dual = _i32(kseg_off), _u8(dual)
    S = len(off) - 1
    if running is None:
        ap, an, acc = np.zeros(S, np.float32), np.zeros(S, np.float32), 0
    else:
        ap, an, acc = _f32(running[0]).copy(), _f32(running[1]).copy(), 1
    sp, sn = np.empty(S, np.float32), np.empty(S, np.float32)
    f = _load().sqo_calibrate_act_percentile
    f.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_double, C.c_int,
                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(f(_p(x), M, K, S, _p(off), _p(dual), float(p), acc, _p(ap), _p(an), _p(sp), _p(sn)),
           "calibrate_act_percentile")
    return sp, sn, ap, an


def quantize_act(x: np.ndarray, kseg_off, dual, s_pos, s_neg):
    """x fp32 [M][K] (bf16 inputs are widened first) -> (xq_pos, xq_neg) int8 [M][K]"""
    x = _f32(x)
    M, K = x.shape
    off, dual, s_pos, s_neg = _i32(kseg_off), _u8(dual), _f32(s_pos), _f32(s_neg)
    S = len(off) - 1
    xp = np.empty((M, K), dtype=np.int8)
    xn = np.empty((M, K), dtype=np.int8)
    _check(_load().sqo_quantize_act(_p(x), M, K, S, _p(off), _p(dual), _p(s_pos), _p(s_neg), _p(xp), _p(xn)),
           "quantize_act")
    return xp, xn


ACT_NONE, ACT_SILU, ACT_GELU = 0, 1, 2


def activation(h: np.ndarray, kseg_off, act):
    """a = act_ks(h) per K-segment (0 none, 1 SiLU, 2 tanh-form GELU), in the bit-specified fp32 arithmetic."""
    h = _f32(h)
    M, K = h.shape
    off, act = _i32(kseg_off), _i32(act)
    a = np.empty((M, K), dtype=np.float32)
    _check(_load().sqo_activation(_p(h), M, K, len(off) - 1, _p(off), _p(act), _p(a)), "activation")
    return a


def quantize_act_fused(h: np.ndarray, kseg_off, dual, act, s_pos, s_neg):
    """h fp32 [M][K] pre-activation -> (xq_pos, xq_neg) int8 [M][K] of Q_dual(act(h))"""
    h = _f32(h)
    M, K = h.shape
    off, dual, act, s_pos, s_neg = _i32(kseg_off), _u8(dual), _i32(act), _f32(s_pos), _f32(s_neg)
    xp = np.empty((M, K), dtype=np.int8)
    xn = np.empty((M, K), dtype=np.int8)
    _check(_load().sqo_quantize_act_fused(_p(h), M, K, len(off) - 1, _p(off), _p(dual), _p(act), _p(s_pos), _p(s_neg),
                                          _p(xp), _p(xn)), "quantize_act_fused")
    return xp, xn


def geglu(h: np.ndarray) -> np.ndarray:
    """GEGLU in front of a DualScale layer (App. B names it next to SiLU and GELU): h fp32 [M][2K] = [value | gate]
    -> value * GELU(gate), fp32 [M][K].  GELU is the bit-specified tanh form of `activation`; the product is one
    IEEE fp32 multiplication (round to nearest even)."""
    h = _f32(h)
    M, K2 = h.shape
    if K2 % 2:
        raise ValueError("GEGLU input has an even number of columns")
    K = K2 // 2
    g = activation(np.ascontiguousarray(h[:, K:]), [0, K], [ACT_GELU])
    return (np.ascontiguousarray(h[:, :K]) * g).astype(np.float32)


def quantize_act_geglu(h: np.ndarray, kseg_off, dual, s_pos, s_neg):
    """h fp32 [M][2K] -> (xq_pos, xq_neg) int8 [M][K] of Q_dual(GEGLU(h)); the K-segments are those of the output."""
    return quantize_act(geglu(h), kseg_off, dual, s_pos, s_neg)


def int_gemm(xq_pos, xq_neg, wq, kseg_off, dual, rows=None):
    """-> (acc_pos, acc_neg) int32 [S][nrows][N]; rows = subset of token rows or None (all)."""
    xq_pos = np.ascontiguousarray(xq_pos, dtype=np.int8)
    xq_neg = np.ascontiguousarray(xq_neg, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    M, K = xq_pos.shape
    N = wq.shape[0]
    off, dual = _i32(kseg_off), _u8(dual)
    S = len(off) - 1
    r = None if rows is None else _i32(rows)
    nrows = M if r is None else len(r)
    ap = np.empty((S, nrows, N), dtype=np.int32)
    an = np.empty((S, nrows, N), dtype=np.int32)
    _check(_load().sqo_int_gemm(_p(xq_pos), _p(xq_neg), _p(wq), M, K, N, S, _p(off), _p(dual), nrows, _p(r),
                                _p(ap), _p(an)), "int_gemm")
    return ap, an


def dequant(acc_pos, acc_neg, nseg_off, dual, s_pos, s_neg, wscale, seg_scale=None, bias=None, want64=True):
    """-> (y32 fp32 [nrows][N], y64 double [nrows][N] or None)"""
    acc_pos = np.ascontiguousarray(acc_pos, dtype=np.int32)
    acc_neg = np.ascontiguousarray(acc_neg, dtype=np.int32)
    S, nrows, N = acc_pos.shape
    noff, dual, s_pos, s_neg, wscale = _i32(nseg_off), _u8(dual), _f32(s_pos), _f32(s_neg), _f32(wscale)
    T = len(noff) - 1
    g = None if seg_scale is None else _f32(seg_scale)
    b = None if bias is None else _f32(bias)
    y32 = np.empty((nrows, N), dtype=np.float32)
    y64 = np.empty((nrows, N), dtype=np.float64) if want64 else None
    _check(_load().sqo_dequant(_p(acc_pos), _p(acc_neg), nrows, N, S, T, _p(noff), _p(dual), _p(s_pos), _p(s_neg),
                               _p(wscale), _p(g), _p(b), _p(y32), _p(y64)), "dequant")
    return y32, y64


def fp_reference(x, w, rows=None, bias=None):
    x, w = _f32(x), _f32(w)
    M, K = x.shape
    N = w.shape[0]
    r = None if rows is None else _i32(rows)
    nrows = M if r is None else len(r)
    b = None if bias is None else _f32(bias)
    y = np.empty((nrows, N), dtype=np.float64)
    _check(_load().sqo_fp_reference(_p(x), _p(w), M, K, N, nrows, _p(r), _p(b), _p(y)), "fp_reference")
    return y


def error_bound(x, w, kseg_off, dual, s_pos, s_neg, wscale, rows=None):
    x, w = _f32(x), _f32(w)
    M, K = x.shape
    N = w.shape[0]
    off, dual, s_pos, s_neg, wscale = _i32(kseg_off), _u8(dual), _f32(s_pos), _f32(s_neg), _f32(wscale)
    S = len(off) - 1
    r = None if rows is None else _i32(rows)
    nrows = M if r is None else len(r)
    out = np.empty((nrows, N), dtype=np.float64)
    _check(_load().sqo_error_bound(_p(x), _p(w), M, K, N, S, _p(off), _p(dual), _p(s_pos), _p(s_neg), _p(wscale),
                                   nrows, _p(r), _p(out)), "error_bound")
    return out


@dataclass
class OracleResult:
    wq: np.ndarray
    wscale: np.ndarray
    xq_pos: np.ndarray
    xq_neg: np.ndarray
    rows: Optional[np.ndarray]
    acc_pos: np.ndarray
    acc_neg: np.ndarray
    y32: np.ndarray
    y64: Optional[np.ndarray]

    @property
    def y_bf16_bits(self) -> np.ndarray:
        return cast_bf16(self.y32)


def seglinear(x, w, kseg_off, nseg_off, dual, s_pos, s_neg, seg_scale=None, bias=None, rows=None, wbits=8) -> OracleResult:
    """The whole layer, step by step: Quant(W) (8-bit, or 4-bit codes when wbits == 4), Q_dual(X), integer GEMM, DeQuant."""
    wq, ws = quantize_weight(w, kseg_off) if wbits == 8 else quantize_weight_w4(w, kseg_off)
    xp, xn = quantize_act(x, kseg_off, dual, s_pos, s_neg)
    ap, an = int_gemm(xp, xn, wq, kseg_off, dual, rows)
    y32, y64 = dequant(ap, an, nseg_off, dual, s_pos, s_neg, ws, seg_scale, bias)
    return OracleResult(wq, ws, xp, xn, None if rows is None else np.asarray(rows), ap, an, y32, y64)


def quantize_act_dynamic(x, kseg_off, dual, abits: int = 8):
    """Dynamic per-token steps (App. B: in the 4-bit settings activations are quantized dynamically per token): every
    token row is calibrated on its own with the min/max rule (calibrate_act on that row) and quantized with its own
    steps.  abits: width of the activation codes, q_max = 2^(abits-1) - 1 (Sec. 3; 127, or 7 for 4-bit activations):
    steps = row extreme / q_max, codes clipped to [-q_max, q_max].
    -> (xq_pos, xq_neg int8 [M][K], s_pos, s_neg fp32 [M][S])"""
    x = _f32(x)
    M, K = x.shape
    S = len(kseg_off) - 1
    q = np.float32(2 ** (abits - 1) - 1)
    xp = np.empty((M, K), np.int8)
    xn = np.empty((M, K), np.int8)
    sp = np.empty((M, S), np.float32)
    sn = np.empty((M, S), np.float32)
    for m in range(M):
        sp[m], sn[m], ap, an = calibrate_act(x[m:m + 1], kseg_off, dual)
        if abits != 8:
            sp[m] = np.where(ap == 0, np.float32(1.0), ap / q)
            sn[m] = np.where(an == 0, np.float32(1.0), an / q)
        xp[m:m + 1], xn[m:m + 1] = quantize_act(x[m:m + 1], kseg_off, dual, sp[m], sn[m])
    return np.clip(xp, -int(q), int(q)), np.clip(xn, -int(q), int(q)), sp, sn


def seglinear_dynamic(x, w, kseg_off, nseg_off, dual, seg_scale=None, bias=None, wbits=8, abits=8) -> OracleResult:
    """The layer with dynamic per-token activation steps: the steps of the dequantization are those of the token."""
    wq, ws = quantize_weight(w, kseg_off) if wbits == 8 else quantize_weight_w4(w, kseg_off)
    xp, xn, sp, sn = quantize_act_dynamic(x, kseg_off, dual, abits)
    ap, an = int_gemm(xp, xn, wq, kseg_off, dual)
    M, N = x.shape[0], w.shape[0]
    y32 = np.empty((M, N), np.float32)
    y64 = np.empty((M, N), np.float64)
    for m in range(M):
        a, b = dequant(ap[:, m:m + 1], an[:, m:m + 1], nseg_off, dual, sp[m], sn[m], ws, seg_scale, bias)
        y32[m], y64[m] = a[0], b[0]
    r = OracleResult(wq, ws, xp, xn, None, ap, an, y32, y64)
    r.tok_steps = np.stack([sp, sn])            # [2][M][S]
    return r


def channel_amax(x: np.ndarray, running=None) -> np.ndarray:
    """max_m |X[m][k]| per input channel k (fp32 [K]), folded into `running` if given."""
    x = _f32(x)
    M, K = x.shape
    a = np.zeros(K, np.float32) if running is None else _f32(running).copy()
    _check(_load().sqo_channel_amax(_p(x), C.c_int(M), C.c_int(K), _p(a), C.c_int(0 if running is None else 1)),
           "channel_amax")
    return a


def smooth_factors(amax_x, amax_w, kseg_off, alpha):
    """SmoothQuant factors with one migration strength per K-segment: s[k] = a_x^alpha / a_w^(1 - alpha).
    -> (smooth fp32 [K], smooth_inv fp32 [K] = 1 / smooth)."""
    ax, aw, off, al = _f32(amax_x), _f32(amax_w), _i32(kseg_off), _f32(alpha)
    K, S = len(ax), len(off) - 1
    s, r = np.empty(K, np.float32), np.empty(K, np.float32)
    _check(_load().sqo_smooth_factors(_p(ax), _p(aw), C.c_int(K), C.c_int(S), _p(off), _p(al), _p(s), _p(r)), "smooth_factors")
    return s, r


def quantize_weight_smoothed(w: np.ndarray, kseg_off, smooth):
    """Quant(W diag(s)): -> (wq int8 [N][K], wscale fp32 [S][N])."""
    w, off, sm = _f32(w), _i32(kseg_off), _f32(smooth)
    N, K = w.shape
    S = len(off) - 1
    wq, ws = np.empty((N, K), np.int8), np.empty((S, N), np.float32)
    _check(_load().sqo_quantize_weight_smoothed(_p(w), C.c_int(N), C.c_int(K), C.c_int(S), _p(off), _p(sm), _p(wq), _p(ws)),
           "quantize_weight_smoothed")
    return wq, ws


def smooth_act(x: np.ndarray, smooth_inv) -> np.ndarray:
    """X diag(s)^-1 as one fp32 multiplication by r[k] = 1 / s[k] per element."""
    x, r = _f32(x), _f32(smooth_inv)
    M, K = x.shape
    out = np.empty((M, K), np.float32)
    _check(_load().sqo_smooth_act(_p(x), C.c_int(M), C.c_int(K), _p(r), _p(out)), "smooth_act")
    return out


def lowrank(x, ld, lu, y_q=None):
    """Low-rank side branch of the 4-bit settings: y = y_q + (X Ld^T) Lu^T, Ld [r][K], Lu [N][r], in double.
    -> (t fp64 [M][r], y fp64 [M][N])"""
    x, ld, lu = _f32(x), _f32(ld), _f32(lu)
    M, K = x.shape
    r, N = ld.shape[0], lu.shape[0]
    assert ld.shape == (r, K) and lu.shape == (N, r)
    yq = None if y_q is None else _f32(y_q)
    t, y = np.empty((M, r), np.float64), np.empty((M, N), np.float64)
    _check(_load().sqo_lowrank(_p(x), _p(ld), _p(lu), _p(yq), C.c_int(M), C.c_int(K), C.c_int(N), C.c_int(r), _p(t), _p(y)),
           "lowrank")
    return t, y


def fp8_encode(v) -> np.ndarray:
    """fp32 -> OCP E4M3 codes (uint8), nearest, ties to even, saturating at +-448."""
    v = _f32(v)
    out = np.empty(v.shape, np.uint8)
    _load().sqo_fp8_encode_array(_p(v), C.c_int64(v.size), _p(out))
    return out


def fp8_decode(c) -> np.ndarray:
    c = _u8(c)
    out = np.empty(c.shape, np.float32)
    _load().sqo_fp8_decode_array(_p(c), C.c_int64(c.size), _p(out))
    return out


def quantize_weight_fp8(w, kseg_off):
    """-> (wq uint8 [N][K] E4M3 codes, wscale fp32 [S][N] = max|w| / 448)"""
    w, off = _f32(w), _i32(kseg_off)
    N, K = w.shape
    S = len(off) - 1
    wq, ws = np.empty((N, K), np.uint8), np.empty((S, N), np.float32)
    _check(_load().sqo_quantize_weight_fp8(_p(w), C.c_int(N), C.c_int(K), C.c_int(S), _p(off), _p(wq), _p(ws)), "quantize_weight_fp8")
    return wq, ws


def quantize_act_fp8(x, kseg_off, dual, s_pos, s_neg):
    """Q_dual with E4M3 codes -> (xq_pos, xq_neg) uint8 [M][K]"""
    x, off, dual, sp, sn = _f32(x), _i32(kseg_off), _u8(dual), _f32(s_pos), _f32(s_neg)
    M, K = x.shape
    xp, xn = np.empty((M, K), np.uint8), np.empty((M, K), np.uint8)
    _check(_load().sqo_quantize_act_fp8(_p(x), C.c_int(M), C.c_int(K), C.c_int(len(off) - 1), _p(off), _p(dual), _p(sp), _p(sn),
                                        _p(xp), _p(xn)), "quantize_act_fp8")
    return xp, xn


def quantize_act_fp8_fused(h, kseg_off, dual, act, s_pos, s_neg):
    """Q_dual(act(h)) with E4M3 codes: the activation (bit-specified fp32, `activation`), then `quantize_act_fp8`."""
    return quantize_act_fp8(activation(h, kseg_off, act), kseg_off, dual, s_pos, s_neg)


def seglinear_fp8(xq_pos, xq_neg, wq, kseg_off, nseg_off, dual, s_pos, s_neg, wscale, seg_scale=None, bias=None):
    """The layer on E4M3 codes in double -> (y fp64 [M][N], mag fp64 [M][N] = the same sum over |terms|)"""
    xp, xn, wq = _u8(xq_pos), _u8(xq_neg), _u8(wq)
    M, K = xp.shape
    N = wq.shape[0]
    koff, noff, dual = _i32(kseg_off), _i32(nseg_off), _u8(dual)
    sp, sn, ws = _f32(s_pos), _f32(s_neg), _f32(wscale)
    sg = None if seg_scale is None else _f32(seg_scale)
    b = None if bias is None else _f32(bias)
    y, mag = np.empty((M, N), np.float64), np.empty((M, N), np.float64)
    _check(_load().sqo_seglinear_fp8(_p(xp), _p(xn), _p(wq), C.c_int(M), C.c_int(K), C.c_int(N), C.c_int(len(koff) - 1), _p(koff),
                                     C.c_int(len(noff) - 1), _p(noff), _p(dual), _p(sp), _p(sn), _p(ws), _p(sg), _p(b), _p(y), _p(mag)),
           "seglinear_fp8")
    return y, mag
