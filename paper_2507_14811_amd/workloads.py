"""Seeded synthetic inputs for the SegLinear + DualScale quantized linear layer.

This module only *generates data*: activations, weights, segment offsets, the
per-K-segment dual flags and the static activation scales that both the HIP
library and the CPU oracle receive as inputs.  It contains none of the
quantize / GEMM / dequant arithmetic and imports neither of the two.

The five named layer shapes stand in for the layer kinds the paper quantizes
(Sec. 4.2.2: output-segmented adaLN / fused QKV, input-segmented concat
projection; Sec. 4.3: SiLU / GELU inputs with a narrow negative range, see the
activation statistics table of Sec. 4.3.1).  All tensors come from
``numpy.random.default_rng(seed)``.

Static activation scales follow the calibration rule of Sec. 4.3.2 (min / max
of the tensor over the quantization range) with the symmetric 8-bit range
[-127, 127]:  s_pos = max(x) / 127 and s_neg = |min(x)| / 127 per K-segment for
a dual segment, absmax / 127 for a single-scale segment; a polarity that never
occurs gets scale 1.0.  They are evaluated on the values the kernels see (after
rounding to bf16 where the layer input is bf16).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

QMAX = 127.0


# ----------------------------------------------------------------------------
# bf16 helpers (data preparation only: round-to-nearest-even on the fp32 bits)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns (RNE, finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 values (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _silu(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.float64)
    return z / (1.0 + np.exp(-z))


def _gelu(z: np.ndarray) -> np.ndarray:
    from scipy.special import erf  # exact erf form, evaluated in float64

    z = z.astype(np.float64)
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


# ----------------------------------------------------------------------------
@dataclass
class Workload:
    """One synthetic layer: everything `sq_*` calls and the oracle take as input."""

    name: str
    M: int
    K: int
    N: int
    kseg_off: np.ndarray          # int32 [S+1]
    nseg_off: np.ndarray          # int32 [T+1]
    dual: np.ndarray              # uint8 [S]
    x: np.ndarray                 # fp32 [M][K] (bf16-representable when x_dtype == "bf16")
    x_dtype: str                  # "bf16" | "f32"
    w: np.ndarray                 # fp32 [N][K]
    s_pos: np.ndarray             # fp32 [S]
    s_neg: np.ndarray             # fp32 [S]
    seg_scale: Optional[np.ndarray] = None   # fp32 [S][T] or None (= all ones)
    bias: Optional[np.ndarray] = None        # fp32 [N] or None
    y_dtype: str = "bf16"
    seed: int = 0
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def S(self) -> int:
        return len(self.kseg_off) - 1

    @property
    def T(self) -> int:
        return len(self.nseg_off) - 1

    @property
    def keff(self) -> int:
        """Sum over K-segments of K_ks * (1 + dual_ks): executed K per output element."""
        ks = np.diff(self.kseg_off).astype(np.int64)
        return int(np.sum(ks * (1 + self.dual.astype(np.int64))))

    @property
    def int8_ops(self) -> int:
        """Executed int8 ops, both polarity paths counted, skipped x- work not counted."""
        return 2 * self.M * self.N * self.keff

    def x_bf16_bits(self) -> np.ndarray:
        assert self.x_dtype == "bf16"
        return f32_to_bf16_bits(self.x)

    def quantize_act_bytes(self) -> int:
        """Algorithmic HBM bytes of the activation quantize pass: the input once, one code byte out
        (both polarity matrices travel in one int8 array: X^ = X^_+ + X^_-)."""
        in_b = 2 if self.x_dtype == "bf16" else 4
        return int(self.M * self.K * (in_b + 1))

    def seglinear_bytes(self, y_dtype: Optional[str] = None) -> int:
        """Compulsory HBM bytes of the GEMM: the merged codes X^ once, W^ once, scales, Y once."""
        yb = 2 if (y_dtype or self.y_dtype) == "bf16" else 4
        return int(self.M * self.K + self.N * self.K + 4 * self.S * self.N + self.M * self.N * yb)


def amax_scales(x: np.ndarray, kseg_off, dual):
    """Static per-K-segment activation scales (Sec. 4.3.2 calibration rule, p = 1.0)."""
    S = len(kseg_off) - 1
    s_pos = np.ones(S, dtype=np.float32)
    s_neg = np.ones(S, dtype=np.float32)
    q = np.float32(QMAX)
    for ks in range(S):
        blk = x[:, kseg_off[ks]:kseg_off[ks + 1]]
        if dual[ks]:
            hi = np.float32(max(float(blk.max()), 0.0))
            lo = np.float32(max(float(-blk.min()), 0.0))
            if hi > 0:
                s_pos[ks] = hi / q
            if lo > 0:
                s_neg[ks] = lo / q
        else:
            a = np.float32(np.abs(blk).max())
            if a > 0:
                s_pos[ks] = a / q
    return s_pos, s_neg


def _finish(name, x, x_dtype, w, kseg, nseg, dual, seed, y_dtype, notes="", **extra) -> Workload:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x_dtype == "bf16":
        x = bf16_bits_to_f32(f32_to_bf16_bits(x))
    w = np.ascontiguousarray(w, dtype=np.float32)
    kseg = np.asarray(kseg, dtype=np.int32)
    nseg = np.asarray(nseg, dtype=np.int32)
    dual = np.asarray(dual, dtype=np.uint8)
    s_pos, s_neg = amax_scales(x, kseg, dual)
    M, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K and kseg[-1] == K and nseg[-1] == N
    return Workload(name, M, K, N, kseg, nseg, dual, x, x_dtype, w, s_pos, s_neg,
                    None, None, y_dtype, seed, notes, dict(extra))


# ----------------------------------------------------------------------------
# The five named configurations
# ----------------------------------------------------------------------------
def cfg1_tiny(seed: int = 0) -> Workload:
    """M=64, K=256 in 2 dual K-segments, N=384 in 3 N-segments; fp32 SiLU input."""
    rng = np.random.default_rng(seed)
    x = _silu(rng.standard_normal((64, 256)))
    w = rng.standard_normal((384, 256)) * 0.02
    return _finish("cfg1_tiny", x, "f32", w, [0, 128, 256], [0, 128, 256, 384], [1, 1], seed, "f32",
                   "correctness only")


def cfg2_dit_fc2(seed: int = 2) -> Workload:
    """DiT MLP fc2: M=2048, K=4608 one dual segment on GELU input, N=1152."""
    rng = np.random.default_rng(seed)
    x = _gelu(rng.standard_normal((2048, 4608), dtype=np.float32))
    w = rng.standard_normal((1152, 4608), dtype=np.float32) * np.float32(0.02)
    return _finish("cfg2_dit_fc2", x, "bf16", w, [0, 4608], [0, 1152], [1], seed, "bf16")


def cfg3_adaln(seed: int = 3) -> Workload:
    """adaLN modulation: M=16, K=1152 dual SiLU input, N=6x1152 with per-N-segment weight std."""
    rng = np.random.default_rng(seed)
    x = _silu(rng.standard_normal((16, 1152), dtype=np.float32))
    sig = np.array([0.01, 0.02, 0.05, 0.1, 0.2, 0.5])[rng.permutation(6)]
    w = rng.standard_normal((6912, 1152), dtype=np.float32)
    for j in range(6):
        w[j * 1152:(j + 1) * 1152] *= np.float32(sig[j])
    return _finish("cfg3_adaln", x, "bf16", w, [0, 1152], [1152 * j for j in range(7)], [1], seed, "bf16",
                   sigma=sig.tolist())


def cfg3_stacked(seed: int = 33, layers: int = 28) -> Workload:
    """The adaLN modulation linears of all `layers` blocks of a DiT stacked along N into one call: they share
    the conditioning input (M=16, K=1152, SiLU), so the stack is one skinny layer with N = layers x 6 x 1152
    (223 MB of int8 weights for 28 blocks) and one N-segment per block.  Chunk-wise weight std as in cfg3."""
    rng = np.random.default_rng(seed)
    x = _silu(rng.standard_normal((16, 1152), dtype=np.float32))
    n_layer = 6 * 1152
    w = rng.standard_normal((layers * n_layer, 1152), dtype=np.float32)
    base = np.array([0.01, 0.02, 0.05, 0.1, 0.2, 0.5])
    for l in range(layers):
        sig = base[rng.permutation(6)]
        for j in range(6):
            w[l * n_layer + j * 1152:l * n_layer + (j + 1) * 1152] *= np.float32(sig[j])
    return _finish(f"cfg3_stacked_x{layers}", x, "bf16", w, [0, 1152], [n_layer * l for l in range(layers + 1)], [1], seed,
                   "bf16")


def cfg4_qkv(seed: int = 4, dual: bool = False) -> Workload:
    """Fused QKV: M=8500 ragged, K=1536 single segment with 15 outlier channels x20, N=3x1536."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((8500, 1536), dtype=np.float32)
    ch = rng.permutation(1536)[:15]
    x[:, ch] *= np.float32(20.0)
    w = rng.standard_normal((4608, 1536), dtype=np.float32) * np.float32(0.02)
    return _finish("cfg4d_qkv_dual" if dual else "cfg4_qkv", x, "bf16", w, [0, 1536],
                   [0, 1536, 3072, 4608], [1 if dual else 0], seed, "bf16", outlier_channels=sorted(ch.tolist()))


def cfg5_outproj(seed: int = 5) -> Workload:
    """Single-stream out-proj: M=4608, K = 3072 (attention out, single scale) + 12288 (GELU, dual), N=3072."""
    rng = np.random.default_rng(seed)
    x = np.empty((4608, 15360), dtype=np.float32)
    x[:, :3072] = rng.standard_normal((4608, 3072), dtype=np.float32)
    x[:, 3072:] = _gelu(rng.standard_normal((4608, 12288), dtype=np.float32))
    w = rng.standard_normal((3072, 15360), dtype=np.float32) * np.float32(0.02)
    return _finish("cfg5_outproj", x, "bf16", w, [0, 3072, 15360], [0, 3072], [0, 1], seed, "bf16")


CONFIGS = {
    "cfg1": cfg1_tiny,
    "cfg2": cfg2_dit_fc2,
    "cfg3": cfg3_adaln,
    "cfg3x28": cfg3_stacked,
    "cfg4": cfg4_qkv,
    "cfg4d": lambda seed=4: cfg4_qkv(seed, dual=True),
    "cfg5": cfg5_outproj,
}


def make(name: str, **kw) -> Workload:
    return CONFIGS[name](**kw)


# ----------------------------------------------------------------------------
# Free-form layers for parity sweeps (ragged tails, many segments, edge cases)
# ----------------------------------------------------------------------------
def random_layer(M, K, N, kseg_off, nseg_off, dual, seed=0, x_dtype="bf16", y_dtype="f32",
                 act="silu", with_seg_scale=False, with_bias=False, w_std=0.02) -> Workload:
    """A seeded layer of arbitrary shape.  act: 'silu' | 'gelu' | 'normal' | 'relu' | 'neg'."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((M, K))
    if act == "silu":
        x = _silu(z)
    elif act == "gelu":
        x = _gelu(z)
    elif act == "relu":
        x = np.maximum(z, 0.0)
    elif act == "neg":
        x = -np.abs(z)
    else:
        x = z
    w = rng.standard_normal((N, K)) * w_std
    wl = _finish(f"rand_{M}x{K}x{N}_s{seed}", x, x_dtype, w, kseg_off, nseg_off, dual, seed, y_dtype)
    if with_seg_scale:
        wl.seg_scale = rng.uniform(0.5, 2.0, size=(wl.S, wl.T)).astype(np.float32)
    if with_bias:
        wl.bias = rng.standard_normal(N).astype(np.float32)
    return wl
