"""Helpers of the GPU parity tests: move a workload to the device, run it through the C ABI, fetch results."""
from __future__ import annotations

import numpy as np
import torch

import paper_2507_14811_amd as sq
from paper_2507_14811_amd import workloads as wl

DEV = "cuda:0"


def to_dev_x(w):
    if w.x_dtype == "bf16":
        bits = wl.f32_to_bf16_bits(w.x)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(w.x).to(DEV)


def bf16_tensor_bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


class GpuLayer:
    """Device buffers of one layer + calls through the binding."""

    def __init__(self, w, w_dtype="f32", poison=True):
        self.w = w
        self.layer = sq.Layer.from_workload(w)
        self.x = to_dev_x(w)
        if w_dtype == "bf16":
            self.wt = torch.from_numpy(wl.f32_to_bf16_bits(w.w).view(np.int16)).view(torch.bfloat16).to(DEV)
        else:
            self.wt = torch.from_numpy(w.w).to(DEV)
        fill = -77 if poison else 0
        self.wq = torch.full((w.N, w.K), fill, dtype=torch.int8, device=DEV)
        self.wscale = torch.full((w.S, w.N), float("nan"), dtype=torch.float32, device=DEV)
        self.xq = torch.full((w.M, w.K), fill, dtype=torch.int8, device=DEV)
        self.bias = None if w.bias is None else torch.from_numpy(w.bias).to(DEV)

    def quantize_weight(self):
        sq.sq_quantize_weight(self.layer, self.wt, self.wq, self.wscale)
        return self.wq.cpu().numpy(), self.wscale.cpu().numpy()

    def quantize_act(self):
        """Runs the activation quantizer; returns the library's polarity-merged codes unpacked into the two
        matrices of Sec. 4.3.2 (X^_+, X^_-) plus the raw merged array."""
        sq.sq_quantize_act(self.layer, self.x, self.xq)
        xq = self.xq.cpu().numpy()
        xp, xn = split_codes(self.w, xq)
        return xp, xn, xq

    def seglinear(self, y_dtype="f32"):
        w = self.w
        if y_dtype == "bf16":
            y = torch.full((w.M, w.N), float("nan"), dtype=torch.bfloat16, device=DEV)
        else:
            y = torch.full((w.M, w.N), float("nan"), dtype=torch.float32, device=DEV)
        sq.sq_seglinear(self.layer, self.xq, self.wq, self.wscale, self.bias, y)
        torch.cuda.synchronize()
        return bf16_tensor_bits(y) if y_dtype == "bf16" else y.cpu().numpy()

    def debug_acc(self):
        w = self.w
        ap = torch.full((w.S, w.M, w.N), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        an = torch.full((w.S, w.M, w.N), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        sq.sq_seglinear_debug_acc(self.layer, self.xq, self.wq, ap, an)
        torch.cuda.synchronize()
        return ap.cpu().numpy(), an.cpu().numpy()


def dual_col_mask(w) -> np.ndarray:
    """Columns that belong to DualScale K-segments."""
    m = np.zeros(w.K, dtype=bool)
    for ks in range(w.S):
        if w.dual[ks]:
            m[w.kseg_off[ks]:w.kseg_off[ks + 1]] = True
    return m


def split_codes(w, xq: np.ndarray):
    """Documented decoding of the merged activation codes: in a dual K-segment X^_+ = max(xq, 0) and
    X^_- = min(xq, 0); elsewhere X^_+ = xq and X^_- = 0 (index work only, none of the method's arithmetic)."""
    mask = dual_col_mask(w)
    xp = xq.copy()
    xn = np.zeros_like(xq)
    xp[:, mask] = np.maximum(xq[:, mask], 0)
    xn[:, mask] = np.minimum(xq[:, mask], 0)
    return xp, xn


def check_bf16_against(y_bits: np.ndarray, ref32: np.ndarray, ref_bits: np.ndarray, tol_abs: float):
    """bf16 outputs: bit-equal to bf16(oracle fp32) except where the fp32 tolerance straddles a rounding
    boundary.  A differing output must still be the bf16 rounding of some value within tol_abs of the
    oracle's fp32 result, i.e. |y - ref32| <= tol_abs + half a bf16 ulp of y; such cases must be rare."""
    neq = y_bits != ref_bits
    rate = float(neq.mean())
    if neq.any():
        yv = wl.bf16_bits_to_f32(y_bits[neq]).astype(np.float64)
        r32 = ref32[neq].astype(np.float64)
        half_ulp = np.abs(yv) * 2.0 ** -8
        assert (np.abs(yv - r32) <= tol_abs + half_ulp * (1 + 1e-6) + 1e-38).all(), \
            "bf16 output is not the rounding of a value within the fp32 tolerance"
    # rare: at most one output in a thousand (two in a small matrix, where a single straddle is already above that rate)
    assert int(neq.sum()) <= max(2, int(1e-3 * neq.size)), f"bf16 mismatch rate {rate}"
    return rate
