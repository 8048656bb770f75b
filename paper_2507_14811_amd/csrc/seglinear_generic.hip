// SegLinear + DualScale GEMM for arbitrary shapes and alignments: one thread per output element.
// Used only when the tile kernels' alignment requirements do not hold (K not a multiple of 16 or a
// K-segment boundary not a multiple of 64).  Same arithmetic: exact int32 per-K-segment accumulators
// (Sec. 4.2.2 item 2), flushed to fp32 with the per-segment steps (Sec. 4.3.2, last display).
#include "sq_kernels.hpp"

namespace sq {

// W4: a.wq points at 4-bit codes packed two per byte, one KiB per (16-row group g, 128-code step t), T = K / 128:
// byte ((g T + t) 16 + r) 64 + j holds code(16 g + r, 128 t + j) (low nibble) and code(16 g + r, 128 t + 64 + j) (high
// nibble), 4-bit two's complement.
template <int MODE, bool W4>
__global__ __launch_bounds__(256) void seglinear_generic_kernel(const GemmArgs a, const GemmTable tb) {
  const int n = blockIdx.y * 64 + (threadIdx.x & 63);
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= a.N || m >= a.M) return;
  const int8_t* xr = a.xq + (size_t)m * a.K;
  const int8_t* wr = W4 ? a.wq + ((size_t)(n >> 4) * (a.K >> 7) * 16 + (n & 15)) * 64 : a.wq + (size_t)n * a.K;
  float y = 0.0f;
  for (int ks = 0; ks < tb.S; ++ks) {
    const bool dual = tb.dual[ks] != 0;
    int ap = 0, an = 0;
    for (int k = tb.kseg_off[ks]; k < tb.kseg_off[ks + 1]; ++k) {
      int wv;
      if (W4) {
        const int byte = wr[((size_t)(k >> 7) << 10) + (k & 63)];   // sign-extended byte: the high nibble keeps its sign
        wv = (k & 64) ? (byte >> 4) : ((int)((unsigned)byte << 28) >> 28);
      } else {
        wv = wr[k];
      }
      const int xv = xr[k];
      if (dual && xv < 0) an += xv * wv;       // X^_- = min(X^, 0): negative codes belong to the s_- path
      else ap += xv * wv;
    }
    if (MODE == OUT_DEBUG_ACC) {
      const size_t o = ((size_t)ks * a.M + m) * a.N + n;
      a.acc_pos[o] = ap;
      a.acc_neg[o] = an;
    } else {
      const float c = seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n];
      float sp = tb.s_pos[ks], sn = tb.s_neg[ks];
      if (a.tok_steps) {                                            // dynamic per-token steps
        sp = a.tok_steps[(size_t)m * tb.S + ks];
        sn = a.tok_steps[((size_t)a.M + m) * tb.S + ks];
      }
      float t = sp * (float)ap;
      if (dual) t += sn * (float)an;
      y += c * t;
    }
  }
  if (MODE != OUT_DEBUG_ACC) {
    if (a.bias) y += a.bias[n];
    const size_t o = (size_t)m * a.N + n;
    if (MODE == OUT_F32) reinterpret_cast<float*>(a.y)[o] = y;
    else reinterpret_cast<uint16_t*>(a.y)[o] = f32_to_bf16(y);
  }
}

template <bool W4>
static hipError_t launch_generic_impl(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st) {
  dim3 grid((a.M + 3) / 4, (a.N + 63) / 64);
  if (mode == OUT_F32) hipLaunchKernelGGL((seglinear_generic_kernel<OUT_F32, W4>), grid, dim3(256), 0, st, a, tb);
  else if (mode == OUT_BF16) hipLaunchKernelGGL((seglinear_generic_kernel<OUT_BF16, W4>), grid, dim3(256), 0, st, a, tb);
  else hipLaunchKernelGGL((seglinear_generic_kernel<OUT_DEBUG_ACC, W4>), grid, dim3(256), 0, st, a, tb);
  return hipGetLastError();
}

hipError_t launch_seglinear_generic(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st) {
  return launch_generic_impl<false>(a, tb, mode, st);
}

hipError_t launch_seglinear_generic_w4(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st) {
  return launch_generic_impl<true>(a, tb, mode, st);
}

}  // namespace sq
