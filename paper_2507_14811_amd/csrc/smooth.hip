// Per-segment smoothing in front of the quantizers (Sec. 4.2.2, last paragraph: SegLinear shares SmoothQuant's
// migration strength alpha across a semantically coherent channel group; App. B: SmoothQuant is the optimizer of the
// 8-bit settings).  The published rule, one alpha per K-segment:
//   a_x[k] = max_m |X[m][k]| over the calibration batches,  a_w[k] = max_n |W[n][k]|,
//   s[k] = a_x[k]^alpha / a_w[k]^(1 - alpha),   X' = X diag(s)^-1,  W' = W diag(s).
// Device side: the per-channel maxima (one read of the matrix), the weight quantizer on W diag(s) and the activation
// quantizer on X diag(r), r = 1 / s.  The factors themselves (K numbers, swept over alpha by the caller) are a host
// computation in double precision.
#include <cmath>

#include "sq_kernels.hpp"

namespace sq {

// ---- per-column maxima of |a[r][k]|, r < R: rows are dealt to the workgroups' y index, columns to threads -----------
// Maxima are >= 0, so their fp32 bit patterns order like unsigned integers and workgroups combine with atomicMax.
constexpr int kColRows = 32;   // rows per workgroup

__global__ void channel_amax_init_kernel(float* __restrict__ amax, int K) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k < K) amax[k] = 0.0f;
}

template <bool BF16>
__global__ __launch_bounds__(256) void channel_amax_kernel(const void* __restrict__ a, int R, int K, float* __restrict__ amax) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= K) return;
  const int r0 = blockIdx.y * kColRows;
  const int r1 = (r0 + kColRows) < R ? (r0 + kColRows) : R;
  float m = 0.0f;
  for (int r = r0; r < r1; ++r) {
    const size_t i = (size_t)r * K + k;
    const float v = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(a)[i]) : reinterpret_cast<const float*>(a)[i];
    m = __builtin_fmaxf(m, __builtin_fabsf(v));
  }
  if (m > 0.0f) atomicMax(reinterpret_cast<unsigned int*>(amax) + k, __float_as_uint(m));
}

hipError_t launch_channel_amax(const void* a, bool is_bf16, int R, int K, float* amax, bool accumulate, hipStream_t st) {
  if (!accumulate) hipLaunchKernelGGL(channel_amax_init_kernel, dim3((K + 255) / 256), dim3(256), 0, st, amax, K);
  dim3 grid((K + 255) / 256, (R + kColRows - 1) / kColRows);
  if (is_bf16) hipLaunchKernelGGL(channel_amax_kernel<true>, grid, dim3(256), 0, st, a, R, K, amax);
  else hipLaunchKernelGGL(channel_amax_kernel<false>, grid, dim3(256), 0, st, a, R, K, amax);
  return hipGetLastError();
}

// ---- s[k] = a_x^alpha / a_w^(1 - alpha) per K-segment, on the host -------------------------------------------------
// A channel whose a_x or a_w is 0, or whose factor (or its reciprocal) is not a finite positive fp32 number, keeps 1.
void smooth_factors_host(const float* amax_x, const float* amax_w, int K, const KsegTable& tb, const float* alpha,
                         float* smooth, float* smooth_inv) {
  for (int ks = 0; ks < tb.S; ++ks) {
    const double al = (double)alpha[ks];
    for (int k = tb.off[ks]; k < tb.off[ks + 1]; ++k) {
      float s = 1.0f;
      if (amax_x[k] > 0.0f && amax_w[k] > 0.0f) {
        s = (float)(std::pow((double)amax_x[k], al) / std::pow((double)amax_w[k], 1.0 - al));
        if (!(s > 0.0f) || !std::isfinite(s) || !std::isfinite(1.0f / s)) s = 1.0f;
      }
      smooth[k] = s;
      smooth_inv[k] = 1.0f / s;
    }
  }
}

// ---- Quant(W diag(s)): one wavefront per (output channel, K-segment); max-reduce, then divide and round -------------
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_weight_smoothed_kernel(const void* __restrict__ w, const float* __restrict__ smooth,
                                                                       int8_t* __restrict__ wq, float* __restrict__ wscale,
                                                                       int N, int K, const KsegTable tb) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);          // (n, ks) pairs, ks fastest
  if (item >= N * tb.S) return;
  const int n = item / tb.S, ks = item - n * tb.S;
  int k0 = 0, k1 = 0;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.off[s]; k1 = tb.off[s + 1]; }
  auto value = [&](int k) {
    const size_t i = (size_t)n * K + k;
    const float v = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(w)[i]) : reinterpret_cast<const float*>(w)[i];
    return __fmul_rn(v, smooth[k]);
  };
  float a = 0.0f;
  for (int k = k0 + lane; k < k1; k += 64) a = __builtin_fmaxf(a, __builtin_fabsf(value(k)));
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) a = __builtin_fmaxf(a, __shfl_xor(a, off, 64));
  const float sw = (a == 0.0f) ? 1.0f : a / kQmax;
  if (lane == 0) wscale[(size_t)ks * N + n] = sw;
  for (int k = k0 + lane; k < k1; k += 64) wq[(size_t)n * K + k] = (int8_t)clip_code(__builtin_rintf(value(k) / sw));
}

hipError_t launch_quantize_weight_smoothed(const void* w, bool w_is_bf16, const float* smooth, int8_t* wq, float* wscale, int N,
                                           int K, const KsegTable& tb, hipStream_t st) {
  const long items = (long)N * tb.S;
  const unsigned blocks = (unsigned)((items + 3) / 4);
  if (w_is_bf16) hipLaunchKernelGGL(quantize_weight_smoothed_kernel<true>, dim3(blocks), dim3(256), 0, st, w, smooth, wq, wscale, N, K, tb);
  else hipLaunchKernelGGL(quantize_weight_smoothed_kernel<false>, dim3(blocks), dim3(256), 0, st, w, smooth, wq, wscale, N, K, tb);
  return hipGetLastError();
}

// ---- Q_dual(X diag(r)): a thread owns 16 consecutive elements of one row and K-segment (K and the segment boundaries
// multiples of 16), else one element per thread.  x' = x * r[k] is one fp32 multiplication, then the quantizer of
// Sec. 4.3.2 as in the plain pass; r (K floats) stays in the caches.
// The aligned kernel: one 16-column chunk per thread; a wave covers 64 / kSmRows chunks of kSmRows consecutive token rows
// (lane -> row lane / CW, chunk lane % CW), a workgroup four times as many chunks of those rows.  The rows of a wave ask
// for the same 16 reciprocal factors per chunk, so the factor loads touch 1 / kSmRows of the cache lines they would with
// one row per wave (with one row per wave the first-level cache moved three times the bytes of X and the pass ran at
// 4.2 TB/s).
constexpr int kSmRows = 8;       // measured on 4608 x 15360 / 8500 x 1536: 45.5 / 11.9 us with 4, 44.5 / 9.6 with 8, 51.6 / 10.0 with 16
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_act_smoothed_fast_kernel(const void* __restrict__ x, const float* __restrict__ rinv,
                                                                         int8_t* __restrict__ xq, int M, uint32_t kchunks,
                                                                         const ActTable tb) {
  constexpr uint32_t CW = 64u / kSmRows;                            // chunks per wave
  const uint32_t nxb = (kchunks + 4u * CW - 1u) / (4u * CW);         // workgroups per group of rows, walked first
  const uint32_t rg = blockIdx.x / nxb;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t cc = (blockIdx.x - rg * nxb) * (4u * CW) + wave * CW + (lane % CW);   // 16-column chunk inside a row
  const int row = (int)(rg * kSmRows + lane / CW);
  if (cc >= kchunks || row >= M) return;
  constexpr int NL = BF16 ? 2 : 4;
  const size_t c = (size_t)row * kchunks + cc;
  v4i raw[NL];
#pragma unroll
  for (int l = 0; l < NL; ++l) raw[l] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(x) + (NL * c + l));
  const int col = (int)(cc * 16u);
  v4f rr[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rr[g] = *reinterpret_cast<const v4f*>(rinv + col + 4 * g);
  float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
  bool dual = tb.dual[0] != 0;
  for (int s = 1; s < tb.S; ++s)
    if (col >= tb.kseg_off[s]) { sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0; }
  v4i out;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    float v[4];
    if (BF16) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const uint32_t u = (uint32_t)raw[BF16 ? g / 2 : 0][(g % 2) * 2 + i];
        v[2 * i] = __uint_as_float(u << 16);
        v[2 * i + 1] = __uint_as_float(u & 0xFFFF0000u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = __int_as_float(raw[BF16 ? 0 : g][i]);
    }
    uint32_t pk = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float xs = __fmul_rn(v[i], rr[g][i]);
      const bool ng = dual && (xs < 0.0f);
      pk |= (uint32_t)(clip_code(round_quotient(xs, ng ? sn : sp, ng ? in : ip)) & 0xFF) << (8 * i);
    }
    out[g] = (int)pk;
  }
  reinterpret_cast<v4i*>(xq)[c] = out;
}

template <bool BF16>
__global__ __launch_bounds__(256) void quantize_act_smoothed_generic_kernel(const void* __restrict__ x, const float* __restrict__ rinv,
                                                                            int8_t* __restrict__ xq, int M, int K, const ActTable tb) {
  const size_t total = (size_t)M * K;
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int col = (int)(i % (size_t)K);
    float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
    bool dual = tb.dual[0] != 0;
    for (int s = 1; s < tb.S; ++s)
      if (col >= tb.kseg_off[s]) { sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0; }
    const float v = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[i]) : reinterpret_cast<const float*>(x)[i];
    const float xs = __fmul_rn(v, rinv[col]);
    const bool ng = dual && (xs < 0.0f);
    xq[i] = (int8_t)clip_code(round_quotient(xs, ng ? sn : sp, ng ? in : ip));
  }
}

hipError_t launch_quantize_act_smoothed(const void* x, bool x_is_bf16, const float* rinv, int8_t* xq, int M, int K,
                                        const ActTable& tb, hipStream_t st) {
  bool aligned = (K % 16 == 0) && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(xq) |
                                    reinterpret_cast<uintptr_t>(rinv)) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) aligned = aligned && (tb.kseg_off[s] % 16 == 0);
  if (aligned) {
    const uint32_t kchunks = (uint32_t)(K / 16);
    const uint32_t cpb = 4u * (64u / kSmRows);                     // chunks per workgroup and row
    const dim3 grid((unsigned)((M + kSmRows - 1) / kSmRows) * ((kchunks + cpb - 1u) / cpb));
    if (x_is_bf16) hipLaunchKernelGGL(quantize_act_smoothed_fast_kernel<true>, grid, dim3(256), 0, st, x, rinv, xq, M, kchunks, tb);
    else hipLaunchKernelGGL(quantize_act_smoothed_fast_kernel<false>, grid, dim3(256), 0, st, x, rinv, xq, M, kchunks, tb);
  } else {
    const size_t total = (size_t)M * K;
    const unsigned blocks = (unsigned)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    if (x_is_bf16) hipLaunchKernelGGL(quantize_act_smoothed_generic_kernel<true>, dim3(blocks), dim3(256), 0, st, x, rinv, xq, M, K, tb);
    else hipLaunchKernelGGL(quantize_act_smoothed_generic_kernel<false>, dim3(blocks), dim3(256), 0, st, x, rinv, xq, M, K, tb);
  }
  return hipGetLastError();
}

}  // namespace sq
