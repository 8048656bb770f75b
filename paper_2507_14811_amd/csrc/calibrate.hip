// Calibration-side kernels: min/max activation steps per K-segment (Sec. 4.3.2: s_- = |min x| / q, s_+ = max x / q;
// App. B sensitivity study: the strict min/max rule) with running maxima over calibration batches.  One pass over
// the activations, HBM-bandwidth-bound.
#include "sq_kernels.hpp"

namespace sq {

constexpr int kCalibRows = 8;   // token rows per workgroup

__global__ void calib_init_kernel(float* __restrict__ amax, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) amax[i] = 0.0f;
}

// grid: (row blocks, K-segments).  Maxima are >= 0, so their fp32 bit patterns order like unsigned integers and
// the cross-workgroup combine is an integer atomic max.
template <bool BF16, bool VEC8>
__global__ __launch_bounds__(256) void calib_amax_kernel(const void* __restrict__ x, int M, int K, const ActTable tb,
                                                         float* __restrict__ amax) {
  const int ks = blockIdx.y;
  int k0 = 0, k1 = 0;
  bool dual = false;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.kseg_off[s]; k1 = tb.kseg_off[s + 1]; dual = tb.dual[s] != 0; }
  const int L = k1 - k0;
  const int r0 = blockIdx.x * kCalibRows;
  const int nrows = (M - r0) < kCalibRows ? (M - r0) : kCalibRows;
  float mp = 0.0f, mn = 0.0f;
  auto take = [&](float v) {
    if (dual) {
      mp = __builtin_fmaxf(mp, v);
      mn = __builtin_fmaxf(mn, -v);
    } else {
      mp = __builtin_fmaxf(mp, __builtin_fabsf(v));
    }
  };
  if (VEC8) {
    const int cpr = L >> 3;                                 // 8-element chunks per row of the segment
    for (int cc = threadIdx.x; cc < cpr; cc += 256) {       // the rows of the block are independent loads in flight
      v4i raw[kCalibRows][BF16 ? 1 : 2];
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        const int rr = r < nrows ? r : nrows - 1;           // ragged M: re-read the last row (a maximum does not mind)
        const size_t e = (size_t)(r0 + rr) * K + k0 + cc * 8;
        if (BF16) {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(x) + e);
        } else {
          raw[r][0] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e);
          raw[r][BF16 ? 0 : 1] = *reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + e + 4);
        }
      }
#pragma unroll
      for (int r = 0; r < kCalibRows; ++r) {
        if (BF16) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t u = (uint32_t)raw[r][0][i];
            take(__uint_as_float(u << 16));
            take(__uint_as_float(u & 0xFFFF0000u));
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) { take(__int_as_float(raw[r][0][i])); take(__int_as_float(raw[r][BF16 ? 0 : 1][i])); }
        }
      }
    }
  } else {
    for (int c = threadIdx.x; c < nrows * L; c += 256) {
      const int r = c / L, cc = c - r * L;
      const size_t e = (size_t)(r0 + r) * K + k0 + cc;
      take(BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[e]) : reinterpret_cast<const float*>(x)[e]);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    mp = __builtin_fmaxf(mp, __shfl_xor(mp, off, 64));
    mn = __builtin_fmaxf(mn, __shfl_xor(mn, off, 64));
  }
  __shared__ float red[2][4];
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = mp; red[1][wave] = mn; }
  __syncthreads();
  if (threadIdx.x == 0) {
    mp = __builtin_fmaxf(__builtin_fmaxf(red[0][0], red[0][1]), __builtin_fmaxf(red[0][2], red[0][3]));
    mn = __builtin_fmaxf(__builtin_fmaxf(red[1][0], red[1][1]), __builtin_fmaxf(red[1][2], red[1][3]));
    atomicMax(reinterpret_cast<unsigned int*>(amax) + ks, __float_as_uint(mp));
    atomicMax(reinterpret_cast<unsigned int*>(amax) + tb.S + ks, __float_as_uint(mn));
  }
}

// steps[ks] = s_+ , steps[S + ks] = s_- : amax / 127, the neutral step 1.0 where the maximum is 0
__global__ void calib_steps_kernel(const float* __restrict__ amax, float* __restrict__ steps, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const float a = amax[i];
    steps[i] = (a == 0.0f) ? 1.0f : a / kQmax;
  }
}

hipError_t launch_calibrate_act(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, float* amax, float* steps,
                                bool accumulate, hipStream_t st) {
  const int n = 2 * tb.S;
  if (!accumulate) hipLaunchKernelGGL(calib_init_kernel, dim3(1), dim3(128), 0, st, amax, n);
  bool vec = (K % 8 == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) vec = vec && (tb.kseg_off[s] % 8 == 0);
  dim3 grid((M + kCalibRows - 1) / kCalibRows, tb.S);
#define SQ_CALIB(B, V) hipLaunchKernelGGL((calib_amax_kernel<B, V>), grid, dim3(256), 0, st, x, M, K, tb, amax)
  if (x_is_bf16) { if (vec) SQ_CALIB(true, true); else SQ_CALIB(true, false); }
  else           { if (vec) SQ_CALIB(false, true); else SQ_CALIB(false, false); }
#undef SQ_CALIB
  hipLaunchKernelGGL(calib_steps_kernel, dim3(1), dim3(128), 0, st, amax, steps, n);
  return hipGetLastError();
}

}  // namespace sq
