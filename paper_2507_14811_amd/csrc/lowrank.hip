// Low-rank side branch of the 4-bit settings (main results, W4A8 rows; App. B: SVDQuant is the optimizer of the 4-bit
// settings, rank fixed at 64).  The weight is W = Lu Ld + R; the residual R is quantized and runs through the SegLinear
// kernels, the rank-r part stays in 16 bit on the unquantized activations:
//   y[m][n] = y_q[m][n] + sum_j T[m][j] Lu[n][j],    T[m][j] = sum_k X[m][k] Ld[j][k]        (Ld [r][K], Lu [N][r]).
// Two kernels:
//   * down projection T = X Ld^T on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): one pass over
//     X, HBM-bound (2 bytes per activation).  A wave owns 32 token rows; the K range is cut into slices so that the
//     launch fills the chip; every slice writes its own fp32 partial T (no atomics: the sum order is fixed).
//   * up projection and add: T (the slices summed in ascending order, fp32) times Lu^T in fp32 FMAs, 64 per output,
//     added to y_q before the single rounding to the output type: one read of y_q, one write of y.
#include "sq_kernels.hpp"

namespace sq {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kLrRowsPerWg = 128;     // down projection: 4 waves x 32 token rows
constexpr int kLrMaxSplit = 32;
constexpr int kLrUpRows = 16, kLrUpCols = 256;

int lowrank_splits(int M, int K, int cus) {
  const int row_blocks = (M + kLrRowsPerWg - 1) / kLrRowsPerWg;
  int s = (2 * cus + row_blocks - 1) / row_blocks;          // about two workgroups per compute unit
  const int max_by_k = K / 256 > 0 ? K / 256 : 1;          // slices of at least 256 features
  s = s < max_by_k ? s : max_by_k;
  s = s < kLrMaxSplit ? s : kLrMaxSplit;
  return s < 1 ? 1 : s;
}

template <bool BF16X, int JB>
__global__ __launch_bounds__(256) void lowrank_down_kernel(const void* __restrict__ x, const uint16_t* __restrict__ ld,
                                                           float* __restrict__ tpart, int M, int K, int slice) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = blockIdx.x * kLrRowsPerWg + wave * 32 + (lane & 31);
  const int mr = m < M ? m : M - 1;                          // rows beyond M re-read the last row, masked at the store
  const int kg = lane >> 5;
  const int k_begin = blockIdx.y * slice;
  const int k_end = (k_begin + slice) < K ? (k_begin + slice) : K;
  v16f acc[JB];
#pragma unroll
  for (int jb = 0; jb < JB; ++jb) acc[jb] = (v16f)(0.0f);
  const size_t xrow = (size_t)mr * K;
  auto load_x = [&](const int k0) __attribute__((always_inline)) {
    if (BF16X) return *reinterpret_cast<const v8bf*>(reinterpret_cast<const uint16_t*>(x) + xrow + k0);
    // fp32 activations enter the 16-bit branch rounded to bf16
    const v4f lo = *reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(x) + xrow + k0);
    const v4f hi = *reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(x) + xrow + k0 + 4);
    v4i p;
    p[0] = (int)f32x2_to_bf16x2(lo[0], lo[1]); p[1] = (int)f32x2_to_bf16x2(lo[2], lo[3]);
    p[2] = (int)f32x2_to_bf16x2(hi[0], hi[1]); p[3] = (int)f32x2_to_bf16x2(hi[2], hi[3]);
    return __builtin_bit_cast(v8bf, p);
  };
  auto load_l = [&](const int jb, const int k0) __attribute__((always_inline)) {
    return *reinterpret_cast<const v8bf*>(ld + (size_t)(jb * 32 + (lane & 31)) * K + k0);
  };
  int k = k_begin + 8 * kg;
  // four 16-feature steps at a time: all loads first (a lane then reads 128 contiguous bytes of its row over the four)
  for (; k + 48 < k_end; k += 64) {
    v8bf xa[4], lb[4][JB];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      xa[t] = load_x(k + 16 * t);
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) lb[t][jb] = load_l(jb, k + 16 * t);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) acc[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lb[t][jb], xa[t], acc[jb], 0, 0, 0);
  }
  for (; k < k_end; k += 16) {
    const v8bf xa = load_x(k);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_l(jb, k), xa, acc[jb], 0, 0, 0);
  }
  if (m < M) {
    // element v of block jb in lane l: row m, column j = 32 jb + 8 (v >> 2) + 4 (l >> 5) + (v & 3)
    float* out = tpart + ((size_t)blockIdx.y * M + m) * (JB * 32);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4f o = {acc[jb][4 * g], acc[jb][4 * g + 1], acc[jb][4 * g + 2], acc[jb][4 * g + 3]};
        *reinterpret_cast<v4f*>(out + jb * 32 + 8 * g + 4 * kg) = o;
      }
  }
}

template <bool YBF16, int R>
__global__ __launch_bounds__(kLrUpCols) void lowrank_up_kernel(const float* __restrict__ tpart, int nsplit, const uint16_t* __restrict__ lu,
                                                               const float* __restrict__ y_in, void* __restrict__ y_out, int M, int N) {
  __shared__ float tsum[kLrUpRows][R];
  const int m0 = blockIdx.y * kLrUpRows;
  for (int idx = threadIdx.x; idx < kLrUpRows * R; idx += kLrUpCols) {
    const int r = idx / R, j = idx - r * R;
    float s = 0.0f;
    if (m0 + r < M)
      for (int sp = 0; sp < nsplit; ++sp) s += tpart[((size_t)sp * M + m0 + r) * R + j];
    tsum[r][j] = s;
  }
  __syncthreads();
  const int n = blockIdx.x * kLrUpCols + threadIdx.x;
  if (n >= N) return;
  float w[R];
#pragma unroll
  for (int c = 0; c < R / 8; ++c) {
    const v4i raw = *reinterpret_cast<const v4i*>(lu + (size_t)n * R + 8 * c);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      w[8 * c + 2 * i] = __uint_as_float((uint32_t)raw[i] << 16);
      w[8 * c + 2 * i + 1] = __uint_as_float((uint32_t)raw[i] & 0xFFFF0000u);
    }
  }
  const int rows = (M - m0) < kLrUpRows ? (M - m0) : kLrUpRows;
  for (int r = 0; r < rows; ++r) {
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < R; ++j) acc = __builtin_fmaf(tsum[r][j], w[j], acc);
    const size_t o = (size_t)(m0 + r) * N + n;
    const float y = (y_in ? y_in[o] : 0.0f) + acc;
    if (YBF16) reinterpret_cast<uint16_t*>(y_out)[o] = f32_to_bf16(y);
    else reinterpret_cast<float*>(y_out)[o] = y;
  }
}

size_t lowrank_workspace_bytes(int M, int K, int rank, int cus) {
  return (size_t)lowrank_splits(M, K, cus) * M * rank * sizeof(float);
}

hipError_t launch_lowrank_add(const void* x, bool x_is_bf16, const uint16_t* ld, const uint16_t* lu, int rank, const float* y_in,
                              void* y_out, bool y_is_bf16, int M, int K, int N, float* workspace, int cus, hipStream_t st) {
  const int nsplit = lowrank_splits(M, K, cus);
  int slice = (K + nsplit - 1) / nsplit;
  slice = (slice + 15) / 16 * 16;
  dim3 gd((M + kLrRowsPerWg - 1) / kLrRowsPerWg, nsplit);
#define SQ_DOWN(B, J) hipLaunchKernelGGL((lowrank_down_kernel<B, J>), gd, dim3(256), 0, st, x, ld, workspace, M, K, slice)
  if (rank == 64) { if (x_is_bf16) SQ_DOWN(true, 2); else SQ_DOWN(false, 2); }
  else            { if (x_is_bf16) SQ_DOWN(true, 1); else SQ_DOWN(false, 1); }
#undef SQ_DOWN
  dim3 gu((N + kLrUpCols - 1) / kLrUpCols, (M + kLrUpRows - 1) / kLrUpRows);
#define SQ_UP(B, R) hipLaunchKernelGGL((lowrank_up_kernel<B, R>), gu, dim3(kLrUpCols), 0, st, workspace, nsplit, lu, y_in, y_out, M, N)
  if (rank == 64) { if (y_is_bf16) SQ_UP(true, 64); else SQ_UP(false, 64); }
  else            { if (y_is_bf16) SQ_UP(true, 32); else SQ_UP(false, 32); }
#undef SQ_UP
  return hipGetLastError();
}

}  // namespace sq
