// Low-rank side branch of the 4-bit settings (main results, W4A8 rows; App. B: SVDQuant is the optimizer of the 4-bit
// settings, rank fixed at 64).  The weight is W = Lu Ld + R; the residual R is quantized and runs through the SegLinear
// kernels, the rank-r part stays in 16 bit on the unquantized activations:
//   y[m][n] = y_q[m][n] + sum_j T[m][j] Lu[n][j],    T[m][j] = sum_k X[m][k] Ld[j][k]        (Ld [r][K], Lu [N][r]).
// Two kernels:
//   * down projection T = X Ld^T on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): one pass over
//     X, HBM-bound (2 bytes per activation).  A wave owns 32 token rows; the K range is cut into slices so that the
//     launch fills the chip; every slice writes its own fp32 partial T (no atomics: the sum order is fixed).
//   * up projection and add: T (the slices summed in ascending order, fp32) times Lu^T on the fp32 matrix cores
//     (T is not rounded to 16 bit), added to y_q before the single rounding to the output type: one read of y_q,
//     one write of y.
#include "sq_kernels.hpp"

namespace sq {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kLrRowsPerWg = 256;     // down projection: 4 waves x 64 token rows
constexpr int kLrMaxSplit = 32;
constexpr int kLrUpCols = 128;        // up projection: output columns per wave (32 token rows)

int lowrank_splits(int M, int K, int cus) {
  const int row_blocks = (M + kLrRowsPerWg - 1) / kLrRowsPerWg;
  int s = (2 * cus + row_blocks - 1) / row_blocks;          // about two workgroups per compute unit
  const int max_by_k = K / 256 > 0 ? K / 256 : 1;          // slices of at least 256 features
  s = s < max_by_k ? s : max_by_k;
  s = s < kLrMaxSplit ? s : kLrMaxSplit;
  return s < 1 ? 1 : s;
}

// A wave owns 64 token rows (two 32-row blocks that share every Ld fragment it fetches) and walks its K slice in
// groups of four 16-feature steps (a lane then reads 128 contiguous bytes of each of its rows per group).  The loads of
// group g + 1 are issued before the matrix instructions of group g, so a wave keeps two groups of loads in flight.
template <bool BF16X, int JB>
__global__ __launch_bounds__(256) void lowrank_down_kernel(const void* __restrict__ x, const uint16_t* __restrict__ ld,
                                                           float* __restrict__ tpart, int M, int K, int slice) {
  constexpr int IM = 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kg = lane >> 5;
  const int k_begin = blockIdx.y * slice;
  const int k_end = (k_begin + slice) < K ? (k_begin + slice) : K;
  int mrow[IM];
  size_t xrow[IM];
#pragma unroll
  for (int i = 0; i < IM; ++i) {
    mrow[i] = blockIdx.x * kLrRowsPerWg + wave * (32 * IM) + i * 32 + (lane & 31);
    xrow[i] = (size_t)(mrow[i] < M ? mrow[i] : M - 1) * K;      // rows beyond M re-read the last row, masked at the store
  }
  v16f acc[IM][JB];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[i][jb] = (v16f)(0.0f);
  auto load_x = [&](const int i, const int k0) __attribute__((always_inline)) {
    if (BF16X) {
      const v4i raw = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(x) + xrow[i] + k0));
      return __builtin_bit_cast(v8bf, raw);
    }
    // fp32 activations enter the 16-bit branch rounded to bf16
    const v4f lo = *reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(x) + xrow[i] + k0);
    const v4f hi = *reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(x) + xrow[i] + k0 + 4);
    v4i p;
    p[0] = (int)f32x2_to_bf16x2(lo[0], lo[1]); p[1] = (int)f32x2_to_bf16x2(lo[2], lo[3]);
    p[2] = (int)f32x2_to_bf16x2(hi[0], hi[1]); p[3] = (int)f32x2_to_bf16x2(hi[2], hi[3]);
    return __builtin_bit_cast(v8bf, p);
  };
  auto load_l = [&](const int jb, const int k0) __attribute__((always_inline)) {
    return *reinterpret_cast<const v8bf*>(ld + (size_t)(jb * 32 + (lane & 31)) * K + k0);
  };
  v8bf xa[2][4][IM], lb[2][4][JB];
  auto load_group = [&](const int buf, const int k) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int i = 0; i < IM; ++i) xa[buf][t][i] = load_x(i, k + 16 * t);
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) lb[buf][t][jb] = load_l(jb, k + 16 * t);
    }
  };
  auto mul_group = [&](const int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
          acc[i][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lb[buf][t][jb], xa[buf][t][i], acc[i][jb], 0, 0, 0);
  };
  int k = k_begin + 8 * kg;
  const int ngroups = (k_end - k_begin) / 64;                    // whole groups of four steps
  if (ngroups > 0) {
    load_group(0, k);
    int g = 0;
    // the scheduling barriers keep the order written here: all loads of the next group go out before the matrix
    // instructions of the current one (left alone, the compiler sinks each load to just in front of its use)
    for (; g + 2 < ngroups; g += 2) {                            // two groups per trip: the buffer index stays static
      load_group(1, k + 64);
      __builtin_amdgcn_sched_barrier(0);
      mul_group(0);
      __builtin_amdgcn_sched_barrier(0);
      load_group(0, k + 128);
      __builtin_amdgcn_sched_barrier(0);
      mul_group(1);
      __builtin_amdgcn_sched_barrier(0);
      k += 128;
    }
    if (g + 1 < ngroups) {
      load_group(1, k + 64);
      __builtin_amdgcn_sched_barrier(0);
      mul_group(0);
      mul_group(1);
      k += 128;
    } else {
      mul_group(0);
      k += 64;
    }
  }
  for (; k < k_end; k += 16) {                                   // fewer than four steps left
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
      const v8bf l = load_l(jb, k);
#pragma unroll
      for (int i = 0; i < IM; ++i) acc[i][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(l, load_x(i, k), acc[i][jb], 0, 0, 0);
    }
  }
  // element v of block (i, jb) in lane l: row mrow[i], column j = 32 jb + 8 (v >> 2) + 4 (l >> 5) + (v & 3)
#pragma unroll
  for (int i = 0; i < IM; ++i) {
    if (mrow[i] >= M) continue;
    float* out = tpart + ((size_t)blockIdx.y * M + mrow[i]) * (JB * 32);
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4f o = {acc[i][jb][4 * g], acc[i][jb][4 * g + 1], acc[i][jb][4 * g + 2], acc[i][jb][4 * g + 3]};
        *reinterpret_cast<v4f*>(out + jb * 32 + 8 * g + 4 * kg) = o;
      }
  }
}

// T = sum of the K slices' partial results, in ascending slice order (fp32): four values per thread.
__global__ __launch_bounds__(256) void lowrank_sum_kernel(const float* __restrict__ tpart, int nsplit, size_t nvec, float* __restrict__ tsum) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  v4f s = reinterpret_cast<const v4f*>(tpart)[i];
  for (int sp = 1; sp < nsplit; ++sp) s += reinterpret_cast<const v4f*>(tpart)[(size_t)sp * nvec + i];
  reinterpret_cast<v4f*>(tsum)[i] = s;
}

// Up projection and addition on the fp32 matrix cores (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation, so T
// is not rounded to 16 bit on the way).  A wave owns 32 token rows and kLrUpCols output columns: its T fragment stays
// in registers, Lu rows (bf16, widened exactly) are the other operand, one 32 x 32 block of outputs at a time.  The
// matrix instruction pairs lane half h of both operands, so half h takes the features [h R/2, (h + 1) R/2) of T and Lu:
// every lane reads one contiguous run of each.  A lane ends up with four runs of four consecutive columns of one row:
// y_q is read and y written 16 (fp32) or 8 (bf16) bytes at a time.
template <bool YBF16, int R>
__global__ __launch_bounds__(256) void lowrank_up_kernel(const float* __restrict__ tsum, const uint16_t* __restrict__ lu,
                                                         const float* y_in, void* y_out, int M, int N) {
  constexpr int KH = R / 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = lane >> 5;
  const int m = blockIdx.y * 32 + (lane & 31);
  const int n_begin = (blockIdx.x * 4 + wave) * kLrUpCols;
  if (n_begin >= N) return;
  const int n_end = (n_begin + kLrUpCols) < N ? (n_begin + kLrUpCols) : N;
  float tf[KH];
  {
    const float* src = tsum + (size_t)(m < M ? m : M - 1) * R + KH * h;
#pragma unroll
    for (int c = 0; c < KH / 4; ++c) {
      const v4f t4 = *reinterpret_cast<const v4f*>(src + 4 * c);
#pragma unroll
      for (int i = 0; i < 4; ++i) tf[4 * c + i] = t4[i];
    }
  }
  const bool vec_ok = (N % 4 == 0) && (reinterpret_cast<uintptr_t>(y_in) % 16 == 0) &&
                      (reinterpret_cast<uintptr_t>(y_out) % (YBF16 ? 8 : 16) == 0);
#pragma unroll 1
  for (int nb = n_begin; nb < n_end; nb += 32) {
    const int na = (nb + (lane & 31)) < N ? (nb + (lane & 31)) : N - 1;       // beyond N: re-read the last row, masked at the store
    float lf[KH];
    const uint16_t* lsrc = lu + (size_t)na * R + KH * h;
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) {
      const v4i raw = *reinterpret_cast<const v4i*>(lsrc + 8 * c);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lf[8 * c + 2 * i] = __uint_as_float((uint32_t)raw[i] << 16);
        lf[8 * c + 2 * i + 1] = __uint_as_float((uint32_t)raw[i] & 0xFFFF0000u);
      }
    }
    // y_q of this block, requested before the matrix instructions
    v4f yq[4];
    const bool full = vec_ok && m < M && nb + 32 <= N;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n0 = nb + 8 * g + 4 * h;
      yq[g] = (v4f)(0.0f);
      if (y_in != nullptr && m < M) {
        if (full) {
          yq[g] = *reinterpret_cast<const v4f*>(y_in + (size_t)m * N + n0);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n0 + r < N) yq[g][r] = y_in[(size_t)m * N + n0 + r];
        }
      }
    }
    v16f acc = (v16f)(0.0f);
#pragma unroll
    for (int t = 0; t < KH; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(lf[t], tf[t], acc, 0, 0, 0);
    if (m < M) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n0 = nb + 8 * g + 4 * h;
        float o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = yq[g][r] + acc[4 * g + r];
        const size_t off = (size_t)m * N + n0;
        if (full) {
          if (YBF16) {
            v2i p;
            p[0] = (int)f32x2_to_bf16x2(o[0], o[1]);
            p[1] = (int)f32x2_to_bf16x2(o[2], o[3]);
            *reinterpret_cast<v2i*>(reinterpret_cast<uint16_t*>(y_out) + off) = p;
          } else {
            const v4f o4 = {o[0], o[1], o[2], o[3]};
            *reinterpret_cast<v4f*>(reinterpret_cast<float*>(y_out) + off) = o4;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n0 + r < N) {
              if (YBF16) reinterpret_cast<uint16_t*>(y_out)[off + r] = f32_to_bf16(o[r]);
              else reinterpret_cast<float*>(y_out)[off + r] = o[r];
            }
        }
      }
    }
  }
}

size_t lowrank_workspace_bytes(int M, int K, int rank, int cus) {
  return (size_t)(lowrank_splits(M, K, cus) + 1) * M * rank * sizeof(float);     // the slices' partial T, then their sum
}

hipError_t launch_lowrank_add(const void* x, bool x_is_bf16, const uint16_t* ld, const uint16_t* lu, int rank, const float* y_in,
                              void* y_out, bool y_is_bf16, int M, int K, int N, float* workspace, int cus, hipStream_t st) {
  const int nsplit = lowrank_splits(M, K, cus);
  int slice = (K + nsplit - 1) / nsplit;
  slice = (slice + 63) / 64 * 64;                              // whole groups of four 16-feature steps, except at the end of K
  dim3 gd((M + kLrRowsPerWg - 1) / kLrRowsPerWg, nsplit);
#define SQ_DOWN(B, J) hipLaunchKernelGGL((lowrank_down_kernel<B, J>), gd, dim3(256), 0, st, x, ld, workspace, M, K, slice)
  if (rank == 64) { if (x_is_bf16) SQ_DOWN(true, 2); else SQ_DOWN(false, 2); }
  else            { if (x_is_bf16) SQ_DOWN(true, 1); else SQ_DOWN(false, 1); }
#undef SQ_DOWN
  const float* tsum = workspace;
  if (nsplit > 1) {
    float* dst = workspace + (size_t)nsplit * M * rank;
    const size_t nvec = (size_t)M * rank / 4;
    hipLaunchKernelGGL(lowrank_sum_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st, workspace, nsplit, nvec, dst);
    tsum = dst;
  }
  dim3 gu((N + 4 * kLrUpCols - 1) / (4 * kLrUpCols), (M + 31) / 32);
#define SQ_UP(B, R) hipLaunchKernelGGL((lowrank_up_kernel<B, R>), gu, dim3(256), 0, st, tsum, lu, y_in, y_out, M, N)
  if (rank == 64) { if (y_is_bf16) SQ_UP(true, 64); else SQ_UP(false, 64); }
  else            { if (y_is_bf16) SQ_UP(true, 32); else SQ_UP(false, 32); }
#undef SQ_UP
  return hipGetLastError();
}

}  // namespace sq
