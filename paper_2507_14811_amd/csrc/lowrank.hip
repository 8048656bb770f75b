// Low-rank side branch of the 4-bit settings (main results, W4A8 rows; App. B: SVDQuant is the optimizer of the 4-bit
// settings, rank fixed at 64).  The weight is W = Lu Ld + R; the residual R is quantized and runs through the SegLinear
// kernels, the rank-r part stays in 16 bit on the unquantized activations:
//   y[m][n] = y_q[m][n] + sum_j T[m][j] Lu[n][j],    T[m][j] = sum_k X[m][k] Ld[j][k]        (Ld [r][K], Lu [N][r]).
// Three kernels:
//   * down projection T = X Ld^T on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): one pass over
//     X, HBM-bound (2 bytes per activation).  The K range is cut into slices so that the launch fills the chip; every
//     slice writes its own fp32 partial T (no atomics: the sum order is fixed).  bf16 activations with K % 64 == 0 are
//     staged through LDS by direct loads of whole 128-byte row pieces; everything else is read straight into fragments.
//   * the slices summed in ascending order (fp32).
//   * up projection and add: T times Lu^T on the bf16 matrix cores with every fp32 T value split exactly into three bf16
//     terms (T is not rounded to 16 bit), added to y_q before the single rounding to the output type: one read of y_q,
//     one write of y, both in whole row pieces.
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

// The same product for bf16 activations with K % 64 == 0, staged through LDS: a workgroup owns 256 token rows, a stage is
// 64 features (128 bytes) of those rows and of the rank rows of Ld, fetched with direct global->LDS loads whose lanes
// cover whole 128-byte row pieces (eight rows per instruction), three stages in a ring (two in flight while one is
// multiplied), one barrier per stage.  The 16-byte chunks of a row are XOR-swizzled with (row >> 1) & 7, which makes the
// fragment reads (lane -> row lane % 32, chunk 2 h + lane / 32) free of bank conflicts.  Every Ld byte is fetched once
// per workgroup instead of once per wave, and every load instruction moves whole cache lines.
constexpr int kLdsRows = 256, kLdsStages = 3;

__device__ __forceinline__ void lr_glds16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

template <int JB>
__global__ __launch_bounds__(256) void lowrank_down_lds_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ ld,
                                                               float* __restrict__ tpart, int M, int K, int nsplit) {
  constexpr int R = JB * 32;
  constexpr int STAGE = (kLdsRows + R) * 128;
  constexpr int GX = kLdsRows / 8 / 4, GL = R / 8 / 4;          // direct loads per wave and stage (8 rows each)
  constexpr int LT = GX + GL;
  __shared__ __attribute__((aligned(1024))) char smem[kLdsStages * STAGE];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // this workgroup's run of 64-feature stages: the K / 64 stages are dealt evenly over the nsplit slices
  const int nst_all = K >> 6, per = nst_all / nsplit, rem = nst_all - per * nsplit;
  const int b = blockIdx.y;
  const int st_begin = b * per + (b < rem ? b : rem);
  const int nst = per + (b < rem ? 1 : 0);
  const int m0 = blockIdx.x * kLdsRows;

  // direct loads: lane -> (row lane / 8 of the instruction's eight rows, slot lane % 8 holding chunk slot ^ swizzle(row))
  const int lrow = lane >> 3, lslot = lane & 7;
  uint32_t voffX[GX], voffL[GL];
#pragma unroll
  for (int g = 0; g < GX; ++g) {
    const int rt = (wave * GX + g) * 8 + lrow;
    int r = m0 + rt;
    r = r < M ? r : M - 1;                                    // rows beyond M re-read the last row, masked at the store
    voffX[g] = ((uint32_t)r * (uint32_t)K) * 2u + (uint32_t)((lslot ^ ((rt >> 1) & 7)) << 4);
  }
#pragma unroll
  for (int g = 0; g < GL; ++g) {
    const int rt = (wave * GL + g) * 8 + lrow;
    voffL[g] = ((uint32_t)rt * (uint32_t)K) * 2u + (uint32_t)((lslot ^ ((rt >> 1) & 7)) << 4);
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  const uint32_t ldsX = lds0 + (uint32_t)(wave * GX) * 1024u;
  const uint32_t ldsL = lds0 + (uint32_t)kLdsRows * 128u + (uint32_t)(wave * GL) * 1024u;
  auto issue_stage = [&](const int s) __attribute__((always_inline)) {       // s: stage index inside this slice
    const size_t kbyte = (size_t)(st_begin + s) * 128;
    // uniform base addresses in scalar registers (the halves go through unsigned 32-bit values: readfirstlane returns a
    // signed int, which would be sign-extended into the upper half)
    auto uniform_ptr = [](const uint16_t* p, size_t byte_off) __attribute__((always_inline)) {
      const uint64_t u = reinterpret_cast<uint64_t>(p) + byte_off;
      const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)u);
      const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
      return reinterpret_cast<const void*>(((uint64_t)hi << 32) | (uint64_t)lo);
    };
    const void* px = uniform_ptr(x, kbyte);
    const void* pl = uniform_ptr(ld, kbyte);
    const uint32_t so = __builtin_amdgcn_readfirstlane((uint32_t)(s % kLdsStages) * (uint32_t)STAGE);
#pragma unroll
    for (int g = 0; g < GX; ++g) lr_glds16(px, voffX[g], ldsX + so + (uint32_t)g * 1024u);
#pragma unroll
    for (int g = 0; g < GL; ++g) lr_glds16(pl, voffL[g], ldsL + so + (uint32_t)g * 1024u);
  };

  // fragments: row lane % 32 of a 32-row block, chunk 2 h + lane / 32 of k-step h
  const int frow = lane & 31, fhi = lane >> 5, fsw = (frow >> 1) & 7;
  int foff[4];
#pragma unroll
  for (int h = 0; h < 4; ++h) foff[h] = frow * 128 + (((2 * h + fhi) ^ fsw) << 4);
  const char* fragX = smem + (wave * 64) * 128;
  const char* fragL = smem + kLdsRows * 128;
  v16f acc[2][JB];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) acc[i][jb] = (v16f)(0.0f);

#pragma unroll 1
  for (int s = 0; s < kLdsStages - 1 && s < nst; ++s) issue_stage(s);
#pragma unroll 1
  for (int s = 0; s < nst; ++s) {
    // stage s has landed in this wave's view (loads return in order): all but the loads of the later stages issued so far
    if (s + kLdsStages - 1 <= nst) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kLdsStages - 2) * LT) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                                          // ... and in every wave's; the buffer of stage s - 1 is free
    if (s + kLdsStages - 1 < nst) issue_stage(s + kLdsStages - 1);
    const int so = (s % kLdsStages) * STAGE;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      v8bf xa[2], lb[JB];
#pragma unroll
      for (int i = 0; i < 2; ++i) xa[i] = *reinterpret_cast<const v8bf*>(fragX + so + i * (32 * 128) + foff[h]);
#pragma unroll
      for (int jb = 0; jb < JB; ++jb) lb[jb] = *reinterpret_cast<const v8bf*>(fragL + so + jb * (32 * 128) + foff[h]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) acc[i][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lb[jb], xa[i], acc[i][jb], 0, 0, 0);
    }
  }
  // element v of block (i, jb) in lane l: row m0 + 64 wave + 32 i + (l & 31), column j = 32 jb + 8 (v >> 2) + 4 (l >> 5) + (v & 3)
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = m0 + wave * 64 + i * 32 + frow;
    if (m >= M) continue;
    float* out = tpart + ((size_t)blockIdx.y * M + m) * R;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4f o = {acc[i][jb][4 * g], acc[i][jb][4 * g + 1], acc[i][jb][4 * g + 2], acc[i][jb][4 * g + 3]};
        *reinterpret_cast<v4f*>(out + jb * 32 + 8 * g + 4 * fhi) = o;
      }
  }
}

// slices of the LDS-staged kernel: one workgroup per compute unit, at least four stages (256 features) per slice
static int lowrank_lds_splits(int M, int K, int cus) {
  const int row_blocks = (M + kLdsRows - 1) / kLdsRows;
  int s = cus / row_blocks;
  const int max_by_k = (K >> 6) / 4;
  s = s < max_by_k ? s : max_by_k;
  s = s < kLrMaxSplit ? s : kLrMaxSplit;
  return s < 1 ? 1 : s;
}
static bool lowrank_lds_usable(const void* x, bool x_is_bf16, const uint16_t* ld, int M, int K) {
  return x_is_bf16 && K % 64 == 0 && K >= 64 && (size_t)M * K * 2 < 0x7FFFFFFFull && (size_t)64 * K * 2 < 0x7FFFFFFFull &&
         (reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(ld)) % 16 == 0;
}

// T = sum of the K slices' partial results, in ascending slice order (fp32): four values per thread.
__global__ __launch_bounds__(256) void lowrank_sum_kernel(const float* __restrict__ tpart, int nsplit, size_t nvec, float* __restrict__ tsum) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  v4f s = reinterpret_cast<const v4f*>(tpart)[i];
  for (int sp = 1; sp < nsplit; ++sp) s += reinterpret_cast<const v4f*>(tpart)[(size_t)sp * nvec + i];
  reinterpret_cast<v4f*>(tsum)[i] = s;
}

// Up projection and addition.  A wave owns 32 token rows and kLrUpCols output columns: its T fragment stays in registers
// as three bf16 terms per value (hi = bf16(t), mid = bf16(t - hi), lo = bf16(t - hi - mid): the differences are exact, so
// hi + mid + lo reproduces t to 2^-25 of its magnitude), Lu rows (bf16) are the other operand, one 32 x 32 block of
// outputs at a time, three v_mfma_f32_32x32x16_bf16 per 16 features (fp32 accumulation; 12 matrix instructions per
// block for rank 64 where the fp32 instruction v_mfma_f32_32x32x2_f32 needs 32 of twice the length).  The matrix
// instruction pairs lane half h of both operands, so half h takes the features [h R/2, (h + 1) R/2) of T and Lu: every lane
// reads one contiguous run of each.  T is the "A" operand: a half-wave then holds 32 consecutive columns of one row.
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
  // this lane's KH features of T, split exactly into three bf16 terms (hi + mid + lo carries the 24-bit mantissa; the
  // last term is rounded at 2^-25 of the value), eight features per matrix instruction
  v8bf thi[KH / 8], tmid[KH / 8], tlo[KH / 8];
  {
    const float* src = tsum + (size_t)(m < M ? m : M - 1) * R + KH * h;
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) {
      const v4f a = *reinterpret_cast<const v4f*>(src + 8 * c), b = *reinterpret_cast<const v4f*>(src + 8 * c + 4);
      const float t[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
      v4i ph, pm, pl;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t hb = f32x2_to_bf16x2(t[2 * i], t[2 * i + 1]);
        const float r0 = t[2 * i] - __uint_as_float(hb << 16), r1 = t[2 * i + 1] - __uint_as_float(hb & 0xFFFF0000u);
        const uint32_t mbits = f32x2_to_bf16x2(r0, r1);
        const float q0 = r0 - __uint_as_float(mbits << 16), q1 = r1 - __uint_as_float(mbits & 0xFFFF0000u);
        ph[i] = (int)hb;
        pm[i] = (int)mbits;
        pl[i] = (int)f32x2_to_bf16x2(q0, q1);
      }
      thi[c] = __builtin_bit_cast(v8bf, ph);
      tmid[c] = __builtin_bit_cast(v8bf, pm);
      tlo[c] = __builtin_bit_cast(v8bf, pl);
    }
  }
  const int mb = blockIdx.y * 32;
  const bool pair_ok = (N % 2 == 0) && (reinterpret_cast<uintptr_t>(y_out) % 4 == 0);     // two bf16 columns per store
#pragma unroll 1
  for (int nb = n_begin; nb < n_end; nb += 32) {
    const int na = (nb + (lane & 31)) < N ? (nb + (lane & 31)) : N - 1;       // beyond N: re-read the last row, masked at the store
    v8bf lf[KH / 8];
    const uint16_t* lsrc = lu + (size_t)na * R + KH * h;
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) lf[c] = *reinterpret_cast<const v8bf*>(lsrc + 8 * c);
    // Element v of the block in lane l: token row mb + 8 (v >> 2) + 4 (l >> 5) + (v & 3), output column nb + (l & 31): the 32
    // lanes of a half-wave hold 32 consecutive columns of one row, so every access below covers whole 128-byte (fp32) or
    // 64-byte (bf16) row pieces.  y_q of this block is requested before the matrix instructions.
    const int n = nb + (lane & 31);
    const bool n_ok = n < N;
    float yq[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int mv = mb + 8 * (v >> 2) + 4 * h + (v & 3);
      yq[v] = (y_in != nullptr && n_ok && mv < M) ? y_in[(size_t)mv * N + n] : 0.0f;
    }
    v16f acc = (v16f)(0.0f);
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tlo[c], lf[c], acc, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tmid[c], lf[c], acc, 0, 0, 0);
#pragma unroll
    for (int c = 0; c < KH / 8; ++c) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(thi[c], lf[c], acc, 0, 0, 0);
    if (YBF16 && pair_ok && nb + 32 <= N) {
      // bf16: neighbouring lanes exchange one value of every row pair, so that a lane stores two adjacent columns (4 bytes):
      // even lanes the row of element 2 u, odd lanes the row of element 2 u + 1
      const bool odd = (lane & 1) != 0;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float o0 = yq[2 * u] + acc[2 * u], o1 = yq[2 * u + 1] + acc[2 * u + 1];
        const float send = odd ? o0 : o1;
        const float recv = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0xB1, 0xF, 0xF, false));   // lane ^ 1
        const int v = 2 * u + (odd ? 1 : 0);
        const int mv = mb + 8 * (v >> 2) + 4 * h + (v & 3);
        const uint32_t pk = odd ? f32x2_to_bf16x2(recv, o1) : f32x2_to_bf16x2(o0, recv);
        if (mv < M) *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(y_out) + (size_t)mv * N + (n & ~1)) = pk;
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int mv = mb + 8 * (v >> 2) + 4 * h + (v & 3);
        const float o = yq[v] + acc[v];
        if (n_ok && mv < M) {
          if (YBF16) reinterpret_cast<uint16_t*>(y_out)[(size_t)mv * N + n] = f32_to_bf16(o);
          else reinterpret_cast<float*>(y_out)[(size_t)mv * N + n] = o;
        }
      }
    }
  }
}

size_t lowrank_workspace_bytes(int M, int K, int rank, int cus) {
  const int a = lowrank_splits(M, K, cus), b = lowrank_lds_splits(M, K, cus);    // whichever down projection runs
  return (size_t)((a > b ? a : b) + 1) * M * rank * sizeof(float);               // the slices' partial T, then their sum
}

hipError_t launch_lowrank_add(const void* x, bool x_is_bf16, const uint16_t* ld, const uint16_t* lu, int rank, const float* y_in,
                              void* y_out, bool y_is_bf16, int M, int K, int N, float* workspace, int cus, hipStream_t st) {
  int nsplit;
  if (lowrank_lds_usable(x, x_is_bf16, ld, M, K)) {
    nsplit = lowrank_lds_splits(M, K, cus);
    dim3 gd((M + kLdsRows - 1) / kLdsRows, nsplit);
    if (rank == 64) hipLaunchKernelGGL(lowrank_down_lds_kernel<2>, gd, dim3(256), 0, st, reinterpret_cast<const uint16_t*>(x), ld, workspace, M, K, nsplit);
    else hipLaunchKernelGGL(lowrank_down_lds_kernel<1>, gd, dim3(256), 0, st, reinterpret_cast<const uint16_t*>(x), ld, workspace, M, K, nsplit);
  } else {
    nsplit = lowrank_splits(M, K, cus);
    int slice = (K + nsplit - 1) / nsplit;
    slice = (slice + 63) / 64 * 64;                              // whole groups of four 16-feature steps, except at the end of K
    dim3 gd((M + kLrRowsPerWg - 1) / kLrRowsPerWg, nsplit);
#define SQ_DOWN(B, J) hipLaunchKernelGGL((lowrank_down_kernel<B, J>), gd, dim3(256), 0, st, x, ld, workspace, M, K, slice)
    if (rank == 64) { if (x_is_bf16) SQ_DOWN(true, 2); else SQ_DOWN(false, 2); }
    else            { if (x_is_bf16) SQ_DOWN(true, 1); else SQ_DOWN(false, 1); }
#undef SQ_DOWN
  }
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
