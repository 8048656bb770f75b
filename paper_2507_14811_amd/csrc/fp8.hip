// The 8-bit floating-point variant of the layer (main results, the 8/8 fp rows): fp8 codes in the published OCP E4M3
// format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinity, largest finite value 448) in
// place of the int8 ones.  Quantizers: code = e4m3(clip(v / s, +-448)), nearest, ties to even, s = range / 448;
// Q_dual (Sec. 4.3.2) keeps its two steps, and the two polarity matrices again travel as one byte matrix: X^_+ holds
// the codes with a clear sign bit, X^_- those with the sign bit set (a zero is stored as +0).  GEMM: the fp8 matrix
// cores of gfx950 (v_mfma_f32_32x32x64_f8f6f4, no block scales: 64 bytes of K per instruction, fp32
// accumulators; inside an aligned group of eight k the instruction keeps 14 bits below the largest product's exponent,
// across groups it adds in fp32), both polarity products fed from the same LDS fragments, the fp32 sums scaled into a running sum at
// every K-segment boundary (Sec. 4.2.2 item 2), per-column constants and bias in the epilogue.
#include "sq_kernels.hpp"

namespace sq {


// v / s for the encoder without the division: q0 = v * (1 / s) is within two units in the last place of the quotient, so
// the quotient lies between q0 (1 - 2^-21) and q0 (1 + 2^-21); the encoder is monotonic, so where both ends of that
// interval get the same code the quotient gets it too.  Only where they differ (a tie of the 3-bit mantissa, or of the
// 2^-9 grid of the subnormal codes, falls inside the interval: about one element in 100 000) the true division is
// evaluated, for the group of four, behind a branch.
constexpr float kFp8Lo = 1.0f - 0x1p-21f, kFp8Hi = 1.0f + 0x1p-21f;

// ---- weight quantizer: one wavefront per (output channel, K-segment) -------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_weight_fp8_kernel(const void* __restrict__ w, uint8_t* __restrict__ wq,
                                                                  float* __restrict__ wscale, int N, int K, const KsegTable tb) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= N * tb.S) return;
  const int n = item / tb.S, ks = item - n * tb.S;
  int k0 = 0, k1 = 0;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.off[s]; k1 = tb.off[s + 1]; }
  auto value = [&](int k) {
    const size_t i = (size_t)n * K + k;
    return BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(w)[i]) : reinterpret_cast<const float*>(w)[i];
  };
  float a = 0.0f;
  for (int k = k0 + lane; k < k1; k += 64) a = __builtin_fmaxf(a, __builtin_fabsf(value(k)));
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) a = __builtin_fmaxf(a, __shfl_xor(a, off, 64));
  const float sw = (a == 0.0f) ? 1.0f : a / kFp8Max;
  if (lane == 0) wscale[(size_t)ks * N + n] = sw;
  for (int k = k0 + lane; k < k1; k += 64) wq[(size_t)n * K + k] = (uint8_t)fp8_encode(value(k) / sw);
}

hipError_t launch_quantize_weight_fp8(const void* w, bool w_is_bf16, uint8_t* wq, float* wscale, int N, int K,
                                      const KsegTable& tb, hipStream_t st) {
  const unsigned blocks = (unsigned)(((long)N * tb.S + 3) / 4);
  if (w_is_bf16) hipLaunchKernelGGL(quantize_weight_fp8_kernel<true>, dim3(blocks), dim3(256), 0, st, w, wq, wscale, N, K, tb);
  else hipLaunchKernelGGL(quantize_weight_fp8_kernel<false>, dim3(blocks), dim3(256), 0, st, w, wq, wscale, N, K, tb);
  return hipGetLastError();
}

// ---- activation quantizer: Q_dual with fp8 codes, one element per thread and loop trip ------------------------------
// ACT: the activation in front of the layer (SiLU / GELU per K-segment, the bit-specified fp32 sequence of sq_common.hpp)
// is applied to the input first: Q_dual(act(h)) in one pass.
template <bool BF16, bool ACT>
__global__ __launch_bounds__(256) void quantize_act_fp8_kernel(const void* __restrict__ x, uint8_t* __restrict__ xq, int M, int K,
                                                               const ActTable tb) {
  const size_t total = (size_t)M * K;
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int col = (int)(i % (size_t)K);
    float sp = tb.s_pos[0], sn = tb.s_neg[0];
    bool dual = tb.dual[0] != 0;
    int acode = tb.act[0];
    for (int s = 1; s < tb.S; ++s)
      if (col >= tb.kseg_off[s]) { sp = tb.s_pos[s]; sn = tb.s_neg[s]; dual = tb.dual[s] != 0; acode = tb.act[s]; }
    float v = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[i]) : reinterpret_cast<const float*>(x)[i];
    if (ACT) v = activate(acode, v);
    const bool ng = dual && (v < 0.0f);
    xq[i] = (uint8_t)fp8_encode(v / (ng ? sn : sp));
  }
}

// aligned shapes: 16 consecutive elements of one row and K-segment per thread (16-byte loads and stores)
template <bool BF16, bool ACT>
__global__ __launch_bounds__(256) void quantize_act_fp8_fast_kernel(const void* __restrict__ x, uint8_t* __restrict__ xq,
                                                                    uint32_t nchunks, uint32_t kchunks, uint32_t kmagic,
                                                                    const ActTable tb) {
  const uint32_t c = blockIdx.x * 256u + threadIdx.x;
  if (c >= nchunks) return;
  constexpr int NL = BF16 ? 2 : 4;
  v4i raw[NL];
#pragma unroll
  for (int l = 0; l < NL; ++l) raw[l] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(x) + ((size_t)NL * c + l));
  float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
  bool dual = tb.dual[0] != 0;
  int acode = ACT ? tb.act[0] : SQ_ACT_NONE;
  if (tb.S > 1) {
    // column of this chunk: c mod kchunks via a reciprocal multiply (the quotient is exact or one too small)
    const uint32_t qc = __umulhi(c, kmagic);
    uint32_t r = c - qc * kchunks;
    if (r >= kchunks) r -= kchunks;
    const int col = (int)(r * 16u);
    for (int s = 1; s < tb.S; ++s)
      if (col >= tb.kseg_off[s]) {
        sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0;
        if (ACT) acode = tb.act[s];
      }
  }
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
    if (ACT) {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = activate(acode, v[i]);
    }
    float q0[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ng = dual && (v[i] < 0.0f);
      q0[i] = v[i] * (ng ? in : ip);
    }
    uint32_t pk = fp8_convert4(q0[0] * kFp8Lo, q0[1] * kFp8Lo, q0[2] * kFp8Lo, q0[3] * kFp8Lo);
    const uint32_t ph = fp8_convert4(q0[0] * kFp8Hi, q0[1] * kFp8Hi, q0[2] * kFp8Hi, q0[3] * kFp8Hi);
    if (__builtin_expect(pk != ph, 0)) {
      asm volatile("" ::: "memory");                       // keeps the divisions behind the branch
      float q[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ng = dual && (v[i] < 0.0f);
        q[i] = v[i] / (ng ? sn : sp);
      }
      pk = fp8_convert4(q[0], q[1], q[2], q[3]);
    }
    pk = fp8_plus_zero(pk);
    out[g] = (int)pk;
  }
  reinterpret_cast<v4i*>(xq)[c] = out;
}

template <bool ACT>
static hipError_t launch_quantize_act_fp8_impl(const void* x, bool x_is_bf16, uint8_t* xq, int M, int K, const ActTable& tb,
                                               hipStream_t st) {
  bool aligned = (K % 16 == 0) && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(xq)) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) aligned = aligned && (tb.kseg_off[s] % 16 == 0);
  for (int s = 0; s < tb.S; ++s)      // the fast kernel multiplies by the reciprocals of the steps: they must be usable
    aligned = aligned && (tb.inv_pos[s] == tb.inv_pos[s]) && (tb.inv_neg[s] == tb.inv_neg[s]);
  if (aligned) {
    const uint32_t kchunks = (uint32_t)(K / 16), nchunks = (uint32_t)(((size_t)M * K) / 16);
    const unsigned blocks = (nchunks + 255u) / 256u;
    const uint32_t kmagic = (uint32_t)(0x100000000ull / kchunks > 0xFFFFFFFFull ? 0xFFFFFFFFull : 0x100000000ull / kchunks);
    if (x_is_bf16) hipLaunchKernelGGL((quantize_act_fp8_fast_kernel<true, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, nchunks, kchunks, kmagic, tb);
    else hipLaunchKernelGGL((quantize_act_fp8_fast_kernel<false, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, nchunks, kchunks, kmagic, tb);
  } else {
    const size_t total = (size_t)M * K;
    const unsigned blocks = (unsigned)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    if (x_is_bf16) hipLaunchKernelGGL((quantize_act_fp8_kernel<true, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, M, K, tb);
    else hipLaunchKernelGGL((quantize_act_fp8_kernel<false, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, M, K, tb);
  }
  return hipGetLastError();
}

// tb.act[] other than SQ_ACT_NONE in any K-segment selects the instantiation with the activation in front
hipError_t launch_quantize_act_fp8(const void* x, bool x_is_bf16, uint8_t* xq, int M, int K, const ActTable& tb, hipStream_t st) {
  bool any = false;
  for (int s = 0; s < tb.S; ++s) any = any || tb.act[s] != SQ_ACT_NONE;
  return any ? launch_quantize_act_fp8_impl<true>(x, x_is_bf16, xq, M, K, tb, st)
             : launch_quantize_act_fp8_impl<false>(x, x_is_bf16, xq, M, K, tb, st);
}

// ---- GEMM ------------------------------------------------------------------------------------------------------------
// 128 x 128 output tile per workgroup, four waves in a 2 x 2 grid, wave tile 64 x 64 = 2 x 2 blocks of 32 x 32.  A stage
// is 128 bytes of K for the 128 X^ rows and the 128 W^ rows of the tile (32 KB; two stages, filled through registers:
// global loads of stage s + 1 are in flight while stage s is multiplied).  Rows are 128 bytes in LDS, the 16-byte
// chunks XOR-swizzled with (row >> 1) & 7 so that the fragment reads (lane -> row lane % 32, 32 bytes at chunk pair
// 2 (2 j + lane / 32)) are free of bank conflicts.  W^ rows are the "A" operand and X^ rows the "B" operand: a lane ends
// up with four runs of four consecutive output columns of one token row.
constexpr int kF8Tile = 128, kF8StageBytes = 2 * kF8Tile * 128;

bool fp8_gemm_supported(const GemmArgs& a, const GemmTable& tb) {
  if (a.K % 128 != 0) return false;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 128 != 0) return false;
  return (reinterpret_cast<uintptr_t>(a.xq) | reinterpret_cast<uintptr_t>(a.wq)) % 16 == 0;
}

template <bool DUAL>
__global__ __launch_bounds__(256) void seglinear_fp8_kernel(const GemmArgs a, const GemmTable tb, const int mode) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * kF8StageBytes];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_n = (a.N + kF8Tile - 1) / kF8Tile;
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x - tm * tiles_n;
  const int m0 = tm * kF8Tile, n0 = tn * kF8Tile;

  // ---- stage fill: thread -> (16-byte chunk t % 8, rows t / 8 + 32 p), rows 0..127 from X^, 128..255 from W^ ----------
  const int lchunk = threadIdx.x & 7, lrow = threadIdx.x >> 3;
  const int8_t* src[8];
  uint32_t dst[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    const int row = p * 32 + lrow;
    if (row < kF8Tile) {
      int r = m0 + row;
      r = r < a.M ? r : a.M - 1;                               // ragged tail: re-read the last row, masked at the store
      src[p] = a.xq + (size_t)r * a.K + lchunk * 16;
    } else {
      int r = n0 + row - kF8Tile;
      r = r < a.N ? r : a.N - 1;
      src[p] = a.wq + (size_t)r * a.K + lchunk * 16;
    }
    dst[p] = (uint32_t)(row * 128 + ((lchunk ^ ((row >> 1) & 7)) << 4));
  }
  v4i stage_regs[8];
  auto fetch = [&](const int s) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < 8; ++p) stage_regs[p] = *reinterpret_cast<const v4i*>(src[p] + (size_t)s * 128);
  };
  auto deposit = [&](const int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < 8; ++p) *reinterpret_cast<v4i*>(smem + buf * kF8StageBytes + dst[p]) = stage_regs[p];
  };

  // ---- fragments -------------------------------------------------------------------------------------------------------
  const int frow = lane & 31, kg = lane >> 5, fsw = (frow >> 1) & 7;      // rows 32 i + frow share the swizzle of frow
  auto frag = [&](const int buf, const int row_base, const int j) __attribute__((always_inline)) {
    const char* base = smem + buf * kF8StageBytes + (row_base + frow) * 128;
    const int c0 = 4 * j + 2 * kg;
    const v4i lo = *reinterpret_cast<const v4i*>(base + ((c0 ^ fsw) << 4));
    const v4i hi = *reinterpret_cast<const v4i*>(base + (((c0 + 1) ^ fsw) << 4));
    v8i f;
    f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
    f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
    return f;
  };
  constexpr int kUnit = 0;                       // constant-zero scale operands select the unscaled instruction
  v16f accp[2][2], accn[2][2], fsum[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      accp[i][j] = (v16f)(0.0f);
      accn[i][j] = (v16f)(0.0f);
      fsum[i][j] = (v16f)(0.0f);
    }
  auto multiply = [&](const int buf, const bool dl) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {                                         // two 64-byte k-steps per stage
      v8i xf[2], nf[2], wf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        xf[i] = frag(buf, wm * 64 + i * 32, j);
        wf[i] = frag(buf, kF8Tile + wn * 64 + i * 32, j);
      }
      if (DUAL && dl) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int d = 0; d < 8; ++d) {                                    // by sign bit: X^_+ / X^_- codes, the others become +0
            const int t = xf[i][d] & (int)0x80808080;
            const int wmask = t - (int)((unsigned)t >> 7);
            const int neg = (xf[i][d] & wmask) | t;
            nf[i][d] = neg;
            xf[i][d] ^= neg;
          }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
          accp[i][jn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[jn], xf[i], accp[i][jn], 0, 0, 0, kUnit, 0, kUnit);
          if (DUAL && dl)
            accn[i][jn] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[jn], nf[i], accn[i][jn], 0, 0, 0, kUnit, 0, kUnit);
        }
    }
  };
  // element v of block (i, jn) in lane l: row m0 + 64 wm + 32 i + (l & 31), column n0 + 64 wn + 32 jn + 8 (v >> 2) + 4 (l >> 5) + (v & 3)
  const int mrow = m0 + wm * 64 + frow, ncol = n0 + wn * 64 + 4 * kg;
  auto flush_segment = [&](const int ks, const bool dl) __attribute__((always_inline)) {
    const float sp = tb.s_pos[ks], sn = dl ? tb.s_neg[ks] : 0.0f;
    const float* ws = a.wscale + (size_t)ks * a.N;
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int n = ncol + jn * 32 + 8 * g + r;
          const float cw = n < a.N ? ws[n] * seg_scale_of(tb, ks, n) : 0.0f;
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            float t = (cw * sp) * accp[i][jn][4 * g + r];
            if (DUAL) t += (cw * sn) * accn[i][jn][4 * g + r];
            fsum[i][jn][4 * g + r] += t;
          }
        }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) {
        accp[i][jn] = (v16f)(0.0f);
        accn[i][jn] = (v16f)(0.0f);
      }
  };

  const int nstage = a.K >> 7;
  int ks = 0, seg_end = tb.kseg_off[1] >> 7;
  fetch(0);
  deposit(0);
  __syncthreads();
#pragma unroll 1
  for (int s = 0; s < nstage; ++s) {
    if (s + 1 < nstage) fetch(s + 1);
    const bool dl = DUAL && (tb.dual[ks] != 0);
    multiply(s & 1, dl);
    if (s + 1 == seg_end) {
      flush_segment(ks, dl);
      if (ks + 1 < tb.S) {
        ++ks;
        seg_end = tb.kseg_off[ks + 1] >> 7;
      }
    }
    if (s + 1 < nstage) deposit((s + 1) & 1);
    __syncthreads();
  }

  const bool vec = (a.N % 4 == 0) && (reinterpret_cast<uintptr_t>(a.y) % 16 == 0);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = mrow + i * 32;
    if (m >= a.M) continue;
#pragma unroll
    for (int jn = 0; jn < 2; ++jn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = ncol + jn * 32 + 8 * g;
        float o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = fsum[i][jn][4 * g + r] + ((a.bias && n + r < a.N) ? a.bias[n + r] : 0.0f);
        const size_t off = (size_t)m * a.N + n;
        if (vec && n + 3 < a.N) {
          if (mode == OUT_BF16) {
            v2i p;
            p[0] = (int)f32x2_to_bf16x2(o[0], o[1]);
            p[1] = (int)f32x2_to_bf16x2(o[2], o[3]);
            *reinterpret_cast<v2i*>(reinterpret_cast<uint16_t*>(a.y) + off) = p;
          } else {
            const v4f o4 = {o[0], o[1], o[2], o[3]};
            *reinterpret_cast<v4f*>(reinterpret_cast<float*>(a.y) + off) = o4;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n + r < a.N) {
              if (mode == OUT_BF16) reinterpret_cast<uint16_t*>(a.y)[off + r] = f32_to_bf16(o[r]);
              else reinterpret_cast<float*>(a.y)[off + r] = o[r];
            }
        }
      }
  }
}

hipError_t launch_seglinear_fp8(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st) {
  bool dual = false;
  for (int s = 0; s < tb.S; ++s) dual = dual || (tb.dual[s] != 0);
  const long tiles = (long)((a.M + kF8Tile - 1) / kF8Tile) * ((a.N + kF8Tile - 1) / kF8Tile);
  if (dual) hipLaunchKernelGGL(seglinear_fp8_kernel<true>, dim3((unsigned)tiles), dim3(256), 0, st, a, tb, (int)mode);
  else hipLaunchKernelGGL(seglinear_fp8_kernel<false>, dim3((unsigned)tiles), dim3(256), 0, st, a, tb, (int)mode);
  return hipGetLastError();
}

}  // namespace sq
