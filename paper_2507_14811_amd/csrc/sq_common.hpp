// Shared device-side declarations of the SegLinear + DualScale HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "segquant.h"

namespace sq {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr float kQmax = 127.0f;

// Segment tables travel by value in the kernel-argument block: no device allocation, stream-ordered,
// safe under graph capture.  Indexing them with wave-uniform indices keeps them in scalar registers.
// Every table is made of 4-byte elements: with byte-sized tables next to int tables the compiler
// shares the byte-granular base "kernarg + index" between both and then issues scalar dword loads
// from a base that is not 4-byte aligned, which the scalar memory unit aligns down: the load returns
// the entry of a neighbouring index.
struct ActTable {                      // for the activation quantize pass
  int S;
  int kseg_off[SQ_MAX_SEGMENTS + 1];
  float s_pos[SQ_MAX_SEGMENTS];
  float s_neg[SQ_MAX_SEGMENTS];
  float inv_pos[SQ_MAX_SEGMENTS];      // 1 / s (NaN = reciprocal not usable, always divide)
  float inv_neg[SQ_MAX_SEGMENTS];
  int dual[SQ_MAX_SEGMENTS];           // 32-bit on purpose, see the note below
  int act[SQ_MAX_SEGMENTS];            // activation fused in front of the quantizer: SQ_ACT_* per K-segment
};

struct GemmTable {                     // for the SegLinear GEMM kernels
  int S, T;
  int has_seg_scale;
  int kseg_off[SQ_MAX_SEGMENTS + 1];
  int nseg_off[SQ_MAX_SEGMENTS + 1];
  float s_pos[SQ_MAX_SEGMENTS];
  float s_neg[SQ_MAX_SEGMENTS];
  int dual[SQ_MAX_SEGMENTS];
  int seg_order[SQ_MAX_SEGMENTS];      // order in which the MFMA kernel visits the K-segments
  float seg_scale[SQ_MAX_SEG_SCALE];   // [ks][ns], valid when has_seg_scale
  int act[SQ_MAX_SEGMENTS];            // weight-stream kernel fed with raw activations: SQ_ACT_* per K-segment
  float inv_pos[SQ_MAX_SEGMENTS];      //   and the reciprocals of the steps for round_quotient (NaN: always divide)
  float inv_neg[SQ_MAX_SEGMENTS];
};

// Slim segment table + per-layer pointers of the grouped skinny call (several layers that share X^ in one launch).
struct GroupSegTable {
  int S;
  int kseg_off[SQ_MAX_SEGMENTS + 1];
  float s_pos[SQ_MAX_SEGMENTS];
  float s_neg[SQ_MAX_SEGMENTS];
  int dual[SQ_MAX_SEGMENTS];
  int act[SQ_MAX_SEGMENTS];                   // raw activations: SQ_ACT_* per K-segment
  float inv_pos[SQ_MAX_SEGMENTS];             //   and the reciprocals of the steps for round_quotient
  float inv_neg[SQ_MAX_SEGMENTS];
  static constexpr int has_seg_scale = 0;     // the grouped call takes no per-block multiplier
};
struct GroupItem {
  const int8_t* wq;      // [N][K]
  const float* wscale;   // [S][N]
  const float* bias;     // [N] or nullptr
  void* y;               // [M][N]
};
struct GroupTable {
  int L;
  GroupItem item[SQ_MAX_GROUP];
};
struct NoGroups {};

struct GemmArgs {
  const int8_t* xq;        // [M][K] polarity-merged activation codes
  const int8_t* wq;        // [N][K]
  const float* wscale;     // [S][N]
  const float* bias;       // [N] or nullptr
  void* y;                 // [M][N] fp32 or bf16
  int32_t* acc_pos;        // debug: [S][M][N]
  int32_t* acc_neg;
  int M, K, N;
  int tiles_m, tiles_n, group_m;   // MFMA kernel: tile grid and panel height of the tile order
  int num_wg;                      // MFMA kernel: persistent workgroups launched
  const float* tok_steps;          // dynamic per-token steps [2][M][S] (s_pos, then s_neg) or nullptr: the layer's static steps
  const void* x_raw;               // weight-stream kernel: activations [M][K] (bf16 or fp32) to be quantized (after the
  int x_raw_bf16;                  // table's activation) into the LDS slab by the kernel itself; nullptr: xq holds codes
  int x_raw_dynamic;               // with x_raw: per-token steps found by the kernel (min/max rule per row and K-segment)
  float act_qmax;                  //   largest activation code of those steps (127, or 7 for 4-bit activation codes)
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round-half-to-even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32), which agrees
// bit for bit with "add 0x7FFF + lsb, drop 16 bits" on every finite input (checked exhaustively over the
// high halves with tie / near-tie low halves).
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  const v2f v = {lo, hi};
  const v2bf b = __builtin_convertvector(v, v2bf);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(f32x2_to_bf16x2(f, 0.0f) & 0xFFFFu); }

// round(v / s) of the Sec. 3 quantizer, bit-identical to an IEEE division followed by
// round-half-to-even.  v * (1/s) is within 2^-14.4 of the correctly rounded quotient whenever the
// quotient matters (|q| <= 256, beyond that both clip), so the cheap product decides unless it lands
// within 2^-13 of a tie; only then (or when inv is NaN/Inf) the true division is evaluated.
__device__ __forceinline__ float round_quotient(float v, float s, float inv) {
  float q0 = v * inv;
  float r = __builtin_rintf(q0);
  float t = q0 - r;
  if (!(__builtin_fabsf(t) < 0.4998779296875f)) r = __builtin_rintf(v / s);
  return r;
}

// The activation in front of a DualScale layer (Sec. 4.3.1: SiLU, GELU), evaluated in fp32 with a fixed
// operation sequence, every operation individually rounded (contraction is switched off in these functions), so that the
// codes decided from its result are reproducible to the bit:
//   exp32(t) = +inf for t > 88; t <- max(t, -87); n = rint(t log2 e); r = t - n ln2 (ln2 in two parts, fma);
//              degree-7 Taylor polynomial in r by Horner with fma; times 2^n
//   SiLU(x) = x / (1 + exp32(-x));   GELU(x) = x / (1 + exp32(-z)), z = (1.59576912 x) fma(0.044715, x x, 1),
//   the tanh form of GELU written with 0.5 (1 + tanh u) = 1 / (1 + e^(-2u)).
__device__ __forceinline__ float exp32(float t) {
#pragma clang fp contract(off)
  const bool over = t > 88.0f;
  t = __builtin_fminf(__builtin_fmaxf(t, -87.0f), 88.0f);
  const float n = __builtin_rintf(__fmul_rn(t, 1.44269504f));
  float r = __fmaf_rn(n, -0.693145751953125f, t);
  r = __fmaf_rn(n, -1.42860682e-6f, r);
  float p = 1.0f / 5040.0f;
  p = __fmaf_rn(p, r, 1.0f / 720.0f);
  p = __fmaf_rn(p, r, 1.0f / 120.0f);
  p = __fmaf_rn(p, r, 1.0f / 24.0f);
  p = __fmaf_rn(p, r, 1.0f / 6.0f);
  p = __fmaf_rn(p, r, 0.5f);
  p = __fmaf_rn(p, r, 1.0f);
  p = __fmaf_rn(p, r, 1.0f);
  const float two_n = __uint_as_float((uint32_t)((int)n + 127) << 23);     // n in [-126, 127]
  return over ? __builtin_inff() : __fmul_rn(p, two_n);
}

__device__ __forceinline__ float activate(int code, float x) {
#pragma clang fp contract(off)
  if (code == SQ_ACT_NONE) return x;
  float z = x;
  if (code == SQ_ACT_GELU) z = __fmul_rn(__fmul_rn(1.59576912f, x), __fmaf_rn(0.044715f, __fmul_rn(x, x), 1.0f));
  return __fdiv_rn(x, __fadd_rn(1.0f, exp32(-z)));
}

__device__ __forceinline__ int clip_code(float r) {
  return (int)__builtin_fminf(__builtin_fmaxf(r, -kQmax), kQmax);
}

constexpr float kFp8Max = 448.0f;     // largest finite OCP E4M3 value

// Nearest E4M3 codes of four finite values, ties to the even mantissa, saturating at +-448: the hardware conversion of
// gfx950 (v_cvt_pk_fp8_f32: OCP E4M3, round to nearest even, subnormals) behind a clip.  fp8_plus_zero then clears the sign
// bit of every byte whose other seven bits are zero (zeros are stored as +0).
__device__ __forceinline__ uint32_t fp8_convert4(float q0, float q1, float q2, float q3) {
  auto clip = [](float q) { return __builtin_fminf(__builtin_fmaxf(q, -kFp8Max), kFp8Max); };
  int p = __builtin_amdgcn_cvt_pk_fp8_f32(clip(q0), clip(q1), 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(clip(q2), clip(q3), p, true);
  return (uint32_t)p;
}
__device__ __forceinline__ uint32_t fp8_plus_zero(uint32_t u) {
  const uint32_t nz = ((u & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) & 0x80808080u;     // bit 7 of the bytes with a non-zero magnitude
  return u & (nz | 0x7F7F7F7Fu);
}
__device__ __forceinline__ uint32_t fp8_encode4(float q0, float q1, float q2, float q3) {
  return fp8_plus_zero(fp8_convert4(q0, q1, q2, q3));
}
__device__ __forceinline__ uint32_t fp8_encode(float v) { return fp8_encode4(v, 0.0f, 0.0f, 0.0f) & 0xFFu; }

// Value of an accumulator register: an exact int32 sum, or (fp8 codes) the bits of an fp32 sum.
template <bool FP8> __device__ __forceinline__ float acc_value(int bits) {
  if constexpr (FP8) return __int_as_float(bits);
  else return (float)bits;
}

// Column-dependent multiplier seg_scale[ks][ns(n)] without per-lane indexing of the by-value table.
__device__ __forceinline__ float seg_scale_of(const GemmTable& tb, int ks, int n) {
  if (!tb.has_seg_scale) return 1.0f;
  float g = tb.seg_scale[ks * tb.T];
  for (int t = 1; t < tb.T; ++t) g = (n >= tb.nseg_off[t]) ? tb.seg_scale[ks * tb.T + t] : g;
  return g;
}

}  // namespace sq
