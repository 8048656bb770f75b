// Quant(.) kernels: the fused polarity-split / DualScale activation quantizer (Sec. 4.3.2) and the
// per-segment symmetric weight quantizer (Sec. 3 quantizer applied per segment, Sec. 4.2.2).
// Both are single-pass, HBM-bandwidth-bound streams.
#include "sq_kernels.hpp"

namespace sq {

// ------------------------------------------------------------------------------------------------
// Activation quantize.  Output: one int8 code per element, X^ = X^_+ + X^_- ("polarity-merged"): in a
// DualScale K-segment the element went through the s_+ branch of Q_dual when x >= 0 (code >= 0) and
// through the s_- branch when x < 0 (code <= 0), so X^_+ = max(X^, 0) and X^_- = min(X^, 0) are recovered
// exactly from the sign; in a single-scale segment the code is the symmetric one.
//
// Fast path: K and every K-segment boundary are multiples of 16, so a thread owns 16 consecutive elements
// of one row and one segment: 32 B (bf16) or 64 B (fp32) in, 16 B out, one chunk per thread (kActUnroll).
// ------------------------------------------------------------------------------------------------
constexpr int kActUnroll = 1;     // measured on the headline layer: 37.4 us with 1, 39.6 with 2, 44 with 4, 52.6 with 8 chunks per thread
constexpr int kActChunk = 16;

__device__ __forceinline__ uint32_t pack4(int c0, int c1, int c2, int c3) {
  return (uint32_t)(c0 & 0xFF) | ((uint32_t)(c1 & 0xFF) << 8) | ((uint32_t)(c2 & 0xFF) << 16) | ((uint32_t)c3 << 24);
}

template <bool BF16, bool ONESEG, bool ACT>
__global__ __launch_bounds__(256) void quantize_act_fast_kernel(const void* __restrict__ x, int8_t* __restrict__ xq,
                                                                uint32_t nchunks, uint32_t kchunks, uint32_t kmagic,
                                                                const ActTable tb) {
  constexpr int NL = BF16 ? 2 : 4;                       // 16-byte loads per chunk
  const uint32_t base = blockIdx.x * (256u * kActUnroll) + threadIdx.x;
  v4i raw[kActUnroll][NL];
#pragma unroll
  for (int j = 0; j < kActUnroll; ++j) {
    const uint32_t c = base + j * 256u;
    if (c < nchunks) {
      // x is read once and dead afterwards: non-temporal loads keep it from displacing X^ (which the GEMM reads
      // next) in the caches; 4.7 -> 5.2 TB/s.  The stores stay ordinary: non-temporal ones were slower.
#pragma unroll
      for (int l = 0; l < NL; ++l) raw[j][l] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(x) + ((size_t)NL * c + l));
    }
  }
#pragma unroll
  for (int j = 0; j < kActUnroll; ++j) {
    const uint32_t c = base + j * 256u;
    if (c >= nchunks) continue;
    float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
    bool dual = tb.dual[0] != 0;
    int acode = ACT ? tb.act[0] : SQ_ACT_NONE;
    if (!ONESEG) {
      // column of this chunk: c mod kchunks via a reciprocal multiply (q is exact or one too small)
      uint32_t q = __umulhi(c, kmagic);
      uint32_t r = c - q * kchunks;
      if (r >= kchunks) r -= kchunks;
      const int col = (int)(r * (uint32_t)kActChunk);
      for (int s = 1; s < tb.S; ++s) {
        if (col >= tb.kseg_off[s]) {
          sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0;
          if (ACT) acode = tb.act[s];
        }
      }
    }
    v4i out;
#pragma unroll
    for (int g = 0; g < 4; ++g) {                        // four output dwords of four codes
      float v[4];
      if (BF16) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const uint32_t u = (uint32_t)raw[j][BF16 ? g / 2 : 0][(g % 2) * 2 + i];
          v[2 * i] = __uint_as_float(u << 16);
          v[2 * i + 1] = __uint_as_float(u & 0xFFFF0000u);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __int_as_float(raw[j][BF16 ? 0 : g][i]);
      }
      if (ACT) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = activate(acode, v[i]);
      }
      int code[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ng = dual && (v[i] < 0.0f);          // X_- = min(X, 0) takes the s_- branch of Q_dual
        code[i] = clip_code(round_quotient(v[i], ng ? sn : sp, ng ? in : ip));
      }
      out[g] = (int)pack4(code[0], code[1], code[2], code[3]);
    }
    reinterpret_cast<v4i*>(xq)[c] = out;
  }
}

// Any K / segment alignment: one element per thread.
template <bool BF16, bool ACT>
__global__ __launch_bounds__(256) void quantize_act_generic_kernel(const void* __restrict__ x, int8_t* __restrict__ xq,
                                                                   int M, int K, const ActTable tb) {
  const size_t total = (size_t)M * K;
  for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
    const int col = (int)(i % (size_t)K);
    float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
    bool dual = tb.dual[0] != 0;
    int acode = ACT ? tb.act[0] : SQ_ACT_NONE;
    for (int s = 1; s < tb.S; ++s) {
      if (col >= tb.kseg_off[s]) {
        sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0;
        if (ACT) acode = tb.act[s];
      }
    }
    float v = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(x)[i]) : reinterpret_cast<const float*>(x)[i];
    if (ACT) v = activate(acode, v);
    const bool ng = dual && (v < 0.0f);
    xq[i] = (int8_t)clip_code(round_quotient(v, ng ? sn : sp, ng ? in : ip));
  }
}

template <bool ACT>
static hipError_t launch_quantize_act_impl(const void* x, bool x_is_bf16, int8_t* xq, int M, int K, const ActTable& tb,
                                           hipStream_t st) {
  bool aligned = (K % kActChunk == 0) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                 (reinterpret_cast<uintptr_t>(xq) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) aligned = aligned && (tb.kseg_off[s] % kActChunk == 0);
  if (aligned) {
    const uint32_t kchunks = (uint32_t)(K / kActChunk);
    const uint32_t nchunks = (uint32_t)(((size_t)M * K) / kActChunk);
    const uint32_t kmagic = (uint32_t)(0x100000000ull / kchunks > 0xFFFFFFFFull ? 0xFFFFFFFFull : 0x100000000ull / kchunks);
    const unsigned blocks = (nchunks + 256u * kActUnroll - 1) / (256u * kActUnroll);
    const bool one = (tb.S == 1);
#define SQ_LAUNCH_ACT(B, O) \
  hipLaunchKernelGGL((quantize_act_fast_kernel<B, O, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, nchunks, kchunks, kmagic, tb)
    if (x_is_bf16) { if (one) SQ_LAUNCH_ACT(true, true); else SQ_LAUNCH_ACT(true, false); }
    else           { if (one) SQ_LAUNCH_ACT(false, true); else SQ_LAUNCH_ACT(false, false); }
#undef SQ_LAUNCH_ACT
  } else {
    const size_t total = (size_t)M * K;
    const unsigned blocks = (unsigned)((total + 255) / 256 > 65536 ? 65536 : (total + 255) / 256);
    if (x_is_bf16) hipLaunchKernelGGL((quantize_act_generic_kernel<true, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, M, K, tb);
    else           hipLaunchKernelGGL((quantize_act_generic_kernel<false, ACT>), dim3(blocks), dim3(256), 0, st, x, xq, M, K, tb);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Fused activation + quantizer for bf16 inputs by table: a bf16 number has 65536 bit patterns, so per K-segment
// the whole map  h -> code of Q_dual(act(h))  is a 64 KiB table.  A small kernel fills the tables with the very
// arithmetic of the direct path (so the codes are the same to the bit); the streaming kernel keeps one segment's
// table in LDS (two workgroups of 64 KiB per CU) and turns every element into one LDS byte read.  The direct path
// costs ~45 ALU instructions per element and is ALU-bound at twice the HBM time; this one is a stream again.
// ------------------------------------------------------------------------------------------------
constexpr int kLutBytes = 65536;
constexpr int kLutThreads = 512;    // 256 and 1024 measured slower

// FP8: the table holds OCP E4M3 codes (nearest value of the IEEE quotient, clipped to +-448, zeros as +0) instead of int8 ones.
template <bool FP8>
__global__ __launch_bounds__(256) void act_lut_build_kernel(const ActTable tb, int8_t* __restrict__ lut) {
  const int ks = blockIdx.y;
  const uint32_t bits = blockIdx.x * 256u + threadIdx.x;                    // grid.x = 256
  float sp = 1.0f, sn = 1.0f, ip = 1.0f, in = 1.0f;
  bool dual = false;
  int acode = SQ_ACT_NONE;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0; acode = tb.act[s]; }
  const float v = activate(acode, __uint_as_float(bits << 16));
  const bool ng = dual && (v < 0.0f);
  if (FP8) lut[(size_t)ks * kLutBytes + bits] = (int8_t)fp8_encode(v / (ng ? sn : sp));
  else lut[(size_t)ks * kLutBytes + bits] = (int8_t)clip_code(round_quotient(v, ng ? sn : sp, ng ? in : ip));
}

struct LutPlan {                         // workgroups [wg_begin[s], wg_begin[s+1]) stream K-segment s
  int wg_begin[SQ_MAX_SEGMENTS + 1];
};

__global__ __launch_bounds__(kLutThreads) void quantize_act_lut_kernel(const uint16_t* __restrict__ h, int8_t* __restrict__ xq,
                                                                       int M, int K, const ActTable tb, const LutPlan plan,
                                                                       const int8_t* __restrict__ lut) {
  __shared__ __attribute__((aligned(16))) uint8_t table[kLutBytes];
  int ks = 0;
  for (int s = 1; s < tb.S; ++s)
    if ((int)blockIdx.x >= plan.wg_begin[s]) ks = s;
  int k0 = 0, k1 = 0, wg0 = 0, wg1 = 1;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.kseg_off[s]; k1 = tb.kseg_off[s + 1]; wg0 = plan.wg_begin[s]; wg1 = plan.wg_begin[s + 1]; }
  {
    const v4i* src = reinterpret_cast<const v4i*>(lut + (size_t)ks * kLutBytes);
    for (int i = threadIdx.x; i < kLutBytes / 16; i += kLutThreads) reinterpret_cast<v4i*>(table)[i] = src[i];
  }
  __syncthreads();
  const uint32_t cps = (uint32_t)(k1 - k0) / kActChunk;                    // 16-element chunks per row of the segment
  const uint32_t nchunks = (uint32_t)M * cps;
  const uint32_t stride = (uint32_t)(wg1 - wg0) * kLutThreads;
  constexpr int U = 1;                                                // chunks in flight per thread: more only hurt (measured)
  for (uint32_t c0 = (uint32_t)((int)blockIdx.x - wg0) * kLutThreads + threadIdx.x; c0 < nchunks; c0 += U * stride) {
    v4i raw[U][2];
    size_t eoff[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t c = c0 + j * stride;
      if (c < nchunks) {
        const uint32_t r = c / cps, cc = c - r * cps;
        eoff[j] = (size_t)r * K + k0 + (size_t)cc * kActChunk;
        const v4i* p = reinterpret_cast<const v4i*>(h + eoff[j]);
        raw[j][0] = __builtin_nontemporal_load(p);
        raw[j][1] = __builtin_nontemporal_load(p + 1);
      }
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
      const uint32_t c = c0 + j * stride;
      if (c >= nchunks) continue;
      v4i out;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint32_t u0 = (uint32_t)raw[j][g / 2][(g % 2) * 2], u1 = (uint32_t)raw[j][g / 2][(g % 2) * 2 + 1];
        const uint32_t b0 = table[u0 & 0xFFFFu], b1 = table[u0 >> 16], b2 = table[u1 & 0xFFFFu], b3 = table[u1 >> 16];
        out[g] = (int)(b0 | (b1 << 8) | (b2 << 16) | (b3 << 24));
      }
      *reinterpret_cast<v4i*>(xq + eoff[j]) = out;
    }
  }
}

size_t quantize_act_fused_workspace_bytes(int S) { return (size_t)S * kLutBytes; }

bool quantize_act_lut_usable(const void* h, bool h_is_bf16, const int8_t* xq, int K, const ActTable& tb) {
  bool ok = h_is_bf16 && (K % kActChunk == 0) && (reinterpret_cast<uintptr_t>(h) % 16 == 0) &&
            (reinterpret_cast<uintptr_t>(xq) % 16 == 0);
  for (int s = 0; s <= tb.S; ++s) ok = ok && (tb.kseg_off[s] % kActChunk == 0);
  return ok;
}

hipError_t launch_quantize_act_lut(const void* h, int8_t* xq, int M, int K, const ActTable& tb, void* workspace, int cus,
                                   hipStream_t st, bool fp8) {
  int8_t* lut = reinterpret_cast<int8_t*>(workspace);
  if (fp8) hipLaunchKernelGGL(act_lut_build_kernel<true>, dim3(256, tb.S), dim3(256), 0, st, tb, lut);
  else hipLaunchKernelGGL(act_lut_build_kernel<false>, dim3(256, tb.S), dim3(256), 0, st, tb, lut);
  // two workgroups per CU, dealt to the K-segments in proportion to their share of the matrix (at least one each)
  const int total = 2 * cus > tb.S ? 2 * cus : tb.S;
  LutPlan plan;
  int given = 0;
  for (int s = 0; s < tb.S; ++s) {
    plan.wg_begin[s] = given;
    const long long share = (long long)(total - tb.S) * (tb.kseg_off[s + 1] - tb.kseg_off[s]) / K;
    given += 1 + (int)share;
  }
  plan.wg_begin[tb.S] = given;
  hipLaunchKernelGGL(quantize_act_lut_kernel, dim3(given), dim3(kLutThreads), 0, st, reinterpret_cast<const uint16_t*>(h), xq,
                     M, K, tb, plan, lut);
  return hipGetLastError();
}

// tb.act is read only when some K-segment has an activation fused in front of it (sq_quantize_act_fused)
hipError_t launch_quantize_act(const void* x, bool x_is_bf16, int8_t* xq, int M, int K, const ActTable& tb,
                               hipStream_t st) {
  bool any = false;
  for (int s = 0; s < tb.S; ++s) any = any || tb.act[s] != SQ_ACT_NONE;
  return any ? launch_quantize_act_impl<true>(x, x_is_bf16, xq, M, K, tb, st)
             : launch_quantize_act_impl<false>(x, x_is_bf16, xq, M, K, tb, st);
}

// ------------------------------------------------------------------------------------------------
// Weight quantize: one wavefront per (output channel n, K-segment ks).  Pass 1 reduces max |w| over the
// row segment, pass 2 re-reads it (L2-resident: a row segment is at most 0.5 MB) and writes the codes.
// ------------------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ float load_w(const void* w, size_t i) {
  return BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(w)[i]) : reinterpret_cast<const float*>(w)[i];
}

// MODE 0: per output channel and K-segment, both passes fused.  MODE 1: first pass only, the row maximum goes to
// wscale[ks][n].  MODE 2: second pass only, with the step found in wscale[ks][n] (block-granular quantizer).
template <bool BF16, bool VEC4, int MODE>
__global__ __launch_bounds__(256) void quantize_weight_kernel(const void* __restrict__ w, int8_t* __restrict__ wq,
                                                              float* __restrict__ wscale, int N, int K,
                                                              const KsegTable tb) {
  const int lane = threadIdx.x & 63;
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= (long)N * tb.S) return;            // whole wave leaves together
  const int n = (int)(item / tb.S), ks = (int)(item % tb.S);
  int k0 = 0, k1 = 0;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.off[s]; k1 = tb.off[s + 1]; }
  const size_t row = (size_t)n * K;
  float sw;
  if (MODE == 2) {
    sw = wscale[(size_t)ks * N + n];
  } else {
    float a = 0.0f;
    if (VEC4) {
      for (int k = k0 + 4 * lane; k < k1; k += 256) {
#pragma unroll
        for (int i = 0; i < 4; ++i) a = __builtin_fmaxf(a, __builtin_fabsf(load_w<BF16>(w, row + k + i)));
      }
    } else {
      for (int k = k0 + lane; k < k1; k += 64) a = __builtin_fmaxf(a, __builtin_fabsf(load_w<BF16>(w, row + k)));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a = __builtin_fmaxf(a, __shfl_xor(a, off, 64));
    if (MODE == 1) {
      if (lane == 0) wscale[(size_t)ks * N + n] = a;
      return;
    }
    sw = (a == 0.0f) ? 1.0f : a / kQmax;
    if (lane == 0) wscale[(size_t)ks * N + n] = sw;
  }
  if (VEC4) {
    for (int k = k0 + 4 * lane; k < k1; k += 256) {
      int c[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) c[i] = clip_code(__builtin_rintf(load_w<BF16>(w, row + k + i) / sw));
      *reinterpret_cast<uint32_t*>(wq + row + k) = pack4(c[0], c[1], c[2], c[3]);
    }
  } else {
    for (int k = k0 + lane; k < k1; k += 64) wq[row + k] = (int8_t)clip_code(__builtin_rintf(load_w<BF16>(w, row + k) / sw));
  }
}

template <int MODE>
static void launch_weight_pass(const void* w, bool w_is_bf16, int8_t* wq, float* wscale, int N, int K, const KsegTable& tb,
                               hipStream_t st) {
  bool vec = (K % 4 == 0) && (reinterpret_cast<uintptr_t>(w) % 16 == 0) && (reinterpret_cast<uintptr_t>(wq) % 4 == 0);
  for (int s = 0; s <= tb.S; ++s) vec = vec && (tb.off[s] % 4 == 0);
  const long items = (long)N * tb.S;
  const unsigned blocks = (unsigned)((items + 3) / 4);
#define SQ_LAUNCH_W(B, V) hipLaunchKernelGGL((quantize_weight_kernel<B, V, MODE>), dim3(blocks), dim3(256), 0, st, w, wq, wscale, N, K, tb)
  if (w_is_bf16) { if (vec) SQ_LAUNCH_W(true, true); else SQ_LAUNCH_W(true, false); }
  else           { if (vec) SQ_LAUNCH_W(false, true); else SQ_LAUNCH_W(false, false); }
#undef SQ_LAUNCH_W
}

hipError_t launch_quantize_weight(const void* w, bool w_is_bf16, int8_t* wq, float* wscale, int N, int K,
                                  const KsegTable& tb, hipStream_t st) {
  launch_weight_pass<0>(w, w_is_bf16, wq, wscale, N, K, tb, st);
  return hipGetLastError();
}

// Block-granular steps: wscale[ks][n] holds the row maxima on entry; one workgroup per (K-segment, N-segment) block
// reduces them and writes the block's step back to every channel of the block.
__global__ __launch_bounds__(256) void weight_block_step_kernel(float* __restrict__ wscale, int N, const KsegTable nt) {
  const int ks = blockIdx.y, ns = blockIdx.x;
  int n0 = 0, n1 = 0;
  for (int t = 0; t < nt.S; ++t)
    if (t == ns) { n0 = nt.off[t]; n1 = nt.off[t + 1]; }
  float* row = wscale + (size_t)ks * N;
  float a = 0.0f;
  for (int n = n0 + threadIdx.x; n < n1; n += 256) a = __builtin_fmaxf(a, row[n]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) a = __builtin_fmaxf(a, __shfl_xor(a, off, 64));
  __shared__ float red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  a = __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
  const float sw = (a == 0.0f) ? 1.0f : a / kQmax;
  __syncthreads();                                       // every thread has read the maxima before they are overwritten
  for (int n = n0 + threadIdx.x; n < n1; n += 256) row[n] = sw;
}

// One step per (K-segment, N-segment) block: row maxima, block reduce + broadcast, quantize with the block's step.
hipError_t launch_quantize_weight_block(const void* w, bool w_is_bf16, int8_t* wq, float* wscale, int N, int K,
                                        const KsegTable& kt, const KsegTable& nt, hipStream_t st) {
  launch_weight_pass<1>(w, w_is_bf16, wq, wscale, N, K, kt, st);
  hipLaunchKernelGGL(weight_block_step_kernel, dim3(nt.S, kt.S), dim3(256), 0, st, wscale, N, nt);
  launch_weight_pass<2>(w, w_is_bf16, wq, wscale, N, K, kt, st);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Dynamic per-token activation steps (App. B: in the 4-bit settings activations are quantized dynamically per
// token): one workgroup per token row; per K-segment the row's extremes give its steps by the min/max rule
// (Sec. 4.3.2: s_+ = max x / 127, s_- = |min x| / 127, 1.0 where the extreme is 0), then the row is quantized with
// them.  This kernel takes any shape; a row is read twice (the second time from cache).  tok_steps: [2][M][S], s_pos
// then s_neg.
// ------------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_act_dynamic_kernel(const void* __restrict__ x, int8_t* __restrict__ xq,
                                                                   float* __restrict__ tok_steps, int M, int K,
                                                                   const ActTable tb, const float qmax) {
  const int m = blockIdx.x;
  const size_t row = (size_t)m * K;
  __shared__ float red[2][4];
  __shared__ float stp[2];
  for (int ks = 0; ks < tb.S; ++ks) {
    const int k0 = tb.kseg_off[ks], k1 = tb.kseg_off[ks + 1];
    const bool dual = tb.dual[ks] != 0;
    float mp = 0.0f, mn = 0.0f;
    for (int k = k0 + threadIdx.x; k < k1; k += 256) {
      const float v = load_w<BF16>(x, row + k);
      if (dual) {
        mp = __builtin_fmaxf(mp, v);
        mn = __builtin_fmaxf(mn, -v);
      } else {
        mp = __builtin_fmaxf(mp, __builtin_fabsf(v));
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      mp = __builtin_fmaxf(mp, __shfl_xor(mp, off, 64));
      mn = __builtin_fmaxf(mn, __shfl_xor(mn, off, 64));
    }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = mp; red[1][threadIdx.x >> 6] = mn; }
    __syncthreads();
    if (threadIdx.x == 0) {
      mp = __builtin_fmaxf(__builtin_fmaxf(red[0][0], red[0][1]), __builtin_fmaxf(red[0][2], red[0][3]));
      mn = __builtin_fmaxf(__builtin_fmaxf(red[1][0], red[1][1]), __builtin_fmaxf(red[1][2], red[1][3]));
      const float sp = (mp == 0.0f) ? 1.0f : mp / qmax, sn = (mn == 0.0f) ? 1.0f : mn / qmax;
      stp[0] = sp;
      stp[1] = sn;
      tok_steps[(size_t)m * tb.S + ks] = sp;
      tok_steps[((size_t)M + m) * tb.S + ks] = sn;
    }
    __syncthreads();
    const float sp = stp[0], sn = stp[1];
    for (int k = k0 + threadIdx.x; k < k1; k += 256) {
      const float v = load_w<BF16>(x, row + k);
      const bool ng = dual && (v < 0.0f);
      xq[row + k] = (int8_t)clip_code(__builtin_rintf(v / (ng ? sn : sp)));
    }
    __syncthreads();                                      // stp and red are reused by the next segment
  }
}

// The same for rows of 16-element chunks (K, the K-segment boundaries multiples of 16, 16-byte aligned pointers, K <=
// 4096 NCH): a thread keeps its NCH chunks of the row in registers between the two passes, so the row is read once
// (at large M the rows in flight on an XCD exceed its L2 and a second read goes back to memory), the loads are 16 bytes
// wide and streaming, the quotient is the reciprocal product of round_quotient (bit-identical to the division) and the
// codes leave as 16-byte stores.
template <bool BF16, int NCH>
__global__ __launch_bounds__(256) void quantize_act_dynamic_fast_kernel(const void* __restrict__ x, int8_t* __restrict__ xq,
                                                                        float* __restrict__ tok_steps, int M, int K,
                                                                        const ActTable tb, const float qmax) {
  constexpr int NL = BF16 ? 2 : 4;                       // 16-byte loads per chunk
  const int m = blockIdx.x;
  const size_t row = (size_t)m * K;
  const int nch = K >> 4;
  __shared__ float red[2][4];
  __shared__ float stp[SQ_MAX_SEGMENTS][4];              // s_+, s_-, and their reciprocals (NaN: always divide)
  v4i raw[NCH][NL];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = threadIdx.x + 256 * j;
#pragma unroll
    for (int l = 0; l < NL; ++l) raw[j][l] = (v4i)(0);
    if (c < nch) {
      const v4i* src = BF16 ? reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(x) + row + 16 * (size_t)c)
                            : reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(x) + row + 16 * (size_t)c);
#pragma unroll
      for (int l = 0; l < NL; ++l) raw[j][l] = __builtin_nontemporal_load(src + l);
    }
  }
  auto value = [&](const int j, const int e) __attribute__((always_inline)) -> float {   // element e of chunk j (constants)
    if (BF16) {
      const uint32_t u = (uint32_t)raw[j][e >> 3][(e >> 1) & 3];
      return __uint_as_float((e & 1) ? (u & 0xFFFF0000u) : (u << 16));
    }
    return __int_as_float(raw[j][BF16 ? 0 : (e >> 2)][e & 3]);
  };
  for (int ks = 0; ks < tb.S; ++ks) {
    const int k0 = tb.kseg_off[ks], k1 = tb.kseg_off[ks + 1];
    const bool dual = tb.dual[ks] != 0;
    float mp = 0.0f, mn = 0.0f;
    if (BF16) {
      // Extremes on the bit patterns, two elements per instruction: as signed 16-bit integers the positive bf16 numbers
      // keep their order and every negative one is below zero (max with 0 = pattern of max(x, 0)); as unsigned ones the
      // negative numbers lie above all positive ones, ordered by magnitude (a maximum >= 0x8000 is the pattern of min x).
      typedef short s16x2 __attribute__((ext_vector_type(2)));
      typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
      s16x2 hi_s = {0, 0};
      u16x2 hi_u = {0, 0};
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int col = (threadIdx.x + 256 * j) << 4;
        if (col < K && col >= k0 && col < k1) {
#pragma unroll
          for (int l = 0; l < 2; ++l)
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const int w = raw[j][BF16 ? l : 0][d];
              if (dual) {
                hi_s = __builtin_elementwise_max(hi_s, __builtin_bit_cast(s16x2, w));
                hi_u = __builtin_elementwise_max(hi_u, __builtin_bit_cast(u16x2, w));
              } else {
                hi_u = __builtin_elementwise_max(hi_u, __builtin_bit_cast(u16x2, w & 0x7FFF7FFF));
              }
            }
        }
      }
      const uint32_t us = (uint32_t)(hi_s[0] > hi_s[1] ? hi_s[0] : hi_s[1]);
      const uint32_t uu = (uint32_t)(hi_u[0] > hi_u[1] ? hi_u[0] : hi_u[1]);
      if (dual) {
        mp = __uint_as_float(us << 16);
        mn = uu >= 0x8000u ? __uint_as_float((uu & 0x7FFFu) << 16) : 0.0f;
      } else {
        mp = __uint_as_float(uu << 16);
      }
    } else {
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int col = (threadIdx.x + 256 * j) << 4;
        if (col < K && col >= k0 && col < k1) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float v = value(j, e);
            if (dual) {
              mp = __builtin_fmaxf(mp, v);
              mn = __builtin_fmaxf(mn, -v);
            } else {
              mp = __builtin_fmaxf(mp, __builtin_fabsf(v));
            }
          }
        }
      }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      mp = __builtin_fmaxf(mp, __shfl_xor(mp, off, 64));
      mn = __builtin_fmaxf(mn, __shfl_xor(mn, off, 64));
    }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = mp; red[1][threadIdx.x >> 6] = mn; }
    __syncthreads();
    if (threadIdx.x == 0) {
      mp = __builtin_fmaxf(__builtin_fmaxf(red[0][0], red[0][1]), __builtin_fmaxf(red[0][2], red[0][3]));
      mn = __builtin_fmaxf(__builtin_fmaxf(red[1][0], red[1][1]), __builtin_fmaxf(red[1][2], red[1][3]));
      const float sp = (mp == 0.0f) ? 1.0f : mp / qmax, sn = (mn == 0.0f) ? 1.0f : mn / qmax;
      stp[ks][0] = sp;
      stp[ks][1] = sn;
      stp[ks][2] = (sp >= 1e-30f && sp <= 1e30f) ? 1.0f / sp : __builtin_nanf("");
      stp[ks][3] = (sn >= 1e-30f && sn <= 1e30f) ? 1.0f / sn : __builtin_nanf("");
      tok_steps[(size_t)m * tb.S + ks] = sp;
      tok_steps[((size_t)M + m) * tb.S + ks] = sn;
    }
    __syncthreads();                                      // red is reused by the next segment; stp is complete after the last
#pragma unroll
    for (int j = 0; j < NCH; ++j)                         // keep the row as loaded: widened copies held across the passes
#pragma unroll
      for (int l = 0; l < NL; ++l) asm volatile("" : "+v"(raw[j][l]));   // would cost half the occupancy
  }
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = threadIdx.x + 256 * j;
    if (c >= nch) continue;
    const int col = c << 4;
    int ks = 0;
    for (int sg = 1; sg < tb.S; ++sg)
      if (col >= tb.kseg_off[sg]) ks = sg;
    bool dual = false;
    for (int sg = 0; sg < tb.S; ++sg)
      if (sg == ks) dual = tb.dual[sg] != 0;
    const float sp = stp[ks][0], sn = stp[ks][1], ip = stp[ks][2], in = stp[ks][3];
    v4i out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int code[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = value(j, 4 * q + i);
        const bool ng = dual && (v < 0.0f);
        code[i] = clip_code(round_quotient(v, ng ? sn : sp, ng ? in : ip));
      }
      out[q] = (int)pack4(code[0], code[1], code[2], code[3]);
    }
    *reinterpret_cast<v4i*>(xq + row + col) = out;
  }
}

hipError_t launch_quantize_act_dynamic(const void* x, bool x_is_bf16, int8_t* xq, float* tok_steps, int M, int K,
                                       const ActTable& tb, float qmax, hipStream_t st) {
  bool fast = K % 16 == 0 && K <= 4096 * 8 && (reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(xq)) % 16 == 0;
  for (int s = 0; s <= tb.S; ++s) fast = fast && tb.kseg_off[s] % 16 == 0;
  if (fast) {
#define SQ_D(B, N) hipLaunchKernelGGL((quantize_act_dynamic_fast_kernel<B, N>), dim3(M), dim3(256), 0, st, x, xq, tok_steps, M, K, tb, qmax)
#define SQ_DN(B) do { if (K <= 4096) SQ_D(B, 1); else if (K <= 8192) SQ_D(B, 2); else if (K <= 16384) SQ_D(B, 4); else SQ_D(B, 8); } while (0)
    if (x_is_bf16) SQ_DN(true); else SQ_DN(false);
#undef SQ_DN
#undef SQ_D
    return hipGetLastError();
  }
  if (x_is_bf16) hipLaunchKernelGGL((quantize_act_dynamic_kernel<true>), dim3(M), dim3(256), 0, st, x, xq, tok_steps, M, K, tb, qmax);
  else           hipLaunchKernelGGL((quantize_act_dynamic_kernel<false>), dim3(M), dim3(256), 0, st, x, xq, tok_steps, M, K, tb, qmax);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// GEGLU in front of the quantizer (App. B lists GEGLU with SiLU and GELU): h [M][2K] = [value | gate],
// xq[m][k] = Q_dual(value[m][k] * GELU(gate[m][k])) with the bit-specified GELU of activate() and one fp32 product.
// VEC: a thread owns 16 consecutive outputs (K, the K-segment boundaries multiples of 16, pointers 16-byte aligned);
// otherwise one output per thread.  HBM-bound where the gate's arithmetic lets it: 2 x 2 (bf16) or 2 x 4 bytes in,
// 1 byte out per element.
// ------------------------------------------------------------------------------------------------
template <bool BF16, bool VEC>
__global__ __launch_bounds__(256) void quantize_act_geglu_kernel(const void* __restrict__ h, int8_t* __restrict__ xq,
                                                                 int M, int K, const ActTable tb) {
#pragma clang fp contract(off)
  constexpr int W = VEC ? 16 : 1;
  const size_t nitem = (size_t)M * (size_t)(K / W);
  const int per_row = K / W;
  for (size_t c = blockIdx.x * (size_t)256 + threadIdx.x; c < nitem; c += (size_t)gridDim.x * 256) {
    const size_t m = c / per_row;
    const int col = (int)(c - m * per_row) * W;
    float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
    bool dual = tb.dual[0] != 0;
    for (int s = 1; s < tb.S; ++s) {
      if (col >= tb.kseg_off[s]) {
        sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0;
      }
    }
    const size_t ev = m * 2 * (size_t)K + col, eg = ev + K;       // value and gate of the first output
    float v[W], g[W];
    if (VEC) {
      if (BF16) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const v4i rv = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(h) + ev + 8 * q));
          const v4i rg = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(reinterpret_cast<const uint16_t*>(h) + eg + 8 * q));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v[8 * q + 2 * i] = __uint_as_float((uint32_t)rv[i] << 16);
            v[8 * q + 2 * i + 1] = __uint_as_float((uint32_t)rv[i] & 0xFFFF0000u);
            g[8 * q + 2 * i] = __uint_as_float((uint32_t)rg[i] << 16);
            g[8 * q + 2 * i + 1] = __uint_as_float((uint32_t)rg[i] & 0xFFFF0000u);
          }
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v4i rv = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(h) + ev + 4 * q));
          const v4i rg = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(reinterpret_cast<const float*>(h) + eg + 4 * q));
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v[4 * q + i] = __int_as_float(rv[i]);
            g[4 * q + i] = __int_as_float(rg[i]);
          }
        }
      }
    } else {
      v[0] = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(h)[ev]) : reinterpret_cast<const float*>(h)[ev];
      g[0] = BF16 ? bf16_to_f32(reinterpret_cast<const uint16_t*>(h)[eg]) : reinterpret_cast<const float*>(h)[eg];
    }
    int code[W];
#pragma unroll
    for (int i = 0; i < W; ++i) {
      const float a = __fmul_rn(v[i], activate(SQ_ACT_GELU, g[i]));
      const bool ng = dual && (a < 0.0f);                 // X_- = min(X, 0) takes the s_- branch of Q_dual
      code[i] = clip_code(round_quotient(a, ng ? sn : sp, ng ? in : ip));
    }
    if (VEC) {
      v4i out;
#pragma unroll
      for (int q = 0; q < 4; ++q) out[q] = (int)pack4(code[4 * q], code[4 * q + 1], code[4 * q + 2], code[4 * q + 3]);
      *reinterpret_cast<v4i*>(xq + m * (size_t)K + col) = out;
    } else {
      xq[m * (size_t)K + col] = (int8_t)code[0];
    }
  }
}

// bf16 input, 16-element chunks: GELU(gate) by table.  A bf16 gate has 2^16 bit patterns, and all but a sliver of a
// layer's gates have magnitudes in [2^-14, 8): the results for the kGegluExps * 128 * 2 patterns of that window (17 KiB
// of fp32, computed by each workgroup with activate(), i.e. the very bits the arithmetic path produces) sit in LDS, and a
// gate costs one ds_read_b32 instead of the ~35-instruction sequence.  A chunk with a gate outside the window (tiny,
// huge, non-finite) is redone with the sequence, in a block of its own so that the common path stays free of it.
// Persistent workgroups (two per CU) so that filling the table is a small part of their work.
constexpr int kGegluExpLo = 113, kGegluExps = 17;        // biased exponents 113 ... 129: 2^-14 <= |gate| < 2^3
constexpr int kGegluThreads = 1024;
__global__ __launch_bounds__(kGegluThreads) void quantize_act_geglu_tab_kernel(const uint16_t* __restrict__ h,
                                                                               int8_t* __restrict__ xq, int M, int K,
                                                                               const ActTable tb, const uint32_t kmagic) {
#pragma clang fp contract(off)
  __shared__ float gelu_tab[2 * kGegluExps * 128];
  for (int i = threadIdx.x; i < 2 * kGegluExps * 128; i += kGegluThreads) {
    const uint32_t sign = (uint32_t)i / (kGegluExps * 128), rest = (uint32_t)i % (kGegluExps * 128);
    const uint32_t bits = (sign << 15) | (((rest >> 7) + kGegluExpLo) << 7) | (rest & 127u);
    gelu_tab[i] = activate(SQ_ACT_GELU, __uint_as_float(bits << 16));
  }
  __syncthreads();
  const uint32_t per_row = (uint32_t)K >> 4;
  const uint32_t nitem = (uint32_t)M * per_row;                    // M * K < 2^31 (checked by the host)
  for (uint32_t c = blockIdx.x * (uint32_t)kGegluThreads + threadIdx.x; c < nitem; c += gridDim.x * (uint32_t)kGegluThreads) {
    uint32_t m = __umulhi(c, kmagic);                              // c / per_row by reciprocal multiply: exact or one too small
    uint32_t rr = c - m * per_row;
    if (rr >= per_row) { rr -= per_row; ++m; }
    const int col = (int)(rr << 4);
    const size_t ev = (size_t)m * 2 * (size_t)K + col, eg = ev + K;
    v4i cv[2], cg[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      cv[q] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(h + ev + 8 * q));
      cg[q] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(h + eg + 8 * q));
    }
    float sp = tb.s_pos[0], sn = tb.s_neg[0], ip = tb.inv_pos[0], in = tb.inv_neg[0];
    bool dual = tb.dual[0] != 0;
    for (int s = 1; s < tb.S; ++s) {
      if (col >= tb.kseg_off[s]) {
        sp = tb.s_pos[s]; sn = tb.s_neg[s]; ip = tb.inv_pos[s]; in = tb.inv_neg[s]; dual = tb.dual[s] != 0;
      }
    }
    float v[16], g[16];
    uint32_t gb[16];
    bool all_in = true;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        v[8 * q + 2 * d] = __uint_as_float((uint32_t)cv[q][d] << 16);
        v[8 * q + 2 * d + 1] = __uint_as_float((uint32_t)cv[q][d] & 0xFFFF0000u);
        gb[8 * q + 2 * d] = (uint32_t)cg[q][d] & 0xFFFFu;
        gb[8 * q + 2 * d + 1] = (uint32_t)cg[q][d] >> 16;
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t rel = ((gb[i] >> 7) & 0xFFu) - (uint32_t)kGegluExpLo;
      const bool inside = rel < (uint32_t)kGegluExps;
      all_in = all_in && inside;
      const uint32_t idx = inside ? (gb[i] >> 15) * (kGegluExps * 128) + rel * 128 + (gb[i] & 127u) : 0u;
      g[i] = gelu_tab[idx];
    }
    if (__builtin_expect(!all_in, 0)) {                            // rare: the whole chunk by the sequence
#pragma unroll 1
      for (int i = 0; i < 16; ++i) g[i] = activate(SQ_ACT_GELU, __uint_as_float(gb[i] << 16));
    }
    v4i out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      int code[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a = __fmul_rn(v[4 * q + i], g[4 * q + i]);
        const bool ng = dual && (a < 0.0f);
        code[i] = clip_code(round_quotient(a, ng ? sn : sp, ng ? in : ip));
      }
      out[q] = (int)pack4(code[0], code[1], code[2], code[3]);
    }
    *reinterpret_cast<v4i*>(xq + (size_t)m * (size_t)K + col) = out;
  }
}

hipError_t launch_quantize_act_geglu(const void* h, bool h_is_bf16, int8_t* xq, int M, int K, const ActTable& tb, int cus,
                                     hipStream_t st) {
  bool vec = K % 16 == 0 && (reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(xq)) % 16 == 0;
  for (int s = 0; s <= tb.S; ++s) vec = vec && tb.kseg_off[s] % 16 == 0;
  const size_t nitem = (size_t)M * (size_t)(vec ? K / 16 : K);
  if (nitem == 0) return hipSuccess;
  if (vec && h_is_bf16 && nitem >= (size_t)cus * 2 * kGegluThreads) {      // enough chunks to pay for the tables
    const uint64_t per_row = (uint64_t)K >> 4;
    const uint32_t kmagic = (uint32_t)(0x100000000ull / per_row > 0xFFFFFFFFull ? 0xFFFFFFFFull : 0x100000000ull / per_row);
    hipLaunchKernelGGL(quantize_act_geglu_tab_kernel, dim3((unsigned)cus * 2), dim3(kGegluThreads), 0, st,
                       reinterpret_cast<const uint16_t*>(h), xq, M, K, tb, kmagic);
    return hipGetLastError();
  }
  size_t blocks = (nitem + 255) / 256;
  const size_t cap = (size_t)cus * 64;
  if (blocks > cap) blocks = cap;
#define SQ_G(B, V) hipLaunchKernelGGL((quantize_act_geglu_kernel<B, V>), dim3((unsigned)blocks), dim3(256), 0, st, h, xq, M, K, tb)
  if (h_is_bf16) { if (vec) SQ_G(true, true); else SQ_G(true, false); }
  else           { if (vec) SQ_G(false, true); else SQ_G(false, false); }
#undef SQ_G
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// 4-bit weights (App. B: per-channel weights in the 4-bit settings): the Sec. 3 quantizer with q_max = 7 per output
// channel and K-segment, codes packed two per byte in the order the weight stream consumes them: rows in groups
// of 16 (the last group padded with zero rows), K in steps of 128 codes (T = K / 128), one contiguous KiB per
// (group, step):  packed[((g T + t) 16 + r) 64 + j] = code(16 g + r, 128 t + j) | code(16 g + r, 128 t + 64 + j) << 4
// (4-bit two's complement).  Shifting a fetched dword left by four and masking gives the 16-fold int8 codes of one
// 64-wide MFMA k-step, masking alone those of the next.  One wavefront per (output channel, K-segment); K and the
// segment boundaries are multiples of 128.  Rows beyond N in the last group are zeroed by their own wavefronts.
// ------------------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void quantize_weight_w4_kernel(const void* __restrict__ w, uint8_t* __restrict__ wq4,
                                                                 float* __restrict__ wscale, int N, int K,
                                                                 const KsegTable tb) {
  const int lane = threadIdx.x & 63;
  const int npad = (N + 15) & ~15;
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= (long)npad * tb.S) return;         // whole wave leaves together
  const int n = (int)(item / tb.S), ks = (int)(item % tb.S);
  int k0 = 0, k1 = 0;
  for (int s = 0; s < tb.S; ++s)
    if (s == ks) { k0 = tb.off[s]; k1 = tb.off[s + 1]; }
  const int T = K >> 7;
  uint8_t* out = wq4 + ((size_t)(n >> 4) * T * 16 + (n & 15)) * 64 + lane;      // + t * 1024 per step
  if (n >= N) {                                  // padding row of the last group
    for (int b = k0; b < k1; b += 128) out[(size_t)(b >> 7) * 1024] = 0;
    return;
  }
  const size_t row = (size_t)n * K;
  float a = 0.0f;
  for (int k = k0 + lane; k < k1; k += 64) a = __builtin_fmaxf(a, __builtin_fabsf(load_w<BF16>(w, row + k)));
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) a = __builtin_fmaxf(a, __shfl_xor(a, off, 64));
  const float sw = (a == 0.0f) ? 1.0f : a / 7.0f;
  if (lane == 0) wscale[(size_t)ks * N + n] = sw;
  for (int b = k0; b < k1; b += 128) {
    const float lo = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(load_w<BF16>(w, row + b + lane) / sw), -7.0f), 7.0f);
    const float hi = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(load_w<BF16>(w, row + b + 64 + lane) / sw), -7.0f), 7.0f);
    out[(size_t)(b >> 7) * 1024] = (uint8_t)(((int)lo & 0xF) | (((int)hi & 0xF) << 4));
  }
}

hipError_t launch_quantize_weight_w4(const void* w, bool w_is_bf16, uint8_t* wq4, float* wscale, int N, int K,
                                     const KsegTable& tb, hipStream_t st) {
  const long items = (long)((N + 15) & ~15) * tb.S;
  const unsigned blocks = (unsigned)((items + 3) / 4);
  if (w_is_bf16) hipLaunchKernelGGL((quantize_weight_w4_kernel<true>), dim3(blocks), dim3(256), 0, st, w, wq4, wscale, N, K, tb);
  else           hipLaunchKernelGGL((quantize_weight_w4_kernel<false>), dim3(blocks), dim3(256), 0, st, w, wq4, wscale, N, K, tb);
  return hipGetLastError();
}

// Packed 4-bit codes back to one int8 code per byte, [N][K] row-major: what the large-M tile kernel consumes (there the
// GEMM is MFMA-bound and 4-bit weights save memory, not time; a caller unpacks a layer into a reusable buffer right
// before its GEMM).  One thread per 16 packed bytes: the low nibbles are 16 consecutive codes of one row, the high nibbles
// the 16 codes 64 columns further on.  Sign extension of a nibble u per byte: u | (u & 8) * 0x1E.
__global__ __launch_bounds__(256) void unpack_w4_kernel(const uint8_t* __restrict__ wq4, int8_t* __restrict__ wq, int N, int K) {
  const int T = K >> 7;
  const long nitem = (long)((N + 15) >> 4) * T * 16 * 4;           // (group, step, row, 16-byte chunk)
  for (long c = blockIdx.x * 256L + threadIdx.x; c < nitem; c += (long)gridDim.x * 256) {
    const int q = (int)(c & 3), r = (int)((c >> 2) & 15);
    const long gt = c >> 6;
    const int t = (int)(gt % T);
    const long n = (gt / T) * 16 + r;
    if (n >= N) continue;                                          // rows of the last group beyond N hold padding
    const v4i p = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wq4) + c);
    v4i lo, hi;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const uint32_t ul = (uint32_t)p[d] & 0x0F0F0F0Fu, uh = ((uint32_t)p[d] >> 4) & 0x0F0F0F0Fu;
      lo[d] = (int)(ul | ((ul & 0x08080808u) * 0x1Eu));
      hi[d] = (int)(uh | ((uh & 0x08080808u) * 0x1Eu));
    }
    int8_t* dst = wq + n * K + 128 * t + 16 * q;
    *reinterpret_cast<v4i*>(dst) = lo;
    *reinterpret_cast<v4i*>(dst + 64) = hi;
  }
}

hipError_t launch_unpack_w4(const uint8_t* wq4, int8_t* wq, int N, int K, int cus, hipStream_t st) {
  const long nitem = (long)((N + 15) >> 4) * (K >> 7) * 64;
  if (nitem == 0) return hipSuccess;
  long blocks = (nitem + 255) / 256;
  if (blocks > (long)cus * 32) blocks = (long)cus * 32;
  hipLaunchKernelGGL(unpack_w4_kernel, dim3((unsigned)blocks), dim3(256), 0, st, wq4, wq, N, K);
  return hipGetLastError();
}

}  // namespace sq
