// Skinny-M (M <= 64) SegLinear + DualScale GEMM: modulation / adaLN-style layers (Sec. 4.2.2 item 1:
// a linear followed by chunk; Sec. 4.3.2: its input comes from SiLU).  The layer is a single pass over
// the int8 weight, so the kernel is an HBM stream: W^ is read exactly once and feeds both polarity
// products; the (polarity-merged) X^ codes are tiny, stay L2-resident and are separated in registers.
//
// Design:
//   * A workgroup (4 waves) owns NT 16-row tiles of W^ (16*NT output columns) and all M rows.  Inside
//     every K-segment the 64-byte K steps are dealt round-robin to the 4 waves; each wave multiplies its
//     steps with v_mfma_i32_16x16x64_i8 (M <= 16 is exactly one MFMA tile; up to 4 tiles for M <= 64).
//   * Every wave streams its operands with direct global->LDS loads into a private ring of R slots, so
//     R-1 steps of W^ (1 KiB per tile and step) are in flight per wave without holding registers, and
//     no workgroup barrier is needed in the stream.  Loads are issued row-contiguous (4 lanes cover the
//     64 bytes of a row) and the 16-byte chunks are XOR-swizzled for conflict-free fragment reads.
//   * At the end of a K-segment the four waves' exact int32 partial sums are added through LDS, then
//     scaled into the fp32 result (or stored raw for the debug entry point).
#include "seglinear_mfma_kernel.hpp"

namespace sq {

template <int MT, int NT, bool DUAL>
struct SkinnyCfg {
  static constexpr int POL = DUAL ? 2 : 1;
  static constexpr int SLOT = (NT + MT) * 1024;
  static constexpr int RAW_R = (72 * 1024) / (4 * SLOT);
  static constexpr int R = RAW_R > 8 ? 8 : (RAW_R < 2 ? 2 : RAW_R);
  static constexpr int RED = 4 * POL * MT * NT * 1024;
  static constexpr int LDS = 4 * R * SLOT + RED;
  static_assert(LDS <= 160 * 1024, "skinny kernel LDS budget");
};

template <int MT, int NT, bool DUAL>
__global__ __launch_bounds__(256) void seglinear_skinny_kernel(const GemmArgs a, const GemmTable tb, const int mode) {
  using C = SkinnyCfg<MT, NT, DUAL>;
  constexpr int R = C::R, SLOT = C::SLOT, POL = C::POL;
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n0 = blockIdx.x * (16 * NT);

  // direct-load source offsets: lane -> (row lane/4, 16 B slot lane%4 holding chunk slot ^ swizzle(row))
  const int lrow = lane >> 2;
  const int lchunk = (lane & 3) ^ ((lrow >> 1) & 3);
  uint32_t voffW[NT], voffX[MT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    int r = n0 + t * 16 + lrow;
    r = r < a.N ? r : a.N - 1;
    voffW[t] = (uint32_t)r * (uint32_t)a.K + (uint32_t)lchunk * 16u;
  }
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    int r = t * 16 + lrow;
    r = r < a.M ? r : a.M - 1;
    voffX[t] = (uint32_t)r * (uint32_t)a.K + (uint32_t)lchunk * 16u;
  }
  char* ring = smem + wave * (R * SLOT);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)SQ_LDS(ring);
  // fragment reads: lane -> row lane%16, chunk lane/16
  const int frow = lane & 15;
  const int foff = frow * 64 + ((((lane >> 4)) ^ ((frow >> 1) & 3)) << 4);

  // ---- this wave's K steps: inside segment ks the steps seg_first + wave, + 4, ... ------------------
  struct Cursor { int ks, t; };
  auto seek = [&](Cursor& c) {   // move to the first valid step at or after (ks, t)
    while (c.ks < tb.S && c.t >= (tb.kseg_off[c.ks + 1] >> 6)) {
      ++c.ks;
      if (c.ks < tb.S) c.t = (tb.kseg_off[c.ks] >> 6) + wave;
    }
  };
  Cursor ic{0, wave}, cc{0, wave};
  seek(ic);
  seek(cc);
  int issued = 0, retired = 0, inflight = 0, islot = 0, cslot = 0;
  auto issue = [&]() {
    const int k0 = ic.t << 6;
    const uint32_t so = ring_lds + (uint32_t)islot * (uint32_t)SLOT;
#pragma unroll
    for (int t = 0; t < NT; ++t) glds16(a.wq + k0, voffW[t], so + t * 1024u);
#pragma unroll
    for (int t = 0; t < MT; ++t) glds16(a.xq + k0, voffX[t], so + (NT + t) * 1024u);
    issued += NT + MT;
    islot = (islot + 1 == R) ? 0 : islot + 1;
    ++inflight;
    ic.t += 4;
    seek(ic);
  };
#pragma unroll 1
  while (inflight < R && ic.ks < tb.S) issue();

  float fsum[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) fsum[i][j] = 0.0f;

  int* red = reinterpret_cast<int*>(smem + 4 * R * SLOT);   // [wave][pol][nt][mt][256]
  const int e = threadIdx.x;                                 // output element this thread finishes:
  const int em = 4 * (e >> 6) + (e & 3);                     //   row inside a 16-row tile (C row = 4*(lane/16) + v)
  const int en = (e >> 2) & 15;                              //   column inside a 16-column tile

#pragma unroll 1
  for (int ks = 0; ks < tb.S; ++ks) {
    const bool dl = DUAL && (tb.dual[ks] != 0);
    v4i accp[NT][MT], accn[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j) { accp[i][j] = (v4i)(0); accn[i][j] = (v4i)(0); }

#pragma unroll 1
    while (cc.ks == ks) {
      retired += NT + MT;
      wait_vmcnt<(R - 1) * (NT + MT), (R - 2) * (NT + MT)>(issued - retired);
      const char* sp = ring + cslot * SLOT + foff;
      v4i wf[NT], xf[MT], nf[MT];
#pragma unroll
      for (int t = 0; t < NT; ++t) wf[t] = *reinterpret_cast<const v4i*>(sp + t * 1024);
#pragma unroll
      for (int t = 0; t < MT; ++t) xf[t] = *reinterpret_cast<const v4i*>(sp + (NT + t) * 1024);
      if (dl) {                                              // X^_+ = max(X^, 0), X^_- = min(X^, 0), byte-wise
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            int pos, neg;
            split_polarity(xf[t][d], pos, neg);
            xf[t][d] = pos;
            nf[t][d] = neg;
          }
      }
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j) {
          accp[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xf[j], wf[i], accp[i][j], 0, 0, 0);
          if (dl) accn[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(nf[j], wf[i], accn[i][j], 0, 0, 0);
        }
      cslot = (cslot + 1 == R) ? 0 : cslot + 1;
      --inflight;
      cc.t += 4;
      seek(cc);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // fragment reads done before the slot is refilled
      if (ic.ks < tb.S) issue();
    }

    // ---- add the four waves' exact partial sums; scale into the fp32 result -------------------------
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        *reinterpret_cast<v4i*>(red + (((wave * POL + 0) * NT + i) * MT + j) * 256 + lane * 4) = accp[i][j];
        if (DUAL) *reinterpret_cast<v4i*>(red + (((wave * POL + (POL - 1)) * NT + i) * MT + j) * 256 + lane * 4) = accn[i][j];
      }
    __syncthreads();
    const float sp_ = tb.s_pos[ks], sn_ = tb.s_neg[ks];
    const bool last = (ks == tb.S - 1);
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const int n = n0 + i * 16 + en;
      const bool nok = n < a.N;
      float cw = 0.0f, bs = 0.0f;
      if (mode != OUT_DEBUG_ACC && nok) {
        cw = seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n];
        if (last && a.bias) bs = a.bias[n];
      }
#pragma unroll
      for (int j = 0; j < MT; ++j) {
        int sump = 0, sumn = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          sump += red[(((w * POL + 0) * NT + i) * MT + j) * 256 + e];
          if (DUAL) sumn += red[(((w * POL + (POL - 1)) * NT + i) * MT + j) * 256 + e];
        }
        if (!dl) sumn = 0;
        const int m = j * 16 + em;
        const bool ok = nok && m < a.M;
        if (mode == OUT_DEBUG_ACC) {
          if (ok) {
            const size_t o = ((size_t)ks * a.M + m) * a.N + n;
            a.acc_pos[o] = sump;
            a.acc_neg[o] = sumn;
          }
        } else {
          float t = cw * sp_ * (float)sump;
          if (DUAL) t += cw * sn_ * (float)sumn;
          t += fsum[i][j];
          fsum[i][j] = t;
          if (last && ok) {
            t += bs;
            const size_t o = (size_t)m * a.N + n;
            if (mode == OUT_F32) reinterpret_cast<float*>(a.y)[o] = t;
            else reinterpret_cast<uint16_t*>(a.y)[o] = f32_to_bf16(t);
          }
        }
      }
    }
    __syncthreads();   // reduction buffer is reused by the next K-segment
  }
}

bool skinny_supported(const GemmArgs& a, const GemmTable& tb) {
  if (a.M > 64 || a.K % 64 != 0) return false;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 64 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.xq) | reinterpret_cast<uintptr_t>(a.wq)) % 16 != 0) return false;
  return true;
}

template <int MT, int NT>
static hipError_t launch_skinny_mn(const GemmArgs& a, const GemmTable& tb, int mode, bool dual, hipStream_t st) {
  const int blocks = (a.N + 16 * NT - 1) / (16 * NT);
  if (dual) hipLaunchKernelGGL((seglinear_skinny_kernel<MT, NT, true>), dim3(blocks), dim3(256), 0, st, a, tb, mode);
  else hipLaunchKernelGGL((seglinear_skinny_kernel<MT, NT, false>), dim3(blocks), dim3(256), 0, st, a, tb, mode);
  return hipGetLastError();
}

hipError_t launch_seglinear_skinny(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st) {
  bool dual = false;
  for (int s = 0; s < tb.S; ++s) dual = dual || tb.dual[s];
  const int mt = (a.M + 15) / 16;
  // Wider workgroup tiles re-use each X^ fragment for more W^ tiles; keep >= 2 workgroups per CU.
  const int nt = (a.N >= 2 * 512 * 32) ? 2 : 1;
  switch (mt) {
    case 1: return nt == 2 ? launch_skinny_mn<1, 2>(a, tb, mode, dual, st) : launch_skinny_mn<1, 1>(a, tb, mode, dual, st);
    case 2: return nt == 2 ? launch_skinny_mn<2, 2>(a, tb, mode, dual, st) : launch_skinny_mn<2, 1>(a, tb, mode, dual, st);
    case 3: return launch_skinny_mn<3, 1>(a, tb, mode, dual, st);
    default: return launch_skinny_mn<4, 1>(a, tb, mode, dual, st);
  }
}

}  // namespace sq
