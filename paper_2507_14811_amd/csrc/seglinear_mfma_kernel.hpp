// Large-M SegLinear + DualScale GEMM on int8 MFMA (gfx950, v_mfma_i32_32x32x32_i8).
//
//   acc_+[ks] = X^_+[:, ks] W^[:, ks]^T ,  acc_-[ks] = X^_-[:, ks] W^[:, ks]^T      (Sec. 4.3.2: the two
//   polarity products against the same quantized weight; Sec. 4.2.2 item 2: one product per K-segment)
//   y = sum_ks c_+[ks][n] acc_+[ks] + c_-[ks][n] acc_-[ks] (+ bias)                  (dequant epilogue)
//
// Design (what is specific to CDNA4):
//   * A workgroup owns a BM x BN output tile; its waves form a WM x WN grid, each wave a TM x TN
//     sub-tile built from 32x32x32 int8 MFMAs.  X rows are the MFMA "A" operand (C rows), W rows the
//     "B" operand (C column = lane & 31), so every lane needs the dequant constants of only TN/32
//     output columns.
//   * Operand tiles are fetched with direct global->LDS loads (global_load_lds_dwordx4): no staging
//     registers and a ring of NSTAGE 64-byte-deep K stages, i.e. NSTAGE-1 stages of prefetch in flight.
//   * One LDS stage holds [X^_+ rows][X^_- rows][W^ rows], 64 B per row; the W^ fragments read from it
//     feed both accumulator sets, so W^ is fetched and read once for the two polarity paths.
//   * Inside a row the four 16-byte chunks are XOR-swizzled with bits 1-2 of the row index.  A direct
//     load writes lane l to byte 16*l of a 1 KiB block (= row l/4, slot l%4), so the swizzle is applied
//     to the *global* column each lane fetches; ds_read_b128 fragment reads (lane -> row l%32) then hit
//     all LDS banks evenly.  The k-order inside a fragment is irrelevant as long as both operands use
//     the same one, which they do.
//   * int32 accumulators are exact; at a K-segment boundary they are scaled into an fp32 running sum
//     (only instantiated when the layer has more than one K-segment) and cleared.  A non-dual segment
//     neither loads X^_- nor issues its MFMAs.
//   * Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works on a
//     contiguous run of tiles, ordered in panels of group_m row-tiles so concurrently resident
//     workgroups of an XCD share X^ and W^ tiles in that XCD's L2.
#pragma once
#include <type_traits>

#include "sq_kernels.hpp"

namespace sq {

// Direct global->LDS 16-byte load: lane l's 16 bytes land at lds_addr + 16*l.  Issued through inline
// assembly so that the compiler does not serialise the software pipeline with vmcnt(0) waits; the
// kernel counts outstanding loads itself (wait_vmcnt).
__device__ __forceinline__ void glds16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr)
               : "memory");
}

// Wait until at most n of this wave's vector-memory loads are outstanding (loads return in order).
// s_waitcnt takes an immediate, so the steady-state counts of the pipeline (FAST0, FAST1) get a direct
// test and everything else (pipeline fill/drain, K-segment transitions) a conservative ladder.
template <int FAST0, int FAST1>
__device__ __forceinline__ void wait_vmcnt(int n) {
#define SQ_WAIT(i) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(i) : "memory")
  if (n == FAST0) { SQ_WAIT(FAST0); }
  else if (n == FAST1) { SQ_WAIT(FAST1); }
  else if (n >= 24) { SQ_WAIT(24); }
  else if (n >= 16) { SQ_WAIT(16); }
  else if (n >= 12) { SQ_WAIT(12); }
  else if (n >= 8) { SQ_WAIT(8); }
  else if (n >= 6) { SQ_WAIT(6); }
  else if (n >= 4) { SQ_WAIT(4); }
  else if (n >= 3) { SQ_WAIT(3); }
  else if (n >= 2) { SQ_WAIT(2); }
  else if (n >= 1) { SQ_WAIT(1); }
  else { SQ_WAIT(0); }
#undef SQ_WAIT
}

#define SQ_LDS(p) ((__attribute__((address_space(3))) char*)(p))

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool MULTI>
struct MfmaCfg {
  static constexpr int NW = WM * WN;
  static constexpr int THREADS = NW * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;
  static constexpr int IM = TM / 32, JN = TN / 32;
  static constexpr int AROWS = BM * (DUAL ? 2 : 1);
  static constexpr int STAGE = (AROWS + BN) * 64;
  static constexpr int GA = BM / 16 / NW;   // 16-row load groups per wave, per polarity
  static constexpr int GB = BN / 16 / NW;
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "load groups must divide evenly over the waves");
  static_assert(NSTAGE * STAGE <= 160 * 1024, "LDS ring exceeds 160 KB");
};

template <int BM, int BN, int WM, int WN, int NSTAGE, bool DUAL, bool MULTI>
__global__ __launch_bounds__(WM * WN * 64, 1) void seglinear_mfma_kernel(const GemmArgs a, const GemmTable tb,
                                                                         const int mode) {
  using C = MfmaCfg<BM, BN, WM, WN, NSTAGE, DUAL, MULTI>;
  constexpr int IM = C::IM, JN = C::JN, GA = C::GA, GB = C::GB, STAGE = C::STAGE;
  __shared__ __attribute__((aligned(1024))) char smem[NSTAGE * STAGE];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- workgroup id -> output tile (XCD-contiguous, panels of group_m row-tiles) -------------------
  int tm, tn;
  {
    const int nblk = gridDim.x, bid = blockIdx.x;
    const int xcd = bid & 7, per = nblk >> 3, rem = nblk & 7;
    const int logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + (bid >> 3);
    const int gsz = a.group_m * a.tiles_n;
    const int g = logical / gsz, in = logical - g * gsz;
    const int first = g * a.group_m;
    const int gm = (a.tiles_m - first) < a.group_m ? (a.tiles_m - first) : a.group_m;
    tn = in / gm;
    tm = first + (in - tn * gm);
  }
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- per-lane source offsets of the direct loads (constant over the K loop) ----------------------
  const int lrow = lane >> 2;                               // row inside a 16-row group
  const int lchunk = (lane & 3) ^ ((lrow >> 1) & 3);        // logical 16 B chunk that belongs in slot lane&3
  uint32_t voffA[GA], voffB[GB];
#pragma unroll
  for (int g = 0; g < GA; ++g) {
    int r = m0 + (wave * GA + g) * 16 + lrow;
    r = r < a.M ? r : a.M - 1;                              // ragged tail: re-read the last row, masked at the store
    voffA[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)lchunk * 16u;
  }
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    int r = n0 + (wave * GB + g) * 16 + lrow;
    r = r < a.N ? r : a.N - 1;
    voffB[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)lchunk * 16u;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)SQ_LDS(smem);
  const uint32_t ldsA = lds0 + (uint32_t)(wave * GA) * 1024u;
  const uint32_t ldsN = ldsA + (uint32_t)BM * 64u;
  const uint32_t ldsB = lds0 + (uint32_t)C::AROWS * 64u + (uint32_t)(wave * GB) * 1024u;

  // ---- per-lane fragment read offsets: row = lane%32, chunk = 2h + lane/32, swizzled ---------------
  const int frow = lane & 31, fsw = (frow >> 1) & 3, fhi = lane >> 5;
  const int foff0 = frow * 64 + (((0 + fhi) ^ fsw) << 4);
  const int foff1 = frow * 64 + (((2 + fhi) ^ fsw) << 4);
  const char* fragA = smem + (wm * C::TM) * 64;
  const char* fragN = fragA + BM * 64;
  const char* fragB = smem + C::AROWS * 64 + (wn * C::TN) * 64;

  v16i accp[IM][JN];
  v16i accn[DUAL ? IM : 1][DUAL ? JN : 1];
  float fsum[MULTI ? IM : 1][MULTI ? JN : 1][16];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      accp[i][j] = (v16i)(0);
      if (DUAL) accn[i][j] = (v16i)(0);
      if (MULTI)
#pragma unroll
        for (int v = 0; v < 16; ++v) fsum[i][j][v] = 0.0f;
    }

  const int nkt = a.K >> 6;
  // issue cursor
  int iks = 0, issued = 0, ikt = 0;
  auto issue = [&]() {
    const int k0 = ikt << 6;
    while (k0 >= tb.kseg_off[iks + 1]) ++iks;
    const bool dl = DUAL && (tb.dual[iks] != 0);
    const uint32_t so = (uint32_t)(ikt % NSTAGE) * (uint32_t)STAGE;
#pragma unroll
    for (int g = 0; g < GA; ++g) glds16(a.xp + k0, voffA[g], ldsA + so + g * 1024u);
    if (dl) {
#pragma unroll
      for (int g = 0; g < GA; ++g) glds16(a.xn + k0, voffA[g], ldsN + so + g * 1024u);
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) glds16(a.wq + k0, voffB[g], ldsB + so + g * 1024u);
    issued += GA * (dl ? 2 : 1) + GB;
    ++ikt;
  };
#pragma unroll 1
  for (int s = 0; s < NSTAGE - 1 && s < nkt; ++s) issue();

  // ---- main loop over one K-segment: DL = this segment runs both polarity paths ----------------------
  int kt = 0, retired = 0;
  auto run_segment = [&](auto dl_tag, const int kt_end) {
    constexpr bool DL = decltype(dl_tag)::value;
#pragma unroll 1
    for (; kt < kt_end; ++kt) {
      retired += GA * (DL ? 2 : 1) + GB;         // loads of stage kt are the oldest outstanding ones
      wait_vmcnt<(NSTAGE - 2) * (2 * GA + GB), (NSTAGE - 2) * (GA + GB)>(issued - retired);
      __syncthreads();                           // stage kt visible to all waves; stage kt-1 free for reuse
      if (ikt < nkt) issue();

      const int so = (kt % NSTAGE) * STAGE;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int fo = so + (h ? foff1 : foff0);
        v4i bf[JN], af[IM], nf[DL ? IM : 1];
#pragma unroll
        for (int j = 0; j < JN; ++j) bf[j] = *reinterpret_cast<const v4i*>(fragB + j * 2048 + fo);
#pragma unroll
        for (int i = 0; i < IM; ++i) af[i] = *reinterpret_cast<const v4i*>(fragA + i * 2048 + fo);
        if (DL) {
#pragma unroll
          for (int i = 0; i < IM; ++i) nf[i] = *reinterpret_cast<const v4i*>(fragN + i * 2048 + fo);
        }
#pragma unroll
        for (int i = 0; i < IM; ++i)
#pragma unroll
          for (int j = 0; j < JN; ++j) {
            accp[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], accp[i][j], 0, 0, 0);
            if (DL)
              accn[DUAL ? i : 0][DUAL ? j : 0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                  nf[DL ? i : 0], bf[j], accn[DUAL ? i : 0][DUAL ? j : 0], 0, 0, 0);
          }
      }
    }
  };

  auto flush = [&](const int ks, const bool dl, const bool last) {
    // ---- K-segment boundary (or end of K): flush the exact int32 sums --------------------------------
    int ncol = n0 + wn * C::TN + (lane & 31);
    int mrow = m0 + wm * C::TM + 4 * (lane >> 5);
    asm volatile("" : "+v"(ncol), "+v"(mrow));   // keep the store addressing out of the K loop's live ranges
    if (mode == OUT_DEBUG_ACC) {
      const int o0 = (ks * a.M + mrow) * a.N + ncol;   // S*M*N < 2^31 is checked by the host
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int dm = i * 32 + 8 * (v >> 2) + (v & 3);
            if (mrow + dm < a.M && ncol + j * 32 < a.N) {
              const int o = o0 + dm * a.N + j * 32;
              a.acc_pos[o] = accp[i][j][v];
              a.acc_neg[o] = (DUAL && dl) ? accn[DUAL ? i : 0][DUAL ? j : 0][v] : 0;
            }
          }
        }
    } else {
      const float sp = tb.s_pos[ks], sn = tb.s_neg[ks];
      const int o0 = mrow * a.N + ncol;
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const int n = ncol + j * 32;
        const bool nok = n < a.N;
        const float cw = nok ? seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n] : 0.0f;
        const float cpos = cw * sp, cneg = dl ? cw * sn : 0.0f;
        const float bs = (last && nok && a.bias) ? a.bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < IM; ++i) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float t = cpos * (float)accp[i][j][v];
            if (DUAL) t += cneg * (float)accn[DUAL ? i : 0][DUAL ? j : 0][v];
            if (MULTI) t += fsum[MULTI ? i : 0][MULTI ? j : 0][v];
            if (!last) {
              if (MULTI) fsum[MULTI ? i : 0][MULTI ? j : 0][v] = t;
            } else {
              t += bs;
              const int dm = i * 32 + 8 * (v >> 2) + (v & 3);
              if (mrow + dm < a.M && nok) {
                const int o = o0 + dm * a.N + j * 32;
                if (mode == OUT_F32) reinterpret_cast<float*>(a.y)[o] = t;
                else reinterpret_cast<uint16_t*>(a.y)[o] = f32_to_bf16(t);
              }
            }
          }
        }
      }
    }
    if (!last) {
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) {
          accp[i][j] = (v16i)(0);
          if (DUAL) accn[i][j] = (v16i)(0);
        }
    }
  };

  if constexpr (!MULTI) {
    // one K-segment: the host selects the DUAL instantiation exactly when that segment is dual
    run_segment(std::integral_constant<bool, DUAL>{}, nkt);
    flush(0, DUAL, true);
  } else {
#pragma unroll 1
    for (int ks = 0; ks < tb.S; ++ks) {
      const bool dl = DUAL && (tb.dual[ks] != 0);
      const int kt_end = tb.kseg_off[ks + 1] >> 6;
      if (dl) run_segment(std::integral_constant<bool, DUAL>{}, kt_end);
      else run_segment(std::integral_constant<bool, false>{}, kt_end);
      flush(ks, dl, ks == tb.S - 1);
    }
  }
}

}  // namespace sq
