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
//     registers, and a ring of NSTAGE stages of SK bytes of K each.  SK = 128 makes every row of a
//     stage one full 128-byte cache line (the default); SK = 64 serves layers whose K-segment
//     boundaries are only 64-aligned.
//   * One LDS stage holds [X^_+ rows][X^_- rows][W^ rows], SK bytes per row; the W^ fragments read from
//     it feed both accumulator sets, so W^ is fetched and read once for the two polarity paths.
//   * Inside a row the 16-byte chunks are XOR-swizzled with row bits chosen so that the 16 lanes the
//     LDS serves per cycle (256 B/clk) fall on distinct bank groups for the MFMA fragment read pattern
//     (lane -> row lane%32): chunk ^= (row >> 1) & 7 for 128-byte rows, (row >> 2) & 3 for 64-byte rows.
//     A direct load writes lane l to byte 16*l of a 1 KiB block, so the swizzle is applied to the
//     *global* column each lane fetches.  The k-order inside a fragment is irrelevant as long as both
//     operands use the same one, which they do.
//   * int32 accumulators are exact; at a K-segment boundary they are scaled into an fp32 running sum
//     (only instantiated when the layer has more than one K-segment) and cleared.  A non-dual segment
//     neither loads X^_- nor issues its MFMAs.
//   * The epilogue stages each 32-row block of the wave's result through (now idle) LDS so that global
//     stores are 16 bytes per lane along N (full cache lines) instead of 2-byte scatters.
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
  else if (n >= 32) { SQ_WAIT(32); }
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

template <int BM, int BN, int WM, int WN, int NSTAGE, int SK, bool DUAL, bool MULTI, bool SHARE>
struct MfmaCfg {
  static constexpr int NW = WM * WN;
  static constexpr int THREADS = NW * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;
  static constexpr int IM = TM / 32, JN = TN / 32;
  static constexpr int AROWS = BM * (DUAL ? 2 : 1);
  static constexpr int STAGE = (AROWS + BN) * SK;
  static constexpr int RPL = 1024 / SK;            // rows covered by one direct-load instruction
  static constexpr int GA = BM / RPL / NW;         // load instructions per wave and stage, per polarity
  static constexpr int GB = BN / RPL / NW;
  static constexpr int SUB = SK / 32;              // 32-byte MFMA k-steps per stage
  static constexpr int CPR = SK / 16;              // 16-byte chunks per row
  static constexpr int EPI_ROW = TN * 4 + 16;      // staging row of the epilogue (fp32 worst case, padded)
  static constexpr int EPI = 32 * EPI_ROW;         // per wave
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static constexpr int LT = 2 * GA + GB;           // direct-load slots of one stage: X^_+ groups, X^_- groups, W^ groups
  static constexpr int NSLOT = SUB * IM;           // points inside a stage's MFMA stream where loads are interleaved
  static_assert(SK == 64 || SK == 128, "stage depth");
  static_assert(!SHARE || (DUAL && MULTI), "register sharing is a mode of dual multi-segment layers");
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "load groups must divide evenly over the waves");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
  static_assert(NW * EPI <= NSTAGE * STAGE, "epilogue staging must fit in the ring");
  static_assert((NSTAGE - 1) * (2 * GA + GB) < 64, "vmcnt is a 6-bit counter");
};

template <int SK> __device__ __forceinline__ int row_swizzle(int row) {
  return SK == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int BM, int BN, int WM, int WN, int NSTAGE, int SK, int MINB, bool DUAL, bool MULTI, bool SHARE>
__global__ __launch_bounds__(WM * WN * 64, MINB) void seglinear_mfma_kernel(const GemmArgs a, const GemmTable tb,
                                                                         const int mode) {
  using C = MfmaCfg<BM, BN, WM, WN, NSTAGE, SK, DUAL, MULTI, SHARE>;
  constexpr bool FSUM = MULTI && !SHARE;      // a separate fp32 running-sum register set
  constexpr int IM = C::IM, JN = C::JN, GA = C::GA, GB = C::GB, STAGE = C::STAGE, RPL = C::RPL, SUB = C::SUB;
  constexpr int KSH = SK == 128 ? 7 : 6;
  constexpr int LT = C::LT, NSLOT = C::NSLOT;
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];

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
  // lane -> (row lane / CPR of the instruction's RPL rows, 16 B slot lane % CPR holding chunk slot ^ swizzle(row))
  const int lrow = lane / C::CPR, lslot = lane % C::CPR;
  uint32_t voffA[GA], voffB[GB];
#pragma unroll
  for (int g = 0; g < GA; ++g) {
    const int rt = (wave * GA + g) * RPL + lrow;            // row inside the tile
    int r = m0 + rt;
    r = r < a.M ? r : a.M - 1;                              // ragged tail: re-read the last row, masked at the store
    voffA[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)((lslot ^ row_swizzle<SK>(rt)) << 4);
  }
#pragma unroll
  for (int g = 0; g < GB; ++g) {
    const int rt = (wave * GB + g) * RPL + lrow;
    int r = n0 + rt;
    r = r < a.N ? r : a.N - 1;
    voffB[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)((lslot ^ row_swizzle<SK>(rt)) << 4);
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)SQ_LDS(smem);
  const uint32_t ldsA = lds0 + (uint32_t)(wave * GA) * 1024u;
  const uint32_t ldsN = ldsA + (uint32_t)BM * SK;
  const uint32_t ldsB = lds0 + (uint32_t)C::AROWS * SK + (uint32_t)(wave * GB) * 1024u;

  // ---- per-lane fragment read offsets: row = lane%32, chunk = 2h + lane/32, swizzled ---------------
  const int frow = lane & 31, fsw = row_swizzle<SK>(frow), fhi = lane >> 5;
  int foff[SUB];
#pragma unroll
  for (int h = 0; h < SUB; ++h) foff[h] = frow * SK + (((2 * h + fhi) ^ fsw) << 4);
  const char* fragA = smem + (wm * C::TM) * SK;
  const char* fragN = fragA + BM * SK;
  const char* fragB = smem + C::AROWS * SK + (wn * C::TN) * SK;

  v16i accp[IM][JN];
  v16i accn[DUAL ? IM : 1][DUAL ? JN : 1];
  float fsum[FSUM ? IM : 1][FSUM ? JN : 1][16];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      accp[i][j] = (v16i)(0);
      if (DUAL) accn[i][j] = (v16i)(0);
      if (FSUM)
#pragma unroll
        for (int v = 0; v < 16; ++v) fsum[i][j][v] = 0.0f;
    }

  const int nkt = a.K >> KSH;
  // ---- direct loads of one stage, issued slot by slot ------------------------------------------------
  // A stage's loads are a list of LT slots (X^_+ groups, X^_- groups, W^ groups).  The pipeline fill issues
  // whole stages; in steady state the slots of the next stage are spread over the current stage's MFMA
  // stream, so that a wave never sits in a burst of load issues while its MFMA pipe is idle.
  // K-segments are visited in the order tb.seg_order (identity unless SHARE); stages are numbered in visit order.
  int issued = 0, ikt = 0;
  int ipos = 0, iks = tb.seg_order[0];
  int ik = tb.kseg_off[iks] >> KSH, ik_end = tb.kseg_off[iks + 1] >> KSH;
  const int8_t* ipA = a.xp;    // operand base pointers of the stage being issued
  const int8_t* ipN = a.xn;
  const int8_t* ipB = a.wq;
  bool idl = false;
  uint32_t iso = 0;
  auto issue_begin = [&]() {
    const int k0 = ik << KSH;
    idl = DUAL && (tb.dual[iks] != 0);
    iso = (uint32_t)(ikt % NSTAGE) * (uint32_t)STAGE;
    ipA = a.xp + k0;
    ipN = a.xn + k0;
    ipB = a.wq + k0;
  };
  auto issue_slot = [&](const int e) {          // e is a compile-time constant after unrolling
    if (e < GA) {
      glds16(ipA, voffA[e < GA ? e : 0], ldsA + iso + (uint32_t)e * 1024u);
      ++issued;
    } else if (e < 2 * GA) {
      if (idl) {
        glds16(ipN, voffA[(e - GA) < GA ? (e >= GA ? e - GA : 0) : 0], ldsN + iso + (uint32_t)(e - GA) * 1024u);
        ++issued;
      }
    } else {
      glds16(ipB, voffB[(e - 2 * GA) < GB ? (e >= 2 * GA ? e - 2 * GA : 0) : 0], ldsB + iso + (uint32_t)(e - 2 * GA) * 1024u);
      ++issued;
    }
  };
  auto issue_end = [&]() {
    ++ikt;
    if (++ik == ik_end && ipos + 1 < tb.S) {
      iks = tb.seg_order[++ipos];
      ik = tb.kseg_off[iks] >> KSH;
      ik_end = tb.kseg_off[iks + 1] >> KSH;
    }
  };
#pragma unroll 1
  for (int s = 0; s < NSTAGE - 1 && s < nkt; ++s) {
    issue_begin();
#pragma unroll
    for (int e = 0; e < LT; ++e) issue_slot(e);
    issue_end();
  }

  // ---- main loop over one K-segment: DL = this segment runs both polarity paths ----------------------
  int kt = 0, retired = 0;
  // One stage of MFMAs; MORE = the next stage's direct loads are interleaved (one share per MFMA row).
  auto compute_stage = [&](auto dl_tag, auto more_tag) {
    constexpr bool DL = decltype(dl_tag)::value;
    constexpr bool MORE = decltype(more_tag)::value;
    const int so = (kt % NSTAGE) * STAGE;
#pragma unroll
    for (int h = 0; h < SUB; ++h) {
      const int fo = so + foff[h];
      v4i bf[JN], af[IM], nf[DL ? IM : 1];
#pragma unroll
      for (int j = 0; j < JN; ++j) bf[j] = *reinterpret_cast<const v4i*>(fragB + j * (32 * SK) + fo);
#pragma unroll
      for (int i = 0; i < IM; ++i) af[i] = *reinterpret_cast<const v4i*>(fragA + i * (32 * SK) + fo);
      if (DL) {
#pragma unroll
        for (int i = 0; i < IM; ++i) nf[i] = *reinterpret_cast<const v4i*>(fragN + i * (32 * SK) + fo);
      }
#pragma unroll
      for (int i = 0; i < IM; ++i) {
#pragma unroll
        for (int j = 0; j < JN; ++j) {
          accp[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], accp[i][j], 0, 0, 0);
          if (DL)
            accn[DUAL ? i : 0][DUAL ? j : 0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                nf[DL ? i : 0], bf[j], accn[DUAL ? i : 0][DUAL ? j : 0], 0, 0, 0);
        }
        if (MORE) {
#pragma unroll
          for (int e = 0; e < LT; ++e)
            if (e * NSLOT / LT == h * IM + i) issue_slot(e);
        }
      }
    }
  };

  // ---- main loop over one K-segment: DL = this segment runs both polarity paths ----------------------
  // Two plain loops (first the stages that still prefetch, then the last NSTAGE-1 stages of K that do not)
  // rather than one loop with a branch: the accumulators then flow through a single MFMA block per loop and
  // stay in accumulation registers.
  auto run_segment = [&](auto dl_tag, const int nstages) {
    constexpr bool DL = decltype(dl_tag)::value;
    // stages of this segment that still prefetch (n_pf) and those at the very end of K that do not
    const int pf_left = nkt - (NSTAGE - 1) - kt;
    const int n_pf = pf_left < 0 ? 0 : (pf_left < nstages ? pf_left : nstages);
    const int kt_pf_end = kt + n_pf;
    const int kt_end = kt + nstages;
    // Start fresh live ranges for the per-lane addresses here: if the register allocator has to spill them
    // around the (register-hungry) flush code, the reload then happens once in front of the loop.  A reload
    // inside the loop would come with compiler-inserted vmcnt waits that drain the direct-load pipeline.
#pragma unroll
    for (int g = 0; g < GA; ++g) asm volatile("" : "+v"(voffA[g]));
#pragma unroll
    for (int g = 0; g < GB; ++g) asm volatile("" : "+v"(voffB[g]));
#pragma unroll
    for (int h = 0; h < SUB; ++h) asm volatile("" : "+v"(foff[h]));
#pragma unroll 1
    for (; kt < kt_pf_end; ++kt) {
      retired += GA * (DL ? 2 : 1) + GB;         // loads of stage kt are the oldest outstanding ones
      wait_vmcnt<(NSTAGE - 2) * (2 * GA + GB), (NSTAGE - 2) * (GA + GB)>(issued - retired);
      __syncthreads();                           // stage kt visible to all waves; stage kt-1 free for reuse
      issue_begin();                             // stage kt + NSTAGE - 1 goes into the buffer just freed
      compute_stage(dl_tag, std::true_type{});
      issue_end();
    }
#pragma unroll 1
    for (; kt < kt_end; ++kt) {
      retired += GA * (DL ? 2 : 1) + GB;
      wait_vmcnt<(NSTAGE - 2) * (2 * GA + GB), (NSTAGE - 2) * (GA + GB)>(issued - retired);
      __syncthreads();
      compute_stage(dl_tag, std::false_type{});
    }
  };

  // Keep the accumulators in accumulation registers at the end of the K loop.  Without this the register
  // allocator starts moving them to ordinary VGPRs inside the last stage (the epilogue's VALU code cannot
  // read AGPRs), which exhausts the VGPR file inside the loop and spills the loop's own address registers.
  auto pin_accumulators = [&]() {
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        asm volatile("" : "+a"(accp[i][j]));
        if (DUAL) asm volatile("" : "+a"(accn[DUAL ? i : 0][DUAL ? j : 0]));
      }
  };

  // ---- K-segment boundary: scale the exact int32 sums into the fp32 running sum, clear them ----------
  // SHARE: the layer has exactly one dual K-segment and it is visited first.  Two int32 sets are live only
  // during that segment; at its end the X^_- set's registers are re-used for the fp32 running sum (its bits
  // are kept in accn), and every later segment accumulates in accp alone.  `first` = first visited segment.
  auto flush_mid = [&](const int ks, const bool dl, const bool first) {
    int ncol = n0 + wn * C::TN + (lane & 31);
    int mrow = m0 + wm * C::TM + 4 * (lane >> 5);
    asm volatile("" : "+v"(ncol), "+v"(mrow));   // keep this addressing out of the K loop's live ranges
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
              a.acc_neg[o] = (DUAL && dl && (!SHARE || first)) ? accn[DUAL ? i : 0][DUAL ? j : 0][v] : 0;
            }
          }
        }
    } else if (SHARE) {
      const float sp = tb.s_pos[ks], sn = tb.s_neg[ks];
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const int n = ncol + j * 32;
        const float cw = (n < a.N) ? seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n] : 0.0f;
        const float cpos = cw * sp, cneg = cw * sn;
#pragma unroll
        for (int i = 0; i < IM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int old = accn[DUAL ? i : 0][DUAL ? j : 0][v];
            const float prev = first ? cneg * (float)old : __int_as_float(old);
            accn[DUAL ? i : 0][DUAL ? j : 0][v] = __float_as_int(prev + cpos * (float)accp[i][j][v]);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (FSUM) {
      const float sp = tb.s_pos[ks], sn = tb.s_neg[ks];
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const int n = ncol + j * 32;
        const float cw = (n < a.N) ? seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n] : 0.0f;
        const float cpos = cw * sp, cneg = dl ? cw * sn : 0.0f;
#pragma unroll
        for (int i = 0; i < IM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float t = cpos * (float)accp[i][j][v];
            if (DUAL) t += cneg * (float)accn[DUAL ? i : 0][DUAL ? j : 0][v];
            fsum[FSUM ? i : 0][FSUM ? j : 0][v] += t;
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        accp[i][j] = (v16i)(0);
        if (DUAL && (!SHARE || mode == OUT_DEBUG_ACC)) accn[i][j] = (v16i)(0);
      }
  };

  // ---- last K-segment: dequantize, add bias, store ----------------------------------------------------
  auto flush_last = [&](const int ks, const bool dl, const bool first) {
    if (mode == OUT_DEBUG_ACC) { flush_mid(ks, dl, first); return; }
    int ncol = n0 + wn * C::TN + (lane & 31);
    int mrow = m0 + wm * C::TM + 4 * (lane >> 5);
    asm volatile("" : "+v"(ncol), "+v"(mrow));
    const float sp = tb.s_pos[ks], sn = tb.s_neg[ks];
    float cpos[JN], cneg[JN], bs[JN];
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      const int n = ncol + j * 32;
      const bool nok = n < a.N;
      const float cw = nok ? seg_scale_of(tb, ks, n) * a.wscale[(size_t)ks * a.N + n] : 0.0f;
      cpos[j] = cw * sp;
      cneg[j] = dl ? cw * sn : 0.0f;
      bs[j] = (nok && a.bias) ? a.bias[n] : 0.0f;
    }
    // 1) dequantize in place: the accumulator registers now hold the fp32 result bits
#pragma unroll
    for (int j = 0; j < JN; ++j) {
#pragma unroll
      for (int i = 0; i < IM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float t = cpos[j] * (float)accp[i][j][v];
          if (SHARE) t += __int_as_float(accn[DUAL ? i : 0][DUAL ? j : 0][v]);   // running sum (never the first segment)
          else if (DUAL) t += cneg[j] * (float)accn[DUAL ? i : 0][DUAL ? j : 0][v];
          if (FSUM) t += fsum[FSUM ? i : 0][FSUM ? j : 0][v];
          t += bs[j];
          accp[i][j][v] = __float_as_int(t);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // 2) store
    const int esz = (mode == OUT_F32) ? 4 : 2;
    const bool vec = (a.N % (16 / esz)) == 0 && (reinterpret_cast<uintptr_t>(a.y) % 16 == 0);
    if (vec) {
      // Stage 32 rows x TN columns at a time through this wave's slice of the (idle) ring, then store
      // 16 bytes per lane along N.
      __syncthreads();                                   // every wave is done reading operand stages
      char* stg = smem + wave * C::EPI;
      const int rowb = C::TN * esz + 16;                 // padded staging row
      const int cpl = 16 / esz;                          // columns per 16-byte store
      const int lpr = C::TN / cpl;                       // lanes that cover one staged row
      const int rows_per_it = 64 / lpr;
      char* wbase = stg + (4 * (lane >> 5)) * rowb + (lane & 31) * esz;
      const char* rbase = stg + (lane / lpr) * rowb + (lane % lpr) * 16;
      const int mbase = m0 + wm * C::TM + lane / lpr;
      const int nst = n0 + wn * C::TN + (lane % lpr) * cpl;
#pragma unroll
      for (int i = 0; i < IM; ++i) {
#pragma unroll
        for (int j = 0; j < JN; ++j) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            char* p = wbase + (8 * (v >> 2) + (v & 3)) * rowb + (j * 32) * esz;
            const float t = __int_as_float(accp[i][j][v]);
            if (mode == OUT_F32) *reinterpret_cast<float*>(p) = t;
            else *reinterpret_cast<uint16_t*>(p) = f32_to_bf16(t);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        // read back row-contiguous and store
#pragma unroll 2
        for (int r0 = 0; r0 < 32; r0 += rows_per_it) {
          const v4i val = *reinterpret_cast<const v4i*>(rbase + r0 * rowb);
          const int m = mbase + i * 32 + r0;
          if (m < a.M && nst < a.N)
            *reinterpret_cast<v4i*>(reinterpret_cast<char*>(a.y) + ((size_t)m * a.N + nst) * esz) = val;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      const int o0 = mrow * a.N + ncol;
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const bool nok = ncol + j * 32 < a.N;
#pragma unroll
        for (int i = 0; i < IM; ++i) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float t = __int_as_float(accp[i][j][v]);
            const int dm = i * 32 + 8 * (v >> 2) + (v & 3);
            if (mrow + dm < a.M && nok) {
              const int o = o0 + dm * a.N + j * 32;
              if (mode == OUT_F32) reinterpret_cast<float*>(a.y)[o] = t;
              else reinterpret_cast<uint16_t*>(a.y)[o] = f32_to_bf16(t);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  };

  if constexpr (!MULTI) {
    // one K-segment: the host selects the DUAL instantiation exactly when that segment is dual
    run_segment(std::integral_constant<bool, DUAL>{}, nkt);
    pin_accumulators();
    flush_last(0, DUAL, true);
  } else if constexpr (SHARE) {
    // the dual K-segment first (both accumulator sets), then the single-scale ones (one set + running sum)
    {
      const int ks = tb.seg_order[0];
      run_segment(std::true_type{}, (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH);
      pin_accumulators();
      flush_mid(ks, true, true);
    }
#pragma unroll 1
    for (int pos = 1; pos < tb.S; ++pos) {
      const int ks = tb.seg_order[pos];
      run_segment(std::false_type{}, (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH);
      pin_accumulators();
      if (pos == tb.S - 1) flush_last(ks, false, false);
      else flush_mid(ks, false, false);
    }
  } else {
#pragma unroll 1
    for (int pos = 0; pos < tb.S; ++pos) {
      const int ks = tb.seg_order[pos];
      const bool dl = DUAL && (tb.dual[ks] != 0);
      const int nst = (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH;
      if (dl) run_segment(std::integral_constant<bool, DUAL>{}, nst);
      else run_segment(std::integral_constant<bool, false>{}, nst);
      pin_accumulators();
      if (pos == tb.S - 1) flush_last(ks, dl, pos == 0);
      else flush_mid(ks, dl, pos == 0);
    }
  }
}

}  // namespace sq
