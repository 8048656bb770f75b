// Large-M SegLinear + DualScale GEMM on int8 MFMA (gfx950, v_mfma_i32_32x32x32_i8).
//
//   acc_+[ks] = X^_+[:, ks] W^[:, ks]^T ,  acc_-[ks] = X^_-[:, ks] W^[:, ks]^T      (Sec. 4.3.2: the two
//   polarity products against the same quantized weight; Sec. 4.2.2 item 2: one product per K-segment)
//   y = sum_ks c_+[ks][n] acc_+[ks] + c_-[ks][n] acc_-[ks] (+ bias)                  (dequant epilogue)
//
// X^_+ >= 0 and X^_- <= 0 have disjoint supports (Sec. 4.3.2: X_+ = max(X, 0), X_- = min(X, 0)), so both
// travel as one int8 matrix X^ = X^_+ + X^_- and are separated again in registers, byte-wise by sign, just
// before the MFMAs: X^_+ = max(X^, 0), X^_- = min(X^, 0).  The dual path therefore costs no operand bytes.
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
//   * One LDS stage holds [X^ rows][W^ rows], SK bytes per row; the X^ and W^ fragments read from it feed
//     both accumulator sets, so each operand is fetched and read once for the two polarity paths.
//   * Inside a row the 16-byte chunks are XOR-swizzled with row bits chosen so that the 16 lanes the
//     LDS serves per cycle (256 B/clk) fall on distinct bank groups for the MFMA fragment read pattern
//     (lane -> row lane%32): chunk ^= (row >> 1) & 7 for 128-byte rows, (row >> 2) & 3 for 64-byte rows.
//     A direct load writes lane l to byte 16*l of a 1 KiB block, so the swizzle is applied to the
//     *global* column each lane fetches.  The k-order inside a fragment is irrelevant as long as both
//     operands use the same one, which they do.
//   * int32 accumulators are exact; at a K-segment boundary they are scaled into an fp32 running sum
//     (only instantiated when the layer has more than one K-segment) and cleared.  A non-dual segment
//     issues only the MFMAs of one set.
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
  static constexpr int AROWS = BM;
  static constexpr int STAGE = (AROWS + BN) * SK;
  static constexpr int RPL = 1024 / SK;            // rows covered by one direct-load instruction
  static constexpr int GA = BM / RPL / NW;         // load instructions per wave and stage
  static constexpr int GB = BN / RPL / NW;
  static constexpr int SUB = SK / 32;              // 32-byte MFMA k-steps per stage
  static constexpr int CPR = SK / 16;              // 16-byte chunks per row
  static constexpr int EPI_ROW = TN * 4 + 16;      // staging row of the epilogue (fp32 worst case, padded)
  static constexpr int EPI = 32 * EPI_ROW;         // per wave
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static constexpr int LT = GA + GB;               // direct-load slots of one stage: X^ groups, W^ groups
  static constexpr int NSLOT = SUB * IM;           // points inside a stage's MFMA stream where loads are interleaved
  static_assert(SK == 64 || SK == 128, "stage depth");
  static_assert(!SHARE || (DUAL && MULTI), "register sharing is a mode of dual multi-segment layers");
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "load groups must divide evenly over the waves");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
  static_assert(NW * EPI <= NSTAGE * STAGE, "epilogue staging must fit in the ring");
  static_assert(NSTAGE * (GA + GB) < 64, "vmcnt is a 6-bit counter");
};

// Polarity split of four packed int8 codes: pos keeps the bytes >= 0, neg the bytes < 0, the others become 0.
//   t = sign bits; w = 0x7F in every negative byte (no borrow crosses a byte); neg = (x & w) | t; pos = x ^ neg
__device__ __forceinline__ void split_polarity(const int x, int& pos, int& neg) {
  const int t = x & (int)0x80808080;
  const int w = t - (int)((unsigned)t >> 7);
  neg = (x & w) | t;
  pos = x ^ neg;
}

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
  const uint32_t ldsB = lds0 + (uint32_t)C::AROWS * SK + (uint32_t)(wave * GB) * 1024u;

  // ---- per-lane fragment read offsets: row = lane%32, chunk = 2h + lane/32, swizzled ---------------
  const int frow = lane & 31, fsw = row_swizzle<SK>(frow), fhi = lane >> 5;
  int foff[SUB];
#pragma unroll
  for (int h = 0; h < SUB; ++h) foff[h] = frow * SK + (((2 * h + fhi) ^ fsw) << 4);
  const char* fragA = smem + (wm * C::TM) * SK;
  const char* fragB = smem + C::AROWS * SK + (wn * C::TN) * SK;

  v16i accp[IM][JN];
  v16i accn[DUAL ? IM : 1][DUAL ? JN : 1];
  v16f fsum[FSUM ? IM : 1][FSUM ? JN : 1];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      accp[i][j] = (v16i)(0);
      if (DUAL) accn[i][j] = (v16i)(0);
      if (FSUM) fsum[i][j] = (v16f)(0.0f);
    }

  const int nkt = a.K >> KSH;
  // ---- direct loads of one stage, issued slot by slot ------------------------------------------------
  // A stage's loads are a list of LT slots (X^ groups, then W^ groups), cut into SUB groups of slots: one
  // group per 32-byte k-step, so that a wave never sits in a burst of load issues while its MFMA pipe idles.
  // K-segments are visited in the order tb.seg_order (identity unless SHARE); stages are numbered in visit
  // order; ikt is the next stage to issue.
  int issued = 0, ikt = 0;
  int ipos = 0, iks = tb.seg_order[0];
  int ik = tb.kseg_off[iks] >> KSH, ik_end = tb.kseg_off[iks + 1] >> KSH;
  const int8_t* ipA = a.xq;    // operand base pointers of the stage being issued
  const int8_t* ipB = a.wq;
  uint32_t iso = 0;
  auto issue_begin = [&]() __attribute__((always_inline)) {
    const int k0 = ik << KSH;
    iso = (uint32_t)(ikt % NSTAGE) * (uint32_t)STAGE;
    ipA = a.xq + k0;
    ipB = a.wq + k0;
  };
  auto issue_slot = [&](const int e) __attribute__((always_inline)) {          // e is a compile-time constant after unrolling
    if (e < GA) glds16(ipA, voffA[e < GA ? e : 0], ldsA + iso + (uint32_t)e * 1024u);
    else glds16(ipB, voffB[e >= GA ? e - GA : 0], ldsB + iso + (uint32_t)(e - GA) * 1024u);
    ++issued;
  };
  auto issue_group = [&](const int g) __attribute__((always_inline)) {         // g is a compile-time constant after unrolling
#pragma unroll
    for (int e = 0; e < LT; ++e)
      if (e * SUB / LT == g) issue_slot(e);
  };
  auto issue_end = [&]() __attribute__((always_inline)) {
    ++ikt;
    if (++ik == ik_end && ipos + 1 < tb.S) {
      iks = tb.seg_order[++ipos];
      ik = tb.kseg_off[iks] >> KSH;
      ik_end = tb.kseg_off[iks + 1] >> KSH;
    }
  };
  // pipeline fill: every buffer of the ring
#pragma unroll 1
  for (int s = 0; s < NSTAGE && s < nkt; ++s) {
    issue_begin();
#pragma unroll
    for (int e = 0; e < LT; ++e) issue_slot(e);
    issue_end();
  }
  // all loads of stage s have landed in this wave's view (loads return in order)
  auto wait_landed = [&](const int s) __attribute__((always_inline)) {
    wait_vmcnt<(NSTAGE - 2) * LT, (NSTAGE - 1) * LT>(issued - (s + 1) * LT);
  };

  // ---- fragments: two register sets, the one being multiplied and the one being fetched ----------------
  v4i bfr[2][JN], afr[2][IM], nfr[2][DUAL ? IM : 1];
  auto load_frags = [&](const int set, const int fo) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IM; ++i) afr[set][i] = *reinterpret_cast<const v4i*>(fragA + i * (32 * SK) + fo);
#pragma unroll
    for (int j = 0; j < JN; ++j) bfr[set][j] = *reinterpret_cast<const v4i*>(fragB + j * (32 * SK) + fo);
  };
  // polarity separation of a fetched X^ fragment set: afr <- X^_+ codes, nfr <- X^_- codes
  auto split_frags = [&](const int set) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        int pos, neg;
        split_polarity(afr[set][i][d], pos, neg);
        afr[set][i][d] = pos;
        nfr[set][DUAL ? i : 0][d] = neg;
      }
  };
  auto stage_off = [&](const int s) __attribute__((always_inline)) { return (s % NSTAGE) * STAGE; };

  // One 32-byte k-step: the MFMAs of fragment set `cur`, while (PF) the fragments of the following k-step
  // are fetched into the other set and separated by polarity, and (GRP >= 0) load group GRP of the stage
  // being issued goes out.  The instruction order is fixed by hand, one MFMA per slot with full scheduling
  // barriers between slots:
  //   * LDS reads are spread over the MFMA stream, X^ fragments first (a burst of reads stalls MFMA issue:
  //     measured 80 % of the MFMA rate with six reads in front of sixteen MFMAs, 94 % with one read per two);
  //   * the separation's VALU work (5 instructions per dword) follows once its fragment had time to arrive,
  //     a dword or two per MFMA, which the matrix pipe (8 issue slots per MFMA) absorbs;
  //   * the direct loads of the group are spread evenly over the slots.
  auto kstep = [&](auto dl_tag, auto pf_tag, auto grp_tag, const int cur, const int fo_next) __attribute__((always_inline)) {
    constexpr bool DL = decltype(dl_tag)::value;
    constexpr bool PF = decltype(pf_tag)::value;
    constexpr int GRP = decltype(grp_tag)::value;
    const int nxt = cur ^ 1;
    constexpr int NM = IM * JN * (DL ? 2 : 1);               // MFMAs of this k-step
    constexpr int NR = PF ? IM + JN : 0;                     // LDS reads (16 bytes per lane each)
    constexpr int RPS = NR > NM ? (NR + NM - 1) / NM : 1;    // LDS reads per slot (1 unless the tile is tiny)
    constexpr int RSTEP = NM * RPS >= 2 * NR ? 2 : 1;        // MFMA slots between reads
    constexpr int ND = (PF && DL) ? IM * 4 : 0;              // dwords to separate
    constexpr int QV_RAW = ((IM - 1) / RPS) * RSTEP + 6;     // first slot with separation work
    constexpr int QV0 = QV_RAW < NM / 2 ? QV_RAW : NM / 2;
    constexpr int DPS = ND ? (ND + (NM - QV0) - 1) / (NM - QV0) : 0;   // dwords per slot
    constexpr int NG = GRP >= 0 ? ((GRP + 1) * LT + SUB - 1) / SUB - (GRP * LT + SUB - 1) / SUB : 0;   // loads of the group
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      {
        const int idx = DL ? (q >> 1) : q;
        const int i = idx / JN, j = idx % JN;
        if (!DL || (q & 1) == 0)
          accp[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afr[cur][i], bfr[cur][j], accp[i][j], 0, 0, 0);
        else
          accn[DUAL ? i : 0][DUAL ? j : 0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
              nfr[cur][DUAL ? i : 0], bfr[cur][j], accn[DUAL ? i : 0][DUAL ? j : 0], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (PF) {
#pragma unroll
        for (int r = 0; r < NR; ++r)                         // read r goes out in slot (r / RPS) * RSTEP
          if ((r / RPS) * RSTEP == q) {
            if (r < IM) afr[nxt][r < IM ? r : 0] = *reinterpret_cast<const v4i*>(fragA + (r < IM ? r : 0) * (32 * SK) + fo_next);
            else bfr[nxt][r >= IM ? r - IM : 0] = *reinterpret_cast<const v4i*>(fragB + (r >= IM ? r - IM : 0) * (32 * SK) + fo_next);
          }
      }
      if (ND && q >= QV0) {
#pragma unroll
        for (int t = 0; t < DPS; ++t) {
          const int w = (q - QV0) * DPS + t;                 // dword index: fragment w / 4, element w % 4
          if (w < ND) {
            int pos, neg;
            split_polarity(afr[nxt][w / 4][w % 4], pos, neg);
            afr[nxt][w / 4][w % 4] = pos;
            nfr[nxt][DUAL ? w / 4 : 0][w % 4] = neg;
          }
        }
      }
      if (GRP >= 0 && NG > 0) {
        int cnt = 0;                                         // the group's loads, spread evenly over the slots
#pragma unroll
        for (int e = 0; e < LT; ++e)
          if (e * SUB / LT == GRP) {
            if (cnt * NM / (NG > 0 ? NG : 1) == q) issue_slot(e);
            ++cnt;
          }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- main loop over one K-segment: DL = this segment runs both polarity paths ----------------------
  // The loop is rotated by one k-step: an iteration starts at the barrier that publishes stage b+1 and frees
  // the buffer of stage b, runs the last k-step of stage b (fetching the first fragments of stage b+1) and
  // the first SUB-1 k-steps of stage b+1, and issues the refill of the freed buffer (stage b+NSTAGE) along
  // the way.  Iterations that still refill and those at the very end of K that do not are separate plain
  // loops, so that the accumulators flow through one MFMA block per loop and stay in accumulation registers.
  int kt = 0;
  auto tail_steps = [&](auto dl_tag, auto more_tag, const int s) __attribute__((always_inline)) {   // k-steps 0 .. SUB-2 of stage s
    constexpr bool MORE = decltype(more_tag)::value;
    const int so = stage_off(s);
#pragma unroll
    for (int h = 0; h + 1 < SUB; ++h) {
      if (h == 0) kstep(dl_tag, std::true_type{}, std::integral_constant<int, MORE ? 1 : -1>{}, 0, so + foff[1]);
      if (h == 1) kstep(dl_tag, std::true_type{}, std::integral_constant<int, MORE ? 2 : -1>{}, 1, so + foff[SUB > 2 ? 2 : 0]);
      if (h == 2) kstep(dl_tag, std::true_type{}, std::integral_constant<int, MORE ? 3 : -1>{}, 0, so + foff[SUB > 3 ? 3 : 0]);
    }
  };
  auto run_segment = [&](auto dl_tag, const int nstages) __attribute__((always_inline)) {
    constexpr bool DL = decltype(dl_tag)::value;
    constexpr int LASTSET = (SUB - 1) & 1;
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
    // segment prologue: stage kt is published, the buffer of stage kt-1 is free; first fragments (exposed once)
    wait_landed(kt);
    __syncthreads();
    load_frags(0, stage_off(kt) + foff[0]);
    if (DL) split_frags(0);
    if (kt > 0 && ikt < nkt) {
      issue_begin();
      issue_group(0);
      tail_steps(dl_tag, std::true_type{}, kt);
      issue_end();
    } else {
      tail_steps(dl_tag, std::false_type{}, kt);
    }
    int b = kt;
    const int b_more_end = (kt_end - 1) < (nkt - NSTAGE) ? (kt_end - 1) : (nkt - NSTAGE);
#pragma unroll 1
    for (; b < b_more_end; ++b) {
      wait_landed(b + 1);
      __syncthreads();
      issue_begin();
      kstep(dl_tag, std::true_type{}, std::integral_constant<int, 0>{}, LASTSET, stage_off(b + 1) + foff[0]);
      tail_steps(dl_tag, std::true_type{}, b + 1);
      issue_end();
    }
#pragma unroll 1
    for (; b < kt_end - 1; ++b) {
      wait_landed(b + 1);
      __syncthreads();
      kstep(dl_tag, std::true_type{}, std::integral_constant<int, -1>{}, LASTSET, stage_off(b + 1) + foff[0]);
      tail_steps(dl_tag, std::false_type{}, b + 1);
    }
    kstep(dl_tag, std::false_type{}, std::integral_constant<int, -1>{}, LASTSET, 0);
    kt = kt_end;
  };

  // Keep the accumulators in accumulation registers at the end of the K loop.  Without this the register
  // allocator starts moving them to ordinary VGPRs inside the last stage (the epilogue's VALU code cannot
  // read AGPRs), which exhausts the VGPR file inside the loop and spills the loop's own address registers.
  auto pin_accumulators = [&]() __attribute__((always_inline)) {
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
  auto flush_mid = [&](const int ks, const bool dl, const bool first) __attribute__((always_inline)) {
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
      // stores share the vector-memory counter with the direct loads but complete out of order with them:
      // drain everything so that the load accounting of the K loop stays valid
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
        // back into accumulation registers at once: left in ordinary VGPRs, the new sums would be spilled to
        // scratch memory around the next K loop
#pragma unroll
        for (int i = 0; i < IM; ++i) asm volatile("" : "+a"(accn[DUAL ? i : 0][DUAL ? j : 0]));
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
  auto flush_last = [&](const int ks, const bool dl, const bool first) __attribute__((always_inline)) {
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
      const int erow = lane / lpr;                       // staged row this lane stores (lanes beyond rows_per_it * lpr idle)
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
          if (erow < rows_per_it && r0 + erow < 32 && m < a.M && nst < a.N)
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
