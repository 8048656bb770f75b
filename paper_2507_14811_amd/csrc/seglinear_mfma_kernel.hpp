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
//     sub-tile built from 32x32x32 int8 MFMAs.  W^ rows are the MFMA "A" operand and X^ rows the "B"
//     operand, so a lane's 16 results of a block are four runs of four consecutive output columns of
//     one token row.
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
//   * The epilogue needs no transpose: each lane scales its runs with per-column constants fetched
//     16 bytes at a time and stores them directly as 16-byte (fp32) or 8-byte (bf16, hardware
//     round-to-nearest-even pack) pieces; the pieces of one row written by a wave are contiguous.
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

template <int BM, int BN, int WM, int WN, int NSTAGE, int SK, bool DUAL, bool MULTI, bool SHARE, bool FP8 = false>
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
  static constexpr int FW = FP8 ? 8 : 4;           // dwords of K per lane and MFMA: int8 32x32x32 / fp8 32x32x64
  static constexpr int SUB = SK / (8 * FW);        // MFMA k-steps per stage (32 bytes of K each, 64 for fp8)
  static constexpr int CPR = SK / 16;              // 16-byte chunks per row
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static constexpr int LT = GA + GB;               // direct-load slots of one stage: X^ groups, W^ groups
  static constexpr int NSLOT = SUB * IM;           // points inside a stage's MFMA stream where loads are interleaved
  static_assert(SK == 64 || SK == 128, "stage depth");
  static_assert(!SHARE || (DUAL && MULTI), "register sharing is a mode of dual multi-segment layers");
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
  static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "load groups must divide evenly over the waves");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS ring exceeds 160 KB");
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

// TOK: dynamic per-token activation steps (App. B, 4-bit settings): the flushes take s_+ / s_- of every lane's own token
// rows from a.tok_steps [2][M][S] instead of the layer's static steps.
// FP8: the codes are OCP E4M3 bytes and the products run on v_mfma_f32_32x32x64_f8f6f4 (no block scales)
// (64 bytes of K per instruction: a lane's operand is two neighbouring 16-byte chunks); the sums are fp32, kept as bits
// in the same accumulator registers; X^_- holds the codes with the sign bit set.
template <int BM, int BN, int WM, int WN, int NSTAGE, int SK, int MINB, bool DUAL, bool MULTI, bool SHARE, bool TOK = false,
          bool FP8 = false>
__global__ __launch_bounds__(WM * WN * 64, MINB) void seglinear_mfma_kernel(const GemmArgs a, const GemmTable tb,
                                                                         const int mode) {
  using C = MfmaCfg<BM, BN, WM, WN, NSTAGE, SK, DUAL, MULTI, SHARE, FP8>;
  constexpr int FW = C::FW, CH = FW / 4;      // dwords / 16-byte chunks of a lane's operand
  using vfrag = std::conditional_t<FP8, v8i, v4i>;
  constexpr bool FSUM = MULTI && !SHARE;      // a separate fp32 running-sum register set
  constexpr int IM = C::IM, JN = C::JN, GA = C::GA, GB = C::GB, STAGE = C::STAGE, RPL = C::RPL, SUB = C::SUB;
  constexpr int KSH = SK == 128 ? 7 : 6;
  constexpr int LT = C::LT, NSLOT = C::NSLOT;
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- persistent workgroups: this workgroup's sequence of output tiles ------------------------------
  // Workgroup ids are dealt round-robin to the 8 XCDs.  Each XCD owns a contiguous run of the (panel-ordered)
  // tile list and its workgroups walk that run side by side, so the tiles in flight on one XCD are
  // neighbours that share X^ and W^ lines in its L2.  The load pipeline runs across tile boundaries: the
  // first stages of the next tile are fetched while the current tile is dequantized and stored.
  const int ntiles = a.tiles_m * a.tiles_n;
  const int xcd = blockIdx.x & 7, xlocal = blockIdx.x >> 3;
  const int xper = ntiles >> 3, xrem = ntiles & 7;
  const int xstart = xcd < xrem ? xcd * (xper + 1) : xrem * (xper + 1) + (xcd - xrem) * xper;
  const int xcnt = xper + (xcd < xrem ? 1 : 0);                       // tiles of this XCD
  const int xwg = (int)(gridDim.x >> 3) + (xcd < (int)(gridDim.x & 7) ? 1 : 0);   // workgroups on this XCD
  const int ntile_wg = xlocal < xcnt ? (xcnt - xlocal + xwg - 1) / xwg : 0;        // tiles of this workgroup
  if (ntile_wg == 0) return;                                          // uniform: the whole workgroup leaves
  auto tile_origin = [&](const int it, int& tm0, int& tn0) __attribute__((always_inline)) {
    const int logical = xstart + it * xwg + xlocal;
    const int gsz = a.group_m * a.tiles_n;
    const int g = logical / gsz, in = logical - g * gsz;
    const int first = g * a.group_m;
    const int gm = (a.tiles_m - first) < a.group_m ? (a.tiles_m - first) : a.group_m;
    const int tn = in / gm;
    tm0 = (first + (in - tn * gm)) * BM;
    tn0 = tn * BN;
  };

  // ---- per-lane source offsets of the direct loads of the tile being fetched --------------------------
  // lane -> (row lane / CPR of the instruction's RPL rows, 16 B slot lane % CPR holding chunk slot ^ swizzle(row))
  const int lrow = lane / C::CPR, lslot = lane % C::CPR;
  uint32_t voffA[GA], voffB[GB];
  auto set_issue_tile = [&](const int it) __attribute__((always_inline)) {
    int im0, in0;
    tile_origin(it, im0, in0);
#pragma unroll
    for (int g = 0; g < GA; ++g) {
      const int rt = (wave * GA + g) * RPL + lrow;            // row inside the tile
      int r = im0 + rt;
      r = r < a.M ? r : a.M - 1;                              // ragged tail: re-read the last row, masked at the store
      voffA[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)((lslot ^ row_swizzle<SK>(rt)) << 4);
    }
#pragma unroll
    for (int g = 0; g < GB; ++g) {
      const int rt = (wave * GB + g) * RPL + lrow;
      int r = in0 + rt;
      r = r < a.N ? r : a.N - 1;
      voffB[g] = (uint32_t)r * (uint32_t)a.K + (uint32_t)((lslot ^ row_swizzle<SK>(rt)) << 4);
    }
  };
  set_issue_tile(0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)SQ_LDS(smem);
  const uint32_t ldsA = lds0 + (uint32_t)(wave * GA) * 1024u;
  const uint32_t ldsB = lds0 + (uint32_t)C::AROWS * SK + (uint32_t)(wave * GB) * 1024u;

  // ---- per-lane fragment read offsets: row = lane%32, chunk = 2h + lane/32, swizzled ---------------
  const int frow = lane & 31, fsw = row_swizzle<SK>(frow), fhi = lane >> 5;
  int foff[SUB];
#pragma unroll
  for (int h = 0; h < SUB; ++h) foff[h] = frow * SK + (((2 * CH * h + CH * fhi) ^ fsw) << 4);   // fp8: second chunk at this ^ 16
  const char* fragA = smem + (wm * C::TM) * SK;
  const char* fragB = smem + C::AROWS * SK + (wn * C::TN) * SK;

  v16i accp[IM][JN];
  v16i accn[DUAL ? IM : 1][DUAL ? JN : 1];
  v16f fsum[FSUM ? IM : 1][FSUM ? JN : 1];
  auto clear_accumulators = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        accp[i][j] = (v16i)(0);
        if (DUAL) accn[i][j] = (v16i)(0);
        if (FSUM) fsum[i][j] = (v16f)(0.0f);
      }
  };

  const int nkt_tile = a.K >> KSH;              // stages of one tile
  const int nkt = nkt_tile * ntile_wg;          // stages of this workgroup, numbered across its tiles
  // ---- direct loads of one stage, issued slot by slot ------------------------------------------------
  // A stage's loads are a list of LT slots (X^ groups, then W^ groups), cut into SUB groups of slots: one
  // group per 32-byte k-step, so that a wave never sits in a burst of load issues while its MFMA pipe idles.
  // K-segments are visited in the order tb.seg_order (identity unless SHARE); stages are numbered in visit
  // order; ikt is the next stage to issue.
  int issued = 0, ikt = 0, iit = 0;
  int ipos = 0, iks = tb.seg_order[0];
  int ik = tb.kseg_off[iks] >> KSH, ik_end = tb.kseg_off[iks + 1] >> KSH;
  const int8_t* ipA = a.xq;    // operand base pointers of the stage being issued
  const int8_t* ipB = a.wq;
  uint32_t iso = 0;
  // The direct loads take their base address and LDS offset in scalar registers.  The values are uniform,
  // but the compiler does not always prove it (it then hands the inline assembly a vector register pair,
  // which does not assemble): readfirstlane states it, and folds away where uniformity is known.
  auto uniform_ptr = [](const int8_t* p) __attribute__((always_inline)) {
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return reinterpret_cast<const int8_t*>(((uint64_t)hi << 32) | lo);
  };
  auto issue_begin = [&]() __attribute__((always_inline)) {
    const int k0 = ik << KSH;
    iso = __builtin_amdgcn_readfirstlane((uint32_t)(ikt % NSTAGE) * (uint32_t)STAGE);
    ipA = uniform_ptr(a.xq + k0);
    ipB = uniform_ptr(a.wq + k0);
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
  // Moving the fetch cursor to the next tile recomputes the per-lane addresses.  It is kept out of the K loops
  // (which run at most to the end of the tile being fetched, see run_segment): inside them the recomputation's
  // spill reloads would come with compiler-inserted vmcnt waits that drain the direct-load pipeline every stage.
  auto issue_next_tile_if_done = [&]() __attribute__((always_inline)) {
    if (ikt == (iit + 1) * nkt_tile && iit + 1 < ntile_wg) {
      set_issue_tile(++iit);
      ipos = 0;
      iks = tb.seg_order[0];
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
    issue_next_tile_if_done();
  }
  // all loads of stage s have landed in this wave's view (loads return in order)
  auto wait_landed = [&](const int s) __attribute__((always_inline)) {
    wait_vmcnt<(NSTAGE - 2) * LT, (NSTAGE - 1) * LT>(issued - (s + 1) * LT);
  };

  // ---- fragments: two register sets, the one being multiplied and the one being fetched ----------------
  vfrag bfr[2][JN], afr[2][IM], nfr[2][DUAL ? IM : 1];
  auto read_chunk = [&](vfrag& f, const int c, const char* p) __attribute__((always_inline)) {   // 16 bytes into dwords 4c .. 4c+3
    const v4i t = *reinterpret_cast<const v4i*>(p);
    if constexpr (FP8) {
#pragma unroll
      for (int d = 0; d < 4; ++d) f[4 * c + d] = t[d];
    } else {
      f = t;
    }
  };
  auto load_frags = [&](const int set, const int fo) __attribute__((always_inline)) {
    if constexpr (FP8) {
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int c = 0; c < CH; ++c) read_chunk(afr[set][i], c, fragA + i * (32 * SK) + (fo ^ (16 * c)));
#pragma unroll
      for (int j = 0; j < JN; ++j)
#pragma unroll
        for (int c = 0; c < CH; ++c) read_chunk(bfr[set][j], c, fragB + j * (32 * SK) + (fo ^ (16 * c)));
    } else {
#pragma unroll
      for (int i = 0; i < IM; ++i) afr[set][i] = *reinterpret_cast<const v4i*>(fragA + i * (32 * SK) + fo);
#pragma unroll
      for (int j = 0; j < JN; ++j) bfr[set][j] = *reinterpret_cast<const v4i*>(fragB + j * (32 * SK) + fo);
    }
  };
  // polarity separation of a fetched X^ fragment set: afr <- X^_+ codes, nfr <- X^_- codes
  auto split_frags = [&](const int set) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int d = 0; d < FW; ++d) {
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
  //   * the direct loads of the group go into the slots that carry neither an LDS read nor separation work.
  auto kstep = [&](auto dl_tag, auto pf_tag, auto grp_tag, const int cur, const int fo_next) __attribute__((always_inline)) {
    constexpr bool DL = decltype(dl_tag)::value;
    constexpr bool PF = decltype(pf_tag)::value;
    constexpr int GRP = decltype(grp_tag)::value;
    const int nxt = cur ^ 1;
    constexpr int NM = IM * JN * (DL ? 2 : 1);               // MFMAs of this k-step
    constexpr int NR = PF ? (IM + JN) * CH : 0;              // LDS reads (16 bytes per lane each)
    constexpr int RPS = NR > NM ? (NR + NM - 1) / NM : 1;    // LDS reads per slot (1 unless the tile is tiny)
    constexpr int RSTEP = NM * RPS >= 2 * NR ? 2 : 1;        // MFMA slots between reads
    constexpr int ND = (PF && DL) ? IM * FW : 0;             // dwords to separate
    constexpr int QV_RAW = ((IM * CH - 1) / RPS) * RSTEP + (FP8 ? 3 : 6);   // first slot with separation work
    constexpr int QV0 = QV_RAW < NM / 2 ? QV_RAW : NM / 2;
    constexpr int DPS = ND ? (ND + (NM - QV0) - 1) / (NM - QV0) : 0;   // dwords per slot
    constexpr int NG = GRP >= 0 ? ((GRP + 1) * LT + SUB - 1) / SUB - (GRP * LT + SUB - 1) / SUB : 0;   // loads of the group
#pragma unroll
    for (int q = 0; q < NM; ++q) {
      {
        const int idx = DL ? (q >> 1) : q;
        const int i = idx / JN, j = idx % JN;
        if constexpr (FP8) {
          constexpr int kUnit = 0;                           // constant-zero scale operands select the unscaled instruction
          if (!DL || (q & 1) == 0)
            accp[i][j] = __builtin_bit_cast(v16i, __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                bfr[cur][j], afr[cur][i], __builtin_bit_cast(v16f, accp[i][j]), 0, 0, 0, kUnit, 0, kUnit));
          else
            accn[DUAL ? i : 0][DUAL ? j : 0] = __builtin_bit_cast(v16i, __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                bfr[cur][j], nfr[cur][DUAL ? i : 0], __builtin_bit_cast(v16f, accn[DUAL ? i : 0][DUAL ? j : 0]), 0, 0, 0, kUnit,
                0, kUnit));
        } else {
          if (!DL || (q & 1) == 0)
            accp[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bfr[cur][j], afr[cur][i], accp[i][j], 0, 0, 0);
          else
            accn[DUAL ? i : 0][DUAL ? j : 0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                bfr[cur][j], nfr[cur][DUAL ? i : 0], accn[DUAL ? i : 0][DUAL ? j : 0], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (PF) {
#pragma unroll
        for (int r = 0; r < NR; ++r)                         // read r goes out in slot (r / RPS) * RSTEP
          if ((r / RPS) * RSTEP == q) {
            if constexpr (FP8) {
              const int f = r / CH, c = r % CH;              // fragment and 16-byte half
              if (f < IM) read_chunk(afr[nxt][f < IM ? f : 0], c, fragA + (f < IM ? f : 0) * (32 * SK) + (fo_next ^ (16 * c)));
              else read_chunk(bfr[nxt][f >= IM ? f - IM : 0], c, fragB + (f >= IM ? f - IM : 0) * (32 * SK) + (fo_next ^ (16 * c)));
            } else {
              if (r < IM) afr[nxt][r < IM ? r : 0] = *reinterpret_cast<const v4i*>(fragA + (r < IM ? r : 0) * (32 * SK) + fo_next);
              else bfr[nxt][r >= IM ? r - IM : 0] = *reinterpret_cast<const v4i*>(fragB + (r >= IM ? r - IM : 0) * (32 * SK) + fo_next);
            }
          }
      }
      if (ND && q >= QV0) {
#pragma unroll
        for (int t = 0; t < DPS; ++t) {
          const int w = (q - QV0) * DPS + t;                 // dword index: fragment w / FW, element w % FW
          if (w < ND) {
            int pos, neg;
            split_polarity(afr[nxt][w / FW][w % FW], pos, neg);
            afr[nxt][w / FW][w % FW] = pos;
            nfr[nxt][DUAL ? w / FW : 0][w % FW] = neg;
          }
        }
      }
      if (GRP >= 0 && NG > 0) {
        // The group's loads go into the slots that carry neither an LDS read nor separation work (a direct load
        // occupies the wave's issue for ~20 clocks, which fits under one MFMA only if nothing else shares the
        // slot); what does not fit there is spread evenly over all slots.
        int nfree = 0, myfree = -1;
#pragma unroll
        for (int qq = 0; qq < NM; ++qq) {
          const bool has_read = PF && (qq % RSTEP == 0) && (qq / RSTEP) * RPS < NR;
          const bool has_valu = ND && qq >= QV0;
          if (!has_read && !has_valu) {
            if (qq == q) myfree = nfree;
            ++nfree;
          }
        }
        const int nplaced = nfree < NG ? nfree : NG;         // loads that get a free slot of their own
        int cnt = 0;
#pragma unroll
        for (int e = 0; e < LT; ++e)
          if (e * SUB / LT == GRP) {
            if (cnt < nplaced) {
              if (cnt == myfree) issue_slot(e);
            } else if ((cnt - nplaced) * NM / (NG - nplaced > 0 ? NG - nplaced : 1) == q) {
              issue_slot(e);
            }
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
      issue_next_tile_if_done();
    } else {
      tail_steps(dl_tag, std::false_type{}, kt);
    }
    int b = kt;
    const int b_more_end = (kt_end - 1) < (nkt - NSTAGE) ? (kt_end - 1) : (nkt - NSTAGE);
#pragma unroll 1
    while (b < b_more_end) {
      // one run of the loop issues one stage per iteration and stays inside the tile being fetched
      const int left = (iit + 1) * nkt_tile - ikt;
      const int stop = (b + left) < b_more_end ? (b + left) : b_more_end;
#pragma unroll 1
      for (; b < stop; ++b) {
        wait_landed(b + 1);
        __syncthreads();
        issue_begin();
        kstep(dl_tag, std::true_type{}, std::integral_constant<int, 0>{}, LASTSET, stage_off(b + 1) + foff[0]);
        tail_steps(dl_tag, std::true_type{}, b + 1);
        issue_end();
      }
      issue_next_tile_if_done();
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

  // The flush code handles one 32x32 block at a time and re-states, right in front of each block, that its
  // sums live in accumulation registers.  Without this the compiler copies all of them to ordinary VGPRs at
  // the end of the K loop, ahead of every use, and spills what does not fit.
  auto pin_block = [&](const int i, const int j) __attribute__((always_inline)) {
    asm volatile("" : "+a"(accp[i][j]));
    if (DUAL) asm volatile("" : "+a"(accn[DUAL ? i : 0][DUAL ? j : 0]));
  };

  // ---- accumulator layout seen by the flush code ------------------------------------------------------
  // W^ is the MFMA "A" operand and X^ the "B" operand, so element v of block (i, j) in lane l is
  //   row    m = m0 + wm*TM + i*32 + (l & 31)
  //   column n = n0 + wn*TN + j*32 + 8*(v >> 2) + 4*(l >> 5) + (v & 3):
  // a lane owns four runs of four consecutive output columns of one row, which it scales with per-column
  // constants fetched 16 bytes at a time and stores directly as 16-byte (fp32, int32) or 8-byte (bf16)
  // pieces; the pieces of the two lane halves and the four runs fill a row's cache lines back to back.
  int mrow = 0, ncol = 0;                                  // of the tile being computed (set_compute_tile)
  bool full_tile = false;
  const bool vec4 = (a.N % 4) == 0;                        // rows of Y / wscale / bias keep 16-byte alignment
  const bool ptr16 = ((reinterpret_cast<uintptr_t>(a.y) | reinterpret_cast<uintptr_t>(a.wscale) |
                       reinterpret_cast<uintptr_t>(a.bias) | reinterpret_cast<uintptr_t>(a.acc_pos) |
                       reinterpret_cast<uintptr_t>(a.acc_neg)) % 16 == 0);
  // FULL: the tile lies inside the matrix and every row piece is 16-byte aligned, so the flush code runs
  // without bounds checks or scalar fallbacks (one uniform branch picks the instantiation).
  auto set_compute_tile = [&](const int it) __attribute__((always_inline)) {
    int m0, n0;
    tile_origin(it, m0, n0);
    mrow = m0 + wm * C::TM + (lane & 31);
    ncol = n0 + wn * C::TN + 4 * (lane >> 5);
    full_tile = vec4 && ptr16 && m0 + BM <= a.M && n0 + BN <= a.N;
  };

  // per-column constants of block column j in K-segment ks: cw[v] = seg_scale * wscale (0 outside N).  fetch_cw only
  // issues the loads of wscale, scale_cw applies the multiplier: the flush code fetches block column j + 1 before it
  // works on block column j, so a tile pays one memory latency for its constants, not one per block column.
  auto fetch_cw = [&](auto full_tag, const int ks, const int j, float (&cw)[16]) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value;
    const float* ws = a.wscale + (size_t)ks * a.N;
    const bool wvec = FULL || (vec4 && (reinterpret_cast<uintptr_t>(ws) % 16 == 0));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = ncol + j * 32 + 8 * g;
      if (FULL || (wvec && n + 3 < a.N)) {
        const v4f w4 = *reinterpret_cast<const v4f*>(ws + n);
#pragma unroll
        for (int r = 0; r < 4; ++r) cw[4 * g + r] = w4[r];
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) cw[4 * g + r] = (n + r < a.N) ? ws[n + r] : 0.0f;
      }
    }
  };
  auto scale_cw = [&](const int ks, const int j, float (&cw)[16]) __attribute__((always_inline)) {
    if (tb.has_seg_scale) {                                // multiplier of block (ks, N-segment of the column)
      float sg[16];
      const float s0 = tb.seg_scale[ks * tb.T];
#pragma unroll
      for (int v = 0; v < 16; ++v) sg[v] = s0;
#pragma unroll 1
      for (int t = 1; t < tb.T; ++t) {
        const int off = tb.nseg_off[t];
        const float st = tb.seg_scale[ks * tb.T + t];
#pragma unroll
        for (int v = 0; v < 16; ++v) sg[v] = (ncol + j * 32 + 8 * (v >> 2) + (v & 3) >= off) ? st : sg[v];
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) cw[v] *= sg[v];
    }
  };

  auto fetch_bias = [&](auto full_tag, const int j, float (&bs)[16]) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value;
    const bool bvec = FULL || (vec4 && (reinterpret_cast<uintptr_t>(a.bias) % 16 == 0));
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = ncol + j * 32 + 8 * g;
      if (a.bias && bvec && (FULL || n + 3 < a.N)) {
        const v4f b4 = *reinterpret_cast<const v4f*>(a.bias + n);
#pragma unroll
        for (int r = 0; r < 4; ++r) bs[4 * g + r] = b4[r];
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) bs[4 * g + r] = (a.bias && n + r < a.N) ? a.bias[n + r] : 0.0f;
      }
    }
  };

  // activation steps of this lane's token rows for K-segment ks: the layer's, or (TOK) each row's own
  auto row_steps = [&](const int ks, const bool dl, float (&spr)[IM], float (&snr)[IM]) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IM; ++i) {
      if (TOK) {
        int m = mrow + i * 32;
        m = m < a.M ? m : a.M - 1;                       // rows beyond M are masked at the store
        spr[i] = a.tok_steps[(size_t)m * tb.S + ks];
        snr[i] = dl ? a.tok_steps[((size_t)a.M + m) * tb.S + ks] : 0.0f;
      } else {
        spr[i] = tb.s_pos[ks];
        snr[i] = dl ? tb.s_neg[ks] : 0.0f;
      }
    }
  };

  // debug entry point: raw int32 sums of segment ks, acc_neg = 0 where the segment ran one path
  auto store_debug = [&](auto full_tag, const int ks, const bool has_neg) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value;
    const bool avec = FULL || (vec4 && ((reinterpret_cast<uintptr_t>(a.acc_pos) | reinterpret_cast<uintptr_t>(a.acc_neg)) % 16 == 0));
#pragma unroll
    for (int i = 0; i < IM; ++i)
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        const int m = mrow + i * 32;
        pin_block(i, j);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = ncol + j * 32 + 8 * g;
          if (FULL || m < a.M) {
            const size_t o = ((size_t)ks * a.M + m) * a.N + n;     // S*M*N < 2^31 is checked by the host
            v4i p, q;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              p[r] = accp[i][j][4 * g + r];
              q[r] = has_neg ? accn[DUAL ? i : 0][DUAL ? j : 0][4 * g + r] : 0;
            }
            if (FULL || (avec && n + 3 < a.N)) {
              *reinterpret_cast<v4i*>(a.acc_pos + o) = p;
              *reinterpret_cast<v4i*>(a.acc_neg + o) = q;
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (n + r < a.N) { a.acc_pos[o + r] = p[r]; a.acc_neg[o + r] = q[r]; }
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    // stores share the vector-memory counter with the direct loads but complete out of order with them:
    // drain everything so that the load accounting of the K loop stays valid
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  // ---- K-segment boundary: scale the exact int32 sums into the fp32 running sum, clear them ----------
  // SHARE: the layer has exactly one dual K-segment and it is visited first.  Two int32 sets are live only
  // during that segment; at its end the X^_- set's registers are re-used for the fp32 running sum (its bits
  // are kept in accn), and every later segment accumulates in accp alone.  `first` = first visited segment.
  auto flush_mid_impl = [&](auto full_tag, const int ks, const bool dl, const bool first) __attribute__((always_inline)) {
    if (mode == OUT_DEBUG_ACC) {
      store_debug(full_tag, ks, DUAL && dl && (!SHARE || first));
    } else if (SHARE || FSUM) {
      float spr[IM], snr[IM];
      row_steps(ks, dl, spr, snr);
      float cwb[2][16];
      fetch_cw(full_tag, ks, 0, cwb[0]);
#pragma unroll
      for (int j = 0; j < JN; ++j) {
        if (j + 1 < JN) fetch_cw(full_tag, ks, j + 1, cwb[(j + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);               // the next block column's loads are out, nothing else moves up
        float (&cw)[16] = cwb[j & 1];
        scale_cw(ks, j, cw);
#pragma unroll
        for (int i = 0; i < IM; ++i) {
          pin_block(i, j);
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float cpos = cw[v] * spr[i], cneg = cw[v] * snr[i];
            if (SHARE) {
              const int old = accn[DUAL ? i : 0][DUAL ? j : 0][v];
              const float prev = first ? cneg * acc_value<FP8>(old) : __int_as_float(old);
              accn[DUAL ? i : 0][DUAL ? j : 0][v] = __float_as_int(prev + cpos * acc_value<FP8>(accp[i][j][v]));
            } else {
              float t = cpos * acc_value<FP8>(accp[i][j][v]);
              if (DUAL) t += cneg * acc_value<FP8>(accn[DUAL ? i : 0][DUAL ? j : 0][v]);
              fsum[FSUM ? i : 0][FSUM ? j : 0][v] += t;
            }
          }
          // back into accumulation registers at once: left in ordinary VGPRs, the new sums would be spilled
          // to scratch memory around the next K loop
          if (SHARE) asm volatile("" : "+a"(accn[DUAL ? i : 0][DUAL ? j : 0]));
          __builtin_amdgcn_sched_barrier(0);
        }
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
  auto flush_mid = [&](const int ks, const bool dl, const bool first) __attribute__((always_inline)) {
    if (full_tile) flush_mid_impl(std::true_type{}, ks, dl, first);
    else flush_mid_impl(std::false_type{}, ks, dl, first);
  };

  // ---- last K-segment: dequantize, add bias, store ----------------------------------------------------
  // bf16 output of an interior tile: the two halves of the wave (lanes l and l + 32 hold the same row, column
  // runs 4 apart) exchange every second run with v_permlane32_swap, so that each lane ends up with eight
  // consecutive columns and stores 16 bytes.
  auto flush_last_impl = [&](auto full_tag, auto bf16_tag, const int ks, const bool dl) __attribute__((always_inline)) {
    constexpr bool FULL = decltype(full_tag)::value;
    constexpr bool BF = decltype(bf16_tag)::value;
    float spr[IM], snr[IM];
    row_steps(ks, dl, spr, snr);
    const bool yvec = FULL || (vec4 && (reinterpret_cast<uintptr_t>(a.y) % 16 == 0));
    float cwb[2][16], bsb[2][16];
    fetch_cw(full_tag, ks, 0, cwb[0]);
    fetch_bias(full_tag, 0, bsb[0]);
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      if (j + 1 < JN) {
        fetch_cw(full_tag, ks, j + 1, cwb[(j + 1) & 1]);
        fetch_bias(full_tag, j + 1, bsb[(j + 1) & 1]);
      }
      __builtin_amdgcn_sched_barrier(0);                 // the next block column's loads are out, nothing else moves up
      float (&cw)[16] = cwb[j & 1];
      float (&bs)[16] = bsb[j & 1];
      scale_cw(ks, j, cw);
#pragma unroll
      for (int i = 0; i < IM; ++i) {
        const int m = mrow + i * 32;
        pin_block(i, j);
        float t[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float u = (cw[v] * spr[i]) * acc_value<FP8>(accp[i][j][v]);
          if (SHARE) u += __int_as_float(accn[DUAL ? i : 0][DUAL ? j : 0][v]);   // running sum (never the first segment)
          else if (DUAL) u += (cw[v] * snr[i]) * acc_value<FP8>(accn[DUAL ? i : 0][DUAL ? j : 0][v]);
          if (FSUM) u += fsum[FSUM ? i : 0][FSUM ? j : 0][v];
          t[v] = u + bs[v];
        }
        if (FULL && BF) {
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t a0 = f32x2_to_bf16x2(t[8 * p + 0], t[8 * p + 1]), a1 = f32x2_to_bf16x2(t[8 * p + 2], t[8 * p + 3]);
            const uint32_t b0 = f32x2_to_bf16x2(t[8 * p + 4], t[8 * p + 5]), b1 = f32x2_to_bf16x2(t[8 * p + 6], t[8 * p + 7]);
            // lanes 32..63 of the first operand <-> lanes 0..31 of the second
            const auto s0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
            const v4i o4 = {(int)s0[0], (int)s1[0], (int)s0[1], (int)s1[1]};
            const size_t o = (size_t)m * a.N + (ncol + j * 32 + 16 * p + 4 * (lane >> 5));
            *reinterpret_cast<v4i*>(reinterpret_cast<uint16_t*>(a.y) + o) = o4;
          }
        } else {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int n = ncol + j * 32 + 8 * g;
            if (FULL || m < a.M) {
              const size_t o = (size_t)m * a.N + n;
              if (FULL || (yvec && n + 3 < a.N)) {
                if (!BF) {
                  const v4f o4 = {t[4 * g], t[4 * g + 1], t[4 * g + 2], t[4 * g + 3]};
                  *reinterpret_cast<v4f*>(reinterpret_cast<float*>(a.y) + o) = o4;
                } else {
                  v2i o2;
                  o2[0] = (int)f32x2_to_bf16x2(t[4 * g], t[4 * g + 1]);
                  o2[1] = (int)f32x2_to_bf16x2(t[4 * g + 2], t[4 * g + 3]);
                  *reinterpret_cast<v2i*>(reinterpret_cast<uint16_t*>(a.y) + o) = o2;
                }
              } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                  if (n + r < a.N) {
                    if (!BF) reinterpret_cast<float*>(a.y)[o + r] = t[4 * g + r];
                    else reinterpret_cast<uint16_t*>(a.y)[o + r] = f32_to_bf16(t[4 * g + r]);
                  }
              }
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto flush_last = [&](const int ks, const bool dl, const bool first) __attribute__((always_inline)) {
    if (mode == OUT_DEBUG_ACC) {
      if (full_tile) store_debug(std::true_type{}, ks, DUAL && dl && (!SHARE || first));
      else store_debug(std::false_type{}, ks, DUAL && dl && (!SHARE || first));
    } else if (mode == OUT_BF16) {
      if (full_tile) flush_last_impl(std::true_type{}, std::true_type{}, ks, dl);
      else flush_last_impl(std::false_type{}, std::true_type{}, ks, dl);
    } else {
      if (full_tile) flush_last_impl(std::true_type{}, std::false_type{}, ks, dl);
      else flush_last_impl(std::false_type{}, std::false_type{}, ks, dl);
    }
  };

#pragma unroll 1
  for (int it = 0; it < ntile_wg; ++it) {
    set_compute_tile(it);
    clear_accumulators();
    if constexpr (!MULTI) {
      // one K-segment: the host selects the DUAL instantiation exactly when that segment is dual
      run_segment(std::integral_constant<bool, DUAL>{}, nkt_tile);
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
      // middle segments in a loop, the last one peeled: with the store epilogue as an alternative inside the
      // loop the accumulators' register assignment has to agree on both ways round it, which costs spills
#pragma unroll 1
      for (int pos = 1; pos + 1 < tb.S; ++pos) {
        const int ks = tb.seg_order[pos];
        run_segment(std::false_type{}, (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH);
        pin_accumulators();
        flush_mid(ks, false, false);
      }
      {
        const int ks = tb.seg_order[tb.S - 1];
        run_segment(std::false_type{}, (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH);
        pin_accumulators();
        flush_last(ks, false, false);
      }
    } else {
#pragma unroll 1
      for (int pos = 0; pos + 1 < tb.S; ++pos) {
        const int ks = tb.seg_order[pos];
        const bool dl = DUAL && (tb.dual[ks] != 0);
        const int nst = (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH;
        if (dl) run_segment(std::integral_constant<bool, DUAL>{}, nst);
        else run_segment(std::integral_constant<bool, false>{}, nst);
        pin_accumulators();
        flush_mid(ks, dl, pos == 0);
      }
      {
        const int ks = tb.seg_order[tb.S - 1];
        const bool dl = DUAL && (tb.dual[ks] != 0);
        const int nst = (tb.kseg_off[ks + 1] - tb.kseg_off[ks]) >> KSH;
        if (dl) run_segment(std::integral_constant<bool, DUAL>{}, nst);
        else run_segment(std::integral_constant<bool, false>{}, nst);
        pin_accumulators();
        flush_last(ks, dl, false);
      }
    }
  }
}

}  // namespace sq
