// Skinny-M (M <= 64) SegLinear + DualScale GEMM for wide layers: a persistent weight stream.
//
// Modulation / adaLN-style layers (Sec. 4.2.2 item 1: a linear followed by chunk; Sec. 4.3.2: its input comes
// from SiLU) have a handful of token rows and a wide output, also when the modulation linears of all blocks
// of a model are stacked along N into one call.  The layer is then one pass over the int8 weight, and this
// kernel is built as an HBM stream:
//   * X^ (polarity-merged codes, at most 64 rows) is copied once per workgroup into an LDS slab and stays there;
//     rows are padded by 16 bytes so that the 16 rows of a fragment read fall on distinct bank groups.
//   * Every wave owns a list of 16-column groups of the output and streams the 16 W^ rows of a group
//     in steps of 128 bytes of K (full cache lines) through a private ring of direct global->LDS loads.  The
//     ring runs ahead across group boundaries.  Sixteen waves per workgroup (four per SIMD; eight when there are
//     more than two 16-row token tiles) and one workgroup per CU: the waves hide each other's LDS and MFMA
//     latencies, which matters more than the depth of a wave's ring.  No workgroup barrier is needed after the
//     slab is filled.
//   * W^ rows are the MFMA "A" operand (v_mfma_i32_16x16x64_i8) and X^ rows the "B" operand, so a lane ends up
//     with four consecutive output columns of one token row: scales are fetched and results stored 16 / 8
//     bytes at a time.  Exact int32 sums per K-segment and polarity are scaled into an fp32 running sum at
//     each segment boundary (Sec. 4.2.2 item 2, Sec. 4.3.2 last display).
//   * Nothing in the group loop is a compiler-visible vector load: the direct loads are counted by hand, scales
//     and biases come through the scalar cache, so no vmcnt(0) ever drains the ring.
#include "seglinear_mfma_kernel.hpp"

namespace sq {

// Waves per workgroup (one workgroup per CU).  With one or two 16-row token tiles a wave needs few registers and
// sixteen waves (four per SIMD) hide each other's LDS and MFMA latencies better than eight with deeper rings
// (measured: ring depth hardly matters, the number of waves does: 5.75 -> 5.97 TB/s, 4-bit weights 4.1 -> 5.1).
constexpr int stream_waves(int mt) { return mt <= 2 ? 16 : 8; }

// The weight stream is read exactly once: the loads carry the non-temporal hint, so that the lines are not kept
// in the caches at the expense of everything else (measured: 5.0 -> 5.8 TB/s for the bare stream from HBM).
__device__ __forceinline__ void glds16_stream(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(voff), "s"(sbase), "s"(lds_addr)
               : "memory");
}

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for outstanding vector memory
// operations, i.e. it leaves the ring's direct loads in flight.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Per-column scales and biases of a 16-column group sit at a wave-uniform address and are never written by the
// kernel: they are fetched through the scalar cache (constant address space).  A vector load here would make the
// compiler wait for vmcnt(0) before its first use, which drains the whole ring of direct loads once per group.
typedef const float __attribute__((address_space(4))) * uniform_f32_ptr;
__device__ __forceinline__ uniform_f32_ptr as_uniform(const float* p) {
  return (uniform_f32_ptr)(reinterpret_cast<uintptr_t>(p));
}
// The 16 values at p, of which the first nvalid exist (a wave-uniform count; the rest read as zero), into scalar
// registers.  Also the ragged last group takes this path: any vector load in the group loop, on any branch,
// would bring the vmcnt(0) waits back at the joins.  Issued before a K loop and picked from after it, the fetch
// hides behind the first wait for stream data.
__device__ __forceinline__ void fetch_group16(const float* p, const int nvalid, float s[16]) {
  uniform_f32_ptr u = as_uniform(p);
  if (nvalid >= 16) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = u[i];
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = i < nvalid ? u[i] : 0.0f;
  }
}
// lane's four consecutive values (columns 4*fq .. 4*fq+3)
__device__ __forceinline__ void pick4(const float s[16], const int fq, float out[4]) {
#pragma unroll
  for (int r = 0; r < 4; ++r) out[r] = fq == 0 ? s[r] : fq == 1 ? s[4 + r] : fq == 2 ? s[8 + r] : s[12 + r];
}

// W4: the weights are 4-bit codes packed two per byte (a step of 128 codes of 16 rows is 1 KiB, one direct load)
// PS: the slab holds X^_+ and X^_- as two planes (split once at the fill instead of in every step); its small size
// class is then 48 KiB instead of 24
template <int MT, int SLAB_KB, bool W4, bool PS>
struct StreamCfg {
  static constexpr int NW = stream_waves(MT);
  static constexpr int SLAB = (PS && SLAB_KB == 24 ? 48 : SLAB_KB) * 1024;
  static constexpr int STEP = W4 ? 1024 : 2048;                   // 16 W^ rows x 128 codes of K
  static constexpr int LPS = W4 ? 1 : 2;                          // direct loads per step
  static constexpr int RAW = (156 * 1024 - SLAB) / (NW * STEP);
  static constexpr int RING = RAW > 28 ? 28 : RAW;                // at most 56 loads in flight: below the 6-bit vmcnt
  static constexpr int LDS = SLAB + NW * RING * STEP;
  static constexpr int TOK = 4096;                                // table of dynamic per-token steps: [64 rows][8 segments][2]
  static_assert(RING >= 2, "ring too shallow");
  static_assert(LDS + 4096 <= 160 * 1024, "LDS budget");
};

// TB: GemmTable (one layer; GT = NoGroups) or GroupSegTable (GT = GroupTable: L layers of the same shape that share
// X^ and its steps; the 16-column groups of all layers form one list, layer = group / groups per layer).
// FP8: the codes are OCP E4M3 bytes; a 128-byte step is one v_mfma_f32_16x16x128_f8f6f4 (no block scales: a lane's operand
// is its two 16-byte chunks of the step, the same k set for W^ and X^), the sums are fp32 kept as bits in the accumulator
// registers, X^_- holds the codes with the sign bit set.  Static steps, code input only.
template <int MT, bool DUAL, int SLAB_KB, class TB, class GT, bool W4 = false, bool PS = false, bool FP8 = false>
__global__ __launch_bounds__(stream_waves(MT) * 64) void seglinear_stream_kernel(const GemmArgs a, const TB tb, const GT gt, const int mode) {
  static_assert(!PS || DUAL, "two slab planes only where both polarity paths run");
  static_assert(!FP8 || !W4, "fp8 codes are bytes");
  using C = StreamCfg<MT, SLAB_KB, W4, PS>;
  constexpr bool GROUPED = std::is_same<GT, GroupTable>::value;
  constexpr int RING = C::RING, STEP = C::STEP, LPS = C::LPS, NW = C::NW;
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS + C::TOK];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* tok = reinterpret_cast<float*>(smem + C::LDS);            // [row][ks][polarity], filled when a.tok_steps is set

  // ---- this wave's run of 16-column groups ------------------------------------------------------------
  const int gpl = (a.N + 15) >> 4;                                 // groups per layer
  int nlayers = 1;
  if constexpr (GROUPED) nlayers = gt.L;
  const int ngroups = gpl * nlayers;
  // Group g of the flat list goes to a wave in one of two ways (both wave-uniform):
  //   * enough groups for every wave of the grid: wave (workgroup b, wave w of NW) takes groups NW b + w, + nwaves, ...
  //     At any moment the chip then reads one contiguous window of the weights (nwaves groups, 18 KB each for
  //     K = 1152) and the waves of a CU read adjacent groups of it, which the memory system (page
  //     translation included) serves measurably better than one far-apart stream per wave: 5.5 vs 4.7 TB/s.
  //   * fewer groups than waves: every workgroup takes a contiguous share of the list and deals it to its
  //     waves, so that a narrow layer still spreads over all CUs.
  const int nwaves = gridDim.x * NW;
  int g_first, g_stride, g_cnt;
  if (ngroups >= nwaves) {
    g_first = blockIdx.x * NW + wave;
    g_stride = nwaves;
    g_cnt = (ngroups - g_first + nwaves - 1) / nwaves;
  } else {
    const int cper = ngroups / (int)gridDim.x, crem = ngroups % (int)gridDim.x, bx = blockIdx.x;
    const int c_begin = bx < crem ? bx * (cper + 1) : crem * (cper + 1) + (bx - crem) * cper;
    const int c_cnt = cper + (bx < crem ? 1 : 0);
    g_first = c_begin + wave;
    g_stride = NW;
    g_cnt = wave < c_cnt ? (c_cnt - wave + NW - 1) / NW : 0;
  }
  auto group_at = [&](const int g) __attribute__((always_inline)) { return g_first + g * g_stride; };
  const int nstep = a.K >> 7;                                      // 128-byte steps per group
  const int total = g_cnt * nstep;                                 // steps of this wave

  // ---- direct loads: lane -> (row lane/8 of 8 rows, 16 B slot lane%8 holding chunk slot ^ swizzle(row)) -----
  char* ring = smem + C::SLAB + wave * (RING * STEP);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)SQ_LDS(ring);
  const int lrow = lane >> 3, lslot = lane & 7;
  int ig = 0, it = 0, issued_steps = 0, islot = 0;
  uint32_t voff[2];
  const int8_t* iwq = a.wq;                                        // weights of the layer being fetched
  auto set_issue_group = [&](const int g) __attribute__((always_inline)) {
    int gl = group_at(g);
    if constexpr (GROUPED) {
      const int l = gl / gpl;
      gl -= l * gpl;
      iwq = gt.item[l].wq;
    }
    if (W4) {
      // packed storage: one contiguous KiB per (16-row group, 128-code step), [16 rows][64 bytes].  lane -> (row
      // lane/4, 16 B slot lane%4 holding chunk slot ^ (row/4 & 3): rows 4 apart share LDS banks, the swizzle keeps
      // a fragment read's 16 rows apart).  Every direct load moves eight full cache lines.
      const int rt = lane >> 2;
      voff[0] = (uint32_t)gl * (uint32_t)(a.K >> 7) * 1024u + (uint32_t)(rt * 64) + (uint32_t)(((lane & 3) ^ ((rt >> 2) & 3)) << 4);
      voff[1] = 0;
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int rt = 8 * h + lrow;
        int r = gl * 16 + rt;
        r = r < a.N ? r : a.N - 1;                                 // ragged N: re-read the last row, masked at the store
        voff[h] = (uint32_t)r * (uint32_t)a.K + (uint32_t)((lslot ^ row_swizzle<128>(rt)) << 4);
      }
    }
  };
  auto issue_step = [&]() __attribute__((always_inline)) {
    const uint64_t u = reinterpret_cast<uint64_t>(iwq + ((size_t)it << (W4 ? 10 : 7)));
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    const int8_t* base = reinterpret_cast<const int8_t*>(((uint64_t)hi << 32) | lo);
    const uint32_t so = __builtin_amdgcn_readfirstlane(ring_lds + (uint32_t)islot * (uint32_t)STEP);
    glds16_stream(base, voff[0], so);
    if (!W4) glds16_stream(base, voff[1], so + 1024u);
    ++issued_steps;
    islot = (islot + 1 == RING) ? 0 : islot + 1;
    if (++it == nstep) {
      it = 0;
      if (++ig < g_cnt) set_issue_group(ig);
    }
  };
  // ---- raw activations (a.x_raw): the activation in front of the layer and Q_dual (Sec. 4.3.2) happen on the way into
  // the slab, in items of four elements.  Every workgroup quantizes the whole of X for itself (M <= 64 rows).  Each
  // thread's first RAWPRE items are requested before the ring is primed, with loads the compiler does not track, and
  // waited for with a count that leaves the ring's direct loads in flight (vector memory loads complete in order), so
  // that the latency of X, the latency of the first weights and the arithmetic overlap.
  constexpr int RAWPRE = 5, NT = NW * 64;
  constexpr int PRIME_LOADS = (RING - 1) * (W4 ? 1 : 2);           // direct loads of a fully primed ring
  static_assert(PRIME_LOADS <= 63, "the wait count is a 6-bit field");
  const int kq = a.K >> 2;                                         // items per row
  const int nitem = a.x_raw ? a.M * kq : 0;
  uint64_t raw2[RAWPRE];                                           // bf16 items: 8 bytes
  v4i raw4[RAWPRE];                                                // fp32 items: 16 bytes
#pragma unroll
  for (int j = 0; j < RAWPRE; ++j) {
    const int c = threadIdx.x + j * NT;
    raw2[j] = 0;
    raw4[j] = (v4i)(0);
    if (c < nitem) {
      if (a.x_raw_bf16)
        asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(raw2[j]) : "v"(reinterpret_cast<const uint16_t*>(a.x_raw) + (size_t)c * 4) : "memory");
      else
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(raw4[j]) : "v"(reinterpret_cast<const float*>(a.x_raw) + (size_t)c * 4) : "memory");
    }
  }

  if (g_cnt > 0) set_issue_group(0);
#pragma unroll 1
  while (issued_steps < RING - 1 && issued_steps < total) issue_step();

  if (a.x_raw) {
#define SQ_RAW_OPERANDS "+v"(raw2[0]), "+v"(raw2[1]), "+v"(raw2[2]), "+v"(raw2[3]), "+v"(raw2[4]), \
                        "+v"(raw4[0]), "+v"(raw4[1]), "+v"(raw4[2]), "+v"(raw4[3]), "+v"(raw4[4])
    static_assert(RAWPRE == 5, "operand list above");
    // One statement carries the registers (a second one on another path would make the compiler merge the two sets
    // with copies, and a copy placed before the wait reads a register the load has not written yet).
    if (issued_steps != RING - 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // ring not fully primed
    asm volatile("s_waitcnt vmcnt(%[cnt])" : SQ_RAW_OPERANDS : [cnt] "n"(PRIME_LOADS) : "memory");
#undef SQ_RAW_OPERANDS
  }

  // ---- X^ slab: [16*MT rows][K + 16] bytes, rows beyond M repeat the last row (masked at the store) ----------
  // PS: a second plane of the same shape behind the first; plane 0 holds X^_+ (the whole code in a single-scale
  // K-segment), plane 1 holds X^_- (zero there): the polarity separation of Sec. 4.3.2 done once per workgroup.
  const int plane = MT * 16 * (a.K + 16);
  if (a.x_raw != nullptr) {
    const int rowb = a.K + 16;
    auto quantize_item = [&](const int c, const uint32_t (&w)[4]) __attribute__((always_inline)) {
      const int r = c / kq, col = (c - r * kq) << 2;
      float sp = 1.0f, sn = 1.0f, ip = 1.0f, in = 1.0f;
      bool dl = false;
      int acode = SQ_ACT_NONE;
      for (int sg = 0; sg < tb.S; ++sg)
        if (col >= tb.kseg_off[sg]) {
          sp = tb.s_pos[sg]; sn = tb.s_neg[sg]; ip = tb.inv_pos[sg]; in = tb.inv_neg[sg]; dl = tb.dual[sg] != 0; acode = tb.act[sg];
        }
      float xv[4];
      if (a.x_raw_bf16) {
        xv[0] = __uint_as_float(w[0] << 16); xv[1] = __uint_as_float(w[0] & 0xFFFF0000u);
        xv[2] = __uint_as_float(w[1] << 16); xv[3] = __uint_as_float(w[1] & 0xFFFF0000u);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) xv[i] = __uint_as_float(w[i]);
      }
      uint32_t pk = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float av = activate(acode, xv[i]);
        const bool ng = dl && (av < 0.0f);                 // X_- = min(X, 0) takes the s_- branch of Q_dual
        const int code = clip_code(round_quotient(av, ng ? sn : sp, ng ? in : ip));
        pk |= (uint32_t)(code & 0xFF) << (8 * i);
      }
      int pos = (int)pk, neg = 0;
      if (PS) {
        if (dl) split_polarity((int)pk, pos, neg);
        *reinterpret_cast<int*>(smem + plane + r * rowb + col) = neg;
      }
      *reinterpret_cast<int*>(smem + r * rowb + col) = pos;
    };
    auto load_item = [&](const int c, uint32_t (&w)[4]) __attribute__((always_inline)) {
      if (a.x_raw_bf16) {
        const uint2 t = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.x_raw) + (size_t)c * 4);
        w[0] = t.x; w[1] = t.y; w[2] = 0; w[3] = 0;
      } else {
        const uint4 t = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(a.x_raw) + (size_t)c * 4);
        w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
      }
    };
    if (a.x_raw_dynamic) {
      // Dynamic per-token steps (App. B, 4-bit settings) found here as well: extremes of act(x) per (token row, K-segment,
      // polarity) through LDS maxima on the bit patterns (non-negative floats order like unsigned integers), the steps by
      // the min/max rule of Sec. 4.3.2 (1.0 where the extreme is 0) into the table the flushes read, then the codes.
      // The activated values of the preloaded items replace the raw ones in their registers between the two passes.
      uint32_t* amax = reinterpret_cast<uint32_t*>(tok);
      const int ntab = MT * 16 * tb.S * 2;
      for (int i = threadIdx.x; i < ntab; i += NT) amax[i] = 0u;
      lds_barrier();
      auto scan_item = [&](const int c, const uint32_t (&w)[4], float (&av)[4]) __attribute__((always_inline)) {
        const int r = c / kq, col = (c - r * kq) << 2;
        int ks = 0, acode = SQ_ACT_NONE;
        bool dl = false;
        for (int sg = 0; sg < tb.S; ++sg)
          if (col >= tb.kseg_off[sg]) { ks = sg; dl = tb.dual[sg] != 0; acode = tb.act[sg]; }
        float mp = 0.0f, mn = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float xv;
          if (a.x_raw_bf16) xv = __uint_as_float((i & 1) ? (w[i >> 1] & 0xFFFF0000u) : (w[i >> 1] << 16));
          else xv = __uint_as_float(w[i]);
          av[i] = activate(acode, xv);
          if (dl) {
            mp = __builtin_fmaxf(mp, av[i]);
            mn = __builtin_fmaxf(mn, -av[i]);
          } else {
            mp = __builtin_fmaxf(mp, __builtin_fabsf(av[i]));
          }
        }
        const int ti = 2 * (r * tb.S + ks);
        if (mp > 0.0f) atomicMax(&amax[ti], __float_as_uint(mp));
        if (mn > 0.0f) atomicMax(&amax[ti + 1], __float_as_uint(mn));
      };
#pragma unroll
      for (int j = 0; j < RAWPRE; ++j) {
        const int c = threadIdx.x + j * NT;
        uint32_t w[4] = {(uint32_t)raw4[j][0], (uint32_t)raw4[j][1], (uint32_t)raw4[j][2], (uint32_t)raw4[j][3]};
        if (a.x_raw_bf16) { w[0] = (uint32_t)raw2[j]; w[1] = (uint32_t)(raw2[j] >> 32); }
        float av[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (c < nitem) scan_item(c, w, av);
#pragma unroll
        for (int i = 0; i < 4; ++i) raw4[j][i] = __float_as_int(av[i]);
      }
#pragma unroll 1
      for (int c = threadIdx.x + RAWPRE * NT; c < nitem; c += NT) {
        uint32_t w[4];
        float av[4];
        load_item(c, w);
        scan_item(c, w, av);
      }
      lds_barrier();
      for (int i = threadIdx.x; i < ntab; i += NT) {
        const float m = __uint_as_float(amax[i]);
        tok[i] = (m == 0.0f) ? 1.0f : m / a.act_qmax;
      }
      lds_barrier();
      auto code_item = [&](const int c, const float (&av)[4]) __attribute__((always_inline)) {
        const int r = c / kq, col = (c - r * kq) << 2;
        int ks = 0;
        bool dl = false;
        for (int sg = 0; sg < tb.S; ++sg)
          if (col >= tb.kseg_off[sg]) { ks = sg; dl = tb.dual[sg] != 0; }
        const float sp = tok[2 * (r * tb.S + ks)], sn = tok[2 * (r * tb.S + ks) + 1];
        const float ip = (sp >= 1e-30f && sp <= 1e30f) ? 1.0f / sp : __builtin_nanf("");
        const float in = (sn >= 1e-30f && sn <= 1e30f) ? 1.0f / sn : __builtin_nanf("");
        uint32_t pk = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool ng = dl && (av[i] < 0.0f);
          const int code = clip_code(round_quotient(av[i], ng ? sn : sp, ng ? in : ip));
          pk |= (uint32_t)(code & 0xFF) << (8 * i);
        }
        int pos = (int)pk, neg = 0;
        if (PS) {
          if (dl) split_polarity((int)pk, pos, neg);
          *reinterpret_cast<int*>(smem + plane + r * rowb + col) = neg;
        }
        *reinterpret_cast<int*>(smem + r * rowb + col) = pos;
      };
#pragma unroll
      for (int j = 0; j < RAWPRE; ++j) {
        const int c = threadIdx.x + j * NT;
        const float av[4] = {__int_as_float(raw4[j][0]), __int_as_float(raw4[j][1]), __int_as_float(raw4[j][2]),
                             __int_as_float(raw4[j][3])};
        if (c < nitem) code_item(c, av);
      }
#pragma unroll 1
      for (int c = threadIdx.x + RAWPRE * NT; c < nitem; c += NT) {
        uint32_t w[4];
        float av[4];
        load_item(c, w);
        const int r = c / kq, col = (c - r * kq) << 2;
        int acode = SQ_ACT_NONE;
        for (int sg = 0; sg < tb.S; ++sg)
          if (col >= tb.kseg_off[sg]) acode = tb.act[sg];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float xv;
          if (a.x_raw_bf16) xv = __uint_as_float((i & 1) ? (w[i >> 1] & 0xFFFF0000u) : (w[i >> 1] << 16));
          else xv = __uint_as_float(w[i]);
          av[i] = activate(acode, xv);
        }
        code_item(c, av);
      }
    } else {
#pragma unroll
      for (int j = 0; j < RAWPRE; ++j) {
        const int c = threadIdx.x + j * NT;
        uint32_t w[4] = {(uint32_t)raw4[j][0], (uint32_t)raw4[j][1], (uint32_t)raw4[j][2], (uint32_t)raw4[j][3]};
        if (a.x_raw_bf16) { w[0] = (uint32_t)raw2[j]; w[1] = (uint32_t)(raw2[j] >> 32); }
        if (c < nitem) quantize_item(c, w);
      }
#pragma unroll 1
      for (int c = threadIdx.x + RAWPRE * NT; c < nitem; c += NT) {  // larger X: plain loads (each wait drains the ring)
        uint32_t w[4];
        load_item(c, w);
        quantize_item(c, w);
      }
    }
    const int cpr = a.K >> 4;                                      // rows beyond M: zero codes (masked at the store)
    for (int c = a.M * cpr + threadIdx.x; c < MT * 16 * cpr; c += NT) {
      const int r = c / cpr, cc = c - r * cpr;
      *reinterpret_cast<v4i*>(smem + r * rowb + cc * 16) = (v4i)(0);
      if (PS) *reinterpret_cast<v4i*>(smem + plane + r * rowb + cc * 16) = (v4i)(0);
    }
  } else {
    const int rowb = a.K + 16, cpr = a.K >> 4;                     // 16-byte chunks per row
    const int nchunk = MT * 16 * cpr;
    for (int c = threadIdx.x; c < nchunk; c += NW * 64) {
      const int r = c / cpr, cc = c - r * cpr;
      const int rs = r < a.M ? r : a.M - 1;
      v4i v = *reinterpret_cast<const v4i*>(a.xq + (size_t)rs * a.K + cc * 16);
      if (PS) {
        bool dl = false;
        for (int sg = 0; sg < tb.S; ++sg)
          if (cc * 16 >= tb.kseg_off[sg]) dl = tb.dual[sg] != 0;
        v4i nv = (v4i)(0);
        if (dl) {
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            int pos, neg;
            split_polarity(v[d], pos, neg);
            v[d] = pos;
            nv[d] = neg;
          }
        }
        *reinterpret_cast<v4i*>(smem + plane + r * rowb + cc * 16) = nv;
      }
      *reinterpret_cast<v4i*>(smem + r * rowb + cc * 16) = v;
    }
  }
  if (a.tok_steps) {                                               // dynamic per-token steps (host: S <= 8)
    for (int i = threadIdx.x; i < MT * 16 * tb.S; i += NW * 64) {
      const int r = i / tb.S, ks = i - r * tb.S;
      const int rs = r < a.M ? r : a.M - 1;
      tok[2 * i] = a.tok_steps[(size_t)rs * tb.S + ks];
      tok[2 * i + 1] = a.tok_steps[((size_t)a.M + rs) * tb.S + ks];
    }
  }
  __syncthreads();   // the only workgroup barrier: slab visible (the compiler drains this thread's loads here, the
                     // direct loads above included; the stream refills right after)

  // ---- fragment offsets ------------------------------------------------------------------------------------
  const int frow = lane & 15, fq = lane >> 4;                      // fragment row, 16-byte k-chunk
  // W^ step slot: row frow, chunk 4h + fq of 8, swizzled; X^ slab: row frow (+16 mt), byte 64*kk + 16*fq
  int woff[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) woff[h] = frow * 128 + (((4 * h + fq) ^ row_swizzle<128>(frow)) << 4);
  if (W4) woff[0] = frow * 64 + ((fq ^ ((frow >> 2) & 3)) << 4);   // packed: one 16-byte chunk holds both k-steps
  const int xrow = frow * (a.K + 16) + 16 * fq;

  const int mlane = lane & 15;                                     // token row inside a 16-row tile
  bool vec4 = (a.N % 4) == 0 &&
              ((reinterpret_cast<uintptr_t>(a.y) | reinterpret_cast<uintptr_t>(a.wscale) | reinterpret_cast<uintptr_t>(a.bias) |
                reinterpret_cast<uintptr_t>(a.acc_pos) | reinterpret_cast<uintptr_t>(a.acc_neg)) % 16 == 0);

  int done_steps = 0, cslot = 0;
#pragma unroll 1
  for (int g = 0; g < g_cnt; ++g) {
    int gl = group_at(g);                                          // group inside its layer
    const float* l_wscale = a.wscale;
    const float* l_bias = a.bias;
    void* l_y = a.y;
    if constexpr (GROUPED) {
      const int l = gl / gpl;
      gl -= l * gpl;
      l_wscale = gt.item[l].wscale;
      l_bias = gt.item[l].bias;
      l_y = gt.item[l].y;
      vec4 = (a.N % 4) == 0 && ((reinterpret_cast<uintptr_t>(l_y) | reinterpret_cast<uintptr_t>(l_wscale) |
                                  reinterpret_cast<uintptr_t>(l_bias)) % 16 == 0);
    }
    const int ncol = gl * 16 + 4 * fq;                             // this lane's four output columns
    v4f fsum[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) fsum[mt] = (v4f)(0.0f);
    int kk = 0;                                                    // 64-byte k-step inside the group
#pragma unroll 1
    for (int ks = 0; ks < tb.S; ++ks) {
      const bool dl = DUAL && (tb.dual[ks] != 0);
      int kk_end = tb.kseg_off[ks + 1] >> 6;

      // two accumulator sets, one per 64-byte half of a step: consecutive MFMAs do not wait on each other
      v4i accp[MT], accn[MT], accp1[MT], accn1[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) { accp[mt] = (v4i)(0); accn[mt] = (v4i)(0); accp1[mt] = (v4i)(0); accn1[mt] = (v4i)(0); }
      // the step loop, once per polarity mode (the test stays out of the loop)
      auto step_loop = [&](auto dl_tag) __attribute__((always_inline)) {
        constexpr bool DL = decltype(dl_tag)::value;
#pragma unroll 1
        while (kk < kk_end) {                                      // one 128-byte step = two MFMA k-steps
          ++done_steps;
          wait_vmcnt<LPS * (RING - 2), 0>(LPS * (issued_steps - done_steps));
          v4i wf[2], xf[2][MT], nfp[2][PS ? MT : 1];
#pragma unroll
          for (int h = 0; h < 2; ++h) {                            // all fragment reads of the step first
            if (!W4 || h == 0) wf[h] = *reinterpret_cast<const v4i*>(ring + cslot * STEP + woff[h]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              xf[h][mt] = *reinterpret_cast<const v4i*>(smem + mt * 16 * (a.K + 16) + xrow + (kk + h) * 64);
              if (PS && DL) nfp[h][mt] = *reinterpret_cast<const v4i*>(smem + plane + mt * 16 * (a.K + 16) + xrow + (kk + h) * 64);
            }
          }
          if (W4) {                                                // nibbles -> 16-fold int8 codes of the two k-steps
#pragma unroll
            for (int d = 0; d < 4; ++d) {
              const int pk = wf[0][d];
              wf[0][d] = (pk << 4) & (int)0xF0F0F0F0u;
              wf[1][d] = pk & (int)0xF0F0F0F0u;
            }
          }
          if constexpr (FP8) {
            v8i w8;
#pragma unroll
            for (int d = 0; d < 4; ++d) { w8[d] = wf[0][d]; w8[4 + d] = wf[1][d]; }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              v8i p8, n8;
#pragma unroll
              for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                  int pos = xf[h][mt][d], neg = 0;
                  if (DL) {
                    if (PS) neg = nfp[h][mt][d];
                    else split_polarity(xf[h][mt][d], pos, neg);
                  }
                  p8[4 * h + d] = pos;
                  n8[4 * h + d] = neg;
                }
              // constant-zero scale operands select the unscaled instruction
              accp[mt] = __builtin_bit_cast(v4i, __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                  w8, p8, __builtin_bit_cast(v4f, accp[mt]), 0, 0, 0, 0, 0, 0));
              if (DL)
                accn[mt] = __builtin_bit_cast(v4i, __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                    w8, n8, __builtin_bit_cast(v4f, accn[mt]), 0, 0, 0, 0, 0, 0));
            }
          } else {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int mt = 0; mt < MT; ++mt) {
                v4i pf = xf[h][mt];
                if (DL) {                                            // X^_+ = max(X^, 0), X^_- = min(X^, 0), byte-wise
                  v4i nf;
                  if (PS) {
                    nf = nfp[h][mt];
                  } else {
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                      int pos, neg;
                      split_polarity(pf[d], pos, neg);
                      pf[d] = pos;
                      nf[d] = neg;
                    }
                  }
                  if (h == 0) accn[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[h], nf, accn[mt], 0, 0, 0);
                  else accn1[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[h], nf, accn1[mt], 0, 0, 0);
                }
                if (h == 0) accp[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[h], pf, accp[mt], 0, 0, 0);
                else accp1[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[h], pf, accp1[mt], 0, 0, 0);
              }
          }
          // step consumed (its fragments are in registers): free the slot, keep the stream going
          cslot = (cslot + 1 == RING) ? 0 : cslot + 1;
          if (issued_steps < total) issue_step();
          kk += 2;
        }
      };
      float ws16[16];                                              // this segment's per-column weight steps
      // The fetch is the last scalar load before the loop (kk_end is pinned into its register first): nothing
      // then waits for it before the loop's first wait for LDS data, which comes after the wait for stream data.
      asm volatile("" : "+s"(kk_end));
      if (mode != OUT_DEBUG_ACC) fetch_group16(l_wscale + (size_t)ks * a.N + gl * 16, a.N - gl * 16, ws16);
      if (dl) step_loop(std::true_type{});
      else step_loop(std::false_type{});
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if (!FP8) { accp[mt] += accp1[mt]; accn[mt] += accn1[mt]; }     // (fp8: one instruction per step, one set)
      }
      // ---- K-segment boundary (kseg boundaries are multiples of 128 here, so a step never straddles one) ------
      if (mode == OUT_DEBUG_ACC) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int m = mt * 16 + mlane;
          if (m < a.M) {
            const size_t o = ((size_t)ks * a.M + m) * a.N + ncol;
            // packed weights enter the MFMA 16-fold: the sums are exact multiples of 16
            const v4i pp = W4 ? (accp[mt] >> 4) : accp[mt];
            const v4i q = dl ? (W4 ? (accn[mt] >> 4) : accn[mt]) : (v4i)(0);
            if (vec4 && ncol + 3 < a.N) {
              *reinterpret_cast<v4i*>(a.acc_pos + o) = pp;
              *reinterpret_cast<v4i*>(a.acc_neg + o) = q;
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (ncol + r < a.N) { a.acc_pos[o + r] = pp[r]; a.acc_neg[o + r] = q[r]; }
            }
          }
        }
      } else {
        float cw[4];
        pick4(ws16, fq, cw);
        if (W4) {                                                  // exact: undoes the 16-fold codes
#pragma unroll
          for (int r = 0; r < 4; ++r) cw[r] *= 0.0625f;
        }
        if constexpr (!GROUPED) {
          if (tb.has_seg_scale) {
#pragma unroll
            for (int r = 0; r < 4; ++r) cw[r] *= seg_scale_of(tb, ks, ncol + r);
          }
        }
        const bool dyn = a.tok_steps != nullptr || a.x_raw_dynamic != 0;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          float sp = tb.s_pos[ks], sn = dl ? tb.s_neg[ks] : 0.0f;
          if (dyn) {                                               // this lane's token row
            const int ti = 2 * ((mt * 16 + mlane) * tb.S + ks);
            sp = tok[ti];
            sn = dl ? tok[ti + 1] : 0.0f;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float t = (cw[r] * sp) * acc_value<FP8>(accp[mt][r]);
            if (DUAL) t += (cw[r] * sn) * acc_value<FP8>(accn[mt][r]);
            fsum[mt][r] += t;
          }
        }
      }
    }
    // ---- group done: bias, cast, store -------------------------------------------------------------------------
    if (mode != OUT_DEBUG_ACC) {
      float bs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      if (l_bias) {
        float b16[16];
        fetch_group16(l_bias + gl * 16, a.N - gl * 16, b16);
        pick4(b16, fq, bs);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + mlane;
        if (m < a.M) {
          const size_t o = (size_t)m * a.N + ncol;
          float t[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) t[r] = fsum[mt][r] + bs[r];
          if (vec4 && ncol + 3 < a.N) {
            if (mode == OUT_F32) {
              const v4f o4 = {t[0], t[1], t[2], t[3]};
              *reinterpret_cast<v4f*>(reinterpret_cast<float*>(l_y) + o) = o4;
            } else {
              v2i o2;
              o2[0] = (int)f32x2_to_bf16x2(t[0], t[1]);
              o2[1] = (int)f32x2_to_bf16x2(t[2], t[3]);
              *reinterpret_cast<v2i*>(reinterpret_cast<uint16_t*>(l_y) + o) = o2;
            }
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (ncol + r < a.N) {
                if (mode == OUT_F32) reinterpret_cast<float*>(l_y)[o + r] = t[r];
                else reinterpret_cast<uint16_t*>(l_y)[o + r] = f32_to_bf16(t[r]);
              }
          }
        }
      }
    }
  }
}

// Wide skinny layers only: enough 16-column groups to give every wave of the chip a run of them; K and every
// K-segment boundary multiples of 128 (a step is a full cache line per row); X^ slab within the LDS budget.
static bool any_dual(const int* dual, int S) {
  bool d = false;
  for (int s = 0; s < S; ++s) d = d || dual[s] != 0;
  return d;
}

// Size class of the X^ slab (24 = small, 80, 0 = does not fit) and whether it holds the two polarity planes
// (dual layers with at most two 16-row tiles whose doubled slab still fits).
static int stream_slab_kb(const GemmArgs& a, bool dual, bool* two_planes) {
  const int mt = (a.M + 15) / 16;
  const long slab = (long)mt * 16 * (a.K + 16);
  *two_planes = dual && mt <= 2 && 2 * slab <= 80 * 1024;
  if (*two_planes) return 2 * slab <= 48 * 1024 ? 24 : 80;
  if (slab <= 24 * 1024) return 24;
  if (slab <= 80 * 1024) return 80;
  return 0;
}

// This file is compiled twice: as it is (int8 and packed 4-bit codes), and with -DSQ_STREAM_FP8=1 for the instantiations
// on fp8 codes only (the kernel is the largest of the library; two translation units build side by side).
#ifndef SQ_STREAM_FP8
bool stream_supported(const GemmArgs& a, const GemmTable& tb) {
  if (a.M > 64 || a.K % 128 != 0 || a.K < 128) return false;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 128 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.xq) | reinterpret_cast<uintptr_t>(a.wq)) % 16 != 0) return false;
  bool ps;
  if (stream_slab_kb(a, any_dual(tb.dual, tb.S), &ps) == 0) return false;
  return true;
}
#endif

template <int MT, int SLAB_KB, bool W4, bool FP8>
static hipError_t launch_stream_ms(const GemmArgs& a, const GemmTable& tb, int mode, bool dual, bool ps, int grid, hipStream_t st) {
#define SQ_K(D, P) hipLaunchKernelGGL((seglinear_stream_kernel<MT, D, SLAB_KB, GemmTable, NoGroups, W4, P, FP8>), dim3(grid), dim3(stream_waves(MT) * 64), 0, st, a, tb, NoGroups{}, mode)
  if constexpr (MT <= 2) {
    if (dual && ps) { SQ_K(true, true); return hipGetLastError(); }
  }
  if (dual) SQ_K(true, false);
  else SQ_K(false, false);
#undef SQ_K
  return hipGetLastError();
}

template <bool W4, bool FP8>
static hipError_t launch_stream_impl(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st) {
  const bool dual = any_dual(tb.dual, tb.S);
  const int mt = (a.M + 15) / 16;
  const int ngroups = (a.N + 15) / 16;
  int grid = ngroups < cus ? ngroups : cus;
  bool ps;
  const int slab = stream_slab_kb(a, dual, &ps);
#define SQ_STREAM(MT_) \
  (slab == 24 ? launch_stream_ms<MT_, 24, W4, FP8>(a, tb, mode, dual, ps, grid, st) : launch_stream_ms<MT_, 80, W4, FP8>(a, tb, mode, dual, ps, grid, st))
  switch (mt) {
    case 1: return SQ_STREAM(1);
    case 2: return SQ_STREAM(2);
    case 3: return SQ_STREAM(3);
    default: return SQ_STREAM(4);
  }
#undef SQ_STREAM
}

#ifdef SQ_STREAM_FP8
// fp8 (E4M3) codes: same shapes as stream_supported(); static steps
hipError_t launch_seglinear_stream_fp8(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st) {
  if (a.x_raw != nullptr || a.tok_steps != nullptr || mode == OUT_DEBUG_ACC) return hipErrorInvalidConfiguration;
  return launch_stream_impl<false, true>(a, tb, mode, cus, st);
}
#else
hipError_t launch_seglinear_stream(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st) {
  return launch_stream_impl<false, false>(a, tb, mode, cus, st);
}

// a.wq points at packed 4-bit codes [N][K/2]
hipError_t launch_seglinear_stream_w4(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st) {
  return launch_stream_impl<true, false>(a, tb, mode, cus, st);
}

// Grouped call: L layers of one shape that share X^ (M <= 32).  a.wq / a.wscale / a.bias / a.y are unused.
bool stream_grouped_supported(const GemmArgs& a, const GroupSegTable& tb) {
  if (a.M > 32 || a.K % 128 != 0 || a.K < 128) return false;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 128 != 0) return false;
  if (reinterpret_cast<uintptr_t>(a.xq) % 16 != 0) return false;
  bool ps;
  return stream_slab_kb(a, any_dual(tb.dual, tb.S), &ps) != 0;
}

#endif

template <int MT, int SLAB_KB, bool W4, bool FP8>
static hipError_t launch_grouped_ms(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, int mode, bool dual,
                                    bool ps, int grid, hipStream_t st) {
#define SQ_K(D, P) hipLaunchKernelGGL((seglinear_stream_kernel<MT, D, SLAB_KB, GroupSegTable, GroupTable, W4, P, FP8>), dim3(grid), dim3(stream_waves(MT) * 64), 0, st, a, tb, gt, mode)
  if (dual && ps) SQ_K(true, true);
  else if (dual) SQ_K(true, false);
  else SQ_K(false, false);
#undef SQ_K
  return hipGetLastError();
}

template <bool W4, bool FP8>
static hipError_t launch_grouped_impl(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, OutMode mode, int cus,
                                      hipStream_t st) {
  const bool dual = any_dual(tb.dual, tb.S);
  const int mt = (a.M + 15) / 16;
  const long ngroups = (long)((a.N + 15) / 16) * gt.L;
  const int grid = (int)(ngroups < cus ? ngroups : cus);
  bool ps;
  const int slab = stream_slab_kb(a, dual, &ps);
  if (mt == 1) return slab == 24 ? launch_grouped_ms<1, 24, W4, FP8>(a, tb, gt, mode, dual, ps, grid, st) : launch_grouped_ms<1, 80, W4, FP8>(a, tb, gt, mode, dual, ps, grid, st);
  return slab == 24 ? launch_grouped_ms<2, 24, W4, FP8>(a, tb, gt, mode, dual, ps, grid, st) : launch_grouped_ms<2, 80, W4, FP8>(a, tb, gt, mode, dual, ps, grid, st);
}

#ifndef SQ_STREAM_FP8
// w4: the items' wq point to packed 4-bit codes (quantize_weight_w4_kernel's layout)
hipError_t launch_seglinear_grouped(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, OutMode mode, int cus,
                                    hipStream_t st, bool w4) {
  return w4 ? launch_grouped_impl<true, false>(a, tb, gt, mode, cus, st) : launch_grouped_impl<false, false>(a, tb, gt, mode, cus, st);
}
#else
// the items' wq point to fp8 (E4M3) codes; static steps, code input
hipError_t launch_seglinear_grouped_fp8(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, OutMode mode, int cus,
                                        hipStream_t st) {
  if (a.x_raw != nullptr || a.tok_steps != nullptr || mode == OUT_DEBUG_ACC) return hipErrorInvalidConfiguration;
  return launch_grouped_impl<false, true>(a, tb, gt, mode, cus, st);
}
#endif

}  // namespace sq
