// Tile configurations of the large-M MFMA kernel.  Each one is compiled in a translation unit of its
// own (seglinear_mfma_inst.hip with -DSQ_VARIANT=<id>) so the library builds in parallel.
#pragma once
#include "sq_kernels.hpp"

namespace sq {

template <int V> struct MfmaVariant;
//             id  block tile  wave grid  stages  K bytes/stage  workgroups per CU   register budget allows: two accumulator sets? /
//                                                                fp32 running sum (multi-K-segment)? / both? /
//                                                                both when the X^_- set's registers double as the running sum?
#define SQ_DEF_VARIANT(V, BM_, BN_, WM_, WN_, NS_, SK_, MINB_, DUAL_OK_, MULTI_OK_, MULTI_DUAL_OK_, SHARE_OK_)                   \
  template <> struct MfmaVariant<V> {                                                                  \
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NS = NS_, SK = SK_, MINB = MINB_;                   \
    static constexpr bool DUAL_OK = DUAL_OK_, MULTI_OK = MULTI_OK_, MULTI_DUAL_OK = MULTI_DUAL_OK_,     \
                          SHARE_OK = SHARE_OK_;                                                    \
    static constexpr bool TOK_OK = (V == 0 || V == 1 || V == 3 || V == 7 || V == 8);   /* instantiated with per-token activation steps */ \
  };
SQ_DEF_VARIANT(0, 128, 256, 2, 2, 3, 128, 1, true, true, false, true)   // wave tile 64 x 128, both polarities: 256 accumulator registers
SQ_DEF_VARIANT(1, 128, 128, 2, 2, 3, 128, 1, true, true, true, true)    // wave tile 64 x 64
SQ_DEF_VARIANT(2, 64, 256, 1, 4, 3, 128, 1, true, true, true, true)     // wave tile 64 x 64, wide-N blocks
SQ_DEF_VARIANT(3, 64, 128, 2, 2, 4, 128, 1, true, true, true, true)     // wave tile 32 x 64, small problems
SQ_DEF_VARIANT(4, 256, 256, 2, 2, 2, 128, 1, false, false, false, false)  // wave tile 128 x 128, single-path layers only
SQ_DEF_VARIANT(5, 128, 256, 2, 4, 2, 128, 1, true, true, true, true)    // 8 waves (2 per SIMD), wave tile 64 x 64
SQ_DEF_VARIANT(6, 128, 128, 2, 2, 4, 64, 1, true, true, true, true)     // 64-byte stages: K-segment boundaries that are only 64-aligned
SQ_DEF_VARIANT(7, 64, 192, 2, 2, 4, 128, 1, true, true, true, true)     // wave tile 32 x 96: N = 192 * odd, mid-size problems
SQ_DEF_VARIANT(8, 128, 192, 2, 2, 3, 128, 1, true, true, true, true)    // wave tile 64 x 96
#undef SQ_DEF_VARIANT
constexpr int kNumMfmaVariants = 9;
// tile configurations also built for fp8 codes (128-byte stages only); listed again in the build script
constexpr bool kMfmaVariantHasFp8[kNumMfmaVariants] = {true, true, false, true, true, true, false, false, true};

struct MfmaVariantInfo { int BM, BN, SK, MINB; bool dual_ok, multi_ok, multi_dual_ok, share_ok, tok_ok; };

template <int V, bool FP8 = false>
hipError_t launch_mfma_variant(const GemmArgs& a, const GemmTable& tb, int mode, bool dual, bool multi, bool share,
                               hipStream_t st);

}  // namespace sq
