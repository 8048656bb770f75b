// Tile configurations of the large-M MFMA kernel.  Each one is compiled in a translation unit of its
// own (seglinear_mfma_inst.hip with -DSQ_VARIANT=<id>) so the library builds in parallel.
#pragma once
#include "sq_kernels.hpp"

namespace sq {

template <int V> struct MfmaVariant;
//                                   block tile   wave grid  LDS stages  dual accumulators fit?  fp32 running sum fits with dual?
#define SQ_DEF_VARIANT(V, BM_, BN_, WM_, WN_, NS_, DUAL_OK_, MULTI_DUAL_OK_)                           \
  template <> struct MfmaVariant<V> {                                                                  \
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, NS = NS_;                             \
    static constexpr bool DUAL_OK = DUAL_OK_, MULTI_DUAL_OK = MULTI_DUAL_OK_;                          \
  };
SQ_DEF_VARIANT(0, 128, 256, 2, 2, 4, true, false)   // wave tile 64 x 128, both polarities: 256 accumulator registers
SQ_DEF_VARIANT(1, 128, 128, 2, 2, 4, true, true)    // wave tile 64 x 64
SQ_DEF_VARIANT(2, 64, 256, 1, 4, 4, true, true)     // wave tile 64 x 64, tall-W blocks
SQ_DEF_VARIANT(3, 64, 128, 2, 2, 4, true, true)     // wave tile 32 x 64, small problems
SQ_DEF_VARIANT(4, 256, 256, 2, 2, 4, false, false)  // wave tile 128 x 128, single-path layers only
SQ_DEF_VARIANT(5, 128, 256, 2, 4, 4, true, true)    // 8 waves (2 per SIMD), wave tile 64 x 64
#undef SQ_DEF_VARIANT
constexpr int kNumMfmaVariants = 6;

struct MfmaVariantInfo { int BM, BN; bool dual_ok, multi_dual_ok; };

template <int V>
hipError_t launch_mfma_variant(const GemmArgs& a, const GemmTable& tb, int mode, bool dual, bool multi, hipStream_t st);

}  // namespace sq
