// One tile configuration of the MFMA kernel (selected with -DSQ_VARIANT=<id>), instantiated for the
// four (dual, multi-K-segment) combinations it supports; -DSQ_FP8=1 builds the same set for fp8 (E4M3) codes.
#include "seglinear_mfma_kernel.hpp"
#include "seglinear_mfma_variants.hpp"

#ifndef SQ_VARIANT
#error "compile with -DSQ_VARIANT=<id>"
#endif
#ifndef SQ_FP8
#define SQ_FP8 0
#endif

namespace sq {

constexpr bool kFp8 = SQ_FP8 != 0;

template <int V, bool DUAL, bool MULTI, bool SHARE>
static hipError_t launch_one(const GemmArgs& a, const GemmTable& tb, int mode, hipStream_t st) {
  using P = MfmaVariant<V>;
  if constexpr (kFp8) {                              // static steps only
    if (a.tok_steps != nullptr) return hipErrorInvalidConfiguration;
    auto kern = seglinear_mfma_kernel<P::BM, P::BN, P::WM, P::WN, P::NS, P::SK, P::MINB, DUAL, MULTI, SHARE, false, true>;
    hipLaunchKernelGGL(kern, dim3(a.num_wg), dim3(P::WM * P::WN * 64), 0, st, a, tb, mode);
    return hipGetLastError();
  } else {
    if (a.tok_steps != nullptr) {                      // dynamic per-token steps: built for the tiles listed in TOK_OK
      if constexpr (P::TOK_OK) {
        auto kern = seglinear_mfma_kernel<P::BM, P::BN, P::WM, P::WN, P::NS, P::SK, P::MINB, DUAL, MULTI, SHARE, true>;
        hipLaunchKernelGGL(kern, dim3(a.num_wg), dim3(P::WM * P::WN * 64), 0, st, a, tb, mode);
        return hipGetLastError();
      } else {
        return hipErrorInvalidConfiguration;
      }
    }
    auto kern = seglinear_mfma_kernel<P::BM, P::BN, P::WM, P::WN, P::NS, P::SK, P::MINB, DUAL, MULTI, SHARE>;
    hipLaunchKernelGGL(kern, dim3(a.num_wg), dim3(P::WM * P::WN * 64), 0, st, a, tb, mode);
    return hipGetLastError();
  }
}

template <int V, bool FP8>
hipError_t launch_mfma_variant(const GemmArgs& a, const GemmTable& tb, int mode, bool dual, bool multi, bool share,
                               hipStream_t st) {
  using P = MfmaVariant<V>;
  if (dual) {
    if constexpr (P::DUAL_OK) {
      if (multi && share) {
        if constexpr (P::SHARE_OK) return launch_one<V, true, true, true>(a, tb, mode, st);
        else return hipErrorInvalidConfiguration;
      }
      if (multi) {
        if constexpr (P::MULTI_DUAL_OK) return launch_one<V, true, true, false>(a, tb, mode, st);
        else return hipErrorInvalidConfiguration;
      }
      return launch_one<V, true, false, false>(a, tb, mode, st);
    } else {
      return hipErrorInvalidConfiguration;
    }
  }
  if (multi) {
    if constexpr (P::MULTI_OK) return launch_one<V, false, true, false>(a, tb, mode, st);
    else return hipErrorInvalidConfiguration;
  }
  return launch_one<V, false, false, false>(a, tb, mode, st);
}

template hipError_t launch_mfma_variant<SQ_VARIANT, kFp8>(const GemmArgs&, const GemmTable&, int, bool, bool, bool, hipStream_t);

}  // namespace sq
