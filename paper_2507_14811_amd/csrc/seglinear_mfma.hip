// Variant table and selection heuristic of the large-M MFMA kernel; the kernels themselves are
// instantiated one variant per translation unit (seglinear_mfma_inst.hip).
#include <utility>

#include "seglinear_mfma_variants.hpp"

namespace sq {

// Per-variant launchers (defined in the per-variant translation units) and properties, as tables.
using LaunchFn = hipError_t (*)(const GemmArgs&, const GemmTable&, int, bool, bool, bool, hipStream_t);
template <int V> static constexpr MfmaVariantInfo info_of() {
  using P = MfmaVariant<V>;
  return {P::BM, P::BN, P::SK, P::MINB, P::DUAL_OK, P::MULTI_OK, P::MULTI_DUAL_OK, P::SHARE_OK, P::TOK_OK};
}
template <int V> static constexpr LaunchFn fp8_launcher() {
  if constexpr (kMfmaVariantHasFp8[V]) return &launch_mfma_variant<V, true>;
  else return nullptr;
}
template <int... V> struct VariantTables {
  static constexpr LaunchFn launch[sizeof...(V)] = {&launch_mfma_variant<V>...};
  static constexpr LaunchFn launch_fp8[sizeof...(V)] = {fp8_launcher<V>()...};
  static constexpr MfmaVariantInfo info[sizeof...(V)] = {info_of<V>()...};
};
template <int... V> static constexpr VariantTables<V...> tables_of(std::integer_sequence<int, V...>) { return {}; }
using Tables = decltype(tables_of(std::make_integer_sequence<int, kNumMfmaVariants>{}));
static MfmaVariantInfo variant_info(int v) { return Tables::info[v]; }
int mfma_num_variants() { return kNumMfmaVariants; }
static int g_group_m = 0;
void mfma_set_group_m(int g) { g_group_m = g; }

// dual: some K-segment runs both polarity paths; multi: more than one K-segment; share: exactly one dual
// segment among several, so it can be visited first and its X^_- accumulator registers re-used as the fp32
// running sum afterwards.
static void layer_flags(const GemmTable& tb, bool& dual, bool& multi, bool& share) {
  int ndual = 0;
  for (int s = 0; s < tb.S; ++s) ndual += (tb.dual[s] != 0);
  dual = ndual > 0;
  multi = tb.S > 1;
  share = multi && ndual == 1;
}

// Largest stage depth (128 or 64 bytes of K) that K and every K-segment boundary are a multiple of.
static int k_alignment(const GemmArgs& a, const GemmTable& tb) {
  int al = (a.K % 128 == 0) ? 128 : 64;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 128 != 0) al = 64;
  return al;
}

static bool variant_ok(int v, bool dual, bool multi, bool share, int kalign, bool tok) {
  if (v < 0 || v >= kNumMfmaVariants) return false;
  const MfmaVariantInfo i = variant_info(v);
  if (tok && !i.tok_ok) return false;
  if (i.SK > kalign) return false;
  if (dual && !i.dual_ok) return false;
  if (dual && multi && !(i.multi_dual_ok || (share && i.share_ok))) return false;
  if (!dual && multi && !i.multi_ok) return false;
  return true;
}

bool mfma_supported(const GemmArgs& a, const GemmTable& tb) {
  if (a.K % 64 != 0) return false;
  for (int s = 0; s <= tb.S; ++s)
    if (tb.kseg_off[s] % 64 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.xq) | reinterpret_cast<uintptr_t>(a.wq)) % 16 != 0) return false;
  return true;
}

// Automatic choice: occupancy of the last round of tiles (fill) times a relative efficiency of the tile
// shape, measured on MI355X per layer class (single-path / dual / dual with several K-segments).
static const float kEffSingle[kNumMfmaVariants] = {1.00f, 0.85f, 0.82f, 0.62f, 0.95f, 0.95f, 0.72f, 0.71f, 0.88f};
static const float kEffDual[kNumMfmaVariants] = {1.00f, 0.78f, 0.77f, 0.65f, 0.00f, 0.76f, 0.70f, 0.77f, 0.88f};
static const float kEffDualMulti[kNumMfmaVariants] = {1.00f, 0.78f, 0.76f, 0.65f, 0.00f, 0.87f, 0.72f, 0.75f, 0.90f};

// Compute units of the current device (MI355X: 256), looked up once per device.
int device_cus() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int cus = 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    cached[dev] = cus;
  }
  return cached[dev];
}

int mfma_pick_variant(const GemmArgs& a, const GemmTable& tb, OutMode) {
  bool dual, multi, share;
  layer_flags(tb, dual, multi, share);
  const int cus = device_cus();
  const float* eff = dual ? (multi ? kEffDualMulti : kEffDual) : kEffSingle;
  int best = -1;
  float best_score = -1.0f;
  for (int v = 0; v < kNumMfmaVariants; ++v) {
    if (!variant_ok(v, dual, multi, share, k_alignment(a, tb), a.tok_steps != nullptr)) continue;
    const MfmaVariantInfo i = variant_info(v);
    const long tiles = (long)((a.M + i.BM - 1) / i.BM) * ((a.N + i.BN - 1) / i.BN);
    const long slots = (long)cus * i.MINB;
    const long rounds = (tiles + slots - 1) / slots;
    const float fill = (float)((double)a.M * a.N / ((double)rounds * slots * i.BM * i.BN));
    const float score = fill * eff[v];
    if (score > best_score) { best_score = score; best = v; }
  }
  return best;
}

// fp8 codes: the tile configurations built for them (128-byte stages, static steps), same fill-times-efficiency choice
// (relative efficiencies measured on MI355X: 8500 x 1536 x 4608 single-path and dual, 4608 x 15360 x 3072 dual with two
// K-segments, 2048 x 4608 x 1152 dual)
static const float kEffFp8Single[kNumMfmaVariants] = {0.76f, 0.68f, 0.0f, 0.52f, 1.00f, 0.83f, 0.0f, 0.0f, 0.87f};
static const float kEffFp8Dual[kNumMfmaVariants] = {0.96f, 0.80f, 0.0f, 0.69f, 0.0f, 0.83f, 0.0f, 0.0f, 1.00f};
static bool fp8_variant_ok(int v, bool dual, bool multi, bool share, int kalign) {
  return kalign == 128 && variant_ok(v, dual, multi, share, kalign, false) && kMfmaVariantHasFp8[v];
}
int mfma_fp8_pick_variant(const GemmArgs& a, const GemmTable& tb) {
  bool dual, multi, share;
  layer_flags(tb, dual, multi, share);
  const int cus = device_cus();
  const float* eff = dual ? kEffFp8Dual : kEffFp8Single;
  int best = -1;
  float best_score = -1.0f;
  for (int v = 0; v < kNumMfmaVariants; ++v) {
    if (!fp8_variant_ok(v, dual, multi, share, k_alignment(a, tb))) continue;
    const MfmaVariantInfo i = variant_info(v);
    const long tiles = (long)((a.M + i.BM - 1) / i.BM) * ((a.N + i.BN - 1) / i.BN);
    const long slots = (long)cus * i.MINB;
    const long rounds = (tiles + slots - 1) / slots;
    const float score = (float)((double)a.M * a.N / ((double)rounds * slots * i.BM * i.BN)) * eff[v];
    if (score > best_score) { best_score = score; best = v; }
  }
  return best;
}

static hipError_t launch_tiles(GemmArgs a, const GemmTable& tb_in, OutMode mode, int variant, bool fp8, hipStream_t st);

hipError_t launch_seglinear_mfma(GemmArgs a, const GemmTable& tb_in, OutMode mode, int variant, hipStream_t st) {
  return launch_tiles(a, tb_in, mode, variant, false, st);
}
hipError_t launch_seglinear_mfma_fp8(GemmArgs a, const GemmTable& tb_in, OutMode mode, int variant, hipStream_t st) {
  if (a.tok_steps != nullptr || mode == OUT_DEBUG_ACC) return hipErrorInvalidConfiguration;
  return launch_tiles(a, tb_in, mode, variant, true, st);
}

static hipError_t launch_tiles(GemmArgs a, const GemmTable& tb_in, OutMode mode, int variant, bool fp8, hipStream_t st) {
  bool dual, multi, share;
  layer_flags(tb_in, dual, multi, share);
  if (fp8 ? !fp8_variant_ok(variant, dual, multi, share, k_alignment(a, tb_in))
          : !variant_ok(variant, dual, multi, share, k_alignment(a, tb_in), a.tok_steps != nullptr))
    return hipErrorInvalidConfiguration;
  const MfmaVariantInfo i = variant_info(variant);
  GemmTable tb = tb_in;
  share = share && i.share_ok;        // prefer the register-sharing mode wherever the tile supports it
  if (share) {                        // visit the dual K-segment first, the others in ascending order
    int pos = 0;
    for (int s = 0; s < tb.S; ++s)
      if (tb.dual[s]) tb.seg_order[pos++] = s;
    for (int s = 0; s < tb.S; ++s)
      if (!tb.dual[s]) tb.seg_order[pos++] = s;
  }
  a.tiles_m = (a.M + i.BM - 1) / i.BM;
  a.tiles_n = (a.N + i.BN - 1) / i.BN;
  const int gm = g_group_m > 0 ? g_group_m : 8;
  a.group_m = a.tiles_m < gm ? a.tiles_m : gm;
  // persistent workgroups: one per compute unit (times the variant's residency), fewer if there are fewer tiles
  const long slots = (long)device_cus() * i.MINB;
  const long tiles = (long)a.tiles_m * a.tiles_n;
  a.num_wg = (int)(tiles < slots ? tiles : slots);
  return (fp8 ? Tables::launch_fp8[variant] : Tables::launch[variant])(a, tb, mode, dual, multi, share, st);
}

}  // namespace sq
