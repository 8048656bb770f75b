// C ABI of the library: host-side validation, table marshalling and kernel selection.  No device
// memory is allocated and no state is kept between calls (apart from the diagnostics overrides).
#include <cmath>
#include <cstring>

#include "sq_kernels.hpp"

namespace {

int g_gemm_variant = -1;   // sq_tuning_set("gemm_variant", v)
int g_force_path = -1;     // sq_tuning_set("force_path", p): 0 generic, 1 MFMA tiles, 2 skinny, 3 skinny weight stream

bool offsets_ok(int n, int cnt, const int32_t* off) {
  if (cnt < 1 || cnt > SQ_MAX_SEGMENTS || off == nullptr) return false;
  if (off[0] != 0 || off[cnt] != n) return false;
  for (int i = 0; i < cnt; ++i)
    if (off[i + 1] <= off[i]) return false;
  return true;
}

bool step_ok(float s) { return std::isfinite(s) && s > 0.0f; }

// Shape / table checks shared by every entry point.  need_scales: s_pos / s_neg are used by the call.
sq_status check_layer(const sq_layer* L, bool need_m, bool need_scales) {
  (void)hipGetLastError();   // every entry point starts here: an error left by an unrelated earlier call is not this call's
  if (L == nullptr) return SQ_ERR_INVALID_ARG;
  if (L->K < 1 || L->N < 1 || (need_m && L->M < 1)) return SQ_ERR_INVALID_ARG;
  if (L->S < 1 || L->T < 1) return SQ_ERR_INVALID_ARG;
  if (L->S > SQ_MAX_SEGMENTS || L->T > SQ_MAX_SEGMENTS) return SQ_ERR_UNSUPPORTED;
  if (!offsets_ok(L->K, L->S, L->kseg_off) || !offsets_ok(L->N, L->T, L->nseg_off)) return SQ_ERR_INVALID_ARG;
  if (L->dual == nullptr) return SQ_ERR_INVALID_ARG;
  if (need_scales) {
    if (L->s_pos == nullptr) return SQ_ERR_INVALID_ARG;
    for (int s = 0; s < L->S; ++s) {
      if (!step_ok(L->s_pos[s])) return SQ_ERR_INVALID_ARG;
      if (L->dual[s]) {
        if (L->s_neg == nullptr || !step_ok(L->s_neg[s])) return SQ_ERR_INVALID_ARG;
      }
    }
  }
  if (L->seg_scale) {                      // read (copied into the kernel's table) by every GEMM entry point
    if ((long)L->S * L->T > SQ_MAX_SEG_SCALE) return SQ_ERR_UNSUPPORTED;
    for (int i = 0; i < L->S * L->T; ++i)
      if (!std::isfinite(L->seg_scale[i])) return SQ_ERR_INVALID_ARG;
  }
  for (int s = 0; s < L->S; ++s)
    if (L->kseg_off[s + 1] - L->kseg_off[s] > SQ_MAX_KSEG_LEN) return SQ_ERR_UNSUPPORTED;
  const long long lim = 0x7FFFFFFFll;
  if ((long long)L->N * L->K > lim) return SQ_ERR_UNSUPPORTED;
  if (need_m && ((long long)L->M * L->K > lim || (long long)L->M * L->N > lim)) return SQ_ERR_UNSUPPORTED;
  return SQ_OK;
}

// Reciprocal used by the fast path of round(x / s); NaN tells the kernel to always divide.
float safe_inv(float s) {
  if (!(s >= 1e-30f && s <= 1e30f)) return std::nanf("");
  return 1.0f / s;
}

void fill_gemm_table(const sq_layer* L, sq::GemmTable& tb) {
  std::memset(&tb, 0, sizeof(tb));
  tb.S = L->S;
  tb.T = L->T;
  for (int s = 0; s <= L->S; ++s) tb.kseg_off[s] = L->kseg_off[s];
  for (int t = 0; t <= L->T; ++t) tb.nseg_off[t] = L->nseg_off[t];
  for (int s = 0; s < L->S; ++s) {
    tb.dual[s] = L->dual[s] ? 1 : 0;
    tb.seg_order[s] = s;
    tb.s_pos[s] = L->s_pos ? L->s_pos[s] : 1.0f;
    tb.s_neg[s] = (L->dual[s] && L->s_neg) ? L->s_neg[s] : 0.0f;
    tb.inv_pos[s] = safe_inv(tb.s_pos[s]);
    tb.inv_neg[s] = safe_inv(tb.s_neg[s]);
  }
  tb.has_seg_scale = L->seg_scale != nullptr;
  if (L->seg_scale) std::memcpy(tb.seg_scale, L->seg_scale, sizeof(float) * L->S * L->T);
}

sq_status run_gemm(const sq_layer* L, const int8_t* xq, const int8_t* wq,
                   const float* wscale, const float* bias, void* y, int32_t* acc_pos, int32_t* acc_neg,
                   sq::OutMode mode, void* stream) {
  sq::GemmTable tb;
  fill_gemm_table(L, tb);
  sq::GemmArgs a{};
  a.xq = xq;
  a.wq = wq;
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.acc_pos = acc_pos;
  a.acc_neg = acc_neg;
  a.M = L->M;
  a.K = L->K;
  a.N = L->N;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  int path = g_force_path;
  if (path == 3 && !sq::stream_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  if (path == 2 && !sq::skinny_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  if (path == 1 && !sq::mfma_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  if (path < 0) {
    // up to two 16-row tiles of tokens: the weight-stream kernel (measured 5.9 TB/s on wide layers); three or four
    // tiles: the MFMA tile kernel with 64-row tiles is as fast or faster; the K-splitting skinny kernel serves
    // the layers whose K-segments are only 64-aligned
    if (a.M <= 32 && sq::stream_supported(a, tb)) path = 3;
    else if (a.M <= 64 && a.M > 32 && sq::mfma_supported(a, tb)) path = 1;
    else if (sq::skinny_supported(a, tb)) path = 2;
    else if (sq::mfma_supported(a, tb)) path = 1;
    else path = 0;
  }
  hipError_t e;
  if (path == 3) {
    e = sq::launch_seglinear_stream(a, tb, mode, sq::device_cus(), st);
  } else if (path == 2) {
    e = sq::launch_seglinear_skinny(a, tb, mode, st);
  } else if (path == 1) {
    int v = g_gemm_variant >= 0 ? g_gemm_variant : sq::mfma_pick_variant(a, tb, mode);
    e = sq::launch_seglinear_mfma(a, tb, mode, v, st);
    if (e == hipErrorInvalidConfiguration) return SQ_ERR_UNSUPPORTED;
  } else {
    e = sq::launch_seglinear_generic(a, tb, mode, st);
  }
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

// 4-bit packed weights: K and every K-segment boundary a multiple of 128.  The weight-stream kernel serves M <= 64
// (this is where halving the weight bytes pays: the pass is HBM-bound); everything else takes the one-thread-per-output
// kernel, which is correct and slow.  force_path 0 selects the latter also for small M.
bool w4_layout_ok(const sq_layer* L) {
  if (L->K < 128 || L->K % 128 != 0) return false;
  for (int s = 0; s <= L->S; ++s)
    if (L->kseg_off[s] % 128 != 0) return false;
  return true;
}

// Dynamic per-token steps: the weight-stream kernel (M <= 64, at most 8 K-segments: its step table is 4 KiB of LDS), the
// MFMA tile kernel (8-bit weights, its alignment rules) or the one-thread-per-output kernel (any shape, 4-bit weights at
// large M).
sq_status run_gemm_dynamic(const sq_layer* L, const int8_t* xq, const float* tok_steps, const void* wq, int w_bits,
                           const float* wscale, const float* bias, void* y, sq::OutMode mode, void* stream) {
  if (w_bits == 4 && !w4_layout_ok(L)) return SQ_ERR_UNSUPPORTED;
  sq::GemmTable tb;
  fill_gemm_table(L, tb);
  for (int s = 0; s < L->S; ++s) { tb.s_pos[s] = 1.0f; tb.s_neg[s] = L->dual[s] ? 1.0f : 0.0f; }
  sq::GemmArgs a{};
  a.xq = xq;
  a.wq = reinterpret_cast<const int8_t*>(wq);
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.M = L->M;
  a.K = L->K;
  a.N = L->N;
  a.tok_steps = tok_steps;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const bool stream_ok = L->S <= 8 && sq::stream_supported(a, tb);
  const bool mfma_ok = w_bits == 8 && sq::mfma_supported(a, tb) && sq::mfma_pick_variant(a, tb, mode) >= 0;
  if (g_force_path == 3 && !stream_ok) return SQ_ERR_UNSUPPORTED;
  if (g_force_path == 1 && !mfma_ok) return SQ_ERR_UNSUPPORTED;
  hipError_t e;
  if (g_force_path != 0 && g_force_path != 1 && stream_ok) {
    e = w_bits == 4 ? sq::launch_seglinear_stream_w4(a, tb, mode, sq::device_cus(), st)
                    : sq::launch_seglinear_stream(a, tb, mode, sq::device_cus(), st);
  } else if (g_force_path != 0 && mfma_ok) {           // large M, 8-bit weights: the MFMA tile kernel with per-row steps
    int v = g_gemm_variant >= 0 ? g_gemm_variant : sq::mfma_pick_variant(a, tb, mode);
    e = sq::launch_seglinear_mfma(a, tb, mode, v, st);
    if (e == hipErrorInvalidConfiguration) return SQ_ERR_UNSUPPORTED;
  } else {
    e = w_bits == 4 ? sq::launch_seglinear_generic_w4(a, tb, mode, st) : sq::launch_seglinear_generic(a, tb, mode, st);
  }
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status run_gemm_w4(const sq_layer* L, const int8_t* xq, const uint8_t* wq4, const float* wscale, const float* bias,
                      void* y, int32_t* acc_pos, int32_t* acc_neg, sq::OutMode mode, void* stream) {
  if (!w4_layout_ok(L)) return SQ_ERR_UNSUPPORTED;
  sq::GemmTable tb;
  fill_gemm_table(L, tb);
  sq::GemmArgs a{};
  a.xq = xq;
  a.wq = reinterpret_cast<const int8_t*>(wq4);
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.acc_pos = acc_pos;
  a.acc_neg = acc_neg;
  a.M = L->M;
  a.K = L->K;
  a.N = L->N;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const bool stream_ok = sq::stream_supported(a, tb);
  if (g_force_path == 3 && !stream_ok) return SQ_ERR_UNSUPPORTED;
  hipError_t e;
  if (g_force_path != 0 && stream_ok) e = sq::launch_seglinear_stream_w4(a, tb, mode, sq::device_cus(), st);
  else e = sq::launch_seglinear_generic_w4(a, tb, mode, st);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

}  // namespace

extern "C" {

sq_status sq_quantize_weight(const sq_layer* layer, const void* w, sq_dtype w_dt, int8_t* wq, float* wscale,
                             void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || wq == nullptr || wscale == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::KsegTable tb;
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.off[s] = layer->kseg_off[s];
  hipError_t e = sq::launch_quantize_weight(w, w_dt == SQ_BF16, wq, wscale, layer->N, layer->K, tb,
                                            reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_quantize_weight_block(const sq_layer* layer, const void* w, sq_dtype w_dt, int8_t* wq, float* wscale,
                                   void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || wq == nullptr || wscale == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::KsegTable kt, nt;
  kt.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) kt.off[s] = layer->kseg_off[s];
  nt.S = layer->T;
  for (int t = 0; t <= layer->T; ++t) nt.off[t] = layer->nseg_off[t];
  hipError_t e = sq::launch_quantize_weight_block(w, w_dt == SQ_BF16, wq, wscale, layer->N, layer->K, kt, nt,
                                                  reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_calibrate_act(const sq_layer* layer, const void* x, sq_dtype x_dt, float* amax, float* steps, int accumulate,
                           void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || amax == nullptr || steps == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) tb.dual[s] = layer->dual[s] ? 1 : 0;
  hipError_t e = sq::launch_calibrate_act(x, x_dt == SQ_BF16, layer->M, layer->K, tb, amax, steps, accumulate != 0,
                                          reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

size_t sq_calibrate_workspace_bytes(void) { return sq::calibrate_workspace_bytes(); }

sq_status sq_calibrate_act_percentile(const sq_layer* layer, const void* x, sq_dtype x_dt, double p, float* amax,
                                      float* steps, void* workspace, size_t workspace_bytes, int accumulate,
                                      void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || amax == nullptr || steps == nullptr || workspace == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (!(p > 0.0 && p <= 1.0)) return SQ_ERR_INVALID_ARG;
  if (workspace_bytes < sq::calibrate_workspace_bytes() || reinterpret_cast<uintptr_t>(workspace) % 4 != 0)
    return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) tb.dual[s] = layer->dual[s] ? 1 : 0;
  hipError_t e = sq::launch_calibrate_act_percentile(x, x_dt == SQ_BF16, layer->M, layer->K, tb, p, amax, steps, workspace,
                                                     accumulate != 0, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_calibrate_act_percentile_static(const sq_layer* layer, const void* x, sq_dtype x_dt, double p, float* amax,
                                             float* steps, int accumulate, void* stream) {
  sq_status st = check_layer(layer, true, false);      // also the size limits of the static scratch: S <= SQ_MAX_SEGMENTS
  if (st != SQ_OK) return st;
  if (x == nullptr || amax == nullptr || steps == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (!(p > 0.0 && p <= 1.0)) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) tb.dual[s] = layer->dual[s] ? 1 : 0;
  hipError_t e = sq::launch_calibrate_act_percentile_static(x, x_dt == SQ_BF16, layer->M, layer->K, tb, p, amax, steps,
                                                            accumulate != 0, reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

size_t sq_calibrate_static_scratch_bytes(void) { return sq::calibrate_static_scratch_bytes(); }

static sq_status quantize_act_common(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, int8_t* xq,
                                     void* workspace, size_t workspace_bytes, void* stream, bool geglu = false) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (x == nullptr || xq == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) {
    tb.dual[s] = layer->dual[s] ? 1 : 0;
    tb.s_pos[s] = layer->s_pos[s];
    tb.inv_pos[s] = safe_inv(layer->s_pos[s]);
    tb.s_neg[s] = layer->dual[s] ? layer->s_neg[s] : 1.0f;
    tb.inv_neg[s] = layer->dual[s] ? safe_inv(layer->s_neg[s]) : 1.0f;
    tb.act[s] = SQ_ACT_NONE;
    if (act != nullptr) {
      if (act[s] != SQ_ACT_NONE && act[s] != SQ_ACT_SILU && act[s] != SQ_ACT_GELU) return SQ_ERR_INVALID_ARG;
      tb.act[s] = act[s];
    }
  }
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  hipError_t e;
  if (geglu) {
    e = sq::launch_quantize_act_geglu(x, x_dt == SQ_BF16, xq, layer->M, layer->K, tb, sq::device_cus(), hs);
  } else if (workspace != nullptr) {
    if (workspace_bytes < sq::quantize_act_fused_workspace_bytes(layer->S) || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
      return SQ_ERR_INVALID_ARG;
    if (sq::quantize_act_lut_usable(x, x_dt == SQ_BF16, xq, layer->K, tb))
      e = sq::launch_quantize_act_lut(x, xq, layer->M, layer->K, tb, workspace, sq::device_cus(), hs);
    else
      e = sq::launch_quantize_act(x, x_dt == SQ_BF16, xq, layer->M, layer->K, tb, hs);
  } else {
    e = sq::launch_quantize_act(x, x_dt == SQ_BF16, xq, layer->M, layer->K, tb, hs);
  }
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_quantize_act(const sq_layer* layer, const void* x, sq_dtype x_dt, int8_t* xq, void* stream) {
  return quantize_act_common(layer, x, x_dt, nullptr, xq, nullptr, 0, stream);
}

sq_status sq_calibrate_channel_amax(const sq_layer* layer, const void* x, sq_dtype x_dt, float* amax_k, int accumulate,
                                    void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || amax_k == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  hipError_t e = sq::launch_channel_amax(x, x_dt == SQ_BF16, layer->M, layer->K, amax_k, accumulate != 0,
                                         reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_weight_channel_amax(const sq_layer* layer, const void* w, sq_dtype w_dt, float* amax_k, void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || amax_k == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  hipError_t e = sq::launch_channel_amax(w, w_dt == SQ_BF16, layer->N, layer->K, amax_k, false,
                                         reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_smooth_factors(const sq_layer* layer, const float* amax_x, const float* amax_w, const float* alpha,
                            float* smooth, float* smooth_inv) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (amax_x == nullptr || amax_w == nullptr || alpha == nullptr || smooth == nullptr || smooth_inv == nullptr)
    return SQ_ERR_INVALID_ARG;
  for (int s = 0; s < layer->S; ++s)
    if (!(alpha[s] >= 0.0f && alpha[s] <= 1.0f)) return SQ_ERR_INVALID_ARG;
  for (int k = 0; k < layer->K; ++k)
    if (!(amax_x[k] >= 0.0f) || !(amax_w[k] >= 0.0f) || !std::isfinite(amax_x[k]) || !std::isfinite(amax_w[k]))
      return SQ_ERR_INVALID_ARG;
  sq::KsegTable tb;
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.off[s] = layer->kseg_off[s];
  sq::smooth_factors_host(amax_x, amax_w, layer->K, tb, alpha, smooth, smooth_inv);
  return SQ_OK;
}

sq_status sq_quantize_weight_smoothed(const sq_layer* layer, const void* w, sq_dtype w_dt, const float* smooth, int8_t* wq,
                                      float* wscale, void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || smooth == nullptr || wq == nullptr || wscale == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::KsegTable tb;
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.off[s] = layer->kseg_off[s];
  hipError_t e = sq::launch_quantize_weight_smoothed(w, w_dt == SQ_BF16, smooth, wq, wscale, layer->N, layer->K, tb,
                                                     reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_quantize_act_smoothed(const sq_layer* layer, const void* x, sq_dtype x_dt, const float* smooth_inv, int8_t* xq,
                                   void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (x == nullptr || smooth_inv == nullptr || xq == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) {
    tb.dual[s] = layer->dual[s] ? 1 : 0;
    tb.s_pos[s] = layer->s_pos[s];
    tb.inv_pos[s] = safe_inv(layer->s_pos[s]);
    tb.s_neg[s] = layer->dual[s] ? layer->s_neg[s] : 1.0f;
    tb.inv_neg[s] = layer->dual[s] ? safe_inv(layer->s_neg[s]) : 1.0f;
    tb.act[s] = SQ_ACT_NONE;
  }
  hipError_t e = sq::launch_quantize_act_smoothed(x, x_dt == SQ_BF16, smooth_inv, xq, layer->M, layer->K, tb,
                                                  reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

size_t sq_lowrank_workspace_bytes(const sq_layer* layer, int32_t rank) {
  if (check_layer(layer, true, false) != SQ_OK || (rank != 32 && rank != 64)) return 0;
  return sq::lowrank_workspace_bytes(layer->M, layer->K, rank, sq::device_cus());
}

sq_status sq_lowrank_add(const sq_layer* layer, const void* x, sq_dtype x_dt, const void* ld, const void* lu, int32_t rank,
                         const float* y_q, void* y, sq_dtype y_dt, void* workspace, size_t workspace_bytes, void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || ld == nullptr || lu == nullptr || y == nullptr || workspace == nullptr) return SQ_ERR_INVALID_ARG;
  if ((x_dt != SQ_F32 && x_dt != SQ_BF16) || (y_dt != SQ_F32 && y_dt != SQ_BF16)) return SQ_ERR_INVALID_ARG;
  if (rank != 32 && rank != 64) return SQ_ERR_UNSUPPORTED;
  if (layer->K % 16 != 0) return SQ_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(ld) | reinterpret_cast<uintptr_t>(lu) |
       reinterpret_cast<uintptr_t>(workspace)) % 16 != 0)
    return SQ_ERR_INVALID_ARG;
  if (workspace_bytes < sq::lowrank_workspace_bytes(layer->M, layer->K, rank, sq::device_cus())) return SQ_ERR_INVALID_ARG;
  hipError_t e = sq::launch_lowrank_add(x, x_dt == SQ_BF16, reinterpret_cast<const uint16_t*>(ld),
                                        reinterpret_cast<const uint16_t*>(lu), rank, y_q, y, y_dt == SQ_BF16, layer->M,
                                        layer->K, layer->N, reinterpret_cast<float*>(workspace), sq::device_cus(),
                                        reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_quantize_weight_fp8(const sq_layer* layer, const void* w, sq_dtype w_dt, uint8_t* wq, float* wscale, void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || wq == nullptr || wscale == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::KsegTable tb;
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.off[s] = layer->kseg_off[s];
  hipError_t e = sq::launch_quantize_weight_fp8(w, w_dt == SQ_BF16, wq, wscale, layer->N, layer->K, tb,
                                                reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

static sq_status quantize_act_fp8_common(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, uint8_t* xq,
                                         void* workspace, size_t workspace_bytes, void* stream);

sq_status sq_quantize_act_fp8(const sq_layer* layer, const void* x, sq_dtype x_dt, uint8_t* xq, void* stream) {
  return quantize_act_fp8_common(layer, x, x_dt, nullptr, xq, nullptr, 0, stream);
}

sq_status sq_quantize_act_fp8_fused(const sq_layer* layer, const void* h, sq_dtype h_dt, const int32_t* act, uint8_t* xq,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  if (act == nullptr) return SQ_ERR_INVALID_ARG;
  return quantize_act_fp8_common(layer, h, h_dt, act, xq, workspace, workspace_bytes, stream);
}

static sq_status quantize_act_fp8_common(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, uint8_t* xq,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (x == nullptr || xq == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) {
    tb.dual[s] = layer->dual[s] ? 1 : 0;
    tb.s_pos[s] = layer->s_pos[s];
    tb.s_neg[s] = layer->dual[s] ? layer->s_neg[s] : 1.0f;
    tb.inv_pos[s] = safe_inv(tb.s_pos[s]);
    tb.inv_neg[s] = safe_inv(tb.s_neg[s]);
    tb.act[s] = SQ_ACT_NONE;
    if (act != nullptr) {
      if (act[s] != SQ_ACT_NONE && act[s] != SQ_ACT_SILU && act[s] != SQ_ACT_GELU) return SQ_ERR_INVALID_ARG;
      tb.act[s] = act[s];
    }
  }
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  if (workspace != nullptr) {            // bf16 inputs by code table, as sq_quantize_act_fused
    if (workspace_bytes < sq::quantize_act_fused_workspace_bytes(layer->S) || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
      return SQ_ERR_INVALID_ARG;
    if (sq::quantize_act_lut_usable(x, x_dt == SQ_BF16, reinterpret_cast<const int8_t*>(xq), layer->K, tb)) {
      hipError_t el = sq::launch_quantize_act_lut(x, reinterpret_cast<int8_t*>(xq), layer->M, layer->K, tb, workspace,
                                                  sq::device_cus(), hs, true);
      return el == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
    }
  }
  hipError_t e = sq::launch_quantize_act_fp8(x, x_dt == SQ_BF16, xq, layer->M, layer->K, tb, hs);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_seglinear_fp8(const sq_layer* layer, const uint8_t* xq, const uint8_t* wq, const float* wscale, const float* bias,
                           void* y, sq_dtype y_dt, void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (xq == nullptr || wq == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if (y_dt != SQ_F32 && y_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  sq::GemmTable tb;
  fill_gemm_table(layer, tb);
  sq::GemmArgs a{};
  a.xq = reinterpret_cast<const int8_t*>(xq);
  a.wq = reinterpret_cast<const int8_t*>(wq);
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.M = layer->M;
  a.K = layer->K;
  a.N = layer->N;
  if (!sq::fp8_gemm_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  const sq::OutMode mode = y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  // up to two 16-row tiles of tokens: the weight-stream kernel; otherwise the pipelined tile kernel shared with the int8
  // path.  force_path 0: the plain tile kernel of fp8.hip, 1: the pipelined tile kernel, 3: the weight-stream kernel
  const bool stream_ok = sq::stream_supported(a, tb);
  if (g_force_path == 3 && !stream_ok) return SQ_ERR_UNSUPPORTED;
  hipError_t e;
  if (g_force_path == 0) {
    e = sq::launch_seglinear_fp8(a, tb, mode, hs);
  } else if (g_force_path == 3 || (g_force_path < 0 && a.M <= 32 && stream_ok)) {
    e = sq::launch_seglinear_stream_fp8(a, tb, mode, sq::device_cus(), hs);
  } else {
    const int v = g_gemm_variant >= 0 ? g_gemm_variant : sq::mfma_fp8_pick_variant(a, tb);
    e = sq::launch_seglinear_mfma_fp8(a, tb, mode, v, hs);
    if (e == hipErrorInvalidConfiguration) return SQ_ERR_UNSUPPORTED;
  }
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

size_t sq_quantize_act_fused_workspace_bytes(const sq_layer* layer) {
  if (layer == nullptr || layer->S < 1 || layer->S > SQ_MAX_SEGMENTS) return 0;
  return sq::quantize_act_fused_workspace_bytes(layer->S);
}

sq_status sq_quantize_act_fused(const sq_layer* layer, const void* h, sq_dtype h_dt, const int32_t* act, int8_t* xq,
                                void* workspace, size_t workspace_bytes, void* stream) {
  if (act == nullptr) return SQ_ERR_INVALID_ARG;
  return quantize_act_common(layer, h, h_dt, act, xq, workspace, workspace_bytes, stream);
}

sq_status sq_quantize_act_geglu(const sq_layer* layer, const void* h, sq_dtype h_dt, int8_t* xq, void* stream) {
  return quantize_act_common(layer, h, h_dt, nullptr, xq, nullptr, 0, stream, true);
}

sq_status sq_seglinear(const sq_layer* layer, const int8_t* xq, const int8_t* wq, const float* wscale,
                       const float* bias, void* y, sq_dtype y_dt, void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (xq == nullptr || wq == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if (y_dt != SQ_F32 && y_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  return run_gemm(layer, xq, wq, wscale, bias, y, nullptr, nullptr,
                  y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32, stream);
}

sq_status sq_seglinear_fused(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, const int8_t* wq,
                             const float* wscale, const float* bias, void* y, sq_dtype y_dt, void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (x == nullptr || wq == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if ((x_dt != SQ_F32 && x_dt != SQ_BF16) || (y_dt != SQ_F32 && y_dt != SQ_BF16)) return SQ_ERR_INVALID_ARG;
  sq::GemmTable tb;
  fill_gemm_table(layer, tb);
  for (int s = 0; s < layer->S; ++s) {
    tb.act[s] = SQ_ACT_NONE;
    if (act != nullptr) {
      if (act[s] != SQ_ACT_NONE && act[s] != SQ_ACT_SILU && act[s] != SQ_ACT_GELU) return SQ_ERR_INVALID_ARG;
      tb.act[s] = act[s];
    }
  }
  sq::GemmArgs a{};
  a.wq = wq;
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.M = layer->M;
  a.K = layer->K;
  a.N = layer->N;
  a.x_raw = x;
  a.x_raw_bf16 = x_dt == SQ_BF16 ? 1 : 0;
  if (reinterpret_cast<uintptr_t>(x) % 16 != 0 || !sq::stream_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  hipError_t e = sq::launch_seglinear_stream(a, tb, y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32, sq::device_cus(),
                                             reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

static sq_status grouped_common(const sq_layer* layer, const int8_t* xq, const void* x_raw, sq_dtype x_dt, const int32_t* act,
                                int32_t L, const sq_group_item* items, sq_dtype y_dt, void* stream, int w_bits = 8,
                                const float* tok_steps = nullptr, bool fp8 = false) {
  sq_status st = check_layer(layer, true, tok_steps == nullptr);
  if (st != SQ_OK) return st;
  if (w_bits != 8 && w_bits != 4) return SQ_ERR_INVALID_ARG;
  if (w_bits == 4 && !w4_layout_ok(layer)) return SQ_ERR_UNSUPPORTED;
  if (tok_steps != nullptr && layer->S > 8) return SQ_ERR_UNSUPPORTED;      // the kernel's step table holds 8 K-segments
  if ((xq == nullptr && x_raw == nullptr) || items == nullptr || L < 1) return SQ_ERR_INVALID_ARG;
  if (x_raw != nullptr && x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (y_dt != SQ_F32 && y_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (L > SQ_MAX_GROUP || layer->seg_scale != nullptr) return SQ_ERR_UNSUPPORTED;
  sq::GroupTable gt;
  std::memset(&gt, 0, sizeof(gt));
  gt.L = L;
  for (int l = 0; l < L; ++l) {
    if (items[l].wq == nullptr || items[l].wscale == nullptr || items[l].y == nullptr) return SQ_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(items[l].wq) % 16 != 0) return SQ_ERR_UNSUPPORTED;
    gt.item[l] = {items[l].wq, items[l].wscale, items[l].bias, items[l].y};
  }
  sq::GroupSegTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) {
    tb.dual[s] = layer->dual[s] ? 1 : 0;
    tb.s_pos[s] = tok_steps ? 1.0f : layer->s_pos[s];
    tb.s_neg[s] = layer->dual[s] ? (tok_steps ? 1.0f : layer->s_neg[s]) : 0.0f;
    tb.inv_pos[s] = safe_inv(tb.s_pos[s]);
    tb.inv_neg[s] = safe_inv(tb.s_neg[s]);
    tb.act[s] = SQ_ACT_NONE;
    if (act != nullptr) {
      if (act[s] != SQ_ACT_NONE && act[s] != SQ_ACT_SILU && act[s] != SQ_ACT_GELU) return SQ_ERR_INVALID_ARG;
      tb.act[s] = act[s];
    }
  }
  sq::GemmArgs a{};
  a.xq = xq;
  a.x_raw = x_raw;
  a.x_raw_bf16 = x_dt == SQ_BF16 ? 1 : 0;
  if (x_raw != nullptr && reinterpret_cast<uintptr_t>(x_raw) % 16 != 0) return SQ_ERR_UNSUPPORTED;
  a.M = layer->M;
  a.K = layer->K;
  a.N = layer->N;
  a.tok_steps = tok_steps;
  if (!sq::stream_grouped_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  const sq::OutMode mode = y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32;
  hipError_t e = fp8 ? sq::launch_seglinear_grouped_fp8(a, tb, gt, mode, sq::device_cus(), reinterpret_cast<hipStream_t>(stream))
                     : sq::launch_seglinear_grouped(a, tb, gt, mode, sq::device_cus(), reinterpret_cast<hipStream_t>(stream),
                                                    w_bits == 4);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_seglinear_grouped(const sq_layer* layer, const int8_t* xq, int32_t L, const sq_group_item* items,
                               sq_dtype y_dt, void* stream) {
  if (xq == nullptr) return SQ_ERR_INVALID_ARG;
  return grouped_common(layer, xq, nullptr, SQ_F32, nullptr, L, items, y_dt, stream);
}

sq_status sq_seglinear_grouped_fp8(const sq_layer* layer, const uint8_t* xq, int32_t L, const sq_group_item* items,
                                   sq_dtype y_dt, void* stream) {
  if (xq == nullptr) return SQ_ERR_INVALID_ARG;
  return grouped_common(layer, reinterpret_cast<const int8_t*>(xq), nullptr, SQ_F32, nullptr, L, items, y_dt, stream, 8, nullptr,
                        true);
}

sq_status sq_seglinear_grouped_w4(const sq_layer* layer, const int8_t* xq, const float* tok_steps, int32_t L,
                                  const sq_group_item* items, sq_dtype y_dt, void* stream) {
  if (xq == nullptr) return SQ_ERR_INVALID_ARG;
  return grouped_common(layer, xq, nullptr, SQ_F32, nullptr, L, items, y_dt, stream, 4, tok_steps);
}

sq_status sq_seglinear_grouped_fused(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, int32_t L,
                                     const sq_group_item* items, sq_dtype y_dt, void* stream) {
  if (x == nullptr) return SQ_ERR_INVALID_ARG;
  return grouped_common(layer, nullptr, x, x_dt, act, L, items, y_dt, stream);
}

sq_status sq_seglinear_debug_acc(const sq_layer* layer, const int8_t* xq, const int8_t* wq, int32_t* acc_pos,
                                 int32_t* acc_neg, void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (xq == nullptr || wq == nullptr || acc_pos == nullptr || acc_neg == nullptr) return SQ_ERR_INVALID_ARG;
  if ((long long)layer->S * layer->M * layer->N > 0x7FFFFFFFll) return SQ_ERR_UNSUPPORTED;
  return run_gemm(layer, xq, wq, nullptr, nullptr, nullptr, acc_pos, acc_neg, sq::OUT_DEBUG_ACC, stream);
}

sq_status sq_quantize_weight_w4(const sq_layer* layer, const void* w, sq_dtype w_dt, uint8_t* wq4, float* wscale,
                                void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (w == nullptr || wq4 == nullptr || wscale == nullptr) return SQ_ERR_INVALID_ARG;
  if (w_dt != SQ_F32 && w_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (!w4_layout_ok(layer)) return SQ_ERR_UNSUPPORTED;
  sq::KsegTable tb;
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.off[s] = layer->kseg_off[s];
  hipError_t e = sq::launch_quantize_weight_w4(w, w_dt == SQ_BF16, wq4, wscale, layer->N, layer->K, tb,
                                               reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_unpack_w4(const sq_layer* layer, const uint8_t* wq4, int8_t* wq, void* stream) {
  sq_status st = check_layer(layer, false, false);
  if (st != SQ_OK) return st;
  if (wq4 == nullptr || wq == nullptr) return SQ_ERR_INVALID_ARG;
  if (!w4_layout_ok(layer)) return SQ_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(wq4) | reinterpret_cast<uintptr_t>(wq)) % 16 != 0) return SQ_ERR_UNSUPPORTED;
  hipError_t e = sq::launch_unpack_w4(wq4, wq, layer->N, layer->K, sq::device_cus(), reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_seglinear_w4(const sq_layer* layer, const int8_t* xq, const uint8_t* wq4, const float* wscale,
                          const float* bias, void* y, sq_dtype y_dt, void* stream) {
  sq_status st = check_layer(layer, true, true);
  if (st != SQ_OK) return st;
  if (xq == nullptr || wq4 == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if (y_dt != SQ_F32 && y_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  return run_gemm_w4(layer, xq, wq4, wscale, bias, y, nullptr, nullptr, y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32,
                     stream);
}

sq_status sq_seglinear_w4_debug_acc(const sq_layer* layer, const int8_t* xq, const uint8_t* wq4, int32_t* acc_pos,
                                    int32_t* acc_neg, void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (xq == nullptr || wq4 == nullptr || acc_pos == nullptr || acc_neg == nullptr) return SQ_ERR_INVALID_ARG;
  if ((long long)layer->S * layer->M * layer->N > 0x7FFFFFFFll) return SQ_ERR_UNSUPPORTED;
  return run_gemm_w4(layer, xq, wq4, nullptr, nullptr, nullptr, acc_pos, acc_neg, sq::OUT_DEBUG_ACC, stream);
}

// Largest code of a_bits-wide symmetric activation codes (Sec. 3: q_max = 2^(b-1) - 1); 0 for widths not offered.
static float act_qmax(int32_t a_bits) { return a_bits == 8 ? 127.0f : a_bits == 4 ? 7.0f : 0.0f; }

sq_status sq_quantize_act_dynamic_bits(const sq_layer* layer, const void* x, sq_dtype x_dt, int32_t a_bits, int8_t* xq,
                                       float* tok_steps, void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || xq == nullptr || tok_steps == nullptr) return SQ_ERR_INVALID_ARG;
  if (x_dt != SQ_F32 && x_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (act_qmax(a_bits) == 0.0f) return SQ_ERR_INVALID_ARG;
  sq::ActTable tb;
  std::memset(&tb, 0, sizeof(tb));
  tb.S = layer->S;
  for (int s = 0; s <= layer->S; ++s) tb.kseg_off[s] = layer->kseg_off[s];
  for (int s = 0; s < layer->S; ++s) tb.dual[s] = layer->dual[s] ? 1 : 0;
  hipError_t e = sq::launch_quantize_act_dynamic(x, x_dt == SQ_BF16, xq, tok_steps, layer->M, layer->K, tb, act_qmax(a_bits),
                                                 reinterpret_cast<hipStream_t>(stream));
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

sq_status sq_quantize_act_dynamic(const sq_layer* layer, const void* x, sq_dtype x_dt, int8_t* xq, float* tok_steps,
                                  void* stream) {
  return sq_quantize_act_dynamic_bits(layer, x, x_dt, 8, xq, tok_steps, stream);
}

sq_status sq_seglinear_dynamic(const sq_layer* layer, const int8_t* xq, const float* tok_steps, const void* wq,
                               int32_t w_bits, const float* wscale, const float* bias, void* y, sq_dtype y_dt,
                               void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (xq == nullptr || tok_steps == nullptr || wq == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if (y_dt != SQ_F32 && y_dt != SQ_BF16) return SQ_ERR_INVALID_ARG;
  if (w_bits != 8 && w_bits != 4) return SQ_ERR_INVALID_ARG;
  return run_gemm_dynamic(layer, xq, tok_steps, wq, w_bits, wscale, bias, y, y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32,
                          stream);
}

sq_status sq_seglinear_fused_dynamic(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, int32_t a_bits,
                                     const void* wq, int32_t w_bits, const float* wscale, const float* bias, void* y,
                                     sq_dtype y_dt, void* stream) {
  sq_status st = check_layer(layer, true, false);
  if (st != SQ_OK) return st;
  if (x == nullptr || wq == nullptr || wscale == nullptr || y == nullptr) return SQ_ERR_INVALID_ARG;
  if ((x_dt != SQ_F32 && x_dt != SQ_BF16) || (y_dt != SQ_F32 && y_dt != SQ_BF16)) return SQ_ERR_INVALID_ARG;
  if ((w_bits != 8 && w_bits != 4) || act_qmax(a_bits) == 0.0f) return SQ_ERR_INVALID_ARG;
  if (w_bits == 4 && !w4_layout_ok(layer)) return SQ_ERR_UNSUPPORTED;
  sq::GemmTable tb;
  fill_gemm_table(layer, tb);
  for (int s = 0; s < layer->S; ++s) {
    tb.s_pos[s] = 1.0f;                                  // the kernel finds every row's steps itself
    tb.s_neg[s] = layer->dual[s] ? 1.0f : 0.0f;
    tb.act[s] = SQ_ACT_NONE;
    if (act != nullptr) {
      if (act[s] != SQ_ACT_NONE && act[s] != SQ_ACT_SILU && act[s] != SQ_ACT_GELU) return SQ_ERR_INVALID_ARG;
      tb.act[s] = act[s];
    }
  }
  sq::GemmArgs a{};
  a.wq = reinterpret_cast<const int8_t*>(wq);
  a.wscale = wscale;
  a.bias = bias;
  a.y = y;
  a.M = layer->M;
  a.K = layer->K;
  a.N = layer->N;
  a.x_raw = x;
  a.x_raw_bf16 = x_dt == SQ_BF16 ? 1 : 0;
  a.x_raw_dynamic = 1;
  a.act_qmax = act_qmax(a_bits);
  if (layer->S > 8 || reinterpret_cast<uintptr_t>(x) % 16 != 0 || !sq::stream_supported(a, tb)) return SQ_ERR_UNSUPPORTED;
  const sq::OutMode mode = y_dt == SQ_BF16 ? sq::OUT_BF16 : sq::OUT_F32;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = w_bits == 4 ? sq::launch_seglinear_stream_w4(a, tb, mode, sq::device_cus(), hs)
                             : sq::launch_seglinear_stream(a, tb, mode, sq::device_cus(), hs);
  return e == hipSuccess ? SQ_OK : SQ_ERR_LAUNCH;
}

const char* sq_status_string(sq_status s) {
  switch (s) {
    case SQ_OK: return "SQ_OK";
    case SQ_ERR_INVALID_ARG: return "SQ_ERR_INVALID_ARG";
    case SQ_ERR_UNSUPPORTED: return "SQ_ERR_UNSUPPORTED";
    case SQ_ERR_LAUNCH: return "SQ_ERR_LAUNCH";
    default: return "SQ_ERR_UNKNOWN";
  }
}

int sq_version(void) { return 400; }   // 0.4.0: smoothing, low-rank branch, fp8 variant, allocation-free calibration entry

sq_status sq_tuning_set(const char* key, int value) {
  if (key == nullptr) return SQ_ERR_INVALID_ARG;
  if (std::strcmp(key, "gemm_variant") == 0) {
    if (value < -1 || value >= sq::mfma_num_variants()) return SQ_ERR_INVALID_ARG;
    g_gemm_variant = value;
    return SQ_OK;
  }
  if (std::strcmp(key, "group_m") == 0) {
    if (value < 0 || value > 1024) return SQ_ERR_INVALID_ARG;
    sq::mfma_set_group_m(value);
    return SQ_OK;
  }
  if (std::strcmp(key, "force_path") == 0) {
    if (value < -1 || value > 3) return SQ_ERR_INVALID_ARG;
    g_force_path = value;
    return SQ_OK;
  }
  return SQ_ERR_INVALID_ARG;
}

}  // extern "C"
