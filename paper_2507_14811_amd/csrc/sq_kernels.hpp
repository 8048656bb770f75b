// Host-side launchers of the HIP kernels (one per source file).  Shapes are validated by the caller.
#pragma once
#include "sq_common.hpp"

namespace sq {

struct KsegTable {
  int S;
  int off[SQ_MAX_SEGMENTS + 1];
};

enum OutMode { OUT_F32 = 0, OUT_BF16 = 1, OUT_DEBUG_ACC = 2 };

// quantize.hip
hipError_t launch_quantize_act(const void* x, bool x_is_bf16, int8_t* xq, int M, int K, const ActTable& tb,
                               hipStream_t st);
// bf16 inputs of the fused activation + quantizer: per-K-segment code tables (S x 64 KiB of workspace), LDS lookups
size_t quantize_act_fused_workspace_bytes(int S);
bool quantize_act_lut_usable(const void* h, bool h_is_bf16, const int8_t* xq, int K, const ActTable& tb);
hipError_t launch_quantize_act_lut(const void* h, int8_t* xq, int M, int K, const ActTable& tb, void* workspace, int cus,
                                   hipStream_t st, bool fp8 = false);     // fp8: the tables (and xq) hold OCP E4M3 codes
hipError_t launch_quantize_weight(const void* w, bool w_is_bf16, int8_t* wq, float* wscale, int N, int K,
                                  const KsegTable& tb, hipStream_t st);

hipError_t launch_quantize_weight_block(const void* w, bool w_is_bf16, int8_t* wq, float* wscale, int N, int K,
                                        const KsegTable& kt, const KsegTable& nt, hipStream_t st);

// calibrate.hip : min/max activation steps per K-segment, running maxima over batches
hipError_t launch_calibrate_act(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, float* amax, float* steps,
                                bool accumulate, hipStream_t st);

// dynamic per-token activation steps: tok_steps [2][M][S]
hipError_t launch_unpack_w4(const uint8_t* wq4, int8_t* wq, int N, int K, int cus, hipStream_t st);
hipError_t launch_quantize_act_geglu(const void* h, bool h_is_bf16, int8_t* xq, int M, int K, const ActTable& tb, int cus,
                                     hipStream_t st);
hipError_t launch_quantize_act_dynamic(const void* x, bool x_is_bf16, int8_t* xq, float* tok_steps, int M, int K,
                                       const ActTable& tb, float qmax, hipStream_t st);

// 4-bit weights, packed two per byte (K and K-segment boundaries multiples of 128)
hipError_t launch_quantize_weight_w4(const void* w, bool w_is_bf16, uint8_t* wq4, float* wscale, int N, int K,
                                     const KsegTable& tb, hipStream_t st);
hipError_t launch_seglinear_generic_w4(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st);
hipError_t launch_seglinear_stream_w4(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st);

// percentile clipping instead of the maximum: exact nearest-rank quantile by radix select; workspace of
// calibrate_workspace_bytes() device bytes
size_t calibrate_workspace_bytes();
hipError_t launch_calibrate_act_percentile(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, double p,
                                           float* amax, float* steps, void* workspace, bool accumulate, hipStream_t st);

// the same with the select state in a file-scope device array of calibrate.hip (no workspace argument, no allocation)
size_t calibrate_static_scratch_bytes();
hipError_t launch_calibrate_act_percentile_static(const void* x, bool x_is_bf16, int M, int K, const ActTable& tb, double p,
                                                  float* amax, float* steps, bool accumulate, hipStream_t st);

// smooth.hip : SmoothQuant factors with one migration strength per K-segment (per-channel maxima, factors on the host,
// quantizers on the smoothed operands)
hipError_t launch_channel_amax(const void* a, bool is_bf16, int R, int K, float* amax, bool accumulate, hipStream_t st);
void smooth_factors_host(const float* amax_x, const float* amax_w, int K, const KsegTable& tb, const float* alpha,
                         float* smooth, float* smooth_inv);
hipError_t launch_quantize_weight_smoothed(const void* w, bool w_is_bf16, const float* smooth, int8_t* wq, float* wscale, int N,
                                           int K, const KsegTable& tb, hipStream_t st);
hipError_t launch_quantize_act_smoothed(const void* x, bool x_is_bf16, const float* rinv, int8_t* xq, int M, int K,
                                        const ActTable& tb, hipStream_t st);

// lowrank.hip : 16-bit low-rank side branch of the 4-bit settings, y = y_q + (X Ld^T) Lu^T (rank 32 or 64, K % 16 == 0)
size_t lowrank_workspace_bytes(int M, int K, int rank, int cus);
hipError_t launch_lowrank_add(const void* x, bool x_is_bf16, const uint16_t* ld, const uint16_t* lu, int rank, const float* y_in,
                              void* y_out, bool y_is_bf16, int M, int K, int N, float* workspace, int cus, hipStream_t st);

// fp8.hip : the 8-bit floating-point variant (OCP E4M3 codes, steps range / 448, fp8 matrix cores with fp32 accumulation).
// The GEMM needs K and every K-segment boundary % 128 == 0 and 16-byte aligned code matrices.
hipError_t launch_quantize_weight_fp8(const void* w, bool w_is_bf16, uint8_t* wq, float* wscale, int N, int K,
                                      const KsegTable& tb, hipStream_t st);
hipError_t launch_quantize_act_fp8(const void* x, bool x_is_bf16, uint8_t* xq, int M, int K, const ActTable& tb, hipStream_t st);
bool fp8_gemm_supported(const GemmArgs& a, const GemmTable& tb);
// seglinear_stream.hip built with -DSQ_STREAM_FP8=1: the weight-stream kernel on fp8 codes (shapes of stream_supported())
hipError_t launch_seglinear_stream_fp8(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st);
hipError_t launch_seglinear_grouped_fp8(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, OutMode mode, int cus,
                                        hipStream_t st);
hipError_t launch_seglinear_fp8(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st);

// seglinear_generic.hip : any shape / alignment, one thread per output element
hipError_t launch_seglinear_generic(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st);

// seglinear_mfma.hip : large-M int8 MFMA tile kernel.  Needs K % 64 == 0 and every K-segment boundary % 64 == 0.
int mfma_num_variants();
void mfma_set_group_m(int g);   // diagnostics: panel height of the tile order (0: default)
bool mfma_supported(const GemmArgs& a, const GemmTable& tb);
int mfma_pick_variant(const GemmArgs& a, const GemmTable& tb, OutMode mode);
hipError_t launch_seglinear_mfma(GemmArgs a, const GemmTable& tb, OutMode mode, int variant, hipStream_t st);
// the same tile kernel on fp8 (E4M3) codes: K and every K-segment boundary % 128 == 0, static steps
int mfma_fp8_pick_variant(const GemmArgs& a, const GemmTable& tb);
hipError_t launch_seglinear_mfma_fp8(GemmArgs a, const GemmTable& tb, OutMode mode, int variant, hipStream_t st);

// seglinear_skinny.hip : M <= 64, weight-streaming kernel.  Same alignment needs as the MFMA kernel.
bool skinny_supported(const GemmArgs& a, const GemmTable& tb);
hipError_t launch_seglinear_skinny(const GemmArgs& a, const GemmTable& tb, OutMode mode, hipStream_t st);

// seglinear_stream.hip : M <= 64 and a wide output: persistent weight stream.  K and K-segment boundaries % 128 == 0.
bool stream_supported(const GemmArgs& a, const GemmTable& tb);
hipError_t launch_seglinear_stream(const GemmArgs& a, const GemmTable& tb, OutMode mode, int cus, hipStream_t st);
bool stream_grouped_supported(const GemmArgs& a, const GroupSegTable& tb);
hipError_t launch_seglinear_grouped(const GemmArgs& a, const GroupSegTable& tb, const GroupTable& gt, OutMode mode, int cus,
                                    hipStream_t st, bool w4 = false);

// compute units of the current device (cached)
int device_cus();

}  // namespace sq
