/*
 * segquant.h - C ABI of the MI355X (gfx950) SegLinear + DualScale quantized linear layer
 * (SegQuant, arXiv 2507.14811).
 *
 * The quantized forward pass is the three-step composition of App. A,
 *     Y ~= DeQuant( Quant(X) . Quant(W) ),
 * with
 *   - SegLinear (Sec. 4.2.2): the weight is cut along its output dimension into N-segments
 *     (item 1, layers followed by chunk/split) and along its input dimension into K-segments
 *     (item 2, layers fed by concat/reshape); every segment has quantization steps of its own
 *     and the K-segment products are summed;
 *   - DualScale (Sec. 4.3.2): an activation that follows SiLU/GELU is split by polarity,
 *     X = X_+ + X_-, each part is quantized with its own step (s_+, s_-), both int8 products
 *     run against the same int8 weight and are recombined as
 *         s_+ s_w (X^_+ W^) + s_- s_w (X^_- W^).
 *
 * Conventions shared by all calls
 *   Memory     "dev" pointers are device (HBM) memory owned by the caller, dense row-major, base
 *              16-byte aligned.  Pointers inside sq_layer are HOST memory, read during the call
 *              only.  The library allocates nothing and keeps no per-call state.
 *   Layout     activations X[M][K] (K contiguous); weights W[N][K] (row = output channel, K
 *              contiguous: the transpose of the paper's k x n matrix); outputs Y[M][N].
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *              enqueued; no call synchronises with the host.
 *   Codes      X^_+ = Quant(max(X, 0)) >= 0 and X^_- = Quant(min(X, 0)) <= 0 are never both non-zero
 *              at one element, so the library stores and consumes them as ONE int8 matrix
 *              X^ = X^_+ + X^_- ("polarity-merged codes"): in a DualScale K-segment
 *              X^_+ = max(X^, 0) and X^_- = min(X^, 0); in a single-scale K-segment X^ is the
 *              symmetric code.  The kernels separate the two operands in registers, so the second
 *              polarity path costs no memory traffic.
 *   Numbers    round() is round-half-to-even, the code range is [-127, 127], x / s is an IEEE
 *              fp32 division; all steps ("scales") are fp32.
 *   Errors     every call returns an sq_status and never throws or aborts.  Host-side checks:
 *              NULL pointers, non-monotone offsets, off[S] != K, off[T] != N, steps that are not
 *              finite and > 0, unknown dtype  -> SQ_ERR_INVALID_ARG;  legal but outside the limits
 *              below -> SQ_ERR_UNSUPPORTED;  a failed launch -> SQ_ERR_LAUNCH.  Device data are
 *              not validated (finite inputs are a precondition).
 *   Limits     1 <= S, T <= SQ_MAX_SEGMENTS; seg_scale needs S*T <= SQ_MAX_SEG_SCALE; every
 *              K-segment is at most SQ_MAX_KSEG_LEN long so that 127*127*K_ks fits int32;
 *              M*K, N*K and M*N below 2^31.
 */
#ifndef SEGQUANT_H
#define SEGQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SQ_MAX_SEGMENTS 64
#define SQ_MAX_SEG_SCALE 512
#define SQ_MAX_KSEG_LEN 133143
#define SQ_MAX_GROUP 64

typedef enum { SQ_OK = 0, SQ_ERR_INVALID_ARG = 1, SQ_ERR_UNSUPPORTED = 2, SQ_ERR_LAUNCH = 3 } sq_status;
typedef enum { SQ_F32 = 0, SQ_BF16 = 1 } sq_dtype;

/*
 * One quantized linear layer: shapes, the segment tables produced by the graph analysis of
 * Sec. 4.2.2 (App. B, pattern detection), and the static activation steps of Sec. 4.3.2.
 * All pointers are HOST memory.
 */
typedef struct sq_layer {
  int32_t M, K, N;         /* tokens, in-features, out-features; all >= 1, M may be ragged        */
  int32_t S;               /* number of K-segments (input-segmented, Sec. 4.2.2 item 2)           */
  const int32_t* kseg_off; /* S+1 entries, 0 = off[0] < ... < off[S] = K                          */
  int32_t T;               /* number of N-segments (output-segmented, Sec. 4.2.2 item 1)          */
  const int32_t* nseg_off; /* T+1 entries, 0 = off[0] < ... < off[T] = N                          */
  const uint8_t* dual;     /* S entries: 1 = DualScale on this K-segment, 0 = one symmetric step  */
  const float* s_pos;      /* S entries: s_+ (or the single step of a non-dual segment)           */
  const float* s_neg;      /* S entries: s_- > 0 (|min x| / 127); ignored where dual[ks] == 0     */
  const float* seg_scale;  /* S*T entries [ks][ns], extra multiplier of block (ks, ns); or NULL   */
} sq_layer;

/*
 * Quant(W), Sec. 3 quantizer with z = 0 applied per segment (Sec. 4.2.2): for every output channel
 * n and K-segment ks:  a = max_k |W[n][k]|,  wscale[ks][n] = a / 127 (1.0 if a == 0),
 * wq[n][k] = clip(round(W[n][k] / wscale[ks][n]), -127, 127).
 *   w      dev, [N][K] of w_dt (SQ_F32 or SQ_BF16)        in
 *   wq     dev, int8 [N][K]                               out
 *   wscale dev, fp32 [S][N]                               out
 * Offline step (once per layer).  M of the layer is ignored.
 */
sq_status sq_quantize_weight(const sq_layer* layer, const void* w, sq_dtype w_dt, int8_t* wq,
                             float* wscale, void* stream);

/*
 * Quant(W) at the granularity the paper uses for 8 bit (App. B, quantization granularity: per tensor, i.e. one
 * step per weight segment under SegLinear): one step per (K-segment, N-segment) block,
 *   a = max |W[n][k]| over the block,  step = a / 127 (1.0 if a == 0),
 * written to wscale[ks][n] of every channel n of the block, so sq_seglinear consumes it unchanged.
 * Arguments as sq_quantize_weight; layer->nseg_off selects the blocks.  wscale is also the scratch of the call.
 */
sq_status sq_quantize_weight_block(const sq_layer* layer, const void* w, sq_dtype w_dt, int8_t* wq,
                                   float* wscale, void* stream);

/*
 * Calibration of the static activation steps (Sec. 4.3.2: s_- = |min x| / q, s_+ = max x / q; App. B sensitivity
 * study: the strict min/max rule, p = 1.0), one pair per K-segment, with running maxima over batches:
 *   dual segment   amax_pos = max(0, max x), amax_neg = max(0, -min x);   single-scale: amax_pos = max |x|
 *   steps[ks] = amax_pos[ks] / 127,  steps[S + ks] = amax_neg[ks] / 127,  1.0 where the maximum is 0.
 *   x      dev, [M][K] of x_dt (one calibration batch)           in
 *   amax   dev, fp32 [2][S] running maxima (pos, then neg)       in/out; ignored on input when accumulate == 0
 *   steps  dev, fp32 [2][S] (s_pos, then s_neg)                  out; copy to the host to fill sq_layer
 * layer->s_pos / s_neg are not read.
 */
sq_status sq_calibrate_act(const sq_layer* layer, const void* x, sq_dtype x_dt, float* amax, float* steps,
                           int accumulate, void* stream);

/*
 * The same calibration with percentile clipping (App. B, dual-scale sensitivity study: p <= 0.9999 against the
 * min/max rule p = 1.0).  The paper names the percentile only; the rule implemented: per K-segment and polarity
 * the clipping threshold of a batch is the nearest-rank p-quantile of the tensor the quantizer sees,
 *   dual segment  V_+ = max(x, 0), V_- = max(-x, 0)  (zeros included);   single-scale: V_+ = |x|,
 * i.e. the k-th smallest of its n = M * K_ks values, k = ceil(p * n) in IEEE double, clamped to [1, n];
 * thresholds combine over batches as running maxima, steps = threshold / 127 (1.0 where it is 0).  p = 1.0 gives
 * sq_calibrate_act.  The order statistic is exact (radix select on the fp32 bit patterns); inputs must be finite.
 *   p          host, 0 < p <= 1
 *   workspace  dev, at least sq_calibrate_workspace_bytes() bytes, 4-byte aligned, contents irrelevant on entry;
 *              owned by the caller, used only during the call (calls that share it must not overlap)
 *   others as sq_calibrate_act.
 * SQ_ERR_INVALID_ARG for p outside (0, 1], a missing or short workspace.
 */
size_t sq_calibrate_workspace_bytes(void);
sq_status sq_calibrate_act_percentile(const sq_layer* layer, const void* x, sq_dtype x_dt, double p, float* amax,
                                      float* steps, void* workspace, size_t workspace_bytes, int accumulate,
                                      void* stream);

/*
 * sq_calibrate_act_percentile for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same results to the bit.  The radix-select state (sq_calibrate_static_scratch_bytes() = 132 608 bytes, enough
 * for the library's maximum of 64 K-segments) lives in a static device array inside the library; every GPU the
 * library runs on holds its own copy until the process ends.  The call allocates and frees nothing (its first
 * call on a device looks the array's address up, which allocates nothing either).  Limits: those of the
 * library, S <= 64 K-segments and M * K < 2^31; beyond them SQ_ERR_UNSUPPORTED, nothing is launched.
 * All calls on one GPU share the array (it keeps the last call's contents; every call re-initialises what it
 * reads): calls that overlap on one GPU — different streams or host threads — race, so serialise them.
 */
size_t sq_calibrate_static_scratch_bytes(void);
sq_status sq_calibrate_act_percentile_static(const sq_layer* layer, const void* x, sq_dtype x_dt, double p, float* amax,
                                             float* steps, int accumulate, void* stream);

/*
 * Smoothing in front of the quantizers with one migration strength per K-segment (Sec. 4.2.2, last paragraph: SegLinear
 * shares SmoothQuant's alpha across a semantically coherent channel group; App. B: SmoothQuant is the optimizer of the
 * 8-bit settings, alpha chosen per layer from 0.0 .. 1.0).  The published rule per input channel k of K-segment ks:
 *   a_x[k] = max_m |X[m][k]| over the calibration batches,   a_w[k] = max_n |W[n][k]|,
 *   s[k] = a_x[k]^alpha[ks] / a_w[k]^(1 - alpha[ks]),   X' = X diag(s)^-1,   W' = W diag(s)   (X' W'^T = X W^T),
 * and X', W' go through the ordinary quantizers (activation steps are calibrated on X').
 *   sq_calibrate_channel_amax   x dev [M][K] -> amax_k dev fp32 [K]; accumulate != 0 folds into the running maxima
 *   sq_weight_channel_amax      w dev [N][K] -> amax_k dev fp32 [K]
 *   sq_smooth_factors           HOST computation on HOST arrays (K numbers; the caller sweeps alpha): amax_x, amax_w
 *                               fp32 [K] in, alpha fp32 [S] in (0 <= alpha <= 1), smooth, smooth_inv fp32 [K] out.
 *                               Powers in double, rounded once to fp32; a channel with a_x = 0 or a_w = 0, or whose
 *                               factor or reciprocal is not a finite positive fp32 number, keeps s = 1;
 *                               smooth_inv[k] = 1 / smooth[k] (one fp32 division).  Launches nothing.
 *   sq_quantize_weight_smoothed sq_quantize_weight of W diag(s): every weight is multiplied by smooth[k] (dev fp32 [K],
 *                               one fp32 multiplication) before the maxima and the codes
 *   sq_quantize_act_smoothed    sq_quantize_act of X diag(smooth_inv): every activation is multiplied by smooth_inv[k]
 *                               (dev fp32 [K], one fp32 multiplication: the form in which the factor is folded into the
 *                               operator in front of the layer) before Q_dual; layer->s_pos / s_neg are steps of X'
 * sq_seglinear is unchanged: it sees the codes and steps of the smoothed operands.
 */
sq_status sq_calibrate_channel_amax(const sq_layer* layer, const void* x, sq_dtype x_dt, float* amax_k, int accumulate,
                                    void* stream);
sq_status sq_weight_channel_amax(const sq_layer* layer, const void* w, sq_dtype w_dt, float* amax_k, void* stream);
sq_status sq_smooth_factors(const sq_layer* layer, const float* amax_x, const float* amax_w, const float* alpha,
                            float* smooth, float* smooth_inv);
sq_status sq_quantize_weight_smoothed(const sq_layer* layer, const void* w, sq_dtype w_dt, const float* smooth, int8_t* wq,
                                      float* wscale, void* stream);
sq_status sq_quantize_act_smoothed(const sq_layer* layer, const void* x, sq_dtype x_dt, const float* smooth_inv, int8_t* xq,
                                   void* stream);

/*
 * Q_dual(X) with the polarity split fused in (Sec. 4.3.2).  For a dual K-segment:
 *   x <  0 : X^_- = max(round(x / s_neg[ks]), -127), X^_+ = 0     -> xq = X^_-  (<= 0)
 *   x >= 0 : X^_+ = min(round(x / s_pos[ks]),  127), X^_- = 0     -> xq = X^_+  (>= 0)
 * For a non-dual K-segment (Sec. 3, z = 0): xq = clip(round(x / s_pos[ks]), -127, 127).
 *   x       dev, [M][K] of x_dt                           in
 *   xq      dev, int8 [M][K], polarity-merged codes       out
 * The two matrices of Sec. 4.3.2 never overlap (X^_+ >= 0 where x >= 0, X^_- <= 0 where x < 0), so they leave as one:
 * the supported decoding is X^_+ = max(xq, 0), X^_- = min(xq, 0) in a dual K-segment, X^_+ = xq elsewhere.
 */
sq_status sq_quantize_act(const sq_layer* layer, const void* x, sq_dtype x_dt, int8_t* xq,
                          void* stream);

/*
 * sq_quantize_act with the polarity-asymmetric activation fused in front of it (Sec. 4.3.1: the layer's input comes
 * from SiLU / GELU; Sec. 4.3.2): xq = Q_dual(act(h)), one pass over the pre-activation instead of an activation
 * pass that writes what the quantizer then reads.  One activation code per K-segment (a concatenated input may
 * carry an activation on one part only).  The codes are integers decided by floating point, so the activation is
 * specified to the bit, in fp32, every operation individually rounded:
 *   exp32(t) = +inf for t > 88;  t <- max(t, -87);  n = round_half_even(t * 1.44269504);
 *              r = fma(n, -0.693145751953125, t);  r = fma(n, -1.42860682e-6, r);
 *              p = 1/5040;  p = fma(p, r, c) for c = 1/720, 1/120, 1/24, 1/6, 1/2, 1, 1;  exp32 = p * 2^n
 *   SQ_ACT_SILU  x / (1 + exp32(-x))
 *   SQ_ACT_GELU  x / (1 + exp32(-z)),  z = (1.59576912 * x) * fma(0.044715, x * x, 1)      (the tanh form)
 * The activation's fp32 value is quantized as it is (no rounding to bf16 in between).
 *   h    dev, [M][K] of h_dt (pre-activation)                in
 *   act  host, int32 [S], SQ_ACT_* per K-segment             in
 *   xq   dev, int8 [M][K], polarity-merged codes             out
 *   workspace  dev or NULL.  With a workspace of at least sq_quantize_act_fused_workspace_bytes(layer) bytes
 *        (16-byte aligned, contents irrelevant on entry, owned by the caller, used only during the call; calls
 *        that share it must not overlap) a bf16 input with 16-aligned K-segments is served by table: the
 *        65536-entry map  bf16 pattern -> code  of every K-segment is filled first with the arithmetic above and
 *        the pass becomes one table read per element (same codes, HBM-bound instead of ALU-bound).  NULL, fp32
 *        input or unaligned segments: the arithmetic runs per element.
 * SQ_ERR_INVALID_ARG for an unknown activation code or a workspace that is too small or misaligned; otherwise as
 * sq_quantize_act.
 */
#define SQ_ACT_NONE 0
#define SQ_ACT_SILU 1
#define SQ_ACT_GELU 2
size_t sq_quantize_act_fused_workspace_bytes(const sq_layer* layer);
sq_status sq_quantize_act_fused(const sq_layer* layer, const void* h, sq_dtype h_dt, const int32_t* act, int8_t* xq,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * GEGLU in front of the quantizer (App. B names GEGLU with SiLU and GELU as the polarity-sensitive activations):
 * the producing projection's output h holds [value | gate] side by side in every row, and
 *   xq[m][k] = Q_dual( value[m][k] * GELU(gate[m][k]) ),   value = h[m][k], gate = h[m][K + k],
 * with the GELU of sq_quantize_act_fused (same fp32 operation sequence), the product one fp32 multiplication
 * (round to nearest even), and the quantizers of sq_quantize_act.  layer->K and the K-segments are those of the
 * OUTPUT (the consuming layer's input features).
 *   h    dev [M][2K] of h_dt (fp32 / bf16)      in
 *   xq   dev int8 [M][K]                        out
 */
sq_status sq_quantize_act_geglu(const sq_layer* layer, const void* h, sq_dtype h_dt, int8_t* xq, void* stream);

/*
 * Dual-path integer GEMM with per-K-segment accumulators and the fused dequant epilogue
 * (Sec. 4.2.2 items 1-2 combined with the last display of Sec. 4.3.2):
 *   acc_+[ks][m][n] = sum_{k in ks} X^_+[m][k] wq[n][k]              (int32, exact)
 *   acc_-[ks][m][n] = sum_{k in ks} X^_-[m][k] wq[n][k]              (dual segments only)
 * with X^_+ = max(xq, 0), X^_- = min(xq, 0) in dual segments and X^_+ = xq elsewhere,
 *   y[m][n] = sum_ks seg_scale[ks][ns(n)] wscale[ks][n] ( s_pos[ks] acc_+ + s_neg[ks] acc_- ) + bias[n]
 * evaluated in fp32 and stored as fp32 or bf16 (round-half-to-even).  Activation and weight tiles
 * are read once and feed both accumulator sets.  Kernel selection: M <= 32 with K and the K-segment boundaries
 * multiples of 128 runs the weight-streaming (bandwidth-bound) kernel; M = 33..64 the MFMA tile kernel with 64-row
 * tiles (K and the boundaries multiples of 64), else the K-splitting skinny kernel; larger M the MFMA tile kernel;
 * shapes none of them takes (unaligned K or boundaries) a plain one-thread-per-output kernel.
 *   xq dev int8 [M][K] (from sq_quantize_act);  wq dev int8 [N][K];  wscale dev fp32 [S][N];
 *   bias dev fp32 [N] or NULL;  y dev [M][N] of y_dt.
 */
sq_status sq_seglinear(const sq_layer* layer, const int8_t* xq, const int8_t* wq,
                       const float* wscale, const float* bias, void* y, sq_dtype y_dt,
                       void* stream);

/*
 * Grouped skinny call: L linear layers of ONE shape (layer->M <= 32 tokens, K, N) that consume the SAME quantized
 * input, e.g. the modulation (adaLN) linears of all blocks of a diffusion transformer, which share the SiLU of the
 * conditioning vector (output-segmented, polarity-asymmetric layers of Sec. 4.2.2 item 1 / Sec. 4.3.2).  One
 * launch streams all L weight matrices; per layer the arithmetic is exactly that of sq_seglinear.
 *   layer   shape, K-segments, dual flags and activation steps shared by the L layers; seg_scale must be NULL
 *   xq      dev int8 [M][K], from sq_quantize_act
 *   items   HOST array of L entries {wq dev int8 [N][K], wscale dev fp32 [S][N], bias dev fp32 [N] or NULL,
 *           y dev [M][N] of y_dt}; read during the call only; wq 16-byte aligned
 * Returns SQ_ERR_UNSUPPORTED when M > 32, L > SQ_MAX_GROUP, K or a K-segment boundary is not a multiple of 128,
 * seg_scale is given, or M*K exceeds the on-chip budget (call sq_seglinear per layer instead).
 */
typedef struct sq_group_item {
  const int8_t* wq;
  const float* wscale;
  const float* bias;
  void* y;
} sq_group_item;

sq_status sq_seglinear_grouped(const sq_layer* layer, const int8_t* xq, int32_t L, const sq_group_item* items,
                               sq_dtype y_dt, void* stream);

/*
 * Skinny layers fed with raw activations: y = SegLinear(Q_dual(act(x))) in ONE launch.  The weight-stream kernel
 * computes the activation in front of the layer (App. B: SiLU / GELU), the polarity split and both quantizers of
 * Sec. 4.3.2 while it fills its on-chip copy of the input, so the code tensor X^ never exists in device memory and
 * the separate quantize launch goes away.  Element by element the codes are those of sq_quantize_act_fused (the same
 * fp32 operation sequence), hence y equals sq_seglinear(sq_quantize_act_fused(x)) bit for bit.
 *   x     dev [M][K] of x_dt (fp32 / bf16), 16-byte aligned      in
 *   act   host, int32 [S], SQ_ACT_* per K-segment, or NULL (no activation)   in
 *   wq, wscale, bias, y   as for sq_seglinear
 * sq_seglinear_grouped_fused is the same for L layers that share x (items as for sq_seglinear_grouped).
 * Returns SQ_ERR_UNSUPPORTED where the weight-stream kernel does not apply (M > 64, or M > 32 for the grouped call, K
 * or a K-segment boundary not a multiple of 128, misaligned pointers, M*K beyond the on-chip budget): run
 * sq_quantize_act_fused + sq_seglinear instead.
 */
sq_status sq_seglinear_fused(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, const int8_t* wq,
                             const float* wscale, const float* bias, void* y, sq_dtype y_dt, void* stream);
sq_status sq_seglinear_grouped_fused(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, int32_t L,
                                     const sq_group_item* items, sq_dtype y_dt, void* stream);

/*
 * The grouped call of the 4-bit settings (App. B): the items' wq point to the packed 4-bit codes of sq_quantize_weight_w4
 * (cast to const int8_t*), wscale are its per-channel scales.  tok_steps: NULL for the layer's static activation steps,
 * or the fp32 [2][M][S] per-token steps of sq_quantize_act_dynamic(_bits) that produced xq (then layer->s_pos / s_neg are
 * not read, and at most 8 K-segments).  Per layer the arithmetic is that of sq_seglinear_w4 / sq_seglinear_dynamic.
 * Limits as for sq_seglinear_grouped.
 */
sq_status sq_seglinear_grouped_w4(const sq_layer* layer, const int8_t* xq, const float* tok_steps, int32_t L,
                                  const sq_group_item* items, sq_dtype y_dt, void* stream);

/*
 * The same with dynamic per-token activation steps (App. B, 4-bit settings: per-channel 4-bit weights, activations
 * quantized dynamically per token): one launch computes act(x), every token row's steps per K-segment by the min/max rule
 * (as sq_quantize_act_dynamic_bits with the same a_bits, 8 or 4), the codes, and the GEMM with 8-bit (w_bits == 8, wq int8 [N][K]) or packed 4-bit weights
 * (w_bits == 4, wq from sq_quantize_weight_w4).  y equals sq_seglinear_dynamic(sq_quantize_act_dynamic(act(x))) bit for
 * bit.  layer->s_pos / s_neg are not read.  Returns SQ_ERR_UNSUPPORTED where the weight-stream kernel does not apply or
 * the layer has more than 8 K-segments; SQ_ERR_INVALID_ARG for a_bits or w_bits other than 4 or 8.
 */
sq_status sq_seglinear_fused_dynamic(const sq_layer* layer, const void* x, sq_dtype x_dt, const int32_t* act, int32_t a_bits,
                                     const void* wq, int32_t w_bits, const float* wscale, const float* bias, void* y,
                                     sq_dtype y_dt, void* stream);

/*
 * Parity instrument: runs the same main loop as sq_seglinear (same kernel selection) and stores the
 * raw int32 accumulators instead of the dequantized output.
 *   acc_pos, acc_neg  dev int32 [S][M][N];  acc_neg[ks] of a non-dual segment is written as 0.
 */
sq_status sq_seglinear_debug_acc(const sq_layer* layer, const int8_t* xq, const int8_t* wq,
                                 int32_t* acc_pos, int32_t* acc_neg, void* stream);

/*
 * 4-bit weights for the skinny layers (App. B, granularity of the 4-bit settings: weights per output channel; the
 * low-rank side branch of the optimizer used there is not part of this library).  The modulation-type layers are one
 * pass over the weights, so halving the weight bytes nearly halves their time.
 *
 * sq_quantize_weight_w4: the Sec. 3 quantizer with q_max = 7 per output channel n and K-segment ks,
 *   a = max_k |W[n][k]|,  wscale[ks][n] = a / 7 (1.0 if a == 0),  code = clip(round(W[n][k] / wscale[ks][n]), -7, 7),
 * codes packed two per byte in the order the weight stream consumes them: rows in groups of 16 (the last group
 * padded with zero rows), K in steps of 128 codes (T = K / 128), one contiguous KiB per (group g, step t):
 *   wq4[((g T + t) 16 + r) 64 + j] = code(16 g + r, 128 t + j)  |  code(16 g + r, 128 t + 64 + j) << 4,
 * 0 <= r < 16, 0 <= j < 64, each code a 4-bit two's-complement number.
 *   w      dev, [N][K] of w_dt                                in
 *   wq4    dev, uint8 [ceil(N / 16) * 16 * K / 2]            out
 *   wscale dev, fp32 [S][N]           out
 * sq_seglinear_w4 / sq_seglinear_w4_debug_acc: as sq_seglinear / sq_seglinear_debug_acc with wq4 in place of wq
 * (activations stay 8-bit polarity-merged codes from sq_quantize_act; the debug sums are those of the 4-bit codes).
 * K and every K-segment boundary must be multiples of 128 (SQ_ERR_UNSUPPORTED otherwise).  M <= 64 with a 16-byte
 * aligned wq4 runs the weight-stream kernel; other shapes run a plain one-thread-per-output kernel.
 */
sq_status sq_quantize_weight_w4(const sq_layer* layer, const void* w, sq_dtype w_dt, uint8_t* wq4, float* wscale,
                                void* stream);
sq_status sq_seglinear_w4(const sq_layer* layer, const int8_t* xq, const uint8_t* wq4, const float* wscale,
                          const float* bias, void* y, sq_dtype y_dt, void* stream);
/*
 * Packed 4-bit weight codes back to int8, one code per byte, [N][K] row-major: the operand of sq_seglinear /
 * sq_seglinear_dynamic (w_bits == 8) with the SAME wscale.  For layers with many token rows, where the GEMM is bound by
 * the matrix units and the 4-bit format saves memory, not time: keep the packed codes resident and unpack a layer into a
 * reusable buffer right before its GEMM.  The result of the GEMM is that of sq_seglinear_w4.
 *   wq4  dev uint8, packed codes of sq_quantize_weight_w4, 16-byte aligned     in
 *   wq   dev int8 [N][K], 16-byte aligned                                      out
 * SQ_ERR_UNSUPPORTED for layouts sq_quantize_weight_w4 does not take or misaligned pointers.
 */
sq_status sq_unpack_w4(const sq_layer* layer, const uint8_t* wq4, int8_t* wq, void* stream);
sq_status sq_seglinear_w4_debug_acc(const sq_layer* layer, const int8_t* xq, const uint8_t* wq4, int32_t* acc_pos,
                                    int32_t* acc_neg, void* stream);

/*
 * Dynamic per-token activation steps (App. B, granularity of the 4-bit settings: activations are quantized dynamically
 * per token).  Every token row m is calibrated on its own with the min/max rule of Sec. 4.3.2, per K-segment ks:
 *   dual          s_pos[m][ks] = max(0, max_k x) / 127,  s_neg[m][ks] = max(0, -min_k x) / 127
 *   single-scale  s_pos[m][ks] = max_k |x| / 127,        s_neg[m][ks] = 1
 * (1.0 where the extreme is 0), quantized with these steps as in sq_quantize_act, and dequantized with them:
 *   y[m][n] = sum_ks seg_scale * wscale[ks][n] * (s_pos[m][ks] acc_pos + s_neg[m][ks] acc_neg) + bias[n].
 * layer->s_pos / s_neg are not read.
 *   x          dev, [M][K] of x_dt                                  in
 *   xq         dev, int8 [M][K], polarity-merged codes              out (sq_quantize_act_dynamic) / in
 *   tok_steps  dev, fp32 [2][M][S]: s_pos, then s_neg               out (sq_quantize_act_dynamic) / in
 *   wq         dev, int8 [N][K] (w_bits == 8) or the packed 4-bit codes of sq_quantize_weight_w4 (w_bits == 4)
 *   others as sq_seglinear.
 * M <= 64 with at most 8 K-segments (and the alignment the weight stream needs) runs the weight-stream kernel; larger
 * M with 8-bit weights runs the MFMA tile kernel (K and the K-segment boundaries multiples of 64), whose flushes read
 * the steps of their token rows; every other shape (4-bit weights at large M included) runs a plain
 * one-thread-per-output kernel.  SQ_ERR_INVALID_ARG for w_bits other than 4 or 8.
 */
sq_status sq_quantize_act_dynamic(const sq_layer* layer, const void* x, sq_dtype x_dt, int8_t* xq, float* tok_steps,
                                  void* stream);
/* The same with a_bits-wide activation codes (Sec. 3: q_max = 2^(a_bits-1) - 1): a_bits == 8 is sq_quantize_act_dynamic,
 * a_bits == 4 gives the 4-bit activations of the paper's W4A4 setting (steps = row extreme / 7, codes in [-7, 7], still
 * one code per byte: the matrix units of this device have no 4-bit integer operands, so the codes run through the int8
 * kernels unchanged and sq_seglinear_dynamic needs no a_bits of its own).  SQ_ERR_INVALID_ARG for other widths. */
sq_status sq_quantize_act_dynamic_bits(const sq_layer* layer, const void* x, sq_dtype x_dt, int32_t a_bits, int8_t* xq,
                                       float* tok_steps, void* stream);
sq_status sq_seglinear_dynamic(const sq_layer* layer, const int8_t* xq, const float* tok_steps, const void* wq,
                               int32_t w_bits, const float* wscale, const float* bias, void* y, sq_dtype y_dt,
                               void* stream);

/*
 * Low-rank side branch of the 4-bit settings (main results, W4A8 rows; App. B: SVDQuant is the optimizer of the 4-bit
 * settings, the rank is fixed at 64).  The published decomposition keeps W = Lu Ld + R: the residual R is quantized
 * (sq_quantize_weight_w4) and runs through sq_seglinear_w4 / sq_seglinear_dynamic, the rank-r part runs in 16 bit on the
 * unquantized activations and is added to the quantized product before the output is rounded:
 *   y[m][n] = y_q[m][n] + sum_j T[m][j] Lu[n][j],     T[m][j] = sum_k X[m][k] Ld[j][k].
 * Arithmetic: X, Ld, Lu are bf16 (fp32 X is rounded to bf16 on entry: the branch is a 16-bit one); T is accumulated
 * and kept in fp32 (bf16 matrix cores, K cut into slices whose partial sums are added in ascending order); for the second
 * product every fp32 T value is split exactly into three bf16 terms (their sum carries its 24-bit mantissa), which run
 * through the bf16 matrix cores with fp32 accumulation, so T is not rounded to 16 bit; then the addition and one rounding
 * to y_dt.  Deterministic.
 *   x     dev [M][K] of x_dt                      ld  dev bf16 [rank][K]            lu  dev bf16 [N][rank]
 *   y_q   dev fp32 [M][N] (the quantized layer's fp32 output) or NULL (= 0)          y   dev [M][N] of y_dt (may be y_q)
 *   rank  32 or 64;  K a multiple of 16 (SQ_ERR_UNSUPPORTED otherwise);  x, ld, lu, workspace 16-byte aligned
 *   workspace  dev, sq_lowrank_workspace_bytes(layer, rank) bytes, contents irrelevant, used only during the call
 */
size_t sq_lowrank_workspace_bytes(const sq_layer* layer, int32_t rank);
sq_status sq_lowrank_add(const sq_layer* layer, const void* x, sq_dtype x_dt, const void* ld, const void* lu, int32_t rank,
                         const float* y_q, void* y, sq_dtype y_dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The 8-bit floating-point variant of the layer (main results, the 8-bit fp rows: weights and activations as fp8 in place
 * of int8).  Codes are bytes in the published OCP 8-bit format E4M3 (1 sign bit, 4 exponent bits with bias 7, 3 mantissa
 * bits, subnormals, no infinities, 0x7F / 0xFF = NaN and never produced, largest finite value 448):
 *   code(v, s) = e4m3(clip(v / s, -448, 448)), nearest value, ties to the even mantissa, the quotient an IEEE fp32 division;
 *   a result of zero is stored as +0 (0x00).
 * The quantizers of Sec. 3 and Sec. 4.3.2 are otherwise unchanged: weight steps are max|w| / 448 per output channel and
 * K-segment (1 where that maximum is 0), written to wscale [S][N]; the activation steps are the layer's s_pos / s_neg
 * (calibrated ranges / 448: the caller divides the amax that sq_calibrate_act* return).  Q_dual splits by the sign of x,
 * so the two polarity matrices travel as one byte matrix: X^_+ = codes with a clear sign bit, X^_- = codes with the sign
 * bit set (the other positions +0).
 *   y[m][n] = sum_ks wscale[ks][n] g(ks, n) (s_pos[ks] X^_+ W^T + s_neg[ks] X^_- W^T)[m][n] + bias[n]
 * with the products of the decoded codes summed on the fp8 matrix cores within a K-segment, fp32 accumulators.  The sum
 * is the hardware's: the eight products of an aligned group of eight k are added after alignment to the group's largest
 * exponent sum E, bits below 2^(E-13) dropped (a product 2^14 below the largest of its group vanishes), the groups and
 * instructions are then added in fp32.  Results are reproducible on this device and lie within
 * (2^-10 + (8 sqrt(K) + 64) 2^-24) of the sum of the terms' magnitudes of the exact value; on layer-like data the error
 * is a few 1e-5 of the largest output.  K, every K-segment boundary: multiples of 128, xq / wq 16-byte aligned
 * (SQ_ERR_UNSUPPORTED otherwise; the quantizers take any shape).  The product runs on the kernels of sq_seglinear with
 * fp8 operands: the weight-stream kernel for M <= 32 (where its X^ slab fits), else the pipelined tile kernel (tile shape
 * chosen per layer; sq_tuning_set "gemm_variant" selects one; "force_path" 3 / 1 force either kernel, 0 a plain tile
 * kernel without the software pipeline).
 *   w   dev [N][K] of w_dt      wq  dev, bytes [N][K]      wscale  dev fp32 [S][N]
 *   x   dev [M][K] of x_dt      xq  dev, bytes [M][K]      bias    dev fp32 [N] or NULL      y  dev [M][N] of y_dt
 */
sq_status sq_quantize_weight_fp8(const sq_layer* layer, const void* w, sq_dtype w_dt, uint8_t* wq, float* wscale, void* stream);
sq_status sq_quantize_act_fp8(const sq_layer* layer, const void* x, sq_dtype x_dt, uint8_t* xq, void* stream);
/* The same with the activation in front of the layer applied first (Sec. 4.3.1-4.3.2; App. B): xq = Q_dual(act(h)) on the
 * fp8 grid, act as for sq_quantize_act_fused (host, int32 [S], SQ_ACT_* per K-segment, must not be NULL; the fp32
 * operation sequence documented there).  workspace as for sq_quantize_act_fused (NULL, or
 * sq_quantize_act_fused_workspace_bytes(layer) device bytes, 16-byte aligned: bf16 inputs are then served by code tables,
 * same codes, two launches); SQ_ERR_INVALID_ARG for a workspace that is too small or misaligned. */
sq_status sq_quantize_act_fp8_fused(const sq_layer* layer, const void* h, sq_dtype h_dt, const int32_t* act, uint8_t* xq,
                                    void* workspace, size_t workspace_bytes, void* stream);
sq_status sq_seglinear_fp8(const sq_layer* layer, const uint8_t* xq, const uint8_t* wq, const float* wscale, const float* bias,
                           void* y, sq_dtype y_dt, void* stream);

/* sq_seglinear_grouped on fp8 codes: xq from sq_quantize_act_fp8, every item's wq / wscale from sq_quantize_weight_fp8
 * (the item's wq member points at E4M3 bytes); per layer the arithmetic is that of sq_seglinear_fp8; limits as for
 * sq_seglinear_grouped. */
sq_status sq_seglinear_grouped_fp8(const sq_layer* layer, const uint8_t* xq, int32_t L, const sq_group_item* items,
                                   sq_dtype y_dt, void* stream);

/* Human-readable name of a status code (static storage). */
const char* sq_status_string(sq_status s);

/* Library version: major * 10000 + minor * 100 + patch. */
int sq_version(void);

/*
 * Diagnostics hook for benchmarks and tests: process-wide override of kernel selection.
 *   key "gemm_variant": -1 = automatic (default), otherwise the index of a tile configuration
 *   key "force_path":   -1 = automatic, 0 = generic kernel, 1 = MFMA tile kernel, 2 = skinny kernel,
 *                       3 = skinny weight-stream kernel
 * Returns SQ_ERR_INVALID_ARG for an unknown key or value.  Not thread-safe against running calls.
 */
sq_status sq_tuning_set(const char* key, int value);

#ifdef __cplusplus
}
#endif
#endif /* SEGQUANT_H */
