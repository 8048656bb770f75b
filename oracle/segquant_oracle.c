/*
 * CPU ORACLE for the SegLinear + DualScale quantized linear layer (arXiv 2507.14811).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C.  Nothing in the
 * product path may call into this file; only tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.  It shares no code, header, table or
 * helper with the HIP library.
 *
 * The method is an encoding + approximation, so the oracle takes the paper's
 * steps in the paper's order:
 *
 *   Quant(W)       uniform symmetric quantizer of Sec. 3 (z = 0), applied
 *                  separately to every segment of the weight (Sec. 4.2.2):
 *                  here per output channel and per K-segment.
 *   Q_dual(X)      Sec. 4.3.2: x < 0 uses the step s_-, x >= 0 uses s_+; the
 *                  matrix is split X = X_+ + X_- (element-wise max / min with 0)
 *                  and each part is quantized with its own step.
 *   integer GEMM   X^_+ W^ and X^_- W^ per K-segment (input-segmented sum of
 *                  Sec. 4.2.2 item 2; output segments of item 1 are column
 *                  blocks of the same product).
 *   DeQuant        Sec. 4.3.2 last display:  s_+ s_w (X^_+ W^) + s_- s_w (X^_- W^),
 *                  summed over K-segments, App. A "symmetric" recovery for a
 *                  single-scale segment.
 *
 * Readings where the paper is silent (listed in the design notes of the repo):
 *   round()            = round-half-to-even (nearbyintf under FE_TONEAREST)
 *   [q_min, q_max]     = [-127, 127]
 *   s_-                = |min x| / 127  (positive step; codes of x < 0 are <= 0)
 *   x / s              = a true IEEE fp32 division
 *   weight layout      = W[n][k] (row = output channel), i.e. the transpose of
 *                        the paper's k x n matrix
 *   percentile clip    = nearest-rank quantile of the tensor the quantizer sees (max(X,0), max(-X,0) or |X|,
 *                        zeros included), per K-segment and batch, running maximum over batches
 *   arithmetic         = fp32, every operation individually rounded (build with
 *                        -ffp-contract=off -fno-fast-math); an fp64 evaluation of
 *                        the same dequant sum is returned beside it.
 *
 * All functions return 0 on success, non-zero on a violated precondition.
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SQO_QMAX 127.0f

int sqo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* bf16 -> fp32: append 16 zero bits (exact). */
static float widen_bf16(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

void sqo_widen_bf16(const uint16_t* in, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = widen_bf16(in[i]);
}

/* fp32 -> bf16 with round-half-to-even on the dropped 16 bits (finite inputs). */
void sqo_cast_bf16(const float* in, int64_t n, uint16_t* out) {
  for (int64_t i = 0; i < n; ++i) {
    uint32_t u;
    memcpy(&u, &in[i], 4);
    uint32_t lower = u & 0xFFFFu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    out[i] = (uint16_t)upper;
  }
}

/* Sec. 3 quantizer with z = 0: clip(round(v / s), -127, 127). */
static int8_t quant_sym(float v, float s) {
  float q = nearbyintf(v / s);
  if (q > SQO_QMAX) q = SQO_QMAX;
  if (q < -SQO_QMAX) q = -SQO_QMAX;
  return (int8_t)q;
}

static int check_offsets(int n, int S, const int32_t* off) {
  if (S < 1 || off[0] != 0 || off[S] != n) return 1;
  for (int i = 0; i < S; ++i)
    if (off[i + 1] <= off[i]) return 1;
  return 0;
}

/*
 * Weight quantization, Sec. 3 quantizer applied per segment (Sec. 4.2.2):
 * for each output channel n and K-segment ks, a = max |W[n][k]| over the segment,
 * step = a / 127 (1.0 if the segment row is all zero), codes = clip(round(W / step)).
 *   w      fp32 [N][K]      wq  int8 [N][K]      wscale fp32 [S][N]
 */
int sqo_quantize_weight(const float* w, int N, int K, int S, const int32_t* kseg_off,
                        int8_t* wq, float* wscale) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off)) return 1;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int ks = 0; ks < S; ++ks) {
      float a = 0.0f;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float v = fabsf(w[(int64_t)n * K + k]);
        if (v > a) a = v;
      }
      float sw = (a == 0.0f) ? 1.0f : a / SQO_QMAX;
      wscale[(int64_t)ks * N + n] = sw;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k)
        wq[(int64_t)n * K + k] = quant_sym(w[(int64_t)n * K + k], sw);
    }
  }
  return 0;
}

/*
 * 4-bit weights (App. B, granularity of the 4-bit settings: weights per output channel): the Sec. 3 quantizer
 * with q_max = 7, per output channel n and K-segment ks,
 *   a = max_k |W[n][k]|,  wscale[ks][n] = a / 7 (1.0 if a == 0),  wq[n][k] = clip(round(W[n][k] / wscale), -7, 7).
 * The codes are returned unpacked (one int8 per weight), so the integer GEMM and DeQuant above apply unchanged.
 */
int sqo_quantize_weight_w4(const float* w, int N, int K, int S, const int32_t* kseg_off, int8_t* wq,
                           float* wscale) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int n = 0; n < N; ++n) {
    for (int ks = 0; ks < S; ++ks) {
      float a = 0.0f;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float v = fabsf(w[(int64_t)n * K + k]);
        if (v > a) a = v;
      }
      float sw = (a == 0.0f) ? 1.0f : a / 7.0f;
      wscale[(int64_t)ks * N + n] = sw;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float q = nearbyintf(w[(int64_t)n * K + k] / sw);
        if (q > 7.0f) q = 7.0f;
        if (q < -7.0f) q = -7.0f;
        wq[(int64_t)n * K + k] = (int8_t)q;
      }
    }
  }
  return 0;
}

/*
 * Storage format of 4-bit weight codes, two per byte (a layout of this library, not of the paper), made so that the
 * 16 rows x 128 codes a streaming step consumes are one contiguous KiB: K is a multiple of 128, T = K / 128; rows are
 * taken in groups of 16 (the last group padded with zero rows), and
 *   packed[((g T + t) 16 + r) 64 + j] = code(16 g + r, 128 t + j)  |  code(16 g + r, 128 t + 64 + j) << 4
 * for 0 <= r < 16, 0 <= j < 64, each code a 4-bit two's-complement number.
 *   wq int8 [N][K] with values in [-8, 7]   ->   packed uint8 [ceil(N / 16) * 16 * K / 2]
 */
int sqo_pack_w4(const int8_t* wq, int N, int K, uint8_t* packed) {
  if (K < 128 || K % 128 != 0) return 1;
  const int T = K / 128, G = (N + 15) / 16;
  for (int g = 0; g < G; ++g)
    for (int t = 0; t < T; ++t)
      for (int r = 0; r < 16; ++r)
        for (int j = 0; j < 64; ++j) {
          const int n = 16 * g + r;
          int lo = 0, hi = 0;
          if (n < N) {
            lo = wq[(int64_t)n * K + 128 * t + j];
            hi = wq[(int64_t)n * K + 128 * t + 64 + j];
          }
          if (lo < -8 || lo > 7 || hi < -8 || hi > 7) return 3;
          packed[(((int64_t)g * T + t) * 16 + r) * 64 + j] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        }
  return 0;
}

/*
 * Activation quantization.  Dual segment (Sec. 4.3.2): X_+ = max(X, 0), X_- = min(X, 0);
 * x < 0 -> code round(x / s_-) in xq_neg (clipped at -127), x >= 0 -> code
 * round(x / s_+) in xq_pos (clipped at 127); the other polarity's code is 0.
 * Single-scale segment (Sec. 3, z = 0): xq_pos = clip(round(x / s_+)), xq_neg = 0.
 *   x fp32 [M][K]     xq_pos, xq_neg int8 [M][K]
 */
int sqo_quantize_act(const float* x, int M, int K, int S, const int32_t* kseg_off,
                     const uint8_t* dual, const float* s_pos, const float* s_neg,
                     int8_t* xq_pos, int8_t* xq_neg) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int ks = 0; ks < S; ++ks) {
    if (!(s_pos[ks] > 0.0f) || !isfinite(s_pos[ks])) return 3;
    if (dual[ks] && (!(s_neg[ks] > 0.0f) || !isfinite(s_neg[ks]))) return 3;
  }
#pragma omp parallel for schedule(static)
  for (int m = 0; m < M; ++m) {
    for (int ks = 0; ks < S; ++ks) {
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        int64_t i = (int64_t)m * K + k;
        float v = x[i];
        if (dual[ks]) {
          float xp = (v > 0.0f) ? v : 0.0f; /* max(x, 0); +-0 land here */
          float xn = (v < 0.0f) ? v : 0.0f; /* min(x, 0) */
          if (v < 0.0f) {
            xq_neg[i] = quant_sym(xn, s_neg[ks]);
            xq_pos[i] = 0;
          } else {
            xq_pos[i] = quant_sym(xp, s_pos[ks]);
            xq_neg[i] = 0;
          }
        } else {
          xq_pos[i] = quant_sym(v, s_pos[ks]);
          xq_neg[i] = 0;
        }
      }
    }
  }
  return 0;
}

/*
 * Integer GEMM per K-segment on a subset of token rows.
 *   acc_pos[ks][r][n] = sum_{k in ks} xq_pos[rows[r]][k] * wq[n][k]     (exact)
 *   acc_neg[ks][r][n] = same with xq_neg for a dual segment, 0 otherwise.
 * Sums are formed in int64 (int32 partial sums over at most 1024 terms, which
 * cannot overflow: 1024 * 127 * 127 < 2^31) and must fit int32, else return 4.
 *   rows == NULL  means rows 0..nrows-1.
 *   acc_* int32 [S][nrows][N]
 */
int sqo_int_gemm(const int8_t* xq_pos, const int8_t* xq_neg, const int8_t* wq, int M, int K, int N,
                 int S, const int32_t* kseg_off, const uint8_t* dual, int nrows, const int32_t* rows,
                 int32_t* acc_pos, int32_t* acc_neg) {
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int r = 0; r < nrows; ++r) {
    int m = rows ? rows[r] : r;
    if (m < 0 || m >= M) return 1;
  }
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 64) reduction(| : overflow)
  for (int r = 0; r < nrows; ++r) {
    for (int n = 0; n < N; ++n) {
      int m = rows ? rows[r] : r;
      const int8_t* xp = xq_pos + (int64_t)m * K;
      const int8_t* xn = xq_neg + (int64_t)m * K;
      const int8_t* wr = wq + (int64_t)n * K;
      for (int ks = 0; ks < S; ++ks) {
        int64_t sp = 0, sn = 0;
        int k0 = kseg_off[ks], k1 = kseg_off[ks + 1];
        for (int kb = k0; kb < k1; kb += 1024) {
          int ke = kb + 1024 < k1 ? kb + 1024 : k1;
          int32_t pp = 0, pn = 0;
          for (int k = kb; k < ke; ++k) pp += (int32_t)xp[k] * (int32_t)wr[k];
          if (dual[ks])
            for (int k = kb; k < ke; ++k) pn += (int32_t)xn[k] * (int32_t)wr[k];
          sp += pp;
          sn += pn;
        }
        if (sp > INT32_MAX || sp < INT32_MIN || sn > INT32_MAX || sn < INT32_MIN) overflow |= 1;
        int64_t o = ((int64_t)ks * nrows + r) * N + n;
        acc_pos[o] = (int32_t)sp;
        acc_neg[o] = (int32_t)sn;
      }
    }
  }
  return overflow ? 4 : 0;
}

/*
 * Dequantization and recombination (Sec. 4.3.2 last display, summed over the
 * K-segments of Sec. 4.2.2 item 2, column n scaled with the step of its own
 * weight segment, item 1).  fp32, in this order:
 *   y = 0
 *   for ks:  c = seg_scale[ks][ns(n)] * wscale[ks][n]
 *            t = s_pos[ks] * (float)acc_pos ;  if dual: t += s_neg[ks] * (float)acc_neg
 *            y += c * t
 *   y += bias[n]
 * y64 (optional) is the same sum evaluated in double.
 *   acc_* int32 [S][nrows][N]; wscale fp32 [S][N]; seg_scale fp32 [S][T] or NULL (= 1);
 *   bias fp32 [N] or NULL;  y32 fp32 [nrows][N]; y64 double [nrows][N] or NULL
 */
int sqo_dequant(const int32_t* acc_pos, const int32_t* acc_neg, int nrows, int N, int S, int T,
                const int32_t* nseg_off, const uint8_t* dual, const float* s_pos, const float* s_neg,
                const float* wscale, const float* seg_scale, const float* bias, float* y32,
                double* y64) {
  if (check_offsets(N, T, nseg_off)) return 1;
  int* nsof = (int*)malloc(sizeof(int) * (size_t)N);
  if (!nsof) return 5;
  for (int t = 0; t < T; ++t)
    for (int n = nseg_off[t]; n < nseg_off[t + 1]; ++n) nsof[n] = t;
#pragma omp parallel for schedule(static)
  for (int r = 0; r < nrows; ++r) {
    for (int n = 0; n < N; ++n) {
      float y = 0.0f;
      double yd = 0.0;
      for (int ks = 0; ks < S; ++ks) {
        float g = seg_scale ? seg_scale[ks * T + nsof[n]] : 1.0f;
        float sw = wscale[(int64_t)ks * N + n];
        int64_t o = ((int64_t)ks * nrows + r) * N + n;
        float c = g * sw;
        float t = s_pos[ks] * (float)acc_pos[o];
        double td = (double)s_pos[ks] * (double)acc_pos[o];
        if (dual[ks]) {
          t += s_neg[ks] * (float)acc_neg[o];
          td += (double)s_neg[ks] * (double)acc_neg[o];
        }
        y += c * t;
        yd += (double)g * (double)sw * td;
      }
      if (bias) {
        y += bias[n];
        yd += (double)bias[n];
      }
      y32[(int64_t)r * N + n] = y;
      if (y64) y64[(int64_t)r * N + n] = yd;
    }
  }
  free(nsof);
  return 0;
}

/* Full-precision layer the quantized one approximates: Y = X W^T (+ bias) in double, selected rows. */
int sqo_fp_reference(const float* x, const float* w, int M, int K, int N, int nrows,
                     const int32_t* rows, const float* bias, double* yfp) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int r = 0; r < nrows; ++r) {
    for (int n = 0; n < N; ++n) {
      int m = rows ? rows[r] : r;
      double s = 0.0;
      for (int k = 0; k < K; ++k) s += (double)x[(int64_t)m * K + k] * (double)w[(int64_t)n * K + k];
      if (bias) s += (double)bias[n];
      yfp[(int64_t)r * N + n] = s;
    }
  }
  (void)M;
  return 0;
}

/*
 * Analytic bound on |y_quantized - y_full_precision| when no value is clipped
 * (steps = absmax / 127) and seg_scale == 1.  Rounding to nearest (Sec. 3) gives
 * |x - s_x x^| <= s_x / 2 and |w - s_w w^| <= s_w / 2, hence per product
 *   |x w - (s_x x^)(s_w w^)| <= |x| s_w / 2 + |w| s_x / 2 + s_x s_w / 4
 * with s_x the step of x's segment and polarity.  Summed over k, in double.
 */
int sqo_error_bound(const float* x, const float* w, int M, int K, int N, int S,
                    const int32_t* kseg_off, const uint8_t* dual, const float* s_pos,
                    const float* s_neg, const float* wscale, int nrows, const int32_t* rows,
                    double* bound) {
  if (check_offsets(K, S, kseg_off)) return 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int r = 0; r < nrows; ++r) {
    for (int n = 0; n < N; ++n) {
      int m = rows ? rows[r] : r;
      double b = 0.0;
      for (int ks = 0; ks < S; ++ks) {
        double sw = wscale[(int64_t)ks * N + n];
        for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
          double xv = x[(int64_t)m * K + k], wv = w[(int64_t)n * K + k];
          double sx = (dual[ks] && xv < 0.0) ? s_neg[ks] : s_pos[ks];
          b += fabs(xv) * sw * 0.5 + fabs(wv) * sx * 0.5 + sx * sw * 0.25;
        }
      }
      bound[(int64_t)r * N + n] = b;
    }
  }
  (void)M;
  return 0;
}

/*
 * Static activation steps from calibration data (Sec. 4.3.2, the two step definitions; App. B sensitivity
 * study: the strict min/max rule, p = 1.0), one pair per K-segment (Sec. 4.2.2 item 2):
 *   dual segment        amax_pos = max(0, max x),  amax_neg = max(0, -min x)
 *   single-scale        amax_pos = max |x|,        amax_neg = 0
 * The running maxima combine over calibration batches (accumulate != 0 keeps what amax_* already hold);
 * steps: s = amax / 127, and 1.0 where amax is 0 (a polarity that never occurred).
 *   x fp32 [M][K]    amax_pos, amax_neg, s_pos, s_neg fp32 [S]
 */
int sqo_calibrate_act(const float* x, int M, int K, int S, const int32_t* kseg_off, const uint8_t* dual,
                      int accumulate, float* amax_pos, float* amax_neg, float* s_pos, float* s_neg) {
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int ks = 0; ks < S; ++ks) {
    float ap = accumulate ? amax_pos[ks] : 0.0f;
    float an = accumulate ? amax_neg[ks] : 0.0f;
    for (int m = 0; m < M; ++m) {
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float v = x[(int64_t)m * K + k];
        if (dual[ks]) {
          if (v > ap) ap = v;
          if (-v > an) an = -v;
        } else {
          float a = fabsf(v);
          if (a > ap) ap = a;
        }
      }
    }
    amax_pos[ks] = ap;
    amax_neg[ks] = an;
    s_pos[ks] = (ap == 0.0f) ? 1.0f : ap / SQO_QMAX;
    s_neg[ks] = (an == 0.0f) ? 1.0f : an / SQO_QMAX;
  }
  return 0;
}

/*
 * The polarity-asymmetric activation in front of a DualScale layer (Sec. 4.3.1: SiLU, GELU), fused with the
 * quantizer: xq = Q_dual(act(h)).  The codes are integers decided by floating point, so the activation is
 * specified to the bit, in fp32 (the precision the kernels compute in), every operation individually rounded:
 *   exp32(t):  +inf for t > 88;  t <- max(t, -87);  n = round_half_even(t * 1.44269504);
 *              r = fma(n, -0.693145751953125, t);  r = fma(n, -1.42860682e-6, r)         (ln 2 in two parts)
 *              p = 1/5040;  p = fma(p, r, c) for c = 1/720, 1/120, 1/24, 1/6, 1/2, 1, 1   (Taylor, |r| <= ln2/2)
 *              exp32 = p * 2^n
 *   SiLU(x)      = x / (1 + exp32(-x))
 *   GELU(x)      = x / (1 + exp32(-z)),  z = (1.59576912 * x) * fma(0.044715, x * x, 1)
 *                  (the tanh form 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))), written with
 *                   0.5 (1 + tanh(u)) = 1 / (1 + e^(-2u)))
 * One activation code per K-segment: 0 none, 1 SiLU, 2 GELU.  The activation's value is quantized as the fp32
 * number it is (no rounding to bf16 in between).
 */
static float exp32(float t) {
  if (t > 88.0f) return INFINITY;
  t = fmaxf(t, -87.0f);
  const float n = nearbyintf(t * 1.44269504f);
  float r = fmaf(n, -0.693145751953125f, t);
  r = fmaf(n, -1.42860682e-6f, r);
  float p = 1.0f / 5040.0f;
  p = fmaf(p, r, 1.0f / 720.0f);
  p = fmaf(p, r, 1.0f / 120.0f);
  p = fmaf(p, r, 1.0f / 24.0f);
  p = fmaf(p, r, 1.0f / 6.0f);
  p = fmaf(p, r, 0.5f);
  p = fmaf(p, r, 1.0f);
  p = fmaf(p, r, 1.0f);
  return ldexpf(p, (int)n);
}

float sqo_silu(float x) { return x / (1.0f + exp32(-x)); }

float sqo_gelu(float x) {
  const float z = (1.59576912f * x) * fmaf(0.044715f, x * x, 1.0f);
  return x / (1.0f + exp32(-z));
}

/* a[m][k] = act_ks(h[m][k]), act[ks] in {0 none, 1 SiLU, 2 GELU};  h, a fp32 [M][K] */
int sqo_activation(const float* h, int M, int K, int S, const int32_t* kseg_off, const int32_t* act, float* a) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int ks = 0; ks < S; ++ks)
    if (act[ks] < 0 || act[ks] > 2) return 1;
  for (int m = 0; m < M; ++m)
    for (int ks = 0; ks < S; ++ks)
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        const float v = h[(int64_t)m * K + k];
        a[(int64_t)m * K + k] = act[ks] == 1 ? sqo_silu(v) : act[ks] == 2 ? sqo_gelu(v) : v;
      }
  return 0;
}

/* xq = Q_dual(act(h)): the activation above, then sqo_quantize_act on its result. */
int sqo_quantize_act_fused(const float* h, int M, int K, int S, const int32_t* kseg_off, const uint8_t* dual,
                           const int32_t* act, const float* s_pos, const float* s_neg, int8_t* xq_pos,
                           int8_t* xq_neg) {
  float* a = (float*)malloc((size_t)M * K * sizeof(float));
  if (!a) return 3;
  int rc = sqo_activation(h, M, K, S, kseg_off, act, a);
  if (rc == 0) rc = sqo_quantize_act(a, M, K, S, kseg_off, dual, s_pos, s_neg, xq_pos, xq_neg);
  free(a);
  return rc;
}

/*
 * Calibration of the activation steps with percentile clipping (App. B, dual-scale sensitivity study: the rule
 * p = 1.0 of sqo_calibrate_act against clipping at p <= 0.9999).  The paper names the percentile only; the
 * reading taken here: the calibrator sees the tensor that the quantizer sees, i.e. per K-segment
 *   dual          V_+ = max(X, 0),  V_- = max(-X, 0)      (Sec. 4.3.2: X = X_+ + X_-, zeros included)
 *   single-scale  V_+ = |X|
 * and the clipping threshold of a batch is the nearest-rank p-quantile of the n = M * K_ks values of V:
 * the k-th smallest with k = ceil(p * n) evaluated in IEEE double, clamped to [1, n]  (p = 1.0: the maximum).
 * Thresholds combine over batches like the maxima do (running maximum); steps: s = threshold / 127, and 1.0
 * where it is 0.  Written as the definition: sort, then index.
 *   x fp32 [M][K]    0 < p <= 1    amax_pos, amax_neg, s_pos, s_neg fp32 [S]
 */
static int cmp_f32(const void* a, const void* b) {
  const float x = *(const float*)a, y = *(const float*)b;
  return (x > y) - (x < y);
}

int sqo_calibrate_act_percentile(const float* x, int M, int K, int S, const int32_t* kseg_off, const uint8_t* dual,
                                 double p, int accumulate, float* amax_pos, float* amax_neg, float* s_pos,
                                 float* s_neg) {
  if (check_offsets(K, S, kseg_off)) return 1;
  if (!(p > 0.0 && p <= 1.0) || M < 1) return 1;
  for (int ks = 0; ks < S; ++ks) {
    const int L = kseg_off[ks + 1] - kseg_off[ks];
    const int64_t n = (int64_t)M * L;
    float* vp = (float*)malloc((size_t)n * sizeof(float));
    float* vn = (float*)malloc((size_t)n * sizeof(float));
    if (!vp || !vn) { free(vp); free(vn); return 3; }
    int64_t i = 0;
    for (int m = 0; m < M; ++m)
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k, ++i) {
        const float v = x[(int64_t)m * K + k];
        if (dual[ks]) {
          vp[i] = v > 0.0f ? v : 0.0f;
          vn[i] = v < 0.0f ? -v : 0.0f;
        } else {
          vp[i] = fabsf(v);
          vn[i] = 0.0f;
        }
      }
    qsort(vp, (size_t)n, sizeof(float), cmp_f32);
    qsort(vn, (size_t)n, sizeof(float), cmp_f32);
    int64_t kth = (int64_t)ceil(p * (double)n);
    if (kth < 1) kth = 1;
    if (kth > n) kth = n;
    const float tp = vp[kth - 1], tn = vn[kth - 1];
    free(vp);
    free(vn);
    float ap = accumulate ? amax_pos[ks] : 0.0f;
    float an = accumulate ? amax_neg[ks] : 0.0f;
    if (tp > ap) ap = tp;
    if (tn > an) an = tn;
    amax_pos[ks] = ap;
    amax_neg[ks] = an;
    s_pos[ks] = (ap == 0.0f) ? 1.0f : ap / SQO_QMAX;
    s_neg[ks] = (an == 0.0f) ? 1.0f : an / SQO_QMAX;
  }
  return 0;
}

/*
 * Quant(W) at the paper's own granularity for 8 bit (App. B, quantization granularity: per-tensor, which
 * under SegLinear means one step per weight segment): one step per (K-segment, N-segment) block,
 *   a = max |W[n][k]| over n in ns, k in ks;  step = a / 127 (1.0 if the block is all zero),
 * written to every channel of the block, so that wscale keeps its [S][N] shape.
 */
int sqo_quantize_weight_block(const float* w, int N, int K, int S, const int32_t* kseg_off, int T,
                              const int32_t* nseg_off, int8_t* wq, float* wscale) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off) || check_offsets(N, T, nseg_off)) return 1;
  for (int ks = 0; ks < S; ++ks) {
    for (int ns = 0; ns < T; ++ns) {
      float a = 0.0f;
      for (int n = nseg_off[ns]; n < nseg_off[ns + 1]; ++n)
        for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
          float v = fabsf(w[(int64_t)n * K + k]);
          if (v > a) a = v;
        }
      float sw = (a == 0.0f) ? 1.0f : a / SQO_QMAX;
      for (int n = nseg_off[ns]; n < nseg_off[ns + 1]; ++n) {
        wscale[(int64_t)ks * N + n] = sw;
        for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k)
          wq[(int64_t)n * K + k] = quant_sym(w[(int64_t)n * K + k], sw);
      }
    }
  }
  return 0;
}

/*
 * Per-segment smoothing in front of the quantizers (Sec. 4.2.2, last paragraph: SegLinear shares the migration
 * strength alpha of SmoothQuant across a semantically coherent channel group; App. B: SmoothQuant is the optimizer of
 * the 8-bit settings, alpha swept per layer).  The published SmoothQuant rule, one alpha per K-segment:
 *   a_x[k] = max_m |X[m][k]|  over the calibration batches,   a_w[k] = max_n |W[n][k]|,
 *   s[k]   = a_x[k]^alpha / a_w[k]^(1 - alpha)   for k in K-segment ks, alpha = alpha[ks],
 *   X' = X diag(s)^-1,   W' = W diag(s)   (per input channel k), so that X' W'^T = X W^T,
 * after which X' and W' go through the ordinary quantizers.
 * Readings: the powers are evaluated in double and rounded once to fp32; a channel whose a_x or a_w is 0, or whose
 * factor is not a finite positive fp32 number, keeps s = 1; the activation side multiplies by the fp32 reciprocal
 * r[k] = 1 / s[k] (one IEEE division, then one multiplication per element: the form in which the factor is folded
 * into the operator in front of the layer).
 */
int sqo_channel_amax(const float* x, int M, int K, float* amax, int accumulate) {
  for (int k = 0; k < K; ++k) {
    float a = accumulate ? amax[k] : 0.0f;
    for (int m = 0; m < M; ++m) {
      float v = fabsf(x[(int64_t)m * K + k]);
      if (v > a) a = v;
    }
    amax[k] = a;
  }
  return 0;
}

int sqo_smooth_factors(const float* amax_x, const float* amax_w, int K, int S, const int32_t* kseg_off,
                       const float* alpha, float* smooth, float* smooth_inv) {
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int ks = 0; ks < S; ++ks) {
    if (!(alpha[ks] >= 0.0f && alpha[ks] <= 1.0f)) return 3;
    for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
      float s = 1.0f;
      if (amax_x[k] > 0.0f && amax_w[k] > 0.0f) {
        double d = pow((double)amax_x[k], (double)alpha[ks]) / pow((double)amax_w[k], 1.0 - (double)alpha[ks]);
        s = (float)d;
        if (!(s > 0.0f) || !isfinite(s) || !isfinite(1.0f / s)) s = 1.0f;
      }
      smooth[k] = s;
      smooth_inv[k] = 1.0f / s;
    }
  }
  return 0;
}

/* W'[n][k] = W[n][k] * s[k] (one fp32 multiplication), then the per-channel, per-K-segment quantizer. */
int sqo_quantize_weight_smoothed(const float* w, int N, int K, int S, const int32_t* kseg_off, const float* smooth,
                                 int8_t* wq, float* wscale) {
  if (fegetround() != FE_TONEAREST) return 2;
  if (check_offsets(K, S, kseg_off)) return 1;
  for (int n = 0; n < N; ++n) {
    for (int ks = 0; ks < S; ++ks) {
      float a = 0.0f;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float v = fabsf(w[(int64_t)n * K + k] * smooth[k]);
        if (v > a) a = v;
      }
      float sw = (a == 0.0f) ? 1.0f : a / SQO_QMAX;
      wscale[(int64_t)ks * N + n] = sw;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k)
        wq[(int64_t)n * K + k] = quant_sym(w[(int64_t)n * K + k] * smooth[k], sw);
    }
  }
  return 0;
}

/* X'[m][k] = X[m][k] * r[k] (one fp32 multiplication), written to xs; Q_dual(X') is sqo_quantize_act on xs. */
int sqo_smooth_act(const float* x, int M, int K, const float* smooth_inv, float* xs) {
  for (int m = 0; m < M; ++m)
    for (int k = 0; k < K; ++k) xs[(int64_t)m * K + k] = x[(int64_t)m * K + k] * smooth_inv[k];
  return 0;
}

/*
 * Low-rank side branch of the 4-bit settings (main results, W4A8 rows; App. B: SVDQuant is the optimizer of the 4-bit
 * settings, "the low-rank setting is fixed at 64").  The published decomposition W = Lu Ld + R keeps a rank-r part in
 * 16 bit next to the quantized residual R; on the forward path
 *   y[m][n] = y_q[m][n] + sum_j ( sum_k X[m][k] Ld[j][k] ) Lu[n][j],      Ld [r][K], Lu [N][r],
 * where y_q is the quantized layer on R (sq-oracle functions above) and X are the unquantized 16-bit activations.
 * Evaluated here in double, in that order (down projection, then up projection); y_q may be NULL (= 0).
 */
int sqo_lowrank(const float* x, const float* ld, const float* lu, const float* y_q, int M, int K, int N, int r,
                double* t_out, double* y_out) {
  if (M < 1 || K < 1 || N < 1 || r < 1) return 1;
#pragma omp parallel for schedule(static)
  for (int m = 0; m < M; ++m) {
    for (int j = 0; j < r; ++j) {
      double acc = 0.0;
      for (int k = 0; k < K; ++k) acc += (double)x[(int64_t)m * K + k] * (double)ld[(int64_t)j * K + k];
      t_out[(int64_t)m * r + j] = acc;
    }
    for (int n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int j = 0; j < r; ++j) acc += t_out[(int64_t)m * r + j] * (double)lu[(int64_t)n * r + j];
      y_out[(int64_t)m * N + n] = acc + (y_q ? (double)y_q[(int64_t)m * N + n] : 0.0);
    }
  }
  return 0;
}

/*
 * The 8-bit floating-point variant (main results, the 8/8 fp rows of the SDXL table): the same layer with fp8 codes in
 * place of int8 ones.  Format: the published OCP 8-bit float E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits, subnormals, no infinity, S.1111.111 = NaN, largest finite value 448).  The Sec. 3 quantizer becomes
 *   code = e4m3( clip(v / s, -448, 448) ),  round to nearest, ties to even,   s = max|v| / 448  (1.0 if 0),
 * Q_dual (Sec. 4.3.2) keeps its two steps s_+ = max x / 448, s_- = |min x| / 448, the products X^_+ W^ and X^_- W^ are
 * sums of exact products of code values, and DeQuant is the same scaled sum.
 */
#define SQO_FP8_MAX 448.0f

float sqo_fp8_decode(uint8_t c) {
  int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
  float v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexpf((float)m, -9);            /* subnormal: m/8 * 2^-6 */
  else v = ldexpf((float)(8 + m), e - 10);         /* (1 + m/8) * 2^(e-7) */
  return sign ? -v : v;
}

/* Nearest E4M3 value to v (finite), ties to the even mantissa, saturating at +-448. */
uint8_t sqo_fp8_encode(float v) {
  uint8_t sign = signbit(v) ? 0x80 : 0x00;
  float a = fabsf(v);
  if (!(a < SQO_FP8_MAX)) return sign | 0x7E;      /* 448 and beyond */
  /* walk the 127 non-negative finite codes: the representable values are ascending in the code */
  int lo = 0;
  for (int c = 1; c <= 0x7E; ++c)
    if (sqo_fp8_decode((uint8_t)c) <= a) lo = c;
  if (lo == 0x7E) return sign | 0x7E;
  float vlo = sqo_fp8_decode((uint8_t)lo), vhi = sqo_fp8_decode((uint8_t)(lo + 1));
  double dlo = (double)a - (double)vlo, dhi = (double)vhi - (double)a;
  int pick = dlo < dhi ? lo : (dhi < dlo ? lo + 1 : ((lo & 1) ? lo + 1 : lo));
  return sign | (uint8_t)pick;
}

void sqo_fp8_encode_array(const float* v, int64_t n, uint8_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = sqo_fp8_encode(v[i]);
}
void sqo_fp8_decode_array(const uint8_t* c, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = sqo_fp8_decode(c[i]);
}

int sqo_quantize_weight_fp8(const float* w, int N, int K, int S, const int32_t* kseg_off, uint8_t* wq, float* wscale) {
  if (check_offsets(K, S, kseg_off)) return 1;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ks = 0; ks < S; ++ks) {
      float a = 0.0f;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        float v = fabsf(w[(int64_t)n * K + k]);
        if (v > a) a = v;
      }
      float sw = (a == 0.0f) ? 1.0f : a / SQO_FP8_MAX;
      wscale[(int64_t)ks * N + n] = sw;
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) wq[(int64_t)n * K + k] = sqo_fp8_encode(w[(int64_t)n * K + k] / sw);
    }
  return 0;
}

/* Q_dual with fp8 codes: x < 0 takes s_-, x >= 0 takes s_+; the other polarity's code is +0. */
int sqo_quantize_act_fp8(const float* x, int M, int K, int S, const int32_t* kseg_off, const uint8_t* dual,
                         const float* s_pos, const float* s_neg, uint8_t* xq_pos, uint8_t* xq_neg) {
  if (check_offsets(K, S, kseg_off)) return 1;
#pragma omp parallel for schedule(static)
  for (int m = 0; m < M; ++m)
    for (int ks = 0; ks < S; ++ks)
      for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
        int64_t i = (int64_t)m * K + k;
        float v = x[i];
        if (dual[ks] && v < 0.0f) {
          xq_neg[i] = sqo_fp8_encode(v / s_neg[ks]);
          xq_pos[i] = 0;
        } else {
          xq_pos[i] = sqo_fp8_encode(v / s_pos[ks]);
          xq_neg[i] = 0;
        }
      }
  return 0;
}

/*
 * The layer on fp8 codes, in double: per K-segment the two products of code VALUES (exact in double: every product is
 * a multiple of 2^-18 below 2^18, a segment has at most 2^17 terms), then
 *   y = sum_ks seg_scale[ks][ns(n)] wscale[ks][n] ( s_+[ks] acc_+ + s_-[ks] acc_- ) + bias[n].
 * Also returns mag[m][n], the same sum over the magnitudes of the terms (the scale of the rounding error of an fp32
 * evaluation).
 */
int sqo_seglinear_fp8(const uint8_t* xq_pos, const uint8_t* xq_neg, const uint8_t* wq, int M, int K, int N, int S,
                      const int32_t* kseg_off, int T, const int32_t* nseg_off, const uint8_t* dual, const float* s_pos,
                      const float* s_neg, const float* wscale, const float* seg_scale, const float* bias, double* y,
                      double* mag) {
  if (check_offsets(K, S, kseg_off) || check_offsets(N, T, nseg_off)) return 1;
  float tab[256];
  for (int c = 0; c < 256; ++c) tab[c] = ((c & 0x7F) == 0x7F) ? 0.0f : sqo_fp8_decode((uint8_t)c);
#pragma omp parallel for schedule(static)
  for (int m = 0; m < M; ++m)
    for (int n = 0; n < N; ++n) {
      int ns = 0;
      while (ns + 1 < T && n >= nseg_off[ns + 1]) ++ns;
      double yy = 0.0, mm = 0.0;
      for (int ks = 0; ks < S; ++ks) {
        double ap = 0.0, an = 0.0, mp = 0.0, mn = 0.0;
        for (int k = kseg_off[ks]; k < kseg_off[ks + 1]; ++k) {
          double wv = tab[wq[(int64_t)n * K + k]];
          double p = (double)tab[xq_pos[(int64_t)m * K + k]] * wv;
          ap += p;
          mp += fabs(p);
          if (dual[ks]) {
            double q = (double)tab[xq_neg[(int64_t)m * K + k]] * wv;
            an += q;
            mn += fabs(q);
          }
        }
        double c = (double)wscale[(int64_t)ks * N + n] * (seg_scale ? (double)seg_scale[ks * T + ns] : 1.0);
        yy += c * ((double)s_pos[ks] * ap + (dual[ks] ? (double)s_neg[ks] * an : 0.0));
        mm += fabs(c) * ((double)s_pos[ks] * mp + (dual[ks] ? (double)s_neg[ks] * mn : 0.0));
      }
      y[(int64_t)m * N + n] = yy + (bias ? (double)bias[n] : 0.0);
      mag[(int64_t)m * N + n] = mm + (bias ? fabs((double)bias[n]) : 0.0);
    }
  return 0;
}
