/*
 * CPU oracle for the tropical convolution operator family.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow loop nest
 * written from the paper's operator definitions.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * What it computes (paper, Sec. 3.1 "Tropical algebra and tropical convolution"):
 *   base operators MinPlus2d / MaxPlus2d: extremum over the KH x KW window of
 *   X[h+i, w+j, c_in] + W[i, j, c_in, c_out]; layers (iv) MinPlus-Min-Conv2d and
 *   (v) MaxPlus-Max-Conv2d then take the same extremum over c_in, i.e. one
 *   reduction over all K = C_in*KH*KW taps.  Sec. 3.3, Definitions "compound"
 *   and "parallel": alpha * (min-plus result) + beta * (max-plus result), with
 *   one shared kernel (compound) or two kernels g1 (min), g2 (max) (parallel).
 *   The discrete operators index X[h+i, w+j] + W[i, j]: cross-correlation.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - tensors are NCHW / OIHW, contiguous; tap index k = (c_in*KH + i)*KW + j;
 *   - padding holds the semiring identity (-inf for max-plus, +inf for
 *     min-plus, Sec. 3.1), so a padded tap can never win: it is skipped;
 *   - ties keep the lowest k (strict compare while k ascends);
 *   - each x + w is one rounded fp32 add; the combine is two rounded fp32
 *     products and one rounded fp32 sum (no fused multiply-add);
 *   - alpha, beta are per-output-channel vectors, NULL meaning all ones
 *     (the direct-summation variants of App. B.4);
 *   - backward routes the whole output gradient through the single winning
 *     tap of each live branch (sub-gradient of max / min); sums are kept in
 *     double so this side is the better-rounded one.
 *
 * Pins (tests/test_oracle_*.py): hand-worked examples, an independent
 * enumerate-everything-then-argmax brute force, the w == 0 max-pool special
 * case against a library routine, the unfold formulation of App. A.1.1,
 * duality / shift / monotonicity invariants, finite differences.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct oracle_shape {
  int32_t N, C_in, H, W;
  int32_t C_out, KH, KW;
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_shape;

enum { ORACLE_MAX = 0, ORACLE_MIN = 1, ORACLE_COMPOUND = 2, ORACLE_PARALLEL = 3 };

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* 1 if some window of one axis has no tap inside the input (written out: every output position, every tap).  The
 * extremum of Sec. 3.1 over an empty set of taps is not defined, so such a layer is rejected. */
static int axis_has_empty_window(long in, long k, long stride, long pad, long dil, long out) {
  for (long o = 0; o < out; ++o) {
    int hit = 0;
    for (long t = 0; t < k; ++t) {
      long i = o * stride - pad + t * dil;
      if (i >= 0 && i < in) hit = 1;
    }
    if (!hit) return 1;
  }
  return 0;
}

int oracle_out_shape(const oracle_shape* s, int32_t* H_out, int32_t* W_out) {
  long eh = (long)s->dil_h * (s->KH - 1) + 1, ew = (long)s->dil_w * (s->KW - 1) + 1;
  long nh = (long)s->H + 2L * s->pad_h - eh, nw = (long)s->W + 2L * s->pad_w - ew;
  if (nh < 0 || nw < 0) return -1;
  *H_out = (int32_t)(nh / s->stride_h + 1);
  *W_out = (int32_t)(nw / s->stride_w + 1);
  return 0;
}

/* Round an fp32 value to the nearest bf16 (ties to even), returned as fp32. */
static float round_to_bf16(float v) {
  uint32_t u;
  memcpy(&u, &v, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return v; /* inf / nan pass through */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float r;
  memcpy(&r, &u, 4);
  return r;
}

/* One output element, one branch: scan the K taps in ascending k. */
static void scan_window(const oracle_shape* s, const float* x_n, const float* w_co, int oh, int ow,
                        int want_max, float* best_out, int32_t* idx_out) {
  float best = 0.0f;
  int32_t bidx = -1;
  for (int c = 0; c < s->C_in; ++c)
    for (int i = 0; i < s->KH; ++i) {
      int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
      if (ih < 0 || ih >= s->H) continue;
      for (int j = 0; j < s->KW; ++j) {
        int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
        if (iw < 0 || iw >= s->W) continue;
        int32_t k = (c * s->KH + i) * s->KW + j;
        volatile float sum = x_n[((size_t)c * s->H + ih) * s->W + iw] + w_co[k];
        float v = sum;
        if (bidx < 0 || (want_max ? (v > best) : (v < best))) {
          best = v;
          bidx = k;
        }
      }
    }
  *best_out = best;
  *idx_out = bidx;
}

/*
 * Forward.  y / y_min / y_max / idx_min / idx_max may each be NULL (not written).
 * mode max: uses w_max, writes y = y_max, idx_max.  mode min: w_min, y = y_min.
 * compound: one kernel (w_min if non-NULL else w_max).  parallel: w_min = g1, w_max = g2.
 * out_bf16 != 0 rounds y, y_min, y_max to bf16-representable values (the index
 * decision is always the fp32 compare).  Returns 0, or -1 on a bad shape
 * (including a window that could lie wholly in the padding).
 */
int oracle_tconv_forward(const oracle_shape* s, int mode, const float* x, const float* w_min,
                         const float* w_max, const float* alpha, const float* beta, float* y,
                         float* y_min, float* y_max, int32_t* idx_min, int32_t* idx_max,
                         int out_bf16) {
  int32_t Ho, Wo;
  if (oracle_out_shape(s, &Ho, &Wo) != 0 || Ho < 1 || Wo < 1) return -1;
  if (s->pad_h > s->dil_h * (s->KH - 1) || s->pad_w > s->dil_w * (s->KW - 1)) return -1;
  if (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, Ho) ||
      axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, Wo))
    return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  const float* wmn = w_min;
  const float* wmx = w_max;
  if (mode == ORACLE_COMPOUND) wmn = wmx = (w_min ? w_min : w_max);
  if ((do_min && !wmn) || (do_max && !wmx)) return -1;
  const size_t K = (size_t)s->C_in * s->KH * s->KW;
  const size_t x_img = (size_t)s->C_in * s->H * s->W;
  const long planes = (long)s->N * s->C_out;
#pragma omp parallel for schedule(dynamic, 1)
  for (long pl = 0; pl < planes; ++pl) {
    int n = (int)(pl / s->C_out), co = (int)(pl % s->C_out);
    const float* x_n = x + (size_t)n * x_img;
    for (int oh = 0; oh < Ho; ++oh)
      for (int ow = 0; ow < Wo; ++ow) {
        size_t o = ((size_t)pl * Ho + oh) * Wo + ow;
        float vmin = 0.0f, vmax = 0.0f;
        int32_t imin = -1, imax = -1;
        if (do_min) scan_window(s, x_n, wmn + (size_t)co * K, oh, ow, 0, &vmin, &imin);
        if (do_max) scan_window(s, x_n, wmx + (size_t)co * K, oh, ow, 1, &vmax, &imax);
        float out;
        if (mode == ORACLE_MAX)
          out = vmax;
        else if (mode == ORACLE_MIN)
          out = vmin;
        else {
          float a = alpha ? alpha[co] : 1.0f, b = beta ? beta[co] : 1.0f;
          volatile float pa = a * vmin;
          volatile float pb = b * vmax;
          volatile float sum = pa + pb;
          out = sum;
        }
        if (out_bf16) {
          out = round_to_bf16(out);
          vmin = round_to_bf16(vmin);
          vmax = round_to_bf16(vmax);
        }
        if (y) y[o] = out;
        if (do_min && y_min) y_min[o] = vmin;
        if (do_max && y_max) y_max[o] = vmax;
        if (do_min && idx_min) idx_min[o] = imin;
        if (do_max && idx_max) idx_max[o] = imax;
      }
  }
  return 0;
}

/*
 * Mixed layers of Sec. 3.1: (iii) MinPlus-Max-Conv2d, y = max over c_in of MinPlus2d(X, W, h, w, c_in, c_out),
 * and (vi) MaxPlus-Min-Conv2d, y = min over c_in of MaxPlus2d(...).  outer_max != 0 selects (iii).
 * The window of every input channel is scanned in ascending tap order with a strict compare (ties:
 * lowest tap, padded taps skipped), then the channels in ascending c_in with a strict compare (ties:
 * lowest channel).  idx receives the flattened tap k = (c*KH + i)*KW + j of the winner, so the backward
 * functions below apply unchanged (mode MIN or MAX: the whole gradient goes through idx).
 */
int oracle_tconv_forward_mixed(const oracle_shape* s, int outer_max, const float* x, const float* w,
                               float* y, int32_t* idx, int out_bf16) {
  int32_t Ho, Wo;
  if (oracle_out_shape(s, &Ho, &Wo) != 0 || Ho < 1 || Wo < 1) return -1;
  if (s->pad_h > s->dil_h * (s->KH - 1) || s->pad_w > s->dil_w * (s->KW - 1)) return -1;
  if (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, Ho) ||
      axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, Wo))
    return -1;
  if (!x || !w) return -1;
  const int KK = s->KH * s->KW;
  const size_t K = (size_t)s->C_in * KK;
  const size_t x_img = (size_t)s->C_in * s->H * s->W;
  const long planes = (long)s->N * s->C_out; /* independent output planes; threads only share inputs */
#pragma omp parallel for schedule(dynamic, 1)
  for (long pl = 0; pl < planes; ++pl) {
    const int n = (int)(pl / s->C_out), co = (int)(pl % s->C_out);
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          float best = 0.0f;
          int32_t bk = -1;
          for (int c = 0; c < s->C_in; ++c) {
            /* base operator of channel c: min-plus for layer (iii), max-plus for layer (vi) */
            float v = 0.0f;
            int32_t t = -1;
            for (int i = 0; i < s->KH; ++i) {
              int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
              if (ih < 0 || ih >= s->H) continue;
              for (int j = 0; j < s->KW; ++j) {
                int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
                if (iw < 0 || iw >= s->W) continue;
                volatile float sum = x[(size_t)n * x_img + ((size_t)c * s->H + ih) * s->W + iw] +
                                     w[(size_t)co * K + (size_t)c * KK + i * s->KW + j];
                float sv = sum;
                if (t < 0 || (outer_max ? (sv < v) : (sv > v))) {
                  v = sv;
                  t = i * s->KW + j;
                }
              }
            }
            if (bk < 0 || (outer_max ? (v > best) : (v < best))) {
              best = v;
              bk = c * KK + t;
            }
          }
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          if (y) y[o] = out_bf16 ? round_to_bf16(best) : best;
          if (idx) idx[o] = bk;
        }
  }
  return 0;
}

/* Gradient that one output sends down one branch. */
static double branch_grad(int mode, int is_max, const float* alpha, const float* beta, int co,
                          float gy) {
  if (mode == ORACLE_MAX || mode == ORACLE_MIN) return (double)gy;
  float coef = is_max ? (beta ? beta[co] : 1.0f) : (alpha ? alpha[co] : 1.0f);
  return (double)coef * (double)gy;
}

/*
 * Backward w.r.t. the input: grad_x[n, c*, ih*, iw*] += g for every output and
 * live branch, (c*, i*, j*) = unflatten(idx).  grad_x (double, NCHW) is overwritten.
 * Serial on purpose: the sums are order-dependent only in the last bits of a
 * double, but a fixed order keeps the oracle reproducible.
 */
int oracle_tconv_backward_input(const oracle_shape* s, int mode, const float* gy, const float* alpha,
                                const float* beta, const int32_t* idx_min, const int32_t* idx_max,
                                double* grad_x) {
  int32_t Ho, Wo;
  if (oracle_out_shape(s, &Ho, &Wo) != 0) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  if ((do_min && !idx_min) || (do_max && !idx_max)) return -1;
  const size_t x_img = (size_t)s->C_in * s->H * s->W;
  memset(grad_x, 0, sizeof(double) * x_img * s->N);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          for (int br = 0; br < 2; ++br) {
            if ((br == 0 && !do_min) || (br == 1 && !do_max)) continue;
            int32_t k = br ? idx_max[o] : idx_min[o];
            int j = k % s->KW, i = (k / s->KW) % s->KH, c = k / (s->KW * s->KH);
            int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
            int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
            if (c < 0 || c >= s->C_in || ih < 0 || ih >= s->H || iw < 0 || iw >= s->W) return -2;
            grad_x[(size_t)n * x_img + ((size_t)c * s->H + ih) * s->W + iw] +=
                branch_grad(mode, br, alpha, beta, co, gy[o]);
          }
        }
  return 0;
}

/*
 * Backward w.r.t. the kernel(s): grad_w_b[c_out, k*] += g summed over (n, oh, ow).
 * max: grad_w_max only; min: grad_w_min only; parallel: both (g1 <- min branch,
 * g2 <- max branch); compound: both branches add into ONE tensor, grad_w_min if
 * non-NULL else grad_w_max.  Outputs (double, OIHW) are overwritten.
 */
int oracle_tconv_backward_weight(const oracle_shape* s, int mode, const float* gy,
                                 const float* alpha, const float* beta, const int32_t* idx_min,
                                 const int32_t* idx_max, double* grad_w_min, double* grad_w_max) {
  int32_t Ho, Wo;
  if (oracle_out_shape(s, &Ho, &Wo) != 0) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  if ((do_min && !idx_min) || (do_max && !idx_max)) return -1;
  const size_t K = (size_t)s->C_in * s->KH * s->KW;
  double* gmn = grad_w_min;
  double* gmx = grad_w_max;
  if (mode == ORACLE_COMPOUND) gmn = gmx = (grad_w_min ? grad_w_min : grad_w_max);
  if ((do_min && !gmn) || (do_max && !gmx)) return -1;
  if (do_min) memset(gmn, 0, sizeof(double) * K * s->C_out);
  if (do_max) memset(gmx, 0, sizeof(double) * K * s->C_out);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          if (do_min) {
            int32_t k = idx_min[o];
            if (k < 0 || (size_t)k >= K) return -2;
            gmn[(size_t)co * K + k] += branch_grad(mode, 0, alpha, beta, co, gy[o]);
          }
          if (do_max) {
            int32_t k = idx_max[o];
            if (k < 0 || (size_t)k >= K) return -2;
            gmx[(size_t)co * K + k] += branch_grad(mode, 1, alpha, beta, co, gy[o]);
          }
        }
  return 0;
}

/*
 * Gradient of the combine step (paper Sec. 3.3: y = alpha*y_min + beta*y_max, alpha and beta
 * learnable; here one pair per output channel): the step is linear in alpha and beta, so
 *   grad_alpha[c] = sum over (n, oh, ow) of gy * y_min,   grad_beta[c] = the same with y_max.
 * y_min, y_max are the branch outputs of the forward pass (fp32 values).  Compound and parallel
 * mode only.  Either output may be NULL.  Outputs (double, [C_out]) are overwritten.
 */
int oracle_tconv_backward_alpha_beta(const oracle_shape* s, int mode, const float* gy,
                                     const float* y_min, const float* y_max, double* grad_alpha,
                                     double* grad_beta) {
  int32_t Ho, Wo;
  if (oracle_out_shape(s, &Ho, &Wo) != 0) return -1;
  if (mode != ORACLE_COMPOUND && mode != ORACLE_PARALLEL) return -1;
  if (!gy || (grad_alpha && !y_min) || (grad_beta && !y_max)) return -1;
  for (int co = 0; co < s->C_out; ++co) {
    double ga = 0.0, gb = 0.0;
    for (int n = 0; n < s->N; ++n)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          if (grad_alpha) ga += (double)gy[o] * (double)y_min[o];
          if (grad_beta) gb += (double)gy[o] * (double)y_max[o];
        }
    if (grad_alpha) grad_alpha[co] = ga;
    if (grad_beta) grad_beta[co] = gb;
  }
  return 0;
}
