/*
 * CPU oracle for the lowered Convolution / FullyConnected hot path of the Glow paper
 * (arXiv 1805.00907).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct statement of what the
 * operators compute, written from the paper's definitions.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares nothing with the GPU library: no headers, no
 * helpers, no tables.  Tensors are passed as plain pointers and plain integers.
 *
 * What each function follows:
 *   - convolution            : Section 3.1 (a convolution is "a sequence of 7 loops"), the IR listing of
 *                              Section 3.5 (input <N x H x W x C>, filter <D x Kx x Ky x C>, bias <D>,
 *                              parameters [kernel stride pad depth]) and the filter-layout figure of
 *                              Section 5.2 ([depth, filter_x, filter_y, channel]).
 *   - fully connected        : Section 3.4 (FullyConnected = matrix multiplication followed by a
 *                              broadcasted add).
 *   - relu                   : the max0 instruction of the Section 3.5 listing.
 *   - quantized tensors      : Section 4.1, value = (input - offset) * scale, int8 range [-128, 127].
 *   - requantize             : Section 4.3 (rescale folded into the numeric-producing operation) and the
 *                              same-scale max of Section 4.3 for the quantized Relu.
 *   - rescale                : Section 4.3 (rescale nodes change the range of the integers).
 *   - chain with a tensor add: Section 5.2 (stacked data-parallel operators work on one memory
 *                              location one after the other; the fused Add + max loop of the
 *                              code-generation figure of Section 5.3): Y = act(conv + bias + addend).
 *                              Quantized: the addend is rescaled (Section 4.3 rescale node) to the
 *                              accumulator's scale sx*sw and added before the one requantize.
 *   - general chains         : Section 5.2 again: ANY run of data-parallel operators behind the
 *                              contraction is stacked.  oracle_conv2d_f32_chain / oracle_qconv2d_chain
 *                              apply a list of {add tensor, multiply by scalar, max with scalar, clip}
 *                              in the order given.
 *   - batch-norm fold        : Section 5.3 (batch normalization is merged into the convolution
 *                              that precedes it before code is generated).
 *
 * Readings taken where the paper is silent (all listed in the design notes of the repository):
 *   cross-correlation (no filter flip); zero padding in the real domain; floor in the output-size
 *   formula; contiguous channel groups; FC weight is [K][N] row-major; int32 bias with scale sx*sw
 *   and offset 0; requantization multiplier sx*sw/sy represented as m * 2^-sh with a 31-bit
 *   mantissa, rounding half up; saturation to [-128, 127]; a quantized addend (scale sr, offset
   r_off) enters the int32 accumulator as round_half_up((r - r_off) * sr / (sx*sw)) with the same
   mantissa/shift representation of sr/(sx*sw).  A general quantized chain runs on the int32
 *   accumulator, whose real value is acc * s with s = sx*sw at first: a scalar multiply by c > 0
 *   changes s to s*c and leaves the integer alone (exact); max / clip thresholds are rounded half up
 *   to the accumulator's grid, T = floor(v / s + 0.5); an added tensor is rescaled to the current s;
 *   the one requantize at the end uses s_final / sy.
 *
 * Floating point: every sum is accumulated in double in the loop order written here and rounded
 * once to float.  Integer: sums are accumulated in 64-bit and must fit 32-bit (checked).
 *
 * Pin status: every function here is pinned by tests that do not call it to produce their expected
 * values (closed forms, numpy matmul on an explicit im2col matrix, exact rationals, hand-worked
 * cases).  The rounding mode of the requantize step is a reading, not something the paper fixes:
 * its pins are the closed forms of that reading plus the 1-LSB distance from the real-valued
 * formula of Section 4.1 ("parity unpinned by the paper" for the tie-break itself).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_OK = 0, ORACLE_BAD_SHAPE = 1, ORACLE_BAD_QUANT = 2, ORACLE_ACC_OVERFLOW = 3 };
enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1 };

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Output extent of one spatial axis: floor((in + pad_lo + pad_hi - kernel) / stride) + 1.
 * The paper's own examples: 28 with kernel 5, stride 1, pad 2 gives 28; the pool example 28 with
 * kernel 3, stride 3, pad 0 gives 9 (so the division floors).  Returns 0 when nothing fits. */
int64_t oracle_out_dim(int64_t in, int64_t kernel, int64_t stride, int64_t pad_lo, int64_t pad_hi) {
  int64_t span = in + pad_lo + pad_hi - kernel;
  if (in <= 0 || kernel <= 0 || stride <= 0 || pad_lo < 0 || pad_hi < 0 || span < 0) return 0;
  return span / stride + 1;
}

typedef struct {
  int64_t n, h, w, c;           /* input  [n][h][w][c]                  */
  int64_t k, r, s;              /* filter [k][r][s][c / groups]         */
  int64_t stride_h, stride_w;
  int64_t pad_t, pad_l, pad_b, pad_r;
  int64_t groups;
  int64_t oh, ow;               /* derived                              */
} conv_shape;

static int conv_shape_init(conv_shape *cs, const int64_t *p) {
  cs->n = p[0]; cs->h = p[1]; cs->w = p[2]; cs->c = p[3];
  cs->k = p[4]; cs->r = p[5]; cs->s = p[6];
  cs->stride_h = p[7]; cs->stride_w = p[8];
  cs->pad_t = p[9]; cs->pad_l = p[10]; cs->pad_b = p[11]; cs->pad_r = p[12];
  cs->groups = p[13];
  if (cs->n <= 0 || cs->h <= 0 || cs->w <= 0 || cs->c <= 0 || cs->k <= 0 || cs->r <= 0 || cs->s <= 0)
    return ORACLE_BAD_SHAPE;
  if (cs->groups <= 0 || cs->c % cs->groups != 0 || cs->k % cs->groups != 0) return ORACLE_BAD_SHAPE;
  cs->oh = oracle_out_dim(cs->h, cs->r, cs->stride_h, cs->pad_t, cs->pad_b);
  cs->ow = oracle_out_dim(cs->w, cs->s, cs->stride_w, cs->pad_l, cs->pad_r);
  if (cs->oh <= 0 || cs->ow <= 0) return ORACLE_BAD_SHAPE;
  return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * fp32 convolution: one output element.  The three inner loops (r, s, c) of the seven.
 * Taps that fall into the padding contribute nothing (zero padding).
 * ---------------------------------------------------------------------------------------------- */
static float conv_f32_one(const float *x, const float *w, const float *bias, const float *addend,
                          const conv_shape *cs, int act, int64_t n, int64_t oh, int64_t ow, int64_t k) {
  const int64_t cg = cs->c / cs->groups;   /* input channels per group  */
  const int64_t kg = cs->k / cs->groups;   /* output channels per group */
  const int64_t g = k / kg;
  double acc = 0.0;
  for (int64_t r = 0; r < cs->r; ++r) {
    const int64_t ih = oh * cs->stride_h - cs->pad_t + r;
    if (ih < 0 || ih >= cs->h) continue;
    for (int64_t s = 0; s < cs->s; ++s) {
      const int64_t iw = ow * cs->stride_w - cs->pad_l + s;
      if (iw < 0 || iw >= cs->w) continue;
      for (int64_t cc = 0; cc < cg; ++cc) {
        const int64_t c = g * cg + cc;
        const double xv = (double)x[((n * cs->h + ih) * cs->w + iw) * cs->c + c];
        const double wv = (double)w[((k * cs->r + r) * cs->s + s) * cg + cc];
        acc += xv * wv;
      }
    }
  }
  if (bias) acc += (double)bias[k];
  /* the next link of the element-wise chain: a tensor of the output's shape */
  if (addend) acc += (double)addend[((n * cs->oh + oh) * cs->ow + ow) * cs->k + k];
  if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;
  return (float)acc;
}

/* p = {n,h,w,c, k,r,s, stride_h,stride_w, pad_t,pad_l,pad_b,pad_r, groups}.  y is [n][oh][ow][k]. */
int oracle_conv2d_f32_add(const float *x, const float *w, const float *bias, const float *addend, float *y,
                          const int64_t *p, int act);

int oracle_conv2d_f32(const float *x, const float *w, const float *bias, float *y, const int64_t *p,
                      int act) {
  return oracle_conv2d_f32_add(x, w, bias, NULL, y, p, act);
}

/* Y = act(conv(X, W) + bias + addend); addend is [n][oh][ow][k] like y, or NULL. */
int oracle_conv2d_f32_add(const float *x, const float *w, const float *bias, const float *addend, float *y,
                          const int64_t *p, int act) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < cs.n; ++n)
    for (int64_t oh = 0; oh < cs.oh; ++oh)
      for (int64_t ow = 0; ow < cs.ow; ++ow)
        for (int64_t k = 0; k < cs.k; ++k)
          y[((n * cs.oh + oh) * cs.ow + ow) * cs.k + k] =
              conv_f32_one(x, w, bias, addend, &cs, act, n, oh, ow, k);
  return ORACLE_OK;
}

/* The same definition evaluated only at the given flat output indices (into [n][oh][ow][k]). */
int oracle_conv2d_f32_add_points(const float *x, const float *w, const float *bias, const float *addend,
                                 const int64_t *p, int act, const int64_t *flat_idx, int64_t n_idx,
                                 float *out);

int oracle_conv2d_f32_points(const float *x, const float *w, const float *bias, const int64_t *p, int act,
                             const int64_t *flat_idx, int64_t n_idx, float *out) {
  return oracle_conv2d_f32_add_points(x, w, bias, NULL, p, act, flat_idx, n_idx, out);
}

int oracle_conv2d_f32_add_points(const float *x, const float *w, const float *bias, const float *addend,
                                 const int64_t *p, int act, const int64_t *flat_idx, int64_t n_idx,
                                 float *out) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
  const int64_t total = cs.n * cs.oh * cs.ow * cs.k;
  for (int64_t i = 0; i < n_idx; ++i)
    if (flat_idx[i] < 0 || flat_idx[i] >= total) return ORACLE_BAD_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n_idx; ++i) {
    int64_t f = flat_idx[i];
    const int64_t k = f % cs.k; f /= cs.k;
    const int64_t ow = f % cs.ow; f /= cs.ow;
    const int64_t oh = f % cs.oh; f /= cs.oh;
    out[i] = conv_f32_one(x, w, bias, addend, &cs, act, f, oh, ow, k);
  }
  return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * fp32 fully connected: Y = A[M][K] * W[K][N], then the broadcast add of bias[N], then the
 * element-wise activation.
 * ---------------------------------------------------------------------------------------------- */
int oracle_fc_f32(const float *a, const float *w, const float *bias, float *y, int64_t M, int64_t K,
                  int64_t N, int act) {
  if (M <= 0 || K <= 0 || N <= 0) return ORACLE_BAD_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double acc = 0.0;
      for (int64_t k = 0; k < K; ++k) acc += (double)a[m * K + k] * (double)w[k * N + n];
      if (bias) acc += (double)bias[n];
      if (act == ORACLE_ACT_RELU && acc < 0.0) acc = 0.0;
      y[m * N + n] = (float)acc;
    }
  return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Quantized tensors: value = (q - offset) * scale with q in [-128, 127].
 * ---------------------------------------------------------------------------------------------- */
void oracle_dequantize(const int8_t *q, int64_t count, float scale, int32_t offset, double *value) {
  for (int64_t i = 0; i < count; ++i) value[i] = ((double)q[i] - (double)offset) * (double)scale;
}

/* Inverse of the above for test data: nearest code (ties to even), saturated.  A NaN has no code;
 * it is given the code of the real value zero (a reading: the paper does not define it, and a cast
 * of NaN to an integer is undefined in C). */
void oracle_quantize(const double *value, int64_t count, float scale, int32_t offset, int8_t *q) {
  for (int64_t i = 0; i < count; ++i) {
    double t = nearbyint(value[i] / (double)scale) + (double)offset;
    if (t != t) t = (double)offset;
    if (t < -128.0) t = -128.0;
    if (t > 127.0) t = 127.0;
    q[i] = (int8_t)t;
  }
}

/* The combined multiplier Mr = sx * sw / sy, written as mant * 2^-shift with mant in [2^30, 2^31).
 * Returns ORACLE_BAD_QUANT when a scale is not a positive finite number or the shift leaves
 * [1, 62]. */
int oracle_requant_params(float sx, float sw, float sy, int32_t *mant, int32_t *shift) {
  if (!(sx > 0.0f) || !(sw > 0.0f) || !(sy > 0.0f) || isinf(sx) || isinf(sw) || isinf(sy))
    return ORACLE_BAD_QUANT;
  const double mr = (double)sx * (double)sw / (double)sy;
  if (!(mr > 0.0) || isinf(mr)) return ORACLE_BAD_QUANT;
  int e = 0;
  const double f = frexp(mr, &e);               /* mr = f * 2^e, f in [0.5, 1) */
  int64_t m = llround(f * 2147483648.0);        /* f * 2^31 */
  if (m == 2147483648LL) { m = 1073741824LL; e += 1; }
  const int sh = 31 - e;
  if (sh < 1 || sh > 62) return ORACLE_BAD_QUANT;
  *mant = (int32_t)m;
  *shift = (int32_t)sh;
  return ORACLE_OK;
}

/* round_half_up(acc * mant / 2^shift) + y_offset, saturated to [lo, 127]. */
int32_t oracle_requantize(int32_t acc, int32_t mant, int32_t shift, int32_t y_offset, int32_t lo) {
  const int64_t prod = (int64_t)acc * (int64_t)mant;
  const int64_t half = (int64_t)1 << (shift - 1);
  /* floor division by 2^shift; written with / and % so that it does not rely on the
   * implementation-defined right shift of a negative value */
  const int64_t t = prod + half;
  const int64_t d = (int64_t)1 << shift;
  int64_t q = t / d;
  if ((t % d) < 0) q -= 1;
  q += y_offset;
  if (q < lo) q = lo;
  if (q > 127) q = 127;
  return (int32_t)q;
}

/* Lower clamp bound: Relu on a quantized tensor is max(q, y_offset) because the real value 0 is
 * the code y_offset and input and output of the max share one scale. */
static int32_t relu_floor(int act, int32_t y_offset) {
  if (act == ORACLE_ACT_RELU && y_offset > -128) return y_offset;
  return -128;
}

static int qconv_acc_one(const int8_t *x, int32_t x_off, const int8_t *w, int32_t w_off,
                         const int32_t *bias, int64_t extra, const conv_shape *cs, int64_t n, int64_t oh,
                         int64_t ow, int64_t k, int32_t *acc_out) {
  const int64_t cg = cs->c / cs->groups;
  const int64_t kg = cs->k / cs->groups;
  const int64_t g = k / kg;
  int64_t acc = 0;
  for (int64_t r = 0; r < cs->r; ++r) {
    const int64_t ih = oh * cs->stride_h - cs->pad_t + r;
    if (ih < 0 || ih >= cs->h) continue;           /* padded tap: real value 0, contributes 0 */
    for (int64_t s = 0; s < cs->s; ++s) {
      const int64_t iw = ow * cs->stride_w - cs->pad_l + s;
      if (iw < 0 || iw >= cs->w) continue;
      for (int64_t cc = 0; cc < cg; ++cc) {
        const int64_t c = g * cg + cc;
        const int64_t xv = (int64_t)x[((n * cs->h + ih) * cs->w + iw) * cs->c + c] - x_off;
        const int64_t wv = (int64_t)w[((k * cs->r + r) * cs->s + s) * cg + cc] - w_off;
        acc += xv * wv;
      }
    }
  }
  if (bias) acc += (int64_t)bias[k];
  acc += extra;                                    /* rescaled addend of the chain, 0 without one */
  if (acc > INT32_MAX || acc < INT32_MIN) return ORACLE_ACC_OVERFLOW;
  *acc_out = (int32_t)acc;
  return ORACLE_OK;
}

static int offsets_ok(int32_t a, int32_t b, int32_t c) {
  return a >= -128 && a <= 127 && b >= -128 && b <= 127 && c >= -128 && c <= 127;
}

/* The rescale node of Section 4.3 on its own: the same real values on another scale/offset,
 * out = sat(round_half_up((in - in_offset) * s_in / s_out) + out_offset), with the multiplier s_in / s_out
 * in the mantissa/shift form of oracle_requant_params. */
int oracle_rescale(const int8_t *in, int64_t count, float s_in, int32_t in_offset, float s_out,
                   int32_t out_offset, int8_t *out) {
  if (in_offset < -128 || in_offset > 127 || out_offset < -128 || out_offset > 127) return ORACLE_BAD_QUANT;
  int32_t mant = 0, shift = 0;
  const int rc = oracle_requant_params(s_in, 1.0f, s_out, &mant, &shift);
  if (rc) return rc;
  for (int64_t i = 0; i < count; ++i)
    out[i] = (int8_t)oracle_requantize((int32_t)in[i] - in_offset, mant, shift, out_offset, -128);
  return ORACLE_OK;
}

/* Rescale of a quantized addend (scale sr) to the accumulator's scale sx*sw: the multiplier
 * sr / (sx*sw) as mant * 2^-shift, mant in [2^30, 2^31), shift in [1, 62]. */
int oracle_rescale_params(float sr, float sx, float sw, int32_t *mant, int32_t *shift) {
  if (!(sr > 0.0f) || !(sx > 0.0f) || !(sw > 0.0f) || isinf(sr) || isinf(sx) || isinf(sw))
    return ORACLE_BAD_QUANT;
  const double mr = (double)sr / ((double)sx * (double)sw);
  if (!(mr > 0.0) || isinf(mr)) return ORACLE_BAD_QUANT;
  int e = 0;
  const double f = frexp(mr, &e);
  int64_t m = llround(f * 2147483648.0);
  if (m == 2147483648LL) { m = 1073741824LL; e += 1; }
  const int sh = 31 - e;
  if (sh < 1 || sh > 62) return ORACLE_BAD_QUANT;
  *mant = (int32_t)m;
  *shift = (int32_t)sh;
  return ORACLE_OK;
}

/* round_half_up(d * mant / 2^shift) for a code difference d = r - r_off (|d| <= 255). */
int64_t oracle_rescale_term(int32_t d, int32_t mant, int32_t shift) {
  const int64_t t = (int64_t)d * (int64_t)mant + ((int64_t)1 << (shift - 1));
  const int64_t den = (int64_t)1 << shift;
  int64_t q = t / den;
  if ((t % den) < 0) q -= 1;                       /* floor */
  return q;
}

int oracle_qconv2d_add(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw, int32_t w_off,
                       const int32_t *bias, const int8_t *addend, float sr, int32_t r_off, int8_t *y,
                       float sy, int32_t y_off, const int64_t *p, int act, int32_t *acc);

/* Quantized convolution.  y (int8) may be NULL, acc (int32 accumulators incl. bias) may be NULL. */
int oracle_qconv2d(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw, int32_t w_off,
                   const int32_t *bias, int8_t *y, float sy, int32_t y_off, const int64_t *p, int act,
                   int32_t *acc) {
  return oracle_qconv2d_add(x, sx, x_off, w, sw, w_off, bias, NULL, 1.0f, 0, y, sy, y_off, p, act, acc);
}

/* Quantized convolution with a quantized addend [n][oh][ow][k] (scale sr, offset r_off; NULL: none):
 * acc = sum + bias + rescale(addend - r_off), y = clamp(requantize(acc)).  acc out includes the term. */
int oracle_qconv2d_add(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw, int32_t w_off,
                       const int32_t *bias, const int8_t *addend, float sr, int32_t r_off, int8_t *y,
                       float sy, int32_t y_off, const int64_t *p, int act, int32_t *acc) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
  if (!offsets_ok(x_off, w_off, y_off)) return ORACLE_BAD_QUANT;
  int32_t mant = 0, shift = 0;
  rc = oracle_requant_params(sx, sw, sy, &mant, &shift);
  if (rc) return rc;
  int32_t r_mant = 0, r_shift = 1;
  if (addend) {
    if (r_off < -128 || r_off > 127) return ORACLE_BAD_QUANT;
    rc = oracle_rescale_params(sr, sx, sw, &r_mant, &r_shift);
    if (rc) return rc;
  }
  const int32_t lo = relu_floor(act, y_off);
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
  for (int64_t n = 0; n < cs.n; ++n)
    for (int64_t oh = 0; oh < cs.oh; ++oh)
      for (int64_t ow = 0; ow < cs.ow; ++ow)
        for (int64_t k = 0; k < cs.k; ++k) {
          int32_t a = 0;
          const int64_t o = ((n * cs.oh + oh) * cs.ow + ow) * cs.k + k;
          const int64_t extra = addend ? oracle_rescale_term((int32_t)addend[o] - r_off, r_mant, r_shift) : 0;
          if (qconv_acc_one(x, x_off, w, w_off, bias, extra, &cs, n, oh, ow, k, &a)) { overflow |= 1; continue; }
          if (acc) acc[o] = a;
          if (y) y[o] = (int8_t)oracle_requantize(a, mant, shift, y_off, lo);
        }
  return overflow ? ORACLE_ACC_OVERFLOW : ORACLE_OK;
}

int oracle_qconv2d_add_points(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw,
                              int32_t w_off, const int32_t *bias, const int8_t *addend, float sr,
                              int32_t r_off, float sy, int32_t y_off, const int64_t *p, int act,
                              const int64_t *flat_idx, int64_t n_idx, int8_t *out);

int oracle_qconv2d_points(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw,
                          int32_t w_off, const int32_t *bias, float sy, int32_t y_off, const int64_t *p,
                          int act, const int64_t *flat_idx, int64_t n_idx, int8_t *out) {
  return oracle_qconv2d_add_points(x, sx, x_off, w, sw, w_off, bias, NULL, 1.0f, 0, sy, y_off, p, act,
                                   flat_idx, n_idx, out);
}

int oracle_qconv2d_add_points(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw,
                              int32_t w_off, const int32_t *bias, const int8_t *addend, float sr,
                              int32_t r_off, float sy, int32_t y_off, const int64_t *p, int act,
                              const int64_t *flat_idx, int64_t n_idx, int8_t *out) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
  if (!offsets_ok(x_off, w_off, y_off)) return ORACLE_BAD_QUANT;
  int32_t mant = 0, shift = 0;
  rc = oracle_requant_params(sx, sw, sy, &mant, &shift);
  if (rc) return rc;
  int32_t r_mant = 0, r_shift = 1;
  if (addend) {
    if (r_off < -128 || r_off > 127) return ORACLE_BAD_QUANT;
    rc = oracle_rescale_params(sr, sx, sw, &r_mant, &r_shift);
    if (rc) return rc;
  }
  const int32_t lo = relu_floor(act, y_off);
  const int64_t total = cs.n * cs.oh * cs.ow * cs.k;
  for (int64_t i = 0; i < n_idx; ++i)
    if (flat_idx[i] < 0 || flat_idx[i] >= total) return ORACLE_BAD_SHAPE;
  int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
  for (int64_t i = 0; i < n_idx; ++i) {
    int64_t f = flat_idx[i];
    const int64_t k = f % cs.k; f /= cs.k;
    const int64_t ow = f % cs.ow; f /= cs.ow;
    const int64_t oh = f % cs.oh; f /= cs.oh;
    int32_t a = 0;
    const int64_t extra =
        addend ? oracle_rescale_term((int32_t)addend[flat_idx[i]] - r_off, r_mant, r_shift) : 0;
    if (qconv_acc_one(x, x_off, w, w_off, bias, extra, &cs, f, oh, ow, k, &a)) { overflow |= 1; continue; }
    out[i] = (int8_t)oracle_requantize(a, mant, shift, y_off, lo);
  }
  return overflow ? ORACLE_ACC_OVERFLOW : ORACLE_OK;
}

/* Quantized fully connected: A[M][K] (int8), W[K][N] (int8), bias[N] (int32). */
int oracle_qfc(const int8_t *a, float sa, int32_t a_off, const int8_t *w, float sw, int32_t w_off,
               const int32_t *bias, int8_t *y, float sy, int32_t y_off, int64_t M, int64_t K, int64_t N,
               int act, int32_t *acc) {
  if (M <= 0 || K <= 0 || N <= 0) return ORACLE_BAD_SHAPE;
  if (!offsets_ok(a_off, w_off, y_off)) return ORACLE_BAD_QUANT;
  int32_t mant = 0, shift = 0;
  int rc = oracle_requant_params(sa, sw, sy, &mant, &shift);
  if (rc) return rc;
  const int32_t lo = relu_floor(act, y_off);
  int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      int64_t s = 0;
      for (int64_t k = 0; k < K; ++k)
        s += ((int64_t)a[m * K + k] - a_off) * ((int64_t)w[k * N + n] - w_off);
      if (bias) s += (int64_t)bias[n];
      if (s > INT32_MAX || s < INT32_MIN) { overflow |= 1; continue; }
      if (acc) acc[m * N + n] = (int32_t)s;
      if (y) y[m * N + n] = (int8_t)oracle_requantize((int32_t)s, mant, shift, y_off, lo);
    }
  return overflow ? ORACLE_ACC_OVERFLOW : ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * General element-wise chains behind the contraction (Section 5.2: operator stacking of consecutive
 * data-parallel operators).  An op list is applied in the order given to every output element.
 * ---------------------------------------------------------------------------------------------- */
enum { ORACLE_OP_ADD_TENSOR = 1, ORACLE_OP_MUL_SCALAR = 2, ORACLE_OP_MAX_SCALAR = 3, ORACLE_OP_CLIP = 4 };

typedef struct {
  int32_t kind;          /* ORACLE_OP_*                                                        */
  float a, b;            /* MUL: factor a; MAX: threshold a; CLIP: bounds a <= b                */
  const void *tensor;    /* ADD_TENSOR: [n][oh][ow][k] like the output (float, or int8 codes)   */
  float t_scale;         /* quantized ADD_TENSOR: the tensor's scale                            */
  int32_t t_offset;      /*                       and offset                                    */
} oracle_chain_op;

/* fp32: y = chain(conv + bias), every step in double, one rounding at the end. */
int oracle_conv2d_f32_chain(const float *x, const float *w, const float *bias, const oracle_chain_op *ops,
                            int32_t n_ops, float *y, const int64_t *p) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
  if (n_ops < 0 || (n_ops > 0 && !ops)) return ORACLE_BAD_SHAPE;
  for (int32_t i = 0; i < n_ops; ++i) {
    if (ops[i].kind < ORACLE_OP_ADD_TENSOR || ops[i].kind > ORACLE_OP_CLIP) return ORACLE_BAD_SHAPE;
    if (ops[i].kind == ORACLE_OP_ADD_TENSOR && !ops[i].tensor) return ORACLE_BAD_SHAPE;
    if (ops[i].kind == ORACLE_OP_CLIP && !(ops[i].a <= ops[i].b)) return ORACLE_BAD_SHAPE;
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < cs.n; ++n)
    for (int64_t oh = 0; oh < cs.oh; ++oh)
      for (int64_t ow = 0; ow < cs.ow; ++ow)
        for (int64_t k = 0; k < cs.k; ++k) {
          const int64_t o = ((n * cs.oh + oh) * cs.ow + ow) * cs.k + k;
          /* the contraction and the bias exactly as in conv_f32_one, kept in double */
          const int64_t cg = cs.c / cs.groups, kg = cs.k / cs.groups, g = k / kg;
          double v = 0.0;
          for (int64_t r = 0; r < cs.r; ++r) {
            const int64_t ih = oh * cs.stride_h - cs.pad_t + r;
            if (ih < 0 || ih >= cs.h) continue;
            for (int64_t s = 0; s < cs.s; ++s) {
              const int64_t iw = ow * cs.stride_w - cs.pad_l + s;
              if (iw < 0 || iw >= cs.w) continue;
              for (int64_t cc = 0; cc < cg; ++cc)
                v += (double)x[((n * cs.h + ih) * cs.w + iw) * cs.c + g * cg + cc] *
                     (double)w[((k * cs.r + r) * cs.s + s) * cg + cc];
            }
          }
          if (bias) v += (double)bias[k];
          for (int32_t i = 0; i < n_ops; ++i) {
            const oracle_chain_op *op = &ops[i];
            if (op->kind == ORACLE_OP_ADD_TENSOR) v += (double)((const float *)op->tensor)[o];
            else if (op->kind == ORACLE_OP_MUL_SCALAR) v *= (double)op->a;
            else if (op->kind == ORACLE_OP_MAX_SCALAR) { if (v < (double)op->a) v = (double)op->a; }
            else { if (v < (double)op->a) v = (double)op->a; if (v > (double)op->b) v = (double)op->b; }
          }
          y[o] = (float)v;
        }
  return ORACLE_OK;
}

/* A positive real multiplier as mant * 2^-shift, mant in [2^30, 2^31), shift in [1, 62]. */
static int multiplier_to_fixed(double mr, int32_t *mant, int32_t *shift) {
  if (!(mr > 0.0) || isinf(mr)) return ORACLE_BAD_QUANT;
  int e = 0;
  const double f = frexp(mr, &e);
  int64_t m = llround(f * 2147483648.0);
  if (m == 2147483648LL) { m = 1073741824LL; e += 1; }
  const int sh = 31 - e;
  if (sh < 1 || sh > 62) return ORACLE_BAD_QUANT;
  *mant = (int32_t)m;
  *shift = (int32_t)sh;
  return ORACLE_OK;
}

/* A real threshold v on the accumulator's grid of step s: floor(v / s + 0.5), saturated to int32. */
int32_t oracle_chain_threshold(float v, double s) {
  const double t = floor((double)v / s + 0.5);
  if (t != t) return 0;
  if (t <= -2147483648.0) return INT32_MIN;
  if (t >= 2147483647.0) return INT32_MAX;
  return (int32_t)t;
}

/* Quantized: the chain on the int32 accumulator (see the readings at the top), then one requantize.
 * acc_out (may be NULL) receives the accumulator after the chain. */
int oracle_qconv2d_chain(const int8_t *x, float sx, int32_t x_off, const int8_t *w, float sw, int32_t w_off,
                         const int32_t *bias, const oracle_chain_op *ops, int32_t n_ops, int8_t *y, float sy,
                         int32_t y_off, const int64_t *p, int32_t *acc_out) {
  conv_shape cs;
  int rc = conv_shape_init(&cs, p);
  if (rc) return rc;
  if (!offsets_ok(x_off, w_off, y_off)) return ORACLE_BAD_QUANT;
  if (!(sx > 0.0f) || !(sw > 0.0f) || !(sy > 0.0f) || isinf(sx) || isinf(sw) || isinf(sy)) return ORACLE_BAD_QUANT;
  if (n_ops < 0 || n_ops > 16 || (n_ops > 0 && !ops)) return ORACLE_BAD_SHAPE;
  /* per-op integer parameters, from the scale the accumulator has when the op is reached */
  int32_t t_lo[16], t_hi[16], a_mant[16], a_shift[16];
  double s = (double)sx * (double)sw;
  for (int32_t i = 0; i < n_ops; ++i) {
    const oracle_chain_op *op = &ops[i];
    t_lo[i] = t_hi[i] = a_mant[i] = 0; a_shift[i] = 1;
    if (op->kind == ORACLE_OP_ADD_TENSOR) {
      if (!op->tensor || op->t_offset < -128 || op->t_offset > 127) return ORACLE_BAD_QUANT;
      if (!(op->t_scale > 0.0f) || isinf(op->t_scale)) return ORACLE_BAD_QUANT;
      rc = multiplier_to_fixed((double)op->t_scale / s, &a_mant[i], &a_shift[i]);
      if (rc) return rc;
    } else if (op->kind == ORACLE_OP_MUL_SCALAR) {
      if (!(op->a > 0.0f) || isinf(op->a)) return ORACLE_BAD_QUANT;
      s = s * (double)op->a;
      if (!(s > 0.0) || isinf(s)) return ORACLE_BAD_QUANT;
    } else if (op->kind == ORACLE_OP_MAX_SCALAR) {
      if (op->a != op->a) return ORACLE_BAD_QUANT;
      t_lo[i] = oracle_chain_threshold(op->a, s);
    } else if (op->kind == ORACLE_OP_CLIP) {
      if (!(op->a <= op->b)) return ORACLE_BAD_QUANT;
      t_lo[i] = oracle_chain_threshold(op->a, s);
      t_hi[i] = oracle_chain_threshold(op->b, s);
    } else {
      return ORACLE_BAD_SHAPE;
    }
  }
  int32_t mant = 0, shift = 0;
  rc = multiplier_to_fixed(s / (double)sy, &mant, &shift);
  if (rc) return rc;
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
  for (int64_t n = 0; n < cs.n; ++n)
    for (int64_t oh = 0; oh < cs.oh; ++oh)
      for (int64_t ow = 0; ow < cs.ow; ++ow)
        for (int64_t k = 0; k < cs.k; ++k) {
          const int64_t o = ((n * cs.oh + oh) * cs.ow + ow) * cs.k + k;
          int32_t a32 = 0;
          if (qconv_acc_one(x, x_off, w, w_off, bias, 0, &cs, n, oh, ow, k, &a32)) { overflow |= 1; continue; }
          int64_t a = a32;
          int bad = 0;
          for (int32_t i = 0; i < n_ops; ++i) {
            const oracle_chain_op *op = &ops[i];
            if (op->kind == ORACLE_OP_ADD_TENSOR) {
              a += oracle_rescale_term((int32_t)((const int8_t *)op->tensor)[o] - op->t_offset, a_mant[i], a_shift[i]);
              if (a > INT32_MAX || a < INT32_MIN) { bad = 1; break; }
            } else if (op->kind == ORACLE_OP_MAX_SCALAR) {
              if (a < t_lo[i]) a = t_lo[i];
            } else if (op->kind == ORACLE_OP_CLIP) {
              if (a < t_lo[i]) a = t_lo[i];
              if (a > t_hi[i]) a = t_hi[i];
            }                                     /* MUL_SCALAR: nothing happens to the integer */
          }
          if (bad) { overflow |= 1; continue; }
          if (acc_out) acc_out[o] = (int32_t)a;
          if (y) y[o] = (int8_t)oracle_requantize((int32_t)a, mant, shift, y_off, -128);
        }
  return overflow ? ORACLE_ACC_OVERFLOW : ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Batch normalization merged into the convolution in front of it (Section 5.3):
 *   gamma * (conv(x, w) + b - mean) / sqrt(var + eps) + beta  ==  conv(x, w') + b'
 *   w'[k][...] = w[k][...] * gamma[k] / sqrt(var[k] + eps)
 *   b'[k]      = (b[k] - mean[k]) * gamma[k] / sqrt(var[k] + eps) + beta[k]
 * evaluated in double, rounded once.  per = elements of one filter; bias may be NULL (zeros).
 * ---------------------------------------------------------------------------------------------- */
int oracle_fold_batchnorm(const float *w, const float *bias, const float *gamma, const float *beta,
                          const float *mean, const float *var, float eps, int64_t k, int64_t per, float *w_out,
                          float *b_out) {
  if (k <= 0 || per <= 0) return ORACLE_BAD_SHAPE;
  for (int64_t i = 0; i < k; ++i) {
    const double denom = (double)var[i] + (double)eps;
    if (!(denom > 0.0) || isinf(denom)) return ORACLE_BAD_SHAPE;
  }
  for (int64_t i = 0; i < k; ++i) {
    const double scale = (double)gamma[i] / sqrt((double)var[i] + (double)eps);
    for (int64_t e = 0; e < per; ++e) w_out[i * per + e] = (float)((double)w[i * per + e] * scale);
    const double b = bias ? (double)bias[i] : 0.0;
    b_out[i] = (float)((b - (double)mean[i]) * scale + (double)beta[i]);
  }
  return ORACLE_OK;
}
