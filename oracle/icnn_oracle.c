/*
 * CPU oracle for the integer-arithmetic-only convolution layer of
 * "Efficient Integer-Arithmetic-Only Convolutional Neural Networks".
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to say what the right answer is:
 * plain loops, 64-bit arithmetic, nothing blocked, fused or reordered.  Only
 * tests, the smoke check and the benchmark's CPU-baseline leg may use it; the
 * GPU library never links, loads or calls it, and shares no code with it.
 *
 * What it computes (Section 3.1, Figure 1 and the requantisation equation of
 * Section 3.2.1; Sections 3.4.1 and 3.4.2; Section 4.1 on residual blocks;
 * Algorithm 2 on concatenation):
 *
 *   U = X (*) W                    integer convolution, zero outside the image
 *   Y = U + b                      int32 bias
 *   T = Y (+ rescaled skip)        ratio synchronisation at a residual merge
 *   V = clamp([T * mul / 2^shift], 0, max_int)   BReLU + activation requantisation
 *
 * Readings fixed where the paper is silent:
 *   - [.] is round-half-up, floor(x + 1/2), for negative values too; a shift of
 *     zero adds no rounding term.
 *   - BReLU followed by requantisation equals requantisation followed by a clamp
 *     to max_int whenever mul > 0 (the map is monotone and sends h_i to max_int),
 *     so the clamp is applied to the requantised value.
 *   - Zero padding is zero in the integer domain, i.e. after the first layer's
 *     "subtract 128" re-normalisation, not before it.
 *   - The skip operand is rescaled by its own multiplier and shift and added in
 *     the Y domain, before BReLU; the sum saturates to int32.
 *   - A regression network's last layer requantises to pixel units, adds the raw
 *     picture and clamps to [0, 255].
 *   - Pooling: max over the valid window; global average is a sum followed by
 *     the same multiply-shift-round-clamp with mul / 2^shift ~ 1 / (H*W).
 *
 *   - Section 3.4.3 trains with one weight step per output channel before batch
 *     normalisation is merged, which leaves every output channel with its own
 *     ratio; orc_conv2d_pc therefore takes the requantisation pair (and the skip
 *     rescale pair) per output channel.  The paper does not spell this out; the
 *     arithmetic per channel is the per-layer one.  Pinned by running the
 *     per-layer function once per channel.
 *
 * Pins (tests marked "not gpu"): the rounding rule against exact rationals,
 * hand-computed cases, the convolution against a seven-loop brute force, a
 * float64 library convolution and an int64 matrix product, shifted-copy and
 * box-sum kernels, add / concat / pool identities.
 */
#include <stdint.h>
#include <stddef.h>

enum { ORC_U8 = 0, ORC_S8 = 1, ORC_S32 = 2 };
enum { ORC_OUT_BRELU_U8 = 0, ORC_OUT_CLAMP_U8 = 1, ORC_OUT_LINEAR_S8 = 2, ORC_OUT_RAW_S32 = 3 };
enum { ORC_RES_NONE = 0, ORC_RES_PRE = 1, ORC_RES_POST = 2 };
enum { ORC_OK = 0, ORC_E_ARG = -1, ORC_E_OVERFLOW = -2 };

typedef struct {
    int32_t n, h, w, cin;
    int32_t in_c_stride;          /* bytes between pixels of x (>= cin)          */
    int32_t in_signed;            /* x bytes are int8 (else uint8)               */
    int32_t in_sub128;            /* x is a raw uint8 picture: use x - 128       */
    int32_t cout, kh, kw, stride_h, stride_w, pad_h, pad_w;
    int32_t out_c_stride, out_c_offset;
    int32_t mul, shift, bound_q;
    int32_t lo, hi;               /* clamp range for ORC_OUT_CLAMP_U8            */
    int32_t out_mode, res_mode, res_dtype, res_c_stride, res_mul, res_shift;
} orc_conv_params;

/* floor(num / 2^s) for any sign, without relying on how >> treats negatives */
static int64_t floor_div_pow2(int64_t num, int s)
{
    int64_t d = (int64_t)1 << s;
    int64_t q = num / d;
    if (num % d < 0) q -= 1;
    return q;
}

/* [v / 2^s]: round half up.  s in [0, 62]; |v| < 2^62 + 2^61 keeps v + half in range. */
int64_t orc_rsr(int64_t v, int32_t s)
{
    if (s <= 0) return v;
    return floor_div_pow2(v + ((int64_t)1 << (s - 1)), s);
}

static int64_t clamp64(int64_t v, int64_t lo, int64_t hi)
{
    return v < lo ? lo : (v > hi ? hi : v);
}

static int64_t sat32(int64_t v)
{
    return clamp64(v, INT32_MIN, INT32_MAX);
}

/* [t * mul / 2^shift] (activation requantisation, Section 3.2.1) */
int64_t orc_requant(int64_t t, int32_t mul, int32_t shift)
{
    return orc_rsr(t * (int64_t)mul, shift);
}

static int64_t load_elem(const void *p, size_t i, int dtype)
{
    switch (dtype) {
    case ORC_U8:  return ((const uint8_t *)p)[i];
    case ORC_S8:  return ((const int8_t *)p)[i];
    default:      return ((const int32_t *)p)[i];
    }
}

static void out_range(int out_mode, int bound_q, int lo, int hi, int64_t *rlo, int64_t *rhi)
{
    if (out_mode == ORC_OUT_BRELU_U8)      { *rlo = 0;    *rhi = bound_q; }
    else if (out_mode == ORC_OUT_CLAMP_U8) { *rlo = lo;   *rhi = hi; }
    else                                   { *rlo = -128; *rhi = 127; }
}

/*
 * One integer conv layer.  x: NHWC 8-bit, pixel pitch in_c_stride.  w: int8
 * [cout][kh][kw][cin].  bias: int32 [cout].  res: skip operand, NHWC over the
 * output pixels with pitch res_c_stride, or NULL.  out: NHWC with pitch
 * out_c_stride; channel co lands at out_c_offset + co (this is how branches of
 * a concatenation share a buffer); elements are uint8, int8 or int32 by out_mode.
 */
/*
 * mul_c, shift_c, res_mul_c, res_shift_c: int32 [cout] each, or NULL to use the
 * per-layer value of *p for that quantity (Section 3.4.3: per-channel ratios).
 */
int orc_conv2d_pc(const orc_conv_params *p, const void *x, const int8_t *w,
                  const int32_t *bias, const void *res, void *out,
                  const int32_t *mul_c, const int32_t *shift_c,
                  const int32_t *res_mul_c, const int32_t *res_shift_c)
{
    if (!p || !x || !w || !bias || !out) return ORC_E_ARG;
    if (p->res_mode != ORC_RES_NONE && !res) return ORC_E_ARG;
    const int ho_n = (p->h + 2 * p->pad_h - p->kh) / p->stride_h + 1;
    const int wo_n = (p->w + 2 * p->pad_w - p->kw) / p->stride_w + 1;
    if (ho_n <= 0 || wo_n <= 0) return ORC_E_ARG;
    int64_t rlo, rhi;
    out_range(p->out_mode, p->bound_q, p->lo, p->hi, &rlo, &rhi);
    int status = ORC_OK;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < p->n; ++n) {
        for (int ho = 0; ho < ho_n; ++ho) {
            for (int wo = 0; wo < wo_n; ++wo) {
                const size_t pix = ((size_t)n * ho_n + ho) * wo_n + wo;
                for (int co = 0; co < p->cout; ++co) {
                    int64_t u = 0;
                    for (int kh = 0; kh < p->kh; ++kh) {
                        const int hi_ = ho * p->stride_h - p->pad_h + kh;
                        if (hi_ < 0 || hi_ >= p->h) continue;          /* zero padding */
                        for (int kw = 0; kw < p->kw; ++kw) {
                            const int wi = wo * p->stride_w - p->pad_w + kw;
                            if (wi < 0 || wi >= p->w) continue;        /* zero padding */
                            const size_t xo = (((size_t)n * p->h + hi_) * p->w + wi) * p->in_c_stride;
                            const int8_t *wr = w + (((size_t)co * p->kh + kh) * p->kw + kw) * p->cin;
                            for (int ci = 0; ci < p->cin; ++ci) {
                                int64_t xv;
                                if (p->in_sub128)      xv = (int64_t)((const uint8_t *)x)[xo + ci] - 128;
                                else if (p->in_signed) xv = ((const int8_t *)x)[xo + ci];
                                else                   xv = ((const uint8_t *)x)[xo + ci];
                                u += xv * (int64_t)wr[ci];
                            }
                        }
                    }
                    if (u > INT32_MAX || u < INT32_MIN) {
#pragma omp atomic write
                        status = ORC_E_OVERFLOW;
                    }
                    int64_t y = u + bias[co];
                    int64_t skip = 0;
                    if (p->res_mode != ORC_RES_NONE) {
                        int64_t r = load_elem(res, pix * p->res_c_stride + co, p->res_dtype);
                        skip = orc_rsr(r * (int64_t)(res_mul_c ? res_mul_c[co] : p->res_mul),
                                       res_shift_c ? res_shift_c[co] : p->res_shift);
                    }
                    int64_t t = (p->res_mode == ORC_RES_PRE) ? sat32(y + skip) : sat32(y);
                    const size_t oi = pix * p->out_c_stride + p->out_c_offset + co;
                    if (p->out_mode == ORC_OUT_RAW_S32) {
                        ((int32_t *)out)[oi] = (int32_t)t;
                        continue;
                    }
                    int64_t q = orc_requant(t, mul_c ? mul_c[co] : p->mul, shift_c ? shift_c[co] : p->shift);
                    if (p->res_mode == ORC_RES_POST) q += skip;
                    q = clamp64(q, rlo, rhi);
                    if (p->out_mode == ORC_OUT_LINEAR_S8) ((int8_t *)out)[oi] = (int8_t)q;
                    else                                  ((uint8_t *)out)[oi] = (uint8_t)q;
                }
            }
        }
    }
    return status;
}

/* The per-layer form: one (mul, shift) and one skip rescale for all channels. */
int orc_conv2d(const orc_conv_params *p, const void *x, const int8_t *w,
               const int32_t *bias, const void *res, void *out)
{
    return orc_conv2d_pc(p, x, w, bias, res, out, NULL, NULL, NULL, NULL);
}

/*
 * Rescaled feature-map addition (ratio synchronisation, Sections 3.4.2 and 4.1):
 *   out = clamp([ sat32(a + [b * b_mul / 2^b_shift]) * mul / 2^shift ], lo, hi)
 * a, b: count_pixels x c elements with pitches a_c_stride / b_c_stride.
 * out_mode ORC_OUT_RAW_S32 stores the saturated sum itself.
 */
int orc_add_rescale(int64_t count_pixels, int32_t c,
                    const void *a, int32_t a_dtype, int32_t a_c_stride,
                    const void *b, int32_t b_dtype, int32_t b_c_stride,
                    int32_t b_mul, int32_t b_shift, int32_t mul, int32_t shift,
                    int32_t lo, int32_t hi, int32_t out_mode,
                    void *out, int32_t out_c_stride, int32_t out_c_offset)
{
    if (!a || !b || !out) return ORC_E_ARG;
    for (int64_t px = 0; px < count_pixels; ++px) {
        for (int ch = 0; ch < c; ++ch) {
            int64_t av = load_elem(a, (size_t)px * a_c_stride + ch, a_dtype);
            int64_t bv = load_elem(b, (size_t)px * b_c_stride + ch, b_dtype);
            int64_t t = sat32(av + orc_rsr(bv * (int64_t)b_mul, b_shift));
            const size_t oi = (size_t)px * out_c_stride + out_c_offset + ch;
            if (out_mode == ORC_OUT_RAW_S32) { ((int32_t *)out)[oi] = (int32_t)t; continue; }
            int64_t q = clamp64(orc_requant(t, mul, shift), lo, hi);
            if (out_mode == ORC_OUT_LINEAR_S8) ((int8_t *)out)[oi] = (int8_t)q;
            else                               ((uint8_t *)out)[oi] = (uint8_t)q;
        }
    }
    return ORC_OK;
}

/*
 * Explicit concatenation with ratio synchronisation (Algorithm 2, online part):
 * input i (uint8, c_in[i] channels) is requantised with its own mul_i, shift_i
 * and clamped to [0, bound_q]; inputs are laid side by side on the channel axis.
 */
int orc_concat(int32_t n_in, const uint8_t *const *in, const int32_t *c_in,
               const int32_t *in_c_stride, const int32_t *mul, const int32_t *shift,
               int32_t bound_q, int64_t count_pixels, uint8_t *out, int32_t out_c_stride)
{
    if (!in || !c_in || !in_c_stride || !mul || !shift || !out) return ORC_E_ARG;
    int off = 0;
    for (int i = 0; i < n_in; ++i) {
        for (int64_t px = 0; px < count_pixels; ++px)
            for (int ch = 0; ch < c_in[i]; ++ch) {
                int64_t v = in[i][(size_t)px * in_c_stride[i] + ch];
                out[(size_t)px * out_c_stride + off + ch] =
                    (uint8_t)clamp64(orc_requant(v, mul[i], shift[i]), 0, bound_q);
            }
        off += c_in[i];
    }
    return ORC_OK;
}

/* Max-pool on uint8 NHWC: maximum over the window positions inside the image. */
int orc_maxpool2d_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t k,
                     int32_t stride, int32_t pad, const uint8_t *x, uint8_t *out)
{
    if (!x || !out) return ORC_E_ARG;
    const int ho_n = (h + 2 * pad - k) / stride + 1, wo_n = (w + 2 * pad - k) / stride + 1;
    for (int in_ = 0; in_ < n; ++in_)
        for (int ho = 0; ho < ho_n; ++ho)
            for (int wo = 0; wo < wo_n; ++wo)
                for (int ch = 0; ch < c; ++ch) {
                    int best = 0;   /* activations are >= 0, so padding never wins */
                    for (int a = 0; a < k; ++a)
                        for (int b = 0; b < k; ++b) {
                            int hi_ = ho * stride - pad + a, wi = wo * stride - pad + b;
                            if (hi_ < 0 || hi_ >= h || wi < 0 || wi >= w) continue;
                            int v = x[(((size_t)in_ * h + hi_) * w + wi) * c + ch];
                            if (v > best) best = v;
                        }
                    out[(((size_t)in_ * ho_n + ho) * wo_n + wo) * c + ch] = (uint8_t)best;
                }
    return ORC_OK;
}

/* Global average pool: clamp([sum * mul / 2^shift], 0, bound_q), out is [n][c]. */
int orc_avgpool_global_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t mul,
                          int32_t shift, int32_t bound_q, const uint8_t *x, uint8_t *out)
{
    if (!x || !out) return ORC_E_ARG;
    for (int in_ = 0; in_ < n; ++in_)
        for (int ch = 0; ch < c; ++ch) {
            int64_t s = 0;
            for (int i = 0; i < h * w; ++i) s += x[((size_t)in_ * h * w + i) * c + ch];
            out[(size_t)in_ * c + ch] = (uint8_t)clamp64(orc_requant(s, mul, shift), 0, bound_q);
        }
    return ORC_OK;
}

/* Re-normalisation of a raw picture (Section 3.4.1): every uint8 sample minus 128, as int8. */
int orc_renormalize_u8(int64_t count, const uint8_t *x, int8_t *out)
{
    if (count < 0 || (count > 0 && (!x || !out))) return ORC_E_ARG;
    for (int64_t i = 0; i < count; ++i) out[i] = (int8_t)((int)x[i] - 128);
    return ORC_OK;
}

/* Threads the parallel loops above will use (for reporting beside timings). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
