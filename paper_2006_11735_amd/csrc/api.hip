// C boundary: argument validation (host only, before any launch) and dispatch.
#include "../../include/icnn.h"
#include "icnn_device.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

using namespace icnn;

namespace icnn {
Tuning g_tuning;
}

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

struct ConvGeom {
    int ho, wo, K, ksteps, chunks;
    long long M;
    // small-cin layers (cin <= 4) run on a zero-bordered 4-channel copy of x in the workspace:
    // rp = bytes of one kernel row there (kw * 4 rounded up to 16), hp x wp = its spatial size
    int rp, hp, wp;
    size_t ws_bytes;
};

int check_conv(const icnn_conv_desc *d, ConvGeom *g)
{
    if (!d) return fail(ICNN_E_NULL, "conv descriptor is NULL");
    if (d->n < 1 || d->h < 1 || d->w < 1 || d->cin < 1 || d->cout < 1 || d->kh < 1 || d->kw < 1)
        return fail(ICNN_E_SHAPE, "n, h, w, cin, cout, kh, kw must be >= 1");
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return fail(ICNN_E_SHAPE, "stride must be >= 1 and pad >= 0");
    if (d->h + 2LL * d->pad_h < d->kh || d->w + 2LL * d->pad_w < d->kw)
        return fail(ICNN_E_SHAPE, "kernel larger than the padded image");
    const int ho = (d->h + 2 * d->pad_h - d->kh) / d->stride_h + 1;
    const int wo = (d->w + 2 * d->pad_w - d->kw) / d->stride_w + 1;
    const long long K = (long long)d->kh * d->kw * d->cin;
    if (K > 65535)
        return fail(ICNN_E_SHAPE, "kh*kw*cin = %lld exceeds 65535: int32 accumulation not provably safe", K);
    if (d->in_signed == ICNN_IN_U8_FULL && K > 32767)
        return fail(ICNN_E_SHAPE, "kh*kw*cin = %lld exceeds 32767 with inputs up to 255: int32 accumulation not provably safe", K);
    const long long M = (long long)d->n * ho * wo;
    if (M > 0x7fffffffLL) return fail(ICNN_E_SHAPE, "n*ho*wo = %lld does not fit int32", M);
    if (d->in_c_stride < d->cin) return fail(ICNN_E_SHAPE, "in_c_stride %d < cin %d", d->in_c_stride, d->cin);
    if (d->out_c_offset < 0 || (long long)d->out_c_offset + d->cout > d->out_c_stride)
        return fail(ICNN_E_SHAPE, "out_c_offset %d + cout %d exceeds out_c_stride %d", d->out_c_offset, d->cout,
                    d->out_c_stride);
    if (d->in_signed < ICNN_IN_U8_LE127 || d->in_signed > ICNN_IN_U8_FULL || (d->in_sub128 != 0 && d->in_sub128 != 1) ||
        (d->in_signed && d->in_sub128))
        return fail(ICNN_E_PARAM, "in_signed must be 0, 1 or 2, in_sub128 0 or 1 and only with in_signed = 0");
    if (d->out_mode < ICNN_OUT_BRELU_U8 || d->out_mode > ICNN_OUT_RAW_S32)
        return fail(ICNN_E_PARAM, "unknown out_mode %d", d->out_mode);
    if (d->res_mode < ICNN_RES_NONE || d->res_mode > ICNN_RES_POST)
        return fail(ICNN_E_PARAM, "unknown res_mode %d", d->res_mode);
    if (d->out_mode != ICNN_OUT_RAW_S32) {
        if (d->mul < 1) return fail(ICNN_E_PARAM, "mul %d must be in [1, 2^31)", d->mul);
        if (d->shift < 0 || d->shift > 62) return fail(ICNN_E_PARAM, "shift %d must be in [0, 62]", d->shift);
    }
    if (d->out_mode == ICNN_OUT_BRELU_U8 && (d->bound_q < 1 || d->bound_q > 255))
        return fail(ICNN_E_PARAM, "bound_q %d must be in [1, 255]", d->bound_q);
    if (d->out_mode == ICNN_OUT_CLAMP_U8 && (d->lo < 0 || d->hi > 255 || d->lo > d->hi))
        return fail(ICNN_E_PARAM, "clamp range [%d, %d] must satisfy 0 <= lo <= hi <= 255", d->lo, d->hi);
    if (d->res_mode != ICNN_RES_NONE) {
        if (d->res_dtype < ICNN_U8 || d->res_dtype > ICNN_S32)
            return fail(ICNN_E_PARAM, "unknown res_dtype %d", d->res_dtype);
        if (d->res_c_stride < d->cout)
            return fail(ICNN_E_SHAPE, "res_c_stride %d < cout %d", d->res_c_stride, d->cout);
        if (d->res_mul < 1) return fail(ICNN_E_PARAM, "res_mul %d must be in [1, 2^31)", d->res_mul);
        if (d->res_shift < 0 || d->res_shift > 62)
            return fail(ICNN_E_PARAM, "res_shift %d must be in [0, 62]", d->res_shift);
        if (d->res_mode == ICNN_RES_POST && d->out_mode == ICNN_OUT_RAW_S32)
            return fail(ICNN_E_PARAM, "a skip operand after requantisation needs a requantised output");
    }
    if (g) {
        g->ho = ho;
        g->wo = wo;
        g->K = (int)K;
        g->M = M;
        g->rp = g->hp = g->wp = 0;
        g->ws_bytes = 0;
        if (d->cin <= 4) {
            g->rp = (d->kw * 4 + 15) / 16 * 16;
            g->hp = d->h + 2 * d->pad_h;
            const int need = (wo - 1) * d->stride_w + g->rp / 4;
            g->wp = d->w + 2 * d->pad_w > need ? d->w + 2 * d->pad_w : need;
            g->K = d->kh * g->rp;
            const unsigned long long wsb = (unsigned long long)d->n * g->hp * g->wp * 4 + 64 + kWsCounterBytes;
            if (wsb > 0x7fffffffull) return fail(ICNN_E_SHAPE, "small-cin workspace of %llu bytes exceeds 2 GiB", wsb);
            g->ws_bytes = (size_t)wsb;
        }
        g->ksteps = (g->K + kStepK - 1) / kStepK;
        g->chunks = ((d->cout + kCoutPad - 1) / kCoutPad) * (kCoutPad / kChunkCout);
    }
    return ICNN_OK;
}

int check_requant(int mul, int shift, const char *what)
{
    if (mul < 1) return fail(ICNN_E_PARAM, "%s multiplier %d must be in [1, 2^31)", what, mul);
    if (shift < 0 || shift > 62) return fail(ICNN_E_PARAM, "%s shift %d must be in [0, 62]", what, shift);
    return ICNN_OK;
}

int launched(hipError_t e, const char *what)
{
    if (e == hipSuccess) return ICNN_OK;
    return fail(ICNN_E_LAUNCH, "%s: %s", what, hipGetErrorString(e));
}

int dtype_bytes(int dt) { return dt == ICNN_S32 ? 4 : 1; }

}  // namespace

extern "C" {

int icnn_version(void) { return 100; }

const char *icnn_last_error(void) { return g_err; }

int icnn_set_tuning(const char *name, int32_t value)
{
    if (!name) return fail(ICNN_E_NULL, "tuning name is NULL");
    struct Entry { const char *name; int Tuning::*field; int lo, hi; };
    static const Entry table[] = {
        {"tile", &Tuning::tile, -1, 4},         {"stages", &Tuning::stages, 0, 6},
        {"no_narrow", &Tuning::no_narrow, 0, 1}, {"no_fc", &Tuning::no_fc, 0, 1},
        {"no_halo", &Tuning::no_halo, 0, 1},     {"halo_tile", &Tuning::halo_tile, 0, 2},
        {"halo_always", &Tuning::halo_always, 0, 1}, {"no_stream", &Tuning::no_stream, 0, 1},
        {"ksplit", &Tuning::ksplit, 0, 8}, {"no_block64", &Tuning::no_block64, 0, 1},
        {"no_plane", &Tuning::no_plane, 0, 1}, {"no_pic", &Tuning::no_pic, 0, 1}, {"block_any_form", &Tuning::block_any_form, 0, 1}, {"plane_no_pipe", &Tuning::plane_no_pipe, 0, 1}, {"plane_always", &Tuning::plane_always, 0, 1},
        {"no_deep", &Tuning::no_deep, 0, 1}, {"deep_always", &Tuning::deep_always, 0, 1}, {"deep_plain_walk", &Tuning::deep_plain_walk, 0, 1},
    };
    if (!strcmp(name, "reset")) {
        g_tuning = Tuning();
        return ICNN_OK;
    }
    for (const Entry &e : table)
        if (!strcmp(name, e.name)) {
            if (value < e.lo || value > e.hi || (e.field == &Tuning::stages && value == 1))
                return fail(ICNN_E_PARAM, "tuning %s = %d outside [%d, %d]", name, value, e.lo, e.hi);
            g_tuning.*(e.field) = value;
            return ICNN_OK;
        }
    return fail(ICNN_E_PARAM, "unknown tuning name %s", name);
}

int iconv2d_validate(const icnn_conv_desc *desc) { return check_conv(desc, nullptr); }

int iconv2d_out_hw(const icnn_conv_desc *desc, int32_t *ho, int32_t *wo)
{
    ConvGeom g;
    const int rc = check_conv(desc, &g);
    if (rc) return rc;
    if (!ho || !wo) return fail(ICNN_E_NULL, "ho / wo is NULL");
    *ho = g.ho;
    *wo = g.wo;
    return ICNN_OK;
}

static int fill_conv_args(const icnn_conv_desc *d, const ConvGeom &g, const void *x, const void *w_packed,
                          const int32_t *bias, const void *res, void *y, ConvArgs &a);

// Workspace of a layer: the padded copy of a small-cin layer, or the partial accumulators of a K axis split over
// workgroups (decided as the launch will decide, for 16-byte aligned tensors), behind the counter block.
static int workspace_need(const icnn_conv_desc *d, const ConvGeom &g, size_t *bytes)
{
    *bytes = g.ws_bytes;
    if (g.ws_bytes) return ICNN_OK;
    ConvArgs a;
    void *const dummy = (void *)(uintptr_t)4096;        // aligned stand-ins: only shapes and parameters matter here
    const int rc = fill_conv_args(d, g, dummy, dummy, (const int32_t *)dummy, d->res_mode != ICNN_RES_NONE ? dummy : nullptr, dummy, a);
    if (rc) return rc;
    const bool vec_in = d->cin % 16 == 0 && d->in_c_stride % 16 == 0;
    a.ws_cnt = (unsigned *)dummy;
    a.ws_part = (int32_t *)dummy;
    const size_t part = conv_split_bytes(a, vec_in);
    *bytes = part ? part + kWsCounterBytes : 0;
    return ICNN_OK;
}

int iconv2d_workspace_bytes(const icnn_conv_desc *desc, size_t *bytes)
{
    ConvGeom g;
    const int rc = check_conv(desc, &g);
    if (rc) return rc;
    if (!bytes) return fail(ICNN_E_NULL, "bytes is NULL");
    return workspace_need(desc, g, bytes);
}

int iconv2d_packed_weight_bytes(const icnn_conv_desc *desc, size_t *bytes)
{
    ConvGeom g;
    const int rc = check_conv(desc, &g);
    if (rc) return rc;
    if (!bytes) return fail(ICNN_E_NULL, "bytes is NULL");
    // the fragment-ordered weights, then one int32 per (padded) output channel: the sum of its weights
    *bytes = (size_t)g.chunks * g.ksteps * kChunkBytes + (size_t)g.chunks * kChunkCout * sizeof(int32_t);
    return ICNN_OK;
}

int iconv2d_prepack_weights(const icnn_conv_desc *desc, const int8_t *w_ohwi, void *w_packed, void *stream)
{
    ConvGeom g;
    const int rc = check_conv(desc, &g);
    if (rc) return rc;
    if (!w_ohwi || !w_packed) return fail(ICNN_E_NULL, "weight pointer is NULL");
    if (!aligned16(w_packed)) return fail(ICNN_E_ALIGN, "w_packed must be 16-byte aligned");
    const hipError_t e = launch_wsum(w_ohwi, (int32_t *)((uint8_t *)w_packed + (size_t)g.chunks * g.ksteps * kChunkBytes),
                                     desc->cout, g.chunks * kChunkCout, desc->kh * desc->kw * desc->cin, (hipStream_t)stream);
    if (e != hipSuccess) return launched(e, "prepack (weight sums)");
    return launched(launch_prepack(w_ohwi, (uint8_t *)w_packed, desc->cout, g.K, g.chunks, g.ksteps, desc->kh,
                                   desc->kw, desc->cin, g.rp, (hipStream_t)stream),
                    "prepack");
}

// Validates pointers and fills the kernel arguments of one conv layer.
static int fill_conv_args(const icnn_conv_desc *d, const ConvGeom &g, const void *x, const void *w_packed,
                          const int32_t *bias, const void *res, void *y, ConvArgs &a)
{
    if (!x || !w_packed || !bias || !y) return fail(ICNN_E_NULL, "x, w_packed, bias and y must not be NULL");
    if (d->res_mode != ICNN_RES_NONE && !res) return fail(ICNN_E_NULL, "res is NULL but res_mode is set");
    if (!aligned16(w_packed)) return fail(ICNN_E_ALIGN, "w_packed must be 16-byte aligned");
    if ((uintptr_t)bias & 3) return fail(ICNN_E_ALIGN, "bias must be 4-byte aligned");
    if (d->out_mode == ICNN_OUT_RAW_S32 && ((uintptr_t)y & 3)) return fail(ICNN_E_ALIGN, "int32 output must be 4-byte aligned");
    if (d->res_mode != ICNN_RES_NONE && d->res_dtype == ICNN_S32 && ((uintptr_t)res & 3))
        return fail(ICNN_E_ALIGN, "int32 skip operand must be 4-byte aligned");

    a.x = (const uint8_t *)x;
    a.wp = (const uint8_t *)w_packed;
    a.bias = bias;
    a.res = d->res_mode != ICNN_RES_NONE ? res : nullptr;
    a.out = y;
    a.N = d->n; a.H = d->h; a.W = d->w; a.Cin = d->cin; a.in_cs = d->in_c_stride;
    a.Cout = d->cout; a.KH = d->kh; a.KW = d->kw;
    a.sh = d->stride_h; a.sw = d->stride_w; a.ph = d->pad_h; a.pw = d->pad_w;
    a.Ho = g.ho; a.Wo = g.wo; a.M = (int)g.M; a.K = g.K; a.ksteps = g.ksteps; a.n_ct = 0;
    a.out_cs = d->out_c_stride; a.out_co = d->out_c_offset;
    a.mul = d->mul; a.shift = d->shift; a.out_mode = d->out_mode;
    switch (d->out_mode) {
    case ICNN_OUT_BRELU_U8: a.lo = 0; a.hi = d->bound_q; break;
    case ICNN_OUT_CLAMP_U8: a.lo = d->lo; a.hi = d->hi; break;
    default: a.lo = -128; a.hi = 127; break;
    }
    if (d->out_mode == ICNN_OUT_RAW_S32) { a.mul = 1; a.shift = 0; }
    // [t * 2m / 2^s] = [t * m / 2^(s-1)] for every t (numerator and denominator halve exactly): the smaller pair
    // lets more layers requantise in 32 bits
    while (a.shift >= 2 && a.mul != 0 && (a.mul & 1) == 0) { a.mul /= 2; --a.shift; }
    a.res_mode = d->res_mode; a.res_dtype = d->res_dtype; a.res_cs = d->res_c_stride;
    a.res_mul = d->res_mode ? d->res_mul : 1; a.res_shift = d->res_mode ? d->res_shift : 0;
    a.in_xor = d->in_sub128 ? 0x80808080u : 0u;
    a.frag_xor = d->in_signed == ICNN_IN_U8_FULL ? 0x80808080u : 0u;
    a.wsum = (const int32_t *)((const uint8_t *)w_packed + (size_t)g.chunks * g.ksteps * kChunkBytes);
    const int ob = d->out_mode == ICNN_OUT_RAW_S32 ? 4 : 1;
    a.vec_out = aligned16(y) && ((long long)d->out_c_stride * ob) % 16 == 0 && ((long long)d->out_c_offset * ob) % 16 == 0;
    a.vec_res = 0;
    a.vec_bias = aligned16(bias) && d->cout % 16 == 0;
    if (d->res_mode != ICNN_RES_NONE) {
        const int rb = dtype_bytes(d->res_dtype);
        a.vec_res = aligned16(res) && ((long long)d->res_c_stride * rb) % 16 == 0;
    }
    {
        // bytes of x up to the end of the last pixel's channel slice, and of the packed weights
        const unsigned long long xb = ((unsigned long long)d->n * d->h * d->w - 1) * d->in_c_stride + d->cin;
        const unsigned long long wb = (unsigned long long)g.chunks * g.ksteps * kChunkBytes;
        a.x_bytes = xb > 0xffffffffull ? 0xffffffffu : (unsigned)xb;
        a.wp_bytes = wb > 0xffffffffull ? 0xffffffffu : (unsigned)wb;
        a.nstages = 0;
        a.div_howo = a.div_wo = FastDiv{0, 0, 0};
    }
    a.n_tiles = a.per_xcd = a.n_vtiles = 0;
    a.pc = nullptr;
    a.pc_fast_ok = 0;
    a.ksplit = 1;
    a.ws_cnt = nullptr;
    a.ws_part = nullptr;
    a.rq_fast = 0;
    a.mul_hi = 0;
    if (d->out_mode != ICNN_OUT_RAW_S32 && a.shift >= 1 && a.shift <= 32 &&
        ((long long)a.mul << (32 - a.shift)) <= 0x7fffffffLL) {
        a.rq_fast = 1;
        a.mul_hi = (int)((long long)a.mul << (32 - a.shift));
    }
    a.rq24 = a.t_hi = a.rnd = 0;
    if (d->out_mode != ICNN_OUT_RAW_S32 && a.lo == 0 && a.hi >= 0 && a.shift >= 1 && a.shift <= 31 && a.mul >= 1 &&
        a.mul < (1 << 24)) {
        const long long half = 1LL << (a.shift - 1);
        const long long num = ((long long)a.hi << a.shift) - half;
        const long long t_hi = num <= 0 ? 0 : (num + a.mul - 1) / a.mul;
        if (t_hi < (1 << 24) && t_hi * a.mul + half <= 0xffffffffLL && ((t_hi * a.mul + half) >> a.shift) == a.hi) {
            a.rq24 = 1;
            a.t_hi = (int)t_hi;
            a.rnd = (int)half;
        }
    }
    a.res_fast = 0;
    if (d->res_mode != ICNN_RES_NONE && d->res_dtype == ICNN_U8 && a.res_shift <= 30 &&
        255LL * a.res_mul + (1LL << a.res_shift) / 2 <= 0x7fffffffLL)
        a.res_fast = 1;
    a.epi_vec = a.vec_out && (d->res_mode == ICNN_RES_NONE || a.vec_res);
    {
        const int res_kind = d->res_mode == ICNN_RES_NONE ? 0 : (d->res_mode == ICNN_RES_PRE && a.res_fast ? 1 : 2);
        const int rq_kind = d->out_mode == ICNN_OUT_RAW_S32 ? 0 : (a.rq24 && res_kind != 2 ? 3 : (a.rq_fast ? 1 : 2));
        a.epi_mode = 4 * res_kind + rq_kind;
    }
    return ICNN_OK;
}

static int conv_layer(const icnn_conv_desc *d, const void *x, const void *w_packed, const int32_t *bias,
                      const void *pc, const void *res, void *y, void *workspace, void *stream,
                      const char *what)
{
    ConvGeom g;
    int rc = check_conv(d, &g);
    if (rc) return rc;
    if (g.ws_bytes && !workspace) return fail(ICNN_E_NULL, "this layer needs a workspace (iconv2d_workspace_bytes)");
    if (workspace && ((uintptr_t)workspace & 15)) return fail(ICNN_E_ALIGN, "workspace must be 16-byte aligned");
    ConvArgs a;
    rc = fill_conv_args(d, g, x, w_packed, bias, res, y, a);
    if (rc) return rc;
    if (pc) {
        if (!aligned16(pc)) return fail(ICNN_E_ALIGN, "packed channel parameters must be 16-byte aligned");
        if (d->out_mode == ICNN_OUT_RAW_S32 && d->res_mode == ICNN_RES_NONE)
            return fail(ICNN_E_PARAM, "a raw int32 output without a skip operand has no per-channel parameter");
        a.pc = (const int32_t *)pc;
        a.pc_fast_ok = d->out_mode != ICNN_OUT_RAW_S32 && a.epi_vec &&
                       (d->res_mode == ICNN_RES_NONE || (d->res_mode == ICNN_RES_PRE && d->res_dtype == ICNN_U8));
    }
    if ((g.rp == 32 || g.rp == 16) && !pc && !g_tuning.no_pic && d->stride_h == 1 && d->stride_w == 1 && d->kh <= 8 && (d->cout == 32 || d->cout == 64) &&
        (d->out_mode == ICNN_OUT_BRELU_U8 || d->out_mode == ICNN_OUT_CLAMP_U8) && d->res_mode == ICNN_RES_NONE &&
        d->in_signed != ICNN_IN_U8_FULL && d->in_signed != ICNN_IN_S8 && a.vec_out && a.vec_bias && a.x_bytes >= 4 &&
        a.x_bytes <= 0x7fffffffu && g.M <= 0x7fffffffLL)
        // a picture's first layer at stride 1: straight off the picture, no padded copy
        return launched(launch_conv_pic(a, (hipStream_t)stream), what);
    if (g.rp) {
        // small cin: pad and re-normalise x into the workspace, then run the layer as a kh x 1
        // convolution with "rp channels" over that copy (see pad_small_cin_kernel)
        uint8_t *padded = (uint8_t *)workspace + kWsCounterBytes;
        const hipError_t e = launch_pad_small_cin(a.x, padded, d->n, d->h, d->w, d->cin, d->in_c_stride, d->pad_h,
                                                  d->pad_w, g.hp, g.wp, a.in_xor, (hipStream_t)stream);
        if (e != hipSuccess) return launched(e, what);
        a.x = padded;
        a.H = g.hp; a.W = g.wp; a.Cin = g.rp; a.in_cs = 4; a.KW = 1; a.ph = 0; a.pw = 0;
        a.in_xor = 0;
        a.x_bytes = (unsigned)(g.ws_bytes - 64 - kWsCounterBytes);
        return launched(launch_conv(a, true, true, (hipStream_t)stream), what);
    }
    const bool vec_in = aligned16(x) && d->cin % 16 == 0 && d->in_c_stride % 16 == 0;
    // layers with few tiles and a long K axis split it over workgroups when the caller brought the workspace
    // iconv2d_workspace_bytes asked for (a workspace passed to a layer that asked for none is not touched)
    if (workspace && conv_split_bytes(a, vec_in) != 0) {
        a.ws_cnt = (unsigned *)workspace;
        a.ws_part = (int32_t *)((uint8_t *)workspace + kWsCounterBytes);
    }
    return launched(launch_conv(a, vec_in, vec_in, (hipStream_t)stream), what);
}

int iconv2d_brelu(const icnn_conv_desc *d, const void *x, const void *w_packed, const int32_t *bias,
                  const void *res, void *y, void *workspace, void *stream)
{
    return conv_layer(d, x, w_packed, bias, nullptr, res, y, workspace, stream, "iconv2d_brelu");
}

// ---- iconv2d_brelu for callers that cannot allocate: the workspace is a fixed array in device memory that the
// code object itself carries (every GPU the library runs on holds its own copy until the process ends).
constexpr size_t kStaticWsBytes = ICNN_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

// In host code `scratch` is only a handle for the symbol, not a device address: the address on the current
// device is asked for once per device and kept; kernels and copies only ever get that pointer.
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_lock;

static int static_workspace(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ICNN_E_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(ICNN_E_UNSUPPORTED, "device index %d beyond %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> g(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(ICNN_E_LAUNCH, "hipGetSymbolAddress(static workspace): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return ICNN_OK;
}

int iconv2d_brelu_static_ws(const icnn_conv_desc *d, const void *x, const void *w_packed, const int32_t *bias,
                            const void *res, void *y, void *stream)
{
    ConvGeom g;
    int rc = check_conv(d, &g);
    if (rc) return rc;
    if (g.ws_bytes > kStaticWsBytes)
        return fail(ICNN_E_SHAPE, "this layer needs a workspace of %zu bytes; the static one holds %zu (use iconv2d_brelu)",
                    g.ws_bytes, kStaticWsBytes);
    size_t need = 0;
    if ((rc = workspace_need(d, g, &need))) return rc;
    void *ws = nullptr;        // a split K axis that would need more than the array holds simply stays whole
    if (need && need <= kStaticWsBytes && (rc = static_workspace(&ws))) return rc;
    return conv_layer(d, x, w_packed, bias, nullptr, res, y, ws, stream, "iconv2d_brelu_static_ws");
}

int iconv2d_packed_channel_params_bytes(const icnn_conv_desc *d, size_t *bytes)
{
    ConvGeom g;
    int rc = check_conv(d, &g);
    if (rc) return rc;
    if (!bytes) return fail(ICNN_E_NULL, "bytes is NULL");
    *bytes = (size_t)((d->cout + 15) / 16) * kPcGroupInts * sizeof(int32_t);
    return ICNN_OK;
}

int iconv2d_prepack_channel_params(const icnn_conv_desc *d, const icnn_channel_params *pc, void *packed, void *stream)
{
    ConvGeom g;
    int rc = check_conv(d, &g);
    if (rc) return rc;
    if (!pc || !packed) return fail(ICNN_E_NULL, "channel parameters and packed buffer must not be NULL");
    const bool requant = d->out_mode != ICNN_OUT_RAW_S32;
    const bool skip = d->res_mode != ICNN_RES_NONE;
    if (requant && (!pc->mul || !pc->shift)) return fail(ICNN_E_NULL, "per-channel mul and shift must not be NULL");
    if (skip && (!pc->res_mul || !pc->res_shift))
        return fail(ICNN_E_NULL, "per-channel res_mul and res_shift must not be NULL when res_mode is set");
    if (!requant && !skip) return fail(ICNN_E_PARAM, "a raw int32 output without a skip operand has no per-channel parameter");
    const int32_t *arrs[4] = {pc->mul, pc->shift, pc->res_mul, pc->res_shift};
    for (const int32_t *q : arrs)
        if ((uintptr_t)q & 3) return fail(ICNN_E_ALIGN, "per-channel arrays must be 4-byte aligned");
    if (!aligned16(packed)) return fail(ICNN_E_ALIGN, "packed channel parameters must be 16-byte aligned");
    return launched(launch_pc_prepack(requant ? pc->mul : nullptr, requant ? pc->shift : nullptr, skip ? pc->res_mul : nullptr,
                                      skip ? pc->res_shift : nullptr, d->cout, (int32_t *)packed, (hipStream_t)stream),
                    "iconv2d_prepack_channel_params");
}

int iconv2d_brelu_pc(const icnn_conv_desc *d, const void *x, const void *w_packed, const int32_t *bias,
                     const void *pc_packed, const void *res, void *y, void *workspace, void *stream)
{
    if (!pc_packed) return fail(ICNN_E_NULL, "packed channel parameters are NULL");
    return conv_layer(d, x, w_packed, bias, pc_packed, res, y, workspace, stream, "iconv2d_brelu_pc");
}

// Y_main + [Y_proj * res_mul / 2^res_shift] inside int32?  |Y_proj| <= Kp*128*128 + 2^28, |Y_main| <= Km*128*128 + 2^28
// under the bias contract (int8 inputs and weights may both be -128)
static bool merged_sum_fits(long long k_main, long long k_proj, int res_mul, int res_shift)
{
    const long long yp = k_proj * 128 * 128 + (1LL << 28);
    const long long ym = k_main * 128 * 128 + (1LL << 28);
    const __int128 s_max = (((__int128)yp * res_mul) >> res_shift) + 2;
    return s_max + ym <= 0x7fffffffLL;
}

static int dual_layer(const icnn_conv_desc *m, const void *x_main, const void *w_main_packed,
                      const int32_t *bias_main, const void *pc, const icnn_conv_desc *p, const void *x_proj,
                      const void *w_proj_packed, const int32_t *bias_proj, void *y, void *stream, const char *what)
{
    ConvGeom gm, gp;
    int rc = check_conv(m, &gm);
    if (rc) return rc;
    rc = check_conv(p, &gp);
    if (rc) return rc;
    if (m->res_mode != ICNN_RES_PRE || m->res_dtype != ICNN_S32)
        return fail(ICNN_E_PARAM, "main layer must describe an int32 skip operand joined before requantisation");
    if (p->out_mode != ICNN_OUT_RAW_S32 || p->res_mode != ICNN_RES_NONE)
        return fail(ICNN_E_PARAM, "projection layer must have a raw int32 output and no skip operand");
    if (m->n != p->n || gm.ho != gp.ho || gm.wo != gp.wo || m->cout != p->cout)
        return fail(ICNN_E_SHAPE, "main and projection layers must produce the same n x ho x wo x cout");
    const icnn_conv_desc *both[2] = {m, p};
    for (const icnn_conv_desc *d : both) {
        if (d->in_signed == ICNN_IN_U8_FULL) return fail(ICNN_E_UNSUPPORTED, "fused block takes inputs up to 127 or int8 only");
        if (d->kh != 1 || d->kw != 1 || d->pad_h != 0 || d->pad_w != 0 || d->cin % 16 != 0 || d->in_c_stride % 16 != 0 ||
            d->in_sub128)
            return fail(ICNN_E_UNSUPPORTED, "fused block needs 1x1 layers without padding, cin and pitch multiples of 16");
    }
    if (!aligned16(x_main) || !aligned16(x_proj) || !aligned16(y))
        return fail(ICNN_E_UNSUPPORTED, "fused block needs 16-byte aligned tensors");
    if (!merged_sum_fits(gm.K, gp.K, m->res_mul, m->res_shift))
        return fail(ICNN_E_UNSUPPORTED, "cannot prove that the merged sum stays inside int32 for these sizes");
    ConvArgs a, b;
    // the main layer's arguments without its skip operand (the projection is accumulated in registers)
    icnn_conv_desc m0 = *m;
    m0.res_mode = ICNN_RES_NONE;
    rc = fill_conv_args(&m0, gm, x_main, w_main_packed, bias_main, nullptr, y, a);
    if (rc) return rc;
    int32_t dummy_out = 0;
    rc = fill_conv_args(p, gp, x_proj, w_proj_packed, bias_proj, nullptr, &dummy_out, b);
    if (rc) return rc;
    if (a.x_bytes >= 0x7fffff00u || b.x_bytes >= 0x7fffff00u || a.wp_bytes >= 0x7fffff00u || b.wp_bytes >= 0x7fffff00u)
        return fail(ICNN_E_UNSUPPORTED, "fused block needs tensors below 2 GiB");
    ProjArgs q;
    q.x = b.x; q.wp = b.wp; q.bias = b.bias;
    q.H = p->h; q.W = p->w; q.Cin = p->cin; q.in_cs = p->in_c_stride; q.sh = p->stride_h; q.sw = p->stride_w;
    q.ksteps = gp.ksteps; q.x_bytes = b.x_bytes; q.wp_bytes = b.wp_bytes;
    q.res_mul = m->res_mul; q.res_shift = m->res_shift; q.vec_bias = b.vec_bias;
    if (pc) {
        if (!aligned16(pc)) return fail(ICNN_E_ALIGN, "packed channel parameters must be 16-byte aligned");
        if (m->out_mode == ICNN_OUT_RAW_S32) return fail(ICNN_E_UNSUPPORTED, "fused block with channel parameters needs an 8-bit output");
        a.pc = (const int32_t *)pc;
        a.pc_fast_ok = a.epi_vec;       // the main layer's arguments carry no skip operand here
    }
    return launched(launch_conv_dual(a, q, (hipStream_t)stream), what);
}

int iconv2d_dual_brelu(const icnn_conv_desc *m, const void *x_main, const void *w_main_packed,
                       const int32_t *bias_main, const icnn_conv_desc *p, const void *x_proj,
                       const void *w_proj_packed, const int32_t *bias_proj, void *y, void *stream)
{
    return dual_layer(m, x_main, w_main_packed, bias_main, nullptr, p, x_proj, w_proj_packed, bias_proj, y, stream,
                      "iconv2d_dual_brelu");
}

int iconv2d_dual_brelu_pc(const icnn_conv_desc *m, const void *x_main, const void *w_main_packed,
                          const int32_t *bias_main, const void *pc_packed_main, const icnn_conv_desc *p,
                          const void *x_proj, const void *w_proj_packed, const int32_t *bias_proj, void *y, void *stream)
{
    if (!pc_packed_main) return fail(ICNN_E_NULL, "packed channel parameters are NULL");
    return dual_layer(m, x_main, w_main_packed, bias_main, pc_packed_main, p, x_proj, w_proj_packed, bias_proj, y, stream,
                      "iconv2d_dual_brelu_pc");
}

int iconv2d_maxpool_brelu(const icnn_conv_desc *d, int32_t pool_k, int32_t pool_stride, int32_t pool_pad, const void *x,
                          const void *w_packed, const int32_t *bias, void *y, void *stream)
{
    ConvGeom g;
    int rc = check_conv(d, &g);
    if (rc) return rc;
    if (pool_k < 1 || pool_stride < 1 || pool_pad < 0 || pool_pad >= pool_k || g.ho + 2 * pool_pad < pool_k || g.wo + 2 * pool_pad < pool_k)
        return fail(ICNN_E_SHAPE, "bad max-pool geometry");
    if (pool_k != 3 || pool_stride != 2 || pool_pad != 1)
        return fail(ICNN_E_UNSUPPORTED, "fused first layer takes a 3x3 / stride 2 / padding 1 max-pool only");
    if (d->cin > 4 || g.rp != 32 || d->kh > 8 || d->stride_h != 2 || d->stride_w != 2 || (d->cout != 32 && d->cout != 64))
        return fail(ICNN_E_UNSUPPORTED, "fused first layer needs cin <= 4, a kernel 5 to 8 pixels wide and at most 8 high, stride 2 and 32 or 64 output channels");
    if ((d->out_mode != ICNN_OUT_BRELU_U8 && d->out_mode != ICNN_OUT_CLAMP_U8) || d->res_mode != ICNN_RES_NONE ||
        d->in_signed == ICNN_IN_U8_FULL || d->in_signed == ICNN_IN_S8)
        return fail(ICNN_E_UNSUPPORTED, "fused first layer stores unsigned bytes, takes no skip operand and unsigned or raw-picture input");
    if (d->out_mode == ICNN_OUT_CLAMP_U8 && d->lo != 0)
        return fail(ICNN_E_UNSUPPORTED, "fused first layer needs a lower clamp of 0 (the pool's padding is zero)");
    ConvArgs a;
    if ((rc = fill_conv_args(d, g, x, w_packed, bias, nullptr, y, a))) return rc;
    if (!a.vec_out || !a.vec_bias) return fail(ICNN_E_UNSUPPORTED, "fused first layer needs 16-byte aligned output and bias");
    const unsigned long long xb = ((unsigned long long)d->n * d->h * d->w - 1) * d->in_c_stride + d->cin;
    if (xb > 0x7fffffffull || g.M > 0x7fffffffLL) return fail(ICNN_E_UNSUPPORTED, "fused first layer needs tensors below 2 GiB");
    if (xb < 4) return fail(ICNN_E_UNSUPPORTED, "fused first layer reads the picture four bytes at a time: it needs at least four");
    const int hp = (g.ho + 2 * pool_pad - pool_k) / pool_stride + 1, wp = (g.wo + 2 * pool_pad - pool_k) / pool_stride + 1;
    return launched(launch_conv_stem_pool(a, hp, wp, (hipStream_t)stream), "iconv2d_maxpool_brelu");
}

int iconv2d_bottleneck_brelu(const icnn_conv_desc *c1, const void *x, const void *w1_packed, const int32_t *bias1,
                             const icnn_conv_desc *c2, const void *w2_packed, const int32_t *bias2,
                             const icnn_conv_desc *c3, const void *w3_packed, const int32_t *bias3, const void *res,
                             void *y, void *stream)
{
    ConvGeom g1, g2, g3;
    int rc = check_conv(c1, &g1);
    if (rc) return rc;
    if ((rc = check_conv(c2, &g2))) return rc;
    if ((rc = check_conv(c3, &g3))) return rc;
    const int mid = c1->cout, c = c1->cin;
    const icnn_conv_desc *all[3] = {c1, c2, c3};
    for (const icnn_conv_desc *d : all) {
        if (d->n != c1->n || d->h != c1->h || d->w != c1->w)
            return fail(ICNN_E_SHAPE, "the three layers of a block must share n, h, w");
        if (d->in_signed != ICNN_IN_U8_LE127 || d->in_sub128)
            return fail(ICNN_E_UNSUPPORTED, "fused block takes unsigned inputs up to 127 only");
        if (d->stride_h != 1 || d->stride_w != 1) return fail(ICNN_E_UNSUPPORTED, "fused block needs stride 1");
    }
    if (c1->kh != 1 || c1->kw != 1 || c1->pad_h || c1->pad_w || c3->kh != 1 || c3->kw != 1 || c3->pad_h || c3->pad_w ||
        c2->kh != 3 || c2->kw != 3 || c2->pad_h != 1 || c2->pad_w != 1)
        return fail(ICNN_E_UNSUPPORTED, "fused block is 1x1, then 3x3 with padding 1, then 1x1");
    if (c2->cin != mid || c2->cout != mid || c3->cin != mid)
        return fail(ICNN_E_SHAPE, "the middle width of the three layers does not match");
    for (const icnn_conv_desc *d : {c1, c2})
        if ((d->out_mode != ICNN_OUT_BRELU_U8 && d->out_mode != ICNN_OUT_CLAMP_U8) || d->res_mode != ICNN_RES_NONE ||
            (d->out_mode == ICNN_OUT_BRELU_U8 ? d->bound_q : d->hi) > 127)
            return fail(ICNN_E_UNSUPPORTED, "the first two layers must store unsigned bytes up to 127 and take no skip operand");
    if ((mid != 64 && mid != 128) || c % 64 != 0 || c3->cout % mid != 0 || c3->cout % 16 != 0)
        return fail(ICNN_E_UNSUPPORTED, "fused block needs a middle width of 64 or 128, cin a multiple of 64 and cout a multiple of the middle width");
    if (conv_block_lds_bytes(mid, c) > 160 * 1024)
        return fail(ICNN_E_UNSUPPORTED, "the block's patch of %d input channels does not fit the on-chip memory", c);
    if (!aligned16(x) || c1->in_c_stride % 16 != 0) return fail(ICNN_E_UNSUPPORTED, "fused block needs a 16-byte aligned input");
    ConvArgs a1, a2, a3;
    int32_t dummy = 0;         // the first two layers' outputs never reach memory
    if ((rc = fill_conv_args(c1, g1, x, w1_packed, bias1, nullptr, &dummy, a1))) return rc;
    if ((rc = fill_conv_args(c2, g2, x, w2_packed, bias2, nullptr, &dummy, a2))) return rc;
    if ((rc = fill_conv_args(c3, g3, x, w3_packed, bias3, res, y, a3))) return rc;
    if (!a3.epi_vec) return fail(ICNN_E_UNSUPPORTED, "fused block needs 16-byte aligned output and skip tensors");
    if (!a1.vec_bias || !a2.vec_bias || !a3.vec_bias) return fail(ICNN_E_UNSUPPORTED, "fused block needs 16-byte aligned bias arrays");
    if (a1.x_bytes >= 0x7fffff00u || a1.wp_bytes >= 0x7fffff00u || a2.wp_bytes >= 0x7fffff00u || a3.wp_bytes >= 0x7fffff00u)
        return fail(ICNN_E_UNSUPPORTED, "fused block needs tensors below 2 GiB");
    BlockArgs b;
    b.x = (const uint8_t *)x; b.x_bytes = a1.x_bytes; b.x_cs = c1->in_c_stride;
    b.N = c1->n; b.H = c1->h; b.W = c1->w;
    if (!conv_block_tile(b.H, b.W, b)) return fail(ICNN_E_UNSUPPORTED, "no tile shape for this image");
    const long long tiles = (long long)b.tiles_per_img * b.N;
    if (tiles > 0x7fffffffLL || g1.M > 0x7fffffffLL) return fail(ICNN_E_SHAPE, "too many tiles");
    b.n_tiles = (int)tiles;
    b.per_xcd = 0;              // set by the launcher
    b.k1 = c / 64;
    b.nchunk3 = c3->cout / mid;
    if (!g_tuning.no_block64 && conv_block64_takes(b, a1, a3) && conv_block64_lds_bytes(c, c, false) <= 160 * 1024)
        return launched(launch_conv_block64(b, a1, a2, a3, nullptr, (hipStream_t)stream), "iconv2d_bottleneck_brelu");
    return launched(launch_conv_block(b, a1, a2, a3, (hipStream_t)stream), "iconv2d_bottleneck_brelu");
}

int iconv2d_bottleneck_dual_brelu(const icnn_conv_desc *c1, const void *x, const void *w1_packed, const int32_t *bias1,
                                  const icnn_conv_desc *c2, const void *w2_packed, const int32_t *bias2,
                                  const icnn_conv_desc *c3, const void *w3_packed, const int32_t *bias3,
                                  const icnn_conv_desc *cp, const void *wp_packed, const int32_t *biasp, void *y, void *stream)
{
    ConvGeom g1, g2, g3, gp;
    int rc = check_conv(c1, &g1);
    if (rc) return rc;
    if ((rc = check_conv(c2, &g2))) return rc;
    if ((rc = check_conv(c3, &g3))) return rc;
    if ((rc = check_conv(cp, &gp))) return rc;
    if (c3->res_mode != ICNN_RES_PRE || c3->res_dtype != ICNN_S32)
        return fail(ICNN_E_PARAM, "the last layer must describe an int32 skip operand joined before requantisation");
    if (cp->out_mode != ICNN_OUT_RAW_S32 || cp->res_mode != ICNN_RES_NONE)
        return fail(ICNN_E_PARAM, "projection layer must have a raw int32 output and no skip operand");
    for (const icnn_conv_desc *d : {c1, c2, c3, cp}) {
        if (d->n != c1->n || d->h != c1->h || d->w != c1->w)
            return fail(ICNN_E_SHAPE, "the layers of a block must share n, h, w");
        if (d->in_signed != ICNN_IN_U8_LE127 || d->in_sub128)
            return fail(ICNN_E_UNSUPPORTED, "fused block takes unsigned inputs up to 127 only");
        if (d->stride_h != 1 || d->stride_w != 1) return fail(ICNN_E_UNSUPPORTED, "fused block needs stride 1");
    }
    for (const icnn_conv_desc *d : {c1, c3, cp})
        if (d->kh != 1 || d->kw != 1 || d->pad_h || d->pad_w) return fail(ICNN_E_UNSUPPORTED, "fused block is 1x1, then 3x3 with padding 1, then 1x1, with a 1x1 projection");
    if (c2->kh != 3 || c2->kw != 3 || c2->pad_h != 1 || c2->pad_w != 1)
        return fail(ICNN_E_UNSUPPORTED, "fused block is 1x1, then 3x3 with padding 1, then 1x1, with a 1x1 projection");
    if (c1->cin != 64 || c1->cout != 64 || c2->cin != 64 || c2->cout != 64 || c3->cin != 64 || c3->cout != 256 || cp->cin != 64 ||
        cp->cout != 256)
        return fail(ICNN_E_UNSUPPORTED, "fused projection block is 64 -> 64 -> 64 -> 256 channels with a 64 -> 256 projection");
    if (cp->in_c_stride != c1->in_c_stride) return fail(ICNN_E_SHAPE, "the projection reads the block input: same pitch as the first layer's input");
    for (const icnn_conv_desc *d : {c1, c2})
        if ((d->out_mode != ICNN_OUT_BRELU_U8 && d->out_mode != ICNN_OUT_CLAMP_U8) || d->res_mode != ICNN_RES_NONE ||
            (d->out_mode == ICNN_OUT_BRELU_U8 ? d->bound_q : d->hi) > 127)
            return fail(ICNN_E_UNSUPPORTED, "the first two layers must store unsigned bytes up to 127 and take no skip operand");
    if (c3->out_mode == ICNN_OUT_RAW_S32) return fail(ICNN_E_UNSUPPORTED, "fused projection block stores 8-bit outputs");
    if (!aligned16(x) || c1->in_c_stride % 16 != 0) return fail(ICNN_E_UNSUPPORTED, "fused block needs a 16-byte aligned input");
    if (!merged_sum_fits(g3.K, gp.K, c3->res_mul, c3->res_shift))
        return fail(ICNN_E_UNSUPPORTED, "cannot prove that the merged sum stays inside int32 for these sizes");
    ConvArgs a1, a2, a3, ap;
    int32_t dummy = 0;
    icnn_conv_desc m0 = *c3;                      // the last layer without its skip operand: the projection is accumulated in registers
    m0.res_mode = ICNN_RES_NONE;
    if ((rc = fill_conv_args(c1, g1, x, w1_packed, bias1, nullptr, &dummy, a1))) return rc;
    if ((rc = fill_conv_args(c2, g2, x, w2_packed, bias2, nullptr, &dummy, a2))) return rc;
    if ((rc = fill_conv_args(&m0, g3, x, w3_packed, bias3, nullptr, y, a3))) return rc;
    if ((rc = fill_conv_args(cp, gp, x, wp_packed, biasp, nullptr, &dummy, ap))) return rc;
    if (!a3.epi_vec) return fail(ICNN_E_UNSUPPORTED, "fused block needs a 16-byte aligned output");
    if (!a1.vec_bias || !a2.vec_bias || !a3.vec_bias || !ap.vec_bias) return fail(ICNN_E_UNSUPPORTED, "fused block needs 16-byte aligned bias arrays");
    if (a1.x_bytes >= 0x7fffff00u || g1.M > 0x7fffffffLL) return fail(ICNN_E_UNSUPPORTED, "fused block needs tensors below 2 GiB");
    ProjArgs q = {};
    q.x = ap.x; q.wp = ap.wp; q.bias = ap.bias;
    q.H = cp->h; q.W = cp->w; q.Cin = cp->cin; q.in_cs = cp->in_c_stride; q.sh = 1; q.sw = 1;
    q.ksteps = gp.ksteps; q.x_bytes = ap.x_bytes; q.wp_bytes = ap.wp_bytes;
    q.res_mul = c3->res_mul; q.res_shift = c3->res_shift; q.vec_bias = ap.vec_bias;
    BlockArgs b;
    b.x = (const uint8_t *)x; b.x_bytes = a1.x_bytes; b.x_cs = c1->in_c_stride;
    b.N = c1->n; b.H = c1->h; b.W = c1->w;
    if (!conv_block_tile(b.H, b.W, b)) return fail(ICNN_E_UNSUPPORTED, "no tile shape for this image");
    const long long tiles = (long long)b.tiles_per_img * b.N;
    if (tiles > 0x7fffffffLL) return fail(ICNN_E_SHAPE, "too many tiles");
    b.n_tiles = (int)tiles;
    b.per_xcd = 0;
    b.k1 = 1;
    b.nchunk3 = 4;
    if (!conv_block64_proj_takes(a1, a3, q)) return fail(ICNN_E_UNSUPPORTED, "fused projection block does not take these layers");
    return launched(launch_conv_block64(b, a1, a2, a3, &q, (hipStream_t)stream), "iconv2d_bottleneck_dual_brelu");
}

int iconv2d_pair_brelu(const icnn_conv_desc *c3, const void *t, const void *w3_packed, const int32_t *bias3, const void *res,
                       void *y, const icnn_conv_desc *c1, const void *w1_packed, const int32_t *bias1, void *z, void *stream)
{
    ConvGeom g3, g1;
    int rc = check_conv(c3, &g3);
    if (rc) return rc;
    if ((rc = check_conv(c1, &g1))) return rc;
    for (const icnn_conv_desc *d : {c3, c1}) {
        if (d->n != c3->n || d->h != c3->h || d->w != c3->w) return fail(ICNN_E_SHAPE, "the two layers of a pair must share n, h, w");
        if (d->kh != 1 || d->kw != 1 || d->pad_h || d->pad_w || d->stride_h != 1 || d->stride_w != 1)
            return fail(ICNN_E_UNSUPPORTED, "fused pair is two 1x1 layers of stride 1 without padding");
        if (d->in_signed != ICNN_IN_U8_LE127 || d->in_sub128)
            return fail(ICNN_E_UNSUPPORTED, "fused pair takes unsigned inputs up to 127 only");
        if (d->out_mode != ICNN_OUT_BRELU_U8 && d->out_mode != ICNN_OUT_CLAMP_U8)
            return fail(ICNN_E_UNSUPPORTED, "both layers of a fused pair store unsigned bytes");
    }
    if (c1->cin != c3->cout || c1->cout != c3->cin) return fail(ICNN_E_SHAPE, "the widths of the two layers do not match");
    if ((c3->cin != 64 && c3->cin != 128 && c3->cin != 256) || c3->cout % 256 != 0 || c3->cout > 2048)
        return fail(ICNN_E_UNSUPPORTED, "fused pair needs a narrow width of 64, 128 or 256 and a wide one that is a multiple of 256 up to 2048");
    if ((c3->out_mode == ICNN_OUT_BRELU_U8 ? c3->bound_q : c3->hi) > 127 || (c3->out_mode == ICNN_OUT_CLAMP_U8 && c3->lo != 0))
        return fail(ICNN_E_UNSUPPORTED, "the first layer of a fused pair must store bytes in 0..127 (the second reads them as signed)");
    if (c1->res_mode != ICNN_RES_NONE) return fail(ICNN_E_UNSUPPORTED, "the second layer of a fused pair takes no skip operand");
    if (c1->out_mode == ICNN_OUT_CLAMP_U8 && c1->lo != 0) return fail(ICNN_E_UNSUPPORTED, "fused pair needs a lower clamp of 0");
    if (!aligned16(t) || c3->in_c_stride % 16 != 0) return fail(ICNN_E_UNSUPPORTED, "fused pair needs a 16-byte aligned input");
    ConvArgs a3, a1;
    if ((rc = fill_conv_args(c3, g3, t, w3_packed, bias3, res, y, a3))) return rc;
    if ((rc = fill_conv_args(c1, g1, y, w1_packed, bias1, nullptr, z, a1))) return rc;
    if (!a3.epi_vec || !a1.epi_vec) return fail(ICNN_E_UNSUPPORTED, "fused pair needs 16-byte aligned output and skip tensors");
    if (!a3.vec_bias || !a1.vec_bias) return fail(ICNN_E_UNSUPPORTED, "fused pair needs 16-byte aligned bias arrays");
    // skip operand kinds the byte epilogue covers: none, or unsigned 8-bit joined before requantisation in 32 bits
    if (a3.epi_mode / 4 == 2) return fail(ICNN_E_UNSUPPORTED, "fused pair takes an unsigned 8-bit skip operand joined before requantisation");
    if (a3.x_bytes >= 0x7fffff00u || g3.M > 0x7fffffffLL - 64 ||
        (unsigned long long)g3.M * c3->out_c_stride >= 0x7fffff00ull ||
        (c3->res_mode != ICNN_RES_NONE && (unsigned long long)g3.M * c3->res_c_stride >= 0x7fffff00ull))
        return fail(ICNN_E_UNSUPPORTED, "fused pair needs tensors below 2 GiB");
    if (conv_pair_lds_bytes(c3->cout, c1->cout) > 160 * 1024) return fail(ICNN_E_UNSUPPORTED, "the tile of the wide tensor does not fit the on-chip memory");
    return launched(launch_conv_pair(a3, a1, g3.M, (hipStream_t)stream), "iconv2d_pair_brelu");
}

int iconv2d_twin_brelu(const icnn_conv_desc *ca, const void *x, const void *wa_packed, const int32_t *bias_a, void *ya,
                       const icnn_conv_desc *cb, const void *wb_packed, const int32_t *bias_b, void *yb, void *stream)
{
    ConvGeom ga, gb;
    int rc = check_conv(ca, &ga);
    if (rc) return rc;
    if ((rc = check_conv(cb, &gb))) return rc;
    if (cb->n != ca->n || cb->h != ca->h || cb->w != ca->w || cb->cin != ca->cin || cb->in_c_stride != ca->in_c_stride ||
        cb->in_signed != ca->in_signed || cb->in_sub128 != ca->in_sub128)
        return fail(ICNN_E_SHAPE, "twin layers read the same input: n, h, w, cin, in_c_stride and the input kind must agree");
    if (ca->res_mode != ICNN_RES_NONE || cb->res_mode != ICNN_RES_NONE)
        return fail(ICNN_E_UNSUPPORTED, "twin layers take no skip operands");
    if (ca->in_signed != ICNN_IN_U8_LE127 || ca->in_sub128) return fail(ICNN_E_UNSUPPORTED, "twin layers take unsigned inputs up to 127 only");
    if (!aligned16(x)) return fail(ICNN_E_UNSUPPORTED, "twin layers need a 16-byte aligned input");
    ConvArgs a, b;
    if ((rc = fill_conv_args(ca, ga, x, wa_packed, bias_a, nullptr, ya, a))) return rc;
    if ((rc = fill_conv_args(cb, gb, x, wb_packed, bias_b, nullptr, yb, b))) return rc;
    if (!conv_plane_twin_ok(a, b))
        return fail(ICNN_E_UNSUPPORTED, "twin layers: a 5x5 layer of 64 channels beside a 3x3, or a 3x3 layer of 48 or 64 channels beside a 1x1, "
                                        "stride 1, \"same\" padding, at most 32 output channels each, tensors below 2 GiB");
    return launched(launch_conv_plane_twin(a, b, (hipStream_t)stream), "iconv2d_twin_brelu");
}

int iadd_rescale(const icnn_add_desc *d, const void *a, const void *b, void *out, void *stream)
{
    if (!d) return fail(ICNN_E_NULL, "add descriptor is NULL");
    if (d->count_pixels < 0 || d->c < 0) return fail(ICNN_E_SHAPE, "count_pixels and c must be >= 0");
    if (d->a_c_stride < d->c || d->b_c_stride < d->c || d->out_c_offset < 0 ||
        (long long)d->out_c_offset + d->c > d->out_c_stride)
        return fail(ICNN_E_SHAPE, "channel pitches must cover c (and out_c_offset + c)");
    if (d->a_dtype < ICNN_U8 || d->a_dtype > ICNN_S32 || d->b_dtype < ICNN_U8 || d->b_dtype > ICNN_S32)
        return fail(ICNN_E_PARAM, "unknown operand dtype");
    if (d->out_mode != ICNN_OUT_CLAMP_U8 && d->out_mode != ICNN_OUT_LINEAR_S8 && d->out_mode != ICNN_OUT_RAW_S32)
        return fail(ICNN_E_PARAM, "iadd_rescale out_mode must be CLAMP_U8, LINEAR_S8 or RAW_S32");
    int rc = check_requant(d->b_mul, d->b_shift, "b");
    if (rc) return rc;
    if (d->out_mode != ICNN_OUT_RAW_S32 && (rc = check_requant(d->mul, d->shift, "output"))) return rc;
    if (d->out_mode == ICNN_OUT_CLAMP_U8 && (d->lo < 0 || d->hi > 255 || d->lo > d->hi))
        return fail(ICNN_E_PARAM, "clamp range [%d, %d] must satisfy 0 <= lo <= hi <= 255", d->lo, d->hi);
    if (d->count_pixels == 0 || d->c == 0) return ICNN_OK;
    if (!a || !b || !out) return fail(ICNN_E_NULL, "a, b and out must not be NULL");
    if ((d->a_dtype == ICNN_S32 && ((uintptr_t)a & 3)) || (d->b_dtype == ICNN_S32 && ((uintptr_t)b & 3)) ||
        (d->out_mode == ICNN_OUT_RAW_S32 && ((uintptr_t)out & 3)))
        return fail(ICNN_E_ALIGN, "int32 tensors must be 4-byte aligned");
    AddArgs k;
    k.a = a; k.b = b; k.out = out; k.px = d->count_pixels; k.c = d->c;
    k.a_cs = d->a_c_stride; k.b_cs = d->b_c_stride; k.out_cs = d->out_c_stride; k.out_co = d->out_c_offset;
    k.a_dt = d->a_dtype; k.b_dt = d->b_dtype; k.out_mode = d->out_mode;
    k.b_mul = d->b_mul; k.b_shift = d->b_shift;
    k.mul = d->out_mode == ICNN_OUT_RAW_S32 ? 1 : d->mul;
    k.shift = d->out_mode == ICNN_OUT_RAW_S32 ? 0 : d->shift;
    k.lo = d->out_mode == ICNN_OUT_LINEAR_S8 ? -128 : d->lo;
    k.hi = d->out_mode == ICNN_OUT_LINEAR_S8 ? 127 : d->hi;
    k.mul_hi = 0;
    k.q24 = Rq24{0, 0, 0, 0, 0};
    const int ab = dtype_bytes(d->a_dtype), bb = dtype_bytes(d->b_dtype);
    const int ob = d->out_mode == ICNN_OUT_RAW_S32 ? 4 : 1;
    const bool vec = d->c % 16 == 0 && aligned16(a) && aligned16(b) && aligned16(out) &&
                     ((long long)d->a_c_stride * ab) % 16 == 0 && ((long long)d->b_c_stride * bb) % 16 == 0 &&
                     ((long long)d->out_c_stride * ob) % 16 == 0 && ((long long)d->out_c_offset * ob) % 16 == 0;
    return launched(launch_add(k, vec, (hipStream_t)stream), "iadd_rescale");
}

int iconcat(int32_t n_in, const void *const *in, const int32_t *c_in, const int32_t *in_c_stride,
            const int32_t *mul, const int32_t *shift, int32_t bound_q, int64_t count_pixels, void *out,
            int32_t out_c_stride, void *stream)
{
    if (n_in < 1 || n_in > 16) return fail(ICNN_E_SHAPE, "n_in %d must be in [1, 16]", n_in);
    if (!in || !c_in || !in_c_stride || !mul || !shift) return fail(ICNN_E_NULL, "an argument array is NULL");
    if (count_pixels < 0) return fail(ICNN_E_SHAPE, "count_pixels must be >= 0");
    if (bound_q < 1 || bound_q > 255) return fail(ICNN_E_PARAM, "bound_q %d must be in [1, 255]", bound_q);
    long long total_c = 0;
    for (int i = 0; i < n_in; ++i) {
        if (c_in[i] < 0 || in_c_stride[i] < c_in[i]) return fail(ICNN_E_SHAPE, "input %d: bad channel count or pitch", i);
        const int rc = check_requant(mul[i], shift[i], "concat input");
        if (rc) return rc;
        total_c += c_in[i];
    }
    if (total_c > out_c_stride) return fail(ICNN_E_SHAPE, "inputs have %lld channels, out_c_stride is %d", total_c, out_c_stride);
    if (count_pixels == 0) return ICNN_OK;
    if (!out) return fail(ICNN_E_NULL, "out is NULL");
    for (int i = 0; i < n_in; ++i)
        if (c_in[i] > 0 && !in[i]) return fail(ICNN_E_NULL, "input %d is NULL", i);
    {
        // every branch aligned: one launch writes whole output rows (branches without channels are left out)
        ConcatArgs k;
        k.n_in = 0;
        bool all_vec = out_c_stride % 16 == 0 && aligned16(out);
        int end = 0;
        for (int i = 0; i < n_in && all_vec; ++i) {
            if (c_in[i] == 0) continue;
            all_vec = c_in[i] % 16 == 0 && in_c_stride[i] % 16 == 0 && aligned16(in[i]);
            const int j = k.n_in++;
            end += c_in[i];
            k.in[j] = (const uint8_t *)in[i]; k.c_end[j] = end; k.in_cs[j] = in_c_stride[i];
            k.mul[j] = mul[i]; k.shift[j] = shift[i]; k.q[j] = make_rq24(mul[i], shift[i], bound_q);
        }
        if (all_vec && k.n_in >= 1) {
            for (int j = k.n_in; j < 16; ++j) {
                k.in[j] = nullptr; k.c_end[j] = end; k.in_cs[j] = 0; k.mul[j] = 1; k.shift[j] = 0; k.q[j] = Rq24{0, 0, 0, 0, 0};
            }
            k.out_cs = out_c_stride; k.bound = bound_q; k.out = (uint8_t *)out;
            return launched(launch_concat_vec(k, count_pixels, (hipStream_t)stream), "iconcat");
        }
        if (all_vec) return ICNN_OK;     // no channels at all
    }
    int off = 0;
    for (int i = 0; i < n_in; ++i) {
        const bool vec = c_in[i] % 16 == 0 && in_c_stride[i] % 16 == 0 && out_c_stride % 16 == 0 && off % 16 == 0 &&
                         aligned16(in[i]) && aligned16(out);
        const int rc = launched(launch_requant_copy((const uint8_t *)in[i], (uint8_t *)out, count_pixels, c_in[i],
                                                    in_c_stride[i], out_c_stride, off, mul[i], shift[i], bound_q, vec,
                                                    (hipStream_t)stream),
                                "iconcat");
        if (rc) return rc;
        off += c_in[i];
    }
    return ICNN_OK;
}

int imaxpool2d_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t k, int32_t stride, int32_t pad,
                  const void *x, void *out, void *stream)
{
    if (n < 1 || h < 1 || w < 1 || c < 1 || k < 1 || stride < 1 || pad < 0 || h + 2 * pad < k || w + 2 * pad < k)
        return fail(ICNN_E_SHAPE, "bad max-pool geometry");
    if (pad >= k) return fail(ICNN_E_SHAPE, "pad must be smaller than the window");
    if (!x || !out) return fail(ICNN_E_NULL, "x and out must not be NULL");
    const int ho = (h + 2 * pad - k) / stride + 1, wo = (w + 2 * pad - k) / stride + 1;
    const bool vec = c % 16 == 0 && aligned16(x) && aligned16(out);
    return launched(launch_maxpool((const uint8_t *)x, (uint8_t *)out, n, h, w, c, k, stride, pad, ho, wo, vec,
                                   (hipStream_t)stream),
                    "imaxpool2d_u8");
}

int iavgpool_global_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t mul, int32_t shift, int32_t bound_q,
                       const void *x, void *out, void *stream)
{
    if (n < 1 || h < 1 || w < 1 || c < 1) return fail(ICNN_E_SHAPE, "n, h, w, c must be >= 1");
    if ((long long)h * w > (1 << 23)) return fail(ICNN_E_SHAPE, "h*w too large for the pooled sum");
    const int rc = check_requant(mul, shift, "average");
    if (rc) return rc;
    if (bound_q < 1 || bound_q > 255) return fail(ICNN_E_PARAM, "bound_q %d must be in [1, 255]", bound_q);
    if (!x || !out) return fail(ICNN_E_NULL, "x and out must not be NULL");
    return launched(launch_avgpool((const uint8_t *)x, (uint8_t *)out, n, h * w, c, mul, shift, bound_q,
                                   (hipStream_t)stream),
                    "iavgpool_global_u8");
}

int irenormalize_u8(int64_t count, const void *x, void *out, void *stream)
{
    if (count < 0) return fail(ICNN_E_SHAPE, "count must be >= 0");
    if (count == 0) return ICNN_OK;
    if (!x || !out) return fail(ICNN_E_NULL, "x and out must not be NULL");
    const bool vec = count % 16 == 0 && aligned16(x) && aligned16(out);
    return launched(launch_renorm((const uint8_t *)x, (uint8_t *)out, count, vec, (hipStream_t)stream),
                    "irenormalize_u8");
}

int icnn_peak_mfma_i8(int32_t blocks, int32_t iters, void *sink, void *stream)
{
    if (blocks < 1 || blocks > (1 << 20) || iters < 1) return fail(ICNN_E_SHAPE, "blocks must be in [1, 2^20] and iters >= 1");
    if (!sink) return fail(ICNN_E_NULL, "sink is NULL");
    if ((uintptr_t)sink & 3) return fail(ICNN_E_ALIGN, "sink must be 4-byte aligned");
    return launched(launch_mfma_loop(blocks, iters, (int *)sink, (hipStream_t)stream), "icnn_peak_mfma_i8");
}

int icnn_peak_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return ICNN_OK;
    if (!src || !dst) return fail(ICNN_E_NULL, "src and dst must not be NULL");
    if (!aligned16(src) || !aligned16(dst) || bytes % 16) return fail(ICNN_E_ALIGN, "src, dst and bytes must be multiples of 16");
    return launched(launch_stream_copy(src, dst, (long long)(bytes / 16), (hipStream_t)stream), "icnn_peak_copy");
}

}  // extern "C"
