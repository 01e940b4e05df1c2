/*
 * icnn.h -- C boundary of the MI355X integer-only CNN inference library.
 *
 * The library implements the inference hot path of "Efficient
 * Integer-Arithmetic-Only Convolutional Neural Networks": an 8-bit integer
 * convolution layer with an integer-only epilogue, the rescaled feature-map
 * addition used at residual merges, and concatenation of branches that carry
 * different scales.
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or keeps device memory.  Descriptor structs and the
 *     small arrays of iconcat are HOST memory, read during the call only.
 *   - Activations are NHWC, 8 bits per element.  "Channel pitch" (c_stride) is
 *     the number of elements between consecutive pixels; it may exceed the
 *     channel count so that a layer can read or write a slice of a wider buffer.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they never synchronise.
 *   - Return value: 0 on success, a negative icnn_status otherwise.  Arguments
 *     are checked on the host before anything is launched; a failed call has
 *     enqueued nothing.  icnn_last_error() describes the last failure on the
 *     calling thread.
 *   - [x] below means round half up, floor(x + 1/2), for negative x too; a
 *     shift of 0 adds no rounding term.  sat32() saturates to int32.
 */
#ifndef ICNN_H
#define ICNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ICNN_OK = 0,
    ICNN_E_NULL = -1,        /* a required pointer is NULL                        */
    ICNN_E_SHAPE = -2,       /* sizes non-positive, inconsistent or too large     */
    ICNN_E_PARAM = -3,       /* mul / shift / bound / mode outside its domain     */
    ICNN_E_ALIGN = -4,       /* pointer or pitch alignment the library needs      */
    ICNN_E_UNSUPPORTED = -5, /* valid request this build does not implement       */
    ICNN_E_LAUNCH = -6       /* the HIP runtime refused a launch                  */
} icnn_status;

typedef enum { ICNN_U8 = 0, ICNN_S8 = 1, ICNN_S32 = 2 } icnn_dtype;

typedef enum {
    ICNN_OUT_BRELU_U8 = 0,   /* clamp to [0, bound_q], store uint8                */
    ICNN_OUT_CLAMP_U8 = 1,   /* clamp to [lo, hi] within [0, 255], store uint8    */
    ICNN_OUT_LINEAR_S8 = 2,  /* clamp to [-128, 127], store int8                  */
    ICNN_OUT_RAW_S32 = 3     /* store T itself as int32: no requantisation        */
} icnn_out_mode;

typedef enum {
    ICNN_IN_U8_LE127 = 0,    /* unsigned bytes, all <= 127 (caller's guarantee)   */
    ICNN_IN_S8 = 1,          /* signed bytes                                      */
    ICNN_IN_U8_FULL = 2      /* unsigned bytes, any value up to 255               */
} icnn_in_kind;

typedef enum {
    ICNN_RES_NONE = 0,
    ICNN_RES_PRE = 1,        /* skip operand joins before BReLU / requantisation  */
    ICNN_RES_POST = 2        /* skip operand joins after requantisation           */
} icnn_res_mode;

/*
 * One quantised convolution layer (Section 3.1 and Figure 1: X_i, W_i, b_i, then
 * BReLU and quantisation to V_i; Section 3.2.1: V = [Y * mul / 2^shift]; Section
 * 3.3: the bound h_i corresponds to max_int = bound_q).
 *
 *   U[n,ho,wo,co] = sum_{kh,kw,ci} x(n, ho*stride_h - pad_h + kh, wo*stride_w - pad_w + kw, ci)
 *                                  * W[co][kh][kw][ci]
 *       x() is 0 outside the image; inside it is the stored byte read as uint8
 *       (in_signed = ICNN_IN_U8_LE127 when the caller guarantees bytes <= 127, as layers
 *       with bound_q <= 127 produce; ICNN_IN_U8_FULL for any byte: the 8-bit activations
 *       of the paper's bit-depth table, bound_q up to 255), as int8 (ICNN_IN_S8), or as
 *       uint8 minus 128 (in_sub128 = 1: the re-normalisation of a raw picture, Section
 *       3.4.1).  ICNN_IN_U8_FULL limits kh*kw*cin to 32767.
 *   Y = U + bias[co]                     (caller guarantees |bias[co]| <= 2^30, so that
 *                                         Y always fits int32; kh*kw*cin <= 65535 bounds U)
 *   S = [res * res_mul / 2^res_shift]                       (res_mode != NONE)
 *   T = sat32(Y + S) if res_mode == PRE, else Y             (Section 4.1: the skip
 *       operand is rescaled to the main path's ratio and added before BReLU)
 *   RAW_S32:  out = T
 *   else:     Q = [T * mul / 2^shift];  if res_mode == POST: Q += S
 *             out = clamp(Q, lo', hi')  with (lo', hi') = (0, bound_q), (lo, hi)
 *             or (-128, 127) by out_mode.
 * Clamping after requantisation equals BReLU before it, because the map is
 * monotone and sends h_i to bound_q.
 *
 * out is NHWC [n, ho, wo, out_c_stride]; channel co is written at
 * out_c_offset + co and no other element is touched, so several layers can fill
 * disjoint channel ranges of one buffer (concatenation without a copy, the
 * online half of Algorithm 2: each branch carries its own mul, shift, bound_q).
 */
typedef struct {
    int32_t n, h, w, cin;          /* logical input shape                          */
    int32_t in_c_stride;           /* channel pitch of x, >= cin                   */
    int32_t in_signed;             /* icnn_in_kind                                 */
    int32_t in_sub128;             /* 1: raw uint8 picture, use x - 128            */
    int32_t cout, kh, kw;
    int32_t stride_h, stride_w, pad_h, pad_w;
    int32_t out_c_stride, out_c_offset;
    int32_t mul, shift;            /* 1 <= mul < 2^31, 0 <= shift <= 62            */
    int32_t bound_q;               /* 1..255; used by ICNN_OUT_BRELU_U8            */
    int32_t lo, hi;                /* 0 <= lo <= hi <= 255; ICNN_OUT_CLAMP_U8 only */
    int32_t out_mode;              /* icnn_out_mode                                */
    int32_t res_mode;              /* icnn_res_mode                                */
    int32_t res_dtype;             /* icnn_dtype of the skip operand               */
    int32_t res_c_stride;          /* channel pitch of res, >= cout                */
    int32_t res_mul, res_shift;    /* 1 <= res_mul < 2^31, 0 <= res_shift <= 62    */
} icnn_conv_desc;

/* Library version, major*10000 + minor*100 + patch. */
int icnn_version(void);

/* Message for the last negative return on this thread ("" if none).  The string
 * is owned by the library and valid until the thread's next failing call. */
const char *icnn_last_error(void);

/* Kernel-selection override, for sweeps and for tests that must reach a kernel the library would not pick
 * for a small shape.  It changes which kernel computes a layer, never a result.  Process-wide, not
 * synchronised: set it while no other thread is inside the library.  `name` (host string) and the values it takes:
 *   "tile"        -1 library's choice; 0..4 force that tile shape of the tap-by-tap convolution kernel
 *   "stages"      0 library's choice; 2..6 LDS ring depth of that kernel
 *   "no_narrow", "no_fc", "no_halo", "no_stream", "no_block64", "no_deep", "no_plane", "no_pic"   1 keeps layers off the respective special kernel
 *   "halo_tile"   0 library's choice; 1 = 128 x 128, 2 = 64 x 256 tiles of the patch-resident 3x3 kernel
 *   "halo_always" 1 lets the patch-resident kernel take layers with several tiles per workgroup
 *   "block_any_form" 1 keeps fused bottleneck blocks on the instantiation that holds every epilogue form
 *   "plane_no_pipe" 1 keeps that kernel off its instantiations with the software-pipelined epilogue
 *   "plane_always" 1 lets the kernel with two-dimensional tiles (few channels, large pictures) take every layer it accepts
 *   "deep_always" 1 lets the 3x3 kernel whose waves split the K axis take every layer whose shape it accepts
 *   "deep_plain_walk" 1 gives that kernel the tile order of the other kernels (pixel tiles, not channel tiles, per XCD)
 *   "ksplit"      0 library's choice; 1 never split the K axis over workgroups; 2..8 that split where it divides the K steps
 *   "reset"       (value ignored) back to the library's choices
 * Unknown names and values outside these ranges return ICNN_E_PARAM and change nothing. */
int icnn_set_tuning(const char *name, int32_t value);

/* Host-only check of a descriptor: the same validation iconv2d_brelu performs,
 * without touching the GPU.  Rejects, among others, kh*kw*cin > 65535 (beyond it
 * the int32 accumulator is no longer provably safe) and unsigned inputs combined
 * with bound semantics the int8 matrix cores cannot take (in_signed = 0 means the
 * caller guarantees bytes <= 127, as produced by bound_q <= 127). */
int iconv2d_validate(const icnn_conv_desc *desc);

/* Output height and width of the layer (host only). */
int iconv2d_out_hw(const icnn_conv_desc *desc, int32_t *ho, int32_t *wo);

/* Bytes of device workspace iconv2d_brelu uses for this layer (may be 0): the padded copy of a layer with cin <= 4,
 * or the partial sums of a layer whose K axis is split over workgroups.  The caller zero-fills a workspace once after
 * allocating it (its first 4096 bytes are counters that every call leaves at zero); one workspace of the largest size
 * may serve all layers that run one after the other on a stream.  Layers that split K also run without a workspace
 * (NULL): then the K axis stays whole.  A layer with cin <= 4 always needs its workspace passed, although the
 * stride-1 forms that the library convolves straight off the picture (8-bit output, 32 or 64 channels, kernel up to
 * 8 x 8, no skip operand) leave it untouched. */
int iconv2d_workspace_bytes(const icnn_conv_desc *desc, size_t *bytes);

/* Bytes of the library's packed weight format for this layer. */
int iconv2d_packed_weight_bytes(const icnn_conv_desc *desc, size_t *bytes);

/* Reorders int8 weights [cout][kh][kw][cin] (device) into the packed format
 * (device, 16-byte aligned, iconv2d_packed_weight_bytes bytes).  Done once per
 * layer, outside the inference loop. */
int iconv2d_prepack_weights(const icnn_conv_desc *desc, const int8_t *w_ohwi,
                            void *w_packed, void *stream);

/* The integer convolution layer defined above.  x: input activations; w_packed:
 * from iconv2d_prepack_weights; bias: int32 [cout]; res: skip operand over the
 * output pixels (NULL iff res_mode == NONE); y: output; workspace: at least
 * iconv2d_workspace_bytes bytes, 16-byte aligned, zero-filled once by the caller (may be NULL when that is 0; a layer
 * that asked for none does not touch it).
 * Alignment: x, y and res 16-byte aligned with pitches that are multiples of 16
 * select the vector paths; anything else takes slower element-wise paths with
 * identical results. */
int iconv2d_brelu(const icnn_conv_desc *desc, const void *x, const void *w_packed,
                  const int32_t *bias, const void *res, void *y, void *workspace,
                  void *stream);

/*
 * iconv2d_brelu for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * iconv2d_brelu, without `workspace`: layers that use one (iconv2d_workspace_bytes > 0) keep their
 * padded copy of x or their partial sums in a fixed array of ICNN_STATIC_WORKSPACE_BYTES bytes of device memory that the library's code
 * object carries (each GPU the library runs on holds its own copy until the process ends).  A layer that needs more
 * padded copy returns ICNN_E_SHAPE having launched nothing (partial sums that would not fit are simply not used: the
 * K axis stays whole).  The call allocates and frees nothing, on the host or the device.  The array's counter block
 * starts at zero when the library is loaded and every call leaves it at zero; all other bytes a layer reads it has
 * written in the same call.  All
 * calls on one GPU share it: calls that may overlap in time on one GPU (different streams, different threads)
 * race on it and must be serialised by the caller.
 */
#define ICNN_STATIC_WORKSPACE_BYTES (16u << 20)
int iconv2d_brelu_static_ws(const icnn_conv_desc *desc, const void *x, const void *w_packed,
                            const int32_t *bias, const void *res, void *y, void *stream);

/*
 * Per-output-channel requantisation (Section 3.4.3: with one weight step per output channel
 * before batch normalisation is merged, every output channel has its own ratio, so the
 * multiplier and shift of the requantisation equation of Section 3.2.1, and of the skip
 * rescale of Section 4.1, become vectors over the output channels).
 * Device arrays of cout int32 each, 4-byte aligned, owned by the caller:
 *   mul[c] in [1, 2^31-1], shift[c] in [0, 62]          (ignored for ICNN_OUT_RAW_S32)
 *   res_mul[c], res_shift[c], same domains              (NULL iff res_mode == NONE)
 * The values live in device memory, so the host cannot check their domains: values outside
 * them give unspecified output bytes for that channel, never a fault.
 */
typedef struct {
    const int32_t *mul;
    const int32_t *shift;
    const int32_t *res_mul;
    const int32_t *res_shift;
} icnn_channel_params;

/* Bytes of the packed form of a layer's per-channel parameters. */
int iconv2d_packed_channel_params_bytes(const icnn_conv_desc *desc, size_t *bytes);

/* Packs per-channel parameters (device arrays) into `packed` (device, 16-byte aligned,
 * iconv2d_packed_channel_params_bytes bytes).  Like the weights, they are constants of the
 * layer: done once, outside the inference loop.  The arrays may be released once the
 * stream has run the call. */
int iconv2d_prepack_channel_params(const icnn_conv_desc *desc, const icnn_channel_params *pc,
                                   void *packed, void *stream);

/* iconv2d_brelu with the layer's mul, shift, res_mul and res_shift replaced channel by channel
 * by the packed parameters (the descriptor's own four values must still be valid, e.g. 1 and
 * 0, and are not used; out_mode and res_mode must be those the parameters were packed for).
 * Everything else, including bound_q / lo / hi, the error codes and the alignment rules, is
 * as for iconv2d_brelu.  A raw int32 output without a skip operand has nothing per channel
 * and is rejected with ICNN_E_PARAM. */
int iconv2d_brelu_pc(const icnn_conv_desc *desc, const void *x, const void *w_packed,
                     const int32_t *bias, const void *pc_packed, const void *res,
                     void *y, void *workspace, void *stream);

/*
 * A residual block's last layer together with its projection skip, as one launch (Section
 * 4.1, the skip connection "after convolution": the projection convolves the quantised block
 * input, its int32 result is rescaled to the main path's ratio and added before BReLU).
 * Result: exactly that of
 *     iconv2d_brelu(proj, x_proj, w_proj_packed, bias_proj, NULL, tmp, ...);   // RAW_S32
 *     iconv2d_brelu(main, x_main, w_main_packed, bias_main, tmp, y, ...);      // res = tmp
 * without the int32 tensor tmp ever existing.  `main` must have res_mode = ICNN_RES_PRE and
 * res_dtype = ICNN_S32 (its res_mul / res_shift rescale the projection); `proj` must have
 * out_mode = ICNN_OUT_RAW_S32 and res_mode = ICNN_RES_NONE.  Both must be 1x1 convolutions
 * without padding (any stride) with cin % 16 == 0 that produce the same n x ho x wo x cout;
 * x, y and pitches 16-byte aligned.
 * Contract: |bias| <= 2^28 for both layers.  With it the library proves from the layer sizes
 * that Y_main + [Y_proj * res_mul / 2^res_shift] cannot leave int32; if it cannot prove that,
 * or a shape restriction fails, the call returns ICNN_E_UNSUPPORTED having launched nothing, and
 * the caller issues the two layers separately.
 */
int iconv2d_dual_brelu(const icnn_conv_desc *main_desc, const void *x_main, const void *w_main_packed,
                       const int32_t *bias_main, const icnn_conv_desc *proj_desc, const void *x_proj,
                       const void *w_proj_packed, const int32_t *bias_proj, void *y, void *stream);

/* iconv2d_dual_brelu with the main layer's mul, shift, res_mul and res_shift per output channel
 * (Section 3.4.3), taken from pc_packed_main = iconv2d_prepack_channel_params(main_desc, ...).
 * The host cannot read the per-channel skip rescales, so the proof that the merged sum stays
 * inside int32 uses main_desc->res_mul / 2^main_desc->res_shift as their upper bound: the
 * caller must set that pair to (at least) the largest per-channel ratio
 * res_mul[c] / 2^res_shift[c]; main_desc->mul and main_desc->shift are not used.  Otherwise as iconv2d_dual_brelu. */
int iconv2d_dual_brelu_pc(const icnn_conv_desc *main_desc, const void *x_main,
                          const void *w_main_packed, const int32_t *bias_main,
                          const void *pc_packed_main, const icnn_conv_desc *proj_desc,
                          const void *x_proj, const void *w_proj_packed,
                          const int32_t *bias_proj, void *y, void *stream);

/*
 * The first layer of a classification network together with the max-pool behind it, as one launch (Sections 3.1 and
 * 3.4.1 for the layer on the raw picture; Section 4.1 mentions the pooling layers of the integer ResNets).  Result:
 * exactly that of
 *     iconv2d_brelu(desc, x, w_packed, bias, NULL, t, workspace, ...);
 *     imaxpool2d_u8(n, ho, wo, cout, pool_k, pool_stride, pool_pad, t, y, ...);
 * without the convolution's output t or the workspace's padded copy of the picture ever existing.  y is NHWC
 * [n, hp, wp, desc->out_c_stride] and desc->out_c_stride / out_c_offset describe y (not t).  Shapes it takes: cin <= 4,
 * kernel 5..8 pixels wide and at most 8 high, stride 2, cout 32 or 64, an unsigned 8-bit output clamped from 0, no skip
 * operand, unsigned (<= 127) or raw-picture (in_sub128) input, pool 3 / 2 / 1, bias and y 16-byte aligned.  Anything else
 * returns ICNN_E_UNSUPPORTED having launched nothing, and the caller issues the two calls.
 */
int iconv2d_maxpool_brelu(const icnn_conv_desc *desc, int32_t pool_k, int32_t pool_stride, int32_t pool_pad,
                          const void *x, const void *w_packed, const int32_t *bias, void *y, void *stream);

/*
 * A whole identity bottleneck block of a residual network as one launch (Section 4.1: the block's layers with the
 * skip connection joining the last one before BReLU; Section 3.1 for each layer).  Result: exactly that of
 *     iconv2d_brelu(c1, x,  w1_packed, bias1, NULL, t1, ...);     // 1x1, stride 1, no padding
 *     iconv2d_brelu(c2, t1, w2_packed, bias2, NULL, t2, ...);     // 3x3, stride 1, padding 1
 *     iconv2d_brelu(c3, t2, w3_packed, bias3, res,  y,  ...);     // 1x1; res: usually x itself
 * without the middle tensors t1 and t2 ever existing in memory (every workgroup takes a spatial tile of the image
 * through all three layers and recomputes the 3x3 layer's one-pixel halo of t1).  c1 and c2 must store unsigned
 * bytes bounded by at most 127 (ICNN_OUT_BRELU_U8 or ICNN_OUT_CLAMP_U8) and take no skip operand; c3 may use any
 * output mode and skip mode.  Shapes it takes: c1->cout = c2->cin = c2->cout = c3->cin in {64, 128}; c1->cin a
 * multiple of 64 (at most 832 for a middle width of 64, 512 for 128); c3->cout a multiple of the middle width; all
 * strides 1; inputs ICNN_IN_U8_LE127; x, y, res and their pitches 16-byte aligned.  The descriptors' pitches and
 * offsets for t1 and t2 (c1->out_*, c2->in_c_stride, c2->out_*, c3->in_c_stride) are not used.  Anything else
 * returns ICNN_E_UNSUPPORTED having launched nothing, and the caller issues the three layers separately.
 */
int iconv2d_bottleneck_brelu(const icnn_conv_desc *c1, const void *x, const void *w1_packed, const int32_t *bias1,
                             const icnn_conv_desc *c2, const void *w2_packed, const int32_t *bias2,
                             const icnn_conv_desc *c3, const void *w3_packed, const int32_t *bias3, const void *res,
                             void *y, void *stream);

/*
 * The bottleneck block that opens a stage, projection skip included, as one launch (Section 4.1, the skip connection
 * "after convolution"; Section 3.1 for each layer).  Result: exactly that of
 *     iconv2d_brelu(c1, x,  w1_packed, bias1, NULL, t1, ...);                      // 1x1, stride 1
 *     iconv2d_brelu(c2, t1, w2_packed, bias2, NULL, t2, ...);                      // 3x3, stride 1, padding 1
 *     iconv2d_dual_brelu(c3, t2, w3_packed, bias3, cp, x, wp_packed, biasp, y, ...);   // 1x1 + 1x1 projection of x
 * without t1, t2 or the projection's int32 result ever existing.  c3 and cp as for iconv2d_dual_brelu (c3: res_mode
 * ICNN_RES_PRE, res_dtype ICNN_S32, its res_mul / res_shift rescale the projection; cp: ICNN_OUT_RAW_S32; |bias| <= 2^28;
 * the same no-overflow proof), c1 and c2 as for iconv2d_bottleneck_brelu.  Shape it takes: 64 -> 64 -> 64 -> 256 channels
 * with a 64 -> 256 projection, all strides 1 (the block after the max-pool in the bottleneck ResNets), an 8-bit output.
 * Anything else returns ICNN_E_UNSUPPORTED having launched nothing.
 */
int iconv2d_bottleneck_dual_brelu(const icnn_conv_desc *c1, const void *x, const void *w1_packed, const int32_t *bias1,
                                  const icnn_conv_desc *c2, const void *w2_packed, const int32_t *bias2,
                                  const icnn_conv_desc *c3, const void *w3_packed, const int32_t *bias3,
                                  const icnn_conv_desc *cp, const void *wp_packed, const int32_t *biasp, void *y, void *stream);

/*
 * Two pointwise layers as one launch: the 1x1 convolution that closes a residual block, skip operand merged in its
 * epilogue (Section 4.1; Section 3.1 for each layer), and the 1x1 convolution that opens the next block and reads
 * that result.  Result: exactly that of
 *     iconv2d_brelu(c3, t, w3_packed, bias3, res,  y, ...);       // 1x1, stride 1, no padding
 *     iconv2d_brelu(c1, y, w1_packed, bias1, NULL, z, ...);       // 1x1, stride 1, no padding
 * Both y and z are written (y is the next block's skip operand); the second layer multiplies y out of on-chip
 * memory instead of reading it back.  Shapes it takes: c3->cin = c1->cout in {64, 128, 256}; c3->cout = c1->cin a
 * multiple of 256 up to 2048; c3 stores unsigned bytes bounded by at most 127 from a lower clamp of 0 and takes
 * either no skip operand or an unsigned 8-bit one joined before requantisation whose rescale fits 32 bits; c1
 * stores unsigned bytes and takes no skip operand; inputs ICNN_IN_U8_LE127; t, res, y, z, the bias arrays and all
 * pitches 16-byte aligned.  c1->in_c_stride is not used (y's layout is c3's output layout).  Anything else returns
 * ICNN_E_UNSUPPORTED having launched nothing, and the caller issues the two layers separately.
 */
int iconv2d_pair_brelu(const icnn_conv_desc *c3, const void *t, const void *w3_packed, const int32_t *bias3, const void *res,
                       void *y, const icnn_conv_desc *c1, const void *w1_packed, const int32_t *bias1, void *z,
                       void *stream);

/*
 * Two branches of one input as one launch: the layers of different kernel sizes whose outputs are concatenated
 * (Section 4.1, zero-copy concatenation: each branch is calibrated to the shared bound and writes its channel range
 * of the common buffer; Section 3.1 for each layer).  Result: exactly that of
 *     iconv2d_brelu(ca, x, wa_packed, bias_a, NULL, ya, ...);
 *     iconv2d_brelu(cb, x, wb_packed, bias_b, NULL, yb, ...);
 * with x read once and, where ya == yb and the two channel ranges are neighbours, whole pixels written.  Every argument
 * is a device pointer; ya and yb may be the same buffer (the descriptors' out_c_stride / out_c_offset place each
 * branch), the two channel ranges must not overlap, and neither output may overlap x.  Shapes it takes: stride 1,
 * "same" padding, ca 5x5 with 64 input channels and cb 3x3, or ca 3x3 with 48 or 64 input channels and cb 1x1; at
 * most 32 output channels each; no skip operands; inputs ICNN_IN_U8_LE127; tensors below 2 GiB; x and
 * in_c_stride 16-byte aligned.  Anything else returns ICNN_E_UNSUPPORTED having launched nothing, and the caller issues
 * the two layers separately.
 */
int iconv2d_twin_brelu(const icnn_conv_desc *ca, const void *x, const void *wa_packed, const int32_t *bias_a, void *ya,
                       const icnn_conv_desc *cb, const void *wb_packed, const int32_t *bias_b, void *yb, void *stream);

/*
 * Rescaled feature-map addition (ratio synchronisation between feature maps,
 * Sections 3.4.2 and 4.1), as a stand-alone pass over memory:
 *   T   = sat32(a + [b * b_mul / 2^b_shift])
 *   out = T                                   (ICNN_OUT_RAW_S32)
 *       = clamp([T * mul / 2^shift], lo, hi)  (ICNN_OUT_CLAMP_U8: 0<=lo<=hi<=255;
 *                                              ICNN_OUT_LINEAR_S8: range is [-128,127])
 * a, b: count_pixels x c elements of a_dtype / b_dtype with the given pitches.
 */
typedef struct {
    int64_t count_pixels;
    int32_t c;
    int32_t a_c_stride, b_c_stride, out_c_stride, out_c_offset;
    int32_t a_dtype, b_dtype;      /* icnn_dtype                                   */
    int32_t out_mode;              /* CLAMP_U8, LINEAR_S8 or RAW_S32               */
    int32_t b_mul, b_shift, mul, shift, lo, hi;
} icnn_add_desc;

int iadd_rescale(const icnn_add_desc *desc, const void *a, const void *b, void *out,
                 void *stream);

/*
 * Explicit concatenation on the channel axis with per-input ratio
 * synchronisation (Algorithm 2, online half): input i (uint8, c_in[i] channels,
 * pitch in_c_stride[i]) lands at channel offset c_in[0] + ... + c_in[i-1] as
 *   clamp([in_i * mul[i] / 2^shift[i]], 0, bound_q).
 * mul = 1, shift = 0 copies.  `in` is a host array of n_in device pointers; the
 * other arrays are host arrays of n_in integers.  1 <= n_in <= 16.
 */
int iconcat(int32_t n_in, const void *const *in, const int32_t *c_in,
            const int32_t *in_c_stride, const int32_t *mul, const int32_t *shift,
            int32_t bound_q, int64_t count_pixels, void *out, int32_t out_c_stride,
            void *stream);

/* Max-pool on uint8 NHWC [n,h,w,c] (contiguous): the maximum over the window
 * positions that fall inside the image (Section 4.1 mentions pooling layers in
 * the integer ResNets; the maximum leaves the ratio unchanged). */
int imaxpool2d_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t k, int32_t stride,
                  int32_t pad, const void *x, void *out, void *stream);

/* Global average pool on uint8 NHWC [n,h,w,c] -> [n,c]:
 *   out = clamp([sum_{h,w} x * mul / 2^shift], 0, bound_q),  mul / 2^shift ~ 1/(h*w). */
int iavgpool_global_u8(int32_t n, int32_t h, int32_t w, int32_t c, int32_t mul,
                       int32_t shift, int32_t bound_q, const void *x, void *out,
                       void *stream);

/* Re-normalisation of a raw uint8 picture as a stand-alone pass (Section 3.4.1):
 * out[i] = x[i] - 128 stored as int8.  `count` elements; in place is allowed.
 * (iconv2d_brelu can do the same on the fly with in_sub128 = 1.) */
int irenormalize_u8(int64_t count, const void *x, void *out, void *stream);

/*
 * Measurement aids: the two roofs a convolution layer is judged against, as they are on the machine at hand
 * (nothing of the method is computed).  The caller times the launches.
 * icnn_peak_mfma_i8: `blocks` workgroups of four waves, each wave issuing iters * 8 register-only
 *   v_mfma_i32_32x32x32_i8 (65536 integer operations each): blocks * 4 * iters * 8 * 65536 operations in all.
 *   sink: device, blocks * 256 int32, overwritten.
 * icnn_peak_copy: dst[i] = src[i] over `bytes` bytes (device, 16-byte aligned, a multiple of 16; the ranges must
 *   not overlap): bytes read plus bytes written.
 */
int icnn_peak_mfma_i8(int32_t blocks, int32_t iters, void *sink, void *stream);
int icnn_peak_copy(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ICNN_H */
