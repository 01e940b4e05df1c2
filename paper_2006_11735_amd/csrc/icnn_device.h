// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace icnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Packed weight format: the cout axis is cut into chunks of 32 output channels and
// the K = kh*kw*cin axis (order kh, kw, ci) into steps of 64.  One (chunk, step) pair
// is 2048 bytes: [k32 half][lane 0..63][16 bytes], exactly the A-operand fragments
// of two v_mfma_i32_32x32x32_i8 issues.  Lane l carries matrix row l%32 and the 16
// k-values (l/32)*16.. of its half.  Matrix row r of a chunk is output channel
// 16*((r>>2)&1) + 4*(r>>3) + (r&3), which makes accumulator register i of a lane
// in half h = l/32 hold channel 16*h + i: sixteen consecutive channels per lane.
constexpr int kChunkCout = 32;
constexpr int kStepK = 64;
constexpr int kChunkBytes = 2048;
constexpr int kCoutPad = 128;   // chunk count is padded so any cout tile can over-read

// floor(n / d) by multiply-high: see fast_div()
struct FastDiv {
    unsigned mul, s1, s2;
};

struct ConvArgs {
    const uint8_t *x;
    const uint8_t *wp;
    const int32_t *bias;
    const void *res;
    void *out;
    int N, H, W, Cin, in_cs, Cout, KH, KW, sh, sw, ph, pw, Ho, Wo;
    int M;        // output pixels N*Ho*Wo
    int K;        // kh*kw*cin
    int ksteps;   // ceil(K / 64)
    int n_ct;     // cout tiles
    int n_tiles;  // cout tiles x pixel tiles
    int per_xcd;  // tiles handed to each of the 8 XCDs
    int n_vtiles; // 8 * per_xcd: tile slots including the padding ones
    unsigned x_bytes;     // extent of x the kernel may touch (direct-to-LDS kernel: < 2 GiB)
    unsigned wp_bytes;    // extent of the packed weights
    int nstages;          // LDS ring depth of the direct-to-LDS kernel
    FastDiv div_howo, div_wo;
    int out_cs, out_co;
    int mul, shift, lo, hi, out_mode;
    int res_mode, res_dtype, res_cs, res_mul, res_shift;
    uint32_t in_xor;   // 0x80808080 when the input is a raw picture (x - 128), else 0
    // Unsigned inputs up to 255 on signed matrix cores: activation fragments are XORed with frag_xor
    // (0x80808080: x - 128) when they leave LDS, and 128 * wsum[co] (wsum = sum of the channel's weights,
    // stored behind the packed weights) is added to the bias.  Zero padding and K tails are zero bytes
    // in LDS, i.e. -128 after the XOR, which the same correction turns back into 0.  Else 0 / unused.
    uint32_t frag_xor;
    const int32_t *wsum;
    int vec_out, vec_res;
    int vec_bias; // bias is 16-byte aligned and cout % 16 == 0
    int rq_fast;  // requantisation as one 32x32->64 multiply-add (mul_hi = mul << (32 - shift))
    int mul_hi;
    // requantisation in 32 bits: with lo = 0, clamping t to [0, t_hi] first (t_hi: the smallest t whose result is
    // hi) leaves the result unchanged, and then t * mul + 2^(shift-1) fits 32 bits unsigned with both factors
    // below 2^24, so one full-rate multiply-add and a shift finish it and no clamp of the result is needed
    int rq24, t_hi, rnd;
    int res_fast; // unsigned 8-bit skip operand whose rescale fits 32 bits
    int epi_vec;  // output (and skip operand) allow 16-byte accesses
    int epi_mode; // 4 * RES + RQ of the vector epilogue
    // per-output-channel requantisation: packed parameters (kPcGroupInts int32 per 16 channels, see
    // pc_prepack_kernel), null for the per-layer form.  pc_fast_ok: shape, alignment and skip operand
    // allow the fast epilogue form where a group's parameters do.
    const int32_t *pc;
    int pc_fast_ok;
    // Split K: the K steps of a tile are cut into ksplit equal ranges, each its own work unit (n_tiles then counts
    // units: unit u is range u % ksplit of tile u / ksplit).  A unit stores its int32 accumulators in ws_part; the
    // unit that arrives last at the tile's counter (ws_cnt, zero before the launch and reset by that unit) adds the
    // others' and runs the epilogue.  1: no split, nothing of this is touched.
    int ksplit;
    unsigned *ws_cnt;
    int32_t *ws_part;
};

// Workspace layout of a convolution call: counters first (zero-filled by the caller once, left zero by every call),
// then data (the padded copy of a small-cin layer, or the partial accumulators of a split K axis).
constexpr size_t kWsCounterBytes = 4096;
constexpr int kWsMaxSplitTiles = (int)(kWsCounterBytes / sizeof(unsigned));

// Packed per-channel parameters, per group of 16 output channels, int32 each:
//   [0,16) A  [16,32) L  [32,48) T  [48,64) C     requantisation of channel c, exact for every valid
//        (mul, shift):  [t*mul/2^shift], once clamped to the 8-bit output range, equals
//        clamp( hi32((clamp(t, ~T, T) << L) * A + 2^(31+C)) >> C )
//   [64,80) mul  [80,96) shift                   as given (general 64-bit form)
//   [96,112) res_mul  [112,128) res_shift
//   [128] flags: bit 0: the skip rescale of every channel of the group fits 32 bits for an 8-bit operand;
//                bit 1: every channel has L = 0, C = 0 and no clamp of t (ratio below one half, shift <= 32)
constexpr int kPcGroupInts = 144;
constexpr int kPcA = 0, kPcL = 16, kPcT = 32, kPcC = 48, kPcMul = 64, kPcShift = 80, kPcResMul = 96, kPcResShift = 112,
              kPcFlags = 128;

// Projection half of a fused type-2 residual block (see conv_dual.hip)
struct ProjArgs {
    const uint8_t *x;
    const uint8_t *wp;
    const int32_t *bias;
    int H, W, Cin, in_cs, sh, sw;
    int ksteps;
    unsigned x_bytes, wp_bytes;
    int res_mul, res_shift;
    int vec_bias;
};

// A fused identity bottleneck block (see conv_block.hip): geometry shared by its three layers
struct BlockArgs {
    const uint8_t *x;
    unsigned x_bytes;
    int x_cs;
    int N, H, W;
    int TH, TW, PW;               // output tile and patch row width TW + 2
    int tiles_x, tiles_per_img, n_tiles;
    int per_xcd;                  // tiles handed to each of the 8 XCDs (set by the launcher)
    unsigned inv_tw, inv_pw;      // q / TW = q * inv_tw >> 16 for q < 128; row / PW likewise for row < 160
    int k1;                       // K steps of the first layer: C / 64
    int nchunk3;                  // output channel chunks of the last layer: C / MID
};

// bytewise maximum of two words: even and odd bytes as 16-bit lanes
__device__ __forceinline__ uint32_t max_bytes(uint32_t x, uint32_t y)
{
    typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
    const uint32_t xe = x & 0x00ff00ffu, ye = y & 0x00ff00ffu, xo = (x >> 8) & 0x00ff00ffu, yo = (y >> 8) & 0x00ff00ffu;
    const u16x2 e = __builtin_elementwise_max(__builtin_bit_cast(u16x2, xe), __builtin_bit_cast(u16x2, ye));
    const u16x2 o = __builtin_elementwise_max(__builtin_bit_cast(u16x2, xo), __builtin_bit_cast(u16x2, yo));
    return __builtin_bit_cast(uint32_t, e) | (__builtin_bit_cast(uint32_t, o) << 8);
}

// [v / 2^s], round half up; arithmetic shift floors for negative values.
__device__ __forceinline__ int64_t rsr64(int64_t v, int s)
{
    return (v + ((int64_t(1) << s) >> 1)) >> s;
}

__device__ __forceinline__ int sat32(int64_t v)
{
    return v > INT32_MAX ? INT32_MAX : (v < INT32_MIN ? INT32_MIN : (int)v);
}

__device__ __forceinline__ int clampi64(int64_t v, int lo, int hi)
{
    return v < lo ? lo : (v > hi ? hi : (int)v);
}

__device__ __forceinline__ int load_elem(const void *p, size_t i, int dtype)
{
    if (dtype == 0) return ((const uint8_t *)p)[i];
    if (dtype == 1) return ((const int8_t *)p)[i];
    return ((const int32_t *)p)[i];
}

// Kernel-selection overrides (icnn_set_tuning): process-wide plain ints, read at every launch.  They change
// which kernel runs, never a result.  -1 / 0 = the library's own choice.
struct Tuning {
    int tile = -1;         // force tile shape 0..4 of the direct-to-LDS kernel (also keeps 3x3 layers off the patch kernel)
    int stages = 0;        // force the LDS ring depth of the direct-to-LDS kernel (2..6)
    int no_narrow = 0;     // keep one-to-four-channel layers on the tile kernels
    int no_fc = 0;         // keep few-pixel pointwise layers on the tile kernels
    int no_halo = 0;       // keep 3x3 layers on the tap-by-tap kernel
    int halo_tile = 0;     // patch-resident kernel: 1 = 128 x 128, 2 = 64 x 256
    int halo_always = 0;   // patch-resident kernel also with several tiles per workgroup and short K loops
    int no_stream = 0;     // single-channel 3x3 layers: lane-group kernel instead of the streaming one
    int no_plane = 0;      // keep few-channel layers on large pictures off the kernel with two-dimensional tiles
    int plane_no_pipe = 0; // that kernel without the instantiations that deal a row's epilogue out between matrix instructions
    int plane_always = 0;  // that kernel for every layer whose shape it accepts
    int no_pic = 0;        // keep stride-1 first layers (cin <= 4) on the padded copy + tile kernel
    int no_deep = 0;       // keep deep 3x3 layers on few pixels off the kernel whose waves split the K axis
    int deep_plain_walk = 0;   // that kernel with the tile order of the other kernels (measurement)
    int deep_always = 0;   // that kernel for every layer whose shape it accepts
    int block_any_form = 0; // LDS-ring block kernel: the instantiation that holds every epilogue form, also where one form would do
    int no_block64 = 0;    // fused bottleneck blocks with 64 middle channels: the LDS-ring kernel instead of the register-resident one
    int ksplit = 0;        // 0 library's choice; 1 never split the K axis; 2..8 this split where it divides the K steps
};
extern Tuning g_tuning;

// launchers (host)
// vec_in: 16-byte pieces of x never straddle a tap (dword aligned); direct_ok: they are also 16-byte aligned
hipError_t launch_conv(const ConvArgs &a, bool vec_in, bool direct_ok, hipStream_t st);
// bytes of split-K partial accumulators launch_conv would use for this layer when given a workspace (0: no split)
size_t conv_split_bytes(const ConvArgs &a, bool direct_ok);
hipError_t launch_conv_dual(const ConvArgs &a, const ProjArgs &q, hipStream_t st);
hipError_t allow_large_lds(const void *kernel);   // > 64 KiB of dynamic LDS, once per kernel function
bool conv_fc_applies(const ConvArgs &a);
hipError_t launch_conv_fc(const ConvArgs &a, hipStream_t st);
bool conv_halo_applies(const ConvArgs &a);
hipError_t launch_conv_halo(const ConvArgs &a, hipStream_t st);
bool conv_plane_applies(const ConvArgs &a);
hipError_t launch_conv_plane(const ConvArgs &a, hipStream_t st);
bool conv_plane_twin_ok(const ConvArgs &a, const ConvArgs &b);
hipError_t launch_conv_plane_twin(const ConvArgs &a, const ConvArgs &b, hipStream_t st);
bool conv_deep_applies(const ConvArgs &a);
hipError_t launch_conv_deep(const ConvArgs &a, hipStream_t st);
hipError_t launch_conv_pic(const ConvArgs &a, hipStream_t st);
hipError_t launch_conv_stem_pool(const ConvArgs &a, int hp, int wp, hipStream_t st);
bool conv_block_tile(int H, int W, BlockArgs &g);
size_t conv_block_lds_bytes(int mid, int c);
hipError_t launch_conv_block(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a2, const ConvArgs &a3, hipStream_t st);
size_t conv_block64_lds_bytes(int c_in, int c_out, bool proj);
bool conv_block64_takes(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a3);
bool conv_block64_proj_takes(const ConvArgs &a1, const ConvArgs &a3, const ProjArgs &pj);
hipError_t launch_conv_block64(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a2, const ConvArgs &a3, const ProjArgs *pj,
                               hipStream_t st);
size_t conv_pair_lds_bytes(int c, int mid2);
hipError_t launch_conv_pair(const ConvArgs &a3, const ConvArgs &a1, long long pixels, hipStream_t st);
bool conv_narrow_applies(const ConvArgs &a);
hipError_t launch_conv_narrow(const ConvArgs &a, hipStream_t st);
hipError_t launch_prepack(const int8_t *w, uint8_t *wp, int Cout, int K, int chunks, int ksteps, int KH, int KW,
                          int Cin, int rp, hipStream_t st);
hipError_t launch_wsum(const int8_t *w, int32_t *wsum, int Cout, int cout_padded, int k_true, hipStream_t st);
hipError_t launch_pc_prepack(const int32_t *mul, const int32_t *shift, const int32_t *res_mul, const int32_t *res_shift,
                             int cout, int32_t *packed, hipStream_t st);
hipError_t launch_pad_small_cin(const uint8_t *x, void *out, int N, int H, int W, int Cin, int in_cs, int ph, int pw,
                                int Hp, int Wp, uint32_t in_xor, hipStream_t st);

// [t * mul / 2^shift] clamped to [0, hi] for t >= 0 in 32 bits: with t first limited to t_hi, the
// smallest t whose result reaches hi, t * mul + 2^(shift-1) stays below 2^32 with both factors below
// 2^24 (one 24-bit multiply-add, one shift, no clamp of the result).  (mul, shift) are the caller's
// pair with common factors of two removed, which changes no result.  ok = 0: the pair does not fit.
struct Rq24 {
    int ok, mul, shift, t_hi, rnd;
};
static inline Rq24 make_rq24(long long mul, int shift, int hi)
{
    Rq24 r = {0, 0, 0, 0, 0};
    while (shift >= 2 && mul != 0 && (mul & 1) == 0) { mul /= 2; --shift; }
    if (hi < 0 || shift < 1 || shift > 31 || mul < 1 || mul >= (1 << 24)) return r;
    const long long half = 1LL << (shift - 1);
    const long long num = ((long long)hi << shift) - half;
    const long long t_hi = num <= 0 ? 0 : (num + mul - 1) / mul;
    if (t_hi >= (1 << 24) || t_hi * mul + half > 0xffffffffLL || ((t_hi * mul + half) >> shift) != hi) return r;
    r.ok = 1; r.mul = (int)mul; r.shift = shift; r.t_hi = (int)t_hi; r.rnd = (int)half;
    return r;
}

struct AddArgs {
    const void *a;
    const void *b;
    void *out;
    int64_t px;
    int c, a_cs, b_cs, out_cs, out_co, a_dt, b_dt, out_mode;
    int b_mul, b_shift, mul, shift, lo, hi;
    int mul_hi;   // mul << (32 - shift) when the fast requantisation applies
    Rq24 q24;     // add_u8_kernel's requantisation
};
hipError_t launch_add(const AddArgs &a, bool vec, hipStream_t st);
hipError_t launch_requant_copy(const uint8_t *in, uint8_t *out, int64_t px, int c, int in_cs,
                               int out_cs, int out_co, int mul, int shift, int bound, bool vec,
                               hipStream_t st);
// All branches of a concatenation in one launch (every branch 16-byte aligned with channel counts and
// pitches that are multiples of 16): a lane handles one 16-byte group of an output pixel.
struct ConcatArgs {
    const uint8_t *in[16];
    int c_end[16];      // first output channel after branch i
    int in_cs[16], mul[16], shift[16];
    Rq24 q[16];
    int n_in, out_cs, bound;
    uint8_t *out;
};
hipError_t launch_concat_vec(const ConcatArgs &a, int64_t px, hipStream_t st);
hipError_t launch_maxpool(const uint8_t *x, uint8_t *out, int n, int h, int w, int c, int k,
                          int stride, int pad, int ho, int wo, bool vec, hipStream_t st);
hipError_t launch_avgpool(const uint8_t *x, uint8_t *out, int n, int hw, int c, int mul, int shift,
                          int bound, hipStream_t st);
hipError_t launch_mfma_loop(int blocks, int iters, int *sink, hipStream_t st);
hipError_t launch_stream_copy(const void *src, void *dst, long long n16, hipStream_t st);
hipError_t launch_renorm(const uint8_t *x, uint8_t *out, int64_t count, bool vec, hipStream_t st);

}  // namespace icnn
