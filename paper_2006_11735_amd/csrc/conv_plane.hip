// Stride-1 "same" convolutions (3x3, 5x5) with few channels on large pictures: the layers of the restoration
// networks (a 5x5 layer 64 -> 32 on a 2560 x 1600 frame is 4 M pixels of K = 1600 for one 32-channel chunk).
//
// The tile kernels cut the flattened pixel axis into runs of consecutive pixels and gather the activation operand tap
// by tap: every K step copies 64 bytes per output pixel from L2 into LDS, i.e. a 5x5 layer moves each input byte 25
// times, and on a picture 2560 pixels wide a run of 256 pixels shares no input rows with its own taps' neighbours, so
// the patch-resident kernel of conv_halo.hip does not apply either.  Here the tile is two-dimensional:
//
//   tile     16 rows x 32 columns of one picture (hanging over its right and bottom edges where the picture is no multiple
//            of that: those outputs are computed and dropped); a pixel group of 32 is one tile row, wave w owns rows 2w and 2w + 1
//            (8 rows x 32 columns, one row per wave, for 3x3 layers of 64 channels on pictures with too few tiles)
//   patch    the (16 + k - 1) x (32 + k - 1) input pixels under the tile, all channels, in LDS (zeros outside the picture:
//            the layer's padding), double-buffered: the next tile's patch travels by direct-to-LDS copies while this
//            one is multiplied.  The 16-byte pieces of 64-channel pixels are swizzled by the pixel's column; 48-byte
//            pixels spread over the banks by themselves.
//   weights  the layer's packed weights (at most 50 KiB) stay in LDS for all the tiles a (persistent) workgroup walks
//   K loop   straight-line over the K fragments of 32: one weight fragment per channel chunk and one activation fragment
//            per tile row from LDS, fetched a step ahead, at addresses that are lane constants plus immediate offsets
//            (64 channels) or plus a per-half constant (48 channels, where the two 16-byte halves of a fragment may
//            lie in different taps).  No barrier inside a tile; one per tile.
//
// Every input byte crosses the memory system once (plus the patch overlap), and what bounds the loop is LDS: 1 + NCH
// fragment reads of 1 KiB per 2 NCH matrix instructions and wave.  Accumulator layout, packed weights and epilogue
// are those of the other kernels, so the results are the same bit for bit.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

constexpr int kPlaneTW = 32;               // tile width; its height is 8 x the rows a wave owns (RPW: 2, or 1 for small pictures)

#ifdef ICNN_PLANE_TRACE      // development aid: one wave of one workgroup stamps the clock; icnn_debug_trace_plane() copies the stamps out
__device__ unsigned long long g_plane_trace[256];
#define PLANE_TR(k)                                                                                              \
    do {                                                                                                         \
        if (blockIdx.x == 3 && wave == (ICNN_PLANE_TRACE) && lane == 0 && trn < 250)                             \
            g_plane_trace[trn++] = ((unsigned long long)(k) << 56) | (__builtin_amdgcn_s_memtime() & 0xffffffffffffffULL); \
    } while (0)
#else
#define PLANE_TR(k)
#endif

struct PlaneArgs {
    int tiles_x, tiles_per_img, n_tiles;
    int per_xcd;                // tiles handed to each of the 8 XCDs
    FastDiv div_tpi, div_tx;    // / tiles_per_img, / tiles_x
};

// Twin layers: a second convolution `b` of the same input whose kernel is the centre (KS - 2) x (KS - 2) of this one's
// (the 3x3 branch beside a 5x5 branch, the 1x1 beside a 3x3 of the restoration network's two-branch layers).  Its
// activation fragments are fragments this layer reads anyway; twin_frag() says which of its weight fragments, if any,
// multiplies the activation fragment f of the main layer.
template <int KS, int CIN>
constexpr int twin_frag(int f)
{
    constexpr int KSB = KS - 2;
    if (CIN == 64) {                                 // two fragments per tap
        const int t = f / 2, dy = t / KS, dx = t % KS;
        if (t >= KS * KS || dy < 1 || dy > KSB || dx < 1 || dx > KSB) return -1;
        return ((dy - 1) * KSB + (dx - 1)) * 2 + (f & 1);
    }
    // 48 channels, 3x3 beside 1x1: the centre tap starts at k = 4 * 48 = 6 * 32; its channels 32..47 share fragment 7 with
    // the next tap's first 16, which meet the zero padding of the twin's K axis
    return f == 6 ? 0 : (f == 7 ? 1 : -1);
}

// kernel size, input channels (48 or 64), 32-channel chunks of the output (1 or 2), chunks of the twin layer (0: none, or 1),
// tile rows per wave (2: tiles of 16 x 32 pixels; 1: 8 x 32, twice the tiles for pictures that have too few).
// PIPE (3x3 layers with the weights in registers, outputs stored as unsigned bytes by the 32-bit requantisation form, no
// skip operand; the host checks): a wave takes its two rows one after the other and deals the first row's epilogue out
// between the second row's matrix instructions.  With a short K loop the epilogue's vector instructions take as long
// as the loop, and because the barrier per tile keeps the two waves of a SIMD in step, both multiplied and then both
// ran epilogues: 2.1 k clocks of matrix work, then 2.9 k of vector work, per tile.
template <int KS, int CIN, int NCH, int NB, int RPW, bool PIPE>
__global__ __launch_bounds__(512, 1) void conv_plane_kernel(const ConvArgs a, const ConvArgs b, const PlaneArgs g)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr unsigned OOB = 0x80000000u;            // beyond any buffer this kernel accepts (< 2 GiB)
    constexpr int PAD = KS / 2;
    constexpr int TH = 8 * RPW;
    constexpr int PH = TH + KS - 1, PW = kPlaneTW + KS - 1;
    constexpr int PWL = (PW + 3) & ~3;               // pixels per patch row in LDS: whole groups of four
    constexpr int PPT = CIN / 16;                    // 16-byte pieces per pixel (= per tap)
    constexpr int ROWB = PWL * CIN;                  // bytes per patch row
    constexpr int K = KS * KS * CIN;
    constexpr int KSTEPS = (K + 63) / 64;
    constexpr int F = 2 * KSTEPS;                    // fragments of 32 k-values, the zero-padded tail included
    constexpr int PIECES = PH * PWL * PPT;
    constexpr int NCOPY = (PIECES + 63) / 64;        // wave-wide 1 KiB copies per patch
    constexpr int CPW = (NCOPY + 7) / 8;             // per wave
    constexpr int PATCH = NCOPY * 1024;
    constexpr int WBYTES = NCH * KSTEPS * kChunkBytes;
    constexpr int KSB = KS - 2;
    constexpr int KSTEPSB = NB ? (KSB * KSB * CIN + 63) / 64 : 0, FB = 2 * KSTEPSB;
    constexpr int WBYTESB = NB * KSTEPSB * kChunkBytes;
    static_assert(CIN == 48 || CIN == 64, "row layouts exist for 48 and 64 channels");
    static_assert(NB == 0 || CIN == 64 || KS == 3, "twin_frag() covers 64 channels, and 48 channels at 3x3 beside 1x1");
    static_assert(WBYTES + WBYTESB + 2 * PATCH <= 160 * 1024, "LDS");
    static_assert((PH + 1) * ROWB < 65536, "fragment reads address rows and taps through the instruction's 16-bit offset");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    uint8_t *const wbuf = lds;
    [[maybe_unused]] uint8_t *const wbufB = lds + WBYTES;
    uint8_t *const pbuf = lds + WBYTES + WBYTESB;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, col = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    [[maybe_unused]] int trn = 0;
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);

    // Work slot v (blockIdx.x, + gridDim.x, ...; the grid is a multiple of 8) is tile (v & 7) * per_xcd + (v >> 3): the
    // workgroups of an XCD walk a contiguous range of tiles, so the patch borders neighbouring tiles share meet in one L2.
    auto tile_of = [&](int v) { return (v & 7) * g.per_xcd + (v >> 3); };
    auto valid = [&](int v) { return (v >> 3) < g.per_xcd && tile_of(v) < g.n_tiles; };
    auto tile_origin = [&](int v, int &n, int &y0, int &x0) {
        const int t = tile_of(v);
        n = fast_div(t, g.div_tpi);
        const int r = t - n * g.tiles_per_img;
        const int ty = fast_div(r, g.div_tx);
        y0 = ty * TH;
        x0 = (r - ty * g.tiles_x) * kPlaneTW;
    };

    // Patch layout in LDS: pixel (py, px) at (py * PWL + px) * CIN.  64-byte pixels: the 16-byte piece c of a pixel lives in
    // slot c ^ ((px >> 2) & 3), so that the fragment reads of 16 consecutive pixels hit every bank once (rows are whole
    // multiples of 256 bytes, so the row does not enter); 48-byte pixels spread over the banks by themselves.
    // Copy e of a patch covers LDS bytes [1024 e, 1024 e + 1024): what this lane fetches for each of its copies does not
    // depend on the tile but for the origin: the piece's offset from the patch's first pixel, and (py, px) for the
    // check against the picture's borders (a lane beyond the patch gets py = 0x7fff, which never passes it).
    int p_rel[CPW], p_yx[CPW];
#pragma unroll
    for (int i = 0; i < CPW; ++i) {
        const int q = (wave + 8 * i) * 64 + lane;
        const int pix = q / PPT, slot = q - pix * PPT;
        const int py = pix / PWL, px = pix - py * PWL;
        const int logical = CIN == 64 ? slot ^ ((px >> 2) & 3) : slot;
        const bool in_patch = q < PIECES && px < PW;
        p_rel[i] = (py * a.W + px) * a.in_cs + logical * 16;
        p_yx[i] = ((in_patch ? py : 0x7fff) << 16) | px;
    }
    // copy i of this wave for the patch whose first pixel is picture pixel (n, y0 - PAD, x0 - PAD), into buffer b
    auto issue_copy = [&](auto i_tag, int base, int y0, int x0, int b) {
        constexpr int i = decltype(i_tag)::value;
        const int e = wave + 8 * i;
        if (e < NCOPY) {                             // wave-uniform
            const int iy = y0 - PAD + (p_yx[i] >> 16), ix = x0 - PAD + (p_yx[i] & 0xffff);
            const bool ok = ((unsigned)iy < (unsigned)a.H) & ((unsigned)ix < (unsigned)a.W);
            const unsigned off = ok ? (unsigned)(base + p_rel[i]) : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)(pbuf + b * PATCH + e * 1024), 16, off,
                                                     0, 0, 0);
        }
    };
    // byte offset of that first pixel (may be negative: only pixels inside the picture use it)
    auto patch_base = [&](int n, int y0, int x0) { return ((n * a.H + y0 - PAD) * a.W + x0 - PAD) * a.in_cs; };
    auto issue_patch = [&](int v, int b) {
        int n, y0, x0;
        tile_origin(v, n, y0, x0);
        const int base = patch_base(n, y0, x0);
        static_for<CPW>([&](auto i_tag) { issue_copy(i_tag, base, y0, x0, b); });
    };

    if (valid(blockIdx.x)) issue_patch(blockIdx.x, 0);
    PLANE_TR(0);
    // weights: a straight copy of the first NCH chunks (the packed order is the fragment order)
    // (direct-to-LDS copies as well, 1 KiB per wave and copy, all in flight together with the first patch: through
    // registers the copy loop waited out one memory latency per 8 KiB, five of them for a 3x3 layer of 64 channels, which
    // is most of the kernel's time on a picture with one tile per workgroup)
    {
        const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, a.wp_bytes, 0x00020000);
#pragma unroll
        for (int e0 = 0; e0 < WBYTES / 1024; e0 += 8) {
            const int e = e0 + wave;
            if (e < WBYTES / 1024)                   // wave-uniform
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (__attribute__((address_space(3))) void *)(wbuf + e * 1024), 16,
                                                         (unsigned)(e * 1024 + lane * 16), 0, 0, 0);
        }
        if constexpr (NB > 0) {
            const __amdgpu_buffer_rsrc_t rs_wb = __builtin_amdgcn_make_buffer_rsrc((void *)b.wp, 0, b.wp_bytes, 0x00020000);
#pragma unroll
            for (int e0 = 0; e0 < WBYTESB / 1024; e0 += 8) {
                const int e = e0 + wave;
                if (e < WBYTESB / 1024)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wb, (__attribute__((address_space(3))) void *)(wbufB + e * 1024), 16,
                                                             (unsigned)(e * 1024 + lane * 16), 0, 0, 0);
            }
        }
    }
    v16i bias[NCH];
    load_bias_rows<NCH>(a, 0, half, bias);
    [[maybe_unused]] v16i biasB[NB ? NB : 1];
    if constexpr (NB > 0) load_bias_rows<NB>(b, 0, half, biasB);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0), lgkmcnt(0): the first patch and the weights are in LDS
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // This lane's output pixels: tile rows 2 wave + j, column col.  Fragment f of tap (dy, dx) is, for this half of the
    // wave, piece pc of patch pixel (2 wave + j + dy, col + dx).  64 channels: both halves read the same tap, pieces 2 k
    // and 2 k + 1, so per dx and k the lane's byte offset within a patch row is a constant of the lane (ex[dx][k]) and
    // row and j go into the read's immediate offset: no address arithmetic in the K loop.  48 channels: the halves may
    // read different taps; the offset is linear, base + a per-half constant.
    const uint8_t *const wlane = wbuf + lane * 16;
    // 3x3 layers with one channel chunk: the weight fragments fit in registers (18 or 14) and stay there for all tiles, which takes a
    // third to a half of the K loop's LDS reads away; 5x5 layers (50 fragments) read them from LDS every time
    constexpr bool AREG = KS == 3 && NCH == 1 && !(NB > 0 && CIN == 64);      // (with a twin at 64 channels they spill)
    [[maybe_unused]] v4i wreg[AREG ? NCH : 1][AREG ? F : 1];
    if constexpr (AREG) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int f = 0; f < F; ++f) wreg[c][f] = *(const v4i *)(wlane + (c * F + f) * 1024);
    }
    [[maybe_unused]] const uint8_t *const wlaneB = wbufB + lane * 16;
    [[maybe_unused]] int ex[KS][2];
    [[maybe_unused]] int lin = 0;
    if constexpr (CIN == 64) {
#pragma unroll
        for (int dx = 0; dx < KS; ++dx)
#pragma unroll
            for (int k = 0; k < 2; ++k)
                ex[dx][k] = (RPW * wave) * ROWB + (col + dx) * 64 + (((2 * k + half) ^ (((col + dx) >> 2) & 3)) << 4);
    } else {
        lin = (RPW * wave) * ROWB + col * CIN;
    }
    // 8-bit output with at most the plain 8-bit skip operand, whole groups of 16 channels: sixteen bytes per lane and
    // pixel straight from epilogue_bytes16 (the general epilogue's dispatch costs as much as a 3x3 tile's K loop here)
    const bool quick = a.epi_vec && a.out_mode <= 1 && a.epi_mode / 4 != 2 && (a.Cout & 15) == 0;
    const bool has_res = a.res_mode != 0;
    // One to four output channels (the regression networks' last layer): a lane of the first half holds them in its
    // first accumulator registers; element-wise epilogue, in 32 bits where the layer's parameters allow, the skip
    // operand fetched before the K loop (a load inside the epilogue would be waited for on the spot)
    constexpr bool THIN_OK = NCH == 1 && NB == 0;        // (the twin instantiations have no registers to spare for it)
    const bool thin = THIN_OK && a.Cout <= 4;
    const bool thin32 = a.out_mode != 3 && a.rq_fast && (a.res_mode == 0 || a.res_fast);
    [[maybe_unused]] const bool quickB = NB && b.epi_vec && b.out_mode <= 1 && b.epi_mode / 4 == 0 && (b.Cout & 15) == 0;

    int buf = 0;
    for (int v = blockIdx.x; valid(v); v += gridDim.x) {
        PLANE_TR(1);
        int n, y0, x0;
        tile_origin(v, n, y0, x0);
        // The next tile's patch travels during this tile.  (A third buffer, i.e. two patches in flight per workgroup, measured
        // no faster: at these sizes the layers with short K loops run at what the memory system gives this access
        // pattern, 3.2 TB/s.)  Its copies are issued one by one between the K steps: issued together at the tile's start
        // they fill the memory pipeline's queue and every wave sits on them for ~ 900 clocks.
        const bool more = valid(v + (int)gridDim.x);
        int nn = 0, ny0 = 0, nx0 = 0;
        if (more) tile_origin(v + (int)gridDim.x, nn, ny0, nx0);
        const int nbase = patch_base(nn, ny0, nx0);
        PLANE_TR(2);
        const uint8_t *const P = pbuf + buf * PATCH;

        if constexpr (PIPE) {
            static_assert(!PIPE || (AREG && RPW == 2 && NCH == 1), "the pipelined form is for register-resident 3x3 weights");
            v16i accp[2], accq[2];                   // [row] of the layer and of its twin
            accp[0] = accp[1] = bias[0];
            if constexpr (NB > 0) accq[0] = accq[1] = biasB[0];
            v4i Bf[2];
            [[maybe_unused]] v4i ABf[2];
            auto fetch1 = [&](auto f_tag, auto j_tag) {
                constexpr int f = decltype(f_tag)::value, j = decltype(j_tag)::value, S = f & 1;
                constexpr int P0 = 2 * f, P1 = 2 * f + 1;
                constexpr int T0 = P0 / PPT < KS * KS ? P0 / PPT : KS * KS - 1, T1 = P1 / PPT < KS * KS ? P1 / PPT : KS * KS - 1;
                if constexpr (NB > 0 && twin_frag<KS, CIN>(f) >= 0) ABf[S] = *(const v4i *)(wlaneB + twin_frag<KS, CIN>(f) * 1024);
                if constexpr (CIN == 64) {
                    constexpr int DY = T0 / KS, DX = T0 % KS, KK = (P0 % PPT) / 2;
                    Bf[S] = *(const v4i *)(P + ex[DX][KK] + (j + DY) * ROWB);
                } else {
                    constexpr int O0 = (T0 / KS) * ROWB + (T0 % KS) * CIN + (P0 % PPT) * 16;
                    constexpr int O1 = (T1 / KS) * ROWB + (T1 % KS) * CIN + (P1 % PPT) * 16;
                    Bf[S] = *(const v4i *)(P + lin + (half ? O1 : O0) + j * ROWB);
                }
            };
            // one K step of row j; g = its position among the 2 F steps of the tile (the next patch's copies are spread over them)
            auto step1 = [&](auto f_tag, auto j_tag) {
                constexpr int f = decltype(f_tag)::value, j = decltype(j_tag)::value, g2 = j * F + f;
                if constexpr (f + 1 < F) fetch1(std::integral_constant<int, f + 1>{}, j_tag);
                constexpr int EVERY = 2 * F / CPW;
                if constexpr (g2 % EVERY == 0 && g2 / EVERY < CPW) {
                    if (more) issue_copy(std::integral_constant<int, g2 / EVERY>{}, nbase, ny0, nx0, buf ^ 1);
                }
                accp[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[0][f], Bf[f & 1], accp[j], 0, 0, 0);
                if constexpr (NB > 0 && twin_frag<KS, CIN>(f) >= 0)
                    accq[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ABf[f & 1], Bf[f & 1], accq[j], 0, 0, 0);
            };
            fetch1(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
            static_for<F>([&](auto f_tag) { step1(f_tag, std::integral_constant<int, 0>{}); });
            mfma_drain(accp[0]);
            if constexpr (NB > 0) mfma_drain(accq[0]);
            // the second row; the first row's 16 (+ 16) outputs are requantised a few at a time behind its matrix instructions
            int wa[4] = {0, 0, 0, 0};
            [[maybe_unused]] int wb[4] = {0, 0, 0, 0};
            const v4i none = {0, 0, 0, 0};
            fetch1(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{});
            static_for<F>([&](auto f_tag) {
                constexpr int f = decltype(f_tag)::value;
                step1(f_tag, std::integral_constant<int, 1>{});
                constexpr int NOUT = 16 + 16 * NB, LO = f * NOUT / F, HI = (f + 1) * NOUT / F;
                constexpr int A0 = LO < 16 ? LO : 16, A1 = HI < 16 ? HI : 16;
                if constexpr (A1 > A0) epilogue_rq24_slice<0, A0, A1 - A0>(a, accp[0], none, wa);
                if constexpr (NB > 0 && HI > 16) {
                    constexpr int B0 = LO > 16 ? LO - 16 : 0, B1 = HI - 16;
                    if constexpr (B1 > B0) epilogue_rq24_slice<0, B0, B1 - B0>(b, accq[0], none, wb);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            const int co0 = half * 16;
            const bool colok = x0 + col < a.W;        // tiles may hang over the picture's right and bottom edges
            if (colok && y0 + 2 * wave < a.H) {
                const size_t p = (size_t)((n * a.H + y0 + 2 * wave) * a.W + x0 + col);
                if (co0 < a.Cout) *(v4i *)((uint8_t *)a.out + p * a.out_cs + a.out_co + co0) = v4i{wa[0], wa[1], wa[2], wa[3]};
                if constexpr (NB > 0)
                    if (co0 < b.Cout) *(v4i *)((uint8_t *)b.out + p * b.out_cs + b.out_co + co0) = v4i{wb[0], wb[1], wb[2], wb[3]};
            }
            mfma_drain(accp[1]);
            if constexpr (NB > 0) mfma_drain(accq[1]);
            if (colok && y0 + 2 * wave + 1 < a.H) {
                const size_t p = (size_t)((n * a.H + y0 + 2 * wave + 1) * a.W + x0 + col);
                if (co0 < a.Cout) *(v4i *)((uint8_t *)a.out + p * a.out_cs + a.out_co + co0) = epilogue_bytes16<0, 3>(a, accp[1], none);
                if constexpr (NB > 0)
                    if (co0 < b.Cout) *(v4i *)((uint8_t *)b.out + p * b.out_cs + b.out_co + co0) = epilogue_bytes16<0, 3>(b, accq[1], none);
            }
        } else {
        [[maybe_unused]] int resv[RPW][THIN_OK ? 4 : 1] = {};
        if (THIN_OK && thin && has_res && half == 0) {
#pragma unroll
            for (int j = 0; j < RPW; ++j)
                if (y0 + RPW * wave + j < a.H && x0 + col < a.W) {
                    const size_t ro = (size_t)((n * a.H + y0 + RPW * wave + j) * a.W + x0 + col) * a.res_cs;
#pragma unroll
                    for (int co = 0; co < 4; ++co)
                        if (co < a.Cout) resv[j][THIN_OK ? co : 0] = load_elem(a.res, ro + co, a.res_dtype);
                }
        }
        v16i acc[RPW][NCH][1];
#pragma unroll
        for (int j = 0; j < RPW; ++j)
#pragma unroll
            for (int c = 0; c < NCH; ++c) acc[j][c][0] = bias[c];
        [[maybe_unused]] v16i accB[RPW][NB ? NB : 1][1];
        if constexpr (NB > 0) {
#pragma unroll
            for (int j = 0; j < RPW; ++j)
#pragma unroll
                for (int c = 0; c < NB; ++c) accB[j][c][0] = biasB[c];
        }
        v4i A[2][NCH], B[2][RPW];
        [[maybe_unused]] v4i AB[2][NB ? NB : 1];
        // pieces in the zero-padded tail of K read the last tap again (their weights are zeros)
        auto fetch = [&](auto f_tag, auto set_tag) {
            constexpr int f = decltype(f_tag)::value, S = decltype(set_tag)::value;
            constexpr int P0 = 2 * f, P1 = 2 * f + 1;
            constexpr int T0 = P0 / PPT < KS * KS ? P0 / PPT : KS * KS - 1, T1 = P1 / PPT < KS * KS ? P1 / PPT : KS * KS - 1;
            if constexpr (!AREG) {
#pragma unroll
                for (int c = 0; c < NCH; ++c) A[S][c] = *(const v4i *)(wlane + (c * F + f) * 1024);
            }
            if constexpr (NB > 0 && twin_frag<KS, CIN>(f) >= 0) {       // the twin's few fragments always come from LDS
#pragma unroll
                for (int c = 0; c < NB; ++c) AB[S][c] = *(const v4i *)(wlaneB + (c * FB + twin_frag<KS, CIN>(f)) * 1024);
            }
            if constexpr (CIN == 64) {
                static_assert(CIN != 64 || T0 == T1, "a fragment of a 64-channel layer lies in one tap");
                constexpr int DY = T0 / KS, DX = T0 % KS, KK = (P0 % PPT) / 2;
#pragma unroll
                for (int j = 0; j < RPW; ++j) B[S][j] = *(const v4i *)(P + ex[DX][KK] + (j + DY) * ROWB);
            } else {
                constexpr int O0 = (T0 / KS) * ROWB + (T0 % KS) * CIN + (P0 % PPT) * 16;
                constexpr int O1 = (T1 / KS) * ROWB + (T1 % KS) * CIN + (P1 % PPT) * 16;
                const int o = lin + (half ? O1 : O0);
#pragma unroll
                for (int j = 0; j < RPW; ++j) B[S][j] = *(const v4i *)(P + o + j * ROWB);
            }
        };
        fetch(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        static_for<F>([&](auto f_tag) {
            constexpr int f = decltype(f_tag)::value;
            if constexpr (f + 1 < F) fetch(std::integral_constant<int, f + 1>{}, std::integral_constant<int, (f + 1) & 1>{});
            constexpr int EVERY = F / CPW;            // a copy of the next patch every so many steps
            if constexpr (f % EVERY == 0 && f / EVERY < CPW) {
                if (more) issue_copy(std::integral_constant<int, f / EVERY>{}, nbase, ny0, nx0, buf ^ 1);
            }
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int j = 0; j < RPW; ++j)
                    acc[j][c][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(AREG ? wreg[AREG ? c : 0][AREG ? f : 0] : A[f & 1][c], B[f & 1][j],
                                                                         acc[j][c][0], 0, 0, 0);
            if constexpr (NB > 0 && twin_frag<KS, CIN>(f) >= 0) {
#pragma unroll
                for (int c = 0; c < NB; ++c)
#pragma unroll
                    for (int j = 0; j < RPW; ++j)
                        accB[j][c][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(AB[f & 1][c], B[f & 1][j], accB[j][c][0], 0, 0, 0);
            }
        });
        PLANE_TR(3);
        static_for<RPW>([&](auto j_tag) {
            constexpr int j = decltype(j_tag)::value;
            mfma_drain(acc[j]);
            // a tile row's 32 pixels are consecutive pixels of the output tensor
            // (tiles may hang over the picture's bottom and right edges: those rows and columns are computed and dropped)
            const int pix_row = (n * a.H + y0 + RPW * wave + j) * a.W + x0;
            const bool rowok = y0 + RPW * wave + j < a.H, pixok = rowok && x0 + col < a.W;
            if (thin) {
                if (pixok && half == 0) {
                    const size_t oo = (size_t)(pix_row + col) * a.out_cs + a.out_co;
                    static_for<4>([&](auto co_tag) {
                        constexpr int co = decltype(co_tag)::value;
                        if (co < a.Cout) epilogue_one(a, acc[j][0][0][co], resv[j][THIN_OK ? co : 0], oo + co, thin32);
                    });
                }
            } else if (quick) {
                const size_t p = (size_t)(pix_row + col);
                static_for<NCH>([&](auto c_tag) {
                    constexpr int c = decltype(c_tag)::value;
                    const int co0 = c * 32 + half * 16;
                    if (co0 < a.Cout && pixok) {
                        v4i r8 = {0, 0, 0, 0};
                        if (has_res) r8 = *(const v4i *)((const uint8_t *)a.res + p * a.res_cs + co0);
                        const v4i w = has_res ? epilogue_bytes16<1>(a, acc[j][c][0], r8) : epilogue_bytes16<0>(a, acc[j][c][0], r8);
                        *(v4i *)((uint8_t *)a.out + p * a.out_cs + a.out_co + co0) = w;
                    }
                });
            } else if (rowok) {
                epilogue_tiles<NCH, 1>(a, acc[j], 0, pixok ? pix_row : a.M, lane);      // a pixel index of M or more is skipped
            }
            if constexpr (NB > 0) {
                mfma_drain(accB[j]);
                if (quickB) {
                    const size_t p = (size_t)(pix_row + col);
                    static_for<NB>([&](auto c_tag) {
                        constexpr int c = decltype(c_tag)::value;
                        const int co0 = c * 32 + half * 16;
                        if (co0 < b.Cout && pixok)
                            *(v4i *)((uint8_t *)b.out + p * b.out_cs + b.out_co + co0) = epilogue_bytes16<0>(b, accB[j][c][0], v4i{0, 0, 0, 0});
                    });
                } else if (rowok) {
                    epilogue_tiles<NB, 1>(b, accB[j], 0, pixok ? pix_row : b.M, lane);
                }
            }
        });
        }
        PLANE_TR(4);
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT(0);                          // the next tile's patch has landed (this wave's copies of it)
        __builtin_amdgcn_s_waitcnt(0xC07F);          // and this wave has read the last of this tile's patch
        PLANE_TR(5);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        buf ^= 1;
    }
#endif
}

#ifdef ICNN_PLANE_TRACE
extern "C" int icnn_debug_trace_plane(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_plane_trace), sizeof(unsigned long long) * 256);
}
#endif

// ------------------------------------------------------------------ dispatch
static int plane_nch(const ConvArgs &a) { return (a.Cout + 31) / 32; }

static bool plane_shape_ok(const ConvArgs &a)
{
    if (a.KH != a.KW || (a.KH != 3 && a.KH != 5) || a.sh != 1 || a.sw != 1 || a.ph != a.KH / 2 || a.pw != a.KW / 2) return false;
    if ((a.Cin != 48 && a.Cin != 64) || a.in_cs % 16 || ((uintptr_t)a.x & 15) || a.in_xor || a.frag_xor || a.pc) return false;
    if (a.Ho != a.H || a.Wo != a.W || a.x_bytes >= 0x7fffff00u) return false;
    if (a.ksteps != (a.KH * a.KW * a.Cin + 63) / 64) return false;
    const int nch = plane_nch(a);
    // the instantiations that exist (launch_conv_plane)
    if (a.KH == 5) return a.Cin == 64 && nch == 1;
    return nch <= 2;
}

// Tile rows per wave: 2 (tiles of 16 x 32 pixels) where the picture gives every compute unit several tiles, else 1 for
// the 3x3 layers of 64 channels; 0: the layer is not worth this kernel.
static int plane_rpw(const ConvArgs &a)
{
    const int tx = (a.W + kPlaneTW - 1) / kPlaneTW;
    const long long tiles8 = (long long)a.N * ((a.H + 7) / 8) * tx;
    // tiles hang over the right and bottom edges of pictures that are no multiples of them: not where that is more than
    // a quarter of the work
    if (!g_tuning.plane_always && (a.W * 4 < tx * kPlaneTW * 3 || a.H < 8)) return 0;
    if (tiles8 >= 2048 || (g_tuning.plane_always && !(a.KH == 3 && a.Cin == 64 && tiles8 < 512))) return 2;
    if (a.KH == 3 && a.Cin == 64 && (tiles8 >= 192 || g_tuning.plane_always)) return 1;
    return g_tuning.plane_always ? 2 : 0;
}

bool conv_plane_applies(const ConvArgs &a)
{
    if (!plane_shape_ok(a)) return false;
    // (pointwise layers gain nothing from a resident patch and are not taken at all: 120 against 101 us at 48 -> 32
    // channels on 2560 x 1600)
    return plane_rpw(a) != 0;
}

template <int KS, int CIN, int NCH, int NB = 0, int RPW = 2, bool PIPE = false>
static hipError_t launch_plane(const ConvArgs &a, const ConvArgs &b, hipStream_t st)
{
    PlaneArgs g;
    g.tiles_x = (a.W + kPlaneTW - 1) / kPlaneTW;
    g.tiles_per_img = g.tiles_x * ((a.H + 8 * RPW - 1) / (8 * RPW));
    const long long tiles = (long long)g.tiles_per_img * a.N;
    if (tiles < 1 || tiles > 0x7ffffff0LL) return hipErrorInvalidValue;
    g.n_tiles = (int)tiles;
    g.per_xcd = (int)((tiles + 7) / 8);
    g.div_tpi = make_fast_div((unsigned)g.tiles_per_img);
    g.div_tx = make_fast_div((unsigned)g.tiles_x);
    constexpr int PH = 8 * RPW + KS - 1, PW = kPlaneTW + KS - 1;
    constexpr int NCOPY = (PH * ((PW + 3) & ~3) * (CIN / 16) + 63) / 64;
    constexpr int KSTEPS = (KS * KS * CIN + 63) / 64;
    constexpr int KSTEPSB = NB ? ((KS - 2) * (KS - 2) * CIN + 63) / 64 : 0;
    const size_t lds_bytes = (size_t)(NCH * KSTEPS + NB * KSTEPSB) * kChunkBytes + 2 * (size_t)NCOPY * 1024;
    const auto kernel = conv_plane_kernel<KS, CIN, NCH, NB, RPW, PIPE>;
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_large_lds((const void *)kernel);
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)(8 * g.per_xcd < 256 ? 8 * g.per_xcd : 256)), block(512);
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a, b, g);
    return hipGetLastError();
}

// what the pipelined instantiations assume of a layer: unsigned bytes by the 32-bit requantisation form, whole groups of
// 16 channels, 16-byte stores, no skip operand
static bool plane_pipe_ok(const ConvArgs &a)
{
    return a.epi_vec && a.out_mode <= 1 && a.res_mode == 0 && (a.Cout & 15) == 0 && a.rq24 && !g_tuning.plane_no_pipe;
}

hipError_t launch_conv_plane(const ConvArgs &a, hipStream_t st)
{
    if (!plane_shape_ok(a)) return hipErrorInvalidValue;
    const int nch = plane_nch(a), rpw = plane_rpw(a);
    if (rpw == 0) return hipErrorInvalidValue;
    if (a.KH == 5) return launch_plane<5, 64, 1>(a, a, st);
    if (a.Cin == 64 && rpw == 1) return nch == 1 ? launch_plane<3, 64, 1, 0, 1>(a, a, st) : launch_plane<3, 64, 2, 0, 1>(a, a, st);
    if (nch == 1 && plane_pipe_ok(a)) return a.Cin == 64 ? launch_plane<3, 64, 1, 0, 2, true>(a, a, st) : launch_plane<3, 48, 1, 0, 2, true>(a, a, st);
    if (a.Cin == 64) return nch == 1 ? launch_plane<3, 64, 1>(a, a, st) : launch_plane<3, 64, 2>(a, a, st);
    return nch == 1 ? launch_plane<3, 48, 1>(a, a, st) : launch_plane<3, 48, 2>(a, a, st);
}

// Two layers of one input in one launch: `a` as above with at most 32 output channels, `b` with the kernel two pixels
// smaller (3x3 beside 5x5, 1x1 beside 3x3), "same" padding, at most 32 output channels, no skip operands.
bool conv_plane_twin_ok(const ConvArgs &a, const ConvArgs &b)
{
    if (!plane_shape_ok(a) || plane_nch(a) != 1 || a.res_mode != 0 || b.res_mode != 0) return false;
    if (b.x != a.x || b.N != a.N || b.H != a.H || b.W != a.W || b.Cin != a.Cin || b.in_cs != a.in_cs || b.Ho != a.H || b.Wo != a.W) return false;
    if (b.KH != a.KH - 2 || b.KW != a.KW - 2 || b.sh != 1 || b.sw != 1 || b.ph != b.KH / 2 || b.pw != b.KW / 2) return false;
    if (b.in_xor || b.frag_xor || b.pc || b.Cout > 32 || b.ksteps != (b.KH * b.KW * b.Cin + 63) / 64) return false;
    return true;
}

hipError_t launch_conv_plane_twin(const ConvArgs &a, const ConvArgs &b, hipStream_t st)
{
    if (!conv_plane_twin_ok(a, b)) return hipErrorInvalidValue;
    if (a.KH == 5) return launch_plane<5, 64, 1, 1>(a, b, st);
    if (a.Cin == 48 && plane_pipe_ok(a) && plane_pipe_ok(b)) return launch_plane<3, 48, 1, 1, 2, true>(a, b, st);
    return a.Cin == 64 ? launch_plane<3, 64, 1, 1>(a, b, st) : launch_plane<3, 48, 1, 1>(a, b, st);
}

}  // namespace icnn
