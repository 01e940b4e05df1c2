// First layer of a picture-to-picture network at stride 1 (cin <= 4, kernel at most 8 pixels wide and high,
// 32 or 64 output channels; Sections 3.1, 3.2.1, 3.4.1): the convolution straight off the raw picture, BReLU /
// requantisation, 8-bit store.  The general path first copies the picture into a padded 4-channel tensor and then
// runs the tile kernel over it with every kernel row padded to a K block of 32; here the picture pixels under a tile
// go to LDS directly (one dword per pixel: channels padded to 4, "- 128" applied, zeros outside the picture = the
// convolution's padding), so the only traffic that counts is the output: 64 bytes per pixel for 1 to 4 bytes read.
//
//   tile    8 rows x 32 columns of output pixels = 8 pixel groups of 32; wave w owns rows 2w and 2w + 1
//   patch   (8 + KH - 1) x (32 + 7) picture pixels, pitch 40 words, double-buffered: the next tile's pixels travel
//           (as loads into registers) while this tile is multiplied
//   conv    D[cout][pixel] with v_mfma_i32_32x32x32_i8, one K block of 32 per kernel row: eight pixels of four
//           channels from column x on (the packed weights of a small-cin layer have exactly this order, zeros in
//           the padding); kernels at most four pixels wide pack two rows of four pixels into a K block; the
//           biases are the C operand of the first block's instructions
//   store   a lane holds 16 consecutive channels of one pixel: one 16-byte store per accumulator tile
//
// 256 threads, persistent workgroups (four per CU), weights resident in LDS.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

constexpr int kPicTH = 8, kPicTW = 32;
constexpr int kPicPitch = kPicTW + 8;                        // patch pitch in pixels
constexpr int kPicMaxRows = kPicTH + 7;                      // patch rows at kernel height 8
constexpr int kPicWords = kPicMaxRows * kPicPitch;
constexpr int kPicPerThread = (kPicWords + 255) / 256;

struct PicArgs {
    int tiles_x, tiles_per_img, n_tiles;
    int per_xcd;                // tiles handed to each of the 8 XCDs
    int patch_rows;             // 8 + KH - 1
    int patch_cols;             // 32 + KW - 1 (<= the pitch)
    FastDiv div_tpi, div_tx;
};

template <int N, class F>
__device__ __forceinline__ void pic_static_for(F &&fn)
{
    if constexpr (N > 0) {
        pic_static_for<N - 1>(fn);
        fn(std::integral_constant<int, N - 1>{});
    }
}

// CG: cout / 32 (1 or 2).  ROW16: kernels at most four pixels wide, whose packed rows are 16 bytes: a K block of 32 is
// two kernel rows of four pixels (this half of the wave the first or the second row) instead of one row of eight.
template <int CG, bool ROW16>
__global__ __launch_bounds__(256, 4) void conv_pic_kernel(const ConvArgs a, const PicArgs g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // weights | patch 0 | patch 1 | biases
    const int w_bytes = CG * a.ksteps * kChunkBytes;
    uint8_t *const wbuf = lds;
    uint32_t *const patch = (uint32_t *)(lds + w_bytes);
    int32_t *const btab = (int32_t *)(lds + w_bytes + 2 * kPicWords * 4);

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, col = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // weights (a straight copy of the first CG chunks: at most 2 chunks x 4 K steps x 2 KiB = 4 pieces per thread) and
    // biases: these loads and the first patch's are all issued before anything is stored, so the prologue costs one
    // memory latency, not five
    constexpr int WPT = 4;
    v4i wv[WPT];
#pragma unroll
    for (int q = 0; q < WPT; ++q) {
        const int i = tid + 256 * q;
        wv[q] = i < w_bytes / 16 ? *(const v4i *)(a.wp + (size_t)i * 16) : v4i{0, 0, 0, 0};
    }
    const int bv = tid < CG * 32 ? a.bias[tid] : 0;

    // Work slot v (blockIdx.x, + gridDim.x, ...; the grid is a multiple of 8) is tile (v & 7) * per_xcd + (v >> 3): the
    // workgroups of one XCD (they are dealt round-robin) walk a contiguous range of tiles, so that the picture rows that
    // neighbouring tiles share meet in one L2.
    auto tile_of = [&](int v) { return (v & 7) * g.per_xcd + (v >> 3); };
    auto valid = [&](int v) { return (v >> 3) < g.per_xcd && tile_of(v) < g.n_tiles; };
    auto tile_origin = [&](int v, int &n, int &oy0, int &ox0) {
        const int t = tile_of(v);
        n = fast_div(t, g.div_tpi);
        const int r = t - n * g.tiles_per_img;
        const int ty = fast_div(r, g.div_tx);
        oy0 = ty * kPicTH;
        ox0 = (r - ty * g.tiles_x) * kPicTW;
    };
    // patch word e = tid + 256 i is patch pixel (e / pitch, e % pitch) = picture pixel (oy0 - pad_h + row, ox0 - pad_w + col)
    uint32_t word[kPicPerThread];          // a patch pixel's channels (and what follows them) as one word, fetched a tile ahead
    int shift_ok[kPicPerThread];           // bit 0: the pixel lies inside the picture; bits 1..: bytes the word was read early
    int rel[kPicPerThread], prow[kPicPerThread], pcol[kPicPerThread];
#pragma unroll
    for (int i = 0; i < kPicPerThread; ++i) {
        const int e = tid + 256 * i;
        prow[i] = e / kPicPitch;
        pcol[i] = e - prow[i] * kPicPitch;
        rel[i] = (prow[i] * a.W + pcol[i]) * a.in_cs;
    }
    typedef uint32_t u32_a1 __attribute__((aligned(1)));
    const uint32_t cmask = a.Cin >= 4 ? 0xffffffffu : (1u << (8 * a.Cin)) - 1u;      // the pixel's own channels
    auto fetch_patch = [&](int v) {
        int n, oy0, ox0;
        tile_origin(v, n, oy0, ox0);
        const int iy0 = oy0 - a.ph, ix0 = ox0 - a.pw;
        const uint8_t *base = a.x + ((ptrdiff_t)(n * a.H + iy0) * a.W + ix0) * a.in_cs;      // may lie before the tensor: only valid pixels are read
#pragma unroll
        for (int i = 0; i < kPicPerThread; ++i) {
            const int iy = iy0 + prow[i], ix = ix0 + pcol[i];
            const bool ok = prow[i] < g.patch_rows && pcol[i] < g.patch_cols && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
            // One unaligned 4-byte load per pixel (its cin <= 4 bytes and whatever follows them), masked to the pixel's
            // channels afterwards.  The tensor's last pixels, where four bytes would run past the end, are read one to
            // three bytes early and shifted down.
            const uint8_t *p = ok ? base + rel[i] : a.x;
            const long long room = (long long)a.x_bytes - (p - a.x);               // bytes from p to the end of the tensor
            const int back = ok && room < 4 ? (int)(4 - room) : 0;
            word[i] = *(const u32_a1 *)(p - back);
            shift_ok[i] = (ok ? 1 : 0) | (back << 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto store_patch = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kPicPerThread; ++i) {
            const int e = tid + 256 * i;
            const uint32_t v = (word[i] >> (8 * (shift_ok[i] >> 1))) & cmask;
            // a pixel outside the picture: zero after the "- 128" too
            if (e < kPicWords) patch[buf * kPicWords + e] = (shift_ok[i] & 1) ? v ^ (a.in_xor & cmask) : 0u;
        }
    };

    const bool first = valid(blockIdx.x);    // (a workgroup whose first slot is a padding slot has no tile at all)
    if (first) fetch_patch(blockIdx.x);
#pragma unroll
    for (int q = 0; q < WPT; ++q)
        if (tid + 256 * q < w_bytes / 16) *(v4i *)(wbuf + (tid + 256 * q) * 16) = wv[q];
    if (tid < CG * 32) btab[tid] = bv;
    if (first) store_patch(0);
    __syncthreads();
    int buf = 0;
    for (int v = blockIdx.x; valid(v); v += gridDim.x) {
        int n, oy0, ox0;
        tile_origin(v, n, oy0, ox0);
        const bool more = valid(v + (int)gridDim.x);
        if (more) fetch_patch(v + (int)gridDim.x);           // travels during the multiplication

        v16i acc[CG][2], bias[CG];
#pragma unroll
        for (int c = 0; c < CG; ++c) bias[c] = bias16(btab + c * 32 + half * 16);
        // fragments of K block kh (one kernel row, or two with ROW16): weights of every chunk, and per pixel group the eight pixels from column x on
        // (this half of the wave the first or the second four) of patch row y + kh
        const uint32_t *P = patch + buf * kPicWords + (2 * wave + (ROW16 ? half : 0)) * kPicPitch + col + (ROW16 ? 0 : 4 * half);
        const int nblk = ROW16 ? (a.KH + 1) >> 1 : a.KH;          // K blocks of 32
        v4i af[CG], bf[2], afn[CG], bfn[2];
        auto fetch_frags = [&](v4i (&fa)[CG], v4i (&fb)[2], int kh) {
#pragma unroll
            for (int c = 0; c < CG; ++c) fa[c] = *(const v4i *)(wbuf + ((c * a.ksteps + (kh >> 1)) * 2 + (kh & 1)) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint32_t *q = P + (j + (ROW16 ? 2 * kh : kh)) * kPicPitch;
                fb[j] = v4i{(int)q[0], (int)q[1], (int)q[2], (int)q[3]};      // dword-aligned only: the column is any
            }
        };
        auto multiply = [&](const v4i (&fa)[CG], const v4i (&fb)[2]) {
#pragma unroll
            for (int c = 0; c < CG; ++c)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[c][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[c], fb[j], acc[c][j], 0, 0, 0);
        };
        // two kernel rows per round: each row's fragments arrive during the previous row's MFMAs, in alternating registers
        fetch_frags(af, bf, 0);
        if (1 < nblk) fetch_frags(afn, bfn, 1);
#pragma unroll
        for (int c = 0; c < CG; ++c)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[c][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[c], bf[j], bias[c], 0, 0, 0);
        if (2 < nblk) fetch_frags(af, bf, 2);
        if (1 < nblk) multiply(afn, bfn);
        for (int kh = 2; kh < nblk; kh += 2) {
            if (kh + 1 < nblk) fetch_frags(afn, bfn, kh + 1);
            multiply(af, bf);
            if (kh + 2 < nblk) fetch_frags(af, bf, kh + 2);
            if (kh + 1 < nblk) multiply(afn, bfn);
        }
        mfma_drain(acc);
        const int ox = ox0 + col;
        pic_static_for<2>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int oy = oy0 + 2 * wave + j;
            if (oy >= a.Ho || ox >= a.Wo) return;
            uint8_t *o = (uint8_t *)a.out + ((size_t)(n * a.Ho + oy) * a.Wo + ox) * a.out_cs + a.out_co + half * 16;
            pic_static_for<CG>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                int t[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = acc[c][j][r];
                *(v4i *)(o + c * 32) = requant16_any(a, t);
            });
        });
        if (more) store_patch(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
}

// a: a small-cin layer's arguments on the ORIGINAL picture (H, W, Cin, in_cs, KH, KW, pads, Ho, Wo as given; the
// packed weights in the small-cin order).  The caller has checked: stride 1, cin <= 4, kernel at most 8 wide and high, 32 or 64 output channels, unsigned 8-bit output with 16-byte aligned pixels, no skip
// operand, per-layer requantisation, input re-normalised by XOR or not at all.
hipError_t launch_conv_pic(const ConvArgs &a, hipStream_t st)
{
    PicArgs g;
    g.tiles_x = (a.Wo + kPicTW - 1) / kPicTW;
    g.tiles_per_img = g.tiles_x * ((a.Ho + kPicTH - 1) / kPicTH);
    const long long tiles = (long long)g.tiles_per_img * a.N;
    if (tiles < 1 || tiles > 0x7fffffffLL / 8) return hipErrorInvalidValue;
    g.n_tiles = (int)tiles;
    g.per_xcd = (g.n_tiles + 7) / 8;
    g.patch_rows = kPicTH + a.KH - 1;
    g.patch_cols = kPicTW + a.KW - 1;
    g.div_tpi = make_fast_div((unsigned)g.tiles_per_img);
    g.div_tx = make_fast_div((unsigned)g.tiles_x);
    const bool row16 = a.KW <= 4;
    if (a.x_bytes < 4 || a.KH > 8 || a.KW > 8 || (a.Cout != 32 && a.Cout != 64) || a.ksteps != (a.KH * (row16 ? 16 : 32) + 63) / 64)
        return hipErrorInvalidValue;
    const size_t lds_bytes = (size_t)(a.Cout / 32) * a.ksteps * kChunkBytes + 2 * (size_t)kPicWords * 4 + (size_t)a.Cout * 4;
    const int slots = 256 * 4;
    const dim3 grid((unsigned)(8 * g.per_xcd < slots ? 8 * g.per_xcd : slots)), block(256);
    if (a.Cout == 64) {
        if (row16) hipLaunchKernelGGL((conv_pic_kernel<2, true>), grid, block, lds_bytes, st, a, g);
        else hipLaunchKernelGGL((conv_pic_kernel<2, false>), grid, block, lds_bytes, st, a, g);
    } else {
        if (row16) hipLaunchKernelGGL((conv_pic_kernel<1, true>), grid, block, lds_bytes, st, a, g);
        else hipLaunchKernelGGL((conv_pic_kernel<1, false>), grid, block, lds_bytes, st, a, g);
    }
    return hipGetLastError();
}

}  // namespace icnn
