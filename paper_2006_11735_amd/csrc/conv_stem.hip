// First layer of a classification network as ONE kernel: strided convolution of a raw picture (cin <= 4, kernel up
// to 8 pixels wide, stride 2), BReLU / requantisation (Sections 3.1, 3.2.1, 3.4.1), then the 3x3 / stride 2 /
// padding 1 max-pool that follows it.  Layer by layer the convolution writes its output (51 MB for a ResNet stem at
// batch 64), the pool reads it back, and the picture is first copied into a padded 4-channel tensor; here a
// workgroup computes the convolution outputs under a tile of pooled pixels, keeps them in LDS, and stores only the
// pooled tile.  Pooling windows overlap by one row and one column, so a tile of PH x PW pooled pixels needs
// (2 PH + 1) x (2 PW + 1) convolution outputs: the overlap is recomputed (14 % at 7 x 8, whose 15 x 17 outputs fill
// eight pixel groups of 32 but for one slot).
//
//   patch   the (4 PH + KH) x (4 PW + KW) input pixels under the tile, in LDS as one dword per pixel
//           (channels padded to 4, "- 128" applied, zeros outside the picture: the convolution's padding), pitch 40
//   conv    D[cout][conv pixel] with v_mfma_i32_32x32x32_i8, one K block of 32 per kernel row: eight pixels of
//           four channels (the packed weights of a small-cin layer have exactly this order, zeros in the padding)
//   pool    conv outputs as bytes in LDS, [pixel][cout]; positions outside the convolution's output are zeros (the
//           pool's padding never wins: activations are not negative); a thread pools 16 channels of one pixel
//
// 256 threads; the next tile's picture pixels travel (as byte loads into registers) while the current tile is
// multiplied; weights stay in LDS for all tiles of the (persistent) workgroup.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

constexpr int kStemPH = 7, kStemPW = 8;                      // pooled tile
constexpr int kStemCH = 2 * kStemPH + 1, kStemCW = 2 * kStemPW + 1;      // convolution outputs under it: 15 x 17
constexpr int kStemGroups = (kStemCH * kStemCW + 31) / 32;   // pixel groups of 32: 8, two per wave
constexpr int kStemPitch = 4 * kStemPW + 8;                  // patch pitch in pixels: 40
static_assert(kStemGroups == 8, "two pixel groups per wave");
constexpr int kStemMaxRows = 4 * kStemPH + 8;                // patch rows at kernel height 8
constexpr int kStemPerThread = (kStemMaxRows * kStemPitch + 255) / 256;

struct StemArgs {
    int Hp, Wp;                 // pooled size
    int tiles_x, tiles_per_img, n_tiles;
    int per_xcd;                // tiles handed to each of the 8 XCDs
    int patch_rows;             // 4 PH + KH
    int patch_cols;             // 4 PW + KW  (<= the pitch)
    int ksteps;                 // K steps of the packed weights: ceil(KH * 32 / 64)
    int cout_chunks;            // packed 32-channel chunks that hold channels: cout / 32
};

template <int N, class F>
__device__ __forceinline__ void stem_static_for(F &&fn)
{
    if constexpr (N > 0) {
        stem_static_for<N - 1>(fn);
        fn(std::integral_constant<int, N - 1>{});
    }
}

template <int CG>           // cout / 32: 1 or 2
__global__ __launch_bounds__(256, 3) void conv_stem_pool_kernel(const ConvArgs a, const StemArgs g)
{
    constexpr int TPX = kStemGroups / 4;             // pixel groups of a wave
    constexpr int ROW_BYTES = CG * 32;               // one convolution pixel's channels
    constexpr int ROW_PITCH = ROW_BYTES + 16;        // rows 20 or 12 banks apart: 16-byte accesses of 16 lanes spread over all banks
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // weights | patch 0 | patch 1 | convolution outputs
    const int w_bytes = CG * g.ksteps * kChunkBytes;
    uint8_t *const wbuf = lds;
    uint32_t *const patch = (uint32_t *)(lds + w_bytes);
    const int patch_words = kStemMaxRows * kStemPitch;
    uint8_t *const cbuf = lds + w_bytes + 2 * patch_words * 4;

    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, col = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pg0 = TPX * wave;                      // first pixel group of the wave

    // weights: a straight copy of the first CG chunks
    for (int i = tid; i < w_bytes / 16; i += 256) {
        const int chunk = i / (g.ksteps * 128), r = i - chunk * (g.ksteps * 128);
        *(v4i *)(wbuf + i * 16) = *(const v4i *)(a.wp + ((size_t)chunk * a.ksteps * kChunkBytes) + (size_t)r * 16);
    }
    // biases in LDS (read again for every tile: the registers are needed elsewhere)
    int32_t *const btab = (int32_t *)(cbuf + kStemGroups * 32 * ROW_PITCH);
    for (int i = tid; i < CG * 32; i += 256) btab[i] = a.bias[i];

    // Workgroups go to the eight XCDs round-robin and every XCD has an L2 of its own: the workgroups of XCD x walk the
    // contiguous tile range [x * per_xcd, (x + 1) * per_xcd), so that the picture rows neighbouring tiles share meet in
    // one L2.  Work slot v (blockIdx.x, + gridDim.x, ...; the grid is a multiple of 8) is tile (v & 7) * per_xcd + (v >> 3);
    // a workgroup's tiles ascend, so its walk ends at the first slot beyond its XCD's range or beyond the last tile.
    auto tile_of = [&](int v) { return (v & 7) * g.per_xcd + (v >> 3); };
    auto valid = [&](int v) { return (v >> 3) < g.per_xcd && tile_of(v) < g.n_tiles; };
    auto tile_origin = [&](int v, int &n, int &py0, int &px0) {
        const int t = tile_of(v);
        n = t / g.tiles_per_img;
        const int r = t - n * g.tiles_per_img;
        const int ty = r / g.tiles_x;
        py0 = ty * kStemPH;
        px0 = (r - ty * g.tiles_x) * kStemPW;
    };
    // picture pixels of a tile's patch: word e = t + 256 i is patch pixel (e / pitch, e % pitch); the patch's first pixel
    // is picture pixel (2 * (2 py0 - 1) - pad_h, 2 * (2 px0 - 1) - pad_w)
    // The channel bytes of a pixel are loaded one by one (a picture's pixels are 1 to 4 bytes apart) and stay in their
    // own registers until store_patch() combines them: the loads of the next tile travel during the multiplication.
    uint32_t word[kStemPerThread];         // a patch pixel's channels (and what follows them) as one word, fetched a tile ahead
    int shift_ok[kStemPerThread];          // bit 0: the pixel lies inside the picture; bits 1..: bytes the word was read early
    int rel[kStemPerThread];        // byte offset of the thread's patch pixels from the patch's first pixel (tile-invariant)
#pragma unroll
    for (int i = 0; i < kStemPerThread; ++i) {
        const int e = tid + 256 * i;
        const int r = e / kStemPitch, c = e - r * kStemPitch;
        rel[i] = (r * a.W + c) * a.in_cs;
    }
    typedef uint32_t u32_a1 __attribute__((aligned(1)));
    const uint32_t cmask = a.Cin >= 4 ? 0xffffffffu : (1u << (8 * a.Cin)) - 1u;      // the pixel's own channels
    auto fetch_patch = [&](int v) {
        int n, py0, px0;
        tile_origin(v, n, py0, px0);
        const int iy0 = 2 * (2 * py0 - 1) - a.ph, ix0 = 2 * (2 * px0 - 1) - a.pw;
        const uint8_t *base = a.x + ((ptrdiff_t)(n * a.H + iy0) * a.W + ix0) * a.in_cs;      // may lie before the tensor: only valid pixels are read
#pragma unroll
        for (int i = 0; i < kStemPerThread; ++i) {
            const int e = tid + 256 * i;
            const int r = e / kStemPitch, c = e - r * kStemPitch;
            const int iy = iy0 + r, ix = ix0 + c;
            const bool ok = n < a.N && r < g.patch_rows && c < g.patch_cols && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
            // One unaligned 4-byte load per pixel (its cin <= 4 bytes and whatever follows them), masked to the pixel's
            // channels afterwards.  The tensor's last pixels, where four bytes would run past the end, are read one to three
            // bytes early and shifted down.
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
        for (int i = 0; i < kStemPerThread; ++i) {
            const int e = tid + 256 * i;
            const uint32_t v = (word[i] >> (8 * (shift_ok[i] >> 1))) & cmask;
            // a pixel outside the picture: zero after the "- 128" too
            if (e < patch_words) patch[buf * patch_words + e] = (shift_ok[i] & 1) ? v ^ (a.in_xor & cmask) : 0u;
        }
    };

    // this lane's convolution pixels: slot q = 32 * (pg0 + j) + col is local output (cy, cx) = (q / CW, q % CW)
    int cy[TPX], cx[TPX];
#pragma unroll
    for (int j = 0; j < TPX; ++j) {
        const int q = 32 * (pg0 + j) + col;
        const bool in = q < kStemCH * kStemCW;
        cy[j] = in ? q / kStemCW : 0;
        cx[j] = in ? q - cy[j] * kStemCW : 0;
        if (!in) cy[j] = -1;
    }

    fetch_patch(blockIdx.x);
    store_patch(0);
    __syncthreads();
    int buf = 0;
    for (int v = blockIdx.x; valid(v); v += gridDim.x) {
        int n, py0, px0;
        tile_origin(v, n, py0, px0);
        const bool more = valid(v + (int)gridDim.x);
        if (more) fetch_patch(v + (int)gridDim.x);           // travels during the multiplication

        // ---- convolution: one K block per kernel row
        // the biases are the first kernel row's C operands (no copies into the accumulators)
        v16i acc[CG][TPX], bias[CG];
#pragma unroll
        for (int c = 0; c < CG; ++c) bias[c] = bias16(btab + c * 32 + half * 16);
        const uint32_t *P = patch + buf * patch_words;
        // fragments of kernel row kh: weights of every chunk, and per pixel group eight pixels from column 2 cx on
        // (this half of the wave the first or the second four)
        int w0[TPX];
#pragma unroll
        for (int j = 0; j < TPX; ++j) w0[j] = 2 * max(cy[j], 0) * kStemPitch + 2 * cx[j] + 4 * half;
        v4i af[CG], bf[TPX], afn[CG], bfn[TPX];
        auto fetch_frags = [&](v4i (&fa)[CG], v4i (&fb)[TPX], int kh) {
#pragma unroll
            for (int c = 0; c < CG; ++c) fa[c] = *(const v4i *)(wbuf + ((c * g.ksteps + (kh >> 1)) * 2 + (kh & 1)) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < TPX; ++j) {
                const uint32_t *q = P + w0[j] + kh * kStemPitch;
                const uint2 lo = *(const uint2 *)q, hi = *(const uint2 *)(q + 2);
                fb[j] = v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
            }
        };
        auto multiply = [&](const v4i (&fa)[CG], const v4i (&fb)[TPX]) {
#pragma unroll
            for (int c = 0; c < CG; ++c)
#pragma unroll
                for (int j = 0; j < TPX; ++j) acc[c][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[c], fb[j], acc[c][j], 0, 0, 0);
        };
        // two kernel rows per round: each row's fragments arrive during the previous row's MFMAs, in alternating registers
        fetch_frags(af, bf, 0);
        if (1 < a.KH) fetch_frags(afn, bfn, 1);
#pragma unroll
        for (int c = 0; c < CG; ++c)
#pragma unroll
            for (int j = 0; j < TPX; ++j) acc[c][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[c], bf[j], bias[c], 0, 0, 0);
        if (2 < a.KH) fetch_frags(af, bf, 2);
        if (1 < a.KH) multiply(afn, bfn);
        for (int kh = 2; kh < a.KH; kh += 2) {
            if (kh + 1 < a.KH) fetch_frags(afn, bfn, kh + 1);
            multiply(af, bf);
            if (kh + 2 < a.KH) fetch_frags(af, bf, kh + 2);
            if (kh + 1 < a.KH) multiply(afn, bfn);
        }
        mfma_drain(acc);
        // ---- requantise; outputs outside the convolution's output range are the pool's padding: zeros
        stem_static_for<TPX>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if (cy[j] < 0) return;
            const int oy = 2 * py0 - 1 + cy[j], ox = 2 * px0 - 1 + cx[j];
            const bool ok = (unsigned)oy < (unsigned)a.Ho && (unsigned)ox < (unsigned)a.Wo;
            const int q = 32 * (pg0 + j) + col;
            stem_static_for<CG>([&](auto cc) {
                constexpr int c = decltype(cc)::value;
                int t[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = acc[c][j][r];
                v4i w = requant16_any(a, t);
                if (!ok) w = v4i{0, 0, 0, 0};
                *(v4i *)(cbuf + q * ROW_PITCH + c * 32 + half * 16) = w;
            });
        });
        if (more) store_patch(buf ^ 1);
        __syncthreads();
        // ---- pool: a thread takes 16 channels of one pooled pixel
        constexpr int GPP = ROW_BYTES / 16;              // 16-channel groups per pixel
        for (int item = tid; item < kStemPH * kStemPW * GPP; item += 256) {
            const int pp = item / GPP, cgp = item - pp * GPP;
            const int ty = pp / kStemPW, tx = pp - ty * kStemPW;
            const int py = py0 + ty, px = px0 + tx;
            if (py >= g.Hp || px >= g.Wp) continue;
            // bytewise maximum in two halves, as 16-bit lanes: the even bytes masked out of every loaded word; the odd
            // bytes need no mask, because a lane's maximum is decided by its high byte (the low byte only breaks ties)
            // and only the high byte of the result is kept
            typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
            u16x2 me[4] = {}, mo[4] = {};
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int jx = 0; jx < 3; ++jx) {
                    const int q = (2 * ty + i) * kStemCW + 2 * tx + jx;
                    const v4i w = *(const v4i *)(cbuf + q * ROW_PITCH + cgp * 16);
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t x = (uint32_t)w[d];
                        me[d] = __builtin_elementwise_max(me[d], __builtin_bit_cast(u16x2, x & 0x00ff00ffu));
                        mo[d] = __builtin_elementwise_max(mo[d], __builtin_bit_cast(u16x2, x));
                    }
                }
            v4i o;
#pragma unroll
            for (int d = 0; d < 4; ++d) o[d] = (int)(__builtin_bit_cast(uint32_t, me[d]) | (__builtin_bit_cast(uint32_t, mo[d]) & 0xff00ff00u));
            *(v4i *)((uint8_t *)a.out + ((size_t)(n * g.Hp + py) * g.Wp + px) * a.out_cs + a.out_co + cgp * 16) = o;
        }
        __syncthreads();
        buf ^= 1;
    }
}

// conv: a small-cin layer's arguments on the ORIGINAL picture (H, W, Cin, in_cs, KH, KW, pads, Ho, Wo as given;
// the packed weights in the small-cin order), out / out_cs / out_co describing the POOLED tensor.
hipError_t launch_conv_stem_pool(const ConvArgs &a, int hp, int wp, hipStream_t st)
{
    StemArgs g;
    g.Hp = hp;
    g.Wp = wp;
    g.tiles_x = (wp + kStemPW - 1) / kStemPW;
    g.tiles_per_img = g.tiles_x * ((hp + kStemPH - 1) / kStemPH);
    const long long tiles = (long long)g.tiles_per_img * a.N;
    if (tiles < 1 || tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    g.n_tiles = (int)tiles;
    g.per_xcd = (g.n_tiles + 7) / 8;
    g.patch_rows = 4 * kStemPH + a.KH;
    g.patch_cols = 4 * kStemPW + a.KW;
    g.ksteps = a.ksteps;
    g.cout_chunks = a.Cout / 32;
    if (a.x_bytes < 4 || a.KH > 8 || a.KW > 8 || g.patch_cols > kStemPitch || g.patch_rows > kStemMaxRows || (a.Cout != 32 && a.Cout != 64) ||
        a.ksteps != (a.KH * 32 + 63) / 64)
        return hipErrorInvalidValue;
    const size_t lds_bytes = (size_t)g.cout_chunks * g.ksteps * kChunkBytes + 2 * (size_t)kStemMaxRows * kStemPitch * 4 +
                             (size_t)kStemGroups * 32 * (a.Cout + 16) + (size_t)a.Cout * 4;
    const int slots = 256 * 3;
    const dim3 grid((unsigned)(8 * g.per_xcd < slots ? 8 * g.per_xcd : slots)), block(256);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a, g);
        return hipGetLastError();
    };
    return a.Cout == 64 ? go(conv_stem_pool_kernel<2>) : go(conv_stem_pool_kernel<1>);
}

}  // namespace icnn
