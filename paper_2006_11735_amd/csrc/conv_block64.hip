// The identity bottleneck block of a network's first stage (1x1 conv to 64 channels, 3x3 conv, 1x1 conv back to C
// channels with the block input as skip operand, Section 4.1) as one kernel whose WEIGHTS LIVE IN REGISTERS.
//
// With 64 middle channels and C <= 256 the three layers' packed weights are 68 KB at most, and what one wave
// multiplies of them -- one 32-channel chunk per layer -- is 28 fragments = 112 registers.  Every wave loads its
// fragments once, when the workgroup starts, and keeps them across all the tiles the workgroup walks: no weight
// traffic per tile at all, no LDS ring, no copy waves and no barrier per K step.  All eight waves multiply.
//
//   tile     TH x TW output pixels (at most 128), patch (TH+2) x (TW+2) input pixels (at most 160), as in
//            conv_block_kernel; two patch buffers, the next tile's patch is copied global -> LDS while this tile runs
//   phase 1  a = BReLU/requant(W1 x + b1) on the patch: ten (chunk, pixel group) items over eight waves; patch
//            pixels outside the image become zeros (the 3x3 layer's padding)
//   phase 2  b = BReLU/requant(W2 (*) a + b2) on the tile: one (chunk, pixel group) item per wave, tap = patch row offset
//   phase 3  y = epilogue(W3 b + b3, skip): a wave owns one of the C/32 output chunks; the skip operand is the block
//            input, read from the patch in LDS (it is still there: nothing overwrites a tile's patch before the
//            tile is finished), so the input crosses the memory system once
// PROJ: the block that opens a stage instead (Section 4.1, skip connection "after convolution"): its skip operand is a
// projection convolution of the block input, W_p x + b_p, rescaled to the main path's ratio and added before the last
// layer's products, exactly as the two-GEMM kernel of the projection blocks does; here its two MFMAs per pixel group
// read the pixel's own patch row, and the last layer's chunk count no longer follows from the input width.
// Four workgroup barriers per tile.  Same MFMA instruction, accumulator layout, packed weights and epilogue
// arithmetic as the other convolution kernels: the result is that of the three separate layers, bit for bit.
#include "conv_common.h"

namespace icnn {

// Development aid, compiled in with -DICNN_B64_TRACE only: wave `ICNN_B64_TRACE` of one workgroup stamps the clock at
// the marked points; icnn_debug_trace_b64() copies the stamps out.
#ifdef ICNN_B64_TRACE
__device__ unsigned long long g_b64_trace[512];
#define B64_TR(k)                                                                                                  \
    do {                                                                                                           \
        if (blockIdx.x == 3 && wave == (ICNN_B64_TRACE) && lane == 0 && trn < 500)                                 \
            g_b64_trace[trn++] = ((unsigned long long)(k) << 56) | (__builtin_amdgcn_s_memtime() & 0xffffffffffffffULL); \
    } while (0)
#else
#define B64_TR(k)
#endif

constexpr int kB64Rows = 160;        // patch rows: five pixel groups of 32 (output pixel slots of a tile: 128, four groups)

template <int K1, int NCH3, bool PROJ>       // input channels / 64 (1, 2 or 4); output channels / 32 (2, 4 or 8); projection skip
__global__ __launch_bounds__(512, 2) void conv_block64_kernel(const BlockArgs g, const ConvArgs a1, const ConvArgs a2, const ConvArgs a3,
                                                              const ProjArgs pj)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int SLICE = kB64Rows * 64;             // one 64-channel slice of a patch
    constexpr int PATCH = K1 * SLICE;
    constexpr int CO = NCH3 * 32;                    // output channels of the last layer
    constexpr int NP3 = NCH3 / 2;                    // pixel groups of a wave in phase 3 (8 waves, 4 * NCH3 items)
    constexpr int NCOPY = 10 * K1;                   // 1 KiB copies of a patch (16 rows of a slice each)
    constexpr int CPW = (NCOPY + 7) / 8;             // copies per wave
    constexpr unsigned OOB = 0x80000000u;

    // LDS: two patches of x | a on the patch (later b on the tile) | biases [64] layer 1, [64] layer 2, [CO] layer 3, [CO] projection
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    uint8_t *const abuf = lds + 2 * PATCH;
    uint8_t *const bbuf = abuf;                      // b overwrites a once every wave has left phase 2
    int32_t *const btab = (int32_t *)(abuf + SLICE);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    const int n_tiles = g.n_tiles;

    // work slot v (blockIdx.x, + gridDim.x, ...) is tile (v & 7) * per_xcd + (v >> 3): the workgroups of an XCD walk a
    // contiguous range of tiles (neighbouring patches share rows: they meet in one L2)
    auto tile_of = [&](int v) { return (v & 7) * g.per_xcd + (v >> 3); };
    auto valid = [&](int v) { return (v >> 3) < g.per_xcd && tile_of(v) < n_tiles; };
    auto tile_origin = [&](int v, int &n, int &y0, int &x0) {
        const int t = tile_of(v);
        n = t / g.tiles_per_img;
        const int r = t - n * g.tiles_per_img;
        const int ty = r / g.tiles_x;
        y0 = ty * g.TH;
        x0 = (r - ty * g.tiles_x) * g.TW;
    };
    // Every barrier first waits for this wave's outstanding LDS accesses (lgkmcnt 0).  For stores that is what makes
    // them visible; for loads it is what makes "all waves are done reading" true: a fragment read that is still queued
    // when the barrier releases the other waves can be overtaken by their stores to the same bytes (the compiler is free
    // to move the MFMA that consumes the fragment, and with it the wait, behind the barrier).
    auto sync = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto sync_lds_written = sync;

    // ---- the patch of tile slot v into buffer b: copy e = wave + 8 i fills rows 16 (e % 10) .. + 16 of slice e / 10;
    // this lane the 16-byte piece lane & 3 of row 16 (e % 10) + (lane >> 2), i.e. logical piece (lane & 3) ^ ((row >> 2) & 3)
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)g.x, 0, g.x_bytes, 0x00020000);
    auto issue_patch = [&](int v, int b) {
        int n, y0, x0;
        tile_origin(v, n, y0, x0);
#pragma unroll
        for (int i = 0; i < CPW; ++i) {
            const int e = wave + 8 * i;
            if (e < NCOPY) {                         // wave-uniform
                const int k = e / 10, rb = e - k * 10;
                const int row = 16 * rb + (lane >> 2);
                const int logical = (lane & 3) ^ ((row >> 2) & 3);
                const int py = (int)(((unsigned)row * g.inv_pw) >> 16);
                const int px = row - py * g.PW;
                const int iy = y0 - 1 + py, ix = x0 - 1 + px;
                const bool ok = py < g.TH + 2 && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
                const unsigned off = ok ? (unsigned)(((n * g.H + iy) * g.W + ix) * g.x_cs) + k * 64 + logical * 16 : OOB;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)(lds + b * PATCH + k * SLICE + rb * 1024),
                                                         16, off, 0, 0, 0);
            }
        }
    };

    // ---- this wave's share of the three layers, for the whole life of the workgroup
    const int c12 = wave & 1;                        // 32-channel chunk of layers 1 and 2
    const int pg12 = wave >> 1;                      // pixel group in phases 1 and 2 (waves 0 and 1 also take group 4 in phase 1)
    const int ch3 = wave % NCH3;                     // chunk of layer 3
    const int pg3_0 = (wave / NCH3) * NP3;           // its first pixel group there
    v4i w1[2 * K1], w2[18], w3[2];
    [[maybe_unused]] v4i wq[2 * K1];                 // the projection's chunk ch3
    {
        const v4i *p1 = (const v4i *)(a1.wp + (size_t)c12 * K1 * kChunkBytes) + lane;
        const v4i *p2 = (const v4i *)(a2.wp + (size_t)c12 * 9 * kChunkBytes) + lane;
        const v4i *p3 = (const v4i *)(a3.wp + (size_t)ch3 * kChunkBytes) + lane;
#pragma unroll
        for (int f = 0; f < 2 * K1; ++f) w1[f] = p1[f * 64];
#pragma unroll
        for (int f = 0; f < 18; ++f) w2[f] = p2[f * 64];
#pragma unroll
        for (int f = 0; f < 2; ++f) w3[f] = p3[f * 64];
        if constexpr (PROJ) {
            const v4i *pq = (const v4i *)(pj.wp + (size_t)ch3 * K1 * kChunkBytes) + lane;
#pragma unroll
            for (int f = 0; f < 2 * K1; ++f) wq[f] = pq[f * 64];
        }
    }
    for (int i = tid; i < 128 + (PROJ ? 2 : 1) * CO; i += 512)
        btab[i] = i < 64 ? a1.bias[i] : (i < 128 ? a2.bias[i - 64] : (i < 128 + CO ? a3.bias[i - 128] : pj.bias[i - 128 - CO]));

    // tile-invariant positions of phase 2: output slot q = 32 pg12 + col is tile pixel (q / TW, q % TW), whose centre
    // tap is patch row (ty + 1) * PW + tx + 1; slots beyond the tile compute on row PW + 1 and are never stored
    int rel2;
    {
        const int q = 32 * pg12 + col;
        const bool in_tile = q < g.TH * g.TW;
        const int ty = in_tile ? (int)(((unsigned)q * g.inv_tw) >> 16) : 0;
        const int tx = in_tile ? q - ty * g.TW : 0;
        rel2 = (ty + 1) * g.PW + tx + 1;
    }
    const bool has_res = a3.res_mode != 0;

    if (valid(blockIdx.x)) issue_patch(blockIdx.x, 0);
    asm volatile("" ::: "memory");
    ICNN_WAIT_VMCNT(0);                              // the first patch (and this wave's weights) have arrived
    sync_lds_written();                              // ... everybody's, and the bias table is written

    int buf = 0;
    [[maybe_unused]] int trn = 0;
    for (int v = blockIdx.x; valid(v); v += gridDim.x) {
        B64_TR(1);
        int n, y0, x0;
        tile_origin(v, n, y0, x0);
        const uint8_t *const xb = lds + buf * PATCH;
        // the next tile's patch travels during this tile (its buffer was last read in the previous tile's phase 3,
        // which every wave left before the barrier at the end of that tile)
        if (valid(v + (int)gridDim.x)) issue_patch(v + (int)gridDim.x, buf ^ 1);
        B64_TR(2);

        // ---------------- phase 1: a = requant(W1 x + b1) on patch rows 32 pg .. + 32, chunk c12
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
            const int pg = pg12 + 4 * rep;
            if (pg < 5) {                            // wave-uniform: the fifth group goes to waves 0 and 1
                const int row = 32 * pg + col;
                v16i acc = bias16(btab + c12 * 32 + half * 16);
#pragma unroll
                for (int f = 0; f < 2 * K1; ++f)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1[f], *(const v4i *)(xb + (f >> 1) * SLICE + b_slot_offset(row, (f & 1) * 2 + half)),
                                                                acc, 0, 0, 0);
                mfma_drain(acc);
                B64_TR(3);
                const int py = (int)(((unsigned)row * g.inv_pw) >> 16);
                const int px = row - py * g.PW;
                const int iy = y0 - 1 + py, ix = x0 - 1 + px;
                const bool ok = py < g.TH + 2 && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
                int t[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = acc[r];
                v4i w = requant16_any(a1, t);
                if (!ok) w = v4i{0, 0, 0, 0};        // outside the image: the next layer's zero padding
                *(v4i *)(abuf + b_slot_offset(row, c12 * 2 + half)) = w;
                B64_TR(4);
            }
        }
        sync_lds_written();
        B64_TR(5);

        // ---------------- phase 2: b = requant(W2 (*) a + b2) on output slots 32 pg12 .. + 32, chunk c12
        {
            v16i acc = bias16(btab + 64 + c12 * 32 + half * 16);
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int row = rel2 + (t / 3 - 1) * g.PW + (t % 3 - 1);
#pragma unroll
                for (int kq = 0; kq < 2; ++kq)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w2[2 * t + kq], *(const v4i *)(abuf + b_slot_offset(row, kq * 2 + half)), acc, 0, 0, 0);
            }
            B64_TR(6);
            sync();                                  // every wave has its last fragments of a: b may overwrite it
            mfma_drain(acc);
            B64_TR(7);
            int t[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) t[r] = acc[r];
            const v4i w = requant16_any(a2, t);      // slots beyond the tile hold values nobody stores
            *(v4i *)(bbuf + b_slot_offset(32 * pg12 + col, c12 * 2 + half)) = w;
            B64_TR(8);
        }
        sync_lds_written();
        B64_TR(9);

        // ---------------- phase 3: y = epilogue(W3 b + b3, skip) on chunk ch3, pixel groups pg3_0 .. + NP3
        static_for<NP3>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int q = 32 * (pg3_0 + j) + col;
            const bool in_tile = q < g.TH * g.TW;
            const int ty = in_tile ? (int)(((unsigned)q * g.inv_tw) >> 16) : 0;
            const int tx = in_tile ? q - ty * g.TW : 0;
            const int oy = y0 + ty, ox = x0 + tx;
            const bool ok = in_tile && oy < g.H && ox < g.W;
            const int prow = (ty + 1) * g.PW + tx + 1;           // the pixel's own patch row
            const int co = ch3 * 32 + half * 16;
            v16i acc;
            if constexpr (PROJ) {
                // the projection's sum on the pixel's own patch row, brought to the main path's ratio; the last layer's bias
                // and products come on top (the host has proved that the sum stays inside int32)
                acc = bias16(btab + 128 + CO + co);
#pragma unroll
                for (int f = 0; f < 2 * K1; ++f)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wq[f], *(const v4i *)(xb + (f >> 1) * SLICE + b_slot_offset(prow, (f & 1) * 2 + half)),
                                                                acc, 0, 0, 0);
                mfma_drain(acc);
                const v16i b3 = bias16(btab + 128 + co);
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = (int)rsr64((int64_t)acc[r] * pj.res_mul, pj.res_shift) + b3[r];
            } else {
                acc = bias16(btab + 128 + co);
            }
#pragma unroll
            for (int kq = 0; kq < 2; ++kq)
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w3[kq], *(const v4i *)(bbuf + b_slot_offset(q, kq * 2 + half)), acc, 0, 0, 0);
            mfma_drain(acc);
            v4i w;
            if constexpr (PROJ) {
                w = epilogue_bytes16<0>(a3, acc, v4i{0, 0, 0, 0});
            } else {
                // the skip operand: channels co .. co + 16 of the pixel's own patch row
                const v4i r8 = *(const v4i *)(xb + (co >> 6) * SLICE + b_slot_offset(prow, (co & 63) >> 4));
                w = has_res ? epilogue_bytes16<1>(a3, acc, r8) : epilogue_bytes16<0>(a3, acc, r8);
            }
            if (ok) *(v4i *)((uint8_t *)a3.out + (size_t)((n * g.H + oy) * g.W + ox) * a3.out_cs + a3.out_co + co) = w;
            B64_TR(10);
        });
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT(0);                          // the next tile's patch has landed (this wave's copies of it)
        B64_TR(11);
        sync();                                      // ... all of it; and nobody reads b or this tile's patch any more
        buf ^= 1;
    }
#endif
}

// ------------------------------------------------------------------ dispatch
size_t conv_block64_lds_bytes(int c_in, int c_out, bool proj)
{
    return (size_t)(2 * (c_in / 64) + 1) * kB64Rows * 64 + (size_t)(128 + (proj ? 2 : 1) * c_out) * 4;
}

// true when the register-resident kernel takes the block: 64 middle channels, 64, 128 or 256 outer channels, an
// 8-bit output, and a skip operand that is the block input itself (unsigned 8-bit, joined before requantisation
// with a rescale that fits 32 bits) or none
bool conv_block64_takes(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a3)
{
    const int c = a1.Cin;
    if (a1.Cout != 64 || a3.Cout != c || (c != 64 && c != 128 && c != 256)) return false;
    if (a3.out_mode == 3 || a3.epi_mode / 4 == 2 || !a3.epi_vec) return false;
    if (a3.res_mode != 0 && ((const uint8_t *)a3.res != g.x || a3.res_cs != g.x_cs)) return false;
    return true;
}

// The block with a projection skip: 64 input and middle channels, 256 output channels (the block that opens the first
// stage of the bottleneck ResNets); a3 carries no skip operand, pj the projection of the block input
bool conv_block64_proj_takes(const ConvArgs &a1, const ConvArgs &a3, const ProjArgs &pj)
{
    return a1.Cin == 64 && a1.Cout == 64 && a3.Cout == 256 && a3.out_mode != 3 && a3.res_mode == 0 && a3.epi_vec && pj.Cin == 64 &&
           pj.ksteps == 1 && pj.sh == 1 && pj.sw == 1 && pj.vec_bias;
}

hipError_t launch_conv_block64(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a2, const ConvArgs &a3, const ProjArgs *pj,
                               hipStream_t st)
{
    const int c = a1.Cin;
    const size_t lds_bytes = conv_block64_lds_bytes(c, a3.Cout, pj != nullptr);
    if (!(pj ? conv_block64_proj_takes(a1, a3, *pj) : conv_block64_takes(g, a1, a3)) || lds_bytes > 160 * 1024 || g.n_tiles < 1)
        return hipErrorInvalidValue;
    BlockArgs gx = g;
    gx.per_xcd = (g.n_tiles + 7) / 8;
    const dim3 grid((unsigned)(8 * gx.per_xcd < 256 ? 8 * gx.per_xcd : 256)), block(512);
    const ProjArgs none = {};
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, gx, a1, a2, a3, pj ? *pj : none);
        return hipGetLastError();
    };
    if (pj) return go(conv_block64_kernel<1, 8, true>);
    return c == 64 ? go(conv_block64_kernel<1, 2, false>) : c == 128 ? go(conv_block64_kernel<2, 4, false>) : go(conv_block64_kernel<4, 8, false>);
}

#ifdef ICNN_B64_TRACE
extern "C" int icnn_debug_trace_b64(unsigned long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_b64_trace), sizeof(unsigned long long) * n);
}
#endif

}  // namespace icnn
