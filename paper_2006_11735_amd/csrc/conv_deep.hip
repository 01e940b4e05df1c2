// 3x3 / stride 1 / padding 1 integer convolution for layers with a deep K axis on few pixels (the late stages of
// the residual networks at moderate batch sizes): the eight waves of a workgroup split the K axis.
//
// The tile kernels (conv_igemm.hip, conv_halo.hip) walk K in 64-byte steps with a workgroup barrier per step, and a
// step costs 0.15-0.2 us whatever the tile shape: a 3x3 layer on 512 channels is 72 such steps in a row on a
// hundred workgroups.  Here nothing inside the K loop is shared between waves except read-only data:
//
//   tile     128 consecutive output pixels (raster order over the batch) x 64 output channels per workgroup
//   patch    the tile's input pixels with their one-pixel surround, ALL channels, in LDS once: rows are indexed by the
//            zero-padded raster index  pi = n*(H+2)*(W+2) + (y+1)*(W+2) + (x+1), so tap (kh, kw) of a pixel is the
//            row at a constant distance (kh-1)*(W+2) + (kw-1); border rows are zeros = the layer's padding
//   K split  wave w multiplies K fragments [w*F/8, (w+1)*F/8) of the F = 9*cin/32 fragments of 32 k-values (order
//            tap, channel), for the whole 128 x 64 tile: 8 accumulator tiles in registers.  Its weights come
//            STRAIGHT FROM GLOBAL MEMORY into A fragments (the packed order is the fragment order; no two waves
//            need the same bytes), nine steps ahead; its activation fragments come from the patch, one step ahead.
//            No barrier, no LDS ring, no copy waves in the loop.
//   reduce   the eight partial tiles of each wave are added into a 32 KiB int32 array in LDS (initialised with the
//            bias) with LDS atomics, register by register so that every wave-wide add is conflict-free; integer
//            addition is associative, so the sums are exact whatever the order.  After one barrier wave w holds
//            accumulator tile w in the usual layout and runs the usual epilogue on it.
//
// A workgroup moves 64 * K bytes of weights and the patch through the compute unit's memory path for 2 * 128 * 64 * K
// operations: about 100 operations per byte, against 128 for a 128 x 128 tile whose weights go through LDS, but twice
// as many workgroups, which is what a layer with a hundred 128 x 128 tiles on 256 compute units lacks.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

constexpr int kDeepBP = 128, kDeepBM = 64;
constexpr int kDeepRedBytes = 8 * 16 * 64 * 4;     // eight accumulator tiles of 32 x 32 int32
constexpr int kDeepRing = 9;                       // weight fragments are requested this many steps ahead
constexpr int kDeepPatchBatch = 16;                // 16-byte pieces of the patch a thread has in flight at once

struct DeepArgs {
    int wp2;            // W + 2
    int img;            // (H + 2) * (W + 2)
    FastDiv div_img, div_wp2, div_ppr;
    int rows;           // patch rows a workgroup copies (upper bound over all tiles)
    int ppr;            // 16-byte pieces per patch row: cin / 16
    int pitch;          // LDS bytes per patch row: cin + 16 (consecutive rows start four banks apart)
    int nchunks;        // cin / 64
    int patch_batches;  // ceil(rows * ppr / (512 * kDeepPatchBatch))
    int pt_per_idx;     // 8 / n_ct when the channel tiles divide the XCDs among themselves (see the kernel), else 0
};

#ifdef ICNN_DEEP_TRACE
__device__ unsigned long long g_deep_trace[8 * 16];
#define DEEP_TR(k)                                                                                              \
    do {                                                                                                        \
        if (blockIdx.x == ICNN_DEEP_TRACE && lane == 0) g_deep_trace[wave * 16 + (k)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#else
#define DEEP_TR(k)
#endif

template <bool U8, int G>          // G: cin / 256
__global__ __launch_bounds__(512, 1) void conv_deep_kernel(const ConvArgs a, const DeepArgs h)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr unsigned OOB = 0x80000000u;            // beyond any buffer this kernel accepts (< 2 GiB)
    constexpr int R = kDeepRing;
    static_assert(9 % R == 0, "the ring slot of a step must be static");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    // Which tile: with n_ct channel tiles dividing 8, XCD x (workgroups are dealt to the eight XCDs round-robin) takes
    // channel tile x % n_ct only, so that each L2 fetches 1/n_ct of the layer's weights instead of all of them
    int ct, pt;
    if (h.pt_per_idx) {
        const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
        ct = xcd % a.n_ct;
        pt = idx * h.pt_per_idx + xcd / a.n_ct;
        if (pt * kDeepBP >= a.M) return;             // whole workgroup
    } else if (!tile_of_block(a, ct, pt)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int32_t *const red = (int32_t *)lds;             // [tile 8][register 16][lane 64]
    uint8_t *const patch = lds + kDeepRedBytes;
    unsigned *const row_off = (unsigned *)(patch + h.rows * h.pitch);      // [rows]
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, a.wp_bytes, 0x00020000);
    DEEP_TR(0);

    // ---- patch: padded raster index of output pixel p (clamped to the last pixel)
    auto pi_of = [&](int p) {
        p = min(p, a.M - 1);
        const int n = fast_div(p, a.div_howo);
        const int r = p - n * a.Ho * a.Wo;
        const int y = fast_div(r, a.div_wo);
        const int x = r - y * a.Wo;
        return n * h.img + (y + 1) * h.wp2 + (x + 1);
    };
    const int pi_base = pi_of(pt * kDeepBP) - h.wp2 - 1;       // row 0: the first pixel's top-left tap
    // where each patch row starts in x (or beyond the buffer: border rows and rows past the last image), once per row
    for (int r = tid; r < h.rows; r += 512) {
        const int pi = pi_base + r;
        const int n = fast_div(pi, h.div_img);
        const int rr = pi - n * h.img;
        const int yy = fast_div(rr, h.div_wp2);
        const int xx = rr - yy * h.wp2;
        const bool ok = (n < a.N) & (yy >= 1) & (yy <= a.H) & (xx >= 1) & (xx <= a.W);
        row_off[r] = ok ? (unsigned)(((n * a.H + yy - 1) * a.W + xx - 1) * a.in_cs) : OOB;
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // All of the prologue's loads are issued before the first one is waited for, the patch first: one memory latency
    const int pieces = h.rows * h.ppr;
    v4i pv[kDeepPatchBatch];
    int pdst[kDeepPatchBatch];
    auto patch_fetch = [&](int b) {
#pragma unroll
        for (int k = 0; k < kDeepPatchBatch; ++k) {
            const int idx = min((b * kDeepPatchBatch + k) * 512 + tid, pieces - 1);     // the tail stores the last piece again
            const int r = fast_div(idx, h.div_ppr);
            const int q = idx - r * h.ppr;
            pv[k] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, row_off[r] + (unsigned)q * 16, 0, 0);   // zeros outside the buffer
            pdst[k] = r * h.pitch + q * 16;
        }
    };
    auto patch_store = [&]() {
#pragma unroll
        for (int k = 0; k < kDeepPatchBatch; ++k) *(v4i *)(patch + pdst[k]) = pv[k];
    };
    patch_fetch(0);
    __builtin_amdgcn_sched_barrier(0);

    // ---- the epilogue tile of this wave: pixel group wave & 3, channel chunk wave >> 2
    const int co_wave = ct * kDeepBM + (wave >> 2) * 32;
    const int pix_wave = pt * kDeepBP + (wave & 3) * 32;
    v4i res8[1][1];
    prefetch_res8<1, 1>(a, co_wave, pix_wave, lane, res8);
    v16i bias[1];
    load_bias_rows<1>(a, co_wave, lane >> 5, bias);
    __builtin_amdgcn_sched_barrier(0);

    // ---- this wave's K range and the first weight fragments
    constexpr int NF = 9 * G;                        // steps (fragments of 32 k-values) of this wave
    const int f0 = wave * NF;
    const unsigned w_tile = (unsigned)(ct * 2) * (unsigned)a.ksteps * kChunkBytes;     // chunk 2*ct, fragment 0
    const unsigned w_lane[2] = {(unsigned)lane * 16, (unsigned)a.ksteps * kChunkBytes + (unsigned)lane * 16};
    v4i A[R][2];
    // fragment i of the wave's range into ring slot SLOT
    auto fetch_a = [&](auto slot_tag, int i) {
        constexpr int SLOT = decltype(slot_tag)::value;
        const unsigned soff = w_tile + (unsigned)(f0 + i) * 1024u;
        A[SLOT][0] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_lane[0], soff, 0);
        A[SLOT][1] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_lane[1], soff, 0);
    };
    static_for<R>([&](auto s) { fetch_a(s, decltype(s)::value); });
    __builtin_amdgcn_sched_barrier(0);

    patch_store();
    for (int b = 1; b < h.patch_batches; ++b) {
        patch_fetch(b);
        patch_store();
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = bias[0][r];
    DEEP_TR(1);
    __builtin_amdgcn_s_waitcnt(0xC07F);              // this wave's LDS stores are done
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    DEEP_TR(2);

    // ---- K loop.  relp[j]: byte offset of pixel group j's centre-tap row for this lane (lanes 32..63: k 16..31)
    int relp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        relp[j] = (pi_of(pt * kDeepBP + j * 32 + (lane & 31)) - pi_base) * h.pitch + (lane >> 5) * 16;
    // Patch position of the next fragment to read.  A tap has 8 * groups fragments and a wave 9 * groups, so wave w
    // starts in tap w at channel fragment w * groups and crosses into tap w + 1 exactly once, n_first fragments in:
    // the byte offset grows by 32 per fragment plus one jump.
    auto tap_off = [&](int t) { return (((t * 11) >> 5) * h.wp2 + (t - 3 * ((t * 11) >> 5)) - h.wp2 - 1) * h.pitch; };
    const int n_first = G * (8 - wave);
    const int jump = tap_off(wave + 1) - tap_off(wave) - a.Cin;
    int soff_b = tap_off(wave) + wave * G * 32;
    auto b_advance = [&](int to) { soff_b += 32 + (to == n_first ? jump : 0); };      // to fragment `to` of the range
    v4i B[2][4];
    auto fetch_b = [&](auto set_tag, auto j_tag) {
        constexpr int SET = decltype(set_tag)::value;
        constexpr int J = decltype(j_tag)::value;
        v4i f = *(const v4i *)(patch + relp[J] + soff_b);
        if constexpr (U8) f ^= v4i{(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
        B[SET][J] = f;
    };
    static_for<4>([&](auto j) { fetch_b(std::integral_constant<int, 0>{}, j); });
    b_advance(1);

    v16i acc[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][j][r] = 0;

    // Straight-line code over all of the wave's steps: the wait counts the compiler derives are exact (around a loop it
    // falls back to waiting for nearly everything in flight at the loop's head)
    static_for<NF>([&](auto i_tag) {
        constexpr int i = decltype(i_tag)::value;
        using SLOT = std::integral_constant<int, i % R>;
        using SET = std::integral_constant<int, i & 1>;
        using NSET = std::integral_constant<int, (i & 1) ^ 1>;
#define ICNN_DEEP_MR(C, J)                                                                                   \
        acc[C][J] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[SLOT::value][C], B[SET::value][J], acc[C][J], 0, 0, 0); \
        if constexpr (C == 0 && i + 1 < NF) fetch_b(NSET{}, std::integral_constant<int, J>{});               \
        __builtin_amdgcn_sched_barrier(0);
        ICNN_DEEP_MR(0, 0) ICNN_DEEP_MR(0, 1) ICNN_DEEP_MR(0, 2) ICNN_DEEP_MR(0, 3)
        ICNN_DEEP_MR(1, 0) ICNN_DEEP_MR(1, 1) ICNN_DEEP_MR(1, 2) ICNN_DEEP_MR(1, 3)
#undef ICNN_DEEP_MR
        if constexpr (i + 2 < NF) b_advance(i + 2);
        if constexpr (i + R < NF) fetch_a(SLOT{}, i + R);
        __builtin_amdgcn_sched_barrier(0);
    });
    DEEP_TR(3);
    mfma_drain(acc);

    // ---- reduce: register r of tile t from every wave into red[t][r][lane]
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                __hip_atomic_fetch_add(red + ((c * 4 + j) * 16 + r) * 64 + lane, acc[c][j][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
    DEEP_TR(4);
    // the skip operand has landed; the adds are done
    __builtin_amdgcn_s_waitcnt(0x0070);              // vmcnt(0), lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    DEEP_TR(5);

    v16i sum[1][1];
#pragma unroll
    for (int r = 0; r < 16; ++r) sum[0][0][r] = red[(wave * 16 + r) * 64 + lane];
    if (a.pc)
        epilogue_pc_tiles<1, 1>(a, sum, co_wave, pix_wave, lane, res8, a.pc + (size_t)((ct * kDeepBM) >> 4) * kPcGroupInts,
                                ct * kDeepBM);
    else epilogue_tiles<1, 1>(a, sum, co_wave, pix_wave, lane, res8);
    DEEP_TR(6);
#endif
}

#ifdef ICNN_DEEP_TRACE
extern "C" int icnn_debug_trace_deep(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_deep_trace), sizeof(unsigned long long) * 8 * 16);
}
#endif

// ------------------------------------------------------------------ dispatch
// Upper bound of the rows of a patch over all pixel tiles: BP pixels, a padded image row and a pixel of taps on
// either side, and the borders crossed (2 per image row, 2 * (W + 2) more per image).
static long long deep_rows(const ConvArgs &a)
{
    const long long wp2 = a.W + 2;
    const long long hw = (long long)a.H * a.W;
    const long long row_crossings = (kDeepBP - 1) / a.W + 1;
    const long long image_crossings = (a.N == 1 || hw % kDeepBP == 0) ? 0 : (kDeepBP - 1) / hw + 1;
    return kDeepBP + 2 * wp2 + 2 + 2 * row_crossings + 2 * wp2 * image_crossings;
}

static bool deep_shape_ok(const ConvArgs &a)
{
    return a.KH == 3 && a.KW == 3 && a.sh == 1 && a.sw == 1 && a.ph == 1 && a.pw == 1 && a.Cin % 256 == 0 && a.Cin >= 256 && a.Cin <= 768 &&
           a.Ho == a.H && a.Wo == a.W && a.in_xor == 0 && a.x_bytes < 0x7fffff00u && a.wp_bytes < 0x7fffff00u &&
           (long long)(a.N + 1) * (a.H + 2) * (a.W + 2) < 0x7fffff00LL && a.ksteps == 9 * (a.Cin / 64) &&
           (a.in_cs & 15) == 0 && ((uintptr_t)a.x & 15) == 0 &&
           kDeepRedBytes + deep_rows(a) * (a.Cin + 16 + 4) <= 160 * 1024;
}

bool conv_deep_applies(const ConvArgs &a)
{
    if (!deep_shape_ok(a)) return false;
    if (g_tuning.deep_always) return true;
    // Worth it where all of its workgroups run at once: a workgroup spends as long before and after its K loop (patch,
    // reduction, epilogue) as in it, and nothing overlaps that with a second round.  Measured at 64 x 7 x 7 x 512 -> 512
    // (200 workgroups): 12.7 us against 17.4 us in the patch-resident kernel; at 64 x 14 x 14 x 256 -> 256 (392
    // workgroups): 18.8 us against 12.3 us.
    const long long wgs = (long long)((a.Cout + kDeepBM - 1) / kDeepBM) * ((a.M + kDeepBP - 1) / kDeepBP);
    return wgs <= 256;
}

hipError_t launch_conv_deep(const ConvArgs &a0, hipStream_t st)
{
    ConvArgs a = a0;
    if (!deep_shape_ok(a) || !finish_args(a, kDeepBM, kDeepBP)) return hipErrorInvalidValue;
    DeepArgs h;
    h.wp2 = a.W + 2;
    h.img = (a.H + 2) * (a.W + 2);
    h.div_img = make_fast_div((unsigned)h.img);
    h.div_wp2 = make_fast_div((unsigned)h.wp2);
    h.rows = (int)deep_rows(a);
    h.ppr = a.Cin / 16;
    h.div_ppr = make_fast_div((unsigned)h.ppr);
    h.pitch = a.Cin + 16;
    h.nchunks = a.Cin / 64;
    const long long pieces = (long long)h.rows * h.ppr;
    h.patch_batches = (int)((pieces + 512 * kDeepPatchBatch - 1) / (512 * kDeepPatchBatch));
    a.div_howo = make_fast_div((unsigned)(a.Ho * a.Wo));
    a.div_wo = make_fast_div((unsigned)a.Wo);
    a.n_vtiles = 8 * a.per_xcd;
    h.pt_per_idx = 0;
    if (8 % a.n_ct == 0 && !g_tuning.deep_plain_walk) {
        h.pt_per_idx = 8 / a.n_ct;
        const int n_pt = (a.M + kDeepBP - 1) / kDeepBP;
        a.n_vtiles = 8 * ((n_pt + h.pt_per_idx - 1) / h.pt_per_idx);
    }
    const size_t lds_bytes = (size_t)kDeepRedBytes + (size_t)h.rows * (h.pitch + 4);
    const dim3 grid((unsigned)a.n_vtiles), block(512);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a, h);
        return hipGetLastError();
    };
    switch (a.Cin / 256) {
    case 1: return a.frag_xor ? go(conv_deep_kernel<true, 1>) : go(conv_deep_kernel<false, 1>);
    case 2: return a.frag_xor ? go(conv_deep_kernel<true, 2>) : go(conv_deep_kernel<false, 2>);
    case 3: return a.frag_xor ? go(conv_deep_kernel<true, 3>) : go(conv_deep_kernel<false, 3>);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace icnn
