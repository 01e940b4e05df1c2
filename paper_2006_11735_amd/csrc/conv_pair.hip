// Two pointwise layers back to back as ONE kernel: the 1x1 convolution that closes a bottleneck block (skip operand
// merged in its epilogue, Section 4.1) and the 1x1 convolution that opens the next block, which reads nothing but
// that result.  Layer by layer the wide tensor between them is written, read back by the second layer and read
// again as the next skip operand; here it is written once and multiplied straight out of LDS, and the two layers
// cost one launch.
//
//   tile     64 consecutive pixels of the flattened N*H*W axis (pointwise layers have no spatial structure)
//   phase 1  y = epilogue(W3 t + b3, skip): all C output channels of the tile.  The tile of t (K3 <= 256 channels)
//            goes through LDS once and then sits in every wave's registers as MFMA B fragments for the whole phase
//            (fetched per wave it would cross the compute unit's memory pipe eight times: measured 20.6 us against
//            17.6 us on 12544 pixels of 256 -> 1024 -> 256); every wave owns C/8 output channels and
//            streams their packed weights from global memory straight into A fragments (the packed order IS the
//            fragment order, and no two waves need the same rows, so LDS would only add a copy).  The 16 bytes a
//            lane produces go to the tile's row of y in LDS; after the phase the tile is stored row by row.
//   phase 2  z = BReLU/requant(W1 y + b1): K = C, activations from LDS, weights again straight from global memory,
//            a 32-channel chunk of the MID2 outputs per wave.
//
// What bounds it is the compute unit's path from L2: a 64-pixel tile pulls both layers' packed weights (512 KB at
// 256 <-> 1024 channels) plus its skip operands through it, at the 25-35 bytes per clock that path delivers, while the
// matrix cores need a quarter of that time; hence one tile per workgroup and nothing fetched twice.
//
// Every product runs on v_mfma_i32_32x32x32_i8 with the accumulator layout, packed weights and epilogue arithmetic
// of the other convolution kernels: y and z are the two separate layers' results, bit for bit.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

constexpr int kPairPix = 64;

// Development aid, compiled in with -DICNN_PAIR_TRACE only: wave 0 of one workgroup stamps the clock at the marked
// points; icnn_debug_trace_pair() copies the stamps out.
#ifdef ICNN_PAIR_TRACE
__device__ unsigned long long g_pair_trace[256];
__device__ unsigned long long g_pair_span[4096];
#define PAIR_TR(k)                                                                                                 \
    do {                                                                                                           \
        if (((k) == 1 || (k) == 8) && lane == 0 && wave == 0 && blockIdx.x < 2048)                                 \
            g_pair_span[blockIdx.x * 2 + ((k) == 8)] = __builtin_amdgcn_s_memtime();                              \
        if (blockIdx.x == 3 && wave == 0 && lane == 0 && trn < 250)                                                \
            g_pair_trace[trn++] = ((unsigned long long)(k) << 56) | (__builtin_amdgcn_s_memtime() & 0xffffffffffffffULL); \
    } while (0)
#define PAIR_TW(k)                                                                                                 \
    do {                                                                                                           \
        if (blockIdx.x == 3 && lane == 0) g_pair_span[4000 + wave * 8 + (k)] = __builtin_amdgcn_s_memtime();       \
    } while (0)
#else
#define PAIR_TR(k)
#define PAIR_TW(k)
#endif

struct PairArgs {
    int P;                      // pixels (N * H * W)
    unsigned res_bytes, y_bytes;
};

// K3 / 32 (fragments of the first layer's K), MID2 / 32 (chunks of the second's outputs); PIPE: the first layer's
// requantisation has the 32-bit form (a3.rq24) and its epilogue is dealt out between the matrix instructions
template <int KF, int MG2, bool PIPE>
__global__ __launch_bounds__(512, KF == 8 ? 1 : 2) void conv_pair_kernel(const ConvArgs a3, const ConvArgs a1, const PairArgs g)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr unsigned OOB = 0x80000000u;
    constexpr int NJ2 = MG2 == 8 ? 2 : 1;             // pixel groups of a wave in phase 2
    constexpr int GF = 8;                             // weight fragments fetched together in phase 2

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int C = a3.Cout;
    const int pitch = C + 16;                         // row pitch of y: the column-wise fragment reads hit every bank once
    uint8_t *const ybuf = lds;
    int32_t *const btab = (int32_t *)(lds + kPairPix * pitch);     // [C] first layer, [MID2] second

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, col = lane & 31;
    const int P = g.P;
    const int p0 = blockIdx.x * kPairPix;
    [[maybe_unused]] int trn = 0;
    PAIR_TR(1);
    PAIR_TW(0);

    // Everything the first chunk needs is requested before anything is waited for: the two layers' biases (for a
    // table in LDS), the tile of t, the first chunk's weights and skip operands.
    constexpr int NB = (2048 + 256) / 512 + 1;        // bias values per thread at the widest shape
    int bv[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int i = tid + q * 512;
        bv[q] = i < C ? a3.bias[i] : (i < C + MG2 * 32 ? a1.bias[i - C] : 0);
    }

    // the tile of t goes through LDS once (every wave needs all of it): 16-byte pieces, rows padded like y's
    constexpr int K3 = KF * 32, TPITCH = K3 + 16, TPIECES = kPairPix * K3 / 16, TQ = (TPIECES + 511) / 512;
    uint8_t *const tbuf = (uint8_t *)(btab + C + MG2 * 32);
    v4i tv[TQ];
    {
        const __amdgpu_buffer_rsrc_t rs_t = __builtin_amdgcn_make_buffer_rsrc((void *)a3.x, 0, a3.x_bytes, 0x00020000);
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
            const int e = tid + q * 512, row = e / (K3 / 16), piece = e % (K3 / 16);
            const unsigned off = e < TPIECES && p0 + row < P ? (unsigned)(p0 + row) * (unsigned)a3.in_cs + piece * 16 : OOB;
            tv[q] = __builtin_amdgcn_raw_buffer_load_b128(rs_t, off, 0, 0);
        }
    }
    int p[2];
    bool okp[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        p[j] = p0 + 32 * j + col;
        okp[j] = p[j] < P;
    }

    // ---------------- phase 1
    // Skip operand and y go through buffer descriptors: a pixel beyond the tensor (or a layer without skip operand: an
    // empty descriptor) reads zeros and stores nothing, without a branch.  Every fetch below is unconditional, so the
    // number of younger loads at each wait is a constant the compiler can count on.
    v4i bt[2][KF];
    const bool has_res = a3.res_mode != 0;
    const __amdgpu_buffer_rsrc_t rs_r =
        __builtin_amdgcn_make_buffer_rsrc(has_res ? (void *)a3.res : (void *)a3.out, 0, has_res ? g.res_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc((void *)a3.out, 0, g.y_bytes, 0x00020000);
    unsigned r_off[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) r_off[j] = okp[j] ? (unsigned)p[j] * (unsigned)a3.res_cs + half * 16 : OOB;
    const int cpw = C >> 8;                           // 32-channel chunks per wave
    const int chunk0 = wave * cpw, chunk_last = chunk0 + cpw - 1;
    auto clamp_chunk = [&](int chunk) { return chunk < chunk_last ? chunk : chunk_last; };   // past the wave's last chunk: fetched again, never used
    auto load_w3 = [&](v4i (&A)[KF], int chunk) __attribute__((always_inline)) {
        const v4i *src = (const v4i *)(a3.wp + (size_t)clamp_chunk(chunk) * (KF * 1024)) + lane;
#pragma unroll
        for (int f = 0; f < KF; ++f) A[f] = src[f * 64];
        __builtin_amdgcn_sched_barrier(0);            // issued here, not wherever the scheduler finds their first use
    };
    auto load_r3 = [&](v4i (&r)[2], int chunk) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 2; ++j) r[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_r, r_off[j], clamp_chunk(chunk) * 32, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    // The products of one 32 x 32 tile (chunk, pixel group J) ...
    auto mul_tile = [&](auto j_tag, const v4i (&A)[KF], int chunk, v16i &acc) __attribute__((always_inline)) {
        constexpr int J = decltype(j_tag)::value;
        acc = bias16(btab + chunk * 32 + half * 16);
#pragma unroll
        for (int f = 0; f < KF; ++f) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[f], bt[J][f], acc, 0, 0, 0);
    };
    // ... and its epilogue: sixteen requantised bytes into the pixel's row of y in LDS.  RQ as in epilogue_bytes16.
    auto fin_tile = [&](auto j_tag, auto rq_tag, const v16i &acc, const v4i &r, int chunk) __attribute__((always_inline)) {
        constexpr int J = decltype(j_tag)::value, RQ = decltype(rq_tag)::value;
        const v4i w = has_res ? epilogue_bytes16<1, RQ>(a3, acc, r) : epilogue_bytes16<0, RQ>(a3, acc, r);
        *(v4i *)(ybuf + (32 * J + col) * pitch + chunk * 32 + half * 16) = w;
    };
    // One step of the software pipeline: a tile's matrix instructions and the previous tile's epilogue are independent.
    // With the 32-bit requantisation form (RQ = 3, straight-line code) the epilogue is dealt out in slices, one after
    // every matrix instruction and pinned there, so that the vector ALUs finish one tile while the matrix core
    // multiplies the next instead of the two waiting for each other (a slice is 16 / KF outputs = about the vector
    // work that fits beside one matrix instruction).  With the form chosen at run time (RQ = 0) the two simply follow
    // each other.
    // JN: pixel group of the new tile (the old one is the other group: of the same chunk for JN = 1, of the chunk
    // before for JN = 0).
    auto step = [&](auto jn_tag, auto rq_tag, const v4i (&A)[KF], int chunk, v16i &acc_new, v16i &acc_old, const v4i &r_old) __attribute__((always_inline)) {
        constexpr int JN = decltype(jn_tag)::value, RQ = decltype(rq_tag)::value;
        const int chunk_old = JN ? chunk : chunk - 1;
        mfma_drain(acc_old);
        if constexpr (RQ == 3) {
            int w[4];
            acc_new = bias16(btab + chunk * 32 + half * 16);
            __builtin_amdgcn_sched_barrier(0);
            static_for<KF>([&](auto f_tag) {
                constexpr int f = decltype(f_tag)::value;
                acc_new = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[f], bt[JN][f], acc_new, 0, 0, 0);
                epilogue_rq24_slice<1, f * (16 / KF), 16 / KF>(a3, acc_old, r_old, w);
                __builtin_amdgcn_sched_barrier(0);
            });
            *(v4i *)(ybuf + (32 * (JN ^ 1) + col) * pitch + chunk_old * 32 + half * 16) = v4i{w[0], w[1], w[2], w[3]};
        } else {
            // kept apart: left to the scheduler, the epilogue's byte extractions move up among the matrix instructions
            // and the registers run out
            fin_tile(std::integral_constant<int, JN ^ 1>{}, rq_tag, acc_old, r_old, chunk_old);
            __builtin_amdgcn_sched_barrier(0);
            mul_tile(jn_tag, A, chunk, acc_new);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    {
        // Weights travel two chunks ahead of their products, skip operands from the end of one step to the epilogue two
        // steps later; every fetch is unconditional (a conditional use would let the compiler move the fetch down to it).
        v4i A0[KF], A1[KF], r0[2], r1[2];
        v16i accx, accy;                              // tiles of pixel group 0 / 1
        load_w3(A0, chunk0);
        load_r3(r0, chunk0);
        PAIR_TR(9);
        PAIR_TW(1);
#pragma unroll
        for (int q = 0; q < NB; ++q)
            if (tid + q * 512 < C + MG2 * 32) btab[tid + q * 512] = bv[q];
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
            const int e = tid + q * 512;
            if (e < TPIECES) *(v4i *)(tbuf + (e / (K3 / 16)) * TPITCH + (e % (K3 / 16)) * 16) = tv[q];
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        PAIR_TR(10);           // the table's writes are done (lgkmcnt 0); the fetches travel on
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        PAIR_TR(2);
        PAIR_TW(3);
        // B fragments of t: fragment f of pixel group j is bytes [32 f + 16 half, + 16) of pixel 32 j + col
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int f = 0; f < KF; ++f) bt[j][f] = *(const v4i *)(tbuf + (32 * j + col) * TPITCH + f * 32 + half * 16);
        load_w3(A1, chunk0 + 1);
        load_r3(r1, chunk0 + 1);
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I3 = std::integral_constant<int, 3>;
        mul_tile(I0{}, A0, chunk0, accx);             // the first tile: nothing to finish yet
        auto rest = [&](auto rq_tag) __attribute__((always_inline)) {
            // chunk c (weights A_cur, skip operands r_cur): its second tile while its first is finished, then the next
            // chunk's first tile (weights A_nxt) while its second is finished; r_cur is free after that and takes the
            // operands of chunk c + 2, A_cur those weights before
            auto chunk_steps = [&](const v4i (&A_cur)[KF], v4i (&A_cur_w)[KF], const v4i (&A_nxt)[KF], v4i (&r_cur)[2], int c) __attribute__((always_inline)) {
                step(I1{}, rq_tag, A_cur, c, accy, accx, r_cur[0]);
                load_w3(A_cur_w, c + 2);
                step(I0{}, rq_tag, A_nxt, c + 1, accx, accy, r_cur[1]);
                load_r3(r_cur, c + 2);
            };
            int c = 0;                                // relative to chunk0
            for (; c + 2 < cpw; c += 2) {
                chunk_steps(A0, A0, A1, r0, chunk0 + c);
                chunk_steps(A1, A1, A0, r1, chunk0 + c + 1);
            }
            if (c + 1 < cpw) {                        // two chunks left: c (A0, r0) and c + 1 (A1, r1)
                chunk_steps(A0, A0, A1, r0, chunk0 + c);
                step(I1{}, rq_tag, A1, chunk0 + c + 1, accy, accx, r1[0]);
                mfma_drain(accy);
                fin_tile(I1{}, rq_tag, accy, r1[1], chunk0 + c + 1);
            } else {                                  // one chunk left: c (A0, r0)
                step(I1{}, rq_tag, A0, chunk0 + c, accy, accx, r0[0]);
                mfma_drain(accy);
                fin_tile(I1{}, rq_tag, accy, r0[1], chunk0 + c);
            }
        };
        // the pipelined form always runs the skip operand's arithmetic: without one the empty descriptor delivers zero
        // bytes and the launcher has set res_mul = 0, res_shift = 0, so that the term is zero
        if constexpr (PIPE) rest(I3{});
        else rest(I0{});
    }

    // ---------------- phase 2
    const bool active = wave < 2 * MG2;               // 2 * MG2 (chunk, pixel group) pairs when a wave takes one group
    const int c2 = wave & (MG2 - 1);
    const int pg = MG2 == 8 ? 0 : wave / MG2;
    const int ng = C / (32 * GF);                     // fragment groups along K = C
    auto load_a1 = [&](v4i (&A)[GF], int gi) {
        gi = gi < ng ? gi : ng - 1;                   // past the last group: fetched again, never used
        const v4i *src = (const v4i *)(a1.wp + ((size_t)c2 * (C >> 5) + (size_t)gi * GF) * 1024) + lane;
#pragma unroll
        for (int f = 0; f < GF; ++f) A[f] = src[f * 64];
        __builtin_amdgcn_sched_barrier(0);
    };
    v4i A0[GF], A1[GF];
    load_a1(A0, 0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);               // this wave's rows of y are in LDS (lgkmcnt 0; the global accesses travel on)
    PAIR_TR(5);
    PAIR_TW(4);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    PAIR_TR(6);
    PAIR_TW(5);
    // y goes to memory from LDS, a pixel's whole row of C bytes per wave and pass in 16-byte pieces of consecutive
    // lanes (stored from the epilogue, 32 bytes per pixel at a time with the rest of the 128-byte line following a
    // chunk later, the writes reached memory as 1.55 times y's size)
    {
        const int pieces = C >> 4;                    // 16-byte pieces of a pixel's row: 16, 32, ... 128
        for (int e = tid; e < kPairPix * pieces; e += 512) {
            const int row = e / pieces, piece = e - row * pieces;
            const v4i w = *(const v4i *)(ybuf + row * pitch + piece * 16);
            const unsigned off = p0 + row < P ? (unsigned)(p0 + row) * (unsigned)a3.out_cs + (unsigned)a3.out_co + piece * 16 : OOB;
            __builtin_amdgcn_raw_buffer_store_b128(w, rs_y, off, 0, 0);
        }
    }
    if (!active) return;
    v16i acc[NJ2];
    {
        const v16i b = bias16(btab + C + c2 * 32 + half * 16);
#pragma unroll
        for (int j = 0; j < NJ2; ++j) acc[j] = b;
    }
    const uint8_t *yrow = ybuf + (32 * pg + col) * pitch + half * 16;
    auto mul_group = [&](const v4i (&A)[GF], int gi) {
        const uint8_t *yg = yrow + gi * (32 * GF);
#pragma unroll
        for (int f = 0; f < GF; ++f)
#pragma unroll
            for (int j = 0; j < NJ2; ++j)
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[f], *(const v4i *)(yg + j * 32 * pitch + f * 32), acc[j], 0, 0, 0);
        PAIR_TR(7);
    };
    int gi = 0;
    if (ng & 1) {                                     // as in phase 1: an odd group count starts with a single group
        load_a1(A1, 1);
        mul_group(A0, 0);
#pragma unroll
        for (int f = 0; f < GF; ++f) A0[f] = A1[f];
        gi = 1;
    }
    for (; gi < ng; gi += 2) {
        load_a1(A1, gi + 1);
        mul_group(A0, gi);
        load_a1(A0, gi + 2);
        mul_group(A1, gi + 1);
    }
    mfma_drain(acc);
    static_for<NJ2>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int pz = p0 + 32 * (pg + j) + col;
        const v4i w = epilogue_bytes16<0>(a1, acc[j], v4i{0, 0, 0, 0});
        if (pz < P) *(v4i *)((uint8_t *)a1.out + (size_t)pz * a1.out_cs + a1.out_co + c2 * 32 + half * 16) = w;
    });
    PAIR_TR(8);
    PAIR_TW(6);
#endif
}

// ------------------------------------------------------------------ dispatch
size_t conv_pair_lds_bytes(int c, int mid2)
{
    return (size_t)kPairPix * (c + 16) + (size_t)(c + mid2) * 4 + (size_t)kPairPix * (mid2 + 16);
}

hipError_t launch_conv_pair(const ConvArgs &a3, const ConvArgs &a1, long long pixels, hipStream_t st)
{
    const int kf = a3.Cin / 32, mg2 = a1.Cout / 32;
    const size_t lds_bytes = conv_pair_lds_bytes(a3.Cout, a1.Cout);
    if (a3.Cin % 64 || a1.Cout % 32 || kf != mg2 || (kf != 2 && kf != 4 && kf != 8) || a3.Cout % 256 || a1.Cin != a3.Cout ||
        lds_bytes > 160 * 1024 || pixels < 1 || pixels > 0x7fffffffLL - kPairPix)
        return hipErrorInvalidValue;
    // byte extents of the skip operand and of y up to the end of the last pixel's channels, for the descriptors
    const unsigned long long rb = a3.res_mode ? (unsigned long long)(pixels - 1) * a3.res_cs + a3.Cout : 0;
    const unsigned long long yb = (unsigned long long)(pixels - 1) * a3.out_cs + a3.out_co + a3.Cout;
    if (rb >= 0x7fffff00ull || yb >= 0x7fffff00ull) return hipErrorInvalidValue;
    PairArgs g;
    g.P = (int)pixels;
    g.res_bytes = (unsigned)rb;
    g.y_bytes = (unsigned)yb;
    const dim3 grid((unsigned)((pixels + kPairPix - 1) / kPairPix)), block(512);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a3, a1, g);
        return hipGetLastError();
    };
    ConvArgs b3 = a3;
    if (!b3.res_mode) b3.res_mul = b3.res_shift = 0;      // the pipelined epilogue always runs the skip operand's arithmetic
    auto go3 = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, b3, a1, g);
        return hipGetLastError();
    };
    if (a3.rq24 && (!a3.res_mode || a3.res_fast))
        return kf == 2 ? go3(conv_pair_kernel<2, 2, true>) : kf == 4 ? go3(conv_pair_kernel<4, 4, true>) : go3(conv_pair_kernel<8, 8, true>);
    return kf == 2 ? go(conv_pair_kernel<2, 2, false>) : kf == 4 ? go(conv_pair_kernel<4, 4, false>) : go(conv_pair_kernel<8, 8, false>);
}

#ifdef ICNN_PAIR_TRACE
extern "C" int icnn_debug_trace_pair(unsigned long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_pair_trace), sizeof(unsigned long long) * n);
}
extern "C" int icnn_debug_span_pair(unsigned long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_pair_span), sizeof(unsigned long long) * n);
}
#endif

}  // namespace icnn
