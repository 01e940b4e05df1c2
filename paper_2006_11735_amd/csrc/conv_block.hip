// A whole identity bottleneck block -- 1x1 conv, 3x3 conv, 1x1 conv with the block input merged in as skip
// operand (Section 4.1) -- as ONE kernel.  Layer by layer the block reads and writes its two narrow middle
// tensors and its wide input twice; here a workgroup takes a spatial tile of the image through all three
// layers, the middle tensors only ever exist in LDS, and the block costs one launch:
//
//   tile: TH x TW output pixels (at most 128), patch: the (TH+2) x (TW+2) input pixels under it (at most 160)
//   phase 1  a = BReLU/requant(conv1x1(x))  on the PATCH (the 3x3 layer's halo is recomputed, not exchanged);
//            patch pixels outside the image become zeros, which is the 3x3 layer's zero padding
//   phase 2  b = BReLU/requant(conv3x3(a))  on the tile: tap (kh, kw) of a pixel is patch row + (kh-1)*PW + (kw-1)
//   phase 3  y = epilogue(conv1x1(b), skip) on the tile, the layer's output channels in chunks of MID
//
// Every phase is a GEMM D[channels][pixels] on v_mfma_i32_32x32x32_i8 with the accumulator layout, packed weights
// and epilogue arithmetic of the other convolution kernels, so each result is the one the three separate layers
// give, bit for bit.
//
// Eight waves with three roles:
//   waves 0-3  multiply: read fragments from LDS, issue MFMAs, run the epilogues (phase 1 and 2 write LDS);
//   waves 4-5  weights:  stream the A operand of every K step (MID rows x 64 bytes) through a ring of six LDS
//              stages, five steps ahead, across phases and tiles;
//   waves 6-7  input:    copy the next tile's whole patch of x (all channels) into LDS while the current tile is
//              in phases 2 and 3.
// One workgroup barrier per K step, one before the first tile, one after phase 1's epilogue, one before and one
// after phase 2's (b overwrites a); all roles run the same loop nest with workgroup-uniform bounds, so the barrier
// counts match.  The multiply waves fetch the fragments of step g + 1 while they multiply step g's: the weight
// fragments right after barrier g, the activation fragments one by one, each into the registers of the fragment
// whose only MFMA has just been issued.  So before barrier g the weight waves have waited for stage g + 1 (loads
// retire in order and every stage is the same number of copies per wave: the wait count is a constant), and after
// it they refill the slot of stage g - 1, whose fragments every multiply wave has multiplied.  The input waves wait
// for everything they issued before a tile's first barrier; they start overwriting the patch only after the
// barrier that follows phase 1's epilogue.
#include "conv_common.h"

namespace icnn {

constexpr int kBlkRows = 160;        // patch rows: five pixel groups of 32
constexpr int kBlkPix = 128;         // output pixel slots of a tile: four groups
constexpr int kBlkStages = 6;        // weight ring
[[maybe_unused]] constexpr int kBlkDepth = kBlkStages - 1;      // stages issued ahead of the step being multiplied

// Development aid, compiled in with -DICNN_BLOCK_TRACE only: multiply wave 0 of one workgroup stamps the clock
// at the marked points; icnn_debug_trace() copies the stamps out.
#ifdef ICNN_BLOCK_TRACE
__device__ unsigned long long g_blk_trace[4096];
#define BLK_TR(k)                                                                                                  \
    do {                                                                                                           \
        if (blockIdx.x == 3 && wave8 == 0 && lane == 0 && trn < 4000)                                              \
            g_blk_trace[trn++] = ((unsigned long long)(k) << 56) | (__builtin_amdgcn_s_memtime() & 0xffffffffffffffULL); \
    } while (0)
#else
#define BLK_TR(k)
#endif

// MG: MID / 32: 2 (two workgroups per compute unit) or 4.  RQ24: all three layers requantise by the 32-bit form and the
// last one stores unsigned bytes with at most the plain 8-bit skip operand (the host checks; every calibrated layer of the
// workloads): the kernel then holds that one epilogue form instead of every form of every layer (a fifth of the code).
template <int MG, bool RQ24>
__global__ __launch_bounds__(512, MG == 2 ? 4 : 2) void conv_block_kernel(const BlockArgs g, const ConvArgs a1, const ConvArgs a2,
                                                                           const ConvArgs a3)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr int ASZ = MG * 2048;                   // one weight stage: MID rows x 64 bytes
    constexpr int WP = 4 / MG;                       // multiply waves along the pixel axis (the others along channels)
    constexpr int TP1 = (5 + WP - 1) / WP;           // pixel groups of a wave in phase 1 (five in all)
    constexpr int TP2 = 4 / WP;                      // ... in phases 2 and 3 (four in all)
    constexpr int SLICE_A = kBlkRows * 64;           // one 64-channel slice of the patch
    constexpr int SLICE_B = kBlkPix * 64;
    constexpr int MID = MG * 32;
    constexpr int NS = kBlkStages;
    // AHEAD: the multiply waves fetch step g + 1's fragments while they multiply step g's.  The 64-wide variant runs
    // two workgroups per compute unit inside 128 registers, where the second fragment set does not fit: it fetches a
    // step's fragments after the step's barrier and leaves the waiting to the other workgroup (measured: 59 us per
    // 64 x 56 x 56 x 256 block against 75 us with the fetch ahead and spills, or with one workgroup per unit).
    constexpr bool AHEAD = MG == 4;
    constexpr unsigned OOB = 0x80000000u;

    // LDS: weight ring | patch of x (k1 slices) | patch of a (s2 slices; later b on the tile, s2 slices) | biases
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int k1 = g.k1, nchunk3 = g.nchunk3;
    constexpr int s2 = MG / 2, k3 = MG / 2;
    uint8_t *const xbuf = lds + NS * ASZ;
    uint8_t *const abuf = xbuf + k1 * SLICE_A;
    uint8_t *const bbuf = abuf;                      // b overwrites a once every wave has left phase 2
    int32_t *const btab = (int32_t *)(abuf + s2 * SLICE_A);        // [MID] layer 1, [MID] layer 2, [C] layer 3

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles = g.n_tiles;

    // Workgroups go to the eight XCDs round-robin and every XCD has an L2 of its own: the workgroups of XCD x walk the
    // contiguous tile range [x * per_xcd, (x + 1) * per_xcd), so that the patch halos neighbouring tiles share meet in
    // one L2.  Work slot v (blockIdx.x, + gridDim.x, ...; the grid is a multiple of 8) is tile (v & 7) * per_xcd + (v >> 3);
    // a workgroup's tiles ascend, so its walk ends at the first slot beyond its XCD's range or beyond the last tile.
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
    // Without the fetch ahead a step's fragment reads are consumed inside the step, and the barrier that ends it lets the
    // weight waves overwrite their ring slot: the reads must have returned by then (lgkmcnt 0), whatever the compiler did
    // with the MFMAs that consume them.  With the fetch ahead the reads in flight at a barrier are those of the NEXT step,
    // whose slot and patch rows nobody writes for another step; they stay in flight on purpose.
    auto sync = [&]() {
        asm volatile("" ::: "memory");
        if (!AHEAD) __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // after LDS was written with ordinary stores: they have to be complete before the barrier lets other waves read
    // them (s_waitcnt lgkmcnt(0); the copy waves' barriers need nothing of the kind)
    auto sync_lds_written = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // Barriers of a workgroup, executed by all eight waves: one before the first tile, then per tile: k1 steps, one after
    // phase 1's epilogue, 9 * s2 steps, one before and one after phase 2's epilogue, nchunk3 * k3 steps.

    if (wave8 >= 6) {
        // ------------------------------------------------------------------ input waves
        const int xw = wave8 - 6;
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)g.x, 0, g.x_bytes, 0x00020000);
        unsigned p_off[5];
        // copy i of this wave fills patch rows 16 * (2i + xw) .. + 16; this lane the 16-byte piece lane & 3 of
        // row 16 * (2i + xw) + (lane >> 2), i.e. logical piece (lane & 3) ^ ((row >> 2) & 3)
        auto setup = [&](int v) {
            int n, y0, x0;
            tile_origin(v, n, y0, x0);
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                const int row = 16 * (2 * i + xw) + (lane >> 2);
                const int logical = (lane & 3) ^ ((row >> 2) & 3);
                const int py = (int)(((unsigned)row * g.inv_pw) >> 16);
                const int px = row - py * g.PW;
                const int iy = y0 - 1 + py, ix = x0 - 1 + px;
                const bool ok = py < g.TH + 2 && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
                p_off[i] = ok ? (unsigned)(((n * g.H + iy) * g.W + ix) * g.x_cs) + logical * 16 : OOB;
            }
        };
        auto issue_patch = [&]() {
            for (int k = 0; k < k1; ++k) {
#pragma unroll
                for (int i = 0; i < 5; ++i)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rs_x, (__attribute__((address_space(3))) void *)(xbuf + k * SLICE_A + (2 * i + xw) * 1024), 16, p_off[i],
                        k * kStepK, 0, 0);
            }
        };
        setup(blockIdx.x);
        issue_patch();
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT(0);
        sync();                                       // the first tile's patch is in LDS
        for (int v = blockIdx.x; valid(v); v += gridDim.x) {
            asm volatile("" ::: "memory");
            ICNN_WAIT_VMCNT(0);                       // this tile's patch is in LDS
            for (int k = 0; k < k1; ++k) sync();
            sync();                                   // phase 1 and its epilogue are over: the patch buffer is free
            if (valid(v + (int)gridDim.x)) {
                setup(v + (int)gridDim.x);
                issue_patch();
            }
            for (int s = 0; s < 9 * s2 + 2 + nchunk3 * k3; ++s) sync();
        }
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT(0);
        return;
    }

    if (wave8 >= 4) {
        // ------------------------------------------------------------------ weight waves
        constexpr int NA = MG;                        // wave-wide 1 KiB copies per stage and wave
        const int aw = wave8 - 4;
        const __amdgpu_buffer_rsrc_t rs_w1 = __builtin_amdgcn_make_buffer_rsrc((void *)a1.wp, 0, a1.wp_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs_w2 = __builtin_amdgcn_make_buffer_rsrc((void *)a2.wp, 0, a2.wp_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs_w3 = __builtin_amdgcn_make_buffer_rsrc((void *)a3.wp, 0, a3.wp_bytes, 0x00020000);
        // copy q of this wave covers packed pieces [64 * m, 64 * m + 64) of the stage, m = 2q + aw: piece e lies in
        // 32-channel chunk e >> 7 at byte (e & 127) * 16 of that chunk's 2 KiB block of the K step
        int chunk_of[NA];
        unsigned piece_off[NA];
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int e = (2 * q + aw) * 64 + lane;
            chunk_of[q] = e >> 7;
            piece_off[q] = (unsigned)(e & 127) * 16u;
        }
        // issue side: tile iv, phase iph (0, 1, 2), position (i0, i1) inside the phase
        int iv = blockIdx.x, iph = 0, i0 = 0, i1 = 0, islot = 0;
        bool imore = valid(iv);
        auto issue_next = [&]() {
            if (!imore) return;
            uint8_t *dst = lds + islot * ASZ;
            if (iph == 0) {                           // layer 1: K step i0 of k1
#pragma unroll
                for (int q = 0; q < NA; ++q)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w1, (__attribute__((address_space(3))) void *)(dst + (2 * q + aw) * 1024), 16,
                                                             (unsigned)(chunk_of[q] * k1) * kChunkBytes + piece_off[q], i0 * kChunkBytes, 0, 0);
                if (++i0 == k1) { i0 = 0; iph = 1; }
            } else if (iph == 1) {                    // layer 2: slice i0, tap i1: packed K step i1 * s2 + i0 of 9 * s2
#pragma unroll
                for (int q = 0; q < NA; ++q)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w2, (__attribute__((address_space(3))) void *)(dst + (2 * q + aw) * 1024), 16,
                                                             (unsigned)(chunk_of[q] * 9 * s2) * kChunkBytes + piece_off[q],
                                                             (i1 * s2 + i0) * kChunkBytes, 0, 0);
                if (++i1 == 9) {
                    i1 = 0;
                    if (++i0 == s2) { i0 = 0; iph = 2; }
                }
            } else {                                  // layer 3: channel chunk i0 (MG packed chunks), K step i1 of k3
#pragma unroll
                for (int q = 0; q < NA; ++q)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w3, (__attribute__((address_space(3))) void *)(dst + (2 * q + aw) * 1024), 16,
                                                             (unsigned)((i0 * MG + chunk_of[q]) * k3) * kChunkBytes + piece_off[q],
                                                             i1 * kChunkBytes, 0, 0);
                if (++i1 == k3) {
                    i1 = 0;
                    if (++i0 == nchunk3) {
                        i0 = 0;
                        iph = 0;
                        iv += gridDim.x;
                        imore = valid(iv);
                    }
                }
            }
            islot = islot + 1 == NS ? 0 : islot + 1;
        };
        // One K step g.  The multiply waves fetch stage g + 1's fragments right after barrier g, so that stage has landed
        // before it: of the stages issued so far (up to g + kBlkDepth - 1) at most kBlkDepth - 2 are younger.  After the
        // barrier the slot of stage g - 1 is free (its fragments were multiplied before the barrier): stage g + kBlkDepth.
        auto step = [&]() {
            asm volatile("" ::: "memory");
            if (imore) ICNN_WAIT_VMCNT((kBlkDepth - (AHEAD ? 2 : 1)) * NA);      // without the fetch ahead: stage g
            else ICNN_WAIT_VMCNT(0);                  // the issue side ran out: fewer younger stages than the count assumes
            sync();
            issue_next();
        };
        for (int d = 0; d < kBlkDepth; ++d) issue_next();      // a tile has more than kBlkDepth steps
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT((kBlkDepth - 1) * NA);        // stage 0
        sync();
        for (int v = blockIdx.x; valid(v); v += gridDim.x) {
            for (int k = 0; k < k1; ++k) step();
            sync();
            for (int s = 0; s < 9 * s2; ++s) step();
            sync();
            sync();
            for (int s = 0; s < nchunk3 * k3; ++s) step();
        }
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT(0);
        return;
    }

    // ---------------------------------------------------------------------- multiply waves
    const int wave = wave8;
    const int wm = MG == 2 ? (wave & 1) : wave;          // 32-channel chunk of the stage this wave multiplies
    const int wp = MG == 2 ? (wave >> 1) : 0;
    const int half = lane >> 5, col = lane & 31;
    const int n1 = MG == 2 ? (wp == 0 ? 3 : 2) : 5;      // pixel groups of this wave in phase 1
    const int pg1_0 = MG == 2 ? (wp == 0 ? 0 : 3) : 0;   // the first of them
    const int co_in_stage = wm * 32 + half * 16;         // this lane's 16 channels inside a stage's MID channels
    int slot = 0;                                        // ring slot of the stage the next step multiplies
    [[maybe_unused]] int trn = 0;

    // the three layers' biases, once per workgroup
    for (int i = tid; i < 2 * MID + g.nchunk3 * MID; i += 256)
        btab[i] = i < MID ? a1.bias[i] : (i < 2 * MID ? a2.bias[i - MID] : a3.bias[i - 2 * MID]);

    // Tile-invariant positions.  (Addresses are rebuilt from these few values inside the K loops, behind an opaque
    // copy: left alone, the compiler hoists dozens of loop-invariant addresses out of the loops and spills them.)
    // Phase 1: pixel group j of the wave is patch rows 32 * (pg1_0 + j) .. + 32
    const int row1_0 = 32 * pg1_0 + col;
    // Phases 2 and 3: pixel group j is output slots q = 32 * (wp * TP2 + j) + col, slot q = ty * TW + tx
    const int q2_0 = 32 * wp * TP2 + col;
    int rel[TP2], ty2[TP2], tx2[TP2];
#pragma unroll
    for (int j = 0; j < TP2; ++j) {
        const int q = q2_0 + 32 * j;
        const bool in_tile = q < g.TH * g.TW;
        ty2[j] = in_tile ? (int)(((unsigned)q * g.inv_tw) >> 16) : 0;
        tx2[j] = in_tile ? q - ty2[j] * g.TW : 0;
        if (!in_tile) ty2[j] = -1;                       // marks a slot beyond the tile
        rel[j] = (max(ty2[j], 0) + 1) * g.PW + tx2[j] + 1;      // patch row of the pixel (centre tap)
    }

    // Fragments.  A: the current step's (afc) and the next step's (afn), fetched one step ahead from the ring.
    // B: every fragment feeds exactly one MFMA (a wave owns one 32-channel chunk), so its registers are refilled with
    // the next step's fragment as soon as that MFMA is issued.
    v4i afc[2], afn[2];
    auto fetch_a = [&](v4i (&dst)[2], int s) {
        const uint8_t *S = lds + s * ASZ + wm * 2048 + lane * 16;
        dst[0] = *(const v4i *)S;
        dst[1] = *(const v4i *)(S + 1024);
    };
    auto next_slot = [&]() { return slot + 1 == NS ? 0 : slot + 1; };

    sync_lds_written();                  // before the first tile: bias table, stage 0 and the first patch are in LDS
    if (AHEAD) fetch_a(afc, 0);

    for (int v = blockIdx.x; valid(v); v += gridDim.x) {
        int n, y0, x0;
        tile_origin(v, n, y0, x0);
        // output pixels of phase 3 and the first chunk's skip operands (they travel during phases 1 and 2)
        int p3[TP2];
        bool ok3[TP2];
#pragma unroll
        for (int j = 0; j < TP2; ++j) {
            const int oy = y0 + ty2[j], ox = x0 + tx2[j];
            ok3[j] = ty2[j] >= 0 && oy < g.H && ox < g.W;
            p3[j] = ok3[j] ? (n * g.H + oy) * g.W + ox : 0;
        }
        const bool fetch_res = res8_applies(a3);
        const bool bytes3 = a3.out_mode != 3 && a3.epi_mode / 4 != 2 && (a3.res_mode == 0 || fetch_res);
        v4i res8[TP2];
        auto fetch_res8 = [&](int ch) {
#pragma unroll
            for (int j = 0; j < TP2; ++j) {
                res8[j] = v4i{0, 0, 0, 0};
                if (fetch_res && ok3[j])
                    res8[j] = *(const v4i *)((const uint8_t *)a3.res + ((size_t)p3[j] * a3.res_cs + ch * MID + co_in_stage));
            }
        };
        fetch_res8(0);
        BLK_TR(1);

        // ---------------- phase 1: a = requant(W1 x + b1) on the patch rows
        {
            v16i acc[TP1];
            {
                const v16i b = bias16(btab + co_in_stage);
#pragma unroll
                for (int j = 0; j < TP1; ++j) acc[j] = b;
            }
            v4i bf[2][TP1];
            for (int k = 0; k < k1; ++k) {
                sync();
                BLK_TR(10);
                int r0 = row1_0;
                asm volatile("" : "+v"(r0));
                if (k == 0 || !AHEAD) {                // (the patch is complete only after a tile's first barrier)
                    const uint8_t *X = xbuf + k * SLICE_A;
#pragma unroll
                    for (int kq = 0; kq < 2; ++kq)
#pragma unroll
                        for (int j = 0; j < TP1; ++j)     // rows 32 apart share the swizzle
                            if (j < n1) bf[kq][j] = *(const v4i *)(X + b_slot_offset(r0, kq * 2 + half) + j * 2048);
                }
                const int ns = next_slot();
                if (AHEAD) fetch_a(afn, ns);
                else fetch_a(afc, slot);
                const bool more = AHEAD && k + 1 < k1;
                const uint8_t *Xn = xbuf + (k + 1) * SLICE_A;
#pragma unroll
                for (int kq = 0; kq < 2; ++kq)
#pragma unroll
                    for (int j = 0; j < TP1; ++j)
                        if (j < n1) {
                            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afc[kq], bf[kq][j], acc[j], 0, 0, 0);
                            if (more) bf[kq][j] = *(const v4i *)(Xn + b_slot_offset(r0, kq * 2 + half) + j * 2048);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                afc[0] = afn[0];
                afc[1] = afn[1];
                slot = ns;
            }
            BLK_TR(3);
            mfma_drain(acc);
            // rows outside the image are the next layer's zero padding
            static_for<TP1>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                if (j >= n1) return;
                const int row = row1_0 + 32 * j;
                const int py = (int)(((unsigned)row * g.inv_pw) >> 16);
                const int px = row - py * g.PW;
                const int iy = y0 - 1 + py, ix = x0 - 1 + px;
                const bool ok = py < g.TH + 2 && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
                int t[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = acc[j][r];
                v4i w = RQ24 ? requant16<3>(a1, t) : requant16_any(a1, t);
                if (!ok) w = v4i{0, 0, 0, 0};
                const int piece = (co_in_stage & 63) >> 4;
                *(v4i *)(abuf + (co_in_stage >> 6) * SLICE_A + row * 64 + (((piece ^ (row >> 2)) & 3) << 4)) = w;
            });
        }
        BLK_TR(4);
        sync_lds_written();
        BLK_TR(5);

        // ---------------- phase 2: b = requant(W2 (*) a + b2) on the tile's pixel slots
        {
            v16i acc[TP2];
            {
                const v16i b = bias16(btab + MID + co_in_stage);
#pragma unroll
                for (int j = 0; j < TP2; ++j) acc[j] = b;
            }
            // fragment of pixel group j for tap offset toff in slice A: pieces 0, 1 hold k 0..31, pieces 2, 3 k 32..63
            v4i bf[2][TP2];
            auto fetch_b2 = [&](const uint8_t *A, int toff) {
#pragma unroll
                for (int j = 0; j < TP2; ++j) {
                    const int row = rel[j] + toff;
                    const int base = row * 64 + (((half ^ (row >> 2)) & 3) << 4);
                    bf[0][j] = *(const v4i *)(A + base);
                    bf[1][j] = *(const v4i *)(A + (base ^ 32));
                }
            };
            if (AHEAD) fetch_b2(abuf, -g.PW - 1);
            for (int c = 0; c < s2; ++c) {
                const uint8_t *A = abuf + c * SLICE_A;
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    sync();
                    BLK_TR(11);
                    const int ns = next_slot();
                    if (AHEAD) fetch_a(afn, ns);
                    else {
                        fetch_a(afc, slot);
                        int toff = (t / 3 - 1) * g.PW + (t % 3 - 1);
                        asm volatile("" : "+s"(toff));
                        fetch_b2(A, toff);
                    }
                    const int tn = t == 8 ? 0 : t + 1;
                    const bool more = AHEAD && (t < 8 || c + 1 < s2);
                    const uint8_t *An = t == 8 ? A + SLICE_A : A;
                    int toffn = (tn / 3 - 1) * g.PW + (tn % 3 - 1);
                    asm volatile("" : "+s"(toffn));
#pragma unroll
                    for (int j = 0; j < TP2; ++j) {
                        const int row = rel[j] + toffn;
                        const int base = row * 64 + (((half ^ (row >> 2)) & 3) << 4);
                        acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afc[0], bf[0][j], acc[j], 0, 0, 0);
                        if (more) bf[0][j] = *(const v4i *)(An + base);
                        if (AHEAD) __builtin_amdgcn_sched_barrier(0);
                        acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afc[1], bf[1][j], acc[j], 0, 0, 0);
                        if (more) bf[1][j] = *(const v4i *)(An + (base ^ 32));
                        if (AHEAD) __builtin_amdgcn_sched_barrier(0);
                    }
                    if (AHEAD) { afc[0] = afn[0]; afc[1] = afn[1]; }
                    slot = ns;
                }
            }
            BLK_TR(6);
            sync();                      // every wave has its last fragments of a: b may overwrite it
            mfma_drain(acc);
            BLK_TR(9);
            static_for<TP2>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                int t[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) t[r] = acc[j][r];
                const v4i w = RQ24 ? requant16<3>(a2, t) : requant16_any(a2, t);      // slots beyond the tile hold values nobody stores
                *(v4i *)(bbuf + (co_in_stage >> 6) * SLICE_B + b_slot_offset(q2_0 + 32 * j, (co_in_stage & 63) >> 4)) = w;
            });
        }
        BLK_TR(7);
        sync_lds_written();
        BLK_TR(8);

        // ---------------- phase 3: y = epilogue(W3 b + b3, skip), MID output channels at a time
        {
            v4i bf[2][TP2];
            auto fetch_b3 = [&](const uint8_t *Bq) {
                int qa = q2_0;
                asm volatile("" : "+v"(qa));
#pragma unroll
                for (int kq = 0; kq < 2; ++kq)
#pragma unroll
                    for (int j = 0; j < TP2; ++j) bf[kq][j] = *(const v4i *)(Bq + b_slot_offset(qa, kq * 2 + half) + j * 2048);
            };
            if (AHEAD) fetch_b3(bbuf);
            for (int ch = 0; ch < nchunk3; ++ch) {
                const int co0 = ch * MID + co_in_stage;
                v16i acc[TP2];
                {
                    const v16i b = bias16(btab + 2 * MID + co0);
#pragma unroll
                    for (int j = 0; j < TP2; ++j) acc[j] = b;
                }
                BLK_TR(20);
#pragma unroll
                for (int k = 0; k < k3; ++k) {
                    sync();
                    BLK_TR(12);
                    const int ns = next_slot();
                    if (AHEAD) fetch_a(afn, ns);
                    else {
                        fetch_a(afc, slot);
                        fetch_b3(bbuf + k * SLICE_B);
                    }
                    const bool more = AHEAD && (k + 1 < k3 || ch + 1 < nchunk3);
                    const uint8_t *Bn = bbuf + (k + 1 < k3 ? k + 1 : 0) * SLICE_B;
                    int qa = q2_0;
                    asm volatile("" : "+v"(qa));
#pragma unroll
                    for (int kq = 0; kq < 2; ++kq)
#pragma unroll
                        for (int j = 0; j < TP2; ++j) {
                            acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(afc[kq], bf[kq][j], acc[j], 0, 0, 0);
                            if (more) bf[kq][j] = *(const v4i *)(Bn + b_slot_offset(qa, kq * 2 + half) + j * 2048);
                            if (AHEAD) __builtin_amdgcn_sched_barrier(0);
                        }
                    if (AHEAD) { afc[0] = afn[0]; afc[1] = afn[1]; }
                    slot = ns;
                }
                BLK_TR(21);
                mfma_drain(acc);
                if constexpr (RQ24) {
                    static_for<TP2>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        const v4i w = fetch_res ? epilogue_bytes16<1, 3>(a3, acc[j], res8[j]) : epilogue_bytes16<0, 3>(a3, acc[j], res8[j]);
                        if (ok3[j]) *(v4i *)((uint8_t *)a3.out + (size_t)p3[j] * a3.out_cs + a3.out_co + co0) = w;
                    });
                } else if (bytes3) {
                    // an 8-bit output whose skip operand, if any, is the 8-bit kind joined before requantisation: the short form
                    static_for<TP2>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        const v4i w = fetch_res ? epilogue_bytes16<1>(a3, acc[j], res8[j]) : epilogue_bytes16<0>(a3, acc[j], res8[j]);
                        if (ok3[j]) *(v4i *)((uint8_t *)a3.out + (size_t)p3[j] * a3.out_cs + a3.out_co + co0) = w;
                    });
                } else {
                    static_for<TP2>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        if (ok3[j]) epilogue_px16(a3, acc[j], p3[j], co0, res8[j]);
                    });
                }
                BLK_TR(22);
                // the next chunk's skip operands travel during its K steps (the first chunk's during phases 1 and 2)
                if (ch + 1 < nchunk3) fetch_res8(ch + 1);
            }
        }
    }
#endif
}

// ------------------------------------------------------------------ dispatch
size_t conv_block_lds_bytes(int mid, int c)
{
    const int mg = mid / 32, k1 = c / 64, s2 = mid / 64;
    return (size_t)kBlkStages * mg * 2048 + (size_t)k1 * kBlkRows * 64 + (size_t)s2 * kBlkRows * 64 + (size_t)(2 * mid + c) * 4;
}

// Output tile TH x TW with TH * TW <= 128 and (TH + 2) * (TW + 2) <= 160 that covers the image with the fewest tiles
// (ties: the widest).  Also the two multiply-shift divisors the kernel uses, checked over their whole ranges.
bool conv_block_tile(int H, int W, BlockArgs &g)
{
    long long best = -1;
    for (int th = 1; th <= 126; ++th)
        for (int tw = 1; tw <= 126; ++tw) {
            if (th * tw > kBlkPix || (th + 2) * (tw + 2) > kBlkRows) continue;
            const long long tiles = (long long)((H + th - 1) / th) * ((W + tw - 1) / tw);
            if (best < 0 || tiles < best || (tiles == best && tw > g.TW)) {
                best = tiles;
                g.TH = th;
                g.TW = tw;
            }
        }
    if (best < 0) return false;
    g.PW = g.TW + 2;
    g.tiles_x = (W + g.TW - 1) / g.TW;
    g.tiles_per_img = g.tiles_x * ((H + g.TH - 1) / g.TH);
    g.inv_tw = 65536u / (unsigned)g.TW + 1;
    g.inv_pw = 65536u / (unsigned)g.PW + 1;
    for (unsigned q = 0; q < (unsigned)kBlkPix; ++q)
        if (((q * g.inv_tw) >> 16) != q / (unsigned)g.TW) return false;
    for (unsigned r = 0; r < (unsigned)kBlkRows; ++r)
        if (((r * g.inv_pw) >> 16) != r / (unsigned)g.PW) return false;
    return true;
}

hipError_t launch_conv_block(const BlockArgs &g, const ConvArgs &a1, const ConvArgs &a2, const ConvArgs &a3, hipStream_t st)
{
    const int mid = a1.Cout;
    const size_t lds_bytes = conv_block_lds_bytes(mid, a1.Cin);
    if (lds_bytes > 160 * 1024 || (mid != 64 && mid != 128) || g.n_tiles < 1) return hipErrorInvalidValue;
    const int per_cu = mid == 64 && 2 * lds_bytes <= 160 * 1024 ? 2 : 1;
    const int slots = 256 * per_cu;
    BlockArgs gx = g;
    gx.per_xcd = (g.n_tiles + 7) / 8;
    const dim3 grid((unsigned)(8 * gx.per_xcd < slots ? 8 * gx.per_xcd : slots)), block(512);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, gx, a1, a2, a3);
        return hipGetLastError();
    };
    const bool res8 = a3.epi_vec && !(a3.Cout & 15) && a3.res_mode != 0 && a3.res_dtype != 2;       // res8_applies(a3)
    const bool rq24 = a1.rq24 && a2.rq24 && a3.rq24 && a3.out_mode != 3 && a3.epi_mode / 4 != 2 && (a3.res_mode == 0 || res8) &&
                      !g_tuning.block_any_form;
    if (mid == 64) return rq24 ? go(conv_block_kernel<2, true>) : go(conv_block_kernel<2, false>);
    return rq24 ? go(conv_block_kernel<4, true>) : go(conv_block_kernel<4, false>);
}

#ifdef ICNN_BLOCK_TRACE
extern "C" int icnn_debug_trace(unsigned long long *host, int n)
{
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_blk_trace), sizeof(unsigned long long) * n);
}
#endif

}  // namespace icnn
