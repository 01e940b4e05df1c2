// 3x3 / stride 1 / padding 1 integer convolution with the input patch resident in LDS and separate
// copy and multiply waves.
//
// Same computation, packed weights, accumulator layout and epilogue as conv_dlds_kernel (conv_igemm.hip).
// That kernel gathers the activation operand tap by tap: every K step copies 64 bytes per output pixel
// from L2 into LDS, so a 3x3 layer moves each input byte nine times, and its K loop runs at the rate the
// compute unit can copy into LDS.  Here the nine taps of a 64-channel slice read one LDS copy of the input:
//
//   * Output pixels are numbered in (n, y, x) raster order and a tile is BP consecutive ones, as before.
//   * Input pixels get a PADDED raster index  pi = n*(H+2)*(W+2) + (y+1)*(W+2) + (x+1): the image with its
//     zero border.  Tap (kh, kw) of output pixel pi sits at  pi + (kh-1)*(W+2) + (kw-1): a constant offset,
//     whatever the pixel, with no border cases.  The taps of a tile cover one contiguous range of pi (the
//     "patch": BP + 2*(W+2) + 2 indices plus the borders it crosses).
//   * The patch of one 64-channel slice is copied to LDS as 64-byte rows, row r = index pi_base + r, by
//     wave-wide direct-to-LDS copies; border rows and rows beyond the tensor ask for an address outside
//     the buffer and receive zeros.  16-byte pieces are swizzled by (pi >> 2) & 3 so that fragment reads
//     of consecutive pixels spread over all banks.
//   * K order is (channel slice c, tap t): packed weight step t * (cin/64) + c.  Weights stream through a
//     ring of LDS stages (A operand only, BM*64 bytes per step); patches alternate between two buffers.
//
// A workgroup has eight waves.  Waves 4..7 only copy: weight stages kHaloDepth steps ahead and, during the
// first kHaloInst steps of a slice, the next slice's patch (the next tile's first one at a tile's end) in
// instalments of PQ wave-wide copies per step.  Waves 0..3 only read fragments and multiply, and run the
// epilogue.  They keep two fragment sets in registers: after the barrier of step g they request the
// fragments of step g + 1 and multiply those of step g, requested a step earlier, so no MFMA waits for
// LDS; this carries over from a tile's last step to the next tile's first.
//
// Synchronisation is one workgroup barrier per K step, executed by all eight waves; steps are counted
// over all tiles of the (persistent) workgroup.  Before barrier g a copy wave waits until its part of
// stage g + 1 (and of every patch instalment older than it) has landed; an extra barrier before the loop
// does the same for stage 0 and the first patch.  After barrier g every multiply wave has finished reading
// stage g - 1 (the MFMAs of step g - 1 are issued, so their operands had arrived), whose slot the copy waves
// refill; the other patch buffer was last read two slices ago.
// Both roles execute the same loop nest (tiles, slices, taps) with workgroup-uniform bounds, so the
// barrier counts match.
#include "conv_common.h"

#include <type_traits>

namespace icnn {

struct HaloArgs {
    int wp2;            // W + 2
    int img;            // (H + 2) * (W + 2)
    FastDiv div_img, div_wp2;
    int npq;            // wave-wide copies per copy wave per patch (always PQ * kHaloInst, so that every instalment
                        // step issues exactly PQ of them): patch buffer = npq * 4096 bytes = npq * 64 rows
    int nchunks;        // cin / 64
};

constexpr int kHaloStages = 6;                    // weight ring
constexpr int kHaloDepth = kHaloStages - 1;       // weight stages issued ahead of the step being multiplied
constexpr int kHaloInst = 10 - kHaloDepth;        // a patch goes out in the first kHaloInst steps of the previous slice
constexpr int kHaloMaxPq = 3;
constexpr int kHaloMaxNpq = kHaloMaxPq * kHaloInst;

// Copy waves, top of a slice's step t: number of this wave's copies that are certainly younger than weight
// stage g + 1 (g = the step).  Stage g + 1 was issued in step g + 1 - D, after that step's instalment;
// steps g + 2 - D .. g - 1 follow it.  Steps before the slice (u < 0) issued a stage each and no instalment
// (instalments stop kHaloInst = 10 - D steps into a slice, and u >= 2 - D).  pnext: this slice carries
// instalments.  Loads retire in order, so s_waitcnt vmcnt(that) proves stage g + 1 and everything older landed.
constexpr int halo_younger(int t, bool pnext, int NA, int PQ)
{
    int n = 0;
    for (int u = t + 2 - kHaloDepth; u < t; ++u) {
        n += NA;
        if (u >= 0 && pnext && u < kHaloInst) n += PQ;
    }
    return n;
}

// PC: per-output-channel requantisation (epilogue_pc_tiles, parameters read from global memory).  Its
// registers do not fit beside the state a workgroup keeps for its next tile, so these instantiations
// handle exactly one tile per workgroup (the launcher sees to it): everything about a next tile folds away.
template <int BM, int BP, int WAVES_M, int WAVES_P, int PQ, bool PC, bool U8>
__global__ __launch_bounds__(512, 1) void conv_halo_kernel(const ConvArgs a, const HaloArgs h)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr int TM = BM / WAVES_M / 32;
    constexpr int TP = BP / WAVES_P / 32;
    constexpr int A_BYTES = BM * kStepK;
    constexpr int A_INSTR = BM / 16;                 // wave-wide 1 KiB copies per weight stage, whole workgroup
    constexpr int NA = A_INSTR / 4;                  // per copy wave
    constexpr int D = kHaloDepth;
    constexpr int nstA = kHaloStages;
    constexpr unsigned OOB = 0x80000000u;            // beyond any buffer this kernel accepts (< 2 GiB)
    static_assert(WAVES_M * WAVES_P == 4 && TM >= 1 && TP >= 1 && NA >= 1, "tile shape");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int patch_bytes = h.npq * 4096;
    uint8_t *const patch0 = lds + nstA * A_BYTES;    // two patch buffers

    auto tile_of = [&](int v, int &ct, int &pt) {
        const int logical = (v & 7) * a.per_xcd + (v >> 3);
        ct = logical % a.n_ct;
        pt = logical / a.n_ct;
        return logical < a.n_tiles;
    };
    {
        int ct, pt;
        if (!tile_of(blockIdx.x, ct, pt)) return;     // whole workgroup
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nchunks = h.nchunks;                   // K steps of a tile: 9 * nchunks

    // padded raster index of output pixel p (clamped to the last pixel)
    auto pi_of = [&](int p) {
        p = min(p, a.M - 1);
        const int n = fast_div(p, a.div_howo);
        const int r = p - n * a.Ho * a.Wo;
        const int y = fast_div(r, a.div_wo);
        const int x = r - y * a.Wo;
        return n * h.img + (y + 1) * h.wp2 + (x + 1);
    };
    // first patch row of pixel tile pt: the row of its first pixel's top-left tap, rounded down to 16
    auto pi_base_of = [&](int pt_) { return (pi_of(pt_ * BP) - h.wp2 - 1) & ~15; };

    if (wave8 >= 4) {
        // ------------------------------------------------------------------ copy waves
        const int wave = wave8 - 4;
        const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, a.wp_bytes, 0x00020000);
        // weights: copy q of this wave covers packed pieces [64*m, 64*m + 64), m = (4*q + wave) % A_INSTR
        unsigned a_off[NA];
        int a_lds[NA];
#pragma unroll
        for (int q = 0; q < NA; ++q) a_lds[q] = ((4 * q + wave) % A_INSTR) * 1024;
        auto setup_weights = [&](int ct_) {
            const int chunk0 = ct_ * (BM / 32);
#pragma unroll
            for (int q = 0; q < NA; ++q) {
                const int e = a_lds[q] / 16 + lane;
                a_off[q] = (unsigned)(chunk0 + (e >> 7)) * (unsigned)(9 * nchunks) * kChunkBytes + (unsigned)(e & 127) * 16;
            }
        };
        // patch: copy q of this wave fills rows 16*(4*q + wave) .. +16; this lane the 16-byte piece lane & 3 of
        // row 16*(4*q + wave) + (lane >> 2).  p_off[q]: byte offset of that piece in x for slice 0, or OOB.
        unsigned p_off[kHaloMaxNpq];
        auto setup_patch = [&](int pt_) {
            const int pb = pi_base_of(pt_);
#pragma unroll
            for (int q = 0; q < kHaloMaxNpq; ++q) {
                p_off[q] = OOB;
                if (q < h.npq) {
                    const int pi = pb + 16 * (4 * q + wave) + (lane >> 2);
                    const int logical = (lane & 3) ^ ((pi >> 2) & 3);
                    const int n = fast_div(pi, h.div_img);
                    const int r = pi - n * h.img;
                    const int yy = fast_div(r, h.div_wp2);
                    const int xx = r - yy * h.wp2;
                    const bool ok = n < a.N && yy >= 1 && yy <= a.H && xx >= 1 && xx <= a.W;
                    if (ok) p_off[q] = (unsigned)(((n * a.H + yy - 1) * a.W + xx - 1) * a.in_cs) + logical * 16;
                }
            }
        };
        auto issue_patch_copy = [&](int c, int pbuf_, int q) {
            if (q < h.npq)     // workgroup-uniform; OOB plus the slice offset stays beyond the buffer
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rs_x, (__attribute__((address_space(3))) void *)(patch0 + pbuf_ * patch_bytes + (4 * q + wave) * 1024), 16,
                    p_off[q], c * kStepK, 0, 0);
        };

        // ---- issue side of the weight ring: (iv, ic, it) = tile, slice and tap of the next stage to copy
        int iv = blockIdx.x, ict, ipt;
        bool imore = tile_of(iv, ict, ipt);
        int ic = 0, it = 0, islot = 0;
        setup_weights(ict);
        auto issue_next_weights = [&]() {
            if (!imore) return;
            const int ps = it * nchunks + ic;
#pragma unroll
            for (int q = 0; q < NA; ++q)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (__attribute__((address_space(3))) void *)(lds + islot * A_BYTES + a_lds[q]),
                                                         16, a_off[q], ps * kChunkBytes, 0, 0);
            islot = islot + 1 == nstA ? 0 : islot + 1;
            if (++it == 9) {
                it = 0;
                if (++ic == nchunks) {
                    ic = 0;
                    iv += gridDim.x;
                    imore = iv < a.n_vtiles && tile_of(iv, ict, ipt);
                    if (imore) setup_weights(ict);
                }
            }
        };

        // ---- first tile: patch of slice 0, then the leading weight stages; barrier -1 once stage 0 landed
        int ct, pt;
        tile_of(blockIdx.x, ct, pt);
        setup_patch(pt);
#pragma unroll
        for (int q = 0; q < kHaloMaxNpq; ++q) issue_patch_copy(0, 0, q);
        for (int d = 0; d < D; ++d) issue_next_weights();
        asm volatile("" ::: "memory");
        ICNN_WAIT_VMCNT((D - 1) * NA);       // at least D stages exist (9 steps per slice)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");

        int pbuf = 0;             // patch buffer of the slice being multiplied
        for (int v = blockIdx.x; v < a.n_vtiles && tile_of(v, ct, pt); v += gridDim.x) {
            int nct = 0, npt = 0;
            const bool more = v + (int)gridDim.x < a.n_vtiles && tile_of(v + (int)gridDim.x, nct, npt);
            for (int c = 0; c < nchunks; ++c) {
                const bool last_chunk = c + 1 == nchunks;
                const bool pnext = !last_chunk || more;        // this slice carries the next patch's instalments
                auto step = [&](auto t_tag) {
                    constexpr int t = decltype(t_tag)::value;
                    asm volatile("" ::: "memory");
                    // once the issue side has run out (the workgroup's last D steps) the counts below would be
                    // too generous: wait for everything
                    if (!imore) ICNN_WAIT_VMCNT(0);
                    else if (pnext) ICNN_WAIT_VMCNT(halo_younger(t, true, NA, PQ));
                    else ICNN_WAIT_VMCNT(halo_younger(t, false, NA, PQ));
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    if (t < kHaloInst && pnext) {
                        if (t == 0 && last_chunk) setup_patch(npt);
#pragma unroll
                        for (int k = 0; k < PQ; ++k) issue_patch_copy(last_chunk ? 0 : c + 1, pbuf ^ 1, t * PQ + k);
                    }
                    issue_next_weights();
                };
                step(std::integral_constant<int, 0>{}); step(std::integral_constant<int, 1>{}); step(std::integral_constant<int, 2>{});
                step(std::integral_constant<int, 3>{}); step(std::integral_constant<int, 4>{}); step(std::integral_constant<int, 5>{});
                step(std::integral_constant<int, 6>{}); step(std::integral_constant<int, 7>{}); step(std::integral_constant<int, 8>{});
                pbuf ^= 1;
            }
        }
        ICNN_WAIT_VMCNT(0);
        return;
    }

    // ---------------------------------------------------------------------- multiply waves
    const int wave = wave8;
    const int wm = wave % WAVES_M;
    const int wp = wave / WAVES_M;
    const int a_rd = wm * TM * 2048 + lane * 16;
    // patch row of this lane's pixel j (centre tap) in tile pt_
    auto rel_of = [&](int pt_, int j) { return pi_of(pt_ * BP + wp * TP * 32 + j * 32 + (lane & 31)) - pi_base_of(pt_); };

    int ct, pt;
    int v = blockIdx.x;
    tile_of(v, ct, pt);
    int rel[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) rel[j] = rel_of(pt, j);

    // Two fragment sets: a step multiplies one while the next step's fragments arrive in the other.  A tile
    // always starts with its first step's fragments in set 0.
    v4i af[2][2][TM], bf[2][2][TP];
    int buf = 0;              // ring slot of the stage whose fragments are requested next
    // read r of the 2 * (TM + TP) fragment reads of a step (r < 2 * TM: weights, then activations) into set SET;
    // brow[j]: byte offset of pixel j's first 16-byte piece (k 0..15 for lanes 0..31, 16..31 for lanes 32..63)
    auto request_one = [&](auto set_tag, auto r_tag, const uint8_t *SA, const uint8_t *SP, const int (&brow)[TP]) {
        constexpr int SET = decltype(set_tag)::value;
        constexpr int r = decltype(r_tag)::value;
        if constexpr (r < 2 * TM) af[SET][r & 1][r >> 1] = *(const v4i *)(SA + a_rd + r * 1024);
        else bf[SET][(r - 2 * TM) & 1][(r - 2 * TM) >> 1] = *(const v4i *)(SP + (brow[(r - 2 * TM) >> 1] ^ (((r - 2 * TM) & 1) << 5)));
    };
    auto b_rows = [&](const int (&rel_)[TP], int toff, int (&brow)[TP]) {
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int row = rel_[j] + toff;
            // 16-byte pieces 0, 1 hold k 0..31, pieces 2, 3 k 32..63; piece index XOR (row >> 2) & 3
            brow[j] = row * 64 + ((((lane >> 5) ^ (row >> 2)) & 3) << 4);
        }
    };
    auto request_all = [&](auto set_tag, int pbuf_, const int (&rel_)[TP], int toff) {
        const uint8_t *SA = lds + buf * A_BYTES;
        const uint8_t *SP = patch0 + pbuf_ * patch_bytes;
        int brow[TP];
        b_rows(rel_, toff, brow);
        request_one(set_tag, std::integral_constant<int, 0>{}, SA, SP, brow);
        request_one(set_tag, std::integral_constant<int, 1>{}, SA, SP, brow);
        if constexpr (TM + TP > 1) { request_one(set_tag, std::integral_constant<int, 2>{}, SA, SP, brow); request_one(set_tag, std::integral_constant<int, 3>{}, SA, SP, brow); }
        if constexpr (TM + TP > 2) { request_one(set_tag, std::integral_constant<int, 4>{}, SA, SP, brow); request_one(set_tag, std::integral_constant<int, 5>{}, SA, SP, brow); }
        if constexpr (TM + TP > 3) { request_one(set_tag, std::integral_constant<int, 6>{}, SA, SP, brow); request_one(set_tag, std::integral_constant<int, 7>{}, SA, SP, brow); }
        buf = buf + 1 == nstA ? 0 : buf + 1;
    };
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();        // barrier -1: stage 0 and the first patch complete
    asm volatile("" ::: "memory");
    request_all(std::integral_constant<int, 0>{}, 0, rel, -h.wp2 - 1);

    v16i bias_next[TM];
    load_bias_rows<TM>(a, ct * BM + wm * TM * 32, lane >> 5, bias_next);
    int pbuf = 0;             // patch buffer of the slice being multiplied

    for (;;) {
        v16i acc[TM][TP];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = bias_next[i];
        const int co_wave = ct * BM + wm * TM * 32;
        const int pix_wave = pt * BP + wp * TP * 32;
        v4i res8[TM][TP];
        prefetch_res8<TM, TP>(a, co_wave, pix_wave, lane, res8);
        int nct = 0, npt = 0;
        const bool more = !PC && v + (int)gridDim.x < a.n_vtiles && tile_of(v + (int)gridDim.x, nct, npt);
        int rel_next[TP];     // this lane's patch rows in the next tile
#pragma unroll
        for (int j = 0; j < TP; ++j) rel_next[j] = more ? rel_of(npt, j) : rel[j];

        // one K step: tap t of slice c multiplies set SET and requests the next step's fragments into the other set
        auto step = [&](auto t_tag, auto set_tag, int c) {
            constexpr int t = decltype(t_tag)::value;
            constexpr int SET = decltype(set_tag)::value;
            constexpr int t2 = t == 8 ? 0 : t + 1;                     // tap of the next step
            const bool last_chunk = c + 1 == nchunks;
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();      // the next step's stage (and patch) complete, see above
            asm volatile("" ::: "memory");
            const int toff2 = (t2 / 3 - 1) * h.wp2 + (t2 % 3 - 1);
            // The next step's fragment reads are issued one by one between this step's MFMAs, so that a read
            // waiting for room in the LDS queue holds up the wave while the matrix core is busy anyway.  They are
            // unconditional: after the workgroup's very last step they read slots nobody writes any more.
            const uint8_t *SA = lds + buf * A_BYTES;
            const uint8_t *SP = patch0 + (t == 8 ? pbuf ^ 1 : pbuf) * patch_bytes;
            int brow[TP];
            if (t == 8 && last_chunk) b_rows(rel_next, toff2, brow);
            else b_rows(rel, toff2, brow);
            buf = buf + 1 == nstA ? 0 : buf + 1;
            using NS = std::integral_constant<int, SET ^ 1>;
            static_assert(TM == 2 && TP == 2, "the interleaving below is written for 2 x 2 MFMA tiles per wave");
            v4i b00 = bf[SET][0][0], b01 = bf[SET][0][1], b10 = bf[SET][1][0], b11 = bf[SET][1][1];
            if constexpr (U8) {
                const v4i m = v4i{(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
                b00 ^= m; b01 ^= m; b10 ^= m; b11 ^= m;
            }
#define ICNN_HALO_MR(I, J, A, B, R)                                                                      \
            acc[I][J] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A, B, acc[I][J], 0, 0, 0);                 \
            request_one(NS{}, std::integral_constant<int, R>{}, SA, SP, brow);                           \
            __builtin_amdgcn_sched_barrier(0);
            ICNN_HALO_MR(0, 0, af[SET][0][0], b00, 0)
            ICNN_HALO_MR(0, 1, af[SET][0][0], b01, 1)
            ICNN_HALO_MR(1, 0, af[SET][0][1], b00, 2)
            ICNN_HALO_MR(1, 1, af[SET][0][1], b01, 3)
            ICNN_HALO_MR(0, 0, af[SET][1][0], b10, 4)
            ICNN_HALO_MR(0, 1, af[SET][1][0], b11, 5)
            ICNN_HALO_MR(1, 0, af[SET][1][1], b10, 6)
            ICNN_HALO_MR(1, 1, af[SET][1][1], b11, 7)
#undef ICNN_HALO_MR
        };
        // the nine steps of slice c, the first one multiplying set S0; the next slice's first fragments end up in S0 ^ 1
        auto slice = [&](auto s0_tag, int c) {
            constexpr int S0 = decltype(s0_tag)::value;
            using A = std::integral_constant<int, S0>;
            using B = std::integral_constant<int, S0 ^ 1>;
            step(std::integral_constant<int, 0>{}, A{}, c); step(std::integral_constant<int, 1>{}, B{}, c);
            step(std::integral_constant<int, 2>{}, A{}, c); step(std::integral_constant<int, 3>{}, B{}, c);
            step(std::integral_constant<int, 4>{}, A{}, c); step(std::integral_constant<int, 5>{}, B{}, c);
            step(std::integral_constant<int, 6>{}, A{}, c); step(std::integral_constant<int, 7>{}, B{}, c);
            step(std::integral_constant<int, 8>{}, A{}, c);
            pbuf ^= 1;
        };
        int c = 0;
        for (; c + 1 < nchunks; c += 2) {
            slice(std::integral_constant<int, 0>{}, c);
            slice(std::integral_constant<int, 1>{}, c + 1);
        }
        if (c < nchunks) {
            // odd number of slices: the next tile's first fragments went to set 1; move them to set 0
            slice(std::integral_constant<int, 0>{}, c);
#pragma unroll
            for (int kq = 0; kq < 2; ++kq) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[0][kq][i] = af[1][kq][i];
#pragma unroll
                for (int j = 0; j < TP; ++j) bf[0][kq][j] = bf[1][kq][j];
            }
        }
        // the skip operands (this wave's only loads) have landed
        ICNN_WAIT_VMCNT(0);
        mfma_drain(acc);

        v += gridDim.x;
        if (more) load_bias_rows<TM>(a, nct * BM + wm * TM * 32, lane >> 5, bias_next);
        if constexpr (PC)
            epilogue_pc_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, res8, a.pc + (size_t)((ct * BM) >> 4) * kPcGroupInts, ct * BM);
        else epilogue_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, res8);
        if (!more) break;
        ct = nct;
        pt = npt;
#pragma unroll
        for (int j = 0; j < TP; ++j) rel[j] = rel_next[j];
    }
#endif
}

// ------------------------------------------------------------------ dispatch
// Upper bound of the rows of a patch over all pixel tiles of BP pixels: BP pixels, two padded image rows and
// two pixels of taps around them, the borders crossed (2 per image row, 2 * (W + 2) more per image) and the
// rounding of the first row down to a multiple of 16.
static int halo_max_rows(const ConvArgs &a, int BP)
{
    const long long wp2 = a.W + 2;
    const long long hw = (long long)a.H * a.W;
    const long long row_crossings = (BP - 1) / a.W + 1;
    // tiles never straddle two images when there is one image or images are whole numbers of tiles
    const long long image_crossings = (a.N == 1 || hw % BP == 0) ? 0 : (BP - 1) / hw + 1;
    const long long rows = BP + 2 * wp2 + 2 + 2 * row_crossings + 2 * wp2 * image_crossings + 15;
    return rows > 1 << 20 ? 1 << 20 : (int)rows;
}

static bool halo_shape_ok(const ConvArgs &a)
{
    return a.KH == 3 && a.KW == 3 && a.sh == 1 && a.sw == 1 && a.ph == 1 && a.pw == 1 && a.Cin % 64 == 0 && a.Cin >= 64 &&
           a.Ho == a.H && a.Wo == a.W && a.in_xor == 0 && a.x_bytes < 0x7fffff00u && a.wp_bytes < 0x7fffff00u &&
           (long long)(a.N + 1) * (a.H + 2) * (a.W + 2) < 0x7fffff00LL && a.M >= 64 && a.ksteps == 9 * (a.Cin / 64);
}

template <int BM, int BP, int WAVES_M, int WAVES_P, int PQ>
static hipError_t launch_halo(const ConvArgs &a0, int rows, hipStream_t st)
{
    ConvArgs a = a0;
    if (!finish_args(a, BM, BP)) return hipErrorInvalidValue;
    HaloArgs h;
    h.wp2 = a.W + 2;
    h.img = (a.H + 2) * (a.W + 2);
    h.div_img = make_fast_div((unsigned)h.img);
    h.div_wp2 = make_fast_div((unsigned)h.wp2);
    if ((rows + 63) / 64 > PQ * kHaloInst) return hipErrorInvalidValue;
    h.npq = PQ * kHaloInst;
    h.nchunks = a.Cin / 64;
    a.nstages = kHaloStages;
    a.div_howo = make_fast_div((unsigned)(a.Ho * a.Wo));
    a.div_wo = make_fast_div((unsigned)a.Wo);
    const size_t lds_bytes = (size_t)kHaloStages * BM * kStepK + 2 * (size_t)h.npq * 4096;
    if (h.npq > kHaloMaxNpq || lds_bytes > 160 * 1024) return hipErrorInvalidValue;
    a.n_vtiles = 8 * a.per_xcd;
    const dim3 grid((unsigned)(a.n_vtiles < 256 ? a.n_vtiles : 256)), block(512);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a, h);
        return hipGetLastError();
    };
    if (a.pc) {
        if (a.n_tiles > (int)grid.x) return hipErrorInvalidValue;          // one tile per workgroup, see halo_choice
        return a.frag_xor ? go(conv_halo_kernel<BM, BP, WAVES_M, WAVES_P, PQ, true, true>)
                          : go(conv_halo_kernel<BM, BP, WAVES_M, WAVES_P, PQ, true, false>);
    }
    return a.frag_xor ? go(conv_halo_kernel<BM, BP, WAVES_M, WAVES_P, PQ, false, true>)
                      : go(conv_halo_kernel<BM, BP, WAVES_M, WAVES_P, PQ, false, false>);
}

// tile shape for a layer: 0 none (not applicable), 1: 128 x 128, 2: 64 x 256
static int halo_choice(const ConvArgs &a, int *rows)
{
    if (!halo_shape_ok(a)) return 0;
    int choice = a.Cout > 64 ? 1 : 2;
    if (g_tuning.halo_tile) choice = g_tuning.halo_tile;
    if (choice != 1 && choice != 2) return 0;
    const int bp = choice == 1 ? 128 : 256, bm = choice == 1 ? 128 : 64;
    *rows = halo_max_rows(a, bp);
    int pq = ((*rows + 63) / 64 + kHaloInst - 1) / kHaloInst;
    if (choice == 2 && pq < 2) pq = 2;    // the instantiations that exist (launch_conv_halo)
    const int npq = pq * kHaloInst;       // patch buffers are whole instalments
    const size_t lds = (size_t)kHaloStages * bm * kStepK + 2 * (size_t)npq * 4096;
    if (pq > (choice == 1 ? 2 : kHaloMaxPq) || lds > 160 * 1024) return 0;
    // One workgroup per compute unit: a tile's epilogue is not hidden behind another workgroup's K loop.  Measured:
    // the kernel wins clearly where a workgroup has one tile and the K loop has 18 steps or more (12.3 against 17 us
    // at 64 x 14 x 14 x 256 -> 256); with several tiles per workgroup it is 3-10 % ahead of the tap-by-tap kernel
    // (two workgroups per unit; 22.8 against 25.5 us at 128 x 14 x 14 x 256 -> 256, 29.2 against 30.6 at
    // 128 x 28 x 28 x 128 -> 128 stand-alone, but the ResNet-18 shape's 18-step layers on 392 tiles came out 2 % slower
    // inside the network), and 9-step tiles lose.  The halo_always override lifts both limits.
    const long long tiles = (long long)((a.Cout + bm - 1) / bm) * ((a.M + bp - 1) / bp);
    if (a.ksteps < (tiles > 256 ? 36 : 18) && !g_tuning.halo_always) return 0;
    if (a.pc && tiles > 256) return 0;       // per-channel instantiations: one tile per workgroup
    return choice;
}

bool conv_halo_applies(const ConvArgs &a)
{
    int rows = 0;
    return halo_choice(a, &rows) != 0;
}

hipError_t launch_conv_halo(const ConvArgs &a, hipStream_t st)
{
    int rows = 0;
    const int choice = halo_choice(a, &rows);
    const int pq = ((rows + 63) / 64 + kHaloInst - 1) / kHaloInst;
    // (128 x 128 tiles with three copies per instalment would need more than 160 KiB of LDS; 256-pixel tiles
    // never get by with one)
    if (choice == 1) {
        if (pq == 1) return launch_halo<128, 128, 2, 2, 1>(a, rows, st);
        if (pq == 2) return launch_halo<128, 128, 2, 2, 2>(a, rows, st);
    }
    if (choice == 2) {
        if (pq <= 2) return launch_halo<64, 256, 1, 4, 2>(a, rows, st);
        if (pq == 3) return launch_halo<64, 256, 1, 4, 3>(a, rows, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace icnn
