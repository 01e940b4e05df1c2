// Integer convolution layer as an implicit GEMM on the gfx950 int8 matrix cores.
//
// Computes, per output pixel p and channel co (Section 3.1 / Figure 1, Section
// 3.2.1's requantisation, Section 4.1's skip merge):
//   U = sum_k X[p, k] * W[co, k],  Y = U + b,  T = Y (+ rescaled skip),
//   V = clamp([T * mul / 2^shift], lo, hi)
// as D = Wmat (cout x K) times Xcol (K x pixels) with v_mfma_i32_32x32x32_i8.
// The weight matrix is the A operand (rows = output channels), the gathered
// activations are the B operand (columns = output pixels), so every lane ends
// up with sixteen consecutive channels of one pixel: the epilogue runs on
// registers and stores 16 bytes per lane; int32 never reaches memory.
//
// One workgroup = 256 threads = 4 waves, tile BM output channels x BP pixels,
// K advanced 64 at a time.  Two kernels share the tile layout and the epilogue:
//   conv_dlds_kernel  cin % 16 == 0, aligned: tiles go from global memory straight
//                     into a ring of LDS stages (global_load_lds_dwordx4), several
//                     stages in flight, one barrier per K step;
//   conv_greg_kernel  any cin / alignment / raw-picture input: tiles are staged
//                     through registers (double-buffered LDS).
#include "conv_common.h"

#include <mutex>
#include <type_traits>
#include <vector>

namespace icnn {

// ------------------------------------------------- direct-to-LDS pipelined kernel
// Tiles travel from global memory into LDS without passing through registers
// (buffer_load_dwordx4 ... lds).  Every lane moves 16 bytes; a wave-wide copy fills
// 1 KiB of consecutive LDS.  Out-of-image pieces (zero padding, the K tail, pixels
// beyond the last one) are given a byte offset beyond the buffer's size: the
// buffer unit returns zeros for those lanes, so padding costs one select.
// MODE 0: 1x1 kernel, stride 1, no padding (input pixel = output pixel);
// MODE 1: cin % 64 == 0 and kh*kw <= 32: a K step lies inside one tap, so the tap
//         position is wave-uniform (scalar registers, one bit test per copy);
// MODE 2: any cin % 16 == 0: every lane tracks the tap of its own 16-byte slot.
// MODE 3: kernel kh x 1 without padding, cin % 16 == 0 (the padded small-cin layout, where "cin" is
//         a kernel row of the picture): every piece lies inside the buffer, so a lane only adds its
//         slot's offset for the K step to the pixel's; nothing to mask but pixels beyond the last.
// PC: requantisation and skip rescale per output channel (epilogue_pc_tiles)
// U8: unsigned inputs up to 255: activation fragments are XORed with 0x80 bytes (x - 128) on their way
//     from LDS to the matrix cores (the bias rows carry the matching correction, see load_bias_rows)
// SPLIT: the K axis of a tile may be cut into ranges that run as separate work units (a.ksplit; instantiated for the
// 128-channel tiles and modes 0 and 1 only: the bookkeeping costs scalar registers the other kernels are short of)
template <int BM, int BP, int WAVES_M, int WAVES_P, int MODE, bool PC, bool U8, bool SPLIT = false>
__global__ __launch_bounds__(256, ((BM / 32) * (BP / 32) > 32 ? 1 : 2)) void conv_dlds_kernel(const ConvArgs a)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr int TM = BM / WAVES_M / 32;
    constexpr int TP = BP / WAVES_P / 32;
    constexpr int A_BYTES = BM * kStepK;
    constexpr int B_BYTES = BP * kStepK;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_INSTR = BM / 16;                 // wave-wide 1 KiB copies per stage, whole workgroup
    constexpr int NA = A_INSTR >= 4 ? A_INSTR / 4 : 1;   // per wave (narrow tiles repeat a copy)
    constexpr int NB = BP / 64;                      // per wave
    constexpr int LPS = NA + NB;                     // loads per stage per wave
    constexpr unsigned OOB = 0x80000000u;            // beyond any buffer this kernel accepts (< 2 GiB)
    static_assert(WAVES_M * WAVES_P == 4 && TM >= 1 && TP >= 1 && NB >= 1, "tile shape");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];   // nstages * STAGE bytes (+ parameter slots; + 16 with SPLIT)

    // Persistent workgroups: this one handles tiles v = blockIdx.x, + gridDim.x, ...  (gridDim.x is a
    // multiple of 8, so all of them map to the same XCD, see tile_of()).
    int vtile = blockIdx.x;
    int ct, pt;
    {
        // XCD x owns the contiguous tile range [x*per_xcd, (x+1)*per_xcd); only its tail can be padding
        const int logical = (vtile & 7) * a.per_xcd + (vtile >> 3);
        if (logical >= a.n_tiles) return;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps LDS targets in scalar registers
    const int wm = wave % WAVES_M;
    const int wp = wave / WAVES_M;
    const int nstages = a.nstages;
    const int ksplit = SPLIT ? a.ksplit : 1;         // K ranges per tile (1: no split); a.n_tiles counts units
    const int ksteps = SPLIT ? a.ksteps / ksplit : a.ksteps;       // K steps of a unit (the host only splits evenly)
    const int depth = min(nstages - 1, ksteps);      // stages of a unit issued ahead of its K loop

    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, a.wp_bytes, 0x00020000);
    // PC: the packed per-channel parameters of a tile's BM channels (PC_BYTES) are copied to LDS at
    // the start of the tile and read from there by the epilogue.  Two slots alternate, so a wave that
    // already started the next tile never overwrites what a slower wave's epilogue still reads (no wave
    // gets two tiles ahead: every K loop has a barrier).
    const __amdgpu_buffer_rsrc_t rs_pc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.pc, 0, PC ? ((a.Cout + 15) >> 4) * kPcGroupInts * 4 : 0, 0x00020000);
    constexpr int PC_BYTES = (BM / 16) * kPcGroupInts * 4;
    constexpr int PC_SLOT = (PC_BYTES + 1023) & ~1023;       // whole wave-wide copies
    uint8_t *const pc_lds = lds + a.nstages * STAGE;
    int pc_slot = 0;
    // split K: one word behind everything else tells the workgroup whether its unit arrived last
    volatile int *const split_flag = (volatile int *)(pc_lds + (PC ? 2 * PC_SLOT : 0));

    // ---- state of the tile whose stages are being issued ("load side")
    // A copy q of this wave covers packed pieces [64*m, 64*m + 64), m = (4*q + wave) % A_INSTR;
    // its byte offset at K step s is a_off[q] + s * 2048
    unsigned a_off[NA];
    int a_lds[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) a_lds[q] = ((4 * q + wave) % A_INSTR) * 1024;
    // B copy j of this wave covers rows 16*(4*j + wave) .. +16 of the tile; this lane fills physical
    // slot lane & 3 of row 16*(4*j + wave) + (lane >> 2), i.e. logical slot ls (same for every j)
    const int ls = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned b_off[NB];      // byte offset of the pixel's first tap (MODE 0, 1: plus the slot's 16*ls)
    unsigned tapmask[NB];    // MODE 1: bit kh*KW + kw set when that tap lies inside the image
    unsigned rowmask[NB];    // MODE 2: bit kh set when the input row of tap kh lies inside the image
    unsigned colmask[NB];    // MODE 2: bit kw likewise for columns
    // K-axis position: MODE 1 wave-uniform (skh, skw, sc0 = first channel of the step);
    // MODE 2 per lane (kh, kw, ci of the lane's slot)
    int skh = 0, skw = 0, sc0 = 0;
    int kh = 0, kw = 0, ci = 0;
    int kh_init = 0, kw_init = 0, ci_init = ls * 16;
    // MODE 3: u = index of the lane's 16-byte piece on the K axis, koff = its byte offset from the pixel's
    // first byte: row u / rp16 of the kernel (rp16 = pieces per kernel row), piece u % rp16 of that row
    const int rp16 = a.Cin >> 4;
    const unsigned rp16_inv = MODE == 3 ? 65535u / (unsigned)rp16 + 1 : 0;   // u / rp16 = u * inv >> 16 for u < 2^16 / rp16
    const unsigned row_bytes = (unsigned)(a.W * a.in_cs);
    auto koff_of = [&](unsigned u) {
        const unsigned row = (u * rp16_inv) >> 16;
        return row * row_bytes + (u - row * (unsigned)rp16) * 16u;
    };
    unsigned ku = 0, koff = 0;
    if (MODE == 2) {
        const int tap = ci_init / a.Cin;
        ci_init -= tap * a.Cin;
        kh_init = tap / a.KW;
        kw_init = tap - kh_init * a.KW;
    }

    int kbase = 0;           // first K step of the unit whose stages are being issued
    auto tile_of = [&](int v, int &ct, int &pt, int &ks) {
        // workgroups are dealt round-robin to the 8 XCDs; XCD x owns units [x*per_xcd, (x+1)*per_xcd): the K ranges
        // of a tile are neighbours there
        const int logical = (v & 7) * a.per_xcd + (v >> 3);
        const int tile = SPLIT ? logical / ksplit : logical;
        ks = SPLIT ? logical - tile * ksplit : 0;
        ct = tile % a.n_ct;
        pt = tile / a.n_ct;
        return logical < a.n_tiles;
    };

    auto setup_load_side = [&](int ct, int pt, int ks) {
        const int pix0 = pt * BP;
        const int chunk0 = ct * (BM / 32);
        kbase = SPLIT ? ks * ksteps : 0;
#pragma unroll
        for (int q = 0; q < NA; ++q) {
            const int e = a_lds[q] / 16 + lane;
            a_off[q] = (unsigned)(chunk0 + (e >> 7)) * (unsigned)a.ksteps * kChunkBytes + (unsigned)(e & 127) * 16;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int p = pix0 + 16 * (4 * j + wave) + (lane >> 2);
            const bool pv = p < a.M;
            tapmask[j] = rowmask[j] = colmask[j] = 0;
            if (MODE == 0) {
                b_off[j] = pv ? (unsigned)p * (unsigned)a.in_cs + ls * 16 : OOB;
            } else if (MODE == 3) {
                const int n = fast_div(p, a.div_howo);
                const int r = p - n * a.Ho * a.Wo;
                const int ho = fast_div(r, a.div_wo);
                const int wo = r - ho * a.Wo;
                // OOB plus any K offset (< 2^31) stays beyond the buffer
                b_off[j] = pv ? (unsigned)(((n * a.H + ho * a.sh) * a.W + wo * a.sw) * a.in_cs) : OOB;
            } else {
                const int pc = pv ? p : 0;
                const int n = fast_div(pc, a.div_howo);
                const int r = pc - n * a.Ho * a.Wo;
                const int ho = fast_div(r, a.div_wo);
                const int wo = r - ho * a.Wo;
                const int hi0 = ho * a.sh - a.ph, wi0 = wo * a.sw - a.pw;
                // may be "negative" (wraps): only used together with a tap that is inside the image
                b_off[j] = (unsigned)(((n * a.H + hi0) * a.W + wi0) * a.in_cs) + (MODE == 1 ? ls * 16 : 0);
                unsigned rm = 0, cm = 0;
                for (int k = 0; k < a.KH; ++k) rm |= (unsigned)((unsigned)(hi0 + k) < (unsigned)a.H) << k;
                for (int k = 0; k < a.KW; ++k) cm |= (unsigned)((unsigned)(wi0 + k) < (unsigned)a.W) << k;
                if (!pv) rm = 0;
                if (MODE == 1) {
                    unsigned tmk = 0;
                    for (int k = 0; k < a.KH; ++k) tmk |= ((rm >> k) & 1u ? cm : 0u) << (k * a.KW);
                    tapmask[j] = tmk;
                } else {
                    rowmask[j] = rm;
                    colmask[j] = cm;
                }
            }
        }
        skh = skw = sc0 = 0;
        if (SPLIT && MODE == 1 && kbase != 0) {       // a later K range starts inside the tap sequence
            const int per_tap = a.Cin / kStepK;
            const int tap = kbase / per_tap;
            sc0 = (kbase - tap * per_tap) * kStepK;
            skh = tap / a.KW;
            skw = tap - skh * a.KW;
        }
        kh = kh_init; kw = kw_init; ci = ci_init;
        if (MODE == 3) { ku = (unsigned)ls; koff = koff_of(ku); }
    };

    // One stage = LPS wave-wide copies.  issue_copy(c, ...) issues copy c (A copies first, then B),
    // advance_k() moves the K-axis position to the next stage; issue_stage() does a whole stage.
    auto issue_copy = [&](int c, int s, uint8_t *stage) {
        if (c < NA) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (__attribute__((address_space(3))) void *)(stage + a_lds[c]),
                                                     16, a_off[c], (kbase + s) * kChunkBytes, 0, 0);
            return;
        }
        const int j = c - NA;
        uint8_t *dst = stage + A_BYTES + (4 * j + wave) * 1024;
        if (MODE == 0) {
            const bool kok = (kbase + s) * kStepK + ls * 16 < a.Cin;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)dst, 16,
                                                     kok ? b_off[j] : OOB, (kbase + s) * kStepK, 0, 0);
        } else if (MODE == 1) {
            const unsigned bit = 1u << (skh * a.KW + skw);
            // added per lane (not as the scalar offset): b_off may have wrapped below zero and the
            // buffer unit range-checks the vector offset alone
            const unsigned soff = (unsigned)((skh * a.W + skw) * a.in_cs + sc0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)dst, 16,
                                                     (tapmask[j] & bit) ? b_off[j] + soff : OOB, 0, 0, 0);
        } else if (MODE == 3) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)dst, 16,
                                                     b_off[j] + koff, 0, 0, 0);
        } else {
            const unsigned tapoff = (unsigned)((kh * a.W + kw) * a.in_cs + ci);
            const bool ok = ((rowmask[j] >> kh) & (colmask[j] >> kw) & 1u) != 0;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)dst, 16,
                                                     ok ? b_off[j] + tapoff : OOB, 0, 0, 0);
        }
    };
    auto advance_k = [&]() {
        if (MODE == 1) {
            sc0 += kStepK;
            if (sc0 == a.Cin) {
                sc0 = 0;
                if (++skw == a.KW) { skw = 0; ++skh; }
            }
        } else if (MODE == 3) {
            ku += 4;
            koff = koff_of(ku);
        } else if (MODE == 2) {
            ci += kStepK;
            while (ci >= a.Cin) {
                ci -= a.Cin;
                if (++kw == a.KW) { kw = 0; ++kh; }
            }
        }
    };
    auto issue_stage = [&](int s, int buf) {
        uint8_t *stage = lds + buf * STAGE;
#pragma unroll
        for (int c = 0; c < LPS; ++c) issue_copy(c, s, stage);
        advance_k();
    };

    // fragment read addresses inside a stage (A: straight; B: swizzled rows, one base per k half)
    const int a_rd = wm * TM * 2048 + lane * 16;
    const int b_rd0 = A_BYTES + b_slot_offset(wp * TP * 32 + (lane & 31), (lane >> 5));
    const int b_rd1 = A_BYTES + b_slot_offset(wp * TP * 32 + (lane & 31), 2 + (lane >> 5));

    // ---- first tile: its leading stages and its bias
    int ks;
    tile_of(vtile, ct, pt, ks);
    setup_load_side(ct, pt, ks);
    int buf = 0;        // ring slot of the next K step to compute
    int ibuf = 0;       // ring slot the next issued stage goes to
    for (int s = 0; s < depth; ++s) {
        issue_stage(s, ibuf);
        if (++ibuf == nstages) ibuf = 0;
    }
    // accumulators start at the bias in a tile's first K range, at zero in the others
    v16i bias_next[TM];
    auto load_unit_bias = [&](int ct_, int ks_) {
        load_bias_rows<TM>(a, ct_ * BM + wm * TM * 32, lane >> 5, bias_next);
        if (SPLIT && ks_ != 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) bias_next[i][r] = 0;
        }
    };
    load_unit_bias(ct, ks);

    for (;;) {
        v16i acc[TM][TP];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = bias_next[i];
        // an 8-bit skip operand travels while the K loop runs
        const int co_wave = ct * BM + wm * TM * 32;
        const int pix_wave = pt * BP + wp * TP * 32;
        const int unit_tile = ct + pt * a.n_ct, unit_ks = ks;
        v4i res8[TM][TP];
        if (!SPLIT || ksplit == 1) prefetch_res8<TM, TP>(a, co_wave, pix_wave, lane, res8);
        if constexpr (PC) {
            pc_slot ^= 1;
#pragma unroll
            for (int c = 0; c * 4096 < PC_SLOT; ++c) {
                const int o = c * 4096 + wave * 1024;
                if (o < PC_SLOT)              // wave-uniform; lanes beyond the tile's parameters and groups beyond cout get zeros
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rs_pc, (__attribute__((address_space(3))) void *)(pc_lds + pc_slot * PC_SLOT + o), 16,
                        o + lane * 16 < PC_BYTES ? (unsigned)(ct * PC_BYTES + o + lane * 16) : OOB, 0, 0, 0);
            }
        }

        // One K step: wait for its stage, barrier, fragments LDS -> registers, MFMAs.  FEED: the
        // copies of stage s + depth are issued between the MFMAs, so the matrix cores work while
        // the wave computes addresses and the memory pipeline accepts them.
        auto k_step = [&](int s, auto feed_tag, auto later_tag, int later) {
            constexpr bool FEED = decltype(feed_tag)::value;
            constexpr int LATER = decltype(later_tag)::value;      // >= 0: known at compile time
            asm volatile("" ::: "memory");
            if constexpr (LATER >= 0) ICNN_WAIT_VMCNT(LATER * LPS);
            else wait_stages_in_flight<LPS>(later);
            // (the previous step's fragment reads have returned: lgkmcnt(0) costs nothing here, but it must hold before the
            // barrier lets other waves refill that step's slot, wherever the compiler put the MFMAs that consumed them)
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();  // every wave's part of stage s is in LDS; the slot of step s-1 is drained
            asm volatile("" ::: "memory");
            uint8_t *istage = lds + ibuf * STAGE;
            const uint8_t *S = lds + buf * STAGE;
            v4i af[2][TM], bf[2][TP];
#pragma unroll
            for (int kq = 0; kq < 2; ++kq) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[kq][i] = *(const v4i *)(S + a_rd + (i * 2 + kq) * 1024);
#pragma unroll
                for (int j = 0; j < TP; ++j) {
                    bf[kq][j] = *(const v4i *)(S + (kq ? b_rd1 : b_rd0) + j * 2048);
                    if constexpr (U8) bf[kq][j] ^= v4i{(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
                }
            }
            // all fragment reads are issued before the first MFMA: left alone, the compiler of a kernel that is
            // short of registers (the per-channel epilogue) reads each fragment just before its MFMA and
            // waits for it there, eight times a step
            __builtin_amdgcn_sched_barrier(0);
            int c = 0;
#pragma unroll
            for (int kq = 0; kq < 2; ++kq)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TP; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[kq][i], bf[kq][j], acc[i][j], 0, 0, 0);
                        if (FEED && c < LPS) {
                            issue_copy(c, s + depth, istage);
                            ++c;
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
            if (FEED) {
#pragma unroll
                for (int cc = 2 * TM * TP; cc < LPS; ++cc) issue_copy(cc, s + depth, istage);   // narrow tiles
                advance_k();
                ibuf = ibuf + 1 == nstages ? 0 : ibuf + 1;
            }
            buf = buf + 1 == nstages ? 0 : buf + 1;
        };
        // steady state: every step feeds the ring and waits with depth - 1 younger stages in flight;
        // the last `depth` steps only drain it
        const int main_steps = ksteps - depth;
        if (depth == 3)
            for (int s = 0; s < main_steps; ++s) k_step(s, std::true_type{}, std::integral_constant<int, 2>{}, 0);
        else if (depth == 2)
            for (int s = 0; s < main_steps; ++s) k_step(s, std::true_type{}, std::integral_constant<int, 1>{}, 0);
        else
            for (int s = 0; s < main_steps; ++s) k_step(s, std::true_type{}, std::integral_constant<int, -1>{}, depth - 1);
        for (int s = main_steps; s < ksteps; ++s)
            k_step(s, std::false_type{}, std::integral_constant<int, -1>{}, ksteps - 1 - s);
        // The last step waited for everything in flight (the skip operands included); saying so
        // here costs nothing and spares the epilogue a wait that would also cover the copies below.
        ICNN_WAIT_VMCNT(0);

        // ---- the next tile's leading stages and bias travel while this tile's epilogue runs.
        // They go to ring slots other than the one of the last K step, which slower waves may
        // still be reading (every wave has passed that step's barrier, so all older slots are free).
        // ---- split K: this unit's accumulators go to the workspace; the unit that arrives last at the tile's counter
        // adds the others' and finishes the tile.  (No spinning anywhere: a unit never waits for another.)  The partial
        // sums travel with system-scope accesses (sc0 sc1: written through to memory, read past the caches), so they
        // are coherent between the chip's L2 caches without any cache-wide write-back or invalidate; a store has reached
        // memory when the wave's counter of outstanding memory operations says so.
        bool finish = true;
        constexpr int UNIT_BYTES = TM * TP * 4 * 256 * 16;                  // a unit's accumulators
        const __amdgpu_buffer_rsrc_t rs_part = __builtin_amdgcn_make_buffer_rsrc((void *)a.ws_part, 0, 0x7ffffff0, 0x00020000);
        mfma_drain(acc);
        if (SPLIT && ksplit > 1) {
            const unsigned mine = (unsigned)(unit_tile * ksplit + unit_ks) * UNIT_BYTES + (wave * (TM * TP * 4 * 64) + lane) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        __builtin_amdgcn_raw_buffer_store_b128(v4i{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]},
                                                               rs_part, mine + ((i * TP + j) * 4 + q) * 1024, 0, 17);
            asm volatile("" ::: "memory");
            ICNN_WAIT_VMCNT(0);
            __syncthreads();                        // every wave's partial sums are in memory
            if (tid == 0) {
                const unsigned arrived = atomicAdd(a.ws_cnt + unit_tile, 1u);
                const bool last = arrived == (unsigned)ksplit - 1;
                if (last) a.ws_cnt[unit_tile] = 0;  // every range has arrived: ready for the next launch
                *split_flag = last ? 1 : 0;
            }
            __syncthreads();
            finish = *split_flag != 0;
        }

        vtile += gridDim.x;
        const bool more = vtile < a.n_vtiles && tile_of(vtile, ct, pt, ks);
        if (more) {
            setup_load_side(ct, pt, ks);
            for (int s = 0; s < depth; ++s) {
                issue_stage(s, ibuf);
                if (++ibuf == nstages) ibuf = 0;
            }
            load_unit_bias(ct, ks);
        }
        if (SPLIT && ksplit > 1 && finish) {
            for (int o = 0; o < ksplit; ++o) {
                if (o == unit_ks) continue;
                const unsigned theirs = (unsigned)(unit_tile * ksplit + o) * UNIT_BYTES + (wave * (TM * TP * 4 * 64) + lane) * 16;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TP; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v4i v = __builtin_amdgcn_raw_buffer_load_b128(rs_part, theirs + ((i * TP + j) * 4 + q) * 1024, 0, 17);
                            acc[i][j][4 * q] += v.x; acc[i][j][4 * q + 1] += v.y; acc[i][j][4 * q + 2] += v.z; acc[i][j][4 * q + 3] += v.w;
                        }
            }
        }
        if (finish) {
            // (with a split K axis the skip operand was not fetched ahead: only one range in ksplit needs it)
            if (SPLIT && ksplit > 1) prefetch_res8<TM, TP>(a, co_wave, pix_wave, lane, res8);
            if constexpr (PC)
                epilogue_pc_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, res8,
                                          (const int32_t *)(pc_lds + pc_slot * PC_SLOT), co_wave - wm * TM * 32);
            else epilogue_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, res8);
        }
        if (!more) break;
        // This tile's stores (and the skip operands of the next) are younger than the stage copies the
        // next K loop waits for.  Loads retire in order among themselves, so a counted wait that leaves
        // n operations in flight still proves every load older than the n youngest has landed: younger
        // operations of any kind make the waits stricter, never unsafe, and no drain is needed here.
    }
#endif
}

// ------------------------------------------------- register-staged general kernel
template <int BM, int BP, int WAVES_M, int WAVES_P, bool VEC, bool PC>
__global__ __launch_bounds__(256) void conv_greg_kernel(const ConvArgs a)
{
    constexpr int TM = BM / WAVES_M / 32;
    constexpr int TP = BP / WAVES_P / 32;
    constexpr int A_BYTES = BM * kStepK;
    constexpr int B_BYTES = BP * kStepK;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int NPA = (BM * 4 + 255) / 256;
    constexpr int NPB = BP * 4 / 256;
    static_assert(WAVES_M * WAVES_P == 4 && TM >= 1 && TP >= 1 && NPB >= 1, "tile shape");

    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE];

    int ct, pt;
    if (!tile_of_block(a, ct, pt)) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WAVES_M;
    const int wp = wave / WAVES_M;
    const int pix0 = pt * BP;
    const int chunk0 = ct * (BM / 32);

    // this thread always fills 16-byte slot `slot` of rows (tid>>2) + 64*j of the B tile
    const int slot = tid & 3;
    int hi0[NPB], wi0[NPB], nrow[NPB];
    bool pv[NPB];
    const int HoWo = a.Ho * a.Wo;
#pragma unroll
    for (int j = 0; j < NPB; ++j) {
        const int p = pix0 + (tid >> 2) + 64 * j;
        pv[j] = p < a.M;
        const int pc = pv[j] ? p : 0;
        const int n = pc / HoWo;
        const int r = pc - n * HoWo;
        const int ho = r / a.Wo;
        const int wo = r - ho * a.Wo;
        hi0[j] = ho * a.sh - a.ph;
        wi0[j] = wo * a.sw - a.pw;
        nrow[j] = n * a.H;
    }
    int kh = 0, kw = 0, ci = 0;
    if (VEC) {
        const int kk = slot * 16;
        const int tap = kk / a.Cin;
        ci = kk - tap * a.Cin;
        kh = tap / a.KW;
        kw = tap - kh * a.KW;
    }

    v4i areg[NPA], breg[NPB];
    bool bok[NPB];

    auto load_tiles = [&](int s) {
#pragma unroll
        for (int i = 0; i < NPA; ++i) {
            const int e = tid + 256 * i;
            if (BM * 4 >= 256 * (i + 1) || e < BM * 4) {
                const size_t off = ((size_t)(chunk0 + (e >> 7)) * a.ksteps + s) * kChunkBytes + (size_t)(e & 127) * 16;
                areg[i] = *(const v4i *)(a.wp + off);
            }
        }
        if (VEC) {
            // branch-free: out-of-image pieces read offset 0 and are zeroed when stored to LDS
#pragma unroll
            for (int j = 0; j < NPB; ++j) {
                const int hi = hi0[j] + kh, wi = wi0[j] + kw;
                const bool ok = pv[j] && kh < a.KH && (unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W;
                const size_t off = ok ? ((size_t)(nrow[j] + hi) * a.W + wi) * a.in_cs + ci : 0;
                breg[j] = *(const v4i_a4 *)(a.x + off);
                bok[j] = ok;
            }
            ci += kStepK;
            while (ci >= a.Cin) {
                ci -= a.Cin;
                if (++kw == a.KW) { kw = 0; ++kh; }
            }
        } else {
            // any cin / pitch: assemble the 16 bytes one by one
            const int kbase = s * kStepK + slot * 16;
#pragma unroll
            for (int j = 0; j < NPB; ++j) {
                uint32_t wd[4] = {0, 0, 0, 0};
                if (pv[j]) {
                    for (int b = 0; b < 16; ++b) {
                        const int kk = kbase + b;
                        if (kk >= a.K) break;
                        const int tap = kk / a.Cin;
                        const int c = kk - tap * a.Cin;
                        const int th = tap / a.KW;
                        const int tw = tap - th * a.KW;
                        const int hi = hi0[j] + th, wi = wi0[j] + tw;
                        if ((unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W) {
                            const size_t off = ((size_t)(nrow[j] + hi) * a.W + wi) * a.in_cs + c;
                            const uint32_t v = (uint32_t)a.x[off] ^ (a.in_xor & 0xffu);
                            wd[b >> 2] |= v << ((b & 3) * 8);
                        }
                    }
                }
                breg[j] = v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
                bok[j] = true;
            }
        }
    };

    auto store_tiles = [&](int buf) {
        uint8_t *A = lds + buf * STAGE;
        uint8_t *B = A + A_BYTES;
#pragma unroll
        for (int i = 0; i < NPA; ++i) {
            const int e = tid + 256 * i;
            if (BM * 4 >= 256 * (i + 1) || e < BM * 4) *(v4i *)(A + e * 16) = areg[i];
        }
#pragma unroll
        for (int j = 0; j < NPB; ++j) {
            v4i v = breg[j];
            if (VEC) {
                const int x = (int)a.in_xor;
                v = bok[j] ? v4i{v.x ^ x, v.y ^ x, v.z ^ x, v.w ^ x} : v4i{0, 0, 0, 0};
            }
            *(v4i *)(B + b_slot_offset((tid >> 2) + 64 * j, slot)) = v;
        }
    };

    v16i acc[TM][TP];
    init_acc_with_bias<TM, TP>(a, ct * BM + wm * TM * 32, lane >> 5, acc);
    const int fxs = (int)a.frag_xor;
    const v4i fx = {fxs, fxs, fxs, fxs};     // x - 128 for unsigned inputs up to 255, else 0

    load_tiles(0);
    store_tiles(0);
    __syncthreads();

    for (int s = 0; s < a.ksteps; ++s) {
        const int buf = s & 1;
        const bool more = s + 1 < a.ksteps;
        if (more) load_tiles(s + 1);

        const uint8_t *A = lds + buf * STAGE;
        const uint8_t *B = A + A_BYTES;
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            v4i af[TM], bf[TP];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *(const v4i *)(A + ((wm * TM + i) * 2 + kq) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < TP; ++j)
                bf[j] = *(const v4i *)(B + b_slot_offset((wp * TP + j) * 32 + (lane & 31), kq * 2 + (lane >> 5))) ^ fx;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_tiles(buf ^ 1);
        __syncthreads();
    }

    mfma_drain(acc);
    if constexpr (PC) {
        v4i res8[TM][TP];
        prefetch_res8<TM, TP>(a, ct * BM + wm * TM * 32, pix0 + wp * TP * 32, lane, res8);
        epilogue_pc_tiles<TM, TP>(a, acc, ct * BM + wm * TM * 32, pix0 + wp * TP * 32, lane, res8,
                                  a.pc + (size_t)(ct * BM >> 4) * kPcGroupInts, ct * BM);
    }
    else epilogue_tiles<TM, TP>(a, acc, ct * BM + wm * TM * 32, pix0 + wp * TP * 32, lane);
}

// ------------------------------------------------------------------ dispatch
// More than 64 KiB of dynamic LDS has to be allowed once per kernel function.
hipError_t allow_large_lds(const void *kernel)
{
    static std::mutex lock;
    static std::vector<const void *> done;
    std::lock_guard<std::mutex> g(lock);
    for (const void *k : done)
        if (k == kernel) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) done.push_back(kernel);
    return e;
}

template <int BM, int BP, int WAVES_M, int WAVES_P>
static hipError_t launch_dlds(const ConvArgs &a0, int max_stages, int per_cu, int ksplit, hipStream_t st)
{
    ConvArgs a = a0;
    if (!finish_args(a, BM, BP)) return hipErrorInvalidValue;
    a.ksplit = ksplit;
    if (ksplit > 1) {                      // units instead of tiles
        if (a.n_tiles > kWsMaxSplitTiles || a.ksteps % ksplit != 0 || !a.ws_cnt || !a.ws_part) return hipErrorInvalidValue;
        a.n_tiles *= ksplit;
        a.per_xcd = (a.n_tiles + 7) / 8;
    }
    if (g_tuning.stages >= 2 && g_tuning.stages <= 6) max_stages = g_tuning.stages;
    const int unit_steps = a.ksteps / ksplit;
    a.nstages = unit_steps + 1 < max_stages ? unit_steps + 1 : max_stages;
    if (a.nstages < 2) a.nstages = 2;
    a.div_howo = make_fast_div((unsigned)(a.Ho * a.Wo));
    a.div_wo = make_fast_div((unsigned)a.Wo);
    // per-channel kernels keep two copies of the tile's packed parameters behind the ring
    const size_t lds_bytes = (size_t)a.nstages * (BM + BP) * kStepK + (a.pc ? 2 * (((BM / 16) * kPcGroupInts * 4 + 1023) & ~1023) : 0) + (ksplit > 1 ? 16 : 0);
    // (the padded copy of a 1x1 small-cin layer is wider than the output: its pixels are not the output's pixels)
    const bool pw = a.KH == 1 && a.KW == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0 && a.Ho == a.H && a.Wo == a.W;
    // kh x 1 kernels whose taps all lie inside the image: no masks (the padded small-cin layout)
    const bool dense = a.KW == 1 && a.ph == 0 && a.pw == 0 && (a.Ho - 1) * a.sh + a.KH <= a.H && (a.Wo - 1) * a.sw + 1 <= a.W &&
                       (long long)(a.K / 16 + 8) * (a.Cin / 16) < 65536;   // the kernel's u / rp16 by multiplication
    const int mode = pw ? 0 : (a.Cin % 64 == 0 && a.KH * a.KW <= 32 ? 1 : (dense ? 3 : 2));
    // persistent workgroups: as many as fit on the chip at once (a multiple of 8, one share per XCD)
    a.n_vtiles = 8 * a.per_xcd;
    const int slots = 256 * per_cu;
    const dim3 grid((unsigned)(a.n_vtiles < slots ? a.n_vtiles : slots)), block(256);
    auto go = [&](auto kernel) -> hipError_t {
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_large_lds((const void *)kernel);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, a);
        return hipGetLastError();
    };
    auto pick = [&](auto pc_tag, auto u8_tag) -> hipError_t {
        constexpr bool PC = decltype(pc_tag)::value;
        constexpr bool U8 = decltype(u8_tag)::value;
        if constexpr (BM == 128) {
            if (ksplit > 1 && mode == 0) return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 0, PC, U8, true>);
            if (ksplit > 1 && mode == 1) return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 1, PC, U8, true>);
        }
        if (ksplit > 1) return hipErrorInvalidValue;          // split_allowed() keeps this from happening
        if (mode == 0) return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 0, PC, U8>);
        if (mode == 1) return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 1, PC, U8>);
        if (mode == 3) return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 3, PC, U8>);
        return go(conv_dlds_kernel<BM, BP, WAVES_M, WAVES_P, 2, PC, U8>);
    };
    if (a.pc) return a.frag_xor ? pick(std::true_type{}, std::true_type{}) : pick(std::true_type{}, std::false_type{});
    return a.frag_xor ? pick(std::false_type{}, std::true_type{}) : pick(std::false_type{}, std::false_type{});
}

template <int BM, int BP, int WAVES_M, int WAVES_P>
static hipError_t launch_greg(const ConvArgs &a0, bool vec_in, hipStream_t st)
{
    ConvArgs a = a0;
    if (!finish_args(a, BM, BP)) return hipErrorInvalidValue;
    const bool pc = a.pc != nullptr;
    const dim3 grid(8u * a.per_xcd), block(256);
    if (vec_in && pc) hipLaunchKernelGGL((conv_greg_kernel<BM, BP, WAVES_M, WAVES_P, true, true>), grid, block, 0, st, a);
    else if (vec_in) hipLaunchKernelGGL((conv_greg_kernel<BM, BP, WAVES_M, WAVES_P, true, false>), grid, block, 0, st, a);
    else if (pc) hipLaunchKernelGGL((conv_greg_kernel<BM, BP, WAVES_M, WAVES_P, false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((conv_greg_kernel<BM, BP, WAVES_M, WAVES_P, false, false>), grid, block, 0, st, a);
    return hipGetLastError();
}

// Tile shapes of the direct-to-LDS kernel: {cout tile, pixel tile, LDS stages, workgroups per CU}
struct TileCfg {
    int bm, bp, stages, per_cu;
};
static const TileCfg kTiles[] = {
    {32, 256, 3, 2}, {64, 128, 4, 2}, {64, 256, 3, 2}, {128, 64, 4, 2}, {128, 128, 4, 2},
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

static hipError_t launch_tile(int t, const ConvArgs &a, int ksplit, hipStream_t st)
{
    switch (t) {
    case 0: return launch_dlds<32, 256, 1, 4>(a, kTiles[0].stages, kTiles[0].per_cu, ksplit, st);
    case 1: return launch_dlds<64, 128, 1, 4>(a, kTiles[1].stages, kTiles[1].per_cu, ksplit, st);
    case 2: return launch_dlds<64, 256, 1, 4>(a, kTiles[2].stages, kTiles[2].per_cu, ksplit, st);
    case 3: return launch_dlds<128, 64, 2, 2>(a, kTiles[3].stages, kTiles[3].per_cu, ksplit, st);
    default: return launch_dlds<128, 128, 2, 2>(a, kTiles[4].stages, kTiles[4].per_cu, ksplit, st);
    }
}

// Estimated cycles of a launch with tile shape c and the K axis cut into ksplit ranges: rounds of resident
// workgroups times the time of one work unit, whose K loop is bound either by the matrix cores or by the
// L2 -> LDS traffic of its tiles (bytes per step = 64 * (bm + bp)).
static double tile_cost(const TileCfg &c, const ConvArgs &a, int ksplit)
{
    const double tiles = (double)((a.Cout + c.bm - 1) / c.bm) * (double)((a.M + c.bp - 1) / c.bp) * ksplit;
    const double slots = 256.0 * c.per_cu;
    const double rounds = (double)(long long)((tiles + slots - 1) / slots);
    const double resident = tiles < slots ? (tiles / 256.0 > 1 ? tiles / 256.0 : 1) : c.per_cu;   // per CU
    const double mfma = (c.bm / 32) * (c.bp / 32) * 2 * 32.0 / 4;          // cycles per step if alone on the CU
    // at ~24 B/clk/CU from L2; gathered activation pieces (taps, padding) cost a little more than the
    // straight weight copies, which decides between transposed shapes (measured on 3x3 layers)
    const bool pointwise = a.KH == 1 && a.KW == 1 && a.sh == 1 && a.sw == 1;
    const double l2 = 64.0 * (c.bm + (pointwise ? 1.0 : 1.1) * c.bp) / 24.0;
    const double step = resident * (mfma > l2 ? mfma : l2) + 150;
    double fixed = 2500 + 1.5 * c.bm * c.bp / 256 * 6;                     // prologue + epilogue
    // partial sums out, their arrival, the counter's round trip, partial sums in: measured 5 to 8 us on layers of
    // 10 us (64 x 7 x 7 x 2048 -> 512: 16.5 us split in two against 10.8 whole; 64 x 14 x 14 x 256 -> 256 3x3 / 2:
    // 23.6 against 12.7), whether the sums travel through memory or stay in L2: a chain of memory latencies at the
    // end of the launch, not bandwidth
    if (ksplit > 1) fixed += 15000;
    return rounds * (a.ksteps / ksplit * step + fixed);
}

// Splits of the K axis the kernel can run for this layer with tile shape c: 128-channel tiles, pointwise and
// 64-channel-aligned layers only (the other addressing modes track taps per lane), even ranges of at least 8 steps, at most one unit per
// compute unit.  Layers with few tiles and a long K loop leave most compute units idle otherwise (a 7 x 7 x
// 512-channel layer at batch 64 has 100 tiles of 128 x 128 for 256 units); whether a split pays is the cost model's
// business (at the workloads' sizes it does not: see tile_cost).
static bool split_allowed(const TileCfg &c, const ConvArgs &a, int s, bool forced)
{
    if (s == 1) return true;
    // (the padded copy of a 1x1 small-cin layer is wider than the output: its pixels are not the output's pixels)
    const bool pw = a.KH == 1 && a.KW == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0 && a.Ho == a.H && a.Wo == a.W;
    if (!(pw || (a.Cin % 64 == 0 && a.KH * a.KW <= 32)) || a.K % kStepK != 0 || a.ksteps % s != 0 || c.bm != 128) return false;
    const long long tiles = (long long)((a.Cout + c.bm - 1) / c.bm) * ((a.M + c.bp - 1) / c.bp);
    if (tiles > kWsMaxSplitTiles) return false;
    return forced ? a.ksteps / s >= 2 : (a.ksteps / s >= 8 && tiles * s <= 256);
}

// Tile shape and K split of the direct-to-LDS kernel for a layer: the cheapest by the cost model, or what the tuning
// overrides ask for.  may_split: the caller brought a workspace.
static void choose_plan(const ConvArgs &a, bool may_split, int &tile, int &ksplit)
{
    tile = -1;
    ksplit = 1;
    double best_cost = 0;
    const int s_lo = !may_split || g_tuning.ksplit == 1 ? 1 : (g_tuning.ksplit > 1 ? g_tuning.ksplit : 1);
    const int s_hi = !may_split || g_tuning.ksplit == 1 ? 1 : (g_tuning.ksplit > 1 ? g_tuning.ksplit : 8);
    for (int t = 0; t < kNumTiles; ++t) {
        if (g_tuning.tile >= 0 && g_tuning.tile < kNumTiles ? t != g_tuning.tile : (kTiles[t].bm / 2 >= a.Cout && t != 0))
            continue;                                                      // forced shape; or more than half the cout tile empty
        for (int s = 1; s <= s_hi; ++s) {
            if (s > 1 && s < s_lo) continue;
            if (!split_allowed(kTiles[t], a, s, g_tuning.ksplit > 1)) continue;
            double c = tile_cost(kTiles[t], a, s);
            if (s > 1 && g_tuning.ksplit > 1) c = 0;                       // a forced split wins wherever it is possible
            if (tile < 0 || c < best_cost) { tile = t; ksplit = s; best_cost = c; }
        }
    }
}

static bool takes_direct(const ConvArgs &a, bool direct_ok)
{
    // the direct-to-LDS kernel addresses x and the packed weights with 32-bit byte offsets
    return direct_ok && a.in_xor == 0 && a.x_bytes < 0x7fffff00u && a.wp_bytes < 0x7fffff00u && a.KH <= 31 && a.KW <= 31;
}

size_t conv_split_bytes(const ConvArgs &a, bool direct_ok)
{
    if (direct_ok && conv_narrow_applies(a) && !g_tuning.no_narrow) return 0;
    if (direct_ok && conv_fc_applies(a) && !g_tuning.no_fc) return 0;
    if (!takes_direct(a, direct_ok)) return 0;
    if (!g_tuning.no_plane && g_tuning.tile < 0 && conv_plane_applies(a)) return 0;
    if (!g_tuning.no_deep && g_tuning.tile < 0 && conv_deep_applies(a)) return 0;
    if (!g_tuning.no_halo && g_tuning.tile < 0 && conv_halo_applies(a)) return 0;
    int t, s;
    choose_plan(a, true, t, s);
    if (s == 1) return 0;
    const size_t tiles = (size_t)((a.Cout + kTiles[t].bm - 1) / kTiles[t].bm) * ((a.M + kTiles[t].bp - 1) / kTiles[t].bp);
    return tiles * s * kTiles[t].bm * kTiles[t].bp * sizeof(int32_t);
}

hipError_t launch_conv(const ConvArgs &a, bool vec_in, bool direct_ok, hipStream_t st)
{
    const bool direct = takes_direct(a, direct_ok);
    // one to four output channels: a lane per pixel and dot products beat tiles that are 7/8 padding
    if (direct_ok && conv_narrow_applies(a) && !g_tuning.no_narrow)
        return launch_conv_narrow(a, st);
    // the classifier: a few pixels, long K
    if (direct_ok && conv_fc_applies(a) && !g_tuning.no_fc) return launch_conv_fc(a, st);
    // few channels on a large picture: two-dimensional tiles, patch and weights resident in LDS
    if (direct && !g_tuning.no_plane && g_tuning.tile < 0 && conv_plane_applies(a)) return launch_conv_plane(a, st);
    // 3x3 / stride 1 / padding 1 with cin % 256 == 0 on few pixels: the waves of a workgroup split the K axis
    if (direct && !g_tuning.no_deep && g_tuning.tile < 0 && conv_deep_applies(a)) return launch_conv_deep(a, st);
    // 3x3 / stride 1 / padding 1 with cin % 64 == 0: the nine taps read one LDS copy of the input
    if (direct && !g_tuning.no_halo && g_tuning.tile < 0 && conv_halo_applies(a)) return launch_conv_halo(a, st);
    if (direct) {
        int tile, ksplit;
        choose_plan(a, a.ws_part != nullptr, tile, ksplit);       // without a workspace the K axis stays whole
        return launch_tile(tile, a, ksplit, st);
    }
    if (a.Cout <= 32) return launch_greg<32, 256, 1, 4>(a, vec_in, st);
    if (a.Cout <= 64) return launch_greg<64, 256, 1, 4>(a, vec_in, st);
    return launch_greg<128, 128, 2, 2>(a, vec_in, st);
}

// One thread per 16-byte piece of the packed weight format.  rp == 0: K index k is
// (kh, kw, ci) in that order.  rp > 0 (small-cin layout): k = kh * rp + kw * 4 + c with
// channels padded to 4 and each kernel row padded to rp bytes; padding weights are 0.
__global__ void prepack_kernel(const int8_t *__restrict__ w, uint8_t *__restrict__ wp, int Cout, int K,
                               int ksteps, long long pieces, int KH, int KW, int Cin, int rp)
{
    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= pieces) return;
    const int l = (int)(e & 63);
    const int kq = (int)((e >> 6) & 1);
    const long long cs = e >> 7;             // chunk * ksteps + step
    const int s = (int)(cs % ksteps);
    const int chunk = (int)(cs / ksteps);
    const int r = l & 31;
    const int co = chunk * 32 + 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
    const int k0 = s * kStepK + kq * 32 + (l >> 5) * 16;
    uint32_t wd[4] = {0, 0, 0, 0};
    if (co < Cout) {
        for (int b = 0; b < 16; ++b) {
            const int k = k0 + b;
            int v = 0;
            if (rp == 0) {
                if (k < K) v = (uint8_t)w[(size_t)co * K + k];
            } else {
                const int kh = k / rp, rem = k - kh * rp;
                const int kw = rem >> 2, c = rem & 3;
                if (kh < KH && kw < KW && c < Cin) v = (uint8_t)w[(((size_t)co * KH + kh) * KW + kw) * Cin + c];
            }
            wd[b >> 2] |= (uint32_t)v << ((b & 3) * 8);
        }
    }
    *(v4i *)(wp + e * 16) = v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
}

// wsum[co] = sum of output channel co's weights (k_true = kh*kw*cin of them), 0 for the padding channels.
// One wave per channel.
__global__ __launch_bounds__(64) void wsum_kernel(const int8_t *__restrict__ w, int32_t *__restrict__ wsum, int Cout,
                                                  int k_true)
{
    const int co = blockIdx.x, lane = threadIdx.x;
    int s = 0;
    if (co < Cout)
        for (int k = lane; k < k_true; k += 64) s += w[(size_t)co * k_true + k];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if (lane == 0) wsum[co] = s;
}

hipError_t launch_wsum(const int8_t *w, int32_t *wsum, int Cout, int cout_padded, int k_true, hipStream_t st)
{
    hipLaunchKernelGGL(wsum_kernel, dim3(cout_padded), dim3(64), 0, st, w, wsum, Cout, k_true);
    return hipGetLastError();
}

hipError_t launch_prepack(const int8_t *w, uint8_t *wp, int Cout, int K, int chunks, int ksteps, int KH, int KW,
                          int Cin, int rp, hipStream_t st)
{
    const long long pieces = (long long)chunks * ksteps * 128;
    const unsigned blocks = (unsigned)((pieces + 255) / 256);
    hipLaunchKernelGGL(prepack_kernel, dim3(blocks), dim3(256), 0, st, w, wp, Cout, K, ksteps, pieces, KH, KW, Cin, rp);
    return hipGetLastError();
}

// Per-channel parameters -> packed groups of 16 channels (layout at kPcGroupInts).  One thread per
// group.  Requantisation of a channel with ratio r = mul / 2^shift as one 32x32 -> 64 bit multiply-add:
//   shift >= 32:             A = mul, C = shift - 32:  hi32(t * mul + 2^(shift-1)) >> (shift - 32), exact
//                            because floor(P / 2^shift) = floor(floor(P / 2^32) / 2^(shift-32));
//   r < 1/2, shift in 1..31: A = mul << (32 - shift) < 2^31:  hi32(t * A + 2^31);
//   r >= 1/2:                outputs saturate once |t| * r >= 257, so t is first clamped to |t| <= T =
//                            ceil(257 / r) + 1 (the final clamp to the 8-bit range hides the difference),
//                            which leaves room to shift it left by L = floor(log2 r) + 2 and use
//                            A = mul << (30 - floor(log2 mul)) < 2^31; ratios of 2^10 and more all behave
//                            like 2^10:  hi32((clamp(t) << L) * A + 2^31).
// The clamp trick needs the 8-bit clamp to follow directly, so a skip operand joined after
// requantisation takes the general form.  Channels beyond cout are neutral.
__global__ __launch_bounds__(64) void pc_prepack_kernel(const int32_t *__restrict__ mul, const int32_t *__restrict__ shift,
                                                        const int32_t *__restrict__ res_mul,
                                                        const int32_t *__restrict__ res_shift, int cout, int groups,
                                                        int32_t *__restrict__ packed)
{
    const int g = blockIdx.x * 64 + threadIdx.x;
    if (g >= groups) return;
    int32_t *o = packed + (size_t)g * kPcGroupInts;
    bool res_fast = true, plain = true;
    for (int r = 0; r < 16; ++r) {
        const int c = g * 16 + r;
        const bool in = c < cout;
        int m = in && mul ? mul[c] : 1, s = in && shift ? shift[c] : 1;
        const int rm = in && res_mul ? res_mul[c] : 1, rs = in && res_shift ? res_shift[c] : 0;
        if (m < 1) m = 1;                       // outside the documented domain: unspecified result, no fault
        s = s < 0 ? 0 : (s > 62 ? 62 : s);
        int A, L = 0, T = 0x7fffffff, C = 0;
        if (s >= 32) {
            A = m;
            C = s - 32;
        } else if (s >= 1 && ((long long)m << (32 - s)) <= 0x7fffffffLL) {
            A = (int)((long long)m << (32 - s));
        } else {
            int mm = m, ss = s;
            if (((long long)mm >> ss) >= 1024) { mm = 1024; ss = 0; }     // r >= 2^10 acts like 2^10
            const int lg = 31 - __clz(mm);
            L = lg - ss + 2;
            A = mm << (30 - lg);
            T = (int)((257LL * (1LL << ss) + mm - 1) / mm) + 1;
        }
        if (in && mul) plain = plain && L == 0 && C == 0;
        if (in && res_mul) res_fast = res_fast && rs >= 0 && rs <= 30 && rm >= 1 && 255LL * rm + ((1LL << rs) >> 1) <= 0x7fffffffLL;
        o[kPcA + r] = A; o[kPcL + r] = L; o[kPcT + r] = T; o[kPcC + r] = C;
        o[kPcMul + r] = m; o[kPcShift + r] = s; o[kPcResMul + r] = rm; o[kPcResShift + r] = rs;
    }
    o[kPcFlags] = (res_fast ? 1 : 0) | (plain ? 2 : 0);
    for (int r = kPcFlags + 1; r < kPcGroupInts; ++r) o[r] = 0;
}

hipError_t launch_pc_prepack(const int32_t *mul, const int32_t *shift, const int32_t *res_mul, const int32_t *res_shift,
                             int cout, int32_t *packed, hipStream_t st)
{
    const int groups = (cout + 15) / 16;
    hipLaunchKernelGGL(pc_prepack_kernel, dim3((groups + 63) / 64), dim3(64), 0, st, mul, shift, res_mul, res_shift, cout,
                       groups, packed);
    return hipGetLastError();
}

// Small-cin layers (cin <= 4: pictures): copies x into a zero-bordered tensor with 4 channels
// per pixel, [n][hp][wp][4] int8, applying the raw picture's "- 128" on the way.  The conv
// then reads 16 contiguous bytes (4 taps x 4 channels) with no bounds checks.
__global__ __launch_bounds__(256) void pad_small_cin_kernel(const uint8_t *__restrict__ x, uint32_t *__restrict__ out,
                                                            long long total, int H, int W, int Cin, int in_cs, int ph,
                                                            int pw, int Hp, int Wp, uint32_t in_xor)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int xp = (int)(e % Wp);
    const long long t = e / Wp;
    const int yp = (int)(t % Hp);
    const long long n = t / Hp;
    const int hi = yp - ph, wi = xp - pw;
    uint32_t v = 0;
    if ((unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W) {
        const uint8_t *p = x + (((size_t)n * H + hi) * W + wi) * in_cs;
        for (int c = 0; c < Cin; ++c) v |= ((uint32_t)p[c] ^ (in_xor & 0xffu)) << (8 * c);
    }
    out[e] = v;
}

// Same copy with the row and the image in the grid's y and z (no per-thread divisions) and four
// pixels per thread (all their byte loads in flight together; the kernel is latency-bound otherwise)
__global__ __launch_bounds__(256) void pad_small_cin_rows_kernel(const uint8_t *__restrict__ x, uint32_t *__restrict__ out,
                                                                 int H, int W, int Cin, int in_cs, int ph, int pw, int Hp,
                                                                 int Wp, uint32_t in_xor)
{
    const int xp0 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (xp0 >= Wp) return;
    const int yp = blockIdx.y, n = blockIdx.z;
    const int hi = yp - ph;
    const bool rowok = (unsigned)hi < (unsigned)H;
    const uint8_t *row = x + ((size_t)n * H + (rowok ? hi : 0)) * W * in_cs;
    const uint32_t m = in_xor & 0xffu;
    uint32_t b[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int wi = xp0 + u - pw;
        const bool ok = rowok && (unsigned)wi < (unsigned)W;
        const uint8_t *p = row + (size_t)(ok ? wi : 0) * in_cs;
#pragma unroll
        for (int c = 0; c < 4; ++c) b[u][c] = (ok && c < Cin) ? ((uint32_t)p[c < Cin ? c : 0] ^ m) : 0u;
    }
    uint32_t *o = out + ((size_t)n * Hp + yp) * Wp + xp0;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (xp0 + u < Wp) o[u] = b[u][0] | (b[u][1] << 8) | (b[u][2] << 16) | (b[u][3] << 24);
}

// Dense three-channel pictures (cin = pitch = 3, W % 4 == 0, 4-byte aligned): a thread turns 12 input
// bytes (three aligned dwords, coalesced across the wave) into four output pixels; byte loads cost
// one address per lane and made the generic kernel address-bound.  Thread W/4 of a row writes the
// left and right border, rows outside the image are all zero.
typedef int v4i_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));
__global__ __launch_bounds__(64) void pad_rgb_rows_kernel(const uint32_t *__restrict__ x, uint32_t *__restrict__ out, int H,
                                                          int W, int ph, int pw, int Hp, int Wp, uint32_t in_xor)
{
    const int t = blockIdx.x * 64 + threadIdx.x;
    const int quads = W >> 2;
    if (t > quads) return;
    const int yp = blockIdx.y, n = blockIdx.z;
    const int hi = yp - ph;
    const bool rowok = (unsigned)hi < (unsigned)H;
    uint32_t *o = out + ((size_t)n * Hp + yp) * Wp;
    if (t == quads) {                               // borders
        for (int c = 0; c < pw; ++c) o[c] = 0;
        for (int c = pw + W; c < Wp; ++c) o[c] = 0;
        return;
    }
    uint32_t d0 = 0, d1 = 0, d2 = 0;
    if (rowok) {
        const uint32_t *p = x + (((size_t)n * H + hi) * W * 3 >> 2) + 3 * t;
        d0 = p[0] ^ in_xor; d1 = p[1] ^ in_xor; d2 = p[2] ^ in_xor;
    }
    // bytes r0 g0 b0 r1 | g1 b1 r2 g2 | b2 r3 g3 b3  ->  one dword per pixel, top byte zero
    const uint32_t m = rowok ? 0x00ffffffu : 0u;
    // one 16-byte store per thread (the left border makes it dword-aligned only)
    *(v4i_dword_aligned *)(o + pw + 4 * t) = v4i_dword_aligned{(int)(d0 & m), (int)(((d0 >> 24) | (d1 << 8)) & m),
                                                               (int)(((d1 >> 16) | (d2 << 16)) & m), (int)((d2 >> 8) & m)};
}

hipError_t launch_pad_small_cin(const uint8_t *x, void *out, int N, int H, int W, int Cin, int in_cs, int ph, int pw,
                                int Hp, int Wp, uint32_t in_xor, hipStream_t st)
{
    if (Cin == 3 && in_cs == 3 && W % 4 == 0 && !((uintptr_t)x & 3) && Wp >= pw + W && N <= 65535 && Hp <= 65535) {
        hipLaunchKernelGGL(pad_rgb_rows_kernel, dim3((unsigned)((W / 4 + 1 + 63) / 64), (unsigned)Hp, (unsigned)N), dim3(64), 0,
                           st, (const uint32_t *)x, (uint32_t *)out, H, W, ph, pw, Hp, Wp, in_xor);
        return hipGetLastError();
    }
    if (N <= 65535 && Hp <= 65535) {
        hipLaunchKernelGGL(pad_small_cin_rows_kernel, dim3((unsigned)((Wp + 1023) / 1024), (unsigned)Hp, (unsigned)N), dim3(256),
                           0, st, x, (uint32_t *)out, H, W, Cin, in_cs, ph, pw, Hp, Wp, in_xor);
        return hipGetLastError();
    }
    const long long total = (long long)N * Hp * Wp;
    hipLaunchKernelGGL(pad_small_cin_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, (uint32_t *)out,
                       total, H, W, Cin, in_cs, ph, pw, Hp, Wp, in_xor);
    return hipGetLastError();
}

}  // namespace icnn
