// Residual block with a projection skip as ONE kernel (Section 4.1, "type 2": the skip
// path convolves the quantised block input, its result is rescaled to the main path's ratio
// and added before BReLU).  Both convolutions are 1x1 (any stride, no padding) and share the
// output pixel grid and channel count, so they are two GEMMs into one accumulator tile:
//
//   phase P:  acc  = b_proj + Xp (*) Wp                       (int32, registers)
//   between:  acc  = [acc * res_mul / 2^res_shift] + b_main   (64-bit multiply, registers)
//   phase M:  acc += Xm (*) Wm
//   epilogue: V = clamp([acc * mul / 2^shift], lo, hi)
//
// which equals sat32(Y_main + [Y_proj * res_mul / 2^res_shift]) exactly whenever that sum
// cannot leave int32; the host proves this from the layer sizes and the bias contract before
// launching (otherwise the caller runs the two layers separately).  The int32 projection tensor
// never exists in memory.  Tile machinery as in conv_dlds_kernel (pointwise addressing).
// PC: res_mul / res_shift and mul / shift per output channel (packed parameters, copied to LDS one
// tile ahead so that they are in place from the first barrier of the tile's K loop on).
#include "conv_common.h"

#include <type_traits>

namespace icnn {

template <int BM, int BP, int WAVES_M, int WAVES_P, bool PC>
__global__ __launch_bounds__(256, 2) void conv_dual_kernel(const ConvArgs a, const ProjArgs q)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    constexpr int TM = BM / WAVES_M / 32;
    constexpr int TP = BP / WAVES_P / 32;
    constexpr int A_BYTES = BM * kStepK;
    constexpr int B_BYTES = BP * kStepK;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_INSTR = BM / 16;
    constexpr int NA = A_INSTR >= 4 ? A_INSTR / 4 : 1;
    constexpr int NB = BP / 64;
    constexpr int LPS = NA + NB;
    constexpr unsigned OOB = 0x80000000u;
    static_assert(WAVES_M * WAVES_P == 4 && TM >= 1 && TP >= 1 && NB >= 1 && LPS <= 2 * TM * TP, "tile shape");

    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    int vtile = blockIdx.x;
    int ct, pt;
    {
        const int logical = (vtile & 7) * a.per_xcd + (vtile >> 3);
        if (logical >= a.n_tiles) return;
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform
    const int wm = wave % WAVES_M;
    const int wp = wave / WAVES_M;
    const int nstages = a.nstages;
    const int kp = q.ksteps, km = a.ksteps;
    const int ksteps = kp + km;                       // projection steps first, then the main path
    const int depth = min(nstages - 1, ksteps);

    const __amdgpu_buffer_rsrc_t rs_xm = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wm = __builtin_amdgcn_make_buffer_rsrc((void *)a.wp, 0, a.wp_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_xp = __builtin_amdgcn_make_buffer_rsrc((void *)q.x, 0, q.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wp = __builtin_amdgcn_make_buffer_rsrc((void *)q.wp, 0, q.wp_bytes, 0x00020000);

    unsigned a_off_m[NA], a_off_p[NA];
    int a_lds[NA];
#pragma unroll
    for (int c = 0; c < NA; ++c) a_lds[c] = ((4 * c + wave) % A_INSTR) * 1024;
    const int ls = (lane & 3) ^ ((lane >> 4) & 3);
    unsigned b_off_m[NB], b_off_p[NB];

    auto tile_of = [&](int v, int &ct_, int &pt_) {
        const int logical = (v & 7) * a.per_xcd + (v >> 3);
        ct_ = logical % a.n_ct;
        pt_ = logical / a.n_ct;
        return logical < a.n_tiles;
    };
    auto setup_load_side = [&](int ct_, int pt_) {
        const int pix0 = pt_ * BP;
        const int chunk0 = ct_ * (BM / 32);
#pragma unroll
        for (int c = 0; c < NA; ++c) {
            const int e = a_lds[c] / 16 + lane;
            const unsigned piece = (unsigned)(e & 127) * 16;
            a_off_m[c] = (unsigned)(chunk0 + (e >> 7)) * (unsigned)km * kChunkBytes + piece;
            a_off_p[c] = (unsigned)(chunk0 + (e >> 7)) * (unsigned)kp * kChunkBytes + piece;
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int p = pix0 + 16 * (4 * j + wave) + (lane >> 2);
            const bool pv = p < a.M;
            const int pc = pv ? p : 0;
            const int n = fast_div(pc, a.div_howo);
            const int r = pc - n * a.Ho * a.Wo;
            const int ho = fast_div(r, a.div_wo);
            const int wo = r - ho * a.Wo;
            b_off_m[j] = pv ? (unsigned)(((n * a.H + ho * a.sh) * a.W + wo * a.sw) * a.in_cs) + ls * 16 : OOB;
            b_off_p[j] = pv ? (unsigned)(((n * q.H + ho * q.sh) * q.W + wo * q.sw) * q.in_cs) + ls * 16 : OOB;
        }
    };
    auto issue_copy = [&](int c, int s, uint8_t *stage) {
        const bool proj = s < kp;
        const int sl = proj ? s : s - kp;
        if (c < NA) {
            if (proj)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wp, (__attribute__((address_space(3))) void *)(stage + a_lds[c]),
                                                         16, a_off_p[c], sl * kChunkBytes, 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wm, (__attribute__((address_space(3))) void *)(stage + a_lds[c]),
                                                         16, a_off_m[c], sl * kChunkBytes, 0, 0);
            return;
        }
        const int j = c - NA;
        uint8_t *dst = stage + A_BYTES + (4 * j + wave) * 1024;
        const bool kok = sl * kStepK + ls * 16 < (proj ? q.Cin : a.Cin);
        if (proj)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_xp, (__attribute__((address_space(3))) void *)dst, 16,
                                                     kok ? b_off_p[j] : OOB, sl * kStepK, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_xm, (__attribute__((address_space(3))) void *)dst, 16,
                                                     kok ? b_off_m[j] : OOB, sl * kStepK, 0, 0);
    };

    const int a_rd = wm * TM * 2048 + lane * 16;
    const int b_rd0 = A_BYTES + b_slot_offset(wp * TP * 32 + (lane & 31), (lane >> 5));
    const int b_rd1 = A_BYTES + b_slot_offset(wp * TP * 32 + (lane & 31), 2 + (lane >> 5));

    // PC: two LDS slots behind the ring take the packed parameters of the current and the next tile
    constexpr int PC_BYTES = (BM / 16) * kPcGroupInts * 4;
    constexpr int PC_SLOT = (PC_BYTES + 1023) & ~1023;
    const __amdgpu_buffer_rsrc_t rs_pc =
        __builtin_amdgcn_make_buffer_rsrc((void *)a.pc, 0, PC ? ((a.Cout + 15) >> 4) * kPcGroupInts * 4 : 0, 0x00020000);
    uint8_t *const pc_lds = lds + nstages * STAGE;
    int pc_slot = 0;
    auto issue_params = [&](int ct_, int slot) {
#pragma unroll
        for (int c = 0; c * 4096 < PC_SLOT; ++c) {
            const int o = c * 4096 + wave * 1024;
            if (o < PC_SLOT)          // wave-uniform; lanes beyond the tile's parameters and groups beyond cout get zeros
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rs_pc, (__attribute__((address_space(3))) void *)(pc_lds + slot * PC_SLOT + o), 16,
                    o + lane * 16 < PC_BYTES ? (unsigned)(ct_ * PC_BYTES + o + lane * 16) : OOB, 0, 0, 0);
        }
    };

    tile_of(vtile, ct, pt);
    setup_load_side(ct, pt);
    if constexpr (PC) issue_params(ct, pc_slot);    // older than every stage copy: landed by the first counted wait
    int buf = 0, ibuf = 0;
    for (int s = 0; s < depth; ++s) {
#pragma unroll
        for (int c = 0; c < LPS; ++c) issue_copy(c, s, lds + ibuf * STAGE);
        if (++ibuf == nstages) ibuf = 0;
    }
    ConvArgs pb = a;            // only .bias / .Cout / .vec_bias are read by load_bias_rows
    pb.bias = q.bias;
    pb.vec_bias = q.vec_bias;
    v16i bias_next[TM];
    load_bias_rows<TM>(pb, ct * BM + wm * TM * 32, lane >> 5, bias_next);

    for (;;) {
        v16i acc[TM][TP];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j) acc[i][j] = bias_next[i];
        v16i bias_main[TM];     // older than every copy issued below, so the counted waits stay valid
        load_bias_rows<TM>(a, ct * BM + wm * TM * 32, lane >> 5, bias_main);

        // One K step (see conv_dlds_kernel): FEED steps issue the copies of stage s + depth between
        // their MFMAs and wait with a compile-time count; the last `depth` steps only drain the ring.
        auto k_step = [&](int s, auto feed_tag, auto later_tag, int later) {
            constexpr bool FEED = decltype(feed_tag)::value;
            constexpr int LATER = decltype(later_tag)::value;
            asm volatile("" ::: "memory");
            if constexpr (LATER >= 0) ICNN_WAIT_VMCNT(LATER * LPS);
            else wait_stages_in_flight<LPS>(later);
            // (the previous step's fragment reads have returned: lgkmcnt(0) costs nothing here, but it must hold before the
            // barrier lets other waves refill that step's slot, wherever the compiler put the MFMAs that consumed them)
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            uint8_t *istage = lds + ibuf * STAGE;
            const uint8_t *S = lds + buf * STAGE;
            v4i af[2][TM], bf[2][TP];
#pragma unroll
            for (int kq = 0; kq < 2; ++kq) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[kq][i] = *(const v4i *)(S + a_rd + (i * 2 + kq) * 1024);
#pragma unroll
                for (int j = 0; j < TP; ++j) bf[kq][j] = *(const v4i *)(S + (kq ? b_rd1 : b_rd0) + j * 2048);
            }
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
            if (FEED) ibuf = ibuf + 1 == nstages ? 0 : ibuf + 1;
            buf = buf + 1 == nstages ? 0 : buf + 1;
            if (s == kp - 1) {
                // the projection sum is complete: bring it to the main path's ratio, add the main bias
                mfma_drain(acc);
                if constexpr (PC) {
                    // every wave's parameter copy landed before this step's barrier (see issue_params)
                    const int32_t *groups = (const int32_t *)(pc_lds + pc_slot * PC_SLOT);
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int32_t *g = groups + (wm * TM * 2 + i * 2 + (lane >> 5)) * kPcGroupInts;
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const v4i rmu = *(const v4i *)(g + kPcResMul + 4 * q4), rsf = *(const v4i *)(g + kPcResShift + 4 * q4);
#pragma unroll
                            for (int j = 0; j < TP; ++j)
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const int r = 4 * q4 + e;
                                    acc[i][j][r] = (int)rsr64((int64_t)acc[i][j][r] * rmu[e], rsf[e] & 63) + bias_main[i][r];
                                }
                        }
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TP; ++j)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                acc[i][j][r] = (int)rsr64((int64_t)acc[i][j][r] * q.res_mul, q.res_shift) + bias_main[i][r];
                }
            }
        };
        const int main_steps = ksteps - depth;
        if (depth == 3)
            for (int s = 0; s < main_steps; ++s) k_step(s, std::true_type{}, std::integral_constant<int, 2>{}, 0);
        else
            for (int s = 0; s < main_steps; ++s) k_step(s, std::true_type{}, std::integral_constant<int, -1>{}, depth - 1);
        for (int s = main_steps; s < ksteps; ++s)
            k_step(s, std::false_type{}, std::integral_constant<int, -1>{}, ksteps - 1 - s);

        const int co_wave = ct * BM + wm * TM * 32;
        const int pix_wave = pt * BP + wp * TP * 32;
        vtile += gridDim.x;
        const bool more = vtile < a.n_vtiles && tile_of(vtile, ct, pt);
        if (more) {
            setup_load_side(ct, pt);
            // the other slot: no wave reads it any more (all have passed this tile's barriers)
            if constexpr (PC) issue_params(ct, pc_slot ^ 1);
            for (int s = 0; s < depth; ++s) {
#pragma unroll
                for (int c = 0; c < LPS; ++c) issue_copy(c, s, lds + ibuf * STAGE);
                if (++ibuf == nstages) ibuf = 0;
            }
            load_bias_rows<TM>(pb, ct * BM + wm * TM * 32, lane >> 5, bias_next);
        }
        mfma_drain(acc);
        if constexpr (PC) {
            v4i no_res[TM][TP];     // the main layer's descriptor carries no skip operand here
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j) no_res[i][j] = v4i{0, 0, 0, 0};
            epilogue_pc_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, no_res, (const int32_t *)(pc_lds + pc_slot * PC_SLOT),
                                      co_wave - wm * TM * 32);
            pc_slot ^= 1;
        } else {
            epilogue_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane);
        }
        if (!more) break;
        // no drain: the stores are younger than the copies the next K loop waits for, and a counted
        // wait only gets stricter with younger operations in flight
    }
#endif
}

template <int BM, int BP, int WAVES_M, int WAVES_P, bool PC>
static hipError_t launch_dual_cfg(const ConvArgs &a0, const ProjArgs &q, hipStream_t st)
{
    ConvArgs a = a0;
    if (!finish_args(a, BM, BP)) return hipErrorInvalidValue;
    const int ksteps = a.ksteps + q.ksteps;
    const int max_stages = 4;
    a.nstages = ksteps + 1 < max_stages ? ksteps + 1 : max_stages;
    if (a.nstages < 2) a.nstages = 2;
    a.div_howo = make_fast_div((unsigned)(a.Ho * a.Wo));
    a.div_wo = make_fast_div((unsigned)a.Wo);
    const size_t lds_bytes = (size_t)a.nstages * (BM + BP) * kStepK + (PC ? 2 * (((BM / 16) * kPcGroupInts * 4 + 1023) & ~1023) : 0);
    a.n_vtiles = 8 * a.per_xcd;
    const int slots = 256 * 2;
    const dim3 grid((unsigned)(a.n_vtiles < slots ? a.n_vtiles : slots)), block(256);
    if (lds_bytes > 64 * 1024) {
        static bool raised = false;                      // once per kernel: allow > 64 KiB dynamic LDS
        if (!raised) {
            const hipError_t e = hipFuncSetAttribute((const void *)conv_dual_kernel<BM, BP, WAVES_M, WAVES_P, PC>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL((conv_dual_kernel<BM, BP, WAVES_M, WAVES_P, PC>), grid, block, lds_bytes, st, a, q);
    return hipGetLastError();
}

hipError_t launch_conv_dual(const ConvArgs &a, const ProjArgs &q, hipStream_t st)
{
    // narrow pixel tiles when the wide ones would leave most CUs without work
    const long long wide = (long long)((a.Cout + 127) / 128) * ((a.M + 127) / 128);
    if (a.pc) {
        if (wide >= 256) return launch_dual_cfg<128, 128, 2, 2, true>(a, q, st);
        return launch_dual_cfg<128, 64, 2, 2, true>(a, q, st);
    }
    if (wide >= 256) return launch_dual_cfg<128, 128, 2, 2, false>(a, q, st);
    return launch_dual_cfg<128, 64, 2, 2, false>(a, q, st);
}

}  // namespace icnn
