// Device and host helpers shared by the convolution kernels (tile layout, epilogue,
// bias rows, fast division, counted waits).  Internal; not installed.
#pragma once
#include "icnn_device.h"

#include <type_traits>

namespace icnn {

typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));   // 16-byte load, dword aligned

// LDS tile layout of one K step (both kernels):
//   A (weights): BM*64 bytes in packed-fragment order, i.e. a straight copy of
//      BM/32 consecutive 2 KiB chunks of the packed weights.
//   B (activations): BP rows of 64 bytes (one output pixel each); the 16-byte slot
//      s of row r lives at slot s ^ ((r >> 2) & 3), which makes both the row-wise
//      fill and the column-wise fragment reads free of bank conflicts.
__device__ __forceinline__ int b_slot_offset(int row, int slot)
{
    return row * 64 + ((slot ^ ((row >> 2) & 3)) << 4);
}

// ---------------------------------------------------------------- epilogue
// Every call handles channels co0..co0+15 (co0 a multiple of 16) of output pixel p,
// held in one lane's accumulator registers, which were initialised with the bias
// (so they hold Y = U + b).  Then (Section 4.1)
// the rescaled skip operand, then (Section 3.2.1) requantisation and the clamp.

// any alignment, any tail: one element at a time, 64-bit arithmetic throughout
__device__ __forceinline__ void epilogue_slow(const ConvArgs &a, const v16i &acc, int p, int co0, int nv)
{
    const size_t ro = (size_t)p * a.res_cs + co0;
    const size_t oo = (size_t)p * a.out_cs + a.out_co + co0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (r >= nv) break;
        int64_t t = acc[r];
        int64_t skip = 0;
        if (a.res_mode != 0) skip = rsr64((int64_t)load_elem(a.res, ro + r, a.res_dtype) * a.res_mul, a.res_shift);
        if (a.res_mode == 1) t += skip;
        const int ti = sat32(t);
        if (a.out_mode == 3) {
            ((int32_t *)a.out)[oo + r] = ti;
        } else {
            int64_t q = rsr64((int64_t)ti * a.mul, a.shift);
            if (a.res_mode == 2) q += skip;
            ((uint8_t *)a.out)[oo + r] = (uint8_t)clampi64(q, a.lo, a.hi);
        }
    }
}

// One output: y = accumulator with the bias in it, resraw = its skip operand as loaded (any kind), oo = its element index
// in the output.  quick32 (wave-uniform; the caller checked a.out_mode != raw, a.rq_fast, and a.res_fast where there is a
// skip operand): the same arithmetic in 32 bits.
__device__ __forceinline__ void epilogue_one(const ConvArgs &a, int y, int resraw, size_t oo, bool quick32)
{
    if (quick32) {
        int skip = 0;
        if (a.res_mode != 0) skip = (int)(((uint32_t)resraw * (uint32_t)a.res_mul + (uint32_t)((1 << a.res_shift) >> 1)) >> a.res_shift);
        const int ti = a.res_mode == 1 ? __builtin_elementwise_add_sat(y, skip) : y;
        int q = (int)(((int64_t)ti * a.mul_hi + 0x80000000LL) >> 32);
        if (a.res_mode == 2) q = __builtin_elementwise_add_sat(q, skip);       // the clamp below makes the saturation exact
        ((uint8_t *)a.out)[oo] = (uint8_t)min(max(q, a.lo), a.hi);
        return;
    }
    int64_t t = y;
    int64_t skip = 0;
    if (a.res_mode != 0) skip = rsr64((int64_t)resraw * a.res_mul, a.res_shift);
    if (a.res_mode == 1) t += skip;
    const int ti = sat32(t);
    if (a.out_mode == 3) {
        ((int32_t *)a.out)[oo] = ti;
    } else {
        int64_t q = rsr64((int64_t)ti * a.mul, a.shift);
        if (a.res_mode == 2) q += skip;
        ((uint8_t *)a.out)[oo] = (uint8_t)clampi64(q, a.lo, a.hi);
    }
}

// min(max(x, lo), hi) as one instruction (the compiler only fuses the pair when it can prove lo <= hi);
// at most one of the three operands may live in a scalar register
__device__ __forceinline__ int med3_v0s(int x, int hi_s)
{
    int r;
    asm("v_med3_i32 %0, %1, 0, %2" : "=v"(r) : "v"(x), "s"(hi_s));
    return r;
}
__device__ __forceinline__ int med3_vvs(int x, int lo_v, int hi_s)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo_v), "s"(hi_s));
    return r;
}
// the low bytes of four values as one word (three byte-permutes)
__device__ __forceinline__ int pack_low_bytes(int v0, int v1, int v2, int v3)
{
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)v1, (uint32_t)v0, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)v3, (uint32_t)v2, 0x0c0c0400u);
    return (int)__builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// byte `pos` (1..3) of w = low byte of x >> sh; the other bytes of w are kept
__device__ __forceinline__ void shift_into_byte(int &w, uint32_t x, int sh_v, int pos)
{
    if (pos == 1)
        asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
            : "+v"(w) : "v"(sh_v), "v"(x));
    else if (pos == 2)
        asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
            : "+v"(w) : "v"(sh_v), "v"(x));
    else
        asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
            : "+v"(w) : "v"(sh_v), "v"(x));
}

// Sixteen values t (bias and skip operand already in) -> sixteen requantised, clamped bytes as four words
// (Section 3.2.1).  RQ as in epilogue_vec: 1 one 32x32->64 multiply-add whose high word is the result;
// 2 general 64-bit multiply, add, shift; 3 in 32 bits after clamping t to [0, t_hi] (see ConvArgs::rq24).
template <int RQ>
__device__ __forceinline__ v4i requant16(const ConvArgs &a, const int (&t)[16])
{
    if (RQ == 3) {
        // clamp, multiply-add, then the shift writes its byte of the output word: three instructions per value
        int w[4];
        const int sh_v = a.shift;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t tc = (uint32_t)med3_v0s(t[r], a.t_hi);
            const uint32_t x = __umul24(tc, (uint32_t)a.mul) + (uint32_t)a.rnd;
            if ((r & 3) == 0) w[r >> 2] = (int)(x >> a.shift);
            else shift_into_byte(w[r >> 2], x, sh_v, r & 3);
        }
        return v4i{w[0], w[1], w[2], w[3]};
    }
    int v[16];
    const int lo_v = a.lo;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (RQ == 1) {
            // [t * mul / 2^shift] = high word of t * (mul << (32 - shift)) + 2^31   (1 <= shift <= 32)
            const int q = (int)(((int64_t)t[r] * a.mul_hi + 0x80000000LL) >> 32);
            v[r] = med3_vvs(q, lo_v, a.hi);
        } else {
            v[r] = clampi64(rsr64((int64_t)t[r] * a.mul, a.shift), a.lo, a.hi);
        }
    }
    return v4i{pack_low_bytes(v[0], v[1], v[2], v[3]), pack_low_bytes(v[4], v[5], v[6], v[7]),
               pack_low_bytes(v[8], v[9], v[10], v[11]), pack_low_bytes(v[12], v[13], v[14], v[15])};
}
// the cheapest exact form the layer's parameters allow (wave-uniform choice)
__device__ __forceinline__ v4i requant16_any(const ConvArgs &a, const int (&t)[16])
{
    if (a.rq24) return requant16<3>(a, t);
    if (a.rq_fast) return requant16<1>(a, t);
    return requant16<2>(a, t);
}

// vector path: all 16 channels valid, 16-byte aligned skip operand and output.
// RES: 0 no skip operand; 1 unsigned 8-bit operand joined before requantisation with a rescale
//      that fits 32 bits; 2 anything else (signed or int32 operand, wide multiplier, join after).
// RQ:  0 raw int32 output; 1 requantisation as one 32x32->64 multiply-add whose high
//      word is the result; 2 general 64-bit multiply, add, shift; 3 in 32 bits after clamping
//      t to [0, t_hi] (see ConvArgs::rq24; never with RES 2).
template <int RES, int RQ>
__device__ __forceinline__ void epilogue_vec(const ConvArgs &a, const v16i &acc, int p, int co0, const v4i &res8)
{
    int t[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) t[r] = acc[r];
    int rv[16];
    if (RES != 0) {
        if (RES == 2 && a.res_dtype == 2) {
            const v4i *rp = (const v4i *)((const int32_t *)a.res + ((size_t)p * a.res_cs + co0));
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4i v = rp[q];
                rv[4 * q] = v.x; rv[4 * q + 1] = v.y; rv[4 * q + 2] = v.z; rv[4 * q + 3] = v.w;
            }
        } else {
            const int wd[4] = {res8.x, res8.y, res8.z, res8.w};
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int b8 = (int)(((uint32_t)wd[r >> 2] >> ((r & 3) * 8)) & 0xffu);
                rv[r] = RES == 2 && a.res_dtype == 1 ? (int)(int8_t)b8 : b8;
            }
        }
    }
    if (RES == 1) {
        const int half = (1 << a.res_shift) >> 1;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            // unsigned operand and 255 * res_mul + half < 2^31 (the host's gate), so res_mul < 2^24: an unsigned
            // 24-bit multiply (the signed one would read multipliers from 2^23 on as negative)
            t[r] = __builtin_elementwise_add_sat(t[r], (int)((__umul24((uint32_t)rv[r], (uint32_t)a.res_mul) + (uint32_t)half) >> a.res_shift));
    }
    if (RES == 2 && a.res_mode == 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) t[r] = sat32((int64_t)t[r] + rsr64((int64_t)rv[r] * a.res_mul, a.res_shift));
    }
    const size_t oo = (size_t)p * a.out_cs + a.out_co + co0;
    if (RQ == 0) {
        v4i *op = (v4i *)((int32_t *)a.out + oo);
#pragma unroll
        for (int q = 0; q < 4; ++q) op[q] = v4i{t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]};
        return;
    }
    if (RQ == 3 || (RQ == 1 && RES != 2)) {
        *(v4i *)((uint8_t *)a.out + oo) = requant16<RQ>(a, t);
        return;
    }
    int v[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        int64_t q = RQ == 1 ? (((int64_t)t[r] * a.mul_hi + 0x80000000LL) >> 32) : rsr64((int64_t)t[r] * a.mul, a.shift);
        if (RES == 2 && a.res_mode == 2) q += rsr64((int64_t)rv[r] * a.res_mul, a.res_shift);
        v[r] = clampi64(q, a.lo, a.hi);
    }
    *(v4i *)((uint8_t *)a.out + oo) = v4i{pack_low_bytes(v[0], v[1], v[2], v[3]), pack_low_bytes(v[4], v[5], v[6], v[7]),
                                          pack_low_bytes(v[8], v[9], v[10], v[11]), pack_low_bytes(v[12], v[13], v[14], v[15])};
}

// True when the call's skip operand is 8-bit and the vector epilogue handles it: then the operands of
// a wave's tiles can be fetched ahead of the K loop (prefetch_res8) and handed to epilogue_tiles.
__device__ __forceinline__ bool res8_applies(const ConvArgs &a)
{
    return a.epi_vec && !(a.Cout & 15) && a.res_mode != 0 && a.res_dtype != 2;
}

// ---- per-output-channel parameters (Section 3.4.3: one weight step per output channel leaves
// every channel its own ratio): channel c is requantised with (pc_mul[c], pc_shift[c]) and its
// skip operand rescaled with (pc_res_mul[c], pc_res_shift[c]).
// General form for one pixel's 16 channels (nv of them valid): any parameters, any alignment, any
// tail; 64-bit arithmetic, four channels at a time.  g: the group's packed parameters.
__device__ __forceinline__ void epilogue_pc_slow(const ConvArgs &a, const v16i &acc, int p, int co0, int nv,
                                                 const int32_t *g)
{
    const bool vec = a.epi_vec && nv == 16;
    const size_t ro = (size_t)p * a.res_cs + co0;
    const size_t oo = (size_t)p * a.out_cs + a.out_co + co0;
    const bool requant = a.out_mode != 3;
    uint32_t wd[4] = {0, 0, 0, 0};
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        const v4i mu = *(const v4i *)(g + kPcMul + 4 * q4), sf = *(const v4i *)(g + kPcShift + 4 * q4);
        const v4i rmu = *(const v4i *)(g + kPcResMul + 4 * q4), rsf = *(const v4i *)(g + kPcResShift + 4 * q4);
        int rv[4] = {0, 0, 0, 0};
        if (a.res_mode != 0) {
            if (vec && a.res_dtype == 2) {
                const v4i v = *(const v4i *)((const int32_t *)a.res + ro + 4 * q4);
                rv[0] = v.x; rv[1] = v.y; rv[2] = v.z; rv[3] = v.w;
            } else if (vec) {
                const int w4 = *(const int *)((const uint8_t *)a.res + ro + 4 * q4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int b8 = (w4 >> (8 * e)) & 0xff;
                    rv[e] = a.res_dtype == 1 ? (int)(int8_t)b8 : b8;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * q4 + e < nv) rv[e] = load_elem(a.res, ro + 4 * q4 + e, a.res_dtype);
            }
        }
        int ti[4];
        int qv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int64_t t = acc[4 * q4 + e];
            const int64_t skip = a.res_mode != 0 ? rsr64((int64_t)rv[e] * rmu[e], rsf[e] & 63) : 0;
            if (a.res_mode == 1) t += skip;
            ti[e] = sat32(t);
            int64_t q = rsr64((int64_t)ti[e] * mu[e], sf[e] & 63);
            if (a.res_mode == 2) q += skip;
            qv[e] = clampi64(q, a.lo, a.hi);
            wd[q4] |= (uint32_t)(qv[e] & 0xff) << (8 * e);
        }
        if (!requant) {
            if (vec) {
                *(v4i *)((int32_t *)a.out + oo + 4 * q4) = v4i{ti[0], ti[1], ti[2], ti[3]};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * q4 + e < nv) ((int32_t *)a.out)[oo + 4 * q4 + e] = ti[e];
            }
        } else if (!vec) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * q4 + e < nv) ((uint8_t *)a.out)[oo + 4 * q4 + e] = (uint8_t)qv[e];
        }
    }
    if (requant && vec) *(v4i *)((uint8_t *)a.out + oo) = v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
}

// One row of a wave's tiles (16 channels per lane, TP pixels) in the single-multiply form of
// pc_prepack_kernel.  skip: an 8-bit skip operand joins before requantisation and its rescale fits 32
// bits.  plain: no channel of the wave's groups needs the clamp, the pre-shift or the post-shift.  Both
// are wave-uniform.  Parameters are fetched four channels at a time and used for all TP pixels before
// the next four (registers are scarce here); the arithmetic variants branch inside that loop.
template <int TP>
__device__ __forceinline__ void epilogue_pc_row(const ConvArgs &a, const v16i (&acc)[TP], int co0, int pix_wave, int lane,
                                                const int32_t *g, const v4i (&rw)[TP], bool skip, bool plain)
{
    uint32_t wd[TP][4];
    const int lo_v = a.lo;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        const v4i A = *(const v4i *)(g + kPcA + 4 * q4);
        v4i L = {0, 0, 0, 0}, T = {0, 0, 0, 0}, C = {0, 0, 0, 0}, rmu = {1, 1, 1, 1}, rsf = {0, 0, 0, 0};
        if (!plain) {
            L = *(const v4i *)(g + kPcL + 4 * q4);
            T = *(const v4i *)(g + kPcT + 4 * q4);
            C = *(const v4i *)(g + kPcC + 4 * q4);
        }
        if (skip) { rmu = *(const v4i *)(g + kPcResMul + 4 * q4); rsf = *(const v4i *)(g + kPcResShift + 4 * q4); }
        auto body = [&](auto res_tag, auto plain_tag) {
            constexpr bool RES = decltype(res_tag)::value;
            constexpr bool PLAIN = decltype(plain_tag)::value;
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const uint32_t w4 = (uint32_t)rw[j][q4];
                int v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int t = acc[j][4 * q4 + e];
                    if (RES) {
                        // unsigned operands only (a.pc_fast_ok) and 255 * rmu + half < 2^31 (group flag bit 0): an
                        // unsigned 24-bit multiply whose sum stays below 2^31
                        const uint32_t rv = (w4 >> (8 * e)) & 0xffu;
                        t = __builtin_elementwise_add_sat(t, (int)((__umul24(rv, (uint32_t)rmu[e]) + ((1u << rsf[e]) >> 1)) >> rsf[e]));
                    }
                    int q;
                    if (PLAIN) {
                        q = (int)(((int64_t)t * A[e] + 0x80000000LL) >> 32);
                    } else {
                        const int tc = min(max(t, ~T[e]), T[e]) << L[e];
                        q = (int)(((int64_t)tc * A[e] + ((int64_t)1 << (31 + C[e]))) >> 32) >> C[e];
                    }
                    v[e] = med3_vvs(q, lo_v, a.hi);
                }
                wd[j][q4] = (uint32_t)pack_low_bytes(v[0], v[1], v[2], v[3]);
            }
        };
        if (skip) {
            if (plain) body(std::true_type{}, std::true_type{});
            else body(std::true_type{}, std::false_type{});
        } else {
            if (plain) body(std::false_type{}, std::true_type{});
            else body(std::false_type{}, std::false_type{});
        }
        __builtin_amdgcn_sched_barrier(0);     // keep the four parameter fetches apart
    }
#pragma unroll
    for (int j = 0; j < TP; ++j) {
        const int p = pix_wave + j * 32 + (lane & 31);
        if (p < a.M)
            *(v4i *)((uint8_t *)a.out + ((size_t)p * a.out_cs + a.out_co + co0)) =
                v4i{(int)wd[j][0], (int)wd[j][1], (int)wd[j][2], (int)wd[j][3]};
    }
}

// Epilogue of a wave's tiles with per-channel parameters.  The single-multiply form is used when the
// call allows it (8-bit output, 16-byte accesses, no skip operand or an 8-bit one joined before
// requantisation: a.pc_fast_ok), the lane's 16 channels are all valid and the skip rescale of its group
// fits 32 bits; the decision is taken for the whole wave, so each form is straight-line code.
// res8: the 8-bit skip operands fetched by prefetch_res8 for the same tile when res8_applies(a).
// groups: packed parameters of the channel group that starts at channel co_base (a multiple of 16),
// followed by those of the next groups (global memory or a copy in LDS).
template <int TM, int TP>
__device__ __forceinline__ void epilogue_pc_tiles(const ConvArgs &a, const v16i (&acc)[TM][TP], int co_wave, int pix_wave,
                                                  int lane, const v4i (&res8)[TM][TP], const int32_t *groups, int co_base)
{
    const bool skip = a.res_mode != 0;
    const bool have_res8 = res8_applies(a);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int co0 = co_wave + i * 32 + (lane >> 5) * 16;
        const int nv = min(16, a.Cout - co0);          // <= 0: this half of the wave has no channels here
        const int32_t *g = groups + ((co0 - co_base) >> 4) * kPcGroupInts;
        const int flags = nv > 0 ? g[kPcFlags] : 3;
        const bool fast = nv <= 0 || (a.pc_fast_ok && nv == 16 && (!skip || (flags & 1)));
        const bool wave_fast = __builtin_amdgcn_ballot_w64(!fast) == 0;
        const bool wave_plain = __builtin_amdgcn_ballot_w64(!(flags & 2)) == 0;
        if (!wave_fast) {
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const int p = pix_wave + j * 32 + (lane & 31);
                if (nv > 0 && p < a.M) epilogue_pc_slow(a, acc[i][j], p, co0, nv, g);
            }
            continue;
        }
        if (nv <= 0) continue;
        v4i rw[TP];
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int p = pix_wave + j * 32 + (lane & 31);
            rw[j] = have_res8 ? res8[i][j] : v4i{0, 0, 0, 0};
            if (skip && !have_res8 && p < a.M) rw[j] = *(const v4i *)((const uint8_t *)a.res + ((size_t)p * a.res_cs + co0));
        }
        epilogue_pc_row<TP>(a, acc[i], co0, pix_wave, lane, g, rw, skip, wave_plain);
    }
}
template <int TM, int TP>
__device__ __forceinline__ void prefetch_res8(const ConvArgs &a, int co_wave, int pix_wave, int lane, v4i (&res8)[TM][TP])
{
    if (!res8_applies(a)) return;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int co0 = co_wave + i * 32 + (lane >> 5) * 16;
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int p = pix_wave + j * 32 + (lane & 31);
            if (co0 < a.Cout && p < a.M)
                res8[i][j] = *(const v4i *)((const uint8_t *)a.res + ((size_t)p * a.res_cs + co0));
        }
    }
}
// res8: the 8-bit skip operands fetched by prefetch_res8 for the same tile (ignored otherwise)
template <int TM, int TP>
__device__ __forceinline__ void epilogue_tiles(const ConvArgs &a, const v16i (&acc)[TM][TP], int co_wave, int pix_wave,
                                               int lane, const v4i (&res8)[TM][TP])
{
    const int half = lane >> 5;
    auto for_tiles = [&](auto fn) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int co0 = co_wave + i * 32 + half * 16;
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const int p = pix_wave + j * 32 + (lane & 31);
                if (co0 < a.Cout && p < a.M) fn(acc[i][j], p, co0, i, j);
            }
        }
    };
    // Unaligned tensors take the element-wise path for the whole call, and so do channel tails (cout % 16 != 0)
    // together with a skip operand (prefetch_res8 does not serve them); otherwise only the last, partial group
    // of 16 channels does.
    const bool all_slow = !a.epi_vec || ((a.Cout & 15) && a.res_mode != 0);
    if (!all_slow) {
        switch (a.epi_mode) {
#define ICNN_EPI_CASE(RES, RQ)                                                                      \
    case RES * 4 + RQ:                                                                              \
        for_tiles([&](const v16i &c, int p, int co0, int i, int j) {                                \
            if (co0 + 16 <= a.Cout) epilogue_vec<RES, RQ>(a, c, p, co0, res8[i][j]);                \
        });                                                                                         \
        break;
            ICNN_EPI_CASE(0, 0) ICNN_EPI_CASE(0, 1) ICNN_EPI_CASE(0, 2) ICNN_EPI_CASE(0, 3)
            ICNN_EPI_CASE(1, 0) ICNN_EPI_CASE(1, 1) ICNN_EPI_CASE(1, 2) ICNN_EPI_CASE(1, 3)
            ICNN_EPI_CASE(2, 0) ICNN_EPI_CASE(2, 1) ICNN_EPI_CASE(2, 2)
#undef ICNN_EPI_CASE
        default: break;
        }
    }
    if (all_slow || (a.Cout & 15)) {
        for_tiles([&](const v16i &c, int p, int co0, int, int) {
            if (all_slow || co0 + 16 > a.Cout) epilogue_slow(a, c, p, co0, min(16, a.Cout - co0));
        });
    }
}
// One pixel's 16 channels co0..co0+15 (all valid; the call allows 16-byte accesses: a.epi_vec) in the form the
// host chose (a.epi_mode).  res8: the 8-bit skip operand's 16 bytes, when there is one.
__device__ __forceinline__ void epilogue_px16(const ConvArgs &a, const v16i &acc, int p, int co0, const v4i &res8)
{
    switch (a.epi_mode) {
#define ICNN_EPI_CASE(RES, RQ) case RES * 4 + RQ: epilogue_vec<RES, RQ>(a, acc, p, co0, res8); break;
        ICNN_EPI_CASE(0, 0) ICNN_EPI_CASE(0, 1) ICNN_EPI_CASE(0, 2) ICNN_EPI_CASE(0, 3)
        ICNN_EPI_CASE(1, 0) ICNN_EPI_CASE(1, 1) ICNN_EPI_CASE(1, 2) ICNN_EPI_CASE(1, 3)
        ICNN_EPI_CASE(2, 0) ICNN_EPI_CASE(2, 1) ICNN_EPI_CASE(2, 2)
#undef ICNN_EPI_CASE
    default: break;
    }
}
// The same arithmetic as epilogue_px16 for a layer that stores unsigned bytes and whose skip operand, if any, is
// the unsigned 8-bit kind joined before requantisation (RES 0 or 1, RQ 1, 2 or 3): the sixteen bytes are returned,
// for callers that keep the result on chip as well.
// RQ: 0 the requantisation form is chosen at run time (wave-uniform branch); 1, 2, 3 that form of requant16, for
// callers that need the epilogue to be straight-line code.
template <int RES, int RQ = 0>
__device__ __forceinline__ v4i epilogue_bytes16(const ConvArgs &a, const v16i &acc, const v4i &res8)
{
    int t[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) t[r] = acc[r];
    if (RES == 1) {
        const int wd[4] = {res8.x, res8.y, res8.z, res8.w};
        const int half = (1 << a.res_shift) >> 1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t b8 = ((uint32_t)wd[r >> 2] >> ((r & 3) * 8)) & 0xffu;
            t[r] = __builtin_elementwise_add_sat(t[r], (int)((__umul24(b8, (uint32_t)a.res_mul) + (uint32_t)half) >> a.res_shift));
        }
    }
    if constexpr (RQ == 0) return requant16_any(a, t);
    else return requant16<RQ>(a, t);
}
// Outputs R0 .. R0 + N - 1 of epilogue_bytes16<RES, 3> (the 32-bit requantisation form, a.rq24): their bytes go into
// the words w[R0 / 4 ..], which the caller collects over the sixteen outputs.  For callers that deal the epilogue out
// in slices between matrix instructions.  R0 and N are multiples of... any; a word is started by its output 4 q.
template <int RES, int R0, int N>
__device__ __forceinline__ void epilogue_rq24_slice(const ConvArgs &a, const v16i &acc, const v4i &res8, int (&w)[4])
{
    const int wd[4] = {res8.x, res8.y, res8.z, res8.w};
    const int half = (1 << a.res_shift) >> 1;
    const int sh_v = a.shift;
#pragma unroll
    for (int r = R0; r < R0 + N; ++r) {
        int t = acc[r];
        if (RES == 1) {
            const uint32_t b8 = ((uint32_t)wd[r >> 2] >> ((r & 3) * 8)) & 0xffu;
            t = __builtin_elementwise_add_sat(t, (int)((__umul24(b8, (uint32_t)a.res_mul) + (uint32_t)half) >> a.res_shift));
        }
        const uint32_t tc = (uint32_t)med3_v0s(t, a.t_hi);
        const uint32_t x = __umul24(tc, (uint32_t)a.mul) + (uint32_t)a.rnd;
        if ((r & 3) == 0) w[r >> 2] = (int)(x >> a.shift);
        else shift_into_byte(w[r >> 2], x, sh_v, r & 3);
    }
}
// Between the last v_mfma of an accumulation and the first instruction that reads the accumulator.  The compiler's
// hazard recogniser does not always keep the two apart (seen in a kernel whose epilogue starts two instructions after
// the last MFMA, behind a branch: the reads returned the sums without the last product, now and then), and the
// hardware does not hold the reader back.  Twenty wait states, what a 16-pass matrix instruction needs; the empty
// statements before and after tie every accumulator tile to the wait, so neither an MFMA nor a reader can cross it.
#ifdef ICNN_NO_DRAIN            // measurement only: what the wait states and the register pinning cost
#define ICNN_DRAIN_NOPS ""
#else
#define ICNN_DRAIN_NOPS "s_nop 15\n\ts_nop 3"
#endif
__device__ __forceinline__ void mfma_drain(v16i &acc)
{
    asm volatile(ICNN_DRAIN_NOPS : "+v"(acc));
}
template <int N>
__device__ __forceinline__ void mfma_drain(v16i (&acc)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(acc[i]));
    asm volatile(ICNN_DRAIN_NOPS);
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(acc[i]));
}
template <int M, int N>
__device__ __forceinline__ void mfma_drain(v16i (&acc)[M][N])
{
#pragma unroll
    for (int i = 0; i < M; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) asm volatile("" : "+v"(acc[i][j]));
    asm volatile(ICNN_DRAIN_NOPS);
#pragma unroll
    for (int i = 0; i < M; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) asm volatile("" : "+v"(acc[i][j]));
}

// fn(integral_constant<int, 0>) ... fn(integral_constant<int, N - 1>): a loop the compiler cannot leave rolled
// (register arrays indexed inside it stay in registers)
template <int N, class F>
__device__ __forceinline__ void static_for(F &&fn)
{
    if constexpr (N > 0) {
        static_for<N - 1>(fn);
        fn(std::integral_constant<int, N - 1>{});
    }
}

// sixteen consecutive int32 of the bias table in LDS
__device__ __forceinline__ v16i bias16(const int32_t *tab)
{
    const v4i *bp = (const v4i *)tab;
    v16i b;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const v4i v = bp[q];
        b[4 * q] = v.x; b[4 * q + 1] = v.y; b[4 * q + 2] = v.z; b[4 * q + 3] = v.w;
    }
    return b;
}

// for callers without a K loop to hide the fetch behind: fetch, then finish
template <int TM, int TP>
__device__ __forceinline__ void epilogue_tiles(const ConvArgs &a, const v16i (&acc)[TM][TP], int co_wave, int pix_wave,
                                               int lane)
{
    v4i res8[TM][TP];
    prefetch_res8<TM, TP>(a, co_wave, pix_wave, lane, res8);
    epilogue_tiles<TM, TP>(a, acc, co_wave, pix_wave, lane, res8);
}
// Maps the hardware workgroup id to a tile.  Workgroups are dealt round-robin to the
// 8 XCDs (each with its own L2); giving XCD x the contiguous tile range
// [x*per_xcd, (x+1)*per_xcd) keeps the cout tiles of one pixel tile, and neighbouring
// pixel tiles (shared halo rows), in one L2.  Returns false for padding workgroups.
__device__ __forceinline__ bool tile_of_block(const ConvArgs &a, int &ct, int &pt)
{
    const int xcd = blockIdx.x & 7;
    const int idx = blockIdx.x >> 3;
    const int logical = xcd * a.per_xcd + idx;
    if (logical >= a.n_tiles) return false;
    ct = logical % a.n_ct;
    pt = logical / a.n_ct;
    return true;
}

// Bias of the channels a lane owns: register r of a lane in half h of tile row i holds
// channel co_base + 32*i + 16*h + r.  Accumulators start at these values.
template <int TM>
__device__ __forceinline__ void load_bias_rows(const ConvArgs &a, int co_base, int half, v16i (&b)[TM])
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int co0 = co_base + i * 32 + half * 16;
        if (a.vec_bias) {
            const v4i *bp = (const v4i *)(a.bias + max(0, min(co0, a.Cout - 16)));
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4i v = bp[q];
                b[i][4 * q] = v.x; b[i][4 * q + 1] = v.y; b[i][4 * q + 2] = v.z; b[i][4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) b[i][r] = a.bias[min(co0 + r, a.Cout - 1)];
        }
        if (a.frag_xor) {
            // unsigned inputs up to 255: the matrix cores see x - 128, so 128 * (sum of the channel's
            // weights) is due (wsum is padded to whole 32-channel chunks and 16-byte aligned)
            const v4i *wp = (const v4i *)(a.wsum + co0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4i v = wp[q];
                b[i][4 * q] += 128 * v.x; b[i][4 * q + 1] += 128 * v.y; b[i][4 * q + 2] += 128 * v.z; b[i][4 * q + 3] += 128 * v.w;
            }
        }
    }
}

template <int TM, int TP>
__device__ __forceinline__ void init_acc_with_bias(const ConvArgs &a, int co_base, int half, v16i (&acc)[TM][TP])
{
    v16i b[TM];
    load_bias_rows<TM>(a, co_base, half, b);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j) acc[i][j] = b[i];
}

#define ICNN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | 0x0F70 | (((n) >> 4) << 14))

// Waits until at most `later` stages' worth of this wave's copies (LPS each) are still in
// flight; the count is an immediate of s_waitcnt (6 bits), hence the switch.
template <int LPS>
__device__ __forceinline__ void wait_stages_in_flight(int later)
{
    constexpr int kMax = 63 / LPS < 7 ? 63 / LPS : 7;
    if (later > kMax) later = kMax;
    switch (later) {
    case 0: ICNN_WAIT_VMCNT(0); break;
    case 1: ICNN_WAIT_VMCNT(LPS); break;
    case 2: ICNN_WAIT_VMCNT(2 * LPS <= 63 ? 2 * LPS : 63); break;
    case 3: ICNN_WAIT_VMCNT(3 * LPS <= 63 ? 3 * LPS : 63); break;
    case 4: ICNN_WAIT_VMCNT(4 * LPS <= 63 ? 4 * LPS : 63); break;
    case 5: ICNN_WAIT_VMCNT(5 * LPS <= 63 ? 5 * LPS : 63); break;
    case 6: ICNN_WAIT_VMCNT(6 * LPS <= 63 ? 6 * LPS : 63); break;
    default: ICNN_WAIT_VMCNT(7 * LPS <= 63 ? 7 * LPS : 63); break;
    }
}

// floor(n / d) for 0 <= n < 2^31 by multiply-high and shifts (Granlund & Montgomery's
// round-up method); the host fills `FastDiv` for d.
__device__ __forceinline__ int fast_div(int n, const FastDiv &d)
{
    const unsigned t = __umulhi((unsigned)n, d.mul);
    return (int)((t + (((unsigned)n - t) >> d.s1)) >> d.s2);
}

static inline bool finish_args(ConvArgs &a, int BM, int BP)
{
    a.n_ct = (a.Cout + BM - 1) / BM;
    const long long tiles = (long long)a.n_ct * ((a.M + BP - 1) / BP);
    if (tiles <= 0 || tiles > 0x7ffffff0LL) return false;
    a.n_tiles = (int)tiles;
    a.per_xcd = (int)((tiles + 7) / 8);
    return true;
}

static inline FastDiv make_fast_div(unsigned d)
{
    // l = ceil(log2 d); mul = floor(2^32 * (2^l - d) / d) + 1; q = (t + ((n - t) >> min(l,1))) >> max(l-1,0)
    FastDiv f;
    unsigned l = 0;
    while ((1ull << l) < d) ++l;
    f.mul = (unsigned)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 1 ? l - 1 : 0;
    return f;
}


}  // namespace icnn
