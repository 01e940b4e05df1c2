// Bandwidth-bound integer kernels: rescaled feature-map addition (Sections 3.4.2
// and 4.1), explicit concatenation with per-branch requantisation (Algorithm 2,
// online half), pooling, and the raw-picture re-normalisation (Section 3.4.1).
// Vector paths move 16 elements per lane (one 128-bit access per 8-bit operand).  The streaming kernels (every
// byte touched once) use non-temporal accesses and one group per lane in a grid that covers the tensor: on a 1 GiB
// copy that shape measured 6.5 TB/s against 6.2 with cached accesses, 5.7 with four groups per lane and 4.3 for a
// persistent grid-stride loop.
#include "icnn_device.h"

namespace icnn {

__device__ __forceinline__ void unpack16(const void *p, size_t i, int dtype, int v[16])
{
    if (dtype == 2) {
        const v4i *q = (const v4i *)((const int32_t *)p + i);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const v4i t = __builtin_nontemporal_load(q + k);
            v[4 * k] = t.x; v[4 * k + 1] = t.y; v[4 * k + 2] = t.z; v[4 * k + 3] = t.w;
        }
    } else {
        const v4i t = __builtin_nontemporal_load((const v4i *)((const uint8_t *)p + i));
        const int wd[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int b8 = (wd[r >> 2] >> ((r & 3) * 8)) & 0xff;
            v[r] = dtype == 1 ? (int)(int8_t)b8 : b8;
        }
    }
}

__device__ __forceinline__ v4i pack16(const int v[16])
{
    uint32_t wd[4] = {0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 16; ++r) wd[r >> 2] |= (uint32_t)(v[r] & 0xff) << ((r & 3) * 8);
    return v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
}

__device__ __forceinline__ int add_one(int av, int bv, const AddArgs &a, bool raw)
{
    const int t = sat32((int64_t)av + rsr64((int64_t)bv * a.b_mul, a.b_shift));
    if (raw) return t;
    return clampi64(rsr64((int64_t)t * a.mul, a.shift), a.lo, a.hi);
}

// vector path: one lane = 16 consecutive channels of one pixel.
// FAST: b is 8 bits wide with a rescale that fits 32 bits and b_mul < 2^23 (a signed 24-bit multiply), and the output requantisation is one
// 32x32->64 multiply-add whose high word is the result (same identities as the conv epilogue).
template <bool FAST>
__global__ __launch_bounds__(256) void add_rescale_vec_kernel(const AddArgs a, int groups_per_px, long long total)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    size_t ao, bo, oo;
    if (groups_per_px == 0) {
        // all three tensors are dense: no pixel / channel split needed
        ao = bo = oo = (size_t)g * 16;
    } else {
        long long px;
        if (total < 0x7fffffffLL) px = (unsigned)g / (unsigned)groups_per_px;
        else px = g / groups_per_px;
        const int c0 = (int)(g - px * groups_per_px) * 16;
        ao = (size_t)px * a.a_cs + c0;
        bo = (size_t)px * a.b_cs + c0;
        oo = (size_t)px * a.out_cs + a.out_co + c0;
    }
    int av[16], bv[16], ov[16];
    unpack16(a.a, ao, a.a_dt, av);
    unpack16(a.b, bo, a.b_dt, bv);
    const bool raw = a.out_mode == 3;
    if (FAST) {
        const int half = (1 << a.b_shift) >> 1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = __builtin_elementwise_add_sat(av[r], (__mul24(bv[r], a.b_mul) + half) >> a.b_shift);
            const int q = (int)(((int64_t)t * a.mul_hi + 0x80000000LL) >> 32);
            ov[r] = raw ? t : min(max(q, a.lo), a.hi);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) ov[r] = add_one(av[r], bv[r], a, raw);
    }
    if (raw) {
        v4i *op = (v4i *)((int32_t *)a.out + oo);
#pragma unroll
        for (int k = 0; k < 4; ++k) __builtin_nontemporal_store(v4i{ov[4 * k], ov[4 * k + 1], ov[4 * k + 2], ov[4 * k + 3]}, op + k);
    } else {
        __builtin_nontemporal_store(pack16(ov), (v4i *)((uint8_t *)a.out + oo));
    }
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

// four bytes of t (each already limited to q.t_hi or not), requantised in 32 bits (see Rq24)
__device__ __forceinline__ int requant4_u24(const uint32_t (&t)[4], const Rq24 &q)
{
    int w = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t x = __umul24(min(t[e], (uint32_t)q.t_hi), (uint32_t)q.mul) + (uint32_t)q.rnd;
        if (e == 0) w = (int)(x >> q.shift);
        else shift_into_byte(w, x, q.shift, e);
    }
    return w;
}

// Both operands unsigned 8-bit, 8-bit output clamped to [0, hi], multipliers that fit 24 bits (see
// launch_add): t = a + [b * b_mul / 2^b_shift] is at most 255 + 2^30, never negative and never
// saturates, and the requantisation runs in 32 bits.  About eight vector instructions per element, so
// the kernel is bound by HBM and not by its arithmetic.
constexpr int kGroupsPerLane = 1;   // 16-byte groups a lane handles (more per lane measured slower on data that
                                    // comes from HBM, see the note at the top)

__global__ __launch_bounds__(256) void add_u8_kernel(const AddArgs a, int groups_per_px, long long total)
{
    const long long g0 = (long long)blockIdx.x * (256 * kGroupsPerLane) + threadIdx.x;
    v4i wa[kGroupsPerLane], wb[kGroupsPerLane];
    size_t oo[kGroupsPerLane];
#pragma unroll
    for (int u = 0; u < kGroupsPerLane; ++u) {
        const long long g = g0 + u * 256;
        if (g >= total) break;
        size_t ao, bo;
        if (groups_per_px == 0) {
            ao = bo = oo[u] = (size_t)g * 16;
        } else {
            long long px;
            if (total < 0x7fffffffLL) px = (unsigned)g / (unsigned)groups_per_px;
            else px = g / groups_per_px;
            const int c0 = (int)(g - px * groups_per_px) * 16;
            ao = (size_t)px * a.a_cs + c0;
            bo = (size_t)px * a.b_cs + c0;
            oo[u] = (size_t)px * a.out_cs + a.out_co + c0;
        }
        wa[u] = __builtin_nontemporal_load((const v4i *)((const uint8_t *)a.a + ao));
        wb[u] = __builtin_nontemporal_load((const v4i *)((const uint8_t *)a.b + bo));
    }
    const uint32_t half = (1u << a.b_shift) >> 1;
#pragma unroll
    for (int u = 0; u < kGroupsPerLane; ++u) {
        if (g0 + u * 256 >= total) break;
        int w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t t[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t av = ((uint32_t)wa[u][k] >> (8 * e)) & 0xffu, bv = ((uint32_t)wb[u][k] >> (8 * e)) & 0xffu;
                t[e] = av + ((__umul24(bv, (uint32_t)a.b_mul) + half) >> a.b_shift);
            }
            w[k] = requant4_u24(t, a.q24);
        }
        __builtin_nontemporal_store(v4i{w[0], w[1], w[2], w[3]}, (v4i *)((uint8_t *)a.out + oo[u]));
    }
}

// int32 + unsigned 8-bit -> 8-bit on dense tensors, the arithmetic of add_rescale_vec_kernel<true>.  The int32
// stream is two thirds of the bytes: a lane takes four separate groups of four elements, so that each of a wave's
// loads of it covers one contiguous KiB (sixteen consecutive elements per lane put every load's 64 pieces 64 bytes
// apart); the 8-bit operand and the output then move as dwords, 256 contiguous bytes per wave and access.
__global__ __launch_bounds__(256) void add_s32_u8_dense_kernel(const AddArgs a, long long elements)
{
    const long long wave_base = ((long long)blockIdx.x * 4 + (threadIdx.x >> 6)) * 1024 + (threadIdx.x & 63) * 4;
    v4i av[4];
    uint32_t bw[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long long e = wave_base + k * 256;
        if (e < elements) {
            av[k] = __builtin_nontemporal_load((const v4i *)((const int32_t *)a.a + e));
            bw[k] = __builtin_nontemporal_load((const uint32_t *)((const uint8_t *)a.b + e));
        }
    }
    const int half = (1 << a.b_shift) >> 1;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const long long e = wave_base + k * 256;
        if (e >= elements) continue;
        uint32_t w = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int bv = (int)((bw[k] >> (8 * r)) & 0xffu);
            const int t = __builtin_elementwise_add_sat(av[k][r], (__mul24(bv, a.b_mul) + half) >> a.b_shift);
            const int q = (int)(((int64_t)t * a.mul_hi + 0x80000000LL) >> 32);
            w |= (uint32_t)(min(max(q, a.lo), a.hi) & 0xff) << (8 * r);
        }
        __builtin_nontemporal_store(w, (uint32_t *)((uint8_t *)a.out + e));
    }
}

__global__ __launch_bounds__(256) void add_rescale_scalar_kernel(const AddArgs a, long long total)
{
    const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const long long px = e / a.c;
    const int ch = (int)(e - px * a.c);
    const int av = load_elem(a.a, (size_t)px * a.a_cs + ch, a.a_dt);
    const int bv = load_elem(a.b, (size_t)px * a.b_cs + ch, a.b_dt);
    const bool raw = a.out_mode == 3;
    const int v = add_one(av, bv, a, raw);
    const size_t oo = (size_t)px * a.out_cs + a.out_co + ch;
    if (raw) ((int32_t *)a.out)[oo] = v;
    else ((uint8_t *)a.out)[oo] = (uint8_t)v;
}

hipError_t launch_add(const AddArgs &a, bool vec, hipStream_t st)
{
    if (a.px == 0 || a.c == 0) return hipSuccess;
    if (vec) {
        const bool dense = a.a_cs == a.c && a.b_cs == a.c && a.out_cs == a.c && a.out_co == 0;
        const long long total = a.px * (a.c / 16);
        const int gpp = dense ? 0 : a.c / 16;
        // fast arithmetic when b is 8 bits with |255 * b_mul| + half < 2^31 and (raw output or
        // 1 <= shift <= 32 with mul << (32 - shift) < 2^31)
        // b_fit32: an 8-bit operand's rescale never leaves 32 bits; b_fast adds what the signed 24-bit multiply
        // of add_rescale_vec_kernel<true> needs (multipliers from 2^23 on would be read as negative)
        const bool b_fit32 = a.b_dt != 2 && a.b_shift <= 30 && 255LL * a.b_mul + (1LL << a.b_shift) / 2 <= 0x7fffffffLL;
        const bool b_fast = b_fit32 && a.b_mul < (1 << 23);
        const bool q_fast = a.out_mode == 3 ||
                            (a.shift >= 1 && a.shift <= 32 && ((long long)a.mul << (32 - a.shift)) <= 0x7fffffffLL);
        const dim3 grid((unsigned)((total + 255) / 256)), block(256);
        // both operands unsigned bytes, output clamped to [0, hi]: everything in 32 bits when the skip term stays
        // below 2^30 and the requantisation pair fits 24 bits
        const Rq24 q24 = make_rq24(a.mul, a.shift, a.hi);
        if (a.a_dt == 0 && a.b_dt == 0 && a.out_mode != 3 && a.lo == 0 && b_fit32 && q24.ok &&      // unsigned 24-bit multiply: b_mul < 2^24
            ((255LL * a.b_mul + (1LL << a.b_shift) / 2) >> a.b_shift) <= (1LL << 30)) {
            AddArgs f = a;
            f.q24 = q24;
            const long long per_block = 256 * kGroupsPerLane;
            hipLaunchKernelGGL(add_u8_kernel, dim3((unsigned)((total + per_block - 1) / per_block)), block, 0, st, f, gpp, total);
        } else if (b_fast && q_fast) {
            AddArgs f = a;
            f.mul_hi = a.out_mode == 3 ? 0 : (int)((long long)a.mul << (32 - a.shift));
            if (dense && a.a_dt == 2 && a.b_dt == 0 && a.out_mode != 3) {
                const long long elements = a.px * a.c;
                hipLaunchKernelGGL(add_s32_u8_dense_kernel, dim3((unsigned)((elements + 4095) / 4096)), block, 0, st, f, elements);
            } else {
                hipLaunchKernelGGL(add_rescale_vec_kernel<true>, grid, block, 0, st, f, gpp, total);
            }
        } else {
            hipLaunchKernelGGL(add_rescale_vec_kernel<false>, grid, block, 0, st, a, gpp, total);
        }
    } else {
        const long long total = a.px * a.c;
        hipLaunchKernelGGL(add_rescale_scalar_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                           st, a, total);
    }
    return hipGetLastError();
}

// out[px, out_co + ch] = clamp([in[px, ch] * mul / 2^shift], 0, bound)
__global__ __launch_bounds__(256) void requant_copy_kernel(const uint8_t *__restrict__ in,
                                                           uint8_t *__restrict__ out, long long total,
                                                           int per_px, int in_cs, int out_cs, int out_co,
                                                           int mul, int shift, int bound, int vec, const Rq24 q24)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    const long long px = g / per_px;
    const int k = (int)(g - px * per_px);
    if (vec && q24.ok) {
        // the multiplier pair fits 24 bits: four instructions per byte
        const v4i wi = __builtin_nontemporal_load((const v4i *)(in + (size_t)px * in_cs + k * 16));
        int w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t t[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = ((uint32_t)wi[q] >> (8 * e)) & 0xffu;
            w[q] = requant4_u24(t, q24);
        }
        __builtin_nontemporal_store(v4i{w[0], w[1], w[2], w[3]}, (v4i *)(out + (size_t)px * out_cs + out_co + k * 16));
    } else if (vec) {
        int v[16];
        unpack16(in, (size_t)px * in_cs + k * 16, 0, v);
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = clampi64(rsr64((int64_t)v[r] * mul, shift), 0, bound);
        *(v4i *)(out + (size_t)px * out_cs + out_co + k * 16) = pack16(v);
    } else {
        const int v = in[(size_t)px * in_cs + k];
        out[(size_t)px * out_cs + out_co + k] = (uint8_t)clampi64(rsr64((int64_t)v * mul, shift), 0, bound);
    }
}

hipError_t launch_requant_copy(const uint8_t *in, uint8_t *out, int64_t px, int c, int in_cs, int out_cs,
                               int out_co, int mul, int shift, int bound, bool vec, hipStream_t st)
{
    if (px == 0 || c == 0) return hipSuccess;
    const int per_px = vec ? c / 16 : c;
    const long long total = (long long)px * per_px;
    hipLaunchKernelGGL(requant_copy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, in, out,
                       total, per_px, in_cs, out_cs, out_co, mul, shift, bound, vec ? 1 : 0, make_rq24(mul, shift, bound));
    return hipGetLastError();
}

// Explicit concatenation, all branches in one launch: each output row is written once, whole.  The
// branch of a lane's group is found by a scan over the (wave-uniform) branch table; its fields are picked
// with selects, so the table stays in scalar registers.
__global__ __launch_bounds__(256) void concat_vec_kernel(const ConcatArgs a, int groups_per_px, long long total)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    long long px;
    if (total < 0x7fffffffLL) px = (unsigned)g / (unsigned)groups_per_px;
    else px = g / groups_per_px;
    const int ch = (int)(g - px * groups_per_px) * 16;
    const uint8_t *src = a.in[0];
    int cs = a.in_cs[0], c0 = 0, mul = a.mul[0], shift = a.shift[0];
    Rq24 q = a.q[0];
    for (int i = 1; i < a.n_in; ++i) {
        const bool later = ch >= a.c_end[i - 1];
        src = later ? a.in[i] : src;
        cs = later ? a.in_cs[i] : cs;
        c0 = later ? a.c_end[i - 1] : c0;
        mul = later ? a.mul[i] : mul;
        shift = later ? a.shift[i] : shift;
        q.ok = later ? a.q[i].ok : q.ok;
        q.mul = later ? a.q[i].mul : q.mul;
        q.shift = later ? a.q[i].shift : q.shift;
        q.t_hi = later ? a.q[i].t_hi : q.t_hi;
        q.rnd = later ? a.q[i].rnd : q.rnd;
    }
    const v4i wi = __builtin_nontemporal_load((const v4i *)(src + (size_t)px * cs + (ch - c0)));
    int w[4];
    if (q.ok) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t t[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = ((uint32_t)wi[k] >> (8 * e)) & 0xffu;
            w[k] = requant4_u24(t, q);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = (int)(((uint32_t)wi[k] >> (8 * e)) & 0xffu);
                word |= (uint32_t)clampi64(rsr64((int64_t)v * mul, shift), 0, a.bound) << (8 * e);
            }
            w[k] = (int)word;
        }
    }
    __builtin_nontemporal_store(v4i{w[0], w[1], w[2], w[3]}, (v4i *)(a.out + (size_t)px * a.out_cs + ch));
}

hipError_t launch_concat_vec(const ConcatArgs &a, int64_t px, hipStream_t st)
{
    const int c_total = a.c_end[a.n_in - 1];
    if (px == 0 || c_total == 0) return hipSuccess;
    const long long total = (long long)px * (c_total / 16);
    hipLaunchKernelGGL(concat_vec_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, c_total / 16, total);
    return hipGetLastError();
}

// max over the window positions inside the image; bytewise max of packed words
__device__ __forceinline__ uint32_t max_u8x4(uint32_t x, uint32_t y)
{
    return max_bytes(x, y);
}

__global__ __launch_bounds__(256) void maxpool_kernel(const uint8_t *__restrict__ x, uint8_t *__restrict__ out,
                                                      long long total, int per_px, int h, int w, int c, int k,
                                                      int stride, int pad, int ho_n, int wo_n, int vec)
{
    // Workgroups go to the eight XCDs round-robin and every XCD has an L2 of its own: workgroup b takes the b/8-th
    // piece of XCD (b % 8)'s contiguous eighth of the output, so that the input rows two neighbouring output rows share
    // are fetched into one L2, not two (workgroups in launch order: every shared row crossed the fabric twice).
    const unsigned nb = gridDim.x, xcd = blockIdx.x & 7, qn = nb >> 3, rn = nb & 7;
    const unsigned piece = xcd * qn + (xcd < rn ? xcd : rn) + (blockIdx.x >> 3);
    const long long g = (long long)piece * 256 + threadIdx.x;
    if (g >= total) return;
    long long px = g / per_px;
    const int q = (int)(g - px * per_px);
    const int wo = (int)(px % wo_n);
    const long long t = px / wo_n;
    const int ho = (int)(t % ho_n);
    const long long n = t / ho_n;
    if (vec && k == 3) {
        // 3x3 window, branch-free: a position outside the image is replaced by the nearest one inside,
        // which the window also contains, so the maximum is unchanged and all nine loads are independent.
        // (A variant in which a lane walks four output rows and carries the shared input row, six loads per output
        // instead of nine, measured slower, 21.8 us against 17.9 us on 64 x 112 x 112 x 64: a quarter of the
        // workgroups, all of them waiting for their loads at the same time.)
        // Bytewise maxima as 16-bit lanes: the even bytes masked out of every loaded word; the odd bytes unmasked, because a
        // lane's maximum is decided by its high byte (the low byte only breaks ties) and only the high byte is kept.
        typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
        u16x2 me[4] = {}, mo[4] = {};
        const uint8_t *base = x + (size_t)n * h * w * c + q * 16;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int hi = min(max(ho * stride - pad + i, 0), h - 1);
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int wi = min(max(wo * stride - pad + j, 0), w - 1);
                const v4i v = *(const v4i *)(base + ((size_t)hi * w + wi) * c);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const uint32_t u = (uint32_t)v[d];
                    me[d] = __builtin_elementwise_max(me[d], __builtin_bit_cast(u16x2, u & 0x00ff00ffu));
                    mo[d] = __builtin_elementwise_max(mo[d], __builtin_bit_cast(u16x2, u));
                }
            }
        }
        v4i o;
#pragma unroll
        for (int d = 0; d < 4; ++d) o[d] = (int)(__builtin_bit_cast(uint32_t, me[d]) | (__builtin_bit_cast(uint32_t, mo[d]) & 0xff00ff00u));
        *(v4i *)(out + (size_t)px * c + q * 16) = o;
    } else if (vec) {
        uint32_t m[4] = {0, 0, 0, 0};
        for (int i = 0; i < k; ++i) {
            const int hi = ho * stride - pad + i;
            if ((unsigned)hi >= (unsigned)h) continue;
            for (int j = 0; j < k; ++j) {
                const int wi = wo * stride - pad + j;
                if ((unsigned)wi >= (unsigned)w) continue;
                const v4i v = *(const v4i *)(x + (((size_t)n * h + hi) * w + wi) * c + q * 16);
                m[0] = max_u8x4(m[0], (uint32_t)v.x); m[1] = max_u8x4(m[1], (uint32_t)v.y);
                m[2] = max_u8x4(m[2], (uint32_t)v.z); m[3] = max_u8x4(m[3], (uint32_t)v.w);
            }
        }
        *(v4i *)(out + (size_t)px * c + q * 16) = v4i{(int)m[0], (int)m[1], (int)m[2], (int)m[3]};
    } else {
        int best = 0;
        for (int i = 0; i < k; ++i) {
            const int hi = ho * stride - pad + i;
            if ((unsigned)hi >= (unsigned)h) continue;
            for (int j = 0; j < k; ++j) {
                const int wi = wo * stride - pad + j;
                if ((unsigned)wi >= (unsigned)w) continue;
                const int v = x[(((size_t)n * h + hi) * w + wi) * c + q];
                best = v > best ? v : best;
            }
        }
        out[(size_t)px * c + q] = (uint8_t)best;
    }
}

hipError_t launch_maxpool(const uint8_t *x, uint8_t *out, int n, int h, int w, int c, int k, int stride,
                          int pad, int ho, int wo, bool vec, hipStream_t st)
{
    const int per_px = vec ? c / 16 : c;
    const long long total = (long long)n * ho * wo * per_px;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, out, total,
                       per_px, h, w, c, k, stride, pad, ho, wo, vec ? 1 : 0);
    return hipGetLastError();
}

// one thread per (image, channel): consecutive lanes read consecutive channels
__global__ __launch_bounds__(256) void avgpool_kernel(const uint8_t *__restrict__ x, uint8_t *__restrict__ out,
                                                      long long total, int hw, int c, int mul, int shift,
                                                      int bound)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    const long long n = g / c;
    const int ch = (int)(g - n * c);
    const uint8_t *p = x + (size_t)n * hw * c + ch;
    int64_t s = 0;
    for (int i = 0; i < hw; ++i) s += p[(size_t)i * c];
    out[g] = (uint8_t)clampi64(rsr64(s * mul, shift), 0, bound);
}

// Same result, c % 4 == 0 and 4-byte aligned tensors: a workgroup sums 256 channels of one image,
// wave w taking positions w, w + 4, ... (four channels per lane and load, 256 contiguous bytes per
// wave and position); the four partial sums meet in LDS.
__global__ __launch_bounds__(256) void avgpool_vec_kernel(const uint8_t *__restrict__ x, uint8_t *__restrict__ out, int hw,
                                                          int c, int mul, int shift, int bound)
{
    __shared__ int part[4][64][4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, split = tid >> 6;
    const int quad = blockIdx.x * 64 + lane;
    const int n = blockIdx.y;
    const bool ok = quad * 4 < c;
    int s[4] = {0, 0, 0, 0};
    if (ok) {
        const uint8_t *p = x + ((size_t)n * hw) * c + (size_t)quad * 4;
        int i = split;
        for (; i + 12 < hw; i += 16) {          // four loads in flight
            const uint32_t v0 = *(const uint32_t *)(p + (size_t)i * c), v1 = *(const uint32_t *)(p + (size_t)(i + 4) * c);
            const uint32_t v2 = *(const uint32_t *)(p + (size_t)(i + 8) * c), v3 = *(const uint32_t *)(p + (size_t)(i + 12) * c);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                s[k] += (int)((v0 >> (8 * k)) & 0xff) + (int)((v1 >> (8 * k)) & 0xff) + (int)((v2 >> (8 * k)) & 0xff) +
                        (int)((v3 >> (8 * k)) & 0xff);
        }
        for (; i < hw; i += 4) {
            const uint32_t v = *(const uint32_t *)(p + (size_t)i * c);
#pragma unroll
            for (int k = 0; k < 4; ++k) s[k] += (int)((v >> (8 * k)) & 0xff);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) part[split][lane][k] = s[k];
    __syncthreads();
    if (split == 0 && ok) {
        uint32_t o = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t t = (int64_t)part[0][lane][k] + part[1][lane][k] + part[2][lane][k] + part[3][lane][k];
            o |= (uint32_t)clampi64(rsr64(t * mul, shift), 0, bound) << (8 * k);
        }
        *(uint32_t *)(out + (size_t)n * c + (size_t)quad * 4) = o;
    }
}

hipError_t launch_avgpool(const uint8_t *x, uint8_t *out, int n, int hw, int c, int mul, int shift, int bound,
                          hipStream_t st)
{
    const long long total = (long long)n * c;
    if (total == 0) return hipSuccess;
    // per-position sums stay below 2^31 for hw < 2^23
    if (c % 4 == 0 && !((uintptr_t)x & 3) && !((uintptr_t)out & 3) && hw < (1 << 23) && n <= 65535) {
        hipLaunchKernelGGL(avgpool_vec_kernel, dim3((unsigned)((c / 4 + 63) / 64), (unsigned)n), dim3(256), 0, st, x, out, hw,
                           c, mul, shift, bound);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(avgpool_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, x, out, total,
                       hw, c, mul, shift, bound);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void renorm_kernel(const uint8_t *__restrict__ x, uint8_t *__restrict__ out,
                                                     long long count, int vec)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (vec) {
        if (g * 16 >= count) return;
        v4i v = __builtin_nontemporal_load((const v4i *)(x + g * 16));
        v.x ^= 0x80808080; v.y ^= 0x80808080; v.z ^= 0x80808080; v.w ^= 0x80808080;
        __builtin_nontemporal_store(v, (v4i *)(out + g * 16));
    } else {
        if (g >= count) return;
        out[g] = x[g] ^ 0x80;
    }
}

hipError_t launch_renorm(const uint8_t *x, uint8_t *out, int64_t count, bool vec, hipStream_t st)
{
    if (count == 0) return hipSuccess;
    const long long threads = vec ? count / 16 : count;
    hipLaunchKernelGGL(renorm_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, x, out,
                       (long long)count, vec ? 1 : 0);
    return hipGetLastError();
}

}  // namespace icnn
