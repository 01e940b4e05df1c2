// Layers with one to four output channels (the last layer of the regression networks: "the overall
// ratio can be reset by rescaling the output", Section 3.1).  On the matrix-core path such a layer pads
// cout to 32 and spends its time moving im2col tiles; here the cin / 16 lanes of a group own one output
// pixel, each lane one 16-channel slice, so that a wave reads whole contiguous runs of NHWC memory
// (16 bytes per lane, neighbouring lanes neighbouring addresses).  Every lane walks the taps with 4-way
// int8 dot products against its slice of the weights (kept in LDS, taken out of the same packed buffer the
// matrix-core kernels use); the slices meet by lane shuffles.  Bound by the L1 path: x is read kh*kw
// times from cache, once from HBM, the output is tiny.
#include "conv_common.h"

namespace icnn {

// Byte offset, inside the packed weights, of the 16 weights k0 .. k0 + 15 (k0 a multiple of 16) of output
// channel co < 4: chunk 0, K step k0 / 64, fragment half (k0 / 32) & 1, lane 32 * ((k0 / 16) & 1) + row,
// and matrix row = channel for the first four channels of a chunk.
__device__ __forceinline__ unsigned packed_weight_offset(int k0, int co)
{
    return (unsigned)(k0 >> 6) * kChunkBytes + (unsigned)((k0 >> 5) & 1) * 1024u + (unsigned)((((k0 >> 4) & 1) * 32 + co) * 16);
}

template <int NCO>
__global__ __launch_bounds__(256) void conv_narrow_kernel(const ConvArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t wl_raw[];     // [tap][slice][co] x 16 bytes
    v4i *wl = (v4i *)wl_raw;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = a.Cin >> 4;                 // lanes per pixel
    const int ppw = 64 / S;                   // pixels per wave
    const int taps = a.KH * a.KW;
    for (int e = tid; e < taps * S * NCO; e += 256) {
        const int co = e % NCO, ts = e / NCO;
        wl[e] = *(const v4i *)(a.wp + packed_weight_offset((ts / S) * a.Cin + (ts % S) * 16, co));
    }
    __syncthreads();

    const int slice = lane % S, lp = lane / S;
    const int p = (blockIdx.x * 4 + wave) * ppw + lp;
    const bool pv = lp < ppw && p < a.M;
    const int pc = pv ? p : 0;
    const int n = fast_div(pc, a.div_howo);
    const int r = pc - n * a.Ho * a.Wo;
    const int ho = fast_div(r, a.div_wo);
    const int wo = r - ho * a.Wo;
    int acc[NCO];
#pragma unroll
    for (int co = 0; co < NCO; ++co) acc[co] = 0;
    const int ix = (int)a.in_xor, fx = (int)a.frag_xor;
    constexpr int BATCH = 5;                  // loads in flight per lane
    for (int kh = 0; kh < a.KH; ++kh) {
        const int hi = ho * a.sh - a.ph + kh;
        const bool rowok = pv && (unsigned)hi < (unsigned)a.H;
        const uint8_t *row = a.x + (rowok ? (size_t)(n * a.H + hi) * a.W * a.in_cs : 0) + slice * 16;
        for (int kw0 = 0; kw0 < a.KW; kw0 += BATCH) {
            v4i v[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int wi = wo * a.sw - a.pw + kw0 + u;
                const bool ok = rowok && kw0 + u < a.KW && (unsigned)wi < (unsigned)a.W;
                const v4i t = *(const v4i *)(row + (ok ? (size_t)wi * a.in_cs : 0));
                // outside the image: zero after the raw picture's "- 128", -128 for full-range unsigned bytes
                // (which the weight-sum term of the bias turns back into zero)
                v[u] = ok ? v4i{t.x ^ ix, t.y ^ ix, t.z ^ ix, t.w ^ ix} : v4i{0, 0, 0, 0};
                v[u] = v4i{v[u].x ^ fx, v[u].y ^ fx, v[u].z ^ fx, v[u].w ^ fx};
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                if (kw0 + u < a.KW) {
                    const v4i *wt = wl + ((kh * a.KW + kw0 + u) * S + slice) * NCO;
#pragma unroll
                    for (int co = 0; co < NCO; ++co) {
                        const v4i w = wt[co];
                        acc[co] = __builtin_amdgcn_sdot4(v[u].x, w.x, acc[co], false);
                        acc[co] = __builtin_amdgcn_sdot4(v[u].y, w.y, acc[co], false);
                        acc[co] = __builtin_amdgcn_sdot4(v[u].z, w.z, acc[co], false);
                        acc[co] = __builtin_amdgcn_sdot4(v[u].w, w.w, acc[co], false);
                    }
                }
            }
        }
    }
    // the S slices of a pixel sit in consecutive lanes: lane slice 0 collects them
#pragma unroll
    for (int co = 0; co < NCO; ++co) {
        int sum = acc[co];
        for (int j = 1; j < S; ++j) sum += __shfl(acc[co], lane + j, 64);
        acc[co] = sum;
    }
    if (!pv || slice != 0) return;
    // epilogue: bias, the rescaled skip operand (Section 4.1), requantisation (Section 3.2.1), clamp
    const size_t ro = (size_t)p * a.res_cs;
    const size_t oo = (size_t)p * a.out_cs + a.out_co;
#pragma unroll
    for (int co = 0; co < NCO; ++co) {
        if (co >= a.Cout) break;
        int64_t t = (int64_t)acc[co] + a.bias[co];
        if (a.frag_xor) t += 128LL * a.wsum[co];     // see ConvArgs::frag_xor
        int64_t skip = 0;
        if (a.res_mode != 0) skip = rsr64((int64_t)load_elem(a.res, ro + co, a.res_dtype) * a.res_mul, a.res_shift);
        if (a.res_mode == 1) t += skip;
        const int ti = sat32(t);
        if (a.out_mode == 3) {
            ((int32_t *)a.out)[oo + co] = ti;
        } else {
            int64_t q = rsr64((int64_t)ti * a.mul, a.shift);
            if (a.res_mode == 2) q += skip;
            ((uint8_t *)a.out)[oo + co] = (uint8_t)clampi64(q, a.lo, a.hi);
        }
    }
}

// 3x3, stride 1: a wave owns a strip of 64 / S output columns and walks down `rseg` output rows of one
// image.  Every input row is fetched once per strip (three 16-byte loads per lane, one per kw) and feeds
// the three output rows it belongs to, whose partial sums rotate through three accumulator sets; the
// row that just became complete is reduced over the S lanes of each pixel and stored.  x is read once
// from HBM and three times (instead of nine) through L1.
// PLAIN: the input bytes are operands as they are (no XOR) and x lies below 2 GiB: the loads go through a buffer
// descriptor, whose range check returns zeros for the padding (an out-of-range offset) at no instruction.
template <int NCO, bool PLAIN>
__global__ __launch_bounds__(256) void conv_narrow3x3_kernel(const ConvArgs a, int rseg, int strips, int segs)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the buffer-resource type exists in the device pass only
    extern __shared__ __attribute__((aligned(16))) uint8_t wl_raw[];     // [tap][slice][co] x 16 bytes
    v4i *wl = (v4i *)wl_raw;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = a.Cin >> 4;
    const int ppw = 64 / S;
    for (int e = tid; e < 9 * S * NCO; e += 256) {
        const int co = e % NCO, ts = e / NCO;
        wl[e] = *(const v4i *)(a.wp + packed_weight_offset((ts / S) * a.Cin + (ts % S) * 16, co));
    }
    __syncthreads();
    const int w = blockIdx.x * 4 + wave;            // wave id -> (image, row segment, column strip)
    if (w >= a.N * segs * strips) return;
    const int strip = w % strips;
    const int seg = (w / strips) % segs;
    const int n = w / (strips * segs);
    const int slice = lane % S, lp = lane / S;
    const int wo = strip * ppw + lp;
    const bool colv = lp < ppw && wo < a.Wo;        // this lane's pixel column exists
    const int r0 = seg * rseg;
    const int rows_out = min(rseg, a.Ho - r0);
    const int ix = (int)a.in_xor, fx = (int)a.frag_xor;
    // this lane's slice of the nine taps' weights
    v4i wreg[9][NCO];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int co = 0; co < NCO; ++co) wreg[t][co] = wl[(t * S + slice) * NCO + co];
    bool cok[3];
    size_t coff[3];
    // PLAIN: offsets from the row's first byte; a column outside the picture gets one beyond any buffer this path takes,
    // and so does a row outside it (their sum stays below 2^32)
    [[maybe_unused]] const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)a.x, 0, a.x_bytes, 0x00020000);
    [[maybe_unused]] unsigned boff[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
        const int wi = wo - a.pw + kw;
        cok[kw] = colv && (unsigned)wi < (unsigned)a.W;
        coff[kw] = cok[kw] ? (size_t)wi * a.in_cs + slice * 16 : 0;
        boff[kw] = cok[kw] ? (unsigned)coff[kw] : 0x7fffff00u;
    }
    // the epilogue in 32 bits where the layer's parameters allow it (wave-uniform): requantisation as one multiply-add
    // whose high word is the result, an unsigned 8-bit skip operand whose rescale fits 32 bits
    const bool quick = a.out_mode != 3 && a.rq_fast && !a.frag_xor && (a.res_mode == 0 || a.res_fast);
    int acc[3][NCO];
#pragma unroll
    for (int q = 0; q < 3; ++q)
#pragma unroll
        for (int co = 0; co < NCO; ++co) acc[q][co] = 0;

    // The skip operand of an output row is fetched one row step before the row is complete: a load inside emit() would
    // have to be waited for on the spot, and that wait also covers the next input row's loads issued just before it,
    // i.e. every row step would expose a full memory latency.
    int rescur[NCO], resnext[NCO];
#pragma unroll
    for (int co = 0; co < NCO; ++co) rescur[co] = resnext[co] = 0;
    auto fetch_res = [&](int j, int (&r)[NCO]) {      // skip operand of output row r0 + j, where that row exists
        if (a.res_mode != 0 && j >= 0 && j < rows_out && colv && slice == 0) {
            const size_t ro = (((size_t)n * a.Ho + r0 + j) * a.Wo + wo) * a.res_cs;
#pragma unroll
            for (int co = 0; co < NCO; ++co)
                if (co < a.Cout) r[co] = load_elem(a.res, ro + co, a.res_dtype);
        }
    };
    // input row i of the segment (image row r0 - ph + i) adds tap row kh to output row r0 + i - kh
    auto emit = [&](int j, int (&sum)[NCO]) {         // output row r0 + j is complete
#pragma unroll
        for (int co = 0; co < NCO; ++co) {
            int t = sum[co];
            for (int q = 1; q < S; ++q) t += __shfl(sum[co], lane + q, 64);
            sum[co] = t;
        }
        if (j >= 0 && j < rows_out && colv && slice == 0) {
            const size_t p = ((size_t)n * a.Ho + r0 + j) * a.Wo + wo;
            const size_t oo = p * a.out_cs + a.out_co;
            if (quick) {
#pragma unroll
                for (int co = 0; co < NCO; ++co) {
                    if (co >= a.Cout) break;
                    int skip = 0;
                    if (a.res_mode != 0) skip = (int)(((uint32_t)rescur[co] * (uint32_t)a.res_mul + (uint32_t)((1 << a.res_shift) >> 1)) >> a.res_shift);
                    const int ti = sat32((int64_t)sum[co] + a.bias[co] + (a.res_mode == 1 ? skip : 0));
                    int q = (int)(((int64_t)ti * a.mul_hi + 0x80000000LL) >> 32);
                    if (a.res_mode == 2) q = __builtin_elementwise_add_sat(q, skip);       // the clamp below makes the saturation exact
                    ((uint8_t *)a.out)[oo + co] = (uint8_t)min(max(q, a.lo), a.hi);
                }
            } else
#pragma unroll
            for (int co = 0; co < NCO; ++co) {
                if (co >= a.Cout) break;
                int64_t t = (int64_t)sum[co] + a.bias[co];
                if (a.frag_xor) t += 128LL * a.wsum[co];     // see ConvArgs::frag_xor
                int64_t skip = 0;
                if (a.res_mode != 0) skip = rsr64((int64_t)rescur[co] * a.res_mul, a.res_shift);
                if (a.res_mode == 1) t += skip;
                const int ti = sat32(t);
                if (a.out_mode == 3) {
                    ((int32_t *)a.out)[oo + co] = ti;
                } else {
                    int64_t q = rsr64((int64_t)ti * a.mul, a.shift);
                    if (a.res_mode == 2) q += skip;
                    ((uint8_t *)a.out)[oo + co] = (uint8_t)clampi64(q, a.lo, a.hi);
                }
            }
        }
#pragma unroll
        for (int co = 0; co < NCO; ++co) sum[co] = 0;
    };
    // raw loads of input row i (nothing touches the data yet, so the loads stay in flight) ...
    auto fetch_row = [&](int i, v4i (&v)[3], bool &rowok) {
        const int hi = r0 - a.ph + i;
        rowok = (unsigned)hi < (unsigned)a.H;
        if constexpr (PLAIN) {
            const unsigned rb = rowok ? (unsigned)((n * a.H + hi) * a.W) * (unsigned)a.in_cs : 0x80000000u;
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) v[kw] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, rb + boff[kw], 0, 0);
        } else {
            const uint8_t *row = a.x + (rowok ? (size_t)(n * a.H + hi) * a.W * a.in_cs : 0);
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) v[kw] = *(const v4i *)(row + coff[kw]);
        }
    };
    // ... and what makes them operands: outside the image zero after the raw picture's "- 128", -128 for
    // full-range unsigned bytes (which the weight-sum term of the bias turns back into zero)
    auto finish_row = [&](const v4i (&raw)[3], bool rowok, v4i (&v)[3]) {
        if constexpr (PLAIN) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) v[kw] = raw[kw];
            return;
        }
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const bool ok = rowok && cok[kw];
            const v4i t = raw[kw];
            v[kw] = ok ? v4i{t.x ^ ix, t.y ^ ix, t.z ^ ix, t.w ^ ix} : v4i{0, 0, 0, 0};
            v[kw] = v4i{v[kw].x ^ fx, v[kw].y ^ fx, v[kw].z ^ fx, v[kw].w ^ fx};
        }
    };
    v4i vcur[3], vnext[3];
    // one input row: the next row's loads are issued first, so they travel during this row's arithmetic
    bool oknext = false;
    auto row_step = [&](int i, int (&a0)[NCO], int (&a1)[NCO], int (&a2)[NCO]) {
        fetch_row(i + 1, vnext, oknext);
        fetch_res(i - 1, resnext);                    // for the row the next step completes
        auto tap_row = [&](int kh, int (&dst)[NCO]) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                for (int co = 0; co < NCO; ++co) {
                    const v4i wv = wreg[kh * 3 + kw][co];
                    dst[co] = __builtin_amdgcn_sdot4(vcur[kw].x, wv.x, dst[co], false);
                    dst[co] = __builtin_amdgcn_sdot4(vcur[kw].y, wv.y, dst[co], false);
                    dst[co] = __builtin_amdgcn_sdot4(vcur[kw].z, wv.z, dst[co], false);
                    dst[co] = __builtin_amdgcn_sdot4(vcur[kw].w, wv.w, dst[co], false);
                }
        };
        tap_row(0, a0);        // output row r0 + i
        tap_row(1, a1);        // output row r0 + i - 1
        tap_row(2, a2);        // output row r0 + i - 2: complete
        emit(i - 2, a2);
        finish_row(vnext, oknext, vcur);
#pragma unroll
        for (int co = 0; co < NCO; ++co) rescur[co] = resnext[co];
    };
    fetch_row(0, vnext, oknext);
    finish_row(vnext, oknext, vcur);
    const int rows_in = rows_out + 2;
    for (int i = 0; i < rows_in; i += 3) {
        row_step(i, acc[0], acc[2], acc[1]);
        if (i + 1 < rows_in) row_step(i + 1, acc[1], acc[0], acc[2]);
        if (i + 2 < rows_in) row_step(i + 2, acc[2], acc[1], acc[0]);
    }
#endif
}

bool conv_narrow_applies(const ConvArgs &a)
{
    // weights of all taps in LDS (16 bytes per tap, slice and channel)
    // (with two to four channels, and on small maps, the matrix-core kernels are as fast or faster: measured)
    return a.Cout == 1 && a.M >= 200000 && a.Cin % 16 == 0 && a.Cin <= 256 && a.in_cs % 16 == 0 && !a.pc &&
           (long long)a.KH * a.KW * (a.Cin / 16) * 4 * 16 <= 48 * 1024;
}

// Requires conv_narrow_applies(a), x 16-byte aligned, packed weights in the ordinary (kh, kw, ci) order.
hipError_t launch_conv_narrow(const ConvArgs &a0, hipStream_t st)
{
    ConvArgs a = a0;
    a.div_howo = make_fast_div((unsigned)(a.Ho * a.Wo));
    a.div_wo = make_fast_div((unsigned)a.Wo);
    const int S = a.Cin / 16, ppb = 4 * (64 / S);
    const int nco = a.Cout == 1 ? 1 : 4;
    const size_t lds = (size_t)a.KH * a.KW * S * nco * 16;
    if (a.KH == 3 && a.KW == 3 && a.sh == 1 && a.sw == 1 && S <= 8 && !g_tuning.no_stream) {
        // row segments short enough to give the chip a few thousand waves, long enough to amortise the
        // two halo rows each segment re-reads
        const int strips = (a.Wo + 64 / S - 1) / (64 / S);
        // ... and few enough that all waves are resident at once (five per SIMD with one output channel, two with four:
        // 256 CUs x 4 SIMDs of them, less a margin for the ragged last segment), or the last ones run alone
        const long long slots = 1024LL * (a.Cout == 1 ? 5 : 2) * 19 / 20;
        long long rseg = ((long long)a.N * a.Ho * strips + slots - 1) / slots;
        rseg = rseg < 4 ? 4 : (rseg > 128 ? 128 : rseg);
        const int segs = (int)((a.Ho + rseg - 1) / rseg);
        const long long waves = (long long)a.N * segs * strips;
        const dim3 grid((unsigned)((waves + 3) / 4)), block(256);
        const bool plain = !a.in_xor && !a.frag_xor && a.x_bytes < 0x7fffff00u;
        if (a.Cout == 1) {
            if (plain) hipLaunchKernelGGL((conv_narrow3x3_kernel<1, true>), grid, block, lds, st, a, (int)rseg, strips, segs);
            else hipLaunchKernelGGL((conv_narrow3x3_kernel<1, false>), grid, block, lds, st, a, (int)rseg, strips, segs);
        } else {
            if (plain) hipLaunchKernelGGL((conv_narrow3x3_kernel<4, true>), grid, block, lds, st, a, (int)rseg, strips, segs);
            else hipLaunchKernelGGL((conv_narrow3x3_kernel<4, false>), grid, block, lds, st, a, (int)rseg, strips, segs);
        }
        return hipGetLastError();
    }
    const dim3 grid((unsigned)((a.M + ppb - 1) / ppb)), block(256);
    if (a.Cout == 1) hipLaunchKernelGGL(conv_narrow_kernel<1>, grid, block, lds, st, a);
    else hipLaunchKernelGGL(conv_narrow_kernel<4>, grid, block, lds, st, a);
    return hipGetLastError();
}

}  // namespace icnn
