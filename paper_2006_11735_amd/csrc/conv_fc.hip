// Pointwise layers on very few pixels (the classifier: a 1x1 convolution over the pooled 1x1 map, one pixel
// per image).  On the tile kernels such a layer has cout/128 workgroups of which each walks the whole K axis
// alone: 8 workgroups read 2 MB of weights for a ResNet head.  Here a workgroup owns 32 output channels and
// its eight waves split the K axis into contiguous ranges; every wave loads its fragments straight from global memory into
// registers (the packed weights are stored in fragment order, an activation fragment is 16 consecutive
// bytes of a pixel: no LDS, no barrier in the loop), multiplies, and the eight partial accumulators are
// summed through LDS.  Same accumulator layout as the tile kernels, hence the same epilogue.
#include "conv_common.h"

namespace icnn {

constexpr int kFcWaves = 8;

template <bool U8>
__global__ __launch_bounds__(64 * kFcWaves) void conv_fc_kernel(const ConvArgs a)
{
    // partial sums: [wave][register 0..31][lane]; reused for the reduced sums [register][lane]
    __shared__ int part[kFcWaves][32][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int chunk = blockIdx.x;                       // 32 output channels
    const int half = lane >> 5;

    // this lane's pixels: (lane & 31) and 32 + (lane & 31); bytes k = 64*s + 32*kq + 16*half .. + 15 of each
    const uint8_t *xp[2];
    bool pv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int p = j * 32 + (lane & 31);
        pv[j] = p < a.M;
        xp[j] = a.x + (size_t)(pv[j] ? p : 0) * a.in_cs + half * 16;
    }
    const uint8_t *wbase = a.wp + (size_t)chunk * a.ksteps * kChunkBytes + lane * 16;

    // the bias travels while the K loop runs (only wave 0 finishes the tile)
    v16i bias[1];
    if (wave == 0) load_bias_rows<1>(a, chunk * 32, half, bias);
    v16i acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0;
    const v4i zero = {0, 0, 0, 0};
    const v4i flip = {(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
    // Wave w owns K steps [w * per, (w + 1) * per): consecutive steps read consecutive bytes of a pixel, so the
    // lanes of a wave use whole cache lines.  The fragments of up to four steps are requested together: one
    // memory latency per batch.
    constexpr int B = 4;
    const int per = (a.ksteps + kFcWaves - 1) / kFcWaves;
    const int s_end = min(a.ksteps, (wave + 1) * per);
    for (int s0 = wave * per; s0 < s_end; s0 += B) {
        v4i fa[B][2], fb[B][2][2];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            // every load is issued (no branch around it, so that all of them are in flight together): steps beyond
            // the last one re-read the last step and get their weights zeroed afterwards; pixels beyond the last
            // one read pixel 0 and contribute nothing that is stored
            const int sc = min(s0 + u, a.ksteps - 1);
            fa[u][0] = *(const v4i *)(wbase + (size_t)sc * kChunkBytes);
            fa[u][1] = *(const v4i *)(wbase + (size_t)sc * kChunkBytes + 1024);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int kq = 0; kq < 2; ++kq) fb[u][j][kq] = *(const v4i *)(xp[j] + sc * kStepK + kq * 32);
        }
        __builtin_amdgcn_sched_barrier(0);      // all requests go out before the first use
#pragma unroll
        for (int u = 0; u < B; ++u) {
            if (s0 + u >= s_end) fa[u][0] = fa[u][1] = zero;
            if (U8) {
#pragma unroll
                for (int j = 0; j < 2; ++j) { fb[u][j][0] ^= flip; fb[u][j][1] ^= flip; }
            }
        }
#pragma unroll
        for (int u = 0; u < B; ++u)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[u][0], fb[u][j][0], acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[u][1], fb[u][j][1], acc[j], 0, 0, 0);
            }
    }
    mfma_drain(acc);
    // ---- sum the eight partial accumulators: wave w sums registers 4w .. 4w + 3 of all waves
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave][j * 16 + r][lane] = acc[j][r];
    __syncthreads();
    int sum[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        sum[q] = 0;
#pragma unroll
        for (int w = 0; w < kFcWaves; ++w) sum[q] += part[w][wave * 4 + q][lane];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) part[0][wave * 4 + q][lane] = sum[q];
    __syncthreads();
    if (wave != 0) return;
    v16i tot[1][2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) tot[0][j][r] = part[0][j * 16 + r][lane] + bias[0][r];
    epilogue_tiles<1, 2>(a, tot, chunk * 32, 0, lane);
}

// 1x1, stride 1, no padding, at most 64 output pixels, whole 64-channel K steps, 16-byte aligned rows
bool conv_fc_applies(const ConvArgs &a)
{
    return a.KH == 1 && a.KW == 1 && a.sh == 1 && a.sw == 1 && a.ph == 0 && a.pw == 0 && a.M <= 64 && a.Cin % 64 == 0 &&
           a.Cin >= 512 && a.in_cs % 16 == 0 && a.in_xor == 0 && !a.pc;
}

// Requires conv_fc_applies(a) and x 16-byte aligned.
hipError_t launch_conv_fc(const ConvArgs &a, hipStream_t st)
{
    const dim3 grid((unsigned)((a.Cout + 31) / 32)), block(64 * kFcWaves);
    if (a.frag_xor) hipLaunchKernelGGL(conv_fc_kernel<true>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(conv_fc_kernel<false>, grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace icnn
