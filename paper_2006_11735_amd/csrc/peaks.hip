// Measured-achievable roofs of the machine the library runs on, as two plain kernels the benchmark times:
// a register-only loop of the int8 matrix instruction the convolution kernels use, and a streaming copy.
// Nothing of the method is computed here.
#include "icnn_device.h"

namespace icnn {

// Every wave keeps four independent 32x32 accumulator tiles and issues `iters` rounds of eight
// v_mfma_i32_32x32x32_i8 (two per tile, the dependency distance of the convolution kernels' K step).
// Operands never change; the sums are stored once so that the loop cannot be dropped.
__global__ __launch_bounds__(256) void mfma_i8_loop_kernel(int iters, int *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const v4i a0 = {lane, lane + 1, lane + 2, lane + 3}, a1 = {~lane, lane ^ 21, lane * 3, lane * 5};
    const v4i b0 = {lane * 7, lane * 11, lane ^ 85, lane + 9}, b1 = {lane * 13, ~lane * 3, lane + 77, lane ^ 51};
    v16i c00 = {}, c01 = {}, c10 = {}, c11 = {};
    for (int i = 0; i < iters; ++i) {
        c00 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, c00, 0, 0, 0);
        c01 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b1, c01, 0, 0, 0);
        c10 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b0, c10, 0, 0, 0);
        c11 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, c11, 0, 0, 0);
        c00 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1, c00, 0, 0, 0);
        c01 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b0, c01, 0, 0, 0);
        c10 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b1, c10, 0, 0, 0);
        c11 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, c11, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c00[r] ^ c01[r] ^ c10[r] ^ c11[r];
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// dst[i] = src[i]: one 16-byte non-temporal load and store per lane, one workgroup per 4 KiB.  (Measured on 1 GiB:
// 6.5 TB/s; the same with cached accesses 6.2, four accesses per lane 5.7, a persistent grid-stride loop 4.3,
// hipMemcpyAsync 5.0.)
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst, long long n16)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

hipError_t launch_mfma_loop(int blocks, int iters, int *sink, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_i8_loop_kernel, dim3((unsigned)blocks), dim3(256), 0, st, iters, sink);
    return hipGetLastError();
}

hipError_t launch_stream_copy(const void *src, void *dst, long long n16, hipStream_t st)
{
    if (n16 == 0) return hipSuccess;
    const long long blocks = (n16 + 255) / 256;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const v4i *)src, (v4i *)dst, n16);
    return hipGetLastError();
}

}  // namespace icnn
