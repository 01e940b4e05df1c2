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
// K advanced 64 at a time through double-buffered LDS.
#include "icnn_device.h"

namespace icnn {

template <int BM, int BP, int WAVES_M, int WAVES_P, bool VEC>
__global__ __launch_bounds__(256) void conv_igemm_kernel(const ConvArgs a)
{
    constexpr int TM = BM / WAVES_M / 32;   // 32x32 tiles per wave along cout
    constexpr int TP = BP / WAVES_P / 32;   // and along pixels
    constexpr int A_BYTES = BM * kStepK;
    constexpr int B_BYTES = BP * kStepK;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int NPA = (BM * 4 + 255) / 256;
    constexpr int NPB = BP * 4 / 256;
    static_assert(WAVES_M * WAVES_P == 4 && TM >= 1 && TP >= 1 && NPB >= 1, "tile shape");

    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WAVES_M;
    const int wp = wave / WAVES_M;
    const int ct = blockIdx.x % a.n_ct;
    const int pt = blockIdx.x / a.n_ct;
    const int pix0 = pt * BP;
    const int chunk0 = ct * (BM / 32);

    // ---- gather bookkeeping: this thread always fills 16-byte slot `slot` of
    // pixels (tid>>2) + 64*j of the tile.
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
    // position of this thread's slot on the K axis, kept as (kh, kw, ci)
    int kh = 0, kw = 0, ci = 0;
    if (VEC) {
        const int kk = slot * 16;
        const int tap = kk / a.Cin;
        ci = kk - tap * a.Cin;
        kh = tap / a.KW;
        kw = tap - kh * a.KW;
    }

    v4i areg[NPA], breg[NPB];

    auto load_tiles = [&](int s) {
#pragma unroll
        for (int i = 0; i < NPA; ++i) {
            const int e = tid + 256 * i;
            if (BM * 4 >= 256 * (i + 1) || e < BM * 4) {
                const size_t off = ((size_t)(chunk0 + (e >> 7)) * a.ksteps + s) * kChunkBytes +
                                   (size_t)(e & 127) * 16;
                areg[i] = *(const v4i *)(a.wp + off);
            }
        }
        if (VEC) {
#pragma unroll
            for (int j = 0; j < NPB; ++j) {
                const int hi = hi0[j] + kh, wi = wi0[j] + kw;
                const bool ok = pv[j] && kh < a.KH && (unsigned)hi < (unsigned)a.H &&
                                (unsigned)wi < (unsigned)a.W;
                v4i v = {0, 0, 0, 0};
                if (ok) {
                    const size_t off = ((size_t)(nrow[j] + hi) * a.W + wi) * a.in_cs + ci;
                    v = *(const v4i *)(a.x + off);
                    v.x ^= a.in_xor; v.y ^= a.in_xor; v.z ^= a.in_xor; v.w ^= a.in_xor;
                }
                breg[j] = v;
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
            const int pl = (tid >> 2) + 64 * j;
            *(v4i *)(B + pl * 64 + ((slot ^ ((pl >> 2) & 3)) << 4)) = breg[j];
        }
    };

    v16i acc[TM][TP];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

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
            for (int i = 0; i < TM; ++i)
                af[i] = *(const v4i *)(A + ((wm * TM + i) * 2 + kq) * 1024 + lane * 16);
#pragma unroll
            for (int j = 0; j < TP; ++j) {
                const int pl = (wp * TP + j) * 32 + (lane & 31);
                const int sl = kq * 2 + (lane >> 5);
                bf[j] = *(const v4i *)(B + pl * 64 + ((sl ^ ((pl >> 2) & 3)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TP; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue on registers: bias, skip merge, requantise, clamp, store
    const int half = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int co0 = ct * BM + (wm * TM + i) * 32 + half * 16;
        if (co0 >= a.Cout) continue;
        const int nv = min(16, a.Cout - co0);
        int bv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) bv[r] = r < nv ? a.bias[co0 + r] : 0;
#pragma unroll
        for (int j = 0; j < TP; ++j) {
            const int p = pix0 + (wp * TP + j) * 32 + (lane & 31);
            if (p >= a.M) continue;
            int t[16];
            int64_t skip[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) t[r] = acc[i][j][r] + bv[r];
            if (a.res_mode != 0) {
                const size_t ro = (size_t)p * a.res_cs + co0;
                int rv[16];
                if (a.vec_res && nv == 16) {
                    if (a.res_dtype == 2) {
                        const v4i *rp = (const v4i *)((const int32_t *)a.res + ro);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const v4i v = rp[q];
                            rv[4 * q] = v.x; rv[4 * q + 1] = v.y; rv[4 * q + 2] = v.z; rv[4 * q + 3] = v.w;
                        }
                    } else {
                        const v4i v = *(const v4i *)((const uint8_t *)a.res + ro);
                        const int wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int b8 = (wd[r >> 2] >> ((r & 3) * 8)) & 0xff;
                            rv[r] = a.res_dtype == 1 ? (int)(int8_t)b8 : b8;
                        }
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) rv[r] = r < nv ? load_elem(a.res, ro + r, a.res_dtype) : 0;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) skip[r] = rsr64((int64_t)rv[r] * a.res_mul, a.res_shift);
                if (a.res_mode == 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) t[r] = sat32((int64_t)t[r] + skip[r]);
                }
            }
            const size_t oo = (size_t)p * a.out_cs + a.out_co + co0;
            if (a.out_mode == 3) {
                int32_t *op = (int32_t *)a.out + oo;
                if (a.vec_out && nv == 16) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        ((v4i *)op)[q] = v4i{t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (r < nv) op[r] = t[r];
                }
            } else {
                uint32_t wd[4] = {0, 0, 0, 0};
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int64_t q = rsr64((int64_t)t[r] * a.mul, a.shift);
                    if (a.res_mode == 2) q += skip[r];
                    const int v = clampi64(q, a.lo, a.hi);
                    wd[r >> 2] |= (uint32_t)(v & 0xff) << ((r & 3) * 8);
                }
                uint8_t *op = (uint8_t *)a.out + oo;
                if (a.vec_out && nv == 16) {
                    *(v4i *)op = v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (r < nv) op[r] = (uint8_t)(wd[r >> 2] >> ((r & 3) * 8));
                }
            }
        }
    }
}

template <int BM, int BP, int WAVES_M, int WAVES_P>
static hipError_t launch_cfg(const ConvArgs &a0, bool vec_in, hipStream_t st)
{
    ConvArgs a = a0;
    a.n_ct = (a.Cout + BM - 1) / BM;
    const long long blocks = (long long)a.n_ct * ((a.M + BP - 1) / BP);
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (vec_in)
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BP, WAVES_M, WAVES_P, true>), dim3((unsigned)blocks),
                           dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((conv_igemm_kernel<BM, BP, WAVES_M, WAVES_P, false>), dim3((unsigned)blocks),
                           dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_conv(const ConvArgs &a, bool vec_in, hipStream_t st)
{
    if (a.Cout <= 32) return launch_cfg<32, 256, 1, 4>(a, vec_in, st);
    if (a.Cout <= 64) return launch_cfg<64, 256, 1, 4>(a, vec_in, st);
    return launch_cfg<128, 128, 2, 2>(a, vec_in, st);
}

// One thread per 16-byte piece of the packed weight format.
__global__ void prepack_kernel(const int8_t *__restrict__ w, uint8_t *__restrict__ wp, int Cout, int K,
                               int ksteps, long long pieces)
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
            if (k < K) wd[b >> 2] |= (uint32_t)(uint8_t)w[(size_t)co * K + k] << ((b & 3) * 8);
        }
    }
    *(v4i *)(wp + e * 16) = v4i{(int)wd[0], (int)wd[1], (int)wd[2], (int)wd[3]};
}

hipError_t launch_prepack(const int8_t *w, uint8_t *wp, int Cout, int K, int chunks, int ksteps,
                          hipStream_t st)
{
    const long long pieces = (long long)chunks * ksteps * 128;
    const unsigned blocks = (unsigned)((pieces + 255) / 256);
    hipLaunchKernelGGL(prepack_kernel, dim3(blocks), dim3(256), 0, st, w, wp, Cout, K, ksteps, pieces);
    return hipGetLastError();
}

}  // namespace icnn
