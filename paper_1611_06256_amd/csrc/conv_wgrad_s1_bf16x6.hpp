// Weight and bias gradient of a stride-1 convolution layer with 64 input
// channels (the third layer of the larger network) on the bf16 matrix cores at
// fp32 accuracy:
//
//   dW[oc][c][u][v] = sum over frames and output pixels (i, j) of dY[oc][i][j] x[c][i+u][j+v]
//   db[oc]          = sum of dY[oc][i][j]
//
// The contraction runs over the output pixels of a frame, numbered on the
// input's grid: pixel (i, j) is k = i W + j, so that tap (u, v) meets the input
// plane read from index k + u W + v on.  dY goes to LDS as [oc][k] (columns OW
// .. W - 1 and the tail of the last group of 32 are zero) and the input as
// [c][k]; both operands of an MFMA are eight consecutive k, and all KS x KS
// shifts of a channel are cut from one 64-byte window of its plane: whole
// dwords for even shifts, a 16-bit funnel shift for odd ones.  Wavefront w owns
// the channels 16 w .. 16 w + 15: KS x KS taps x 2 filter tiles of accumulators
// [16 filters] x [16 channels], kept over all frames of its block.  The bias
// gradient is one more product, dY times a column of ones.
//
// Both operands are split into three bf16 terms (x = hi + mid + lo exactly)
// while they are staged, and a product is evaluated as the six largest of the
// nine term products (dense_gemm_bf16x6.hpp).
//
// A block takes 32 filters, 32 blockIdx.y .. (gridDim.y = OC / 32), of frames
// blockIdx.x, + gridDim.x, .. and writes its rows of one partial gradient,
// part[blockIdx.x][OC][K + 1] (the last column is the bias gradient), which a
// second kernel adds up in block order: no atomics, the result does not depend
// on timing.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"

namespace ga3c {

template <class SP>
struct ConvWgradS1Bf16Geom {
    static constexpr int MS = 2;                                   // filter tiles of 16 per block
    static constexpr int KTOT = (SP::OH - 1) * SP::W + SP::OW;     // k = i * W + j
    static constexpr int NKB = (KTOT + 31) / 32;                   // groups of 32 k
    static constexpr int DROW = NKB * 32 + 8;                      // bf16 per filter row of dY (36 dwords: 16 rows hit all banks)
    static constexpr int WIN = 32;                                 // elements of a plane row a lane reads per group and term
    static constexpr int SHIFT = (SP::KS - 1) * SP::W + SP::KS - 1;         // the largest shift
    static constexpr int PROW = ((NKB * 32 + WIN - 8) / 8) * 8 + 16;        // bf16 per channel row of the input (52 dwords)
    static constexpr int DTERM = MS * 16 * DROW, PTERM = SP::C * PROW;      // elements per term
    static constexpr int OTP = SP::K + 4;                          // floats per filter row of a tile's result in LDS
    __host__ __device__ static constexpr int lds_bytes(bool one) {
        const int stage = (one ? 1 : 3) * (DTERM + PTERM) * 2, out = 16 * OTP * 4;
        return stage > out ? stage : out;
    }
};

// ONE: operands rounded to bfloat16 (the reduced-precision variant): one term, one product.
template <class SP, bool ONE>
__global__ __launch_bounds__(256, 2) void conv_wgrad_s1_bf16x6_kernel(const float *__restrict__ x, const float *__restrict__ dy,
                                                                      float *__restrict__ part, int nframes, float scale) {
    typedef ConvWgradS1Bf16Geom<SP> G;
    static_assert(SP::S == 1 && SP::C == 64 && SP::OC % 32 == 0, "stride 1, 64 channels in (16 per wavefront), filters in groups of 32");
    static_assert(G::SHIFT + 8 <= G::WIN && G::NKB * 32 - 8 + G::WIN <= G::PROW, "the window holds every shift and stays in its row");
    static_assert(SP::H * SP::W <= G::PROW, "a plane fits its row");
    static_assert((SP::CHW % 4) == 0 && (32 * SP::NPIX) % 4 == 0 && (G::DTERM % 8) == 0 && (G::PTERM % 8) == 0, "16-byte steps");
    static_assert((G::PROW / 2) % 8 == 4 && (G::DROW / 2) % 8 == 4, "16 rows of 16 bytes must fall on all banks");
    constexpr int MS = G::MS, NKB = G::NKB, DROW = G::DROW, PROW = G::PROW, KS = SP::KS, NTAP = KS * KS;
    constexpr int DTERM = G::DTERM, PTERM = G::PTERM, OTP = G::OTP, HW = SP::H * SP::W;
    constexpr int NTERM = ONE ? 1 : 3;
    constexpr int XV = SP::CHW / 4, XPT = (XV + 255) / 256;                // float4 of the input frame
    constexpr int NDV = MS * 16 * SP::NPIX / 4, DPT = (NDV + 255) / 256;    // float4 of my filters' dY
    constexpr int K1 = SP::K + 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __bf16 *dsm = (__bf16 *)smem;                      // [term][oc][DROW]
    __bf16 *psm = dsm + NTERM * DTERM;                 // [term][c][PROW]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int oc0 = blockIdx.y * MS * 16;

    for (int e = tid; e < NTERM * (DTERM + PTERM) / 8; e += 256) ((u32x4 *)smem)[e] = u32x4{0u, 0u, 0u, 0u};   // padding stays zero

    // staging descriptors: element -> its place in LDS (term 0)
    int xdst[XPT][4], ddst[DPT][4];
#pragma unroll
    for (int i = 0; i < XPT; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int el = min(4 * (tid + 256 * i) + j, SP::CHW - 1);
            xdst[i][j] = (el / HW) * PROW + el % HW;
        }
#pragma unroll
    for (int i = 0; i < DPT; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int el = min(4 * (tid + 256 * i) + j, MS * 16 * SP::NPIX - 1);
            const int oc = el / SP::NPIX, pix = el % SP::NPIX;
            ddst[i][j] = oc * DROW + (pix / SP::OW) * SP::W + pix % SP::OW;
        }

    floatx4 acc[NTAP][MS], bacc[MS];
#pragma unroll
    for (int m = 0; m < MS; ++m) {
        bacc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NTAP; ++s) acc[s][m] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    Bf16x8Bits ones;
    ones.u = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};

    float4 xpre[XPT], dpre[DPT];
    auto fetch = [&](int f) {
        const float4 *xs = (const float4 *)(x + (size_t)f * SP::CHW);
#pragma unroll
        for (int i = 0; i < XPT; ++i) xpre[i] = xs[min(tid + 256 * i, XV - 1)];
        const float4 *ds = (const float4 *)(dy + ((size_t)f * SP::OC + oc0) * SP::NPIX);
#pragma unroll
        for (int i = 0; i < DPT; ++i) dpre[i] = ds[min(tid + 256 * i, NDV - 1)];
    };
    auto stash4 = [&](const float4 v, __bf16 *base, int tstride, const int (&dst)[4]) {
        uint32_t t0[3], t1[3];
        split3_pair(v.x, v.y, t0[0], t0[1], t0[2]);
        split3_pair(v.z, v.w, t1[0], t1[1], t1[2]);
        uint16_t *o = (uint16_t *)base;
#pragma unroll
        for (int t = 0; t < NTERM; ++t) {
            o[t * tstride + dst[0]] = (uint16_t)(t0[t] & 0xffffu);
            o[t * tstride + dst[1]] = (uint16_t)(t0[t] >> 16);
            o[t * tstride + dst[2]] = (uint16_t)(t1[t] & 0xffffu);
            o[t * tstride + dst[3]] = (uint16_t)(t1[t] >> 16);
        }
    };
    int f = blockIdx.x;
    fetch(min(f, nframes - 1));
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();                      // the last frame's operands have been read
#pragma unroll
        for (int i = 0; i < XPT; ++i)
            if (tid + 256 * i < XV) stash4(xpre[i], psm, PTERM, xdst[i]);
#pragma unroll
        for (int i = 0; i < DPT; ++i)
            if (tid + 256 * i < NDV) stash4(dpre[i], dsm, DTERM, ddst[i]);
        __syncthreads();
        fetch(min(f + (int)gridDim.x, nframes - 1));
        // the loads above go out before the products start (the compiler would otherwise sink them below the MFMAs)
        __builtin_amdgcn_sched_barrier(0);
        constexpr int NPROD = ONE ? 1 : 6;
        constexpr int PA[6] = {2, 1, 0, 1, 0, 0}, PB[6] = {0, 1, 2, 0, 1, 0};      // smallest products first
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            Bf16x8Bits a[MS][NTERM];
            uint32_t dw[NTERM][16];
#pragma unroll
            for (int m = 0; m < MS; ++m)
#pragma unroll
                for (int t = 0; t < NTERM; ++t)
                    a[m][t].u = *(const u32x4 *)(dsm + t * DTERM + (m * 16 + l16) * DROW + 32 * kb + 8 * g);
#pragma unroll
            for (int t = 0; t < NTERM; ++t) {
                const u32x4 *src = (const u32x4 *)(psm + t * PTERM + (wave * 16 + l16) * PROW + 32 * kb + 8 * g);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const u32x4 w = src[q];
                    dw[t][4 * q] = w[0]; dw[t][4 * q + 1] = w[1]; dw[t][4 * q + 2] = w[2]; dw[t][4 * q + 3] = w[3];
                }
            }
            if (kb % 4 == wave) {             // bias: the terms add up to dY exactly, smallest first
#pragma unroll
                for (int t = NTERM - 1; t >= 0; --t)
#pragma unroll
                    for (int m = 0; m < MS; ++m)
                        bacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m][t].v, ones.v, bacc[m], 0, 0, 0);
            }
            // one row of taps at a time: KS shifts x MS filter tiles of independent accumulators
#pragma unroll
            for (int u = 0; u < KS; ++u) {
                Bf16x8Bits b[KS][NTERM];
#pragma unroll
                for (int v = 0; v < KS; ++v) {
                    const int sh = u * SP::W + v, o = sh / 2;
#pragma unroll
                    for (int t = 0; t < NTERM; ++t) {
                        if (sh % 2 == 0)
                            b[v][t].u = u32x4{dw[t][o], dw[t][o + 1], dw[t][o + 2], dw[t][o + 3]};
                        else
                            b[v][t].u = u32x4{__builtin_amdgcn_alignbit(dw[t][o + 1], dw[t][o], 16), __builtin_amdgcn_alignbit(dw[t][o + 2], dw[t][o + 1], 16),
                                              __builtin_amdgcn_alignbit(dw[t][o + 3], dw[t][o + 2], 16), __builtin_amdgcn_alignbit(dw[t][o + 4], dw[t][o + 3], 16)};
                    }
                }
#pragma unroll
                for (int q = 0; q < NPROD; ++q) {
                    const int ai = ONE ? 0 : PA[q], bi = ONE ? 0 : PB[q];
#pragma unroll
                    for (int v = 0; v < KS; ++v)
#pragma unroll
                        for (int m = 0; m < MS; ++m)
                            acc[u * KS + v][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m][ai % NTERM].v, b[v][bi % NTERM].v,
                                                                                         acc[u * KS + v][m], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
    }
    // lane (l16, g), register r of acc[tap][m]: filter oc0 + 16 m + 4 g + r, channel 16 wave + l16.  One filter tile at a
    // time is put together in LDS and leaves in rows.
    __shared__ float bsh[4][MS * 16];                  // bias sums of the four wavefronts
    float *ot = (float *)smem;                         // [16 filters][OTP]
    typedef float f32x4_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));
#pragma unroll
    for (int m = 0; m < MS; ++m) {
        __syncthreads();
        if (l16 == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) bsh[wave][m * 16 + 4 * g + r] = bacc[m][r];
        }
#pragma unroll
        for (int s = 0; s < NTAP; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) ot[(4 * g + r) * OTP + (wave * 16 + l16) * NTAP + s] = acc[s][m][r];
        __syncthreads();
        float *pb = part + ((size_t)blockIdx.x * SP::OC + oc0 + m * 16) * K1;
        for (int it = tid; it < 16 * (SP::K / 4); it += 256) {
            const int oc = it / (SP::K / 4), kq = it % (SP::K / 4);
            const float4 v = *(const float4 *)(ot + oc * OTP + 4 * kq);
            *(f32x4_dword_aligned *)(pb + (size_t)oc * K1 + 4 * kq) = f32x4_dword_aligned{v.x * scale, v.y * scale, v.z * scale, v.w * scale};
        }
    }
    if (tid < MS * 16)
        part[((size_t)blockIdx.x * SP::OC + oc0 + tid) * K1 + SP::K] = (bsh[0][tid] + bsh[1][tid]) + (bsh[2][tid] + bsh[3][tid]);
}

// One partial dW per block: fewer blocks where a partial is large.
template <class SP>
inline int conv_wgrad_s1_bf16x6_blocks(int nframes) {
    constexpr int LIMIT = SP::OC * (SP::K + 1) > 16384 ? 256 : 512;
    return nframes < LIMIT ? nframes : LIMIT;
}

// x: [n][C][H][W] and dy: [n][OC][OH][OW], both 16-byte aligned; part: [conv_wgrad_s1_bf16x6_blocks(n)][OC][K + 1].
template <class SP>
inline hipError_t launch_conv_wgrad_s1_bf16x6(const float *x, const float *dy, float *part, int nframes, float scale,
                                              hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    typedef ConvWgradS1Bf16Geom<SP> G;
    static bool attr_set = false;          // once per layer shape: let the kernels use more than 64 KB of LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_wgrad_s1_bf16x6_kernel<SP, false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(false));
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_wgrad_s1_bf16x6_kernel<SP, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(true));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid(conv_wgrad_s1_bf16x6_blocks<SP>(nframes), SP::OC / 32);
    if (rb)
        ga3c::launch((conv_wgrad_s1_bf16x6_kernel<SP, true>), grid, dim3(256), G::lds_bytes(true), s, x, dy, part, nframes, scale);
    else
        ga3c::launch((conv_wgrad_s1_bf16x6_kernel<SP, false>), grid, dim3(256), G::lds_bytes(false), s, x, dy, part, nframes, scale);
    return hipGetLastError();
}

}  // namespace ga3c
