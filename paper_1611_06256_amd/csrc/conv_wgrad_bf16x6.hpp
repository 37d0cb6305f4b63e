// Weight and bias gradient of a 4x4, stride-2 convolution layer on the bf16
// matrix cores at fp32 accuracy (backward pass of the network of Sec. 3.2; the
// layer is the second convolution of both networks):
//
//   dW[oc][c][u][v] = sum over frames and output pixels (i, j) of dY[oc][i][j] x[c][2i+u][2j+v]
//   db[oc]          = sum of dY[oc][i][j]
//
// The contraction runs over the output pixels of a frame.  The input falls
// into 2 x 2 stride phases P[ry][rx][c][y'][x'] = x[c][2y'+ry][2x'+rx], and
// with u = ry + 2a, v = rx + 2e the tap (u, v) meets P[ry][rx][c][i+a][j+e]:
// on the phase grid (GW = W / 2 wide) pixel (i, j) is index k = i GW + j, and
// the tap's operand is the phase plane read from index k + a GW + e on.  So
// dY goes to LDS as [oc][k] (column GW - 1 and the tail of the last group of
// 32 are zero) and every phase plane as [c][k]; both operands of an MFMA are
// eight consecutive k, and the four shifts (a, e) of a phase are cut from one
// 48-byte window of the plane: whole dwords for e = 0, a 16-bit funnel shift
// for e = 1.  Wavefront w owns phase w: 4 shifts x OC / 16 filter tiles of
// accumulators [16 filters] x [16 channels], kept over all frames of its block.
// The bias gradient is one more product, dY times a column of ones, which the
// wavefronts of channel slice 0 share by groups of 32 k.
//
// Both operands are split into three bf16 terms (x = hi + mid + lo exactly)
// while they are staged, and a product is evaluated as the six largest of the
// nine term products (dense_gemm_bf16x6.hpp): 6 x 16 cycles per 32 pixels
// instead of 8 x 32 on the fp32 instruction.
//
// A block takes 16 input channels, 16 blockIdx.y .. (gridDim.y = C / 16), and
// OCB filters, OCB blockIdx.z .. (all of them, or 32 where two blocks then fit
// a compute unit's LDS), of
// frames blockIdx.x, + gridDim.x, .. and writes its part of one partial gradient,
// part[blockIdx.x][OC][K + 1] (K = 16 C; the last column is the bias gradient,
// written by the blocks of channel slice 0), which a second kernel adds up in
// block order: no atomics, the result does not depend on timing.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"

namespace ga3c {

// OCB: filters per block (a multiple of 16; blockIdx.z takes the slices of OCB filters)
template <class SP, int OCB = SP::OC>
struct ConvWgradBf16Geom {
    static constexpr int CS = 16;
    static constexpr int GH = SP::H / 2, GW = SP::W / 2;
    static constexpr int KTOT = SP::OH * GW;                       // k = i * GW + j
    static constexpr int NKB = (KTOT + 31) / 32;                   // groups of 32 k
    static constexpr int DROW = NKB * 32 + 8;                      // bf16 per filter row of dY (52 dwords: 16 rows hit all banks)
    static constexpr int WIN = 24;                                 // elements of a plane row a lane reads per group and term
    static constexpr int PROW = NKB * 32 + WIN;                    // bf16 per channel row of a phase plane (60 dwords)
    static constexpr int MT = OCB / 16;
    static constexpr int DTERM = OCB * DROW, PTERM = 4 * CS * PROW;         // elements per term
    static constexpr int OTP = CS * 16 + 4;                        // floats per filter row of the block's result in LDS
    __host__ __device__ static constexpr int lds_bytes(bool one) {
        const int stage = (one ? 1 : 3) * (DTERM + PTERM) * 2, out = OCB * OTP * 4;
        return stage > out ? stage : out;
    }
    static constexpr int PER_CU = 2 * lds_bytes(false) <= 160 * 1024 ? 2 : 1;
};

// ONE: operands rounded to bfloat16 (the reduced-precision variant): one term, one product.
template <class SP, bool ONE, int OCB = SP::OC>
__global__ __launch_bounds__(256, (ConvWgradBf16Geom<SP, OCB>::PER_CU)) void conv_wgrad_bf16x6_kernel(const float *__restrict__ x,
                                                                                              const float *__restrict__ dy,
                                                                                              float *__restrict__ part,
                                                                                              int nframes, float scale) {
    typedef ConvWgradBf16Geom<SP, OCB> G;
    static_assert(SP::OC % OCB == 0 && OCB % 16 == 0, "whole slices of filters");
    static_assert(SP::KS == 4 && SP::S == 2, "kernel must be 4x4 with stride 2");
    static_assert(SP::C % 16 == 0 && SP::OC % 16 == 0 && SP::OC <= 256, "channels and filters in groups of 16");
    static_assert(SP::H % 2 == 0 && SP::W % 4 == 0 && G::GW % 2 == 0, "rows are read four values at a time; shifts are whole dwords");
    static_assert(G::GW + 9 <= G::WIN, "the window must hold the largest shift plus eight elements");
    static_assert(SP::OW + 1 <= G::GW && SP::OH + 1 <= G::GH, "shifted pixels must stay on the phase grid");
    static_assert((OCB * SP::NPIX) % 4 == 0 && (G::DTERM % 8) == 0 && (G::PTERM % 8) == 0, "16-byte steps");
    constexpr int CS = G::CS, GW = G::GW, NKB = G::NKB, DROW = G::DROW, PROW = G::PROW, MT = G::MT;
    constexpr int DTERM = G::DTERM, PTERM = G::PTERM, OTP = G::OTP;
    constexpr int NTERM = ONE ? 1 : 3;
    constexpr int W4 = SP::W / 4, XV = CS * SP::H * W4, XPT = (XV + 255) / 256;       // float4 of the input slice
    constexpr int NDV = OCB * SP::NPIX / 4, DPT = (NDV + 255) / 256;                   // float4 of my filters' dY
    constexpr int K1 = SP::K + 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __bf16 *dsm = (__bf16 *)smem;                      // [term][oc][DROW]
    __bf16 *psm = dsm + NTERM * DTERM;                 // [term][phase][c][PROW]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int ry = wave / 2, rx = wave % 2;
    const int c0 = blockIdx.y * CS, oc0 = blockIdx.z * OCB;

    for (int e = tid; e < NTERM * (DTERM + PTERM) / 8; e += 256) ((u32x4 *)smem)[e] = u32x4{0u, 0u, 0u, 0u};   // padding stays zero

    // staging descriptors.  Input: float4 item -> (c, y, x = 4q..4q+3): x, x+2 are neighbours in phase column 0 and
    // x+1, x+3 in phase column 1 of phase row y % 2.
    int xdst[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
        const int e = min(tid + 256 * i, XV - 1);
        const int c = e / (SP::H * W4), rem = e % (SP::H * W4), y = rem / W4, q = rem % W4;
        xdst[i] = ((y % 2) * 2 * CS + c) * PROW + (y / 2) * GW + 2 * q;
    }
    int ddst[DPT][4];
#pragma unroll
    for (int i = 0; i < DPT; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int el = min(4 * (tid + 256 * i) + j, OCB * SP::NPIX - 1);
            const int oc = el / SP::NPIX, pix = el % SP::NPIX;
            ddst[i][j] = oc * DROW + (pix / SP::OW) * GW + pix % SP::OW;
        }

    floatx4 acc[4][MT];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[s][m] = floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 bacc[MT];                                  // dY times ones: every column holds the row sums
#pragma unroll
    for (int m = 0; m < MT; ++m) bacc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
    Bf16x8Bits ones;
    ones.u = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};

    float4 xpre[XPT], dpre[DPT];
    auto fetch = [&](int f) {
        const float4 *xs = (const float4 *)(x + (size_t)f * SP::CHW + (size_t)c0 * (SP::H * SP::W));
#pragma unroll
        for (int i = 0; i < XPT; ++i) xpre[i] = xs[min(tid + 256 * i, XV - 1)];
        const float4 *ds = (const float4 *)(dy + ((size_t)f * SP::OC + oc0) * SP::NPIX);
#pragma unroll
        for (int i = 0; i < DPT; ++i) dpre[i] = ds[min(tid + 256 * i, NDV - 1)];
    };
    int f = blockIdx.x;
    fetch(min(f, nframes - 1));
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();                      // the last frame's operands have been read
#pragma unroll
        for (int i = 0; i < XPT; ++i)
            if (tid + 256 * i < XV) {
                uint32_t t0[3], t1[3];
                split3_pair(xpre[i].x, xpre[i].z, t0[0], t0[1], t0[2]);
                split3_pair(xpre[i].y, xpre[i].w, t1[0], t1[1], t1[2]);
#pragma unroll
                for (int t = 0; t < NTERM; ++t) {
                    *(uint32_t *)(psm + t * PTERM + xdst[i]) = t0[t];
                    *(uint32_t *)(psm + t * PTERM + xdst[i] + CS * PROW) = t1[t];
                }
            }
#pragma unroll
        for (int i = 0; i < DPT; ++i)
            if (tid + 256 * i < NDV) {
                uint32_t t0[3], t1[3];
                split3_pair(dpre[i].x, dpre[i].y, t0[0], t0[1], t0[2]);
                split3_pair(dpre[i].z, dpre[i].w, t1[0], t1[1], t1[2]);
                uint16_t *dst = (uint16_t *)dsm;
#pragma unroll
                for (int t = 0; t < NTERM; ++t) {
                    dst[t * DTERM + ddst[i][0]] = (uint16_t)(t0[t] & 0xffffu);
                    dst[t * DTERM + ddst[i][1]] = (uint16_t)(t0[t] >> 16);
                    dst[t * DTERM + ddst[i][2]] = (uint16_t)(t1[t] & 0xffffu);
                    dst[t * DTERM + ddst[i][3]] = (uint16_t)(t1[t] >> 16);
                }
            }
        __syncthreads();
        fetch(min(f + (int)gridDim.x, nframes - 1));
        // the loads above go out before the products start (the compiler would otherwise sink them below the MFMAs)
        __builtin_amdgcn_sched_barrier(0);
        constexpr int NPROD = ONE ? 1 : 6;
        constexpr int PA[6] = {2, 1, 0, 1, 0, 0}, PB[6] = {0, 1, 2, 0, 1, 0};      // smallest products first
        // the operand reads of the next group of 32 k are issued before the products of this one
        Bf16x8Bits a[2][MT][NTERM];
        u32x4 win[2][NTERM][3];
        auto read_operands = [&](int kb, Bf16x8Bits (&ad)[MT][NTERM], u32x4 (&wd)[NTERM][3]) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < NTERM; ++t)
                    ad[m][t].u = *(const u32x4 *)(dsm + t * DTERM + (m * 16 + l16) * DROW + 32 * kb + 8 * g);
#pragma unroll
            for (int t = 0; t < NTERM; ++t) {
                const u32x4 *src = (const u32x4 *)(psm + t * PTERM + (wave * CS + l16) * PROW + 32 * kb + 8 * g);
                wd[t][0] = src[0]; wd[t][1] = src[1]; wd[t][2] = src[2];
            }
        };
        read_operands(0, a[0], win[0]);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            if (kb + 1 < NKB) read_operands(kb + 1, a[(kb + 1) & 1], win[(kb + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            Bf16x8Bits b[4][NTERM];
#pragma unroll
            for (int t = 0; t < NTERM; ++t) {
                const u32x4 w0 = win[kb & 1][t][0], w1 = win[kb & 1][t][1], w2 = win[kb & 1][t][2];
                const uint32_t dw[12] = {w0[0], w0[1], w0[2], w0[3], w1[0], w1[1], w1[2], w1[3], w2[0], w2[1], w2[2], w2[3]};
#pragma unroll
                for (int av = 0; av < 2; ++av) {
                    const int o = av * (GW / 2);          // a shift of a rows of the phase grid is GW / 2 dwords
                    b[2 * av][t].u = u32x4{dw[o], dw[o + 1], dw[o + 2], dw[o + 3]};
                    b[2 * av + 1][t].u = u32x4{__builtin_amdgcn_alignbit(dw[o + 1], dw[o], 16), __builtin_amdgcn_alignbit(dw[o + 2], dw[o + 1], 16),
                                               __builtin_amdgcn_alignbit(dw[o + 3], dw[o + 2], 16), __builtin_amdgcn_alignbit(dw[o + 4], dw[o + 3], 16)};
                }
            }
            if (blockIdx.y == 0 && kb % 4 == wave) {      // bias: the terms add up to dY exactly, smallest first
#pragma unroll
                for (int t = NTERM - 1; t >= 0; --t)
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        bacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kb & 1][m][t].v, ones.v, bacc[m], 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < NPROD; ++q) {
                const int ai = ONE ? 0 : PA[q], bi = ONE ? 0 : PB[q];
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        acc[s][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kb & 1][m][ai % NTERM].v, b[s][bi % NTERM].v, acc[s][m], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    }
    // lane (l16, g), register r of acc[s = 2a + e][m]: filter 16 m + 4 g + r, channel c0 + l16, tap (ry + 2a, rx + 2e).
    // The block's result is put together in LDS and leaves in rows.
    __syncthreads();
    float *ot = (float *)smem;                         // [oc][OTP]
    __shared__ float bsh[4][OCB];                      // bias sums of the four wavefronts
    if (l16 == 0) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) bsh[wave][m * 16 + 4 * g + r] = bacc[m][r];
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int u = ry + 2 * (s / 2), v = rx + 2 * (s % 2);
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) ot[(m * 16 + 4 * g + r) * OTP + l16 * 16 + u * 4 + v] = acc[s][m][r];
    }
    __syncthreads();
    typedef float f32x4_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));
    float *pb = part + ((size_t)blockIdx.x * SP::OC + oc0) * K1 + c0 * 16;
    for (int it = tid; it < OCB * CS * 4; it += 256) {
        const int oc = it / (CS * 4), kq = it % (CS * 4);
        const float4 v = *(const float4 *)(ot + oc * OTP + 4 * kq);
        *(f32x4_dword_aligned *)(pb + (size_t)oc * K1 + 4 * kq) = f32x4_dword_aligned{v.x * scale, v.y * scale, v.z * scale, v.w * scale};
    }
    if (blockIdx.y == 0 && tid < OCB)
        part[((size_t)blockIdx.x * SP::OC + oc0 + tid) * K1 + SP::K] = (bsh[0][tid] + bsh[1][tid]) + (bsh[2][tid] + bsh[3][tid]);
}

// One partial dW per block: fewer blocks where a partial is large.
template <class SP>
inline int conv_wgrad_bf16x6_blocks(int nframes) {
    constexpr int LIMIT = SP::OC * (SP::K + 1) > 16384 ? 256 : 512;
    return nframes < LIMIT ? nframes : LIMIT;
}

// x: [n][C][H][W] and dy: [n][OC][OH][OW], both 16-byte aligned; part: [conv_wgrad_bf16x6_blocks(n)][OC][K + 1].
template <class SP, int OCB = SP::OC>
inline hipError_t launch_conv_wgrad_bf16x6(const float *x, const float *dy, float *part, int nframes, float scale,
                                           hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    typedef ConvWgradBf16Geom<SP, OCB> G;
    static bool attr_set = false;          // once per layer shape: let the kernels use more than 64 KB of LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_wgrad_bf16x6_kernel<SP, false, OCB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(false));
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_wgrad_bf16x6_kernel<SP, true, OCB>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(true));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const dim3 grid(conv_wgrad_bf16x6_blocks<SP>(nframes), SP::C / 16, SP::OC / OCB);
    if (rb)
        ga3c::launch((conv_wgrad_bf16x6_kernel<SP, true, OCB>), grid, dim3(256), G::lds_bytes(true), s, x, dy, part, nframes, scale);
    else
        ga3c::launch((conv_wgrad_bf16x6_kernel<SP, false, OCB>), grid, dim3(256), G::lds_bytes(false), s, x, dy, part, nframes, scale);
    return hipGetLastError();
}

}  // namespace ga3c
