// Frame-resident weight-gradient kernels on the fp32 matrix cores, compiled for
// a fixed layer geometry (the layers of the networks
// of Sec. 3.2 and of the larger network of the workload list).
//
// One block keeps a whole input frame (and the layer's output gradient) in LDS
// and walks over the frames assigned to it, so that every byte of the frame is
// fetched from HBM once and the im2col gather happens between LDS and
// registers.  The products run on v_mfma_f32_16x16x4_f32.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "gemm_mfma.hpp"

namespace ga3c {

template <class TIn_, int C_, int H_, int W_, int OC_, int KS_, int S_>
struct ConvSpec {
    typedef TIn_ TIn;
    static constexpr int C = C_, H = H_, W = W_, OC = OC_, KS = KS_, S = S_;
    static constexpr int OH = (H - KS) / S + 1, OW = (W - KS) / S + 1;
    static constexpr int K = C * KS * KS, NPIX = OH * OW, CHW = C * H * W;
    static constexpr int NT = (NPIX + 15) / 16;      // pixel tiles per frame
    static constexpr int OT = OC / 16;               // filter tiles
    static_assert(OC % 16 == 0 && (OT == 1 || OT == 2 || OT == 4), "filter count must be 16, 32 or 64");
    static_assert(K % 16 == 0, "filter length must be a multiple of 16");
    // element offset inside a frame of filter tap k = (c, u, v)
    __host__ __device__ static constexpr int koff(int k) {
        return (k / (KS * KS)) * H * W + ((k / KS) % KS) * W + (k % KS);
    }
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Four floats held as raw bits, each rounded to bfloat16 and back (the
// reduced-precision variant rounds float operands while they are staged; bytes
// are exact and pass unchanged).
template <class TIn>
__device__ __forceinline__ u32x4 stage_round(u32x4 v, int rb) {
    if (sizeof(TIn) == 4 && rb) {
#pragma unroll
        for (int d = 0; d < 4; ++d) v[d] = __float_as_uint(bf16_rne(__uint_as_float(v[d])));
    }
    return v;
}

__device__ __forceinline__ floatx4 mfma4(float a, float b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Weight and bias gradient of the same layers.
//   dW[oc][k] = sum over frames and output pixels of dY[oc][pix] * x[tap k at pix]
//   db[oc]    = sum of dY[oc][pix]
// The sum over pixels is the contraction index of the MFMA (4 pixels per
// instruction, one per lane group), the filters are the rows and 16 filter
// taps the columns of an output tile.  A wave owns K/64 tap tiles times all
// filter tiles and keeps them in registers over all frames of its block; each
// block then writes one partial dW, which a second kernel adds up in block
// order (no atomics, so the result does not depend on timing).
// part: [gridDim.x][OC][K+1], the last column is the bias gradient.
// KSL > 1 cuts the filter taps into KSL slices (blockIdx.y) where one block's
// accumulators for all of them would not fit the register file.
template <class SP, int KSL = 1, int NW = 4>
__global__ __launch_bounds__(64 * NW, 2) void conv_wgrad_frame_kernel(const typename SP::TIn *__restrict__ x,
                                                                  const float *__restrict__ dy,
                                                                  float *__restrict__ part, int nframes, float scale,
                                                                  int rb) {
    // rb: dY and (float) frames are rounded to bfloat16 on their way to LDS; the bias sums take the rounded dY
    typedef typename SP::TIn TIn;
    constexpr int FRAME_BYTES = SP::CHW * (int)sizeof(TIn);
    constexpr int NTHR = 64 * NW;                                // NW wavefronts share the tap tiles
    constexpr int NV = FRAME_BYTES / 16, VPT = (NV + NTHR - 1) / NTHR;
    constexpr int NS = (SP::NPIX + 3) / 4;                       // contraction steps per frame
    constexpr int DPITCH = ((4 * NS + 31) / 32) * 32 + 4;        // row pitch of dY in LDS: 4 mod 32 banks
    constexpr int NDY = SP::OC * SP::NPIX, DPT = (NDY + NTHR - 1) / NTHR;
    constexpr int KT = SP::K / 16, KTW = KT / (NW * KSL);        // tap tiles in all / per wave
    static_assert(KT % (NW * KSL) == 0, "tap tiles must split evenly over the slices and waves");
    static_assert(256 % SP::OC == 0, "bias sums use 256/OC threads per filter");
    constexpr int TPO = 256 / SP::OC;                            // threads per filter in the bias sum
    __shared__ __attribute__((aligned(16))) unsigned char xs_raw[VPT * NTHR * 16];
    __shared__ __attribute__((aligned(16))) float ds[SP::OC * DPITCH];
    const TIn *xs = (const TIn *)xs_raw;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;

    for (int e = tid; e < SP::OC * DPITCH; e += NTHR) ds[e] = 0.f;   // the padding stays zero

    int tapoff[KTW];                                             // my tap in each of my tiles
#pragma unroll
    for (int t = 0; t < KTW; ++t) tapoff[t] = SP::koff(16 * ((blockIdx.y * NW + wave) * KTW + t) + l16);
    // pixel 4s+g of a frame -> offset of its window
    int pixoff[SP::OW % 4 == 0 ? 1 : NS];
    if (SP::OW % 4 != 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            int p = 4 * s + g;
            if (p >= SP::NPIX) p = 0;                             // dY is zero there
            pixoff[SP::OW % 4 == 0 ? 0 : s] = (p / SP::OW) * SP::S * SP::W + (p % SP::OW) * SP::S;
        }
    }
    int vidx[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) vidx[i] = min(tid + NTHR * i, NV - 1);
    int didx[DPT], dlds[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) {
        const int e = min(tid + NTHR * i, NDY - 1);
        didx[i] = e;
        dlds[i] = (e / SP::NPIX) * DPITCH + e % SP::NPIX;
    }

    floatx4 acc[SP::OT][KTW];
#pragma unroll
    for (int o = 0; o < SP::OT; ++o)
#pragma unroll
        for (int t = 0; t < KTW; ++t) acc[o][t] = floatx4{0.f, 0.f, 0.f, 0.f};
    float bsum = 0.f;

    u32x4 pre[VPT];
    float dpre[DPT];
    int f = blockIdx.x;
    {
        const int ff = min(f, nframes - 1);
        const u32x4 *src = (const u32x4 *)(x + (size_t)ff * SP::CHW);
#pragma unroll
        for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
        const float *dsrc = dy + (size_t)ff * NDY;
#pragma unroll
        for (int i = 0; i < DPT; ++i) dpre[i] = dsrc[didx[i]];
    }
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < VPT; ++i) ((u32x4 *)xs_raw)[tid + NTHR * i] = stage_round<TIn>(pre[i], rb);
#pragma unroll
        for (int i = 0; i < DPT; ++i) ds[dlds[i]] = rb ? bf16_rne(dpre[i]) : dpre[i];
        __syncthreads();
        {
            const int ff = min(f + (int)gridDim.x, nframes - 1);
            const u32x4 *src = (const u32x4 *)(x + (size_t)ff * SP::CHW);
#pragma unroll
            for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
            const float *dsrc = dy + (size_t)ff * NDY;
#pragma unroll
            for (int i = 0; i < DPT; ++i) dpre[i] = dsrc[didx[i]];
        }
        if (tid < 256) {   // bias: TPO threads share a filter row, combined in lane order
            const int oc = tid / TPO, part_id = tid % TPO;
            float sum = 0.f;
            for (int pp = part_id; pp < SP::NPIX; pp += TPO) sum += ds[oc * DPITCH + pp];
#pragma unroll
            for (int o = TPO / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
            bsum += sum;
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            int po;
            if (SP::OW % 4 == 0) {
                constexpr int dummy = 0; (void)dummy;
                po = ((4 * s) / SP::OW) * SP::S * SP::W + ((4 * s) % SP::OW + g) * SP::S;
            } else {
                po = pixoff[SP::OW % 4 == 0 ? 0 : s];
            }
            float a[SP::OT];
#pragma unroll
            for (int o = 0; o < SP::OT; ++o) a[o] = ds[(o * 16 + l16) * DPITCH + 4 * s + g];
#pragma unroll
            for (int t = 0; t < KTW; ++t) {
                const float b = (float)xs[po + tapoff[t]];
#pragma unroll
                for (int o = 0; o < SP::OT; ++o) acc[o][t] = mfma4(a[o], b, acc[o][t]);
            }
        }
    }
    // lane (l16, g) register r of tile (o, t): filter o*16 + 4g + r, tap 16*((slice*NW+wave)*KTW+t) + l16
    float *pb = part + (size_t)blockIdx.x * SP::OC * (SP::K + 1);
#pragma unroll
    for (int o = 0; o < SP::OT; ++o)
#pragma unroll
        for (int t = 0; t < KTW; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                pb[(o * 16 + 4 * g + r) * (SP::K + 1) + 16 * ((blockIdx.y * NW + wave) * KTW + t) + l16] = acc[o][t][r] * scale;
    if (blockIdx.y == 0 && tid < 256 && tid % TPO == 0) pb[(tid / TPO) * (SP::K + 1) + SP::K] = bsum;
}

// One partial dW per block: fewer blocks where a partial is large.
template <class SP>
inline int conv_wgrad_frame_blocks(int nframes) {
    constexpr int LIMIT = SP::OC * (SP::K + 1) > 16384 ? 256 : 512;
    return nframes < LIMIT ? nframes : LIMIT;
}

template <class SP, int KSL = 1, int NW = 4>
inline hipError_t launch_conv_wgrad_frame(const typename SP::TIn *x, const float *dy, float *part, int nframes,
                                          float scale, hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    ga3c::launch((conv_wgrad_frame_kernel<SP, KSL, NW>), dim3(conv_wgrad_frame_blocks<SP>(nframes), KSL), dim3(64 * NW), 0,
                       s, x, dy, part, nframes, scale, rb);
    return hipGetLastError();
}


}  // namespace ga3c
