// Second convolution layer of the small network (32 filters 4x4 stride 2 on
// 16x20x20 activations; paper Sec. 3.2) on the bf16 matrix cores at fp32
// accuracy: activations and filters are split into three bf16 terms each and
// the six largest term products are accumulated in fp32 (see
// dense_gemm_bf16x6.hpp for the error argument).  The frame sits in LDS as
// three bf16 planes, the split filters in registers.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"

namespace ga3c {

// y[b][oc][pix] = max(0, sum_k W[oc][k] x[b][tap k at pix] + bias[oc]).
// Block = 4 wavefronts; wave w: filter tile w % 2, pixel tiles w/2, w/2 + 2, w/2 + 4.
// A lane (pixel p, group g) supplies, for tap block kb, the 8 taps
// k = 32 kb + 8 g + e: channel 2 kb + g/2, filter rows 2 (g%2) and 2 (g%2) + 1, 4 columns.
__global__ __launch_bounds__(256, 2) void conv2_bf16x6_fwd_kernel(const float *__restrict__ x,
                                                                  const float *__restrict__ w,
                                                                  const float *__restrict__ bias, float *__restrict__ y,
                                                                  int nframes, int rb) {
    constexpr int C = 16, H = 20, W = 20, OC = 32, S = 2, OW = 9, NPIX = 81, K = 256, CHW = C * H * W;
    constexpr int NV = CHW / 4, VPT = (NV + 255) / 256;      // float4 per frame / per thread
    constexpr int TPW = 3;
    __shared__ __attribute__((aligned(16))) __bf16 xs[3][VPT * 256 * 4];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int ot = wave % 2;

    bf16x8 wq[3][8];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) {
        const float *src = w + (size_t)(ot * 16 + l16) * K + 32 * kb + 8 * g;
        const float4 a = *(const float4 *)src, b = *(const float4 *)(src + 4);
        const float f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __bf16 h, m, l;
            split3(f[e], h, m, l, rb);
            wq[0][kb][e] = h; wq[1][kb][e] = m; wq[2][kb][e] = l;
        }
    }
    float bv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = bias[ot * 16 + 4 * g + r];

    int pixbase[TPW], pixidx[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        int p = (wave / 2 + 2 * i) * 16 + l16;
        pixidx[i] = p < NPIX ? p : -1;
        if (p >= NPIX) p = 0;
        // element (channel g/2 of the pair, row 2*(g%2), column 0) of the window of pixel p
        pixbase[i] = (g / 2) * (H * W) + ((p / OW) * S + 2 * (g % 2)) * W + (p % OW) * S;
    }
    int vidx[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) vidx[i] = min(tid + 256 * i, NV - 1);

    float4 pre[VPT];
    int f = blockIdx.x;
    {
        const float4 *src = (const float4 *)(x + (size_t)min(f, nframes - 1) * CHW);
#pragma unroll
        for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
    }
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const float v[4] = {pre[i].x, pre[i].y, pre[i].z, pre[i].w};
            union { __bf16 h[4]; uint2 u; } o[3];
#pragma unroll
            for (int t = 0; t < 4; ++t) split3(v[t], o[0].h[t], o[1].h[t], o[2].h[t], rb);
#pragma unroll
            for (int term = 0; term < 3; ++term) *(uint2 *)(&xs[term][(tid + 256 * i) * 4]) = o[term].u;
        }
        __syncthreads();
        {
            const float4 *src = (const float4 *)(x + (size_t)min(f + (int)gridDim.x, nframes - 1) * CHW);
#pragma unroll
            for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
        }
        floatx4 acc[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int off = pixbase[i] + 2 * kb * (H * W);       // even: 4-byte aligned in bf16
                Bf16x8Bits xv[3];
#pragma unroll
                for (int term = 0; term < 3; ++term) {
                    const uint32_t *r0 = (const uint32_t *)(&xs[term][off]);
                    const uint32_t *r1 = (const uint32_t *)(&xs[term][off + W]);
                    xv[term].u = u32x4{r0[0], r0[1], r1[0], r1[1]};
                }
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[2][kb], xv[0].v, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[1][kb], xv[1].v, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[0][kb], xv[2].v, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[1][kb], xv[0].v, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[0][kb], xv[1].v, acc[i], 0, 0, 0);
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[0][kb], xv[0].v, acc[i], 0, 0, 0);
            }
        }
        float *yb = y + (size_t)f * OC * NPIX;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            if (pixidx[i] >= 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float v = acc[i][r] + bv[r];
                    yb[(ot * 16 + 4 * g + r) * NPIX + pixidx[i]] = v > 0.f ? v : 0.f;
                }
            }
        }
    }
}

inline hipError_t launch_conv2_bf16x6_fwd(const float *x, const float *w, const float *bias, float *y, int nframes,
                                          hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    const int grid = nframes < 512 ? nframes : 512;
    ga3c::launch(conv2_bf16x6_fwd_kernel, dim3(grid), dim3(256), 0, s, x, w, bias, y, nframes, rb);
    return hipGetLastError();
}

}  // namespace ga3c
