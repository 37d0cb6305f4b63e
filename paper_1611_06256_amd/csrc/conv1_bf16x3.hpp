// First convolution layer (8x8 filters, stride 4, on 4x84x84 byte frames;
// paper Sec. 3.2) on the bf16 matrix cores without losing fp32 accuracy.
//
// A byte 0..255 has at most 8 significant bits, which is exactly what a bf16
// holds, so the frame converts to bf16 without rounding.  An fp32 number is the
// exact sum of three bf16 numbers (hi + mid + lo, 8 bits each).  The product of
// a byte and a bf16 term has 16 bits and is exact in the fp32 accumulator.  So
//   sum_k W[k] x[k] = sum_k (hi[k] + mid[k] + lo[k]) x[k]
// evaluated with three v_mfma_f32_16x16x32_bf16 per 32 taps rounds only where
// the fp32 MFMA path rounds too (in the accumulation), at 5x its rate.  The
// layer then runs at the speed of fetching frames and storing activations.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include <type_traits>

#include "conv_frame.hpp"

namespace ga3c {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

union Bf16x8Bits {
    bf16x8 v;
    u32x4 u;
};

// Sum step inside a row of 16 lanes (DPP control CTRL).
template <int CTRL>
__device__ __forceinline__ float dpp_row_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// hi/mid/lo with f == hi + mid + lo exactly (round-to-nearest-even casts).
__device__ __forceinline__ void split3(float f, __bf16 &hi, __bf16 &mid, __bf16 &lo) {
    hi = (__bf16)f;
    const float r1 = f - (float)hi;
    mid = (__bf16)r1;
    lo = (__bf16)(r1 - (float)mid);
}
// The same with a switch: rb != 0 keeps only hi, i.e. the operand rounded to
// bfloat16 (the reduced-precision variant of the network); the kernels then
// multiply zeros in the other two terms.
__device__ __forceinline__ void split3(float f, __bf16 &hi, __bf16 &mid, __bf16 &lo, int rb) {
    split3(f, hi, mid, lo);
    if (rb) { mid = (__bf16)0.f; lo = (__bf16)0.f; }
}

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// two floats -> two bfloat16 (round to nearest even) in one register, x in the low half
__device__ __forceinline__ uint32_t pack_bf16_rne(float x, float y) {
    union { bf16x2_t v; uint32_t u; } c;
    c.v = __builtin_convertvector(f32x2_t{x, y}, bf16x2_t);
    return c.u;
}

// split3 for two values at a time (the same roundings, one conversion instruction per pair and term):
// x in the low halves of hi, mid, lo and y in the high halves
__device__ __forceinline__ void split3_pair(float x, float y, uint32_t &hi, uint32_t &mid, uint32_t &lo) {
    hi = pack_bf16_rne(x, y);
    const float rx = x - __uint_as_float(hi << 16), ry = y - __uint_as_float(hi & 0xffff0000u);
    mid = pack_bf16_rne(rx, ry);
    lo = pack_bf16_rne(rx - __uint_as_float(mid << 16), ry - __uint_as_float(mid & 0xffff0000u));
}

// 16 bytes -> 16 bf16 (two 16-byte vectors)
__device__ __forceinline__ void bytes_to_bf16(const u32x4 b, u32x4 &lo8, u32x4 &hi8) {
    Bf16x8Bits o[2];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t v = b[d];
        o[d / 2].v[(d % 2) * 4 + 0] = (__bf16)(float)(v & 0xff);
        o[d / 2].v[(d % 2) * 4 + 1] = (__bf16)(float)((v >> 8) & 0xff);
        o[d / 2].v[(d % 2) * 4 + 2] = (__bf16)(float)((v >> 16) & 0xff);
        o[d / 2].v[(d % 2) * 4 + 3] = (__bf16)(float)(v >> 24);
    }
    lo8 = o[0].u;
    hi8 = o[1].u;
}

// y[b][oc][pix] = max(0, scale * sum_k W[oc][k] x[b][tap k at pix] + bias[oc]),  OC = 16 or 32.
// Block = 4 wavefronts, frames blockIdx.x, blockIdx.x + gridDim.x, ...  The
// frame sits in LDS as bf16 [4][84][84]; a lane (pixel p, group g) reads the 8
// taps of filter row u = 4*(kb%2) + g of channel kb/2 in one go, which is the
// k = 8g..8g+7 share of a 16x16x32 MFMA.  The split filters stay in registers.
template <int OC>
__global__ __launch_bounds__(256, 2) void conv1_bf16x3_fwd_kernel(const uint8_t *__restrict__ x,
                                                                  const float *__restrict__ w,
                                                                  const float *__restrict__ bias, float *__restrict__ y,
                                                                  int nframes, float scale, int rb) {
    constexpr int C = 4, H = 84, W = 84, S = 4, OW = 20, NPIX = 400, K = 256, CHW = C * H * W;
    constexpr int NV = CHW / 16, VPT = (NV + 255) / 256;           // 16-byte vectors of the byte frame
    constexpr int OT = OC / 16, JOBS = 25 * OT, TPW = (JOBS + 3) / 4;
    constexpr int FULL = JOBS % 4 == 0 ? TPW : TPW - 1, NLAST = JOBS - 4 * FULL;
    static_assert(OC == 16 || OC == 32, "16 or 32 filters");
    __shared__ __attribute__((aligned(16))) __bf16 xs[VPT * 256 * 16];

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave that gets the odd tile rotates with the block, so that two
    // blocks sharing a compute unit do not load the same SIMD
    const int wave = __builtin_amdgcn_readfirstlane(((tid >> 6) + (OT == 1 ? blockIdx.x : 2 * (blockIdx.x & 1))) & 3);
    const int l16 = lane & 15, g = lane >> 4;
    const int ot = wave % OT;

    // my filter (row l16 of tile ot), split into three bf16 terms, 8 taps per 32-tap block
    bf16x8 wq[3][8];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) {
        const float *src = w + (size_t)(ot * 16 + l16) * K + (kb / 2) * 64 + (4 * (kb % 2) + g) * 8;
        const float4 a = *(const float4 *)src, b = *(const float4 *)(src + 4);
        const float f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __bf16 h, m, l;
            split3(f[e], h, m, l, rb);
            wq[0][kb][e] = h; wq[1][kb][e] = m; wq[2][kb][e] = l;
        }
    }
    // The MFMAs take the pixels as rows and the filters as columns: a lane ends up with four consecutive pixels
    // (16 tile + 4 g + r) of filter ot * 16 + l16, which it stores as one 16-byte vector.
    const float bv = bias[ot * 16 + l16];

    int pixbase[TPW], pixidx[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int job = wave + 4 * i;
        int p = (job / OT) * 16 + l16;
        pixidx[i] = (job < JOBS && p < NPIX) ? (job / OT) * 16 + 4 * g : -1;       // first of my four output pixels
        if (p >= NPIX) p = 0;
        pixbase[i] = (p / OW) * S * W + (p % OW) * S + g * W;     // + row g of the 4 rows of a tap block
    }
    int vidx[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) vidx[i] = min(tid + 256 * i, NV - 1);

    u32x4 pre[VPT];
    int f = blockIdx.x;
    {
        const u32x4 *src = (const u32x4 *)(x + (size_t)min(f, nframes - 1) * CHW);
#pragma unroll
        for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
    }
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            u32x4 a, b;
            bytes_to_bf16(pre[i], a, b);
            u32x4 *dst = (u32x4 *)(xs + (size_t)(tid + 256 * i) * 16);
            dst[0] = a; dst[1] = b;
        }
        __syncthreads();
        {
            const u32x4 *src = (const u32x4 *)(x + (size_t)min(f + (int)gridDim.x, nframes - 1) * CHW);
#pragma unroll
            for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
        }
        floatx4 acc[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        auto tile_step = [&](int i, int kb) {
            const __bf16 *src = xs + pixbase[i] + (kb / 2) * (H * W) + 4 * (kb % 2) * W;   // 8-byte aligned
            const uint2 lo = *(const uint2 *)src, hi = *(const uint2 *)(src + 4);
            Bf16x8Bits xv;
            xv.u = u32x4{lo.x, lo.y, hi.x, hi.y};
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xv.v, wq[2][kb], acc[i], 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xv.v, wq[1][kb], acc[i], 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xv.v, wq[0][kb], acc[i], 0, 0, 0);
        };
#pragma unroll
        for (int kb = 0; kb < 8; ++kb)
#pragma unroll
            for (int i = 0; i < FULL; ++i) tile_step(i, kb);
        if (NLAST > 0 && wave < NLAST) {
#pragma unroll
            for (int kb = 0; kb < 8; ++kb) tile_step(TPW - 1, kb);
        }
        float *yb = y + (size_t)f * OC * NPIX;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            if (pixidx[i] >= 0) {
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v[r] = acc[i][r] * scale + bv;
                    v[r] = v[r] > 0.f ? v[r] : 0.f;
                }
                *(float4 *)(yb + (ot * 16 + l16) * NPIX + pixidx[i]) = float4{v[0], v[1], v[2], v[3]};      // NPIX % 4 == 0
            }
        }
    }
}

template <int OC>
inline hipError_t launch_conv1_bf16x3_fwd(const uint8_t *x, const float *w, const float *bias, float *y, int nframes,
                                          float scale, hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    const int grid = nframes < 512 ? nframes : 512;
    ga3c::launch((conv1_bf16x3_fwd_kernel<OC>), dim3(grid), dim3(256), 0, s, x, w, bias, y, nframes, scale, rb);
    return hipGetLastError();
}


// Weight and bias gradient of the same layer, same arithmetic: the frame is
// exact in bf16 and dY is split into three bf16 terms.
//   dW[oc][c][u][v] = sum_{i,j} dY[oc][i][j] x[c][4i+u][4j+v],   db[oc] = sum dY[oc][i][j]
// The contraction runs over output pixels, 8 consecutive pixels of a row per
// lane, so the frame is re-laid in LDS "space to depth": with u = 4a + u',
// v = 4b + v' the pixel x[c][4i+u][4j+v] is X[(c,u',v')][i+a][j+b], and 8
// consecutive j are 8 consecutive elements of a row of plane (c,u',v').  Plane
// index q = (c,u',v') is the column of the MFMA tile (wave w owns channel w and
// its 16 planes), the filters are the rows, and the four (a,b) are four
// accumulators.  Shift b = 1 is made from the b = 0 vector and one more dword.
// Rows of 20 pixels are padded to 24 = 3 blocks of 8 with zero dY.
// part: [gridDim.x][OCT][257]; the last column is the bias gradient.  A layer
// with OCT = 32 filters is done in two slices of 16 (blockIdx.y).
template <int OCT, int NPART>
__global__ __launch_bounds__(256 * NPART) void conv1_bf16x3_wgrad_kernel(const uint8_t *__restrict__ x,
                                                                 const float *__restrict__ dy,
                                                                 float *__restrict__ part, int nframes, float scale,
                                                                 int rb) {
    // rb: dY enters the products (and the bias sums) rounded to bfloat16
    constexpr int C = 4, H = 84, W = 84, OC = 16, OH = 20, NPIX = 400, K = 256, CHW = C * H * W;
    constexpr int XROW = 32, XPLANE = 21 * XROW + 8;       // bf16 elements; plane pitch 20 mod 32 dwords
    constexpr int DROW = 24, DOC = OH * DROW + 8;          // dY rows padded to 24, filter pitch 20 mod 32 dwords
    constexpr int NTHR = 256 * NPART;                      // NPART wavefronts per SIMD, so that one's LDS and
                                                           // conversion work fills another's MFMA waits
    constexpr int NITEM = 336 * 6, IPT = (NITEM + NTHR - 1) / NTHR;    // (frame row, group of 4 dwords)
    constexpr int NDV = OC * NPIX / 4, DPT = (NDV + NTHR - 1) / NTHR;  // float4 of dY per frame
    constexpr int NSTEP = OH * 3 / 4;                      // 60 blocks of 8 pixels, 4 per MFMA
    __shared__ __attribute__((aligned(16))) __bf16 xp[64 * XPLANE];
    __shared__ __attribute__((aligned(16))) __bf16 dp[3 * OC * DOC];
    __shared__ float bsh[NDV];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int oc0 = blockIdx.y * OC;                       // my slice of the filters
    static_assert(OCT % OC == 0, "whole slices of 16 filters");

    for (int e = tid; e < 64 * XPLANE / 2; e += NTHR) ((uint32_t *)xp)[e] = 0u;     // padding stays zero
    for (int e = tid; e < 3 * OC * DOC / 2; e += NTHR) ((uint32_t *)dp)[e] = 0u;

    // staging descriptors: where my dwords come from and where they go.  A row of 21 dwords is five groups of four
    // and a last group of one; that one is fetched as the last of the row's dwords 17..20, so that every fetch is one
    // 16-byte load (4-byte aligned) that stays inside the frame.
    int xsrc[IPT], xdst[IPT], xcnt[IPT];
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int it = min(tid + NTHR * i, NITEM - 1);
        const int row = it / 6, gq = it % 6;               // row = c*84 + r
        const int c = row / H, r = row % H;
        xsrc[i] = row * (W / 4) + (gq == 5 ? 17 : 4 * gq); // dword index in the frame
        xcnt[i] = (tid + NTHR * i < NITEM) ? (gq == 5 ? 1 : 4) : 0;
        xdst[i] = ((c * 4 + r % 4) * 4) * XPLANE + (r / 4) * XROW + 4 * gq;   // plane (c, u'=r%4, v'=0)
    }
    int dsrc[DPT], ddst[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) {
        const int e = min(tid + NTHR * i, NDV - 1);
        dsrc[i] = e;
        const int oc = e / (NPIX / 4), pq = e % (NPIX / 4);           // 5 float4 per row of 20
        ddst[i] = oc * DOC + (pq / 5) * DROW + 4 * (pq % 5);
    }

    floatx4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
    float bsum = 0.f;

    typedef uint32_t u32x4_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));
    u32x4 xpre[IPT];
    float4 dpre[DPT];
    auto fetch = [&](int ff) {
        const uint32_t *xs = (const uint32_t *)(x + (size_t)ff * CHW);
#pragma unroll
        for (int i = 0; i < IPT; ++i) xpre[i] = *(const u32x4_dword_aligned *)(xs + xsrc[i]);
        const float4 *ds = (const float4 *)(dy + ((size_t)ff * OCT + oc0) * NPIX);
#pragma unroll
        for (int i = 0; i < DPT; ++i) dpre[i] = ds[dsrc[i]];
    };
    int f = blockIdx.x;
    fetch(min(f, nframes - 1));
    const int ch = wave & 3, prt = wave >> 2;        // wavefronts w, w + 4, ... share channel w and divide the pixel blocks
    const __bf16 *xq = xp + (ch * 16 + l16) * XPLANE;                // my plane
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < IPT; ++i) {
            if (xcnt[i] > 0) {
                // a last group holds its dword in the fourth place; the other three places become zero padding
                const u32x4 xv = xcnt[i] == 4 ? xpre[i] : u32x4{xpre[i][3], 0u, 0u, 0u};
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {             // plane v' = vq gets byte vq of each dword
                    union { __bf16 h[4]; uint2 u; } o;
#pragma unroll
                    for (int t = 0; t < 4; ++t) o.h[t] = (__bf16)(float)((xv[t] >> (8 * vq)) & 0xff);
                    *(uint2 *)(xp + xdst[i] + vq * XPLANE) = o.u;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < DPT; ++i) {
            if (tid + NTHR * i < NDV) {
                const float v[4] = {dpre[i].x, dpre[i].y, dpre[i].z, dpre[i].w};
                union { __bf16 h[4]; uint2 u; } o[3];
                split3_pair(v[0], v[1], o[0].u.x, o[1].u.x, o[2].u.x);
                split3_pair(v[2], v[3], o[0].u.y, o[1].u.y, o[2].u.y);
                if (rb) { o[1].u = uint2{0u, 0u}; o[2].u = uint2{0u, 0u}; }
#pragma unroll
                for (int term = 0; term < 3; ++term) *(uint2 *)(dp + term * OC * DOC + ddst[i]) = o[term].u;
                bsh[tid + NTHR * i] = rb ? ((float)o[0].h[0] + (float)o[0].h[1]) + ((float)o[0].h[2] + (float)o[0].h[3])
                                        : (v[0] + v[1]) + (v[2] + v[3]);
            }
        }
        __syncthreads();
        fetch(min(f + (int)gridDim.x, nframes - 1));
        if (tid < 256) {   // bias: 16 lanes share a filter, 100 partial sums each
            const int oc = tid / 16, pt = tid % 16;
            float sum = 0.f;
            for (int m = pt; m < NPIX / 4; m += 16) sum += bsh[oc * (NPIX / 4) + m];
            sum += dpp_row_f32<0xB1>(sum); sum += dpp_row_f32<0x4E>(sum);
            sum += dpp_row_f32<0x141>(sum); sum += dpp_row_f32<0x140>(sum);
            bsum += sum;
        }
        auto steps = [&](auto first, auto last) {
#pragma unroll
            for (int st = decltype(first)::value; st < decltype(last)::value; ++st) {
                const int blk = 4 * st + g, i = blk / 3, jb = blk % 3;
                Bf16x8Bits d[3];
#pragma unroll
                for (int term = 0; term < 3; ++term)
                    d[term].u = *(const u32x4 *)(dp + term * OC * DOC + l16 * DOC + i * DROW + 8 * jb);
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const __bf16 *src = xq + (i + a) * XROW + 8 * jb;
                    const u32x4 c0 = *(const u32x4 *)src;
                    const uint32_t c4 = *(const uint32_t *)(src + 8);
                    Bf16x8Bits x0, x1;
                    x0.u = c0;
                    x1.u = u32x4{__builtin_amdgcn_alignbit(c0[1], c0[0], 16), __builtin_amdgcn_alignbit(c0[2], c0[1], 16),
                                 __builtin_amdgcn_alignbit(c0[3], c0[2], 16), __builtin_amdgcn_alignbit(c4, c0[3], 16)};
#pragma unroll
                    for (int term = 2; term >= 0; --term) {
                        acc[a][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(d[term].v, x0.v, acc[a][0], 0, 0, 0);
                        acc[a][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(d[term].v, x1.v, acc[a][1], 0, 0, 0);
                    }
                }
            }
        };
        static_assert(NPART == 1 || NPART == 2 || NPART == 4, "one, two or four wavefronts per SIMD");
        constexpr int Q1 = NSTEP / NPART, Q2 = 2 * NSTEP / NPART, Q3 = 3 * NSTEP / NPART;
        typedef std::integral_constant<int, 0> I0;
        typedef std::integral_constant<int, NSTEP> IN;
        if (NPART == 1) steps(I0{}, IN{});
        else if (NPART == 2) {
            if (prt == 0) steps(I0{}, std::integral_constant<int, Q1>{});
            else steps(std::integral_constant<int, Q1>{}, IN{});
        } else {
            if (prt == 0) steps(I0{}, std::integral_constant<int, Q1>{});
            else if (prt == 1) steps(std::integral_constant<int, Q1>{}, std::integral_constant<int, Q2>{});
            else if (prt == 2) steps(std::integral_constant<int, Q2>{}, std::integral_constant<int, Q3>{});
            else steps(std::integral_constant<int, Q3>{}, IN{});
        }
    }
    if (NPART > 1) {   // the parts of a channel's pixel blocks are added through LDS (the frame planes are no longer needed)
        __syncthreads();
        float *xch = (float *)xp;
        if (prt > 0) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        xch[(((prt - 1) * 4 + ch) * 16 + (a * 2 + b) * 4 + r) * 64 + lane] = acc[a][b][r];
        }
        __syncthreads();
        if (prt > 0) return;
#pragma unroll
        for (int q = 0; q < NPART - 1; ++q)
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[a][b][r] += xch[((q * 4 + ch) * 16 + (a * 2 + b) * 4 + r) * 64 + lane];
    }
    // lane (l16, g), register r of acc[a][b]: filter 4g + r, tap (c = wave, u = 4a + l16/4, v = 4b + l16%4)
    float *pb = part + ((size_t)blockIdx.x * OCT + oc0) * (K + 1);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                pb[(4 * g + r) * (K + 1) + ch * 64 + (4 * a + l16 / 4) * 8 + 4 * b + l16 % 4] = acc[a][b][r] * scale;
    if (tid % 16 == 0) pb[(tid / 16) * (K + 1) + K] = bsum;      // tid < 256 here
}

inline int conv1_bf16x3_wgrad_blocks(int nframes) { return nframes < 256 ? nframes : 256; }

template <int OCT = 16, int NPART = 4>
inline hipError_t launch_conv1_bf16x3_wgrad(const uint8_t *x, const float *dy, float *part, int nframes, float scale,
                                            hipStream_t s, int rb = 0) {
    if (nframes <= 0) return hipSuccess;
    ga3c::launch((conv1_bf16x3_wgrad_kernel<OCT, NPART>), dim3(conv1_bf16x3_wgrad_blocks(nframes), OCT / 16),
                       dim3(256 * NPART), 0, s, x, dy, part, nframes, scale, rb);
    return hipGetLastError();
}

}  // namespace ga3c
