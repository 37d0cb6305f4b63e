// Input gradient of a 4x4, stride-2 convolution layer on the bf16 matrix cores
// at fp32 accuracy (backward pass of the network of Sec. 3.2; the layer is the
// second convolution of both networks):
//
//   dX[c][y][x] = [xin[c][y][x] > 0] * sum_{oc,u,v} dY[oc][(y-u)/2][(x-v)/2] W[oc][c][u][v]
//
// The input pixels fall into 2 x 2 stride phases (y%2, x%2), one per wavefront
// of a block; a phase only meets the filter taps u = y%2 + 2a, v = x%2 + 2e
// (a, e in {0, 1}), so on the phase grid the layer is a dense 2 x 2
// convolution of the zero-padded dY with a sub-filter: a product
// [16 channels] x [4 OC] x [pixels of the phase].  The four phases are
// interleaved in an LDS copy of the output frame, which is then masked and
// stored with full-width writes.  A block computes 16 input channels,
// 16 blockIdx.y .. (gridDim.y = C / 16), of frames blockIdx.x, + gridDim.x, ...
//
// Both operands are split into
// three bf16 terms (x = hi + mid + lo exactly) and a product is evaluated as the
// six largest of the nine term products (dense_gemm_bf16x6.hpp), on
// v_mfma_f32_16x16x32_bf16: 6 x 16 cycles per 32 k instead of 8 x 32 on the
// fp32 instruction.  The contraction index is ordered (tap, oc), and dY sits in
// LDS as [padded pixel][oc] per term, so the 8 consecutive k a lane feeds to an
// MFMA are 8 consecutive filters of one pixel: one 16-byte LDS read per term.
// The pixel pitch is 2 OC + 16 bytes, which spreads 16 consecutive pixels over
// all banks.  The sub-filters of a wavefront's phase stay in registers as split
// fragments for the whole launch.  A block can take them ready-made (`wfrag`:
// the register image of every wavefront, which the kernel that updates the
// parameters keeps current): gathering them from the filter tensor costs 32
// scattered loads per lane, 64 cache lines each, a quarter of the life of a
// block that only computes five frames.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"

namespace ga3c {

// Optional instrumentation (the micro-benchmark program defines GA3C_BLOCK_STAMPS before it includes this file; the
// library does not): thread 0 of every block of channel slice 0 records the wall clock (100 MHz) and the core clock at
// its start (slot 0), after its prologue (1) and at its end (2).
#ifdef GA3C_BLOCK_STAMPS
__device__ long long conv_dgrad_block_stamps[1024 * 6];
#define CONV_DGRAD_STAMP(slot)                                                                   \
    do {                                                                                         \
        if (threadIdx.x == 0 && blockIdx.x < 1024 && blockIdx.y == 0) {                          \
            conv_dgrad_block_stamps[blockIdx.x * 6 + 2 * (slot)] = wall_clock64();               \
            conv_dgrad_block_stamps[blockIdx.x * 6 + 2 * (slot) + 1] = clock64();                \
        }                                                                                        \
    } while (0)
#else
#define CONV_DGRAD_STAMP(slot)
#endif

template <class SP>
struct ConvDgradBf16Geom {
    static constexpr int CS = 16, S = 2;
    static constexpr int GH = SP::H / S, GW = SP::W / S, GP = GH * GW;
    static constexpr int NT = (GP + 15) / 16;
    static constexpr int PH = SP::OH + 2, PW = SP::OW + 2;
    static constexpr int OCB = SP::OC / 32, KB = 4 * OCB;          // k-blocks of 32: (tap, 32 filters)
    static constexpr int PIT = 2 * SP::OC + 16;                    // bytes per padded pixel and term
    static constexpr int PLANE = PH * PW * PIT;
    static constexpr int NX = CS * SP::H * SP::W;
    __host__ __device__ static constexpr int lds_bytes(bool one) { return (one ? 1 : 3) * PLANE + NX * 4; }
    // ready-made filter fragments: [channel slice][wavefront = phase][k-block][term][lane] vectors of 8 bf16
    static constexpr int FRAG_VECS = (SP::C / CS) * 4 * KB * 3 * 64;
};

// Writes the terms of four filter taps into the ready-made fragments: `rel` (a multiple of 4) is the index of v.x in
// the filter tensor [oc][c][4][4], so the four values are row u = (rel / 4) % 4, columns 0..3 of filter oc, channel c.
template <class SP>
__device__ __forceinline__ void conv_dgrad_store_fragment4(u32x4 *__restrict__ wfrag, int rel, const float4 v) {
    typedef ConvDgradBf16Geom<SP> G;
    const int oc = rel / (SP::C * 16), c = (rel / 16) % SP::C, u = (rel / 4) % 4;
    const int ry = u % 2, a = u / 2;
    const int lane = ((oc % 32) / 8) * 16 + c % 16, j = oc % 8;
    const float f[4] = {v.x, v.y, v.z, v.w};
    __bf16 *dst = (__bf16 *)wfrag;
#pragma unroll
    for (int col = 0; col < 4; ++col) {
        const int rx = col % 2, e = col / 2;
        const int wave = ry * 2 + rx, kb = (a * 2 + e) * G::OCB + oc / 32;
        __bf16 t[3];
        split3(f[col], t[0], t[1], t[2]);
#pragma unroll
        for (int x = 0; x < 3; ++x)
            dst[((size_t)((((c / 16) * 4 + wave) * G::KB + kb) * 3 + x) * 64 + lane) * 8 + j] = t[x];
    }
}

// All fragments from the filter tensor w [oc][c][4][4] (16-byte aligned).
template <class SP>
__global__ __launch_bounds__(256) void conv_dgrad_filter_fragments_kernel(const float *__restrict__ w, u32x4 *__restrict__ wfrag) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < SP::OC * SP::C * 4) conv_dgrad_store_fragment4<SP>(wfrag, 4 * i, ((const float4 *)w)[i]);
}

template <class SP>
inline hipError_t launch_conv_dgrad_filter_fragments(const float *w, u32x4 *wfrag, hipStream_t s) {
    ga3c::launch((conv_dgrad_filter_fragments_kernel<SP>), dim3((SP::OC * SP::C * 4 + 255) / 256), dim3(256), 0, s, w, wfrag);
    return hipGetLastError();
}

// ONE: operands rounded to bfloat16 (the reduced-precision variant): one term, one product.
template <class SP, bool ONE>
__global__ __launch_bounds__(256, 2) void conv_dgrad_bf16x6_kernel(const float *__restrict__ dy, const float *__restrict__ w,
                                                                   const float *__restrict__ xin, float *__restrict__ dx,
                                                                   int nframes, const u32x4 *__restrict__ wfrag) {
    typedef ConvDgradBf16Geom<SP> G;
    static_assert(SP::KS == 4 && SP::S == 2, "kernel must be 4x4 with stride 2");
    static_assert(SP::C % 16 == 0 && SP::OC % 32 == 0, "16 input channels per block, filters in groups of 32");
    static_assert(SP::H % 2 == 0 && SP::W % 2 == 0, "phases must tile the input");
    static_assert(G::GH <= SP::OH + 1 && G::GW <= SP::OW + 1, "phase grid must fit the padded dY");
    constexpr int CS = G::CS, S = G::S, GW = G::GW, GP = G::GP, NT = G::NT, PW = G::PW;
    constexpr int OCB = G::OCB, KB = G::KB, PIT = G::PIT, PLANE = G::PLANE, NX = G::NX;
    constexpr int NTERM = ONE ? 1 : 3;
    constexpr int NITEM = (SP::OC / 4) * SP::NPIX, DPT = (NITEM + 255) / 256;      // items: 4 filters of one pixel
    constexpr int XV = NX / 4, XPT = (XV + 255) / 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *dp = smem;                                   // [term][padded pixel][oc] bf16
    float *outs = (float *)(smem + NTERM * PLANE);              // [c][H][W]

    CONV_DGRAD_STAMP(0);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int ry = wave / S, rx = wave % S;
    const int c0 = blockIdx.y * CS;

    for (int e = tid; e < NTERM * PLANE / 16; e += 256) ((u32x4 *)dp)[e] = u32x4{0u, 0u, 0u, 0u};     // zero border

    int pbyte[NT], obase[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        int p = 16 * i + l16;
        const bool ok = p < GP;
        if (!ok) p = 0;
        const int iy = p / GW, ix = p % GW;
        // tap (a, e) reads padded pixel (iy - a + 1, ix - e + 1)
        pbyte[i] = (iy * PW + ix) * PIT + 16 * g;
        obase[i] = ok ? (S * iy + ry) * SP::W + S * ix + rx : -1;
    }
    int dsrc_off[DPT], dlds[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) {
        const int e = min(tid + 256 * i, NITEM - 1);
        const int ocq = e / SP::NPIX, pix = e % SP::NPIX;
        dsrc_off[i] = 4 * ocq * SP::NPIX + pix;
        dlds[i] = ((pix / SP::OW + 1) * PW + pix % SP::OW + 1) * PIT + 8 * ocq;
    }
    int xidx[XPT];
#pragma unroll
    for (int i = 0; i < XPT; ++i) xidx[i] = min(tid + 256 * i, XV - 1);

    float dpre[DPT][4];
    auto fetch_dy = [&](int f) {
        const float *dsrc = dy + (size_t)f * (SP::OC * SP::NPIX);
#pragma unroll
        for (int i = 0; i < DPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) dpre[i][j] = dsrc[dsrc_off[i] + j * SP::NPIX];
    };
    int f = blockIdx.x;
    fetch_dy(min(f, nframes - 1));       // on its way while the filters arrive
    // sub-filter fragments of my phase: row = channel l16, k = (tap, filter 8g..8g+7 of the block's 32)
    Bf16x8Bits af[KB][NTERM];
    if (wfrag) {
        const u32x4 *src = wfrag + (size_t)((blockIdx.y * 4 + wave) * KB) * 3 * 64 + lane;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int x = 0; x < NTERM; ++x) af[kb][x].u = src[(kb * 3 + x) * 64];
    } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int tap = kb / OCB, a = tap / 2, e = tap % 2;
            const int u = ry + S * a, v = rx + S * e;
            const int oc0 = (kb % OCB) * 32 + 8 * g;
            Bf16x8Bits t[3];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float f = w[((size_t)((oc0 + j) * SP::C + c0 + l16) * SP::KS + u) * SP::KS + v];
                __bf16 h, m, l;
                split3(f, h, m, l);
                t[0].v[j] = h; t[1].v[j] = m; t[2].v[j] = l;
            }
#pragma unroll
            for (int x = 0; x < NTERM; ++x) af[kb][x] = t[x];
        }
    }
    CONV_DGRAD_STAMP(1);
    for (; f < nframes; f += gridDim.x) {
        __syncthreads();                      // the border is zero; the last frame's dY and outs have been read
#pragma unroll
        for (int i = 0; i < DPT; ++i)
            if (tid + 256 * i < NITEM) {
                uint2 o3[3];
                split3_pair(dpre[i][0], dpre[i][1], o3[0].x, o3[1].x, o3[2].x);
                split3_pair(dpre[i][2], dpre[i][3], o3[0].y, o3[1].y, o3[2].y);
#pragma unroll
                for (int x = 0; x < NTERM; ++x) *(uint2 *)(dp + x * PLANE + dlds[i]) = o3[x];
            }
        __syncthreads();
        fetch_dy(min(f + (int)gridDim.x, nframes - 1));
        float4 mask[XPT];
        {
            const float4 *msrc = (const float4 *)(xin + (size_t)f * SP::CHW + (size_t)c0 * (SP::H * SP::W));
#pragma unroll
            for (int i = 0; i < XPT; ++i) mask[i] = msrc[xidx[i]];
        }
        // the loads above go out before the products start (the compiler would otherwise sink them below the MFMAs,
        // and their latency would be paid after the next barrier)
        __builtin_amdgcn_sched_barrier(0);
        floatx4 acc[NT];
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        // pixel tiles in groups of up to four: the accumulators of a group take one term product each in turn.  A step is
        // one k-block of one group; where the registers allow (32 filters), the operand reads of the next step are
        // issued before the products of this one, so that no product waits for LDS.
        constexpr int IG = 4, NSTEP = ((NT + IG - 1) / IG) * KB;
        constexpr bool AHEAD = KB * NTERM <= 12;
        constexpr int NPROD = ONE ? 1 : 6;
        constexpr int PA[6] = {2, 1, 0, 1, 0, 0}, PB[6] = {0, 1, 2, 0, 1, 0};      // smallest products first
        Bf16x8Bits b[AHEAD ? 2 : 1][IG][NTERM];
        auto read_b = [&](int step, Bf16x8Bits (&dst)[IG][NTERM]) {
            const int i0 = (step / KB) * IG, kb = step % KB;
            const int tap = kb / OCB, a = tap / 2, e = tap % 2;
            const int koff = ((1 - a) * PW + (1 - e)) * PIT + (kb % OCB) * 64;
#pragma unroll
            for (int ii = 0; ii < IG; ++ii)
                if (i0 + ii < NT) {
#pragma unroll
                    for (int x = 0; x < NTERM; ++x) dst[ii][x].u = *(const u32x4 *)(dp + x * PLANE + pbyte[i0 + ii] + koff);
                }
        };
        __builtin_amdgcn_s_setprio(1);         // the products first: measured 2 % over equal priorities
        if (AHEAD) read_b(0, b[0]);
#pragma unroll
        for (int step = 0; step < NSTEP; ++step) {
            if (!AHEAD) read_b(step, b[0]);
            else if (step + 1 < NSTEP) read_b(step + 1, b[(step + 1) & 1]);
            if (AHEAD) __builtin_amdgcn_sched_barrier(0);
            const int i0 = (step / KB) * IG, kb = step % KB;
#pragma unroll
            for (int q = 0; q < NPROD; ++q) {
                const int ai = ONE ? 0 : PA[q], bi = ONE ? 0 : PB[q];
#pragma unroll
                for (int ii = 0; ii < IG; ++ii)
                    if (i0 + ii < NT)
                        acc[i0 + ii] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[kb][ai % NTERM].v, b[AHEAD ? step & 1 : 0][ii][bi % NTERM].v,
                                                                               acc[i0 + ii], 0, 0, 0);
            }
            if (AHEAD) __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int i = 0; i < NT; ++i)
            if (obase[i] >= 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) outs[(4 * g + r) * (SP::H * SP::W) + obase[i]] = acc[i][r];
            }
        __syncthreads();
        float4 *dst = (float4 *)(dx + (size_t)f * SP::CHW + (size_t)c0 * (SP::H * SP::W));
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int e = tid + 256 * i;
            if (e < XV) {
                float4 v = ((const float4 *)outs)[e];
                v.x = mask[i].x > 0.f ? v.x : 0.f; v.y = mask[i].y > 0.f ? v.y : 0.f;
                v.z = mask[i].z > 0.f ? v.z : 0.f; v.w = mask[i].w > 0.f ? v.w : 0.f;
                dst[e] = v;
            }
        }
    }
    CONV_DGRAD_STAMP(2);
}

// `blocks`: how many blocks the chip holds at once (two per CU), shared out over the channel slices.
template <class SP>
inline hipError_t launch_conv_dgrad_bf16x6(const float *dy, const float *w, const float *xin, float *dx, int nframes,
                                           hipStream_t s, int blocks = 512, int rb = 0, const u32x4 *wfrag = nullptr) {
    if (nframes <= 0) return hipSuccess;
    typedef ConvDgradBf16Geom<SP> G;
    constexpr int SLICES = SP::C / 16;
    const int per = blocks / SLICES;
    const int grid = nframes < per ? nframes : per;
    static bool attr_set = false;          // once per layer shape: let the kernels use more than 64 KB of LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_dgrad_bf16x6_kernel<SP, false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(false));
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_dgrad_bf16x6_kernel<SP, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(true));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (rb)
        ga3c::launch((conv_dgrad_bf16x6_kernel<SP, true>), dim3(grid, SLICES), dim3(256), G::lds_bytes(true), s, dy, w, xin,
                           dx, nframes, wfrag);
    else
        ga3c::launch((conv_dgrad_bf16x6_kernel<SP, false>), dim3(grid, SLICES), dim3(256), G::lds_bytes(false), s, dy, w,
                           xin, dx, nframes, wfrag);
    return hipGetLastError();
}

}  // namespace ga3c
