// Forward pass of a convolution layer with 32 k input channels and 64 filters
// (the second and third layers of the larger network) on the bf16 matrix cores
// at fp32 accuracy:
//
//   y[oc][oy][ox] = max(0, b[oc] + sum_{c,u,v} W[oc][c][u][v] x[c][S oy + u][S ox + v])
//
// Activations and filters are split into three bf16 terms each (x = hi + mid + lo
// exactly) and a product is evaluated as the six largest of the nine term
// products (dense_gemm_bf16x6.hpp has the error argument), 6 x 16 cycles per 32 k
// on v_mfma_f32_16x16x32_bf16 instead of 8 x 32 on the fp32 instruction.
//
// The contraction index is ordered (u, v, c): a k-block of 32 is 32 channels of
// one tap.  The frame sits in LDS as [pixel][channel] per term (pitch 2 C + 16
// bytes), so the 8 consecutive k a lane feeds to an MFMA are 8 consecutive
// channels of one input pixel: one 16-byte LDS read per term.  With stride 2 the
// even and the odd columns of a row are stored apart, so that the 16 output
// pixels of a tile read 16 consecutive LDS pixels (and with them all banks)
// instead of every other one.  A block works on
// whole frames (blockIdx.x, + gridDim.x, ...): wavefront w computes filter tile
// w % 4 for the pixel tiles w / 4, w / 4 + NW / 4, ... and keeps its tile's
// filters for all k in registers as split fragments for the whole launch (that
// is 12 registers per k-block: hence one or two wavefronts per SIMD).  The next
// frame travels from memory while the current one is multiplied.  The fragments
// can be handed in ready-made (`wfrag`, the register image of the four filter
// tiles, built once per parameter copy): gathering them costs 8 KB scattered
// loads per lane, more than a frame's products when a block sees one frame.
//
// The input gradient of a stride-1 layer is the same computation with other
// operands (DGRAD): dX = [xin > 0] * (dY zero-padded by KS - 1 on every side,
// convolved with the filters flipped in both directions and transposed),
//   dX[c][y][x] = sum_{oc,u,v} dY[oc][y - u][x - v] W[oc][c][u][v].
// The kernel is then instantiated on that pseudo-layer: SP::C = the layer's
// filter count, SP::H x SP::W = the padded dY, SP::OC = the layer's input
// channels, SP::OH x SP::OW = the layer's input size; the border of the LDS
// planes is zeroed once and only the interior is staged.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"
#include "conv_frame.hpp"

namespace ga3c {

template <class SP>
struct ConvFwdBf16Geom {
    static constexpr int CG = SP::C / 32;                          // channel groups of 32 per tap
    static constexpr int KB = SP::KS * SP::KS * CG;                // k-blocks of 32
    static constexpr int NT = (SP::NPIX + 15) / 16;                // pixel tiles
    static constexpr int PIT = 2 * SP::C + 16;                     // bytes per input pixel and term
    static constexpr int PLANE = SP::H * SP::W * PIT;
    static_assert(SP::S == 1 || (SP::S == 2 && SP::W % 2 == 0), "stride 1, or stride 2 on an even width");
    // where input pixel (row, column x) sits in a plane
    __host__ __device__ static constexpr int pixel(int row, int xcol) {
        return row * SP::W + (SP::S == 2 ? (xcol & 1) * (SP::W / 2) + (xcol >> 1) : xcol);
    }
    __host__ __device__ static constexpr int lds_bytes(bool one) { return (one ? 1 : 3) * PLANE; }
    static constexpr int FRAG_VECS = 4 * KB * 3 * 64;             // ready-made fragments: [filter tile][k-block][term][lane]
};

// The value that sits at row (filter o of the tile layout), k = (tap, channel ic) of the kernel's filter operand.
template <class SP, bool DGRAD>
__device__ __forceinline__ float conv_fwd_filter_value(const float *__restrict__ w, int o, int ic, int u, int v) {
    constexpr int KS = SP::KS;
    return DGRAD ? w[((size_t)(ic * SP::OC + o) * KS + (KS - 1 - u)) * KS + (KS - 1 - v)]
                 : w[((size_t)(o * SP::C + ic) * KS + u) * KS + v];
}

// All fragments of a layer (for DGRAD: of its pseudo-layer SP) from the filter tensor: thread i of 4 * KB * 64 writes
// the three vectors of one (filter tile, k-block, lane).
template <class SP, bool DGRAD>
__device__ __forceinline__ void conv_fwd_filter_fragments_thread(const float *__restrict__ w, u32x4 *__restrict__ wfrag, int i) {
    typedef ConvFwdBf16Geom<SP> G;
    if (i >= 4 * G::KB * 64) return;
    const int lane = i % 64, kb = (i / 64) % G::KB, ot = i / (64 * G::KB);
    const int l16 = lane & 15, g = lane >> 4;
    const int tap = kb / G::CG, cg = kb % G::CG, u = tap / SP::KS, v = tap % SP::KS;
    Bf16x8Bits t[3];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        __bf16 h, m, l;
        split3(conv_fwd_filter_value<SP, DGRAD>(w, ot * 16 + l16, cg * 32 + 8 * g + j, u, v), h, m, l);
        t[0].v[j] = h; t[1].v[j] = m; t[2].v[j] = l;
    }
#pragma unroll
    for (int q = 0; q < 3; ++q) wfrag[(size_t)((ot * G::KB + kb) * 3 + q) * 64 + lane] = t[q].u;
}
template <class SP, bool DGRAD>
__global__ __launch_bounds__(256) void conv_fwd_filter_fragments_kernel(const float *__restrict__ w, u32x4 *__restrict__ wfrag) {
    conv_fwd_filter_fragments_thread<SP, DGRAD>(w, wfrag, blockIdx.x * 256 + threadIdx.x);
}

// NW wavefronts per block (4 or 8).  ONE: operands rounded to bfloat16 (the reduced-precision variant): one term,
// one product.  DGRAD: x = dY [SP::C][SP::H - 2 PAD][SP::W - 2 PAD], w = the layer's filters [SP::C][SP::OC][KS][KS],
// aux = the layer's input (ReLU mask), y = dX; otherwise aux = bias.
template <class SP, int NW, bool ONE, bool DGRAD>
__global__ __launch_bounds__(64 * NW, 1) void conv_fwd_bf16x6_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                                     const float *__restrict__ aux, float *__restrict__ y,
                                                                     int nframes, const u32x4 *__restrict__ wfrag) {
    typedef ConvFwdBf16Geom<SP> G;
    static_assert(SP::C % 32 == 0 && SP::OC == 64, "32 k channels in, 64 filters out");
    static_assert(NW == 4 || NW == 8, "one or two wavefronts per SIMD");
    constexpr int C = SP::C, HW = SP::H * SP::W, KS = SP::KS, S = SP::S, OW = SP::OW, NPIX = SP::NPIX;
    constexpr int CG = G::CG, KB = G::KB, NT = G::NT, PIT = G::PIT, PLANE = G::PLANE;
    constexpr int NTERM = ONE ? 1 : 3, NTHR = 64 * NW;
    constexpr int PG = NW / 4, TPW = (NT + PG - 1) / PG;           // pixel groups; pixel tiles per wavefront
    static_assert(!DGRAD || S == 1, "input gradient: stride 1 only");
    constexpr int PAD = DGRAD ? KS - 1 : 0;
    constexpr int SH = SP::H - 2 * PAD, SW = SP::W - 2 * PAD, SHW = SH * SW;  // the frame as it sits in memory
    constexpr int NITEM = (C / 4) * SHW, DPT = (NITEM + NTHR - 1) / NTHR;     // items: 4 channels of one pixel
    extern __shared__ __attribute__((aligned(16))) unsigned char cf_smem[];   // [term][pixel][channel] bf16

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int ot = wave % 4, pg = wave / 4;

    // the first frame is asked for before the filters are prepared
    int src_off[DPT], dst_off[DPT];
#pragma unroll
    for (int i = 0; i < DPT; ++i) {
        const int e = min(tid + NTHR * i, NITEM - 1);
        const int cq = e / SHW, pix = e % SHW;
        src_off[i] = 4 * cq * SHW + pix;
        dst_off[i] = G::pixel(pix / SW + PAD, pix % SW + PAD) * PIT + 8 * cq;
    }
    float pre[DPT][4];
    auto fetch = [&](int f) {
        const float *src = x + (size_t)f * (C * SHW);
#pragma unroll
        for (int i = 0; i < DPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) pre[i][j] = src[src_off[i] + j * SHW];
    };
    int f = blockIdx.x;
    fetch(min(f, nframes - 1));

    // filter fragments of my tile: row = filter 16 ot + l16, k = (tap, channel 32 cg + 8 g .. + 7)
    Bf16x8Bits wq[KB][NTERM];
    if (wfrag) {
        const u32x4 *src = wfrag + (size_t)(ot * KB) * 3 * 64 + lane;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int q = 0; q < NTERM; ++q) wq[kb][q].u = src[(kb * 3 + q) * 64];
    } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int tap = kb / CG, cg = kb % CG, u = tap / KS, v = tap % KS;
            Bf16x8Bits t[3];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                __bf16 h, m, l;
                split3(conv_fwd_filter_value<SP, DGRAD>(w, ot * 16 + l16, cg * 32 + 8 * g + j, u, v), h, m, l);
                t[0].v[j] = h; t[1].v[j] = m; t[2].v[j] = l;
            }
#pragma unroll
            for (int q = 0; q < NTERM; ++q) wq[kb][q] = t[q];
        }
    }
    float bv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = DGRAD ? 0.f : aux[ot * 16 + 4 * g + r];
    if (DGRAD)                                // the border stays zero: staging writes the interior only
        for (int e = tid; e < NTERM * PLANE / 16; e += NTHR) ((u32x4 *)cf_smem)[e] = u32x4{0u, 0u, 0u, 0u};

    int pbyte[TPW], pidx[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int t = pg + PG * i;
        int p = 16 * t + l16;
        const bool ok = t < NT && p < NPIX;
        if (!ok) p = 0;
        pbyte[i] = ((p / OW) * S * SP::W + (p % OW)) * PIT + 16 * g;        // pixel (S oy, S ox) of the plane
        pidx[i] = ok ? p : -1;
    }

    for (; f < nframes; f += gridDim.x) {
        __syncthreads();                      // the last frame's planes have been read
#pragma unroll
        for (int i = 0; i < DPT; ++i)
            if (tid + NTHR * i < NITEM) {
                uint2 o3[3];
                split3_pair(pre[i][0], pre[i][1], o3[0].x, o3[1].x, o3[2].x);
                split3_pair(pre[i][2], pre[i][3], o3[0].y, o3[1].y, o3[2].y);
#pragma unroll
                for (int q = 0; q < NTERM; ++q) *(uint2 *)(cf_smem + q * PLANE + dst_off[i]) = o3[q];
            }
        __syncthreads();
        fetch(min(f + (int)gridDim.x, nframes - 1));
        float mk[DGRAD ? TPW : 1][4];
        if (DGRAD) {
            const float *mb = aux + (size_t)f * SP::OC * NPIX;
#pragma unroll
            for (int i = 0; i < TPW; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) mk[i][r] = mb[(ot * 16 + 4 * g + r) * NPIX + max(pidx[i], 0)];
        }
        floatx4 acc[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
        // pixel tiles in groups of at most four: the accumulators of a group take one term product each in turn
        constexpr int IG = TPW <= 4 ? TPW : 3;
#pragma unroll
        for (int i0 = 0; i0 < TPW; i0 += IG) {
            // the operands of k-block kb + 1 are read while the products of k-block kb run (one wavefront per SIMD:
            // nobody else hides the LDS latency)
            Bf16x8Bits b[2][IG][NTERM];
            auto read_b = [&](int kb, int buf) {
                const int tap = kb / CG, cg = kb % CG, u = tap / KS, v = tap % KS;
                const int koff = G::pixel(u, v) * PIT + cg * 64;         // pixel (S oy + u, S ox + v) from there
#pragma unroll
                for (int ii = 0; ii < IG; ++ii)
                    if (i0 + ii < TPW) {
#pragma unroll
                        for (int q = 0; q < NTERM; ++q)
                            b[buf][ii][q].u = *(const u32x4 *)(cf_smem + q * PLANE + pbyte[i0 + ii] + koff);
                    }
            };
            read_b(0, 0);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                if (kb + 1 < KB) read_b(kb + 1, (kb + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
                constexpr int NPROD = ONE ? 1 : 6;
                constexpr int PA[6] = {2, 1, 0, 1, 0, 0}, PB[6] = {0, 1, 2, 0, 1, 0};      // smallest products first
#pragma unroll
                for (int q = 0; q < NPROD; ++q) {
                    const int ai = ONE ? 0 : PA[q], bi = ONE ? 0 : PB[q];
#pragma unroll
                    for (int ii = 0; ii < IG; ++ii)
                        if (i0 + ii < TPW)
                            acc[i0 + ii] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[kb][ai % NTERM].v, b[kb & 1][ii][bi % NTERM].v,
                                                                                   acc[i0 + ii], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        float *yb = y + (size_t)f * SP::OC * NPIX;
#pragma unroll
        for (int i = 0; i < TPW; ++i)
            if (pidx[i] >= 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float val = acc[i][r] + bv[r];
                    yb[(ot * 16 + 4 * g + r) * NPIX + pidx[i]] = DGRAD ? (mk[i][r] > 0.f ? val : 0.f) : (val > 0.f ? val : 0.f);
                }
            }
    }
}

// `blocks`: how many blocks the chip holds at once.
template <class SP, int NW, bool DGRAD>
inline hipError_t launch_conv_bf16x6_impl(const float *x, const float *w, const float *aux, float *y, int nframes,
                                          hipStream_t s, int blocks, int rb, const u32x4 *wfrag) {
    if (nframes <= 0) return hipSuccess;
    typedef ConvFwdBf16Geom<SP> G;
    const int grid = nframes < blocks ? nframes : blocks;
    static bool attr_set = false;          // once per layer shape: let the kernels use more than 64 KB of LDS
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)conv_fwd_bf16x6_kernel<SP, NW, false, DGRAD>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(false));
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)conv_fwd_bf16x6_kernel<SP, NW, true, DGRAD>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, G::lds_bytes(true));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    if (rb)
        ga3c::launch((conv_fwd_bf16x6_kernel<SP, NW, true, DGRAD>), dim3(grid), dim3(64 * NW), G::lds_bytes(true), s, x, w,
                           aux, y, nframes, wfrag);
    else
        ga3c::launch((conv_fwd_bf16x6_kernel<SP, NW, false, DGRAD>), dim3(grid), dim3(64 * NW), G::lds_bytes(false), s, x,
                           w, aux, y, nframes, wfrag);
    return hipGetLastError();
}

template <class SP, int NW>
inline hipError_t launch_conv_fwd_bf16x6(const float *x, const float *w, const float *bias, float *y, int nframes,
                                         hipStream_t s, int blocks, int rb = 0, const u32x4 *wfrag = nullptr) {
    return launch_conv_bf16x6_impl<SP, NW, false>(x, w, bias, y, nframes, s, blocks, rb, wfrag);
}

// The ready-made fragments of layer SP's forward pass: wfrag [ConvFwdBf16Geom<SP>::FRAG_VECS].
template <class SP>
inline hipError_t launch_conv_fwd_filter_fragments(const float *w, u32x4 *wfrag, hipStream_t s) {
    ga3c::launch((conv_fwd_filter_fragments_kernel<SP, false>), dim3(ConvFwdBf16Geom<SP>::KB), dim3(256), 0, s, w, wfrag);
    return hipGetLastError();
}

// Input gradient of the stride-1 layer SP: dy [n][OC][OH][OW], w the layer's filters, xin the layer's input
// [n][C][H][W] (its ReLU mask), dx [n][C][H][W].
template <class SP, int NW>
inline hipError_t launch_conv_dgrad_s1_bf16x6(const float *dy, const float *w, const float *xin, float *dx, int nframes,
                                              hipStream_t s, int blocks, int rb = 0, const u32x4 *wfrag = nullptr) {
    static_assert(SP::S == 1, "stride 1");
    typedef ConvSpec<float, SP::OC, SP::OH + 2 * (SP::KS - 1), SP::OW + 2 * (SP::KS - 1), SP::C, SP::KS, 1> Pseudo;
    static_assert(Pseudo::OH == SP::H && Pseudo::OW == SP::W, "the padded correlation gives back the input size");
    return launch_conv_bf16x6_impl<Pseudo, NW, true>(dy, w, xin, dx, nframes, s, blocks, rb, wfrag);
}

// The ready-made fragments of that input gradient (of the pseudo-layer: as many vectors as conv_dgrad_s1_frag_vecs).
template <class SP>
constexpr int conv_dgrad_s1_frag_vecs() {
    return ConvFwdBf16Geom<ConvSpec<float, SP::OC, SP::OH + 2 * (SP::KS - 1), SP::OW + 2 * (SP::KS - 1), SP::C, SP::KS, 1>>::FRAG_VECS;
}
template <class SP>
inline hipError_t launch_conv_dgrad_s1_filter_fragments(const float *w, u32x4 *wfrag, hipStream_t s) {
    typedef ConvSpec<float, SP::OC, SP::OH + 2 * (SP::KS - 1), SP::OW + 2 * (SP::KS - 1), SP::C, SP::KS, 1> Pseudo;
    ga3c::launch((conv_fwd_filter_fragments_kernel<Pseudo, true>), dim3(ConvFwdBf16Geom<Pseudo>::KB), dim3(256), 0, s, w, wfrag);
    return hipGetLastError();
}

}  // namespace ga3c
