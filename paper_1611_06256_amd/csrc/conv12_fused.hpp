// First two convolution layers of the small network (paper Sec. 3.2) in one
// kernel: 16 filters 8x8 stride 4 on the 4x84x84 byte frame, ReLU, 32 filters
// 4x4 stride 2, ReLU.  The 16x20x20 activations between the two layers never
// leave the compute unit unless the caller wants them (training keeps them for
// the backward pass).
//
// Arithmetic as in conv1_bf16x3.hpp and conv2_bf16x6.hpp: bytes are exact in
// bf16, fp32 numbers are split into three bf16 terms, products accumulate in
// fp32 on v_mfma_f32_16x16x32_bf16.
//
// One block of 8 wavefronts per compute unit works as a two-stage pipeline:
// wavefronts 0..3 run layer 1 of frame i (and split its output into three bf16
// planes in LDS) while wavefronts 4..7 run layer 2 of frame i - 1 from the planes
// written one iteration earlier.  The two groups hold only their own filters in
// registers and share the matrix cores of each SIMD.
//
// Matrix and vector instructions of the two groups share each SIMD and their times add up (about 2 us of MFMAs and
// 1.3 us of vector work per frame); the LDS layout is chosen so that operand reads stay out of the way:
//  * the planes hold each channel as 2x2 pixel blocks, [row pair][column pair]
//    [2][2]: the 2 rows x 4 columns a lane feeds to one MFMA are 16 contiguous
//    bytes (the filter taps are permuted to that order when they are loaded);
//  * a layer-2 wavefront computes both filter tiles from one fetch of the
//    activations and takes half of the 256 taps instead; the two wavefronts of
//    a pair swap half of their partial sums through LDS and finish one filter
//    tile each, one iteration later, so that no extra barrier is needed.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"
#include "dense_gemm_bf16x6.hpp"

namespace ga3c {

constexpr int C12_XS = 7 * 256 * 16;                 // bf16 elements of the staged frame (28 224 used)
constexpr int C12_Y1 = 16 * 400;                     // elements of one plane of the layer-1 output
constexpr int C12_EX = 4 * 3 * 4 * 64;               // floats one exchange buffer holds: [wavefront][tile][r][lane]
constexpr size_t C12_LDS_BYTES = sizeof(__bf16) * (C12_XS + 2 * 3 * C12_Y1) + sizeof(float) * 2 * C12_EX;

// Where the single-frame variant leaves the layer-2 output: the second buffer of layer-1 planes, which one frame never
// uses; everything below this offset is free once layer 2 has run.
constexpr size_t C12_Y2S_OFF = sizeof(__bf16) * (C12_XS + 3 * C12_Y1);

constexpr int C12_FRAG_SET = 3 * 8 * 64;             // 16-byte vectors of one fragment set: [term][slot][lane]

// Filters of both layers as MFMA operand fragments, split into three bf16 terms
// (w = hi + mid + lo exactly), in the order the forward kernel's lanes hold them.
// Set 0: layer 1, slot j = tap block j of filter l16 (taps 32 j + 8 g ..).
// Sets 1 + kh: layer 2, slot j = tap block 4 kh + j/2 of filter 16 (j%2) + l16, taps in the
// order of a 2x2-block pair: (r0c0 r0c1 r1c0 r1c1 r0c2 r0c3 r1c2 r1c3).
// One block of 192 threads; runs whenever the parameters change.
__global__ __launch_bounds__(192) void conv12_filter_fragments_kernel(const float *__restrict__ w1,
                                                                      const float *__restrict__ w2,
                                                                      u32x4 *__restrict__ frag, int rb) {
    constexpr int K = 256;
    const int lane = threadIdx.x & 63, set = threadIdx.x >> 6;
    const int l16 = lane & 15, g = lane >> 4, kh = set - 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float *src = set == 0 ? w1 + (size_t)l16 * K + 32 * j + 8 * g
                                    : w2 + (size_t)((j & 1) * 16 + l16) * K + 32 * (4 * kh + (j >> 1)) + 8 * g;
        const float4 a = *(const float4 *)src, b = *(const float4 *)(src + 4);
        const float f[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        constexpr int PERM[8] = {0, 1, 4, 5, 2, 3, 6, 7};
        Bf16x8Bits h, m, l;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            __bf16 th, tm, tl;
            split3(set == 0 ? f[e] : f[PERM[e]], th, tm, tl, rb);
            h.v[e] = th; m.v[e] = tm; l.v[e] = tl;
        }
        u32x4 *dst = frag + (size_t)set * C12_FRAG_SET + lane;
        dst[(0 * 8 + j) * 64] = h.u;
        dst[(1 * 8 + j) * 64] = m.u;
        dst[(2 * 8 + j) * 64] = l.u;
    }
}

// The same fragments, four filter taps at a time: `rel` (a multiple of 4) is the index of v.x in the layer's
// filter tensor [oc][256].  Lets the kernel that updates the parameters keep the fragments current.
__device__ __forceinline__ void conv12_store_fragment4(u32x4 *__restrict__ frag, int layer2, int rel, const float4 v,
                                                       int rb) {
    const int oc = rel >> 8, k = rel & 255;
    const int kb = k >> 5, g = (k >> 3) & 3, e0 = k & 7;               // e0 = 0 or 4
    const float f[4] = {v.x, v.y, v.z, v.w};
    union { __bf16 h[4]; uint32_t u[2]; } o[3];
#pragma unroll
    for (int e = 0; e < 4; ++e) split3(f[e], o[0].h[e], o[1].h[e], o[2].h[e], rb);
    if (!layer2) {
        uint32_t *dst = (uint32_t *)(frag + (size_t)kb * 64 + g * 16 + oc) + e0 / 2;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            dst[(size_t)t * 8 * 64 * 4] = o[t].u[0];
            dst[(size_t)t * 8 * 64 * 4 + 1] = o[t].u[1];
        }
    } else {
        const int kh = kb >> 2, j = 2 * (kb & 3) + (oc >> 4);
        // taps e0, e0+1 go to positions e0/2, e0/2+1 of the vector; taps e0+2, e0+3 to positions 4 + e0/2, ..
        uint32_t *dst = (uint32_t *)(frag + (size_t)(1 + kh) * C12_FRAG_SET + (size_t)j * 64 + g * 16 + (oc & 15)) + e0 / 4;
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            dst[(size_t)t * 8 * 64 * 4] = o[t].u[0];
            dst[(size_t)t * 8 * 64 * 4 + 2] = o[t].u[1];
        }
    }
}

inline hipError_t launch_conv12_filter_fragments(const float *w1, const float *w2, u32x4 *frag, hipStream_t s, int rb) {
    ga3c::launch(conv12_filter_fragments_kernel, dim3(1), dim3(192), 0, s, w1, w2, frag, rb);
    return hipGetLastError();
}

// x: [n][4][84][84] bytes; frag: the three fragment sets; b1 [16], b2 [32];
// y1: [n][16][400] or nullptr; y2: [n][32][81].  Frames blockIdx.x, + gridDim.x, ...
// ONE: the reduced-precision variant (operands rounded to bfloat16): only the first
// term of every operand exists, so one MFMA per tap block replaces three / six and
// only the first plane of the layer-1 output is written and read.
// KEEP: the layer-1 output is also written to y1 (a template parameter rather than a test of the pointer, so that
// the stores do not cut the epilogue into a basic block each).
//
// The body is a device function so that a second kernel can run it on one frame and go on with the rest of the
// network: the block works on frames first, first + stride, ... below nframes.  TO_LDS: the layer-2 output of the
// (single) frame goes to LDS instead of y2, as floats [32][81] at C12_Y2S_OFF; the caller synchronises before
// reading it.  idle(it) is called by the layer-1 wavefronts in the iterations in which they have no frame left to
// work on (while layer 2 runs), idle2() by the layer-2 wavefronts in the first iteration, when there is no layer-1
// output yet.
template <bool ONE, bool KEEP, bool TO_LDS, class Idle, class Idle2>
__device__ __forceinline__ void conv12_fused_block(const uint8_t *__restrict__ x, const u32x4 *__restrict__ frag,
                                                   const float *__restrict__ b1, const float *__restrict__ b2,
                                                   float *__restrict__ y1, float *__restrict__ y2, int first, int stride,
                                                   int nframes, float scale, unsigned char *c12_smem, Idle idle, Idle2 idle2) {
    constexpr int CHW1 = 4 * 84 * 84, W1 = 84, NPIX1 = 400, OW1 = 20;
    constexpr int NV = CHW1 / 16, VPT = 7;                         // 16-byte vectors of a frame, per layer-1 thread
    constexpr int HW2 = 400, NPIX2 = 81, OW2 = 9, OC2 = 32;
    __bf16 *xs = (__bf16 *)c12_smem;
    __bf16 *ys = xs + C12_XS;                                      // [2][3][C12_Y1]
    float *exb = (float *)(ys + 2 * 3 * C12_Y1);                   // [2][C12_EX]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool layer1 = wave < 4;
    const int rw = wave & 3;                                       // wavefront within its group
    const int rt = tid & 255;                                      // thread within its group
    const int l16 = lane & 15, g = lane >> 4;
    const int pg = rw >> 1, kh = rw & 1;                           // layer 2: pixel tiles pg, pg+2, pg+4; taps 128 kh ..

    // the first frame is requested before anything else, so that it travels while the filters are prepared
    u32x4 pre[VPT];
    int vidx[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) vidx[i] = min(rt + 256 * i, NV - 1);
    if (layer1) {
        const u32x4 *src = (const u32x4 *)(x + (size_t)first * CHW1);
#pragma unroll
        for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
    }

    // My filter fragments, split into three bf16 terms ahead of time (conv12_filter_fragments_kernel).  Every block
    // of the launch wants the same 72 KB at the same moment, and a wavefront's copy is 24 KB, so what the blocks ask
    // of the L2 in their first microsecond is kept small: the four layer-1 wavefronts fetch their common set once
    // between them and hand it round through LDS (the exchange buffers, which nobody uses before the second
    // iteration); the layer-2 wavefronts fetch theirs during the first iteration, in which they have nothing else to
    // do and the layer-1 set has already arrived.
    constexpr int NTERM = ONE ? 1 : 3;
    constexpr int FPT = NTERM * 8 * 64 / 256;                      // vectors of the layer-1 set per layer-1 thread
    static_assert(sizeof(u32x4) * NTERM * 8 * 64 <= sizeof(float) * 2 * C12_EX, "the layer-1 set fits the exchange buffers");
    bf16x8 wq[3][8];
    u32x4 fpre[FPT];
    if (layer1) {
#pragma unroll
        for (int i = 0; i < FPT; ++i) fpre[i] = frag[rt + 256 * i];
    }
    float bv[4];                                                   // layer 1: bv[0] = bias of filter l16; layer 2 finishes filter tile kh
#pragma unroll
    for (int r = 0; r < 4; ++r) bv[r] = layer1 ? b1[l16] : b2[kh * 16 + 4 * g + r];

    const int grid = stride;
    const int n = TO_LDS ? 1 : (nframes - first + grid - 1) / grid;      // frames of this block (>= 1)

    floatx4 keep[3];                                               // layer 2: my filter tile's sums of the previous frame
#pragma unroll
    for (int i = 0; i < 3; ++i) keep[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    // iteration it: layer 1 of frame it, layer 2 of frame it - 1, last step of layer 2 of frame it - 2
    // (one frame: the three iterations are written out, so that each keeps only what it needs in registers)
    auto stage_frame = [&]() {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            u32x4 a, b;
            bytes_to_bf16(pre[i], a, b);
            u32x4 *dst = (u32x4 *)(xs + (size_t)(rt + 256 * i) * 16);
            dst[0] = a; dst[1] = b;
        }
    };
    // before the first iteration: the first frame and the layer-1 filter set go to LDS, then everybody takes its filters
    if (layer1) {
        stage_frame();
#pragma unroll
        for (int i = 0; i < FPT; ++i) ((u32x4 *)exb)[rt + 256 * i] = fpre[i];
    }
    __syncthreads();
    {
        if (layer1) {
            const u32x4 *src = (const u32x4 *)exb + lane;
#pragma unroll
            for (int t = 0; t < NTERM; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    Bf16x8Bits v;
                    v.u = src[(t * 8 + j) * 64];
                    wq[t][j] = v.v;
                }
        } else {
            const u32x4 *src = frag + (size_t)(1 + kh) * C12_FRAG_SET + lane;
#pragma unroll
            for (int t = 0; t < NTERM; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    Bf16x8Bits v;
                    v.u = src[(t * 8 + j) * 64];
                    wq[t][j] = v.v;
                }
        }
    }
#pragma unroll(TO_LDS ? 3 : 1)
    for (int it = 0; it <= n + 1; ++it) {
        if (it > 0) {
            __syncthreads();          // layer 1 of the previous frame has read xs; layer 2 has read its planes
            if (layer1 && it < n) stage_frame();
            __syncthreads();
        }
        if (layer1) {
            if (it < n) {
                const int f = first + it * grid;
                {
                    const u32x4 *src = (const u32x4 *)(x + (size_t)min(f + grid, nframes - 1) * CHW1);
#pragma unroll
                    for (int i = 0; i < VPT; ++i) pre[i] = src[vidx[i]];
                }
                __bf16 *yp = ys + (it & 1) * 3 * C12_Y1;
                float *yb = KEEP ? y1 + (size_t)f * 16 * NPIX1 : nullptr;
                // pixel tiles rw, rw + 4, ...: 25 tiles, wavefront 0 takes seven, the others six.
                // Six independent accumulators: consecutive MFMAs never depend on each other.
                auto tile_base = [&](int t) {
                    const int p = t * 16 + l16;
                    return (p / OW1) * 4 * W1 + (p % OW1) * 4 + g * W1;
                };
                auto operand = [&](int base, int kb) {
                    const __bf16 *src = xs + base + (kb / 2) * (84 * 84) + 4 * (kb % 2) * W1;   // 8-byte aligned
                    const uint2 lo = *(const uint2 *)src, hi = *(const uint2 *)(src + 4);
                    Bf16x8Bits xv;
                    xv.u = u32x4{lo.x, lo.y, hi.x, hi.y};
                    return xv.v;
                };
                // The MFMAs below take the pixels as rows and the filters as columns, so a lane ends up with four
                // consecutive pixels (16 t + 4 g + r) of filter l16: one 16-byte store to y1, and pixel pairs that are
                // neighbours in the planes' 2x2-block layout (one 4-byte LDS store per pair and term).
                auto finish = [&](int t, const floatx4 acc) {
                    const int p = t * 16 + 4 * g;                           // a multiple of 4: the four pixels share a row
                    const int row = p / OW1, col = p % OW1;
                    const int blk = (row >> 1) * 40 + (col >> 1) * 4 + (row & 1) * 2;      // pixels col, col+1; +4: col+2, col+3
                    float v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        v[r] = acc[r] * scale + bv[0];
                        v[r] = v[r] > 0.f ? v[r] : 0.f;
                    }
                    if (KEEP) *(float4 *)(yb + l16 * NPIX1 + p) = float4{v[0], v[1], v[2], v[3]};
                    // split two values per conversion instruction (v = hi + mid + lo exactly; ONE: v rounded)
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const float a = v[2 * q], b = v[2 * q + 1];
                        const int e0 = l16 * HW2 + blk + 4 * q;             // even: 4-byte aligned
                        const uint32_t hi = pack_bf16_rne(a, b);
                        *(uint32_t *)(yp + e0) = hi;
                        if (!ONE) {
                            const float ra = a - __uint_as_float(hi << 16), rb2 = b - __uint_as_float(hi & 0xffff0000u);
                            const uint32_t mid = pack_bf16_rne(ra, rb2);
                            const uint32_t lo = pack_bf16_rne(ra - __uint_as_float(mid << 16), rb2 - __uint_as_float(mid & 0xffff0000u));
                            *(uint32_t *)(yp + C12_Y1 + e0) = mid;
                            *(uint32_t *)(yp + 2 * C12_Y1 + e0) = lo;
                        }
                    }
                };
                {
                    int base[6];
                    floatx4 acc[6];
#pragma unroll
                    for (int j = 0; j < 6; ++j) {
                        base[j] = tile_base(rw + 4 * j);
                        acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                    for (int kb = 0; kb < 8; ++kb) {
                        bf16x8 xv[6];
#pragma unroll
                        for (int j = 0; j < 6; ++j) xv[j] = operand(base[j], kb);
#pragma unroll
                        for (int term = ONE ? 0 : 2; term >= 0; --term)
#pragma unroll
                            for (int j = 0; j < 6; ++j)
                                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xv[j], wq[term][kb], acc[j], 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < 6; ++j) finish(rw + 4 * j, acc[j]);
                }
                if (rw == 0) {
                    const int base = tile_base(24);
                    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kb = 0; kb < 8; ++kb) {
                        const bf16x8 xv = operand(base, kb);
#pragma unroll
                        for (int term = ONE ? 0 : 2; term >= 0; --term)
                            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xv, wq[term][kb], acc, 0, 0, 0);
                    }
                    finish(24, acc);
                }
            } else {
                idle(it);
            }
        } else {
            if (TO_LDS && it == 0) idle2();
            if (it >= 2) {       // frame it - 2: add what my partner summed over its taps, bias, ReLU, store
                const float *ex = exb + ((it - 1) & 1) * C12_EX + (rw ^ 1) * (3 * 4 * 64);
                float *yb = TO_LDS ? (float *)(c12_smem + C12_Y2S_OFF) : y2 + (size_t)(first + (it - 2) * grid) * OC2 * NPIX2;
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int p = (pg + 2 * i) * 16 + l16;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float v = keep[i][r] + ex[(i * 4 + r) * 64 + lane] + bv[r];
                        if (p < NPIX2) yb[(kh * 16 + 4 * g + r) * NPIX2 + p] = v > 0.f ? v : 0.f;
                    }
                }
            }
            if (it >= 1 && it <= n) {
                const __bf16 *yp = ys + ((it - 1) & 1) * 3 * C12_Y1;
                // a lane's taps of block kb: channel 2 kb + g/2, window rows 2 (g%2) and 2 (g%2) + 1, 4 columns,
                // = column pairs ox and ox + 1 of row pair oy + g%2
                floatx4 acc[3][2];
                int off[3];
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    int p = (pg + 2 * i) * 16 + l16;
                    if (p >= NPIX2) p = 0;
                    off[i] = (g / 2) * HW2 + ((p / OW2) + (g % 2)) * 40 + (p % OW2) * 4 + 2 * (4 * kh) * HW2;
                    acc[i][0] = floatx4{0.f, 0.f, 0.f, 0.f};
                    acc[i][1] = floatx4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int kbl = 0; kbl < 4; ++kbl) {
                    Bf16x8Bits xv[3][3];                             // [tile][term]
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
#pragma unroll
                        for (int term = 0; term < (ONE ? 1 : 3); ++term) {
                            const uint2 *q = (const uint2 *)(yp + term * C12_Y1 + off[i] + 2 * kbl * HW2);   // 8-byte aligned
                            const uint2 lo = q[0], hi = q[1];
                            xv[i][term].u = u32x4{lo.x, lo.y, hi.x, hi.y};
                        }
                    }
                    // the six largest term products, smallest first; six accumulators alternate
                    constexpr int WT[6] = {2, 1, 0, 1, 0, 0}, XT[6] = {0, 1, 2, 0, 1, 0};
#pragma unroll
                    for (int q = ONE ? 5 : 0; q < 6; ++q)          // q = 5 is the product of the two first terms
#pragma unroll
                        for (int i = 0; i < 3; ++i)
#pragma unroll
                            for (int o = 0; o < 2; ++o)
                                acc[i][o] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wq[WT[q]][2 * kbl + o], xv[i][XT[q]].v,
                                                                                    acc[i][o], 0, 0, 0);
                }
                // my partner finishes the other filter tile
                float *ex = exb + (it & 1) * C12_EX + rw * (3 * 4 * 64);
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const floatx4 mine = kh ? acc[i][1] : acc[i][0], other = kh ? acc[i][0] : acc[i][1];
                    keep[i] = mine;
#pragma unroll
                    for (int r = 0; r < 4; ++r) ex[(i * 4 + r) * 64 + lane] = other[r];
                }
            }
        }
    }
}

template <bool ONE, bool KEEP>
__global__ __launch_bounds__(512, 1) void conv12_fused_fwd_kernel(const uint8_t *__restrict__ x,
                                                                  const u32x4 *__restrict__ frag,
                                                                  const float *__restrict__ b1,
                                                                  const float *__restrict__ b2, float *__restrict__ y1,
                                                                  float *__restrict__ y2, int nframes, float scale,
                                                                  int rb) {
    extern __shared__ __attribute__((aligned(16))) unsigned char c12_smem[];
    conv12_fused_block<ONE, KEEP, false>(x, frag, b1, b2, y1, y2, (int)blockIdx.x, (int)gridDim.x, nframes, scale,
                                         c12_smem, [](int) {}, []() {});
}

inline int conv12_fused_blocks(int nframes) { return nframes < 256 ? nframes : 256; }

inline hipError_t launch_conv12_fused_fwd(const uint8_t *x, const u32x4 *frag, const float *b1, const float *b2, float *y1,
                                          float *y2, int nframes, float scale, hipStream_t s, int rb) {
    if (nframes <= 0) return hipSuccess;
    static bool attr_set = false;     // the kernels need more LDS than the default limit
    if (!attr_set) {
        const void *ks[4] = {(const void *)conv12_fused_fwd_kernel<false, false>, (const void *)conv12_fused_fwd_kernel<false, true>,
                             (const void *)conv12_fused_fwd_kernel<true, false>, (const void *)conv12_fused_fwd_kernel<true, true>};
        for (const void *k : ks) {
            const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C12_LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const dim3 grid(conv12_fused_blocks(nframes)), block(512);
#define GA3C_C12_LAUNCH(ONE_, KEEP_)                                                                                          \
    ga3c::launch((conv12_fused_fwd_kernel<ONE_, KEEP_>), grid, block, C12_LDS_BYTES, s, x, frag, b1, b2, y1, y2, nframes, \
                       scale, rb)
    if (rb) { if (y1) GA3C_C12_LAUNCH(true, true); else GA3C_C12_LAUNCH(true, false); }
    else { if (y1) GA3C_C12_LAUNCH(false, true); else GA3C_C12_LAUNCH(false, false); }
#undef GA3C_C12_LAUNCH
    return hipGetLastError();
}

}  // namespace ga3c
