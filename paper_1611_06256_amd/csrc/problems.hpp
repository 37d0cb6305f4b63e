// Operand gathers and epilogues that turn the layers of the policy/value
// network (paper Sec. 3.2) and their gradients into instances of the tiled
// MFMA product in gemm_mfma.hpp.  All tensors are NCHW fp32 except the input
// frames, which are raw bytes.
#pragma once
#include "gemm_mfma.hpp"

namespace ga3c {

// One convolution layer: VALID cross-correlation, C x H x W -> OC x OH x OW,
// kernel KS x KS, stride S.
struct ConvGeom {
    int C, H, W, OC, KS, S, OH, OW;
    int K;       // C*KS*KS, the length of one filter
    int OHW;     // OH*OW
    int CHW;     // C*H*W
    FastDiv dOHW, dOW;
    const int *koff;  // device table, K entries rounded up to 4: c*H*W + u*W + v of filter tap k
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(uint8_t v) { return (float)v; }

__device__ __forceinline__ bool aligned16(const void *p) { return (((uintptr_t)p) & 15) == 0; }

// ---- convolution forward -------------------------------------------------
// D[oc][P] = sum_k W[oc][k] * x[frame(P)][tap k at pixel(P)],  P = frame*OHW + pixel.
// Epilogue: y = max(0, scale*D + bias[oc]); scale = 1/255 for the byte input.
template <class TIn>
struct ConvFwdP {
    int M, N, K;
    ConvGeom g;
    const TIn *x;
    const float *w, *bias;
    float *y;
    float scale;
    int rb = 0;          // round operands to bfloat16

    __device__ __forceinline__ void krange(int, int &kbeg, int &kend) const { kbeg = 0; kend = K; }

    __device__ __forceinline__ float4 loadA(int m, int k, int kend, int) const {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m >= M) return v;
        const float *p = w + (size_t)m * K + k;
        if (k + 3 < kend && aligned16(p)) return *(const float4 *)p;
        if (k < kend) v.x = p[0];
        if (k + 1 < kend) v.y = p[1];
        if (k + 2 < kend) v.z = p[2];
        if (k + 3 < kend) v.w = p[3];
        return v;
    }
    __device__ __forceinline__ float4 loadB(int n, int k, int kend, int) const {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n >= N || k >= kend) return v;
        uint32_t b, pix, i, j;
        g.dOHW.divmod((uint32_t)n, b, pix);
        g.dOW.divmod(pix, i, j);
        const TIn *base = x + (size_t)b * g.CHW + (i * g.S) * g.W + j * g.S;
        const int4 ko = *(const int4 *)(g.koff + k);   // table is padded to a multiple of 4
        v.x = to_f32(base[ko.x]);
        if (k + 1 < kend) v.y = to_f32(base[ko.y]);
        if (k + 2 < kend) v.z = to_f32(base[ko.z]);
        if (k + 3 < kend) v.w = to_f32(base[ko.w]);
        return v;
    }
    __device__ __forceinline__ void store(int m, int n, float v, int) const {
        uint32_t b, pix;
        g.dOHW.divmod((uint32_t)n, b, pix);
        float r = v * scale + bias[m];
        y[((size_t)b * g.OC + m) * g.OHW + pix] = r > 0.f ? r : 0.f;
    }
};

// ---- convolution weight gradient -------------------------------------------
// D[oc][kk] = sum_P dY[P][oc] * x[frame(P)][tap kk at pixel(P)], with one more
// column kk = K whose operand is 1, which yields the bias gradient.  The sum
// over P is cut into chunks (blockIdx.z); each chunk writes its own partial
// D, and a second kernel adds the partials in a fixed order.  The input scale
// (1/255 for bytes) multiplies the finished sums, not the operands.
template <class TIn>
struct ConvWgradP {
    int M, N, K;        // M = OC, N = g.K + 1, K = frames*OHW
    int kchunk;
    ConvGeom g;
    const TIn *x;
    const float *dy;
    float *ws;
    float scale;
    int rb = 0;          // round operands to bfloat16

    __device__ __forceinline__ void krange(int z, int &kbeg, int &kend) const {
        kbeg = z * kchunk;
        kend = min(K, kbeg + kchunk);
    }
    __device__ __forceinline__ float4 loadA(int m, int k, int kend, int) const {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m >= M || k >= kend) return v;
        uint32_t b, pix;
        g.dOHW.divmod((uint32_t)k, b, pix);
        float r[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (k + t < kend) r[t] = dy[((size_t)b * g.OC + m) * g.OHW + pix];
            if (++pix == (uint32_t)g.OHW) { pix = 0; ++b; }
        }
        return make_float4(r[0], r[1], r[2], r[3]);
    }
    __device__ __forceinline__ float4 loadB(int n, int k, int kend, int) const {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n >= N || k >= kend) return v;
        float r[4] = {0.f, 0.f, 0.f, 0.f};
        if (n == g.K) {
#pragma unroll
            for (int t = 0; t < 4; ++t) r[t] = (k + t < kend) ? 1.f : 0.f;
            return make_float4(r[0], r[1], r[2], r[3]);
        }
        const int ko = g.koff[n];
        uint32_t b, pix, i, j;
        g.dOHW.divmod((uint32_t)k, b, pix);
        g.dOW.divmod(pix, i, j);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (k + t < kend) r[t] = to_f32(x[(size_t)b * g.CHW + (i * g.S) * g.W + j * g.S + ko]);
            if (++j == (uint32_t)g.OW) { j = 0; if (++i == (uint32_t)g.OH) { i = 0; ++b; } }
        }
        return make_float4(r[0], r[1], r[2], r[3]);
    }
    __device__ __forceinline__ void store(int m, int n, float v, int z) const {
        ws[((size_t)z * M + m) * N + n] = n == g.K ? v : v * scale;
    }
};

// ---- convolution input gradient, one stride phase ---------------------------
// Input pixel (y, x) = (S*iy + ry, S*ix + rx) of phase (ry, rx) receives
//   dX[c][y][x] = sum_{oc,a,e} dY[oc][iy-a][ix-e] * W[oc][c][ry+S*a][rx+S*e]
// over the taps that exist, i.e. a stride-1 correlation of dY with the
// sub-sampled, flipped filter.  D[c][Pp], Pp = frame*nH*nW + iy*nW + ix.
// Epilogue: multiply by the ReLU mask of the layer below (its saved output).
struct ConvDgradP {
    int M, N, K;        // M = C, N = frames*nH*nW, K = OC*TA*TB
    ConvGeom g;
    int ry, rx, nH, nW, TA, TB;
    FastDiv dNHW, dNW, dTAB, dTB;
    const float *w, *dy, *xmask;
    float *dx;
    int rb = 0;          // round operands to bfloat16

    __device__ __forceinline__ void krange(int, int &kbeg, int &kend) const { kbeg = 0; kend = K; }

    __device__ __forceinline__ float4 loadA(int m, int k, int kend, int) const {
        float r[4] = {0.f, 0.f, 0.f, 0.f};
        if (m < M) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k + t >= kend) break;
                uint32_t oc, rem, a, e;
                dTAB.divmod((uint32_t)(k + t), oc, rem);
                dTB.divmod(rem, a, e);
                const int u = ry + g.S * a, v = rx + g.S * e;
                if (u < g.KS && v < g.KS) r[t] = w[(size_t)oc * g.K + (m * g.KS + u) * g.KS + v];
            }
        }
        return make_float4(r[0], r[1], r[2], r[3]);
    }
    __device__ __forceinline__ float4 loadB(int n, int k, int kend, int) const {
        float r[4] = {0.f, 0.f, 0.f, 0.f};
        if (n < N) {
            uint32_t b, rem, iy, ix;
            dNHW.divmod((uint32_t)n, b, rem);
            dNW.divmod(rem, iy, ix);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k + t >= kend) break;
                uint32_t oc, r2, a, e;
                dTAB.divmod((uint32_t)(k + t), oc, r2);
                dTB.divmod(r2, a, e);
                const int yy = (int)iy - (int)a, xx = (int)ix - (int)e;
                if ((unsigned)yy < (unsigned)g.OH && (unsigned)xx < (unsigned)g.OW)
                    r[t] = dy[((size_t)b * g.OC + oc) * g.OHW + yy * g.OW + xx];
            }
        }
        return make_float4(r[0], r[1], r[2], r[3]);
    }
    __device__ __forceinline__ void store(int m, int n, float v, int) const {
        uint32_t b, rem, iy, ix;
        dNHW.divmod((uint32_t)n, b, rem);
        dNW.divmod(rem, iy, ix);
        const size_t idx = ((size_t)b * g.C + m) * (g.H * g.W) + (g.S * iy + ry) * g.W + g.S * ix + rx;
        dx[idx] = xmask[idx] > 0.f ? v : 0.f;
    }
};

// ---- plain strided product ---------------------------------------------------
// A(m,k) = A[m*sAm + k*sAk], B(n,k) = B[n*sBn + k*sBk]; optional last column of
// ones in B (bias gradients).  Epilogues: partial sums for split-k, bias+ReLU,
// or the ReLU mask of a saved activation.
enum { EPI_PARTIAL = 0, EPI_BIAS_RELU = 1, EPI_MASK = 2 };

template <int EPI, bool ONES_COL>
struct GemmP {
    int M, N, K;
    int kchunk;
    const float *A, *B;
    long sAm, sAk, sBn, sBk;
    float *C;            // EPI_PARTIAL: workspace [z][M][N]; otherwise output with row pitch ldc
    long ldc;
    const float *aux;    // bias[n] or mask[m*ldc + n]
    int rb = 0;          // round operands to bfloat16

    __device__ __forceinline__ void krange(int z, int &kbeg, int &kend) const {
        kbeg = z * kchunk;
        kend = min(K, kbeg + kchunk);
    }
    __device__ __forceinline__ static float4 ld(const float *p, long sk, int k, int kend) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (sk == 1 && k + 3 < kend && aligned16(p)) return *(const float4 *)p;
        if (k < kend) v.x = p[0];
        if (k + 1 < kend) v.y = p[sk];
        if (k + 2 < kend) v.z = p[2 * sk];
        if (k + 3 < kend) v.w = p[3 * sk];
        return v;
    }
    __device__ __forceinline__ float4 loadA(int m, int k, int kend, int) const {
        if (m >= M) return make_float4(0.f, 0.f, 0.f, 0.f);
        return ld(A + m * sAm + k * sAk, sAk, k, kend);
    }
    __device__ __forceinline__ float4 loadB(int n, int k, int kend, int) const {
        if (n >= N) return make_float4(0.f, 0.f, 0.f, 0.f);
        if (ONES_COL && n == N - 1)
            return make_float4(k < kend ? 1.f : 0.f, k + 1 < kend ? 1.f : 0.f, k + 2 < kend ? 1.f : 0.f,
                               k + 3 < kend ? 1.f : 0.f);
        return ld(B + n * sBn + k * sBk, sBk, k, kend);
    }
    __device__ __forceinline__ void store(int m, int n, float v, int z) const {
        if (EPI == EPI_PARTIAL) {
            C[((size_t)z * M + m) * N + n] = v;
        } else if (EPI == EPI_BIAS_RELU) {
            float r = v + aux[n];
            C[m * ldc + n] = r > 0.f ? r : 0.f;
        } else {
            C[m * ldc + n] = aux[m * ldc + n] > 0.f ? v : 0.f;
        }
    }
};

}  // namespace ga3c
