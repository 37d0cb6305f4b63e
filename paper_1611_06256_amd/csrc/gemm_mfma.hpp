// Tiled fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_16x16x4_f32) with
// pluggable operand gathers and epilogues.
//
//   D[m][n] = sum_k A(m,k) * B(n,k)            m < M, n < N, k in [kbeg, kend)
//
// With P::rb set, both operands are rounded to bfloat16 as they are fetched
// (products of two bfloat16 numbers are exact in fp32, so this is what a bf16
// MFMA with fp32 accumulation computes).
//
// A problem type P supplies the two gathers and the store, so that the same
// kernel serves convolution forward (B = implicit im2col), weight gradients
// (reduction over pixels, split over blockIdx.z), the stride-phase form of the
// transposed convolution, and the plain fully connected products.
//
// Tile: BM = 16*TM*WM rows by BN = 16*TN*WN columns per block of WM*WN
// wavefronts, BK = 32.  Both operands are staged in LDS as float4 "k-quads":
// tile element (row, k) lives at quad[k/4][row].{x,y,z,w}[k%4], one spare row
// per quad line so that writes along k and reads along rows are both free of
// bank conflicts.  A lane (l16 = lane%16, g = lane/16) reads quad 4*kb+g of
// its row once and feeds it to four MFMAs; MFMA number t of that group sums
// over k = {16*kb + 4*g + t : g = 0..3}.  A and B use the same partition of k,
// which is all a dot product needs.
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

namespace ga3c {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// n / d for 0 <= n < 2^31 by multiply-high and shift (d >= 1 fixed on the host).
struct FastDiv {
    uint32_t d, mul, shift;
    FastDiv() : d(1), mul(1), shift(0) {}
    explicit FastDiv(uint32_t dd) : d(dd) {
        shift = 0;
        while ((1ull << shift) < dd) ++shift;
        mul = (uint32_t)(((1ull << 32) * ((1ull << shift) - dd)) / dd + 1);
    }
    __device__ __forceinline__ uint32_t div(uint32_t n) const {
        return (__umulhi(n, mul) + n) >> shift;
    }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t &q, uint32_t &r) const {
        q = div(n);
        r = n - q * d;
    }
};

// Round to bfloat16 (nearest even) and back: the reduced-precision variant of
// the network feeds every contraction operands that have gone through this.
__device__ __forceinline__ float bf16_rne(float f) { return (float)(__bf16)f; }
__device__ __forceinline__ float4 bf16_rne(float4 v) {
    return make_float4(bf16_rne(v.x), bf16_rne(v.y), bf16_rne(v.z), bf16_rne(v.w));
}

constexpr int GEMM_BK = 32;

// A_ROWS / B_ROWS pick how the 256-odd threads walk an operand tile when they
// fetch it: false = consecutive lanes along k (operand contiguous in k),
// true = consecutive lanes along rows (operand contiguous or strided in rows).
template <int TM, int TN, int WM, int WN, bool A_ROWS, bool B_ROWS, class P>
__global__ __launch_bounds__(WM *WN * 64) void gemm_mfma_kernel(const P p) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN, BK = GEMM_BK, NT = WM * WN * 64;
    constexpr int QK = BK / 4;
    __shared__ float4 As[QK][BM + 1];
    __shared__ float4 Bs[QK][BN + 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int wm = wave / WN, wn = wave % WN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int z = blockIdx.z;
    int kbeg, kend;
    p.krange(z, kbeg, kend);

    floatx4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // The next k-tile is fetched into registers while the current one, already
    // in LDS, is multiplied.
    constexpr int AI = (BM * QK + NT - 1) / NT, BI = (BN * QK + NT - 1) / NT;
    float4 ra[AI], rb[BI];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int it = 0; it < AI; ++it) {
            const int e = tid + it * NT;
            int row, q;
            if (A_ROWS) { row = e % BM; q = e / BM; } else { q = e % QK; row = e / QK; }
            ra[it] = (BM * QK % NT == 0 || e < BM * QK) ? p.loadA(m0 + row, k0 + 4 * q, kend, z)
                                                        : make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.rb) ra[it] = bf16_rne(ra[it]);
        }
#pragma unroll
        for (int it = 0; it < BI; ++it) {
            const int e = tid + it * NT;
            int row, q;
            if (B_ROWS) { row = e % BN; q = e / BN; } else { q = e % QK; row = e / QK; }
            rb[it] = (BN * QK % NT == 0 || e < BN * QK) ? p.loadB(n0 + row, k0 + 4 * q, kend, z)
                                                        : make_float4(0.f, 0.f, 0.f, 0.f);
            if (p.rb) rb[it] = bf16_rne(rb[it]);
        }
    };
    if (kbeg < kend) fetch(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < AI; ++it) {
            const int e = tid + it * NT;
            int row, q;
            if (A_ROWS) { row = e % BM; q = e / BM; } else { q = e % QK; row = e / QK; }
            if (BM * QK % NT == 0 || e < BM * QK) As[q][row] = ra[it];
        }
#pragma unroll
        for (int it = 0; it < BI; ++it) {
            const int e = tid + it * NT;
            int row, q;
            if (B_ROWS) { row = e % BN; q = e / BN; } else { q = e % QK; row = e / QK; }
            if (BN * QK % NT == 0 || e < BN * QK) Bs[q][row] = rb[it];
        }
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
        for (int kb = 0; kb < QK / 4; ++kb) {
            float4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = As[4 * kb + g][(wm * TM + i) * 16 + l16];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bs[4 * kb + g][(wn * TN + j) * 16 + l16];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i].x, b[j].x, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i].y, b[j].y, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i].z, b[j].z, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i].w, b[j].w, acc[i][j], 0, 0, 0);
                }
        }
    }

    // Accumulator register r of lane (l16, g) holds D[4*g + r][l16] of its tile.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + (wn * TN + j) * 16 + l16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + (wm * TM + i) * 16 + 4 * g + r;
                if (m < p.M && n < p.N) p.store(m, n, acc[i][j][r], z);
            }
        }
}

template <int TM, int TN, int WM, int WN, bool A_ROWS, bool B_ROWS, class P>
inline hipError_t launch_gemm(const P &p, int nz, hipStream_t s) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN;
    if (p.M <= 0 || p.N <= 0) return hipSuccess;
    dim3 grid((p.N + BN - 1) / BN, (p.M + BM - 1) / BM, nz);
    ga3c::launch((gemm_mfma_kernel<TM, TN, WM, WN, A_ROWS, B_ROWS, P>), grid, dim3(WM * WN * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace ga3c
