// Dense fp32 products for the fully connected layer (forward, input gradient,
// weight gradient) on v_mfma_f32_16x16x4_f32.
//
//   D[m][n] = sum_{k in chunk z} A(m,k) * B(n,k)
//
// Each operand is either "k-major" (stored [row][k], k contiguous) or
// "row-major" (stored [k][row], rows contiguous); both are fetched with
// 16-byte loads that are clamped to the matrix and zeroed outside, so the
// fetch has no divergent branches.  Host code checks the alignment rules
// (leading dimensions and the contiguous extent multiples of 4, 16-byte bases).
//
// Work placement.  The chip has 8 accelerator dies (XCDs) with a private L2
// each, and consecutive workgroup ids go to consecutive XCDs.  A product whose
// operands exceed one L2 would pull every tile across the fabric many times.
// The grid is therefore 1-D and block id b works for XCD b % 8 on a slice of
// the problem chosen so that the slices of different XCDs are disjoint in one
// dimension (k-chunks, or column tiles): each L2 then holds only its slice.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_mfma.hpp"

namespace ga3c {

enum { DG_PARTIAL = 0, DG_BIAS_RELU = 1, DG_MASK = 2 };
enum { DG_SPLIT_Z = 0, DG_SPLIT_N = 1 };

struct DenseGemmArgs {
    int M, N, K;
    int kchunk, nz;          // k is cut into nz chunks of kchunk (a multiple of 32)
    int ntm, ntn;            // tiles along m and n
    int split;               // DG_SPLIT_Z: chunk z belongs to XCD z % 8; DG_SPLIT_N: column tile tn to XCD tn % 8
    int per_xcd;             // blocks per XCD; grid = 8 * per_xcd
    const float *A, *B;
    long lda, ldb;
    float *C;                // DG_PARTIAL: [nz][M][N]; otherwise [M][ldc]
    long ldc;
    const float *aux;        // bias[n] or mask[m*ldc + n]
    int rb;                  // round both operands to bfloat16 on the way to LDS
};

constexpr int DG_XCDS = 8;

template <int TM, int TN, int WM, int WN, bool A_ROWMAJOR, bool B_ROWMAJOR, int EPI>
__global__ __launch_bounds__(WM *WN * 64, 2) void dense_gemm_kernel(const DenseGemmArgs p) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN, BK = 32, NT = WM * WN * 64;
    constexpr int QK = BK / 4;
    constexpr int A_FLOATS = A_ROWMAJOR ? BK * (BM + 4) : QK * (BM + 1) * 4;
    constexpr int B_FLOATS = B_ROWMAJOR ? BK * (BN + 4) : QK * (BN + 1) * 4;
    __shared__ __attribute__((aligned(16))) float As[A_FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[B_FLOATS];
    constexpr int AI = BM * QK / NT, BI = BN * QK / NT;       // float4 per thread per k-tile
    static_assert(BM * QK % NT == 0 && BN * QK % NT == 0, "tile must divide evenly over the threads");

    // which (tm, tn, z) is mine
    const int xcd = blockIdx.x % DG_XCDS, local = blockIdx.x / DG_XCDS;
    int tm, tn, z;
    if (p.split == DG_SPLIT_Z) {
        const int tiles = p.ntm * p.ntn;
        const int zi = local / tiles, t = local % tiles;
        z = zi * DG_XCDS + xcd;
        tm = t / p.ntn; tn = t % p.ntn;
        if (z >= p.nz) return;
    } else {
        const int per_col = p.ntm * p.nz;
        const int ci = local / per_col, t = local % per_col;
        tn = ci * DG_XCDS + xcd;
        tm = t % p.ntm; z = t / p.ntm;
        if (tn >= p.ntn) return;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int kbeg = z * p.kchunk, kend = min(p.K, kbeg + p.kchunk);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, g = lane >> 4;
    const int wm = wave / WN, wn = wave % WN;

    floatx4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Fetch one operand tile into registers.  k-major: thread -> (row, k-quad),
    // 8 consecutive lanes read 128 contiguous bytes of one row.  row-major:
    // thread -> (k, row-quad), BM/4 consecutive lanes read one k line.
    auto fetchA = [&](int k0, float4 (&r)[AI]) {
#pragma unroll
        for (int it = 0; it < AI; ++it) {
            const int e = tid + it * NT;
            if (!A_ROWMAJOR) {
                const int row = e / QK, q = e % QK;
                const int m = m0 + row, k = k0 + 4 * q;
                const float4 v = *(const float4 *)(p.A + (long)min(m, p.M - 1) * p.lda + min(k, p.K - 4));
                r[it] = (m < p.M && k < kend) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                const int k = e / (BM / 4), mq = e % (BM / 4);
                const int m = m0 + 4 * mq, kk = k0 + k;
                const float4 v = *(const float4 *)(p.A + (long)min(kk, p.K - 1) * p.lda + min(m, p.M - 4));
                r[it] = (m < p.M && kk < kend) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    auto fetchB = [&](int k0, float4 (&r)[BI]) {
#pragma unroll
        for (int it = 0; it < BI; ++it) {
            const int e = tid + it * NT;
            if (!B_ROWMAJOR) {
                const int row = e / QK, q = e % QK;
                const int n = n0 + row, k = k0 + 4 * q;
                const float4 v = *(const float4 *)(p.B + (long)min(n, p.N - 1) * p.ldb + min(k, p.K - 4));
                r[it] = (n < p.N && k < kend) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                const int k = e / (BN / 4), nq = e % (BN / 4);
                const int n = n0 + 4 * nq, kk = k0 + k;
                const float4 v = *(const float4 *)(p.B + (long)min(kk, p.K - 1) * p.ldb + min(n, p.N - 4));
                r[it] = (n < p.N && kk < kend) ? v : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    auto stashA = [&](const float4 (&r)[AI]) {
#pragma unroll
        for (int it = 0; it < AI; ++it) {
            const int e = tid + it * NT;
            const float4 v = p.rb ? bf16_rne(r[it]) : r[it];
            if (!A_ROWMAJOR) *(float4 *)(As + ((e % QK) * (BM + 1) + e / QK) * 4) = v;
            else *(float4 *)(As + (e / (BM / 4)) * (BM + 4) + 4 * (e % (BM / 4))) = v;
        }
    };
    auto stashB = [&](const float4 (&r)[BI]) {
#pragma unroll
        for (int it = 0; it < BI; ++it) {
            const int e = tid + it * NT;
            const float4 v = p.rb ? bf16_rne(r[it]) : r[it];
            if (!B_ROWMAJOR) *(float4 *)(Bs + ((e % QK) * (BN + 1) + e / QK) * 4) = v;
            else *(float4 *)(Bs + (e / (BN / 4)) * (BN + 4) + 4 * (e % (BN / 4))) = v;
        }
    };

    float4 ra[AI], rb[BI];
    if (kbeg < kend) { fetchA(kbeg, ra); fetchB(kbeg, rb); }
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
        stashA(ra); stashB(rb);
        __syncthreads();
        if (k0 + BK < kend) { fetchA(k0 + BK, ra); fetchB(k0 + BK, rb); }
        // MFMA number t of group kb sums over k = 16*kb + 4*g + t, g = 0..3
#pragma unroll
        for (int kb = 0; kb < QK / 4; ++kb) {
            float a[TM][4], b[TN][4];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = (wm * TM + i) * 16 + l16;
                if (!A_ROWMAJOR) {
                    const float4 v = *(const float4 *)(As + ((4 * kb + g) * (BM + 1) + row) * 4);
                    a[i][0] = v.x; a[i][1] = v.y; a[i][2] = v.z; a[i][3] = v.w;
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) a[i][t] = As[(16 * kb + 4 * g + t) * (BM + 4) + row];
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = (wn * TN + j) * 16 + l16;
                if (!B_ROWMAJOR) {
                    const float4 v = *(const float4 *)(Bs + ((4 * kb + g) * (BN + 1) + row) * 4);
                    b[j][0] = v.x; b[j][1] = v.y; b[j][2] = v.z; b[j][3] = v.w;
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) b[j][t] = Bs[(16 * kb + 4 * g + t) * (BN + 4) + row];
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i][t], b[j][t], acc[i][j], 0, 0, 0);
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
                if (m < p.M && n < p.N) {
                    const float v = acc[i][j][r];
                    if (EPI == DG_PARTIAL) {
                        p.C[((size_t)z * p.M + m) * p.N + n] = v;
                    } else if (EPI == DG_BIAS_RELU) {
                        const float t = v + p.aux[n];
                        p.C[m * p.ldc + n] = t > 0.f ? t : 0.f;
                    } else {
                        p.C[m * p.ldc + n] = p.aux[m * p.ldc + n] > 0.f ? v : 0.f;
                    }
                }
            }
        }
}

// Fills the placement fields and launches.  kchunk/nz must be set already.
template <int TM, int TN, int WM, int WN, bool A_ROWMAJOR, bool B_ROWMAJOR, int EPI>
inline hipError_t launch_dense_gemm(DenseGemmArgs p, int split, hipStream_t s) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN;
    if (p.M <= 0 || p.N <= 0) return hipSuccess;
    p.ntm = (p.M + BM - 1) / BM;
    p.ntn = (p.N + BN - 1) / BN;
    p.split = split;
    if (split == DG_SPLIT_Z) p.per_xcd = ((p.nz + DG_XCDS - 1) / DG_XCDS) * p.ntm * p.ntn;
    else p.per_xcd = ((p.ntn + DG_XCDS - 1) / DG_XCDS) * p.ntm * p.nz;
    hipLaunchKernelGGL((dense_gemm_kernel<TM, TN, WM, WN, A_ROWMAJOR, B_ROWMAJOR, EPI>), dim3(DG_XCDS * p.per_xcd),
                       dim3(WM * WN * 64), 0, s, p);
    return hipGetLastError();
}

// Alignment rules of the 16-byte fetches.
inline bool dense_operand_ok(const float *base, long ld, int contiguous_extent) {
    return (((uintptr_t)base) & 15) == 0 && ld % 4 == 0 && contiguous_extent % 4 == 0 && contiguous_extent >= 4;
}

}  // namespace ga3c
