// Dense products of the fully connected layer on the bf16 matrix cores at
// fp32 accuracy.  Each fp32 operand is split into three bf16 terms
// (a = a0 + a1 + a2 exactly, 8 significant bits each) while its tile is staged
// into LDS, and a product a*b is evaluated as the six largest of the nine term
// products (a0b0, a0b1, a1b0, a0b2, a1b1, a2b0), each exact in the fp32
// accumulator; what is dropped is below 2^-23 of |a*b|, the size of fp32
// rounding itself.  Six v_mfma_f32_16x16x32_bf16 replace eight
// v_mfma_f32_16x16x4_f32 at a quarter of their cycles, and the operands take
// 96 instead of 256 bytes of LDS traffic per lane.
//
// Same interface, tiling freedom and XCD-partitioned 1-D grid as
// dense_gemm.hpp (see there).
#pragma once
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include <stdint.h>

#include "conv1_bf16x3.hpp"
#include "dense_gemm.hpp"

namespace ga3c {

// 8 floats -> three bf16x8 vectors (hi, mid, lo) with f = hi + mid + lo exactly, two values per conversion
// instruction (the same roundings as split3, 5.5 instead of 7.5 vector instructions per value)
__device__ __forceinline__ void split3x8(const float (&f)[8], u32x4 &hi, u32x4 &mid, u32x4 &lo, int rb = 0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        uint32_t h, m, l;
        split3_pair(f[2 * e], f[2 * e + 1], h, m, l);
        hi[e] = h; mid[e] = rb ? 0u : m; lo[e] = rb ? 0u : l;
    }
}

// Fetch the thread's share of a ROWS x 32 operand tile into registers: an item
// is 8 consecutive k of one row, which is what one lane feeds to an MFMA.
// k-major operand ([row][k]): two 16-byte loads; 4 consecutive lanes cover 128
// contiguous bytes of a row.  row-major operand ([k][row]): eight 4-byte loads
// with consecutive lanes on consecutive rows.  Loads are clamped into the
// matrix.  ZERO_TAIL: values at k >= kend are replaced by zeros (needed only
// in a chunk's last, partial group of 32).  Rows beyond the matrix repeat its
// last row: they only feed outputs that are never stored.
template <bool ROWMAJOR, int ROWS, int ITEMS, int NT, bool ZERO_TAIL = true, bool PTR_STEPS = false>
__device__ __forceinline__ void fetch_tile(const float *__restrict__ X, long ld, int R0, int R, int K, int k0, int kend,
                                           int tid, float (&r)[ITEMS][8]) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int e = tid + it * NT;
        if (!ROWMAJOR) {
            const int row = e / 4, kg = e % 4;
            const float *src = X + (long)min(R0 + row, R - 1) * ld;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kk = k0 + 8 * kg + 4 * h;
                const float4 v = *(const float4 *)(src + min(kk, K - 4));
                const bool ok = !ZERO_TAIL || kk < kend;
                r[it][4 * h + 0] = ok ? v.x : 0.f; r[it][4 * h + 1] = ok ? v.y : 0.f;
                r[it][4 * h + 2] = ok ? v.z : 0.f; r[it][4 * h + 3] = ok ? v.w : 0.f;
            }
        } else {
            const int kg = e / ROWS, row = e % ROWS;
            const int m = min(R0 + row, R - 1);
            if (!ZERO_TAIL && PTR_STEPS) {      // every k is inside the matrix: plain pointer steps, no 64-bit products per
                                                // load (pays when both operands are read this way, measured)
                const float *src = X + ((long)(8 * kg) * ld + m) + (long)k0 * ld;
#pragma unroll
                for (int h = 0; h < 8; ++h) r[it][h] = src[(long)h * ld];
            } else {
#pragma unroll
                for (int h = 0; h < 8; ++h) {
                    const int kk = k0 + 8 * kg + h;
                    const float v = X[(long)min(kk, K - 1) * ld + m];
                    r[it][h] = (!ZERO_TAIL || kk < kend) ? v : 0.f;
                }
            }
        }
    }
}

// Split what fetch_tile brought and store it as S[term][k-group][row].
template <bool ROWMAJOR, int ROWS, int ITEMS, int NT, bool ONE = false>
__device__ __forceinline__ void stash_tile(u32x4 (&S)[3][4][ROWS + 1], int tid, const float (&r)[ITEMS][8], int rb) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int e = tid + it * NT;
        const int row = ROWMAJOR ? e % ROWS : e / 4, kg = ROWMAJOR ? e / ROWS : e % 4;
        if (ONE) {       // only the first term exists
            u32x4 hi, mid, lo;
            split3x8(r[it], hi, mid, lo, 1);
            S[0][kg][row] = hi;
        } else {
            split3x8(r[it], S[0][kg][row], S[1][kg][row], S[2][kg][row]);      // all three terms (rb runs the ONE kernel)
        }
    }
}

// ONE: the reduced-precision variant (operands rounded to bfloat16): one term per operand, one MFMA per tile pair.
template <int TM, int TN, int WM, int WN, bool A_ROWMAJOR, bool B_ROWMAJOR, int EPI, bool ONE>
__global__ __launch_bounds__(WM *WN * 64, 2) void dense_gemm_bf16x6_kernel(const DenseGemmArgs p) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN, BK = 32, NT = WM * WN * 64;
    constexpr bool SWAP = EPI == DG_MASK;            // the input gradient: output and mask are read and written in rows
    // LDS: [term][k-group of 8][row] in 16-byte units, one spare unit per line
    __shared__ u32x4 As[3][4][BM + 1];
    __shared__ u32x4 Bs[3][4][BN + 1];
    constexpr int A_ITEMS = BM * 4 / NT, B_ITEMS = BN * 4 / NT;      // (row, k-group) items per thread
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0 && A_ITEMS >= 1 && B_ITEMS >= 1, "tile does not fit the block");

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

    float ra[A_ITEMS][8], rb[B_ITEMS][8];
    if (kbeg < kend) {
        fetch_tile<A_ROWMAJOR, BM, A_ITEMS, NT>(p.A, p.lda, m0, p.M, p.K, kbeg, kend, tid, ra);
        fetch_tile<B_ROWMAJOR, BN, B_ITEMS, NT>(p.B, p.ldb, n0, p.N, p.K, kbeg, kend, tid, rb);
    }
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        __syncthreads();
        stash_tile<A_ROWMAJOR, BM, A_ITEMS, NT, ONE>(As, tid, ra, p.rb);
        stash_tile<B_ROWMAJOR, BN, B_ITEMS, NT, ONE>(Bs, tid, rb, p.rb);
        __syncthreads();
        if (k0 + 2 * BK <= kend) {          // a whole group of 32 comes next: nothing to zero
            constexpr bool PS = A_ROWMAJOR && B_ROWMAJOR;
            fetch_tile<A_ROWMAJOR, BM, A_ITEMS, NT, false, PS>(p.A, p.lda, m0, p.M, p.K, k0 + BK, kend, tid, ra);
            fetch_tile<B_ROWMAJOR, BN, B_ITEMS, NT, false, PS>(p.B, p.ldb, n0, p.N, p.K, k0 + BK, kend, tid, rb);
        } else if (k0 + BK < kend) {
            fetch_tile<A_ROWMAJOR, BM, A_ITEMS, NT>(p.A, p.lda, m0, p.M, p.K, k0 + BK, kend, tid, ra);
            fetch_tile<B_ROWMAJOR, BN, B_ITEMS, NT>(p.B, p.ldb, n0, p.N, p.K, k0 + BK, kend, tid, rb);
        }
        Bf16x8Bits a[TM][3], b[TN][3];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < (ONE ? 1 : 3); ++t) a[i][t].u = As[t][g][(wm * TM + i) * 16 + l16];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int t = 0; t < (ONE ? 1 : 3); ++t) b[j][t].u = Bs[t][g][(wn * TN + j) * 16 + l16];
        // smallest products first.  SWAP: the instruction takes B's rows as its rows, so that a lane ends up with
        // C[m = its l16][n = 4 g .. 4 g + 3] (four consecutive columns) instead of four rows of one column
        auto mma = [&](const bf16x8 x, const bf16x8 y, floatx4 &c) {
            c = SWAP ? __builtin_amdgcn_mfma_f32_16x16x32_bf16(y, x, c, 0, 0, 0) : __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, c, 0, 0, 0);
        };
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (!ONE) {
                    mma(a[i][2].v, b[j][0].v, acc[i][j]);
                    mma(a[i][1].v, b[j][1].v, acc[i][j]);
                    mma(a[i][0].v, b[j][2].v, acc[i][j]);
                    mma(a[i][1].v, b[j][0].v, acc[i][j]);
                    mma(a[i][0].v, b[j][1].v, acc[i][j]);
                }
                mma(a[i][0].v, b[j][0].v, acc[i][j]);
            }
    }

    if (SWAP) {
        // one 16-byte store (and one 16-byte load of the mask) per tile instead of four scattered 4-byte ones, where
        // the row pitch and the pointers allow it
        const bool vec = p.N % 4 == 0 && p.ldc % 4 == 0 && (uintptr_t)p.C % 16 == 0 && (uintptr_t)p.aux % 16 == 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int m = m0 + (wm * TM + i) * 16 + l16;
                const int n = n0 + (wn * TN + j) * 16 + 4 * g;
                if (m >= p.M || n >= p.N) continue;
                float *dst = p.C + (size_t)m * p.ldc + n;
                const float *msk = p.aux + (size_t)m * p.ldc + n;
                if (vec) {
                    const float4 k4 = *(const float4 *)msk;
                    float4 v = float4{acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
                    v.x = k4.x > 0.f ? v.x : 0.f; v.y = k4.y > 0.f ? v.y : 0.f; v.z = k4.z > 0.f ? v.z : 0.f; v.w = k4.w > 0.f ? v.w : 0.f;
                    *(float4 *)dst = v;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (n + r < p.N) dst[r] = msk[r] > 0.f ? acc[i][j][r] : 0.f;
                }
            }
        return;
    }

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

template <int TM, int TN, int WM, int WN, bool A_ROWMAJOR, bool B_ROWMAJOR, int EPI>
inline hipError_t launch_dense_gemm_bf16x6(DenseGemmArgs p, int split, hipStream_t s) {
    constexpr int BM = 16 * TM * WM, BN = 16 * TN * WN;
    if (p.M <= 0 || p.N <= 0) return hipSuccess;
    p.ntm = (p.M + BM - 1) / BM;
    p.ntn = (p.N + BN - 1) / BN;
    p.split = split;
    if (split == DG_SPLIT_Z) p.per_xcd = ((p.nz + DG_XCDS - 1) / DG_XCDS) * p.ntm * p.ntn;
    else p.per_xcd = ((p.ntn + DG_XCDS - 1) / DG_XCDS) * p.ntm * p.nz;
    if (p.rb)
        ga3c::launch((dense_gemm_bf16x6_kernel<TM, TN, WM, WN, A_ROWMAJOR, B_ROWMAJOR, EPI, true>),
                           dim3(DG_XCDS * p.per_xcd), dim3(WM * WN * 64), 0, s, p);
    else
        ga3c::launch((dense_gemm_bf16x6_kernel<TM, TN, WM, WN, A_ROWMAJOR, B_ROWMAJOR, EPI, false>),
                           dim3(DG_XCDS * p.per_xcd), dim3(WM * WN * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace ga3c
