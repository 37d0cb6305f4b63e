// Dense products for the fully connected layer (forward, input gradient,
// weight gradient): the problem description and the placement of the work.
// The kernel is in dense_gemm_bf16x6.hpp.
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

// Alignment rules of the 16-byte fetches.
inline bool dense_operand_ok(const float *base, long ld, int contiguous_extent) {
    return (((uintptr_t)base) & 15) == 0 && ld % 4 == 0 && contiguous_extent % 4 == 0 && contiguous_extent >= 4;
}

}  // namespace ga3c
