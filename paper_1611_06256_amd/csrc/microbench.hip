// Micro-benchmarks of the chip properties the kernel designs of this library rest on (gfx950): the rate of the
// bf16 MFMA, whether vector-ALU work, LDS traffic and MFMAs of different wavefronts of a SIMD overlap, LDS read and
// write rates for the address patterns of the convolution and GEMM kernels, how fast operand tiles stream from L2 to
// the compute units, and what a 16-byte global load costs its wavefront to issue for several lane-to-address maps.
// One section runs a kernel of the library itself (the conv2 input gradient, with the clock stamps its header offers
// to this program) and shows what counters average away: when the blocks of a launch start and end, what a block's
// prologue costs with gathered and with ready-made filter fragments, and the core clock inside the kernel.
// A standalone program (no part of the library): built by paper_1611_06256_amd/build.py (build_microbench) and run as
//   paper_1611_06256_amd/microbench [mfma_rate|overlap|lds_read|lds_write|l2_stream|load_issue|block_lives ...]   (default: all)
// Every kernel indexes inside its own buffers for the fixed launch shapes used below; nothing is read from files.
#include <hip/hip_runtime.h>

#define GA3C_BLOCK_STAMPS
#include "conv_frame.hpp"
#include "conv_dgrad_bf16x6.hpp"

#include <cstdint>
#include <cstdio>
#include <algorithm>
#include <cstring>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace mfma_rate {
// cycles per v_mfma_f32_16x16x32_bf16 for one or more wavefronts per SIMD and different dependency distances
template <int NACC>
__global__ __launch_bounds__(1024) void k(float *out, int iters, long long *cyc) {
    floatx4 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)(e * 3 + 1); }
    const long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < NACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    const long long t1 = clock64();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.f) out[threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) *cyc = t1 - t0;
}
template <int NACC> int run(int threads) {
    float *out; long long *cyc, h; CK(hipMalloc(&out, 4096)); CK(hipMalloc(&cyc, 8));
    const int iters = 2000;
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(k<NACC>, dim3(256), dim3(threads), 0, 0, out, iters, cyc);
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL(k<NACC>, dim3(256), dim3(threads), 0, 0, out, iters, cyc);
    CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    CK(hipMemcpy(&h, cyc, 8, hipMemcpyDeviceToHost));
    const double n = (double)iters * 4 * NACC;          // MFMAs per wave
    const double waves = threads / 64.0;
    printf("NACC %2d, %2.0f waves/CU: %.1f clock64 ticks per MFMA per wave, %.3f ms, %.0f TFLOP/s chip\n", NACC, waves, h / n, ms,
           n * waves * 256 * 16384.0 / (ms * 1e-3) / 1e12);
    return 0;
}
int run_all() {
    for (int threads : {256, 512, 1024}) {
        if (run<1>(threads) || run<2>(threads) || run<4>(threads) || run<8>(threads) || run<16>(threads)) return 1;
    }
    return 0;
}
}  // namespace mfma_rate

namespace overlap {
// Do the vector ALU work of one wavefront and the MFMAs of another overlap on a SIMD?
// block of 512 threads: waves 0-3 (one per SIMD) role A, waves 4-7 role B.  mode bits: 1 = A runs MFMAs, 2 = B runs VALU,
// 4 = B runs LDS writes, 8 = B runs LDS reads, 16 = B runs MFMAs too
__global__ __launch_bounds__(512) void k(float *out, int iters, int mode) {
    __shared__ u32x4 lds[2048];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    floatx4 acc[8];
    for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x + e); b[e] = (__bf16)(float)(e * 3 + 1); }
    float v[16];
    for (int e = 0; e < 16; ++e) v[e] = threadIdx.x * 0.001f + e;
    u32x4 w = u32x4{(unsigned)lane, 1u, 2u, 3u};
    if (wave < 4) {
        if (mode & 1)
            for (int it = 0; it < iters; ++it)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    } else {
        if (mode & 2)
            for (int it = 0; it < iters; ++it)
#pragma unroll
                for (int r = 0; r < 8; ++r)
#pragma unroll
                    for (int e = 0; e < 16; ++e) v[e] = v[e] * 1.0001f + 0.5f;          // 128 VALU per iteration
        if (mode & 4)
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int r = 0; r < 8; ++r) { lds[(wave - 4) * 512 + r * 64 + lane] = w; w[0] += 1; }
                asm volatile("" ::: "memory");
            }
        if (mode & 8)
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int r = 0; r < 8; ++r) { const u32x4 q = lds[(wave - 4) * 512 + r * 64 + lane]; w[1] ^= q[0] + q[3]; }
                asm volatile("" ::: "memory");
            }
        if (mode & 16)
            for (int it = 0; it < iters; ++it)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = w[0] + w[1];
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3];
    for (int e = 0; e < 16; ++e) s += v[e];
    if (s == 12345.f) out[threadIdx.x] = s;
}
int run(const char *name, int mode) {
    float *out; CK(hipMalloc(&out, 4096));
    const int iters = 2000;
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(k, dim3(256), dim3(512), 0, 0, out, iters, mode);
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL(k, dim3(256), dim3(512), 0, 0, out, iters, mode);
    CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    printf("%-52s %8.1f us\n", name, ms * 1e3);
    return 0;
}
int run_all() {
    if (run("A: 32 MFMA/iter alone", 1)) return 1;
    if (run("B: 128 VALU/iter alone", 2)) return 1;
    if (run("A MFMA + B VALU", 3)) return 1;
    if (run("B: 8 ds_write_b128/iter alone", 4)) return 1;
    if (run("A MFMA + B LDS writes", 5)) return 1;
    if (run("B: 8 ds_read_b128/iter alone", 8)) return 1;
    if (run("A MFMA + B LDS reads", 9)) return 1;
    if (run("A MFMA + B MFMA (two waves per SIMD)", 17)) return 1;
    if (run("A MFMA + B VALU + LDS writes + reads", 15)) return 1;
    return 0;
}
}  // namespace overlap

namespace lds_read {
// LDS read throughput for the address patterns of the convolution kernels.
constexpr int LDS_BYTES = 64 * 1024;
// mode 0: b64 contiguous; 1: b128 contiguous; 2: conv1 pattern 2 x b64; 3: conv2 pattern (4 dwords as 2 x read2_b32)
// 4: b32 contiguous; 5: conv1 pattern, one b64 only; 6: conv1 pattern with row pitch padded (g*176 B)
template <int MODE>
__global__ __launch_bounds__(1024) void lds_kernel(unsigned *out, int iters, int dppdummy) {
    __shared__ __attribute__((aligned(16))) unsigned char sm[LDS_BYTES];
    for (int i = threadIdx.x; i < LDS_BYTES / 4; i += 1024) ((unsigned *)sm)[i] = i * 2654435761u;
    __syncthreads();
    const int lane = threadIdx.x & 63, l16 = lane & 15, g = lane >> 4, wave = (threadIdx.x >> 6) & 3;
    unsigned acc = 0;
    int base;
    if (MODE == 0) base = lane * 8;
    else if (MODE == 1) base = lane * 16;
    else if (MODE == 2 || MODE == 5) { int p = wave * 16 + l16; base = ((p / 20) * 4 * 84 + (p % 20) * 4 + g * 84) * 2; }
    else if (MODE == 6) { int p = wave * 16 + l16; base = ((p / 20) * 4 * 88 + (p % 20) * 4 + g * 88) * 2; }
    else if (MODE == 3) { int p = wave * 16 + l16; if (p >= 81) p = 0; base = ((g / 2) * 400 + ((p / 9) * 2 + 2 * (g % 2)) * 20 + (p % 9) * 2) * 2; }
    else base = lane * 4;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
        const int off = u * 1024 * 4;      // stays inside the array with every pattern
        const unsigned char *q = sm + base + off;
        if (MODE == 0 || MODE == 5) { uint2 v = *(const uint2 *)q; acc ^= v.x + v.y; }
        else if (MODE == 1) { u32x4 v = *(const u32x4 *)q; acc ^= v[0] + v[1] + v[2] + v[3]; }
        else if (MODE == 2 || MODE == 6) { uint2 v = *(const uint2 *)q, w = *(const uint2 *)(q + 8); acc ^= v.x + v.y + w.x + w.y; }
        else if (MODE == 3) { const unsigned *r0 = (const unsigned *)q, *r1 = (const unsigned *)(q + 40); acc ^= r0[0] + r0[1] + r1[0] + r1[1]; }
        else { acc ^= *(const unsigned *)q; }
        }
        asm volatile("" ::: "memory");
    }
    if (acc == 0x12345u + dppdummy) out[(blockIdx.x * 256 + threadIdx.x) & 65535] = acc;
}
template <int MODE> int run(const char *name, int bytes_per_lane) {
    unsigned *out; CK(hipMalloc(&out, 256 * 256 * 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int iters = 4000;
    for (int rep = 0; rep < 2; ++rep) {
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(lds_kernel<MODE>, dim3(256), dim3(1024), 0, 0, out, iters, 7);
        CK(hipEventRecord(e1, 0)); CK(hipDeviceSynchronize());
    }
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    double bytes = (double)iters * 8 * 1024 * bytes_per_lane;       // per CU (one block per CU)
    printf("%-34s %7.3f ms  %6.1f B/clk/CU (at 2.4 GHz)\n", name, ms, bytes / (ms * 1e-3 * 2.4e9));
    CK(hipFree(out)); return 0;
}
int run_all() {
    if (run<4>("b32 contiguous", 4)) return 1;
    if (run<0>("b64 contiguous", 8)) return 1;
    if (run<1>("b128 contiguous", 16)) return 1;
    if (run<5>("conv1 pattern, first b64 only", 8)) return 1;
    if (run<2>("conv1 pattern, 2 x b64", 16)) return 1;
    if (run<6>("conv1 pattern, pitch 88, 2 x b64", 16)) return 1;
    if (run<3>("conv2 pattern, 4 dwords", 16)) return 1;
    return 0;
}
}  // namespace lds_read

namespace lds_write {
// LDS write throughput for candidate stash layouts of the GEMM tiles.
constexpr int LDS_BYTES = 64 * 1024;
// MODE 0: b128 contiguous, 1: b64 contiguous, 2: b32 contiguous,
// 10+PAD: stash pattern: lane e -> row e/4, kg e%4, unit kg*(64+PAD)+row, three planes
// 40: lane -> row = e%64, kg = e/64 (consecutive lanes consecutive rows)
// 50+S: swizzled: unit = kg*64 + (row ^ (kg*S))
template <int MODE>
__global__ __launch_bounds__(256) void k(unsigned *out, int iters, unsigned seed) {
    __shared__ __attribute__((aligned(16))) unsigned char sm[LDS_BYTES];
    const int tid = threadIdx.x;
    u32x4 v; v[0] = seed + tid; v[1] = seed * 3 + tid; v[2] = seed ^ tid; v[3] = tid;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            unsigned char *q = sm + u * 13 * 1024;
            if (MODE == 0) { *(u32x4 *)(q + tid * 16) = v; *(u32x4 *)(q + 4096 + tid * 16) = v; *(u32x4 *)(q + 8192 + tid * 16) = v; }
            else if (MODE == 1) { for (int j = 0; j < 6; ++j) *(uint2 *)(q + j * 2048 + tid * 8) = uint2{v[0], v[1]}; }
            else if (MODE == 2) { for (int j = 0; j < 12; ++j) *(unsigned *)(q + j * 1024 + tid * 4) = v[0]; }
            else if (MODE >= 10 && MODE < 40) {
                constexpr int P = 64 + (MODE - 10);
                const int row = tid / 4, kg = tid % 4;
#pragma unroll
                for (int t = 0; t < 3; ++t) *(u32x4 *)(q + ((t * 4 + kg) * P + row) * 16) = v;
            } else if (MODE == 40) {
                const int row = tid % 64, kg = tid / 64;
#pragma unroll
                for (int t = 0; t < 3; ++t) *(u32x4 *)(q + ((t * 4 + kg) * 65 + row) * 16) = v;
            } else {
                constexpr int S = MODE - 50;
                const int row = tid / 4, kg = tid % 4;
#pragma unroll
                for (int t = 0; t < 3; ++t) *(u32x4 *)(q + ((t * 4 + kg) * 64 + (row ^ (kg * S))) * 16) = v;
            }
            v[0] += 1;
        }
        asm volatile("" ::: "memory");
    }
    __syncthreads();
    unsigned acc = ((unsigned *)sm)[tid];
    if (acc == 0x12345u + seed) out[(blockIdx.x * 256 + threadIdx.x) & 65535] = acc;
}
template <int MODE> int run(const char *name) {
    unsigned *out; CK(hipMalloc(&out, 256 * 256 * 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int iters = 4000;
    for (int rep = 0; rep < 2; ++rep) {
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(k<MODE>, dim3(512), dim3(256), 0, 0, out, iters, 7u);     // 2 blocks per CU
        CK(hipEventRecord(e1, 0)); CK(hipDeviceSynchronize());
    }
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    double bytes = 2.0 * iters * 4 * 256 * 48;       // per CU
    printf("%-44s %7.3f ms  %6.1f B/clk/CU (at 2.4 GHz)\n", name, ms, bytes / (ms * 1e-3 * 2.4e9));
    CK(hipFree(out)); return 0;
}
int run_all() {
    if (run<0>("write b128 contiguous")) return 1;
    if (run<1>("write b64 contiguous")) return 1;
    if (run<2>("write b32 contiguous")) return 1;
    if (run<11>("stash pattern pitch 65")) return 1;
    if (run<12>("stash pattern pitch 66")) return 1;
    if (run<14>("stash pattern pitch 68")) return 1;
    if (run<18>("stash pattern pitch 72")) return 1;
    if (run<26>("stash pattern pitch 80")) return 1;
    if (run<40>("rows across lanes, pitch 65")) return 1;
    if (run<54>("xor swizzle 4")) return 1;
    if (run<58>("xor swizzle 8")) return 1;
    if (run<66>("xor swizzle 16")) return 1;
    return 0;
}
}  // namespace lds_write

namespace l2_stream {
// How fast can the CUs pull GEMM operand tiles through L2?  No LDS, no MFMA: loads + checksum.
// Each block "owns" a tile of ROWS rows x 32 k per step, walks nsteps steps along k (row pitch ld floats).
// PAT 0: lane e -> row e/4, 32 B at k = 8*(e%4) (two 16 B loads, 16 B apart)   [the GEMM's pattern]
// PAT 1: lane e -> row e/8, 16 B at k = 4*(e%8)  (one 16 B load; a row's 128 B by 8 consecutive lanes)
template <int PAT, int UNROLL>
__global__ __launch_bounds__(256) void stream_kernel(const float *__restrict__ X, long ld, int rows_per_block, int nsteps, int share, float *out) {
    // blocks b and b ^ 1 read the same rows if share (second reader hits L2)
    const int tile = (blockIdx.x / (8 * share)) * 8 + blockIdx.x % 8;      // `share` blocks of one XCD, adjacent ids, read the same rows
    const float *base = X + (long)tile * rows_per_block * ld;
    const int tid = threadIdx.x;
    float acc = 0.f;
    const int items = rows_per_block * 4;          // 32-byte items per step
    for (int s0 = 0; s0 < nsteps; s0 += UNROLL) {
        float4 v[UNROLL][4];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int k0 = (s0 + u) * 32;
#pragma unroll
            for (int it = 0; it < 2; ++it) {        // 512 items per step: 128 rows
                const int e = (tid + it * 256) % items;
                if (PAT == 0) {
                    const float *p = base + (long)(e / 4) * ld + k0 + 8 * (e % 4);
                    v[u][2 * it] = *(const float4 *)p; v[u][2 * it + 1] = *(const float4 *)(p + 4);
                } else {
                    const int e0 = (tid + it * 256) * 2;     // 16-byte pieces
                    const float *p0 = base + (long)((e0 / 8) % rows_per_block) * ld + k0 + 4 * (e0 % 8);
                    v[u][2 * it] = *(const float4 *)p0; v[u][2 * it + 1] = *(const float4 *)(p0 + 4);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc += v[u][j].x + v[u][j].y + v[u][j].z + v[u][j].w;
    }
    if (acc == 12345.f) out[blockIdx.x * 256 + tid] = acc;
}
template <int PAT, int UNROLL>
int run(const float *X, float *out, int blocks, int share, const char *name) {
    const long ld = 2592; const int rows = 128, nsteps = 80;
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    for (int i = 0; i < 2; ++i) hipLaunchKernelGGL((stream_kernel<PAT, UNROLL>), dim3(blocks), dim3(256), 0, 0, X, ld, rows, nsteps, share, out);
    CK(hipEventRecord(a, 0));
    for (int i = 0; i < 10; ++i) hipLaunchKernelGGL((stream_kernel<PAT, UNROLL>), dim3(blocks), dim3(256), 0, 0, X, ld, rows, nsteps, share, out);
    CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b)); ms /= 10;
    const double bytes = (double)blocks * nsteps * 512 * 32;
    printf("%-28s blocks %5d share %d unroll %d: %7.1f us  %6.2f TB/s to the CUs\n", name, blocks, share, UNROLL, ms * 1e3, bytes / (ms * 1e-3) / 1e12);
    return 0;
}
int run_all() {
    float *X, *out; const size_t rows = 2048 * 128;      // enough for 2048 distinct tiles
    CK(hipMalloc(&X, rows * 2592 * 4)); CK(hipMemset(X, 0, rows * 2592 * 4)); CK(hipMalloc(&out, 4096 * 256 * 4));
    for (int blocks : {512, 2048}) {
        for (int share : {1, 2, 4, 16}) {
            if (run<0, 1>(X, out, blocks, share, "gemm pattern")) return 1;
            if (run<0, 2>(X, out, blocks, share, "gemm pattern")) return 1;
            if (run<0, 4>(X, out, blocks, share, "gemm pattern")) return 1;
            if (run<1, 2>(X, out, blocks, share, "row-contiguous pattern")) return 1;
            if (run<1, 4>(X, out, blocks, share, "row-contiguous pattern")) return 1;
        }
    }
    return 0;
}
}  // namespace l2_stream

namespace load_issue {
// Issue cost of a 16-byte global load per wavefront for several lane->address patterns (L2-resident data)
// PAT 0: lane -> row lane/4, bytes 32*(lane%4)      (16 rows, 4 pieces of 16 B, 32 B apart)      [current fetch, h = 0]
// PAT 1: lane -> row lane%16, bytes 16*(lane/16)    (A fragment pattern)
// PAT 2: lane -> row lane/8, bytes 16*(lane%8)      (8 rows x 128 B contiguous)
// PAT 3: lane -> row lane/16, bytes 16*(lane%16)    (4 rows x 256 B)
// PAT 4: contiguous 1 KB
template <int PAT>
__global__ __launch_bounds__(256) void k(const float *X, long ld, int iters, float *out, long long *cyc) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int row, off;
    if (PAT == 0) { row = lane / 4; off = 8 * (lane % 4); }
    else if (PAT == 1) { row = lane % 16; off = 4 * (lane / 16); }
    else if (PAT == 2) { row = lane / 8; off = 4 * (lane % 8); }
    else if (PAT == 3) { row = lane / 16; off = 4 * (lane % 16); }
    else { row = 0; off = 4 * lane; }
    const float *p = X + (long)(blockIdx.x * 64 + wave * 16 + row) * ld + off;
    float acc = 0.f;
    long long tot = 0;
    for (int it = 0; it < iters; ++it) {
        float4 v[8];
        const long long t0 = clock64();
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = *(const float4 *)(p + ((it * 8 + j) % 64) * 32);
        __builtin_amdgcn_sched_barrier(0);
        const long long t1 = clock64();
        __builtin_amdgcn_sched_barrier(0);
        tot += t1 - t0;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += v[j].x + v[j].w;
    }
    if (acc == 12345.f) out[threadIdx.x] = acc;
    if (blockIdx.x == 3 && threadIdx.x == 0) *cyc = tot;
}
template <int PAT> int run(const float *X, const char *name, int blocks) {
    float *out; long long *cyc, h; CK(hipMalloc(&out, 4096)); CK(hipMalloc(&cyc, 8));
    const int iters = 200;
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(k<PAT>, dim3(blocks), dim3(256), 0, 0, X, 2592L, iters, out, cyc);
    CK(hipEventRecord(a, 0));
    hipLaunchKernelGGL(k<PAT>, dim3(blocks), dim3(256), 0, 0, X, 2592L, iters, out, cyc);
    CK(hipEventRecord(b, 0)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b)); CK(hipMemcpy(&h, cyc, 8, hipMemcpyDeviceToHost));
    printf("%-44s blocks %4d: %6.1f cycles to issue one load, kernel %7.1f us, %5.2f TB/s\n", name, blocks, (double)h / (iters * 8), ms * 1e3,
           (double)blocks * 4 * iters * 8 * 1024 / (ms * 1e-3) / 1e12);
    return 0;
}
int run_all() {
    float *X; CK(hipMalloc(&X, (size_t)256 * 64 * 2592 * 4 + 65536)); CK(hipMemset(X, 0, (size_t)256 * 64 * 2592 * 4 + 65536));
    for (int blocks : {16, 256}) {
        if (run<0>(X, "16 rows, 16 B pieces 32 B apart", blocks)) return 1;
        if (run<1>(X, "16 rows x 4 pieces of 16 B (fragment order)", blocks)) return 1;
        if (run<2>(X, "8 rows x 128 B", blocks)) return 1;
        if (run<3>(X, "4 rows x 256 B", blocks)) return 1;
        if (run<4>(X, "1 KB contiguous", blocks)) return 1;
    }
    return 0;
}
}  // namespace load_issue

namespace block_lives {
typedef ga3c::ConvSpec<float, 16, 20, 20, 32, 4, 2> Conv2;      // conv2 of the small net (Sec. 3.2)
__global__ void fill(float *p, size_t n, unsigned seed) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        unsigned h = (unsigned)i * 2654435761u + seed;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        p[i] = (float)((int)(h % 2001u) - 1000) * 1e-3f;          // [-1, 1]: about half of the mask entries positive
    }
}
static double quantile(std::vector<double> v, double q) {
    std::sort(v.begin(), v.end());
    return v[(size_t)(q * (v.size() - 1))];
}
int run_all() {
    const int B = 2560, NBLK = 512;
    const size_t ndy = (size_t)B * Conv2::OC * Conv2::NPIX, nx = (size_t)B * Conv2::CHW, nw = (size_t)Conv2::OC * Conv2::K;
    float *dy, *w, *xin, *dx;
    ga3c::u32x4 *frag;
    CK(hipMalloc(&dy, ndy * 4)); CK(hipMalloc(&w, nw * 4)); CK(hipMalloc(&xin, nx * 4)); CK(hipMalloc(&dx, nx * 4));
    CK(hipMalloc(&frag, sizeof(ga3c::u32x4) * ga3c::ConvDgradBf16Geom<Conv2>::FRAG_VECS));
    hipLaunchKernelGGL(fill, dim3(1024), dim3(256), 0, 0, dy, ndy, 1u);
    hipLaunchKernelGGL(fill, dim3(64), dim3(256), 0, 0, w, nw, 2u);
    hipLaunchKernelGGL(fill, dim3(1024), dim3(256), 0, 0, xin, nx, 3u);
    CK(ga3c::launch_conv_dgrad_filter_fragments<Conv2>(w, frag, 0));
    CK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    for (int variant = 0; variant < 2; ++variant) {
        const ga3c::u32x4 *wf = variant == 0 ? nullptr : frag;
        float ms = 0.f;
        for (int rep = 0; rep < 4; ++rep) {          // the last launch is the one reported
            CK(hipEventRecord(e0, 0));
            CK(ga3c::launch_conv_dgrad_bf16x6<Conv2>(dy, w, xin, dx, B, 0, NBLK, 0, wf));
            CK(hipEventRecord(e1, 0));
            CK(hipEventSynchronize(e1));
            CK(hipEventElapsedTime(&ms, e0, e1));
        }
        std::vector<long long> st(1024 * 6);
        CK(hipMemcpyFromSymbol(st.data(), HIP_SYMBOL(ga3c::conv_dgrad_block_stamps), sizeof(long long) * st.size()));
        long long t0 = st[0], t1 = 0;
        for (int i = 0; i < NBLK; ++i) { t0 = std::min(t0, st[6 * i]); t1 = std::max(t1, st[6 * i + 4]); }
        std::vector<double> start, pro, life[2];
        double ghz = 0.0;
        for (int i = 0; i < NBLK; ++i) {
            start.push_back((st[6 * i] - t0) * 0.01);                     // wall clock: 10 ns per tick
            pro.push_back((st[6 * i + 2] - st[6 * i]) * 0.01);
            life[i < NBLK / 2 ? 0 : 1].push_back((st[6 * i + 4] - st[6 * i]) * 0.01);
            ghz += (double)(st[6 * i + 5] - st[6 * i + 1]) / ((st[6 * i + 4] - st[6 * i]) * 10.0) / NBLK;
        }
        printf("%-34s %d frames, %d blocks (two per CU), five frames each: first start to last end %.1f us (event pair %.1f us)\n",
               variant == 0 ? "filters gathered by every block:" : "ready-made filter fragments:", B, NBLK, (t1 - t0) * 0.01, ms * 1e3);
        printf("    block starts, us after the first: median %.2f, last %.2f; prologue (entry to first frame): median %.2f us, longest %.2f us\n",
               quantile(start, 0.5), quantile(start, 1.0), quantile(pro, 0.5), quantile(pro, 1.0));
        printf("    block lives, us (min / median / max): blocks 0..255 %.1f / %.1f / %.1f, blocks 256..511 %.1f / %.1f / %.1f\n",
               quantile(life[0], 0.0), quantile(life[0], 0.5), quantile(life[0], 1.0), quantile(life[1], 0.0), quantile(life[1], 0.5), quantile(life[1], 1.0));
        printf("    core clock over the blocks' lives (clock64 ticks per wall-clock ns): %.2f GHz\n", ghz);
    }
    return 0;
}
}  // namespace block_lives

int main(int argc, char **argv) {
    struct Section { const char *name; int (*fn)(); const char *what; };
    const Section sections[] = {
        {"mfma_rate", mfma_rate::run_all, "v_mfma_f32_16x16x32_bf16: clock ticks per MFMA and wavefront, chip rate, by independent accumulators and wavefronts per CU"},
        {"overlap", overlap::run_all, "wavefronts 0-3 of a block (one per SIMD) run MFMAs, wavefronts 4-7 run vector ALU / LDS work: alone and together"},
        {"lds_read", lds_read::run_all, "LDS read rate per compute unit for contiguous accesses and for the operand patterns of the convolution kernels"},
        {"lds_write", lds_write::run_all, "LDS write rate per compute unit for contiguous accesses and for tile layouts of the GEMM staging"},
        {"l2_stream", l2_stream::run_all, "operand tiles from L2 / HBM to the compute units without LDS or MFMA work (share = blocks of an XCD reading the same rows)"},
        {"load_issue", load_issue::run_all, "cycles a wavefront needs to issue one 16-byte global load, by lane-to-address map (L2-resident data)"},
        {"block_lives", block_lives::run_all, "the library's conv2 input-gradient kernel at 2560 frames: when its blocks start and end, their prologues, the core clock"},
    };
    for (const Section &s : sections) {
        bool want = argc < 2;
        for (int i = 1; i < argc; ++i) want = want || !strcmp(argv[i], s.name);
        if (!want) continue;
        printf("== %s: %s\n", s.name, s.what);
        fflush(stdout);
        if (s.fn()) return 1;
        CK(hipDeviceSynchronize());
    }
    return 0;
}
