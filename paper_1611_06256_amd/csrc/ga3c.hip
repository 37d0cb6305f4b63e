// GA3C hot path on MI355X (gfx950): the C ABI declared in include/ga3c.h and
// the kernels behind it that are not matrix products (heads + softmax +
// sampling, returns + loss, reductions, RMSProp, parameter initialisation).
// The matrix products are instances of gemm_mfma.hpp / problems.hpp.
#include <hip/hip_runtime.h>

#include "launch.hpp"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/ga3c.h"
#include "problems.hpp"
#include "conv_frame.hpp"
#include "dense_gemm.hpp"
#include "conv1_bf16x3.hpp"
#include "dense_gemm_bf16x6.hpp"
#include "conv2_bf16x6.hpp"
#include "conv12_fused.hpp"
#include "conv_fwd_bf16x6.hpp"
#include "conv_dgrad_bf16x6.hpp"
#include "conv_wgrad_bf16x6.hpp"
#include "conv_wgrad_s1_bf16x6.hpp"

using namespace ga3c;

// Fixed-geometry kernels exist for the layers of the paper's networks.
typedef ConvSpec<uint8_t, 4, 84, 84, 16, 8, 4> SpecS1;    // small net, conv1
typedef ConvSpec<float, 16, 20, 20, 32, 4, 2> SpecS2;     // small net, conv2
typedef ConvSpec<uint8_t, 4, 84, 84, 32, 8, 4> SpecL1;    // large net, conv1
typedef ConvSpec<float, 32, 20, 20, 64, 4, 2> SpecL2;     // large net, conv2
typedef ConvSpec<float, 64, 9, 9, 64, 3, 1> SpecL3;       // large net, conv3
typedef ConvSpec<float, 32, 20, 20, 32, 4, 2> SpecP2;     // the paper's larger-network family (Sec. 5), stride-4 member, conv2
// 16-byte vectors of a small-net fragment buffer: the filters of conv1 / conv2 for the fused forward kernel, then
// those of conv2 for its input-gradient kernel
constexpr int CFRAG_FWD_VECS = 3 * C12_FRAG_SET, CFRAG_VECS = CFRAG_FWD_VECS + ConvDgradBf16Geom<SpecS2>::FRAG_VECS;
// parts of a larger-net fragment buffer: conv2 forward, conv2 input gradient, conv3 forward, conv3 input gradient
constexpr int LFRAG_FWD2 = 0, LFRAG_DGRAD2 = LFRAG_FWD2 + ConvFwdBf16Geom<SpecL2>::FRAG_VECS,
              LFRAG_FWD3 = LFRAG_DGRAD2 + ConvDgradBf16Geom<SpecL2>::FRAG_VECS, LFRAG_DGRAD3 = LFRAG_FWD3 + ConvFwdBf16Geom<SpecL3>::FRAG_VECS,
              LFRAG_VECS = LFRAG_DGRAD3 + conv_dgrad_s1_frag_vecs<SpecL3>();

// All four parts in one launch (w2, w3: the filter tensors of conv2 and conv3).
typedef ConvSpec<float, SpecL3::OC, SpecL3::OH + 2 * (SpecL3::KS - 1), SpecL3::OW + 2 * (SpecL3::KS - 1), SpecL3::C, SpecL3::KS, 1> SpecL3Dgrad;
constexpr int LFRAG_B0 = ConvFwdBf16Geom<SpecL2>::KB, LFRAG_B1 = LFRAG_B0 + (SpecL2::OC * SpecL2::C * 4 + 255) / 256,
              LFRAG_B2 = LFRAG_B1 + ConvFwdBf16Geom<SpecL3>::KB, LFRAG_B3 = LFRAG_B2 + ConvFwdBf16Geom<SpecL3Dgrad>::KB;
__global__ __launch_bounds__(256) void large_filter_fragments_kernel(const float *__restrict__ w2, const float *__restrict__ w3,
                                                                     u32x4 *__restrict__ lfrag) {
    const int b = blockIdx.x, t = threadIdx.x;
    if (b < LFRAG_B0) conv_fwd_filter_fragments_thread<SpecL2, false>(w2, lfrag + LFRAG_FWD2, b * 256 + t);
    else if (b < LFRAG_B1) {
        const int i = (b - LFRAG_B0) * 256 + t;
        if (i < SpecL2::OC * SpecL2::C * 4) conv_dgrad_store_fragment4<SpecL2>(lfrag + LFRAG_DGRAD2, 4 * i, ((const float4 *)w2)[i]);
    } else if (b < LFRAG_B2) conv_fwd_filter_fragments_thread<SpecL3, false>(w3, lfrag + LFRAG_FWD3, (b - LFRAG_B1) * 256 + t);
    else conv_fwd_filter_fragments_thread<SpecL3Dgrad, true>(w3, lfrag + LFRAG_DGRAD3, (b - LFRAG_B2) * 256 + t);
}

// ---------------------------------------------------------------- errors ----

static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                   \
    do {                                                                                \
        hipError_t e_ = (expr);                                                         \
        if (e_ != hipSuccess)                                                           \
            return fail(e_ == hipErrorOutOfMemory ? GA3C_ENOMEM : GA3C_EHIP, "%s: %s", \
                        #expr, hipGetErrorString(e_));                                  \
    } while (0)

extern "C" const char *ga3c_last_error(void) { return g_err; }

// ---------------------------------------------------------------- context ---

namespace {

constexpr int LOSS_THREADS = 64;    // frames per block in the returns/loss kernel

struct Work {            // activations of one call; predict and train own one each
    int cap = 0;         // frames
    float *act[GA3C_MAX_CONV] = {nullptr, nullptr, nullptr, nullptr};   // conv outputs, NCHW, post-ReLU
    float *h = nullptr;  // fc output [cap][F], post-ReLU
    float *zv = nullptr; // logits and value [cap][A+1]
    float *ws = nullptr; // split-k partial products of this call
    size_t ws_floats = 0;
    const float *fc_ws = nullptr;   // where the last forward left the fc partial sums, and how many
    int fc_nz = 1;
};

}  // namespace

namespace {
// Optional per-stage timing: the execution times of the kernels of each stage (an event pair per launch).
struct ProfStage { const char *name; long calls; double ms, flop, bytes; };
struct ProfRec { int stage; hipEvent_t a, b; };
struct Profiler {
    bool on = false;
    std::vector<ProfStage> stages;
    std::vector<ProfRec> recs;          // recorded, not yet read
    std::vector<hipEvent_t> pool;       // idle events
};
}  // namespace

struct ga3c_ctx {
    Profiler *prof;
    bool fast;                    // use the fixed-geometry kernels where they apply
    bool small_predict;           // predictions of a handful of frames go out as one launch
    int rb;                       // desc.math == 1: operands of every contraction are rounded to bfloat16
    ga3c_net_desc desc;
    int nconv, F, A, flat;
    ConvGeom geom[GA3C_MAX_CONV];
    int *koff[GA3C_MAX_CONV];
    int64_t off[2 * GA3C_MAX_CONV + 7];
    int noff;
    size_t P;
    int max_pred, max_train;
    // Two copies of the parameters.  theta2[cur] is the published snapshot that
    // predictions and the forward/backward of an update read; RMSProp writes the
    // other copy and publishes it.  ev_ready[i]: copy i has been written;
    // ev_readers[i]: the last prediction that read copy i has finished.
    float *theta2[2];
    int cur;
    hipEvent_t ev_ready[2], ev_readers[2];
    hipStream_t ready_stream[2], readers_stream[2];   // where each event was last recorded
    bool ready_set[2], readers_set[2];
    float *g, *grad;
    // small net: conv1/conv2 filters of each parameter copy as split MFMA fragments (nullptr for other nets), forward
    // kernel's first, then (at CFRAG_FWD_VECS) the input-gradient kernel's; refreshed by whoever writes the copy
    u32x4 *cfrag[2];
    bool cfrag_dgrad;             // the buffers hold the second part too (a context that can train)
    // larger net: the filters of conv2 and conv3 of each parameter copy as ready-made fragments for the forward and the
    // input-gradient kernels (LFRAG_* give the parts); rebuilt by whoever writes the copy
    u32x4 *lfrag[2];
    int *ticket;                  // predict_small_kernel's per-frame counters, zero between launches
    Work pred, train;
    // training only
    float *dact[GA3C_MAX_CONV];   // dL/d(pre-activation) of each conv output
    float *dh;                    // dL/d(pre-activation) of the fc output
    float *dzv;                   // dL/d(logits, value) [cap][A+1]
    float *R;                     // returns [cap]
    float *partials;              // one squared-norm partial per reduce block, then 3 per loss block
    int max_norm_parts;
    float *colpart;               // per-block column sums of dh [cap/HD_FRAMES + 1][F]
    float *scale;                 // clip scale of the last step (1 float)
    ga3c_train_stats *stats;      // stats of the last step
    int last_frames;
};

namespace {

// ------------------------------------------------------------ small kernels -

// Wavefront-wide sum and max in registers: butterflies inside each row of 16
// lanes with DPP (quad permutes, then the two mirror patterns), then the four
// row results are combined through scalar registers.  Every lane gets the
// result; no LDS traffic, unlike __shfl_xor.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_f32(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<0xB1>(v);      // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E>(v);      // quad_perm [2,3,0,1]
    v += dpp_f32<0x141>(v);     // row_half_mirror
    v += dpp_f32<0x140>(v);     // row_mirror
    return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    v = fmaxf(v, dpp_f32<0x141>(v));
    v = fmaxf(v, dpp_f32<0x140>(v));
    return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

// Global memory answers in roughly half a microsecond, so short kernels are
// bound by the number of dependent load rounds, not by bytes.  These helpers
// issue a batch of independent loads (indices past the end are clamped, the
// values then ignored) before any of them is used.
template <int BATCH>
__device__ __forceinline__ void copy_to_lds(float *dst, const float *__restrict__ src, int n, int tid, int nthreads) {
    for (int e0 = 0; e0 < n; e0 += BATCH * nthreads) {
        float v[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) v[j] = src[min(e0 + j * nthreads + tid, n - 1)];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const int idx = e0 + j * nthreads + tid;
            if (idx < n) dst[idx] = v[j];
        }
    }
}

// Policy and value heads (Sec. 3.2: softmax policy output, linear value
// output), then softmax and inverse-CDF sampling; optionally preceded by the
// last step of a split-k fully connected layer.  A block takes 4 frames.
//   ws != null: h[b][o] = max(0, bias[o] + sum_z ws[z][b][o]) is formed first
//               (and written to h); otherwise h is read.
//   h [B][F]; Wp [A][F], bp [A], Wv [F], bv [1].  zv [B][A+1] is written when
//   not null (training keeps it); logits / values / probs / actions are the
//   caller's optional outputs.
// Dynamic LDS: heads_lds_floats(F, A) floats: the 4 rows of h, both weight
// matrices (rows padded to a multiple of 4 plus 4, so that rows start 16-byte
// aligned in different banks), the partial dot products.  Global memory answers
// in about a microsecond, so every load a thread needs (weights, partial sums,
// biases, its uniform number) is issued before the first one is used.
__host__ __device__ inline int heads_f4(int F) { return (F + 3) / 4 * 4; }
__host__ __device__ inline int heads_lds_floats(int F, int A) { return 4 * heads_f4(F) + (A + 1) * (heads_f4(F) + 4 + 12); }

// Both weight matrices into the block's LDS in the layout heads_fwd_body reads, by threads t = 0 .. NT-1.
template <int NT>
__device__ __forceinline__ void heads_stage_weights(float *hs, const int t, int F, int A, const float *__restrict__ Wp,
                                                    const float *__restrict__ Wv, int rb) {
    const int F4 = heads_f4(F), WP = F4 + 4;
    float *wsh = hs + 4 * F4;
    for (int e = t; e < (A + 1) * (WP - F); e += NT) wsh[(e / (WP - F)) * WP + F + e % (WP - F)] = 0.f;
    const int nw = (A + 1) * F;
    for (int e0 = 0; e0 < nw; e0 += 24 * NT) {
        float wv[24];
#pragma unroll
        for (int j = 0; j < 24; ++j) {
            const int e = min(e0 + j * NT + t, nw - 1);
            wv[j] = e < A * F ? Wp[e] : Wv[e - A * F];
        }
#pragma unroll
        for (int j = 0; j < 24; ++j) {
            const int e = e0 + j * NT + t;
            if (e < nw) wsh[(e / F) * WP + e % F] = rb ? bf16_rne(wv[j]) : wv[j];
        }
    }
}

// The same in two steps for at most 24 * NT weights: the loads first, the stores whenever the caller has time.
template <int NT>
__device__ __forceinline__ void heads_load_weights(float (&wv)[24], const int t, int F, int A, const float *__restrict__ Wp,
                                                   const float *__restrict__ Wv) {
    const int nw = (A + 1) * F;
#pragma unroll
    for (int j = 0; j < 24; ++j) {
        const int e = min(j * NT + t, nw - 1);
        wv[j] = e < A * F ? Wp[e] : Wv[e - A * F];
    }
}
template <int NT>
__device__ __forceinline__ void heads_store_weights(float *hs, const float (&wv)[24], const int t, int F, int A, int rb) {
    const int F4 = heads_f4(F), WP = F4 + 4;
    float *wsh = hs + 4 * F4;
    for (int e = t; e < (A + 1) * (WP - F); e += NT) wsh[(e / (WP - F)) * WP + F + e % (WP - F)] = 0.f;
    const int nw = (A + 1) * F;
#pragma unroll
    for (int j = 0; j < 24; ++j) {
        const int e = j * NT + t;
        if (e < nw) wsh[(e / F) * WP + e % F] = rb ? bf16_rne(wv[j]) : wv[j];
    }
}

// The loads of a heads block as 16-byte vectors (a quarter of the load instructions: a wavefront spends about a
// hundred cycles issuing each one, whatever its width): the split-k partial sums of the fc layer for NF frames are
// added up in chunk order, bias and ReLU follow, the result goes to h and (rounded if rb) to hs [NF][F4]; the heads'
// weights go to wsh [A+1][WP] (the value head's row with 4-byte loads: it follows the policy biases in the parameter
// vector and is not aligned).  Needs F % 4 == 0 and 16-byte aligned pointers (heads_vec4_ok).  Every load of a round
// is issued before the first one is used.
__device__ __forceinline__ bool heads_vec4_ok(int F, const void *ws, const void *fcb, const void *h, const void *Wp) {
    return F % 4 == 0 && (((uintptr_t)ws | (uintptr_t)fcb | (uintptr_t)h | (uintptr_t)Wp) & 15) == 0;
}
template <int NT, int NF, int CH>
__device__ __forceinline__ void heads_load_vec4(float *hs, float *wsh, const int tid, const int b0, const int nf,
                                                const float *__restrict__ ws, int nz, const float *__restrict__ fcb,
                                                float *__restrict__ h, int B, int F, int F4, int WP, int A,
                                                const float *__restrict__ Wp, const float *__restrict__ Wv, int rb) {
    const int FQ = F >> 2, nwq = A * FQ;
    const size_t stride4 = (size_t)B * FQ;
    for (int q0 = 0; q0 < nwq || q0 == 0; q0 += 8 * NT) {
        float4 wv4[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) wv4[j] = ((const float4 *)Wp)[min(q0 + j * NT + tid, nwq - 1)];
        if (q0 == 0) {
            for (int k = tid; k < F; k += NT) wsh[A * WP + k] = rb ? bf16_rne(Wv[k]) : Wv[k];
            for (int it = tid; it < NF * FQ; it += NT) {
                const int fb = it / FQ, oq = it % FQ;
                const float4 bias = ((const float4 *)fcb)[oq];
                const float4 *src = (const float4 *)(ws + (size_t)(b0 + min(fb, nf - 1)) * F) + oq;
                float4 acc = float4{0.f, 0.f, 0.f, 0.f};
                for (int z = 0; z < nz; z += CH) {
                    float4 v[CH];
#pragma unroll
                    for (int i = 0; i < CH; ++i) v[i] = src[(size_t)min(z + i, nz - 1) * stride4];
#pragma unroll
                    for (int i = 0; i < CH; ++i) {
                        const bool in = z + i < nz;
                        acc.x += in ? v[i].x : 0.f; acc.y += in ? v[i].y : 0.f;
                        acc.z += in ? v[i].z : 0.f; acc.w += in ? v[i].w : 0.f;
                    }
                }
                float4 r = float4{acc.x + bias.x, acc.y + bias.y, acc.z + bias.z, acc.w + bias.w};
                r.x = r.x > 0.f ? r.x : 0.f; r.y = r.y > 0.f ? r.y : 0.f; r.z = r.z > 0.f ? r.z : 0.f; r.w = r.w > 0.f ? r.w : 0.f;
                if (fb < nf) *(float4 *)(h + (size_t)(b0 + fb) * F + 4 * oq) = r;
                *(float4 *)(hs + fb * F4 + 4 * oq) = rb ? bf16_rne(r) : r;
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int q = q0 + j * NT + tid;
            if (q < nwq) *(float4 *)(wsh + (q / FQ) * WP + 4 * (q % FQ)) = rb ? bf16_rne(wv4[j]) : wv4[j];
        }
    }
}

// The body, for a block of NT threads (all of them must call it) that works on frames b0 .. min(b0 + 4, B) - 1;
// hs is the block's LDS.  COHERENT: h was written by other blocks of the same launch, so it is read past the
// caches that are not kept coherent within a launch.  WSTAGED: heads_stage_weights has already run on hs.
template <int NT, bool COHERENT, bool WSTAGED>
__device__ __forceinline__ void heads_fwd_body(float *hs, const int tid, const int b0, const float *__restrict__ ws, int nz,
                                               const float *__restrict__ fcb, float *__restrict__ h, int B, int F, int A,
                                               const float *__restrict__ Wp, const float *__restrict__ bp,
                                               const float *__restrict__ Wv, const float *__restrict__ bv, float *zv,
                                               float *logits, float *values, float *probs, const float *uniforms,
                                               int32_t *actions, int rb) {
    // rb: the products of the heads take h and the weights rounded to bfloat16 (h itself is stored as computed)
    const int F4 = heads_f4(F), WP = F4 + 4;                        // hs: [4][F4], weights [A+1][F4+4], partial dots
    float *wsh = hs + 4 * F4;
    const int nf = min(4, B - b0);
    const int nout = nf * (A + 1);
    // thread tid < nout finishes output a of frame fb
    const int ofb = min(tid / (A + 1), nf - 1), oa = tid % (A + 1);
    const float obias = oa < A ? bp[oa] : bv[0];
    const float ou = (actions && tid < nout) ? uniforms[b0 + ofb] : 0.f;
    // padding columns of the LDS rows stay zero
    for (int e = tid; e < 4 * (F4 - F); e += NT) hs[(e / (F4 - F)) * F4 + F + e % (F4 - F)] = 0.f;
    if (!WSTAGED)
        for (int e = tid; e < (A + 1) * (WP - F); e += NT) wsh[(e / (WP - F)) * WP + F + e % (WP - F)] = 0.f;
    const int nw = (A + 1) * F;                 // Wp [A][F] and Wv [F] are adjacent in LDS, not in global memory
    const bool vec4 = !WSTAGED && ws && heads_vec4_ok(F, ws, fcb, h, Wp);
    if (vec4) heads_load_vec4<NT, 4, 16>(hs, wsh, tid, b0, nf, ws, nz, fcb, h, B, F, F4, WP, A, Wp, Wv, rb);
    for (int e0 = 0; !vec4 && ((!WSTAGED && e0 < nw) || e0 == 0); e0 += 24 * NT) {
        float wv[24];
        if (!WSTAGED) {
#pragma unroll
            for (int j = 0; j < 24; ++j) {
                const int e = min(e0 + j * NT + tid, nw - 1);
                wv[j] = e < A * F ? Wp[e] : Wv[e - A * F];
            }
        }
        if (e0 == 0) {
            for (int o = tid; o < F; o += NT) {
                if (ws) {
                    const float bias = fcb[o];
                    const size_t stride = (size_t)B * F;
                    const float *src = ws + (size_t)b0 * F + o;
                    float acc4[4] = {0.f, 0.f, 0.f, 0.f};
                    for (int z = 0; z < nz; z += 16) {
                        float v[4][16];
#pragma unroll
                        for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                v[fb][i] = src[min(z + i, nz - 1) * stride + (size_t)min(fb, nf - 1) * F];
#pragma unroll
                        for (int fb = 0; fb < 4; ++fb)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc4[fb] += (z + i < nz) ? v[fb][i] : 0.f;
                    }
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb) {
                        float v = acc4[fb] + bias;
                        v = v > 0.f ? v : 0.f;
                        if (fb < nf) h[(size_t)(b0 + fb) * F + o] = v;
                        hs[fb * F4 + o] = rb ? bf16_rne(v) : v;
                    }
                } else {
                    float v[4];
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb) {
                        const float *src = h + (size_t)(b0 + min(fb, nf - 1)) * F + o;
                        v[fb] = COHERENT ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
                    }
#pragma unroll
                    for (int fb = 0; fb < 4; ++fb) hs[fb * F4 + o] = rb ? bf16_rne(v[fb]) : v[fb];
                }
            }
        }
        if (!WSTAGED) {
#pragma unroll
            for (int j = 0; j < 24; ++j) {
                const int e = e0 + j * NT + tid;
                if (e < nw) wsh[(e / F) * WP + e % F] = rb ? bf16_rne(wv[j]) : wv[j];
            }
        }
    }
    __syncthreads();
    // Dot products from LDS, 16 bytes per read, without cross-lane traffic:
    // thread (frame, output, part of k) adds its share; KP shares make one output (three where the block has
    // threads for them, fewer when there are many actions).
    float *zs = wsh + (A + 1) * WP;                  // [4][A+1][3] partial dots, then [4][A+1] values
    const int KP = max(1, min(3, 256 / (4 * (A + 1))));      // the first 256 threads finish the outputs
    if (tid < KP * nout) {
        const int kp = tid / nout, r = tid % nout;
        const int fb = r / (A + 1), a = r % (A + 1);
        const int nk = F4 / 4;
        const int klo = (nk * kp) / KP, khi = (nk * (kp + 1)) / KP;
        const float4 *hb = (const float4 *)(hs + fb * F4), *wr = (const float4 *)(wsh + a * WP);
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 4
        for (int k = klo; k < khi; ++k) {
            const float4 x = hb[k], w = wr[k];
            s0 += x.x * w.x; s1 += x.y * w.y; s2 += x.z * w.z; s3 += x.w * w.w;
        }
        zs[(fb * (A + 1) + a) * 3 + kp] = (s0 + s1) + (s2 + s3);
    }
    __syncthreads();
    float z = 0.f;
    const bool mine = tid < nout;
    const int b = b0 + ofb;
    if (mine) {
        z = zs[tid * 3];
        for (int kp = 1; kp < KP; ++kp) z += zs[tid * 3 + kp];
        z += obias;
        if (zv) zv[(size_t)b * (A + 1) + oa] = z;
        if (oa < A && logits) logits[(size_t)b * A + oa] = z;
        if (oa == A && values) values[b] = z;
    }
    if (!probs && !actions) return;
    // Softmax and the draw, one thread per (frame, action).  The sums run left to
    // right in fp32 exactly as a single thread would form them, so the sampled
    // action is a pure function of the probabilities written out.
    const bool pol = mine && oa < A;
    float *zr = zs + ofb * (A + 1);
    __syncthreads();                                  // all partials are consumed
    if (mine) zs[tid] = z;
    __syncthreads();
    float e = 0.f;
    if (pol) {
        float zmax = zr[0];
        for (int j = 1; j < A; ++j) zmax = fmaxf(zmax, zr[j]);
        e = expf(z - zmax);
    }
    __syncthreads();
    if (pol) zr[oa] = e;
    __syncthreads();
    float pr = 0.f;
    if (pol) {
        float S = 0.f;
        for (int j = 0; j < A; ++j) S += zr[j];
        pr = e / S;
        if (probs) probs[(size_t)b * A + oa] = pr;
    }
    if (!actions) return;
    __syncthreads();
    if (pol) zr[oa] = pr;
    __syncthreads();
    if (pol) {
        float c = 0.f, cprev = 0.f;
        for (int j = 0; j <= oa; ++j) { cprev = c; c += zr[j]; }
        // the first action whose running sum exceeds u; the last one if none does
        if (c > ou && !(oa > 0 && cprev > ou)) actions[b] = oa;
        else if (oa == A - 1 && !(c > ou)) actions[b] = A - 1;
    }
}

__global__ __launch_bounds__(256) void heads_fwd_kernel(const float *__restrict__ ws, int nz,
                                                        const float *__restrict__ fcb, float *__restrict__ h, int B,
                                                        int F, int A, const float *__restrict__ Wp,
                                                        const float *__restrict__ bp, const float *__restrict__ Wv,
                                                        const float *__restrict__ bv, float *zv, float *logits,
                                                        float *values, float *probs, const float *uniforms,
                                                        int32_t *actions, int rb) {
    extern __shared__ __attribute__((aligned(16))) float heads_smem[];
    heads_fwd_body<256, false, false>(heads_smem, threadIdx.x, blockIdx.x * 4, ws, nz, fcb, h, B, F, A, Wp, bp, Wv, bv, zv, logits,
                               values, probs, uniforms, actions, rb);
}

// The whole forward pass of the small network (Sec. 3.2) for a handful of frames in ONE launch, for the latency of a
// small prediction batch (the paper's Sec. 5.2 finds the per-call overhead, not the arithmetic, dominant there).
// SLICES blocks work on each frame (32 for up to 8 frames, 16 for up to 16, 8 for up to 32, 4 for up to 64: at most one
// block per compute unit either way):
// every one of them runs both convolution layers of the frame (the same work SLICES times: the chip is otherwise
// idle), keeps the result in LDS and computes its own 256 / SLICES outputs of the fully connected layer, two per
// wavefront: the idle layer-1 wavefronts fetch their weight rows while layer 2 runs; with 16 slices the layer-2
// wavefronts take two rows each as well and fetch them when they are done.  The block that finishes a frame's fc
// outputs last (a ticket counter per frame; nobody waits for anybody) runs the heads, the softmax and the draw for
// that frame.  h [B][256]; ticket [B][SP_TICKET_PITCH], zero before the launch and zero
// again after it.
constexpr int SP_FC = 256, SP_FLAT = 2592, SP_MAX_FRAMES = 64;
constexpr int SP_TICKET_PITCH = 32;                        // ints between two frames' counters: a cache line each
// LDS of the heads: the 4 KB of fc outputs end where the layer-2 output ends, the weights follow in the part of the
// second layer-1 buffer that a single frame never touches, so that they can be staged while the convolutions run.
constexpr size_t SP_HEADS_OFF = C12_Y2S_OFF + sizeof(float) * (SP_FLAT - 4 * SP_FC);
constexpr size_t SP_HEADS_MAX = sizeof(__bf16) * (C12_XS + 2 * 3 * C12_Y1) - SP_HEADS_OFF;
constexpr int SP_ROWS = 2;                                 // fc outputs per wavefront
constexpr int SP_WJ = (SP_FLAT / 4 + 63) / 64;             // 16-byte vectors of one fc row per lane

template <bool ONE, int SLICES>
__global__ __launch_bounds__(512, 1) void predict_small_kernel(
    const uint8_t *__restrict__ x, const u32x4 *__restrict__ frag, const float *__restrict__ b1,
    const float *__restrict__ b2, const float *__restrict__ Wfc, const float *__restrict__ fcb, float *__restrict__ h,
    int *__restrict__ ticket, int A, const float *__restrict__ Wp, const float *__restrict__ bp,
    const float *__restrict__ Wv, const float *__restrict__ bv, float *logits, float *values, float *probs,
    const float *uniforms, int32_t *actions, float scale, int rb) {
    extern __shared__ __attribute__((aligned(16))) unsigned char sp_smem[];
    __shared__ int last;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // fc rows of a block: 256 / SLICES.  32 slices: the four layer-1 wavefronts take two rows each; 16 or fewer
    // slices: all eight wavefronts take two rows per pass, in 1, 2 or 4 passes.
    constexpr bool ALL_WAVES_FC = SLICES <= 16;
    constexpr int PASSES = ALL_WAVES_FC ? SP_FC / (SLICES * 8 * SP_ROWS) : 1;
    static_assert(SLICES * 4 * SP_ROWS == SP_FC || SLICES * 8 * SP_ROWS * PASSES == SP_FC, "two fc outputs per wavefront and pass");
    const int frame = blockIdx.x / SLICES, slice = blockIdx.x % SLICES;
    // first fc output of my wavefront in pass p
    auto row0 = [&](int p) { return slice * (SP_FC / SLICES) + (p * (ALL_WAVES_FC ? 8 : 4) + wave) * SP_ROWS; };

    // the layer-2 wavefronts ask for the heads' weights now (with their filters, before the first barrier waits for
    // both) and put them into LDS while layer 1 runs
    float hw[24];
    const bool hw_early = (A + 1) * SP_FC <= 24 * 256;
    if (wave >= 4 && hw_early) heads_load_weights<256>(hw, tid - 256, SP_FC, A, Wp, Wv);
    float4 wreg[PASSES > 1 ? 2 : 1][SP_ROWS][SP_WJ];
    float fbias[PASSES > 1 ? 2 : 1][SP_ROWS];
    auto load_rows = [&](int set, int p) {
        const int o0 = row0(p);
#pragma unroll
        for (int r = 0; r < SP_ROWS; ++r) fbias[set][r] = fcb[min(o0 + r, SP_FC - 1)];
#pragma unroll
        for (int r = 0; r < SP_ROWS; ++r)
#pragma unroll
            for (int j = 0; j < SP_WJ; ++j)          // rows are 16-byte aligned: the tensor starts on one and a row is 2592 floats
                wreg[set][r][j] = ((const float4 *)(Wfc + (size_t)min(o0 + r, SP_FC - 1) * SP_FLAT))[min(lane + 64 * j, SP_FLAT / 4 - 1)];
    };
    // the loads happen where this is called, and not where the compiler finds their first use
    auto pin_rows = [&](int set) {
#pragma unroll
        for (int r = 0; r < SP_ROWS; ++r)
#pragma unroll
            for (int j = 0; j < SP_WJ; ++j)
                asm volatile("" : "+v"(wreg[set][r][j].x), "+v"(wreg[set][r][j].y), "+v"(wreg[set][r][j].z), "+v"(wreg[set][r][j].w));
#pragma unroll
        for (int r = 0; r < SP_ROWS; ++r) asm volatile("" : "+v"(fbias[set][r]));
    };
    auto fetch_rows = [&](int it) {      // the idle layer-1 wavefronts, while layer 2 runs
        if (it != 1) return;
        load_rows(0, 0);
        pin_rows(0);
    };
    auto store_heads_weights = [&]() {
        if (hw_early) heads_store_weights<256>((float *)(sp_smem + SP_HEADS_OFF), hw, tid - 256, SP_FC, A, rb);
        else heads_stage_weights<256>((float *)(sp_smem + SP_HEADS_OFF), tid - 256, SP_FC, A, Wp, Wv, rb);
    };
    conv12_fused_block<ONE, false, true>(x, frag, b1, b2, nullptr, nullptr, frame, 1 << 24, frame + 1, scale, sp_smem,
                                         fetch_rows, store_heads_weights);
    if (ALL_WAVES_FC && wave >= 4) { load_rows(0, 0); pin_rows(0); }
    __syncthreads();
    if (ALL_WAVES_FC || wave < 4) {
        const float *y2s = (const float *)(sp_smem + C12_Y2S_OFF);
        float4 yreg[PASSES > 1 ? SP_WJ : 1];     // several passes: the layer-2 output is read from LDS once
        if (PASSES > 1) {
#pragma unroll
            for (int j = 0; j < SP_WJ; ++j) {
                yreg[j] = ((const float4 *)y2s)[min(lane + 64 * j, SP_FLAT / 4 - 1)];
                if (rb) yreg[j] = bf16_rne(yreg[j]);
            }
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int set = p & 1;
            if (p + 1 < PASSES) load_rows(set ^ 1, p + 1);      // the next pass's rows travel while this pass adds up
            const int o0 = row0(p);
#pragma unroll
            for (int r = 0; r < SP_ROWS; ++r) {
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < SP_WJ; ++j) {
                    const int k4 = lane + 64 * j;
                    float4 y, w = wreg[set][r][j];
                    if (PASSES > 1) y = yreg[j];
                    else {
                        y = ((const float4 *)y2s)[min(k4, SP_FLAT / 4 - 1)];
                        if (rb) y = bf16_rne(y);
                    }
                    if (rb) w = bf16_rne(w);
                    const float d = (y.x * w.x + y.y * w.y) + (y.z * w.z + y.w * w.w);
                    sum += k4 < SP_FLAT / 4 ? d : 0.f;
                }
#pragma unroll
                for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
                if (lane == 0) {
                    const float v = sum + fbias[set][r];
                    // written through to where every compute unit sees it (a device-wide fence instead would write
                    // back and invalidate the whole L2 of this block's XCD, once per block)
                    __hip_atomic_store(h + (size_t)frame * SP_FC + o0 + r, v > 0.f ? v : 0.f, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    }
    // Hand-off to whichever block finishes the frame last.  Order of events that makes its reads of h safe:
    //  1. every wavefront waits until the memory system has acknowledged its own stores of h (they are device-scope
    //     atomic stores, which the hardware writes through to the level all compute units share, and a store leaves
    //     the wavefront's count of outstanding memory operations only when that write is acknowledged);
    //  2. the barrier: all of the block's stores of h are therefore acknowledged before thread 0 goes on;
    //  3. thread 0 draws the ticket with a device-scope read-modify-write and waits for its result;
    //  4. the block that draws the last ticket knows that steps 1-3 of every other block are complete, and reads h
    //     with device-scope atomic loads issued after its ticket returned: they are served from the shared level.
    // No fence is used: a device-scope release or acquire fence writes back / invalidates the whole L2 of the XCD,
    // which costs more than the three kernels this one replaces when a training step shares the chip.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
        int *mine = ticket + frame * SP_TICKET_PITCH;
        const int t = __hip_atomic_fetch_add(mine, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = t == SLICES - 1;
        // for the next launch (stream order puts it after this kernel's end, which completes the store)
        if (last) __hip_atomic_store(mine, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!last) return;
    heads_fwd_body<512, true, true>((float *)(sp_smem + SP_HEADS_OFF), tid, frame, nullptr, 0, fcb, h, frame + 1, SP_FC, A, Wp, bp, Wv, bv, nullptr,
                              logits, values, probs, uniforms, actions, rb);
}

// n-step return (text after Eq. 1) of frame i when the segments have unequal
// lengths (Sec. 4.1: an agent hands in fewer than t_max experiences when its
// episode ends): segment n is the frames seg_start[n] .. seg_start[n+1]-1 and
// the return after its last frame is bootstrap[n].  The segment of frame i is
// the last n with seg_start[n] <= i, so empty segments are passed over.  The
// walk is bounded by the frame count whatever the table holds.
__device__ __forceinline__ float ragged_return(const float *__restrict__ rewards, const uint8_t *__restrict__ dones,
                                               const int32_t *__restrict__ seg_start, const float *__restrict__ bootstrap,
                                               int N, int B, int i, float gamma) {
    int lo = 0, hi = N - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (seg_start[mid] <= i) lo = mid; else hi = mid - 1;
    }
    const int end = min(seg_start[lo + 1], B);
    float next = bootstrap ? bootstrap[lo] : 0.f;
    for (int j = end - 1; j >= i; --j) next = rewards[j] + gamma * (dones[j] ? 0.f : 1.f) * next;
    return next;
}

// n-step returns (text after Eq. 1) and the loss with its gradient w.r.t. the
// head outputs (Eq. 1, 2, 5), one thread per frame (n, t).  The thread walks
// its agent's steps T-1 .. t to get R_t, in the order of the recursion.  The
// block first copies the head outputs of its frames to LDS in one sweep.
// Per-block sums of the three loss pieces go to part[3*block..].
// Dynamic LDS: LOSS_THREADS * (A + 1) floats.
__global__ __launch_bounds__(LOSS_THREADS) void returns_loss_kernel(
    const float *__restrict__ zv, const int32_t *__restrict__ actions, const float *__restrict__ rewards,
    const uint8_t *__restrict__ dones, const float *__restrict__ bootstrap, const int32_t *__restrict__ seg_start, int N,
    int T, int B, int A, float gamma, float beta, float cv, float eps, float *__restrict__ R, float *__restrict__ dzv,
    float *__restrict__ part) {
    extern __shared__ float zsh[];     // [LOSS_THREADS][A+1]
    const int i0 = blockIdx.x * LOSS_THREADS;
    const int i = i0 + threadIdx.x;
    const int nrows = min(LOSS_THREADS, B - i0);
    copy_to_lds<8>(zsh, zv + (size_t)i0 * (A + 1), nrows * (A + 1), threadIdx.x, LOSS_THREADS);
    float s_pl = 0.f, s_vl = 0.f, s_en = 0.f;
    float next = 0.f;
    int a = 0;
    if (i < B) {
        a = actions[i];
        if (seg_start) {
            next = ragged_return(rewards, dones, seg_start, bootstrap, N, B, i, gamma);
        } else {
            const int n = i / T, t = i % T;
            next = bootstrap ? bootstrap[n] : 0.f;
            for (int tt = T - 1; tt >= t; --tt) {
                const size_t j = (size_t)n * T + tt;
                next = rewards[j] + gamma * (dones[j] ? 0.f : 1.f) * next;
            }
        }
        R[i] = next;
    }
    __syncthreads();
    if (i < B) {
        const float *z = zsh + threadIdx.x * (A + 1);
        float *dz = dzv + (size_t)i * (A + 1);
        const float V = z[A];
        const float adv = next - V;
        float zmax = z[0];
        for (int j = 1; j < A; ++j) zmax = fmaxf(zmax, z[j]);
        float S = 0.f;
        for (int j = 0; j < A; ++j) S += expf(z[j] - zmax);
        const float logS = logf(S), invS = 1.f / S;
        // dL/dp_k = beta (lg_k + r_k) - [k=a] adv/(p_a+eps);  lg = log(p+eps), r = p/(p+eps)
        float H = 0.f, dot = 0.f, lga = 0.f, ra = 1.f;
        for (int j = 0; j < A; ++j) {
            const float p = expf(z[j] - zmax) * invS;
            float lg, r;
            if (eps == 0.f) { lg = z[j] - zmax - logS; r = 1.f; }
            else { lg = logf(p + eps); r = p / (p + eps); }
            H -= p * lg;
            dot += p * beta * (lg + r);
            if (j == a) { lga = lg; ra = r; }
        }
        dot -= adv * ra;
        for (int j = 0; j < A; ++j) {
            const float p = expf(z[j] - zmax) * invS;
            float lg, r;
            if (eps == 0.f) { lg = z[j] - zmax - logS; r = 1.f; }
            else { lg = logf(p + eps); r = p / (p + eps); }
            dz[j] = p * (beta * (lg + r) - dot) - (j == a ? adv * ra : 0.f);
        }
        dz[A] = -2.f * cv * adv;
        s_pl = -lga * adv;
        s_vl = adv * adv;
        s_en = H;
    }
    __shared__ float sh[3][LOSS_THREADS / 64];
    s_pl = wave_sum(s_pl); s_vl = wave_sum(s_vl); s_en = wave_sum(s_en);
    if ((threadIdx.x & 63) == 0) {
        sh[0][threadIdx.x >> 6] = s_pl; sh[1][threadIdx.x >> 6] = s_vl; sh[2][threadIdx.x >> 6] = s_en;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        float s = 0.f;
        for (int w = 0; w < LOSS_THREADS / 64; ++w) s += sh[threadIdx.x][w];
        part[3 * blockIdx.x + threadIdx.x] = s;
    }
}

// dL/d(pre-activation of fc)[b][k] = [h > 0] * (sum_a dz[b][a] Wp[a][k] + dv[b] Wv[k]).
// A block takes HD_FRAMES frames; both weight matrices and the frames' dz rows
// are first copied to LDS.  colpart[block][k] receives the block's sum over
// its frames, which a reduction turns into the fc bias gradient.  Dynamic LDS: (A + 1) * (F + HD_FRAMES) floats.
constexpr int HD_FRAMES = 8;
__global__ __launch_bounds__(256) void heads_dgrad_kernel(const float *__restrict__ dzv, const float *__restrict__ h,
                                                          const float *__restrict__ Wp, const float *__restrict__ Wv,
                                                          int B, int F, int A, float *__restrict__ dh,
                                                          float *__restrict__ colpart, float *__restrict__ wpart, int rb) {
    // rb: every product takes its operands rounded to bfloat16, and the sums that are products with ones
    // (the bias gradients) take rounded terms; dh is stored as computed
    extern __shared__ float sm[];
    float *wsh = sm;                        // [A+1][F]
    float *dzs = sm + (A + 1) * F;          // [HD_FRAMES][A+1]
    const int tid = threadIdx.x;
    const int b0 = blockIdx.x * HD_FRAMES;
    const int nf = min(HD_FRAMES, B - b0);
    copy_to_lds<8>(wsh, Wp, A * F, tid, 256);
    copy_to_lds<2>(wsh + A * F, Wv, F, tid, 256);
    copy_to_lds<1>(dzs, dzv + (size_t)b0 * (A + 1), nf * (A + 1), tid, 256);
    __syncthreads();
    if (rb) {
        for (int e = tid; e < (A + 1) * F; e += 256) wsh[e] = bf16_rne(wsh[e]);
        for (int e = tid; e < nf * (A + 1); e += 256) dzs[e] = bf16_rne(dzs[e]);
        __syncthreads();
    }
    for (int k = tid; k < F; k += 256) {
        float hv[HD_FRAMES];
#pragma unroll
        for (int fb = 0; fb < HD_FRAMES; ++fb) hv[fb] = h[(size_t)(b0 + min(fb, nf - 1)) * F + k];
        float s[HD_FRAMES];
#pragma unroll
        for (int fb = 0; fb < HD_FRAMES; ++fb) s[fb] = 0.f;
        // wpart (optional): this block's share of the heads' weight gradient,
        // [block][A+1][F+1] with the bias gradient in the last column
        float *wp = wpart ? wpart + (size_t)blockIdx.x * (A + 1) * (F + 1) + k : nullptr;
        for (int a = 0; a <= A; ++a) {
            const float wv = wsh[a * F + k];
            float gw = 0.f;
#pragma unroll
            for (int fb = 0; fb < HD_FRAMES; ++fb) {
                const float d = dzs[min(fb, nf - 1) * (A + 1) + a];
                s[fb] += d * wv;
                gw += fb < nf ? d * (rb ? bf16_rne(hv[fb]) : hv[fb]) : 0.f;
            }
            if (wp) wp[(size_t)a * (F + 1)] = gw;
        }
        float col = 0.f;
#pragma unroll
        for (int fb = 0; fb < HD_FRAMES; ++fb)
            if (fb < nf) {
                const float v = hv[fb] > 0.f ? s[fb] : 0.f;
                dh[(size_t)(b0 + fb) * F + k] = v;
                col += rb ? bf16_rne(v) : v;
            }
        colpart[(size_t)blockIdx.x * F + k] = col;      // this block's share of the fc bias gradient
    }
    if (wpart && tid <= A) {
        float gb = 0.f;
        for (int fb = 0; fb < nf; ++fb) gb += dzs[fb * (A + 1) + tid];
        wpart[((size_t)blockIdx.x * (A + 1) + tid) * (F + 1) + F] = gb;
    }
}

// Training only: everything between the fc products and the fc backward in one
// kernel, for HD_FRAMES frames per block.  (1) last step of the split-k fc layer:
// h = max(0, bias + sum_z ws[z]); (2) heads: z = W h + b; (3) n-step returns
// (text after Eq. 1), loss and its gradient w.r.t. the head outputs (Eq. 1, 2,
// 5), one thread per (frame, action), sums taken in action order so that they
// do not depend on the thread layout; (4) heads backward: dh = [h > 0] dz W,
// and the block's shares of the heads' weight and bias gradients (wpart
// [block][A+1][F+1]) and of the fc bias gradient (colpart [block][F]): a
// thread takes four consecutive k and every fourth output (its wavefront's),
// so that weights, activations and gradients move as 16-byte vectors; the four
// partial sums of dh meet in LDS.
// Writes h, zv, R, dzv (kept for inspection), dh, colpart, wpart and three loss
// sums per block.  rb: operands of every product rounded to bfloat16.
// Dynamic LDS: heads_train_lds_floats(F, A) floats.
__host__ __device__ inline int heads_train_kparts(int F, int A) {
    const int kp = 256 / (A + 1), nk = heads_f4(F) / 4;
    return kp < nk ? kp : nk;
}
__host__ __device__ inline int heads_train_lds_floats(int F, int A) {
    return HD_FRAMES * heads_f4(F) + (A + 1) * (heads_f4(F) + 4) + 4 * HD_FRAMES * 256 + (A + 1) * HD_FRAMES +
           3 * HD_FRAMES * heads_f4(A + 1) + HD_FRAMES * (A + 1) * heads_train_kparts(F, A) + 512;
}

__global__ __launch_bounds__(256) void heads_train_kernel(
    const float *__restrict__ ws, int nz, const float *__restrict__ fcb, int B, int F, int A,
    const float *__restrict__ Wp, const float *__restrict__ bp, const float *__restrict__ Wv, const float *__restrict__ bv,
    const int32_t *__restrict__ actions, const float *__restrict__ rewards, const uint8_t *__restrict__ dones,
    const float *__restrict__ bootstrap, const int32_t *__restrict__ seg_start, int N, int T, float gamma, float beta,
    float cv, float eps, float *__restrict__ h, float *__restrict__ zv, float *__restrict__ R, float *__restrict__ dzv,
    float *__restrict__ dh, float *__restrict__ colpart, float *__restrict__ wpart, float *__restrict__ losspart, int rb) {
    extern __shared__ __attribute__((aligned(16))) float sm[];
    constexpr int NF = HD_FRAMES;
    const int F4 = heads_f4(F), WP = F4 + 4, A1 = A + 1, KP = heads_train_kparts(F, A);
    const int ZR = heads_f4(A1);             // row pitch of the per-(frame, output) arrays: rows start on 16 bytes
    float *hs = sm;                          // [NF][F4]   fc output of my frames (rounded if rb)
    float *wsh = hs + NF * F4;               // [A1][WP]   head weights (rounded if rb)
    float *red = wsh + A1 * WP;              // [4][NF][256] partial sums of dh, one set per wavefront
    float *zt = red + 4 * NF * 256;          // [A1][NF]   gradients of the head outputs, transposed
    float *zs = zt + A1 * NF;                // [NF][ZR]   head outputs, later their gradients
    float *ex = zs + NF * ZR;                // [NF][ZR]   exp / per-action terms
    float *tm = ex + NF * ZR;                // [NF][ZR]   per-action terms
    float *zp = tm + NF * ZR;                // [NF][A1][KP] partial dots
    float *rw = zp + NF * A1 * KP;           // [256]      rewards of the agents my frames belong to
    float *dn = rw + 256;                    // [256]      1 - done
    const int tid = threadIdx.x;
    const int b0 = blockIdx.x * NF;
    const int nf = min(NF, B - b0);

    // ---- everything from global memory is requested first
    const int n0 = b0 / T, n1 = (b0 + nf - 1) / T;          // agents of my frames
    const int nrw = (n1 - n0 + 1) * T;
    const bool rw_lds = !seg_start && nrw <= 256;      // segments of unequal length read their rewards from global memory
    float my_rw = 0.f, my_dn = 0.f;
    if (rw_lds && tid < nrw) { my_rw = rewards[(size_t)n0 * T + tid]; my_dn = dones[(size_t)n0 * T + tid] ? 0.f : 1.f; }
    const int ofb = min(tid / A1, nf - 1), oa = tid % A1;   // thread tid < nf*A1 owns output oa of frame ofb
    const bool mine = tid < nf * A1;
    const int ob = b0 + ofb;
    const float obias = oa < A ? bp[oa] : bv[0];
    const int oact = actions[ob];
    const float oboot = bootstrap && !seg_start ? bootstrap[ob / T] : 0.f;
    for (int e = tid; e < NF * (F4 - F); e += 256) hs[(e / (F4 - F)) * F4 + F + e % (F4 - F)] = 0.f;
    for (int e = tid; e < A1 * (WP - F); e += 256) wsh[(e / (WP - F)) * WP + F + e % (WP - F)] = 0.f;
    const int nw = A1 * F;
    const bool vec4 = heads_vec4_ok(F, ws, fcb, h, Wp);
    if (vec4) heads_load_vec4<256, NF, 8>(hs, wsh, tid, b0, nf, ws, nz, fcb, h, B, F, F4, WP, A, Wp, Wv, rb);
    for (int e0 = 0; !vec4 && (e0 < nw || e0 == 0); e0 += 24 * 256) {
        float wv[24];
#pragma unroll
        for (int j = 0; j < 24; ++j) {
            const int e = min(e0 + j * 256 + tid, nw - 1);
            wv[j] = e < A * F ? Wp[e] : Wv[e - A * F];
        }
        if (e0 == 0) {
            for (int o = tid; o < F; o += 256) {
                const float bias = fcb[o];
                const size_t stride = (size_t)B * F;
                const float *src = ws + (size_t)b0 * F + o;
                float acc[NF];
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) acc[fb] = 0.f;
                for (int z = 0; z < nz; z += 8) {
                    float v[NF][8];
#pragma unroll
                    for (int fb = 0; fb < NF; ++fb)
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            v[fb][i] = src[min(z + i, nz - 1) * stride + (size_t)min(fb, nf - 1) * F];
#pragma unroll
                    for (int fb = 0; fb < NF; ++fb)
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[fb] += (z + i < nz) ? v[fb][i] : 0.f;
                }
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) {
                    float v = acc[fb] + bias;
                    v = v > 0.f ? v : 0.f;
                    if (fb < nf) h[(size_t)(b0 + fb) * F + o] = v;
                    hs[fb * F4 + o] = rb ? bf16_rne(v) : v;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < 24; ++j) {
            const int e = e0 + j * 256 + tid;
            if (e < nw) wsh[(e / F) * WP + e % F] = rb ? bf16_rne(wv[j]) : wv[j];
        }
    }
    if (rw_lds && tid < nrw) { rw[tid] = my_rw; dn[tid] = my_dn; }
    __syncthreads();

    // ---- heads: thread (action a, part kp of k) for all frames, then the parts are added in order
    {
        const int a = tid % A1, kp = tid / A1;
        if (kp < KP) {
            const int nk = F4 / 4;
            const int klo = (nk * kp) / KP, khi = (nk * (kp + 1)) / KP;
            const float4 *wr = (const float4 *)(wsh + a * WP);
            float s[NF];
#pragma unroll
            for (int fb = 0; fb < NF; ++fb) s[fb] = 0.f;
            for (int k = klo; k < khi; ++k) {
                const float4 w = wr[k];
#pragma unroll
                for (int fb = 0; fb < NF; ++fb) {
                    const float4 x = ((const float4 *)(hs + fb * F4))[k];
                    s[fb] += (x.x * w.x + x.y * w.y) + (x.z * w.z + x.w * w.w);
                }
            }
#pragma unroll
            for (int fb = 0; fb < NF; ++fb) zp[(fb * A1 + a) * KP + kp] = s[fb];
        }
    }
    __syncthreads();
    float z = 0.f;
    if (mine) {
        const float *q = zp + (ofb * A1 + oa) * KP;
        for (int kp = 0; kp < KP; ++kp) z += q[kp];
        z += obias;
        zv[(size_t)ob * A1 + oa] = z;
        zs[ofb * ZR + oa] = z;
    }
    // ---- n-step return of my frame (threads with oa == A: one per frame)
    float Rt = 0.f;
    if (mine && oa == A) {
        const int n = ob / T, t = ob % T;
        float next = oboot;
        if (seg_start) {
            next = ragged_return(rewards, dones, seg_start, bootstrap, N, B, ob, gamma);
        } else if (rw_lds) {
            for (int tt = T - 1; tt >= t; --tt) { const int j = (n - n0) * T + tt; next = rw[j] + gamma * dn[j] * next; }
        } else {
            for (int tt = T - 1; tt >= t; --tt) {
                const size_t j = (size_t)n * T + tt;
                next = rewards[j] + gamma * (dones[j] ? 0.f : 1.f) * next;
            }
        }
        Rt = next;
        R[ob] = next;
        tm[ofb * ZR + A] = next;             // the policy threads of the frame read it from here
    }
    __syncthreads();
    // ---- loss and dL/dz, thread (frame, action); sums over the actions run in index order
    const bool pol = mine && oa < A;
    // rows are read four values at a time; sums still add one value after the other, in index order
    const float *zr = zs + ofb * ZR;
    float zmax = 0.f, e = 0.f;
    if (pol) {
        zmax = zr[0];
        for (int j = 0; j < A; j += 4) {
            const float4 q = *(const float4 *)(zr + j);
            zmax = fmaxf(zmax, q.x);
            if (j + 1 < A) zmax = fmaxf(zmax, q.y);
            if (j + 2 < A) zmax = fmaxf(zmax, q.z);
            if (j + 3 < A) zmax = fmaxf(zmax, q.w);
        }
        e = expf(z - zmax);
        ex[ofb * ZR + oa] = e;
    }
    __syncthreads();
    float p = 0.f, lg = 0.f, r = 1.f, adv = 0.f;
    if (mine) {
        const float V = zr[A];
        adv = tm[ofb * ZR + A] - V;
    }
    if (pol) {
        float S = 0.f;
        for (int j = 0; j < A; j += 4) {
            const float4 q = *(const float4 *)(ex + ofb * ZR + j);
            S += q.x;
            if (j + 1 < A) S += q.y;
            if (j + 2 < A) S += q.z;
            if (j + 3 < A) S += q.w;
        }
        const float logS = logf(S), invS = 1.f / S;
        p = e * invS;
        if (eps == 0.f) { lg = z - zmax - logS; r = 1.f; }
        else { lg = logf(p + eps); r = p / (p + eps); }
    }
    __syncthreads();                                  // every exp has been read
    if (pol) {
        ex[ofb * ZR + oa] = p * lg;                   // -H terms
        tm[ofb * ZR + oa] = p * beta * (lg + r);      // dot terms
    }
    __syncthreads();
    float dzo = 0.f, s_pl = 0.f, s_vl = 0.f, s_en = 0.f;
    // the thread of the action taken publishes its lg and r
    if (pol && oa == oact) { dn[ofb * 2] = lg; dn[ofb * 2 + 1] = r; }      // (rw, dn are free again by now)
    __syncthreads();
    if (mine) {
        float H = 0.f, dot = 0.f;
        for (int j = 0; j < A; j += 4) {
            const float4 q = *(const float4 *)(ex + ofb * ZR + j), u = *(const float4 *)(tm + ofb * ZR + j);
            H -= q.x; dot += u.x;
            if (j + 1 < A) { H -= q.y; dot += u.y; }
            if (j + 2 < A) { H -= q.z; dot += u.z; }
            if (j + 3 < A) { H -= q.w; dot += u.w; }
        }
        const bool known = (unsigned)oact < (unsigned)A;
        const float lga = known ? dn[ofb * 2] : 0.f, ra = known ? dn[ofb * 2 + 1] : 1.f;
        dot -= adv * ra;
        if (oa < A) dzo = p * (beta * (lg + r) - dot) - (oa == oact ? adv * ra : 0.f);
        else {
            dzo = -2.f * cv * adv;
            s_pl = -lga * adv; s_vl = adv * adv; s_en = H;
        }
        dzv[(size_t)ob * A1 + oa] = dzo;
    }
    // the gradients go to zt[output][frame] (zero for frames the block does not have) for the backward pass
    if (tid < NF * A1) zt[oa * NF + tid / A1] = mine ? (rb ? bf16_rne(dzo) : dzo) : 0.f;
    // loss sums of the block, frames in order (threads oa == A hold them)
    if (mine && oa == A) { rw[ofb] = s_pl; rw[NF + ofb] = s_vl; rw[2 * NF + ofb] = s_en; }
    __syncthreads();
    if (tid < 3) {
        const float *src = rw + tid * NF;
        float sum = 0.f;
        for (int fb = 0; fb < nf; ++fb) sum += src[fb];
        losspart[3 * blockIdx.x + tid] = sum;
    }
    // ---- heads backward (zt holds dz of my frames).  Wavefront ag takes the outputs ag, ag + 4, ..; lane kl the four
    // k starting at kbase + 4 kl, 256 k per pass.
    typedef float f32x4_dword_aligned __attribute__((ext_vector_type(4), aligned(4)));
    const int ag = tid >> 6, kl = tid & 63;
    for (int kbase = 0; kbase < F; kbase += 256) {
        const int k4 = kbase + 4 * kl;
        const bool kin = k4 < F4;
        float4 hv[NF], sd[NF];
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) {
            hv[fb] = kin ? *(const float4 *)(hs + fb * F4 + k4) : float4{0.f, 0.f, 0.f, 0.f};
            sd[fb] = float4{0.f, 0.f, 0.f, 0.f};
        }
        float *wp = wpart + (size_t)blockIdx.x * A1 * (F + 1) + k4;
        for (int a = ag; a < A1; a += 4) {
            const float4 wv = kin ? *(const float4 *)(wsh + a * WP + k4) : float4{0.f, 0.f, 0.f, 0.f};
            const float4 d0 = *(const float4 *)(zt + a * NF), d1 = *(const float4 *)(zt + a * NF + 4);
            const float d[NF] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
            float4 gw = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int fb = 0; fb < NF; ++fb) {
                sd[fb].x += d[fb] * wv.x; sd[fb].y += d[fb] * wv.y; sd[fb].z += d[fb] * wv.z; sd[fb].w += d[fb] * wv.w;
                gw.x += d[fb] * hv[fb].x; gw.y += d[fb] * hv[fb].y; gw.z += d[fb] * hv[fb].z; gw.w += d[fb] * hv[fb].w;
            }
            float *dst = wp + (size_t)a * (F + 1);
            if (k4 + 3 < F) {
                *(f32x4_dword_aligned *)dst = f32x4_dword_aligned{gw.x, gw.y, gw.z, gw.w};
            } else {
                if (k4 < F) dst[0] = gw.x;
                if (k4 + 1 < F) dst[1] = gw.y;
                if (k4 + 2 < F) dst[2] = gw.z;
            }
        }
#pragma unroll
        for (int fb = 0; fb < NF; ++fb) *(float4 *)(red + (ag * NF + fb) * 256 + 4 * kl) = sd[fb];
        __syncthreads();
        const int k = kbase + tid;
        if (k < F) {
            float col = 0.f;
#pragma unroll
            for (int fb = 0; fb < NF; ++fb)
                if (fb < nf) {
                    const float sum = (red[fb * 256 + tid] + red[(NF + fb) * 256 + tid]) +
                                      (red[(2 * NF + fb) * 256 + tid] + red[(3 * NF + fb) * 256 + tid]);
                    const float v = hs[fb * F4 + k] > 0.f ? sum : 0.f;
                    dh[(size_t)(b0 + fb) * F + k] = v;
                    col += rb ? bf16_rne(v) : v;
                }
            colpart[(size_t)blockIdx.x * F + k] = col;
        }
        __syncthreads();                              // red is written again in the next pass
    }
    if (tid <= A) {
        float gb = 0.f;
        for (int fb = 0; fb < nf; ++fb) gb += zt[tid * NF + fb];
        wpart[((size_t)blockIdx.x * A1 + tid) * (F + 1) + F] = gb;
    }
}

// One launch adds up the partial weight gradients of every layer and, on the
// way, the squares of the results (for the global norm).
// A segment is a stack of nz partial matrices ws[z][M][N].  Rows [r0, r0+rows)
// go to gW[(m-r0)*(N-1) + n] for n < N-1 and gb[m-r0] for n = N-1 (bias_col),
// or all N columns to gW[(m-r0)*N + n] (no bias_col).  A block handles 256/zg
// outputs with zg threads each: thread j adds z = j, j+zg, ... (eight loads in
// flight at a time), then the zg sums are added in order of j.  Nothing depends
// on timing, so the gradient is reproducible bit for bit.
// Block ids go round-robin over the 8 XCDs; the ids of one XCD take consecutive
// groups of outputs, so that blocks which share 128-byte lines of the partial
// sums also share an L2.  Where the first row of the segment and the planes of the stack start on 16-byte
// boundaries a thread takes four consecutive outputs and reads its partial sums as 16-byte vectors (a quarter of the
// load instructions); the sums of an output are formed in the same order either way.
struct ReduceSeg {
    const float *ws;
    float *gW, *gb;
    int nz, M, N, r0, rows, bias_col, zg, first_block;
    int per_xcd;         // the segment owns 8 * per_xcd block ids, first_block is a multiple of 8
    int vec;             // a thread takes four consecutive outputs and reads 16-byte vectors (the stack allows it)
};
constexpr int MAX_REDUCE_SEGS = 12;
struct ReduceArgs {
    ReduceSeg seg[MAX_REDUCE_SEGS];
    int nseg;
    float *normpart;     // one partial sum of squares per block
};

__global__ __launch_bounds__(256) void reduce_all_kernel(const ReduceArgs a) {
    __shared__ float4 sh[256];
    __shared__ float wsum[4];
    int si = 0;
    while (si + 1 < a.nseg && (int)blockIdx.x >= a.seg[si + 1].first_block) ++si;
    const ReduceSeg &g = a.seg[si];
    const int opb = 256 / g.zg;
    const int o = threadIdx.x % opb, zi = threadIdx.x / opb;
    const size_t cnt = (size_t)g.rows * g.N;
    const int lb = blockIdx.x - g.first_block;
    const int per = g.vec ? 4 : 1;                      // outputs per thread
    const size_t i = (((size_t)(lb % 8) * g.per_xcd + lb / 8) * opb + o) * per;
    float4 s = float4{0.f, 0.f, 0.f, 0.f};
    const size_t src = (size_t)g.r0 * g.N + i, stride = (size_t)g.M * g.N;
    if (g.vec && i + 3 < cnt) {
        for (int z = zi; z < g.nz; z += 8 * g.zg) {
            float4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = *(const float4 *)(g.ws + (size_t)min(z + j * g.zg, g.nz - 1) * stride + src);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = z + j * g.zg < g.nz;
                s.x += in ? v[j].x : 0.f; s.y += in ? v[j].y : 0.f; s.z += in ? v[j].z : 0.f; s.w += in ? v[j].w : 0.f;
            }
        }
    } else if (i < cnt) {                               // one output, or the last, partial group of four
        const int ne = (int)min((size_t)per, cnt - i);
        for (int e = 0; e < ne; ++e) {
            float t = 0.f;
            for (int z = zi; z < g.nz; z += 8 * g.zg) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = g.ws[(size_t)min(z + j * g.zg, g.nz - 1) * stride + src + e];
#pragma unroll
                for (int j = 0; j < 8; ++j) t += (z + j * g.zg < g.nz) ? v[j] : 0.f;
            }
            if (e == 0) s.x = t; else if (e == 1) s.y = t; else if (e == 2) s.z = t; else s.w = t;
        }
    }
    sh[threadIdx.x] = s;
    __syncthreads();
    float sq = 0.f;
    if (zi == 0 && i < cnt) {
        float4 t = sh[o];
        for (int j = 1; j < g.zg; ++j) {
            const float4 u = sh[j * opb + o];
            t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
        }
        const float te[4] = {t.x, t.y, t.z, t.w};
        const int ne = (int)min((size_t)per, cnt - i);
        for (int e = 0; e < ne; ++e) {
            const size_t ie = i + e;
            const int m = (int)(ie / g.N), n = (int)(ie % g.N);
            if (!g.bias_col) g.gW[ie] = te[e];
            else if (n < g.N - 1) g.gW[(size_t)m * (g.N - 1) + n] = te[e];
            else g.gb[m] = te[e];
            sq += te[e] * te[e];
        }
    }
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) a.normpart[blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// Eq. 3 on a flat buffer: d = s*grad; g = alpha g + (1-alpha) d^2;
// theta_out = theta_in - lr d / sqrt(g + eps) (the two may be the same buffer).  20 bytes of traffic per parameter.
// s comes from one of three places: scale_host (normpart == nullptr and scale_dev == nullptr), scale_dev[0], or,
// inside a training step, the per-block squared norms of the gradient (normpart, nnorm of them): every block adds
// them up in the same fixed order and forms s = min(1, clip / norm) itself, and block 0 also writes the loss sums
// and the statistics, which saves the launch of a kernel of one block between the reduction and this one.
// A thread keeps four 16-byte vectors of each array in flight, which is what a streaming kernel needs to approach
// the memory's bandwidth on a buffer far larger than the caches.  VARIANT bit 0: loads, bit 1: stores bypass the caches.
struct RmsClip {
    const float *normpart; int nnorm;          // squared-norm partials of the gradient
    const float *losspart; int nloss;          // three loss sums per loss block
    float clip;                                // threshold of the global-norm rescale, <= 0: off
    float *scale_out;                          // receives s (1 float)
    ga3c_train_stats *own, *user;              // statistics (user may be null)
};

// streaming accesses: the line is not kept in the caches after use
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load(const float4 *p) {
    const f32x4_t v = __builtin_nontemporal_load((const f32x4_t *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store(const float4 v, float4 *p) {
    __builtin_nontemporal_store(f32x4_t{v.x, v.y, v.z, v.w}, (f32x4_t *)p);
}

__device__ __forceinline__ void rmsprop4(float4 &t, float4 &gg, float4 d, float s, float lr, float alpha, float oma, float eps) {
    d.x *= s; d.y *= s; d.z *= s; d.w *= s;
    gg.x = alpha * gg.x + oma * d.x * d.x; gg.y = alpha * gg.y + oma * d.y * d.y;
    gg.z = alpha * gg.z + oma * d.z * d.z; gg.w = alpha * gg.w + oma * d.w * d.w;
    t.x -= lr * d.x / sqrtf(gg.x + eps); t.y -= lr * d.y / sqrtf(gg.y + eps);
    t.z -= lr * d.z / sqrtf(gg.z + eps); t.w -= lr * d.w / sqrtf(gg.w + eps);
}

template <int VARIANT, int VPT>
__global__ __launch_bounds__(256) void rmsprop_kernel(const float *theta_in, float *theta_out, float *__restrict__ g,
                                                      const float *__restrict__ grad, size_t n,
                                                      const float *__restrict__ scale_dev, float scale_host, float lr,
                                                      float alpha, float eps, u32x4 *__restrict__ frag, unsigned w1_off,
                                                      unsigned w2_off, int frag_rb, const RmsClip clipargs) {
    // frag (optional): split MFMA fragments of the small net's conv filters, kept current with theta_out;
    // w1_off / w2_off: where the two filter tensors start in the flat buffer (multiples of 4)
    float s = scale_dev ? scale_dev[0] : scale_host;
    if (clipargs.normpart) {
        __shared__ float sh[4][4];
        const int tid = threadIdx.x;
        float acc[4] = {0.f, 0.f, 0.f, 0.f};     // norm^2, policy loss, value loss, entropy
        for (int i = tid; i < clipargs.nnorm; i += 8 * 256) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = clipargs.normpart[min(i + 256 * j, clipargs.nnorm - 1)];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[0] += (i + 256 * j < clipargs.nnorm) ? v[j] : 0.f;
        }
        if (blockIdx.x == 0)
            for (int i = tid; i < clipargs.nloss; i += 256)
                for (int c = 0; c < 3; ++c) acc[1 + c] += clipargs.losspart[3 * i + c];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            acc[c] = wave_sum(acc[c]);
            if ((tid & 63) == 0) sh[c][tid >> 6] = acc[c];
        }
        __syncthreads();
        float t[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) t[c] = (sh[c][0] + sh[c][1]) + (sh[c][2] + sh[c][3]);
        const float norm = sqrtf(t[0]);
        s = 1.f;
        if (clipargs.clip > 0.f && norm > clipargs.clip) s = clipargs.clip / norm;
        if (blockIdx.x == 0 && tid == 0) {
            clipargs.scale_out[0] = s;
            ga3c_train_stats st;
            st.policy_loss = t[1]; st.value_loss = t[2]; st.entropy = t[3];
            st.grad_norm = norm; st.clip_scale = s; st.nonfinite = !(norm <= 3.0e38f) ? 1 : 0;
            *clipargs.own = st;
            if (clipargs.user) *clipargs.user = st;
        }
    }
    const float oma = 1.f - alpha;
    const size_t n4 = n / 4;
    const size_t stride = (size_t)gridDim.x * 256;
    const float4 *t4 = (const float4 *)theta_in;
    float4 *o4 = (float4 *)theta_out;
    float4 *g4 = (float4 *)g;
    const float4 *d4 = (const float4 *)grad;
    // a block works on tiles of 256 * VPT consecutive vectors (16 KB of each array for VPT = 4): thread t takes vectors
    // t, t + 256, ... of the tile, all requested before the first is used
    const size_t ntile = n4 / (256 * VPT);
    for (size_t tile = blockIdx.x; tile < ntile; tile += gridDim.x) {
        const size_t i = tile * (256 * VPT) + threadIdx.x;
        float4 t[VPT], gg[VPT], d[VPT];
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            t[j] = VARIANT & 1 ? nt_load(t4 + i + 256 * j) : t4[i + 256 * j];
            gg[j] = VARIANT & 1 ? nt_load(g4 + i + 256 * j) : g4[i + 256 * j];
            d[j] = VARIANT & 1 ? nt_load(d4 + i + 256 * j) : d4[i + 256 * j];
        }
#pragma unroll
        for (int j = 0; j < VPT; ++j) {
            rmsprop4(t[j], gg[j], d[j], s, lr, alpha, oma, eps);
            if (VARIANT & 2) { nt_store(gg[j], g4 + i + 256 * j); nt_store(t[j], o4 + i + 256 * j); }
            else { g4[i + 256 * j] = gg[j]; o4[i + 256 * j] = t[j]; }
            if (frag) {
                const unsigned r1 = (unsigned)(4 * (i + 256 * j)) - w1_off, r2 = (unsigned)(4 * (i + 256 * j)) - w2_off;
                if (r1 < 16u * 256u) conv12_store_fragment4(frag, 0, (int)r1, t[j], frag_rb);
                else if (r2 < 32u * 256u) {
                    conv12_store_fragment4(frag, 1, (int)r2, t[j], frag_rb);
                    conv_dgrad_store_fragment4<SpecS2>(frag + CFRAG_FWD_VECS, (int)r2, t[j]);
                }
            }
        }
    }
    for (size_t i = ntile * (256 * VPT) + (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        float4 t = t4[i], gg = g4[i];
        rmsprop4(t, gg, d4[i], s, lr, alpha, oma, eps);
        g4[i] = gg; o4[i] = t;
        if (frag) {
            const unsigned r1 = (unsigned)(4 * i) - w1_off, r2 = (unsigned)(4 * i) - w2_off;
            if (r1 < 16u * 256u) conv12_store_fragment4(frag, 0, (int)r1, t, frag_rb);
            else if (r2 < 32u * 256u) {
                conv12_store_fragment4(frag, 1, (int)r2, t, frag_rb);
                conv_dgrad_store_fragment4<SpecS2>(frag + CFRAG_FWD_VECS, (int)r2, t);
            }
        }
    }
    for (size_t k = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) {
        const float d = s * grad[k];
        const float gg = alpha * g[k] + oma * d * d;
        g[k] = gg;
        theta_out[k] = theta_in[k] - lr * d / sqrtf(gg + eps);
    }
}

// Counter-based normal deviates: splitmix64 of (seed, index) gives two
// 24-bit uniforms, Box-Muller turns them into one N(0,1) value.
__device__ __forceinline__ uint64_t splitmix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
__global__ __launch_bounds__(256) void init_normal_kernel(float *__restrict__ dst, size_t base, size_t n, float std,
                                                          uint64_t seed) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint64_t r = splitmix64(seed * 0xD1342543DE82EF95ull + (base + i));
    const float u1 = ((float)((r >> 40) & 0xFFFFFF) + 1.f) * (1.f / 16777216.f);   // (0, 1]
    const float u2 = (float)((r >> 8) & 0xFFFFFF) * (1.f / 16777216.f);             // [0, 1)
    dst[i] = std * sqrtf(-2.f * logf(u1)) * cosf(6.28318530717958647692f * u2);
}
__global__ __launch_bounds__(256) void fill_kernel(float *__restrict__ dst, size_t n, float v) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = v;
}

// ------------------------------------------------------------ host helpers --

// Event fences between the calls of a context.  A wait is skipped when the
// event was last recorded on the same stream (stream order already holds) or
// never recorded.
int fence_wait(hipStream_t s, hipEvent_t ev, bool set, hipStream_t where) {
    if (!set || where == s) return GA3C_OK;
    HIP_TRY(hipStreamWaitEvent(s, ev, 0));
    return GA3C_OK;
}
int wait_ready(ga3c_ctx *c, int i, hipStream_t s) { return fence_wait(s, c->ev_ready[i], c->ready_set[i], c->ready_stream[i]); }
int wait_readers(ga3c_ctx *c, int i, hipStream_t s) { return fence_wait(s, c->ev_readers[i], c->readers_set[i], c->readers_stream[i]); }
int mark_ready(ga3c_ctx *c, int i, hipStream_t s) {
    HIP_TRY(hipEventRecord(c->ev_ready[i], s));
    c->ready_set[i] = true; c->ready_stream[i] = s;
    return GA3C_OK;
}
int mark_readers(ga3c_ctx *c, int i, hipStream_t s) {
    HIP_TRY(hipEventRecord(c->ev_readers[i], s));
    c->readers_set[i] = true; c->readers_stream[i] = s;
    return GA3C_OK;
}
#define TRY(expr) do { int rc_ = (expr); if (rc_ != GA3C_OK) return rc_; } while (0)

// While one of these is alive and profiling is on, every kernel launched by this host thread carries an event pair
// of its own (launch.hpp), booked to the stage: the stage's time is the sum of its kernels' execution times.  Costs
// one branch when profiling is off.
struct ProfScope final : ga3c::LaunchTimer {
    Profiler *p; int sid;
    ProfScope(ga3c_ctx *c, hipStream_t, const char *name, double flop, double bytes) : p(c->prof), sid(-1) {
        if (!p || !p->on) { p = nullptr; return; }
        for (size_t i = 0; i < p->stages.size(); ++i) if (!strcmp(p->stages[i].name, name)) { sid = (int)i; break; }
        if (sid < 0) { p->stages.push_back({name, 0, 0.0, 0.0, 0.0}); sid = (int)p->stages.size() - 1; }
        p->stages[sid].calls += 1; p->stages[sid].flop += flop; p->stages[sid].bytes += bytes;
        ga3c::launch_timer = this;
    }
    bool next_events(hipEvent_t *start, hipEvent_t *stop) override {
        ProfRec r; r.stage = sid; r.a = r.b = nullptr;
        for (hipEvent_t *e : {&r.a, &r.b}) {
            if (!p->pool.empty()) { *e = p->pool.back(); p->pool.pop_back(); }
            else if (hipEventCreate(e) != hipSuccess) { *e = nullptr; }
        }
        if (!r.a || !r.b) {
            for (hipEvent_t e : {r.a, r.b}) if (e) p->pool.push_back(e);
            return false;
        }
        p->recs.push_back(r);
        *start = r.a; *stop = r.b;
        return true;
    }
    ~ProfScope() { if (p) ga3c::launch_timer = nullptr; }
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;
};
#define STAGE(name, flop, bytes) ProfScope prof_scope_(c, s, name, (double)(flop), (double)(bytes))

const char *const CONV_FWD[GA3C_MAX_CONV] = {"conv1_fwd", "conv2_fwd", "conv3_fwd", "conv4_fwd"};
const char *const CONV_WGRAD[GA3C_MAX_CONV] = {"conv1_wgrad", "conv2_wgrad", "conv3_wgrad", "conv4_wgrad"};
const char *const CONV_DGRAD[GA3C_MAX_CONV] = {"conv1_dgrad", "conv2_dgrad", "conv3_dgrad", "conv4_dgrad"};

inline unsigned blocks_for(size_t n, int per = 256) { return (unsigned)((n + per - 1) / per); }

// Number of k-chunks for a split-k product with `tiles` output tiles and a
// reduction of length K: enough blocks to fill 256 compute units a few times
// over, chunks a multiple of the k-tile and at least two k-tiles long.
inline void pick_split(int tiles, int K, int &nz, int &kchunk) {
    int want = (512 + tiles - 1) / tiles;
    int maxz = std::max(1, K / (2 * GEMM_BK));
    want = std::max(1, std::min(want, maxz));
    kchunk = (K + want - 1) / want;
    kchunk = (kchunk + GEMM_BK - 1) / GEMM_BK * GEMM_BK;
    nz = (K + kchunk - 1) / kchunk;
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// k-chunks for the XCD-partitioned dense product: a multiple of 8 chunks (one
// or more per XCD) when the reduction is long enough, about `target` blocks in
// all (fewer chunks mean fewer partial sums to write and add up again).
inline void pick_split_xcd(int tiles, int K, int &nz, int &kchunk, int target = 512) {
    int want = 8 * std::max(1, (target + 8 * tiles - 1) / (8 * tiles));
    const int maxz = std::max(1, K / (2 * GEMM_BK));
    if (want > maxz) want = maxz >= 8 ? maxz / 8 * 8 : maxz;
    kchunk = (K + want - 1) / want;
    kchunk = (kchunk + GEMM_BK - 1) / GEMM_BK * GEMM_BK;
    nz = (K + kchunk - 1) / kchunk;
}

int alloc_work(Work &w, const ga3c_ctx *c, int cap) {
    w.cap = cap;
    if (cap <= 0) return GA3C_OK;
    for (int l = 0; l < c->nconv; ++l)
        HIP_TRY(hipMalloc(&w.act[l], sizeof(float) * (size_t)cap * c->geom[l].OC * c->geom[l].OHW));
    HIP_TRY(hipMalloc(&w.h, sizeof(float) * (size_t)cap * c->F));
    HIP_TRY(hipMalloc(&w.zv, sizeof(float) * (size_t)cap * (c->A + 1)));
    return GA3C_OK;
}

void free_work(Work &w) {
    (void)hipFree(w.ws);
    for (int l = 0; l < GA3C_MAX_CONV; ++l) (void)hipFree(w.act[l]);
    (void)hipFree(w.h);
    (void)hipFree(w.zv);
}

// Tile shapes: output channels are few (16..64), pixels are many.
template <class P>
hipError_t launch_conv_like(const P &p, int nz, hipStream_t s, bool a_rows_unused = false) {
    (void)a_rows_unused;
    if (p.M <= 16) return launch_gemm<1, 4, 1, 4, false, true>(p, nz, s);   // 16 x 256
    if (p.M <= 32) return launch_gemm<2, 2, 1, 4, false, true>(p, nz, s);   // 32 x 128
    return launch_gemm<2, 2, 2, 2, false, true>(p, nz, s);                  // 64 x 64
}
inline int conv_like_tiles(int M, int N) {
    if (M <= 16) return cdiv(N, 256);
    if (M <= 32) return cdiv(N, 128);
    return cdiv(M, 64) * cdiv(N, 64);
}

// LDS the fused training heads kernel may ask for; larger heads fall back to the separate kernels.
constexpr size_t HEADS_TRAIN_MAX_LDS = 128 * 1024;
constexpr size_t HEADS_FWD_MAX_LDS = 160 * 1024;      // all of a compute unit's LDS

// A kernel may take more than 64 KB of dynamic LDS only after its limit has
// been raised; `set` remembers the largest size asked for so far.
static hipError_t allow_dynamic_lds(const void *kernel, size_t bytes, size_t &set) {
    if (bytes <= 64 * 1024 || bytes <= set) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) set = bytes;
    return e;
}

template <class SP>
inline bool spec_matches(const ConvGeom &g, bool byte_input) {
    return g.C == SP::C && g.H == SP::H && g.W == SP::W && g.OC == SP::OC && g.KS == SP::KS && g.S == SP::S &&
           byte_input == (sizeof(typename SP::TIn) == 1);
}
inline bool is_aligned16(const void *p) { return (((uintptr_t)p) & 15) == 0; }

// Things derived from parameter copy i, rebuilt on s after that copy was written there.
int refresh_derived(ga3c_ctx *c, int i, hipStream_t s) {
    if (c->cfrag[i]) {
        HIP_TRY(launch_conv12_filter_fragments(c->theta2[i] + c->off[0], c->theta2[i] + c->off[2], c->cfrag[i], s, c->rb));
        if (c->cfrag_dgrad)
            HIP_TRY(launch_conv_dgrad_filter_fragments<SpecS2>(c->theta2[i] + c->off[2], c->cfrag[i] + CFRAG_FWD_VECS, s));
    }
    if (c->lfrag[i]) {
        const float *w2 = c->theta2[i] + c->off[2], *w3 = c->theta2[i] + c->off[4];
        ga3c::launch(large_filter_fragments_kernel, dim3(LFRAG_B3), dim3(256), 0, s, w2, w3, c->lfrag[i]);
        HIP_TRY(hipGetLastError());
    }
    return GA3C_OK;
}

// Forward pass of `B` frames into `w`; heads outputs to the optional pointers.
int forward(ga3c_ctx *c, int which, Work &w, const uint8_t *frames, int B, bool keep_zv, float *logits, float *values,
            float *probs, const float *uniforms, int32_t *actions, hipStream_t s, bool with_heads = true) {
    const float *th = c->theta2[which];
    const int nb = 2 * c->nconv;
    int first = 0;
    if (c->fast && c->small_predict && c->ticket && c->cfrag[which] && is_aligned16(frames) && !keep_zv && with_heads &&
        B <= SP_MAX_FRAMES && c->nconv == 2 && c->F == SP_FC && c->flat == SP_FLAT && c->off[nb] % 4 == 0 &&
        sizeof(float) * heads_lds_floats(c->F, c->A) <= SP_HEADS_MAX) {
        // a handful of frames: one launch for the whole network
        static bool attr_set = false;
        if (!attr_set) {
            const void *ks[8] = {(const void *)predict_small_kernel<false, 32>, (const void *)predict_small_kernel<true, 32>,
                                 (const void *)predict_small_kernel<false, 16>, (const void *)predict_small_kernel<true, 16>,
                                 (const void *)predict_small_kernel<false, 8>, (const void *)predict_small_kernel<true, 8>,
                                 (const void *)predict_small_kernel<false, 4>, (const void *)predict_small_kernel<true, 4>};
            for (const void *k : ks) HIP_TRY(hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C12_LDS_BYTES));
            attr_set = true;
        }
        const ConvGeom &g0 = c->geom[0], &g1 = c->geom[1];
        STAGE("predict_small", 2.0 * B * (g0.OHW * g0.OC * g0.K + g1.OHW * g1.OC * g1.K + (double)c->flat * c->F + c->F * (c->A + 1)),
              (double)B * g0.CHW + 4.0 * c->flat * c->F);
        const int slices = B <= 8 ? 32 : B <= 16 ? 16 : B <= 32 ? 8 : 4;
        const dim3 grid(B * slices), block(512);
#define GA3C_SP_LAUNCH(ONE_, SL_)                                                                                              \
    ga3c::launch((predict_small_kernel<ONE_, SL_>), grid, block, C12_LDS_BYTES, s, frames, c->cfrag[which],             \
                       th + c->off[1], th + c->off[3], th + c->off[nb], th + c->off[nb + 1], w.h, c->ticket, c->A,            \
                       th + c->off[nb + 2], th + c->off[nb + 3], th + c->off[nb + 4], th + c->off[nb + 5], logits, values,    \
                       probs, uniforms, actions, 1.f / 255.f, c->rb)
#define GA3C_SP_PICK(ONE_)                                                                                                     \
    do {                                                                                                                       \
        if (slices == 32) GA3C_SP_LAUNCH(ONE_, 32); else if (slices == 16) GA3C_SP_LAUNCH(ONE_, 16);                           \
        else if (slices == 8) GA3C_SP_LAUNCH(ONE_, 8); else GA3C_SP_LAUNCH(ONE_, 4);                                           \
    } while (0)
        if (c->rb) GA3C_SP_PICK(true); else GA3C_SP_PICK(false);
#undef GA3C_SP_PICK
#undef GA3C_SP_LAUNCH
        HIP_TRY(hipGetLastError());
        return GA3C_OK;
    }
    if (c->fast && c->cfrag[which] && is_aligned16(frames)) {
        // small net: both convolution layers in one kernel; layer-1 activations go to HBM only when training
        const ConvGeom &g0 = c->geom[0], &g1 = c->geom[1];
        STAGE("conv12_fwd", 2.0 * B * (g0.OHW * g0.OC * g0.K + g1.OHW * g1.OC * g1.K),
              (double)B * (g0.CHW + (keep_zv ? 4.0 * g0.OC * g0.OHW : 0.0) + 4.0 * g1.OC * g1.OHW));
        HIP_TRY(launch_conv12_fused_fwd(frames, c->cfrag[which], th + c->off[1], th + c->off[3],
                                        keep_zv ? w.act[0] : nullptr, w.act[1], B, 1.f / 255.f, s, c->rb));
        first = 2;
    }
    for (int l = first; l < c->nconv; ++l) {
        const ConvGeom &g = c->geom[l];
        STAGE(CONV_FWD[l], 2.0 * B * g.OHW * g.OC * g.K, (double)B * ((l == 0 ? 1.0 : 4.0) * g.CHW + 4.0 * g.OC * g.OHW));
        const float *wl = th + c->off[2 * l], *bl = th + c->off[2 * l + 1];
        const void *xin = l == 0 ? (const void *)frames : (const void *)w.act[l - 1];
        if (c->fast && is_aligned16(wl) && is_aligned16(xin)) {
            if (spec_matches<SpecS1>(g, l == 0)) {
                HIP_TRY(launch_conv1_bf16x3_fwd<16>((const uint8_t *)xin, wl, bl, w.act[l], B, 1.f / 255.f, s, c->rb));
                continue;
            }
            if (spec_matches<SpecL1>(g, l == 0)) {
                HIP_TRY(launch_conv1_bf16x3_fwd<32>((const uint8_t *)xin, wl, bl, w.act[l], B, 1.f / 255.f, s, c->rb));
                continue;
            }
            if (spec_matches<SpecS2>(g, l == 0)) {
                HIP_TRY(launch_conv2_bf16x6_fwd((const float *)xin, wl, bl, w.act[l], B, s, c->rb));
                continue;
            }
            if (spec_matches<SpecL2>(g, l == 0)) {      // the frame as split bf16 planes in LDS: one block per CU
                HIP_TRY((launch_conv_fwd_bf16x6<SpecL2, 4>((const float *)xin, wl, bl, w.act[l], B, s, 256, c->rb,
                                                           c->lfrag[which] && l == 1 ? c->lfrag[which] + LFRAG_FWD2 : nullptr)));
                continue;
            }
            if (spec_matches<SpecL3>(g, l == 0)) {
                HIP_TRY((launch_conv_fwd_bf16x6<SpecL3, 4>((const float *)xin, wl, bl, w.act[l], B, s, 256, c->rb,
                                                           c->lfrag[which] && l == 2 ? c->lfrag[which] + LFRAG_FWD3 : nullptr)));
                continue;
            }
        }
        if (l == 0) {
            ConvFwdP<uint8_t> p; p.rb = c->rb;
            p.M = g.OC; p.N = B * g.OHW; p.K = g.K; p.g = g;
            p.x = frames; p.w = th + c->off[0]; p.bias = th + c->off[1];
            p.y = w.act[0]; p.scale = 1.f / 255.f;
            HIP_TRY(launch_conv_like(p, 1, s));
        } else {
            ConvFwdP<float> p; p.rb = c->rb;
            p.M = g.OC; p.N = B * g.OHW; p.K = g.K; p.g = g;
            p.x = w.act[l - 1]; p.w = th + c->off[2 * l]; p.bias = th + c->off[2 * l + 1];
            p.y = w.act[l]; p.scale = 1.f;
            HIP_TRY(launch_conv_like(p, 1, s));
        }
    }
    const float *fc_ws = nullptr;
    int fc_nz = 1;
    {   // fully connected: h[b][o] = max(0, b[o] + sum_i x[b][i] Wfc[o][i])
        const float *x = w.act[c->nconv - 1];
        const float *wfc = th + c->off[nb];
        STAGE("fc_fwd", 2.0 * B * c->F * c->flat, 0);
        int nz, kchunk;
        if (c->fast && dense_operand_ok(x, c->flat, c->flat) && dense_operand_ok(wfc, c->flat, c->flat)) {
            pick_split_xcd(cdiv(B, 64) * cdiv(c->F, 64), c->flat, nz, kchunk);
            DenseGemmArgs p{}; p.rb = c->rb;
            p.M = B; p.N = c->F; p.K = c->flat; p.kchunk = kchunk; p.nz = nz;
            p.A = x; p.lda = c->flat; p.B = wfc; p.ldb = c->flat;
            p.C = w.ws; p.ldc = c->F; p.aux = nullptr;
            if ((size_t)nz * B * c->F > w.ws_floats) return fail(GA3C_EINVAL, "internal: split-k workspace too small (fc)");
            HIP_TRY((launch_dense_gemm_bf16x6<2, 2, 2, 2, false, false, DG_PARTIAL>(p, DG_SPLIT_Z, s)));
            fc_ws = w.ws; fc_nz = nz;
        } else {
            pick_split(cdiv(B, 64) * cdiv(c->F, 64), c->flat, nz, kchunk);
            GemmP<EPI_PARTIAL, false> p; p.rb = c->rb;
            p.M = B; p.N = c->F; p.K = c->flat; p.kchunk = kchunk;
            p.A = x; p.sAm = c->flat; p.sAk = 1;
            p.B = wfc; p.sBn = c->flat; p.sBk = 1;
            p.C = w.ws; p.ldc = c->F; p.aux = nullptr;
            if ((size_t)nz * B * c->F > w.ws_floats) return fail(GA3C_EINVAL, "internal: split-k workspace too small (fc)");
            HIP_TRY((launch_gemm<2, 2, 2, 2, false, false>(p, nz, s)));
            fc_ws = w.ws; fc_nz = nz;
        }
    }
    w.fc_ws = fc_ws; w.fc_nz = fc_nz;
    if (!with_heads) return GA3C_OK;          // the caller finishes the fc layer and the heads itself
    const size_t hf_lds = sizeof(float) * heads_lds_floats(c->F, c->A);
    static size_t hf_lds_set = 0;
    HIP_TRY(allow_dynamic_lds((const void *)heads_fwd_kernel, hf_lds, hf_lds_set));
    STAGE("heads_fwd", 2.0 * B * c->F * (c->A + 1), 4.0 * (fc_nz + 1) * B * c->F);
    ga3c::launch(heads_fwd_kernel, dim3(cdiv(B, 4)), dim3(256), hf_lds, s, fc_ws, fc_nz,
                       th + c->off[nb + 1], w.h, B, c->F, c->A, th + c->off[nb + 2],
                       th + c->off[nb + 3], th + c->off[nb + 4], th + c->off[nb + 5],
                       keep_zv ? w.zv : nullptr, logits, values, probs, uniforms, actions, c->rb);
    HIP_TRY(hipGetLastError());
    return GA3C_OK;
}

// Floats of split-k workspace a call on up to `cap` frames can need.
size_t workspace_floats(const ga3c_ctx *c, int cap, bool training) {
    size_t need = 0;
    for (int B = 1; B <= cap; ++B) {        // fc forward: depends on the batch
        int nz, kc;
        pick_split(cdiv(B, 64) * cdiv(c->F, 64), c->flat, nz, kc);
        need = std::max(need, (size_t)nz * B * c->F);
        pick_split_xcd(cdiv(B, 64) * cdiv(c->F, 64), c->flat, nz, kc);
        need = std::max(need, (size_t)nz * B * c->F);
    }
    const int B = cap;
    if (training && B > 0) {       // every weight gradient has a region of its own (rounded up to 64 floats)
        size_t sum = 0;
        auto add = [&](size_t floats) { sum += (floats + 63) / 64 * 64; };
        int nz, kc;
        for (int l = 0; l < c->nconv; ++l) {
            const ConvGeom &g = c->geom[l];
            pick_split(conv_like_tiles(g.OC, g.K + 1), B * g.OHW, nz, kc);
            add((size_t)std::max(nz, std::min(B, 512)) * g.OC * (g.K + 1));      // generic or frame-resident kernel
        }
        int nz2;
        pick_split(cdiv(c->F, 64) * cdiv(c->flat + 1, 64), B, nz, kc);
        pick_split_xcd(cdiv(c->F, 64) * cdiv(c->flat, 64), B, nz2, kc, 256);
        add((size_t)std::max(nz, nz2) * c->F * (c->flat + 1));
        pick_split(conv_like_tiles(c->A + 1, c->F + 1), B, nz, kc);
        add((size_t)std::max(nz, cdiv(B, HD_FRAMES)) * (c->A + 1) * (c->F + 1));
        need = (need + 63) / 64 * 64 + sum;      // the regions follow the fc partial sums
    }
    return need;
}

}  // namespace

// Host-only part of setting up a context: layer geometry, parameter offsets, counts.  Touches no device memory.
// On a layer that does not fit its input, returns GA3C_EINVAL with c->nconv set to that layer's index.
static int init_shape(ga3c_ctx *c, const ga3c_net_desc *d) {
    c->rb = d->math;
    c->desc = *d;
    c->nconv = d->n_conv; c->F = d->fc_units; c->A = d->n_actions;
    int C = d->in_c, H = d->in_h, W = d->in_w;
    int64_t pos = 0; int no = 0;
    for (int l = 0; l < c->nconv; ++l) {
        const int oc = d->conv[l].oc, ks = d->conv[l].k, st = d->conv[l].stride;
        if (oc < 1 || ks < 1 || st < 1 || ks > H || ks > W) { c->nconv = l; return GA3C_EINVAL; }
        ConvGeom &g = c->geom[l];
        g.C = C; g.H = H; g.W = W; g.OC = oc; g.KS = ks; g.S = st;
        g.OH = (H - ks) / st + 1; g.OW = (W - ks) / st + 1;
        g.K = C * ks * ks; g.OHW = g.OH * g.OW; g.CHW = C * H * W;
        g.dOHW = FastDiv(g.OHW); g.dOW = FastDiv(g.OW);
        g.koff = nullptr;
        c->off[no++] = pos; pos += (int64_t)oc * g.K;
        c->off[no++] = pos; pos += oc;
        C = oc; H = g.OH; W = g.OW;
    }
    c->flat = C * H * W;
    c->off[no++] = pos; pos += (int64_t)c->flat * c->F;
    c->off[no++] = pos; pos += c->F;
    c->off[no++] = pos; pos += (int64_t)c->A * c->F;
    c->off[no++] = pos; pos += c->A;
    c->off[no++] = pos; pos += c->F;
    c->off[no++] = pos; pos += 1;
    c->off[no++] = pos;
    c->noff = no; c->P = (size_t)pos;
    return GA3C_OK;
}

// ------------------------------------------------------------------ C ABI ---

extern "C" int ga3c_create(const ga3c_net_desc *d, int max_predict_batch, int max_train_frames, ga3c_ctx **out) {
    if (out) *out = nullptr;
    if (!d || !out) return fail(GA3C_EINVAL, "ga3c_create: null argument");
    if (d->n_conv < 1 || d->n_conv > GA3C_MAX_CONV) return fail(GA3C_EINVAL, "ga3c_create: n_conv must be 1..4");
    if (d->n_actions < 1 || d->n_actions > GA3C_MAX_ACTIONS)
        return fail(GA3C_EINVAL, "ga3c_create: n_actions must be 1..%d", GA3C_MAX_ACTIONS);
    if (d->in_c < 1 || d->in_h < 1 || d->in_w < 1 || d->fc_units < 1) return fail(GA3C_EINVAL, "ga3c_create: bad sizes");
    if (d->math != 0 && d->math != 1) return fail(GA3C_EINVAL, "ga3c_create: math must be 0 (fp32) or 1 (bfloat16 operands)");
    if (max_predict_batch < 0 || max_train_frames < 0) return fail(GA3C_EINVAL, "ga3c_create: negative capacity");
    if ((size_t)heads_lds_floats(d->fc_units, d->n_actions) * sizeof(float) > HEADS_FWD_MAX_LDS)
        return fail(GA3C_EINVAL, "ga3c_create: (n_actions + 5) * (fc_units + 16) must not exceed 40960");

    ga3c_ctx *c = new (std::nothrow) ga3c_ctx();
    if (!c) return fail(GA3C_ENOMEM, "ga3c_create: host allocation failed");
    memset((void *)c, 0, sizeof(*c));
    c->prof = new (std::nothrow) Profiler();
    c->fast = true;
    c->small_predict = true;
    c->max_pred = max_predict_batch; c->max_train = max_train_frames;

    if (init_shape(c, d) != GA3C_OK) {
        const int l = c->nconv;      // init_shape leaves the index of the offending layer here
        delete c->prof;
        delete c;
        return fail(GA3C_EINVAL, "ga3c_create: conv layer %d does not fit its input", l);
    }
    // 32-bit index limits of the kernels
    const int maxB = std::max(max_predict_batch, max_train_frames);
    for (int l = 0; l < c->nconv; ++l)
        if ((double)maxB * std::max(c->geom[l].OHW, c->geom[l].H * c->geom[l].W) >= 2.0e9) {
            delete c->prof;
            delete c;
            return fail(GA3C_EINVAL, "ga3c_create: capacity too large for 32-bit pixel indices");
        }

    int rc = GA3C_OK;
    auto guard = [&](int r) { if (r != GA3C_OK && rc == GA3C_OK) rc = r; return r == GA3C_OK; };
    auto dmalloc = [&](void **p, size_t bytes) -> int {
        HIP_TRY(hipMalloc(p, bytes ? bytes : 16));
        return GA3C_OK;
    };
    // filter-tap offset tables
    for (int l = 0; l < c->nconv && rc == GA3C_OK; ++l) {
        ConvGeom &g = c->geom[l];
        const int n = (g.K + 3) / 4 * 4;
        std::vector<int> t(n, 0);
        for (int cc = 0; cc < g.C; ++cc)
            for (int u = 0; u < g.KS; ++u)
                for (int v = 0; v < g.KS; ++v) t[(cc * g.KS + u) * g.KS + v] = cc * g.H * g.W + u * g.W + v;
        if (!guard(dmalloc((void **)&c->koff[l], sizeof(int) * n))) break;
        hipError_t e = hipMemcpy(c->koff[l], t.data(), sizeof(int) * n, hipMemcpyHostToDevice);
        if (e != hipSuccess) { guard(fail(GA3C_EHIP, "hipMemcpy: %s", hipGetErrorString(e))); break; }
        g.koff = c->koff[l];
    }
    for (int i = 0; i < 2 && rc == GA3C_OK; ++i) {
        guard(dmalloc((void **)&c->theta2[i], sizeof(float) * c->P));
        if (rc == GA3C_OK && hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming) != hipSuccess)
            guard(fail(GA3C_EHIP, "hipEventCreate failed"));
        if (rc == GA3C_OK && hipEventCreateWithFlags(&c->ev_readers[i], hipEventDisableTiming) != hipSuccess)
            guard(fail(GA3C_EHIP, "hipEventCreate failed"));
    }
    if (rc == GA3C_OK) guard(dmalloc((void **)&c->g, sizeof(float) * c->P));
    if (rc == GA3C_OK) guard(dmalloc((void **)&c->grad, sizeof(float) * c->P));
    if (rc == GA3C_OK) {
        hipError_t e = hipMemset(c->theta2[0], 0, sizeof(float) * c->P);
        if (e == hipSuccess) e = hipMemset(c->theta2[1], 0, sizeof(float) * c->P);
        if (e == hipSuccess) e = hipMemset(c->g, 0, sizeof(float) * c->P);
        if (e == hipSuccess) e = hipMemset(c->grad, 0, sizeof(float) * c->P);
        if (e != hipSuccess) guard(fail(GA3C_EHIP, "hipMemset: %s", hipGetErrorString(e)));
    }
    if (rc == GA3C_OK && c->nconv >= 2 && spec_matches<SpecS1>(c->geom[0], true) && spec_matches<SpecS2>(c->geom[1], false) &&
        c->off[0] % 4 == 0 && c->off[2] % 4 == 0) {
        c->cfrag_dgrad = true;
        for (int i = 0; i < 2 && rc == GA3C_OK; ++i) {
            guard(dmalloc((void **)&c->cfrag[i], sizeof(u32x4) * CFRAG_VECS));
            if (rc == GA3C_OK) guard(refresh_derived(c, i, nullptr));
        }
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->ticket, sizeof(int) * SP_MAX_FRAMES * SP_TICKET_PITCH));
        if (rc == GA3C_OK) {
            const hipError_t e = hipMemset(c->ticket, 0, sizeof(int) * SP_MAX_FRAMES * SP_TICKET_PITCH);
            if (e != hipSuccess) guard(fail(GA3C_EHIP, "hipMemset: %s", hipGetErrorString(e)));
        }
    }
    if (rc == GA3C_OK && c->nconv == 3 && spec_matches<SpecL2>(c->geom[1], false) && spec_matches<SpecL3>(c->geom[2], false) &&
        c->off[2] % 4 == 0 && c->off[4] % 4 == 0) {
        for (int i = 0; i < 2 && rc == GA3C_OK; ++i) {
            guard(dmalloc((void **)&c->lfrag[i], sizeof(u32x4) * LFRAG_VECS));
            if (rc == GA3C_OK) guard(refresh_derived(c, i, nullptr));
        }
    }
    if (rc == GA3C_OK) guard(alloc_work(c->pred, c, max_predict_batch));
    if (rc == GA3C_OK) guard(alloc_work(c->train, c, max_train_frames));
    if (rc == GA3C_OK && max_train_frames > 0) {
        const size_t B = (size_t)max_train_frames;
        for (int l = 0; l < c->nconv && rc == GA3C_OK; ++l)
            guard(dmalloc((void **)&c->dact[l], sizeof(float) * B * c->geom[l].OC * c->geom[l].OHW));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->dh, sizeof(float) * B * c->F));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->dzv, sizeof(float) * B * (c->A + 1)));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->R, sizeof(float) * B));
        c->max_norm_parts = (int)(c->P / 4 + 24 * MAX_REDUCE_SEGS);   // a reduce block covers at least 4 outputs
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->partials, sizeof(float) * (c->max_norm_parts + 3 * (B / HD_FRAMES + 1))));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->colpart, sizeof(float) * (B / HD_FRAMES + 1) * c->F));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->scale, sizeof(float)));
        if (rc == GA3C_OK) guard(dmalloc((void **)&c->stats, sizeof(ga3c_train_stats)));
        if (rc == GA3C_OK) {
            hipError_t e = hipMemset(c->stats, 0, sizeof(ga3c_train_stats));
            if (e != hipSuccess) guard(fail(GA3C_EHIP, "hipMemset: %s", hipGetErrorString(e)));
        }
    }
    if (rc == GA3C_OK) {
        c->pred.ws_floats = workspace_floats(c, max_predict_batch, false);
        guard(dmalloc((void **)&c->pred.ws, sizeof(float) * c->pred.ws_floats));
    }
    if (rc == GA3C_OK) {
        c->train.ws_floats = workspace_floats(c, max_train_frames, true);
        guard(dmalloc((void **)&c->train.ws, sizeof(float) * c->train.ws_floats));
    }
    if (rc != GA3C_OK) {
        char keep[sizeof(g_err)];
        memcpy(keep, g_err, sizeof(keep));
        ga3c_destroy(c);
        memcpy(g_err, keep, sizeof(keep));
        return rc;
    }
    *out = c;
    return GA3C_OK;
}

extern "C" int ga3c_destroy(ga3c_ctx *c) {
    if (!c) return GA3C_OK;
    (void)hipDeviceSynchronize();
    for (int l = 0; l < GA3C_MAX_CONV; ++l) { (void)hipFree(c->koff[l]); (void)hipFree(c->dact[l]); }
    for (int i = 0; i < 2; ++i) {
        (void)hipFree(c->theta2[i]);
        if (c->ev_ready[i]) (void)hipEventDestroy(c->ev_ready[i]);
        if (c->ev_readers[i]) (void)hipEventDestroy(c->ev_readers[i]);
    }
    (void)hipFree(c->g); (void)hipFree(c->grad);
    (void)hipFree(c->cfrag[0]); (void)hipFree(c->cfrag[1]); (void)hipFree(c->ticket); (void)hipFree(c->lfrag[0]); (void)hipFree(c->lfrag[1]);
    free_work(c->pred); free_work(c->train);
    (void)hipFree(c->dh); (void)hipFree(c->dzv); (void)hipFree(c->R);
    (void)hipFree(c->partials); (void)hipFree(c->colpart); (void)hipFree(c->scale); (void)hipFree(c->stats);
    if (c->prof) {
        for (ProfRec &r : c->prof->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (hipEvent_t e : c->prof->pool) (void)hipEventDestroy(e);
        delete c->prof;
    }
    delete c;
    return GA3C_OK;
}

extern "C" size_t ga3c_params_count(const ga3c_ctx *c) { return c ? c->P : 0; }

extern "C" int ga3c_params_offsets(const ga3c_ctx *c, int64_t *off, int cap) {
    if (!c || !off || cap < c->noff) return fail(GA3C_EINVAL, "ga3c_params_offsets: null argument or cap too small");
    for (int i = 0; i < c->noff; ++i) off[i] = c->off[i];
    return c->noff;
}

extern "C" int ga3c_params_init(ga3c_ctx *c, uint64_t seed, void *stream) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_params_init: null context");
    hipStream_t s = (hipStream_t)stream;
    float *theta = c->theta2[c->cur];
    // wait for whoever wrote or still reads this copy
    TRY(wait_ready(c, c->cur, s));
    TRY(wait_readers(c, c->cur, s));
    ga3c::launch(fill_kernel, dim3(blocks_for(c->P)), dim3(256), 0, s, theta, c->P, 0.f);
    ga3c::launch(fill_kernel, dim3(blocks_for(c->P)), dim3(256), 0, s, c->g, c->P, 0.f);
    HIP_TRY(hipGetLastError());
    const int nb = 2 * c->nconv;
    // weight tensors and their fan-in; biases stay zero
    struct { int64_t off; size_t n; int fan_in; } t[GA3C_MAX_CONV + 3];
    int nt = 0;
    for (int l = 0; l < c->nconv; ++l) t[nt++] = {c->off[2 * l], (size_t)c->geom[l].OC * c->geom[l].K, c->geom[l].K};
    t[nt++] = {c->off[nb], (size_t)c->flat * c->F, c->flat};
    t[nt++] = {c->off[nb + 2], (size_t)c->A * c->F, c->F};
    t[nt++] = {c->off[nb + 4], (size_t)c->F, c->F};
    for (int i = 0; i < nt; ++i) {
        ga3c::launch(init_normal_kernel, dim3(blocks_for(t[i].n)), dim3(256), 0, s, theta + t[i].off,
                           (size_t)t[i].off, t[i].n, sqrtf(2.f / (float)t[i].fan_in), seed);
        HIP_TRY(hipGetLastError());
    }
    TRY(refresh_derived(c, c->cur, s));
    TRY(mark_ready(c, c->cur, s));
    return GA3C_OK;
}

static float *select_buffer(ga3c_ctx *c, int which) {
    return which == 0 ? c->theta2[c->cur] : which == 1 ? c->g : which == 2 ? c->grad : nullptr;
}

extern "C" int ga3c_params_get(ga3c_ctx *c, int which, float *dst, size_t n, void *stream) {
    if (!c || !dst) return fail(GA3C_EINVAL, "ga3c_params_get: null argument");
    float *src = select_buffer(c, which);
    if (!src || n != c->P) return fail(GA3C_EINVAL, "ga3c_params_get: which must be 0..2 and n the parameter count");
    TRY(wait_ready(c, c->cur, (hipStream_t)stream));
    HIP_TRY(hipMemcpyAsync(dst, src, sizeof(float) * n, hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return GA3C_OK;
}

extern "C" int ga3c_params_set(ga3c_ctx *c, int which, const float *src, size_t n, void *stream) {
    if (!c || !src) return fail(GA3C_EINVAL, "ga3c_params_set: null argument");
    if ((which != 0 && which != 1) || n != c->P)
        return fail(GA3C_EINVAL, "ga3c_params_set: which must be 0 or 1 and n the parameter count");
    hipStream_t s = (hipStream_t)stream;
    TRY(wait_ready(c, c->cur, s));
    TRY(wait_readers(c, c->cur, s));
    HIP_TRY(hipMemcpyAsync(select_buffer(c, which), src, sizeof(float) * n, hipMemcpyDeviceToDevice, s));
    if (which == 0) {
        TRY(refresh_derived(c, c->cur, s));
        TRY(mark_ready(c, c->cur, s));
    }
    return GA3C_OK;
}

extern "C" int ga3c_predict(ga3c_ctx *c, const uint8_t *frames, int B, const float *uniforms, float *logits,
                            float *values, float *probs, int32_t *actions, void *stream) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_predict: null context");
    if (B < 0 || B > c->max_pred) return fail(GA3C_EINVAL, "ga3c_predict: B = %d outside [0, %d]", B, c->max_pred);
    if (B == 0) return GA3C_OK;
    if (!frames) return fail(GA3C_EINVAL, "ga3c_predict: null frames");
    if (actions && !uniforms) return fail(GA3C_EINVAL, "ga3c_predict: actions requested without uniforms");
    hipStream_t s = (hipStream_t)stream;
    const int cur = c->cur;
    TRY(wait_ready(c, cur, s));
    const int rc = forward(c, cur, c->pred, frames, B, false, logits, values, probs, uniforms, actions, s);
    if (rc != GA3C_OK) return rc;
    TRY(mark_readers(c, cur, s));
    return GA3C_OK;
}

// One update on B frames.  seg_start == nullptr: N segments of T frames each
// (B = N*T); otherwise N segments of unequal length, T = 1.
static int train_step_impl(ga3c_ctx *c, const uint8_t *frames, const int32_t *actions, const float *rewards,
                           const uint8_t *dones, const float *bootstrap, const int32_t *seg_start, int N, int T, int B,
                           const ga3c_hparams *hp, ga3c_train_stats *stats, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    Work &w = c->train;
    const int nb = 2 * c->nconv, A = c->A, F = c->F;
    c->last_frames = B;

    const int cur = c->cur;
    const float *th = c->theta2[cur];
    TRY(wait_ready(c, cur, s));
    // One kernel finishes the fc layer, runs the heads, the loss and the heads' backward pass, if its LDS fits.
    const size_t ht_lds = sizeof(float) * (size_t)heads_train_lds_floats(F, A);
    const bool fused_heads = c->fast && ht_lds <= HEADS_TRAIN_MAX_LDS && HD_FRAMES * (A + 1) <= 256;      // a thread per (frame, output)
    int rc = forward(c, cur, w, frames, B, true, nullptr, nullptr, nullptr, nullptr, nullptr, s, !fused_heads);
    if (rc != GA3C_OK) return rc;

    const int nloss = fused_heads ? cdiv(B, HD_FRAMES) : cdiv(B, LOSS_THREADS);
    float *losspart = c->partials + c->max_norm_parts;
    if (!fused_heads) {
        STAGE("returns_loss", 0, 4.0 * B * (2 * (A + 1) + 4));
        ga3c::launch(returns_loss_kernel, dim3(nloss), dim3(LOSS_THREADS), sizeof(float) * LOSS_THREADS * (A + 1), s, w.zv, actions, rewards, dones,
                           bootstrap, seg_start, N, T, B, A, hp->gamma, hp->beta, hp->value_coef, hp->log_eps, c->R, c->dzv, losspart);
        HIP_TRY(hipGetLastError());
    }

    const float *Wp = th + c->off[nb + 2], *Wv = th + c->off[nb + 4];
    int nz, kchunk;
    // Every weight gradient leaves its partial sums in a region of its own; one kernel adds them all up at the end.
    ReduceArgs red;
    red.nseg = 0; red.normpart = c->partials;
    // the fused heads kernel still reads the fc partial sums, which sit at the start of the workspace
    size_t ws_used = fused_heads ? ((size_t)w.fc_nz * B * F + 63) / 64 * 64 : 0;
    int red_blocks = 0;
    double red_bytes = 0;
    auto region = [&](size_t floats) -> float * {
        float *r = ws_used + floats <= w.ws_floats ? w.ws + ws_used : nullptr;
        ws_used += (floats + 63) / 64 * 64;
        return r;
    };
    bool seg_overflow = false;
    auto add_seg = [&](const float *ws, int nz_, int M, int Ncols, int r0, int rows, float *gW, float *gb, int bias_col) {
        if (red.nseg >= MAX_REDUCE_SEGS) { seg_overflow = true; return; }
        ReduceSeg &g = red.seg[red.nseg++];
        g.ws = ws; g.nz = nz_; g.M = M; g.N = Ncols; g.r0 = r0; g.rows = rows; g.gW = gW; g.gb = gb; g.bias_col = bias_col;
        int zg = 1;
        while (zg < 64 && zg * 16 < nz_) zg *= 2;      // at most two rounds of eight loads per thread
        g.zg = zg; g.first_block = red_blocks;
        g.vec = ((size_t)r0 * Ncols) % 4 == 0 && ((size_t)M * Ncols) % 4 == 0 && (uintptr_t)ws % 16 == 0;
        const size_t per_block = (size_t)(256 / zg) * (g.vec ? 4 : 1);
        const int nblk = (int)(((size_t)rows * Ncols + per_block - 1) / per_block);
        g.per_xcd = (nblk + 7) / 8;
        red_blocks += 8 * g.per_xcd;
        red_bytes += 4.0 * (nz_ + 1) * rows * Ncols;
    };
    const size_t hd_lds = sizeof(float) * (A + 1) * (F + HD_FRAMES);      // heads_dgrad_kernel's LDS
    static size_t hd_lds_set = 0;
    if (fused_heads) {
        const int nblk = cdiv(B, HD_FRAMES);
        float *part = region((size_t)nblk * (A + 1) * (F + 1));
        if (!part) return fail(GA3C_EINVAL, "internal: split-k workspace too small (heads)");
        static size_t ht_lds_set = 0;
        HIP_TRY(allow_dynamic_lds((const void *)heads_train_kernel, ht_lds, ht_lds_set));
        STAGE("heads_train", 6.0 * B * (A + 1) * F, 4.0 * (w.fc_nz + 1) * B * F);
        ga3c::launch(heads_train_kernel, dim3(nblk), dim3(256), ht_lds, s, w.fc_ws, w.fc_nz, th + c->off[nb + 1], B, F, A, Wp,
                           th + c->off[nb + 3], Wv, th + c->off[nb + 5], actions, rewards, dones, bootstrap, seg_start, N, T, hp->gamma, hp->beta,
                           hp->value_coef, hp->log_eps, w.h, w.zv, c->R, c->dzv, c->dh, c->colpart, part, losspart, c->rb);
        HIP_TRY(hipGetLastError());
        add_seg(part, nblk, A + 1, F + 1, 0, A, c->grad + c->off[nb + 2], c->grad + c->off[nb + 3], 1);
        add_seg(part, nblk, A + 1, F + 1, A, 1, c->grad + c->off[nb + 4], c->grad + c->off[nb + 5], 1);
    } else if (c->fast) {   // heads: input gradient and, per block of frames, the block's share of the weight and bias gradients
        const int nblk = cdiv(B, HD_FRAMES);
        float *part = region((size_t)nblk * (A + 1) * (F + 1));
        if (!part) return fail(GA3C_EINVAL, "internal: split-k workspace too small (heads)");
        STAGE("heads_bwd", 4.0 * B * (A + 1) * F, 0);
        HIP_TRY(allow_dynamic_lds((const void *)heads_dgrad_kernel, hd_lds, hd_lds_set));
        ga3c::launch(heads_dgrad_kernel, dim3(nblk), dim3(256), hd_lds, s, c->dzv, w.h, Wp, Wv, B,
                           F, A, c->dh, c->colpart, part, c->rb);
        HIP_TRY(hipGetLastError());
        add_seg(part, nblk, A + 1, F + 1, 0, A, c->grad + c->off[nb + 2], c->grad + c->off[nb + 3], 1);
        add_seg(part, nblk, A + 1, F + 1, A, 1, c->grad + c->off[nb + 4], c->grad + c->off[nb + 5], 1);
    } else {   // heads: weight and bias gradients as a product, then the input gradient
        GemmP<EPI_PARTIAL, true> p; p.rb = c->rb;
        p.M = A + 1; p.N = F + 1; p.K = B;
        pick_split(conv_like_tiles(p.M, p.N), B, nz, kchunk);
        p.kchunk = kchunk;
        p.A = c->dzv; p.sAm = 1; p.sAk = A + 1;
        p.B = w.h; p.sBn = 1; p.sBk = F;
        p.C = region((size_t)nz * p.M * p.N); p.ldc = 0; p.aux = nullptr;
        if (!p.C) return fail(GA3C_EINVAL, "internal: split-k workspace too small (heads)");
        {
            STAGE("heads_wgrad", 2.0 * B * (A + 1) * F, 0);
            HIP_TRY(launch_conv_like(p, nz, s));
        }
        add_seg(p.C, nz, A + 1, F + 1, 0, A, c->grad + c->off[nb + 2], c->grad + c->off[nb + 3], 1);
        add_seg(p.C, nz, A + 1, F + 1, A, 1, c->grad + c->off[nb + 4], c->grad + c->off[nb + 5], 1);
        STAGE("heads_dgrad", 2.0 * B * (A + 1) * F, 0);
        HIP_TRY(allow_dynamic_lds((const void *)heads_dgrad_kernel, hd_lds, hd_lds_set));
        ga3c::launch(heads_dgrad_kernel, dim3(cdiv(B, HD_FRAMES)), dim3(256), hd_lds, s, c->dzv, w.h, Wp, Wv, B,
                           F, A, c->dh, c->colpart, (float *)nullptr, c->rb);
        HIP_TRY(hipGetLastError());
    }
    const float *xfc = w.act[c->nconv - 1];
    const float *wfc = th + c->off[nb];
    const bool fc_dense = c->fast && dense_operand_ok(c->dh, F, F) && dense_operand_ok(xfc, c->flat, c->flat) &&
                          dense_operand_ok(wfc, c->flat, c->flat);
    if (fc_dense) {   // fc weight gradient: D[o][i] = sum_b dh[b][o] x[b][i]; bias from the column sums of dh
        pick_split_xcd(cdiv(F, 64) * cdiv(c->flat, 64), B, nz, kchunk, 256);
        DenseGemmArgs p{}; p.rb = c->rb;
        p.M = F; p.N = c->flat; p.K = B; p.kchunk = kchunk; p.nz = nz;
        p.A = c->dh; p.lda = F; p.B = xfc; p.ldb = c->flat;
        p.C = region((size_t)nz * p.M * p.N); p.ldc = 0; p.aux = nullptr;
        if (!p.C) return fail(GA3C_EINVAL, "internal: split-k workspace too small (fc wgrad)");
        {
            STAGE("fc_wgrad", 2.0 * B * F * c->flat, 0);
            HIP_TRY((launch_dense_gemm_bf16x6<2, 2, 2, 2, true, true, DG_PARTIAL>(p, DG_SPLIT_Z, s)));
        }
        add_seg(p.C, nz, p.M, p.N, 0, p.M, c->grad + c->off[nb], nullptr, 0);
        add_seg(c->colpart, cdiv(B, HD_FRAMES), 1, F, 0, 1, c->grad + c->off[nb + 1], nullptr, 0);
    } else {   // general shapes: one more column of ones yields the bias gradient
        GemmP<EPI_PARTIAL, true> p; p.rb = c->rb;
        p.M = F; p.N = c->flat + 1; p.K = B;
        pick_split(cdiv(p.M, 64) * cdiv(p.N, 64), B, nz, kchunk);
        p.kchunk = kchunk;
        p.A = c->dh; p.sAm = 1; p.sAk = F;
        p.B = xfc; p.sBn = 1; p.sBk = c->flat;
        p.C = region((size_t)nz * p.M * p.N); p.ldc = 0; p.aux = nullptr;
        if (!p.C) return fail(GA3C_EINVAL, "internal: split-k workspace too small (fc wgrad)");
        {
            STAGE("fc_wgrad", 2.0 * B * F * c->flat, 0);
            HIP_TRY((launch_gemm<2, 2, 2, 2, true, true>(p, nz, s)));
        }
        add_seg(p.C, nz, p.M, p.N, 0, p.M, c->grad + c->off[nb], c->grad + c->off[nb + 1], 1);
    }
    {   // fc input gradient, masked by the ReLU of the last conv layer
        STAGE("fc_dgrad", 2.0 * B * F * c->flat, 0);
        if (fc_dense) {
            DenseGemmArgs p{}; p.rb = c->rb;
            p.M = B; p.N = c->flat; p.K = F; p.kchunk = (F + GEMM_BK - 1) / GEMM_BK * GEMM_BK; p.nz = 1;
            p.A = c->dh; p.lda = F; p.B = wfc; p.ldb = c->flat;
            p.C = c->dact[c->nconv - 1]; p.ldc = c->flat; p.aux = xfc;
            HIP_TRY((launch_dense_gemm_bf16x6<4, 2, 2, 2, false, true, DG_MASK>(p, DG_SPLIT_N, s)));
        } else {
            GemmP<EPI_MASK, false> p; p.rb = c->rb;
            p.M = B; p.N = c->flat; p.K = F; p.kchunk = (F + GEMM_BK - 1) / GEMM_BK * GEMM_BK;
            p.A = c->dh; p.sAm = F; p.sAk = 1;
            p.B = wfc; p.sBn = 1; p.sBk = c->flat;
            p.C = c->dact[c->nconv - 1]; p.ldc = c->flat; p.aux = xfc;
            HIP_TRY((launch_gemm<2, 2, 2, 2, false, true>(p, 1, s)));
        }
    }
    for (int l = c->nconv - 1; l >= 0; --l) {
        const ConvGeom &g = c->geom[l];
        // weight + bias gradient
        {
            const void *xin = l == 0 ? (const void *)frames : (const void *)w.act[l - 1];
            const bool ok = c->fast && is_aligned16(xin);
            const int kind = !ok ? 0 : (spec_matches<SpecS1>(g, l == 0) && is_aligned16(c->dact[l])) ? 1
                                     : (spec_matches<SpecL1>(g, l == 0) && is_aligned16(c->dact[l])) ? 2
                                     : spec_matches<SpecS2>(g, l == 0) ? (is_aligned16(c->dact[l]) ? 6 : 3)
                                     : spec_matches<SpecL2>(g, l == 0) ? (is_aligned16(c->dact[l]) ? 7 : 4)
                                     : spec_matches<SpecL3>(g, l == 0) ? (is_aligned16(c->dact[l]) ? 8 : 5)
                                     : (spec_matches<SpecP2>(g, l == 0) && is_aligned16(c->dact[l])) ? 9 : 0;
            if (kind == 1) nz = conv1_bf16x3_wgrad_blocks(B);
            else if (kind == 2) nz = conv1_bf16x3_wgrad_blocks(B);
            else if (kind == 3) nz = conv_wgrad_frame_blocks<SpecS2>(B);
            else if (kind == 4) nz = conv_wgrad_frame_blocks<SpecL2>(B);
            else if (kind == 5) nz = conv_wgrad_frame_blocks<SpecL3>(B);
            else if (kind == 6) nz = conv_wgrad_bf16x6_blocks<SpecS2>(B);
            else if (kind == 7) nz = conv_wgrad_bf16x6_blocks<SpecL2>(B);
            else if (kind == 8) nz = conv_wgrad_s1_bf16x6_blocks<SpecL3>(B);
            else if (kind == 9) nz = conv_wgrad_bf16x6_blocks<SpecP2>(B);
            else pick_split(conv_like_tiles(g.OC, g.K + 1), B * g.OHW, nz, kchunk);
            float *part = region((size_t)nz * g.OC * (g.K + 1));
            if (!part) return fail(GA3C_EINVAL, "internal: split-k workspace too small (conv)");
            STAGE(CONV_WGRAD[l], 2.0 * B * g.OHW * g.OC * g.K, (double)B * ((l == 0 ? 1.0 : 4.0) * g.CHW + 4.0 * g.OC * g.OHW));
            if (kind == 1) {
                HIP_TRY(launch_conv1_bf16x3_wgrad((const uint8_t *)xin, c->dact[l], part, B, 1.f / 255.f, s, c->rb));
            } else if (kind == 2) {
                HIP_TRY(launch_conv1_bf16x3_wgrad<32>((const uint8_t *)xin, c->dact[l], part, B, 1.f / 255.f, s, c->rb));
            } else if (kind == 3) {
                HIP_TRY((launch_conv_wgrad_frame<SpecS2, 1, 8>)((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (kind == 4) {
                HIP_TRY((launch_conv_wgrad_frame<SpecL2, 4, 8>)((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (kind == 5) {
                HIP_TRY((launch_conv_wgrad_frame<SpecL3, 3>)((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (kind == 6) {
                HIP_TRY(launch_conv_wgrad_bf16x6<SpecS2>((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (kind == 7) {
                HIP_TRY((launch_conv_wgrad_bf16x6<SpecL2, 32>((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb)));
            } else if (kind == 8) {
                HIP_TRY(launch_conv_wgrad_s1_bf16x6<SpecL3>((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (kind == 9) {
                HIP_TRY(launch_conv_wgrad_bf16x6<SpecP2>((const float *)xin, c->dact[l], part, B, 1.f, s, c->rb));
            } else if (l == 0) {
                ConvWgradP<uint8_t> p; p.rb = c->rb;
                p.M = g.OC; p.N = g.K + 1; p.K = B * g.OHW; p.kchunk = kchunk; p.g = g;
                p.x = frames; p.dy = c->dact[0]; p.ws = part; p.scale = 1.f / 255.f;
                HIP_TRY(launch_conv_like(p, nz, s));
            } else {
                ConvWgradP<float> p; p.rb = c->rb;
                p.M = g.OC; p.N = g.K + 1; p.K = B * g.OHW; p.kchunk = kchunk; p.g = g;
                p.x = w.act[l - 1]; p.dy = c->dact[l]; p.ws = part; p.scale = 1.f;
                HIP_TRY(launch_conv_like(p, nz, s));
            }
            add_seg(part, nz, g.OC, g.K + 1, 0, g.OC, c->grad + c->off[2 * l], c->grad + c->off[2 * l + 1], 1);
        }
        if (l == 0) break;   // the input is data: no gradient needed
        // input gradient
        // bytes: dY in, the layer's input (for the ReLU mask) in, dX out
        STAGE(CONV_DGRAD[l], 2.0 * B * g.OHW * g.OC * g.K, 4.0 * B * (g.OC * g.OHW + 2.0 * g.C * g.H * g.W));
        if (c->fast && spec_matches<SpecS2>(g, false) && is_aligned16(th + c->off[2 * l])) {
            // the fragments of the copy being trained on, when the context keeps them (it does when conv1 is the small net's too)
            const u32x4 *wfrag = c->cfrag[cur] && c->cfrag_dgrad ? c->cfrag[cur] + CFRAG_FWD_VECS : nullptr;
            HIP_TRY(launch_conv_dgrad_bf16x6<SpecS2>(c->dact[l], th + c->off[2 * l], w.act[l - 1], c->dact[l - 1], B, s, 512, c->rb, wfrag));
            continue;
        }
        if (c->fast && spec_matches<SpecL2>(g, false) && is_aligned16(th + c->off[2 * l])) {
            HIP_TRY(launch_conv_dgrad_bf16x6<SpecL2>(c->dact[l], th + c->off[2 * l], w.act[l - 1], c->dact[l - 1], B, s, 512, c->rb,
                                                     c->lfrag[cur] && l == 1 ? c->lfrag[cur] + LFRAG_DGRAD2 : nullptr));
            continue;
        }
        if (c->fast && spec_matches<SpecP2>(g, false) && is_aligned16(th + c->off[2 * l])) {
            HIP_TRY(launch_conv_dgrad_bf16x6<SpecP2>(c->dact[l], th + c->off[2 * l], w.act[l - 1], c->dact[l - 1], B, s, 512, c->rb));
            continue;
        }
        if (c->fast && spec_matches<SpecL3>(g, false)) {
            HIP_TRY((launch_conv_dgrad_s1_bf16x6<SpecL3, 4>(c->dact[l], th + c->off[2 * l], w.act[l - 1], c->dact[l - 1], B, s, 256, c->rb,
                                                            c->lfrag[cur] && l == 2 ? c->lfrag[cur] + LFRAG_DGRAD3 : nullptr)));
            continue;
        }
        // general shapes: one launch per stride phase
        for (int ry = 0; ry < g.S; ++ry)
            for (int rx = 0; rx < g.S; ++rx) {
                ConvDgradP p; p.rb = c->rb;
                p.g = g; p.ry = ry; p.rx = rx;
                p.nH = ry < g.H ? (g.H - ry + g.S - 1) / g.S : 0;
                p.nW = rx < g.W ? (g.W - rx + g.S - 1) / g.S : 0;
                if (p.nH == 0 || p.nW == 0) continue;
                p.TA = (g.KS + g.S - 1) / g.S; p.TB = p.TA;
                p.dNHW = FastDiv(p.nH * p.nW); p.dNW = FastDiv(p.nW);
                p.dTAB = FastDiv(p.TA * p.TB); p.dTB = FastDiv(p.TB);
                p.M = g.C; p.N = B * p.nH * p.nW; p.K = g.OC * p.TA * p.TB;
                p.w = th + c->off[2 * l]; p.dy = c->dact[l]; p.xmask = w.act[l - 1]; p.dx = c->dact[l - 1];
                HIP_TRY(launch_conv_like(p, 1, s));
            }
    }
    // all partial gradients -> gradient and its squared norm; then clip scale and stats; then RMSProp
    if (seg_overflow) return fail(GA3C_EINVAL, "internal: more partial-gradient segments than the reduction kernel takes");
    if (red_blocks > c->max_norm_parts) return fail(GA3C_EINVAL, "internal: too many reduce blocks");
    {
        STAGE("wgrad_reduce", 0, red_bytes);
        ga3c::launch(reduce_all_kernel, dim3(red_blocks), dim3(256), 0, s, red);
        HIP_TRY(hipGetLastError());
    }
    STAGE("rmsprop", 8.0 * c->P, 20.0 * c->P);
    // one float4 per thread at these sizes; the clip factor and the statistics are formed in the kernel's prologue
    const unsigned rb = std::min<unsigned>(blocks_for(c->P / 4 + 1), 2048u);
    // the copy about to be overwritten may still be read by predictions issued before the last update
    TRY(wait_readers(c, cur ^ 1, s));
    RmsClip ca;
    ca.normpart = c->partials; ca.nnorm = red_blocks; ca.losspart = losspart; ca.nloss = nloss; ca.clip = hp->clip_norm;
    ca.scale_out = c->scale; ca.own = c->stats; ca.user = stats;
    ga3c::launch((rmsprop_kernel<0, 1>), dim3(rb), dim3(256), 0, s, th, c->theta2[cur ^ 1], c->g, c->grad, c->P, (const float *)nullptr,
                       1.f, hp->lr, hp->rms_decay, hp->rms_eps, c->cfrag[cur ^ 1], (unsigned)c->off[0], (unsigned)c->off[2], c->rb, ca);
    HIP_TRY(hipGetLastError());
    if (c->lfrag[cur ^ 1]) TRY(refresh_derived(c, cur ^ 1, s));      // the larger net's fragments follow the new parameters
    TRY(mark_ready(c, cur ^ 1, s));
    c->cur = cur ^ 1;        // calls enqueued from now on see the new parameters
    return GA3C_OK;
}

extern "C" int ga3c_train_step(ga3c_ctx *c, const uint8_t *frames, const int32_t *actions, const float *rewards,
                               const uint8_t *dones, const float *bootstrap, int N, int T, const ga3c_hparams *hp,
                               ga3c_train_stats *stats, void *stream) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_train_step: null context");
    if (N < 0 || T < 0) return fail(GA3C_EINVAL, "ga3c_train_step: negative N or T");
    const long long BL = (long long)N * T;
    if (BL > c->max_train) return fail(GA3C_EINVAL, "ga3c_train_step: N*T = %lld above capacity %d", BL, c->max_train);
    if (BL == 0) return GA3C_OK;
    if (!frames || !actions || !rewards || !dones || !hp) return fail(GA3C_EINVAL, "ga3c_train_step: null argument");
    return train_step_impl(c, frames, actions, rewards, dones, bootstrap, nullptr, N, T, (int)BL, hp, stats, stream);
}

extern "C" int ga3c_train_step_ragged(ga3c_ctx *c, const uint8_t *frames, const int32_t *actions, const float *rewards,
                                      const uint8_t *dones, const int32_t *seg_start, const float *bootstrap, int N,
                                      int n_frames, const ga3c_hparams *hp, ga3c_train_stats *stats, void *stream) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_train_step_ragged: null context");
    if (N < 0 || n_frames < 0) return fail(GA3C_EINVAL, "ga3c_train_step_ragged: negative N or n_frames");
    if (n_frames > c->max_train)
        return fail(GA3C_EINVAL, "ga3c_train_step_ragged: %d frames above capacity %d", n_frames, c->max_train);
    if (n_frames == 0) return GA3C_OK;
    if (N == 0) return fail(GA3C_EINVAL, "ga3c_train_step_ragged: frames without a segment");
    if (!frames || !actions || !rewards || !dones || !seg_start || !hp)
        return fail(GA3C_EINVAL, "ga3c_train_step_ragged: null argument");
    return train_step_impl(c, frames, actions, rewards, dones, bootstrap, seg_start, N, 1, n_frames, hp, stats, stream);
}

extern "C" int ga3c_train_debug_get(ga3c_ctx *c, int which, float *dst, size_t n, void *stream) {
    if (!c || !dst) return fail(GA3C_EINVAL, "ga3c_train_debug_get: null argument");
    const size_t B = (size_t)c->last_frames;
    const float *src = nullptr;
    size_t cap = 0;
    if (which == 0) { src = c->R; cap = B; }
    else if (which == 3) { src = c->dzv; cap = B * (c->A + 1); }
    else if (which == 1 || which == 2) { src = c->train.zv; cap = B * (c->A + 1); }
    else if (which >= 4 && which < 4 + c->nconv) { src = c->train.act[which - 4]; cap = B * c->geom[which - 4].OC * c->geom[which - 4].OHW; }
    else if (which == 8) { src = c->train.h; cap = B * c->F; }
    else if (which == 9) { src = c->dh; cap = B * c->F; }
    else if (which >= 10 && which < 10 + c->nconv) { src = c->dact[which - 10]; cap = B * c->geom[which - 10].OC * c->geom[which - 10].OHW; }
    if (!src || n > (which == 1 ? B * c->A : which == 2 ? B : cap))
        return fail(GA3C_EINVAL, "ga3c_train_debug_get: bad selector or size");
    hipStream_t s = (hipStream_t)stream;
    if (which == 1 || which == 2) {
        // strided copy out of the packed [B][A+1] buffer
        const size_t rows = which == 1 ? n / c->A : n;
        HIP_TRY(hipMemcpy2DAsync(dst, sizeof(float) * (which == 1 ? c->A : 1), src + (which == 2 ? c->A : 0),
                                 sizeof(float) * (c->A + 1), sizeof(float) * (which == 1 ? c->A : 1), rows,
                                 hipMemcpyDeviceToDevice, s));
        return GA3C_OK;
    }
    HIP_TRY(hipMemcpyAsync(dst, src, sizeof(float) * n, hipMemcpyDeviceToDevice, s));
    return GA3C_OK;
}

extern "C" int ga3c_rmsprop_flat(float *theta, float *g, const float *grad, size_t n, float scale, float lr,
                                 float rms_decay, float rms_eps, void *stream) {
    if (!theta || !g || !grad) return fail(GA3C_EINVAL, "ga3c_rmsprop_flat: null argument");
    if (n == 0) return GA3C_OK;
    if ((((uintptr_t)theta) | ((uintptr_t)g) | ((uintptr_t)grad)) & 15)
        return fail(GA3C_EINVAL, "ga3c_rmsprop_flat: buffers must be 16-byte aligned");
    // one tile of 1024 vectors per block (measured: 6.0 TB/s on 2^28 parameters, against 5.3 with 4096 blocks that
    // loop over tiles and 4.3 with one vector per thread and iteration).  Buffers far larger than the last-level
    // cache are streamed past the caches (non-temporal loads and stores: 5.5 -> 6.0 TB/s); smaller ones are not,
    // since whoever uses theta next finds it in the cache.
    const unsigned rb = (unsigned)std::min<size_t>(std::max<size_t>(n / 4096, 1), (size_t)1 << 20);
    const bool stream_past_caches = 20.0 * (double)n > 1.0e9;
    RmsClip none;
    memset(&none, 0, sizeof(none));
#define GA3C_RMS_LAUNCH(V)                                                                                               \
    ga3c::launch((rmsprop_kernel<V, 4>), dim3(rb), dim3(256), 0, (hipStream_t)stream, theta, theta, g, grad, n,         \
                       (const float *)nullptr, scale, lr, rms_decay, rms_eps, (u32x4 *)nullptr, 0u, 0u, 0, none)
    if (stream_past_caches) GA3C_RMS_LAUNCH(3); else GA3C_RMS_LAUNCH(0);
#undef GA3C_RMS_LAUNCH
    HIP_TRY(hipGetLastError());
    return GA3C_OK;
}

extern "C" int ga3c_profile_enable(ga3c_ctx *c, int on) {
    if (!c || !c->prof) return fail(GA3C_EINVAL, "ga3c_profile_enable: null context");
    c->prof->on = on != 0;
    return GA3C_OK;
}

extern "C" int ga3c_profile_read(ga3c_ctx *c, char *buf, size_t cap) {
    if (!c || !c->prof || !buf || cap == 0) return fail(GA3C_EINVAL, "ga3c_profile_read: null argument");
    Profiler *p = c->prof;
    for (ProfRec &r : p->recs) {
        HIP_TRY(hipEventSynchronize(r.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        p->stages[r.stage].ms += ms;
        p->pool.push_back(r.a); p->pool.push_back(r.b);
    }
    p->recs.clear();
    size_t pos = 0;
    buf[0] = 0;
    for (const ProfStage &st : p->stages) {
        int n = snprintf(buf + pos, cap - pos, "%s %ld %.6f %.6e %.6e\n", st.name, st.calls, st.ms, st.flop, st.bytes);
        if (n < 0 || (size_t)n >= cap - pos) return fail(GA3C_EINVAL, "ga3c_profile_read: buffer too small");
        pos += (size_t)n;
    }
    p->stages.clear();
    return GA3C_OK;
}

extern "C" int ga3c_use_generic_kernels(ga3c_ctx *c, int on) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_use_generic_kernels: null context");
    c->fast = on == 0;
    return GA3C_OK;
}

extern "C" int ga3c_get_desc(const ga3c_ctx *c, ga3c_net_desc *desc, int *max_predict_batch, int *max_train_frames) {
    if (!c) return fail(GA3C_EINVAL, "ga3c_get_desc: null context");
    if (desc) *desc = c->desc;
    if (max_predict_batch) *max_predict_batch = c->max_pred;
    if (max_train_frames) *max_train_frames = c->max_train;
    return GA3C_OK;
}

// ---------------------------------------------- prediction without allocation ---
//
// ga3c_predict_static: the prediction of the Sec. 3.2 network for callers that cannot allocate device memory.
// Everything ga3c_predict keeps in buffers that ga3c_create allocates (filter fragments, layer-2 activations, split-k
// partial sums of the fc layer, fc outputs, the one-launch path's tickets) lives in one file-scope device array here.
// Each GPU holds its own copy of the array; its address on a device is looked up once, with that device current,
// and kernels and copies only ever get that looked-up address.
namespace {
constexpr int STATIC_MAX_FRAMES = GA3C_STATIC_MAX_FRAMES;
constexpr int STATIC_MAX_SPLITS = 40;                                    // k-chunks of the fc product: 2592 / 64
constexpr size_t up256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t ST_FRAG_OFF = 0;
constexpr size_t ST_TICKET_OFF = ST_FRAG_OFF + up256(sizeof(u32x4) * 3 * C12_FRAG_SET);
constexpr size_t ST_H_OFF = ST_TICKET_OFF + up256(sizeof(int) * SP_MAX_FRAMES * SP_TICKET_PITCH);
constexpr size_t ST_Y2_OFF = ST_H_OFF + up256(sizeof(float) * STATIC_MAX_FRAMES * SP_FC);
constexpr size_t ST_WS_OFF = ST_Y2_OFF + up256(sizeof(float) * STATIC_MAX_FRAMES * SP_FLAT);
constexpr size_t ST_WS_FLOATS = (size_t)STATIC_MAX_SPLITS * STATIC_MAX_FRAMES * SP_FC;
constexpr size_t ST_BYTES = ST_WS_OFF + up256(sizeof(float) * ST_WS_FLOATS);
static_assert(ST_BYTES <= (size_t)GA3C_STATIC_SCRATCH_BYTES, "the header promises a smaller array");

constexpr int ST_MAX_DEVICES = 64;
unsigned char *g_static_ptr[ST_MAX_DEVICES];      // device address of the array on each GPU, nullptr until looked up
std::mutex g_static_mutex;
}  // namespace

static __device__ __align__(256) unsigned char ga3c_static_scratch[ST_BYTES];

// Address of the array on the current device (looked up on the first call there).
static int static_scratch(unsigned char **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= ST_MAX_DEVICES) return fail(GA3C_EINVAL, "ga3c_predict_static: device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(ga3c_static_scratch)));
        if (!p) return fail(GA3C_EHIP, "ga3c_predict_static: the scratch array has no address on device %d", dev);
        g_static_ptr[dev] = (unsigned char *)p;
    }
    *out = g_static_ptr[dev];
    return GA3C_OK;
}

extern "C" int ga3c_predict_static(int n_actions, int math, const float *theta, const uint8_t *frames, int B,
                                   const float *uniforms, float *logits, float *values, float *probs, int32_t *actions,
                                   void *stream) {
    if (n_actions < 1 || n_actions > GA3C_MAX_ACTIONS)
        return fail(GA3C_EINVAL, "ga3c_predict_static: n_actions must be 1..%d", GA3C_MAX_ACTIONS);
    if (math != 0 && math != 1) return fail(GA3C_EINVAL, "ga3c_predict_static: math must be 0 or 1");
    if (B < 0 || B > STATIC_MAX_FRAMES)
        return fail(GA3C_EINVAL, "ga3c_predict_static: B = %d outside [0, %d] (the scratch array is sized for %d frames)", B,
                    STATIC_MAX_FRAMES, STATIC_MAX_FRAMES);
    if (B == 0) return GA3C_OK;
    if (!theta || !frames) return fail(GA3C_EINVAL, "ga3c_predict_static: null theta or frames");
    if (actions && !uniforms) return fail(GA3C_EINVAL, "ga3c_predict_static: actions requested without uniforms");
    if (!is_aligned16(theta) || !is_aligned16(frames))
        return fail(GA3C_EINVAL, "ga3c_predict_static: theta and frames must be 16-byte aligned");

    // a context on the stack that owns nothing: shape and offsets on the host, every buffer inside the array
    ga3c_ctx c;
    memset((void *)&c, 0, sizeof(c));
    ga3c_net_desc d;
    memset(&d, 0, sizeof(d));
    d.in_c = 4; d.in_h = 84; d.in_w = 84; d.n_conv = 2;
    d.conv[0].oc = 16; d.conv[0].k = 8; d.conv[0].stride = 4;
    d.conv[1].oc = 32; d.conv[1].k = 4; d.conv[1].stride = 2;
    d.fc_units = SP_FC; d.n_actions = n_actions; d.math = math;
    TRY(init_shape(&c, &d));
    if (c.flat != SP_FLAT || c.off[2] % 4 != 0 || c.off[4] % 4 != 0)
        return fail(GA3C_EINVAL, "ga3c_predict_static: internal: unexpected layout");
    unsigned char *base = nullptr;
    TRY(static_scratch(&base));
    c.fast = true; c.small_predict = true; c.max_pred = STATIC_MAX_FRAMES;
    c.theta2[0] = const_cast<float *>(theta);
    c.cfrag[0] = (u32x4 *)(base + ST_FRAG_OFF);
    c.ticket = (int *)(base + ST_TICKET_OFF);
    c.pred.cap = STATIC_MAX_FRAMES;
    c.pred.h = (float *)(base + ST_H_OFF);
    c.pred.act[1] = (float *)(base + ST_Y2_OFF);
    c.pred.ws = (float *)(base + ST_WS_OFF);
    c.pred.ws_floats = ST_WS_FLOATS;
    hipStream_t s = (hipStream_t)stream;
    // the filters as split MFMA fragments, from the caller's parameters (a context does this when they change)
    TRY(refresh_derived(&c, 0, s));
    return forward(&c, 0, c.pred, frames, B, false, logits, values, probs, uniforms, actions, s);
}
