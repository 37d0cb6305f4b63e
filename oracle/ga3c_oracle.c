/*
 * fp64 CPU oracle for the GA3C hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library computes:
 * the batched policy/value CNN forward pass and one A3C update (n-step
 * returns, advantage, policy + entropy + value loss, backward by the chain
 * rule, global-norm clip, non-centred RMSProp).  It is used by the tests,
 * the smoke check and the cpu_baseline leg of the benchmark, and by nothing
 * on the product path.  It shares no code, header or table with the HIP
 * library.
 *
 * Citations are to the paper (arXiv 1611.06256):
 *   Sec. 3.2           network shape; rectifier after each hidden layer;
 *                      softmax policy head and linear value head
 *   Eq. 1              policy objective  log pi(a|s) (R - V) + beta H(pi)
 *   text after Eq. 1   n-step return R_t = sum_i gamma^i r_{t+i} + gamma^k V
 *   Eq. 2              value cost (R - V)^2
 *   Eq. 3              RMSProp  g = a g + (1-a) d^2 ; th -= eta d / sqrt(g+eps)
 *   Eq. 5              epsilon-stabilised log(pi+eps), H with log(pi+eps)
 *   Sec. 5.3           gradients are SUMMED over the training batch
 *
 * Everything is double precision, NCHW, naive loops.  Convolutions are VALID
 * cross-correlations.  OpenMP is used only as "parallel for" over frames or
 * over output rows; no loop is blocked, fused or reordered.
 *
 * Flat parameter order (shared convention with any caller, stated here in
 * full so this file stands alone): for each conv layer W[oc][ic][kh][kw] then
 * b[oc]; fc W[out][in] with in = c*H*W + h*W + w, fc b[out]; policy W[A][F],
 * policy b[A]; value W[F], value b.
 *
 * math = 1 is the reduced-precision variant of the same network: every
 * contraction (convolution, fully connected layer, heads, and each of their
 * weight, bias and input gradients) takes both of its operands rounded to
 * bfloat16 (8 significant bits, round to nearest even), multiplies them exactly
 * and accumulates without further rounding; everything else (biases, ReLU,
 * softmax, loss, clip, RMSProp, the stored parameters) is as for math = 0.  The
 * input bytes are exact in bfloat16, so layer 1 multiplies the raw bytes and
 * applies the 1/255 afterwards.  A bias gradient is the contraction of the
 * output gradient with a vector of ones, so its terms are rounded too.
 * The code for math = 0 is untouched by this: every use is behind `if (bf)`.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAX_CONV 4

typedef struct {
    int in_c, in_h, in_w;
    int n_conv;
    int oc[ORC_MAX_CONV], k[ORC_MAX_CONV], stride[ORC_MAX_CONV];
    int fc_units;
    int n_actions;
    int math;           /* 0: plain fp64; 1: operands of every contraction rounded to bfloat16 */
} orc_net;

typedef struct {
    double gamma, beta, value_coef, log_eps;
    double lr, rms_decay, rms_eps, clip_norm;
} orc_hparams;

typedef struct {
    double policy_loss, value_loss, entropy, grad_norm, clip_scale;
} orc_stats;

/* ---- shapes ------------------------------------------------------------ */

/* channels / height / width of the input of conv layer l (l == n_conv gives
 * the shape that is flattened into the fc layer). */
static void layer_in_shape(const orc_net *net, int l, int *c, int *h, int *w) {
    int cc = net->in_c, hh = net->in_h, ww = net->in_w;
    for (int i = 0; i < l; ++i) {
        hh = (hh - net->k[i]) / net->stride[i] + 1;
        ww = (ww - net->k[i]) / net->stride[i] + 1;
        cc = net->oc[i];
    }
    *c = cc; *h = hh; *w = ww;
}

/* Offsets of every tensor in the flat parameter vector.
 * off[2l], off[2l+1] = conv l weight, bias; then fcW, fcb, polW, polb, valW,
 * valb, and finally the total count.  Returns the number of entries. */
int orc_offsets(const orc_net *net, int64_t *off) {
    int64_t p = 0; int n = 0;
    for (int l = 0; l < net->n_conv; ++l) {
        int c, h, w; layer_in_shape(net, l, &c, &h, &w);
        off[n++] = p; p += (int64_t)net->oc[l] * c * net->k[l] * net->k[l];
        off[n++] = p; p += net->oc[l];
    }
    int c, h, w; layer_in_shape(net, net->n_conv, &c, &h, &w);
    int64_t flat = (int64_t)c * h * w;
    off[n++] = p; p += flat * net->fc_units;
    off[n++] = p; p += net->fc_units;
    off[n++] = p; p += (int64_t)net->n_actions * net->fc_units;
    off[n++] = p; p += net->n_actions;
    off[n++] = p; p += net->fc_units;
    off[n++] = p; p += 1;
    off[n++] = p;
    return n;
}

int64_t orc_param_count(const orc_net *net) {
    int64_t off[2 * ORC_MAX_CONV + 8];
    int n = orc_offsets(net, off);
    return off[n - 1];
}

/* Number of doubles of saved activations per frame: the scaled input, every
 * conv output (post-ReLU) and the fc output (post-ReLU), in that order. */
int64_t orc_acts_per_frame(const orc_net *net) {
    int64_t s = (int64_t)net->in_c * net->in_h * net->in_w;
    for (int l = 1; l <= net->n_conv; ++l) {
        int c, h, w; layer_in_shape(net, l, &c, &h, &w);
        s += (int64_t)c * h * w;
    }
    return s + net->fc_units;
}

/* ---- bfloat16 rounding (math = 1) --------------------------------------- */

/* Nearest bfloat16 (1 sign, 8 exponent, 7 fraction bits), ties to even. */
double orc_bf16_round(double v) {
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f;      /* inf, nan */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}
#define Q(v) orc_bf16_round(v)

/* ---- forward ----------------------------------------------------------- */

/* VALID cross-correlation + bias + ReLU for one frame (Sec. 3.2). */
/* bf != 0: operands rounded to bfloat16; xs = 255 for the first layer, whose
 * stored input x = byte / 255 enters the products as the byte itself. */
static void conv_relu(const double *x, int C, int H, int W,
                      const double *wt, const double *bias, int OC, int K, int S,
                      double *y, int bf, double xs) {
    int OH = (H - K) / S + 1, OW = (W - K) / S + 1;
    for (int o = 0; o < OC; ++o)
        for (int i = 0; i < OH; ++i)
            for (int j = 0; j < OW; ++j) {
                double acc = bias[o];
                if (!bf) {
                    for (int c = 0; c < C; ++c)
                        for (int u = 0; u < K; ++u)
                            for (int v = 0; v < K; ++v)
                                acc += wt[((o * C + c) * K + u) * K + v] *
                                       x[(c * H + i * S + u) * W + j * S + v];
                } else {
                    double dot = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int u = 0; u < K; ++u)
                            for (int v = 0; v < K; ++v)
                                dot += Q(wt[((o * C + c) * K + u) * K + v]) *
                                       Q(xs * x[(c * H + i * S + u) * W + j * S + v]);
                    acc += dot / xs;
                }
                y[(o * OH + i) * OW + j] = acc > 0.0 ? acc : 0.0;
            }
}

/* Fully connected layer of one frame: y[o] = bias[o] + sum_i W[o][i] x[i],
 * followed by the rectifier when relu != 0 (Sec. 3.2).  bf != 0: both operands
 * of every product rounded to bfloat16. */
static void dense(const double *x, int64_t I, const double *W, const double *bias, int O,
                  int relu, int bf, double *y) {
    for (int o = 0; o < O; ++o) {
        double acc = bias[o];
        if (!bf) for (int64_t i = 0; i < I; ++i) acc += W[o * I + i] * x[i];
        else for (int64_t i = 0; i < I; ++i) acc += Q(W[o * I + i]) * Q(x[i]);
        y[o] = (relu && !(acc > 0.0)) ? 0.0 : acc;
    }
}

static void softmax(const double *z, int A, double *p) {
    double m = z[0];
    for (int j = 1; j < A; ++j) if (z[j] > m) m = z[j];
    double s = 0.0;
    for (int j = 0; j < A; ++j) { p[j] = exp(z[j] - m); s += p[j]; }
    for (int j = 0; j < A; ++j) p[j] /= s;
}

/* Forward pass of one frame.  acts (may not be NULL) receives the saved
 * activations in the order of orc_acts_per_frame. */
static void forward_one(const orc_net *net, const double *theta, const int64_t *off,
                        const uint8_t *frame, double *acts,
                        double *logits, double *value, double *probs) {
    int64_t in_sz = (int64_t)net->in_c * net->in_h * net->in_w;
    double *x = acts;
    for (int64_t i = 0; i < in_sz; ++i) x[i] = frame[i] / 255.0;
    double *cur = x; int64_t cur_sz = in_sz;
    for (int l = 0; l < net->n_conv; ++l) {
        int c, h, w; layer_in_shape(net, l, &c, &h, &w);
        double *y = cur + cur_sz;
        conv_relu(cur, c, h, w, theta + off[2 * l], theta + off[2 * l + 1],
                  net->oc[l], net->k[l], net->stride[l], y, net->math, l == 0 ? 255.0 : 1.0);
        int c2, h2, w2; layer_in_shape(net, l + 1, &c2, &h2, &w2);
        cur = y; cur_sz = (int64_t)c2 * h2 * w2;
    }
    int nb = 2 * net->n_conv;
    const double *Wf = theta + off[nb], *bf = theta + off[nb + 1];
    const double *Wp = theta + off[nb + 2], *bp = theta + off[nb + 3];
    const double *Wv = theta + off[nb + 4], *bv = theta + off[nb + 5];
    int F = net->fc_units, A = net->n_actions;
    double *hfc = cur + cur_sz;
    const int q = net->math;
    dense(cur, cur_sz, Wf, bf, F, 1, q, hfc);
    dense(hfc, F, Wp, bp, A, 0, q, logits);
    dense(hfc, F, Wv, bv, 1, 0, q, value);
    if (probs) softmax(logits, A, probs);
}

/* Batched forward.  acts may be NULL (then a scratch frame buffer is used);
 * probs may be NULL. */
int orc_forward(const orc_net *net, const double *theta, const uint8_t *frames, int B,
                double *acts, double *logits, double *values, double *probs) {
    int64_t off[2 * ORC_MAX_CONV + 8]; orc_offsets(net, off);
    int64_t apf = orc_acts_per_frame(net);
    int64_t in_sz = (int64_t)net->in_c * net->in_h * net->in_w;
    int A = net->n_actions;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        double *a = acts ? acts + (int64_t)b * apf : (double *)malloc(sizeof(double) * apf);
        if (!a) { fail = 1; continue; }
        forward_one(net, theta, off, frames + (int64_t)b * in_sz, a,
                    logits + (int64_t)b * A, values + b, probs ? probs + (int64_t)b * A : NULL);
        if (!acts) free(a);
    }
    return fail ? -1 : 0;
}

/* Inverse-CDF sampling: the first action whose running sum of probabilities
 * exceeds u; the last action if none does (Sec. 4.1: the agent chooses
 * actions according to the policy). */
int orc_sample(const double *p, int A, double u) {
    double c = 0.0;
    for (int j = 0; j < A; ++j) { c += p[j]; if (c > u) return j; }
    return A - 1;
}

/* ---- returns (text after Eq. 1) ----------------------------------------- */

/* R[n][T] = bootstrap[n];  R[n][t] = r[n][t] + gamma (1 - done[n][t]) R[n][t+1].
 * A terminal at step t cuts the sum there, which is the k < t_max case. */
void orc_returns(const double *rewards, const uint8_t *dones, const double *bootstrap,
                 int N, int T, double gamma, double *R) {
    for (int n = 0; n < N; ++n) {
        double next = bootstrap ? bootstrap[n] : 0.0;
        for (int t = T - 1; t >= 0; --t) {
            double cont = dones[n * T + t] ? 0.0 : 1.0;
            next = rewards[n * T + t] + gamma * cont * next;
            R[n * T + t] = next;
        }
    }
}

/* The same for segments of unequal length laid end to end (Sec. 4.1: an agent
 * hands in its experiences after t_max actions or when its episode ends, so a
 * training batch also holds shorter segments).  Segment n is the frames
 * seg_start[n] .. seg_start[n+1]-1; the return after its last frame is
 * bootstrap[n]. */
void orc_returns_ragged(const double *rewards, const uint8_t *dones, const int32_t *seg_start,
                        const double *bootstrap, int N, double gamma, double *R) {
    for (int n = 0; n < N; ++n) {
        double next = bootstrap ? bootstrap[n] : 0.0;
        for (int i = seg_start[n + 1] - 1; i >= seg_start[n]; --i) {
            double cont = dones[i] ? 0.0 : 1.0;
            next = rewards[i] + gamma * cont * next;
            R[i] = next;
        }
    }
}

/* ---- loss and its gradient w.r.t. the two heads (Eq. 1, 2, 5) ----------- */

/* Minimised quantity per frame:
 *   L = -log(p[a] + e) * adv - beta * H + cv * (R - V)^2,
 *   H = -sum_j p_j log(p_j + e),  adv = R - V held constant in the first term.
 * Outputs dz[A] = dL/dz, *dv = dL/dV and the three loss pieces. */
static void loss_one(const double *z, double V, int a, double R, int A,
                     double beta, double cv, double e,
                     double *dz, double *dv, double *pl, double *vl, double *ent) {
    double p[64];
    softmax(z, A, p);
    double adv = R - V;
    double H = 0.0;
    for (int j = 0; j < A; ++j) if (p[j] + e > 0.0) H -= p[j] * log(p[j] + e);
    *pl = -log(p[a] + e) * adv;
    *vl = (R - V) * (R - V);
    *ent = H;
    /* dL/dp_k, then through the softmax Jacobian dp_k/dz_j = p_k (1[k=j] - p_j). */
    double dp[64], dot = 0.0;
    for (int k = 0; k < A; ++k) {
        double lg = (p[k] + e > 0.0) ? log(p[k] + e) : 0.0;
        double r = (p[k] + e > 0.0) ? p[k] / (p[k] + e) : 0.0;
        dp[k] = beta * (lg + r);
        if (k == a) dp[k] -= adv / (p[k] + e);
        dot += p[k] * dp[k];
    }
    for (int j = 0; j < A; ++j) dz[j] = p[j] * (dp[j] - dot);
    *dv = -2.0 * cv * (R - V);
}

void orc_loss_grad(const double *logits, const double *values, const int32_t *actions,
                   const double *R, int B, int A, double beta, double cv, double e,
                   double *dZ, double *dV, double *sums /* policy, value, entropy */) {
    sums[0] = sums[1] = sums[2] = 0.0;
    for (int b = 0; b < B; ++b) {
        double pl, vl, en;
        loss_one(logits + (int64_t)b * A, values[b], actions[b], R[b], A, beta, cv, e,
                 dZ + (int64_t)b * A, dV + b, &pl, &vl, &en);
        sums[0] += pl; sums[1] += vl; sums[2] += en;
    }
}

/* ---- backward ----------------------------------------------------------- */

/* Backward of a fully connected layer for one frame, by the chain rule:
 * dy[O] = dL/d(pre-activation).  ADDS gW[o][i] += dy[o] x[i], gb[o] += dy[o]
 * and, when dx is not NULL, dx[i] += sum_o dy[o] W[o][i] (rows in order).
 * bf != 0: operands of every product rounded to bfloat16; the bias gradient is
 * the product with ones, so its terms are the rounded dy. */
static void dense_backward(const double *x, int64_t I, const double *W, int O, const double *dy,
                           int bf, double *gW, double *gb, double *dx) {
    for (int o = 0; o < O; ++o) {
        if (!bf) {
            gb[o] += dy[o];
            for (int64_t i = 0; i < I; ++i) {
                gW[o * I + i] += dy[o] * x[i];
                if (dx) dx[i] += dy[o] * W[o * I + i];
            }
        } else {
            const double d = Q(dy[o]);
            gb[o] += d;
            for (int64_t i = 0; i < I; ++i) {
                gW[o * I + i] += d * Q(x[i]);
                if (dx) dx[i] += d * Q(W[o * I + i]);
            }
        }
    }
}

/* Backward of one convolution layer for one frame (the transposes of
 * conv_relu): y is the layer's output (post-ReLU, gives the mask), dy the
 * gradient w.r.t. that output before the mask is applied.  ADDS to gw and gb;
 * dx (may be NULL: the first layer's input is data) must be zero on entry and
 * receives the gradient w.r.t. the layer's input.  bf, xs as in conv_relu: the
 * first layer multiplies the raw bytes and divides by xs afterwards. */
static void conv_backward(const double *x, int C, int H, int W, const double *wt, int OC, int K, int S,
                          const double *y, const double *dy, int bf, double xs,
                          double *gw, double *gb, double *dx) {
    int OH = (H - K) / S + 1, OW = (W - K) / S + 1;
    for (int o = 0; o < OC; ++o)
        for (int i = 0; i < OH; ++i)
            for (int j = 0; j < OW; ++j) {
                int64_t yi = (o * OH + i) * OW + j;
                if (!(y[yi] > 0.0)) continue;          /* ReLU */
                double d = dy[yi];
                if (bf) {
                    d = Q(d);
                    gb[o] += d;
                    for (int cc = 0; cc < C; ++cc)
                        for (int u = 0; u < K; ++u)
                            for (int v = 0; v < K; ++v) {
                                int64_t wi = ((o * C + cc) * K + u) * K + v;
                                int64_t xi = (cc * H + i * S + u) * W + j * S + v;
                                gw[wi] += d * Q(xs * x[xi]) / xs;
                                if (dx) dx[xi] += d * Q(wt[wi]);
                            }
                    continue;
                }
                gb[o] += d;
                for (int cc = 0; cc < C; ++cc)
                    for (int u = 0; u < K; ++u)
                        for (int v = 0; v < K; ++v) {
                            int64_t wi = ((o * C + cc) * K + u) * K + v;
                            int64_t xi = (cc * H + i * S + u) * W + j * S + v;
                            gw[wi] += d * x[xi];
                            if (dx) dx[xi] += d * wt[wi];
                        }
            }
}

/* Gradient of one frame's loss w.r.t. all parameters, ADDED into grad.
 * dz[A], dv are dL/dlogits and dL/dvalue for this frame. */
static void backward_one(const orc_net *net, const double *theta, const int64_t *off,
                         const double *acts, const double *dz, double dv, double *grad,
                         double *scratch /* 2 * acts_per_frame doubles */) {
    int nb = 2 * net->n_conv;
    int F = net->fc_units, A = net->n_actions;
    int c, h, w; layer_in_shape(net, net->n_conv, &c, &h, &w);
    int64_t flat = (int64_t)c * h * w;
    /* locate saved activations */
    const double *layer_in[ORC_MAX_CONV + 1];
    int64_t pos = 0;
    for (int l = 0; l <= net->n_conv; ++l) {
        int cc, hh, ww; layer_in_shape(net, l, &cc, &hh, &ww);
        layer_in[l] = acts + pos; pos += (int64_t)cc * hh * ww;
    }
    const double *hfc = acts + pos;
    const int q = net->math;

    /* heads: policy rows first, then the value row */
    double *dh = scratch;                    /* F */
    for (int i = 0; i < F; ++i) dh[i] = 0.0;
    dense_backward(hfc, F, theta + off[nb + 2], A, dz, q, grad + off[nb + 2], grad + off[nb + 3], dh);
    dense_backward(hfc, F, theta + off[nb + 4], 1, &dv, q, grad + off[nb + 4], grad + off[nb + 5], dh);
    for (int i = 0; i < F; ++i) if (!(hfc[i] > 0.0)) dh[i] = 0.0;   /* ReLU of fc */

    /* fc */
    double *dcur = scratch + F;              /* gradient w.r.t. current layer input */
    for (int64_t i = 0; i < flat; ++i) dcur[i] = 0.0;
    dense_backward(layer_in[net->n_conv], flat, theta + off[nb], F, dh, q, grad + off[nb], grad + off[nb + 1], dcur);

    /* conv layers, last to first.  dcur holds dL/d(output of conv l) before
     * that layer's ReLU mask.  The two buffers swap roles per layer, so each
     * is as large as the largest conv output (2*acts_per_frame covers it). */
    int64_t maxsz = flat;
    for (int l = 1; l <= net->n_conv; ++l) {
        int cc, hh, ww; layer_in_shape(net, l, &cc, &hh, &ww);
        if ((int64_t)cc * hh * ww > maxsz) maxsz = (int64_t)cc * hh * ww;
    }
    double *dprev = dcur + maxsz;
    for (int l = net->n_conv - 1; l >= 0; --l) {
        int C, H, W; layer_in_shape(net, l, &C, &H, &W);
        int64_t in_sz = (int64_t)C * H * W;
        if (l > 0) for (int64_t i = 0; i < in_sz; ++i) dprev[i] = 0.0;
        /* the input of layer 0 is data: no gradient needed */
        conv_backward(layer_in[l], C, H, W, theta + off[2 * l], net->oc[l], net->k[l], net->stride[l],
                      layer_in[l + 1], dcur, q, l == 0 ? 255.0 : 1.0,
                      grad + off[2 * l], grad + off[2 * l + 1], l > 0 ? dprev : NULL);
        double *t = dcur; dcur = dprev; dprev = t;
    }
}

/* Sum over the batch (Sec. 5.3) of the per-frame parameter gradients.
 * grad is overwritten.  Frames are processed in index order by each thread
 * on a private accumulator; the accumulators are then added in thread order,
 * so the result does not depend on scheduling. */
int orc_backward(const orc_net *net, const double *theta, const double *acts, int B,
                 const double *dZ, const double *dV, double *grad) {
    int64_t off[2 * ORC_MAX_CONV + 8]; orc_offsets(net, off);
    int64_t P = orc_param_count(net), apf = orc_acts_per_frame(net);
    int A = net->n_actions;
    int nthreads = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    nthreads = omp_get_max_threads();
#endif
    if (nthreads > B) nthreads = B > 0 ? B : 1;
    double *priv = (double *)calloc((size_t)nthreads * P, sizeof(double));
    double *scr = (double *)malloc(sizeof(double) * (size_t)nthreads * 2 * apf);
    if (!priv || !scr) { free(priv); free(scr); return -1; }
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int t = 0; t < nthreads; ++t) {
        int b0 = (int)((int64_t)B * t / nthreads), b1 = (int)((int64_t)B * (t + 1) / nthreads);
        for (int b = b0; b < b1; ++b)
            backward_one(net, theta, off, acts + (int64_t)b * apf, dZ + (int64_t)b * A, dV[b],
                         priv + (int64_t)t * P, scr + (int64_t)t * 2 * apf);
    }
    for (int64_t i = 0; i < P; ++i) {
        double s = 0.0;
        for (int t = 0; t < nthreads; ++t) s += priv[(int64_t)t * P + i];
        grad[i] = s;
    }
    free(priv); free(scr);
    return 0;
}

/* ---- clip and RMSProp --------------------------------------------------- */

double orc_grad_norm(const double *grad, int64_t P) {
    double s = 0.0;
    for (int64_t i = 0; i < P; ++i) s += grad[i] * grad[i];
    return sqrt(s);
}

/* Global L2-norm rescale: s = min(1, c / ||grad||); c <= 0 disables. */
double orc_clip_scale(double norm, double c) {
    if (!(c > 0.0)) return 1.0;
    return norm > c ? c / norm : 1.0;
}

/* Eq. 3 with d = scale * grad; eps inside the root. */
void orc_rmsprop(double *theta, double *g, const double *grad, int64_t P,
                 double scale, double lr, double alpha, double eps) {
    for (int64_t i = 0; i < P; ++i) {
        double d = scale * grad[i];
        g[i] = alpha * g[i] + (1.0 - alpha) * d * d;
        theta[i] -= lr * d / sqrt(g[i] + eps);
    }
}

/* ---- one whole update --------------------------------------------------- */

/* frames [N][T][C][H][W]; actions, rewards, dones [N][T]; bootstrap [N] or NULL.
 * theta and g are updated in place; grad (P doubles) receives the unclipped
 * summed gradient.  Optional outputs (may be NULL): R_out [N*T], dZ_out
 * [N*T][A], dV_out [N*T], logits_out [N*T][A], values_out [N*T]. */
int orc_train_step(const orc_net *net, double *theta, double *g, double *grad,
                   const uint8_t *frames, const int32_t *actions, const double *rewards,
                   const uint8_t *dones, const double *bootstrap, int N, int T,
                   const orc_hparams *hp, orc_stats *stats,
                   double *R_out, double *dZ_out, double *dV_out,
                   double *logits_out, double *values_out) {
    int B = N * T, A = net->n_actions;
    int64_t P = orc_param_count(net), apf = orc_acts_per_frame(net);
    double *acts = (double *)malloc(sizeof(double) * (size_t)B * apf);
    double *logits = (double *)malloc(sizeof(double) * (size_t)B * A);
    double *values = (double *)malloc(sizeof(double) * B);
    double *R = (double *)malloc(sizeof(double) * B);
    double *dZ = (double *)malloc(sizeof(double) * (size_t)B * A);
    double *dV = (double *)malloc(sizeof(double) * B);
    int rc = -1;
    if (acts && logits && values && R && dZ && dV) {
        double sums[3];
        rc = orc_forward(net, theta, frames, B, acts, logits, values, NULL);
        if (rc == 0) {
            orc_returns(rewards, dones, bootstrap, N, T, hp->gamma, R);
            orc_loss_grad(logits, values, actions, R, B, A, hp->beta, hp->value_coef, hp->log_eps,
                          dZ, dV, sums);
            rc = orc_backward(net, theta, acts, B, dZ, dV, grad);
        }
        if (rc == 0) {
            double norm = orc_grad_norm(grad, P);
            double s = orc_clip_scale(norm, hp->clip_norm);
            orc_rmsprop(theta, g, grad, P, s, hp->lr, hp->rms_decay, hp->rms_eps);
            if (stats) {
                stats->policy_loss = sums[0]; stats->value_loss = sums[1]; stats->entropy = sums[2];
                stats->grad_norm = norm; stats->clip_scale = s;
            }
            if (R_out) memcpy(R_out, R, sizeof(double) * B);
            if (dZ_out) memcpy(dZ_out, dZ, sizeof(double) * (size_t)B * A);
            if (dV_out) memcpy(dV_out, dV, sizeof(double) * B);
            if (logits_out) memcpy(logits_out, logits, sizeof(double) * (size_t)B * A);
            if (values_out) memcpy(values_out, values, sizeof(double) * B);
        }
    }
    free(acts); free(logits); free(values); free(R); free(dZ); free(dV);
    return rc;
}

/* ---- single layers, batched ---------------------------------------------- */

/* The layers above one at a time, so that a test can hand each layer the
 * inputs another implementation actually used (for math = 1 this makes both
 * sides round the same numbers).  They call the same routines as the whole
 * network, frame by frame in index order.
 *
 * Convolution: x [B][C][H][W] is the layer's stored input (for the first layer
 * byte / 255, with xs = 255; otherwise xs = 1), y [B][OC][OH][OW]. */
void orc_conv_layer_forward(int B, const double *x, int C, int H, int W, const double *wt,
                            const double *bias, int OC, int K, int S, int math, double xs, double *y) {
    int OH = (H - K) / S + 1, OW = (W - K) / S + 1;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        conv_relu(x + (int64_t)b * C * H * W, C, H, W, wt, bias, OC, K, S, y + (int64_t)b * OC * OH * OW, math, xs);
}

/* Frames are spread over threads as in orc_backward: each thread adds its
 * frames, in index order, into private sums, which are then added in thread
 * order.  Returns the number of threads to use for B frames. */
static int frame_threads(int B) {
    int nthreads = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    nthreads = omp_get_max_threads();
#endif
    if (nthreads > B) nthreads = B > 0 ? B : 1;
    return nthreads;
}

/* gw [OC][C][K][K] and gb [OC] are overwritten with the sums over the frames;
 * dx [B][C][H][W] (may be NULL) is overwritten.  dy is taken before the
 * layer's ReLU mask, which comes from y. */
int orc_conv_layer_backward(int B, const double *x, int C, int H, int W, const double *wt, int OC,
                            int K, int S, const double *y, const double *dy, int math, double xs,
                            double *gw, double *gb, double *dx) {
    int OH = (H - K) / S + 1, OW = (W - K) / S + 1;
    int64_t in_sz = (int64_t)C * H * W, out_sz = (int64_t)OC * OH * OW, nw = (int64_t)OC * C * K * K;
    int nthreads = frame_threads(B);
    double *priv = (double *)calloc((size_t)nthreads * (nw + OC), sizeof(double));
    if (!priv) return -1;
    if (dx) for (int64_t i = 0; i < B * in_sz; ++i) dx[i] = 0.0;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int t = 0; t < nthreads; ++t) {
        int b0 = (int)((int64_t)B * t / nthreads), b1 = (int)((int64_t)B * (t + 1) / nthreads);
        double *pw = priv + (int64_t)t * (nw + OC);
        for (int b = b0; b < b1; ++b)
            conv_backward(x + b * in_sz, C, H, W, wt, OC, K, S, y + b * out_sz, dy + b * out_sz, math, xs,
                          pw, pw + nw, dx ? dx + b * in_sz : NULL);
    }
    for (int64_t i = 0; i < nw + OC; ++i) {
        double sum = 0.0;
        for (int t = 0; t < nthreads; ++t) sum += priv[(int64_t)t * (nw + OC) + i];
        if (i < nw) gw[i] = sum; else gb[i - nw] = sum;
    }
    free(priv);
    return 0;
}

/* x [B][I], W [O][I], bias [O] -> y [B][O]. */
void orc_dense_forward(int B, const double *x, int64_t I, const double *W, const double *bias, int O,
                       int relu, int math, double *y) {
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) dense(x + b * I, I, W, bias, O, relu, math, y + (int64_t)b * O);
}

/* dy [B][O] = dL/d(pre-activation).  gW [O][I], gb [O] are overwritten with the
 * sums over the frames, dx [B][I] (may be NULL) is overwritten. */
int orc_dense_backward(int B, const double *x, int64_t I, const double *W, int O, const double *dy,
                       int math, double *gW, double *gb, double *dx) {
    int64_t nw = (int64_t)O * I;
    int nthreads = frame_threads(B);
    double *priv = (double *)calloc((size_t)nthreads * (nw + O), sizeof(double));
    if (!priv) return -1;
    if (dx) for (int64_t i = 0; i < B * I; ++i) dx[i] = 0.0;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int t = 0; t < nthreads; ++t) {
        int b0 = (int)((int64_t)B * t / nthreads), b1 = (int)((int64_t)B * (t + 1) / nthreads);
        double *pw = priv + (int64_t)t * (nw + O);
        for (int b = b0; b < b1; ++b)
            dense_backward(x + b * I, I, W, O, dy + (int64_t)b * O, math, pw, pw + nw, dx ? dx + b * I : NULL);
    }
    for (int64_t i = 0; i < nw + O; ++i) {
        double sum = 0.0;
        for (int t = 0; t < nthreads; ++t) sum += priv[(int64_t)t * (nw + O) + i];
        if (i < nw) gW[i] = sum; else gb[i - nw] = sum;
    }
    free(priv);
    return 0;
}
