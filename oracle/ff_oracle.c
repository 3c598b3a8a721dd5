/*
 * CPU oracle for the FF-INT8 layer-local training step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * method computes; the HIP library never links, loads or calls it.  It shares
 * no code, header, table or constant generator with the HIP path.
 *
 * Every function follows the paper's Section IV-B (single-layer dataflow:
 * quantise the input with a symmetric uniform quantiser and stochastic
 * rounding, int8 x int8 -> int32 multiply-accumulate, loss from the goodness,
 * gradient of the layer output quantised to int8, weight gradient only, no
 * input gradient), Eq. (1)/(2) (losses), Section IV-C with Eq. (3)/(4) and
 * Algorithm 1 (look-ahead: one forward pass, goodness of every layer, loss of
 * layer i plus lambda times the losses of the later layers).
 *
 * Where a floating-point value decides an integer (a quantised code), the
 * operation order is fixed here in fp32 with IEEE round-to-nearest-even, one
 * rounding per written operation (compile with -ffp-contract=off; fmaf() only
 * where it is written).  Loops are in definition order: no blocking, no fusion.
 * OpenMP is used over independent output rows only.
 *
 * Pins (tests/test_oracle_*.py): closed forms of Eq. (1)/(2) at G = theta and
 * their symmetries, goodness of hand-built vectors, quantise->dequantise error
 * bounds and unbiasedness of stochastic rounding, brute-force integer dot
 * products, 1x1 convolution == dense, padded constant image, direct convolution
 * == explicit im2col + library matmul, finite differences of the un-quantised
 * loss for the local gradient, a hand-computed look-ahead example, and for
 * the residual-block functions: zero skip == plain layer, zero weights ==
 * dequantised input, exact goodness of power-of-two activities, order
 * independence and agreement with the fp64 sum of squares; depthwise
 * convolution == full convolution with channel-diagonal weights; for the
 * exact-derivative look-ahead: brute-force input-gradient contraction, a hand
 * example and the lambda = 0 / top-layer reductions of the combination, and
 * finite differences of L_new on an fp64 model of a three-layer stack within
 * the int8 quantisation error.
 * The look-ahead *semantics* (which reading of Eq. (4) is meant) has no pin in
 * the paper: parity unpinned for that choice; its arithmetic is pinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FFO_OK 0
#define FFO_ERR_ARG (-1)
#define FFO_ERR_OVERFLOW (-5)

#define FFO_ROUND_NEAREST 0
#define FFO_ROUND_STOCHASTIC 1

/* ------------------------------------------------------------------------
 * Counter-based random numbers for stochastic rounding (the paper cites
 * stochastic rounding for the input quantiser in Section IV-B and fixes no
 * generator).  One 32-bit hash per (seed, tag, element index):
 *   key  = finalise64(seed + 0x9E3779B97F4A7C15 * (tag + 1))
 *   k    = lo32(key) + hi32(idx) * (hi32(key) | 1)
 *   v    = lo32(idx) ^ k, then two multiply / xor-shift stages.
 * u = (h >> 8) * 2^-24 is uniform on the 2^24-point grid in [0, 1).
 * ---------------------------------------------------------------------- */
static uint64_t finalise64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint64_t ffo_key(uint64_t seed, uint64_t tag)
{
    return finalise64(seed + 0x9E3779B97F4A7C15ull * (tag + 1ull));
}

uint32_t ffo_hash(uint64_t seed, uint64_t tag, uint64_t idx)
{
    uint64_t key = ffo_key(seed, tag);
    uint32_t k = (uint32_t)key + (uint32_t)(idx >> 32) * ((uint32_t)(key >> 32) | 1u);
    uint32_t v = (uint32_t)idx ^ k;
    v ^= v >> 16;
    v *= 0x7FEB352Du;
    v ^= v >> 15;
    v *= 0x846CA68Bu;
    v ^= v >> 16;
    return v;
}

float ffo_uniform(uint64_t seed, uint64_t tag, uint64_t idx)
{
    return (float)(ffo_hash(seed, tag, idx) >> 8) * 0x1p-24f;
}

/* ------------------------------------------------------------------------
 * Symmetric uniform quantiser, per tensor, codes in [-127, 127]
 * (Section IV, Section IV-B).  n elements, element i uses random index i
 * (the linear index of the logical row-major tensor).  The range is max|x|
 * over the tensor itself.
 * The paper fixes no behaviour for a vanishing range; see the comment below.
 * ---------------------------------------------------------------------- */
static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

int ffo_quantize(const float *x, int64_t n, int mode, uint64_t seed, uint64_t tag,
                 int8_t *q, float *scale_out)
{
    if (!x || !q || !scale_out || n < 0) return FFO_ERR_ARG;
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > amax) amax = a;
    }
    /* A vanishing range (absmax below 2^-100, which includes the all-zero tensor) quantises to
     * all-zero codes with scale 1: 127/absmax must stay a finite fp32 number, and magnitudes this
     * small cannot move an fp32 weight. */
    if (amax < 0x1p-100f) {
        *scale_out = 1.0f;
        memset(q, 0, (size_t)n);
        return FFO_OK;
    }
    const float scale = amax / 127.0f;
    const float inv = 127.0f / amax;
    for (int64_t i = 0; i < n; ++i) {
        const float t = x[i] * inv;
        int code;
        if (mode == FFO_ROUND_NEAREST) {
            code = (int)rintf(t); /* ties to even */
        } else {
            const float f = floorf(t);
            const float frac = t - f;
            const float u = ffo_uniform(seed, tag, (uint64_t)i);
            code = (int)f + (u < frac ? 1 : 0);
        }
        q[i] = (int8_t)clampi(code, -127, 127);
    }
    *scale_out = scale;
    return FFO_OK;
}

void ffo_dequantize(const int8_t *q, int64_t n, float scale, float *x)
{
    for (int64_t i = 0; i < n; ++i) x[i] = (float)q[i] * scale;
}

/* ------------------------------------------------------------------------
 * Forward contraction, dense: acc[m][n] = sum_k A_q[m][k] * W_q[n][k]
 * (Section IV-B: int8 inputs, int32 accumulation).  Accumulated in int64 and
 * required to fit int32.
 * ---------------------------------------------------------------------- */
int ffo_dense_forward(const int8_t *a_q, const int8_t *w_q, int64_t M, int64_t K, int64_t N,
                      int32_t *acc)
{
    if (!a_q || !w_q || !acc) return FFO_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)a_q[m * K + k] * (int32_t)w_q[n * K + k];
            if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
            acc[m * N + n] = (int32_t)s;
        }
    }
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* Forward contraction, convolution (NHWC input, weights [C_out][kh][kw][C_in]);
 * taps that fall outside the image contribute zero. */
int ffo_conv_forward(const int8_t *a_q, const int8_t *w_q, int64_t B, int64_t H, int64_t W,
                     int64_t Cin, int64_t Cout, int64_t ks, int64_t stride, int64_t pad,
                     int32_t *acc)
{
    if (!a_q || !w_q || !acc || stride < 1 || ks < 1) return FFO_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t bh = 0; bh < B * Ho; ++bh) {
        const int64_t b = bh / Ho, ho = bh % Ho;
        for (int64_t wo = 0; wo < Wo; ++wo)
            for (int64_t co = 0; co < Cout; ++co) {
                int64_t s = 0;
                for (int64_t kh = 0; kh < ks; ++kh)
                    for (int64_t kw = 0; kw < ks; ++kw) {
                        const int64_t hi = ho * stride + kh - pad, wi = wo * stride + kw - pad;
                        if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                        for (int64_t ci = 0; ci < Cin; ++ci)
                            s += (int32_t)a_q[((b * H + hi) * W + wi) * Cin + ci] *
                                 (int32_t)w_q[((co * ks + kh) * ks + kw) * Cin + ci];
                    }
                if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                acc[((b * Ho + ho) * Wo + wo) * Cout + co] = (int32_t)s;
            }
    }
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* Depthwise convolution (one filter per channel; the inverted-bottleneck stacks of Table II are built from it):
 * acc[b][ho][wo][c] = sum over taps of a_q[b][hi][wi][c] * w_q[c][kh][kw]; NHWC input, weights [C][kh][kw]. */
int ffo_dwconv_forward(const int8_t *a_q, const int8_t *w_q, int64_t B, int64_t H, int64_t W, int64_t C,
                       int64_t ks, int64_t stride, int64_t pad, int32_t *acc)
{
    if (!a_q || !w_q || !acc || stride < 1 || ks < 1) return FFO_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < B * Ho; ++bh) {
        const int64_t b = bh / Ho, ho = bh % Ho;
        for (int64_t wo = 0; wo < Wo; ++wo)
            for (int64_t c = 0; c < C; ++c) {
                int64_t s = 0;
                for (int64_t kh = 0; kh < ks; ++kh)
                    for (int64_t kw = 0; kw < ks; ++kw) {
                        const int64_t hi = ho * stride + kh - pad, wi = wo * stride + kw - pad;
                        if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                        s += (int32_t)a_q[((b * H + hi) * W + wi) * C + c] * (int32_t)w_q[(c * ks + kh) * ks + kw];
                    }
                acc[((b * Ho + ho) * Wo + wo) * C + c] = (int32_t)s;
            }
    }
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * Activity and goodness (Section III: goodness = sum of squared activities;
 * Algorithm 1: G = ||y||^2).  y = act(s_y * acc), s_y = s_a * s_w, act = ReLU
 * (relu != 0) or identity.  `terms` consecutive accumulators belong to one
 * sample (dense: N; conv: H_out * W_out * C_out).
 *
 * Reproducible form: G_int = sum (v*v >> r) with v = act(acc) as an integer,
 * r = ffo_goodness_shift(K, terms);  G = fp32( fp64(G_int) * 2^r * s_y * s_y ),
 * the two factors s_y widened to fp64, products left to right.
 * Also returned: the plain fp64 sum of y^2 (for the 1e-6 agreement check) and
 * vmax[b] = max over the sample of |act(acc)|.
 * ---------------------------------------------------------------------- */
int ffo_goodness_shift(int64_t K, int64_t terms)
{
    /* smallest r >= 0 with (127^2 K)^2 * terms / 2^r < 2^64 */
    unsigned __int128 a = (unsigned __int128)16129u * (unsigned __int128)K;
    unsigned __int128 bound = a * a * (unsigned __int128)terms;
    int r = 0;
    while ((bound >> r) >> 64) ++r;
    return r;
}

int ffo_goodness(const int32_t *acc, int64_t B, int64_t terms, int relu, int r, float s_a,
                 float s_w, uint64_t *g_int, int32_t *vmax, float *G, double *G_plain)
{
    if (!acc || !g_int || !vmax || !G || !G_plain || r < 0 || r > 62) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t b = 0; b < B; ++b) {
        uint64_t gi = 0;
        int32_t vm = 0;
        double plain = 0.0;
        for (int64_t t = 0; t < terms; ++t) {
            const int32_t a = acc[b * terms + t];
            const int64_t v = (relu && a < 0) ? 0 : (int64_t)a;
            const int64_t av = v < 0 ? -v : v;
            if (av > vm) vm = (int32_t)(av > INT32_MAX ? INT32_MAX : av);
            gi += ((uint64_t)(v * v)) >> r;
            float y = (float)a * s_y;
            if (relu && y < 0.0f) y = 0.0f;
            plain += (double)y * (double)y;
        }
        g_int[b] = gi;
        vmax[b] = vm;
        G_plain[b] = plain;
        double g = (double)gi;
        g = g * ldexp(1.0, r);
        g = g * (double)s_y;
        g = g * (double)s_y;
        G[b] = (float)g;
    }
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * exp(z) for z <= 0 with a fixed operation sequence (it feeds the gradient
 * quantiser through the sigmoid, so both sides must agree bit for bit):
 * z clamped to >= -87; k = rint(z * log2(e)); Cody-Waite reduction with a
 * two-part ln 2; degree-7 Taylor polynomial in Horner form; scale by 2^k.
 * ---------------------------------------------------------------------- */
float ffo_exp_spec(float z)
{
    if (z < -87.0f) z = -87.0f;
    if (z > 0.0f) z = 0.0f;
    const float kf = rintf(z * 0x1.715476p+0f);
    float r = fmaf(-kf, 0x1.62e4p-1f, z);
    r = fmaf(-kf, 0x1.7f7d1cp-20f, r);
    float p = 0x1.a01a02p-13f;          /* 1/5040 */
    p = fmaf(p, r, 0x1.6c16c2p-10f);    /* 1/720  */
    p = fmaf(p, r, 0x1.111112p-7f);     /* 1/120  */
    p = fmaf(p, r, 0x1.555556p-5f);     /* 1/24   */
    p = fmaf(p, r, 0x1.555556p-3f);     /* 1/6    */
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)kf);
}

/* Loss and its derivative w.r.t. the goodness.  x = G - theta.
 * Positive pass, Eq. (1): L = log(1 + exp(-x)), c = dL/dG = -sigmoid(-x).
 * Negative pass, Eq. (2): L = log(1 + exp(+x)), c = dL/dG = +sigmoid(+x).
 * sigmoid(|x|) = 1/(1+e), sigmoid(-|x|) = e/(1+e), e = exp_spec(-|x|).
 * The loss value itself feeds no quantiser: computed in fp64 with libm. */
int ffo_loss_coeff(const float *G, int64_t B, int pass_sign, float theta, float *coeff,
                   float *loss, double *loss_mean)
{
    if (!G || !coeff || !loss || !loss_mean || (pass_sign != 1 && pass_sign != -1))
        return FFO_ERR_ARG;
    double sum = 0.0;
    for (int64_t b = 0; b < B; ++b) {
        const float x = G[b] - theta;
        const float e = ffo_exp_spec(-fabsf(x));
        const float den = 1.0f + e;
        const float sig_big = 1.0f / den; /* sigmoid(+|x|) */
        const float sig_small = e / den;  /* sigmoid(-|x|) */
        if (pass_sign > 0) {
            coeff[b] = -(x >= 0.0f ? sig_small : sig_big);
            const double xd = -(double)x;
            const double l = (xd > 0.0 ? xd : 0.0) + log1p(exp(-fabs(xd)));
            loss[b] = (float)l;
            sum += l;
        } else {
            coeff[b] = (x >= 0.0f ? sig_big : sig_small);
            const double xd = (double)x;
            const double l = (xd > 0.0 ? xd : 0.0) + log1p(exp(-fabs(xd)));
            loss[b] = (float)l;
            sum += l;
        }
    }
    *loss_mean = B > 0 ? sum / (double)B : 0.0;
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * Input of the next layer (Algorithm 1: one full forward pass):
 * a_next = y, or y / sqrt(G[b]) when the layer normalises its output length
 * (0 when G[b] == 0).
 * ---------------------------------------------------------------------- */
int ffo_handoff(const int32_t *acc, int64_t B, int64_t terms, int relu, int l2norm, float s_a,
                float s_w, const float *G, float *a_next)
{
    if (!acc || !a_next || (l2norm && !G)) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t b = 0; b < B; ++b) {
        const float nrm = l2norm ? sqrtf(G[b]) : 1.0f;
        for (int64_t t = 0; t < terms; ++t) {
            float y = (float)acc[b * terms + t] * s_y;
            if (relu && y < 0.0f) y = 0.0f;
            if (l2norm) y = (nrm > 0.0f) ? y / nrm : 0.0f;
            a_next[b * terms + t] = y;
        }
    }
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * Look-ahead (Eq. (3), Eq. (4), Algorithm 1).  With L_new,i = L_i +
 * lambda * (L_{i+1} + ... + L_k) and every L_j a function of G_j alone, the
 * later layers enter layer i's update through their per-sample dL_j/dG_j:
 *   S_k = 0,  S_i = S_{i+1} + c_{i+1},  ctil_i = fma(lambda, S_i, c_i).
 * c and ctil are [k][B], layer-major.
 * ---------------------------------------------------------------------- */
int ffo_lookahead(const float *c, int k, int64_t B, float lambda, float *ctil)
{
    if (!c || !ctil || k < 1) return FFO_ERR_ARG;
    for (int64_t b = 0; b < B; ++b) {
        float S = 0.0f;
        for (int i = k - 1; i >= 0; --i) {
            ctil[(int64_t)i * B + b] = fmaf(lambda, S, c[(int64_t)i * B + b]);
            S = S + c[(int64_t)i * B + b];
        }
    }
    return FFO_OK;
}

/* Gradient of the layer output before quantisation (Section IV-B):
 * dG/dacc is 2*y through the ReLU, so g = (2 * ctil[b]) * y. */
int ffo_local_grad(const int32_t *acc, int64_t B, int64_t terms, int relu, float s_a, float s_w,
                   const float *ctil, float *g)
{
    if (!acc || !ctil || !g) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t b = 0; b < B; ++b) {
        const float d = 2.0f * ctil[b];
        for (int64_t t = 0; t < terms; ++t) {
            float y = (float)acc[b * terms + t] * s_y;
            if (relu && y < 0.0f) y = 0.0f;
            g[b * terms + t] = d * y;
        }
    }
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * Residual blocks (Section IV-C names ResNet-style blocks; it gives no
 * mechanics, so this is a reading).  The second convolution of a basic block
 * is the FF layer whose activity is the BLOCK OUTPUT
 *     y = act( fp32(acc) * (s_a * s_w)  +  u ),
 * u = the skip value: the dequantised int8 block input fp32(x_q) * s_x
 * (identity), or the output of the 1x1 projection fp32(acc_p) * (s_a_p * s_w_p)
 * (down-sampling blocks).  One rounding per written operation.
 * ---------------------------------------------------------------------- */
int ffo_skip_identity(const int8_t *x_q, int64_t n, float s_x, float *u)
{
    if (!x_q || !u) return FFO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) u[i] = (float)x_q[i] * s_x;
    return FFO_OK;
}

int ffo_skip_projection(const int32_t *acc_p, int64_t n, float s_a, float s_w, float *u)
{
    if (!acc_p || !u) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t i = 0; i < n; ++i) u[i] = (float)acc_p[i] * s_y;
    return FFO_OK;
}

int ffo_residual_act(const int32_t *acc, const float *u, int64_t n, int relu, float s_a, float s_w,
                     float *y)
{
    if (!acc || !u || !y) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t i = 0; i < n; ++i) {
        const float t = (float)acc[i] * s_y;
        float v = t + u[i];
        if (relu && v < 0.0f) v = 0.0f;
        y[i] = v;
    }
    return FFO_OK;
}

/* Goodness of an fp32 activity tensor, made order-free: with amax = max |y| over
 * the whole tensor of the pass, each term enters as the integer
 *     floor( r * r * 2^40 ),  r = y * (1 / amax)   (r, 1/amax in fp32; r*r*2^40 exact in fp64)
 * and G = fp32( fp64(sum) * 2^-40 * amax * amax ).  amax < 2^-100: G = 0.
 * Also returns max |y| per sample and the plain fp64 sum of squares. */
int ffo_goodness_fx(const float *y, int64_t B, int64_t terms, float amax, uint64_t *g_int,
                    float *ymax, float *G, double *G_plain)
{
    if (!y || !g_int || !ymax || !G || !G_plain || terms > ((int64_t)1 << 22)) return FFO_ERR_ARG;
    const int live = amax >= 0x1p-100f;
    const float inv = live ? 1.0f / amax : 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        uint64_t gi = 0;
        float vm = 0.0f;
        double plain = 0.0;
        for (int64_t t = 0; t < terms; ++t) {
            const float v = y[b * terms + t];
            const float av = fabsf(v);
            if (av > vm) vm = av;
            const float r = v * inv;
            gi += (uint64_t)((double)r * (double)r * 0x1p40);
            plain += (double)v * (double)v;
        }
        g_int[b] = gi;
        ymax[b] = vm;
        G_plain[b] = plain;
        double g = (double)gi;
        g = g * 0x1p-40;
        g = g * (double)amax;
        g = g * (double)amax;
        G[b] = live ? (float)g : 0.0f;
    }
    return FFO_OK;
}

/* Local gradient from fp32 activities: g = (2 * ctil[b]) * y. */
int ffo_local_grad_f32(const float *y, int64_t B, int64_t terms, const float *ctil, float *g)
{
    if (!y || !ctil || !g) return FFO_ERR_ARG;
    for (int64_t b = 0; b < B; ++b) {
        const float d = 2.0f * ctil[b];
        for (int64_t t = 0; t < terms; ++t) g[b * terms + t] = d * y[b * terms + t];
    }
    return FFO_OK;
}

/* ------------------------------------------------------------------------
 * Weight-gradient contraction (Section IV-B: only g^W is formed).
 * Dense: dw[n][k] = sum_m gy_q[m][n] * a_q[m][k].
 * ---------------------------------------------------------------------- */
int ffo_dense_wgrad(const int8_t *gy_q, const int8_t *a_q, int64_t M, int64_t K, int64_t N,
                    int32_t *dw)
{
    if (!gy_q || !a_q || !dw) return FFO_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t n = 0; n < N; ++n) {
        /* row n of dw: sum over m of gy_q[m][n] * (row m of a_q), in exact 64-bit integers */
        int64_t *row = (int64_t *)calloc((size_t)(K > 0 ? K : 1), sizeof(int64_t));
        if (!row) { bad |= 2; continue; }
        for (int64_t m = 0; m < M; ++m) {
            const int32_t g = (int32_t)gy_q[m * N + n];
            for (int64_t k = 0; k < K; ++k) row[k] += g * (int32_t)a_q[m * K + k];
        }
        for (int64_t k = 0; k < K; ++k) {
            if (row[k] > INT32_MAX || row[k] < INT32_MIN) bad |= 1;
            dw[n * K + k] = (int32_t)row[k];
        }
        free(row);
    }
    if (bad & 2) return FFO_ERR_ARG;
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* ------------------------------------------------------------------------
 * Exact-derivative variant of the look-ahead (Eq. (4) read literally: the
 * derivative of the later layers' losses with respect to this layer's weights
 * is taken through those layers).  Dense ReLU stacks without normalisation.
 * With z_i the pre-activation in activity units, y_i = act(z_i), and
 * E_i = d(L_{i+1} + ... + L_k)/dy_i:
 *     H_i = d(L_i + ... + L_k)/dz_i = (2 c_i y_i + E_i) * act'(z_i)
 *     E_{i-1} = H_i W_i                          (a_i = y_{i-1})
 *     g^Y_i = dL_new_i/dz_i = (2 c_i y_i + lambda E_i) * act'(z_i)
 * c_i = dL_i/dG_i per sample (NOT the combined coefficient of the default
 * reading).  H_i and g^Y_i are each quantised to int8 (a reading: the paper
 * gives no int8 form of this chain and states that FF avoids it).
 *
 * Input-gradient contraction: e[m][k] = sum_n h_q[m][n] * w_q[n][k].
 * ---------------------------------------------------------------------- */
int ffo_dense_input_grad(const int8_t *h_q, const int8_t *w_q, int64_t M, int64_t K, int64_t N,
                         int32_t *e)
{
    if (!h_q || !w_q || !e) return FFO_ERR_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t k = 0; k < K; ++k) {
            int64_t sum = 0;
            for (int64_t n = 0; n < N; ++n) sum += (int32_t)h_q[m * N + n] * (int32_t)w_q[n * K + k];
            if (sum > INT32_MAX || sum < INT32_MIN) bad |= 1;
            e[m * K + k] = (int32_t)sum;
        }
    }
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* The two gradients of one layer and one pass, before quantisation:
 *   y = act(fp32(acc) * (s_a * s_w));  t = (2 c[b]) * y;  E = fp32(e_acc) * s_e  (0 when e_acc is NULL)
 *   h = (t + E) * mask;   g = fma(lambda, E, t) * mask;   mask = acc > 0 (ReLU) or 1 (identity). */
int ffo_chain_combine(const int32_t *acc, int64_t B, int64_t terms, int relu, float s_a, float s_w,
                      const float *c, const int32_t *e_acc, float s_e, float lambda, float *h, float *g)
{
    if (!acc || !c || !h || !g) return FFO_ERR_ARG;
    const float s_y = s_a * s_w;
    for (int64_t b = 0; b < B; ++b) {
        const float d = 2.0f * c[b];
        for (int64_t j = 0; j < terms; ++j) {
            const int64_t i = b * terms + j;
            float y = (float)acc[i] * s_y;
            if (relu && y < 0.0f) y = 0.0f;
            const float t = d * y;
            const float E = e_acc ? (float)e_acc[i] * s_e : 0.0f;
            const int live = !relu || acc[i] > 0;
            h[i] = live ? t + E : 0.0f;
            g[i] = live ? fmaf(lambda, E, t) : 0.0f;
        }
    }
    return FFO_OK;
}

/* Convolution: dw[co][kh][kw][ci] = sum over samples b0 <= b < b1 and output
 * pixels of gy_q[b][ho][wo][co] * a_q[b][ho*s+kh-pad][wo*s+kw-pad][ci].
 * The sample range lets the caller split a reduction that could overflow
 * int32 into chunks with separate accumulators. */
int ffo_conv_wgrad(const int8_t *gy_q, const int8_t *a_q, int64_t b0, int64_t b1, int64_t H,
                   int64_t W, int64_t Cin, int64_t Cout, int64_t ks, int64_t stride, int64_t pad,
                   int32_t *dw)
{
    if (!gy_q || !a_q || !dw || stride < 1 || ks < 1) return FFO_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t co = 0; co < Cout; ++co)
        for (int64_t kh = 0; kh < ks; ++kh)
            for (int64_t kw = 0; kw < ks; ++kw)
                for (int64_t ci = 0; ci < Cin; ++ci) {
                    int64_t s = 0;
                    for (int64_t b = b0; b < b1; ++b)
                        for (int64_t ho = 0; ho < Ho; ++ho) {
                            const int64_t hi = ho * stride + kh - pad;
                            if (hi < 0 || hi >= H) continue;
                            for (int64_t wo = 0; wo < Wo; ++wo) {
                                const int64_t wi = wo * stride + kw - pad;
                                if (wi < 0 || wi >= W) continue;
                                s += (int32_t)gy_q[((b * Ho + ho) * Wo + wo) * Cout + co] *
                                     (int32_t)a_q[((b * H + hi) * W + wi) * Cin + ci];
                            }
                        }
                    if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                    dw[((co * ks + kh) * ks + kw) * Cin + ci] = (int32_t)s;
                }
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* Weight gradient of a depthwise convolution over the samples [b0, b1):
 * dw[c][kh][kw] = sum over (b, ho, wo) of gy_q[b][ho][wo][c] * a_q[b][hi][wi][c]. */
int ffo_dwconv_wgrad(const int8_t *gy_q, const int8_t *a_q, int64_t b0, int64_t b1, int64_t H, int64_t W,
                     int64_t C, int64_t ks, int64_t stride, int64_t pad, int32_t *dw)
{
    if (!gy_q || !a_q || !dw || stride < 1 || ks < 1 || b1 < b0) return FFO_ERR_ARG;
    const int64_t Ho = (H + 2 * pad - ks) / stride + 1, Wo = (W + 2 * pad - ks) / stride + 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t c = 0; c < C; ++c)
        for (int64_t kh = 0; kh < ks; ++kh)
            for (int64_t kw = 0; kw < ks; ++kw) {
                int64_t s = 0;
                for (int64_t b = b0; b < b1; ++b)
                    for (int64_t ho = 0; ho < Ho; ++ho)
                        for (int64_t wo = 0; wo < Wo; ++wo) {
                            const int64_t hi = ho * stride + kh - pad, wi = wo * stride + kw - pad;
                            if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                            s += (int32_t)gy_q[((b * Ho + ho) * Wo + wo) * C + c] *
                                 (int32_t)a_q[((b * H + hi) * W + wi) * C + c];
                        }
                if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
                dw[(c * ks + kh) * ks + kw] = (int32_t)s;
            }
    return bad ? FFO_ERR_OVERFLOW : FFO_OK;
}

/* ------------------------------------------------------------------------
 * Weight update (Algorithm 1: update the weights with the int8 gradients).
 * Plain SGD on the fp32 master weights, one combined update from all
 * `n_terms` integer accumulators (positive pass chunks first, then negative):
 *   g = fp32(dw_0) * (s_g0 * s_a0);  g = fma(fp32(dw_j), s_gj * s_aj, g) ...
 *   w = fma(-(lr / total_samples), g, w).
 * ---------------------------------------------------------------------- */
int ffo_update(float *w, int64_t n, const int32_t *const *dw, const float *s_g, const float *s_a,
               int n_terms, float lr, int total_samples)
{
    if (!w || !dw || !s_g || !s_a || n_terms < 1 || total_samples < 1) return FFO_ERR_ARG;
    const float lr_eff = lr / (float)total_samples;
    for (int64_t i = 0; i < n; ++i) {
        float g = (float)dw[0][i] * (s_g[0] * s_a[0]);
        for (int j = 1; j < n_terms; ++j) g = fmaf((float)dw[j][i], s_g[j] * s_a[j], g);
        w[i] = fmaf(-lr_eff, g, w[i]);
    }
    return FFO_OK;
}
