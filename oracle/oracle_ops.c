/*
 * CPU oracle: plain direct-loop definitions of every operator a tenant graph
 * may contain.  TEST INFRASTRUCTURE ONLY -- it is used by the test-suite, by
 * the smoke check and as the reported CPU baseline; the product (the HIP
 * library) never links, imports or calls it, and the two share no code.
 *
 * The method under test (operator resizing, Eq. 5, and pointer-based
 * reordering, Section 4.3) is required to leave every tenant's result equal
 * to that of its plain forward pass ("without sacrificing model accuracy",
 * Section 4.2).  The oracle is therefore the textbook definition of each
 * operator, written as loops over the output with one fp64 accumulator per
 * output element; nothing is blocked, fused or reordered.
 *
 * Layout: activations are logical NCHW, weights [out][in/groups][kh][kw],
 * all stored as float.  Every function computes in double and rounds once
 * when it stores.  OpenMP, when enabled, only distributes independent output
 * elements over threads; the order of additions inside one output element
 * never changes.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3, ACT_HSWISH = 4, ACT_HSIGMOID = 5 };

/* The piecewise-linear gate of MobileNetV3 (Howard et al. 2019, Section 5.2): ReLU6(v + 3) / 6. */
static double hard_sigmoid(double v)
{
    const double t = v + 3.0;
    return (t < 0.0 ? 0.0 : (t > 6.0 ? 6.0 : t)) / 6.0;
}

static double apply_act(double v, int act)
{
    switch (act) {
    case ACT_RELU:  return v > 0.0 ? v : 0.0;
    case ACT_RELU6: return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
    case ACT_GELU:  return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));   /* exact (erf) form */
    case ACT_HSWISH:   return v * hard_sigmoid(v);
    case ACT_HSIGMOID: return hard_sigmoid(v);
    default:        return v;
    }
}

/* Round-to-nearest-even float -> bfloat16 -> float, in place (storage model of
 * the bf16 configurations: every graph tensor is held in bfloat16). */
void orc_round_bf16(float *a, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        union { float f; uint32_t u; } v;
        v.f = a[i];
        if (v.f != v.f) { v.u |= 0x00400000u; v.u &= 0xFFFF0000u; a[i] = v.f; continue; }
        uint32_t lsb = (v.u >> 16) & 1u;
        v.u += 0x7FFFu + lsb;
        v.u &= 0xFFFF0000u;
        a[i] = v.f;
    }
}

/*
 * Grouped 2-D cross-correlation with fused epilogue:
 *   y[n,co,oh,ow] = act( b[co] + sum_{ci,r,s} x[n, g*Cg+ci, oh*st-p+r, ow*st-p+s] * w[co,ci,r,s] + res[n,co,oh,ow] )
 * g = co / (Cout/groups), Cg = Cin/groups; taps outside the image contribute 0.
 * Only images n in [n_lo, n_hi) and channels co in [c_lo, c_hi) are written, so
 * the same routine serves an operator chunk (Eq. 5) and the whole operator.
 */
void orc_conv2d(const float *x, const float *w, const float *b, const float *res, float *y,
                int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride, int pad,
                int groups, int act, int n_lo, int n_hi, int c_lo, int c_hi)
{
    const int Ho = (H + 2 * pad - kh) / stride + 1;
    const int Wo = (W + 2 * pad - kw) / stride + 1;
    const int Cg = Cin / groups, Og = Cout / groups;
    (void)N;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = n_lo; n < n_hi; ++n)
        for (int co = c_lo; co < c_hi; ++co) {
            const int g = co / Og;
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = b ? (double)b[co] : 0.0;
                    for (int ci = 0; ci < Cg; ++ci)
                        for (int r = 0; r < kh; ++r) {
                            const int ih = oh * stride - pad + r;
                            if (ih < 0 || ih >= H) continue;
                            for (int s = 0; s < kw; ++s) {
                                const int iw = ow * stride - pad + s;
                                if (iw < 0 || iw >= W) continue;
                                acc += (double)x[(((size_t)n * Cin + g * Cg + ci) * H + ih) * W + iw] *
                                       (double)w[(((size_t)co * Cg + ci) * kh + r) * kw + s];
                            }
                        }
                    const size_t o = (((size_t)n * Cout + co) * Ho + oh) * Wo + ow;
                    if (res) acc += (double)res[o];
                    y[o] = (float)apply_act(acc, act);
                }
        }
}

/*
 * Fully connected layer on rows:  y[r,o] = act( b[o] + sum_k x[r,k]*w[o,k] + res[r,o] ),
 * x is [rows][K], w is [Nout][K], y is [rows][Nout]; rows [r_lo,r_hi), outputs [o_lo,o_hi).
 */
void orc_gemm(const float *x, const float *w, const float *b, const float *res, float *y,
              int rows, int K, int Nout, int act, int r_lo, int r_hi, int o_lo, int o_hi)
{
    (void)rows;
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = r_lo; r < r_hi; ++r)
        for (int o = o_lo; o < o_hi; ++o) {
            double acc = b ? (double)b[o] : 0.0;
            for (int k = 0; k < K; ++k)
                acc += (double)x[(size_t)r * K + k] * (double)w[(size_t)o * K + k];
            if (res) acc += (double)res[(size_t)r * Nout + o];
            y[(size_t)r * Nout + o] = (float)apply_act(acc, act);
        }
}

/*
 * Attention scores.  qkv is [B][3*D][S] (logical n,c,h with w=1), D = heads*dh.
 *   out[b*heads+hd, j, i] = alpha * sum_d qkv[b, hd*dh+d, i] * qkv[b, D+hd*dh+d, j]
 * (query position i, key position j); out is [B*heads][S(j)][S(i)].
 */
void orc_bgemm_qk(const float *qkv, float *out, int B, int heads, int dh, int S, double alpha,
                  int b_lo, int b_hi)
{
    const int D = heads * dh;
    (void)B;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = b_lo; b < b_hi; ++b)
        for (int hd = 0; hd < heads; ++hd)
            for (int j = 0; j < S; ++j)
                for (int i = 0; i < S; ++i) {
                    double acc = 0.0;
                    for (int d = 0; d < dh; ++d)
                        acc += (double)qkv[((size_t)b * 3 * D + hd * dh + d) * S + i] *
                               (double)qkv[((size_t)b * 3 * D + D + hd * dh + d) * S + j];
                    out[(((size_t)b * heads + hd) * S + j) * S + i] = (float)(alpha * acc);
                }
}

/*
 * Attention context.  p is [B*heads][S(j)][S(i)], qkv as above.
 *   out[b, hd*dh+d, i] = sum_j p[b*heads+hd, j, i] * qkv[b, 2*D+hd*dh+d, j];  out is [B][D][S].
 */
void orc_bgemm_pv(const float *p, const float *qkv, float *out, int B, int heads, int dh, int S,
                  int b_lo, int b_hi)
{
    const int D = heads * dh;
    (void)B;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = b_lo; b < b_hi; ++b)
        for (int hd = 0; hd < heads; ++hd)
            for (int d = 0; d < dh; ++d)
                for (int i = 0; i < S; ++i) {
                    double acc = 0.0;
                    for (int j = 0; j < S; ++j)
                        acc += (double)p[(((size_t)b * heads + hd) * S + j) * S + i] *
                               (double)qkv[((size_t)b * 3 * D + 2 * D + hd * dh + d) * S + j];
                    out[((size_t)b * D + hd * dh + d) * S + i] = (float)acc;
                }
}

/* Max pooling; positions outside the image never win (they act as -infinity). */
void orc_maxpool(const float *x, float *y, int N, int C, int H, int W, int k, int stride, int pad,
                 int n_lo, int n_hi, int c_lo, int c_hi)
{
    const int Ho = (H + 2 * pad - k) / stride + 1;
    const int Wo = (W + 2 * pad - k) / stride + 1;
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double m = -INFINITY;
                    for (int r = 0; r < k; ++r) {
                        const int ih = oh * stride - pad + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int s = 0; s < k; ++s) {
                            const int iw = ow * stride - pad + s;
                            if (iw < 0 || iw >= W) continue;
                            const double v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (v > m) m = v;
                        }
                    }
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] = (float)m;
                }
}

/* Global average pooling: y[n,c] = (1/(H*W)) * sum_{h,w} x[n,c,h,w]. */
void orc_gavgpool(const float *x, float *y, int N, int C, int H, int W,
                  int n_lo, int n_hi, int c_lo, int c_hi)
{
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c) {
            double acc = 0.0;
            for (int i = 0; i < H * W; ++i) acc += (double)x[((size_t)n * C + c) * H * W + i];
            y[(size_t)n * C + c] = (float)(acc / (double)(H * W));
        }
}

/* Per-channel affine + residual + activation: y = act(x*scale[c] + shift[c] + res). */
void orc_affine_act(const float *x, const float *scale, const float *shift, const float *res, float *y,
                    int N, int C, int HW, int act, int n_lo, int n_hi, int c_lo, int c_hi)
{
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                double v = (double)x[o] * (double)scale[c] + (double)shift[c];
                if (res) v += (double)res[o];
                y[o] = (float)apply_act(v, act);
            }
}

/* Channel gate (squeeze-and-excitation): y[n,c,i] = act(x[n,c,i] * g[n,c]) over a logical [N][C][HW] tensor. */
void orc_scale(const float *x, const float *g, float *y, int N, int C, int HW, int act,
               int n_lo, int n_hi, int c_lo, int c_hi)
{
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c)
            for (int i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = (float)apply_act((double)x[o] * (double)g[(size_t)n * C + c], act);
            }
}

/* Channel concatenation of a [N][Ca][HW] and a [N][Cb][HW] tensor: y[n,c] = c < Ca ? a[n,c] : b[n,c-Ca]. */
void orc_concat(const float *a, const float *b, float *y, int N, int Ca, int Cb, int HW,
                int n_lo, int n_hi, int c_lo, int c_hi)
{
    (void)N;
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * (Ca + Cb) + c) * HW + i] = c < Ca ? a[((size_t)n * Ca + c) * HW + i] : b[((size_t)n * Cb + (c - Ca)) * HW + i];
}

/* Unpadded mean pooling: y[n,c,oh,ow] = (1/k^2) * sum_{r,s<k} x[n,c,oh*stride+r,ow*stride+s]. */
void orc_avgpool(const float *x, float *y, int N, int C, int H, int W, int k, int stride,
                 int n_lo, int n_hi, int c_lo, int c_hi)
{
    const int Ho = (H - k) / stride + 1, Wo = (W - k) / stride + 1;
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int c = c_lo; c < c_hi; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int r = 0; r < k; ++r)
                        for (int s = 0; s < k; ++s) acc += (double)x[(((size_t)n * C + c) * H + oh * stride + r) * W + ow * stride + s];
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] = (float)(acc / (double)(k * k));
                }
}

/* y = act(a + b), elementwise over [lo, hi). */
void orc_add(const float *a, const float *b, float *y, int act, size_t lo, size_t hi)
{
    for (size_t i = lo; i < hi; ++i) y[i] = (float)apply_act((double)a[i] + (double)b[i], act);
}

/* y = act(x), elementwise over [lo, hi). */
void orc_act(const float *x, float *y, int act, size_t lo, size_t hi)
{
    for (size_t i = lo; i < hi; ++i) y[i] = (float)apply_act((double)x[i], act);
}

/*
 * Layer normalisation over the channel axis of a logical [N][C][P] tensor
 * (P = h*w positions), with an optional residual added first:
 *   v = x + res;  mu = mean_c v;  var = mean_c (v-mu)^2  (biased);
 *   y = (v-mu)/sqrt(var+eps) * gamma[c] + beta[c].
 */
void orc_layernorm(const float *x, const float *res, const float *gamma, const float *beta, float *y,
                   int N, int C, int P, double eps, int n_lo, int n_hi)
{
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int p = 0; p < P; ++p) {
            double mu = 0.0, var = 0.0;
            for (int c = 0; c < C; ++c) {
                const size_t o = ((size_t)n * C + c) * P + p;
                mu += (double)x[o] + (res ? (double)res[o] : 0.0);
            }
            mu /= (double)C;
            for (int c = 0; c < C; ++c) {
                const size_t o = ((size_t)n * C + c) * P + p;
                const double d = (double)x[o] + (res ? (double)res[o] : 0.0) - mu;
                var += d * d;
            }
            var /= (double)C;
            const double inv = 1.0 / sqrt(var + eps);
            for (int c = 0; c < C; ++c) {
                const size_t o = ((size_t)n * C + c) * P + p;
                const double v = (double)x[o] + (res ? (double)res[o] : 0.0);
                y[o] = (float)((v - mu) * inv * (double)gamma[c] + (double)beta[c]);
            }
        }
}

/* Softmax over the channel axis of a logical [N][C][P] tensor: exp(x-max)/sum. */
void orc_softmax(const float *x, float *y, int N, int C, int P, int n_lo, int n_hi)
{
    (void)N;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n_lo; n < n_hi; ++n)
        for (int p = 0; p < P; ++p) {
            double m = -INFINITY, s = 0.0;
            for (int c = 0; c < C; ++c) {
                const double v = x[((size_t)n * C + c) * P + p];
                if (v > m) m = v;
            }
            for (int c = 0; c < C; ++c) s += exp((double)x[((size_t)n * C + c) * P + p] - m);
            for (int c = 0; c < C; ++c) {
                const size_t o = ((size_t)n * C + c) * P + p;
                y[o] = (float)(exp((double)x[o] - m) / s);
            }
        }
}
