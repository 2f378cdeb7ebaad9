/*
 * CPU oracle for the fused DNN operators of transfer-tuning's kernel classes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against; it is never part of the product path and it
 * shares no code, header, table or helper with the HIP kernels.
 *
 * A schedule only changes HOW a kernel's loop nest is executed, never WHAT it
 * computes (paper Section 2 on schedules, Section 4.1 on transformations), so
 * the reference for every (kernel, schedule) pair is the operator's plain
 * definition written as the unscheduled loop nest:
 *
 *   - class E (paper Algorithm 2): pad, conv2d, add bias, ReLU;
 *   - class A (paper Table 1, "conv2d_add"): conv2d plus a per-channel vector;
 *   - class F (paper Table 1, "conv2d_bias_add_relu"): conv2d, bias, residual
 *     tensor add, ReLU;
 *   - class D (paper Table 1, "dense_add") and the dense-only class Q of
 *     Section 4.4.1: y = x W^T (+ b) (+ activation);
 *   - batch matmul: C[b] = A[b] B[b];
 *   - depthwise 3x3 (MobileNetV2-shaped kernels of Section 5.1): per-channel
 *     conv, bias, clamp to [0, 6].
 *
 * The convolution is a cross-correlation with zero padding, dilation 1 and
 * groups 1; the GEMM of paper Algorithm 1 (unmodified row-major loop nest) is
 * tt_oracle_batch_matmul with batch = 1 and trans_b = 0.
 *
 * Data are float32 (for the bf16 configurations the caller passes float32
 * arrays whose values are already bf16-representable).  Sums run in the order
 * the definition states; `acc64` selects a double accumulator (the parity
 * reference) or a float accumulator (the "naive fp32 loop" whose distance
 * from the double result bounds the summation-order error).
 *
 * Pins (tests/test_oracle_ops.py): brute-force re-derivations with another
 * loop order on tiny shapes, 1x1 conv == matmul, delta filter == identity,
 * zero filter == act(bias), linearity, shift equivariance, dense == batch
 * matmul with batch 1, depthwise == dense conv with block-diagonal weights,
 * exhaustive bf16 round trip and closed-form ties.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { TT_ORACLE_ACT_NONE = 0, TT_ORACLE_ACT_RELU = 1, TT_ORACLE_ACT_RELU6 = 2, TT_ORACLE_ACT_GELU = 3 };

static double activate(double v, int act)
{
    switch (act) {
    case TT_ORACLE_ACT_RELU:
        return v > 0.0 ? v : 0.0;
    case TT_ORACLE_ACT_RELU6:
        return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
    case TT_ORACLE_ACT_GELU: /* exact form: x/2 * (1 + erf(x / sqrt 2)) */
        return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));
    default:
        return v;
    }
}

/* Output size of one spatial axis of a padded, strided convolution. */
static int out_extent(int in, int filt, int stride, int pad)
{
    return (in + 2 * pad - filt) / stride + 1;
}

int tt_oracle_conv_out_extent(int in, int filt, int stride, int pad)
{
    return out_extent(in, filt, stride, pad);
}

/*
 * y[n,k,p,q] = act( bias[k] + res[n,k,p,q] + sum_{c,r,s} xpad[n,c,p*sh+r,q*sw+s] * w[k,c,r,s] )
 * x: [N,C,H,W], w: [K,C,R,S], bias: [K] or NULL, res: [N,K,Ho,Wo] or NULL,
 * y: [N,K,Ho,Wo].  Paper Algorithm 2 gives the op order: pad, conv, +bias, act.
 */
void tt_oracle_conv2d(const float *x, const float *w, const float *bias, const float *res, float *y,
                      int N, int C, int H, int W, int K, int R, int S, int stride_h, int stride_w,
                      int pad_h, int pad_w, int act, int acc64)
{
    const int Ho = out_extent(H, R, stride_h, pad_h);
    const int Wo = out_extent(W, S, stride_w, pad_w);
    const long long planes = (long long)N * K;
#pragma omp parallel for schedule(static)
    for (long long nk = 0; nk < planes; ++nk) {
        const int n = (int)(nk / K), k = (int)(nk % K);
        for (int p = 0; p < Ho; ++p) {
            for (int q = 0; q < Wo; ++q) {
                double acc_d = 0.0;
                float acc_f = 0.0f;
                for (int c = 0; c < C; ++c) {
                    for (int r = 0; r < R; ++r) {
                        const int ih = p * stride_h + r - pad_h;
                        for (int s = 0; s < S; ++s) {
                            const int iw = q * stride_w + s - pad_w;
                            /* the padded border contributes zeros */
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                continue;
                            const float xv = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            const float wv = w[(((size_t)k * C + c) * R + r) * S + s];
                            if (acc64)
                                acc_d += (double)xv * (double)wv;
                            else
                                acc_f += xv * wv;
                        }
                    }
                }
                const size_t o = (((size_t)n * K + k) * Ho + p) * Wo + q;
                double v = acc64 ? acc_d : (double)acc_f;
                if (bias)
                    v += (double)bias[k];
                if (res)
                    v += (double)res[o];
                y[o] = (float)activate(v, act);
            }
        }
    }
}

/*
 * The same definition evaluated at selected output coordinates only (coords: npts x 4 ints
 * n, k, p, q), for checks at sizes where the whole tensor would take too long.
 */
void tt_oracle_conv2d_points(const float *x, const float *w, const float *bias, const float *res, const int *coords,
                             float *out, long long npts, int N, int C, int H, int W, int K, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w, int act)
{
    const int Ho = out_extent(H, R, stride_h, pad_h);
    const int Wo = out_extent(W, S, stride_w, pad_w);
    (void)N;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < npts; ++i) {
        const int n = coords[4 * i], k = coords[4 * i + 1], p = coords[4 * i + 2], q = coords[4 * i + 3];
        double acc = 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r) {
                const int ih = p * stride_h + r - pad_h;
                for (int s = 0; s < S; ++s) {
                    const int iw = q * stride_w + s - pad_w;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                        continue;
                    acc += (double)x[(((size_t)n * C + c) * H + ih) * W + iw] *
                           (double)w[(((size_t)k * C + c) * R + r) * S + s];
                }
            }
        if (bias)
            acc += (double)bias[k];
        if (res)
            acc += (double)res[(((size_t)n * K + k) * Ho + p) * Wo + q];
        out[i] = (float)activate(acc, act);
    }
}

/*
 * y[m,o] = act( bias[o] + sum_i x[m,i] * w[o,i] );  x: [M,I], w: [O,I] (out, in), y: [M,O].
 */
void tt_oracle_dense(const float *x, const float *w, const float *bias, float *y, int M, int O, int I,
                     int act, int acc64)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int o = 0; o < O; ++o) {
            double acc_d = 0.0;
            float acc_f = 0.0f;
            for (int i = 0; i < I; ++i) {
                const float xv = x[(size_t)m * I + i], wv = w[(size_t)o * I + i];
                if (acc64)
                    acc_d += (double)xv * (double)wv;
                else
                    acc_f += xv * wv;
            }
            double v = acc64 ? acc_d : (double)acc_f;
            if (bias)
                v += (double)bias[o];
            y[(size_t)m * O + o] = (float)activate(v, act);
        }
    }
}

/*
 * c[b,m,n] = sum_k a[b,m,k] * B(b,k,n); a: [B,M,K]; b: [B,K,N] when trans_b == 0, [B,N,K] when 1.
 * With batch 1 and trans_b 0 this is the unmodified loop nest of paper Algorithm 1.
 */
void tt_oracle_batch_matmul(const float *a, const float *b, float *c, int B, int M, int N, int K,
                            int trans_b, int acc64)
{
    const long long rows = (long long)B * M;
#pragma omp parallel for schedule(static)
    for (long long bm = 0; bm < rows; ++bm) {
        const int bi = (int)(bm / M), m = (int)(bm % M);
        for (int n = 0; n < N; ++n) {
            double acc_d = 0.0;
            float acc_f = 0.0f;
            for (int k = 0; k < K; ++k) {
                const float av = a[((size_t)bi * M + m) * K + k];
                const float bv = trans_b ? b[((size_t)bi * N + n) * K + k] : b[((size_t)bi * K + k) * N + n];
                if (acc64)
                    acc_d += (double)av * (double)bv;
                else
                    acc_f += av * bv;
            }
            c[((size_t)bi * M + m) * N + n] = acc64 ? (float)acc_d : acc_f;
        }
    }
}

/*
 * Depthwise convolution, channel multiplier 1:
 * y[n,c,p,q] = act( bias[c] + sum_{r,s} xpad[n,c,p*sh+r,q*sw+s] * w[c,0,r,s] );  w: [C,1,R,S].
 */
void tt_oracle_dwconv(const float *x, const float *w, const float *bias, float *y, int N, int C, int H,
                      int W, int R, int S, int stride_h, int stride_w, int pad_h, int pad_w, int act,
                      int acc64)
{
    const int Ho = out_extent(H, R, stride_h, pad_h);
    const int Wo = out_extent(W, S, stride_w, pad_w);
    const long long planes = (long long)N * C;
#pragma omp parallel for schedule(static)
    for (long long nc = 0; nc < planes; ++nc) {
        const int c = (int)(nc % C);
        const float *xp = x + (size_t)nc * H * W;
        for (int p = 0; p < Ho; ++p) {
            for (int q = 0; q < Wo; ++q) {
                double acc_d = 0.0;
                float acc_f = 0.0f;
                for (int r = 0; r < R; ++r) {
                    const int ih = p * stride_h + r - pad_h;
                    for (int s = 0; s < S; ++s) {
                        const int iw = q * stride_w + s - pad_w;
                        if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                            continue;
                        const float xv = xp[(size_t)ih * W + iw];
                        const float wv = w[((size_t)c * R + r) * S + s];
                        if (acc64)
                            acc_d += (double)xv * (double)wv;
                        else
                            acc_f += xv * wv;
                    }
                }
                double v = acc64 ? acc_d : (double)acc_f;
                if (bias)
                    v += (double)bias[c];
                y[((size_t)nc * Ho + p) * Wo + q] = (float)activate(v, act);
            }
        }
    }
}

/*
 * bfloat16 = the upper 16 bits of an IEEE-754 binary32.  Conversion rounds to
 * nearest, ties to even, on the 16 discarded bits; NaN stays NaN (quiet).
 */
uint16_t tt_oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN: keep sign, force a quiet payload */
        return (uint16_t)((u >> 16) | 0x0040u);
    const uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u; /* carries into the exponent correctly, up to infinity */
    return (uint16_t)upper;
}

float tt_oracle_bf16_to_f32(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

void tt_oracle_round_to_bf16(const float *in, float *out, size_t count)
{
    for (size_t i = 0; i < count; ++i)
        out[i] = tt_oracle_bf16_to_f32(tt_oracle_f32_to_bf16(in[i]));
}
