/*
 * CPU oracle for the convolution front-end of the fused operator:
 *
 *     S[n,oh,ow,co] = sum_{kh<KH} sum_{kw<KW} sum_{c<Cin}
 *                       X[n, oh*sh - ph + kh*dh, ow*sw - pw + kw*dw, c] * Wt[co, kh, kw, c]
 *     v             = alpha * S + bias[co] + beta * R[n,oh,ow,co]
 *     Y[n,oh,ow,co] = round_out( min(max(act(v), lo), hi) )
 *
 * with X read as zero outside [0,H) x [0,W) (zero padding) and
 *     OH = (H + 2 ph - dh (KH-1) - 1) / sh + 1,   OW likewise.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain reference for the GPU library's convolution entry
 * point; nothing on the product path may call it and it shares no code with the HIP kernels.
 *
 * Where the paper fixes it, and this repository's readings:
 *   - the sum is the direct convolution (cross-correlation, as deep-learning frameworks define
 *     it) that the paper's convolution guidance starts from ("direct convolution" before
 *     "implicit GEMM"); the GPU path evaluates the same sum as a GEMM with
 *     M = output positions, N = output channels, K = KH*KW*Cin and an im2col tile gathered on
 *     the fly (optimisation prompt, convolution section), which changes the order of the
 *     additions, not the sum;
 *   - layout is channels-last (X: [N,H,W,Cin], Wt: [Cout,KH,KW,Cin], Y: [N,OH,OW,Cout]): a
 *     reading of this repository (the paper's examples use the framework default), chosen
 *     because 8 consecutive channels of one tap are then 16 contiguous bytes;
 *   - the consumer chain (bias per output channel, residual, activation, clamp, rounding of the
 *     output) and its order are those of the fused GEMM oracle (Level-2 optimisation prompt,
 *     "Fusion");
 *   - precision is never lowered inside: products and sums are fp64; only the final store may
 *     round (fp32, or bf16 by rounding that fp32 value to nearest-even).
 *
 * Pins (tests/test_oracle_conv_pins.py): a library convolution in fp64 over strides, paddings
 * and dilations, exact rational brute force on tiny inputs, the 1x1 case against the pinned GEMM
 * oracle, a one-hot kernel that shifts the input, zero padding, output-size formula.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { CONV_ACT_NONE = 0, CONV_ACT_RELU = 1, CONV_ACT_GELU_TANH = 2 };
enum { CONV_F64 = 0, CONV_F32 = 1, CONV_BF16 = 2 };

static double conv_element(const void *base, int kind, size_t index)
{
    if (kind == CONV_F64) return ((const double *)base)[index];
    if (kind == CONV_F32) return (double)((const float *)base)[index];
    uint32_t w = ((uint32_t)((const uint16_t *)base)[index]) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static float conv_round_bf16(float x)
{
    uint32_t w;
    memcpy(&w, &x, sizeof w);
    if ((w & 0x7F800000u) == 0x7F800000u) {
        if (w & 0x007FFFFFu) w |= 0x00400000u;
        w &= 0xFFFF0000u;
    } else {
        uint32_t lower = w & 0xFFFFu;
        w &= 0xFFFF0000u;
        if (lower > 0x8000u || (lower == 0x8000u && (w & 0x10000u))) w += 0x10000u;
    }
    float r;
    memcpy(&r, &w, sizeof r);
    return r;
}

static double conv_act(double v, int act)
{
    if (act == CONV_ACT_RELU) return v > 0.0 ? v : 0.0;
    if (act == CONV_ACT_GELU_TANH) {
        const double c = 0.7978845608028654; /* sqrt(2/pi) */
        return 0.5 * v * (1.0 + tanh(c * (v + 0.044715 * v * v * v)));
    }
    return v;
}

int oracle_conv_out_size(int in, int k, int stride, int pad, int dil)
{
    int span = in + 2 * pad - dil * (k - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

/*
 * X, Wt: in_kind elements (CONV_*), packed channels-last.  bias (fp64[Cout]) and R (r_kind,
 * packed [N,OH,OW,Cout]) may be NULL.  lo <= hi (+-inf for no clamp).  out_kind: CONV_F64 = no
 * rounding, CONV_F32, CONV_BF16.  Y: fp64 [N,OH,OW,Cout].  Returns 0, or -1 on a bad argument
 * (including an empty output).
 */
int oracle_conv2d_nhwc(int Nb, int H, int W, int Cin, int Cout, int KH, int KW,
                       int sh, int sw, int ph, int pw, int dh, int dw,
                       const void *X, const void *Wt, int in_kind,
                       double alpha, const double *bias,
                       const void *R, int r_kind, double beta,
                       int act, double lo, double hi, int out_kind, double *Y)
{
    if (Nb < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1 || KH < 1 || KW < 1) return -1;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1 || !X || !Wt || !Y) return -1;
    if (act < CONV_ACT_NONE || act > CONV_ACT_GELU_TANH) return -1;
    if (in_kind < CONV_F64 || in_kind > CONV_BF16 || out_kind < CONV_F64 || out_kind > CONV_BF16) return -1;
    if (R && (r_kind < CONV_F64 || r_kind > CONV_BF16)) return -1;
    if (!(lo <= hi)) return -1;
    const int OH = oracle_conv_out_size(H, KH, sh, ph, dh), OW = oracle_conv_out_size(W, KW, sw, pw, dw);
    if (OH < 1 || OW < 1) return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < Nb; ++n) {
        for (int oh = 0; oh < OH; ++oh) {
            for (int ow = 0; ow < OW; ++ow) {
                for (int co = 0; co < Cout; ++co) {
                    double s = 0.0;
                    for (int kh = 0; kh < KH; ++kh) {
                        const int ih = oh * sh - ph + kh * dh;
                        if (ih < 0 || ih >= H) continue;           /* zero padding */
                        for (int kw = 0; kw < KW; ++kw) {
                            const int iw = ow * sw - pw + kw * dw;
                            if (iw < 0 || iw >= W) continue;
                            const size_t xi = (((size_t)n * H + ih) * W + iw) * Cin;
                            const size_t wi = (((size_t)co * KH + kh) * KW + kw) * Cin;
                            for (int c = 0; c < Cin; ++c)
                                s += conv_element(X, in_kind, xi + c) * conv_element(Wt, in_kind, wi + c);
                        }
                    }
                    const size_t yi = (((size_t)n * OH + oh) * OW + ow) * Cout + co;
                    double v = alpha * s;
                    if (bias) v = v + bias[co];
                    if (R) v = v + beta * conv_element(R, r_kind, yi);
                    double y = conv_act(v, act);
                    if (y < lo) y = lo;
                    if (y > hi) y = hi;
                    if (out_kind == CONV_F32) y = (double)(float)y;
                    if (out_kind == CONV_BF16) y = (double)conv_round_bf16((float)y);
                    Y[yi] = y;
                }
            }
        }
    }
    return 0;
}
