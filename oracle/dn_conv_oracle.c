/*
 * dn_conv_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain CPU statement of the two remaining layer types the paper lists for the Deep Netts engine
 * (section "Deep Netts Deep Learning Engine": fully connected, convolutional, maximum pooling,
 * softmax output) and names as the next ones to accelerate (section "Summary"): a
 * two-dimensional convolutional layer and a maximum-pooling layer, forward and backward.
 * The paper gives no formulas for them, so these are the textbook definitions, written as
 * scalar loops in a fixed summation order, with no blocking, fusion or reordering:
 *
 *   convolutional layer (images as [batch][channel][row][column], filters as
 *   [out channel][in channel][filter row][filter column], zero padding `pad` on all four sides,
 *   the same stride in both directions; the filter is applied without flipping):
 *     z[b][co][i][j] = bias[co] + sum_{ci,u,v} W[co][ci][u][v] x[b][ci][i*stride+u-pad][j*stride+v-pad]
 *     y = f(z)                              (f as for the fully connected layers)
 *   backward, given dA = dE/dy for every sample (E the loss of one sample):
 *     delta = dA * f'(y)                    (f' from the stored output, as for the dense layers)
 *     dW[co][ci][u][v] = (1/B) sum_{b,i,j} delta[b][co][i][j] x[b][ci][i*stride+u-pad][j*stride+v-pad]
 *     dbias[co]        = (1/B) sum_{b,i,j} delta[b][co][i][j]
 *     dX[b][ci][r][c]  = sum_{co,u,v : r = i*stride+u-pad, c = j*stride+v-pad} delta[b][co][i][j] W[co][ci][u][v]
 *   (parameter gradients are means over the batch, like the dense layers'; dX is per sample).
 *
 *   maximum pooling (window k x k, stride s, no padding; output rows floor((H-k)/s)+1):
 *     y[b][c][i][j] = max over the window;  backward: dX gets dY[b][c][i][j] added at the
 *     position of the window's maximum, the first one in row-major window order if several
 *     are equal; windows may overlap (s < k), then contributions add up.
 *
 * Compiled twice like dn_oracle.c: STORE_T=float (fp32 storage, fp64 accumulation, one rounding per
 * stored element; symbols o32_*) and STORE_T=double (symbols o64_*).
 * Shares no code with the device library.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef STORE_T
#error "compile with -DSTORE_T=float|double and -DPFX(x)=..."
#endif

typedef STORE_T real;

enum { ACT_LINEAR = 0, ACT_SIGMOID = 1, ACT_TANH = 2, ACT_RELU = 3 };

static double conv_act(int act, double z)
{
    switch (act) {
    case ACT_SIGMOID: return 1.0 / (1.0 + exp(-z));
    case ACT_TANH: return tanh(z);
    case ACT_RELU: return z > 0.0 ? z : 0.0;
    default: return z;
    }
}

static double conv_act_deriv(int act, double a)
{
    switch (act) {
    case ACT_SIGMOID: return a * (1.0 - a);
    case ACT_TANH: return 1.0 - a * a;
    case ACT_RELU: return a > 0.0 ? 1.0 : 0.0;
    default: return 1.0;
    }
}

int PFX(conv_out_size)(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

#define X4(t, b, c, i, j, C, H, W) (t)[(((size_t)(b) * (C) + (c)) * (H) + (i)) * (W) + (j)]

void PFX(conv_forward)(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act,
                       const real *X, const real *Wt, const real *bias, real *Y)
{
    const int Ho = PFX(conv_out_size)(H, KH, stride, pad), Wo = PFX(conv_out_size)(W, KW, stride, pad);
    for (int b = 0; b < B; ++b)
        for (int co = 0; co < Cout; ++co)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double z = (double)bias[co];
                    for (int ci = 0; ci < Cin; ++ci)
                        for (int u = 0; u < KH; ++u)
                            for (int v = 0; v < KW; ++v) {
                                const int r = i * stride + u - pad, c = j * stride + v - pad;
                                if (r < 0 || r >= H || c < 0 || c >= W) continue;
                                z += (double)X4(Wt, co, ci, u, v, Cin, KH, KW) * (double)X4(X, b, ci, r, c, Cin, H, W);
                            }
                    X4(Y, b, co, i, j, Cout, Ho, Wo) = (real)conv_act(act, z);
                }
}

/* delta [B][Cout][Ho][Wo] is an output (the layer's error term); dX may be NULL. */
void PFX(conv_backward)(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act,
                        const real *X, const real *Wt, const real *Y, const real *dA, real *delta, real *dX,
                        real *dW, real *dbias)
{
    const int Ho = PFX(conv_out_size)(H, KH, stride, pad), Wo = PFX(conv_out_size)(W, KW, stride, pad);
    const size_t ny = (size_t)B * Cout * Ho * Wo;
    for (size_t e = 0; e < ny; ++e) delta[e] = (real)((double)dA[e] * conv_act_deriv(act, (double)Y[e]));
    for (int co = 0; co < Cout; ++co) {
        double sb = 0.0;
        for (int b = 0; b < B; ++b)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) sb += (double)X4(delta, b, co, i, j, Cout, Ho, Wo);
        dbias[co] = (real)(sb / (double)B);
        for (int ci = 0; ci < Cin; ++ci)
            for (int u = 0; u < KH; ++u)
                for (int v = 0; v < KW; ++v) {
                    double s = 0.0;
                    for (int b = 0; b < B; ++b)
                        for (int i = 0; i < Ho; ++i)
                            for (int j = 0; j < Wo; ++j) {
                                const int r = i * stride + u - pad, c = j * stride + v - pad;
                                if (r < 0 || r >= H || c < 0 || c >= W) continue;
                                s += (double)X4(delta, b, co, i, j, Cout, Ho, Wo) * (double)X4(X, b, ci, r, c, Cin, H, W);
                            }
                    X4(dW, co, ci, u, v, Cin, KH, KW) = (real)(s / (double)B);
                }
    }
    if (!dX) return;
    for (int b = 0; b < B; ++b)
        for (int ci = 0; ci < Cin; ++ci)
            for (int r = 0; r < H; ++r)
                for (int c = 0; c < W; ++c) {
                    double s = 0.0;
                    for (int co = 0; co < Cout; ++co)
                        for (int u = 0; u < KH; ++u)
                            for (int v = 0; v < KW; ++v) {
                                const int ri = r + pad - u, cj = c + pad - v;
                                if (ri < 0 || cj < 0 || ri % stride != 0 || cj % stride != 0) continue;
                                const int i = ri / stride, j = cj / stride;
                                if (i >= Ho || j >= Wo) continue;
                                s += (double)X4(delta, b, co, i, j, Cout, Ho, Wo) * (double)X4(Wt, co, ci, u, v, Cin, KH, KW);
                            }
                    X4(dX, b, ci, r, c, Cin, H, W) = (real)s;
                }
}

void PFX(maxpool_forward)(int B, int C, int H, int W, int K, int stride, const real *X, real *Y)
{
    const int Ho = (H - K) / stride + 1, Wo = (W - K) / stride + 1;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    real m = X4(X, b, c, i * stride, j * stride, C, H, W);
                    for (int u = 0; u < K; ++u)
                        for (int v = 0; v < K; ++v) {
                            const real x = X4(X, b, c, i * stride + u, j * stride + v, C, H, W);
                            if (x > m) m = x;
                        }
                    X4(Y, b, c, i, j, C, Ho, Wo) = m;
                }
}

void PFX(maxpool_backward)(int B, int C, int H, int W, int K, int stride, const real *X, const real *dY, real *dX)
{
    const int Ho = (H - K) / stride + 1, Wo = (W - K) / stride + 1;
    const size_t nx = (size_t)B * C * H * W;
    double *acc = (double *)calloc(nx ? nx : 1, sizeof(double));
    if (!acc) return;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    int bu = 0, bv = 0;
                    real m = X4(X, b, c, i * stride, j * stride, C, H, W);
                    for (int u = 0; u < K; ++u)
                        for (int v = 0; v < K; ++v) {
                            const real x = X4(X, b, c, i * stride + u, j * stride + v, C, H, W);
                            if (x > m) { m = x; bu = u; bv = v; }   /* strictly greater: the first maximum wins */
                        }
                    X4(acc, b, c, i * stride + bu, j * stride + bv, C, H, W) += (double)X4(dY, b, c, i, j, C, Ho, Wo);
                }
    for (size_t e = 0; e < nx; ++e) dX[e] = (real)acc[e];
    free(acc);
}
