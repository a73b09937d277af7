/*
 * Driver for running the CPU checker under AddressSanitizer and
 * UndefinedBehaviorSanitizer (host code only; test infrastructure).
 *
 * Compiled once per precision together with the checker's two C files:
 *   gcc -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan
 *       -DSTORE_T=float|double "-DPFX(x)=o32_##x|o64_##x"
 *       oracle_sanitize_main.c ../../oracle/dn_oracle.c ../../oracle/dn_conv_oracle.c -lm
 * It calls every exported function of the checker on small, ragged shapes (batch sizes
 * that do not divide the sample count, widths of one, every activation and both losses,
 * strided and padded convolutions, overlapping pooling windows) with all buffers
 * allocated at their exact sizes, so that an out-of-bounds index, a misaligned or
 * overflowing computation ends the run; it also checks two closed forms so that the run
 * is not only a memory check.  Exit status 0 means clean.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef STORE_T real;
enum { ACT_LINEAR = 0, ACT_SIGMOID = 1, ACT_TANH = 2, ACT_RELU = 3, ACT_SOFTMAX = 4 };
enum { LOSS_MSE = 0, LOSS_CE = 1 };

/* the checker's exported functions (oracle/dn_oracle.c, oracle/dn_conv_oracle.c) */
size_t PFX(param_count)(int L, const int32_t *n);
size_t PFX(act_count)(int L, const int32_t *n, int B);
void PFX(forward)(int L, const int32_t *n, const int32_t *acts, const real *params, const real *X, int B, real *A);
int64_t PFX(forward_census)(int L, const int32_t *n, const int32_t *acts, const real *params, const real *X, int B,
                            real *A, double kink_eps, int64_t *kink_list, int64_t kink_cap);
double PFX(backward)(int L, const int32_t *n, const int32_t *acts, int loss, const real *params, const real *X,
                     const int32_t *labels, int B, const real *A, real *D, real *grads);
void PFX(input_gradient)(int L, const int32_t *n, const real *params, const real *D, int B, real *dX);
void PFX(update)(size_t P, real *params, real *vel, const real *grads, real lr, real mu);
double PFX(train_epoch)(int L, const int32_t *n, const int32_t *acts, int loss, real *params, real *vel, const real *X,
                        const int32_t *labels, int64_t N, int B, real lr, real mu, int64_t n_steps_limit,
                        double kink_eps, int64_t *kinks, int64_t *kink_list, int64_t kink_cap);
double PFX(evaluate)(int L, const int32_t *n, const int32_t *acts, int loss, const real *params, const real *X,
                     const int32_t *labels, int64_t N, int64_t *correct);
int PFX(conv_out_size)(int in, int k, int stride, int pad);
void PFX(conv_forward)(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act,
                       const real *X, const real *Wt, const real *bias, real *Y);
void PFX(conv_backward)(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act,
                        const real *X, const real *Wt, const real *Y, const real *dA, real *delta, real *dX, real *dW,
                        real *dbias);
void PFX(maxpool_forward)(int B, int C, int H, int W, int K, int stride, const real *X, real *Y);
void PFX(maxpool_backward)(int B, int C, int H, int W, int K, int stride, const real *X, const real *dY, real *dX);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) /* uniform in (-1, 1) */
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

static real *buf(size_t n, int random)
{
    real *p = (real *)malloc((n ? n : 1) * sizeof(real));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) p[i] = random ? (real)rnd() : (real)0;
    return p;
}

static void check(int ok, const char *what)
{
    if (!ok) { fprintf(stderr, "FAILED: %s\n", what); exit(1); }
}

static void all_finite(const real *p, size_t n, const char *what)
{
    for (size_t i = 0; i < n; ++i) check(isfinite((double)p[i]), what);
}

static void dense_case(int L, const int32_t *n, const int32_t *acts, int loss, int N, int B)
{
    const size_t P = PFX(param_count)(L, n), na = PFX(act_count)(L, n, B);
    real *params = buf(P, 1), *vel = buf(P, 0), *grads = buf(P, 0);
    real *X = buf((size_t)N * n[0], 1), *A = buf(na, 0), *D = buf(na, 0), *dX = buf((size_t)B * n[0], 0);
    int32_t *labels = (int32_t *)malloc((size_t)N * sizeof(int32_t));
    for (int i = 0; i < N; ++i) labels[i] = (int32_t)(i % n[L]);
    const int b = B < N ? B : N;
    PFX(forward)(L, n, acts, params, X, b, A);
    int64_t list[3 * 4];
    const int64_t hits = PFX(forward_census)(L, n, acts, params, X, b, A, 0.5, list, 4);
    check(hits >= 0, "census count");
    const double lb = PFX(backward)(L, n, acts, loss, params, X, labels, b, A, D, grads);
    check(isfinite(lb), "batch loss");
    PFX(input_gradient)(L, n, params, D, b, dX);
    PFX(update)(P, params, vel, grads, (real)0.05, (real)0.9);
    int64_t kinks = 0, klist[3 * 8];
    const double le = PFX(train_epoch)(L, n, acts, loss, params, vel, X, labels, N, B, (real)0.05, (real)0.9, 0, 0.5,
                                       &kinks, klist, 8);
    check(isfinite(le), "epoch loss");
    const double ll = PFX(train_epoch)(L, n, acts, loss, params, vel, X, labels, N, B, (real)0.05, (real)0.0, 2, 0.0,
                                       NULL, NULL, 0);
    check(isfinite(ll), "epoch loss with a step limit");
    int64_t correct = -1;
    const double ev = PFX(evaluate)(L, n, acts, loss, params, X, labels, N, &correct);
    check(isfinite(ev) && correct >= 0 && correct <= N, "evaluate");
    all_finite(params, P, "parameters"); all_finite(vel, P, "velocity"); all_finite(dX, (size_t)b * n[0], "input gradient");
    free(params); free(vel); free(grads); free(X); free(A); free(D); free(dX); free(labels);
}

/* one linear layer with squared error: G = (W x + b - y) x^T, g = W x + b - y */
static void closed_form_linear(void)
{
    const int32_t n[2] = {3, 2}, acts[1] = {ACT_LINEAR};
    real params[8] = {(real)0.5, (real)-1, (real)2, (real)0.25, (real)3, (real)-0.5, (real)0.1, (real)-0.2};
    real X[3] = {(real)1, (real)2, (real)-1}, A[2], D[2], G[8];
    const int32_t label[1] = {1};
    PFX(forward)(1, n, acts, params, X, 1, A);
    PFX(backward)(1, n, acts, LOSS_MSE, params, X, label, 1, A, D, G);
    const double z0 = 0.5 * 1 - 1 * 2 + 2 * -1 + 0.1, z1 = 0.25 * 1 + 3 * 2 - 0.5 * -1 - 0.2;
    const double e0 = z0 - 0.0, e1 = z1 - 1.0;
    const double want[8] = {e0 * 1, e0 * 2, e0 * -1, e1 * 1, e1 * 2, e1 * -1, e0, e1};
    for (int i = 0; i < 8; ++i) check(fabs((double)G[i] - want[i]) < 1e-5, "closed-form gradient of a linear layer");
}

static void conv_case(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act)
{
    const int Ho = PFX(conv_out_size)(H, KH, stride, pad), Wo = PFX(conv_out_size)(W, KW, stride, pad);
    const size_t nx = (size_t)B * Cin * H * W, ny = (size_t)B * Cout * Ho * Wo, nw = (size_t)Cout * Cin * KH * KW;
    real *X = buf(nx, 1), *Wt = buf(nw, 1), *bias = buf((size_t)Cout, 1), *Y = buf(ny, 0), *dA = buf(ny, 1);
    real *delta = buf(ny, 0), *dX = buf(nx, 0), *dW = buf(nw, 0), *db = buf((size_t)Cout, 0);
    PFX(conv_forward)(B, Cin, H, W, Cout, KH, KW, stride, pad, act, X, Wt, bias, Y);
    PFX(conv_backward)(B, Cin, H, W, Cout, KH, KW, stride, pad, act, X, Wt, Y, dA, delta, dX, dW, db);
    PFX(conv_backward)(B, Cin, H, W, Cout, KH, KW, stride, pad, act, X, Wt, Y, dA, delta, NULL, dW, db);
    all_finite(Y, ny, "conv output"); all_finite(dX, nx, "conv input gradient"); all_finite(dW, nw, "conv filter gradient");
    free(X); free(Wt); free(bias); free(Y); free(dA); free(delta); free(dX); free(dW); free(db);
}

static void pool_case(int B, int C, int H, int W, int K, int stride)
{
    const int Ho = (H - K) / stride + 1, Wo = (W - K) / stride + 1;
    const size_t nx = (size_t)B * C * H * W, ny = (size_t)B * C * Ho * Wo;
    real *X = buf(nx, 1), *Y = buf(ny, 0), *dY = buf(ny, 1), *dX = buf(nx, 0);
    PFX(maxpool_forward)(B, C, H, W, K, stride, X, Y);
    PFX(maxpool_backward)(B, C, H, W, K, stride, X, dY, dX);
    double sy = 0.0, sx = 0.0;          /* every window hands its gradient to exactly one input */
    for (size_t i = 0; i < ny; ++i) sy += (double)dY[i];
    for (size_t i = 0; i < nx; ++i) sx += (double)dX[i];
    check(fabs(sx - sy) < 1e-4 * (1.0 + fabs(sy)), "pooling gradient sums");
    free(X); free(Y); free(dY); free(dX);
}

int main(void)
{
    closed_form_linear();
    { const int32_t n[] = {4, 16, 3}, a[] = {ACT_SIGMOID, ACT_SIGMOID}; dense_case(2, n, a, LOSS_MSE, 10, 1); }
    { const int32_t n[] = {5, 7, 6, 4}, a[] = {ACT_RELU, ACT_TANH, ACT_SOFTMAX}; dense_case(3, n, a, LOSS_CE, 11, 4); }
    { const int32_t n[] = {1, 1, 2}, a[] = {ACT_TANH, ACT_SOFTMAX}; dense_case(2, n, a, LOSS_CE, 3, 5); }
    { const int32_t n[] = {9, 1}, a[] = {ACT_SIGMOID}; dense_case(1, n, a, LOSS_MSE, 7, 3); }
    { const int32_t n[] = {3, 5, 2}, a[] = {ACT_RELU, ACT_LINEAR}; dense_case(2, n, a, LOSS_MSE, 64 + 5, 64); }
    conv_case(2, 3, 7, 6, 4, 3, 2, 1, 0, ACT_TANH);
    conv_case(1, 1, 5, 5, 1, 3, 3, 1, 1, ACT_LINEAR);
    conv_case(3, 2, 9, 8, 5, 3, 3, 2, 1, ACT_SIGMOID);
    conv_case(2, 2, 6, 7, 3, 5, 5, 3, 2, ACT_RELU);
    pool_case(2, 3, 6, 6, 2, 2);
    pool_case(1, 2, 7, 5, 3, 2);
    pool_case(1, 1, 3, 3, 3, 1);
    printf("sanitize ok\n");
    return 0;
}
