/*
 * dn_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow CPU statement of what one training step of a fully connected
 * feed-forward network computes: feed forward, loss error assessment, back
 * propagation through every layer in reverse order, and the learning-rate
 * scaled update of weights and biases (the three training parts listed in the
 * paper's section "The Deep Netts Work-flow"; the neuron model -- net input =
 * weights . inputs + bias, output = activation(net input) -- is the one of the
 * section "Deep Learning Overview").  Backpropagation reaches the exact
 * gradient of the stated loss, so this file is that definition written out
 * with scalar loops in a fixed summation order (inner index ascending, then
 * sample index ascending).  There is no blocking, fusion or reordering.
 *
 * It shares no code with the device library and is only called by the tests,
 * the smoke check and the CPU-baseline leg of the benchmark.
 *
 * The file is compiled twice:
 *   -DSTORE_T=float  -DPFX(x)=o32_##x : every tensor a device implementation
 *        would store (W, b, velocity, activations, deltas, gradients) is held
 *        in fp32, each dot product / sum is accumulated in fp64 and rounded to
 *        fp32 once per stored element ("correctly rounded fp32 training").
 *   -DSTORE_T=double -DPFX(x)=o64_##x : everything in fp64 (used for finite
 *        differences and closed-form checks).
 *   -DSTORE_T=float -DACC_T=float -DPFX(x)=o32a_##x : not a reference; see ACC_T below.
 *
 * Readings taken where the paper is silent (it prints no formulas):
 *   - minibatch gradient = mean over the samples of the batch; a short last
 *     batch divides by its own size;
 *   - squared error per sample E = 1/2 sum_k (a_k - y_k)^2, targets one-hot;
 *   - cross-entropy E = -log softmax(z)[label], output delta = p - y;
 *   - activation derivatives are evaluated from the stored activation:
 *     sigmoid a(1-a), tanh 1-a^2, ReLU [a>0], linear 1;
 *   - classic momentum: dW <- mu*dW - lr*G ; W <- W + dW  (mu = 0: plain SGD);
 *   - every delta of a step uses the weights as they were before that step's
 *     update; samples are visited in index order, no shuffling;
 *   - back propagation runs on every step (no max-error gate).
 *
 * Flat layouts (row-major, C order):
 *   params / vel / grads : for l = 1..L : W_l [n_l][n_{l-1}] then b_l [n_l]
 *   acts / deltas        : for l = 1..L : A_l [B][n_l]
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

/* Type the long sums (net inputs, delta propagation, gradients) are accumulated in.  fp64 for the
 * two reference builds.  A third build (o32a_: fp32 storage AND fp32 accumulation, inner index
 * ascending) is not a reference: it is the same definition evaluated with rounding errors of the
 * size an fp32 device path has, and serves to measure how far two valid fp32 evaluations can
 * drift apart on ill-conditioned quantities (ReLU derivatives of net inputs next to zero). */
#ifndef ACC_T
#define ACC_T double
#endif
typedef ACC_T acc_t;

enum { ACT_LINEAR = 0, ACT_SIGMOID = 1, ACT_TANH = 2, ACT_RELU = 3, ACT_SOFTMAX = 4 };
enum { LOSS_MSE = 0, LOSS_CE = 1 };

size_t PFX(param_count)(int L, const int32_t *n)
{
    size_t p = 0;
    for (int l = 1; l <= L; ++l)
        p += (size_t)n[l] * (size_t)n[l - 1] + (size_t)n[l];
    return p;
}

size_t PFX(act_count)(int L, const int32_t *n, int B)
{
    size_t p = 0;
    for (int l = 1; l <= L; ++l)
        p += (size_t)B * (size_t)n[l];
    return p;
}

static size_t w_offset(const int32_t *n, int l) /* offset of W_l, l = 1..L */
{
    size_t p = 0;
    for (int j = 1; j < l; ++j)
        p += (size_t)n[j] * (size_t)n[j - 1] + (size_t)n[j];
    return p;
}

static size_t a_offset(const int32_t *n, int l, int B) /* offset of A_l, l = 1..L */
{
    size_t p = 0;
    for (int j = 1; j < l; ++j)
        p += (size_t)B * (size_t)n[j];
    return p;
}

static double act_apply(int act, double z)
{
    switch (act) {
    case ACT_SIGMOID: return 1.0 / (1.0 + exp(-z));
    case ACT_TANH:    return tanh(z);
    case ACT_RELU:    return z > 0.0 ? z : 0.0;
    default:          return z; /* linear; softmax is handled per row */
    }
}

static double act_deriv_from_output(int act, double a)
{
    switch (act) {
    case ACT_SIGMOID: return a * (1.0 - a);
    case ACT_TANH:    return 1.0 - a * a;
    case ACT_RELU:    return a > 0.0 ? 1.0 : 0.0;
    default:          return 1.0;
    }
}

/*
 * Feed forward: a_0 = x; for each layer, net input z = W a_prev + b and
 * a = f(z).  A softmax layer turns its row of net inputs into
 * exp(z - max z) / sum exp(z - max z).
 * kink_eps > 0 additionally counts ReLU units with |z| < kink_eps (the "kink
 * census": units whose derivative a rounding difference could flip) and, when
 * a log is given, records the first log->cap of them as triples
 * (sample index = log->base + row, layer, unit).
 */
typedef struct {
    int64_t *triples; /* [cap][3] */
    int64_t cap, n, base;
} kink_log;

static void forward_impl(int L, const int32_t *n, const int32_t *acts, const real *params,
                         const real *X, int B, real *A, double kink_eps, int64_t *kinks, kink_log *log)
{
    for (int l = 1; l <= L; ++l) {
        const real *W = params + w_offset(n, l);
        const real *b = W + (size_t)n[l] * (size_t)n[l - 1];
        const real *Ain = (l == 1) ? X : A + a_offset(n, l - 1, B);
        real *Aout = A + a_offset(n, l, B);
        const int nin = n[l - 1], nout = n[l], act = acts[l - 1];
        int64_t kink_local = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : kink_local)
        for (int s = 0; s < B; ++s) {
            for (int o = 0; o < nout; ++o) {
                acc_t z = (acc_t)b[o];
                for (int k = 0; k < nin; ++k)
                    z += (acc_t)W[(size_t)o * nin + k] * (acc_t)Ain[(size_t)s * nin + k];
                if (act == ACT_RELU && kink_eps > 0.0 && fabs((double)z) < kink_eps) {
                    kink_local++;
                    if (log) {
#pragma omp critical(kink_log_append)
                        if (log->n < log->cap) {
                            int64_t *t = log->triples + 3 * log->n++;
                            t[0] = log->base + s; t[1] = l; t[2] = o;
                        }
                    }
                }
                Aout[(size_t)s * nout + o] = (real)act_apply(act, (double)z);
            }
        }
        if (kinks)
            *kinks += kink_local;
        if (act == ACT_SOFTMAX) {
#pragma omp parallel for schedule(static)
            for (int s = 0; s < B; ++s) {
                real *row = Aout + (size_t)s * nout;
                double m = (double)row[0];
                for (int o = 1; o < nout; ++o)
                    if ((double)row[o] > m) m = (double)row[o];
                double sum = 0.0;
                for (int o = 0; o < nout; ++o)
                    sum += exp((double)row[o] - m);
                for (int o = 0; o < nout; ++o)
                    row[o] = (real)(exp((double)row[o] - m) / sum);
            }
        }
    }
}

void PFX(forward)(int L, const int32_t *n, const int32_t *acts, const real *params,
                  const real *X, int B, real *A)
{
    forward_impl(L, n, acts, params, X, B, A, 0.0, NULL, NULL);
}

/*
 * Feed forward with the kink census of this batch: returns the number of ReLU units with
 * |net input| < kink_eps and lists the first kink_cap of them in kink_list (may be NULL) as
 * triples (row of the batch, layer, unit).  Activations are those of forward().
 */
int64_t PFX(forward_census)(int L, const int32_t *n, const int32_t *acts, const real *params,
                            const real *X, int B, real *A, double kink_eps, int64_t *kink_list,
                            int64_t kink_cap)
{
    int64_t kinks = 0;
    kink_log log = {kink_list, kink_list ? kink_cap : 0, 0, 0};
    forward_impl(L, n, acts, params, X, B, A, kink_eps, &kinks, kink_list ? &log : NULL);
    return kinks;
}

/*
 * Loss error assessment and back propagation for one batch, given the
 * activations of the forward pass.  Writes deltas D (same layout as A) and the
 * batch-mean gradients (same layout as params).  Returns the batch-mean loss.
 *
 * Output layer:   cross-entropy + softmax : delta = p - y
 *                 squared error           : delta = (a - y) * f'(a)
 * Hidden layers:  delta_{l-1}[i] = (sum_o W_l[o][i] delta_l[o]) * f'_{l-1}(a_{l-1}[i])
 * Gradients:      G_l[o][i] = (1/B) sum_s delta_l[s][o] a_{l-1}[s][i]
 *                 g_l[o]    = (1/B) sum_s delta_l[s][o]
 * For B = 1 the weight gradient is the rank-1 outer product delta x input,
 * i.e. the two nested loops over (inputs, outputs) that the paper offloads in
 * the softmax output layer's backward method (section "How Deep Netts is
 * parallelized with TornadoVM?").
 */
double PFX(backward)(int L, const int32_t *n, const int32_t *acts, int loss, const real *params,
                     const real *X, const int32_t *labels, int B, const real *A, real *D,
                     real *grads)
{
    const int nL = n[L];
    const real *AL = A + a_offset(n, L, B);
    real *DL = D + a_offset(n, L, B);
    double loss_sum = 0.0;
    for (int s = 0; s < B; ++s) {
        const real *a = AL + (size_t)s * nL;
        real *d = DL + (size_t)s * nL;
        const int y = labels[s];
        double e = 0.0;
        if (loss == LOSS_CE) {
            e = -log((double)a[y] > 0.0 ? (double)a[y] : 1e-300);
            for (int o = 0; o < nL; ++o)
                d[o] = (real)((double)a[o] - (o == y ? 1.0 : 0.0));
        } else {
            for (int o = 0; o < nL; ++o) {
                double diff = (double)a[o] - (o == y ? 1.0 : 0.0);
                e += 0.5 * diff * diff;
                d[o] = (real)(diff * act_deriv_from_output(acts[L - 1], (double)a[o]));
            }
        }
        loss_sum += e;
    }

    for (int l = L; l >= 1; --l) {
        const real *W = params + w_offset(n, l);
        const real *Dl = D + a_offset(n, l, B);
        const real *Aprev = (l == 1) ? X : A + a_offset(n, l - 1, B);
        const int nin = n[l - 1], nout = n[l];
        if (l > 1) {
            real *Dprev = D + a_offset(n, l - 1, B);
            const int actp = acts[l - 2];
#pragma omp parallel for collapse(2) schedule(static)
            for (int s = 0; s < B; ++s) {
                for (int i = 0; i < nin; ++i) {
                    acc_t t = 0;
                    for (int o = 0; o < nout; ++o)
                        t += (acc_t)W[(size_t)o * nin + i] * (acc_t)Dl[(size_t)s * nout + o];
                    Dprev[(size_t)s * nin + i] =
                        (real)((double)t * act_deriv_from_output(actp, (double)Aprev[(size_t)s * nin + i]));
                }
            }
        }
        real *G = grads + w_offset(n, l);
        real *g = G + (size_t)nout * (size_t)nin;
#pragma omp parallel for schedule(static)
        for (int o = 0; o < nout; ++o) {
            for (int i = 0; i < nin; ++i) {
                acc_t acc = 0;
                for (int s = 0; s < B; ++s)
                    acc += (acc_t)Dl[(size_t)s * nout + o] * (acc_t)Aprev[(size_t)s * nin + i];
                G[(size_t)o * nin + i] = (real)((double)acc / (double)B);
            }
            acc_t accb = 0;
            for (int s = 0; s < B; ++s)
                accb += (acc_t)Dl[(size_t)s * nout + o];
            g[o] = (real)((double)accb / (double)B);
        }
    }
    return loss_sum / (double)B;
}

/*
 * Derivative of each sample's loss with respect to that sample's input, from the deltas the
 * backward pass left: dX[s][i] = sum_o W_1[o][i] delta_1[s][o]  (the propagation rule for
 * the hidden layers taken one layer further; the input has no activation, so no derivative
 * factor).  Per sample, not a batch mean: it is what a layer in front of the net receives as
 * the derivative with respect to its own output.
 */
void PFX(input_gradient)(int L, const int32_t *n, const real *params, const real *D, int B, real *dX)
{
    (void)L;
    const real *W = params + w_offset(n, 1);
    const real *D1 = D + a_offset(n, 1, B);
    const int nin = n[0], nout = n[1];
    for (int s = 0; s < B; ++s)
        for (int i = 0; i < nin; ++i) {
            double t = 0.0;
            for (int o = 0; o < nout; ++o)
                t += (double)W[(size_t)o * nin + i] * (double)D1[(size_t)s * nout + o];
            dX[(size_t)s * nin + i] = (real)t;
        }
}

/* Update: dW <- mu*dW - lr*G ; W <- W + dW, for weights and biases alike. */
void PFX(update)(size_t P, real *params, real *vel, const real *grads, real lr, real mu)
{
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < P; ++p) {
        real v = (real)((double)mu * (double)vel[p] - (double)lr * (double)grads[p]);
        vel[p] = v;
        params[p] = (real)((double)params[p] + (double)v);
    }
}

/*
 * One epoch: batches of B consecutive samples in index order (the last one
 * may be short); each batch runs forward, loss + backward, update.  Returns
 * the epoch loss = sum over batches of (batch-mean loss * batch size) / N,
 * every batch's loss being taken before its own update.  n_steps_limit > 0
 * stops after that many batches (the returned loss then averages over the
 * samples actually visited).  Returns NaN if scratch memory cannot be had.
 * kink_list (may be NULL) receives the first kink_cap census hits as triples
 * (sample, layer, unit) in no particular order; *kinks is the full count.
 */
double PFX(train_epoch)(int L, const int32_t *n, const int32_t *acts, int loss, real *params,
                        real *vel, const real *X, const int32_t *labels, int64_t N, int B,
                        real lr, real mu, int64_t n_steps_limit, double kink_eps,
                        int64_t *kinks, int64_t *kink_list, int64_t kink_cap)
{
    kink_log log = {kink_list, kink_list ? kink_cap : 0, 0, 0};
    const size_t P = PFX(param_count)(L, n);
    const size_t na = PFX(act_count)(L, n, B);
    real *A = (real *)malloc(na * sizeof(real));
    real *D = (real *)malloc(na * sizeof(real));
    real *G = (real *)malloc(P * sizeof(real));
    if (!A || !D || !G) {
        free(A); free(D); free(G);
        return NAN;
    }
    double loss_total = 0.0;
    int64_t seen = 0, step = 0;
    if (kinks) *kinks = 0;
    for (int64_t s0 = 0; s0 < N; s0 += B, ++step) {
        if (n_steps_limit > 0 && step >= n_steps_limit) break;
        const int b = (int)((N - s0) < B ? (N - s0) : B);
        const real *Xb = X + (size_t)s0 * (size_t)n[0];
        log.base = s0;
        forward_impl(L, n, acts, params, Xb, b, A, kink_eps, kinks, kink_list ? &log : NULL);
        double lb = PFX(backward)(L, n, acts, loss, params, Xb, labels + s0, b, A, D, G);
        PFX(update)(P, params, vel, G, lr, mu);
        loss_total += lb * (double)b;
        seen += b;
    }
    free(A); free(D); free(G);
    return seen ? loss_total / (double)seen : 0.0;
}

/*
 * Loss error assessment without training (the work-flow's comparison of the
 * network output with the desired output through the loss function, and the
 * paper's test step on held-out data): forward pass over all N samples at the
 * current parameters.  Returns the mean loss; *correct receives the number of
 * samples whose largest output sits at the label's index (the lowest index wins
 * a tie; outputs are compared as stored).
 */
double PFX(evaluate)(int L, const int32_t *n, const int32_t *acts, int loss, const real *params,
                     const real *X, const int32_t *labels, int64_t N, int64_t *correct)
{
    const int chunk = 64;
    const int nL = n[L];
    const size_t na = PFX(act_count)(L, n, chunk);
    real *A = (real *)malloc(na * sizeof(real));
    if (!A)
        return NAN;
    double loss_total = 0.0;
    int64_t hits = 0;
    for (int64_t s0 = 0; s0 < N; s0 += chunk) {
        const int b = (int)((N - s0) < chunk ? (N - s0) : chunk);
        forward_impl(L, n, acts, params, X + (size_t)s0 * (size_t)n[0], b, A, 0.0, NULL, NULL);
        const real *AL = A + a_offset(n, L, b);
        for (int s = 0; s < b; ++s) {
            const real *a = AL + (size_t)s * nL;
            const int y = labels[s0 + s];
            if (loss == LOSS_CE) {
                loss_total += -log((double)a[y] > 0.0 ? (double)a[y] : 1e-300);
            } else {
                for (int o = 0; o < nL; ++o) {
                    double diff = (double)a[o] - (o == y ? 1.0 : 0.0);
                    loss_total += 0.5 * diff * diff;
                }
            }
            int best = 0;
            for (int o = 1; o < nL; ++o)
                if (a[o] > a[best]) best = o;
            if (best == y) hits++;
        }
    }
    free(A);
    if (correct) *correct = hits;
    return N > 0 ? loss_total / (double)N : 0.0;
}

/* Number of threads the loops above will use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int PFX(threads)(void) { return omp_get_max_threads(); }
/* Threads for the following calls (n < 1: leave as is).  Results do not depend on it. */
void PFX(set_threads)(int n) { if (n >= 1) omp_set_num_threads(n); }
#else
int PFX(threads)(void) { return 1; }
void PFX(set_threads)(int n) { (void)n; }
#endif
