// Row-wise and elementwise kernels of a training step: output-layer error
// (softmax, loss, Delta_L), loss reduction, and the elementwise parameter
// update used by dn_update.
#include "dn_internal.h"
#include "dn_wave.h"
#include "dn_narrow.h"

namespace dn {

// Block-wide reductions over 256 threads (4 waves); every thread gets the result.
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ float block_max(float v, float *red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__device__ __forceinline__ float activate(int act, float z)
{
    switch (act) {
    case DN_ACT_SIGMOID: return 1.0f / (1.0f + expf(-z));
    case DN_ACT_TANH: return tanhf(z);
    case DN_ACT_RELU: return z > 0.0f ? z : 0.0f;
    default: return z;
    }
}

__device__ __forceinline__ float deriv_from_output(int act, float a)
{
    switch (act) {
    case DN_ACT_SIGMOID: return a * (1.0f - a);
    case DN_ACT_TANH: return 1.0f - a * a;
    case DN_ACT_RELU: return a > 0.0f ? 1.0f : 0.0f;
    default: return 1.0f;
    }
}

// One workgroup per sample.
// Cross-entropy, phase OUT_FUSED: the row of A_L holds net inputs z; it is replaced by
// p = softmax(z), Delta_L = p - y, loss = log sum exp(z - max) - (z_y - max).
// Phase OUT_SOFTMAX_ONLY does only z -> p (no labels needed); phase OUT_FROM_P starts from
// a row that already holds p: Delta_L = p - y, loss = -log p_y.
// Squared error: the row holds a = f(z); Delta_L = (a - y) f'(a), loss = 1/2 sum (a - y)^2.
// With `loss_sums` the sample's loss is also added to loss_sums[s] (one running sum per batch
// row, so no two workgroups touch the same word): an epoch then needs one reduction at its end
// instead of one per step.
__global__ __launch_bounds__(256) void output_delta_kernel(float *__restrict__ AL, float *__restrict__ DL,
                                                           const int32_t *__restrict__ labels,
                                                           float *__restrict__ loss_rows, int nL, int act,
                                                           int loss, int phase, float *__restrict__ hit_rows,
                                                           double *__restrict__ loss_sums)
{
    __shared__ float red[4];
    const int s = blockIdx.x, tid = threadIdx.x;
    float *a = AL + (size_t)s * nL;
    float *d = DL + (size_t)s * nL;
    int y = (phase == OUT_SOFTMAX_ONLY) ? 0 : labels[s];
    y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);  // labels are the caller's; never index outside the row
    if (phase == OUT_EVAL) {
        // loss and hit flag only; the largest output wins, the lowest index among equals
        // (softmax is monotone, so for cross-entropy the net inputs z are compared)
        float m = -INFINITY;
        for (int o = tid; o < nL; o += 256) m = fmaxf(m, a[o]);
        m = block_max(m, red);
        float first = (float)nL;
        for (int o = tid; o < nL; o += 256)
            if (a[o] == m) { first = (float)o; break; }
        first = -block_max(-first, red);
        float e;
        if (loss == DN_LOSS_CROSS_ENTROPY) {
            float sum = 0.f;
            for (int o = tid; o < nL; o += 256) sum += expf(a[o] - m);
            sum = block_sum(sum, red);
            e = logf(sum) - (a[y] - m);
        } else {
            e = 0.f;
            for (int o = tid; o < nL; o += 256) {
                const float diff = a[o] - (o == y ? 1.0f : 0.0f);
                e += 0.5f * diff * diff;
            }
            e = block_sum(e, red);
        }
        if (tid == 0) {
            loss_rows[s] = e;
            hit_rows[s] = ((int)first == y) ? 1.0f : 0.0f;
        }
        return;
    }
    if (loss == DN_LOSS_CROSS_ENTROPY && phase != OUT_FROM_P) {
        float m = -INFINITY;
        for (int o = tid; o < nL; o += 256) m = fmaxf(m, a[o]);
        m = block_max(m, red);
        float sum = 0.f;
        for (int o = tid; o < nL; o += 256) sum += expf(a[o] - m);
        sum = block_sum(sum, red);
        const float zy = a[y];
        __syncthreads();  // every thread has read a[y] before the row is overwritten
        const float inv = 1.0f / sum;
        for (int o = tid; o < nL; o += 256) {
            const float p = expf(a[o] - m) * inv;
            a[o] = p;
            if (phase == OUT_FUSED) d[o] = p - (o == y ? 1.0f : 0.0f);
        }
        if (phase == OUT_FUSED && tid == 0) {
            const float e = logf(sum) - (zy - m);
            loss_rows[s] = e;
            if (loss_sums) loss_sums[s] += (double)e;
        }
    } else if (loss == DN_LOSS_CROSS_ENTROPY) {
        for (int o = tid; o < nL; o += 256) d[o] = a[o] - (o == y ? 1.0f : 0.0f);
        if (tid == 0) loss_rows[s] = -logf(fmaxf(a[y], 1e-37f));
    } else if (phase != OUT_SOFTMAX_ONLY) {
        float e = 0.f;
        for (int o = tid; o < nL; o += 256) {
            const float diff = a[o] - (o == y ? 1.0f : 0.0f);
            e += 0.5f * diff * diff;
            d[o] = diff * deriv_from_output(act, a[o]);
        }
        e = block_sum(e, red);
        if (tid == 0) {
            loss_rows[s] = e;
            if (loss_sums) loss_sums[s] += (double)e;
        }
    }
}

template <class In>
__global__ __launch_bounds__(256) void loss_reduce_kernel(const In *__restrict__ loss_rows, int B,
                                                          float *__restrict__ mean_out,
                                                          double *__restrict__ epoch_acc)
{
    __shared__ double red[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < B; i += 256) s += (double)loss_rows[i];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double t = red[0] + red[1] + red[2] + red[3];
        if (mean_out) *mean_out = (float)(t / (double)B);
        if (epoch_acc) *epoch_acc += t;
    }
}

__global__ __launch_bounds__(256) void update_kernel(float *__restrict__ p, float *__restrict__ v,
                                                     const float *__restrict__ g, size_t count, float lr,
                                                     float mu)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) {
        const float dw = mu * v[i] - lr * g[i];
        v[i] = dw;
        p[i] = p[i] + dw;
    }
}

__global__ __launch_bounds__(256) void copy_kernel(float *__restrict__ dst, const float *__restrict__ src,
                                                   size_t count)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256)
        dst[i] = src[i];
}

hipError_t launch_output_delta(float *AL, float *DL, const int32_t *labels, float *loss_rows, int B,
                               int nL, int act, int loss, int phase, hipStream_t stream, float *hit_rows,
                               double *loss_sums)
{
    if (phase == OUT_EVAL && !hit_rows) return hipErrorInvalidValue;
    launch_kernel(output_delta_kernel, dim3(B), dim3(256), 0, stream, AL, DL, labels, loss_rows, nL, act, loss, phase,
                  hit_rows, loss_sums);
    return hipGetLastError();
}

hipError_t launch_loss_reduce(const float *loss_rows, int B, float *loss_mean_out, double *epoch_acc,
                              hipStream_t stream)
{
    hipLaunchKernelGGL(loss_reduce_kernel<float>, dim3(1), dim3(256), 0, stream, loss_rows, B, loss_mean_out,
                       epoch_acc);
    return hipGetLastError();
}

hipError_t launch_loss_sums_reduce(const double *loss_sums, int B, double *epoch_acc, hipStream_t stream)
{
    hipLaunchKernelGGL(loss_reduce_kernel<double>, dim3(1), dim3(256), 0, stream, loss_sums, B, (float *)nullptr,
                       epoch_acc);
    return hipGetLastError();
}

// The two-index (inputs x outputs) loop of the paper's offloaded backward method for one
// sample: gradients[o][i] = deltas[o] * inputs[i], deltaWeights[o][i] = -lr * gradients[o][i],
// deltaBiases[o] = -lr * deltas[o].  One thread per run of four (VEC) or one weight.
template <int VEC>
__global__ __launch_bounds__(256) void layer_backward_kernel(const float *__restrict__ deltas,
                                                             const float *__restrict__ inputs, float lr,
                                                             int cols_out, int cols_in, float *__restrict__ G,
                                                             float *__restrict__ dW, float *__restrict__ dB)
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    const size_t total = (size_t)cols_out * (size_t)cols_in / VEC;
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < total; q += (size_t)gridDim.x * 256) {
        const size_t e = q * VEC;
        const int o = (int)(e / (size_t)cols_in);
        const int i = (int)(e - (size_t)o * cols_in);
        const float d = deltas[o];
        if (VEC == 4) {
            const v4 x = *reinterpret_cast<const v4 *>(inputs + i);
            const v4 g = x * d;
            *reinterpret_cast<v4 *>(G + e) = g;
            *reinterpret_cast<v4 *>(dW + e) = g * (-lr);
        } else {
            const float g = d * inputs[i];
            G[e] = g;
            dW[e] = -lr * g;
        }
    }
    for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < (size_t)cols_out; o += (size_t)gridDim.x * 256)
        dB[o] = -lr * deltas[o];
}

hipError_t launch_layer_backward(const float *deltas, const float *inputs, float lr, int cols_out, int cols_in,
                                 float *G, float *dW, float *dB, hipStream_t stream)
{
    const bool vec = cols_in % 4 == 0;
    size_t work = (size_t)cols_out * cols_in / (vec ? 4 : 1);
    size_t g = (work + 255) / 256;
    if (g > 256 * 32) g = 256 * 32;
    if (g < 1) g = 1;
    if (vec)
        hipLaunchKernelGGL(layer_backward_kernel<4>, dim3((unsigned)g), dim3(256), 0, stream, deltas, inputs, lr,
                           cols_out, cols_in, G, dW, dB);
    else
        hipLaunchKernelGGL(layer_backward_kernel<1>, dim3((unsigned)g), dim3(256), 0, stream, deltas, inputs, lr,
                           cols_out, cols_in, G, dW, dB);
    return hipGetLastError();
}

// ---- layers with at most 16 outputs (the 10-class output layer of the benchmark nets) ----------
// Their delta and gradient products have one side of at most 16: on 32- or 64-wide matrix-core
// tiles most of the work would be padding, and a width that is not a multiple of four rules out
// vector loads there.  These kernels use plain FMAs instead; both are bound by launch latency.
// Delta_{l-1}[b][j] = f'(A_{l-1}[b][j]) * sum_o Delta_l[b][o] W_l[o][j] for n_l <= 16.
// One thread per VEC adjacent columns j; it keeps its columns of W_l in registers and walks the
// rows of its block's row range (row addresses are uniform, so Delta_l comes through scalar loads).
template <int VEC>
__global__ __launch_bounds__(256) void narrow_delta_kernel(const float *__restrict__ D, const float *__restrict__ W,
                                                           const float *__restrict__ Aprev, float *__restrict__ C,
                                                           int B, int nl, int nin, int act, int rows_per_block)
{
    const int j = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (j >= nin) return;
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    vec_t w[kNarrow];
#pragma unroll
    for (int o = 0; o < kNarrow; ++o) {
        w[o] = 0.f;
        if (o < nl) w[o] = *reinterpret_cast<const vec_t *>(W + (size_t)o * nin + j);
    }
    const int b0 = blockIdx.y * rows_per_block;
    const int b1 = min(B, b0 + rows_per_block);
    for (int b = b0; b < b1; ++b) {
        const float *d = D + (size_t)b * nl;
        vec_t sum = 0.f;
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            if (o < nl) {
                const float dv = d[o];
#pragma unroll
                for (int v = 0; v < VEC; ++v) sum[v] = fmaf(dv, w[o][v], sum[v]);
            }
        }
        const size_t e = (size_t)b * nin + j;
        const vec_t a = *reinterpret_cast<const vec_t *>(Aprev + e);
#pragma unroll
        for (int v = 0; v < VEC; ++v) sum[v] *= deriv_from_output(act, a[v]);
        *reinterpret_cast<vec_t *>(C + e) = sum;
    }
}

// The weight gradient / update of such a layer (narrow_grad_block, dn_narrow.h) as a kernel of its own.
template <int VEC>
__global__ __launch_bounds__(256) void narrow_grad_kernel(NarrowGradArgs g)
{
    narrow_grad_block<VEC>(g, (int)blockIdx.x, (int)gridDim.x);
}

bool narrow_layer(int n_out) { return n_out >= 1 && n_out <= kNarrow; }

// Forward pass and output error of a last layer with at most 16 outputs in one launch:
// z = A_{L-1} W_L^T + b_L, then what output_delta_kernel's phase OUT_FUSED does with the row
// (softmax, loss, Delta_L; or activation, loss, Delta_L for squared error).  A workgroup takes R
// rows of the batch; its 256 threads split k (each W_L element a lane loads serves R rows), the
// R * n_L dot products are summed across each wave and then across the four waves through LDS,
// and wave w finishes rows w, w + 4, ... with every lane holding the row's z.
// With Dprev given the launch also propagates the error one layer down: Delta_{L-1}[b][k] =
// f'_{L-1}(A_{L-1}[b][k]) * sum_o Delta_L[b][o] W_L[o][k] -- every thread already holds its k
// columns of W_L and of the row, so the delta product through a narrow last layer costs no
// launch of its own.  Same arithmetic, in the same order, as narrow_delta_kernel.
struct NarrowOutArgs {
    const float *Aprev, *W, *bias;
    const int32_t *labels;
    float *AL, *DL, *loss_rows;
    double *loss_sums;
    int B, nl, nin, act, loss;
    float *Dprev;     // [B][nin] or nullptr
    int act_prev;     // activation of layer L-1 (its derivative multiplies Dprev)
};

template <int R, int VEC>
__global__ __launch_bounds__(256) void narrow_output_kernel(NarrowOutArgs g)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    __shared__ float part[4][R][kNarrow];
    __shared__ float dsh[R][kNarrow];   // Delta_L of the workgroup's rows, for the propagation phase
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * R;
    // what the last phase needs, requested before the k loop so that it is there by then
    const float my_bias = lane < g.nl ? g.bias[lane] : 0.f;
    int label[(R + 3) / 4];
#pragma unroll
    for (int i = 0; i < (R + 3) / 4; ++i) label[i] = g.labels[min(row0 + wave + 4 * i, g.B - 1)];
    // the epoch's running loss sum of the row this lane will finish: read now, added to at the end
    double sum_pre[(R + 3) / 4];
#pragma unroll
    for (int i = 0; i < (R + 3) / 4; ++i) {
        const int row = row0 + wave + 4 * i;
        sum_pre[i] = (g.loss_sums && lane == 0 && wave + 4 * i < R && row < g.B) ? g.loss_sums[row] : 0.0;
    }
    float acc[R][kNarrow];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) acc[r][o] = 0.f;
    // The thread's first piece of k stays in registers (its VEC columns of every row of W_L and of the
    // R input rows): up to 256 * VEC inputs that is all of k, and the propagation phase at the end
    // then needs no second trip to memory.
    const int k_first = threadIdx.x * VEC;
    const bool has_first = k_first < g.nin;
    vec_t a0[R], w0[kNarrow];
#pragma unroll
    for (int r = 0; r < R; ++r)   // rows past the batch repeat the last row; their results are dropped
        a0[r] = has_first ? *reinterpret_cast<const vec_t *>(g.Aprev + (size_t)min(row0 + r, g.B - 1) * g.nin + k_first) : (vec_t)0.f;
#pragma unroll
    for (int o = 0; o < kNarrow; ++o)
        w0[o] = (has_first && o < g.nl) ? *reinterpret_cast<const vec_t *>(g.W + (size_t)o * g.nin + k_first) : (vec_t)0.f;
#pragma unroll
    for (int o = 0; o < kNarrow; ++o)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[r][o] = fmaf(a0[r][v], w0[o][v], acc[r][o]);
    for (int k = k_first + 256 * VEC; k < g.nin; k += 256 * VEC) {
        vec_t a[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            a[r] = *reinterpret_cast<const vec_t *>(g.Aprev + (size_t)min(row0 + r, g.B - 1) * g.nin + k);
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            if (o < g.nl) {
                const vec_t w = *reinterpret_cast<const vec_t *>(g.W + (size_t)o * g.nin + k);
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[r][o] = fmaf(a[r][v], w[v], acc[r][o]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            const float total = (o < g.nl) ? wave_sum(acc[r][o]) : 0.f;
            if (lane == 0) part[wave][r][o] = total;
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < (R + 3) / 4; ++i) {
        const int r = wave + 4 * i;
        const int row = row0 + r;
        if (r >= R || row >= g.B) continue;
        float z[kNarrow];
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_bias), o));
            z[o] = ((part[0][r][o] + part[1][r][o]) + (part[2][r][o] + part[3][r][o])) + b;
        }
        int y = label[i];
        y = y < 0 ? 0 : (y >= g.nl ? g.nl - 1 : y);
        float mine = 0.f, e;   // lane o keeps output o
        if (g.loss == DN_LOSS_CROSS_ENTROPY) {
            float m = -INFINITY, zy = 0.f;
#pragma unroll
            for (int o = 0; o < kNarrow; ++o)
                if (o < g.nl) {
                    m = fmaxf(m, z[o]);
                    zy = (o == y) ? z[o] : zy;
                }
            float sum = 0.f;
#pragma unroll
            for (int o = 0; o < kNarrow; ++o)
                if (o < g.nl) {
                    z[o] = expf(z[o] - m);
                    sum += z[o];
                }
            const float inv = 1.0f / sum;
#pragma unroll
            for (int o = 0; o < kNarrow; ++o) mine = (o == lane) ? z[o] * inv : mine;
            e = logf(sum) - (zy - m);
            if (lane < g.nl) {
                const float d = mine - (lane == y ? 1.0f : 0.0f);
                g.AL[(size_t)row * g.nl + lane] = mine;
                g.DL[(size_t)row * g.nl + lane] = d;
                dsh[r][lane] = d;
            }
        } else {
            e = 0.f;
#pragma unroll
            for (int o = 0; o < kNarrow; ++o)
                if (o < g.nl) {
                    const float a = activate(g.act, z[o]);
                    const float diff = a - (o == y ? 1.0f : 0.0f);
                    e += 0.5f * diff * diff;
                    mine = (o == lane) ? a : mine;
                }
            if (lane < g.nl) {
                const float diff = mine - (lane == y ? 1.0f : 0.0f);
                const float d = diff * deriv_from_output(g.act, mine);
                g.AL[(size_t)row * g.nl + lane] = mine;
                g.DL[(size_t)row * g.nl + lane] = d;
                dsh[r][lane] = d;
            }
        }
        if (lane == 0) {
            g.loss_rows[row] = e;
            if (g.loss_sums) g.loss_sums[row] = sum_pre[i] + (double)e;
        }
    }
    if (!g.Dprev) return;
    __syncthreads();
    for (int k = k_first; k < g.nin; k += 256 * VEC) {
        const bool first = k == k_first;
        vec_t sum[R];
#pragma unroll
        for (int r = 0; r < R; ++r) sum[r] = 0.f;
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            if (o < g.nl) {
                const vec_t w = first ? w0[o] : *reinterpret_cast<const vec_t *>(g.W + (size_t)o * g.nin + k);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const float dv = dsh[r][o];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) sum[r][v] = fmaf(dv, w[v], sum[r][v]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (row0 + r < g.B) {
                const size_t e = (size_t)(row0 + r) * g.nin + k;
                const vec_t a = first ? a0[r] : *reinterpret_cast<const vec_t *>(g.Aprev + e);
#pragma unroll
                for (int v = 0; v < VEC; ++v) sum[r][v] *= deriv_from_output(g.act_prev, a[v]);
                *reinterpret_cast<vec_t *>(g.Dprev + e) = sum[r];
            }
        }
    }
}

hipError_t launch_narrow_output(const float *Aprev, const float *W, const float *bias, const int32_t *labels,
                                float *AL, float *DL, float *loss_rows, double *loss_sums, int B, int nl, int nin,
                                int act, int loss, hipStream_t stream, float *Dprev, int act_prev)
{
    if (!narrow_layer(nl) || B < 1 || nin < 1) return hipErrorInvalidValue;
    const bool vec = nin % 4 == 0 && ((reinterpret_cast<uintptr_t>(Aprev) | reinterpret_cast<uintptr_t>(W) |
                                        reinterpret_cast<uintptr_t>(Dprev)) & 15) == 0;
    NarrowOutArgs g{Aprev, W, bias, labels, AL, DL, loss_rows, loss_sums, B, nl, nin, act, loss, Dprev, act_prev};
    const int R = B > 1024 ? 4 : 1;
    const unsigned grid = (unsigned)((B + R - 1) / R);
    if (R == 4 && vec) launch_kernel(narrow_output_kernel<4, 4>, dim3(grid), dim3(256), 0, stream, g);
    else if (R == 4) launch_kernel(narrow_output_kernel<4, 1>, dim3(grid), dim3(256), 0, stream, g);
    else if (vec) launch_kernel(narrow_output_kernel<1, 4>, dim3(grid), dim3(256), 0, stream, g);
    else launch_kernel(narrow_output_kernel<1, 1>, dim3(grid), dim3(256), 0, stream, g);
    return hipGetLastError();
}


hipError_t launch_narrow_delta(const float *D, const float *W, const float *Aprev, float *C, int B, int nl, int nin,
                               int act, hipStream_t stream)
{
    if (!narrow_layer(nl) || B < 1 || nin < 1) return hipErrorInvalidValue;
    const bool vec = nin % 4 == 0 && ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(Aprev) |
                                        reinterpret_cast<uintptr_t>(C)) & 15) == 0;
    const int groups = vec ? nin / 4 : nin;
    const unsigned gx = (unsigned)((groups + 255) / 256);
    int rows = (int)(((long)B * gx + 511) / 512);   // about 512 workgroups
    if (rows < 4) rows = 4;
    const unsigned gy = (unsigned)((B + rows - 1) / rows);
    if (vec)
        launch_kernel(narrow_delta_kernel<4>, dim3(gx, gy), dim3(256), 0, stream, D, W, Aprev, C, B, nl, nin, act, rows);
    else
        launch_kernel(narrow_delta_kernel<1>, dim3(gx, gy), dim3(256), 0, stream, D, W, Aprev, C, B, nl, nin, act, rows);
    return hipGetLastError();
}

hipError_t launch_narrow_grad(const float *D, const float *Aprev, float *C, float *V, float *gb, float *vb, int B,
                              int nl, int nin, int mode, float scale, float mu, hipStream_t stream)
{
    if (!narrow_layer(nl) || B < 1 || nin < 1) return hipErrorInvalidValue;
    const bool vec = nin % 4 == 0 && ((reinterpret_cast<uintptr_t>(Aprev) | reinterpret_cast<uintptr_t>(C) |
                                        reinterpret_cast<uintptr_t>(V)) & 15) == 0;
    NarrowGradArgs g{D, Aprev, C, V, gb, vb, B, nl, nin, mode, scale, mu};
    const unsigned grid = (unsigned)(vec ? nin / 4 : nin) + 1;
    if (vec)
        launch_kernel(narrow_grad_kernel<4>, dim3(grid), dim3(256), 0, stream, g);
    else
        launch_kernel(narrow_grad_kernel<1>, dim3(grid), dim3(256), 0, stream, g);
    return hipGetLastError();
}

static unsigned grid_for(size_t count)
{
    size_t g = (count + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    return (unsigned)(g ? g : 1);
}

__global__ __launch_bounds__(256) void descent_kernel(float *__restrict__ p, const float *__restrict__ g, size_t count,
                                                      float lr)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256)
        p[i] = p[i] + (-lr * g[i]);
}

hipError_t launch_update(float *p, float *v, const float *g, size_t count, float lr, float mu,
                         hipStream_t stream)
{
    // without a velocity buffer (momentum 0 only): plain gradient descent
    if (!v) hipLaunchKernelGGL(descent_kernel, dim3(grid_for(count)), dim3(256), 0, stream, p, g, count, lr);
    else hipLaunchKernelGGL(update_kernel, dim3(grid_for(count)), dim3(256), 0, stream, p, v, g, count, lr, mu);
    return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, size_t count, hipStream_t stream)
{
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for(count)), dim3(256), 0, stream, dst, src, count);
    return hipGetLastError();
}

}  // namespace dn
