// Row-wise and elementwise kernels of a training step: output-layer error
// (softmax, loss, Delta_L), loss reduction, and the elementwise parameter
// update used by dn_update.
#include "dn_internal.h"

namespace dn {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

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
    hipLaunchKernelGGL(output_delta_kernel, dim3(B), dim3(256), 0, stream, AL, DL, labels, loss_rows, nL, act,
                       loss, phase, hit_rows, loss_sums);
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

static unsigned grid_for(size_t count)
{
    size_t g = (count + 255) / 256;
    if (g > 256 * 16) g = 256 * 16;
    return (unsigned)(g ? g : 1);
}

hipError_t launch_update(float *p, float *v, const float *g, size_t count, float lr, float mu,
                         hipStream_t stream)
{
    hipLaunchKernelGGL(update_kernel, dim3(grid_for(count)), dim3(256), 0, stream, p, v, g, count, lr, mu);
    return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, size_t count, hipStream_t stream)
{
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for(count)), dim3(256), 0, stream, dst, src, count);
    return hipGetLastError();
}

}  // namespace dn
