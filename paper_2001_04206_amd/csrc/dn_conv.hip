// Convolutional and maximum-pooling layers, forward and backward, as stateless calls on device
// tensors (the layer types the paper's engine offers besides the fully connected and softmax ones
// and names as the next to accelerate; it gives no formulas, these are the usual definitions, stated
// in include/dn.h).  Direct (gather) form throughout: every output element is owned by one thread or
// one workgroup, so nothing is accumulated with atomics and every sum has a fixed order.
#include "dn_internal.h"
#include "dn_wave.h"

namespace dn {

namespace {

constexpr int kMaxFilter = 7;   // largest filter edge

__device__ __forceinline__ float conv_act(int act, float z)
{
    switch (act) {
    case DN_ACT_SIGMOID: return 1.0f / (1.0f + expf(-z));
    case DN_ACT_TANH: return tanhf(z);
    case DN_ACT_RELU: return z > 0.0f ? z : 0.0f;
    default: return z;
    }
}

__device__ __forceinline__ float conv_deriv(int act, float a)
{
    switch (act) {
    case DN_ACT_SIGMOID: return a * (1.0f - a);
    case DN_ACT_TANH: return 1.0f - a * a;
    case DN_ACT_RELU: return a > 0.0f ? 1.0f : 0.0f;
    default: return 1.0f;
    }
}

struct ConvShape {
    int B, Cin, H, W, Cout, KH, KW, stride, pad, Ho, Wo, act;
};

// y[b][o][i][j] for CO output channels o at a time: a thread owns one pixel (b, i, j) of a group of
// CO channels, so each input value it loads serves CO filters; filter values are uniform across
// the wave (scalar loads).  Adjacent threads own adjacent j: input rows are read coalesced.
template <int CO>
__global__ __launch_bounds__(256) void conv_forward_kernel(ConvShape s, const float *__restrict__ X,
                                                           const float *__restrict__ Wt,
                                                           const float *__restrict__ bias, float *__restrict__ Y)
{
    const int pix = s.Ho * s.Wo;
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int og = blockIdx.y, b = blockIdx.z;
    if (p >= pix) return;
    const int i = p / s.Wo, j = p - i * s.Wo;
    float acc[CO];
    int oc[CO];
#pragma unroll
    for (int q = 0; q < CO; ++q) {
        oc[q] = min(og * CO + q, s.Cout - 1);   // channels past the end repeat the last one; not stored
        acc[q] = bias[oc[q]];
    }
    const int r0 = i * s.stride - s.pad, c0 = j * s.stride - s.pad;
    for (int ci = 0; ci < s.Cin; ++ci) {
        const float *x = X + ((size_t)b * s.Cin + ci) * s.H * s.W;
        for (int u = 0; u < s.KH; ++u) {
            const int r = r0 + u;
            if (r < 0 || r >= s.H) continue;
            for (int v = 0; v < s.KW; ++v) {
                const int c = c0 + v;
                if (c < 0 || c >= s.W) continue;
                const float xv = x[(size_t)r * s.W + c];
#pragma unroll
                for (int q = 0; q < CO; ++q)
                    acc[q] = fmaf(Wt[(((size_t)oc[q] * s.Cin + ci) * s.KH + u) * s.KW + v], xv, acc[q]);
            }
        }
    }
#pragma unroll
    for (int q = 0; q < CO; ++q)
        if (og * CO + q < s.Cout) Y[((size_t)b * s.Cout + og * CO + q) * pix + p] = conv_act(s.act, acc[q]);
}

__global__ __launch_bounds__(256) void conv_delta_kernel(const float *__restrict__ dA, const float *__restrict__ Y,
                                                         float *__restrict__ delta, size_t count, int act)
{
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (size_t)gridDim.x * 256)
        delta[e] = dA[e] * conv_deriv(act, Y[e]);
}

// dW[o][c][u][v] = (1/B) sum_{b,i,j} delta[b][o][i][j] x[b][c][i*stride+u-pad][j*stride+v-pad]:
// one workgroup per (o, c) pair holds all kh x kw sums; its threads take the positions (b, i, j)
// in turn (adjacent threads adjacent j), each delta value a thread loads serving the whole
// filter window; the threads' partial sums are then added in a fixed order.  Workgroups past the
// (o, c) pairs, one per output channel, add up delta for the bias.
__global__ __launch_bounds__(256) void conv_dw_kernel(ConvShape s, const float *__restrict__ X,
                                                      const float *__restrict__ delta, float *__restrict__ dW,
                                                      float *__restrict__ dbias)
{
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pix = s.Ho * s.Wo;
    const int total = s.B * pix;
    const float inv_b = 1.0f / (float)s.B;
    if ((int)blockIdx.x >= s.Cout * s.Cin) {
        const int o = blockIdx.x - s.Cout * s.Cin;
        float part = 0.f;
        for (int t = tid; t < total; t += 256) {
            const int b = t / pix, p = t - b * pix;
            part += delta[((size_t)b * s.Cout + o) * pix + p];
        }
        part = wave_sum(part);
        if (lane == 0) red[wave] = part;
        __syncthreads();
        if (tid == 0) dbias[o] = ((red[0] + red[1]) + (red[2] + red[3])) * inv_b;
        return;
    }
    const int o = blockIdx.x / s.Cin, c = blockIdx.x - o * s.Cin;
    float acc[kMaxFilter][kMaxFilter];
#pragma unroll
    for (int u = 0; u < kMaxFilter; ++u)
#pragma unroll
        for (int v = 0; v < kMaxFilter; ++v) acc[u][v] = 0.f;
    for (int t = tid; t < total; t += 256) {
        const int b = t / pix, p = t - b * pix;
        const int i = p / s.Wo, j = p - i * s.Wo;
        const float d = delta[((size_t)b * s.Cout + o) * pix + p];
        const float *x = X + ((size_t)b * s.Cin + c) * s.H * s.W;
        const int r0 = i * s.stride - s.pad, c0 = j * s.stride - s.pad;
#pragma unroll
        for (int u = 0; u < kMaxFilter; ++u) {
            if (u < s.KH) {
                const int r = r0 + u;
                const bool row_ok = r >= 0 && r < s.H;
#pragma unroll
                for (int v = 0; v < kMaxFilter; ++v) {
                    if (v < s.KW) {
                        const int cc = c0 + v;
                        const bool ok = row_ok && cc >= 0 && cc < s.W;
                        const float xv = ok ? x[(size_t)r * s.W + cc] : 0.f;
                        acc[u][v] = fmaf(d, xv, acc[u][v]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kMaxFilter; ++u) {
#pragma unroll
        for (int v = 0; v < kMaxFilter; ++v) {
            if (u < s.KH && v < s.KW) {   // uniform
                const float w_sum = wave_sum(acc[u][v]);
                __syncthreads();            // red is free again
                if (lane == 0) red[wave] = w_sum;
                __syncthreads();
                if (tid == 0)
                    dW[(((size_t)o * s.Cin + c) * s.KH + u) * s.KW + v] = ((red[0] + red[1]) + (red[2] + red[3])) * inv_b;
            }
        }
    }
}

// dX[b][c][r][col] = sum over (o, u, v) with r = i*stride+u-pad, col = j*stride+v-pad of
// delta[b][o][i][j] W[o][c][u][v]: a thread owns one input pixel of one channel.
__global__ __launch_bounds__(256) void conv_dx_kernel(ConvShape s, const float *__restrict__ Wt,
                                                      const float *__restrict__ delta, float *__restrict__ dX)
{
    const int hw = s.H * s.W;
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y, b = blockIdx.z;
    if (p >= hw) return;
    const int r = p / s.W, col = p - r * s.W;
    const int pix = s.Ho * s.Wo;
    float acc = 0.f;
    for (int o = 0; o < s.Cout; ++o) {
        const float *d = delta + ((size_t)b * s.Cout + o) * pix;
        const float *wf = Wt + ((size_t)o * s.Cin + c) * s.KH * s.KW;
        for (int u = 0; u < s.KH; ++u) {
            const int ri = r + s.pad - u;
            if (ri < 0 || ri % s.stride != 0) continue;
            const int i = ri / s.stride;
            if (i >= s.Ho) continue;
            for (int v = 0; v < s.KW; ++v) {
                const int cj = col + s.pad - v;
                if (cj < 0 || cj % s.stride != 0) continue;
                const int j = cj / s.stride;
                if (j >= s.Wo) continue;
                acc = fmaf(d[(size_t)i * s.Wo + j], wf[u * s.KW + v], acc);
            }
        }
    }
    dX[((size_t)b * s.Cin + c) * hw + p] = acc;
}

struct PoolShape {
    int planes, H, W, K, stride, Ho, Wo;   // planes = batch * channels
};

__global__ __launch_bounds__(256) void maxpool_forward_kernel(PoolShape s, const float *__restrict__ X,
                                                              float *__restrict__ Y)
{
    const int pix = s.Ho * s.Wo;
    const int p = blockIdx.x * 256 + threadIdx.x, plane = blockIdx.y;
    if (p >= pix) return;
    const int i = p / s.Wo, j = p - i * s.Wo;
    const float *x = X + (size_t)plane * s.H * s.W + (size_t)(i * s.stride) * s.W + j * s.stride;
    float m = x[0];
    for (int u = 0; u < s.K; ++u)
        for (int v = 0; v < s.K; ++v) m = fmaxf(m, x[(size_t)u * s.W + v]);
    Y[(size_t)plane * pix + p] = m;
}

// A thread owns one input pixel: for every window that contains it, it finds the window's first
// maximum (row-major order) again and takes the window's dY if that is its own position.
__global__ __launch_bounds__(256) void maxpool_backward_kernel(PoolShape s, const float *__restrict__ X,
                                                               const float *__restrict__ dY, float *__restrict__ dX)
{
    const int hw = s.H * s.W;
    const int p = blockIdx.x * 256 + threadIdx.x, plane = blockIdx.y;
    if (p >= hw) return;
    const int r = p / s.W, c = p - r * s.W;
    const float *x = X + (size_t)plane * hw;
    const float mine = x[p];
    // windows i with i*stride <= r < i*stride + K
    const int i_hi = min(r / s.stride, s.Ho - 1), j_hi = min(c / s.stride, s.Wo - 1);
    const int i_lo = max(0, (r - s.K + s.stride) / s.stride), j_lo = max(0, (c - s.K + s.stride) / s.stride);
    float acc = 0.f;
    for (int i = i_lo; i <= i_hi; ++i)
        for (int j = j_lo; j <= j_hi; ++j) {
            const float *w0 = x + (size_t)(i * s.stride) * s.W + j * s.stride;
            const int mu = r - i * s.stride, mv = c - j * s.stride;   // own position inside the window
            bool wins = true;
            for (int u = 0; u < s.K && wins; ++u)
                for (int v = 0; v < s.K; ++v) {
                    const float other = w0[(size_t)u * s.W + v];
                    const bool before = u < mu || (u == mu && v < mv);
                    if (before ? other >= mine : other > mine) { wins = false; break; }
                }
            if (wins) acc += dY[((size_t)plane * s.Ho + i) * s.Wo + j];
        }
    dX[(size_t)plane * hw + p] = acc;
}

bool fits_int(long long v) { return v >= 1 && v <= 0x7fffffffLL; }

dn_status conv_shape(int B, int Cin, int H, int W, int Cout, int KH, int KW, int stride, int pad, int act, ConvShape &s)
{
    if (B < 1 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || KH < 1 || KW < 1 || stride < 1 || pad < 0) return DN_ERR_INVALID_ARG;
    if (KH > kMaxFilter || KW > kMaxFilter || pad >= KH || pad >= KW) return DN_ERR_INVALID_ARG;
    if (act == DN_ACT_SOFTMAX) return DN_ERR_UNSUPPORTED;
    if (act < DN_ACT_LINEAR || act > DN_ACT_SOFTMAX) return DN_ERR_INVALID_ARG;
    if (H + 2 * pad < KH || W + 2 * pad < KW) return DN_ERR_INVALID_ARG;
    const int Ho = (H + 2 * pad - KH) / stride + 1, Wo = (W + 2 * pad - KW) / stride + 1;
    if (!fits_int((long long)B * Cin * H * W) || !fits_int((long long)B * Cout * Ho * Wo) ||
        !fits_int((long long)Cout * Cin * KH * KW) || Cout > 65535 || Cin > 65535 || B > 65535)
        return DN_ERR_INVALID_ARG;
    s = ConvShape{B, Cin, H, W, Cout, KH, KW, stride, pad, Ho, Wo, act};
    return DN_OK;
}

dn_status pool_shape(int B, int C, int H, int W, int K, int stride, PoolShape &s)
{
    if (B < 1 || C < 1 || H < 1 || W < 1 || K < 1 || stride < 1 || K > H || K > W) return DN_ERR_INVALID_ARG;
    const int Ho = (H - K) / stride + 1, Wo = (W - K) / stride + 1;
    if (!fits_int((long long)B * C * H * W) || (long long)B * C > 65535) return DN_ERR_INVALID_ARG;
    s = PoolShape{B * C, H, W, K, stride, Ho, Wo};
    return DN_OK;
}

dn_status launched() { return hipGetLastError() == hipSuccess ? DN_OK : DN_ERR_DEVICE; }

}  // namespace

}  // namespace dn

using namespace dn;

extern "C" {

dn_status dn_conv_forward(const float *X_dev, const float *W_dev, const float *bias_dev, float *Y_dev, int32_t batch,
                          int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh, int32_t kw, int32_t stride,
                          int32_t pad, dn_act act, void *hip_stream)
{
    if (!X_dev || !W_dev || !bias_dev || !Y_dev) return DN_ERR_INVALID_ARG;
    ConvShape s;
    const dn_status st = conv_shape(batch, c_in, h, w, c_out, kh, kw, stride, pad, (int)act, s);
    if (st != DN_OK) return st;
    constexpr int CO = 4;
    const dim3 grid((unsigned)((s.Ho * s.Wo + 255) / 256), (unsigned)((s.Cout + CO - 1) / CO), (unsigned)s.B);
    hipLaunchKernelGGL(conv_forward_kernel<CO>, grid, dim3(256), 0, (hipStream_t)hip_stream, s, X_dev, W_dev, bias_dev,
                       Y_dev);
    return launched();
}

dn_status dn_conv_backward(const float *X_dev, const float *W_dev, const float *Y_dev, const float *dA_dev,
                           float *delta_dev, float *dX_dev, float *dW_dev, float *dbias_dev, int32_t batch,
                           int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh, int32_t kw, int32_t stride,
                           int32_t pad, dn_act act, void *hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || !dA_dev || !delta_dev || !dW_dev || !dbias_dev) return DN_ERR_INVALID_ARG;
    ConvShape s;
    const dn_status st = conv_shape(batch, c_in, h, w, c_out, kh, kw, stride, pad, (int)act, s);
    if (st != DN_OK) return st;
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t ny = (size_t)s.B * s.Cout * s.Ho * s.Wo;
    size_t blocks = (ny + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(conv_delta_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dA_dev, Y_dev, delta_dev, ny,
                       s.act);
    if (launched() != DN_OK) return DN_ERR_DEVICE;
    hipLaunchKernelGGL(conv_dw_kernel, dim3((unsigned)(s.Cout * s.Cin + s.Cout)), dim3(256), 0, stream, s, X_dev,
                       delta_dev, dW_dev, dbias_dev);
    if (launched() != DN_OK) return DN_ERR_DEVICE;
    if (dX_dev) {
        const dim3 grid((unsigned)((s.H * s.W + 255) / 256), (unsigned)s.Cin, (unsigned)s.B);
        hipLaunchKernelGGL(conv_dx_kernel, grid, dim3(256), 0, stream, s, W_dev, delta_dev, dX_dev);
        if (launched() != DN_OK) return DN_ERR_DEVICE;
    }
    return DN_OK;
}

dn_status dn_maxpool_forward(const float *X_dev, float *Y_dev, int32_t batch, int32_t channels, int32_t h, int32_t w,
                             int32_t k, int32_t stride, void *hip_stream)
{
    if (!X_dev || !Y_dev) return DN_ERR_INVALID_ARG;
    PoolShape s;
    const dn_status st = pool_shape(batch, channels, h, w, k, stride, s);
    if (st != DN_OK) return st;
    const dim3 grid((unsigned)((s.Ho * s.Wo + 255) / 256), (unsigned)s.planes);
    hipLaunchKernelGGL(maxpool_forward_kernel, grid, dim3(256), 0, (hipStream_t)hip_stream, s, X_dev, Y_dev);
    return launched();
}

dn_status dn_maxpool_backward(const float *X_dev, const float *dY_dev, float *dX_dev, int32_t batch, int32_t channels,
                              int32_t h, int32_t w, int32_t k, int32_t stride, void *hip_stream)
{
    if (!X_dev || !dY_dev || !dX_dev) return DN_ERR_INVALID_ARG;
    PoolShape s;
    const dn_status st = pool_shape(batch, channels, h, w, k, stride, s);
    if (st != DN_OK) return st;
    const dim3 grid((unsigned)((s.H * s.W + 255) / 256), (unsigned)s.planes);
    hipLaunchKernelGGL(maxpool_backward_kernel, grid, dim3(256), 0, (hipStream_t)hip_stream, s, X_dev, dY_dev, dX_dev);
    return launched();
}

}  // extern "C"
