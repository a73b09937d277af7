// A convolutional classifier as one network: convolution (+ maximum pooling) blocks in front of
// a fully connected net, the layer sequence of the paper's engine (section "Deep Netts Deep
// Learning Engine": convolutional, maximum pooling, fully connected, softmax output layers), with
// the work-flow's three training parts (section "The Deep Netts Work-flow") run for every batch
// of an epoch without returning to the host between steps.
//
// Nothing is computed here: every step is one of the library's own entry points (dn_conv_*,
// dn_maxpool_*, dn_forward / dn_backward / dn_input_gradient / dn_update, dn_sgd_step) enqueued
// on one stream in the order of the chain rule.  This file owns the layout of the arena (filters,
// their velocities and gradients, the activations and gradients between the blocks, the
// convolution workspaces, the fully connected net's own arena) and the epoch loop.
#include <hip/hip_runtime.h>

#include <cmath>
#include <new>
#include <vector>

#include "../../include/dn.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int kLossSlots = 4096;   // per-step losses kept on the device between two read-backs

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Block {
    dn_conv_block spec{};
    int c_in = 0, h = 0, w = 0;      // input image
    int ho = 0, wo = 0;              // convolution output
    int hp = 0, wp = 0;              // block output (after pooling, if any)
    size_t filt = 0;                 // c_out * c_in * k * k
    size_t ws_bytes = 0;
    // byte offsets into the arena
    size_t W = 0, b = 0, vW = 0, vb = 0, dW = 0, db = 0;
    size_t Y = 0, P = 0, dOut = 0, dY = 0, delta = 0, ws = 0;
    bool pooled() const { return spec.pool_k > 0; }
    size_t out_per_sample() const { return (size_t)spec.c_out * hp * wp; }
    size_t y_per_sample() const { return (size_t)spec.c_out * ho * wo; }
};

struct Layout {
    std::vector<Block> blocks;
    std::vector<int32_t> widths;     // of the fully connected part: [flat, dense widths ...]
    size_t off_loss = 0, off_dense = 0, dense_bytes = 0, total = 0;
};

// Sizes and offsets of everything; false if a size is invalid or a tensor would pass 2^31 - 1 elements.
bool plan(int32_t c, int32_t h, int32_t w, const dn_conv_block *blocks, int32_t n_blocks, const int32_t *dense_widths,
          int32_t n_dense, int32_t max_batch, Layout &lo)
{
    if (c < 1 || h < 1 || w < 1 || !blocks || n_blocks < 1 || n_blocks > 64 || !dense_widths || n_dense < 1 || max_batch < 1)
        return false;
    const size_t limit = 0x7fffffffu;
    size_t o = 0;
    int ci = c, hi = h, wi = w;
    lo.blocks.assign((size_t)n_blocks, Block{});
    for (int i = 0; i < n_blocks; ++i) {
        Block &bk = lo.blocks[(size_t)i];
        bk.spec = blocks[i];
        const dn_conv_block &s = bk.spec;
        if (s.c_out < 1 || s.k < 1 || s.k > 7 || s.stride < 1 || s.pad < 0 || s.pad >= s.k || s.pool_k < 0 ||
            (s.pool_k > 0 && s.pool_stride < 1) || s.act < DN_ACT_LINEAR || s.act >= DN_ACT_SOFTMAX)
            return false;
        bk.c_in = ci; bk.h = hi; bk.w = wi;
        bk.ho = (hi + 2 * s.pad - s.k) / s.stride + 1;
        bk.wo = (wi + 2 * s.pad - s.k) / s.stride + 1;
        if (hi + 2 * s.pad < s.k || wi + 2 * s.pad < s.k || bk.ho < 1 || bk.wo < 1) return false;
        bk.hp = bk.ho; bk.wp = bk.wo;
        if (bk.pooled()) {
            if (s.pool_k > bk.ho || s.pool_k > bk.wo) return false;
            bk.hp = (bk.ho - s.pool_k) / s.pool_stride + 1;
            bk.wp = (bk.wo - s.pool_k) / s.pool_stride + 1;
        }
        bk.filt = (size_t)s.c_out * ci * s.k * s.k;
        if ((size_t)max_batch * bk.y_per_sample() > limit || (size_t)max_batch * ci * hi * wi > limit || bk.filt > limit)
            return false;
        bk.ws_bytes = dn_conv_backward_workspace_bytes(max_batch, ci, hi, wi, s.c_out, s.k, s.k, s.stride, s.pad);
        if (bk.ws_bytes == 0) return false;
        const size_t fb = bk.filt * sizeof(float), bb = (size_t)s.c_out * sizeof(float);
        bk.W = o; o += align_up(fb);
        bk.b = o; o += align_up(bb);
        bk.vW = o; o += align_up(fb);
        bk.vb = o; o += align_up(bb);
        bk.dW = o; o += align_up(fb);
        bk.db = o; o += align_up(bb);
        const size_t yb = (size_t)max_batch * bk.y_per_sample() * sizeof(float);
        const size_t pb = (size_t)max_batch * bk.out_per_sample() * sizeof(float);
        bk.Y = o; o += align_up(yb);
        bk.delta = o; o += align_up(yb);
        if (bk.pooled()) {
            bk.P = o; o += align_up(pb);
            bk.dY = o; o += align_up(yb);
        }
        bk.dOut = o; o += align_up(pb);
        bk.ws = o; o += align_up(bk.ws_bytes);
        ci = s.c_out; hi = bk.hp; wi = bk.wp;
    }
    const size_t flat = (size_t)ci * hi * wi;
    if (flat > limit) return false;
    lo.widths.clear();
    lo.widths.push_back((int32_t)flat);
    for (int i = 0; i < n_dense; ++i) lo.widths.push_back(dense_widths[i]);
    lo.off_loss = o; o += align_up(kLossSlots * sizeof(float));
    lo.dense_bytes = dn_net_arena_bytes(lo.widths.data(), (int32_t)lo.widths.size(), max_batch);
    if (lo.dense_bytes == 0) return false;
    lo.off_dense = o; o += align_up(lo.dense_bytes);
    lo.total = o;
    return true;
}

}  // namespace

struct dn_cnn {
    Layout lo;
    int c = 0, h = 0, w = 0, max_batch = 0;
    char *arena = nullptr;
    hipStream_t stream = nullptr;
    dn_net *dense = nullptr;
    float *at(size_t off) const { return reinterpret_cast<float *>(arena + off); }
};

namespace {

// Convolution / pooling blocks on `batch` images at X; returns the last block's output.
dn_status blocks_forward(dn_cnn *net, const float *X, int batch, const float **out)
{
    const float *a = X;
    for (Block &bk : net->lo.blocks) {
        const dn_conv_block &s = bk.spec;
        dn_status st = dn_conv_forward(a, net->at(bk.W), net->at(bk.b), net->at(bk.Y), batch, bk.c_in, bk.h, bk.w, s.c_out,
                                       s.k, s.k, s.stride, s.pad, (dn_act)s.act, net->stream);
        if (st != DN_OK) return st;
        a = net->at(bk.Y);
        if (bk.pooled()) {
            st = dn_maxpool_forward(net->at(bk.Y), net->at(bk.P), batch, s.c_out, bk.ho, bk.wo, s.pool_k, s.pool_stride,
                                    net->stream);
            if (st != DN_OK) return st;
            a = net->at(bk.P);
        }
    }
    *out = a;
    return DN_OK;
}

}  // namespace

extern "C" {

size_t dn_cnn_arena_bytes(int32_t c, int32_t h, int32_t w, const dn_conv_block *blocks, int32_t n_blocks,
                          const int32_t *dense_widths, int32_t n_dense, int32_t max_batch)
{
    Layout lo;
    return plan(c, h, w, blocks, n_blocks, dense_widths, n_dense, max_batch, lo) ? lo.total : 0;
}

dn_status dn_cnn_create(int32_t c, int32_t h, int32_t w, const dn_conv_block *blocks, int32_t n_blocks,
                        const int32_t *dense_widths, int32_t n_dense, const dn_act *dense_acts, dn_loss loss,
                        int32_t max_batch, void *arena_dev, size_t arena_bytes, void *hip_stream, dn_cnn **out)
{
    if (!out) return DN_ERR_INVALID_ARG;
    *out = nullptr;
    if (!blocks || !dense_widths || !dense_acts || !arena_dev) return DN_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(arena_dev) & (kAlign - 1)) != 0) return DN_ERR_INVALID_ARG;
    dn_cnn *net = new (std::nothrow) dn_cnn;
    if (!net) return DN_ERR_OOM;
    if (!plan(c, h, w, blocks, n_blocks, dense_widths, n_dense, max_batch, net->lo) || arena_bytes < net->lo.total) {
        delete net;
        return DN_ERR_SHAPE;
    }
    net->c = c; net->h = h; net->w = w; net->max_batch = max_batch;
    net->arena = static_cast<char *>(arena_dev);
    net->stream = static_cast<hipStream_t>(hip_stream);
    // filters, velocities and gradients start at zero, like the parameters of a fully connected net
    for (const Block &bk : net->lo.blocks) {
        if (hipMemsetAsync(net->arena + bk.W, 0, bk.Y - bk.W, net->stream) != hipSuccess) {
            delete net;
            return DN_ERR_DEVICE;
        }
    }
    const dn_status st = dn_net_create(net->lo.widths.data(), (int32_t)net->lo.widths.size(), dense_acts, loss, max_batch,
                                       net->arena + net->lo.off_dense, net->lo.dense_bytes, hip_stream, &net->dense);
    if (st != DN_OK) {
        delete net;
        return st;
    }
    *out = net;
    return DN_OK;
}

dn_status dn_cnn_destroy(dn_cnn *net)
{
    if (!net) return DN_ERR_INVALID_ARG;
    dn_status st = DN_OK;
    if (net->dense) st = dn_net_destroy(net->dense);   // waits for the stream
    delete net;
    return st;
}

dn_net *dn_cnn_dense(dn_cnn *net) { return net ? net->dense : nullptr; }

int32_t dn_cnn_flat_size(const dn_cnn *net) { return net ? net->lo.widths[0] : 0; }

dn_status dn_cnn_set_filters(dn_cnn *net, int32_t block, const float *W_host, const float *bias_host)
{
    if (!net || block < 0 || block >= (int32_t)net->lo.blocks.size()) return DN_ERR_INVALID_ARG;
    const Block &bk = net->lo.blocks[(size_t)block];
    const size_t fb = bk.filt * sizeof(float), bb = (size_t)bk.spec.c_out * sizeof(float);
    if (hipStreamSynchronize(net->stream) != hipSuccess) return DN_ERR_DEVICE;
    if (W_host && (hipMemcpy(net->arena + bk.W, W_host, fb, hipMemcpyHostToDevice) != hipSuccess ||
                   hipMemset(net->arena + bk.vW, 0, fb) != hipSuccess))
        return DN_ERR_DEVICE;
    if (bias_host && (hipMemcpy(net->arena + bk.b, bias_host, bb, hipMemcpyHostToDevice) != hipSuccess ||
                      hipMemset(net->arena + bk.vb, 0, bb) != hipSuccess))
        return DN_ERR_DEVICE;
    return DN_OK;
}

dn_status dn_cnn_get_filters(dn_cnn *net, int32_t block, float *W_host, float *bias_host)
{
    if (!net || block < 0 || block >= (int32_t)net->lo.blocks.size()) return DN_ERR_INVALID_ARG;
    const Block &bk = net->lo.blocks[(size_t)block];
    if (hipStreamSynchronize(net->stream) != hipSuccess) return DN_ERR_DEVICE;
    if (W_host && hipMemcpy(W_host, net->arena + bk.W, bk.filt * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
        return DN_ERR_DEVICE;
    if (bias_host &&
        hipMemcpy(bias_host, net->arena + bk.b, (size_t)bk.spec.c_out * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
        return DN_ERR_DEVICE;
    return DN_OK;
}

dn_status dn_cnn_get_filter_grads(dn_cnn *net, int32_t block, float *dW_host, float *dbias_host)
{
    if (!net || block < 0 || block >= (int32_t)net->lo.blocks.size()) return DN_ERR_INVALID_ARG;
    const Block &bk = net->lo.blocks[(size_t)block];
    if (hipStreamSynchronize(net->stream) != hipSuccess) return DN_ERR_DEVICE;
    if (dW_host && hipMemcpy(dW_host, net->arena + bk.dW, bk.filt * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
        return DN_ERR_DEVICE;
    if (dbias_host &&
        hipMemcpy(dbias_host, net->arena + bk.db, (size_t)bk.spec.c_out * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
        return DN_ERR_DEVICE;
    return DN_OK;
}

dn_status dn_cnn_forward(dn_cnn *net, const float *X_dev, int32_t batch, float *out_dev)
{
    if (!net || !X_dev) return DN_ERR_INVALID_ARG;
    if (batch < 1 || batch > net->max_batch) return DN_ERR_SHAPE;
    const float *a = nullptr;
    const dn_status st = blocks_forward(net, X_dev, batch, &a);
    if (st != DN_OK) return st;
    return dn_forward(net->dense, a, batch, out_dev);
}

dn_status dn_cnn_train_epoch(dn_cnn *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples, int32_t batch,
                             float lr, float momentum, float *mean_loss_host)
{
    if (!net || !X_dev || !labels_dev || n_samples <= 0) return DN_ERR_INVALID_ARG;
    if (!std::isfinite(lr) || !std::isfinite(momentum) || lr < 0.f || momentum < 0.f || momentum >= 1.f)
        return DN_ERR_INVALID_ARG;
    if (batch < 1 || batch > net->max_batch) return DN_ERR_SHAPE;
    const size_t image = (size_t)net->c * net->h * net->w;
    float *loss_slots = net->at(net->lo.off_loss);
    std::vector<float> host_loss((size_t)kLossSlots);
    std::vector<int> step_size;
    double acc = 0.0;
    auto drain = [&]() -> dn_status {   // per-step losses of the steps enqueued since the last read-back
        if (step_size.empty()) return DN_OK;
        if (hipMemcpyAsync(host_loss.data(), loss_slots, step_size.size() * sizeof(float), hipMemcpyDeviceToHost,
                           net->stream) != hipSuccess ||
            hipStreamSynchronize(net->stream) != hipSuccess)
            return DN_ERR_DEVICE;
        for (size_t i = 0; i < step_size.size(); ++i) acc += (double)host_loss[i] * step_size[i];
        step_size.clear();
        return DN_OK;
    };
    const size_t nb = net->lo.blocks.size();
    for (int64_t s0 = 0; s0 < n_samples; s0 += batch) {
        const int B = (int)((n_samples - s0) < batch ? (n_samples - s0) : batch);
        const float *Xb = X_dev + (size_t)s0 * image;
        // part 1: feed forward
        const float *a = nullptr;
        dn_status st = blocks_forward(net, Xb, B, &a);
        if (st != DN_OK) return st;
        if ((st = dn_forward(net->dense, a, B, nullptr)) != DN_OK) return st;
        // parts 2 and 3: loss, then the error backwards through every layer
        if ((st = dn_backward(net->dense, labels_dev + s0, B, loss_slots + step_size.size())) != DN_OK) return st;
        step_size.push_back(B);
        if ((st = dn_input_gradient(net->dense, B, net->at(net->lo.blocks[nb - 1].dOut))) != DN_OK) return st;
        for (size_t i = nb; i-- > 0;) {
            Block &bk = net->lo.blocks[i];
            const dn_conv_block &s = bk.spec;
            const float *dA = net->at(bk.dOut);
            if (bk.pooled()) {
                st = dn_maxpool_backward(net->at(bk.Y), net->at(bk.dOut), net->at(bk.dY), B, s.c_out, bk.ho, bk.wo, s.pool_k,
                                         s.pool_stride, net->stream);
                if (st != DN_OK) return st;
                dA = net->at(bk.dY);
            }
            const float *in = i == 0 ? Xb : (net->lo.blocks[i - 1].pooled() ? net->at(net->lo.blocks[i - 1].P)
                                                                             : net->at(net->lo.blocks[i - 1].Y));
            float *dX = i == 0 ? nullptr : net->at(net->lo.blocks[i - 1].dOut);
            st = dn_conv_backward(in, net->at(bk.W), net->at(bk.Y), dA, net->at(bk.delta), dX, net->at(bk.dW), net->at(bk.db),
                                  net->arena + bk.ws, bk.ws_bytes, B, bk.c_in, bk.h, bk.w, s.c_out, s.k, s.k, s.stride, s.pad,
                                  (dn_act)s.act, net->stream);
            if (st != DN_OK) return st;
        }
        // the update, every layer by the same rule
        if ((st = dn_update(net->dense, lr, momentum)) != DN_OK) return st;
        for (Block &bk : net->lo.blocks) {
            float *vW = momentum != 0.f ? net->at(bk.vW) : nullptr, *vb = momentum != 0.f ? net->at(bk.vb) : nullptr;
            if ((st = dn_sgd_step(net->at(bk.W), net->at(bk.dW), vW, (int64_t)bk.filt, lr, momentum, net->stream)) != DN_OK)
                return st;
            if ((st = dn_sgd_step(net->at(bk.b), net->at(bk.db), vb, bk.spec.c_out, lr, momentum, net->stream)) != DN_OK)
                return st;
        }
        if ((int)step_size.size() == kLossSlots && (st = drain()) != DN_OK) return st;
    }
    const dn_status st = drain();
    if (st != DN_OK) return st;
    if (mean_loss_host) *mean_loss_host = (float)(acc / (double)n_samples);
    return DN_OK;
}

}  // extern "C"
