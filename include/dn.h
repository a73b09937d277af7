/*
 * dn.h -- C ABI of libdn: training of fully connected feed-forward networks
 * on one AMD MI355X (gfx950).
 *
 * The library runs the training loop the paper describes in its section "The
 * Deep Netts Work-flow": feed forward, loss error assessment, back propagation
 * through the layers in reverse order, and the learning-rate scaled update of
 * the weights and biases of every neuron.  The neuron model (net input =
 * weights . inputs + bias, output = activation(net input)) is that of the
 * section "Deep Learning Overview".  The two methods the paper offloads -- the
 * backward step of the fully connected layer and of the softmax output layer
 * (section "How Deep Netts is parallelized with TornadoVM?") -- correspond to
 * dn_backward / dn_update here; dn_train_epoch runs whole epochs with all state
 * resident on the device, which removes the per-call host<->device copies the
 * paper's task schedule performs and names as its main overhead (sections
 * "Performance Analysis" and "Conclusions").
 *
 * Conventions
 *   - All arithmetic and all tensors are fp32, row-major, contiguous.
 *   - Layers l = 1..L, widths n_0 (input) .. n_L (output).  W_l is
 *     [n_l][n_{l-1}], b_l is [n_l].  A batch of B samples is [B][n].
 *   - Labels are int32 class ids in [0, n_L); targets are their one-hot rows
 *     (for squared error too).
 *   - "_dev" pointers are device memory, "_host" pointers host memory.
 *   - The library never allocates or frees device memory: the caller hands it
 *     one arena (dn_net_arena_bytes) that holds parameters, velocities,
 *     gradients, activations, deltas and kernel workspace, and the caller owns
 *     it and every other device buffer.  The arena must stay alive, and must
 *     not be written by the caller, until dn_net_destroy.
 *   - All device work is enqueued on the HIP stream given at creation.
 *     dn_forward / dn_backward / dn_update return without waiting for it;
 *     dn_set_params / dn_get_params / dn_get_grads / dn_train_epoch wait for
 *     the stream before they return.
 *   - Every function returns a dn_status; none throws or aborts.  Arguments
 *     are validated on the host before anything is launched.
 *   - A net is not thread safe; different nets may be used from different
 *     threads.
 */
#ifndef DN_H
#define DN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dn_net dn_net; /* opaque host-side handle */

typedef enum {
    DN_OK = 0,
    DN_ERR_INVALID_ARG = 1, /* NULL pointer, value out of range, call out of order */
    DN_ERR_SHAPE = 2,       /* widths / batch / arena size do not fit */
    DN_ERR_UNSUPPORTED = 3, /* activation / loss combination not provided */
    DN_ERR_OOM = 4,         /* host allocation of the handle failed */
    DN_ERR_DEVICE = 5       /* a HIP call or a kernel reported an error */
} dn_status;

typedef enum {
    DN_ACT_LINEAR = 0,
    DN_ACT_SIGMOID = 1,
    DN_ACT_TANH = 2,
    DN_ACT_RELU = 3,
    DN_ACT_SOFTMAX = 4 /* last layer only, and only with DN_LOSS_CROSS_ENTROPY */
} dn_act;

typedef enum {
    DN_LOSS_MSE = 0,          /* per sample 1/2 sum_k (a_k - y_k)^2 */
    DN_LOSS_CROSS_ENTROPY = 1 /* per sample -log softmax(z)[label]; needs a softmax last layer */
} dn_loss;

/* Short static description of a status code (never NULL). */
const char *dn_status_string(dn_status s);

/*
 * Bytes of device arena a net of these widths needs for batches up to
 * max_batch.  Returns 0 if the arguments are invalid (NULL, n_widths < 2, a
 * width <= 0, max_batch <= 0, or sizes that overflow).
 */
size_t dn_net_arena_bytes(const int32_t *widths, int32_t n_widths, int32_t max_batch);

/*
 * Build a network (the network construction step of section "The Deep Netts
 * Work-flow"; layer types and counts are the configuration parameters it lists).
 *   widths      n_0..n_L, n_widths = L+1 >= 2, all > 0           (host)
 *   acts        L activations, one per layer                     (host)
 *   loss        loss function of the output layer
 *   max_batch   largest batch any later call may pass
 *   arena_dev   device memory, 256-byte aligned, >= dn_net_arena_bytes(...)
 *   hip_stream  a hipStream_t (NULL = the default stream)
 *   out         receives the handle
 * Parameters, velocities and gradients start at zero; call dn_set_params.
 * Errors: INVALID_ARG (NULL, bad enum, misaligned arena), SHAPE (widths,
 * max_batch, arena too small), UNSUPPORTED (softmax not last / softmax without
 * cross-entropy / cross-entropy without softmax), OOM, DEVICE.
 */
dn_status dn_net_create(const int32_t *widths, int32_t n_widths, const dn_act *acts,
                        dn_loss loss, int32_t max_batch, void *arena_dev, size_t arena_bytes,
                        void *hip_stream, dn_net **out);

/* Free the host handle (waits for the stream first).  The arena is the caller's. */
dn_status dn_net_destroy(dn_net *net);

/*
 * Copy parameters of layer `layer` (1..L) between host and device.  W_host is
 * [n_l][n_{l-1}], b_host is [n_l]; either may be NULL to skip it.
 * dn_set_params also zeroes that layer's velocity (the weight and bias
 * initialisation step of section "The Deep Netts Work-flow" is done by the caller,
 * who passes the initial values here).  dn_get_grads reads the batch-mean gradients left by
 * the last dn_backward.
 */
dn_status dn_set_params(dn_net *net, int32_t layer, const float *W_host, const float *b_host);
dn_status dn_get_params(dn_net *net, int32_t layer, float *W_host, float *b_host);
dn_status dn_get_grads(dn_net *net, int32_t layer, float *G_host, float *g_host);

/*
 * Feed forward (training part 1): A_0 = X; Z_l = A_{l-1} W_l^T + b_l;
 * A_l = f_l(Z_l); softmax rows are exp(z - max z) / sum exp(z - max z).
 *   X_dev    [batch][n_0]  (device; read only; must stay valid until the
 *            matching dn_backward has been enqueued and the stream has passed it)
 *   out_dev  [batch][n_L]  (device) receives A_L; may be NULL
 * 1 <= batch <= max_batch, else DN_ERR_SHAPE.
 */
dn_status dn_forward(dn_net *net, const float *X_dev, int32_t batch, float *out_dev);

/*
 * Loss error assessment and back propagation (training parts 2 and 3, without
 * the update) for the batch of the last dn_forward:
 *   output layer    cross-entropy: Delta_L = P - Y ;  squared error:
 *                   Delta_L = (A_L - Y) * f'_L(A_L)
 *   hidden layers   Delta_{l-1} = (Delta_l W_l) * f'_{l-1}(A_{l-1}),  l = L..2
 *   gradients       G_l = (1/B) Delta_l^T A_{l-1},  g_l = (1/B) column sums of Delta_l
 * (for B = 1, G_l is the outer product delta x input that the paper's offloaded
 * two-index loop fills).  Derivatives are taken from the stored activations:
 * sigmoid a(1-a), tanh 1-a^2, ReLU [a>0], linear 1.
 *   labels_dev [batch] int32 (device);  loss_dev (device, 1 float) receives the
 *   batch-mean loss, may be NULL.  batch must equal the last dn_forward's batch
 *   (DN_ERR_SHAPE); calling it before any dn_forward is DN_ERR_INVALID_ARG.
 */
dn_status dn_backward(dn_net *net, const int32_t *labels_dev, int32_t batch, float *loss_dev);

/*
 * Derivative of every sample's loss with respect to that sample's input, for the batch
 * of the last dn_backward: dX = Delta_1 W_1, the delta propagation above taken one layer
 * further (the input has no activation, hence no derivative factor).  Per sample, not a
 * batch mean.  It is what a layer placed in front of the net takes as the derivative with
 * respect to its output (dn_maxpool_backward's dY_dev, dn_conv_backward's dA_dev), which
 * makes the convolutional and pooling layers of the paper's engine ("Deep Netts Deep
 * Learning Engine") trainable in front of a fully connected net.
 *   dX_dev [batch][n_0] (device, written).  batch must equal the last dn_forward's batch
 *   (DN_ERR_SHAPE).  DN_ERR_INVALID_ARG unless dn_backward was the last call to touch the
 *   net's state: W_1 must still be the matrix the deltas were propagated through, so not
 *   after dn_update, dn_set_params of layer 1, a new dn_forward, or the epoch calls.
 */
dn_status dn_input_gradient(dn_net *net, int32_t batch, float *dX_dev);

/*
 * Update from the gradients of the last dn_backward (the paper's
 * learning-rate scaled weight and bias deltas):
 *   dW_l <- momentum * dW_l - lr * G_l ;  W_l <- W_l + dW_l     (same for b_l)
 * momentum = 0 is plain gradient descent.  lr >= 0 and 0 <= momentum < 1 and
 * both finite, else DN_ERR_INVALID_ARG; DN_ERR_INVALID_ARG before any dn_backward.
 */
dn_status dn_update(dn_net *net, float lr, float momentum);

/*
 * One epoch: samples 0..n_samples-1 in index order, `batch` per step (the last
 * step may be short and averages over its own size); each step is forward,
 * loss + back propagation (every delta from the weights as they were before
 * this step's update), update.  Nothing returns to the host between steps.
 *   X_dev [n_samples][n_0], labels_dev [n_samples] int32     (device)
 *   mean_loss_host  receives sum over steps of (step-mean loss * step size) /
 *                   n_samples, each step's loss taken before its update; may be NULL
 * Gradient buffers read by dn_get_grads are not maintained by this call.
 * Errors: INVALID_ARG (NULL, n_samples <= 0, bad lr/momentum), SHAPE (batch
 * outside 1..max_batch), DEVICE.
 */
dn_status dn_train_epoch(dn_net *net, const float *X_dev, const int32_t *labels_dev,
                         int64_t n_samples, int32_t batch, float lr, float momentum,
                         float *mean_loss_host);

/*
 * Training run with the work-flow's stopping rule (section "The Deep Netts Work-flow"): a
 * largest tolerated error is among the configuration parameters, and back propagation goes on
 * while the loss error assessment finds the network above it.  Here the rule is applied per
 * epoch: epochs of dn_train_epoch are run until an epoch's loss (as dn_train_epoch reports
 * it) is <= max_error or max_epochs epochs have run.
 *   epochs_run_host   receives the number of epochs run (>= 1); may be NULL
 *   last_loss_host    receives the last epoch's loss; may be NULL
 * Errors: those of dn_train_epoch; INVALID_ARG also for max_epochs <= 0 or a NaN max_error.
 */
dn_status dn_train(dn_net *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples,
                   int32_t batch, float lr, float momentum, float max_error, int32_t max_epochs,
                   int32_t *epochs_run_host, float *last_loss_host);

/*
 * Loss error assessment without training (the paper's benchmark application ends with a test
 * of the trained network on the held-out part of its data set): feed forward over
 * n_samples samples in chunks of `batch` at the current parameters.
 *   mean_loss_host   receives the mean loss per sample; may be NULL
 *   correct_host     receives the number of samples whose largest output is at the label's
 *                    index (lowest index among equal outputs); may be NULL
 * Parameters are not changed; activations left by dn_forward are overwritten (a following
 * dn_backward needs a new dn_forward).  Errors: INVALID_ARG (NULL, n_samples <= 0), SHAPE
 * (batch outside 1..max_batch), DEVICE.
 */
dn_status dn_evaluate(dn_net *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples,
                      int32_t batch, float *mean_loss_host, int64_t *correct_host);

/*
 * The paper's offloaded method, call for call (section "How Deep Netts is parallelized with
 * TornadoVM?"): the backward step of one layer for one sample as a task that streams its
 * operands in from the host, runs the two-index (inputs x outputs) loop on the device and
 * streams the results out again:
 *     gradients[o][i]    = deltas[o] * inputs[i]
 *     deltaWeights[o][i] = -learning_rate * gradients[o][i]
 *     deltaBiases[o]     = -learning_rate * deltas[o]
 * (the argument list is the one the paper prints for its softmax output layer: deltas, inputs,
 * gradients, deltaWeights, deltaBiases, colsOut, colsInput, learningRate; the sign is read so
 * that a delta is the quantity added to the weight).  It exists to measure that execution
 * model -- copies around every call -- next to the device-resident dn_train_epoch; the paper
 * finds the copies dominate for small data and names their removal as future work.
 *   deltas_host [cols_out], inputs_host [cols_input]                              (host, read)
 *   gradients_host, delta_weights_host [cols_out][cols_input], delta_biases_host [cols_out]
 *                                                                                 (host, written)
 *   workspace_dev   device memory, 256-byte aligned, >= dn_layer_backward_workspace_bytes(...)
 *   hip_stream      stream to work on (NULL = default); the call returns after it has drained
 *   ms_copy_in / ms_kernel / ms_copy_out   device times of the three stages; each may be NULL
 * Errors: INVALID_ARG (NULL, non-finite rate, misaligned workspace), SHAPE (sizes <= 0, more
 * than 2^31 weights, workspace too small), DEVICE.
 */
size_t dn_layer_backward_workspace_bytes(int32_t cols_out, int32_t cols_input);
dn_status dn_layer_backward_host(const float *deltas_host, const float *inputs_host, float learning_rate,
                                 int32_t cols_out, int32_t cols_input, float *gradients_host,
                                 float *delta_weights_host, float *delta_biases_host, void *workspace_dev,
                                 size_t workspace_bytes, void *hip_stream, float *ms_copy_in, float *ms_kernel,
                                 float *ms_copy_out);

/* ---- convolutional and maximum-pooling layers ---------------------------------
 * The two remaining layer types of the engine ("Deep Netts Deep Learning
 * Engine": fully connected, convolutional, maximum pooling, softmax output), which
 * the paper leaves on the CPU and names as the next to accelerate ("Summary").  It
 * gives no formulas for them; these are the usual definitions:
 *   images [batch][channel][row][column] (row-major, dense), filters
 *   [c_out][c_in][kh][kw], zero padding `pad` on all four sides, one stride for
 *   both directions, the filter applied without flipping:
 *     y[b][o][i][j] = f(bias[o] + sum_{c,u,v} W[o][c][u][v] x[b][c][i*stride+u-pad][j*stride+v-pad])
 *   with h_out = (h + 2 pad - kh) / stride + 1 (rounded down), w_out alike.
 *   Backward, from dA = dE/dy of every sample: delta = dA * f'(y) (f' from the stored
 *   output), dW and dbias = means over the batch of the per-sample gradients (as for
 *   the dense layers), dX = dE/dx per sample.
 *   Pooling: window k x k, stride s, no padding, h_out = (h - k) / s + 1; backward
 *   adds dY to the position of each window's maximum (the first in row-major window
 *   order among equals); windows may overlap.
 * These calls are stateless: every pointer is device memory owned by the caller, work
 * is enqueued on `hip_stream` (NULL = default stream) and nothing is synchronised.
 * All tensors fp32.
 * Errors: NULL pointers (dX_dev may be NULL: then no input gradient is computed),
 * sizes < 1, kh or kw > 7, pad >= kh or kw, an empty output, or more than 2^31 - 1
 * elements in a tensor -> DN_ERR_INVALID_ARG; softmax as activation ->
 * DN_ERR_UNSUPPORTED; launch failures -> DN_ERR_DEVICE.
 */
dn_status dn_conv_forward(const float *X_dev, const float *W_dev, const float *bias_dev, float *Y_dev,
                          int32_t batch, int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh,
                          int32_t kw, int32_t stride, int32_t pad, dn_act act, void *hip_stream);
/* delta_dev [batch][c_out][h_out][w_out] is written (the layer's error term, read by
 * the other outputs' kernels); dW_dev [c_out][c_in][kh][kw], dbias_dev [c_out],
 * dX_dev [batch][c_in][h][w] or NULL.  workspace_dev: device memory of at least
 * dn_conv_backward_workspace_bytes(...) bytes (partial sums of the filter and bias gradients
 * over chunks of the batch, and a rearranged copy of the filters for the input gradient; 0
 * from the query means the sizes are invalid); too small ->
 * DN_ERR_SHAPE.  Sums are taken in a fixed order: results are bitwise reproducible. */
size_t dn_conv_backward_workspace_bytes(int32_t batch, int32_t c_in, int32_t h, int32_t w, int32_t c_out,
                                        int32_t kh, int32_t kw, int32_t stride, int32_t pad);
dn_status dn_conv_backward(const float *X_dev, const float *W_dev, const float *Y_dev, const float *dA_dev,
                           float *delta_dev, float *dX_dev, float *dW_dev, float *dbias_dev,
                           void *workspace_dev, size_t workspace_bytes, int32_t batch, int32_t c_in, int32_t h,
                           int32_t w, int32_t c_out, int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                           dn_act act, void *hip_stream);
/*
 * dn_conv_backward for callers that cannot allocate device memory at the point of the call and
 * have no workspace to pass (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same launches, with the workspace taken from a fixed array that lives
 * in the library's device image.  No device or host memory is allocated or freed by the call.
 *   - Limit: the layer's dn_conv_backward_workspace_bytes(...) must not exceed
 *     dn_conv_backward_static_limit() (32 MiB); larger layers -> DN_ERR_SHAPE, nothing launched.
 *   - Every device the library runs on holds its own copy of the array (32 MiB of device memory
 *     per device until the process ends).  The first call on a device looks its address up once;
 *     that device must be current, as for every other call here.
 *   - All calls on one device share the array: two calls whose device work may overlap (different
 *     streams, or different host threads on one device) race on it.  Calls on one stream are
 *     ordered and safe.  The array keeps the previous call's contents; each call writes every
 *     word it reads before reading it, so nothing needs clearing.
 * Arguments, results and all other errors are those of dn_conv_backward; results are the same bits.
 */
dn_status dn_conv_backward_static(const float *X_dev, const float *W_dev, const float *Y_dev, const float *dA_dev,
                                  float *delta_dev, float *dX_dev, float *dW_dev, float *dbias_dev, int32_t batch,
                                  int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh, int32_t kw,
                                  int32_t stride, int32_t pad, dn_act act, void *hip_stream);
size_t dn_conv_backward_static_limit(void);
dn_status dn_maxpool_forward(const float *X_dev, float *Y_dev, int32_t batch, int32_t channels, int32_t h,
                             int32_t w, int32_t k, int32_t stride, void *hip_stream);
/* dX_dev [batch][channels][h][w] is overwritten (not accumulated into). */
dn_status dn_maxpool_backward(const float *X_dev, const float *dY_dev, float *dX_dev, int32_t batch,
                              int32_t channels, int32_t h, int32_t w, int32_t k, int32_t stride,
                              void *hip_stream);

/*
 * The update rule of dn_update for parameters the caller keeps itself (the filters and
 * biases of a convolutional layer):  d <- momentum * d - lr * G ;  P <- P + d.
 *   param_dev, grad_dev [count] (device); velocity_dev [count] (device) holds d between
 *   calls (zero it before the first) and may be NULL when momentum is 0.
 * Errors: INVALID_ARG (NULL param / grad, rates outside lr >= 0, 0 <= momentum < 1 or not
 * finite, momentum > 0 without a velocity buffer), SHAPE (count < 1), DEVICE.
 */
dn_status dn_sgd_step(float *param_dev, const float *grad_dev, float *velocity_dev, int64_t count, float lr,
                      float momentum, void *hip_stream);

/* ---- a convolutional classifier as one network ---------------------------------
 * The layer sequence of the paper's engine (section "Deep Netts Deep Learning Engine":
 * convolutional, maximum pooling, fully connected and softmax output layers) as one
 * object: n_blocks blocks of [convolution -> activation -> optional maximum pooling] on
 * images [c][h][w], the last block's output flattened ([channel][row][column] order) into
 * a fully connected net of widths [flat, dense_widths[0], ..., dense_widths[n_dense-1]].
 * dn_cnn_train_epoch runs the work-flow's three training parts (section "The Deep Netts
 * Work-flow") for every batch of an epoch -- feed forward through every layer, loss, the
 * error backwards through every layer (each delta from the parameters as they were before
 * this step's update), then the update of every layer by the rule of dn_update -- without
 * returning to the host between steps.  Every step is one of the calls above, enqueued on
 * one stream; results are those calls' results.
 *   blocks        n_blocks >= 1 descriptions (host): square k x k filters (k <= 7, pad < k),
 *                 `act` a dn_act other than softmax, pool_k = 0 for no pooling
 *   dense_widths  n_dense >= 1 widths after the flatten (host); dense_acts one dn_act each
 *   arena_dev     device memory, 256-byte aligned, >= dn_cnn_arena_bytes(...) (0 from the
 *                 query: invalid sizes); holds filters, their velocities and gradients, the
 *                 activations and gradients between the layers, the convolution workspaces
 *                 and the fully connected net's arena.  It must stay alive, and must not be
 *                 written by the caller, until dn_cnn_destroy.
 * Filters, biases and velocities start at zero: call dn_cnn_set_filters (W_host
 * [c_out][c_in][k][k], bias_host [c_out]; either may be NULL; zeroes that block's
 * velocity) and, for the fully connected part, dn_set_params on dn_cnn_dense(net), a handle
 * that lives as long as the dn_cnn and must not be destroyed by the caller (layer l of it
 * is the l-th fully connected layer; dn_cnn_flat_size gives its n_0).
 * dn_cnn_get_filter_grads reads the batch-mean filter gradients of the last training step.
 * dn_cnn_forward: out_dev [batch][n_L] (device) receives the output layer; may be NULL.
 * dn_cnn_train_epoch: X_dev [n_samples][c][h][w], labels_dev [n_samples] int32 (device);
 * samples in index order, `batch` per step, the last step may be short; mean_loss_host as
 * for dn_train_epoch.
 * Errors: INVALID_ARG (NULL, misaligned arena, bad rates, block index), SHAPE (invalid
 * sizes, arena too small, batch outside 1..max_batch), UNSUPPORTED / OOM / DEVICE as for
 * dn_net_create and the layer calls.
 */
typedef struct dn_cnn dn_cnn;
typedef struct {
    int32_t c_out, k, stride, pad; /* convolution */
    int32_t act;                   /* dn_act applied to its output */
    int32_t pool_k, pool_stride;   /* maximum pooling after it; pool_k = 0: none */
} dn_conv_block;
size_t dn_cnn_arena_bytes(int32_t c, int32_t h, int32_t w, const dn_conv_block *blocks, int32_t n_blocks,
                          const int32_t *dense_widths, int32_t n_dense, int32_t max_batch);
dn_status dn_cnn_create(int32_t c, int32_t h, int32_t w, const dn_conv_block *blocks, int32_t n_blocks,
                        const int32_t *dense_widths, int32_t n_dense, const dn_act *dense_acts, dn_loss loss,
                        int32_t max_batch, void *arena_dev, size_t arena_bytes, void *hip_stream, dn_cnn **out);
dn_status dn_cnn_destroy(dn_cnn *net);
dn_net *dn_cnn_dense(dn_cnn *net);
int32_t dn_cnn_flat_size(const dn_cnn *net);
dn_status dn_cnn_set_filters(dn_cnn *net, int32_t block, const float *W_host, const float *bias_host);
dn_status dn_cnn_get_filters(dn_cnn *net, int32_t block, float *W_host, float *bias_host);
dn_status dn_cnn_get_filter_grads(dn_cnn *net, int32_t block, float *dW_host, float *dbias_host);
dn_status dn_cnn_forward(dn_cnn *net, const float *X_dev, int32_t batch, float *out_dev);
dn_status dn_cnn_train_epoch(dn_cnn *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples,
                             int32_t batch, float lr, float momentum, float *mean_loss_host);

/*
 * Measurement hooks (the paper times its two offloaded methods with wall-clock
 * timers, section "Experimental Evaluation"; here the device itself is timed).
 *
 * dn_last_epoch_ms: milliseconds the device spent between the first and the
 * last kernel of the last dn_train_epoch, from HIP events on the net's stream.
 *
 * dn_kernel_time: with dn_set_option("time_kernels", 1), every kernel launch of
 * dn_train_epoch is timed with a pair of HIP events on the net's stream (up to
 * 16384 launches per epoch; later ones run untimed).  The launches of the
 * launch-per-product path carry their events themselves (the kernel's own start
 * and end, as a profiler's kernel trace shows them); a persistent whole-epoch
 * kernel is bracketed by recorded events.  After the epoch this returns, for
 * one kernel class, the summed duration and the number of timed launches.
 */
typedef enum {
    DN_K_FORWARD = 0,     /* Z = A W^T + b, activation                       */
    DN_K_DELTA = 1,       /* Delta_{l-1} = (Delta_l W_l) * f' (a narrow last layer's gradient may ride along) */
    DN_K_GRAD_UPDATE = 2, /* G = Delta^T A / B and bias gradient, fused with the update; several layers may share a launch */
    DN_K_OUTPUT = 3,      /* softmax / loss / Delta_L and loss reduction     */
    DN_K_ONLINE = 4,      /* persistent whole-epoch kernels                  */
    DN_K_CLASSES = 5
} dn_kernel_class;

dn_status dn_last_epoch_ms(dn_net *net, float *epoch_ms);
/* How the last dn_train_epoch of this net ran its steps (the epoch loop of section "The Deep Netts
 * Work-flow"): DN_SCHED_NONE before the first call. */
enum {
    DN_SCHED_NONE = 0,
    DN_SCHED_LAUNCHES = 1,        /* one launch per product (or per few products) of every step */
    DN_SCHED_PER_SAMPLE = 2,      /* batch 1: the general persistent whole-epoch kernel */
    DN_SCHED_TWO_COPY = 3,        /* batch 1: the persistent kernel with row and column copies of the inner weights */
    DN_SCHED_MINIBATCH = 4,       /* the persistent minibatch kernel for one- and two-layer nets */
    DN_SCHED_MINIBATCH_DEEP = 5,  /* the persistent minibatch kernel for deeper nets */
    DN_SCHED_ONE_WAVE = 6,        /* batch 1, every layer at most 64 wide: one wavefront runs the epoch */
    DN_SCHED_WIDE_HIDDEN = 7,     /* batch 1, two layers, a hidden layer too wide for LDS: rows in LDS, registers and memory */
    DN_SCHED_ONE_WAVE_REGISTERS = 8, /* batch 1, two layers at most 64 wide, no momentum: one wavefront, the net in its registers */
    DN_SCHED_ONE_WORKGROUP = 9     /* batch 1, two layers, no momentum, W_1 within one compute unit's registers: one workgroup
                                      (the last few samples of a call may run on another batch-1 schedule) */
};
dn_status dn_last_schedule(dn_net *net, int32_t *schedule);
dn_status dn_kernel_time(dn_net *net, int32_t kernel_class, float *ms_total, int64_t *launches);
/* Algorithmic floating-point operations (2 x rows x columns x contraction length per product)
 * of the timed launches of one class of the last dn_train_epoch; 0 for the classes that are not
 * matrix products (DN_K_OUTPUT, DN_K_ONLINE). */
dn_status dn_kernel_flops(dn_net *net, int32_t kernel_class, double *flops);

/*
 * Tuning and diagnostics switches (all default 0):
 *   "time_kernels"   1: collect per-launch times in dn_train_epoch (see above)
 *   "gemm_variant"   -1 (default): pick the tile configuration of each
 *                    contraction from its shape; >= 0: force that configuration
 *   "split_k"        1 (default): forward / delta products with few output tiles split k across
 *                    workgroups (partials summed in a fixed order); 0: never
 *   "merge_launches" 1 (default): the gradient / update products of a backward pass, independent of one
 *                    another once every delta exists, share one launch where their shapes allow; 0: one
 *                    launch per product
 *   "online_mode"    0: choose automatically; 1: per-phase launches for batch 1;
 *                    2: persistent whole-epoch kernel for batch 1 (dn_train_epoch
 *                    returns DN_ERR_UNSUPPORTED if the net does not fit it: more than
 *                    8 layers, an output layer wider than 128, or too wide for LDS)
 *   "batch_mode"     minibatches: 0: choose automatically (a persistent whole-epoch minibatch
 *                    kernel while a step is launch bound); 1: always one launch per product;
 *                    2: always a persistent kernel (DN_ERR_UNSUPPORTED from dn_train_epoch if
 *                    the net fits none.  One or two layers: max_batch <= 256, n_0 <= 2048 and a
 *                    multiple of 4, output width <= 128, LDS.  Three to eight layers: momentum 0,
 *                    max_batch <= 64, every width but the last a multiple of 4, output width
 *                    <= 128, LDS)
 *   "online_min_tile"  weights of one layer a workgroup of the persistent kernel should
 *                    own before the layer is spread over more workgroups (default 4096)
 *   "online_resident"  1 (default): the persistent kernel keeps its weight slices in LDS
 *                    when they fit; 0: always stream them from device memory
 *   "online_twin"    1 (default): batch 1 with momentum 0 on a net of two to eight layers, every
 *                    width but the last a multiple of 4, whose slices fit in LDS (the inner layers'
 *                    twice, the last layer whole), runs on the persistent kernel that keeps a row copy
 *                    and a column copy of the inner weights and repeats the last layer in every
 *                    workgroup (no partial sums cross workgroups); 0: always the general persistent kernel
 *   "online_wide"    1 (default): batch 1 on a two-layer net whose hidden layer does not fit in LDS,
 *                    with at most 384 inputs (a multiple of 4) and at most 16 outputs -- the paper's
 *                    340-100000-10 network -- runs on the persistent kernel that keeps most rows of W_1
 *                    (with momentum: and of its velocities) in LDS and in registers for the whole epoch
 *                    and streams the rest; 0: such nets take the general persistent kernel
 *   "online_solo"    1 (default): batch 1 without momentum on a two-layer net with at most 256 hidden units,
 *                    at most 16 outputs and at most 1568 / 784 / 392 inputs (for up to 64 / 128 / 256
 *                    hidden units) runs on ONE workgroup that keeps W_1 in its registers and reads the
 *                    samples through scalar loads; 0: such nets take the other batch-1 schedules
 *   "online_tiny"    1 (default): batch 1 on a net whose layers are all at most 64 wide (and whose
 *                    parameters fit in LDS, twice with momentum) runs on a single wavefront that keeps
 *                    the whole net in LDS -- in its registers, for two layers and momentum 0; 2: the
 *                    same wavefront, always with the net in LDS; 0: such nets take the other batch-1
 *                    schedules
 * Unknown names or values out of range give DN_ERR_INVALID_ARG.
 */
dn_status dn_set_option(dn_net *net, const char *name, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* DN_H */
