// Internal declarations shared by the host API (dn_api.hip) and the kernel
// launchers (dn_gemm.hip, dn_small.hip).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/dn.h"

namespace dn {

// Per-launch timing.  Events recorded around a launch also count the time between the marker and
// the kernel's start (measured: 2.4 us, a sixth of a 14 us product); events handed to the launch
// itself carry the kernel's own start and end, as a profiler's trace shows them.  The caller that
// wants its next launch timed leaves an event pair here (per host thread); launch_kernel binds
// the pair to the kernel and says so in `bound`.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
    bool bound = false;
};
LaunchEvents &launch_events();

template <class K, class... Args>
inline void launch_kernel(K kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, Args... args)
{
    LaunchEvents &ev = launch_events();
    if (ev.start && !ev.bound) {
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, ev.start, ev.stop, 0, args...);
        ev.bound = true;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
    }
}

// ---- contraction kernels ---------------------------------------------------
// C[m][n] = sum_k A(m,k) * B(k,n), followed by one of the fused epilogues.
// An operand is either contiguous along k ("KC": row-major [m][k] resp. [n][k])
// or contiguous along its own m/n index ("MC": stored [k][m] resp. [k][n]).
enum GemmKind : int {
    GEMM_FWD = 0,    // A = A_{l-1} [B][n_in] (KC), B = W_l [n_out][n_in] (KC): Z = A W^T; + bias, activation
    GEMM_DELTA = 1,  // A = Delta_l [B][n_l] (KC), B = W_l [n_l][n_{l-1}] (MC): (Delta W) * f'(A_{l-1})
    GEMM_GRAD = 2,   // A = Delta_l stored [B][n_l] (MC), B = A_{l-1} stored [B][n_{l-1}] (MC): Delta^T A, and the
                     // column sums of Delta (bias gradient) computed by the first tile column
    GEMM_KINDS = 3
};

enum GradMode : int {
    GRAD_STORE = 0,      // G = acc / B
    GRAD_SGD = 1,        // W += -(lr/B) acc                         (velocity untouched)
    GRAD_SGD_KEEPV = 2,  // dW = -(lr/B) acc ; V = dW ; W += dW       (velocity written, not read)
    GRAD_MOMENTUM = 3    // dW = mu V - (lr/B) acc ; V = dW ; W += dW
};

struct GemmArgs {
    const float *A;  // first operand
    const float *B;  // second operand
    int lda, ldb;    // leading dimensions (elements) of the stored matrices
    int M, N, K;
    // epilogue
    float *C;          // FWD: A_l ; DELTA: Delta_{l-1} ; GRAD_STORE: G ; update modes: W (in place)
    int ldc;
    const float *bias; // FWD
    int act;           // FWD: activation of this layer (softmax stores z) ; DELTA: activation of layer l-1
    const float *aux;  // DELTA: A_{l-1} [M][ldc]
    float *V;          // update modes: velocity, same shape as W
    float *gb;         // GEMM_GRAD: bias gradient (GRAD_STORE) or bias b_l updated in place (update modes)
    float *vb;         // GEMM_GRAD update modes: bias velocity
    float scale;       // GRAD_STORE: 1/B ; update modes: lr/B
    float mu;          // GRAD_MOMENTUM
    int mode;          // GradMode for GEMM_GRAD
    // k split across workgroups (FWD / DELTA with few output tiles): workspace for the partial
    // tiles and one arrival counter per tile (zero before the launch; left zero by it).
    // ws == nullptr: never split.  sk is chosen by launch_gemm.
    float *ws;
    unsigned *counters;
    size_t ws_floats;  // capacity of ws
    int n_counters;    // capacity of counters
    int sk;
};

constexpr size_t GEMM_WS_FLOATS = (size_t)2 << 20;  // 8 MB of partial tiles
constexpr int GEMM_COUNTERS = 1024;

// Enqueue one contraction on `stream`.  Returns hipSuccess or the launch error.
// `variant` < 0 picks a tile configuration from the shape; >= 0 forces one.
hipError_t launch_gemm(GemmKind kind, const GemmArgs &a, int variant, hipStream_t stream);
// A delta product through W_{l-1} and the gradient / update of a NARROW layer l (at most 16
// outputs, vector units) in one launch: the two do not depend on each other.
bool delta_narrow_grad_fits(const GemmArgs &delta, const GemmArgs &grad, int variant);
hipError_t launch_delta_with_narrow_grad(const GemmArgs &delta, const GemmArgs &grad, hipStream_t stream);
// The gradient / update products of several layers (GEMM_GRAD, same mode), which no longer depend
// on one another once every delta of the backward pass exists: those whose shapes suit it share
// one launch, the rest are launched one by one.  merged_out: products in the shared launch.
hipError_t launch_gemm_grads(const GemmArgs *grads, int n, int variant, bool merge, hipStream_t stream, int *merged_out);
// The selection launch_gemm_grads makes: in_shared[i] says whether product i goes into the shared launch.
void gemm_grads_plan(const GemmArgs *grads, int n, int variant, bool merge, bool *in_shared, int *merged_out);
int gemm_variant_count();
const char *gemm_variant_name(int variant);

// ---- small kernels -----------------------------------------------------------
// Output layer: softmax (cross-entropy: in place on A_L, which holds z after the forward
// contraction), per-sample loss, Delta_L.  One workgroup per sample.
enum OutPhase : int {
    OUT_FUSED = 0,         // z -> p, Delta_L, loss            (training step)
    OUT_SOFTMAX_ONLY = 1,  // z -> p                           (dn_forward; labels unused)
    OUT_FROM_P = 2,        // p -> Delta_L, loss               (dn_backward)
    OUT_EVAL = 3           // z (cross-entropy) or a (squared error) -> loss and hit flag, rows untouched (dn_evaluate)
};
// hit_rows (OUT_EVAL only): 1.0 where the row's largest output is at the label, else 0.0.
// loss_sums (optional, phases that produce a loss): loss_sums[row] += the row's loss.
hipError_t launch_output_delta(float *AL, float *DL, const int32_t *labels, float *loss_rows,
                               int B, int nL, int act, int loss, int phase, hipStream_t stream,
                               float *hit_rows = nullptr, double *loss_sums = nullptr);
// Sum loss_rows[0..B): *loss_mean_out = sum / B (if non-null); *epoch_acc += sum (if non-null).
hipError_t launch_loss_reduce(const float *loss_rows, int B, float *loss_mean_out,
                              double *epoch_acc, hipStream_t stream);
// *epoch_acc += sum of loss_sums[0..B) (the per-row running sums of launch_output_delta).
hipError_t launch_loss_sums_reduce(const double *loss_sums, int B, double *epoch_acc, hipStream_t stream);
// Products of a layer with at most 16 outputs, without the matrix cores (same results as
// launch_gemm's GEMM_DELTA / GEMM_GRAD for that layer, same fused stores and updates).
bool narrow_layer(int n_out);
// C[b][j] = f'(Aprev[b][j]) * sum_o D[b][o] W[o][j];  D [B][nl], W [nl][nin], Aprev and C [B][nin], all dense.
hipError_t launch_narrow_delta(const float *D, const float *W, const float *Aprev, float *C, int B, int nl, int nin,
                               int act, hipStream_t stream);
// sum_b D[b][o] Aprev[b][j] into C / V [nl][nin] and the column sums of D into gb / vb, per GradMode.
hipError_t launch_narrow_grad(const float *D, const float *Aprev, float *C, float *V, float *gb, float *vb, int B,
                              int nl, int nin, int mode, float scale, float mu, hipStream_t stream);
// Last layer with at most 16 outputs, training step: forward product, then softmax / loss / Delta_L as
// launch_output_delta's phase OUT_FUSED, in one launch.  Aprev [B][nin], W [nl][nin], AL and DL [B][nl].
// Dprev (optional, [B][nin]): also receives Delta_{L-1} = (Delta_L W_L) * f'_{act_prev}(Aprev), as
// launch_narrow_delta would compute it.
hipError_t launch_narrow_output(const float *Aprev, const float *W, const float *bias, const int32_t *labels,
                                float *AL, float *DL, float *loss_rows, double *loss_sums, int B, int nl, int nin,
                                int act, int loss, hipStream_t stream, float *Dprev = nullptr, int act_prev = 0);
// Elementwise update of a parameter vector from a stored gradient (dn_update).
hipError_t launch_update(float *p, float *v, const float *g, size_t count, float lr, float mu,
                         hipStream_t stream);
hipError_t launch_copy(float *dst, const float *src, size_t count, hipStream_t stream);
// One sample's backward outputs of one layer (gradients, lr-scaled weight and bias deltas).
hipError_t launch_layer_backward(const float *deltas, const float *inputs, float lr, int cols_out, int cols_in,
                                 float *G, float *dW, float *dB, hipStream_t stream);

// ---- persistent batch-1 epoch kernel (dn_online.hip) ----------------------------
constexpr int ON_MAX_L = 8;         // layers
constexpr int ON_MAX_WG = 256;      // workgroups (one per compute unit)
constexpr int ON_MAX_NL = 128;      // width of the output layer
constexpr int ON_THREADS = 512;     // threads per workgroup
constexpr int ON_TMP_FLOATS = 4096; // reduction scratch in LDS
constexpr size_t ON_MAX_LDS_BYTES = 156 * 1024;
constexpr int ON_DEFAULT_MIN_TILE = 4096;  // weights a workgroup should own per layer before rows are spread further

// How the layers are cut into per-workgroup slices, where the exchange buffers sit inside
// the exchange region (in 64-bit words) and where each piece of LDS starts (in floats).
struct OnlineGeom {
    bool ok;
    int L, grid;
    int per[ON_MAX_L + 1];    // rows per workgroup (layers < L); columns per workgroup (layer L)
    int P[ON_MAX_L + 1];      // workgroups that own a slice of the layer
    int kf[ON_MAX_L + 1];     // forward: segments a row's dot product is split into (a power of two)
    int kshift[ON_MAX_L + 1]; // log2 of it
    int seg[ON_MAX_L + 1];    // forward: segment length
    int vec4[ON_MAX_L + 1];   // rows are whole float4s
    size_t off_act[ON_MAX_L + 1], off_part[ON_MAX_L + 1], off_z, words;
    int lds_x, lds_a[ON_MAX_L + 1], lds_own_a[ON_MAX_L + 1], lds_own_d[ON_MAX_L + 1];
    int lds_b[ON_MAX_L + 1];  // own biases, then their velocities
    int lds_w[ON_MAX_L + 1], lds_v[ON_MAX_L + 1];   // own weight / velocity slices when resident
    int resident;             // bit l: layer l's slices are kept in LDS
    int part_rows;            // layer 1 not resident: this many rows of each workgroup's block are kept in LDS anyway
    int lds_out, lds_kpart, lds_tmp, lds_work_floats, lds_floats;
};

struct OnlineLayer {
    float *W, *b, *VW, *Vb;
    int n_in, n_out, act, per, P, kshift, seg, vec4;
};

struct OnlinePlan {
    int L;
    OnlineLayer layer[ON_MAX_L + 1];            // 1..L
    unsigned long long *act_x[ON_MAX_L + 1];    // [2][n_l]            activations of layers 1..L-2
    unsigned long long *part_x[ON_MAX_L + 1];   // [2][P_l][n_{l-1}]   partials of W_l^T delta_l, l = 2..L-1
    unsigned long long *z_x;                    // [2][P_L][n_L]       partials of the output net inputs
    int *abort_flag;
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    float lr, mu;
    int loss, keep_v;
    uint32_t seq0;                              // step numbers seq0+1 .. seq0+n_samples stamp the exchange words
    int lds_x, lds_a[ON_MAX_L + 1], lds_own_a[ON_MAX_L + 1], lds_own_d[ON_MAX_L + 1];
    int lds_b[ON_MAX_L + 1], lds_w[ON_MAX_L + 1], lds_v[ON_MAX_L + 1];
    int resident;                               // bit l: layer l's weight slice is kept in LDS for the whole launch
    int part_rows;                              // rows of layer 1's block kept in LDS when the whole block does not fit
    int lds_out, lds_kpart, lds_tmp;
};

// ---- persistent minibatch epoch kernel for nets of one or two layers (dn_online.hip) ----
// Same ownership as the per-sample kernel (rows of W_1, matching columns of the last layer),
// B samples per step.  With at most two layers the only data that crosses workgroups are the
// partial net inputs of the output layer and its deltas.
constexpr int PB_MAX_BATCH = 256;
constexpr int PB_MAX_N0 = 2048;       // a sample's features are held in registers: 8 float4 per lane
constexpr int PB_MAX_ROWS = 16;       // rows of W_1 per workgroup
constexpr int PB_MAX_OUT_FLOATS = 8192;   // batch x (n_L + 1) in LDS

struct BatchGeom {
    bool ok;
    int L, grid, per, P, spw;   // per: hidden units (L = 2) or input features (L = 1) per workgroup; spw: samples per workgroup in the output stage
    size_t off_z, off_d, words;
    int lds_w1, lds_v1, lds_b1, lds_w2, lds_v2, lds_bL, lds_a1, lds_d1, lds_d2, lds_zs, lds_tmp, lds_floats;
};

struct BatchPlan {
    int L;
    float *W1, *b1, *VW1, *Vb1;     // L = 2 only
    float *W2, *b2, *VW2, *Vb2;     // the last layer [nL][n_mid]
    int n0, n_mid, nL, act1, actL;  // n_mid: width feeding the last layer (n_1, or n_0 when L = 1)
    int per, P, spw, max_batch;
    unsigned long long *z_x;        // [2][P][max_batch * nL]     partial net inputs of the output layer
    unsigned long long *d_x;        // [2][max_batch * (nL + 1)]  output deltas and per-sample losses
    int *abort_flag;
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    int batch;
    float lr, mu;
    int loss, keep_v, with_v;
    uint32_t seq0;
    int lds_w1, lds_v1, lds_b1, lds_w2, lds_v2, lds_bL, lds_a1, lds_d1, lds_d2, lds_zs, lds_tmp;
};

bool batch_geometry(const int32_t *n, int L, int max_batch, int min_tile, bool want_v, BatchGeom &g);
size_t batch_exchange_bytes_bound(const int32_t *n, int L, int max_batch);
hipError_t batch_prepare();
hipError_t launch_batch_epoch(const BatchGeom &g, const BatchPlan &plan, hipStream_t stream);

// ---- persistent minibatch epoch kernel for deeper nets, plain gradient descent (dn_online.hip) ----
// Every hidden layer is owned by rows as before; to keep the backward pass free of partial sums
// over workgroups, a workgroup also keeps, for each layer l >= 2, a second copy of the weights that
// leave its own units of layer l-1 (the columns of W_l, stored transposed) and updates both copies
// with the same arithmetic.  What crosses workgroups is then only whole activation / delta matrices
// of the batch, written once and read by everyone.
constexpr int PD_MAX_BATCH = 64;

struct DeepGeom {
    bool ok;
    int L, grid, spw, halves;
    int per[ON_MAX_L + 1], P[ON_MAX_L + 1];
    size_t off_z, off_d, off_ea[ON_MAX_L + 1], off_ed[ON_MAX_L + 1], off_fa[ON_MAX_L + 1], off_fd[ON_MAX_L + 1], bytes;
    int lds_r[ON_MAX_L + 1], lds_ct[ON_MAX_L + 1], lds_b[ON_MAX_L + 1], lds_a[ON_MAX_L + 1], lds_dl[ON_MAX_L + 1];
    int lds_w2, lds_bL, lds_d2, lds_zs, lds_tmp, lds_floats;
};

struct DeepLayer {
    float *W, *b, *VW, *Vb;
    int n_in, n_out, act, per, P;
};

struct DeepPlan {
    int L;
    DeepLayer layer[ON_MAX_L + 1];
    int grid, spw, max_batch, halves;
    unsigned long long *z_x, *d_x;                 // as in the two-layer kernel, over `grid` producers
    float *ea[ON_MAX_L + 1], *ed[ON_MAX_L + 1];    // [2][max_batch][n_l]: activations (l = 1..L-2), deltas (l = 2..L-1)
    unsigned long long *fa[ON_MAX_L + 1], *fd[ON_MAX_L + 1];   // [2][grid] "my slice is written" stamps
    int *abort_flag;
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    int batch;
    float lr;
    int loss, keep_v;
    uint32_t seq0;
    int lds_r[ON_MAX_L + 1], lds_ct[ON_MAX_L + 1], lds_b[ON_MAX_L + 1], lds_a[ON_MAX_L + 1], lds_dl[ON_MAX_L + 1];
    int lds_w2, lds_bL, lds_d2, lds_zs, lds_tmp;
};

bool deep_geometry(const int32_t *n, int L, int max_batch, int min_tile, DeepGeom &g);
size_t deep_exchange_bytes_bound(const int32_t *n, int L, int max_batch);
hipError_t deep_prepare();
hipError_t launch_deep_epoch(const DeepGeom &g, const DeepPlan &plan, hipStream_t stream);

// ---- persistent batch-1 epoch kernel with two copies of the inner weights (dn_twin.hip) ----
// Plain gradient descent, two or more layers, everything resident in LDS.  A workgroup owns a
// block of units of every hidden layer and keeps their rows of W_l (forward, update) and, for
// l >= 2, the columns of W_l that leave its units of layer l-1 (stored transposed: delta
// propagation without partial sums over workgroups); the narrow last layer is kept whole by every
// workgroup.  Both copies of a weight receive the same fused multiply-add from the same operands,
// so they stay equal bit for bit.  What crosses workgroups per step: the activation vectors of
// layers 1..L-1 and the delta vectors of layers L-1..2, one stamped word per number.
struct TwinGeom {
    bool ok;
    int L, grid;
    int per[ON_MAX_L + 1], P[ON_MAX_L + 1];            // hidden layers 1..L-1: units per workgroup, owners
    int r_kshift[ON_MAX_L + 1], r_seg[ON_MAX_L + 1];   // own rows x a_{l-1}: segments per row (log2), segment length
    int c_kshift[ON_MAX_L + 1], c_seg[ON_MAX_L + 1];   // own columns x delta_l, l = 2..L-1
    size_t off_act[ON_MAX_L + 1], off_dl[ON_MAX_L + 1], words;   // exchange region, in 64-bit words
    int lds_x, lds_a[ON_MAX_L + 1], lds_d, lds_own_a[ON_MAX_L + 1], lds_own_d[ON_MAX_L + 1], lds_b[ON_MAX_L + 1];
    int lds_r[ON_MAX_L + 1], lds_c[ON_MAX_L + 1], lds_wL, lds_out, lds_kpart, lds_floats;
};

struct TwinLayer {
    float *W, *b, *VW, *Vb;
    int n_in, n_out, act, per, P, r_kshift, r_seg, c_kshift, c_seg;
    // a thread walks an LDS tile of rows of n floats in strides of ON_THREADS float4s: quotient and
    // remainder of that stride by n, and 1 / n, for tiles with rows of n_in (r_*) and n_out (c_*) floats
    float inv_in, inv_out;
    int r_rs, r_ks, c_rs, c_ks;
};

struct TwinPlan {
    int L;
    TwinLayer layer[ON_MAX_L + 1];              // 1..L
    unsigned long long *act_x[ON_MAX_L + 1];    // [2][n_l]  activations of layers 1..L-1
    unsigned long long *dl_x[ON_MAX_L + 1];     // [2][n_l]  deltas of layers 2..L-1
    int *abort_flag;
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    float lr;
    int loss, keep_v;
    uint32_t seq0;
    int lds_x, lds_a[ON_MAX_L + 1], lds_d, lds_own_a[ON_MAX_L + 1], lds_own_d[ON_MAX_L + 1], lds_b[ON_MAX_L + 1];
    int lds_r[ON_MAX_L + 1], lds_c[ON_MAX_L + 1], lds_wL, lds_out, lds_kpart;
};

// false if the net does not suit the kernel (fewer than two layers, a width that is not a multiple
// of 4, output layer too wide, slices beyond LDS).
bool twin_geometry(const int32_t *n, int L, int min_tile, TwinGeom &g);
size_t twin_exchange_bytes_bound(const int32_t *n, int L);
hipError_t twin_prepare();
hipError_t launch_twin_epoch(const TwinGeom &g, const TwinPlan &plan, hipStream_t stream);

// ---- batch-1 epochs of two-layer nets with a wide hidden layer and a narrow output layer (dn_wide.hip) ----
// A workgroup (256 threads: one wave per SIMD, so a lane may hold 512 registers) owns a block of hidden
// units; their rows of W_1 live in LDS, in registers (WIDE_REG_ROWS rows per group of sixteen lanes,
// WIDE_NI float4 pieces per lane and row) and, for the rest, in device memory.  What crosses workgroups
// per step: one partial net input per output unit and workgroup.
constexpr int WIDE_THREADS = 256;
constexpr int WIDE_NI = 6;          // rows of at most 64 * WIDE_NI = 384 inputs
constexpr int WIDE_REG_ROWS = 12;   // 24 registers each per lane: 288 of a lane's 512 (13 rows spill)
constexpr int WIDE_REG_ROWS_MOMENTUM = 4;   // with momentum a row brings its velocities: 48 registers each
constexpr int WIDE_MAX_NL = 16;     // output units
struct WideGeom {
    bool ok;
    int per, grid;        // hidden units per workgroup, workgroups
    int lds_rows;         // rows of a workgroup's block that live in LDS
    size_t words;         // exchange region, in 64-bit words
    int lds_x, lds_a, lds_d, lds_b, lds_z, lds_w2, lds_vb, lds_vw2, lds_zall, lds_out, lds_w1, lds_floats;
};

struct WidePlan {
    float *W1, *b1, *W2, *b2, *VW1, *Vb1, *VW2, *Vb2;
    unsigned long long *z_x;    // [2][grid][nL] partial net inputs of the output layer
    int *abort_flag;
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    int n0, n1, nL, act1, actL, loss, per, lds_rows, keep_v;
    float lr, mu;
    uint32_t seq0;
    int lds_x, lds_a, lds_d, lds_b, lds_z, lds_w2, lds_vb, lds_vw2, lds_zall, lds_out, lds_w1;
};

// false if the net does not suit the kernel (not two layers, inputs not a multiple of 4 or above 384,
// more than 16 outputs, or a hidden layer whose rows all fit in LDS anyway).
bool wide_geometry(const int32_t *n, int L, int max_wg, bool want_v, WideGeom &g);
size_t wide_exchange_bytes_bound(const int32_t *n, int L);
hipError_t wide_prepare();
hipError_t launch_wide_epoch(const WideGeom &g, const WidePlan &plan, hipStream_t stream);

// ---- batch-1 epochs of very small nets on one wavefront (dn_tiny.hip) ----
// Every width at most 64: lane j is unit j of each layer; parameters, activations and deltas in LDS.
struct TinyLayer {
    float *W, *b, *VW, *Vb;
    int n_in, n_out, act;
    int pitch;                    // floats between rows of W_l in LDS (odd)
    int rs, ks;                   // quotient and remainder of 64 by n_in
    int lds_w, lds_v, lds_b, lds_vb;
};

struct TinyPlan {
    int L;
    TinyLayer layer[ON_MAX_L + 1];                   // 1..L
    int lds_act[ON_MAX_L + 1], lds_dl[ON_MAX_L + 1]; // activations (0: the features, two buffers) and deltas
    double *loss_acc;
    const float *X;
    const int32_t *labels;
    int64_t n_samples;
    float lr, mu;
    int loss, keep_v;
    int lds_floats;
    int in_registers;   // two-layer nets without momentum may take the form that keeps the net in registers
};

// Fills the shape-dependent fields; false if a layer is wider than 64 or the parameters (with their
// velocities if want_v) exceed LDS.
bool tiny_plan(const int32_t *n, int L, bool want_v, TinyPlan &p);
hipError_t tiny_prepare();
hipError_t launch_tiny_epoch(const TinyPlan &plan, hipStream_t stream);

// ---- two-layer nets on one workgroup (dn_solo.hip) ----
constexpr int SOLO_THREADS = 512;   // eight waves, two per SIMD: 256 registers a lane
constexpr int SOLO_MAX_OUT = 16;

struct SoloGeom {
    int ug;           // groups of 64 hidden units (1, 2 or 4); 8 / ug column segments
    int c;            // columns of W_1 per lane (the kernel is compiled per value)
    int tail_steps;   // last steps of a sample array the kernel must not be given (its reads would pass the array's end)
};

struct SoloPlan {
    float *W1, *b1, *W2, *b2, *VW1, *Vb1, *VW2, *Vb2;
    double *loss_acc;
    const float *X;          // only ever read (the kernel reads it through the constant address space)
    const int32_t *labels;
    int64_t n_samples;
    int n0, n1, n2, act1, act2, loss, keep_v;
    float lr;
};

// False unless the net has two layers, at most 256 hidden units, at most SOLO_MAX_OUT outputs and a
// row of W_1 fits the registers of the lanes that share it.
bool solo_geometry(const int32_t *n, int L, SoloGeom &g);
hipError_t launch_solo_epoch(const SoloGeom &g, const SoloPlan &plan, hipStream_t stream);

// Slices and buffer offsets for widths n[0..L]; false if the net does not fit the kernel
// (too many layers, output layer too wide, LDS).  want_v: velocity slices are read every step
// (momentum), so they must fit in LDS next to the weights for the slices to be resident.
bool online_geometry(const int32_t *n, int L, int min_tile, bool want_v, OnlineGeom &g);
// Upper bound of the exchange region in bytes for any min_tile (0 if the net can never fit).
size_t online_exchange_bytes_bound(const int32_t *n, int L);
hipError_t online_prepare();
hipError_t launch_online_epoch(const OnlineGeom &g, const OnlinePlan &plan, hipStream_t stream);

}  // namespace dn
