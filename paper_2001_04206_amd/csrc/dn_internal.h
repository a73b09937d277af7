// Internal declarations shared by the host API (dn_api.hip) and the kernel
// launchers (dn_gemm.hip, dn_small.hip).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dn.h"

namespace dn {

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
};

// Enqueue one contraction on `stream`.  Returns hipSuccess or the launch error.
// `variant` < 0 picks a tile configuration from the shape; >= 0 forces one.
hipError_t launch_gemm(GemmKind kind, const GemmArgs &a, int variant, hipStream_t stream);
int gemm_variant_count();
const char *gemm_variant_name(int variant);

// ---- small kernels -----------------------------------------------------------
// Output layer: softmax (cross-entropy: in place on A_L, which holds z after the forward
// contraction), per-sample loss, Delta_L.  One workgroup per sample.
enum OutPhase : int {
    OUT_FUSED = 0,         // z -> p, Delta_L, loss            (training step)
    OUT_SOFTMAX_ONLY = 1,  // z -> p                           (dn_forward; labels unused)
    OUT_FROM_P = 2         // p -> Delta_L, loss               (dn_backward)
};
hipError_t launch_output_delta(float *AL, float *DL, const int32_t *labels, float *loss_rows,
                               int B, int nL, int act, int loss, int phase, hipStream_t stream);
// Sum loss_rows[0..B): *loss_mean_out = sum / B (if non-null); *epoch_acc += sum (if non-null).
hipError_t launch_loss_reduce(const float *loss_rows, int B, float *loss_mean_out,
                              double *epoch_acc, hipStream_t stream);
// Elementwise update of a parameter vector from a stored gradient (dn_update).
hipError_t launch_update(float *p, float *v, const float *g, size_t count, float lr, float mu,
                         hipStream_t stream);
hipError_t launch_copy(float *dst, const float *src, size_t count, hipStream_t stream);

}  // namespace dn
