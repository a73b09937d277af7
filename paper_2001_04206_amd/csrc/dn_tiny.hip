// Per-sample (batch 1) training of very small nets -- every layer at most 64 units wide -- as one
// wavefront that runs the whole epoch.
//
// A net like 4-16-3 has a few hundred weights: spread over workgroups, or even over the waves of one
// workgroup, a training step is nothing but barriers and exchanges.  Here lane j of a single wave is
// unit j of every layer.  Weights, biases, (with momentum) their velocities, the activations and the
// deltas of one sample live in LDS; a step is the textbook sequence -- feed forward, output error and
// loss, deltas through the weights from before the update, rank-1 update of every layer -- with no
// waiting on anybody.  Weight rows sit an odd number of floats apart, so the lanes of a forward
// product (one row each, same column) and of a delta product (same row, one column each) touch
// different LDS banks.  The next sample's features are requested a step ahead.
#include <algorithm>

#include "dn_internal.h"
#include "dn_persist.h"
#include "dn_wave.h"

namespace dn {
namespace {

// L is a template parameter so that the layer loops unroll and every layer's shape and LDS offsets
// stay in scalar registers for the whole epoch (read from the argument block each time, they cost a
// scalar-memory round trip per use, several per layer and step).
template <int L>
__global__ __launch_bounds__(64) void tiny_epoch_kernel(TinyPlan p)
{
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x;
    const int n0 = p.layer[1].n_in, nL = p.layer[L].n_out;
    const bool with_v = p.mu != 0.f;

    // ---- prologue: parameters (and velocities, if they are read) into LDS ----
#pragma unroll
    for (int l = 1; l <= L; ++l) {
        const TinyLayer &ly = p.layer[l];
        for (int e = lane; e < ly.n_out * ly.n_in; e += 64) {
            const int j = e / ly.n_in, k = e - j * ly.n_in;
            lds[ly.lds_w + j * ly.pitch + k] = ly.W[e];
            if (with_v) lds[ly.lds_v + j * ly.pitch + k] = ly.VW[e];
        }
        if (lane < ly.n_out) {
            lds[ly.lds_b + lane] = ly.b[lane];
            if (with_v) lds[ly.lds_vb + lane] = ly.Vb[lane];
        }
    }
    if (lane < n0) lds[p.lds_act[0] + lane] = p.X[lane];
    // Features travel two steps ahead of their use, labels 64 at a time (lane i holds the label of
    // step 64 b + i), both as vector loads: a scalar load in flight would hold up every wait for LDS.
    float x_1 = (1 < p.n_samples && lane < n0) ? p.X[(size_t)n0 + lane] : 0.f;   // features of step s + 1
    int y_block = 0;
    double loss_acc = 0.0;
    __syncthreads();

    for (int64_t s = 0; s < p.n_samples; ++s) {
        const int mode = with_v ? UPD_MOMENTUM : ((p.keep_v && s == p.n_samples - 1) ? UPD_KEEPV : UPD_SGD);
        const float *x = lds + p.lds_act[0] + (int)(s & 1) * 64;
        const bool more = s + 1 < p.n_samples;
        if ((s & 63) == 0) y_block = p.labels[min(s + lane, p.n_samples - 1)];
        const int y_cur = __builtin_amdgcn_readlane(y_block, (int)(s & 63));
        const float x_2 = (s + 2 < p.n_samples && lane < n0) ? p.X[(size_t)(s + 2) * n0 + lane] : 0.f;

        // ---- feed forward: lane j is unit j ----
        const float *ain = x;
#pragma unroll
        for (int l = 1; l <= L; ++l) {
            const TinyLayer &ly = p.layer[l];
            float *aout = lds + p.lds_act[l];
            if (lane < ly.n_out) {
                const float *wr = lds + ly.lds_w + lane * ly.pitch;
                float z = lds[ly.lds_b + lane];
                int k = 0;
                for (; k + 4 <= ly.n_in; k += 4)
                    z += wr[k] * ain[k] + wr[k + 1] * ain[k + 1] + wr[k + 2] * ain[k + 2] + wr[k + 3] * ain[k + 3];
                for (; k < ly.n_in; ++k) z += wr[k] * ain[k];
                aout[lane] = act_fn(ly.act, z);   // a softmax layer keeps its net inputs here
            }
            __syncthreads();
            ain = aout;
        }

        // ---- output error and loss ----
        {
            const TinyLayer &ly = p.layer[L];
            const float *aL = lds + p.lds_act[L];
            int y = y_cur;
            y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
            const bool on = lane < nL;
            const float t = lane == y ? 1.0f : 0.0f;
            float d, e;
            if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                const float z = on ? aL[lane] : -INFINITY;
                const float m = wave_max(z);
                const float ex = on ? expf(z - m) : 0.f;
                const float sum = wave_sum(ex);
                d = ex * (1.0f / sum) - t;
                e = logf(sum) - (aL[y] - m);
            } else {
                const float a = on ? aL[lane] : 0.f;
                const float f = a - t;
                d = f * act_deriv(ly.act, a);
                e = wave_sum(on ? 0.5f * f * f : 0.f);
            }
            if (on) lds[p.lds_dl[L] + lane] = d;
            if (lane == 0) loss_acc += (double)e;
            __syncthreads();
        }

        // ---- back propagation in reverse order: delta of the layer below from the weights before
        //      their update, then the update of this layer ----
#pragma unroll
        for (int l = L; l >= 1; --l) {
            const TinyLayer &ly = p.layer[l];
            const float *dl = lds + p.lds_dl[l];
            const float *aprev = (l == 1) ? x : (lds + p.lds_act[l - 1]);
            float *W = lds + ly.lds_w, *V = lds + ly.lds_v;
            if (l > 1) {
                if (lane < ly.n_in) {   // lane k is unit k of layer l-1
                    float sacc = 0.f;
                    for (int j = 0; j < ly.n_out; ++j) sacc += W[j * ly.pitch + lane] * dl[j];
                    lds[p.lds_dl[l - 1] + lane] = sacc * act_deriv(p.layer[l - 1].act, aprev[lane]);
                }
                __syncthreads();
            }
            // rank-1 update: element e = lane + 64 i of the n_out x n_in matrix, (row, column) advanced
            // by the quotient and remainder of 64 by n_in
            int j = lane / ly.n_in, k = lane - j * ly.n_in;
            for (int e = lane; e < ly.n_out * ly.n_in; e += 64) {
                const int idx = j * ly.pitch + k;
                float v = with_v ? V[idx] : 0.f;
                W[idx] = apply_update(W[idx], (p.lr * dl[j]) * aprev[k], v, p.mu, mode);
                if (mode == UPD_MOMENTUM) V[idx] = v;
                else if (mode == UPD_KEEPV) ly.VW[j * ly.n_in + k] = v;
                j += ly.rs;
                k += ly.ks;
                if (k >= ly.n_in) { k -= ly.n_in; ++j; }
            }
            if (lane < ly.n_out) {
                float v = with_v ? lds[ly.lds_vb + lane] : 0.f;
                lds[ly.lds_b + lane] = apply_update(lds[ly.lds_b + lane], p.lr * dl[lane], v, p.mu, mode);
                if (mode == UPD_MOMENTUM) lds[ly.lds_vb + lane] = v;
                else if (mode == UPD_KEEPV) ly.Vb[lane] = v;
            }
            __syncthreads();
        }

        if (more && lane < n0) lds[p.lds_act[0] + (int)((s + 1) & 1) * 64 + lane] = x_1;
        x_1 = x_2;
        __syncthreads();
    }

    // ---- epilogue: parameters back to device memory ----
#pragma unroll
    for (int l = 1; l <= L; ++l) {
        const TinyLayer &ly = p.layer[l];
        for (int e = lane; e < ly.n_out * ly.n_in; e += 64) {
            const int j = e / ly.n_in, k = e - j * ly.n_in;
            ly.W[e] = lds[ly.lds_w + j * ly.pitch + k];
            if (with_v) ly.VW[e] = lds[ly.lds_v + j * ly.pitch + k];
        }
        if (lane < ly.n_out) {
            ly.b[lane] = lds[ly.lds_b + lane];
            if (with_v) ly.Vb[lane] = lds[ly.lds_vb + lane];
        }
    }
    if (lane == 0) *p.loss_acc += loss_acc;
}

// ---- two-layer nets, plain gradient descent: the whole net in the wave's registers ----
// With two layers the LDS round trips of the kernel above (one per dependent phase, ~120 cycles each,
// and nothing else for the lone wave to do meanwhile) can go entirely.  Lane j is hidden unit j and
// keeps row j of W_1; lane k is output unit k and keeps row k of W_2; lane j also keeps column j of
// W_2 (the weights that leave its unit), so that the delta of unit j is a product of registers too.
// A vector that every lane needs -- the features, the hidden activations, the output deltas -- is
// read lane by lane into scalar registers (one cross-lane read per element) and enters the
// multiply-adds as a scalar operand.  Both copies of W_2 take the same fused multiply-add from the
// same operands and stay equal bit for bit; the row copy goes back to device memory at the end.
// N0 / N1 / N2: compile-time bounds of the three widths (the loops unroll to them; entries past the
// real widths hold zeros).  No LDS, no barrier, nobody to wait for.
__device__ __forceinline__ float lane_read(float v, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

// Elements base .. base + Q - 1 of a vector spread over the lanes, as Q scalar registers at once: the
// empty statement needs all of them together, so the cross-lane reads are issued back to back and
// the multiply-adds that use them follow without the wait states a scalar register needs right after
// a vector instruction has written it.  (Left alone the compiler reads, waits and uses one at a time.)
template <int Q>
struct LaneQ { float v[Q]; };
template <int Q>
__device__ __forceinline__ LaneQ<Q> lane_read_q(float v, int base)
{
    static_assert(Q == 4 || Q == 8, "four or eight at a time");
    LaneQ<Q> r;
#pragma unroll
    for (int q = 0; q < Q; ++q) r.v[q] = lane_read(v, base + q);
    if constexpr (Q == 4)
        asm volatile("" : "+s"(r.v[0]), "+s"(r.v[1]), "+s"(r.v[2]), "+s"(r.v[3]));
    else
        asm volatile("" : "+s"(r.v[0]), "+s"(r.v[1]), "+s"(r.v[2]), "+s"(r.v[3]), "+s"(r.v[4]), "+s"(r.v[5]), "+s"(r.v[6]), "+s"(r.v[7]));
    return r;
}

template <int N0, int N1, int N2>
__global__ __launch_bounds__(64) void tiny_regs_epoch_kernel(TinyPlan p)
{
    constexpr int Q0 = N0 >= 8 ? 8 : 4, Q1 = N1 >= 8 ? 8 : 4, Q2 = N2 >= 8 ? 8 : 4;   // cross-lane reads at a time
    const int lane = threadIdx.x;
    const TinyLayer &l1 = p.layer[1], &l2 = p.layer[2];
    const int n0 = l1.n_in, n1 = l1.n_out, n2 = l2.n_out;
    const bool hid = lane < n1, outl = lane < n2;
    float w1[N0], w2r[N1], w2c[N2];
#pragma unroll
    for (int i = 0; i < N0; ++i) w1[i] = (hid && i < n0) ? l1.W[lane * n0 + i] : 0.f;
#pragma unroll
    for (int j = 0; j < N1; ++j) w2r[j] = (outl && j < n1) ? l2.W[lane * n1 + j] : 0.f;
#pragma unroll
    for (int k = 0; k < N2; ++k) w2c[k] = (hid && k < n2) ? l2.W[k * n1 + lane] : 0.f;
    float b1 = hid ? l1.b[lane] : 0.f, b2 = outl ? l2.b[lane] : 0.f;
    // features travel two steps ahead of their use (lane i holds feature i), labels 64 at a time
    float x_cur = lane < n0 ? p.X[lane] : 0.f;
    float x_1 = (1 < p.n_samples && lane < n0) ? p.X[(size_t)n0 + lane] : 0.f;
    int y_block = 0;
    double loss_acc = 0.0;

    for (int64_t s = 0; s < p.n_samples; ++s) {
        const bool keepv = p.keep_v && s == p.n_samples - 1;   // the epoch's last step also leaves the applied change as velocity
        if ((s & 63) == 0) y_block = p.labels[min(s + lane, p.n_samples - 1)];
        int y = __builtin_amdgcn_readlane(y_block, (int)(s & 63));
        y = y < 0 ? 0 : (y >= n2 ? n2 - 1 : y);
        const float x_2 = (s + 2 < p.n_samples && lane < n0) ? p.X[(size_t)(s + 2) * n0 + lane] : 0.f;

        // ---- feed forward ----
        float z1 = b1;
#pragma unroll
        for (int i = 0; i < N0; i += Q0) {
            const LaneQ<Q0> xs = lane_read_q<Q0>(x_cur, i);
#pragma unroll
            for (int q = 0; q < Q0; ++q) z1 = __builtin_fmaf(w1[i + q], xs.v[q], z1);
        }
        const float a1 = hid ? act_fn(l1.act, z1) : 0.f;
        float z2 = b2;
#pragma unroll
        for (int j = 0; j < N1; j += Q1) {
            const LaneQ<Q1> as = lane_read_q<Q1>(a1, j);
#pragma unroll
            for (int q = 0; q < Q1; ++q) z2 = __builtin_fmaf(w2r[j + q], as.v[q], z2);
        }

        // ---- output error and loss ----
        const float t = lane == y ? 1.0f : 0.0f;
        float d2, e;
        if (p.loss == DN_LOSS_CROSS_ENTROPY) {
            const float z = outl ? z2 : -INFINITY;
            const float m = wave_max(z);
            const float ex = outl ? expf(z - m) : 0.f;
            const float sum = wave_sum(ex);
            d2 = outl ? ex * (1.0f / sum) - t : 0.f;
            e = lane == 0 ? logf(sum) - (lane_read(z2, y) - m) : 0.f;
        } else {
            const float a2 = outl ? act_fn(l2.act, z2) : 0.f;
            const float f = outl ? a2 - t : 0.f;
            d2 = f * act_deriv(l2.act, a2);
            e = 0.5f * f * f;   // this lane's share: the lanes' sums meet once, after the last step
        }
        loss_acc += (double)e;

        // ---- deltas of the hidden units through W_2 as it was ----
        float sacc = 0.f;
#pragma unroll
        for (int k = 0; k < N2; k += Q2) {
            const LaneQ<Q2> ds = lane_read_q<Q2>(d2, k);
#pragma unroll
            for (int q = 0; q < Q2; ++q) sacc = __builtin_fmaf(w2c[k + q], ds.v[q], sacc);
        }
        const float d1 = hid ? sacc * act_deriv(l1.act, a1) : 0.f;

        // ---- updates: w = fma(-(lr delta), input, w) ----
        const float nld2 = -(p.lr * d2), nld1 = -(p.lr * d1);
#pragma unroll
        for (int j = 0; j < N1; j += Q1) {
            const LaneQ<Q1> as = lane_read_q<Q1>(a1, j);
#pragma unroll
            for (int q = 0; q < Q1; ++q) w2r[j + q] = __builtin_fmaf(nld2, as.v[q], w2r[j + q]);
        }
#pragma unroll
        for (int k = 0; k < N2; k += Q2) {
            const LaneQ<Q2> gs = lane_read_q<Q2>(nld2, k);
#pragma unroll
            for (int q = 0; q < Q2; ++q) w2c[k + q] = __builtin_fmaf(gs.v[q], a1, w2c[k + q]);
        }
        b2 += nld2;
#pragma unroll
        for (int i = 0; i < N0; i += Q0) {
            const LaneQ<Q0> xs = lane_read_q<Q0>(x_cur, i);
#pragma unroll
            for (int q = 0; q < Q0; ++q) w1[i + q] = __builtin_fmaf(nld1, xs.v[q], w1[i + q]);
        }
        b1 += nld1;
        if (keepv) {
            // (the widths as the compiler cannot see through them: the bounds tests below would
            // otherwise be computed once before the loop and held in scalar registers through every step)
            int n0v = n0, n1v = n1;
            asm volatile("" : "+s"(n0v), "+s"(n1v));
#pragma unroll
            for (int j = 0; j < N1; ++j)
                if (outl && j < n1v) l2.VW[lane * n1v + j] = nld2 * lane_read(a1, j);
#pragma unroll
            for (int i = 0; i < N0; ++i)
                if (hid && i < n0v) l1.VW[lane * n0v + i] = nld1 * lane_read(x_cur, i);
            if (outl) l2.Vb[lane] = nld2;
            if (hid) l1.Vb[lane] = nld1;
        }
        x_cur = x_1;
        x_1 = x_2;
    }

    // ---- epilogue ----
#pragma unroll
    for (int i = 0; i < N0; ++i)
        if (hid && i < n0) l1.W[lane * n0 + i] = w1[i];
#pragma unroll
    for (int j = 0; j < N1; ++j)
        if (outl && j < n1) l2.W[lane * n1 + j] = w2r[j];
    if (hid) l1.b[lane] = b1;
    if (outl) l2.b[lane] = b2;
    // the lanes' loss sums, added in lane order
    double total = 0.0;
    for (int l = 0; l < 64; ++l) {
        const unsigned lo = __builtin_amdgcn_readlane((int)(__builtin_bit_cast(unsigned long long, loss_acc) & 0xffffffffu), l);
        const unsigned hi = __builtin_amdgcn_readlane((int)(__builtin_bit_cast(unsigned long long, loss_acc) >> 32), l);
        total += __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
    }
    if (lane == 0) *p.loss_acc += total;
}

}  // namespace

// ---- host side -------------------------------------------------------------------

bool tiny_plan(const int32_t *n, int L, bool want_v, TinyPlan &p)
{
    p = TinyPlan{};
    if (L < 1 || L > ON_MAX_L) return false;
    for (int l = 0; l <= L; ++l)
        if (n[l] > 64) return false;
    p.L = L;
    int f = 0;
    p.lds_act[0] = f; f += 2 * 64;                      // the sample's features, two buffers
    for (int l = 1; l <= L; ++l) {
        p.lds_act[l] = f; f += 64;
        p.lds_dl[l] = f; f += 64;
    }
    for (int l = 1; l <= L; ++l) {
        TinyLayer &y = p.layer[l];
        y.n_in = n[l - 1]; y.n_out = n[l];
        y.pitch = n[l - 1] | 1;                          // odd: rows start in different banks
        y.rs = 64 / y.n_in; y.ks = 64 % y.n_in;
        y.lds_w = f; f += y.n_out * y.pitch;
        y.lds_v = f; if (want_v) f += y.n_out * y.pitch;
        y.lds_b = f; f += 64;
        y.lds_vb = f; if (want_v) f += 64;
    }
    if ((size_t)f * sizeof(float) > ON_MAX_LDS_BYTES) return false;
    p.lds_floats = f;
    return true;
}

namespace {

template <int L>
hipError_t tiny_prepare_one()
{
    return hipFuncSetAttribute((const void *)tiny_epoch_kernel<L>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)ON_MAX_LDS_BYTES);
}

template <int L>
void tiny_launch_one(const TinyPlan &plan, hipStream_t stream)
{
    hipLaunchKernelGGL(tiny_epoch_kernel<L>, dim3(1), dim3(64), (size_t)plan.lds_floats * sizeof(float), stream, plan);
}

}  // namespace

hipError_t tiny_prepare()
{
    static_assert(ON_MAX_L == 8, "one instantiation per depth");
    const hipError_t e[] = {tiny_prepare_one<1>(), tiny_prepare_one<2>(), tiny_prepare_one<3>(), tiny_prepare_one<4>(),
                            tiny_prepare_one<5>(), tiny_prepare_one<6>(), tiny_prepare_one<7>(), tiny_prepare_one<8>()};
    for (hipError_t x : e)
        if (x != hipSuccess) return x;
    return hipSuccess;
}

namespace {

// The register form's compile-time bounds: the smallest of {4, 16, 64} x {16, 64} x {4, 16, 64} that holds the widths.
template <int N0, int N1>
void tiny_regs_launch_n2(const TinyPlan &plan, hipStream_t stream)
{
    const int n2 = plan.layer[2].n_out;
    if (n2 <= 4) hipLaunchKernelGGL((tiny_regs_epoch_kernel<N0, N1, 4>), dim3(1), dim3(64), 0, stream, plan);
    else if (n2 <= 16) hipLaunchKernelGGL((tiny_regs_epoch_kernel<N0, N1, 16>), dim3(1), dim3(64), 0, stream, plan);
    else hipLaunchKernelGGL((tiny_regs_epoch_kernel<N0, N1, 64>), dim3(1), dim3(64), 0, stream, plan);
}

template <int N0>
void tiny_regs_launch_n1(const TinyPlan &plan, hipStream_t stream)
{
    if (plan.layer[1].n_out <= 16) tiny_regs_launch_n2<N0, 16>(plan, stream);
    else tiny_regs_launch_n2<N0, 64>(plan, stream);
}

}  // namespace

hipError_t launch_tiny_epoch(const TinyPlan &plan, hipStream_t stream)
{
    if (plan.in_registers) {   // two layers, plain gradient descent: no LDS at all
        if (plan.L != 2 || plan.mu != 0.f) return hipErrorInvalidValue;
        const int n0 = plan.layer[1].n_in;
        if (n0 <= 4) tiny_regs_launch_n1<4>(plan, stream);
        else if (n0 <= 16) tiny_regs_launch_n1<16>(plan, stream);
        else tiny_regs_launch_n1<64>(plan, stream);
        return hipGetLastError();
    }
    switch (plan.L) {
    case 1: tiny_launch_one<1>(plan, stream); break;
    case 2: tiny_launch_one<2>(plan, stream); break;
    case 3: tiny_launch_one<3>(plan, stream); break;
    case 4: tiny_launch_one<4>(plan, stream); break;
    case 5: tiny_launch_one<5>(plan, stream); break;
    case 6: tiny_launch_one<6>(plan, stream); break;
    case 7: tiny_launch_one<7>(plan, stream); break;
    case 8: tiny_launch_one<8>(plan, stream); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace dn
