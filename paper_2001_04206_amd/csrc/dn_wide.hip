// Per-sample (batch 1) training, with or without momentum, of two-layer nets whose hidden layer is
// too wide for LDS and whose output layer is narrow -- the shape of the network the paper trains
// (340 inputs, 100000 hidden units, 10 softmax outputs; section "Experimental Evaluation") -- as
// ONE persistent kernel per epoch that keeps most of W_1 on the chip.
//
// A workgroup owns a block of hidden units: their rows of W_1, their biases, their columns of W_2.
// What a step needs from other workgroups is one number per output unit and workgroup (the partial
// net inputs of the output layer), exchanged as stamped words (dn_persist.h); everything else is
// local.  The cost of a step is then the sweep over the own rows of W_1 -- the rank-1 update
// W_1[r] -= lr delta_r x, fused with the next sample's product z_r = W_1[r] x' on the row while it
// is at hand -- and the sweep is as fast as the rows are near:
//   tier 1   rows in LDS (what is left of it after the small vectors and the columns of W_2);
//   tier 2   rows in REGISTERS: sixteen lanes share a row, a lane keeps its 6 float4 pieces of RR
//            rows for the whole launch (24 RR registers), so 16 RR rows per workgroup never leave
//            the register file between the launch's first and last step;
//   tier 3   the remaining rows stream from and to device memory, 8 bytes per weight and step.
// A workgroup has 256 threads, one wave per SIMD, which lets a lane hold 512 registers (256 plus the
// 256 accumulation registers, which the compiler uses as a second home for values it cannot keep in
// the first 256): the sweep's working set is about 170 registers per lane whatever the thread count,
// so fewer, fatter threads leave more of the register file to the weights.  RR = 12 keeps 288
// registers per lane for them.  For the paper's network (391 rows of 340 floats per workgroup) that is
// 93 rows in LDS, 192 in registers and 106 streamed: a quarter of the bytes the all-streaming sweep moves.
// With momentum every row brings its row of velocities along, in the same tier (LDS rows side by side,
// 48 registers per register row, four of them; streamed rows move 16 bytes per weight and step).
// At the end of the launch tiers 1 and 2, the biases and the columns of W_2 go back to device memory.
#include <algorithm>
#include <type_traits>

#define DN_PERSIST_THREADS 256   // = WIDE_THREADS
#include "dn_internal.h"
#include "dn_persist.h"
#include "dn_wave.h"

namespace dn {
namespace {

static_assert(kThreads == WIDE_THREADS, "the thread count is set before dn_persist.h is included");
constexpr int WNI = WIDE_NI;   // float4 pieces of a row per lane (rows of up to 64 * WNI floats)
constexpr int kPass = kWaves * 4;   // rows a workgroup works on at a time: sixteen lanes each

// This lane's pieces of a vector of n4 float4s (zeros past the end).
__device__ __forceinline__ void lane_pieces(v4f (&dst)[WNI], const float *src, int n4, int g)
{
#pragma unroll
    for (int j = 0; j < WNI; ++j) {
        const int c = g + 16 * j;
        dst[j] = c < n4 ? *(const v4f *)(src + 4 * c) : (v4f){0.f, 0.f, 0.f, 0.f};
    }
}

__device__ __forceinline__ float dot_pieces(const v4f (&w)[WNI], const v4f (&x)[WNI])
{
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < WNI; ++j) acc += w[j].x * x[j].x + w[j].y * x[j].y + w[j].z * x[j].z + w[j].w * x[j].w;
    return acc;
}

// A lane's part of one row: its pieces of the weights and, with momentum, of the velocities.
template <bool MOM>
struct RowPart {
    v4f w[WNI];
    v4f v[WNI];
};
template <>
struct RowPart<false> {
    v4f w[WNI];
};

__device__ __forceinline__ v4f fma4(float s, const v4f &a, const v4f &w)
{
    return (v4f){__builtin_fmaf(s, a.x, w.x), __builtin_fmaf(s, a.y, w.y), __builtin_fmaf(s, a.z, w.z), __builtin_fmaf(s, a.w, w.w)};
}

// The update of one row part by the rule of dn_update, g = (lr delta_r) a_k:
//   plain gradient descent   w = fma(-(lr delta_r), a_k, w)
//   momentum                 v = fma(mu, v, -(lr delta_r) a_k);  w = w + v
template <bool MOM>
__device__ __forceinline__ void update_piece(RowPart<MOM> &r, int j, float nld, float mu, const v4f (&a4)[WNI])
{
    if constexpr (MOM) {
        r.v[j] = fma4(mu, r.v[j], a4[j] * nld);
        r.w[j] = r.w[j] + r.v[j];
    } else {
        r.w[j] = fma4(nld, a4[j], r.w[j]);
    }
}

// Rows in memory (LDS or device): nr rows of n floats at Wt (their velocities at Vt); row r of the
// block takes delta dl[r] and leaves its product with the next sample in out[r].  Sixteen lanes per
// row, four rows per wave at a time, RU such groups in flight.  A pass is split in two -- its loads,
// and everything that needs them -- so that other work can be put between the two.  Loads are
// unconditional (clamped addresses); columns past the end hold zeros in a4 / x4 and are never stored.
// Without momentum Vt is written only when keepv is set (the applied change, for a later momentum epoch).
template <bool MOM, int RU>
__device__ __forceinline__ void pass_load(RowPart<MOM> (&r)[RU], const float *__restrict__ Wt, const float *__restrict__ Vt,
                                          int n, int nr, int base)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int n4 = n >> 2;
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int row = base + u * kPass + wave * 4 + sg;
        const size_t at = (size_t)min(row, nr - 1) * n;
#pragma unroll
        for (int j = 0; j < WNI; ++j) {
            const int c4 = 4 * min(g + 16 * j, n4 - 1);
            r[u].w[j] = *(const v4f *)(Wt + at + c4);
            if constexpr (MOM) r[u].v[j] = *(const v4f *)(Vt + at + c4);
        }
    }
}

template <bool MOM, bool UPDATE, bool DOT, int RU>
__device__ __forceinline__ void pass_finish(RowPart<MOM> (&r)[RU], float *__restrict__ Wt, float *__restrict__ Vt, int n, int nr,
                                            int base, const float *dl, const v4f (&a4)[WNI], const v4f (&x4)[WNI], float lr,
                                            float mu, bool keepv, float *out)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int n4 = n >> 2;
#pragma unroll
    for (int u = 0; u < RU; ++u) {
        const int row = base + u * kPass + wave * 4 + sg;
        const bool rin = row < nr;
        const int rc = min(row, nr - 1);
        if (UPDATE) {
            const float nld = -(lr * dl[rc]);
            const size_t at = (size_t)rc * n;
#pragma unroll
            for (int j = 0; j < WNI; ++j) {
                const int c = g + 16 * j;
                update_piece<MOM>(r[u], j, nld, mu, a4);
                if (rin && c < n4) {
                    *(v4f *)(Wt + at + 4 * c) = r[u].w[j];
                    if constexpr (MOM) {
                        *(v4f *)(Vt + at + 4 * c) = r[u].v[j];
                    } else {
                        if (keepv) *(v4f *)(Vt + at + 4 * c) = a4[j] * nld;
                    }
                }
            }
        }
        if (DOT) {
            const float acc = row16_sum(dot_pieces(r[u].w, x4));
            if (g == 0 && rin) out[row] = acc;
        }
    }
}

template <bool MOM, bool UPDATE, bool DOT, int RU>
__device__ __forceinline__ void sweep_mem(float *__restrict__ Wt, float *__restrict__ Vt, int n, int nr, const float *dl,
                                          const v4f (&a4)[WNI], const v4f (&x4)[WNI], float lr, float mu, bool keepv, float *out,
                                          int first_base = 0)
{
    for (int base = first_base; base < nr; base += kPass * RU) {
        RowPart<MOM> r[RU];
        pass_load<MOM, RU>(r, Wt, Vt, n, nr, base);
        pass_finish<MOM, UPDATE, DOT, RU>(r, Wt, Vt, n, nr, base, dl, a4, x4, lr, mu, keepv, out);
    }
}

// A row in registers: r is this lane's part of row `row` of the tier (nr rows).
template <bool MOM, bool UPDATE, bool DOT>
__device__ __forceinline__ void reg_row(RowPart<MOM> &r, int row, float *__restrict__ Vt, int n, int nr, const float *dl,
                                        const v4f (&a4)[WNI], const v4f (&x4)[WNI], float lr, float mu, bool keepv, float *out)
{
    const int g = threadIdx.x & 15;
    const int n4 = n >> 2;
    const bool rin = row < nr;
    const int rc = rin ? row : 0;
    if (UPDATE) {
        const float nld = rin ? -(lr * dl[rc]) : 0.f;
#pragma unroll
        for (int j = 0; j < WNI; ++j) {
            update_piece<MOM>(r, j, nld, mu, a4);
            if (!MOM && keepv && rin && g + 16 * j < n4) *(v4f *)(Vt + (size_t)rc * n + 4 * (g + 16 * j)) = a4[j] * nld;
        }
    }
    if (DOT) {
        const float acc = row16_sum(dot_pieces(r.w, x4));
        if (g == 0 && rin) out[row] = acc;
    }
}

// The three tiers of a workgroup's rows: streamed (ns rows at Ws), registers (nrr), LDS (nl rows at Wl,
// with momentum their velocities at Vl); local row numbers run LDS, registers, streamed.  V: the
// block's rows of the velocity in device memory.
struct SweepArgs {
    float *Ws, *Wl, *Vl, *V;
    const float *d;
    float *z;
    int n, nl, nrr, ns;
    float lr, mu;
};

// One stage of the sweep: streamed pass i (in cur, loaded two stages ago) is finished, the loads of
// pass i + 2 go out into the buffer this frees, and register row i and LDS pass i are worked on while
// they travel.  Passes are sixteen rows (one row per group of sixteen lanes).
struct StageArgs {
    float *Ws, *Vs, *Vr, *Wl, *Vl;
    const float *ds, *dr, *dl;
    float *zs, *zr, *zl;
    int n, ns, nrr, nl, npass, nlpass;
    float lr, mu;
    bool keepv;
};

template <bool MOM, bool U, bool D>
__device__ __forceinline__ void sweep_stage(RowPart<MOM> (&cur)[1], RowPart<MOM> &wrow, int i, int last, const StageArgs &t,
                                            const v4f (&a4)[WNI], const v4f (&x4)[WNI])
{
    const int wave = threadIdx.x >> 6, sg = (threadIdx.x & 63) >> 4;
    // (the pass's first row is made opaque: as a constant, every address of every unrolled stage is
    // loop invariant over the steps, and the compiler computes them all once and keeps them in registers)
    int base = i * kPass;
    asm volatile("" : "+s"(base));
    if (i < t.npass) pass_finish<MOM, U, D, 1>(cur, t.Ws, t.Vs, t.n, t.ns, base, t.ds, a4, x4, t.lr, t.mu, t.keepv, t.zs);
    if (i + 2 < t.npass && i + 2 < last) pass_load<MOM, 1>(cur, t.Ws, t.Vs, t.n, t.ns, base + 2 * kPass);
    reg_row<MOM, U, D>(wrow, i * kPass + wave * 4 + sg, t.Vr, t.n, t.nrr, t.dr, a4, x4, t.lr, t.mu, t.keepv, t.zr);
    if (i < t.nlpass) {
        RowPart<MOM> wl[1];
        pass_load<MOM, 1>(wl, t.Wl, t.Vl, t.n, t.nl, base);
        pass_finish<MOM, U, D, 1>(wl, t.Wl, t.Vl, t.n, t.nl, base, t.dl, a4, x4, t.lr, t.mu, t.keepv, t.zl);
    }
}

// The first two streamed passes of the NEXT sweep, requested as soon as a sweep has written them (a
// thread reads back the rows and columns it wrote itself): they travel while the step's small
// phases -- the exchange of the partial net inputs, the output stage, the deltas -- run.
template <bool MOM>
__device__ __forceinline__ void sweep_preload(RowPart<MOM> (&bufa)[1], RowPart<MOM> (&bufb)[1], const float *Ws, const float *Vs,
                                              int n, int ns)
{
    int base = 0;
    asm volatile("" : "+s"(base));
    if (ns > 0) pass_load<MOM, 1>(bufa, Ws, Vs, n, ns, base);
    if (ns > kPass) pass_load<MOM, 1>(bufb, Ws, Vs, n, ns, base + kPass);
}

// One sweep over all three tiers.  The streamed rows wait for memory, the register and LDS rows for
// next to nothing, and with one wave per SIMD there is nobody else to fill the wait: the tiers are
// therefore interleaved by hand, one stage per register row (RR of them), the streamed
// passes two ahead in two buffers.  On entry bufa / bufb hold streamed passes 0 and 1 (sweep_preload);
// on exit they hold them again, for the next sweep.  Streamed and LDS passes beyond RR follow in plain loops.
// res[i] is this lane's part of row i * kPass + wave * 4 + sg of the register tier.
template <bool MOM, bool U, bool D, int RR>
__device__ __forceinline__ void sweep_all(RowPart<MOM> (&res)[RR > 0 ? RR : 1], RowPart<MOM> (&bufa)[1], RowPart<MOM> (&bufb)[1],
                                          const SweepArgs &sa, const v4f (&a4)[WNI], const v4f (&x4)[WNI], bool keepv)
{
    const int first_s = sa.nl + sa.nrr;
    StageArgs t;
    t.Ws = sa.Ws; t.Vs = sa.V + (size_t)first_s * sa.n; t.Vr = sa.V + (size_t)sa.nl * sa.n; t.Wl = sa.Wl;
    t.Vl = MOM ? sa.Vl : sa.V;   // the LDS rows' velocities: beside them with momentum, else device memory (written on request)
    t.ds = sa.d + first_s; t.dr = sa.d + sa.nl; t.dl = sa.d;
    t.zs = sa.z + first_s; t.zr = sa.z + sa.nl; t.zl = sa.z;
    t.n = sa.n; t.ns = sa.ns; t.nrr = sa.nrr; t.nl = sa.nl;
    t.npass = (sa.ns + kPass - 1) / kPass;
    t.nlpass = (sa.nl + kPass - 1) / kPass;
    t.lr = sa.lr; t.mu = sa.mu; t.keepv = keepv;
#pragma unroll
    for (int i = 0; i + 1 < RR; i += 2) {   // stages in pairs: even streamed passes go through bufa, odd ones through bufb
        sweep_stage<MOM, U, D>(bufa, res[i], i, RR, t, a4, x4);
        sweep_stage<MOM, U, D>(bufb, res[i + 1], i + 1, RR, t, a4, x4);
    }
    if (RR % 2 == 1) sweep_stage<MOM, U, D>(bufa, res[RR - 1], RR - 1, RR, t, a4, x4);
    if (t.npass > RR) sweep_mem<MOM, U, D, 1>(t.Ws, t.Vs, t.n, t.ns, t.ds, a4, x4, t.lr, t.mu, keepv, t.zs, RR * kPass);
    if (t.nlpass > RR) sweep_mem<MOM, U, D, 1>(t.Wl, t.Vl, t.n, t.nl, t.dl, a4, x4, t.lr, t.mu, keepv, t.zl, RR * kPass);
    sweep_preload<MOM>(bufa, bufb, t.Ws, t.Vs, t.n, t.ns);
}

template <int RR, bool MOM>
__global__ __launch_bounds__(kThreads) void wide_epoch_kernel(WidePlan p)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ int s_abort;
    const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int n0 = p.n0, n1 = p.n1, nL = p.nL, per = p.per, perp = (per + 3) & ~3, grid = (int)gridDim.x;
    const int n4 = n0 >> 2, n0p = (n0 + 3) & ~3;
    const int r0 = w * per, nr = max(0, min(per, n1 - r0));
    // the three tiers of the own rows
    const int nl = min(p.lds_rows, nr);
    const int nrr = min(kPass * RR, nr - nl);
    const int ns = nr - nl - nrr;
    float *xbuf = lds + p.lds_x;
    float *a_own = lds + p.lds_a, *d_own = lds + p.lds_d, *b1 = lds + p.lds_b, *z1 = lds + p.lds_z;
    float *W2c = lds + p.lds_w2;                    // [nL][perp]: the own columns of W_2
    float *zall = lds + p.lds_zall;                 // [grid][nL] partial net inputs of the output layer
    float *zL = lds + p.lds_out, *dL = zL + WIDE_MAX_NL, *bL = dL + WIDE_MAX_NL;
    float *W1l = lds + p.lds_w1;                    // tier 1 (with momentum its velocities follow at V1l)
    float *V1l = W1l + (size_t)p.lds_rows * n0;
    float *vb1 = lds + p.lds_vb, *VW2c = lds + p.lds_vw2, *vbL = bL + WIDE_MAX_NL;   // velocities of b_1, the W_2 columns, b_2 (momentum)
    float *W1r = p.W1 + (size_t)(r0 + nl) * n0;     // tier 2's rows in device memory (prologue / epilogue)
    float *W1s = p.W1 + (size_t)(r0 + nl + nrr) * n0;   // tier 3
    float *V1 = p.VW1 + (size_t)r0 * n0;

    // ---- prologue ----
    if (tid == 0) s_abort = 0;
    for (int k = tid; k < nL; k += kThreads) bL[k] = p.b2[k];
    for (int j = tid; j < nr; j += kThreads) b1[j] = p.b1[r0 + j];
    for (int i = tid; i < nL * perp; i += kThreads) {
        const int k = i / perp, j = i - k * perp;
        W2c[i] = j < nr ? p.W2[(size_t)k * n1 + r0 + j] : 0.f;
    }
    copy_floats(W1l, p.W1 + (size_t)r0 * n0, nl * n0);
    if (MOM) {
        copy_floats(V1l, V1, nl * n0);
        for (int k = tid; k < nL; k += kThreads) vbL[k] = p.Vb2[k];
        for (int j = tid; j < nr; j += kThreads) vb1[j] = p.Vb1[r0 + j];
        for (int i = tid; i < nL * perp; i += kThreads) {
            const int k = i / perp, j = i - k * perp;
            VW2c[i] = j < nr ? p.VW2[(size_t)k * n1 + r0 + j] : 0.f;
        }
    }
    RowPart<MOM> wres[RR > 0 ? RR : 1];
#pragma unroll
    for (int i = 0; i < RR; ++i) {
        const int row = min(i * kPass + wave * 4 + sg, max(nrr - 1, 0));
#pragma unroll
        for (int j = 0; j < WNI; ++j) {
            const int c = g + 16 * j;
            const bool on = nrr > 0 && c < n4;
            const size_t at = (size_t)(nl + row) * n0 + 4 * min(c, n4 - 1);
            wres[i].w[j] = on ? *(const v4f *)(p.W1 + (size_t)r0 * n0 + at) : (v4f){0.f, 0.f, 0.f, 0.f};
            if constexpr (MOM) wres[i].v[j] = on ? *(const v4f *)(V1 + at) : (v4f){0.f, 0.f, 0.f, 0.f};
        }
    }
    for (int k = tid; k < n0; k += kThreads) xbuf[k] = p.X[k];
    int y_cur = p.labels[0];
    double loss_acc = 0.0;
    __syncthreads();

    // one sweep over all three tiers: rows take d_own, products with x4 go to z1
    const SweepArgs sa{W1s, W1l, V1l, V1, d_own, z1, n0, nl, nrr, ns, p.lr, p.mu};
    RowPart<MOM> bufa[1], bufb[1];   // streamed passes 0 and 1 of the next sweep, in flight between sweeps
    {   // the first sample's products with W_1
        v4f a4[WNI], x4[WNI];
        lane_pieces(x4, xbuf, n4, g);
#pragma unroll
        for (int j = 0; j < WNI; ++j) a4[j] = (v4f){0.f, 0.f, 0.f, 0.f};
        sweep_preload<MOM>(bufa, bufb, W1s, V1 + (size_t)(nl + nrr) * n0, n0, ns);
        sweep_all<MOM, false, true, RR>(wres, bufa, bufb, sa, a4, x4, false);
    }
    __syncthreads();

    for (int64_t s = 0; s < p.n_samples; ++s) {
        const uint32_t seq = p.seq0 + 1u + (uint32_t)s;
        const int par = (int)(seq & 1u);
        const bool more = s + 1 < p.n_samples;
        const bool keepv = !MOM && p.keep_v && !more;   // plain gradient descent: the epoch's last step also leaves the applied change as velocity
        const float *x = xbuf + (size_t)(s & 1) * n0p;
        float *xn = xbuf + (size_t)((s + 1) & 1) * n0p;

        // ---- hidden layer: activations of the own units, then their share of the output layer's net inputs ----
        for (int j = tid; j < nr; j += kThreads) a_own[j] = act_fn(p.act1, z1[j] + b1[j]);
        for (int j = nr + tid; j < perp; j += kThreads) a_own[j] = 0.f;
        __syncthreads();
        u64 *pub = p.z_x + ((size_t)par * grid + w) * nL;
        for (int k = wave; k < nL; k += kWaves) {
            const float *wr = W2c + k * perp;
            float acc = 0.f;
            for (int j = lane * 4; j < perp; j += 256) {
                const v4f av = *(const v4f *)(a_own + j), wv = *(const v4f *)(wr + j);
                acc += wv.x * av.x + wv.y * av.y + wv.z * av.z + wv.w * av.w;
            }
            acc = wave_sum(acc);
            if (lane == 0) {
                if (grid > 1) ll_store(pub + k, acc, seq);
                else zall[k] = acc;
            }
        }
        // while the partials travel: the next sample's features and label
        constexpr int XR = (64 * WNI + kThreads - 1) / kThreads;
        float xr[XR];
        int y_next = 0;
        if (more) {
#pragma unroll
            for (int u = 0; u < XR; ++u) {
                const int k = tid + u * kThreads;
                xr[u] = k < n0 ? p.X[(size_t)(s + 1) * n0 + k] : 0.f;
            }
            y_next = p.labels[s + 1];
        }
        if (grid > 1) {
            const u64 *src = p.z_x + (size_t)par * grid * nL;
            poll_words(grid * nL, seq, [&](int q) { return src + q; }, [&](int q, float v) { zall[q] = v; }, p.abort_flag,
                       &s_abort);
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < XR; ++u) {
                const int k = tid + u * kThreads;
                if (k < n0) xn[k] = xr[u];
            }
        }
        __syncthreads();
        if (s_abort) break;
        // z_L = sum of the partials in workgroup order (the same order everywhere) + b_L
        for (int k = wave; k < nL; k += kWaves) {
            float acc = 0.f;
            for (int q = lane; q < grid; q += 64) acc += zall[q * nL + k];
            acc = wave_sum(acc);
            if (lane == 0) zL[k] = acc + bL[k];
        }
        __syncthreads();

        // ---- output layer, repeated by every workgroup: loss and delta_L (wave 0) ----
        int y = y_cur;
        y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
        if (wave == 0) {
            const int k0 = lane;
            const float z0 = k0 < nL ? zL[k0] : -INFINITY;
            float d0, e;
            if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                const float e_m = wave_max(z0);
                const float e0 = k0 < nL ? expf(z0 - e_m) : 0.f;
                const float e_sum = wave_sum(e0);
                d0 = e0 * (1.0f / e_sum) - (k0 == y ? 1.0f : 0.0f);
                e = logf(e_sum) - (zL[y] - e_m);
            } else {
                const float a0 = act_fn(p.actL, z0);
                const float f0 = a0 - (k0 == y ? 1.0f : 0.0f);
                d0 = f0 * act_deriv(p.actL, a0);
                e = wave_sum(k0 < nL ? 0.5f * f0 * f0 : 0.f);
            }
            if (k0 < nL) {
                dL[k0] = d0;
                if (MOM) {
                    const float vv = p.mu * vbL[k0] - p.lr * d0;
                    vbL[k0] = vv;
                    bL[k0] = bL[k0] + vv;
                } else {
                    bL[k0] = bL[k0] - p.lr * d0;
                    if (keepv && w == 0) p.Vb2[k0] = -(p.lr * d0);
                }
            }
            if (w == 0 && lane == 0) loss_acc += (double)e;
        }
        __syncthreads();

        // ---- deltas of the own hidden units through W_2 as it was; W_2's own columns and b_1 updated ----
        for (int j = tid; j < nr; j += kThreads) {
            const float a = a_own[j];
            float sacc = 0.f;
            for (int k = 0; k < nL; ++k) {
                const float wv = W2c[k * perp + j], dk = dL[k];
                sacc += wv * dk;
                float ch = -((p.lr * dk) * a);
                if (MOM) {
                    ch = __builtin_fmaf(p.mu, VW2c[k * perp + j], ch);
                    VW2c[k * perp + j] = ch;
                }
                W2c[k * perp + j] = wv + ch;
                if (keepv) p.VW2[(size_t)k * n1 + r0 + j] = ch;
            }
            const float d = sacc * act_deriv(p.act1, a);
            d_own[j] = d;
            if (MOM) {
                const float vv = p.mu * vb1[j] - p.lr * d;
                vb1[j] = vv;
                b1[j] = b1[j] + vv;
            } else {
                b1[j] = b1[j] - p.lr * d;
                if (keepv) p.Vb1[r0 + j] = -(p.lr * d);
            }
        }
        __syncthreads();

        // ---- the sweep over the own rows of W_1: this step's update, the next step's products ----
        {
            v4f a4[WNI], x4[WNI];
            lane_pieces(a4, x, n4, g);
            // (ONE instance of the sweep inside the loop: with one per case -- more steps to come, last
            // step, last step leaving velocities -- the register rows met in a join after three separate
            // updates and the compiler kept a second set of registers for them.  After the last step the
            // products are taken with whatever the other input buffer holds and nobody reads them.)
            lane_pieces(x4, xn, n4, g);
            sweep_all<MOM, true, true, RR>(wres, bufa, bufb, sa, a4, x4, keepv);
        }
        __syncthreads();
        y_cur = y_next;
    }

    // ---- epilogue: everything the workgroup kept on the chip goes back to device memory ----
    __syncthreads();
    copy_floats(p.W1 + (size_t)r0 * n0, W1l, nl * n0);
    if (MOM) copy_floats(V1, V1l, nl * n0);
#pragma unroll
    for (int i = 0; i < RR; ++i) {
        const int row = i * kPass + wave * 4 + sg;
#pragma unroll
        for (int j = 0; j < WNI; ++j) {
            const int c = g + 16 * j;
            if (row < nrr && c < n4) {
                *(v4f *)(W1r + (size_t)row * n0 + 4 * c) = wres[i].w[j];
                if constexpr (MOM) *(v4f *)(V1 + (size_t)(nl + row) * n0 + 4 * c) = wres[i].v[j];
            }
        }
    }
    for (int j = tid; j < nr; j += kThreads) {
        p.b1[r0 + j] = b1[j];
        if (MOM) p.Vb1[r0 + j] = vb1[j];
    }
    for (int i = tid; i < nL * perp; i += kThreads) {
        const int k = i / perp, j = i - k * perp;
        if (j < nr) {
            p.W2[(size_t)k * n1 + r0 + j] = W2c[i];
            if (MOM) p.VW2[(size_t)k * n1 + r0 + j] = VW2c[i];
        }
    }
    if (w == 0) {
        for (int k = tid; k < nL; k += kThreads) {
            p.b2[k] = bL[k];
            if (MOM) p.Vb2[k] = vbL[k];
        }
        if (tid == 0) *p.loss_acc += loss_acc;
    }
}

}  // namespace

// ---- host side -------------------------------------------------------------------

bool wide_geometry(const int32_t *n, int L, int max_wg, bool want_v, WideGeom &g)
{
    g = WideGeom{};
    if (L != 2) return false;
    const int n0 = n[0], n1 = n[1], nL = n[2];
    if (n0 % 4 != 0 || n0 < 4 || n0 > 64 * WIDE_NI || nL > WIDE_MAX_NL || n1 < 1) return false;
    if (max_wg < 1) return false;
    if (max_wg > ON_MAX_WG) max_wg = ON_MAX_WG;
    auto pad4 = [](int v) { return (v + 3) & ~3; };
    const int per = (n1 + max_wg - 1) / max_wg;
    const int grid = (n1 + per - 1) / per;
    if ((int64_t)per * n0 > ((int64_t)1 << 24)) return false;
    g.per = per;
    g.grid = grid;
    int64_t f = 0;
    g.lds_x = (int)f; f += 2 * pad4(n0);
    g.lds_a = (int)f; f += pad4(per);
    g.lds_d = (int)f; f += pad4(per);
    g.lds_b = (int)f; f += pad4(per);
    g.lds_z = (int)f; f += pad4(per);
    g.lds_w2 = (int)f; f += (int64_t)nL * pad4(per);
    g.lds_vb = (int)f; if (want_v) f += pad4(per);
    g.lds_vw2 = (int)f; if (want_v) f += (int64_t)nL * pad4(per);
    g.lds_zall = (int)f; f += pad4(grid * nL);
    g.lds_out = (int)f; f += 4 * WIDE_MAX_NL;
    g.lds_w1 = (int)f;
    const int64_t room = (int64_t)(ON_MAX_LDS_BYTES / sizeof(float)) - f;
    if (room < 0) return false;
    // rows of W_1 in LDS; with momentum each brings its row of velocities
    int rows = (int)std::min<int64_t>(room / ((int64_t)n0 * (want_v ? 2 : 1)), per);
    // the kernel is for layers that do NOT fit: a net whose rows all fit in LDS belongs to the kernels that
    // keep every weight there
    if ((int64_t)per * n0 <= room) return false;
    g.lds_rows = rows;
    f += (int64_t)rows * n0 * (want_v ? 2 : 1);
    g.lds_floats = (int)f;
    g.words = 2 * (size_t)grid * nL;
    g.ok = true;
    return true;
}

size_t wide_exchange_bytes_bound(const int32_t *n, int L)
{
    if (L != 2 || n[2] > WIDE_MAX_NL) return 0;
    return 2 * (size_t)ON_MAX_WG * WIDE_MAX_NL * sizeof(u64);
}

hipError_t wide_prepare()
{
    hipError_t e = hipFuncSetAttribute((const void *)wide_epoch_kernel<WIDE_REG_ROWS, false>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)ON_MAX_LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)wide_epoch_kernel<WIDE_REG_ROWS_MOMENTUM, true>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)ON_MAX_LDS_BYTES);
}

hipError_t launch_wide_epoch(const WideGeom &g, const WidePlan &plan, hipStream_t stream)
{
    if (plan.mu != 0.f)
        return launch_resident(wide_epoch_kernel<WIDE_REG_ROWS_MOMENTUM, true>, plan, g.grid, (size_t)g.lds_floats * sizeof(float),
                               stream);
    return launch_resident(wide_epoch_kernel<WIDE_REG_ROWS, false>, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
}

}  // namespace dn
