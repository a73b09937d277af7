// Per-sample (batch 1) training as ONE persistent kernel per epoch.
//
// With one sample per step every phase of back propagation is a matrix-vector
// product that depends on the previous phase, and the next step depends on this
// step's update, so a step is a chain of short phases.  Launching a kernel per
// phase makes the chain cost a launch per link.  Here up to 256 workgroups (one
// per compute unit) stay resident for the whole epoch and each OWNS a fixed slice
// of every layer:
//
//   layers 1..L-1   a block of rows of W_l (a block of that layer's neurons):
//                   forward   a_l[rows]   = f(W_l[rows,:] a_{l-1} + b_l[rows])   (needs all of a_{l-1})
//                   backward  one sweep over the same rows reads each weight once and
//                             (i) adds W_l[r,:] delta_l[r] into this workgroup's partial of W_l^T delta_l,
//                             (ii) writes W_l[r,:] - lr delta_l[r] a_{l-1}  -- the two-index
//                             (inputs x outputs) loop the paper offloads, fused with the update
//   layer L         the block of COLUMNS of W_L that matches its rows of layer L-1
//                   (its own hidden units feed these columns), so the last layer needs
//                   no input exchange: forward gives a partial of z_L (n_L numbers),
//                   backward gives delta_{L-1} for its own units directly.
//
// What has to cross between workgroups is small: the activations of layers
// 1..L-2, one n_L-vector of partial net inputs per workgroup, and the partials of
// W_l^T delta_l for l = 2..L-1.  It is exchanged through device memory as 64-bit
// words {value, step number}: a consumer polls the word until the step number is
// the current one, so publishing and signalling are a single store and a single
// load apart (no grid-wide barrier).  Two copies of every exchange buffer, used
// on alternating steps, keep a fast producer from overwriting a word a slow
// consumer has not read yet: before a workgroup publishes step s+2 it has
// consumed data that every one of its consumers published after they finished
// reading step s.
//
// A workgroup's slices never change hands, so when they fit (with the velocity slices
// when momentum is used) they are copied into LDS at the start of the epoch and written
// back once at its end: weights of small and medium nets then never touch device memory
// between steps and a step costs little more than its exchanges.  Larger slices stay in
// device memory and are streamed (each weight read once forward, read and written once
// backward).
//
// Every wait is bounded: a poll that does not complete within kSpinLimit
// attempts raises an abort flag that ends every workgroup, and the host reports
// DN_ERR_DEVICE.  All sums are taken in a fixed order, so an epoch is
// reproducible bit for bit.
#include <algorithm>

#include "dn_internal.h"
#include "dn_persist.h"
#include "dn_wave.h"

namespace dn {
namespace {

// out[e] = sum over w < P of the word at src[w * stride + base + e], e < count, summed in a
// fixed order: 16 lanes per element each add every 16th partial, then a butterfly over the 16.
// `scale_fn(e, sum)` finishes the element.  tmp holds kTmp floats.  Ends with a barrier.
template <class Finish>
__device__ __forceinline__ void gather_partials(const u64 *src, int P, int stride, int base, int count,
                                                uint32_t seq, float *tmp, Finish finish, int *abort_flag,
                                                volatile int *s_abort)
{
    const int ecap = min(kTmp / P, kThreads);   // elements per pass (P <= ON_MAX_WG <= kTmp)
    for (int e0 = 0; e0 < count; e0 += ecap) {
        const int ne = min(ecap, count - e0);
        // threads form groups of G = 2^lg >= ne lanes; a group reads the ne words of one producer
        const int lg = 32 - __clz(ne - 1), G = 1 << lg;
        const int e = threadIdx.x & (G - 1), ww0 = threadIdx.x >> lg, wstep = kThreads >> lg;
        if (e < ne) {
            const u64 *col = src + base + e0 + e;
            for (int wb = ww0; wb < P; wb += wstep * kPollBatch) {
                u64 v[kPollBatch];
                bool ok[kPollBatch];
                bool all = true;
#pragma unroll
                for (int u = 0; u < kPollBatch; ++u) {
                    const int ww = wb + u * wstep;
                    v[u] = 0;
                    ok[u] = true;
                    if (ww < P) {
                        v[u] = ll_load(col + (size_t)ww * stride);
                        ok[u] = (uint32_t)(v[u] >> 32) == seq;
                    }
                    all = all && ok[u];
                }
                int spins = 0;
                while (!all) {
                    all = true;
#pragma unroll
                    for (int u = 0; u < kPollBatch; ++u) {
                        if (!ok[u]) {
                            v[u] = ll_load(col + (size_t)(wb + u * wstep) * stride);
                            ok[u] = (uint32_t)(v[u] >> 32) == seq;
                            all = all && ok[u];
                        }
                    }
                    if (all) break;
                    ++spins;
                    if (spins > kSpinLimit) {
                        __hip_atomic_store(abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        *s_abort = 1;
                        break;
                    }
                    if ((spins & 255) == 0 &&
                        __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                        *s_abort = 1;
                        break;
                    }
                }
#pragma unroll
                for (int u = 0; u < kPollBatch; ++u) {
                    const int ww = wb + u * wstep;
                    if (ww < P) tmp[e * P + ww] = __uint_as_float((uint32_t)v[u]);
                }
            }
        }
        __syncthreads();
        const int g = threadIdx.x & 15;
        for (int e = threadIdx.x >> 4; e < ne; e += kThreads / 16) {
            float s = 0.f;
            for (int ww = g; ww < P; ww += 16) s += tmp[e * P + ww];
            s = row16_sum(s);
            if (g == 0) finish(e0 + e, s);
        }
        __syncthreads();
    }
}

// Backward sweep over a block of rows of a layer whose input layer needs a delta:
// every weight is read once; s[k] accumulates W[r][k] delta[r] over the block's rows and the
// weight is rewritten with the update.  Waves split the columns in chunks of 64*VEC and,
// when there are fewer chunks than waves, the rows as well (partials meet in sred).
// The block's partial of W^T delta is published to part_out[k], k < n_in.
// (MODE, the update rule, is a template parameter of the three backward sweeps: tested per element
// at run time it puts a branch around every multiply-add of the unrolled loops.)
template <int VEC, int RU, int MODE>
__device__ __forceinline__ void bwd_rows_m(float *__restrict__ Wt, float *Vt, int n_in, int nr,
                                           const float *dl, const float *ain, float lr, float mu,
                                           float *sred, u64 *part_out, uint32_t seq)
{
    constexpr int mode = MODE;
    constexpr int CW = 64 * VEC;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int C = (n_in + CW - 1) / CW;
    int RG, rg, c_first, c_step;
    if (C >= kWaves) {
        RG = 1; rg = 0; c_first = wave; c_step = kWaves;
    } else {
        RG = kWaves / C; rg = wave / C; c_first = wave - rg * C; c_step = C;   // one chunk per wave
        if (rg >= RG) c_first = C;                                             // spare waves idle
    }
    for (int c = c_first; c < C; c += c_step) {
        const int k = c * CW + lane * VEC;
        const bool kin = k < n_in;
        const int kc = kin ? k : 0;
        float a[VEC], s[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) { a[e] = ain[kc + e]; s[e] = 0.f; }
        for (int r = rg; r < nr; r += RG * RU) {
            float wv[RU][VEC], vv[RU][VEC];
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int ru = r + u * RG;
                const int rc = ru < nr ? ru : r;
                const float *wp = Wt + (size_t)rc * n_in + kc;
                if (VEC == 4) {
                    const v4f t = *(const v4f *)wp;
                    wv[u][0] = t.x; wv[u][1 % VEC] = t.y; wv[u][2 % VEC] = t.z; wv[u][3 % VEC] = t.w;
                } else {
                    wv[u][0] = wp[0];
                }
            }
            if (mode == UPD_MOMENTUM) {
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int ru = r + u * RG;
                    const int rc = ru < nr ? ru : r;
                    const float *vp = Vt + (size_t)rc * n_in + kc;
                    if (VEC == 4) {
                        const v4f t = *(const v4f *)vp;
                        vv[u][0] = t.x; vv[u][1 % VEC] = t.y; vv[u][2 % VEC] = t.z; vv[u][3 % VEC] = t.w;
                    } else {
                        vv[u][0] = vp[0];
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < RU; ++u)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) vv[u][e] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int ru = r + u * RG;
                if (ru < nr) {
                    const float d = dl[ru];
                    const float ld = lr * d;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        s[e] += wv[u][e] * d;
                        wv[u][e] = apply_update(wv[u][e], ld * a[e], vv[u][e], mu, mode);
                    }
                    if (kin) {
                        float *wp = Wt + (size_t)ru * n_in + k;
                        float *vp = Vt + (size_t)ru * n_in + k;
                        if (VEC == 4) {
                            v4f t; t.x = wv[u][0]; t.y = wv[u][1 % VEC]; t.z = wv[u][2 % VEC]; t.w = wv[u][3 % VEC];
                            *(v4f *)wp = t;
                            if (mode != UPD_SGD) {
                                v4f q; q.x = vv[u][0]; q.y = vv[u][1 % VEC]; q.z = vv[u][2 % VEC]; q.w = vv[u][3 % VEC];
                                *(v4f *)vp = q;
                            }
                        } else {
                            wp[0] = wv[u][0];
                            if (mode != UPD_SGD) vp[0] = vv[u][0];
                        }
                    }
                }
            }
        }
        if (kin) {
            if (RG == 1) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) ll_store(part_out + k + e, s[e], seq);
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) sred[rg * n_in + k + e] = s[e];
            }
        }
    }
    if (RG > 1) {
        __syncthreads();
        for (int j = threadIdx.x; j < n_in; j += kThreads) {
            float t = 0.f;
            for (int g = 0; g < RG; ++g) t += sred[g * n_in + j];
            ll_store(part_out + j, t, seq);
        }
    }
}

template <int VEC, int RU>
__device__ __forceinline__ void bwd_rows(float *__restrict__ Wt, float *Vt, int n_in, int nr,
                                         const float *dl, const float *ain, float lr, float mu, int mode,
                                         float *sred, u64 *part_out, uint32_t seq)
{
    if (mode == UPD_SGD) bwd_rows_m<VEC, RU, UPD_SGD>(Wt, Vt, n_in, nr, dl, ain, lr, mu, sred, part_out, seq);
    else if (mode == UPD_KEEPV) bwd_rows_m<VEC, RU, UPD_KEEPV>(Wt, Vt, n_in, nr, dl, ain, lr, mu, sred, part_out, seq);
    else bwd_rows_m<VEC, RU, UPD_MOMENTUM>(Wt, Vt, n_in, nr, dl, ain, lr, mu, sred, part_out, seq);
}

// Backward of a block of rows of the first layer (no delta is needed for the input): the
// block is a contiguous run of nr * n_in weights, updated in place.
template <int VEC, int RU, int MODE>
__device__ __forceinline__ void bwd_flat_m(float *__restrict__ Wb, float *Vb, int n_in, int nr,
                                           const float *dl, const float *ain, float lr, float mu)
{
    constexpr int mode = MODE;
    const int total = nr * n_in;
    const float inv_n = 1.0f / (float)n_in;
    for (int i0 = threadIdx.x * VEC; i0 < total; i0 += kThreads * VEC * RU) {
        float wv[RU][VEC], vv[RU][VEC];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int i = i0 + u * kThreads * VEC;
            const int ic = i < total ? i : i0;
            if (VEC == 4) {
                const v4f t = *(const v4f *)(Wb + ic);
                wv[u][0] = t.x; wv[u][1 % VEC] = t.y; wv[u][2 % VEC] = t.z; wv[u][3 % VEC] = t.w;
            } else {
                wv[u][0] = Wb[ic];
            }
        }
        if (mode == UPD_MOMENTUM) {
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int i = i0 + u * kThreads * VEC;
                const int ic = i < total ? i : i0;
                if (VEC == 4) {
                    const v4f t = *(const v4f *)(Vb + ic);
                    vv[u][0] = t.x; vv[u][1 % VEC] = t.y; vv[u][2 % VEC] = t.z; vv[u][3 % VEC] = t.w;
                } else {
                    vv[u][0] = Vb[ic];
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < RU; ++u)
#pragma unroll
                for (int e = 0; e < VEC; ++e) vv[u][e] = 0.f;
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int i = i0 + u * kThreads * VEC;
            if (i < total) {
                // row of element i: below 2^22 elements a float estimate is off by at most one
                // row and is corrected exactly; larger blocks divide
                int r;
                if (total < (1 << 22)) {
                    r = min((int)((float)i * inv_n), nr - 1);
                    if (r * n_in > i) --r;
                    else if ((r + 1) * n_in <= i) ++r;
                } else {
                    r = (int)((unsigned)i / (unsigned)n_in);
                }
                const int k = i - r * n_in;
                const float ld = lr * dl[r];
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    wv[u][e] = apply_update(wv[u][e], ld * ain[k + e], vv[u][e], mu, mode);
                if (VEC == 4) {
                    v4f t; t.x = wv[u][0]; t.y = wv[u][1 % VEC]; t.z = wv[u][2 % VEC]; t.w = wv[u][3 % VEC];
                    *(v4f *)(Wb + i) = t;
                    if (mode != UPD_SGD) {
                        v4f q; q.x = vv[u][0]; q.y = vv[u][1 % VEC]; q.z = vv[u][2 % VEC]; q.w = vv[u][3 % VEC];
                        *(v4f *)(Vb + i) = q;
                    }
                } else {
                    Wb[i] = wv[u][0];
                    if (mode != UPD_SGD) Vb[i] = vv[u][0];
                }
            }
        }
    }
}

template <int VEC, int RU>
__device__ __forceinline__ void bwd_flat(float *__restrict__ Wb, float *Vb, int n_in, int nr,
                                         const float *dl, const float *ain, float lr, float mu, int mode)
{
    if (mode == UPD_SGD) bwd_flat_m<VEC, RU, UPD_SGD>(Wb, Vb, n_in, nr, dl, ain, lr, mu);
    else if (mode == UPD_KEEPV) bwd_flat_m<VEC, RU, UPD_KEEPV>(Wb, Vb, n_in, nr, dl, ain, lr, mu);
    else bwd_flat_m<VEC, RU, UPD_MOMENTUM>(Wb, Vb, n_in, nr, dl, ain, lr, mu);
}

// One sweep over a block of rows of the FIRST layer, for rows of at most 512 floats (whole float4s):
//   UPDATE  W[r][k] = update(W[r][k], (lr dl[r]) a[k])          (the rank-1 step; no delta is needed below layer 1)
//   DOT     out[r]  = sum_k W[r][k] xd[k], from the row as just updated
// Per-sample training allows both in one pass: the update of W_1 is the last thing a step does and
// the product W_1 x of the next sample the first thing the next step does, so the row that was just
// updated is multiplied with the next sample while it is still in registers -- 8 bytes per weight
// and step through memory (read, write) instead of 12 (read; read, write).
// Sixteen lanes share a row (four rows per wave at a time, two such groups in flight): a lane owns
// the float4 columns g, g + 16, ... of every row and keeps its pieces of a and xd in registers, so a
// row costs its loads, its multiply-adds, its stores and one four-step butterfly -- no index
// arithmetic and no LDS traffic per element.  Wt / Vt: LDS or device memory.
// NI: float4 columns per lane (rows of up to 64 NI floats).  Every load is issued unconditionally (clamped
// address, contribution masked): loads behind a branch make the compiler wait for each before the next.
// MODE (the update rule) is a template parameter as well: tested per element at run time it put a
// branch around every multiply-add (measured: 7 us per 64 rows against 0.5 us).
template <bool UPDATE, bool DOT, int NI, int MODE>
__device__ __forceinline__ void sweep_rows16_n(float *__restrict__ Wt, float *__restrict__ Vt, int n, int nr, const float *dl,
                                               const float *a, const float *xd, float lr, float mu, float *out)
{
    constexpr int mode = MODE;
    constexpr int RU = 2;   // row groups in flight
    constexpr int jn = NI;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int n4 = n >> 2;
    v4f a4[NI], x4[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int c = g + 16 * j;
        const bool on = c < n4;
        a4[j] = (UPDATE && on) ? *(const v4f *)(a + 4 * c) : (v4f){0.f, 0.f, 0.f, 0.f};
        x4[j] = (DOT && on) ? *(const v4f *)(xd + 4 * c) : (v4f){0.f, 0.f, 0.f, 0.f};
    }
    for (int base = 0; base < nr; base += 32 * RU) {
        v4f wv[RU][NI];
        int row[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            row[u] = base + u * 32 + wave * 4 + sg;
            const float *wp = Wt + (size_t)min(row[u], nr - 1) * n;
#pragma unroll
            for (int j = 0; j < NI; ++j)
                if (j < jn) wv[u][j] = *(const v4f *)(wp + 4 * min(g + 16 * j, n4 - 1));
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const bool rin = row[u] < nr;
            const int rc = min(row[u], nr - 1);
            float acc = 0.f;
            if (UPDATE) {
                const float ld = lr * dl[rc];
                float *wp = Wt + (size_t)rc * n, *vp = Vt + (size_t)rc * n;
                v4f vrow[NI];
                if (mode == UPD_MOMENTUM) {
#pragma unroll
                    for (int j = 0; j < NI; ++j) vrow[j] = *(const v4f *)(vp + 4 * min(g + 16 * j, n4 - 1));
                } else {
#pragma unroll
                    for (int j = 0; j < NI; ++j) vrow[j] = (v4f){0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    if (j < jn) {
                        const int c = g + 16 * j;
                        const bool on = rin && c < n4;
                        const v4f vv = vrow[j];
                        v4f t;
                        float v0 = vv.x, v1 = vv.y, v2 = vv.z, v3 = vv.w;
                        t.x = apply_update(wv[u][j].x, ld * a4[j].x, v0, mu, mode);
                        t.y = apply_update(wv[u][j].y, ld * a4[j].y, v1, mu, mode);
                        t.z = apply_update(wv[u][j].z, ld * a4[j].z, v2, mu, mode);
                        t.w = apply_update(wv[u][j].w, ld * a4[j].w, v3, mu, mode);
                        wv[u][j] = t;
                        if (on) {
                            *(v4f *)(wp + 4 * c) = t;
                            if (mode != UPD_SGD) *(v4f *)(vp + 4 * c) = (v4f){v0, v1, v2, v3};
                        }
                    }
                }
            }
            if (DOT) {
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    if (j < jn)
                        acc += wv[u][j].x * x4[j].x + wv[u][j].y * x4[j].y + wv[u][j].z * x4[j].z + wv[u][j].w * x4[j].w;
                acc = row16_sum(acc);
                if (g == 0 && rin) out[row[u]] = acc;
            }
        }
    }
}

template <bool UPDATE, bool DOT, int MODE>
__device__ __forceinline__ void sweep_rows16_m(float *__restrict__ Wt, float *__restrict__ Vt, int n, int nr, const float *dl,
                                               const float *a, const float *xd, float lr, float mu, float *out)
{
    if ((n >> 2) <= 64) sweep_rows16_n<UPDATE, DOT, 4, MODE>(Wt, Vt, n, nr, dl, a, xd, lr, mu, out);
    else sweep_rows16_n<UPDATE, DOT, 8, MODE>(Wt, Vt, n, nr, dl, a, xd, lr, mu, out);
}

template <bool UPDATE, bool DOT>
__device__ __forceinline__ void sweep_rows16(float *__restrict__ Wt, float *__restrict__ Vt, int n, int nr, const float *dl,
                                             const float *a, const float *xd, float lr, float mu, int mode, float *out)
{
    if (!UPDATE || mode == UPD_SGD) sweep_rows16_m<UPDATE, DOT, UPD_SGD>(Wt, Vt, n, nr, dl, a, xd, lr, mu, out);
    else if (mode == UPD_KEEPV) sweep_rows16_m<UPDATE, DOT, UPD_KEEPV>(Wt, Vt, n, nr, dl, a, xd, lr, mu, out);
    else sweep_rows16_m<UPDATE, DOT, UPD_MOMENTUM>(Wt, Vt, n, nr, dl, a, xd, lr, mu, out);
}

// Last layer, forward: this workgroup's partial of z_L from its nc own columns of W_L
// (Wt = first own column of row 0, rows `stride` apart).
__device__ __forceinline__ void fwd_cols(const float *__restrict__ Wt, int stride, int nL, int nc,
                                         const float *a_own, u64 *zout, uint32_t seq)
{
    constexpr int JU = 4;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int k = wave; k < nL; k += kWaves) {
        const float *wp = Wt + (size_t)k * stride;
        float acc = 0.f;
        for (int j0 = lane; j0 < nc; j0 += 64 * JU) {
            float wv[JU];
#pragma unroll
            for (int u = 0; u < JU; ++u) {
                const int j = j0 + u * 64;
                wv[u] = wp[j < nc ? j : j0];
            }
#pragma unroll
            for (int u = 0; u < JU; ++u) {
                const int j = j0 + u * 64;
                acc += j < nc ? wv[u] * a_own[j] : 0.f;
            }
        }
        acc = wave_sum(acc);
        if (lane == 0) ll_store(zout + k, acc, seq);
    }
}

// Last layer, backward: for each own column j: s_j = sum_k W_L[k][j] delta_L[k] from the
// weights before the update, then the column is updated.  d_own[j] = s_j f'(a_own[j]) when
// a previous layer exists.
template <int MODE>
__device__ __forceinline__ void bwd_cols_m(float *__restrict__ Wt, int stride, float *Vt, int vstride, int nL,
                                           int nc, const float *a_own, const float *dL, float lr, float mu,
                                           float *d_own, int act_prev)
{
    constexpr int mode = MODE;
    constexpr int KB = 16;
    for (int j = threadIdx.x; j < nc; j += kThreads) {
        const float a = a_own[j];
        float s = 0.f;
        for (int k0 = 0; k0 < nL; k0 += KB) {
            float wv[KB], vv[KB];
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const int k = min(k0 + u, nL - 1);
                wv[u] = Wt[(size_t)k * stride + j];
            }
            if (mode == UPD_MOMENTUM) {
#pragma unroll
                for (int u = 0; u < KB; ++u) {
                    const int k = min(k0 + u, nL - 1);
                    vv[u] = Vt[(size_t)k * vstride + j];
                }
            } else {
#pragma unroll
                for (int u = 0; u < KB; ++u) vv[u] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const int k = k0 + u;
                if (k < nL) {
                    const float d = dL[k];
                    s += wv[u] * d;
                    const float nw = apply_update(wv[u], (lr * d) * a, vv[u], mu, mode);
                    Wt[(size_t)k * stride + j] = nw;
                    if (mode != UPD_SGD) Vt[(size_t)k * vstride + j] = vv[u];
                }
            }
        }
        if (d_own) d_own[j] = s * act_deriv(act_prev, a);
    }
}

__device__ __forceinline__ void bwd_cols(float *__restrict__ Wt, int stride, float *Vt, int vstride, int nL,
                                         int nc, const float *a_own, const float *dL, float lr, float mu,
                                         int mode, float *d_own, int act_prev)
{
    if (mode == UPD_SGD) bwd_cols_m<UPD_SGD>(Wt, stride, Vt, vstride, nL, nc, a_own, dL, lr, mu, d_own, act_prev);
    else if (mode == UPD_KEEPV) bwd_cols_m<UPD_KEEPV>(Wt, stride, Vt, vstride, nL, nc, a_own, dL, lr, mu, d_own, act_prev);
    else bwd_cols_m<UPD_MOMENTUM>(Wt, stride, Vt, vstride, nL, nc, a_own, dL, lr, mu, d_own, act_prev);
}

__global__ __launch_bounds__(ON_THREADS) void online_epoch_kernel(OnlinePlan p)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ int s_abort;
    const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int L = p.L;
    const int n0 = p.layer[1].n_in;
    const int nL = p.layer[L].n_out;
    const OnlineLayer &last = p.layer[L];
    // layer l's weight slice lives in LDS (bit l of p.resident), and with momentum its velocity slice too
    auto res_of = [&](int l) { return ((p.resident >> l) & 1) != 0; };
    // layer 1 too large for LDS: the first p.part_rows rows of the workgroup's block live there all
    // the same (every weight kept in LDS saves its three trips through device memory per step)
    const int part1 = (L >= 2 && !res_of(1)) ? max(0, min(p.part_rows, min(p.layer[1].per, p.layer[1].n_out - w * p.layer[1].per))) : 0;
    const bool with_v = p.mu != 0.f;

    // slices owned by this workgroup
    const int c0 = w * last.per;                                  // columns of W_L
    const int nc = max(0, min(last.per, last.n_in - c0));
    const int ncp = (last.per + 3) & ~3;                          // row pitch of the LDS image of those columns
    bool any = (w == 0) || nc > 0;
    for (int l = 1; l < L; ++l) any = any || (w * p.layer[l].per < p.layer[l].n_out);
    if (!any) return;
    const bool need_x = (L == 1) ? (nc > 0) : (w * p.layer[1].per < p.layer[1].n_out);
    const bool need_z = (w == 0) || nc > 0;

    float *xa0 = lds + p.lds_x;
    float *zL = lds + p.lds_out, *dL = zL + ON_MAX_NL, *bL = dL + ON_MAX_NL, *vbL = bL + ON_MAX_NL;
    float *kpart = lds + p.lds_kpart;
    float *tmp = lds + p.lds_tmp;
    const int n0p = (n0 + 3) & ~3;

    // ---- prologue: biases of own rows (always) and own weight slices (if resident) into LDS ----
    if (tid == 0) s_abort = 0;
    for (int k = tid; k < nL; k += kThreads) {
        bL[k] = last.b[k];
        vbL[k] = last.Vb[k];
    }
    for (int l = 1; l < L; ++l) {
        const OnlineLayer &ly = p.layer[l];
        const int r0 = w * ly.per;
        const int nr = max(0, min(ly.per, ly.n_out - r0));
        float *bl = lds + p.lds_b[l], *vbl = bl + ((ly.per + 3) & ~3);
        for (int r = tid; r < nr; r += kThreads) {
            bl[r] = ly.b[r0 + r];
            vbl[r] = ly.Vb[r0 + r];
        }
        if (res_of(l) && nr > 0) copy_floats(lds + p.lds_w[l], ly.W + (size_t)r0 * ly.n_in, nr * ly.n_in);
        if (res_of(l) && with_v && nr > 0) copy_floats(lds + p.lds_v[l], ly.VW + (size_t)r0 * ly.n_in, nr * ly.n_in);
        if (l == 1 && part1 > 0) {
            copy_floats(lds + p.lds_w[1], ly.W + (size_t)r0 * ly.n_in, part1 * ly.n_in);
            if (with_v) copy_floats(lds + p.lds_v[1], ly.VW + (size_t)r0 * ly.n_in, part1 * ly.n_in);
        }
    }
    const bool res_last = res_of(L), vres_last = res_last && with_v;
    if (res_last)
        for (int i = tid; i < nL * nc; i += kThreads) {
            const int k = i / nc, j = i - k * nc;
            lds[p.lds_w[L] + k * ncp + j] = last.W[(size_t)k * last.n_in + c0 + j];
            if (vres_last) lds[p.lds_v[L] + k * ncp + j] = last.VW[(size_t)k * last.n_in + c0 + j];
        }
    if (need_x)
        for (int k = tid; k < n0; k += kThreads) xa0[k] = p.X[k];
    int y_cur = p.labels[0];
    double loss_acc = 0.0;
    __syncthreads();

    // A first layer that is streamed (wholly or in part) and has short rows takes the one-pass
    // sweep: update of W_1 and the next sample's products with it together (sweep_rows16).
    const bool fast1 = L >= 2 && !res_of(1) && p.layer[1].vec4 != 0 && n0 <= 512 && p.layer[1].kshift == 0;
    bool have_z1 = false;   // kpart already holds layer 1's products with the current sample

    constexpr int XR = 4;
    for (int64_t s = 0; s < p.n_samples; ++s) {
        const uint32_t seq = p.seq0 + 1u + (uint32_t)s;
        const int par = (int)(seq & 1u);
        const int mode = (p.mu != 0.f) ? UPD_MOMENTUM : ((p.keep_v && s == p.n_samples - 1) ? UPD_KEEPV : UPD_SGD);
        const float *x = xa0 + (size_t)(s & 1) * n0p;
        float xr[XR];
        int y_next = 0;
        bool aborted = false;
        const bool more = s + 1 < p.n_samples;

#define DN_PREFETCH_X()                                                                           \
        do {                                                                                      \
            if (more) {                                                                           \
                const float *xn = p.X + (size_t)(s + 1) * n0;                                     \
                _Pragma("unroll") for (int u = 0; u < XR; ++u) {                                  \
                    const int k = tid + u * kThreads;                                             \
                    xr[u] = (need_x && k < n0) ? xn[k] : 0.f;                                     \
                }                                                                                 \
                y_next = p.labels[s + 1];                                                         \
            }                                                                                     \
        } while (0)
        // the prefetched features of the next sample into the other input buffer
        auto store_next_x = [&]() {
            float *xn = xa0 + (size_t)((s + 1) & 1) * n0p;
            if (need_x) {
#pragma unroll
                for (int u = 0; u < XR; ++u) {
                    const int k = tid + u * kThreads;
                    if (k < n0) xn[k] = xr[u];
                }
                for (int k = tid + XR * kThreads; k < n0; k += kThreads) xn[k] = p.X[(size_t)(s + 1) * n0 + k];
            }
        };

        // ---- forward through the row-split layers 1..L-1 -------------------------------
        for (int l = 1; l < L; ++l) {
            const OnlineLayer &ly = p.layer[l];
            const int r0 = w * ly.per;
            const int nr = max(0, min(ly.per, ly.n_out - r0));
            if (nr > 0) {
                const float *xin = x;
                if (l > 1) {
                    float *dst = lds + p.lds_a[l - 1];
                    const u64 *src = p.act_x[l - 1] + (size_t)par * ly.n_in;
                    poll_words(ly.n_in, seq, [&](int q) { return src + q; }, [&](int q, float v) { dst[q] = v; },
                               p.abort_flag, &s_abort);
                    __syncthreads();
                    if (s_abort) { aborted = true; break; }
                    xin = dst;
                }
                if (res_of(l)) {
                    const float *Wt = lds + p.lds_w[l];
                    if ((nr << ly.kshift) <= kWaves) {      // one (row, segment) per wave: no batching needed
                        if (ly.vec4) fwd_rows<4, 1>(Wt, ly.n_in, nr, ly.kshift, ly.seg, xin, kpart);
                        else fwd_rows<1, 1>(Wt, ly.n_in, nr, ly.kshift, ly.seg, xin, kpart);
                    } else {
                        if (ly.vec4) fwd_rows<4, 4>(Wt, ly.n_in, nr, ly.kshift, ly.seg, xin, kpart);
                        else fwd_rows<1, 4>(Wt, ly.n_in, nr, ly.kshift, ly.seg, xin, kpart);
                    }
                } else if (l == 1 && fast1) {
                    if (!have_z1) {   // (otherwise the previous step's sweep left the products in kpart)
                        if (part1 > 0)
                            sweep_rows16<false, true>(lds + p.lds_w[1], nullptr, ly.n_in, part1, nullptr, nullptr, xin, 0.f, 0.f,
                                                      UPD_SGD, kpart);
                        sweep_rows16<false, true>(ly.W + (size_t)(r0 + part1) * ly.n_in, nullptr, ly.n_in, nr - part1, nullptr,
                                                  nullptr, xin, 0.f, 0.f, UPD_SGD, kpart + part1);
                    }
                } else {
                    const int nl = (l == 1) ? part1 : 0;   // rows held in LDS; the rest is streamed
                    if (nl > 0) {
                        if (ly.vec4) fwd_rows<4, 4>(lds + p.lds_w[1], ly.n_in, nl, ly.kshift, ly.seg, xin, kpart);
                        else fwd_rows<1, 4>(lds + p.lds_w[1], ly.n_in, nl, ly.kshift, ly.seg, xin, kpart);
                    }
                    const float *Wt = ly.W + (size_t)(r0 + nl) * ly.n_in;   // streamed: four rows of loads in flight per wave (two and eight measured slower)
                    if (ly.vec4) fwd_rows<4, 4>(Wt, ly.n_in, nr - nl, ly.kshift, ly.seg, xin, kpart + (nl << ly.kshift));
                    else fwd_rows<1, 4>(Wt, ly.n_in, nr - nl, ly.kshift, ly.seg, xin, kpart + (nl << ly.kshift));
                }
                __syncthreads();
                float *a_own = lds + p.lds_own_a[l];
                const float *bl = lds + p.lds_b[l];
                for (int r = tid; r < nr; r += kThreads) {
                    float z = bl[r];
                    for (int ks = 0; ks < (1 << ly.kshift); ++ks) z += kpart[(r << ly.kshift) + ks];
                    const float a = act_fn(ly.act, z);
                    a_own[r] = a;
                    if (l <= L - 2) ll_store(p.act_x[l] + (size_t)par * ly.n_out + r0 + r, a, seq);
                }
                __syncthreads();
            }
            if (l == 1) DN_PREFETCH_X();
        }
        if (aborted) break;

        // ---- last layer: partial net inputs from own columns ---------------------------
        const float *a_last = (L == 1) ? (x + c0) : (lds + p.lds_own_a[L - 1]);
        if (nc > 0) {
            u64 *zout = p.z_x + ((size_t)par * last.P + w) * nL;
            if (res_last) fwd_cols(lds + p.lds_w[L], ncp, nL, nc, a_last, zout, seq);
            else fwd_cols(last.W + c0, last.n_in, nL, nc, a_last, zout, seq);
        }
        if (L == 1) DN_PREFETCH_X();

        // ---- output layer: z_L, loss, Delta_L (every owner of last-layer columns repeats it) ----
        if (need_z) {
            gather_partials(p.z_x + (size_t)par * last.P * nL, last.P, nL, 0, nL, seq, tmp,
                            [&](int k, float sum) { zL[k] = sum + bL[k]; }, p.abort_flag, &s_abort);
            if (s_abort) break;
            if (wave == 0) {
                int y = y_cur;
                y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
                const int k0 = lane, k1 = lane + 64;
                const float z0 = k0 < nL ? zL[k0] : -INFINITY, z1 = k1 < nL ? zL[k1] : -INFINITY;
                float d0, d1, e;
                if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                    const float m = wave_max(fmaxf(z0, z1));
                    const float e0 = k0 < nL ? expf(z0 - m) : 0.f, e1 = k1 < nL ? expf(z1 - m) : 0.f;
                    const float sum = wave_sum(e0 + e1);
                    const float inv = 1.0f / sum;
                    d0 = e0 * inv - (k0 == y ? 1.0f : 0.0f);
                    d1 = e1 * inv - (k1 == y ? 1.0f : 0.0f);
                    e = logf(sum) - (zL[y] - m);
                } else {
                    const float a0 = act_fn(last.act, z0), a1 = act_fn(last.act, z1);
                    const float f0 = a0 - (k0 == y ? 1.0f : 0.0f), f1 = a1 - (k1 == y ? 1.0f : 0.0f);
                    d0 = f0 * act_deriv(last.act, a0);
                    d1 = f1 * act_deriv(last.act, a1);
                    e = wave_sum((k0 < nL ? 0.5f * f0 * f0 : 0.f) + (k1 < nL ? 0.5f * f1 * f1 : 0.f));
                }
                if (k0 < nL) {
                    dL[k0] = d0;
                    bL[k0] = apply_update(bL[k0], p.lr * d0, vbL[k0], p.mu, mode);
                }
                if (k1 < nL) {
                    dL[k1] = d1;
                    bL[k1] = apply_update(bL[k1], p.lr * d1, vbL[k1], p.mu, mode);
                }
                if (lane == 0) loss_acc += (double)e;
            }
            __syncthreads();
            if (nc > 0) {
                float *d_prev = (L >= 2) ? (lds + p.lds_own_d[L - 1]) : nullptr;
                const int act_prev = (L >= 2) ? p.layer[L - 1].act : 0;
                float *Vt = vres_last ? (lds + p.lds_v[L]) : (last.VW + c0);
                const int vstride = vres_last ? ncp : last.n_in;
                if (res_last)
                    bwd_cols(lds + p.lds_w[L], ncp, Vt, vstride, nL, nc, a_last, dL, p.lr, p.mu, mode, d_prev,
                             act_prev);
                else
                    bwd_cols(last.W + c0, last.n_in, Vt, vstride, nL, nc, a_last, dL, p.lr, p.mu, mode, d_prev,
                             act_prev);
                __syncthreads();
            }
        }

        // ---- backward through the row-split layers L-1..1 ------------------------------
        for (int l = L - 1; l >= 1; --l) {
            const OnlineLayer &ly = p.layer[l];
            const int r0 = w * ly.per;
            const int nr = max(0, min(ly.per, ly.n_out - r0));
            if (nr <= 0) continue;
            float *d_own = lds + p.lds_own_d[l];
            const float *a_own = lds + p.lds_own_a[l];
            if (l < L - 1) {
                const OnlineLayer &up = p.layer[l + 1];
                gather_partials(p.part_x[l + 1] + (size_t)par * up.P * ly.n_out, up.P, ly.n_out, r0, nr, seq, tmp,
                                [&](int r, float sum) { d_own[r] = sum * act_deriv(ly.act, a_own[r]); },
                                p.abort_flag, &s_abort);
                if (s_abort) { aborted = true; break; }
            }
            const float *ain = (l == 1) ? x : (lds + p.lds_a[l - 1]);
            const bool res = res_of(l);
            float *Vt = (res && with_v) ? (lds + p.lds_v[l]) : (ly.VW + (size_t)r0 * ly.n_in);
            u64 *pout = (l >= 2) ? p.part_x[l] + ((size_t)par * ly.P + w) * ly.n_in : nullptr;
#define DN_BWD_ROWS(WT, RU)                                                                                   \
            do {                                                                                              \
                if (l >= 2) {                                                                                 \
                    if (ly.vec4) bwd_rows<4, RU>(WT, Vt, ly.n_in, nr, d_own, ain, p.lr, p.mu, mode, tmp, pout, seq); \
                    else bwd_rows<1, RU>(WT, Vt, ly.n_in, nr, d_own, ain, p.lr, p.mu, mode, tmp, pout, seq);  \
                } else {                                                                                      \
                    if (ly.vec4) bwd_flat<4, RU>(WT, Vt, ly.n_in, nr, d_own, ain, p.lr, p.mu, mode);          \
                    else bwd_flat<1, RU>(WT, Vt, ly.n_in, nr, d_own, ain, p.lr, p.mu, mode);                  \
                }                                                                                             \
            } while (0)
            if (res) {
                // small slices: one row (or one vector) per wave (thread), no batching of loads needed
                const int vec = ly.vec4 ? 4 : 1;
                const int C = (ly.n_in + 64 * vec - 1) / (64 * vec);
                const bool small = (l >= 2) ? (nr <= (C >= kWaves ? 1 : kWaves / C)) : (nr * ly.n_in <= kThreads * vec);
                if (small) DN_BWD_ROWS(lds + p.lds_w[l], 1);
                else DN_BWD_ROWS(lds + p.lds_w[l], 4);
            } else if (l == 1 && fast1) {
                // The next sample's features go to the other input buffer first: the sweep multiplies
                // each row with them right after updating it, which is layer 1's forward product of
                // the next step.  Rows held in LDS first, then the streamed rest of the block.
                float *xnext = xa0 + (size_t)((s + 1) & 1) * n0p;
                if (more) {
                    store_next_x();
                    __syncthreads();
                }
                float *Vl = with_v ? (lds + p.lds_v[1]) : (ly.VW + (size_t)r0 * ly.n_in);
                float *Wg = ly.W + (size_t)(r0 + part1) * ly.n_in, *Vg = ly.VW + (size_t)(r0 + part1) * ly.n_in;
                if (more) {
                    if (part1 > 0)
                        sweep_rows16<true, true>(lds + p.lds_w[1], Vl, ly.n_in, part1, d_own, ain, xnext, p.lr, p.mu, mode, kpart);
                    sweep_rows16<true, true>(Wg, Vg, ly.n_in, nr - part1, d_own + part1, ain, xnext, p.lr, p.mu, mode,
                                             kpart + part1);
                } else {
                    if (part1 > 0)
                        sweep_rows16<true, false>(lds + p.lds_w[1], Vl, ly.n_in, part1, d_own, ain, nullptr, p.lr, p.mu, mode, kpart);
                    sweep_rows16<true, false>(Wg, Vg, ly.n_in, nr - part1, d_own + part1, ain, nullptr, p.lr, p.mu, mode,
                                              kpart + part1);
                }
                have_z1 = more;
            } else if (l == 1 && part1 > 0) {
                // the rows held in LDS, then the streamed rest of the block
                float *Vl = with_v ? (lds + p.lds_v[1]) : (ly.VW + (size_t)r0 * ly.n_in);
                float *Wg = ly.W + (size_t)(r0 + part1) * ly.n_in, *Vg = ly.VW + (size_t)(r0 + part1) * ly.n_in;
                if (ly.vec4) {
                    bwd_flat<4, 4>(lds + p.lds_w[1], Vl, ly.n_in, part1, d_own, ain, p.lr, p.mu, mode);
                    bwd_flat<4, 4>(Wg, Vg, ly.n_in, nr - part1, d_own + part1, ain, p.lr, p.mu, mode);
                } else {
                    bwd_flat<1, 4>(lds + p.lds_w[1], Vl, ly.n_in, part1, d_own, ain, p.lr, p.mu, mode);
                    bwd_flat<1, 4>(Wg, Vg, ly.n_in, nr - part1, d_own + part1, ain, p.lr, p.mu, mode);
                }
            } else {
                DN_BWD_ROWS(ly.W + (size_t)r0 * ly.n_in, 4);
            }
#undef DN_BWD_ROWS
            float *bl = lds + p.lds_b[l], *vbl = bl + ((ly.per + 3) & ~3);
            for (int r = tid; r < nr; r += kThreads) {
                float vb = vbl[r];
                bl[r] = apply_update(bl[r], p.lr * d_own[r], vb, p.mu, mode);
                if (mode != UPD_SGD) vbl[r] = vb;
            }
            __syncthreads();
        }
        if (aborted) break;

        // ---- next sample into the other input buffer (the one-pass sweep has done it already) ----
        if (more) {
            if (!fast1) store_next_x();
            y_cur = y_next;
        }
        __syncthreads();
    }
#undef DN_PREFETCH_X

    // ---- epilogue: LDS images back to device memory -------------------------------------
    __syncthreads();
    const bool v_touched = p.mu != 0.f || p.keep_v;
    for (int l = 1; l < L; ++l) {
        const OnlineLayer &ly = p.layer[l];
        const int r0 = w * ly.per;
        const int nr = max(0, min(ly.per, ly.n_out - r0));
        const float *bl = lds + p.lds_b[l], *vbl = bl + ((ly.per + 3) & ~3);
        for (int r = tid; r < nr; r += kThreads) {
            ly.b[r0 + r] = bl[r];
            if (v_touched) ly.Vb[r0 + r] = vbl[r];
        }
        if (res_of(l) && nr > 0) copy_floats(ly.W + (size_t)r0 * ly.n_in, lds + p.lds_w[l], nr * ly.n_in);
        if (res_of(l) && with_v && nr > 0) copy_floats(ly.VW + (size_t)r0 * ly.n_in, lds + p.lds_v[l], nr * ly.n_in);
        if (l == 1 && part1 > 0) {
            copy_floats(ly.W + (size_t)r0 * ly.n_in, lds + p.lds_w[1], part1 * ly.n_in);
            if (with_v) copy_floats(ly.VW + (size_t)r0 * ly.n_in, lds + p.lds_v[1], part1 * ly.n_in);
        }
    }
    if (res_last)
        for (int i = tid; i < nL * nc; i += kThreads) {
            const int k = i / nc, j = i - k * nc;
            last.W[(size_t)k * last.n_in + c0 + j] = lds[p.lds_w[L] + k * ncp + j];
            if (vres_last) last.VW[(size_t)k * last.n_in + c0 + j] = lds[p.lds_v[L] + k * ncp + j];
        }
    if (w == 0) {
        if (tid == 0) *p.loss_acc += loss_acc;
        for (int k = tid; k < nL; k += kThreads) {
            last.b[k] = bL[k];
            if (v_touched) last.Vb[k] = vbL[k];
        }
    }
}


// Rank-B update of four consecutive columns of NQ own rows (persistent minibatch kernel):
// acc[q] += delta1[b][rc + q] * x_b[columns] over samples [bbeg, bend), sixteen samples' loads in flight.
template <int NQ>
__device__ __forceinline__ void w1_accumulate(v4f (&acc)[4], const float *__restrict__ Xcol, int n0, int bbeg, int bend,
                                              int Bs, const float *d1, int per, int rc)
{
    for (int bb0 = bbeg; bb0 < bend; bb0 += 16) {
        v4f x[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) x[u] = *(const v4f *)(Xcol + (size_t)min(bb0 + u, Bs - 1) * n0);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const float on = (bb0 + u < bend) ? 1.f : 0.f;   // a factor, not a branch
            const float *dr = d1 + min(bb0 + u, Bs - 1) * per + rc;
#pragma unroll
            for (int q = 0; q < NQ; ++q) acc[q] += x[u] * (dr[q] * on);
        }
    }
}

// Forward of a workgroup's own units for every sample of a batch (persistent minibatch kernel):
// a1[b * per + r] = f(W1[r] . x_b + b1[r]).  Sixteen lanes share one sample (four samples per wave
// at a time): a lane covers every sixteenth float4 of the row, keeps its part of W1[r] in
// registers for all samples, and one four-step DPP butterfly finishes four dot products at
// once.  Rows longer than 1024 go in chunks of 1024 columns.
__device__ __forceinline__ void fwd_batch(const float *__restrict__ Xb, int n0, int Bs, const float *w1, const float *b1,
                                          int nr, int per, int act, float *a1)
{
    constexpr int MAXIT = PB_MAX_BATCH / (kWaves * 4);   // sample slots a lane group may have to serve
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int nk4 = n0 / 4;
    const int nit = (Bs + kWaves * 4 - 1) / (kWaves * 4);
    const int nchunk = (nk4 + 255) / 256;
    for (int r = 0; r < nr; ++r) {
        float acc[MAXIT];
#pragma unroll
        for (int i = 0; i < MAXIT; ++i) acc[i] = 0.f;
        for (int c = 0; c < nchunk; ++c) {
            v4f wv[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int k4 = (c * 16 + j) * 16 + g;
                wv[j] = (k4 < nk4) ? *(const v4f *)(w1 + r * n0 + k4 * 4) : (v4f){0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int it = 0; it < MAXIT; ++it) {
                if (it < nit) {
                    const int b = min(it * (kWaves * 4) + wave * 4 + sg, Bs - 1);
                    v4f x[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int k4 = (c * 16 + j) * 16 + g;
                        x[j] = *(const v4f *)(Xb + (size_t)b * n0 + (k4 < nk4 ? k4 : 0) * 4);
                    }
                    float t = 0.f;
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        t += wv[j].x * x[j].x + wv[j].y * x[j].y + wv[j].z * x[j].z + wv[j].w * x[j].w;
                    acc[it] += t;
                }
            }
        }
        const float bias = b1[r];
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
            if (it < nit) {
                const int b = it * (kWaves * 4) + wave * 4 + sg;
                const float sum = row16_sum(acc[it]);
                if (g == 0 && b < Bs) a1[b * per + r] = act_fn(act, sum + bias);
            }
        }
    }
}

// ---- minibatch epochs of one- and two-layer nets as one persistent kernel ----------------
//
// Small nets at small and medium batch sizes are bound by launches when every product is its
// own kernel (a 784-128-10 net at batch 128 spends 50 us per step in eight launches that each
// do a few microseconds of work).  With at most two layers the ownership scheme of the
// per-sample kernel carries over to a batch without any wide exchange: a workgroup owns `per`
// hidden units -- their rows of W_1 and their columns of W_2, resident in LDS -- and needs
// from the others only the sum of the partial output net inputs.  That sum is taken per
// sample by the workgroup that owns the sample (reduce-scatter), which also computes the
// sample's loss and output delta and publishes them to everyone (all-gather): two hops per
// step, B * n_L numbers each.  Everything else (forward of the own units for all B samples,
// their deltas, the rank-B updates of the own rows and columns) is local; X is read from
// device memory (L2) twice per step.  A one-layer net is the same with its input features in
// the role of the hidden units.
template <int LT>   // the depth, one or two layers, at compile time: the branches on it go
__global__ __launch_bounds__(ON_THREADS) void batch_epoch_kernel(BatchPlan p)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ int s_abort;
    const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    constexpr int L = LT;
    const int n0 = p.n0, nL = p.nL, nL1 = p.nL + 1, per = p.per, maxB = p.max_batch;
    const int c0 = w * per;
    const int nr = max(0, min(per, p.n_mid - c0));   // own hidden units (L = 2) or input features (L = 1)
    const bool with_v = p.with_v != 0;
    float *w1 = lds + p.lds_w1, *v1 = lds + p.lds_v1, *b1 = lds + p.lds_b1, *vb1 = b1 + ((per + 3) & ~3);
    float *w2 = lds + p.lds_w2, *v2 = lds + p.lds_v2, *bL = lds + p.lds_bL, *vbL = bL + ON_MAX_NL;
    float *a1 = lds + p.lds_a1, *d1 = lds + p.lds_d1, *d2 = lds + p.lds_d2, *zs = lds + p.lds_zs;
    float *tmp = lds + p.lds_tmp;

    // ---- prologue: own slices into LDS ----
    if (tid == 0) s_abort = 0;
    for (int k = tid; k < nL; k += kThreads) {
        bL[k] = p.b2[k];
        vbL[k] = p.Vb2[k];
    }
    if (L == 2) {
        for (int r = tid; r < nr; r += kThreads) {
            b1[r] = p.b1[c0 + r];
            vb1[r] = p.Vb1[c0 + r];
        }
        copy_floats(w1, p.W1 + (size_t)c0 * n0, nr * n0);
        if (with_v) copy_floats(v1, p.VW1 + (size_t)c0 * n0, nr * n0);
    }
    for (int i = tid; i < nL * nr; i += kThreads) {
        const int k = i / nr, j = i - k * nr;
        w2[k * per + j] = p.W2[(size_t)k * p.n_mid + c0 + j];
        if (with_v) v2[k * per + j] = p.VW2[(size_t)k * p.n_mid + c0 + j];
    }
    double loss_acc = 0.0;
    float pf_sink = 0.f;   // keeps the prefetch loads alive
    __syncthreads();

    const int64_t nsteps = (p.n_samples + p.batch - 1) / p.batch;
    for (int64_t step = 0; step < nsteps; ++step) {
        const int64_t s0 = step * p.batch;
        const int Bs = (int)min((int64_t)p.batch, p.n_samples - s0);   // the last batch may be short
        const uint32_t seq = p.seq0 + 1u + (uint32_t)step;
        const int par = (int)(seq & 1u);
        const int mode = (p.mu != 0.f) ? UPD_MOMENTUM : ((p.keep_v && step == nsteps - 1) ? UPD_KEEPV : UPD_SGD);
        const float scale = p.lr / (float)Bs;
        const float *Xb = p.X + (size_t)s0 * n0;
        const int32_t *yb = p.labels + s0;

        // ---- 1. activations of the own units for every sample of the batch ----
        if (L == 2) {
            if (nr > 0) {
                fwd_batch(Xb, n0, Bs, w1, b1, nr, per, p.act1, a1);
            }
        } else {
            for (int q = tid; q < Bs * nr; q += kThreads) {
                const int b = q / nr, j = q - b * nr;
                a1[b * per + j] = Xb[(size_t)b * n0 + c0 + j];
            }
        }
        __syncthreads();

        // ---- 2. partial output net inputs from the own columns of the last layer ----
        if (nr > 0) {
            u64 *zout = p.z_x + ((size_t)par * p.P + w) * ((size_t)maxB * nL);
            for (int q = tid; q < Bs * nL; q += kThreads) {
                const int b = q / nL, k = q - b * nL;
                float z = 0.f;
                for (int j = 0; j < nr; ++j) z += w2[k * per + j] * a1[b * per + j];
                ll_store(zout + q, z, seq);
            }
        }

        // The next batch's features are pulled towards the L2 now, one word per 128-byte line,
        // so that the next step's passes over them do not start from device memory.  The
        // workgroups that (by the usual round-robin placement) share an XCD share the lines.
        if (L == 2 && step + 1 < nsteps) {
            const int64_t s1 = s0 + p.batch;
            const int64_t words = (int64_t)min((int64_t)p.batch, p.n_samples - s1) * n0;
            const float *Xn = p.X + (size_t)s1 * n0;
            const int nlocal = (p.P + 7) / 8, local = w / 8;
            for (int64_t line = (int64_t)local * kThreads + tid; line * 32 < words; line += (int64_t)nlocal * kThreads)
                pf_sink += Xn[line * 32];
        }

        // ---- 3. output stage for the samples this workgroup owns ----
        const int b0 = w * p.spw;
        const int nb = max(0, min(p.spw, Bs - b0));
        if (nb > 0) {
            gather_partials(p.z_x + (size_t)par * p.P * ((size_t)maxB * nL), p.P, maxB * nL, b0 * nL, nb * nL, seq, tmp,
                            [&](int e, float sum) { zs[e] = sum; }, p.abort_flag, &s_abort);
            if (s_abort) break;
            for (int bb = wave; bb < nb; bb += kWaves) {
                const float *z = zs + bb * nL;
                int y = yb[b0 + bb];
                y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
                const int k0 = lane, k1 = lane + 64;
                const float z0 = k0 < nL ? z[k0] + bL[k0] : -INFINITY, z1 = k1 < nL ? z[k1] + bL[k1] : -INFINITY;
                float d0, d1v, e;
                if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                    const float m = wave_max(fmaxf(z0, z1));
                    const float e0 = k0 < nL ? expf(z0 - m) : 0.f, e1 = k1 < nL ? expf(z1 - m) : 0.f;
                    const float sum = wave_sum(e0 + e1);
                    const float inv = 1.0f / sum;
                    d0 = e0 * inv - (k0 == y ? 1.0f : 0.0f);
                    d1v = e1 * inv - (k1 == y ? 1.0f : 0.0f);
                    e = logf(sum) - ((z[y] + bL[y]) - m);
                } else {
                    const float a0 = act_fn(p.actL, z0), a1v = act_fn(p.actL, z1);
                    const float f0 = a0 - (k0 == y ? 1.0f : 0.0f), f1 = a1v - (k1 == y ? 1.0f : 0.0f);
                    d0 = f0 * act_deriv(p.actL, a0);
                    d1v = f1 * act_deriv(p.actL, a1v);
                    e = wave_sum((k0 < nL ? 0.5f * f0 * f0 : 0.f) + (k1 < nL ? 0.5f * f1 * f1 : 0.f));
                }
                u64 *dout = p.d_x + (size_t)par * ((size_t)maxB * nL1) + (size_t)(b0 + bb) * nL1;
                if (k0 < nL) ll_store(dout + k0, d0, seq);
                if (k1 < nL) ll_store(dout + k1, d1v, seq);
                if (lane == 0) ll_store(dout + nL, e, seq);   // the sample's loss rides along
            }
        }

        // ---- 4. every workgroup takes in all output deltas ----
        {
            const u64 *dsrc = p.d_x + (size_t)par * ((size_t)maxB * nL1);
            poll_words(Bs * nL1, seq, [&](int q) { return dsrc + q; }, [&](int q, float v) { d2[q] = v; }, p.abort_flag,
                       &s_abort);
        }
        __syncthreads();
        if (s_abort) break;
        if (w == 0 && wave == 0) {   // the batch's losses, summed in a fixed tree
            double part = 0.0;
            for (int b = lane; b < Bs; b += 64) part += (double)d2[b * nL1 + nL];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o, 64);
            loss_acc += part;
        }
        // output bias (every workgroup keeps its own copy in step): 16 lanes per bias
        for (int t = tid; t < nL * 16; t += kThreads) {
            const int k = t >> 4, gq = t & 15;
            float g = 0.f;
            for (int b = gq; b < Bs; b += 16) g += d2[b * nL1 + k];
            g = row16_sum(g);
            if (gq == 0) bL[k] = apply_update(bL[k], scale * g, vbL[k], p.mu, mode);
        }

        // ---- 5. deltas of the own units (through the last layer's weights before their update) ----
        if (L == 2) {
            for (int q = tid; q < Bs * nr; q += kThreads) {
                const int b = q / nr, j = q - b * nr;
                float sacc = 0.f;
                for (int k = 0; k < nL; ++k) sacc += w2[k * per + j] * d2[b * nL1 + k];
                d1[b * per + j] = sacc * act_deriv(p.act1, a1[b * per + j]);
            }
        }
        __syncthreads();
        // ---- 6. rank-B update of the own columns of the last layer ----
        for (int t = tid; t < nL * nr * 16; t += kThreads) {
            const int q = t >> 4, gq = t & 15;
            const int k = q / nr, j = q - k * nr;
            float g = 0.f;
            for (int b = gq; b < Bs; b += 16) g += d2[b * nL1 + k] * a1[b * per + j];
            g = row16_sum(g);
            if (gq == 0) {
                const int idx = k * per + j;
                float v = with_v ? v2[idx] : 0.f;
                w2[idx] = apply_update(w2[idx], scale * g, v, p.mu, mode);
                if (mode == UPD_MOMENTUM) v2[idx] = v;
                else if (mode == UPD_KEEPV) p.VW2[(size_t)k * p.n_mid + c0 + j] = v;
            }
        }
        // ---- 7. rank-B update of the own rows of the first layer ----
        if (L == 2 && nr > 0) {
            // A thread owns four consecutive input columns and adds up, over the samples,
            // delta1[b][r] * x_b[columns] for four own rows at a time, sixteen samples' loads in
            // flight.  When the columns occupy at most half the threads the samples are split
            // between two halves of the workgroup; the second half hands its sums over through
            // LDS (a two-term sum: no order to fix).
            const int nk4 = n0 / 4;
            const int halves = (2 * nk4 <= kThreads && 4 * n0 <= kTmp) ? 2 : 1;
            const int half = (halves == 2 && tid >= kThreads / 2) ? 1 : 0;
            const int t0 = halves == 2 ? tid - half * (kThreads / 2) : tid;
            const int tstep = halves == 2 ? kThreads / 2 : kThreads;
            const int bmid = halves == 2 ? (Bs + 1) / 2 : Bs;
            const int bbeg = half ? bmid : 0, bend = half ? Bs : bmid;
            for (int rc = 0; rc < nr; rc += 4) {
                for (int kb = 0; kb < nk4; kb += tstep) {     // one pass unless there are more columns than threads
                    const int k4 = kb + t0;
                    const bool on = k4 < nk4;
                    v4f acc[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
                    if (on) {
                        const float *Xcol = Xb + k4 * 4;
                        switch (min(4, nr - rc)) {
                        case 1: w1_accumulate<1>(acc, Xcol, n0, bbeg, bend, Bs, d1, per, rc); break;
                        case 2: w1_accumulate<2>(acc, Xcol, n0, bbeg, bend, Bs, d1, per, rc); break;
                        case 3: w1_accumulate<3>(acc, Xcol, n0, bbeg, bend, Bs, d1, per, rc); break;
                        default: w1_accumulate<4>(acc, Xcol, n0, bbeg, bend, Bs, d1, per, rc); break;
                        }
                    }
                    if (halves == 2) {
                        if (half == 1 && on) {
#pragma unroll
                            for (int q = 0; q < 4; ++q) *(v4f *)(tmp + q * n0 + k4 * 4) = acc[q];
                        }
                        __syncthreads();
                        if (half == 0 && on) {
#pragma unroll
                            for (int q = 0; q < 4; ++q) acc[q] += *(const v4f *)(tmp + q * n0 + k4 * 4);
                        }
                    }
                    if (half == 0 && on) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int r = rc + q;
                            if (r < nr) {
                                const int idx = r * n0 + k4 * 4;
                                v4f wv = *(v4f *)(w1 + idx);
                                v4f vv = with_v ? *(v4f *)(v1 + idx) : (v4f){0.f, 0.f, 0.f, 0.f};
                                float wn[4], vn[4];
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    vn[e] = vv[e];
                                    wn[e] = apply_update(wv[e], scale * acc[q][e], vn[e], p.mu, mode);
                                }
                                *(v4f *)(w1 + idx) = (v4f){wn[0], wn[1], wn[2], wn[3]};
                                if (mode == UPD_MOMENTUM) *(v4f *)(v1 + idx) = (v4f){vn[0], vn[1], vn[2], vn[3]};
                                else if (mode == UPD_KEEPV)
                                    *(v4f *)(p.VW1 + (size_t)(c0 + r) * n0 + k4 * 4) = (v4f){vn[0], vn[1], vn[2], vn[3]};
                            }
                        }
                    }
                    if (halves == 2) __syncthreads();   // tmp is free again
                }
            }
            for (int t = tid; t < nr * 16; t += kThreads) {   // biases of the own units, 16 lanes each
                const int r = t >> 4, gq = t & 15;
                float g = 0.f;
                for (int b = gq; b < Bs; b += 16) g += d1[b * per + r];
                g = row16_sum(g);
                if (gq == 0) b1[r] = apply_update(b1[r], scale * g, vb1[r], p.mu, mode);
            }
        }
        __syncthreads();
    }

    // ---- epilogue: LDS images back to device memory ----
    __syncthreads();
    const bool v_touched = p.mu != 0.f || p.keep_v;
    if (L == 2) {
        for (int r = tid; r < nr; r += kThreads) {
            p.b1[c0 + r] = b1[r];
            if (v_touched) p.Vb1[c0 + r] = vb1[r];
        }
        if (nr > 0) copy_floats(p.W1 + (size_t)c0 * n0, w1, nr * n0);
        if (with_v && nr > 0) copy_floats(p.VW1 + (size_t)c0 * n0, v1, nr * n0);
    }
    for (int i = tid; i < nL * nr; i += kThreads) {
        const int k = i / nr, j = i - k * nr;
        p.W2[(size_t)k * p.n_mid + c0 + j] = w2[k * per + j];
        if (with_v) p.VW2[(size_t)k * p.n_mid + c0 + j] = v2[k * per + j];
    }
    if (pf_sink == 1.2345678e-30f) *p.abort_flag = 0;   // never true in practice; the loads must not be dropped
    if (w == 0) {
        if (tid == 0) *p.loss_acc += loss_acc;
        for (int k = tid; k < nL; k += kThreads) {
            p.b2[k] = bL[k];
            if (v_touched) p.Vb2[k] = vbL[k];
        }
    }
}


// ---- minibatch epochs of deeper nets (plain gradient descent) as one persistent kernel ----

// How a matrix in device memory is read: plainly (the caller's X, read-only), or with relaxed
// device-scope atomic loads that bypass the per-XCD L2 (matrices other workgroups wrote moments
// ago).  (Invalidating the caches once per exchange and then loading plainly was measured: the
// invalidation alone costs about 10 us per exchange, more than the bypassing loads.)
// A loader is built from the matrix's first element (wave uniform) and reads the four floats at an
// element offset.  The bypassing form is one 16-byte buffer load with the device-scope cache policy
// (the policy a device-scope atomic load gets); four 4-byte atomic loads per float4 were the first
// version and cost four times the memory instructions.  The data needs no atomicity: it was complete
// before its producer's stamp became visible, and is read after the stamp was seen.
struct PlainLoad {
    const float *base;
    __device__ __forceinline__ explicit PlainLoad(const float *b) : base(b) {}
    __device__ __forceinline__ v4f ld(int off) const { return *(const v4f *)(base + off); }
};
struct CoherentLoad {
    typedef unsigned int v4u __attribute__((ext_vector_type(4)));
    __amdgpu_buffer_rsrc_t rsrc;
    // raw buffer over [b, b + 2 GB): 32-bit byte offsets, no stride; 0x00020000: 32-bit data format
    __device__ __forceinline__ explicit CoherentLoad(const float *b)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(b), 0, 0x7fffffff, 0x00020000)) {}
    __device__ __forceinline__ v4f ld(int off) const
    {
        constexpr int kDeviceScope = 16;   // the sc1 bit of the cache policy operand
        const v4u u = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off * 4, 0, kDeviceScope);
        return (v4f){__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w)};
    }
};

// The same product for batches of at most 16 rows of M, where a lane group per row of M would leave
// most waves idle: the 32 lane groups of the workgroup split into (row of M) x (part of k), a lane
// issues JN loads, the parts' sums meet in tmp (one barrier per four tile rows).  Bp: the power of
// two >= Bs that divides 32.  Contains barriers: call from uniform control flow.
template <class Load, int JN, class Fin>
__device__ __forceinline__ void tile_times_rows_split(const float *__restrict__ M, int n, int Bs, int Bp, const float *T, int nr,
                                                      float *tmp, Fin fin)
{
    const Load load(M);
    const int grp = threadIdx.x >> 4, g = threadIdx.x & 15;
    const int b = grp & (Bp - 1), part = grp / Bp, parts = 32 / Bp;
    const int nk4 = n / 4;
    const int cols = ((nk4 + parts - 1) / parts + 15) & ~15;   // float4 columns per part, whole lane strides
    const int kbeg = part * cols, kend = min(nk4, kbeg + cols);
    const int bc = min(b, Bs - 1);
    for (int rc = 0; rc < nr; rc += 4) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c0 = kbeg; c0 < kbeg + cols; c0 += 16 * JN) {
            v4f x[JN];
#pragma unroll
            for (int j = 0; j < JN; ++j) {
                const int k4 = c0 + j * 16 + g;
                x[j] = load.ld(bc * n + (k4 < kend ? k4 : 0) * 4);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row = min(rc + q, nr - 1);
                float t = 0.f;
#pragma unroll
                for (int j = 0; j < JN; ++j) {
                    const int k4 = c0 + j * 16 + g;
                    const v4f wv = *(const v4f *)(T + row * n + (k4 < kend ? k4 : 0) * 4);
                    const float d = wv.x * x[j].x + wv.y * x[j].y + wv.z * x[j].z + wv.w * x[j].w;
                    t += k4 < kend ? d : 0.f;
                }
                acc[q] += t;
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float sum = row16_sum(acc[q]);
            if (g == 0) tmp[(part * Bp + b) * 4 + q] = sum;
        }
        __syncthreads();
        for (int t = threadIdx.x; t < Bs * 4; t += kThreads) {
            const int bb = t >> 2, q = t & 3;
            if (rc + q < nr) {
                float sum = 0.f;
                for (int pp = 0; pp < parts; ++pp) sum += tmp[(pp * Bp + bb) * 4 + q];
                fin(bb, rc + q, sum);
            }
        }
        __syncthreads();
    }
}

// out(b, r) = sum_k T[r][k] * M[b][k] for the nr rows of an LDS tile T (pitch n) and every row b
// of a device matrix M (Bs x n, pitch n): sixteen lanes per row of M, four rows of M per wave at a
// time, four tile rows per pass over M.  fin(b, r, sum) finishes an element.
template <class Load, class Fin>
__device__ __forceinline__ void tile_times_rows(const float *__restrict__ M, int n, int Bs, const float *T, int nr, Fin fin)
{
    constexpr int MAXIT = PD_MAX_BATCH / (kWaves * 4);
    const Load load(M);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sg = lane >> 4, g = lane & 15;
    const int nk4 = n / 4;
    const int nit = (Bs + kWaves * 4 - 1) / (kWaves * 4);
    const int nchunk = (nk4 + 255) / 256;
    for (int rc = 0; rc < nr; rc += 4) {
        float acc[MAXIT][4];
#pragma unroll
        for (int i = 0; i < MAXIT; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[i][q] = 0.f;
        for (int c = 0; c < nchunk; ++c) {
#pragma unroll
            for (int it = 0; it < MAXIT; ++it) {
                if (it < nit && it * (kWaves * 4) + wave * 4 < Bs) {   // waves whose four slots are all past the batch sit out
                    const int b = min(it * (kWaves * 4) + wave * 4 + sg, Bs - 1);
                    v4f x[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int k4 = (c * 16 + j) * 16 + g;
                        x[j] = load.ld(b * n + (k4 < nk4 ? k4 : 0) * 4);
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (rc + q < nr) {
                            float t = 0.f;
#pragma unroll
                            for (int j = 0; j < 16; ++j) {
                                // (unconditional load from a clamped address, masked product: a load
                                // behind a test is waited for before the next one is issued)
                                const int k4 = (c * 16 + j) * 16 + g;
                                const v4f wv = *(const v4f *)(T + (rc + q) * n + (k4 < nk4 ? k4 : 0) * 4);
                                const float d = wv.x * x[j].x + wv.y * x[j].y + wv.z * x[j].z + wv.w * x[j].w;
                                t += k4 < nk4 ? d : 0.f;
                            }
                            acc[it][q] += t;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int it = 0; it < MAXIT; ++it) {
            if (it < nit && it * (kWaves * 4) + wave * 4 < Bs) {
                const int b = it * (kWaves * 4) + wave * 4 + sg;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (rc + q < nr) {
                        const float sum = row16_sum(acc[it][q]);
                        if (g == 0 && b < Bs) fin(b, rc + q, sum);
                    }
                }
            }
        }
    }
}

// The product in the form that suits the batch: up to 16 rows of M split k among lane groups
// (measured on 1024-wide layers, batch 8: 3.6 -> 2.x us per product), larger batches give every
// lane group a row of M.  Contains barriers for small batches: call from uniform control flow.
template <class Load, class Fin>
__device__ __forceinline__ void tile_product(const float *__restrict__ M, int n, int Bs, const float *T, int nr, float *tmp,
                                             Fin fin)
{
    if (Bs <= 4) tile_times_rows_split<Load, 4>(M, n, Bs, 4, T, nr, tmp, fin);
    else if (Bs <= 8) tile_times_rows_split<Load, 4>(M, n, Bs, 8, T, nr, tmp, fin);
    else if (Bs <= 16) tile_times_rows_split<Load, 8>(M, n, Bs, 16, T, nr, tmp, fin);
    else tile_times_rows<Load>(M, n, Bs, T, nr, fin);
}

template <int NQ, class Load>
__device__ __forceinline__ void rank_accumulate(v4f (&acc)[4], const Load &load, int col, int n, int bbeg, int bend,
                                                int Bs, const float *D, int dper, int rc)
{
    for (int bb0 = bbeg; bb0 < bend; bb0 += 8) {
        v4f x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = load.ld(min(bb0 + u, Bs - 1) * n + col);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float on = (bb0 + u < bend) ? 1.f : 0.f;
            const float *dr = D + min(bb0 + u, Bs - 1) * dper + rc;
#pragma unroll
            for (int q = 0; q < NQ; ++q) acc[q] += x[u] * (dr[q] * on);
        }
    }
}

// T[r][k] -= scale * sum_b D[b][r] * M[b][k] for an LDS tile T (nr rows, pitch n), D in LDS
// (pitch dper), M a device matrix (Bs x n).  With `halves` == 2 the samples are split between the
// two halves of the workgroup (second half hands its sums over through tmp).  On the last step of
// a plain-gradient-descent epoch (keepv) the applied change is also written to Vrows (device rows
// of the velocity, pitch n), if given.  Contains barriers: call from uniform control flow.
template <class Load>
__device__ __forceinline__ void tile_rank_update(float *T, float *Vrows, int n, int nr, const float *D, int dper,
                                                 const float *__restrict__ M, int Bs, float scale, bool keepv, float *tmp,
                                                 int halves)
{
    const Load load(M);
    const int tid = threadIdx.x;
    const int nk4 = n / 4;
    const int half = (halves == 2 && tid >= kThreads / 2) ? 1 : 0;
    const int t0 = halves == 2 ? tid - half * (kThreads / 2) : tid;
    const int tstep = halves == 2 ? kThreads / 2 : kThreads;
    const int bmid = halves == 2 ? (Bs + 1) / 2 : Bs;
    const int bbeg = half ? bmid : 0, bend = half ? Bs : bmid;
    for (int rc = 0; rc < nr; rc += 4) {
        for (int kb = 0; kb < nk4; kb += tstep) {
            const int k4 = kb + t0;
            const bool on = k4 < nk4;
            v4f acc[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = (v4f){0.f, 0.f, 0.f, 0.f};
            if (on) {
                const int col = k4 * 4;
                switch (min(4, nr - rc)) {
                case 1: rank_accumulate<1, Load>(acc, load, col, n, bbeg, bend, Bs, D, dper, rc); break;
                case 2: rank_accumulate<2, Load>(acc, load, col, n, bbeg, bend, Bs, D, dper, rc); break;
                case 3: rank_accumulate<3, Load>(acc, load, col, n, bbeg, bend, Bs, D, dper, rc); break;
                default: rank_accumulate<4, Load>(acc, load, col, n, bbeg, bend, Bs, D, dper, rc); break;
                }
            }
            if (halves == 2) {
                if (half == 1 && on) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) *(v4f *)(tmp + q * n + k4 * 4) = acc[q];
                }
                __syncthreads();
                if (half == 0 && on) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[q] += *(const v4f *)(tmp + q * n + k4 * 4);
                }
            }
            if (half == 0 && on) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int r = rc + q;
                    if (r < nr) {
                        const int idx = r * n + k4 * 4;
                        const v4f wv = *(const v4f *)(T + idx);
                        const v4f dv = acc[q] * (-scale);
                        *(v4f *)(T + idx) = wv + dv;
                        if (keepv && Vrows) *(v4f *)(Vrows + (size_t)r * n + k4 * 4) = dv;
                    }
                }
            }
            if (halves == 2) __syncthreads();
        }
    }
}

__global__ __launch_bounds__(ON_THREADS) void deep_batch_epoch_kernel(DeepPlan p)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ int s_abort;
    const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int L = p.L, nL = p.layer[L].n_out, nL1 = nL + 1, maxB = p.max_batch, n0 = p.layer[1].n_in;
    const DeepLayer &last = p.layer[L];
    const int perL = p.layer[L - 1].per;                 // own units of layer L-1 = own columns of W_L
    const int cL = w * perL;
    const int ncL = max(0, min(perL, last.n_in - cL));
    float *w2 = lds + p.lds_w2, *bL = lds + p.lds_bL, *d2 = lds + p.lds_d2, *zs = lds + p.lds_zs, *tmp = lds + p.lds_tmp;
    auto own_c0 = [&](int l) { return w * p.layer[l].per; };
    auto own_nr = [&](int l) { return max(0, min(p.layer[l].per, p.layer[l].n_out - w * p.layer[l].per)); };

    // ---- prologue: own slices into LDS ----
    if (tid == 0) s_abort = 0;
    for (int k = tid; k < nL; k += kThreads) bL[k] = last.b[k];
    for (int l = 1; l < L; ++l) {
        const DeepLayer &ly = p.layer[l];
        const int c0 = own_c0(l), nr = own_nr(l);
        float *bl = lds + p.lds_b[l];
        for (int r = tid; r < nr; r += kThreads) bl[r] = ly.b[c0 + r];
        if (nr > 0) copy_floats(lds + p.lds_r[l], ly.W + (size_t)c0 * ly.n_in, nr * ly.n_in);
        if (l >= 2) {   // transposed copy of the weights leaving this workgroup's units of layer l-1
            const int cp = own_c0(l - 1), np = own_nr(l - 1);
            float *ct = lds + p.lds_ct[l];
            for (int i = tid; i < np * ly.n_out; i += kThreads) {
                const int j = i / ly.n_out, o = i - j * ly.n_out;
                ct[j * ly.n_out + o] = ly.W[(size_t)o * ly.n_in + cp + j];
            }
        }
    }
    for (int i = tid; i < nL * ncL; i += kThreads) {
        const int k = i / ncL, j = i - k * ncL;
        w2[k * perL + j] = last.W[(size_t)k * last.n_in + cL + j];
    }
    double loss_acc = 0.0;
    float pf_sink = 0.f;
    __syncthreads();

    const int64_t nsteps = (p.n_samples + p.batch - 1) / p.batch;
    for (int64_t step = 0; step < nsteps; ++step) {
        const int64_t s0 = step * p.batch;
        const int Bs = (int)min((int64_t)p.batch, p.n_samples - s0);
        const uint32_t seq = p.seq0 + 1u + (uint32_t)step;
        const int par = (int)(seq & 1u);
        const bool keepv = p.keep_v && step == nsteps - 1;
        const float scale = p.lr / (float)Bs;
        const float *Xb = p.X + (size_t)s0 * n0;
        const int32_t *yb = p.labels + s0;
        bool aborted = false;

        // ---- forward through the hidden layers ----
        for (int l = 1; l < L; ++l) {
            const DeepLayer &ly = p.layer[l];
            const int c0 = own_c0(l), nr = own_nr(l);
            float *a_own = lds + p.lds_a[l];
            if (nr > 0) {
                const float *bl = lds + p.lds_b[l];
                const float *T = lds + p.lds_r[l];
                const int per = ly.per, act = ly.act;
                auto fin = [&](int b, int r, float sum) { a_own[b * per + r] = act_fn(act, sum + bl[r]); };
                if (l == 1) {
                    tile_product<PlainLoad>(Xb, ly.n_in, Bs, T, nr, tmp, fin);
                } else {
                    const u64 *flags = p.fa[l - 1] + (size_t)par * p.grid;
                    poll_words(p.layer[l - 1].P, seq, [&](int q) { return flags + q; }, [&](int, float) {}, p.abort_flag,
                               &s_abort);
                    __syncthreads();
                    if (s_abort) { aborted = true; break; }
                    tile_product<CoherentLoad>(p.ea[l - 1] + (size_t)par * maxB * ly.n_in, ly.n_in, Bs, T, nr, tmp, fin);
                }
            }
            __syncthreads();
            if (l <= L - 2 && nr > 0) {   // publish the own slice, then say so
                float *dst = p.ea[l] + (size_t)par * maxB * ly.n_out;
                for (int q = tid; q < Bs * nr; q += kThreads) {
                    const int b = q / nr, r = q - b * nr;
                    __hip_atomic_store(dst + (size_t)b * ly.n_out + c0 + r, a_own[b * ly.per + r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                }
                drain_device_scope_stores();   // every wave: its part of the slice has reached device scope
                __syncthreads();               // ... before thread 0 announces the slice
                if (tid == 0) ll_store(p.fa[l] + (size_t)par * p.grid + w, 0.f, seq);
            }
        }
        if (aborted) break;

        // ---- output layer: partial net inputs from own columns (every workgroup publishes) ----
        const float *aL = lds + p.lds_a[L - 1];
        {
            u64 *zout = p.z_x + ((size_t)par * p.grid + w) * ((size_t)maxB * nL);
            for (int q = tid; q < Bs * nL; q += kThreads) {
                const int b = q / nL, k = q - b * nL;
                float z = 0.f;
                for (int j = 0; j < ncL; ++j) z += w2[k * perL + j] * aL[b * perL + j];
                ll_store(zout + q, z, seq);
            }
        }
        if (step + 1 < nsteps) {   // next batch towards the L2, one word per 128-byte line
            const int64_t s1 = s0 + p.batch;
            const int64_t words = (int64_t)min((int64_t)p.batch, p.n_samples - s1) * n0;
            const float *Xn = p.X + (size_t)s1 * n0;
            const int nlocal = (p.grid + 7) / 8, local = w / 8;
            for (int64_t line = (int64_t)local * kThreads + tid; line * 32 < words; line += (int64_t)nlocal * kThreads)
                pf_sink += Xn[line * 32];
        }
        const int b0 = w * p.spw;
        const int nb = max(0, min(p.spw, Bs - b0));
        if (nb > 0) {
            gather_partials(p.z_x + (size_t)par * p.grid * ((size_t)maxB * nL), p.grid, maxB * nL, b0 * nL, nb * nL, seq,
                            tmp, [&](int e, float sum) { zs[e] = sum; }, p.abort_flag, &s_abort);
            if (s_abort) break;
            for (int bb = wave; bb < nb; bb += kWaves) {
                const float *z = zs + bb * nL;
                int y = yb[b0 + bb];
                y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
                const int k0 = lane, k1 = lane + 64;
                const float z0 = k0 < nL ? z[k0] + bL[k0] : -INFINITY, z1 = k1 < nL ? z[k1] + bL[k1] : -INFINITY;
                float d0, d1v, e;
                if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                    const float m = wave_max(fmaxf(z0, z1));
                    const float e0 = k0 < nL ? expf(z0 - m) : 0.f, e1 = k1 < nL ? expf(z1 - m) : 0.f;
                    const float sum = wave_sum(e0 + e1);
                    const float inv = 1.0f / sum;
                    d0 = e0 * inv - (k0 == y ? 1.0f : 0.0f);
                    d1v = e1 * inv - (k1 == y ? 1.0f : 0.0f);
                    e = logf(sum) - ((z[y] + bL[y]) - m);
                } else {
                    const float a0 = act_fn(last.act, z0), a1v = act_fn(last.act, z1);
                    const float f0 = a0 - (k0 == y ? 1.0f : 0.0f), f1 = a1v - (k1 == y ? 1.0f : 0.0f);
                    d0 = f0 * act_deriv(last.act, a0);
                    d1v = f1 * act_deriv(last.act, a1v);
                    e = wave_sum((k0 < nL ? 0.5f * f0 * f0 : 0.f) + (k1 < nL ? 0.5f * f1 * f1 : 0.f));
                }
                u64 *dout = p.d_x + (size_t)par * ((size_t)maxB * nL1) + (size_t)(b0 + bb) * nL1;
                if (k0 < nL) ll_store(dout + k0, d0, seq);
                if (k1 < nL) ll_store(dout + k1, d1v, seq);
                if (lane == 0) ll_store(dout + nL, e, seq);
            }
        }
        {
            const u64 *dsrc = p.d_x + (size_t)par * ((size_t)maxB * nL1);
            poll_words(Bs * nL1, seq, [&](int q) { return dsrc + q; }, [&](int q, float v) { d2[q] = v; }, p.abort_flag,
                       &s_abort);
        }
        __syncthreads();
        if (s_abort) break;
        if (w == 0 && wave == 0) {
            double part = 0.0;
            for (int b = lane; b < Bs; b += 64) part += (double)d2[b * nL1 + nL];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o, 64);
            loss_acc += part;
        }
        for (int t = tid; t < nL * 16; t += kThreads) {
            const int k = t >> 4, gq = t & 15;
            float g = 0.f;
            for (int b = gq; b < Bs; b += 16) g += d2[b * nL1 + k];
            g = row16_sum(g);
            if (gq == 0) {
                const float dv = -scale * g;
                bL[k] += dv;
                if (keepv && w == 0) last.Vb[k] = dv;
            }
        }
        // deltas of the own units of layer L-1 through the last layer's weights before their update
        {
            float *dl = lds + p.lds_dl[L - 1];
            const int actp = p.layer[L - 1].act;
            for (int q = tid; q < Bs * ncL; q += kThreads) {
                const int b = q / ncL, j = q - b * ncL;
                float sacc = 0.f;
                for (int k = 0; k < nL; ++k) sacc += w2[k * perL + j] * d2[b * nL1 + k];
                dl[b * perL + j] = sacc * act_deriv(actp, aL[b * perL + j]);
            }
        }
        __syncthreads();
        for (int t = tid; t < nL * ncL * 16; t += kThreads) {
            const int q = t >> 4, gq = t & 15;
            const int k = q / ncL, j = q - k * ncL;
            float g = 0.f;
            for (int b = gq; b < Bs; b += 16) g += d2[b * nL1 + k] * aL[b * perL + j];
            g = row16_sum(g);
            if (gq == 0) {
                const float dv = -scale * g;
                w2[k * perL + j] += dv;
                if (keepv) last.VW[(size_t)k * last.n_in + cL + j] = dv;
            }
        }

        // ---- backward through the hidden layers ----
        // the own slice of layer l's deltas to the exchange matrix, then the stamp that says so (l >= 2)
        auto publish_delta = [&](int l) {
            const DeepLayer &ly = p.layer[l];
            const int c0 = own_c0(l), nr = own_nr(l);
            if (l < 2 || nr <= 0) return;
            const float *dl = lds + p.lds_dl[l];
            float *dst = p.ed[l] + (size_t)par * maxB * ly.n_out;
            for (int q = tid; q < Bs * nr; q += kThreads) {
                const int b = q / nr, r = q - b * nr;
                __hip_atomic_store(dst + (size_t)b * ly.n_out + c0 + r, dl[b * ly.per + r], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            drain_device_scope_stores();
            __syncthreads();
            if (tid == 0) ll_store(p.fd[l] + (size_t)par * p.grid + w, 0.f, seq);
        };
        for (int l = L - 1; l >= 1; --l) {
            const DeepLayer &ly = p.layer[l];
            const int c0 = own_c0(l), nr = own_nr(l);
            float *dl = lds + p.lds_dl[l];
            // everyone needs this layer's deltas.  Layer L-1's slice is published here; the slices of
            // the layers below were published as soon as they existed (further down), before the
            // column copy's update, so that the update runs while the exchange is in flight
            if (l == L - 1) publish_delta(l);
            if (nr > 0) {   // own rows of W_l and their biases
                float *Vrows = ly.VW + (size_t)c0 * ly.n_in;
                if (l == 1)
                    tile_rank_update<PlainLoad>(lds + p.lds_r[l], Vrows, ly.n_in, nr, dl, ly.per, Xb, Bs, scale, keepv, tmp,
                                                p.halves);
                else
                    tile_rank_update<CoherentLoad>(lds + p.lds_r[l], Vrows, ly.n_in, nr, dl, ly.per,
                                                   p.ea[l - 1] + (size_t)par * maxB * ly.n_in, Bs, scale, keepv, tmp,
                                                   p.halves);
                float *bl = lds + p.lds_b[l];
                for (int t = tid; t < nr * 16; t += kThreads) {
                    const int r = t >> 4, gq = t & 15;
                    float g = 0.f;
                    for (int b = gq; b < Bs; b += 16) g += dl[b * ly.per + r];
                    g = row16_sum(g);
                    if (gq == 0) {
                        const float dv = -scale * g;
                        bl[r] += dv;
                        if (keepv) ly.Vb[c0 + r] = dv;
                    }
                }
            }
            if (l >= 2) {
                const DeepLayer &lp = p.layer[l - 1];
                const int np = own_nr(l - 1);
                if (np > 0) {   // deltas of the own units of layer l-1, then the second copy's update
                    const u64 *flags = p.fd[l] + (size_t)par * p.grid;
                    poll_words(ly.P, seq, [&](int q) { return flags + q; }, [&](int, float) {}, p.abort_flag, &s_abort);
                    __syncthreads();
                    if (s_abort) { aborted = true; break; }
                    const float *Dm = p.ed[l] + (size_t)par * maxB * ly.n_out;
                    float *dp = lds + p.lds_dl[l - 1];
                    const float *ap = lds + p.lds_a[l - 1];
                    const int pper = lp.per, actp = lp.act;
                    tile_product<CoherentLoad>(Dm, ly.n_out, Bs, lds + p.lds_ct[l], np, tmp, [&](int b, int j, float sum) {
                        dp[b * pper + j] = sum * act_deriv(actp, ap[b * pper + j]);
                    });
                    __syncthreads();
                    publish_delta(l - 1);
                    tile_rank_update<CoherentLoad>(lds + p.lds_ct[l], nullptr, ly.n_out, np, ap, pper, Dm, Bs, scale, false,
                                                   tmp, p.halves);
                }
            }
            __syncthreads();
        }
        if (aborted) break;
    }

    // ---- epilogue: LDS images back to device memory ----
    __syncthreads();
    for (int l = 1; l < L; ++l) {
        const DeepLayer &ly = p.layer[l];
        const int c0 = own_c0(l), nr = own_nr(l);
        const float *bl = lds + p.lds_b[l];
        for (int r = tid; r < nr; r += kThreads) ly.b[c0 + r] = bl[r];
        if (nr > 0) copy_floats(ly.W + (size_t)c0 * ly.n_in, lds + p.lds_r[l], nr * ly.n_in);
    }
    for (int i = tid; i < nL * ncL; i += kThreads) {
        const int k = i / ncL, j = i - k * ncL;
        last.W[(size_t)k * last.n_in + cL + j] = w2[k * perL + j];
    }
    if (pf_sink == 1.2345678e-30f) *p.abort_flag = 0;
    if (w == 0) {
        if (tid == 0) *p.loss_acc += loss_acc;
        for (int k = tid; k < nL; k += kThreads) last.b[k] = bL[k];
    }
}

}  // namespace

// ---- host side -------------------------------------------------------------------

bool online_geometry(const int32_t *n, int L, int min_tile, bool want_v, OnlineGeom &g)
{
    g = OnlineGeom{};
    if (L < 1 || L > ON_MAX_L) return false;
    if (n[L] > ON_MAX_NL) return false;
    if (min_tile < 1) min_tile = 1;
    auto cdiv = [](int64_t a, int64_t b) { return (int)((a + b - 1) / b); };
    auto pad4 = [](int v) { return (v + 3) & ~3; };
    g.L = L;
    int grid = 1;
    for (int l = 1; l <= L; ++l) {
        // rows (layers < L) or, for a one-layer net, input columns of the last layer
        const int units = (l < L) ? n[l] : n[L - 1];
        const int other = (l < L) ? n[l - 1] : n[L];
        int per;
        if (l == L && L >= 2) {
            per = g.per[L - 1];   // the last layer's column blocks are the row blocks of layer L-1
        } else {
            per = std::max(cdiv(units, ON_MAX_WG), cdiv(min_tile, other));
            per = std::min(per, units);
        }
        if ((int64_t)per * n[l - 1] > ((int64_t)1 << 30)) return false;
        g.per[l] = per;
        g.P[l] = cdiv(units, per);
        grid = std::max(grid, g.P[l]);
        const bool vec4 = (n[l - 1] % 4) == 0;
        g.vec4[l] = vec4 ? 1 : 0;
        if (l < L) {
            // forward: a row's dot product is cut into 2^kshift segments of whole wave strides so
            // that a small block still occupies every wave
            const int vec = vec4 ? 4 : 1;
            int kf = 1;
            while (kf * 2 * per <= kWaves) kf *= 2;
            auto seg_of = [&](int f) { return cdiv(cdiv(n[l - 1], f), 64 * vec) * 64 * vec; };
            while (kf > 1 && (int64_t)seg_of(kf) * (kf - 1) >= n[l - 1]) kf /= 2;   // no empty segments
            g.seg[l] = seg_of(kf);
            g.kf[l] = kf;
            int sh = 0;
            while ((1 << sh) < kf) ++sh;
            g.kshift[l] = sh;
        }
    }
    g.grid = grid;
    // exchange buffers (64-bit words, two copies each)
    size_t words = 0;
    for (int l = 1; l <= L - 2; ++l) { g.off_act[l] = words; words += 2 * (size_t)n[l]; }
    for (int l = 2; l <= L - 1; ++l) { g.off_part[l] = words; words += 2 * (size_t)g.P[l] * n[l - 1]; }
    g.off_z = words; words += 2 * (size_t)g.P[L] * n[L];
    g.words = words;
    // LDS (floats; every piece a multiple of 4)
    int64_t f = 0;
    g.lds_x = (int)f; f += 2 * pad4(n[0]);
    for (int l = 1; l <= L - 2; ++l) { g.lds_a[l] = (int)f; f += pad4(n[l]); }
    int kp = 16;
    for (int l = 1; l <= L - 1; ++l) {
        g.lds_own_a[l] = (int)f; f += pad4(g.per[l]);
        g.lds_own_d[l] = (int)f; f += pad4(g.per[l]);
        g.lds_b[l] = (int)f; f += 2 * pad4(g.per[l]);
        kp = std::max(kp, g.per[l] * g.kf[l]);
    }
    g.lds_out = (int)f; f += 4 * ON_MAX_NL;
    g.lds_kpart = (int)f; f += pad4(kp);
    g.lds_tmp = (int)f; f += ON_TMP_FLOATS;
    if (f * (int64_t)sizeof(float) > (int64_t)ON_MAX_LDS_BYTES) return false;
    g.lds_work_floats = (int)f;
    // The workgroup's weight slices (with their velocity slices when those are read every step)
    // go to LDS layer by layer, smallest first, while they fit.
    const int64_t copies = want_v ? 2 : 1;
    const int64_t budget = (int64_t)ON_MAX_LDS_BYTES / (int64_t)sizeof(float);
    bool taken[ON_MAX_L + 1] = {false};
    for (;;) {
        int best = 0;
        int64_t best_t = 0;
        for (int l = 1; l <= L; ++l) {
            if (taken[l]) continue;
            const int64_t t = (l < L) ? (int64_t)g.per[l] * pad4(n[l - 1]) : (int64_t)n[L] * pad4(g.per[L]);
            if (best == 0 || t < best_t) { best = l; best_t = t; }
        }
        if (best == 0 || f + copies * best_t > budget) break;
        taken[best] = true;
        g.resident |= 1 << best;
        g.lds_w[best] = (int)f; f += best_t;
        if (want_v) { g.lds_v[best] = (int)f; f += best_t; }
    }
    // What is left takes the first rows of layer 1's block when the whole block does not fit (a
    // multiple of four rows, so that every piece stays 16-byte aligned).
    if (L >= 2 && !taken[1]) {
        const int64_t rows = ((budget - f) / (copies * (int64_t)n[0])) & ~(int64_t)3;
        if (rows >= 4 && rows < g.per[1]) {
            g.part_rows = (int)rows;
            g.lds_w[1] = (int)f; f += rows * n[0];
            if (want_v) { g.lds_v[1] = (int)f; f += rows * n[0]; }
        }
    }
    g.lds_floats = (int)f;
    g.ok = true;
    return true;
}

size_t online_exchange_bytes_bound(const int32_t *n, int L)
{
    if (L < 1 || L > ON_MAX_L || n[L] > ON_MAX_NL) return 0;
    size_t words = 0;
    for (int l = 1; l <= L - 2; ++l) words += 2 * (size_t)n[l];
    for (int l = 2; l <= L - 1; ++l) words += 2 * (size_t)ON_MAX_WG * n[l - 1];
    words += 2 * (size_t)ON_MAX_WG * n[L];
    const size_t bytes = words * sizeof(u64);
    return bytes > ((size_t)1 << 30) ? 0 : bytes;
}

hipError_t online_prepare()
{
    return hipFuncSetAttribute((const void *)online_epoch_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)ON_MAX_LDS_BYTES);
}

hipError_t launch_online_epoch(const OnlineGeom &g, const OnlinePlan &plan, hipStream_t stream)
{
    return launch_resident(online_epoch_kernel, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
}

bool batch_geometry(const int32_t *n, int L, int max_batch, int min_tile, bool want_v, BatchGeom &g)
{
    g = BatchGeom{};
    if (L < 1 || L > 2) return false;
    const int nL = n[L], n_mid = n[L - 1];
    if (nL > ON_MAX_NL || max_batch < 1 || max_batch > PB_MAX_BATCH) return false;
    if ((int64_t)max_batch * (nL + 1) > PB_MAX_OUT_FLOATS) return false;
    if (L == 2 && (n[0] > PB_MAX_N0 || n[0] % 4 != 0)) return false;
    if (min_tile < 1) min_tile = 1;
    auto cdiv = [](int64_t a, int64_t b) { return (int)((a + b - 1) / b); };
    auto pad4 = [](int v) { return (v + 3) & ~3; };
    const int other = (L == 2) ? n[0] : nL;
    int per = std::max(cdiv(n_mid, ON_MAX_WG), cdiv(min_tile, (int64_t)other * max_batch));
    per = std::min(per, n_mid);
    if (per > PB_MAX_ROWS) per = PB_MAX_ROWS;
    if (cdiv(n_mid, per) > ON_MAX_WG) return false;
    g.L = L;
    g.per = per;
    g.P = cdiv(n_mid, per);
    g.grid = g.P;
    g.spw = cdiv(max_batch, g.P);
    size_t words = 0;
    g.off_z = words; words += 2 * (size_t)g.P * max_batch * nL;
    g.off_d = words; words += 2 * (size_t)max_batch * (nL + 1);
    g.words = words;
    int64_t f = 0;
    const int64_t t1 = (L == 2) ? (int64_t)per * n[0] : 0, t2 = (int64_t)nL * per;
    g.lds_w1 = (int)f; f += pad4((int)t1);
    g.lds_v1 = (int)f; if (want_v) f += pad4((int)t1);
    g.lds_b1 = (int)f; f += 2 * pad4(per);
    g.lds_w2 = (int)f; f += pad4((int)t2);
    g.lds_v2 = (int)f; if (want_v) f += pad4((int)t2);
    g.lds_bL = (int)f; f += 2 * ON_MAX_NL;
    g.lds_a1 = (int)f; f += pad4(max_batch * per);
    g.lds_d1 = (int)f; f += pad4(max_batch * per);
    g.lds_d2 = (int)f; f += pad4(max_batch * (nL + 1));
    g.lds_zs = (int)f; f += pad4(g.spw * nL);
    g.lds_tmp = (int)f; f += ON_TMP_FLOATS;
    if (f * (int64_t)sizeof(float) > (int64_t)ON_MAX_LDS_BYTES) return false;
    g.lds_floats = (int)f;
    g.ok = true;
    return true;
}

size_t batch_exchange_bytes_bound(const int32_t *n, int L, int max_batch)
{
    if (L < 1 || L > 2 || n[L] > ON_MAX_NL || max_batch < 2 || max_batch > PB_MAX_BATCH) return 0;
    if ((int64_t)max_batch * (n[L] + 1) > PB_MAX_OUT_FLOATS) return 0;
    const size_t words = 2 * (size_t)ON_MAX_WG * max_batch * n[L] + 2 * (size_t)max_batch * (n[L] + 1);
    return words * sizeof(u64);
}

hipError_t batch_prepare()
{
    hipError_t e = hipFuncSetAttribute((const void *)batch_epoch_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)ON_MAX_LDS_BYTES);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)batch_epoch_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)ON_MAX_LDS_BYTES);
}

hipError_t launch_batch_epoch(const BatchGeom &g, const BatchPlan &plan, hipStream_t stream)
{
    if (plan.L == 1) return launch_resident(batch_epoch_kernel<1>, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
    if (plan.L == 2) return launch_resident(batch_epoch_kernel<2>, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
    return hipErrorInvalidValue;
}

bool deep_geometry(const int32_t *n, int L, int max_batch, int min_tile, DeepGeom &g)
{
    g = DeepGeom{};
    if (L < 3 || L > ON_MAX_L) return false;
    const int nL = n[L];
    if (nL > ON_MAX_NL || max_batch < 2 || max_batch > PD_MAX_BATCH) return false;
    for (int l = 0; l < L; ++l)
        if (n[l] % 4 != 0) return false;     // tile rows are read as float4
    if (min_tile < 1) min_tile = 1;
    auto cdiv = [](int64_t a, int64_t b) { return (int)((a + b - 1) / b); };
    auto pad4 = [](int v) { return (v + 3) & ~3; };
    g.L = L;
    int grid = 1, nmax = 0;
    for (int l = 1; l < L; ++l) {
        int per = std::max(cdiv(n[l], ON_MAX_WG), cdiv(min_tile, (int64_t)n[l - 1] * max_batch));
        per = std::min(per, n[l]);
        g.per[l] = per;
        g.P[l] = cdiv(n[l], per);
        grid = std::max(grid, g.P[l]);
        nmax = std::max(nmax, std::max(n[l - 1], n[l]));
    }
    g.per[L] = g.per[L - 1];
    g.P[L] = g.P[L - 1];
    g.grid = grid;
    g.spw = cdiv(max_batch, grid);
    // the two halves of a workgroup split the samples of a rank-B update only if every tile allows it
    g.halves = (2 * (nmax / 4) <= kThreads && 4 * nmax <= kTmp) ? 2 : 1;
    size_t bytes = 0;
    auto take = [&](size_t b) { const size_t o = bytes; bytes += (b + 255) / 256 * 256; return o; };
    g.off_z = take(2 * (size_t)grid * max_batch * nL * sizeof(u64));
    g.off_d = take(2 * (size_t)max_batch * (nL + 1) * sizeof(u64));
    for (int l = 1; l <= L - 1; ++l) {
        if (l <= L - 2) { g.off_ea[l] = take(2 * (size_t)max_batch * n[l] * sizeof(float)); g.off_fa[l] = take(2 * (size_t)grid * sizeof(u64)); }
        if (l >= 2) { g.off_ed[l] = take(2 * (size_t)max_batch * n[l] * sizeof(float)); g.off_fd[l] = take(2 * (size_t)grid * sizeof(u64)); }
    }
    g.bytes = bytes;
    int64_t f = 0;
    for (int l = 1; l < L; ++l) {
        g.lds_r[l] = (int)f; f += pad4(g.per[l] * n[l - 1]);
        if (l >= 2) { g.lds_ct[l] = (int)f; f += pad4(g.per[l - 1] * n[l]); }
        g.lds_b[l] = (int)f; f += pad4(g.per[l]);
        g.lds_a[l] = (int)f; f += pad4(max_batch * g.per[l]);
        g.lds_dl[l] = (int)f; f += pad4(max_batch * g.per[l]);
    }
    g.lds_w2 = (int)f; f += pad4(nL * g.per[L - 1]);
    g.lds_bL = (int)f; f += ON_MAX_NL;
    g.lds_d2 = (int)f; f += pad4(max_batch * (nL + 1));
    g.lds_zs = (int)f; f += pad4(g.spw * nL);
    g.lds_tmp = (int)f; f += ON_TMP_FLOATS;
    if (f * (int64_t)sizeof(float) > (int64_t)ON_MAX_LDS_BYTES) return false;
    g.lds_floats = (int)f;
    g.ok = true;
    return true;
}

size_t deep_exchange_bytes_bound(const int32_t *n, int L, int max_batch)
{
    if (L < 3 || L > ON_MAX_L || n[L] > ON_MAX_NL || max_batch < 2 || max_batch > PD_MAX_BATCH) return 0;
    for (int l = 0; l < L; ++l)
        if (n[l] % 4 != 0) return 0;
    size_t bytes = 0;
    auto take = [&](size_t b) { bytes += (b + 255) / 256 * 256; };
    take(2 * (size_t)ON_MAX_WG * max_batch * n[L] * sizeof(u64));
    take(2 * (size_t)max_batch * (n[L] + 1) * sizeof(u64));
    for (int l = 1; l <= L - 1; ++l) {
        take(2 * (size_t)max_batch * n[l] * sizeof(float)); take(2 * (size_t)ON_MAX_WG * sizeof(u64));
        take(2 * (size_t)max_batch * n[l] * sizeof(float)); take(2 * (size_t)ON_MAX_WG * sizeof(u64));
    }
    return bytes > ((size_t)1 << 30) ? 0 : bytes;
}

hipError_t deep_prepare()
{
    return hipFuncSetAttribute((const void *)deep_batch_epoch_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)ON_MAX_LDS_BYTES);
}

hipError_t launch_deep_epoch(const DeepGeom &g, const DeepPlan &plan, hipStream_t stream)
{
    return launch_resident(deep_batch_epoch_kernel, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
}

}  // namespace dn
