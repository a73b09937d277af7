// Per-sample (batch 1) training of nets with two or more layers, plain gradient descent, as ONE
// persistent kernel per epoch with every weight resident in LDS -- the inner ones twice.
//
// The general per-sample kernel (dn_online.hip) keeps one copy of each weight (the rows of W_l
// with the workgroup that owns the layer's units), so propagating a delta through W_l gives every
// workgroup a PARTIAL of W_l^T delta_l, and every other workgroup has to fetch and add up to 256
// of them per unit: an exchange of P x n numbers per layer and step, plus one of P x n_L partial net
// inputs for the output layer.  When LDS has the room, a second copy removes the partial sums:
//
//   layers 1..L-1   a workgroup owns a block of units of each layer.  It keeps their ROWS of W_l
//                   (forward product, weight update) and, for l >= 2, the COLUMNS of W_l that leave
//                   its own units of layer l-1, stored transposed: delta_{l-1} of its own units is
//                   then one local product with the whole vector delta_l.
//   layer L         narrow (a few outputs): every workgroup keeps all of W_L and b_L and repeats
//                   the output stage; no partial net inputs cross workgroups.
//
// Both copies of a weight are updated by the same fused multiply-add from the same three numbers
// (the learning rate times the published delta of the row's unit, the published activation of the
// column's unit, the weight), so they stay equal bit for bit; at the end of the launch the row copies
// and workgroup 0's image of the last layer go back to device memory and the column copies are
// dropped (the next launch rebuilds them).
//
// What crosses workgroups per step is the least a layer-by-layer method allows: the activation
// vectors a_1 .. a_{L-1} and the delta vectors delta_{L-1} .. delta_2, each number once, as 64-bit
// words {value, step number} that consumers poll (see dn_persist.h).  The weight updates of a layer
// are issued after the delta the next layer down is waiting for has been published, so they run
// while that exchange is in flight.  Two copies of every exchange vector serve alternating steps: a
// workgroup that publishes step s+2 has taken in the last hidden layer's activations of step s+1,
// and those exist only after every workgroup finished reading step s.
#include <algorithm>

#include "dn_internal.h"
#include "dn_persist.h"
#include "dn_wave.h"

namespace dn {
namespace {

// Exchange words sit kWordStride 64-bit words apart.  Dense is best: every workgroup reads every
// word, so spreading them over more memory lines only adds lines to fetch (measured on
// 1024-1024-1024-1024-10, us per step: stride 1: 14.0, 2: 13.9, 8: 15.2, 16: 17.5).
constexpr int kWordStride = 1;

// T[r][k] = fma(-(lr * d), a, T[r][k]) over an LDS tile of nr rows of n floats (n a multiple of 4,
// nr * n below 2^24); the delta d belongs to the row (ON_ROWS: d = dv[r], a = av[k]) or to the column
// (d = dv[k], a = av[r]).  vel (optional, device memory, rows `n` apart): receives the applied change.
// A thread walks the tile in steps of kThreads float4s: (row, column) advance by (rs, ks), the
// quotient and remainder of that stride by n, which the host supplies with 1 / n.
template <bool ON_ROWS>
__device__ __forceinline__ void rank1_update(float *T, int n, int nr, const float *dv, const float *av, float lr,
                                             float *vel, float inv_n, int rs, int ks)
{
    const int total = nr * n;
    int i = threadIdx.x * 4;
    int r = (int)((float)i * inv_n);   // off by at most one: corrected exactly
    if (r * n > i) --r;
    else if ((r + 1) * n <= i) ++r;
    int k = i - r * n;
    for (; i < total; i += kThreads * 4) {
        v4f w = *(const v4f *)(T + i);
        v4f nld, a;
        if (ON_ROWS) {
            const float t = -(lr * dv[r]);
            nld = (v4f){t, t, t, t};
            a = *(const v4f *)(av + k);
        } else {
            const v4f d4 = *(const v4f *)(dv + k);
            nld = (v4f){-(lr * d4.x), -(lr * d4.y), -(lr * d4.z), -(lr * d4.w)};
            const float t = av[r];
            a = (v4f){t, t, t, t};
        }
        w.x = __builtin_fmaf(nld.x, a.x, w.x);
        w.y = __builtin_fmaf(nld.y, a.y, w.y);
        w.z = __builtin_fmaf(nld.z, a.z, w.z);
        w.w = __builtin_fmaf(nld.w, a.w, w.w);
        *(v4f *)(T + i) = w;
        if (vel) *(v4f *)(vel + (size_t)r * n + k) = (v4f){nld.x * a.x, nld.y * a.y, nld.z * a.z, nld.w * a.w};
        r += rs;
        k += ks;
        if (k >= n) { k -= n; ++r; }
    }
}

// (The depth is a template parameter: with the layer loops of a step unrolled, a layer's shape, pointers
// and LDS offsets are fixed places in the argument block, which the compiler reads once and keeps in
// scalar registers -- or in the lanes of a vector register when those run out -- for the whole
// epoch.  With a run-time depth every use was a scalar load from the argument block, several dozen
// a step, each a round trip a lone wave waits out.)
template <int LT>
__global__ __launch_bounds__(ON_THREADS) void twin_epoch_kernel(TwinPlan p)
{
    extern __shared__ __align__(16) float lds[];
    __shared__ int s_abort;
    const int w = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    constexpr int L = LT;
    const int n0 = p.layer[1].n_in;
    const TwinLayer &last = p.layer[L];
    const int nL = last.n_out, nLin = last.n_in;
    auto r0_of = [&](int l) { return w * p.layer[l].per; };
    auto nr_of = [&](int l) { return max(0, min(p.layer[l].per, p.layer[l].n_out - w * p.layer[l].per)); };

    float *xa0 = lds + p.lds_x;
    float *zL = lds + p.lds_out, *dL = zL + ON_MAX_NL, *bL = dL + ON_MAX_NL;
    float *kpart = lds + p.lds_kpart;
    float *d_full = lds + p.lds_d;
    float *WL = lds + p.lds_wL;
    const int n0p = (n0 + 3) & ~3;
    const bool need_x = nr_of(1) > 0;

    // ---- prologue: own slices, both copies, and the whole last layer into LDS ----
    if (tid == 0) s_abort = 0;
    for (int k = tid; k < nL; k += kThreads) bL[k] = last.b[k];
    copy_floats(WL, last.W, nL * nLin);
    for (int l = 1; l < L; ++l) {
        const TwinLayer &ly = p.layer[l];
        const int r0 = r0_of(l), nr = nr_of(l);
        float *bl = lds + p.lds_b[l];
        for (int r = tid; r < nr; r += kThreads) bl[r] = ly.b[r0 + r];
        if (nr > 0) copy_floats(lds + p.lds_r[l], ly.W + (size_t)r0 * ly.n_in, nr * ly.n_in);
        if (l >= 2) {   // columns of W_l that leave the own units of layer l-1, one LDS row per unit
            const int cp = r0_of(l - 1), np = nr_of(l - 1);
            float *ct = lds + p.lds_c[l];
            for (int i = tid; i < np * ly.n_out; i += kThreads) {
                const int j = i / ly.n_out, o = i - j * ly.n_out;
                ct[i] = ly.W[(size_t)o * ly.n_in + cp + j];
            }
        }
    }
    if (need_x)
        for (int k = tid; k < n0; k += kThreads) xa0[k] = p.X[k];
    int y_cur = p.labels[0];
    double loss_acc = 0.0;
    __syncthreads();

    // rows of an LDS tile T (nr of them, n long) times the vector v; fin(r, sum) finishes a row.  A
    // row is cut into 2^kshift segments so that a few rows still occupy every wave; the segment sums
    // meet in kpart (one barrier), and a second barrier holds the other waves back while a few threads
    // finish the rows: waves that run ahead into the next poll spin on loads and take issue slots from
    // the waves that still compute (measured: 14.8 -> 14.0 us per step on 1024-1024-1024-1024-10; one
    // wave per row without any barrier: 17.2 us).
    auto product = [&](const float *T, int n, int nr, int kshift, int seg, const float *v, auto fin) {
        if ((nr << kshift) <= kWaves) fwd_rows<4, 1>(T, n, nr, kshift, seg, v, kpart);
        else fwd_rows<4, 4>(T, n, nr, kshift, seg, v, kpart);
        __syncthreads();
        for (int r = tid; r < nr; r += kThreads) {
            float sum = 0.f;
            for (int ks = 0; ks < (1 << kshift); ++ks) sum += kpart[(r << kshift) + ks];
            fin(r, sum);
        }
        __syncthreads();
    };

    // Takes in a whole exchange vector (n words at src) into dst.  A net that one workgroup owns
    // alone has nobody to wait for: its own values (own[0..n)) are copied instead.
    const bool single = gridDim.x == 1;
    auto take_in = [&](const u64 *src, int n, float *dst, const float *own, uint32_t seq) {
        if (single) {
            for (int q = tid; q < n; q += kThreads) dst[q] = own[q];
        } else {
            poll_words(n, seq, [&](int q) { return src + (size_t)q * kWordStride; }, [&](int q, float v) { dst[q] = v; },
                       p.abort_flag, &s_abort);
        }
        __syncthreads();
    };

    const int per1p = (p.layer[1].per + 3) & ~3;
    bool pending_c2 = false;   // the column copy of W_2 still lacks the previous step's update
    constexpr int XR = 4;
    for (int64_t s = 0; s < p.n_samples; ++s) {
        const uint32_t seq = p.seq0 + 1u + (uint32_t)s;
        const int par = (int)(seq & 1u);
        const bool keepv = p.keep_v && s == p.n_samples - 1;   // the epoch's last step also leaves the applied change as velocity
        const float *x = xa0 + (size_t)(s & 1) * n0p;
        const bool more = s + 1 < p.n_samples;
        // layer 1's own activations alternate between two buffers: the deferred update of the
        // column copy of W_2 (below) still needs the previous step's
        float *a1_cur = lds + p.lds_own_a[1] + (int)(s & 1) * per1p;
        const float *a1_prev = lds + p.lds_own_a[1] + (int)((s + 1) & 1) * per1p;
        auto own_a = [&](int l) { return l == 1 ? a1_cur : lds + p.lds_own_a[l]; };
        float xr[XR];
        int y_next = 0;
        bool aborted = false;

        // ---- forward through the hidden layers ----
#pragma unroll
        for (int l = 1; l < L; ++l) {
            const TwinLayer &ly = p.layer[l];
            const int r0 = r0_of(l), nr = nr_of(l);
            if (nr > 0) {
                const float *xin = x;
                if (l > 1) {
                    float *dst = lds + p.lds_a[l - 1];
                    const u64 *src = p.act_x[l - 1] + (size_t)par * ly.n_in * kWordStride;
                    take_in(src, ly.n_in, dst, own_a(l - 1), seq);
                    if (s_abort) { aborted = true; break; }
                    xin = dst;
                }
                float *a_own = own_a(l);
                const float *bl = lds + p.lds_b[l];
                u64 *pub = p.act_x[l] + ((size_t)par * ly.n_out + r0) * kWordStride;
                const int act = ly.act;
                product(lds + p.lds_r[l], ly.n_in, nr, ly.r_kshift, ly.r_seg, xin, [&](int r, float sum) {
                    const float a = act_fn(act, sum + bl[r]);
                    a_own[r] = a;
                    if (!single) ll_store(pub + (size_t)r * kWordStride, a, seq);
                });
            }
            if (l == 1) {
                // work that fits the wait for the other workgroups' activations: the next sample's
                // features are requested, and the column copy of W_2 takes the previous step's update
                if (more) {
                    const float *xn = p.X + (size_t)(s + 1) * n0;
#pragma unroll
                    for (int u = 0; u < XR; ++u) {
                        const int k = tid + u * kThreads;
                        xr[u] = (need_x && k < n0) ? xn[k] : 0.f;
                    }
                    y_next = p.labels[s + 1];
                }
                if (pending_c2) {
                    const TwinLayer &l2 = p.layer[2];
                    rank1_update<false>(lds + p.lds_c[2], l2.n_out, nr_of(1), d_full, a1_prev, p.lr, nullptr, l2.inv_out,
                                        l2.c_rs, l2.c_ks);
                    pending_c2 = false;
                }
            }
            if (l == L - 1 && more && need_x) {   // the features requested above go to the other input buffer
                float *xn = xa0 + (size_t)((s + 1) & 1) * n0p;
#pragma unroll
                for (int u = 0; u < XR; ++u) {
                    const int k = tid + u * kThreads;
                    if (k < n0) xn[k] = xr[u];
                }
                for (int k = tid + XR * kThreads; k < n0; k += kThreads) xn[k] = p.X[(size_t)(s + 1) * n0 + k];
            }
        }
        if (aborted) break;

        // ---- output layer, repeated by every workgroup: z_L, loss, delta_L ----
        {
            float *aLm1 = lds + p.lds_a[L - 1];
            const u64 *src = p.act_x[L - 1] + (size_t)par * nLin * kWordStride;
            take_in(src, nLin, aLm1, own_a(L - 1), seq);
            if (s_abort) break;
            for (int k = wave; k < nL; k += 2 * kWaves) {   // two rows of W_L per wave at a time
                const int k2 = k + kWaves;
                const float *wr = WL + k * nLin, *wr2 = WL + (k2 < nL ? k2 : k) * nLin;
                float acc = 0.f, acc2 = 0.f;
                for (int j = lane * 4; j < nLin; j += 256) {
                    const v4f av = *(const v4f *)(aLm1 + j);
                    const v4f wv = *(const v4f *)(wr + j), wv2 = *(const v4f *)(wr2 + j);
                    acc += wv.x * av.x + wv.y * av.y + wv.z * av.z + wv.w * av.w;
                    acc2 += wv2.x * av.x + wv2.y * av.y + wv2.z * av.z + wv2.w * av.w;
                }
                acc = wave_sum(acc);
                acc2 = wave_sum(acc2);
                if (lane == 0) {
                    zL[k] = acc + bL[k];
                    if (k2 < nL) zL[k2] = acc2 + bL[k2];
                }
            }
            __syncthreads();
            // wave 0: delta_L first (everyone waits for it); the loss and the bias update follow
            // after the barrier, beside the other waves' work
            int y = y_cur;
            y = y < 0 ? 0 : (y >= nL ? nL - 1 : y);
            const int k0 = lane, k1 = lane + 64;
            float d0 = 0.f, d1 = 0.f, e_m = 0.f, e_sum = 1.f, f0 = 0.f, f1 = 0.f;
            if (wave == 0) {
                const float z0 = k0 < nL ? zL[k0] : -INFINITY, z1 = k1 < nL ? zL[k1] : -INFINITY;
                if (p.loss == DN_LOSS_CROSS_ENTROPY) {
                    e_m = wave_max(fmaxf(z0, z1));
                    const float e0 = k0 < nL ? expf(z0 - e_m) : 0.f, e1 = k1 < nL ? expf(z1 - e_m) : 0.f;
                    e_sum = wave_sum(e0 + e1);
                    const float inv = 1.0f / e_sum;
                    d0 = e0 * inv - (k0 == y ? 1.0f : 0.0f);
                    d1 = e1 * inv - (k1 == y ? 1.0f : 0.0f);
                } else {
                    const float a0 = act_fn(last.act, z0), a1 = act_fn(last.act, z1);
                    f0 = a0 - (k0 == y ? 1.0f : 0.0f);
                    f1 = a1 - (k1 == y ? 1.0f : 0.0f);
                    d0 = f0 * act_deriv(last.act, a0);
                    d1 = f1 * act_deriv(last.act, a1);
                }
                if (k0 < nL) dL[k0] = d0;
                if (k1 < nL) dL[k1] = d1;
            }
            __syncthreads();
            if (wave == 0) {
                if (w == 0) {
                    float e;
                    if (p.loss == DN_LOSS_CROSS_ENTROPY) e = logf(e_sum) - (zL[y] - e_m);
                    else e = wave_sum((k0 < nL ? 0.5f * f0 * f0 : 0.f) + (k1 < nL ? 0.5f * f1 * f1 : 0.f));
                    if (lane == 0) loss_acc += (double)e;
                }
                if (k0 < nL) {
                    bL[k0] = bL[k0] - p.lr * d0;
                    if (keepv && w == 0) last.Vb[k0] = -(p.lr * d0);
                }
                if (k1 < nL) {
                    bL[k1] = bL[k1] - p.lr * d1;
                    if (keepv && w == 0) last.Vb[k1] = -(p.lr * d1);
                }
            } else {
                // deltas of the own units of layer L-1 through the last layer's weights before their
                // update: sixteen lanes per unit, on the waves beside wave 0
                const int c0 = r0_of(L - 1), nc = nr_of(L - 1);
                const float *a_own = own_a(L - 1);
                float *d_own = lds + p.lds_own_d[L - 1];
                const int actp = p.layer[L - 1].act;
                for (int t = tid - 64; t < nc * 16; t += kThreads - 64) {
                    const int j = t >> 4, g = t & 15;
                    float sacc = 0.f;
                    for (int k = g; k < nL; k += 16) sacc += WL[k * nLin + c0 + j] * dL[k];
                    sacc = row16_sum(sacc);
                    if (g == 0) {
                        const float d = sacc * act_deriv(actp, a_own[j]);
                        d_own[j] = d;
                        if (L >= 3 && !single) ll_store(p.dl_x[L - 1] + ((size_t)par * nLin + c0 + j) * kWordStride, d, seq);
                    }
                }
            }
            __syncthreads();
            rank1_update<true>(WL, nLin, nL, dL, aLm1, p.lr, (keepv && w == 0) ? last.VW : nullptr, last.inv_in, last.r_rs,
                               last.r_ks);
        }

        // ---- backward through the hidden layers ----
#pragma unroll
        for (int l = L - 1; l >= 1; --l) {
            const TwinLayer &ly = p.layer[l];
            const int r0 = r0_of(l), nr = nr_of(l);
            if (nr > 0) {   // own rows of W_l and their biases
                const float *d_own = lds + p.lds_own_d[l];
                const float *ain = (l == 1) ? x : (lds + p.lds_a[l - 1]);
                rank1_update<true>(lds + p.lds_r[l], ly.n_in, nr, d_own, ain, p.lr,
                                   keepv ? ly.VW + (size_t)r0 * ly.n_in : nullptr, ly.inv_in, ly.r_rs, ly.r_ks);
                float *bl = lds + p.lds_b[l];
                for (int r = tid; r < nr; r += kThreads) {
                    bl[r] = bl[r] - p.lr * d_own[r];
                    if (keepv) ly.Vb[r0 + r] = -(p.lr * d_own[r]);
                }
            }
            if (l >= 2) {
                const TwinLayer &lp = p.layer[l - 1];
                const int c0 = r0_of(l - 1), np = nr_of(l - 1);
                if (np > 0) {   // deltas of the own units of layer l-1, then the column copy's update
                    const u64 *src = p.dl_x[l] + (size_t)par * ly.n_out * kWordStride;
                    take_in(src, ly.n_out, d_full, lds + p.lds_own_d[l], seq);
                    if (s_abort) { aborted = true; break; }
                    const float *a_own = own_a(l - 1);
                    float *d_prev = lds + p.lds_own_d[l - 1];
                    u64 *pub = p.dl_x[l - 1] + ((size_t)par * lp.n_out + c0) * kWordStride;
                    const int actp = lp.act;
                    const bool publish = l - 1 >= 2 && !single;
                    product(lds + p.lds_c[l], ly.n_out, np, ly.c_kshift, ly.c_seg, d_full, [&](int j, float sum) {
                        const float d = sum * act_deriv(actp, a_own[j]);
                        d_prev[j] = d;
                        if (publish) ll_store(pub + (size_t)j * kWordStride, d, seq);
                    });
                    if (l == 2 && more) {
                        // nothing waits for this update before the next step's backward pass: it runs
                        // in the next step, while layer 1's activations travel
                        pending_c2 = true;
                    } else {
                        __syncthreads();
                        rank1_update<false>(lds + p.lds_c[l], ly.n_out, np, d_full, a_own, p.lr, nullptr, ly.inv_out, ly.c_rs,
                                            ly.c_ks);
                    }
                }
            }
            __syncthreads();
        }
        if (aborted) break;
        y_cur = y_next;
    }

    // ---- epilogue: row copies (and workgroup 0's last layer) back to device memory ----
    __syncthreads();
    for (int l = 1; l < L; ++l) {
        const TwinLayer &ly = p.layer[l];
        const int r0 = r0_of(l), nr = nr_of(l);
        const float *bl = lds + p.lds_b[l];
        for (int r = tid; r < nr; r += kThreads) ly.b[r0 + r] = bl[r];
        if (nr > 0) copy_floats(ly.W + (size_t)r0 * ly.n_in, lds + p.lds_r[l], nr * ly.n_in);
    }
    if (w == 0) {
        copy_floats(last.W, WL, nL * nLin);
        for (int k = tid; k < nL; k += kThreads) last.b[k] = bL[k];
        if (tid == 0) *p.loss_acc += loss_acc;
    }
}

}  // namespace

// ---- host side -------------------------------------------------------------------

bool twin_geometry(const int32_t *n, int L, int min_tile, TwinGeom &g)
{
    g = TwinGeom{};
    if (L < 2 || L > ON_MAX_L) return false;
    if (n[L] > ON_MAX_NL) return false;
    for (int l = 0; l < L; ++l)
        if (n[l] % 4 != 0) return false;     // LDS rows are read and written as float4
    if (min_tile < 1) min_tile = 1;
    auto cdiv = [](int64_t a, int64_t b) { return (int)((a + b - 1) / b); };
    auto pad4 = [](int v) { return (v + 3) & ~3; };
    // segments a row's dot product is cut into so that a small block still occupies every wave
    auto segments = [&](int rows, int len, int &kshift, int &seg) {
        int kf = 1;
        while (kf * 2 * rows <= kWaves) kf *= 2;
        auto seg_of = [&](int f) { return cdiv(cdiv(len, f), 256) * 256; };
        while (kf > 1 && (int64_t)seg_of(kf) * (kf - 1) >= len) kf /= 2;   // no empty segments
        seg = seg_of(kf);
        kshift = 0;
        while ((1 << kshift) < kf) ++kshift;
        return kf;
    };
    g.L = L;
    int grid = 1, kp = 16;
    for (int l = 1; l < L; ++l) {
        int per = std::max(cdiv(n[l], ON_MAX_WG), cdiv(min_tile, n[l - 1]));
        per = std::min(per, n[l]);
        if ((int64_t)per * n[l - 1] > ((int64_t)1 << 24)) return false;
        g.per[l] = per;
        g.P[l] = cdiv(n[l], per);
        grid = std::max(grid, g.P[l]);
        kp = std::max(kp, per * segments(per, n[l - 1], g.r_kshift[l], g.r_seg[l]));
        if (l >= 2) kp = std::max(kp, g.per[l - 1] * segments(g.per[l - 1], n[l], g.c_kshift[l], g.c_seg[l]));
    }
    g.grid = grid;
    size_t words = 0;
    for (int l = 1; l <= L - 1; ++l) { g.off_act[l] = words; words += 2 * (size_t)n[l] * kWordStride; }
    for (int l = 2; l <= L - 1; ++l) { g.off_dl[l] = words; words += 2 * (size_t)n[l] * kWordStride; }
    g.words = words;
    int64_t f = 0;
    int dmax = 4;
    g.lds_x = (int)f; f += 2 * pad4(n[0]);
    for (int l = 1; l <= L - 1; ++l) {
        g.lds_a[l] = (int)f; f += pad4(n[l]);
        g.lds_own_a[l] = (int)f; f += (l == 1 ? 2 : 1) * pad4(g.per[l]);   // layer 1: two buffers, alternating steps
        g.lds_own_d[l] = (int)f; f += pad4(g.per[l]);
        g.lds_b[l] = (int)f; f += pad4(g.per[l]);
        if (l >= 2) dmax = std::max(dmax, pad4(n[l]));
    }
    g.lds_d = (int)f; f += dmax;
    g.lds_out = (int)f; f += 3 * ON_MAX_NL;
    g.lds_kpart = (int)f; f += pad4(kp);
    for (int l = 1; l <= L - 1; ++l) {
        g.lds_r[l] = (int)f; f += (int64_t)g.per[l] * n[l - 1];
        if (l >= 2) { g.lds_c[l] = (int)f; f += (int64_t)g.per[l - 1] * n[l]; }
    }
    g.lds_wL = (int)f; f += (int64_t)pad4(n[L] * n[L - 1]);
    if (f * (int64_t)sizeof(float) > (int64_t)ON_MAX_LDS_BYTES) return false;
    g.lds_floats = (int)f;
    g.ok = true;
    return true;
}

size_t twin_exchange_bytes_bound(const int32_t *n, int L)
{
    if (L < 2 || L > ON_MAX_L || n[L] > ON_MAX_NL) return 0;
    size_t words = 0;
    for (int l = 1; l <= L - 1; ++l) words += 4 * (size_t)n[l] * kWordStride;
    const size_t bytes = words * sizeof(u64);
    return bytes > ((size_t)1 << 30) ? 0 : bytes;
}

namespace {

template <int LT>
hipError_t twin_prepare_one()
{
    return hipFuncSetAttribute((const void *)twin_epoch_kernel<LT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)ON_MAX_LDS_BYTES);
}

template <int LT>
hipError_t twin_launch_one(const TwinGeom &g, const TwinPlan &plan, hipStream_t stream)
{
    return launch_resident(twin_epoch_kernel<LT>, plan, g.grid, (size_t)g.lds_floats * sizeof(float), stream);
}

}  // namespace

hipError_t twin_prepare()
{
    static_assert(ON_MAX_L == 8, "one instantiation per depth from two layers on");
    const hipError_t e[] = {twin_prepare_one<2>(), twin_prepare_one<3>(), twin_prepare_one<4>(), twin_prepare_one<5>(),
                            twin_prepare_one<6>(), twin_prepare_one<7>(), twin_prepare_one<8>()};
    for (hipError_t x : e)
        if (x != hipSuccess) return x;
    return hipSuccess;
}

hipError_t launch_twin_epoch(const TwinGeom &g, const TwinPlan &plan, hipStream_t stream)
{
    switch (plan.L) {
    case 2: return twin_launch_one<2>(g, plan, stream);
    case 3: return twin_launch_one<3>(g, plan, stream);
    case 4: return twin_launch_one<4>(g, plan, stream);
    case 5: return twin_launch_one<5>(g, plan, stream);
    case 6: return twin_launch_one<6>(g, plan, stream);
    case 7: return twin_launch_one<7>(g, plan, stream);
    case 8: return twin_launch_one<8>(g, plan, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace dn
