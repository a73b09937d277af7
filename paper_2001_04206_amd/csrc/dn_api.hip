// Host side of libdn: argument validation, arena layout, the schedule of
// kernel launches for each entry point of include/dn.h, and launch timing.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "dn_internal.h"

using namespace dn;

namespace {

constexpr size_t kAlign = 256;
constexpr int kMaxTimed = 16384;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Offsets (bytes) of everything the arena holds.
struct Layout {
    std::vector<size_t> W, b;   // per layer, relative to the start of a parameter-shaped region
    size_t region = 0;          // bytes of one parameter-shaped region (params / velocity / gradients)
    std::vector<size_t> A, D;   // activations / deltas of layers 1..L, absolute
    size_t off_params = 0, off_vel = 0, off_grads = 0;
    size_t off_loss_rows = 0, off_hit_rows = 0, off_loss_sums = 0, off_scalars = 0;
    size_t off_online = 0, online_bytes = 0;   // exchange buffers of the persistent batch-1 kernel
    size_t off_gemm_ws = 0, off_gemm_counters = 0;   // partial tiles / arrival counters of k-split contractions
    size_t off_batch = 0, batch_bytes = 0;           // exchange buffers of the persistent minibatch kernel
    size_t off_deep = 0, deep_bytes = 0;             // exchange buffers of the persistent minibatch kernel for deeper nets
    size_t total = 0;
};

bool compute_layout(const int32_t *widths, int32_t n_widths, int32_t max_batch, Layout &lo)
{
    if (!widths || n_widths < 2 || max_batch <= 0) return false;
    const int L = n_widths - 1;
    for (int i = 0; i < n_widths; ++i)
        if (widths[i] <= 0) return false;
    lo.W.assign(L + 1, 0);
    lo.b.assign(L + 1, 0);
    lo.A.assign(L + 1, 0);
    lo.D.assign(L + 1, 0);
    const size_t lim = (size_t)1 << 46;  // refuse absurd sizes before they overflow
    size_t p = 0;
    for (int l = 1; l <= L; ++l) {
        const size_t nw = (size_t)widths[l] * (size_t)widths[l - 1];
        if (nw > lim / 4) return false;
        lo.W[l] = p;
        p += align_up(nw * sizeof(float));
        lo.b[l] = p;
        p += align_up((size_t)widths[l] * sizeof(float));
        if (p > lim) return false;
    }
    lo.region = p;
    size_t o = 0;
    lo.off_params = o; o += lo.region;
    lo.off_vel = o; o += lo.region;
    lo.off_grads = o; o += lo.region;
    for (int l = 1; l <= L; ++l) {
        const size_t na = align_up((size_t)max_batch * (size_t)widths[l] * sizeof(float));
        if (na > lim) return false;
        lo.A[l] = o; o += na;
        lo.D[l] = o; o += na;
        if (o > lim) return false;
    }
    lo.off_loss_rows = o; o += align_up((size_t)max_batch * sizeof(float));
    lo.off_hit_rows = o; o += align_up((size_t)max_batch * sizeof(float));
    lo.off_loss_sums = o; o += align_up((size_t)max_batch * sizeof(double));
    lo.off_scalars = o; o += kAlign;
    lo.online_bytes = std::max({online_exchange_bytes_bound(widths, L), twin_exchange_bytes_bound(widths, L),
                                wide_exchange_bytes_bound(widths, L)});
    lo.off_online = o; o += align_up(lo.online_bytes);
    lo.off_gemm_ws = o; o += align_up(GEMM_WS_FLOATS * sizeof(float));
    lo.off_gemm_counters = o; o += align_up(GEMM_COUNTERS * sizeof(unsigned));
    lo.batch_bytes = batch_exchange_bytes_bound(widths, L, max_batch);
    lo.off_batch = o; o += align_up(lo.batch_bytes);
    lo.deep_bytes = deep_exchange_bytes_bound(widths, L, max_batch);
    lo.off_deep = o; o += align_up(lo.deep_bytes);
    lo.total = o;
    return true;
}

struct TimedLaunch {
    hipEvent_t start, stop;
    int cls;
    double flop;   // algorithmic flops of the launch (2 M N K per product)
};

}  // namespace

struct dn_net {
    int L = 0;
    std::vector<int32_t> n;     // widths n_0..n_L
    std::vector<int32_t> act;   // act[l], l = 1..L (index 0 unused)
    int loss = 0;
    int max_batch = 0;
    char *arena = nullptr;
    Layout lo;
    hipStream_t stream = nullptr;
    // state of the split API
    const float *X = nullptr;
    int fwd_batch = 0;
    bool have_fwd = false, have_bwd = false;
    bool w1_as_in_bwd = false;   // W_1 is still the matrix the last dn_backward propagated through
    // options
    int time_kernels = 0, gemm_variant = -1, online_mode = 0, online_min_tile = ON_DEFAULT_MIN_TILE,
        online_resident = 1, online_twin = 1, online_tiny = 1, online_solo = 1, online_wide = 1, split_k_on = 1, merge_launches = 1;
    // persistent batch-1 kernel
    OnlineGeom geom{};
    bool online_ok = false;
    bool online_prepared = false, batch_prepared = false, deep_prepared = false;   // LDS limits raised at creation
    bool twin_ready = false;   // the two-copy batch-1 kernel's LDS limit is raised
    bool tiny_ready = false;   // the one-wave batch-1 kernel's LDS limit is raised
    bool wide_ready = false;   // the wide-hidden-layer batch-1 kernel's LDS limit is raised
    bool wide_ok = false;      // ... and the net suits it
    int last_schedule = DN_SCHED_NONE;   // how the last dn_train_epoch ran
    uint32_t online_seq = 0;   // last step number stamped into the exchange buffers
    // persistent minibatch kernel (one- and two-layer nets)
    bool batch_ok = false, deep_ok = false;
    int batch_mode = 0;
    uint32_t batch_seq = 0, deep_seq = 0;
    int device_cus = 0;
    // timing
    hipEvent_t ev_epoch0 = nullptr, ev_epoch1 = nullptr;
    std::vector<TimedLaunch> pool;
    int timed = 0;
    float epoch_ms = 0.f;
    double cls_ms[DN_K_CLASSES] = {0};
    double cls_flop[DN_K_CLASSES] = {0};
    int64_t cls_launches[DN_K_CLASSES] = {0};

    float *W(int l) const { return (float *)(arena + lo.off_params + lo.W[l]); }
    float *b(int l) const { return (float *)(arena + lo.off_params + lo.b[l]); }
    float *VW(int l) const { return (float *)(arena + lo.off_vel + lo.W[l]); }
    float *Vb(int l) const { return (float *)(arena + lo.off_vel + lo.b[l]); }
    float *GW(int l) const { return (float *)(arena + lo.off_grads + lo.W[l]); }
    float *Gb(int l) const { return (float *)(arena + lo.off_grads + lo.b[l]); }
    float *A(int l) const { return (float *)(arena + lo.A[l]); }
    float *D(int l) const { return (float *)(arena + lo.D[l]); }
    float *loss_rows() const { return (float *)(arena + lo.off_loss_rows); }
    float *hit_rows() const { return (float *)(arena + lo.off_hit_rows); }
    double *loss_sums() const { return (double *)(arena + lo.off_loss_sums); }
    double *hit_acc() const { return (double *)(arena + lo.off_scalars + 16); }   // after epoch_acc and the abort flag
    double *epoch_acc() const { return (double *)(arena + lo.off_scalars); }
    int *abort_flag() const { return (int *)(arena + lo.off_scalars + sizeof(double)); }
    unsigned long long *exchange() const { return (unsigned long long *)(arena + lo.off_online); }
    unsigned long long *batch_exchange() const { return (unsigned long long *)(arena + lo.off_batch); }
    char *deep_exchange() const { return arena + lo.off_deep; }
    void split_k(GemmArgs &g) const
    {
        g.ws = split_k_on ? (float *)(arena + lo.off_gemm_ws) : nullptr;
        g.counters = (unsigned *)(arena + lo.off_gemm_counters);
        g.ws_floats = GEMM_WS_FLOATS;
        g.n_counters = GEMM_COUNTERS;
    }
};

LaunchEvents &dn::launch_events()
{
    static thread_local LaunchEvents ev;
    return ev;
}

namespace {

#define DN_HIP(expr)                                   \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return DN_ERR_DEVICE;    \
    } while (0)

// Which persistent kernels this net fits with the current tile option ("online_min_tile").
void refresh_persistent(dn_net *net)
{
    const int L = net->L;
    net->online_ok = net->batch_ok = net->deep_ok = net->wide_ok = false;
    if (net->device_cus <= 0) return;
    if (net->wide_ready) {
        WideGeom wg;
        net->wide_ok = wide_geometry(net->n.data(), L, net->device_cus, false, wg) &&
                       wg.words * sizeof(unsigned long long) <= net->lo.online_bytes;
    }
    if (net->online_prepared && online_geometry(net->n.data(), L, net->online_min_tile, false, net->geom))
        net->online_ok = net->geom.grid <= net->device_cus;
    if (net->batch_prepared) {
        BatchGeom bg;   // with velocities: the larger of the two LDS layouts
        net->batch_ok = batch_geometry(net->n.data(), L, net->max_batch, net->online_min_tile, true, bg) &&
                        bg.grid <= net->device_cus;
    }
    if (net->deep_prepared) {
        DeepGeom dg;
        net->deep_ok = deep_geometry(net->n.data(), L, net->max_batch, net->online_min_tile, dg) &&
                       dg.grid <= net->device_cus;
    }
}

double product_flop(const GemmArgs &g) { return 2.0 * (double)g.M * (double)g.N * (double)g.K; }

bool rate_ok(float lr, float mu)
{
    return std::isfinite(lr) && std::isfinite(mu) && lr >= 0.f && mu >= 0.f && mu < 1.f;
}

// Times one launch when per-launch timing is on.  bind: the scope holds exactly one kernel launch
// made through launch_kernel, which takes the event pair along (the kernel's own start and end);
// otherwise the events are recorded around whatever the scope enqueues.
struct ScopedTimer {
    dn_net *net;
    TimedLaunch *t = nullptr;
    bool bind;
    ScopedTimer(dn_net *n, int cls, bool enabled, double flop = 0.0, bool bind_to_launch = false) : net(n), bind(bind_to_launch)
    {
        if (!enabled || net->timed >= kMaxTimed) return;
        if ((int)net->pool.size() <= net->timed) {
            TimedLaunch tl{};
            if (hipEventCreate(&tl.start) != hipSuccess) return;
            if (hipEventCreate(&tl.stop) != hipSuccess) {
                (void)hipEventDestroy(tl.start);
                return;
            }
            net->pool.push_back(tl);
        }
        t = &net->pool[net->timed++];
        t->cls = cls;
        t->flop = flop;
        if (bind) {
            LaunchEvents &ev = launch_events();
            ev.start = t->start;
            ev.stop = t->stop;
            ev.bound = false;
        } else {
            (void)hipEventRecord(t->start, net->stream);
        }
    }
    ~ScopedTimer()
    {
        if (!t) return;
        if (bind) {
            LaunchEvents &ev = launch_events();
            if (!ev.bound) --net->timed;   // nothing was launched (an error on the way): the pair stays unused
            ev = LaunchEvents{};
        } else {
            (void)hipEventRecord(t->stop, net->stream);
        }
    }
};

// Forward pass of one batch; leaves A_1..A_L in the arena.  The softmax layer's
// row normalisation is left to the caller (it is fused with the loss in training).
dn_status run_forward(dn_net *net, const float *X, int B, bool timing, int last_layer = -1)
{
    if (last_layer < 0) last_layer = net->L;
    for (int l = 1; l <= last_layer; ++l) {
        GemmArgs g{};
        g.A = (l == 1) ? X : net->A(l - 1);
        g.lda = net->n[l - 1];
        g.B = net->W(l);
        g.ldb = net->n[l - 1];
        g.M = B; g.N = net->n[l]; g.K = net->n[l - 1];
        g.C = net->A(l); g.ldc = net->n[l];
        g.bias = net->b(l);
        g.act = net->act[l];
        net->split_k(g);
        ScopedTimer st(net, DN_K_FORWARD, timing, product_flop(g), true);
        DN_HIP(launch_gemm(GEMM_FWD, g, net->gemm_variant, net->stream));
    }
    return DN_OK;
}

// Back propagation of one batch from Delta_L.  mode GRAD_STORE leaves gradients in the gradient
// region; the other modes update parameters in place.  With T_l the delta product through W_l
// (giving Delta_{l-1}) and G_l the gradient / update of layer l, the order is
//     T_L, T_{L-1}, ..., T_2 (each needs the one before), then G_L .. G_1:
// every T_l has read W_l before any G writes it, and once all deltas exist the G_l are independent
// of one another, so those whose shapes allow share ONE launch (launch_gemm_grads).  A narrow last
// layer's G_L rides with T_{L-1} instead (launch_delta_with_narrow_grad): its vector-unit work fits
// beside the few tiles of a delta product.  merge_launches = 0: one launch per product.
// have_top_delta: Delta_{L-1} came with the output error already (narrow last layer).
dn_status run_backward(dn_net *net, const float *X, int B, int mode, float lr, float mu, bool timing,
                       bool have_top_delta = false)
{
    const float scale = (mode == GRAD_STORE) ? 1.0f / (float)B : lr / (float)B;
    const int L = net->L;
    const bool merge = net->merge_launches != 0;
    auto delta_args = [&](int l) {   // T_l, l >= 2
        GemmArgs g{};
        g.A = net->D(l); g.lda = net->n[l];
        g.B = net->W(l); g.ldb = net->n[l - 1];
        g.M = B; g.N = net->n[l - 1]; g.K = net->n[l];
        g.C = net->D(l - 1); g.ldc = net->n[l - 1];
        g.aux = net->A(l - 1);
        g.act = net->act[l - 1];
        net->split_k(g);
        return g;
    };
    auto grad_args = [&](int l) {    // G_l
        GemmArgs g{};
        g.A = net->D(l); g.lda = net->n[l];
        g.B = (l == 1) ? X : net->A(l - 1); g.ldb = net->n[l - 1];
        g.M = net->n[l]; g.N = net->n[l - 1]; g.K = B;
        g.C = (mode == GRAD_STORE) ? net->GW(l) : net->W(l);
        g.ldc = net->n[l - 1];
        g.V = net->VW(l);
        g.gb = (mode == GRAD_STORE) ? net->Gb(l) : net->b(l);   // bias gradient / update rides along
        g.vb = net->Vb(l);
        g.scale = scale; g.mu = mu; g.mode = mode;
        return g;
    };
    if (L > ON_MAX_L + 56) return DN_ERR_UNSUPPORTED;
    int top_grad = L;                // gradients L .. 1 are still to do
    for (int l = L; l >= 2; --l) {
        if (l == L && have_top_delta) continue;
        const GemmArgs d = delta_args(l);
        if (merge && l == L - 1 && top_grad == L) {
            const GemmArgs gl = grad_args(L);
            if (delta_narrow_grad_fits(d, gl, net->gemm_variant)) {
                ScopedTimer st(net, DN_K_DELTA, timing, product_flop(d) + product_flop(gl), true);
                DN_HIP(launch_delta_with_narrow_grad(d, gl, net->stream));
                top_grad = L - 1;
                continue;
            }
        }
        ScopedTimer st(net, DN_K_DELTA, timing, product_flop(d), true);
        DN_HIP(launch_gemm(GEMM_DELTA, d, net->gemm_variant, net->stream));
    }
    GemmArgs grads[ON_MAX_L + 56];
    int n = 0;
    for (int l = top_grad; l >= 1; --l) grads[n++] = grad_args(l);
    if (!timing) {
        DN_HIP(launch_gemm_grads(grads, n, net->gemm_variant, merge, net->stream, nullptr));
        return DN_OK;
    }
    // timed: the shared launch (if any) and every single launch get an event pair of their own
    int merged = 0;
    {
        // a dry run tells which products share the launch: they are timed together, the others one by one
        bool in_shared[ON_MAX_L + 56];
        gemm_grads_plan(grads, n, net->gemm_variant, merge, in_shared, &merged);
        if (merged >= 2) {
            GemmArgs shared[ON_MAX_L + 56];
            int ns = 0;
            double fs = 0.0;
            for (int i = 0; i < n; ++i)
                if (in_shared[i]) { shared[ns++] = grads[i]; fs += product_flop(grads[i]); }
            ScopedTimer st(net, DN_K_GRAD_UPDATE, timing, fs, true);
            DN_HIP(launch_gemm_grads(shared, ns, net->gemm_variant, true, net->stream, nullptr));
        }
        for (int i = 0; i < n; ++i) {
            if (merged >= 2 && in_shared[i]) continue;
            ScopedTimer st(net, DN_K_GRAD_UPDATE, timing, product_flop(grads[i]), true);
            DN_HIP(launch_gemm(GEMM_GRAD, grads[i], net->gemm_variant, net->stream));
        }
    }
    return DN_OK;
}

// A whole batch-1 epoch of a very small net on one wavefront.
dn_status run_tiny(dn_net *net, TinyPlan &p, const float *X, const int32_t *labels, int64_t n_samples, float lr, float mu,
                   bool timing)
{
    for (int l = 1; l <= net->L; ++l) {
        TinyLayer &y = p.layer[l];
        y.W = net->W(l); y.b = net->b(l); y.VW = net->VW(l); y.Vb = net->Vb(l);
        y.act = net->act[l];
    }
    p.loss_acc = net->epoch_acc();
    p.X = X; p.labels = labels; p.n_samples = n_samples;
    p.lr = lr; p.mu = mu; p.loss = net->loss; p.keep_v = 1;
    p.in_registers = (net->online_tiny == 1 && net->L == 2 && mu == 0.f) ? 1 : 0;
    net->last_schedule = p.in_registers ? DN_SCHED_ONE_WAVE_REGISTERS : DN_SCHED_ONE_WAVE;
    ScopedTimer st(net, DN_K_ONLINE, timing);
    DN_HIP(launch_tiny_epoch(p, net->stream));
    return DN_OK;
}

// A whole batch-1 epoch of plain gradient descent with the two-copy kernel (same exchange region
// and step numbering as run_online, so either may follow the other).
dn_status run_twin(dn_net *net, const TwinGeom &g, const float *X, const int32_t *labels, int64_t n_samples, float lr,
                   bool timing)
{
    const int L = net->L;
    TwinPlan p{};
    p.L = L;
    for (int l = 1; l <= L; ++l) {
        TwinLayer &y = p.layer[l];
        y.W = net->W(l); y.b = net->b(l); y.VW = net->VW(l); y.Vb = net->Vb(l);
        y.n_in = net->n[l - 1]; y.n_out = net->n[l]; y.act = net->act[l];
        y.per = g.per[l]; y.P = g.P[l];
        y.r_kshift = g.r_kshift[l]; y.r_seg = g.r_seg[l]; y.c_kshift = g.c_kshift[l]; y.c_seg = g.c_seg[l];
        const int stride = ON_THREADS * 4;
        y.inv_in = 1.0f / (float)y.n_in; y.r_rs = stride / y.n_in; y.r_ks = stride % y.n_in;
        y.inv_out = 1.0f / (float)y.n_out; y.c_rs = stride / y.n_out; y.c_ks = stride % y.n_out;
        p.act_x[l] = net->exchange() + g.off_act[l];
        p.dl_x[l] = net->exchange() + g.off_dl[l];
        p.lds_a[l] = g.lds_a[l]; p.lds_own_a[l] = g.lds_own_a[l]; p.lds_own_d[l] = g.lds_own_d[l];
        p.lds_b[l] = g.lds_b[l]; p.lds_r[l] = g.lds_r[l]; p.lds_c[l] = g.lds_c[l];
    }
    p.abort_flag = net->abort_flag();
    p.loss_acc = net->epoch_acc();
    p.lr = lr; p.loss = net->loss;
    p.lds_x = g.lds_x; p.lds_d = g.lds_d; p.lds_wL = g.lds_wL; p.lds_out = g.lds_out; p.lds_kpart = g.lds_kpart;
    const int64_t chunk = (int64_t)1 << 30;
    for (int64_t s0 = 0; s0 < n_samples; s0 += chunk) {
        const int64_t n = (n_samples - s0) < chunk ? (n_samples - s0) : chunk;
        if ((uint64_t)net->online_seq + (uint64_t)n + 2 > 0xffffffffull) {   // step numbers would wrap
            DN_HIP(hipMemsetAsync(net->exchange(), 0, net->lo.online_bytes, net->stream));
            net->online_seq = 0;
        }
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (s0 + n >= n_samples) ? 1 : 0;
        p.seq0 = net->online_seq;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_twin_epoch(g, p, net->stream));
        net->online_seq += (uint32_t)n;
    }
    return DN_OK;
}

// Batch-1 epochs of a two-layer net with a wide hidden layer: most of W_1 stays in LDS and registers.
dn_status run_wide(dn_net *net, const WideGeom &g, const float *X, const int32_t *labels, int64_t n_samples, float lr,
                   float mu, bool timing)
{
    WidePlan p{};
    p.W1 = net->W(1); p.b1 = net->b(1); p.VW1 = net->VW(1); p.Vb1 = net->Vb(1);
    p.W2 = net->W(2); p.b2 = net->b(2); p.VW2 = net->VW(2); p.Vb2 = net->Vb(2);
    p.z_x = net->exchange();
    p.abort_flag = net->abort_flag();
    p.loss_acc = net->epoch_acc();
    p.n0 = net->n[0]; p.n1 = net->n[1]; p.nL = net->n[2];
    p.act1 = net->act[1]; p.actL = net->act[2]; p.loss = net->loss;
    p.per = g.per; p.lds_rows = g.lds_rows;
    p.lr = lr; p.mu = mu;
    p.lds_x = g.lds_x; p.lds_a = g.lds_a; p.lds_d = g.lds_d; p.lds_b = g.lds_b; p.lds_z = g.lds_z; p.lds_w2 = g.lds_w2;
    p.lds_vb = g.lds_vb; p.lds_vw2 = g.lds_vw2;
    p.lds_zall = g.lds_zall; p.lds_out = g.lds_out; p.lds_w1 = g.lds_w1;
    const int64_t chunk = (int64_t)1 << 30;
    for (int64_t s0 = 0; s0 < n_samples; s0 += chunk) {
        const int64_t n = (n_samples - s0) < chunk ? (n_samples - s0) : chunk;
        if ((uint64_t)net->online_seq + (uint64_t)n + 2 > 0xffffffffull) {   // step numbers would wrap
            DN_HIP(hipMemsetAsync(net->exchange(), 0, net->lo.online_bytes, net->stream));
            net->online_seq = 0;
        }
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (s0 + n >= n_samples) ? 1 : 0;
        p.seq0 = net->online_seq;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_wide_epoch(g, p, net->stream));
        net->online_seq += (uint32_t)n;
    }
    return DN_OK;
}

// Batch-1 steps of a two-layer net on one workgroup that keeps W_1 in its registers (plain gradient descent).
dn_status run_solo(dn_net *net, const SoloGeom &g, const float *X, const int32_t *labels, int64_t n_samples, float lr,
                   bool keep_v, bool timing)
{
    SoloPlan p{};
    p.W1 = net->W(1); p.b1 = net->b(1); p.VW1 = net->VW(1); p.Vb1 = net->Vb(1);
    p.W2 = net->W(2); p.b2 = net->b(2); p.VW2 = net->VW(2); p.Vb2 = net->Vb(2);
    p.loss_acc = net->epoch_acc();
    p.n0 = net->n[0]; p.n1 = net->n[1]; p.n2 = net->n[2];
    p.act1 = net->act[1]; p.act2 = net->act[2]; p.loss = net->loss;
    p.lr = lr;
    const int64_t chunk = (int64_t)1 << 30;   // the kernel counts its steps in 32 bits
    for (int64_t s0 = 0; s0 < n_samples; s0 += chunk) {
        const int64_t n = (n_samples - s0) < chunk ? (n_samples - s0) : chunk;
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (keep_v && s0 + n >= n_samples) ? 1 : 0;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_solo_epoch(g, p, net->stream));
    }
    return DN_OK;
}

dn_status run_online_shared(dn_net *net, const float *X, const int32_t *labels, int64_t n_samples, float lr, float mu,
                            bool timing);

// A whole batch-1 epoch on the persistent kernel that suits the net.
dn_status run_online(dn_net *net, const float *X, const int32_t *labels, int64_t n_samples, float lr, float mu,
                     bool timing)
{
    const int L = net->L;
    if (net->online_tiny && net->tiny_ready) {
        TinyPlan tp;   // every layer at most 64 wide: one wavefront runs the epoch
        if (tiny_plan(net->n.data(), L, mu != 0.f, tp)) {
            return run_tiny(net, tp, X, labels, n_samples, lr, mu, timing);
        }
    }
    bool solo_ran = false;
    if (mu == 0.f && net->online_solo) {
        // two layers, W_1 within one compute unit's registers: one workgroup, no exchange through memory.
        // Its scalar reads of a sample may run past the row's end; the last tail_steps samples, where
        // that would leave the array, go to the kernels below (which must then be known to fit).
        SoloGeom sg;
        if (solo_geometry(net->n.data(), L, sg) && n_samples > sg.tail_steps && (sg.tail_steps == 0 || net->online_ok)) {
            const int64_t n_solo = n_samples - sg.tail_steps;
            dn_status st = run_solo(net, sg, X, labels, n_solo, lr, sg.tail_steps == 0, timing);
            if (st != DN_OK) return st;
            net->last_schedule = DN_SCHED_ONE_WORKGROUP;
            if (sg.tail_steps == 0) return DN_OK;
            X += (size_t)n_solo * net->n[0];
            labels += n_solo;
            n_samples = sg.tail_steps;
            solo_ran = true;
        }
    }
    dn_status st = run_online_shared(net, X, labels, n_samples, lr, mu, timing);
    if (solo_ran && st == DN_OK) net->last_schedule = DN_SCHED_ONE_WORKGROUP;
    return st;
}

// ... on the kernels whose workgroups exchange through device memory, in launches of at most 2^30 steps each.
dn_status run_online_shared(dn_net *net, const float *X, const int32_t *labels, int64_t n_samples, float lr, float mu,
                            bool timing)
{
    const int L = net->L;
    if (mu == 0.f && net->online_twin && net->twin_ready) {
        // slices that fit in LDS with a second copy of the inner layers: no partial sums cross workgroups
        TwinGeom tg;
        if (twin_geometry(net->n.data(), L, net->online_min_tile, tg) && tg.grid <= net->device_cus) {
            net->last_schedule = DN_SCHED_TWO_COPY;
            return run_twin(net, tg, X, labels, n_samples, lr, timing);
        }
    }
    if (net->online_wide && net->wide_ok) {
        // two layers, the hidden one too wide for LDS: most of its rows stay in LDS and registers
        WideGeom wg;
        if (wide_geometry(net->n.data(), L, net->device_cus, mu != 0.f, wg)) {
            net->last_schedule = DN_SCHED_WIDE_HIDDEN;
            return run_wide(net, wg, X, labels, n_samples, lr, mu, timing);
        }
    }
    OnlineGeom g;   // same slices as net->geom; LDS residency depends on whether velocities are read
    if (!online_geometry(net->n.data(), L, net->online_min_tile, mu != 0.f, g)) return DN_ERR_UNSUPPORTED;
    OnlinePlan p{};
    p.L = L;
    for (int l = 1; l <= L; ++l) {
        OnlineLayer &y = p.layer[l];
        y.W = net->W(l); y.b = net->b(l); y.VW = net->VW(l); y.Vb = net->Vb(l);
        y.n_in = net->n[l - 1]; y.n_out = net->n[l]; y.act = net->act[l];
        y.per = g.per[l]; y.P = g.P[l]; y.kshift = g.kshift[l]; y.seg = g.seg[l]; y.vec4 = g.vec4[l];
        p.act_x[l] = net->exchange() + g.off_act[l];
        p.part_x[l] = net->exchange() + g.off_part[l];
        p.lds_a[l] = g.lds_a[l]; p.lds_own_a[l] = g.lds_own_a[l]; p.lds_own_d[l] = g.lds_own_d[l];
        p.lds_b[l] = g.lds_b[l]; p.lds_w[l] = g.lds_w[l]; p.lds_v[l] = g.lds_v[l];
    }
    p.z_x = net->exchange() + g.off_z;
    p.abort_flag = net->abort_flag();
    p.loss_acc = net->epoch_acc();
    p.lr = lr; p.mu = mu; p.loss = net->loss;
    p.resident = g.resident;
    p.part_rows = g.part_rows;
    if (net->online_resident == 0) {   // slice images are laid out last: drop them
        p.resident = 0;
        p.part_rows = 0;
        g.lds_floats = g.lds_work_floats;
    }
    p.lds_x = g.lds_x; p.lds_out = g.lds_out; p.lds_kpart = g.lds_kpart; p.lds_tmp = g.lds_tmp;
    const int64_t chunk = (int64_t)1 << 30;
    for (int64_t s0 = 0; s0 < n_samples; s0 += chunk) {
        const int64_t n = (n_samples - s0) < chunk ? (n_samples - s0) : chunk;
        if ((uint64_t)net->online_seq + (uint64_t)n + 2 > 0xffffffffull) {   // step numbers would wrap
            DN_HIP(hipMemsetAsync(net->exchange(), 0, net->lo.online_bytes, net->stream));
            net->online_seq = 0;
        }
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (s0 + n >= n_samples) ? 1 : 0;
        p.seq0 = net->online_seq;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_online_epoch(g, p, net->stream));
        net->online_seq += (uint32_t)n;
    }
    return DN_OK;
}

// Automatic choice between the persistent minibatch kernel and one launch per product: the
// persistent kernel does its products on the vector units, so it only pays while a step is
// launch bound, i.e. while the step's contraction work is small.
bool batch_pays(const dn_net *net, int batch)
{
    double flop = 0.0;
    for (int l = 1; l <= net->L; ++l) flop += 6.0 * batch * (double)net->n[l] * (double)net->n[l - 1];
    return flop <= 4.0e8;
}

// The same question for the deeper-net kernel, which reads whole activation / delta matrices of
// the batch past the L2 in every phase: it pays while those matrices are small.
bool deep_pays(const dn_net *net, int batch)
{
    (void)net;
    // 1024-1024-1024-1024-10, us/step persistent against one launch per product (7 launches): batch 4: 37 / 76,
    // batch 8: 38 / 76, batch 16: 43 / 77, batch 24: 57 / 77, batch 32: 58 / 75, batch 48: 77 / 72, batch 64: 85 / 71
    return batch <= 32;
}

// A whole minibatch epoch of a one- or two-layer net in persistent-kernel launches.
dn_status run_batch_persistent(dn_net *net, const float *X, const int32_t *labels, int64_t n_samples, int batch,
                               float lr, float mu, bool timing)
{
    const int L = net->L;
    BatchGeom g;
    if (!batch_geometry(net->n.data(), L, net->max_batch, net->online_min_tile, mu != 0.f, g)) return DN_ERR_UNSUPPORTED;
    BatchPlan p{};
    p.L = L;
    if (L == 2) { p.W1 = net->W(1); p.b1 = net->b(1); p.VW1 = net->VW(1); p.Vb1 = net->Vb(1); p.act1 = net->act[1]; }
    p.W2 = net->W(L); p.b2 = net->b(L); p.VW2 = net->VW(L); p.Vb2 = net->Vb(L); p.actL = net->act[L];
    p.n0 = net->n[0]; p.n_mid = net->n[L - 1]; p.nL = net->n[L];
    p.per = g.per; p.P = g.P; p.spw = g.spw; p.max_batch = net->max_batch;
    p.z_x = net->batch_exchange() + g.off_z;
    p.d_x = net->batch_exchange() + g.off_d;
    p.abort_flag = net->abort_flag();
    p.loss_acc = net->epoch_acc();
    p.batch = batch;
    p.lr = lr; p.mu = mu; p.loss = net->loss; p.with_v = (mu != 0.f) ? 1 : 0;
    p.lds_w1 = g.lds_w1; p.lds_v1 = g.lds_v1; p.lds_b1 = g.lds_b1; p.lds_w2 = g.lds_w2; p.lds_v2 = g.lds_v2;
    p.lds_bL = g.lds_bL; p.lds_a1 = g.lds_a1; p.lds_d1 = g.lds_d1; p.lds_d2 = g.lds_d2; p.lds_zs = g.lds_zs;
    p.lds_tmp = g.lds_tmp;
    const int64_t chunk_steps = (int64_t)1 << 30;
    const int64_t total_steps = (n_samples + batch - 1) / batch;
    for (int64_t t0 = 0; t0 < total_steps; t0 += chunk_steps) {
        const int64_t nt = (total_steps - t0) < chunk_steps ? (total_steps - t0) : chunk_steps;
        if ((uint64_t)net->batch_seq + (uint64_t)nt + 2 > 0xffffffffull) {   // step numbers would wrap
            DN_HIP(hipMemsetAsync(net->batch_exchange(), 0, net->lo.batch_bytes, net->stream));
            net->batch_seq = 0;
        }
        const int64_t s0 = t0 * batch;
        const int64_t n = ((t0 + nt) * batch < n_samples ? (t0 + nt) * batch : n_samples) - s0;
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (t0 + nt >= total_steps) ? 1 : 0;
        p.seq0 = net->batch_seq;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_batch_epoch(g, p, net->stream));
        net->batch_seq += (uint32_t)nt;
    }
    return DN_OK;
}

// A whole plain-gradient-descent minibatch epoch of a net of three or more layers in
// persistent-kernel launches.
dn_status run_deep_persistent(dn_net *net, const float *X, const int32_t *labels, int64_t n_samples, int batch,
                              float lr, bool timing)
{
    const int L = net->L;
    DeepGeom g;
    if (!deep_geometry(net->n.data(), L, net->max_batch, net->online_min_tile, g)) return DN_ERR_UNSUPPORTED;
    DeepPlan p{};
    p.L = L;
    char *ex = net->deep_exchange();
    for (int l = 1; l <= L; ++l) {
        DeepLayer &y = p.layer[l];
        y.W = net->W(l); y.b = net->b(l); y.VW = net->VW(l); y.Vb = net->Vb(l);
        y.n_in = net->n[l - 1]; y.n_out = net->n[l]; y.act = net->act[l];
        y.per = g.per[l]; y.P = g.P[l];
        p.ea[l] = (float *)(ex + g.off_ea[l]); p.ed[l] = (float *)(ex + g.off_ed[l]);
        p.fa[l] = (unsigned long long *)(ex + g.off_fa[l]); p.fd[l] = (unsigned long long *)(ex + g.off_fd[l]);
        p.lds_r[l] = g.lds_r[l]; p.lds_ct[l] = g.lds_ct[l]; p.lds_b[l] = g.lds_b[l]; p.lds_a[l] = g.lds_a[l];
        p.lds_dl[l] = g.lds_dl[l];
    }
    p.grid = g.grid; p.spw = g.spw; p.max_batch = net->max_batch; p.halves = g.halves;
    p.z_x = (unsigned long long *)(ex + g.off_z);
    p.d_x = (unsigned long long *)(ex + g.off_d);
    p.abort_flag = net->abort_flag();
    p.loss_acc = net->epoch_acc();
    p.batch = batch;
    p.lr = lr; p.loss = net->loss;
    p.lds_w2 = g.lds_w2; p.lds_bL = g.lds_bL; p.lds_d2 = g.lds_d2; p.lds_zs = g.lds_zs; p.lds_tmp = g.lds_tmp;
    const int64_t chunk_steps = (int64_t)1 << 30;
    const int64_t total_steps = (n_samples + batch - 1) / batch;
    for (int64_t t0 = 0; t0 < total_steps; t0 += chunk_steps) {
        const int64_t nt = (total_steps - t0) < chunk_steps ? (total_steps - t0) : chunk_steps;
        if ((uint64_t)net->deep_seq + (uint64_t)nt + 2 > 0xffffffffull) {
            DN_HIP(hipMemsetAsync(net->deep_exchange(), 0, net->lo.deep_bytes, net->stream));
            net->deep_seq = 0;
        }
        const int64_t s0 = t0 * batch;
        const int64_t n = ((t0 + nt) * batch < n_samples ? (t0 + nt) * batch : n_samples) - s0;
        p.X = X + (size_t)s0 * net->n[0];
        p.labels = labels + s0;
        p.n_samples = n;
        p.keep_v = (t0 + nt >= total_steps) ? 1 : 0;
        p.seq0 = net->deep_seq;
        ScopedTimer st(net, DN_K_ONLINE, timing);
        DN_HIP(launch_deep_epoch(g, p, net->stream));
        net->deep_seq += (uint32_t)nt;
    }
    return DN_OK;
}

void collect_times(dn_net *net)
{
    for (int c = 0; c < DN_K_CLASSES; ++c) {
        net->cls_ms[c] = 0.0;
        net->cls_flop[c] = 0.0;
        net->cls_launches[c] = 0;
    }
    for (int i = 0; i < net->timed; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, net->pool[i].start, net->pool[i].stop) == hipSuccess) {
            net->cls_ms[net->pool[i].cls] += ms;
            net->cls_flop[net->pool[i].cls] += net->pool[i].flop;
            net->cls_launches[net->pool[i].cls] += 1;
        }
    }
}

}  // namespace

extern "C" {

const char *dn_status_string(dn_status s)
{
    switch (s) {
    case DN_OK: return "ok";
    case DN_ERR_INVALID_ARG: return "invalid argument";
    case DN_ERR_SHAPE: return "shape mismatch";
    case DN_ERR_UNSUPPORTED: return "unsupported activation/loss combination";
    case DN_ERR_OOM: return "out of host memory";
    case DN_ERR_DEVICE: return "device error";
    default: return "unknown status";
    }
}

size_t dn_net_arena_bytes(const int32_t *widths, int32_t n_widths, int32_t max_batch)
{
    Layout lo;
    return compute_layout(widths, n_widths, max_batch, lo) ? lo.total : 0;
}

dn_status dn_net_create(const int32_t *widths, int32_t n_widths, const dn_act *acts, dn_loss loss,
                        int32_t max_batch, void *arena_dev, size_t arena_bytes, void *hip_stream,
                        dn_net **out)
{
    if (!out) return DN_ERR_INVALID_ARG;
    *out = nullptr;
    if (!widths || !acts || !arena_dev) return DN_ERR_INVALID_ARG;
    if (n_widths < 2 || max_batch <= 0) return DN_ERR_SHAPE;
    for (int i = 0; i < n_widths; ++i)
        if (widths[i] <= 0) return DN_ERR_SHAPE;
    if (loss != DN_LOSS_MSE && loss != DN_LOSS_CROSS_ENTROPY) return DN_ERR_INVALID_ARG;
    const int L = n_widths - 1;
    for (int l = 0; l < L; ++l) {
        if ((int)acts[l] < DN_ACT_LINEAR || (int)acts[l] > DN_ACT_SOFTMAX) return DN_ERR_INVALID_ARG;
        if (acts[l] == DN_ACT_SOFTMAX && l != L - 1) return DN_ERR_UNSUPPORTED;
    }
    const bool softmax_last = acts[L - 1] == DN_ACT_SOFTMAX;
    if (softmax_last != (loss == DN_LOSS_CROSS_ENTROPY)) return DN_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(arena_dev) % kAlign != 0) return DN_ERR_INVALID_ARG;
    Layout lo;
    if (!compute_layout(widths, n_widths, max_batch, lo)) return DN_ERR_SHAPE;
    if (arena_bytes < lo.total) return DN_ERR_SHAPE;

    dn_net *net = new (std::nothrow) dn_net();
    if (!net) return DN_ERR_OOM;
    try {
        net->n.assign(widths, widths + n_widths);
        net->act.assign(L + 1, 0);
        for (int l = 1; l <= L; ++l) net->act[l] = (int)acts[l - 1];
        net->lo = lo;
    } catch (...) {
        delete net;
        return DN_ERR_OOM;
    }
    net->L = L;
    net->loss = (int)loss;
    net->max_batch = max_batch;
    net->arena = (char *)arena_dev;
    net->stream = (hipStream_t)hip_stream;
    // persistent kernels: slices per workgroup, if the net fits them and the device has the units
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&net->device_cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            net->device_cus = 0;
        (void)hipGetLastError();
    }
    if (net->device_cus > 0) {
        // the kernels' LDS limits are raised once; whether a net fits follows the tile option
        net->online_prepared = lo.online_bytes > 0 && online_prepare() == hipSuccess;
        net->twin_ready = lo.online_bytes > 0 && twin_exchange_bytes_bound(net->n.data(), L) > 0 && twin_prepare() == hipSuccess;
        net->tiny_ready = tiny_prepare() == hipSuccess;
        net->wide_ready = lo.online_bytes > 0 && wide_exchange_bytes_bound(net->n.data(), L) > 0 && wide_prepare() == hipSuccess;
        net->batch_prepared = lo.batch_bytes > 0 && batch_prepare() == hipSuccess;
        net->deep_prepared = lo.deep_bytes > 0 && deep_prepare() == hipSuccess;
        (void)hipGetLastError();
    }
    refresh_persistent(net);
    // parameters, velocities and gradients start at zero; exchange words start unstamped
    if (hipMemsetAsync(net->arena, 0, 3 * lo.region, net->stream) != hipSuccess ||
        hipMemsetAsync(net->arena + lo.off_scalars, 0, kAlign, net->stream) != hipSuccess ||
        (lo.online_bytes > 0 &&
         hipMemsetAsync(net->arena + lo.off_online, 0, lo.online_bytes, net->stream) != hipSuccess) ||
        hipMemsetAsync(net->arena + lo.off_gemm_counters, 0, GEMM_COUNTERS * sizeof(unsigned), net->stream) != hipSuccess ||
        (lo.batch_bytes > 0 &&
         hipMemsetAsync(net->arena + lo.off_batch, 0, lo.batch_bytes, net->stream) != hipSuccess) ||
        (lo.deep_bytes > 0 &&
         hipMemsetAsync(net->arena + lo.off_deep, 0, lo.deep_bytes, net->stream) != hipSuccess) ||
        hipEventCreate(&net->ev_epoch0) != hipSuccess || hipEventCreate(&net->ev_epoch1) != hipSuccess ||
        hipStreamSynchronize(net->stream) != hipSuccess) {
        if (net->ev_epoch0) (void)hipEventDestroy(net->ev_epoch0);
        if (net->ev_epoch1) (void)hipEventDestroy(net->ev_epoch1);
        delete net;
        return DN_ERR_DEVICE;
    }
    *out = net;
    return DN_OK;
}

dn_status dn_net_destroy(dn_net *net)
{
    if (!net) return DN_ERR_INVALID_ARG;
    dn_status st = DN_OK;
    if (hipStreamSynchronize(net->stream) != hipSuccess) st = DN_ERR_DEVICE;
    for (auto &t : net->pool) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    (void)hipEventDestroy(net->ev_epoch0);
    (void)hipEventDestroy(net->ev_epoch1);
    delete net;
    return st;
}

dn_status dn_set_params(dn_net *net, int32_t layer, const float *W_host, const float *b_host)
{
    if (!net || layer < 1 || layer > net->L) return DN_ERR_INVALID_ARG;
    if (layer == 1 && W_host) net->w1_as_in_bwd = false;
    const size_t nw = (size_t)net->n[layer] * net->n[layer - 1], nb = (size_t)net->n[layer];
    if (W_host) {
        DN_HIP(hipMemcpyAsync(net->W(layer), W_host, nw * sizeof(float), hipMemcpyHostToDevice, net->stream));
        DN_HIP(hipMemsetAsync(net->VW(layer), 0, nw * sizeof(float), net->stream));
    }
    if (b_host) {
        DN_HIP(hipMemcpyAsync(net->b(layer), b_host, nb * sizeof(float), hipMemcpyHostToDevice, net->stream));
        DN_HIP(hipMemsetAsync(net->Vb(layer), 0, nb * sizeof(float), net->stream));
    }
    DN_HIP(hipStreamSynchronize(net->stream));
    return DN_OK;
}

static dn_status read_pair(dn_net *net, int32_t layer, const float *Wd, const float *bd, float *W_host,
                           float *b_host)
{
    const size_t nw = (size_t)net->n[layer] * net->n[layer - 1], nb = (size_t)net->n[layer];
    if (W_host) DN_HIP(hipMemcpyAsync(W_host, Wd, nw * sizeof(float), hipMemcpyDeviceToHost, net->stream));
    if (b_host) DN_HIP(hipMemcpyAsync(b_host, bd, nb * sizeof(float), hipMemcpyDeviceToHost, net->stream));
    DN_HIP(hipStreamSynchronize(net->stream));
    return DN_OK;
}

dn_status dn_get_params(dn_net *net, int32_t layer, float *W_host, float *b_host)
{
    if (!net || layer < 1 || layer > net->L) return DN_ERR_INVALID_ARG;
    return read_pair(net, layer, net->W(layer), net->b(layer), W_host, b_host);
}

dn_status dn_get_grads(dn_net *net, int32_t layer, float *G_host, float *g_host)
{
    if (!net || layer < 1 || layer > net->L) return DN_ERR_INVALID_ARG;
    if (!net->have_bwd) return DN_ERR_INVALID_ARG;
    return read_pair(net, layer, net->GW(layer), net->Gb(layer), G_host, g_host);
}

dn_status dn_forward(dn_net *net, const float *X_dev, int32_t batch, float *out_dev)
{
    if (!net || !X_dev) return DN_ERR_INVALID_ARG;
    if (batch < 1 || batch > net->max_batch) return DN_ERR_SHAPE;
    net->have_fwd = false;
    net->have_bwd = false;
    net->w1_as_in_bwd = false;
    dn_status st = run_forward(net, X_dev, batch, false);
    if (st != DN_OK) return st;
    const int L = net->L;
    if (net->loss == DN_LOSS_CROSS_ENTROPY)
        DN_HIP(launch_output_delta(net->A(L), net->D(L), nullptr, net->loss_rows(), batch, net->n[L],
                                   net->act[L], net->loss, OUT_SOFTMAX_ONLY, net->stream));
    if (out_dev) DN_HIP(launch_copy(out_dev, net->A(L), (size_t)batch * net->n[L], net->stream));
    net->X = X_dev;
    net->fwd_batch = batch;
    net->have_fwd = true;
    return DN_OK;
}

dn_status dn_backward(dn_net *net, const int32_t *labels_dev, int32_t batch, float *loss_dev)
{
    if (!net || !labels_dev) return DN_ERR_INVALID_ARG;
    if (!net->have_fwd) return DN_ERR_INVALID_ARG;
    if (batch != net->fwd_batch) return DN_ERR_SHAPE;
    const int L = net->L;
    DN_HIP(launch_output_delta(net->A(L), net->D(L), labels_dev, net->loss_rows(), batch, net->n[L],
                               net->act[L], net->loss, OUT_FROM_P, net->stream));
    if (loss_dev) DN_HIP(launch_loss_reduce(net->loss_rows(), batch, loss_dev, nullptr, net->stream));
    dn_status st = run_backward(net, net->X, batch, GRAD_STORE, 0.f, 0.f, false);
    if (st != DN_OK) return st;
    net->have_bwd = true;
    net->w1_as_in_bwd = true;
    return DN_OK;
}

dn_status dn_input_gradient(dn_net *net, int32_t batch, float *dX_dev)
{
    if (!net || !dX_dev) return DN_ERR_INVALID_ARG;
    if (!net->have_bwd || !net->w1_as_in_bwd) return DN_ERR_INVALID_ARG;
    if (batch != net->fwd_batch) return DN_ERR_SHAPE;
    // the delta propagation of the hidden layers, one layer further: the input has no activation,
    // so the derivative factor is that of the identity (the kernel still reads an operand of the
    // output's shape for it, whose values the identity's derivative ignores: the output buffer
    // itself, so that the caller's X need not outlive dn_backward)
    GemmArgs g{};
    g.A = net->D(1); g.lda = net->n[1];
    g.B = net->W(1); g.ldb = net->n[0];
    g.M = batch; g.N = net->n[0]; g.K = net->n[1];
    g.C = dX_dev; g.ldc = net->n[0];
    g.aux = dX_dev;
    g.act = DN_ACT_LINEAR;
    net->split_k(g);
    DN_HIP(launch_gemm(GEMM_DELTA, g, net->gemm_variant, net->stream));
    return DN_OK;
}

dn_status dn_update(dn_net *net, float lr, float momentum)
{
    if (!net || !rate_ok(lr, momentum)) return DN_ERR_INVALID_ARG;
    if (!net->have_bwd) return DN_ERR_INVALID_ARG;
    net->w1_as_in_bwd = false;
    // parameters, velocities and gradients are three regions of one shape (padding holds zeros)
    DN_HIP(launch_update((float *)(net->arena + net->lo.off_params), (float *)(net->arena + net->lo.off_vel),
                         (const float *)(net->arena + net->lo.off_grads), net->lo.region / sizeof(float), lr,
                         momentum, net->stream));
    return DN_OK;
}

dn_status dn_sgd_step(float *param_dev, const float *grad_dev, float *velocity_dev, int64_t count, float lr,
                      float momentum, void *hip_stream)
{
    if (!param_dev || !grad_dev || !rate_ok(lr, momentum)) return DN_ERR_INVALID_ARG;
    if (momentum != 0.f && !velocity_dev) return DN_ERR_INVALID_ARG;
    if (count < 1) return DN_ERR_SHAPE;
    DN_HIP(launch_update(param_dev, velocity_dev, grad_dev, (size_t)count, lr, momentum, (hipStream_t)hip_stream));
    return DN_OK;
}

dn_status dn_train_epoch(dn_net *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples,
                         int32_t batch, float lr, float momentum, float *mean_loss_host)
{
    if (!net || !X_dev || !labels_dev || n_samples <= 0 || !rate_ok(lr, momentum)) return DN_ERR_INVALID_ARG;
    if (batch < 1 || batch > net->max_batch) return DN_ERR_SHAPE;
    net->have_fwd = net->have_bwd = net->w1_as_in_bwd = false;  // activations / gradients of the split API are overwritten
    const bool timing = net->time_kernels != 0;
    net->timed = 0;
    const int L = net->L;
    // (a two-layer net with a very wide hidden layer may suit only the kernel for such nets)
    bool wide_fit = false;
    if (net->online_wide && net->wide_ok) {
        WideGeom wg;
        wide_fit = wide_geometry(net->n.data(), net->L, net->device_cus, momentum != 0.f, wg);
    }
    const bool online_fit = net->online_ok || wide_fit;
    bool persistent = batch == 1 && net->online_mode != 1 && online_fit;
    if (batch == 1 && net->online_mode == 2 && !online_fit) return DN_ERR_UNSUPPORTED;
    const bool pbatch = batch > 1 && net->batch_mode != 1 && net->batch_ok &&
                        (net->batch_mode == 2 || batch_pays(net, batch));
    const bool pdeep = batch > 1 && net->batch_mode != 1 && net->deep_ok && momentum == 0.f &&
                       (net->batch_mode == 2 || deep_pays(net, batch));
    if (batch > 1 && net->batch_mode == 2 && !pbatch && !pdeep) return DN_ERR_UNSUPPORTED;
    DN_HIP(hipMemsetAsync(net->epoch_acc(), 0, sizeof(double) + sizeof(int), net->stream));
    DN_HIP(hipEventRecord(net->ev_epoch0, net->stream));
    // A persistent path that turns out not to fit (its geometry is recomputed for this call's momentum
    // and the current tile option) reports DN_ERR_UNSUPPORTED before it launches anything: in automatic
    // mode the epoch then runs with one launch per product instead.
    net->last_schedule = DN_SCHED_LAUNCHES;
    if (persistent) {
        net->last_schedule = DN_SCHED_PER_SAMPLE;   // run_online changes it if the two-copy kernel takes the pass
        dn_status st = run_online(net, X_dev, labels_dev, n_samples, lr, momentum, timing);
        if (st == DN_ERR_UNSUPPORTED && net->online_mode == 0) persistent = false;
        else if (st != DN_OK) return st;
    } else if (pbatch) {
        net->last_schedule = DN_SCHED_MINIBATCH;
        dn_status st = run_batch_persistent(net, X_dev, labels_dev, n_samples, batch, lr, momentum, timing);
        if (st == DN_OK) persistent = true;
        else if (st != DN_ERR_UNSUPPORTED || net->batch_mode != 0) return st;
    } else if (pdeep) {
        net->last_schedule = DN_SCHED_MINIBATCH_DEEP;
        dn_status st = run_deep_persistent(net, X_dev, labels_dev, n_samples, batch, lr, timing);
        if (st == DN_OK) persistent = true;
        else if (st != DN_ERR_UNSUPPORTED || net->batch_mode != 0) return st;
    }
    if (!persistent) net->last_schedule = DN_SCHED_LAUNCHES;
    // Launch-per-product path.  The epoch's loss is kept as one running sum per batch row, added
    // to by the output kernel of each step, and reduced once after the last step.
    const int rows_used = (int)(n_samples < batch ? n_samples : batch);
    if (!persistent) DN_HIP(hipMemsetAsync(net->loss_sums(), 0, (size_t)rows_used * sizeof(double), net->stream));
    for (int64_t s0 = persistent ? n_samples : 0; s0 < n_samples; s0 += batch) {
        const int B = (int)((n_samples - s0) < batch ? (n_samples - s0) : batch);
        const float *Xb = X_dev + (size_t)s0 * net->n[0];
        const bool last = s0 + batch >= n_samples;
        const int mode = (momentum != 0.f) ? GRAD_MOMENTUM : (last ? GRAD_SGD_KEEPV : GRAD_SGD);
        // a last layer of at most 16 outputs: its forward product and the output error in one launch
        const bool fused_out = net->gemm_variant < 0 && narrow_layer(net->n[L]);
        dn_status st = run_forward(net, Xb, B, timing, fused_out ? L - 1 : L);
        if (st != DN_OK) return st;
        {
            // with a narrow last layer the launch also holds that layer's forward product and its delta product
            const double out_flop = fused_out ? 2.0 * B * (double)net->n[L] * net->n[L - 1] * (L > 1 ? 2.0 : 1.0) : 0.0;
            ScopedTimer t(net, DN_K_OUTPUT, timing, out_flop, true);
            if (fused_out)
                DN_HIP(launch_narrow_output(L == 1 ? Xb : net->A(L - 1), net->W(L), net->b(L), labels_dev + s0, net->A(L),
                                            net->D(L), net->loss_rows(), net->loss_sums(), B, net->n[L], net->n[L - 1],
                                            net->act[L], net->loss, net->stream, L > 1 ? net->D(L - 1) : nullptr,
                                            L > 1 ? net->act[L - 1] : 0));
            else
                DN_HIP(launch_output_delta(net->A(L), net->D(L), labels_dev + s0, net->loss_rows(), B, net->n[L],
                                           net->act[L], net->loss, OUT_FUSED, net->stream, nullptr, net->loss_sums()));
        }
        st = run_backward(net, Xb, B, mode, lr, momentum, timing, fused_out && L > 1);
        if (st != DN_OK) return st;
    }
    if (!persistent) DN_HIP(launch_loss_sums_reduce(net->loss_sums(), rows_used, net->epoch_acc(), net->stream));
    DN_HIP(hipEventRecord(net->ev_epoch1, net->stream));
    struct { double acc; int aborted; int pad; } res = {0.0, 0, 0};
    DN_HIP(hipMemcpyAsync(&res, net->epoch_acc(), sizeof(double) + sizeof(int), hipMemcpyDeviceToHost, net->stream));
    DN_HIP(hipStreamSynchronize(net->stream));
    DN_HIP(hipEventElapsedTime(&net->epoch_ms, net->ev_epoch0, net->ev_epoch1));
    collect_times(net);
    if (res.aborted) return DN_ERR_DEVICE;   // a workgroup of the persistent kernel gave up waiting
    const double acc = res.acc;
    if (mean_loss_host) *mean_loss_host = (float)(acc / (double)n_samples);
    return DN_OK;
}

dn_status dn_train(dn_net *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples, int32_t batch,
                   float lr, float momentum, float max_error, int32_t max_epochs, int32_t *epochs_run_host,
                   float *last_loss_host)
{
    if (!net || max_epochs <= 0 || std::isnan(max_error)) return DN_ERR_INVALID_ARG;
    float loss = 0.f;
    int32_t e = 0;
    while (e < max_epochs) {
        dn_status st = dn_train_epoch(net, X_dev, labels_dev, n_samples, batch, lr, momentum, &loss);
        if (st != DN_OK) return st;
        ++e;
        if (loss <= max_error) break;
    }
    if (epochs_run_host) *epochs_run_host = e;
    if (last_loss_host) *last_loss_host = loss;
    return DN_OK;
}

dn_status dn_evaluate(dn_net *net, const float *X_dev, const int32_t *labels_dev, int64_t n_samples, int32_t batch,
                      float *mean_loss_host, int64_t *correct_host)
{
    if (!net || !X_dev || !labels_dev || n_samples <= 0) return DN_ERR_INVALID_ARG;
    if (batch < 1 || batch > net->max_batch) return DN_ERR_SHAPE;
    net->have_fwd = net->have_bwd = net->w1_as_in_bwd = false;  // the activations of the split API are overwritten
    const int L = net->L;
    DN_HIP(hipMemsetAsync(net->epoch_acc(), 0, 24, net->stream));
    for (int64_t s0 = 0; s0 < n_samples; s0 += batch) {
        const int B = (int)((n_samples - s0) < batch ? (n_samples - s0) : batch);
        dn_status st = run_forward(net, X_dev + (size_t)s0 * net->n[0], B, false);
        if (st != DN_OK) return st;
        DN_HIP(launch_output_delta(net->A(L), net->D(L), labels_dev + s0, net->loss_rows(), B, net->n[L],
                                   net->act[L], net->loss, OUT_EVAL, net->stream, net->hit_rows()));
        DN_HIP(launch_loss_reduce(net->loss_rows(), B, nullptr, net->epoch_acc(), net->stream));
        DN_HIP(launch_loss_reduce(net->hit_rows(), B, nullptr, net->hit_acc(), net->stream));
    }
    struct { double loss; int aborted; int pad; double hits; } res = {0.0, 0, 0, 0.0};
    DN_HIP(hipMemcpyAsync(&res, net->epoch_acc(), 24, hipMemcpyDeviceToHost, net->stream));
    DN_HIP(hipStreamSynchronize(net->stream));
    if (mean_loss_host) *mean_loss_host = (float)(res.loss / (double)n_samples);
    if (correct_host) *correct_host = (int64_t)(res.hits + 0.5);
    return DN_OK;
}

size_t dn_layer_backward_workspace_bytes(int32_t cols_out, int32_t cols_input)
{
    if (cols_out <= 0 || cols_input <= 0) return 0;
    const size_t nw = (size_t)cols_out * (size_t)cols_input;
    if (nw > ((size_t)1 << 31)) return 0;
    return align_up((size_t)cols_out * 4) * 2 + align_up((size_t)cols_input * 4) + 2 * align_up(nw * 4);
}

dn_status dn_layer_backward_host(const float *deltas_host, const float *inputs_host, float learning_rate,
                                 int32_t cols_out, int32_t cols_input, float *gradients_host,
                                 float *delta_weights_host, float *delta_biases_host, void *workspace_dev,
                                 size_t workspace_bytes, void *hip_stream, float *ms_copy_in, float *ms_kernel,
                                 float *ms_copy_out)
{
    if (!deltas_host || !inputs_host || !gradients_host || !delta_weights_host || !delta_biases_host ||
        !workspace_dev || !std::isfinite(learning_rate))
        return DN_ERR_INVALID_ARG;
    const size_t need = dn_layer_backward_workspace_bytes(cols_out, cols_input);
    if (need == 0 || workspace_bytes < need) return DN_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign != 0) return DN_ERR_INVALID_ARG;
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t nw = (size_t)cols_out * (size_t)cols_input;
    char *w = (char *)workspace_dev;
    float *d_dev = (float *)w; w += align_up((size_t)cols_out * 4);
    float *db_dev = (float *)w; w += align_up((size_t)cols_out * 4);
    float *x_dev = (float *)w; w += align_up((size_t)cols_input * 4);
    float *g_dev = (float *)w; w += align_up(nw * 4);
    float *dw_dev = (float *)w;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    dn_status st = DN_OK;
    for (auto &e : ev)
        if (hipEventCreate(&e) != hipSuccess) st = DN_ERR_DEVICE;
    auto ok = [&](hipError_t e) { if (e != hipSuccess) st = DN_ERR_DEVICE; return st == DN_OK; };
    if (st == DN_OK) {
        // the task schedule of the paper: stream in, run the task, stream out
        ok(hipEventRecord(ev[0], stream)) &&
        ok(hipMemcpyAsync(d_dev, deltas_host, (size_t)cols_out * 4, hipMemcpyHostToDevice, stream)) &&
        ok(hipMemcpyAsync(x_dev, inputs_host, (size_t)cols_input * 4, hipMemcpyHostToDevice, stream)) &&
        ok(hipEventRecord(ev[1], stream)) &&
        ok(launch_layer_backward(d_dev, x_dev, learning_rate, cols_out, cols_input, g_dev, dw_dev, db_dev, stream)) &&
        ok(hipEventRecord(ev[2], stream)) &&
        ok(hipMemcpyAsync(gradients_host, g_dev, nw * 4, hipMemcpyDeviceToHost, stream)) &&
        ok(hipMemcpyAsync(delta_weights_host, dw_dev, nw * 4, hipMemcpyDeviceToHost, stream)) &&
        ok(hipMemcpyAsync(delta_biases_host, db_dev, (size_t)cols_out * 4, hipMemcpyDeviceToHost, stream)) &&
        ok(hipEventRecord(ev[3], stream)) &&
        ok(hipStreamSynchronize(stream));
    }
    if (st == DN_OK) {
        float a = 0.f, b = 0.f, c = 0.f;
        if (hipEventElapsedTime(&a, ev[0], ev[1]) != hipSuccess || hipEventElapsedTime(&b, ev[1], ev[2]) != hipSuccess ||
            hipEventElapsedTime(&c, ev[2], ev[3]) != hipSuccess)
            st = DN_ERR_DEVICE;
        if (ms_copy_in) *ms_copy_in = a;
        if (ms_kernel) *ms_kernel = b;
        if (ms_copy_out) *ms_copy_out = c;
    }
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    return st;
}

dn_status dn_last_epoch_ms(dn_net *net, float *epoch_ms)
{
    if (!net || !epoch_ms) return DN_ERR_INVALID_ARG;
    *epoch_ms = net->epoch_ms;
    return DN_OK;
}

dn_status dn_last_schedule(dn_net *net, int32_t *schedule)
{
    if (!net || !schedule) return DN_ERR_INVALID_ARG;
    *schedule = net->last_schedule;
    return DN_OK;
}

dn_status dn_kernel_time(dn_net *net, int32_t kernel_class, float *ms_total, int64_t *launches)
{
    if (!net || kernel_class < 0 || kernel_class >= DN_K_CLASSES) return DN_ERR_INVALID_ARG;
    if (ms_total) *ms_total = (float)net->cls_ms[kernel_class];
    if (launches) *launches = net->cls_launches[kernel_class];
    return DN_OK;
}

dn_status dn_kernel_flops(dn_net *net, int32_t kernel_class, double *flops)
{
    if (!net || !flops || kernel_class < 0 || kernel_class >= DN_K_CLASSES) return DN_ERR_INVALID_ARG;
    *flops = net->cls_flop[kernel_class];
    return DN_OK;
}

dn_status dn_set_option(dn_net *net, const char *name, int64_t value)
{
    if (!net || !name) return DN_ERR_INVALID_ARG;
    if (!strcmp(name, "time_kernels")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->time_kernels = (int)value;
    } else if (!strcmp(name, "gemm_variant")) {
        if (value < -1 || value >= gemm_variant_count()) return DN_ERR_INVALID_ARG;
        net->gemm_variant = (int)value;
    } else if (!strcmp(name, "online_mode")) {
        if (value < 0 || value > 2) return DN_ERR_INVALID_ARG;
        net->online_mode = (int)value;
    } else if (!strcmp(name, "online_min_tile")) {
        if (value < 1 || value > ((int64_t)1 << 30) || net->lo.online_bytes == 0) return DN_ERR_INVALID_ARG;
        OnlineGeom g;
        if (!online_geometry(net->n.data(), net->L, (int)value, false, g) || g.grid > net->device_cus)
            return DN_ERR_INVALID_ARG;
        if (hipStreamSynchronize(net->stream) != hipSuccess) return DN_ERR_DEVICE;
        net->online_min_tile = (int)value;
        refresh_persistent(net);   // the minibatch kernels cut their slices by the same option
    } else if (!strcmp(name, "batch_mode")) {
        if (value < 0 || value > 2) return DN_ERR_INVALID_ARG;
        net->batch_mode = (int)value;
    } else if (!strcmp(name, "merge_launches")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->merge_launches = (int)value;
    } else if (!strcmp(name, "split_k")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->split_k_on = (int)value;
    } else if (!strcmp(name, "online_resident")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->online_resident = (int)value;
    } else if (!strcmp(name, "online_tiny")) {
        if (value < 0 || value > 2) return DN_ERR_INVALID_ARG;
        net->online_tiny = (int)value;
    } else if (!strcmp(name, "online_solo")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->online_solo = (int)value;
    } else if (!strcmp(name, "online_twin")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->online_twin = (int)value;
    } else if (!strcmp(name, "online_wide")) {
        if (value != 0 && value != 1) return DN_ERR_INVALID_ARG;
        net->online_wide = (int)value;
    } else {
        return DN_ERR_INVALID_ARG;
    }
    return DN_OK;
}

}  // extern "C"
