// Convolutional and maximum-pooling layers, forward and backward, as stateless calls on device
// tensors (the layer types the paper's engine offers besides the fully connected and softmax ones
// and names as the next to accelerate; it gives no formulas, these are the usual definitions, stated
// in include/dn.h).  Gather form throughout: every output element is owned by one thread, wave or
// workgroup, so nothing is accumulated with atomics and every sum has a fixed order.  Stride-1
// layers wide enough for 32 x 32 tiles run their forward product and input gradient on the matrix
// cores (corr_mfma_kernel), with square filters of odd edge the filter gradient too (conv_dw_mfma_kernel);
// everything else uses register-tiled vector kernels.
#include <atomic>
#include <mutex>

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

constexpr int kStageFloats = 8192;   // filter values staged in LDS at a time (32 KB)

// y[b][o][i][j] for CO output channels o at a time: a thread owns one pixel (b, i, j) of a group of
// CO channels, so each input value it loads serves CO filters.  The group's filter values are
// staged through LDS, a range of input channels at a time, laid out [channel][tap][CO] so that a
// thread reads the CO values of a tap as 16-byte broadcasts.  Adjacent threads own adjacent j:
// input rows are read coalesced.
template <int CO>
__global__ __launch_bounds__(256) void conv_forward_kernel(ConvShape s, const float *__restrict__ X,
                                                           const float *__restrict__ Wt,
                                                           const float *__restrict__ bias, float *__restrict__ Y)
{
    __shared__ __attribute__((aligned(16))) float wl[kStageFloats];
    const int pix = s.Ho * s.Wo, taps = s.KH * s.KW;
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int og = blockIdx.y, b = blockIdx.z;
    const bool live = p < pix;
    const int i = live ? p / s.Wo : 0, j = live ? p - i * s.Wo : 0;
    float acc[CO];
#pragma unroll
    for (int q = 0; q < CO; ++q) acc[q] = bias[min(og * CO + q, s.Cout - 1)];   // past the end: repeats, not stored
    const int r0 = i * s.stride - s.pad, c0 = j * s.stride - s.pad;
    const int per_stage = max(1, kStageFloats / (taps * CO));   // input channels per stage
    for (int ci0 = 0; ci0 < s.Cin; ci0 += per_stage) {
        const int n = min(per_stage, s.Cin - ci0);
        __syncthreads();   // the previous stage has been used
        for (int e = threadIdx.x; e < n * taps * CO; e += 256) {
            const int q = e % CO, tap = (e / CO) % taps, cl = e / (CO * taps);
            wl[e] = Wt[((size_t)min(og * CO + q, s.Cout - 1) * s.Cin + ci0 + cl) * taps + tap];
        }
        __syncthreads();
        if (!live) continue;
        // the taps that fall inside the image, once per thread instead of a test per tap
        const int u_lo = max(0, -r0), u_hi = min(s.KH, s.H - r0), v_lo = max(0, -c0), v_hi = min(s.KW, s.W - c0);
        for (int cl = 0; cl < n; ++cl) {
            const float *x = X + ((size_t)b * s.Cin + ci0 + cl) * s.H * s.W + (size_t)r0 * s.W + c0;
            const float *wc = wl + (size_t)cl * taps * CO;
            for (int u = u_lo; u < u_hi; ++u) {
                for (int v = v_lo; v < v_hi; ++v) {
                    const float xv = x[u * s.W + v];
                    const float *wq = wc + (u * s.KW + v) * CO;
#pragma unroll
                    for (int q = 0; q < CO; ++q) acc[q] = fmaf(wq[q], xv, acc[q]);
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int q = 0; q < CO; ++q)
        if (og * CO + q < s.Cout) Y[((size_t)b * s.Cout + og * CO + q) * pix + p] = conv_act(s.act, acc[q]);
}

// Stride 1, both directions.  The forward product and the input gradient of a stride-1 layer are
// the same computation, a correlation of a multi-channel image with a filter bank:
//   out[b][oc][i][j] = fin(bias[oc] + sum_{ic,u,v} w(oc, ic, u, v) in[b][ic][i+u-pad_h][j+v-pad_w])
// forward: in = x, w = W[oc][ic][u][v], pads = pad; input gradient: in = delta, oc = the layer's input
// channel, ic = its output channel, w = W[ic][oc][kh-1-u][kw-1-v] (the flipped filter),
// pads = kh-1-pad and kw-1-pad, no bias, no activation.
// A thread owns RT consecutive output rows of one column j for a group of CO output channels.  Per
// input channel it loads the RT + kh - 1 input rows of its kw columns once into registers and
// uses each value for up to kh x CO products; filter values come from LDS ([ic][tap][CO], staged a
// range of input channels at a time) as 16-byte broadcasts.  No index arithmetic or bounds tests
// in the product loops: rows and columns outside the image are loaded as zeros.
struct CorrShape {
    int B, Cin, H, W, Cout, KH, KW, pad_h, pad_w, Ho, Wo, act;
    int w_out_stride, w_in_stride, flip;   // filter element (oc, ic, tap) at oc*w_out_stride + ic*w_in_stride + tap'
};

template <int CO, int RT, int KMAX>
__global__ __launch_bounds__(256) void corr_rows_kernel(CorrShape s, const float *__restrict__ In,
                                                        const float *__restrict__ Wt, const float *__restrict__ bias,
                                                        float *__restrict__ Out)
{
    __shared__ __attribute__((aligned(16))) float wl[kStageFloats];
    const int taps = s.KH * s.KW;
    const int tiles = (s.Ho + RT - 1) / RT;
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int og = blockIdx.y, b = blockIdx.z;
    const bool live = p < tiles * s.Wo;
    const int tile = live ? p / s.Wo : 0, j = live ? p - tile * s.Wo : 0;
    const int i0 = tile * RT;
    float acc[RT][CO];
#pragma unroll
    for (int q = 0; q < CO; ++q) {
        const float bq = bias ? bias[min(og * CO + q, s.Cout - 1)] : 0.f;   // past the end: repeats, not stored
#pragma unroll
        for (int t = 0; t < RT; ++t) acc[t][q] = bq;
    }
    const int c0 = j - s.pad_w, r0 = i0 - s.pad_h;
    bool col_ok[KMAX];
#pragma unroll
    for (int v = 0; v < KMAX; ++v) col_ok[v] = live && v < s.KW && c0 + v >= 0 && c0 + v < s.W;
    const int per_stage = max(1, kStageFloats / (taps * CO));   // input channels per stage
    for (int ic0 = 0; ic0 < s.Cin; ic0 += per_stage) {
        const int n = min(per_stage, s.Cin - ic0);
        __syncthreads();   // the previous stage has been used
        for (int e = threadIdx.x; e < n * taps * CO; e += 256) {
            const int q = e % CO, tap = (e / CO) % taps, cl = e / (CO * taps);
            wl[e] = Wt[(size_t)min(og * CO + q, s.Cout - 1) * s.w_out_stride + (size_t)(ic0 + cl) * s.w_in_stride +
                       (s.flip ? taps - 1 - tap : tap)];
        }
        __syncthreads();
        for (int cl = 0; cl < n; ++cl) {
            const float *x = In + ((size_t)b * s.Cin + ic0 + cl) * s.H * s.W;
            float xw[RT + KMAX - 1][KMAX];
#pragma unroll
            for (int k = 0; k < RT + KMAX - 1; ++k) {
                const int r = r0 + k;
                const bool row_ok = k < RT + s.KH - 1 && r >= 0 && r < s.H;
#pragma unroll
                for (int v = 0; v < KMAX; ++v) xw[k][v] = (row_ok && col_ok[v]) ? x[(size_t)r * s.W + c0 + v] : 0.f;
            }
            const float *wc = wl + (size_t)cl * taps * CO;
#pragma unroll
            for (int u = 0; u < KMAX; ++u) {
                if (u < s.KH) {
#pragma unroll
                    for (int v = 0; v < KMAX; ++v) {
                        if (v < s.KW) {
                            const float *wq = wc + (u * s.KW + v) * CO;
                            float w8[CO];
#pragma unroll
                            for (int q = 0; q < CO; ++q) w8[q] = wq[q];
#pragma unroll
                            for (int t = 0; t < RT; ++t)
#pragma unroll
                                for (int q = 0; q < CO; ++q) acc[t][q] = fmaf(w8[q], xw[t + u][v], acc[t][q]);
                        }
                    }
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int q = 0; q < CO; ++q)
            if (i0 + t < s.Ho && og * CO + q < s.Cout)
                Out[(((size_t)b * s.Cout + og * CO + q) * s.Ho + i0 + t) * s.Wo + j] = conv_act(s.act, acc[t][q]);
}

template <int CO>
hipError_t launch_corr_rows(const CorrShape &s, const float *In, const float *Wt, const float *bias, float *Out,
                            hipStream_t stream)
{
    const int kmax = s.KH > s.KW ? s.KH : s.KW;
    const int rt = kmax <= 5 ? 4 : 2;
    const int tiles = (s.Ho + rt - 1) / rt;
    const dim3 grid((unsigned)((tiles * s.Wo + 255) / 256), (unsigned)((s.Cout + CO - 1) / CO), (unsigned)s.B);
    if (kmax <= 3) hipLaunchKernelGGL((corr_rows_kernel<CO, 4, 3>), grid, dim3(256), 0, stream, s, In, Wt, bias, Out);
    else if (kmax <= 5) hipLaunchKernelGGL((corr_rows_kernel<CO, 4, 5>), grid, dim3(256), 0, stream, s, In, Wt, bias, Out);
    else hipLaunchKernelGGL((corr_rows_kernel<CO, 2, 7>), grid, dim3(256), 0, stream, s, In, Wt, bias, Out);
    return hipGetLastError();
}

// The same correlation (stride 1) on the matrix cores, for layers wide enough to fill their 32 x 32
// tiles.  Per image it is the product out[oc][pixel] = sum_k w[oc][k] patch[k][pixel] with
// k = (input channel, tap).  A workgroup owns 32 OT output channels x (8 output rows x 32 columns);
// wave r of its four owns output rows 2r and 2r + 1: 2 OT accumulator tiles of 32 channels x 32
// pixels.  One matrix instruction (32x32x2) takes two k values: lane (idx, h) supplies, for k slot h,
// the filter value of channel idx and the input value under pixel idx.  The two slots are two
// input channels at the same tap, so the input value's LDS address is the pixel's base plus one
// offset per (channel pair, tap) and there is no index arithmetic in the loop; every filter value
// read from LDS serves two instructions and so does every input value (OT = 2).  Input channels
// are staged through LDS eight at a time: the filters as [k][32 OT channels] with a row stride of
// 80 words (staging writes run along k for a few channels at a time: stride 16 mod 32 spreads them
// over the banks), the input as [channel][8 + kh - 1 rows][32 + kw - 1 columns], zeros outside
// the image.  Filters must be stored [oc][ic][tap] (w_in_stride = taps, no flip): the input
// gradient passes a flipped, transposed copy (written by conv_delta_kernel).
constexpr int MC_IC = 8, MC_WSTRIDE = 80;
typedef float v16f_t __attribute__((ext_vector_type(16)));

// KS: filter edge known at compile time (3: the tap loop is unrolled), 0: any.  TW: columns of the
// workgroup's pixel tile, 32 (a 32-pixel accumulator tile is one output row) or 16 (two rows of 16:
// images of at most 16 columns would leave half of every 32-column tile empty).
template <int OT, int RW, int KS, int TW = 32>
__global__ __launch_bounds__(256) void corr_mfma_kernel(CorrShape s, const float *__restrict__ In,
                                                        const float *__restrict__ Wt, const float *__restrict__ bias,
                                                        float *__restrict__ Out)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int OC = 32 * OT, RPT = 32 / TW, MC_ROWS = 4 * RW * RPT;   // RPT: output rows per accumulator tile
    const int taps = s.KH * s.KW, kstage = MC_IC * taps;
    const int prow = MC_ROWS + s.KH - 1, pcol = TW + s.KW - 1;   // staged input patch per channel
    float *wl = lds;                                   // [kstage][MC_WSTRIDE]
    float *pl = lds + (size_t)kstage * MC_WSTRIDE;     // [MC_IC][prow][pcol]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int idx = lane & 31, h = lane >> 5;
    const int col_tiles = (s.Wo + TW - 1) / TW;
    const int i0 = (blockIdx.x / col_tiles) * MC_ROWS, j0 = (blockIdx.x % col_tiles) * TW;
    const int oc0 = blockIdx.y * OC, b = blockIdx.z;
    v16f_t acc[OT][RW];
#pragma unroll
    for (int t = 0; t < OT; ++t)
#pragma unroll
        for (int q = 0; q < RW; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][q][r] = 0.f;
    const int r_in0 = i0 - s.pad_h, c_in0 = j0 - s.pad_w;   // image position of the patch's corner
    // staging roles: filters - four threads per output channel, each every fourth k of the stage;
    // input - one thread per patch column, a wave per patch row in turn
    const int w_ocl = tid >> 2, w_k0 = tid & 3;
    const bool w_on = w_ocl < OC;
    const int w_oc = min(oc0 + w_ocl, s.Cout - 1);
    const bool w_real = oc0 + w_ocl < s.Cout;
    // Filter edge known (3 x 3, 5 x 5): every load of a stage is requested at once, into registers, before the
    // first value is stored; the staging indices are recomputed from the thread
    // index every time rather than kept in registers across the product loop (the empty asm hides
    // that they repeat)
    constexpr int TAPS3 = KS * KS, PROW3 = MC_ROWS + KS - 1, PCOL3 = TW + KS - 1, NP3 = MC_IC * PROW3 * PCOL3;
    constexpr int XP3 = KS > 0 ? (NP3 + 255) / 256 : 1, WP3 = KS > 0 ? MC_IC * TAPS3 / 4 : 1;
    [[maybe_unused]] float wreg[WP3], xreg[XP3];
    [[maybe_unused]] auto stage_request = [&](int ic0) {
        const int st = tid;
        const int kvalid = min(MC_IC, s.Cin - ic0) * TAPS3;
        const int ocl = st >> 2, kq = st & 3;
        const bool real = ocl < OC && oc0 + ocl < s.Cout;
        const float *src = Wt + (size_t)min(oc0 + ocl, s.Cout - 1) * s.w_out_stride + (size_t)ic0 * TAPS3;
#pragma unroll
        for (int m = 0; m < WP3; ++m) {
            const int kl = kq + 4 * m;
            wreg[m] = (real && kl < kvalid) ? src[kl] : 0.f;
        }
        const float *img = In + ((size_t)b * s.Cin + ic0) * s.H * s.W;
#pragma unroll
        for (int m = 0; m < XP3; ++m) {
            const int e = st + 256 * m;
            const int c = e % PCOL3, pr = (e / PCOL3) % PROW3, icl = e / (PCOL3 * PROW3);
            const int r_img = r_in0 + pr, c_img = c_in0 + c;
            const bool ok = e < NP3 && ic0 + icl < s.Cin && r_img >= 0 && r_img < s.H && c_img >= 0 && c_img < s.W;
            xreg[m] = ok ? img[(unsigned)((icl * s.H + r_img) * s.W + c_img)] : 0.f;
        }
    };
    [[maybe_unused]] auto stage_store = [&]() {
        const int st = tid;
        const int ocl = st >> 2, kq = st & 3;
        if (ocl < OC) {
#pragma unroll
            for (int m = 0; m < WP3; ++m) wl[(kq + 4 * m) * MC_WSTRIDE + ocl] = wreg[m];
        }
#pragma unroll
        for (int m = 0; m < XP3; ++m) {
            const int e = st + 256 * m;
            if (e < NP3) pl[e] = xreg[m];
        }
    };
    if constexpr (KS > 0) stage_request(0);
    for (int ic0 = 0; ic0 < s.Cin; ic0 += MC_IC) {
        [[maybe_unused]] const int kvalid = min(MC_IC, s.Cin - ic0) * taps;   // k values of this stage that exist
        __syncthreads();   // the previous stage has been used
        if constexpr (KS > 0) {
            stage_store();
        } else {
        // (loads in batches, all of a batch in flight before the first is stored)
        constexpr int WB = 9, PB = 6;
        if (w_on) {
            const float *src = Wt + (size_t)w_oc * s.w_out_stride + (size_t)ic0 * taps;
            for (int k0 = w_k0; k0 < kstage; k0 += 4 * WB) {
                float tmp[WB];
#pragma unroll
                for (int m = 0; m < WB; ++m) {
                    const int kl = k0 + 4 * m;
                    tmp[m] = (w_real && kl < kvalid) ? src[kl] : 0.f;
                }
#pragma unroll
                for (int m = 0; m < WB; ++m) {
                    const int kl = k0 + 4 * m;
                    if (kl < kstage) wl[kl * MC_WSTRIDE + w_ocl] = tmp[m];
                }
            }
        }
        for (int row0 = wave; row0 < MC_IC * prow; row0 += 4 * PB) {
            float tmp[PB];
#pragma unroll
            for (int m = 0; m < PB; ++m) {
                const int row = row0 + 4 * m;
                const int icl = row / prow, pr = row - icl * prow;   // uniform across the wave
                const int r = r_in0 + pr, c = c_in0 + lane, ic = ic0 + icl;
                const bool ok = row < MC_IC * prow && lane < pcol && ic < s.Cin && r >= 0 && r < s.H && c >= 0 && c < s.W;
                tmp[m] = ok ? In[(((size_t)b * s.Cin + ic) * s.H + r) * s.W + c] : 0.f;
            }
#pragma unroll
            for (int m = 0; m < PB; ++m) {
                const int row = row0 + 4 * m;
                if (row < MC_IC * prow && lane < pcol) pl[row * pcol + lane] = tmp[m];
            }
        }
        }
        __syncthreads();
        if constexpr (KS > 0) {
            if (ic0 + MC_IC < s.Cin) stage_request(ic0 + MC_IC);
        }
        // k slot h of every instruction: input channel 2 * pair + h at one tap
        const float *wa = wl + (size_t)(h * taps) * MC_WSTRIDE + idx;
        const float *pb = pl + (size_t)h * prow * pcol + (RW * wave * RPT + idx / TW) * pcol + idx % TW;
#pragma unroll
        for (int pair = 0; pair < MC_IC / 2; ++pair) {
            const float *wp = wa + (size_t)(2 * pair * taps) * MC_WSTRIDE;
            const float *pp = pb + (size_t)(2 * pair) * prow * pcol;
            auto one_tap = [&](int tap, int po) {   // po: patch offset u * pcol + v of the tap
                float xv[RW];
#pragma unroll
                for (int q = 0; q < RW; ++q) xv[q] = pp[po + q * RPT * pcol];
                const float *wq = wp + tap * MC_WSTRIDE;
#pragma unroll
                for (int t = 0; t < OT; ++t) {
                    const float wv = wq[32 * t];
#pragma unroll
                    for (int q = 0; q < RW; ++q)
                        acc[t][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(wv, xv[q], acc[t][q], 0, 0, 0);
                }
            };
            if (KS > 0) {
#pragma unroll
                for (int u = 0; u < KS; ++u)
#pragma unroll
                    for (int v = 0; v < KS; ++v) one_tap(u * KS + v, u * pcol + v);
            } else {
                for (int u = 0; u < s.KH; ++u)
                    for (int v = 0; v < s.KW; ++v) one_tap(u * s.KW + v, u * pcol + v);
            }
        }
    }
    // the workgroup's biases go through LDS: one read from memory each instead of one per output
    // (the condition is the same for the whole grid)
    if (bias) {
        __syncthreads();
        if (tid < OC) wl[tid] = oc0 + tid < s.Cout ? bias[oc0 + tid] : 0.f;
        __syncthreads();
    }
    // register r of lane (idx, h): output channel 8 (r / 4) + 4 h + r % 4 of the tile, pixel idx of the tile's row(s)
    const int j = j0 + idx % TW;
    if (j >= s.Wo) return;
#pragma unroll
    for (int q = 0; q < RW; ++q) {
        const int i = i0 + (RW * wave + q) * RPT + idx / TW;
        if (i >= s.Ho) continue;
#pragma unroll
        for (int t = 0; t < OT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ocl = 32 * t + 8 * (r >> 2) + 4 * h + (r & 3);
                if (oc0 + ocl < s.Cout)
                    Out[(((size_t)b * s.Cout + oc0 + ocl) * s.Ho + i) * s.Wo + j] =
                        conv_act(s.act, acc[t][q][r] + (bias ? wl[ocl] : 0.f));
            }
    }
}

// Wide enough for the matrix-core form?  (Narrow layers would mostly multiply padding.)
bool corr_mfma_fits(const CorrShape &s)
{
    // (3 x 3 filters have 16-column pixel tiles; the others' tiles are 32 columns wide)
    const int min_w = s.KH == 3 && s.KW == 3 ? 12 : 16;
    return s.Cout >= 32 && s.Cin >= 8 && s.Wo >= min_w && s.w_in_stride == s.KH * s.KW && !s.flip;
}

template <int OT, int RW, int KS, int TW = 32>
hipError_t launch_corr_mfma_as(const CorrShape &s, const float *In, const float *Wt, const float *bias, float *Out,
                               hipStream_t stream)
{
    constexpr int rows = 4 * RW * (32 / TW);
    const int taps = s.KH * s.KW;
    const size_t lds = sizeof(float) * ((size_t)MC_IC * taps * MC_WSTRIDE +
                                        (size_t)MC_IC * (rows + s.KH - 1) * (TW + s.KW - 1));
    // 7 x 7 filters need up to 146 KB, more than the default limit of dynamic LDS (the calls are stateless and
    // may come from several threads: setting the limit twice is harmless, the flag is read and written atomically)
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&corr_mfma_kernel<OT, RW, KS, TW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const dim3 grid((unsigned)(((s.Ho + rows - 1) / rows) * ((s.Wo + TW - 1) / TW)),
                    (unsigned)((s.Cout + 32 * OT - 1) / (32 * OT)), (unsigned)s.B);
    hipLaunchKernelGGL((corr_mfma_kernel<OT, RW, KS, TW>), grid, dim3(256), lds, stream, s, In, Wt, bias, Out);
    return hipGetLastError();
}

hipError_t launch_corr_mfma(const CorrShape &s, const float *In, const float *Wt, const float *bias, float *Out,
                            hipStream_t stream)
{
    const bool k3 = s.KH == 3 && s.KW == 3, k5 = s.KH == 5 && s.KW == 5;
    // 3 x 3: pixel tiles of 16 rows x 16 columns instead of 8 x 32 where they cover the image with less padding
    const auto padded = [&](int rows, int cols) {
        return (long)((s.Ho + rows - 1) / rows * rows) * ((s.Wo + cols - 1) / cols * cols);
    };
    const bool narrow = k3 && padded(16, 16) < padded(8, 32);
    // ... and of half the rows when the full tiles would leave CUs without a workgroup
    const long wg16 = (long)((s.Ho + 15) / 16) * ((s.Wo + 15) / 16) * s.B * ((s.Cout + 63) / 64);
    const bool small = narrow && wg16 < 512;
    if (s.Cout > 32) {
        if (small) return launch_corr_mfma_as<2, 1, 3, 16>(s, In, Wt, bias, Out, stream);
        if (narrow) return launch_corr_mfma_as<2, 2, 3, 16>(s, In, Wt, bias, Out, stream);
        if (k5) return launch_corr_mfma_as<2, 2, 5>(s, In, Wt, bias, Out, stream);
        return k3 ? launch_corr_mfma_as<2, 2, 3>(s, In, Wt, bias, Out, stream)
                  : launch_corr_mfma_as<2, 2, 0>(s, In, Wt, bias, Out, stream);
    }
    if (small) return launch_corr_mfma_as<1, 1, 3, 16>(s, In, Wt, bias, Out, stream);
    if (narrow) return launch_corr_mfma_as<1, 2, 3, 16>(s, In, Wt, bias, Out, stream);
    if (k5) return launch_corr_mfma_as<1, 2, 5>(s, In, Wt, bias, Out, stream);
    return k3 ? launch_corr_mfma_as<1, 2, 3>(s, In, Wt, bias, Out, stream)
              : launch_corr_mfma_as<1, 2, 0>(s, In, Wt, bias, Out, stream);
}

// The first `delta_blocks` workgroups write delta = dA f'(Y).  The others, if there are any, write
// the flipped, transposed filter copy the matrix-core input gradient reads, one element per thread:
// Wf[c][o][tap] = W[o][c][taps - 1 - tap], the filters of the input gradient seen as a correlation.
__global__ __launch_bounds__(256) void conv_delta_kernel(const float *__restrict__ dA, const float *__restrict__ Y,
                                                         float *__restrict__ delta, size_t count, int act,
                                                         unsigned delta_blocks, const float *__restrict__ Wt,
                                                         float *__restrict__ Wf, int c_out, int c_in, int taps)
{
    if (blockIdx.x >= delta_blocks) {
        const size_t e = (size_t)(blockIdx.x - delta_blocks) * 256 + threadIdx.x;
        if (e >= (size_t)c_out * c_in * taps) return;
        const int tap = (int)(e % taps);
        const int o = (int)((e / taps) % c_out), c = (int)(e / ((size_t)taps * c_out));
        Wf[e] = Wt[((size_t)o * c_in + c) * taps + (taps - 1 - tap)];
        return;
    }
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (size_t)delta_blocks * 256)
        delta[e] = dA[e] * conv_deriv(act, Y[e]);
}

// dW[o][c][u][v] = (1/B) sum_{b,i,j} delta[b][o][i][j] x[b][c][i*stride+u-pad][j*stride+v-pad].
// A workgroup owns one input channel c, a group of CO output channels and a chunk of the batch's
// images, and holds all CO x kh x kw sums of that chunk in registers: its threads take the
// positions (b, i, j) in turn (adjacent threads adjacent j); every input value a thread loads
// serves CO filters and every delta value the whole filter window.  The threads' sums are added
// in a fixed order (lane butterfly, then the four waves) and written to part[chunk][o][c][u][v];
// conv_dw_reduce_kernel adds the chunks in order and divides by the batch.  Chunks exist so
// that layers with few channels still fill the device.
template <int KMAX, int CO>
__global__ __launch_bounds__(256) void conv_dw_kernel(ConvShape s, const float *__restrict__ X,
                                                      const float *__restrict__ delta, float *__restrict__ part,
                                                      int images_per_chunk)
{
    __shared__ float red[4][CO * KMAX * KMAX + CO];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pix = s.Ho * s.Wo;
    const int c = blockIdx.x % s.Cin, og = blockIdx.x / s.Cin;
    const int b0 = blockIdx.y * images_per_chunk, b1 = min(s.B, b0 + images_per_chunk);
    const int total = (b1 - b0) * pix;
    int oc[CO];
#pragma unroll
    for (int q = 0; q < CO; ++q) oc[q] = min(og * CO + q, s.Cout - 1);   // past the end: repeats, not stored
    float acc[CO][KMAX][KMAX];
#pragma unroll
    for (int q = 0; q < CO; ++q)
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
#pragma unroll
            for (int v = 0; v < KMAX; ++v) acc[q][u][v] = 0.f;
    float bsum[CO];   // the chunk's sum of delta per channel: the bias gradient (kept by the workgroups of c = 0)
#pragma unroll
    for (int q = 0; q < CO; ++q) bsum[q] = 0.f;
    for (int t = tid; t < total; t += 256) {
        const int b = b0 + t / pix, p = t % pix;
        const int i = p / s.Wo, j = p - i * s.Wo;
        float d[CO];
#pragma unroll
        for (int q = 0; q < CO; ++q) {
            d[q] = delta[((size_t)b * s.Cout + oc[q]) * pix + p];
            bsum[q] += d[q];
        }
        const float *x = X + ((size_t)b * s.Cin + c) * s.H * s.W;
        const int r0 = i * s.stride - s.pad, c0 = j * s.stride - s.pad;
#pragma unroll
        for (int u = 0; u < KMAX; ++u) {
            if (u < s.KH) {
                const int r = r0 + u;
                const bool row_ok = r >= 0 && r < s.H;
#pragma unroll
                for (int v = 0; v < KMAX; ++v) {
                    if (v < s.KW) {
                        const int cc = c0 + v;
                        const bool ok = row_ok && cc >= 0 && cc < s.W;
                        const float xv = ok ? x[(size_t)r * s.W + cc] : 0.f;
#pragma unroll
                        for (int q = 0; q < CO; ++q) acc[q][u][v] = fmaf(d[q], xv, acc[q][u][v]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < CO; ++q)
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
#pragma unroll
            for (int v = 0; v < KMAX; ++v) {
                if (u < s.KH && v < s.KW) {   // uniform
                    const float w_sum = wave_sum(acc[q][u][v]);
                    if (lane == 0) red[wave][(q * KMAX + u) * KMAX + v] = w_sum;
                }
            }
    if (c == 0) {
#pragma unroll
        for (int q = 0; q < CO; ++q) {
            const float b_sum = wave_sum(bsum[q]);
            if (lane == 0) red[wave][CO * KMAX * KMAX + q] = b_sum;
        }
    }
    __syncthreads();
    const size_t filt = (size_t)s.Cout * s.Cin * s.KH * s.KW;
    const size_t per_chunk = filt + s.Cout;   // filter sums, then bias sums
    if (c == 0 && tid < CO && og * CO + tid < s.Cout) {
        const int e = CO * KMAX * KMAX + tid;
        part[(size_t)blockIdx.y * per_chunk + filt + og * CO + tid] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    }
    for (int e = tid; e < CO * KMAX * KMAX; e += 256) {
        const int q = e / (KMAX * KMAX), u = (e / KMAX) % KMAX, v = e % KMAX;
        if (u < s.KH && v < s.KW && og * CO + q < s.Cout)
            part[(size_t)blockIdx.y * per_chunk + (((size_t)(og * CO + q) * s.Cin + c) * s.KH + u) * s.KW + v] =
                (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    }
}

// The same for stride 1, where consecutive output rows share all but one row of their input
// windows: a thread owns one output column j of one image and walks down the rows, keeping the
// kh x kw window in registers and loading only its new bottom row per step (no index arithmetic
// in the loop).  Window rows sit at the bottom of a KMAX-row register array so that the row that
// is replaced has a fixed register position whatever kh is.
template <int KMAX, int CO>
__global__ __launch_bounds__(256) void conv_dw_slide_kernel(ConvShape s, const float *__restrict__ X,
                                                            const float *__restrict__ delta, float *__restrict__ part,
                                                            int images_per_chunk, int bands, int rows_per_band)
{
    __shared__ float red[4][CO * KMAX * KMAX + CO];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pix = s.Ho * s.Wo;
    const int c = blockIdx.x % s.Cin, og = blockIdx.x / s.Cin;
    // a chunk is a group of images and a band of their output rows
    const int band = blockIdx.y % bands;
    const int b0 = (blockIdx.y / bands) * images_per_chunk, b1 = min(s.B, b0 + images_per_chunk);
    const int i_lo = band * rows_per_band, i_hi = min(s.Ho, i_lo + rows_per_band);
    const int total = (b1 - b0) * s.Wo;
    const int off = KMAX - s.KH;   // window row u lives at index u + off
    int oc[CO];
#pragma unroll
    for (int q = 0; q < CO; ++q) oc[q] = min(og * CO + q, s.Cout - 1);   // past the end: repeats, not stored
    float acc[CO][KMAX][KMAX];
#pragma unroll
    for (int q = 0; q < CO; ++q)
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
#pragma unroll
            for (int v = 0; v < KMAX; ++v) acc[q][u][v] = 0.f;
    float bsum[CO];   // the chunk's sum of delta per channel: the bias gradient (kept by the workgroups of c = 0)
#pragma unroll
    for (int q = 0; q < CO; ++q) bsum[q] = 0.f;
    for (int t = tid; t < total; t += 256) {
        const int b = b0 + t / s.Wo, j = t % s.Wo;
        const float *x = X + ((size_t)b * s.Cin + c) * s.H * s.W;
        const float *d = delta + (size_t)b * s.Cout * pix + j;
        const int c0 = j - s.pad;
        bool col_ok[KMAX];
#pragma unroll
        for (int v = 0; v < KMAX; ++v) col_ok[v] = v < s.KW && c0 + v >= 0 && c0 + v < s.W;
        float win[KMAX][KMAX];
        // the window of the output row before the band: its rows 1 .. kh-1 are rows 0 .. kh-2 of the band's first
#pragma unroll
        for (int u = 0; u < KMAX; ++u) {
            const int r = i_lo - 1 - s.pad + (u - off);
            const bool row_ok = u >= off && r >= 0 && r < s.H;
#pragma unroll
            for (int v = 0; v < KMAX; ++v) win[u][v] = (row_ok && col_ok[v]) ? x[(size_t)r * s.W + c0 + v] : 0.f;
        }
        for (int i = i_lo; i < i_hi; ++i) {
#pragma unroll
            for (int u = 0; u < KMAX - 1; ++u)
#pragma unroll
                for (int v = 0; v < KMAX; ++v) win[u][v] = win[u + 1][v];
            const int r = i - s.pad + s.KH - 1;
            const bool row_ok = r >= 0 && r < s.H;
#pragma unroll
            for (int v = 0; v < KMAX; ++v) win[KMAX - 1][v] = (row_ok && col_ok[v]) ? x[(size_t)r * s.W + c0 + v] : 0.f;
            float dv[CO];
#pragma unroll
            for (int q = 0; q < CO; ++q) {
                dv[q] = d[(size_t)oc[q] * pix + (size_t)i * s.Wo];
                bsum[q] += dv[q];
            }
#pragma unroll
            for (int u = 0; u < KMAX; ++u) {
                if (u >= off) {
#pragma unroll
                    for (int v = 0; v < KMAX; ++v) {
                        if (v < s.KW) {
#pragma unroll
                            for (int q = 0; q < CO; ++q) acc[q][u][v] = fmaf(dv[q], win[u][v], acc[q][u][v]);
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < CO; ++q)
#pragma unroll
        for (int u = 0; u < KMAX; ++u)
#pragma unroll
            for (int v = 0; v < KMAX; ++v) {
                if (u >= off && v < s.KW) {   // uniform
                    const float w_sum = wave_sum(acc[q][u][v]);
                    if (lane == 0) red[wave][(q * KMAX + u) * KMAX + v] = w_sum;
                }
            }
    if (c == 0) {
#pragma unroll
        for (int q = 0; q < CO; ++q) {
            const float b_sum = wave_sum(bsum[q]);
            if (lane == 0) red[wave][CO * KMAX * KMAX + q] = b_sum;
        }
    }
    __syncthreads();
    const size_t filt = (size_t)s.Cout * s.Cin * s.KH * s.KW;
    const size_t per_chunk = filt + s.Cout;   // filter sums, then bias sums
    if (c == 0 && tid < CO && og * CO + tid < s.Cout) {
        const int e = CO * KMAX * KMAX + tid;
        part[(size_t)blockIdx.y * per_chunk + filt + og * CO + tid] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    }
    for (int e = tid; e < CO * KMAX * KMAX; e += 256) {
        const int q = e / (KMAX * KMAX), u = (e / KMAX) % KMAX, v = e % KMAX;
        if (u >= off && v < s.KW && og * CO + q < s.Cout)
            part[(size_t)blockIdx.y * per_chunk + (((size_t)(og * CO + q) * s.Cin + c) * s.KH + (u - off)) * s.KW + v] =
                (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
    }
}

// The stride-1 filter gradient of square filters of edge 3, 5 or 7 on the matrix cores, for wide
// layers (described for 3 x 3).  Per image it is the product
// dW[oc][n] = sum_pixel delta[oc][pixel] xs[n][pixel] with n = (input channel, tap) and xs the
// input shifted by the tap.  A workgroup of four waves owns 64 output channels, a group of up to
// 17 input channels (153 columns n in five 32-column tiles) and a part of the batch's pixels
// (several images, one image, or a band of its rows).  Wave w owns column tile w over all pixels
// and column tile 4 over a quarter of them (the four quarters are added through LDS at the end, in
// wave order),
// each for both 32-channel halves: four accumulator tiles.  One matrix instruction takes two
// pixels: lane (idx, h) supplies delta of channel idx and the input under its column, both at
// pixel 2 t + h; one input value read from LDS serves both channel halves.  The pixels are walked
// in blocks of 128 / TW output rows x TW columns staged through LDS - delta as [channel][128 pixels]
// (row stride 129 words; read from memory 16 bytes at a time where the caller's pointer allows),
// the input as [channel][block rows + 2][TW + 2] with zeros outside the image - all of a block's
// loads requested before the first is stored.  A column's
// LDS address is a per-lane base (its channel and tap, and the lane's pixel of the pair) plus a
// constant per pixel pair.  The partial result goes to part[chunk][oc][ic][tap] like the other
// filter-gradient kernels', the bias sums (input-channel group 0: sums of the delta values the
// workgroup stages) behind it; conv_dw_reduce_kernel adds the chunks.
// TW: columns of a pixel block, 32 (4 rows) or 16 (8 rows; images of at most 16 columns would leave
// half of every 32-column block empty).  KS: filter edge, 3, 5 or 7 (5 x 5: groups of up to 6 input
// channels, 150 columns; 7 x 7: 3 channels, 147 columns; the text above gives the figures for 3 x 3).
constexpr int DWM_THREADS = 256, DWM_DSTRIDE = 129;
constexpr int dwm_group(int ks) { return 160 / (ks * ks); }     // input channels whose columns fit five 32-column tiles
constexpr int DWM_DP = (2048 + DWM_THREADS - 1) / DWM_THREADS;   // delta pieces per thread
constexpr int DWM_XMAX = 17 * 6 * 34;                            // staged input values: the largest of the block shapes

template <int TW, int KS>
__global__ __launch_bounds__(DWM_THREADS, 3) void conv_dw_mfma_kernel(ConvShape s, const float *__restrict__ X,
                                                                      const float *__restrict__ delta,
                                                                      float *__restrict__ part, int ig, int bands,
                                                                      int rows_per_band, int images_per_chunk,
                                                                      int delta_vec)
{
    __shared__ __attribute__((aligned(16))) float dl[64 * DWM_DSTRIDE];
    __shared__ float xl[DWM_XMAX];
    constexpr int taps = KS * KS, DWM_IG = dwm_group(KS);
    constexpr int BR = 128 / TW, DWM_PROW = BR + KS - 1, DWM_PCOL = TW + KS - 1;   // block rows; staged input rows and columns
    constexpr int NX = DWM_IG * DWM_PROW * DWM_PCOL, DWM_XP = (NX + DWM_THREADS - 1) / DWM_THREADS;
    static_assert(NX <= DWM_XMAX, "staged input exceeds its LDS array");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int idx = lane & 31, h = lane >> 5;
    const int groups = (s.Cin + ig - 1) / ig;
    const int icg = blockIdx.x % groups, ocg = blockIdx.x / groups;
    const int ic0 = icg * ig, oc0 = ocg * 64;
    const int nic = min(ig, s.Cin - ic0);   // input channels of this workgroup that exist
    const int band = blockIdx.y % bands;
    const int b_lo = (blockIdx.y / bands) * images_per_chunk, b_hi = min(s.B, b_lo + images_per_chunk);
    const int row_lo = band * rows_per_band, row_hi = min(s.Ho, row_lo + rows_per_band);
    const int pix = s.Ho * s.Wo;
    // a column's channel and tap as an offset into the staged input (0 for columns past the last one)
    auto column_base = [&](int n) {
        const int n_ic = n / taps, n_tap = n - n_ic * taps;
        return n < nic * taps ? (n_ic * DWM_PROW + n_tap / KS) * DWM_PCOL + n_tap % KS : 0;
    };
    const int n_own = 32 * wave + idx, n_shared = 128 + idx;
    const bool shared_on = nic * taps > 128;   // the fifth tile has columns
    const float *xb = xl + column_base(n_own) + h;
    const float *xs = xl + column_base(n_shared) + h;
    const float *da = dl + idx * DWM_DSTRIDE + h;
    v16f_t acc0, acc1, acc2, acc3;   // own tile: channels 0..31, 32..63; shared tile likewise
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = acc2[r] = acc3[r] = 0.f;
    typedef float v4_t __attribute__((ext_vector_type(4)));
    float bsum[DWM_DP];   // sums of the delta values this thread stages, per staged piece (a piece has one channel)
#pragma unroll
    for (int m = 0; m < DWM_DP; ++m) bsum[m] = 0.f;
    for (int b = b_lo; b < b_hi; ++b)
    for (int i0 = row_lo; i0 < row_hi; i0 += BR)
        for (int j0 = 0; j0 < s.Wo; j0 += TW) {
            __syncthreads();   // the previous block has been used
            // The staging indices are recomputed from the thread index in every block rather than
            // kept in registers across the product loop (the empty asm hides that they repeat).
            int st = tid;
            asm volatile("" : "+v"(st));
            // delta: 64 channels x BR rows x TW / 4 pieces of four pixels = 2048 pieces; input: nic x (BR + 2) x (TW + 2) values
            v4_t dreg[DWM_DP];
            float xreg[DWM_XP];
            const float *dblk = delta + ((size_t)b * s.Cout + oc0) * pix + (size_t)i0 * s.Wo + j0;
#pragma unroll
            for (int m = 0; m < DWM_DP; ++m) {
                const int e = st + DWM_THREADS * m;
                const int q = e % (TW / 4), row = (e / (TW / 4)) % BR, ocl = e >> 5;
                const int left = s.Wo - (j0 + 4 * q);   // pixels of the row from this piece on
                const bool ok = e < 2048 && oc0 + ocl < s.Cout && i0 + row < row_hi && left > 0;
                v4_t v = {0.f, 0.f, 0.f, 0.f};
                if (ok) {
                    const float *src = dblk + (unsigned)(ocl * pix + row * s.Wo + 4 * q);
                    // 16 bytes at once if the caller's pointer is 16-byte aligned and the rows are whole pieces
                    if (delta_vec) v = *reinterpret_cast<const v4_t *>(src);
                    else {
                        v[0] = src[0];
                        if (left > 1) v[1] = src[1];
                        if (left > 2) v[2] = src[2];
                        if (left > 3) v[3] = src[3];
                    }
                }
                dreg[m] = v;
            }
            const float *xblk = X + ((size_t)b * s.Cin + ic0) * s.H * s.W;
#pragma unroll
            for (int m = 0; m < DWM_XP; ++m) {
                const int e = st + DWM_THREADS * m;
                const int c = e % DWM_PCOL, pr = (e / DWM_PCOL) % DWM_PROW, icl = e / (DWM_PCOL * DWM_PROW);
                const int r_img = i0 - s.pad + pr, c_img = j0 - s.pad + c;
                // rows beyond the band carry no delta of this workgroup but are still inputs of its last rows
                const bool ok = icl < nic && r_img >= 0 && r_img < s.H && c_img >= 0 && c_img < s.W;
                xreg[m] = ok ? xblk[(unsigned)((icl * s.H + r_img) * s.W + c_img)] : 0.f;
            }
#pragma unroll
            for (int m = 0; m < DWM_DP; ++m) {
                const int e = st + DWM_THREADS * m;
                if (e < 2048) {
                    float *dst = dl + (e >> 5) * DWM_DSTRIDE + 4 * (e & 31);   // pixel (row, 4 q) of the block = row * TW + 4 q
                    dst[0] = dreg[m][0]; dst[1] = dreg[m][1]; dst[2] = dreg[m][2]; dst[3] = dreg[m][3];
                    bsum[m] += (dreg[m][0] + dreg[m][1]) + (dreg[m][2] + dreg[m][3]);
                }
            }
#pragma unroll
            for (int m = 0; m < DWM_XP; ++m) {
                const int e = st + DWM_THREADS * m;
                if (e < NX) xl[e] = xreg[m];
            }
            __syncthreads();
            // 64 pixel pairs: pair t holds pixels 2 t and 2 t + 1 of the block (row 2 t / TW, column 2 t % TW);
            // the wave multiplies the shared tile over the pairs of quarter `wave`.  (The lane's half h is in its base
            // addresses, so every offset below is a constant.)
#pragma unroll
            for (int row = 0; row < 4; ++row) {
                if (row == wave && shared_on) {
#pragma unroll
                    for (int t = 16 * row; t < 16 * row + 16; ++t) {
                        const int xo = (2 * t / TW) * DWM_PCOL + (2 * t) % TW;
                        const float d0 = da[2 * t], d1 = da[32 * DWM_DSTRIDE + 2 * t];
                        const float x = xb[xo], x4 = xs[xo];
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(d0, x, acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(d1, x, acc1, 0, 0, 0);
                        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(d0, x4, acc2, 0, 0, 0);
                        acc3 = __builtin_amdgcn_mfma_f32_32x32x2f32(d1, x4, acc3, 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int t = 16 * row; t < 16 * row + 16; ++t) {
                        const float x = xb[(2 * t / TW) * DWM_PCOL + (2 * t) % TW];
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(da[2 * t], x, acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(da[32 * DWM_DSTRIDE + 2 * t], x, acc1, 0, 0, 0);
                    }
                }
            }
        }
    // register r of lane (idx, h): output channel 8 (r / 4) + 4 h + r % 4 of the tile, the lane's column
    const size_t filt = (size_t)s.Cout * s.Cin * taps;
    const size_t per_chunk = filt + s.Cout;
    float *out = part + (size_t)blockIdx.y * per_chunk;
    if (n_own < nic * taps) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int ocl = 8 * (r >> 2) + 4 * h + (r & 3);
            if (oc0 + ocl < s.Cout) out[((size_t)(oc0 + ocl) * s.Cin + ic0) * taps + n_own] = acc0[r];
            if (oc0 + 32 + ocl < s.Cout) out[((size_t)(oc0 + 32 + ocl) * s.Cin + ic0) * taps + n_own] = acc1[r];
        }
    }
    // the shared tile: every wave leaves its quarter in LDS as [wave][register][lane]; wave w
    // then adds the four quarters of registers 8 w .. 8 w + 7 (of 32: both channel halves)
    __syncthreads();
    float *quarter = dl;   // 4 * 32 * 64 words
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        quarter[(wave * 32 + r) * 64 + lane] = acc2[r];
        quarter[(wave * 32 + 16 + r) * 64 + lane] = acc3[r];
    }
    __syncthreads();
    if (n_shared < nic * taps) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int rr = 8 * wave + k;   // 0..15: channels 0..31, 16..31: channels 32..63
            float sum = quarter[rr * 64 + lane];
#pragma unroll
            for (int w = 1; w < 4; ++w) sum += quarter[(w * 32 + rr) * 64 + lane];
            const int r = rr & 15;
            const int ocl = 32 * (rr >> 4) + 8 * (r >> 2) + 4 * h + (r & 3);
            if (oc0 + ocl < s.Cout) out[((size_t)(oc0 + ocl) * s.Cin + ic0) * taps + n_shared] = sum;
        }
    }
    if (icg == 0) {
        // piece e = tid + 256 m belongs to channel e >> 5: add the pieces per channel through LDS, in order
        __syncthreads();
        float *red = dl;   // [2048] piece sums
#pragma unroll
        for (int m = 0; m < DWM_DP; ++m) {
            const int e = tid + DWM_THREADS * m;
            if (e < 2048) red[e] = bsum[m];
        }
        __syncthreads();
        if (tid < 64 && oc0 + tid < s.Cout) {
            float sum = 0.f;
            for (int k = 0; k < 32; ++k) sum += red[tid * 32 + k];
            out[filt + oc0 + tid] = sum;
        }
    }
}

// dW and dbias = (1/B) sum over chunks (in order) of part; one thread per filter element / channel.
__global__ __launch_bounds__(256) void conv_dw_reduce_kernel(const float *__restrict__ part, float *__restrict__ dW,
                                                             float *__restrict__ dbias, size_t filt, int c_out,
                                                             int chunks, float inv_b)
{
    // 32 elements per block; the chunks are cut into 8 runs, one per group of 32 threads, whose
    // sums are added in run order
    __shared__ float run_sum[8][32];
    const int el = threadIdx.x & 31, run = threadIdx.x >> 5;
    const size_t e = (size_t)blockIdx.x * 32 + el;
    const size_t per_chunk = filt + c_out;
    const int per_run = (chunks + 7) / 8;
    const int k_lo = run * per_run, k_hi = min(chunks, k_lo + per_run);
    float sum = 0.f;
    if (e < per_chunk) {
#pragma unroll 8
        for (int k = k_lo; k < k_hi; ++k) sum += part[(size_t)k * per_chunk + e];
    }
    run_sum[run][el] = sum;
    __syncthreads();
    if (run != 0 || e >= per_chunk) return;
    for (int r = 1; r < 8; ++r) sum += run_sum[r][el];
    if (e < filt) dW[e] = sum * inv_b;
    else dbias[e - filt] = sum * inv_b;
}

// dX[b][c][r][col] = sum over (o, u, v) with r = i*stride+u-pad, col = j*stride+v-pad of
// delta[b][o][i][j] W[o][c][u][v]: a thread owns one input pixel of a group of CI channels, so each
// delta value it loads serves CI filters.  The group's filter values are staged through LDS, a
// range of output channels at a time, laid out [output channel][tap][CI].
template <int CI>
__global__ __launch_bounds__(256) void conv_dx_kernel(ConvShape s, const float *__restrict__ Wt,
                                                      const float *__restrict__ delta, float *__restrict__ dX)
{
    __shared__ __attribute__((aligned(16))) float wl[kStageFloats];
    const int hw = s.H * s.W;
    const int p = blockIdx.x * 256 + threadIdx.x;
    const int cg = blockIdx.y, b = blockIdx.z;
    const bool live = p < hw;
    const int r = live ? p / s.W : 0, col = live ? p - r * s.W : 0;
    const int pix = s.Ho * s.Wo;
    const int taps = s.KH * s.KW;
    float acc[CI];
#pragma unroll
    for (int q = 0; q < CI; ++q) acc[q] = 0.f;
    const int per_stage = max(1, kStageFloats / (taps * CI));   // output channels per stage
    for (int o0 = 0; o0 < s.Cout; o0 += per_stage) {
        const int n = min(per_stage, s.Cout - o0);
        __syncthreads();   // the previous stage has been used
        for (int e = threadIdx.x; e < n * taps * CI; e += 256) {
            const int q = e % CI, tap = (e / CI) % taps, ol = e / (CI * taps);
            wl[e] = Wt[((size_t)(o0 + ol) * s.Cin + min(cg * CI + q, s.Cin - 1)) * taps + tap];   // past the end: repeats
        }
        __syncthreads();
        if (!live) continue;
        if (s.stride == 1) {
            // output rows i = r + pad - u and columns j = col + pad - v inside the output: the
            // valid taps form a rectangle, found once per thread
            const int u_lo = max(0, r + s.pad - s.Ho + 1), u_hi = min(s.KH, r + s.pad + 1);
            const int v_lo = max(0, col + s.pad - s.Wo + 1), v_hi = min(s.KW, col + s.pad + 1);
            const float *d0 = delta + ((size_t)b * s.Cout + o0) * pix + (size_t)(r + s.pad) * s.Wo + (col + s.pad);
            for (int ol = 0; ol < n; ++ol) {
                const float *d = d0 + (size_t)ol * pix;
                const float *wo = wl + (size_t)ol * taps * CI;
                for (int u = u_lo; u < u_hi; ++u)
                    for (int v = v_lo; v < v_hi; ++v) {
                        const float dv = d[-(u * s.Wo + v)];
                        const float *wq = wo + (u * s.KW + v) * CI;
#pragma unroll
                        for (int q = 0; q < CI; ++q) acc[q] = fmaf(dv, wq[q], acc[q]);
                    }
            }
            continue;
        }
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
                const float *d = delta + ((size_t)b * s.Cout + o0) * pix + (size_t)i * s.Wo + j;
                const float *wt = wl + (size_t)(u * s.KW + v) * CI;
                for (int ol = 0; ol < n; ++ol) {
                    const float dv = d[(size_t)ol * pix];
                    const float *wq = wt + (size_t)ol * taps * CI;
#pragma unroll
                    for (int q = 0; q < CI; ++q) acc[q] = fmaf(dv, wq[q], acc[q]);
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int q = 0; q < CI; ++q)
        if (cg * CI + q < s.Cin) dX[((size_t)b * s.Cin + cg * CI + q) * hw + p] = acc[q];
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

// Windows that tile the image exactly (stride = k, h and w multiples of k): every input pixel
// belongs to one window, so a thread owns a window, finds its first maximum and writes all of the
// window's input gradients (dY at the maximum, zero elsewhere).
__global__ __launch_bounds__(256) void maxpool_backward_tiles_kernel(PoolShape s, const float *__restrict__ X,
                                                                     const float *__restrict__ dY,
                                                                     float *__restrict__ dX)
{
    const int pix = s.Ho * s.Wo;
    const int p = blockIdx.x * 256 + threadIdx.x, plane = blockIdx.y;
    if (p >= pix) return;
    const int i = p / s.Wo, j = p - i * s.Wo;
    const size_t base = (size_t)plane * s.H * s.W + (size_t)(i * s.K) * s.W + j * s.K;
    const float *x = X + base;
    float m = x[0];
    int best = 0;
    for (int u = 0; u < s.K; ++u)
        for (int v = 0; v < s.K; ++v) {
            const float xv = x[(size_t)u * s.W + v];
            if (xv > m) {   // strictly greater: the first maximum wins
                m = xv;
                best = u * s.K + v;
            }
        }
    const float g = dY[(size_t)plane * pix + p];
    float *d = dX + base;
    for (int u = 0; u < s.K; ++u)
        for (int v = 0; v < s.K; ++v) d[(size_t)u * s.W + v] = (u * s.K + v == best) ? g : 0.f;
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

// How the weight-gradient kernel splits the batch: CO output channels per workgroup by filter
// size, and as many chunks of images as it takes to put about a thousand workgroups on the device.
struct DwPlan {
    int co, groups, chunks, images_per_chunk;
    size_t filt;
    int mfma_ig, mfma_tw, bands, rows_per_band;   // mfma_ig > 0: the matrix-core kernel, pixel blocks mfma_tw columns wide
};

DwPlan dw_plan(const ConvShape &s)
{
    DwPlan p;
    const int kmax = s.KH > s.KW ? s.KH : s.KW;
    p.co = kmax <= 3 ? 8 : (kmax <= 5 ? 4 : 2);
    p.groups = (s.Cout + p.co - 1) / p.co;
    const long per_chunk = (long)p.groups * s.Cin;
    long chunks = (1024 + per_chunk - 1) / per_chunk;
    if (chunks > s.B) chunks = s.B;
    if (chunks < 1) chunks = 1;
    p.images_per_chunk = (int)((s.B + chunks - 1) / chunks);
    // the stride-1 kernel gives a thread one output column of one image: a chunk should hold enough
    // images to keep a workgroup's 256 threads busy
    if (s.stride == 1) {
        const int fill = (256 + s.Wo - 1) / s.Wo;
        if (p.images_per_chunk < fill) p.images_per_chunk = fill < s.B ? fill : s.B;
    }
    p.chunks = (s.B + p.images_per_chunk - 1) / p.images_per_chunk;
    p.filt = (size_t)s.Cout * s.Cin * s.KH * s.KW;
    p.mfma_ig = 0;
    p.mfma_tw = 32;
    p.bands = 1;
    p.rows_per_band = s.Ho;
    // few channels and a small batch: the stride-1 kernel also cuts the images into bands of at
    // least four output rows (a band reloads kh - 1 rows above it), towards two workgroups per CU
    if (s.stride == 1 && per_chunk * p.chunks < 512) {
        long bands = (512 + per_chunk * p.chunks - 1) / (per_chunk * p.chunks);
        const long max_bands = s.Ho / 4 > 1 ? s.Ho / 4 : 1;
        if (bands > max_bands) bands = max_bands;
        p.rows_per_band = (int)((s.Ho + bands - 1) / bands);
        p.bands = (s.Ho + p.rows_per_band - 1) / p.rows_per_band;
        p.chunks *= p.bands;
    }
    if (s.stride == 1 && s.KH == s.KW && (s.KH == 3 || s.KH == 5 || s.KH == 7) && s.Cout >= 32 && s.Cin >= 8 && s.Wo >= 12) {
        const int max_group = s.KH == 3 ? dwm_group(3) : (s.KH == 5 ? dwm_group(5) : dwm_group(7));
        const int groups = (s.Cin + max_group - 1) / max_group;
        const int ig = (s.Cin + groups - 1) / groups;   // even groups
        // about three workgroups per CU: several images per chunk if the batch gives more, else
        // one image per chunk cut into bands of rows
        const long wg_per_image = (long)groups * ((s.Cout + 63) / 64);
        const long want = 768;
        int ipc = (int)(wg_per_image * s.B / want);
        if (ipc < 1) ipc = 1;
        int bands = ipc > 1 ? 1 : (int)((want + wg_per_image * s.B - 1) / (wg_per_image * s.B));
        // pixel blocks of 8 rows x 16 columns instead of 4 x 32 where they cover the image with less padding
        const auto padded = [&](int rows, int cols) {
            return (long)((s.Ho + rows - 1) / rows * rows) * ((s.Wo + cols - 1) / cols * cols);
        };
        p.mfma_tw = padded(8, 16) < padded(4, 32) ? 16 : 32;
        const int br = 128 / p.mfma_tw;
        const int max_bands = (s.Ho + br - 1) / br;
        if (bands > max_bands) bands = max_bands;
        const int rows = ((s.Ho + bands - 1) / bands + br - 1) / br * br;   // whole blocks
        bands = (s.Ho + rows - 1) / rows;
        const int image_groups = (s.B + ipc - 1) / ipc;
        if (wg_per_image * image_groups * bands >= 192) {   // else too few workgroups to be worth it
            p.mfma_ig = ig;
            p.bands = bands;
            p.rows_per_band = rows;
            p.images_per_chunk = ipc;
            p.chunks = image_groups * bands;
        }
    }
    return p;
}

size_t conv_backward_scratch_bytes(const ConvShape &s, const DwPlan &p)
{
    return ((p.filt + (size_t)s.Cout) * (size_t)p.chunks + p.filt) * sizeof(float);   // partial sums, flipped filters
}

dn_status conv_backward_run(const ConvShape &s, const DwPlan &p, const float *X_dev, const float *W_dev,
                            const float *Y_dev, const float *dA_dev, float *delta_dev, float *dX_dev, float *dW_dev,
                            float *dbias_dev, float *part, hipStream_t stream);

// ---- scratch memory of dn_conv_backward_static ---------------------------------------------
// A fixed device array takes the place of the caller's workspace.  Each device the library runs
// on holds its own copy at its own address for the life of the process; the address is looked up
// once per device (with that device current) and only that pointer -- never the array's name,
// which is a host-side stand-in -- is handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
}  // namespace dn

static __device__ __align__(256) unsigned char scratch[dn::kStaticScratchBytes];

namespace dn {
namespace {
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

dn_status static_scratch(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DN_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return DN_ERR_DEVICE;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<float *>(g_scratch_ptr[dev]);
    return DN_OK;
}

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
    hipStream_t stream = (hipStream_t)hip_stream;
    const int co = s.Cout >= 8 ? 8 : 4;
    if (s.stride == 1) {
        const int taps = s.KH * s.KW;
        const CorrShape c{s.B, s.Cin, s.H, s.W, s.Cout, s.KH, s.KW, s.pad, s.pad, s.Ho, s.Wo, s.act, s.Cin * taps, taps, 0};
        const hipError_t e = corr_mfma_fits(c) ? launch_corr_mfma(c, X_dev, W_dev, bias_dev, Y_dev, stream)
                             : co == 8         ? launch_corr_rows<8>(c, X_dev, W_dev, bias_dev, Y_dev, stream)
                                               : launch_corr_rows<4>(c, X_dev, W_dev, bias_dev, Y_dev, stream);
        return e == hipSuccess ? DN_OK : DN_ERR_DEVICE;
    }
    const dim3 grid((unsigned)((s.Ho * s.Wo + 255) / 256), (unsigned)((s.Cout + co - 1) / co), (unsigned)s.B);
    if (co == 8)
        hipLaunchKernelGGL(conv_forward_kernel<8>, grid, dim3(256), 0, stream, s, X_dev, W_dev, bias_dev, Y_dev);
    else
        hipLaunchKernelGGL(conv_forward_kernel<4>, grid, dim3(256), 0, stream, s, X_dev, W_dev, bias_dev, Y_dev);
    return launched();
}

size_t dn_conv_backward_workspace_bytes(int32_t batch, int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh,
                                        int32_t kw, int32_t stride, int32_t pad)
{
    ConvShape s;
    if (conv_shape(batch, c_in, h, w, c_out, kh, kw, stride, pad, DN_ACT_LINEAR, s) != DN_OK) return 0;
    return conv_backward_scratch_bytes(s, dw_plan(s));
}

dn_status dn_conv_backward(const float *X_dev, const float *W_dev, const float *Y_dev, const float *dA_dev,
                           float *delta_dev, float *dX_dev, float *dW_dev, float *dbias_dev, void *workspace_dev,
                           size_t workspace_bytes, int32_t batch, int32_t c_in, int32_t h, int32_t w, int32_t c_out,
                           int32_t kh, int32_t kw, int32_t stride, int32_t pad, dn_act act, void *hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || !dA_dev || !delta_dev || !dW_dev || !dbias_dev || !workspace_dev)
        return DN_ERR_INVALID_ARG;
    ConvShape s;
    const dn_status st = conv_shape(batch, c_in, h, w, c_out, kh, kw, stride, pad, (int)act, s);
    if (st != DN_OK) return st;
    const DwPlan p = dw_plan(s);
    if (workspace_bytes < conv_backward_scratch_bytes(s, p)) return DN_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(workspace_dev) & 3) != 0) return DN_ERR_INVALID_ARG;
    return conv_backward_run(s, p, X_dev, W_dev, Y_dev, dA_dev, delta_dev, dX_dev, dW_dev, dbias_dev,
                             static_cast<float *>(workspace_dev), (hipStream_t)hip_stream);
}

dn_status dn_conv_backward_static(const float *X_dev, const float *W_dev, const float *Y_dev, const float *dA_dev,
                                  float *delta_dev, float *dX_dev, float *dW_dev, float *dbias_dev, int32_t batch,
                                  int32_t c_in, int32_t h, int32_t w, int32_t c_out, int32_t kh, int32_t kw,
                                  int32_t stride, int32_t pad, dn_act act, void *hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || !dA_dev || !delta_dev || !dW_dev || !dbias_dev) return DN_ERR_INVALID_ARG;
    ConvShape s;
    const dn_status st = conv_shape(batch, c_in, h, w, c_out, kh, kw, stride, pad, (int)act, s);
    if (st != DN_OK) return st;
    const DwPlan p = dw_plan(s);
    if (conv_backward_scratch_bytes(s, p) > kStaticScratchBytes) return DN_ERR_SHAPE;   // layer too large for the fixed buffer
    float *part = nullptr;
    const dn_status sp = static_scratch(&part);
    if (sp != DN_OK) return sp;
    return conv_backward_run(s, p, X_dev, W_dev, Y_dev, dA_dev, delta_dev, dX_dev, dW_dev, dbias_dev, part,
                             (hipStream_t)hip_stream);
}

size_t dn_conv_backward_static_limit(void) { return kStaticScratchBytes; }

}  // extern "C"

namespace dn {
namespace {

// The launches of dn_conv_backward / dn_conv_backward_static; `part` is the scratch memory (partial
// sums of the filter and bias gradients, then the flipped filters), every word of which is written
// by this call before it is read.
dn_status conv_backward_run(const ConvShape &s, const DwPlan &p, const float *X_dev, const float *W_dev,
                            const float *Y_dev, const float *dA_dev, float *delta_dev, float *dX_dev, float *dW_dev,
                            float *dbias_dev, float *part, hipStream_t stream)
{
    const size_t ny = (size_t)s.B * s.Cout * s.Ho * s.Wo;
    size_t blocks = (ny + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    // the stride-1 input gradient is a correlation of delta with the flipped filters; on the matrix
    // cores it reads a flipped, transposed copy of them, kept behind the partial sums
    const int taps = s.KH * s.KW;
    const CorrShape cm{s.B, s.Cout, s.Ho, s.Wo, s.Cin, s.KH, s.KW, s.KH - 1 - s.pad, s.KW - 1 - s.pad, s.H, s.W,
                       DN_ACT_LINEAR, s.Cout * taps, taps, 0};
    const bool dx_mfma = dX_dev && s.stride == 1 && corr_mfma_fits(cm);
    float *flipped = part + (p.filt + (size_t)s.Cout) * (size_t)p.chunks;
    const size_t flip_blocks = dx_mfma ? (p.filt + 255) / 256 : 0;
    hipLaunchKernelGGL(conv_delta_kernel, dim3((unsigned)(blocks + flip_blocks)), dim3(256), 0, stream, dA_dev, Y_dev,
                       delta_dev, ny, s.act, (unsigned)blocks, W_dev, flipped, s.Cout, s.Cin, taps);
    if (launched() != DN_OK) return DN_ERR_DEVICE;
    const dim3 grid_dw((unsigned)(p.groups * s.Cin), (unsigned)p.chunks);
    if (p.mfma_ig > 0) {
        const int groups = (s.Cin + p.mfma_ig - 1) / p.mfma_ig;
        const dim3 grid((unsigned)(groups * ((s.Cout + 63) / 64)), (unsigned)p.chunks);
        const int vec = (int)(reinterpret_cast<uintptr_t>(delta_dev) % 16 == 0 && s.Wo % 4 == 0);
        auto *kernel = s.KH == 3   ? (p.mfma_tw == 16 ? conv_dw_mfma_kernel<16, 3> : conv_dw_mfma_kernel<32, 3>)
                       : s.KH == 5 ? (p.mfma_tw == 16 ? conv_dw_mfma_kernel<16, 5> : conv_dw_mfma_kernel<32, 5>)
                                   : (p.mfma_tw == 16 ? conv_dw_mfma_kernel<16, 7> : conv_dw_mfma_kernel<32, 7>);
        hipLaunchKernelGGL(kernel, grid, dim3(DWM_THREADS), 0, stream, s, X_dev, delta_dev, part, p.mfma_ig, p.bands,
                           p.rows_per_band, p.images_per_chunk, vec);
    } else if (s.stride == 1 && p.co == 8)
        hipLaunchKernelGGL((conv_dw_slide_kernel<3, 8>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk, p.bands, p.rows_per_band);
    else if (s.stride == 1 && p.co == 4)
        hipLaunchKernelGGL((conv_dw_slide_kernel<5, 4>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk, p.bands, p.rows_per_band);
    else if (s.stride == 1)
        hipLaunchKernelGGL((conv_dw_slide_kernel<7, 2>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk, p.bands, p.rows_per_band);
    else if (p.co == 8)
        hipLaunchKernelGGL((conv_dw_kernel<3, 8>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk);
    else if (p.co == 4)
        hipLaunchKernelGGL((conv_dw_kernel<5, 4>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk);
    else
        hipLaunchKernelGGL((conv_dw_kernel<7, 2>), grid_dw, dim3(256), 0, stream, s, X_dev, delta_dev, part,
                           p.images_per_chunk);
    if (launched() != DN_OK) return DN_ERR_DEVICE;
    hipLaunchKernelGGL(conv_dw_reduce_kernel, dim3((unsigned)((p.filt + s.Cout + 31) / 32)), dim3(256), 0, stream, part,
                       dW_dev, dbias_dev, p.filt, s.Cout, p.chunks, 1.0f / (float)s.B);
    if (launched() != DN_OK) return DN_ERR_DEVICE;
    if (dX_dev && s.stride == 1) {
        const CorrShape c{s.B, s.Cout, s.Ho, s.Wo, s.Cin, s.KH, s.KW, s.KH - 1 - s.pad, s.KW - 1 - s.pad, s.H, s.W,
                          DN_ACT_LINEAR, taps, s.Cin * taps, 1};
        hipError_t e;
        if (dx_mfma) e = launch_corr_mfma(cm, delta_dev, flipped, nullptr, dX_dev, stream);
        else
            e = s.Cin >= 8 ? launch_corr_rows<8>(c, delta_dev, W_dev, nullptr, dX_dev, stream)
                           : launch_corr_rows<4>(c, delta_dev, W_dev, nullptr, dX_dev, stream);
        if (e != hipSuccess) return DN_ERR_DEVICE;
    } else if (dX_dev) {
        const int ci = s.Cin >= 8 ? 8 : (s.Cin >= 2 ? 4 : 1);
        const dim3 grid((unsigned)((s.H * s.W + 255) / 256), (unsigned)((s.Cin + ci - 1) / ci), (unsigned)s.B);
        if (ci == 8) hipLaunchKernelGGL(conv_dx_kernel<8>, grid, dim3(256), 0, stream, s, W_dev, delta_dev, dX_dev);
        else if (ci == 4) hipLaunchKernelGGL(conv_dx_kernel<4>, grid, dim3(256), 0, stream, s, W_dev, delta_dev, dX_dev);
        else hipLaunchKernelGGL(conv_dx_kernel<1>, grid, dim3(256), 0, stream, s, W_dev, delta_dev, dX_dev);
        if (launched() != DN_OK) return DN_ERR_DEVICE;
    }
    return DN_OK;
}

}  // namespace
}  // namespace dn

extern "C" {

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
    if (s.stride == s.K && s.H % s.K == 0 && s.W % s.K == 0) {
        const dim3 grid((unsigned)((s.Ho * s.Wo + 255) / 256), (unsigned)s.planes);
        hipLaunchKernelGGL(maxpool_backward_tiles_kernel, grid, dim3(256), 0, (hipStream_t)hip_stream, s, X_dev, dY_dev,
                           dX_dev);
        return launched();
    }
    const dim3 grid((unsigned)((s.H * s.W + 255) / 256), (unsigned)s.planes);
    hipLaunchKernelGGL(maxpool_backward_kernel, grid, dim3(256), 0, (hipStream_t)hip_stream, s, X_dev, dY_dev, dX_dev);
    return launched();
}

}  // extern "C"
