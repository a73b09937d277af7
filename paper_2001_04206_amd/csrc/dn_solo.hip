// Per-sample (batch 1) training of two-layer nets whose first weight matrix fits the register file
// of ONE compute unit, plain gradient descent: a single workgroup of eight wavefronts runs the epoch.
//
// A net like 784-128-10 has 100 000 weights in W_1: too many for one wavefront, few enough for the
// 128 K registers of a compute unit.  Spread over several workgroups, every step pays an exchange
// through device memory (several microseconds); inside one workgroup the same exchange is an LDS
// write, a barrier and an LDS read.  So the whole epoch runs on one compute unit:
//
//  * The 8 waves form a UG x SEGS grid (UG = groups of 64 hidden units, SEGS = 8 / UG segments of
//    C input columns).  Lane j of wave (ug, seg) is hidden unit 64 ug + j and keeps the C weights of
//    its row that fall into segment seg in registers, for the whole epoch.
//  * The features of a sample are the same for every lane of a wave, so they are read through the
//    constant address space: scalar loads into scalar registers, which enter the multiply-adds as a
//    scalar operand.  No vector register, LDS read or cross-lane move is spent on them, in the forward
//    product and again in the rank-1 update.  (The samples are only ever read.)
//  * Step: every wave forms its part of z_1 (C multiply-adds per lane), the parts meet in LDS
//    [barrier]; every wave assembles all of a_1; wave w forms output units w and w + 8 from rows of
//    W_2 it keeps spread over its lanes, one wave-wide sum each, and leaves them in LDS [barrier];
//    every wave then computes the output error (and thread 0 the loss) redundantly and, from its two
//    rows of W_2, a part of W_2^T delta_2 for every hidden unit; the eight parts meet in LDS [barrier];
//    every wave sums them for its own 64 units and applies the updates to what it holds.  Copies of a
//    value held by several waves (the biases) take the same operation from the same operands and
//    stay equal bit for bit.  Three barriers per step, no wait on anything outside the compute unit.
//  * Rows of future samples are touched with one vector load per 128 bytes a few steps ahead, so that
//    the scalar loads find them in the L2.
//
// The scalar loads of a step read C columns per segment whether or not the row is that long
// (weights past the row's end are zero); the host keeps the steps whose over-read would leave the
// sample array for another schedule.
#include <algorithm>

#include "dn_internal.h"
#include "dn_persist.h"
#include "dn_wave.h"

namespace dn {
namespace {

typedef const float __attribute__((address_space(4))) *const_floats;
typedef const int32_t __attribute__((address_space(4))) *const_ints;

// Scalar loads of 16 (4) consecutive features into scalar registers, issued by hand so that the next
// chunk travels while the current one is used (scalar loads return in any order, so the only wait
// there is waits for all of them: chunk i is awaited BEFORE chunk i + 1 is requested).  The compiler
// does not know that DST is pending between the two statements; ARRIVED both waits and hands the
// value on, so every use comes after it.  AFTER names a result of the chunk before, which keeps the
// compiler from moving the wait up over that chunk's arithmetic; BEFORE names an operand of the
// current chunk's arithmetic, which keeps the request for the next chunk ahead of it (without the two
// the compiler orders request, wait, use with nothing in between).
typedef float xs16 __attribute__((ext_vector_type(16)));
typedef float xs4 __attribute__((ext_vector_type(4)));
#define SOLO_LOAD16(DST, BASE, BYTES, BEFORE) \
    asm volatile("s_load_dwordx16 %0, %2, %3" : "=s"(DST), "+v"(BEFORE) : "s"(BASE), "s"((int)(BYTES)))
#define SOLO_LOAD4(DST, BASE, BYTES, BEFORE) \
    asm volatile("s_load_dwordx4 %0, %2, %3" : "=s"(DST), "+v"(BEFORE) : "s"(BASE), "s"((int)(BYTES)))
#define SOLO_ARRIVED(V, AFTER) asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(V), "+v"(AFTER))

__device__ __forceinline__ float solo_lane_read(float v, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}

template <int UG, int C>
__global__ __launch_bounds__(SOLO_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void solo_epoch_kernel(SoloPlan p)
{
    constexpr int SEGS = 8 / UG, N2 = SOLO_MAX_OUT, KK = SOLO_MAX_OUT / 8, PF = 4;
    constexpr int NFULL = C / 16, REM = C % 16;   // chunks of 16 features, and what is left
    static_assert(NFULL >= 1 && (REM == 0 || REM == 4), "feature chunks are 16 wide, a last one may be 4 wide");
    __shared__ float part[SEGS][64 * UG];   // parts of z_1, one per column segment
    __shared__ float z2s[N2];               // z_2 without the biases
    __shared__ float dpart[8][64 * UG];     // parts of W_2^T delta_2, one per wave (its two rows of W_2)
    __shared__ double loss_sum;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int ug = wave % UG, seg = wave / UG;
    const int n0 = p.n0, n1 = p.n1, n2 = p.n2;
    const int unit = 64 * ug + lane;
    const int c0 = seg * C;
    const int nv = max(0, min(C, p.n0 - c0));   // columns of this segment that exist
    const bool hid = unit < n1, outl = lane < n2;

    // ---- prologue: what this wave keeps ----
    float w[C];      // row `unit` of W_1, columns c0 .. c0 + C - 1
#pragma unroll
    for (int c = 0; c < C; ++c) w[c] = (hid && c0 + c < n0) ? p.W1[(size_t)unit * n0 + c0 + c] : 0.f;
    float w2r[KK][UG];   // rows wave + 8 kk of W_2, columns lane + 64 u
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int u = 0; u < UG; ++u)
            w2r[kk][u] = (wave + 8 * kk < n2 && lane + 64 * u < n1) ? p.W2[(wave + 8 * kk) * n1 + lane + 64 * u] : 0.f;
    float b1 = hid ? p.b1[unit] : 0.f;    // every wave of the unit group keeps a copy; segment 0 adds it to its part
    float b2 = outl ? p.b2[lane] : 0.f;   // every wave keeps a copy

    const const_floats xc = (const_floats)(uintptr_t)p.X;
    const const_ints yc = (const_ints)(uintptr_t)p.labels;
    // one float per 128 bytes of the row PF steps ahead, to bring it into the L2
    const int pf_col = (int)threadIdx.x * 32;
    float pf = 0.f;
    if (threadIdx.x == 0) loss_sum = 0.0;
    const int n_steps = (int)p.n_samples;   // (the host keeps a launch within 2^30 steps)

    for (int s = 0; s < n_steps; ++s) {
        const bool keepv = p.keep_v && s == n_steps - 1;   // the epoch's last step also leaves the applied change as velocity
        const const_floats x = xc + (size_t)s * n0 + c0;
        asm volatile("" ::"v"(pf));
        pf = (pf_col < n0) ? p.X[(size_t)min(s + PF, n_steps - 1) * n0 + pf_col] : 0.f;
        int y = yc[s];
        y = y < 0 ? 0 : (y >= n2 ? n2 - 1 : y);

        // ---- this wave's part of z_1: chunk i + 1 of the features is on its way while chunk i is used ----
        float zq[4] = {seg == 0 ? b1 : 0.f, 0.f, 0.f, 0.f};
        {
            xs16 xa, xb;
            xs4 xr;
            SOLO_LOAD16(xa, x, 0, w[0]);
#pragma unroll
            for (int i = 0; i < NFULL; ++i) {
                if (i & 1) SOLO_ARRIVED(xb, zq[(i + 3) & 3]); else SOLO_ARRIVED(xa, zq[(i + 3) & 3]);
                if (i + 1 < NFULL) {
                    if (i & 1) SOLO_LOAD16(xa, x, (i + 1) * 64, w[16 * i]); else SOLO_LOAD16(xb, x, (i + 1) * 64, w[16 * i]);
                } else if (REM) {
                    SOLO_LOAD4(xr, x, NFULL * 64, w[16 * i]);
                }
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    zq[i & 3] = __builtin_fmaf(w[16 * i + j], (i & 1) ? xb[j] : xa[j], zq[i & 3]);
            }
            if (REM) {
                SOLO_ARRIVED(xr, zq[(NFULL + 3) & 3]);
#pragma unroll
                for (int j = 0; j < REM; ++j) zq[NFULL & 3] = __builtin_fmaf(w[16 * NFULL + j], xr[j], zq[NFULL & 3]);
            }
        }
        part[seg][unit] = (zq[0] + zq[1]) + (zq[2] + zq[3]);
        __syncthreads();

        // ---- all of a_1 (lane j: units j + 64 u), this wave's output units ----
        float a1[UG];
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            float t = part[0][64 * u + lane];
#pragma unroll
            for (int g = 1; g < SEGS; ++g) t += part[g][64 * u + lane];
            a1[u] = (64 * u + lane < n1) ? act_fn(p.act1, t) : 0.f;
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            float t = 0.f;
#pragma unroll
            for (int u = 0; u < UG; ++u) t = __builtin_fmaf(w2r[kk][u], a1[u], t);
            t = wave_sum(t);
            if (lane == 0) z2s[wave + 8 * kk] = t;
        }
        __syncthreads();

        // ---- output error and loss (every wave alike; lane k is output unit k) ----
        const float z2 = outl ? z2s[lane] + b2 : 0.f;
        const float t1 = lane == y ? 1.0f : 0.0f;
        float d2, e;
        if (p.loss == DN_LOSS_CROSS_ENTROPY) {
            const float zz = outl ? z2 : -INFINITY;
            const float m = wave_max(zz);
            const float ex = outl ? expf(zz - m) : 0.f;
            const float sum = wave_sum(ex);
            d2 = outl ? ex * (1.0f / sum) - t1 : 0.f;
            e = logf(sum) - (solo_lane_read(z2, y) - m);
        } else {
            const float a2 = outl ? act_fn(p.act2, z2) : 0.f;
            const float f = outl ? a2 - t1 : 0.f;
            d2 = f * act_deriv(p.act2, a2);
            e = wave_sum(0.5f * f * f);
        }
        if (threadIdx.x == 0) loss_sum += (double)e;

        // ---- deltas of the hidden units through W_2 as it was: this wave's rows give a part for every
        //      unit, the eight parts meet in LDS ----
#pragma unroll
        for (int u = 0; u < UG; ++u) {
            float t = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) t = __builtin_fmaf(w2r[kk][u], solo_lane_read(d2, (wave + 8 * kk) & 63), t);
            dpart[wave][64 * u + lane] = t;
        }
        __syncthreads();
        float a_own = a1[0];
#pragma unroll
        for (int u = 1; u < UG; ++u) a_own = ug == u ? a1[u] : a_own;
        float sacc = dpart[0][unit];
#pragma unroll
        for (int g = 1; g < 8; ++g) sacc += dpart[g][unit];
        const float d1 = hid ? sacc * act_deriv(p.act1, a_own) : 0.f;

        // ---- updates: w = fma(-(lr delta), input, w) ----
        const float nld2 = -(p.lr * d2), nld1 = -(p.lr * d1);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int k = wave + 8 * kk;
            const float g = solo_lane_read(nld2, k & 63);
#pragma unroll
            for (int u = 0; u < UG; ++u) {
                w2r[kk][u] = __builtin_fmaf(g, a1[u], w2r[kk][u]);
            }
        }
        b2 += nld2;
        b1 += nld1;
        {   // W_1: the same pipeline over the features.  Columns past the row's end keep their zeros: a
            // chunk that lies past it is skipped, the chunk that holds it is put right afterwards.
            int nvv = __builtin_amdgcn_readfirstlane(nv);
            asm volatile("" : "+s"(nvv));   // (keeps the comparisons below inside the loop, in scalar registers only while they are used)
            xs16 xa, xb;
            xs4 xr;
            SOLO_LOAD16(xa, x, 0, w[0]);
#pragma unroll
            for (int i = 0; i < NFULL; ++i) {
                if (i & 1) SOLO_ARRIVED(xb, w[i ? 16 * i - 1 : 0]); else SOLO_ARRIVED(xa, w[i ? 16 * i - 1 : 0]);
                if (i + 1 < NFULL) {
                    if (i & 1) SOLO_LOAD16(xa, x, (i + 1) * 64, w[16 * i]); else SOLO_LOAD16(xb, x, (i + 1) * 64, w[16 * i]);
                } else if (REM) {
                    SOLO_LOAD4(xr, x, NFULL * 64, w[16 * i]);
                }
                if (16 * i < nvv) {
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        w[16 * i + j] = __builtin_fmaf(nld1, (i & 1) ? xb[j] : xa[j], w[16 * i + j]);
                    if (16 * (i + 1) > nvv) {
#pragma unroll
                        for (int j = 1; j < 16; ++j) w[16 * i + j] = (16 * i + j < nvv) ? w[16 * i + j] : 0.f;
                    }
                }
            }
            if (REM) {
                SOLO_ARRIVED(xr, w[16 * NFULL - 1]);
                if (16 * NFULL < nvv) {
#pragma unroll
                    for (int j = 0; j < REM; ++j) w[16 * NFULL + j] = __builtin_fmaf(nld1, xr[j], w[16 * NFULL + j]);
                    if (16 * NFULL + REM > nvv) {
#pragma unroll
                        for (int j = 1; j < REM; ++j) w[16 * NFULL + j] = (16 * NFULL + j < nvv) ? w[16 * NFULL + j] : 0.f;
                    }
                }
            }
        }
        if (keepv) {
            // (the widths as the compiler cannot see through them: the bounds tests below would otherwise be
            // computed once before the loop and held in scalar registers through every step)
            int n0v = n0, n1v = n1, n2v = n2;
            asm volatile("" : "+s"(n0v), "+s"(n1v), "+s"(n2v));
#pragma unroll
            for (int c = 0; c < C; ++c)
                if (hid && c0 + c < n0v) p.VW1[(size_t)unit * n0v + c0 + c] = nld1 * x[c];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int k = wave + 8 * kk;
                const float g = solo_lane_read(nld2, k & 63);
#pragma unroll
                for (int u = 0; u < UG; ++u)
                    if (k < n2v && lane + 64 * u < n1v) p.VW2[k * n1v + lane + 64 * u] = g * a1[u];
            }
            if (seg == 0 && hid) p.Vb1[unit] = nld1;
            if (wave == 0 && outl) p.Vb2[lane] = nld2;
        }
    }
    asm volatile("" ::"v"(pf));

    // ---- epilogue ----
    // (the widths once more as the compiler cannot see through them: the prologue's bounds tests are
    // the same ones, and it would keep all of them in scalar registers across the whole step loop)
    int n0e = n0, n1e = n1, n2e = n2;
    asm volatile("" : "+s"(n0e), "+s"(n1e), "+s"(n2e));
#pragma unroll
    for (int c = 0; c < C; ++c)
        if (unit < n1e && c0 + c < n0e) p.W1[(size_t)unit * n0e + c0 + c] = w[c];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int u = 0; u < UG; ++u)
            if (wave + 8 * kk < n2e && lane + 64 * u < n1e) p.W2[(wave + 8 * kk) * n1e + lane + 64 * u] = w2r[kk][u];
    if (seg == 0 && hid) p.b1[unit] = b1;
    if (wave == 0 && outl) p.b2[lane] = b2;
    if (threadIdx.x == 0) *p.loss_acc += loss_sum;
}

template <int UG>
void solo_launch_c(const SoloPlan &plan, int C, hipStream_t stream)
{
    switch (C) {
    case 32: hipLaunchKernelGGL((solo_epoch_kernel<UG, 32>), dim3(1), dim3(SOLO_THREADS), 0, stream, plan); break;
    case 64: hipLaunchKernelGGL((solo_epoch_kernel<UG, 64>), dim3(1), dim3(SOLO_THREADS), 0, stream, plan); break;
    case 128: hipLaunchKernelGGL((solo_epoch_kernel<UG, 128>), dim3(1), dim3(SOLO_THREADS), 0, stream, plan); break;
    default: hipLaunchKernelGGL((solo_epoch_kernel<UG, 196>), dim3(1), dim3(SOLO_THREADS), 0, stream, plan); break;
    }
}

}  // namespace

// ---- host side -------------------------------------------------------------------

bool solo_geometry(const int32_t *n, int L, SoloGeom &g)
{
    g = SoloGeom{};
    if (L != 2 || n[0] < 1 || n[1] < 1 || n[2] < 1 || n[1] > 256 || n[2] > SOLO_MAX_OUT) return false;
    g.ug = n[1] <= 64 ? 1 : (n[1] <= 128 ? 2 : 4);
    const int segs = 8 / g.ug;
    const int need = (n[0] + segs - 1) / segs;
    static const int kC[] = {32, 64, 128, 196};
    g.c = 0;
    for (int c : kC)
        if (c >= need) { g.c = c; break; }
    if (!g.c) return false;
    // a step reads segs * c floats from its row's start: the last tail_steps steps would read past the array
    const int over = segs * g.c - n[0];
    g.tail_steps = (over + n[0] - 1) / n[0];
    return true;
}

hipError_t launch_solo_epoch(const SoloGeom &g, const SoloPlan &plan, hipStream_t stream)
{
    if (plan.n_samples < 1) return hipErrorInvalidValue;
    switch (g.ug) {
    case 1: solo_launch_c<1>(plan, g.c, stream); break;
    case 2: solo_launch_c<2>(plan, g.c, stream); break;
    case 4: solo_launch_c<4>(plan, g.c, stream); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace dn
