// Pieces shared by the persistent epoch kernels (dn_online.hip, dn_twin.hip): the stamped exchange
// words and their bounded polls, activation functions, and the row-block matrix-vector product.
// Every definition is local to the translation unit that includes this header.
#pragma once

#include "dn_internal.h"
#include "dn_wave.h"

namespace dn {
namespace {

typedef unsigned long long u64;
typedef float v4f __attribute__((ext_vector_type(4)));

// Threads per workgroup: ON_THREADS unless the including file sets DN_PERSIST_THREADS first (a
// kernel that wants fewer, fatter threads: half the threads may hold twice the registers each).
#ifdef DN_PERSIST_THREADS
constexpr int kThreads = DN_PERSIST_THREADS;
#else
constexpr int kThreads = ON_THREADS;
#endif
constexpr int kWaves = kThreads / 64;
constexpr int kSpinLimit = 1 << 21;   // polls of ~0.5 us each: about a second
constexpr int kPollBatch = 4;         // words each thread keeps in flight while polling (eight measured no faster)
constexpr int kTmp = ON_TMP_FLOATS;

enum UpdMode : int { UPD_SGD = 0, UPD_KEEPV = 1, UPD_MOMENTUM = 2 };

__device__ __forceinline__ void ll_store(u64 *p, float v, uint32_t seq)
{
    const u64 word = ((u64)seq << 32) | (u64)__float_as_uint(v);
    __hip_atomic_store(p, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ u64 ll_load(const u64 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float act_fn(int act, float z)
{
    switch (act) {
    case DN_ACT_SIGMOID: return 1.0f / (1.0f + expf(-z));
    case DN_ACT_TANH: return tanhf(z);
    case DN_ACT_RELU: return z > 0.0f ? z : 0.0f;
    default: return z;
    }
}

__device__ __forceinline__ float act_deriv(int act, float a)
{
    switch (act) {
    case DN_ACT_SIGMOID: return a * (1.0f - a);
    case DN_ACT_TANH: return 1.0f - a * a;
    case DN_ACT_RELU: return a > 0.0f ? 1.0f : 0.0f;
    default: return 1.0f;
    }
}

// dW = mu dW - g ; w += dW, with g already scaled by the learning rate.
__device__ __forceinline__ float apply_update(float w, float g, float &v, float mu, int mode)
{
    if (mode == UPD_SGD) return w - g;
    v = (mode == UPD_MOMENTUM) ? mu * v - g : -g;
    return w + v;
}

// Polls `total` exchange words; word q lives at addr(q) and its value goes to sink(q, value).
// Each thread keeps kPollBatch loads in flight and re-reads only the words that are not
// yet stamped with `seq`.  On a timeout (or when another workgroup has already given up)
// *s_abort is set; the caller tests it after its next barrier.
template <class Addr, class Sink>
__device__ __forceinline__ void poll_words(int total, uint32_t seq, Addr addr, Sink sink, int *abort_flag,
                                           volatile int *s_abort)
{
    for (int q0 = threadIdx.x; q0 < total; q0 += kThreads * kPollBatch) {
        u64 v[kPollBatch];
        bool ok[kPollBatch];
#pragma unroll
        for (int u = 0; u < kPollBatch; ++u) {
            const int q = q0 + u * kThreads;
            v[u] = 0;
            if (q < total) v[u] = ll_load(addr(q));
        }
        bool all = true;
#pragma unroll
        for (int u = 0; u < kPollBatch; ++u) {
            ok[u] = (q0 + u * kThreads >= total) || (uint32_t)(v[u] >> 32) == seq;
            all = all && ok[u];
        }
        int spins = 0;
        while (!all) {
            all = true;
#pragma unroll
            for (int u = 0; u < kPollBatch; ++u) {
                if (!ok[u]) {
                    v[u] = ll_load(addr(q0 + u * kThreads));
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
            const int q = q0 + u * kThreads;
            if (q < total) sink(q, __uint_as_float((uint32_t)v[u]));
        }
    }
}

// Forward of a block of rows (Wt = first row of the block, in LDS or device memory):
// kpart[r * kf + ks] = sum over segment ks of Wt[r][k] xin[k].
// One wave per (row, segment), kf = 2^kshift segments per row; a wave works on RU of them at a
// time so that their loads are in flight together.  Loads are unconditional (clamped addresses, masked values).
template <int VEC, int RU>
__device__ __forceinline__ void fwd_rows(const float *__restrict__ Wt, int n_in, int nr, int kshift, int seg,
                                         const float *xin, float *kpart)
{
    const int kf = 1 << kshift;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int items = nr * kf;
    for (int it0 = wave; it0 < items; it0 += kWaves * RU) {
        float acc[RU];
        const float *wp[RU];
        int kbeg[RU], kend[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int it = it0 + u * kWaves;
            const bool on = it < items;
            const int r = on ? it >> kshift : 0;
            const int ks = on ? it & (kf - 1) : 0;
            kbeg[u] = ks * seg;
            kend[u] = on ? min(n_in, kbeg[u] + seg) : 0;
            wp[u] = Wt + (size_t)r * n_in;
            acc[u] = 0.f;
        }
        for (int kk = lane * VEC; kk < seg; kk += 64 * VEC) {
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int k = kbeg[u] + kk;
                const bool in = k < kend[u];
                const int kc = in ? k : 0;
                if (VEC == 4) {
                    const v4f wv = *(const v4f *)(wp[u] + kc);
                    const v4f xv = *(const v4f *)(xin + kc);
                    const float d = wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
                    acc[u] += in ? d : 0.f;
                } else {
                    const float d = wp[u][kc] * xin[kc];
                    acc[u] += in ? d : 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const float s = wave_sum(acc[u]);
            const int it = it0 + u * kWaves;
            if (lane == 0 && it < items) kpart[it] = s;
        }
    }
}

// Copies between a block of device memory rows and its LDS image (count floats, contiguous).
__device__ __forceinline__ void copy_floats(float *dst, const float *src, int count)
{
    for (int i = threadIdx.x; i < count; i += kThreads) dst[i] = src[i];
}

}  // namespace

// The persistent kernels' workgroups wait for one another, so all of them must be on the device at
// once.  That holds for an ordinary launch when the grid is no larger than what the device can hold
// of this kernel at this LDS size (checked here from the occupancy query: workgroups per compute
// unit x compute units) and nothing else occupies the compute units for long; work queued earlier on
// the same stream has finished by the time the kernel starts.  Should a workgroup be kept waiting
// anyway (other long-running work of the process on another stream), the bounded polls end the
// launch with the abort flag instead of hanging.  (A cooperative launch gives the same residency
// through a separate device queue; that queue's teardown crashed at process exit under the
// profiler, and its only service here -- refusing grids that cannot be resident -- is this check.)
template <class Kernel, class Plan>
static hipError_t launch_resident(Kernel kernel, const Plan &plan, int grid, size_t lds_bytes, hipStream_t stream)
{
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kernel), kThreads, lds_bytes);
    if (e != hipSuccess) return e;
    if (grid < 1 || per_cu < 1 || (long)grid > (long)per_cu * cus) return hipErrorCooperativeLaunchTooLarge;
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(kThreads), lds_bytes, stream, plan);
    return hipGetLastError();
}

}  // namespace dn
