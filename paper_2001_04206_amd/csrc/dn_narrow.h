// Weight gradient / update of a layer with at most 16 outputs on the vector units: the work of one
// workgroup as a device function, so that it can run as a kernel of its own (dn_small.hip) or in
// extra workgroups of a matrix-core launch that does not depend on it (dn_gemm.hip).
#pragma once
#include "dn_internal.h"
#include "dn_wave.h"

namespace dn {

constexpr int kNarrow = 16;

// acc[o][j] = sum_b Delta_l[b][o] A_{l-1}[b][j] for n_l <= 16, then the same fused store / update
// as the matrix-core gradient product.  The output is small (n_l x n_{l-1}) and the sum runs over
// the batch, so the parallelism is taken from both: a workgroup owns VEC adjacent columns j, its
// 256 threads take the rows b, b + 256, ... and the threads' partial sums are added in a fixed
// order (lane butterfly, then the four waves).  A_{l-1} is read in 16-byte pieces, one row per
// lane; it is small enough to come from the L2 for all but the first reader of a line.  One
// extra workgroup (the last) does the bias: column sums of Delta_l.
struct NarrowGradArgs {
    const float *D, *Aprev;
    float *C, *V, *gb, *vb;
    int B, nl, nin, mode;
    float scale, mu;
};

__device__ __forceinline__ void narrow_apply(int mode, float scale, float mu, float sum, float *c, float *v)
{
    if (mode == GRAD_STORE) {
        *c = sum * scale;
    } else if (mode == GRAD_SGD) {
        *c = *c + (-scale * sum);
    } else if (mode == GRAD_SGD_KEEPV) {
        const float dw = -scale * sum;
        *v = dw;
        *c = *c + dw;
    } else {
        const float dw = mu * *v - scale * sum;
        *v = dw;
        *c = *c + dw;
    }
}

// Work of workgroup `block` of `nblocks` (256 threads): blocks 0 .. nblocks-2 own VEC adjacent
// columns each, the last one sums Delta_l's columns for the bias.
template <int VEC>
__device__ __forceinline__ void narrow_grad_block(const NarrowGradArgs &g, int block, int nblocks)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    __shared__ float red[4][kNarrow * VEC];   // per wave: [o][column]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (block == nblocks - 1) {
        // bias: the same sum with 1 in the place of A_{l-1}
        float part[kNarrow];
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) part[o] = 0.f;
        for (int b = tid; b < g.B; b += 256) {
            const float *d = g.D + (size_t)b * g.nl;
#pragma unroll
            for (int o = 0; o < kNarrow; ++o)
                if (o < g.nl) part[o] += d[o];
        }
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            const float total = wave_sum(part[o]);
            if (lane == 0) red[wave][o] = total;
        }
        __syncthreads();
        if (tid < g.nl) {
            const float sum = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
            narrow_apply(g.mode, g.scale, g.mu, sum, g.gb + tid, g.vb + tid);
        }
        return;
    }
    const int j = block * VEC;   // one workgroup per column group
    float acc[kNarrow][VEC];
#pragma unroll
    for (int o = 0; o < kNarrow; ++o)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[o][v] = 0.f;
    for (int b = tid; b < g.B; b += 256) {
        const vec_t a = *reinterpret_cast<const vec_t *>(g.Aprev + (size_t)b * g.nin + j);
        const float *d = g.D + (size_t)b * g.nl;
#pragma unroll
        for (int o = 0; o < kNarrow; ++o) {
            if (o < g.nl) {
                const float dv = d[o];
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[o][v] = fmaf(dv, a[v], acc[o][v]);
            }
        }
    }
#pragma unroll
    for (int o = 0; o < kNarrow; ++o)
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float total = wave_sum(acc[o][v]);
            if (lane == 0) red[wave][o * VEC + v] = total;
        }
    __syncthreads();
    if (tid < g.nl * VEC) {
        const int o = tid / VEC, v = tid % VEC;
        const float sum = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        const size_t at = (size_t)o * g.nin + j + v;
        narrow_apply(g.mode, g.scale, g.mu, sum, g.C + at, g.V + at);
    }
}


}  // namespace dn
