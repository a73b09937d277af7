// fp32 MFMA contraction kernels for the three dense products of a training
// step (forward, delta propagation, weight gradient) with fused epilogues.
//
// One workgroup computes a BM x BN tile of C.  The k range is walked in steps
// of KT through double-buffered LDS tiles; waves are arranged WM x WN over the
// tile and, when WK > 1, additionally split each KT step among WK wave groups
// whose partial tiles are summed through LDS before the epilogue (this keeps
// every CU busy when the output has few tiles, e.g. batch x width products).
// Each wave owns TM x TN accumulator blocks of v_mfma_f32_32x32x2_f32.
//
// Lane layout of v_mfma_f32_32x32x2_f32 (64 lanes, lane = 32*h + i):
//   A operand: row i of the 32-row block, k index h of the pair
//   B operand: column i of the 32-column block, k index h of the pair
//   D, register r in 0..15: row 8*(r/4) + 4*h + (r%4), column i
// The sum over k is order-free, so a group of eight k values is fed as four
// instructions pairing k = j (h = 0) with k = 4 + j (h = 1): a lane then needs
// four consecutive k values of its row, one 128-bit LDS read when the tile is
// stored k-contiguous.
#include "dn_internal.h"

namespace dn {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float act_fn(int act, float z)
{
    switch (act) {
    case DN_ACT_SIGMOID: return 1.0f / (1.0f + expf(-z));
    case DN_ACT_TANH: return tanhf(z);
    case DN_ACT_RELU: return z > 0.0f ? z : 0.0f;
    default: return z;  // linear; a softmax layer stores z and is normalised by the output kernel
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

template <int BM_, int BN_, int KT_, int WM_, int WN_, int WK_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, KT = KT_, WM = WM_, WN = WN_, WK = WK_;
    static constexpr int NT = 64 * WM * WN * WK;
    static constexpr int WTM = BM / WM, WTN = BN / WN;  // wave tile
    static constexpr int TM = WTM / 32, TN = WTN / 32;  // 32x32 blocks per wave
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32x32");
    static_assert(KT % (8 * WK) == 0, "KT must hold a group of eight k per k-split wave");
    static_assert((BM * KT / 4) % NT == 0 && (BN * KT / 4) % NT == 0, "tile loads must divide evenly");
};

// Row stride (floats) of an LDS tile: k-contiguous tiles are [rows][KT+4],
// m/n-contiguous tiles are [KT][rows+8]; both keep 16-byte alignment of float4
// accesses and spread the two lane halves over different banks.
template <bool KC, int ROWS, int KT>
struct Lds {
    static constexpr int STRIDE = KC ? KT + 4 : ROWS + 8;
    static constexpr int FLOATS = KC ? ROWS * STRIDE : KT * STRIDE;
};

// Global -> register load of one operand tile (ROWS x KT), zero-filled outside
// the matrix.  KC: rows of the matrix are rows of the tile, contiguous in k.
// MC: rows of the stored matrix are k, contiguous along the tile's rows.
template <bool KC, int ROWS, int KT, int NT>
__device__ __forceinline__ void load_tile(v4f (&reg)[ROWS * KT / 4 / NT], const float *__restrict__ P,
                                          int ld, int r0, int k0, int R, int K, bool vec_ok, int tid)
{
    constexpr int N = ROWS * KT / 4 / NT;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int f = tid + i * NT;
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (KC) {
            const int r = f / (KT / 4), c = (f % (KT / 4)) * 4;
            const int gr = r0 + r, gk = k0 + c;
            if (gr < R) {
                const float *src = P + (size_t)gr * ld + gk;
                if (vec_ok && gk + 3 < K) {
                    v = *reinterpret_cast<const v4f *>(src);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (gk + j < K) v[j] = src[j];
                }
            }
        } else {
            const int k = f / (ROWS / 4), c = (f % (ROWS / 4)) * 4;
            const int gk = k0 + k, gr = r0 + c;
            if (gk < K) {
                const float *src = P + (size_t)gk * ld + gr;
                if (vec_ok && gr + 3 < R) {
                    v = *reinterpret_cast<const v4f *>(src);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (gr + j < R) v[j] = src[j];
                }
            }
        }
        reg[i] = v;
    }
}

template <bool KC, int ROWS, int KT, int NT>
__device__ __forceinline__ void store_tile(float *__restrict__ S, const v4f (&reg)[ROWS * KT / 4 / NT], int tid)
{
    constexpr int N = ROWS * KT / 4 / NT;
    constexpr int STRIDE = Lds<KC, ROWS, KT>::STRIDE;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int f = tid + i * NT;
        int off;
        if (KC) {
            const int r = f / (KT / 4), c = (f % (KT / 4)) * 4;
            off = r * STRIDE + c;
        } else {
            const int k = f / (ROWS / 4), c = (f % (ROWS / 4)) * 4;
            off = k * STRIDE + c;
        }
        *reinterpret_cast<v4f *>(S + off) = reg[i];
    }
}

// Fetch the four k values (group kk, lane half h) of tile row `row`.
template <bool KC, int ROWS, int KT>
__device__ __forceinline__ v4f fetch_frag(const float *__restrict__ S, int row, int kk, int h)
{
    constexpr int STRIDE = Lds<KC, ROWS, KT>::STRIDE;
    if (KC) {
        return *reinterpret_cast<const v4f *>(S + row * STRIDE + kk * 8 + h * 4);
    } else {
        v4f v;
        const float *p = S + (kk * 8 + h * 4) * STRIDE + row;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = p[j * STRIDE];
        return v;
    }
}

template <class T, bool A_KC, bool B_KC, int KIND>
__global__ __launch_bounds__(T::NT) void gemm_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    constexpr int BM = T::BM, BN = T::BN, KT = T::KT, NT = T::NT;
    constexpr int TM = T::TM, TN = T::TN, WK = T::WK;
    using LA = Lds<A_KC, BM, KT>;
    using LB = Lds<B_KC, BN, KT>;
    constexpr int STAGE = LA::FLOATS + LB::FLOATS;
    constexpr int RED = (WK > 1) ? (WK / 2) * BM * BN : 0;
    constexpr int SMEM = (2 * STAGE > RED) ? 2 * STAGE : RED;
    __shared__ __attribute__((aligned(16))) float smem[SMEM];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // run of tiles (m fastest) so tiles sharing a B panel meet in one L2.
    const int nt = tiles_m * tiles_n;
    const int per_xcd = (nt + 7) / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (v >= nt) return;
    const int m0 = (v % tiles_m) * BM, n0 = (v / tiles_m) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int idx = lane & 31, h = lane >> 5;
    const int wk = wave / (T::WM * T::WN);
    const int wm = (wave % (T::WM * T::WN)) / T::WN, wn = wave % T::WN;

    const bool a_vec = (g.lda % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.A) & 15) == 0);
    const bool b_vec = (g.ldb % 4 == 0) && ((reinterpret_cast<uintptr_t>(g.B) & 15) == 0);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    v4f ra[BM * KT / 4 / NT], rb[BN * KT / 4 / NT];
    const int nk = (g.K + KT - 1) / KT;

    load_tile<A_KC, BM, KT, NT>(ra, g.A, g.lda, m0, 0, g.M, g.K, a_vec, tid);
    load_tile<B_KC, BN, KT, NT>(rb, g.B, g.ldb, n0, 0, g.N, g.K, b_vec, tid);
    store_tile<A_KC, BM, KT, NT>(smem, ra, tid);
    store_tile<B_KC, BN, KT, NT>(smem + LA::FLOATS, rb, tid);
    __syncthreads();

    for (int t = 0; t < nk; ++t) {
        const float *As = smem + (t & 1) * STAGE;
        const float *Bs = As + LA::FLOATS;
        if (t + 1 < nk) {
            load_tile<A_KC, BM, KT, NT>(ra, g.A, g.lda, m0, (t + 1) * KT, g.M, g.K, a_vec, tid);
            load_tile<B_KC, BN, KT, NT>(rb, g.B, g.ldb, n0, (t + 1) * KT, g.N, g.K, b_vec, tid);
        }
#pragma unroll
        for (int kk = 0; kk < KT / 8; kk += WK) {
            v4f fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = fetch_frag<A_KC, BM, KT>(As, wm * T::WTM + i * 32 + idx, kk + wk, h);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = fetch_frag<B_KC, BN, KT>(Bs, wn * T::WTN + j * 32 + idx, kk + wk, h);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][q], fb[j][q], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < nk) {
            float *An = smem + ((t + 1) & 1) * STAGE;
            store_tile<A_KC, BM, KT, NT>(An, ra, tid);
            store_tile<B_KC, BN, KT, NT>(An + LA::FLOATS, rb, tid);
        }
        __syncthreads();
    }

    // Sum the k-split partial tiles (tree over wk, through LDS).
    if (WK > 1) {
        const int wpos = wm * T::WN + wn;
#pragma unroll
        for (int s = WK / 2; s >= 1; s /= 2) {
            if (wk >= s && wk < 2 * s) {
                float *dst = smem + ((size_t)((wk - s) * T::WM * T::WN + wpos) * TM * TN) * 1024;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) dst[((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
            }
            __syncthreads();
            if (wk < s) {
                const float *src = smem + ((size_t)(wk * T::WM * T::WN + wpos) * TM * TN) * 1024;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[i][j][r] += src[((i * TN + j) * 16 + r) * 64 + lane];
            }
            __syncthreads();
        }
        if (wk != 0) return;
    }

    // Epilogue.  Lanes of one register cover 32 consecutive columns of one row.
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * T::WTN + j * 32 + idx;
            if (col >= g.N) continue;
            float bias = 0.f;
            if (KIND == GEMM_FWD) bias = g.bias[col];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (row >= g.M) continue;
                const size_t o = (size_t)row * g.ldc + col;
                const float s = acc[i][j][r];
                if (KIND == GEMM_FWD) {
                    g.C[o] = act_fn(g.act, s + bias);
                } else if (KIND == GEMM_DELTA) {
                    g.C[o] = s * act_deriv(g.act, g.aux[o]);
                } else {
                    if (g.mode == GRAD_STORE) {
                        g.C[o] = s * g.scale;
                    } else if (g.mode == GRAD_SGD) {
                        g.C[o] = g.C[o] + (-g.scale * s);
                    } else if (g.mode == GRAD_SGD_KEEPV) {
                        const float dw = -g.scale * s;
                        g.V[o] = dw;
                        g.C[o] = g.C[o] + dw;
                    } else {
                        const float dw = g.mu * g.V[o] - g.scale * s;
                        g.V[o] = dw;
                        g.C[o] = g.C[o] + dw;
                    }
                }
            }
        }
    }
}

// ---- tile configurations and dispatch ----------------------------------------
using T128 = Tile<128, 128, 16, 2, 2, 1>;   // many-tile outputs (weight gradients, large batches)
using T64K4 = Tile<64, 64, 32, 1, 1, 4>;    // few-tile outputs: batch x width with batch <= a few hundred
using T32K4 = Tile<32, 64, 32, 1, 1, 4>;    // very small batches

static const char *kVariantNames[] = {"128x128x16_w2x2", "64x64x32_k4", "32x64x32_k4"};
int gemm_variant_count() { return 3; }
const char *gemm_variant_name(int v) { return (v >= 0 && v < 3) ? kVariantNames[v] : "?"; }

template <class T, bool A_KC, bool B_KC, int KIND>
static hipError_t launch_one(const GemmArgs &a, hipStream_t stream)
{
    const int tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const long nt = (long)tiles_m * tiles_n;
    const long grid = 8 * ((nt + 7) / 8);
    if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_kernel<T, A_KC, B_KC, KIND>), dim3((unsigned)grid), dim3(T::NT), 0, stream, a,
                       tiles_m, tiles_n);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_kind(GemmKind kind, const GemmArgs &a, hipStream_t stream)
{
    switch (kind) {
    case GEMM_FWD: return launch_one<T, true, true, GEMM_FWD>(a, stream);
    case GEMM_DELTA: return launch_one<T, true, false, GEMM_DELTA>(a, stream);
    case GEMM_GRAD: return launch_one<T, false, false, GEMM_GRAD>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

static int pick_variant(const GemmArgs &a)
{
    const long t128 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (t128 >= 192) return 0;
    if (a.M <= 32) return 2;
    return 1;
}

hipError_t launch_gemm(GemmKind kind, const GemmArgs &a, int variant, hipStream_t stream)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (variant < 0) variant = pick_variant(a);
    switch (variant) {
    case 0: return launch_kind<T128>(kind, a, stream);
    case 1: return launch_kind<T64K4>(kind, a, stream);
    case 2: return launch_kind<T32K4>(kind, a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace dn
