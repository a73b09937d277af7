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
#include <atomic>
#include <type_traits>

#include "dn_internal.h"
#include "dn_narrow.h"
#include "dn_wave.h"

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

template <int BM_, int BN_, int KT_, int WM_, int WN_, int WK_, int R_, int PC_ = 0, int OCC_ = 1, bool PV_ = true>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, KT = KT_, WM = WM_, WN = WN_, WK = WK_, R = R_;
    static constexpr int PC = PC_;    // peeled k steps that carry the epilogue-operand prefetch (update kernels)
    static constexpr int OCC = OCC_;  // waves per SIMD the register budget must allow
    static constexpr bool PV = PV_;   // momentum update: prefetch the velocity too (else read it in the epilogue)
    static_assert(R >= 1 && R <= 4, "register stages");
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

// Operand tiles travel global -> registers -> LDS.  KC: rows of the matrix are
// rows of the tile, contiguous in k.  MC: rows of the stored matrix are k,
// contiguous along the tile's own index.
//
// load_tile only issues loads: the address is clamped into the matrix so that
// no branch and no use of the loaded value follows, and all loads of a tile
// (and of the tiles behind it) stay in flight while the matrix cores work.
// store_tile, called one or more k-steps later, replaces elements that lie
// outside the matrix by zero and writes the tile to LDS.
// VEC (chosen on the host, a separate instantiation so the fast path is straight-line
// code) means that for both operands the contiguous extent and the leading dimension
// are multiples of 4 and the base is 16-byte aligned; otherwise elements are loaded singly.
template <bool KC, int ROWS, int KT>
__device__ __forceinline__ void tile_coords(int f, int j, int r0, int k0, int &gr, int &gk)
{
    if (KC) {
        gr = r0 + f / (KT / 4);
        gk = k0 + (f % (KT / 4)) * 4 + j;
    } else {
        gk = k0 + f / (ROWS / 4);
        gr = r0 + (f % (ROWS / 4)) * 4 + j;
    }
}

template <bool KC, int ROWS, int KT, int NT, bool VEC>
__device__ __forceinline__ void load_tile(v4f (&reg)[ROWS * KT / 4 / NT], const float *__restrict__ P,
                                          int ld, int r0, int k0, int R, int K, int tid)
{
    constexpr int N = ROWS * KT / 4 / NT;
    if (VEC) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            int gr, gk;
            tile_coords<KC, ROWS, KT>(tid + i * NT, 0, r0, k0, gr, gk);
            const bool ok = gr < R && gk < K;
            const int cr = ok ? gr : 0, ck = ok ? gk : 0;
            const float *src = KC ? P + (size_t)cr * ld + ck : P + (size_t)ck * ld + cr;
            reg[i] = *reinterpret_cast<const v4f *>(src);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int gr, gk;
                tile_coords<KC, ROWS, KT>(tid + i * NT, j, r0, k0, gr, gk);
                const bool ok = gr < R && gk < K;
                const int cr = ok ? gr : 0, ck = ok ? gk : 0;
                reg[i][j] = KC ? P[(size_t)cr * ld + ck] : P[(size_t)ck * ld + cr];
            }
        }
    }
}

template <bool KC, int ROWS, int KT, int NT>
__device__ __forceinline__ void store_tile(float *__restrict__ S, const v4f (&reg)[ROWS * KT / 4 / NT], int r0,
                                           int k0, int R, int K, int tid)
{
    constexpr int N = ROWS * KT / 4 / NT;
    constexpr int STRIDE = Lds<KC, ROWS, KT>::STRIDE;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int f = tid + i * NT;
        v4f v = reg[i];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int gr, gk;
            tile_coords<KC, ROWS, KT>(f, j, r0, k0, gr, gk);
            v[j] = (gr < R && gk < K) ? v[j] : 0.f;
        }
        const int off = KC ? (f / (KT / 4)) * STRIDE + (f % (KT / 4)) * 4 : (f / (ROWS / 4)) * STRIDE + (f % (ROWS / 4)) * 4;
        *reinterpret_cast<v4f *>(S + off) = v;
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

// Epilogue selector of the kernel template.
enum Epi : int { EPI_FWD = 0, EPI_DELTA = 1, EPI_GRAD_STORE = 2, EPI_GRAD_SGD = 3, EPI_GRAD_SGD_KEEPV = 4, EPI_GRAD_MOMENTUM = 5 };

// One element of the fused epilogue.  `pre_w` / `pre_v` are the values of the in-place
// operands (W and velocity for the update modes, A_{l-1} for DELTA) that were fetched
// before the k loop so their latency hides behind the contraction.
template <int EPI>
__device__ __forceinline__ void epilogue_store(const GemmArgs &g, size_t o, float s, float bias, float pre_w, float pre_v)
{
    if (EPI == EPI_FWD) {
        g.C[o] = act_fn(g.act, s + bias);
    } else if (EPI == EPI_DELTA) {
        g.C[o] = s * act_deriv(g.act, pre_w);
    } else if (EPI == EPI_GRAD_STORE) {
        g.C[o] = s * g.scale;
    } else if (EPI == EPI_GRAD_SGD) {
        g.C[o] = pre_w + (-g.scale * s);
    } else if (EPI == EPI_GRAD_SGD_KEEPV) {
        const float dw = -g.scale * s;
        g.V[o] = dw;
        g.C[o] = pre_w + dw;
    } else {
        const float dw = g.mu * pre_v - g.scale * s;
        g.V[o] = dw;
        g.C[o] = pre_w + dw;
    }
}

// Interior-tile variants of the tile movers: the tile lies wholly inside the matrix in its
// own index and in k, so addresses are one wave-uniform base plus a per-lane offset that
// never changes (no address arithmetic, no clamps, no masks inside the k loop).
template <bool KC, int ROWS, int KT, int NT>
__device__ __forceinline__ void lane_offsets(unsigned (&off)[ROWS * KT / 4 / NT], int ld, int tid)
{
#pragma unroll
    for (int i = 0; i < ROWS * KT / 4 / NT; ++i) {
        const int f = tid + i * NT;
        off[i] = KC ? (unsigned)(f / (KT / 4)) * (unsigned)ld + (unsigned)(f % (KT / 4)) * 4u
                    : (unsigned)(f / (ROWS / 4)) * (unsigned)ld + (unsigned)(f % (ROWS / 4)) * 4u;
    }
}

template <int N>
__device__ __forceinline__ void load_tile_fast(v4f (&reg)[N], const float *__restrict__ base, const unsigned (&off)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i) reg[i] = *reinterpret_cast<const v4f *>(base + off[i]);
}

template <bool KC, int ROWS, int KT, int NT>
__device__ __forceinline__ void store_tile_fast(float *__restrict__ S, const v4f (&reg)[ROWS * KT / 4 / NT], int tid)
{
    constexpr int STRIDE = Lds<KC, ROWS, KT>::STRIDE;
#pragma unroll
    for (int i = 0; i < ROWS * KT / 4 / NT; ++i) {
        const int f = tid + i * NT;
        const int off = KC ? (f / (KT / 4)) * STRIDE + (f % (KT / 4)) * 4 : (f / (ROWS / 4)) * STRIDE + (f % (ROWS / 4)) * 4;
        *reinterpret_cast<v4f *>(S + off) = reg[i];
    }
}

// Emits the requested instruction order of one k step for the machine scheduler: FILL times
// (BASE matrix instructions, then one LDS read while I < NRD, else one LDS write).
template <int I, int FILL, int NRD, int BASE>
struct SchedPattern {
    static __device__ __forceinline__ void emit()
    {
        __builtin_amdgcn_sched_group_barrier(0x008, BASE, 0);
        __builtin_amdgcn_sched_group_barrier(I < NRD ? 0x100 : 0x200, 1, 0);
        SchedPattern<I + 1, FILL, NRD, BASE>::emit();
    }
};
template <int FILL, int NRD, int BASE>
struct SchedPattern<FILL, FILL, NRD, BASE> {
    static __device__ __forceinline__ void emit() {}
};

// Work of one workgroup on the tile at (m0, n0).  FAST: the tile is interior in m and n and
// both operands are vector-loadable; only a ragged last k step takes the clamped path.
template <class T, bool A_KC, bool B_KC, int EPI, bool VEC, bool FAST>
__device__ __forceinline__ void gemm_tile(const GemmArgs &g0, float *smem, const int m0, const int n0, const int tile_id,
                                          const int split)
{
    // k split across workgroups: this one contracts k steps [split * per, (split + 1) * per) of the
    // KT-step sequence, i.e. the same product on operands advanced along k and a shorter K.
    GemmArgs g = g0;
    if (g0.sk > 1) {
        const int per = (((g0.K + T::KT - 1) / T::KT) + g0.sk - 1) / g0.sk * T::KT;
        const int kb = split * per;
        g.A = A_KC ? g0.A + kb : g0.A + (size_t)kb * g0.lda;
        g.B = B_KC ? g0.B + kb : g0.B + (size_t)kb * g0.ldb;
        g.K = min(per, g0.K - kb);
    }
    constexpr int BM = T::BM, BN = T::BN, KT = T::KT, NT = T::NT, R = T::R;
    constexpr int TM = T::TM, TN = T::TN, WK = T::WK;
    constexpr bool IS_GRAD = EPI >= EPI_GRAD_STORE;
    constexpr bool PRE_W = EPI == EPI_DELTA || EPI >= EPI_GRAD_SGD;
    constexpr bool PRE_V = EPI == EPI_GRAD_MOMENTUM && T::PV;
    using LA = Lds<A_KC, BM, KT>;
    using LB = Lds<B_KC, BN, KT>;
    constexpr int STAGE = LA::FLOATS + LB::FLOATS;
    static_assert(!IS_GRAD || NT >= BM, "bias reduction needs one thread per tile row");
    static_assert(!IS_GRAD || WK * BM <= 2 * (Lds<A_KC, BM, KT>::FLOATS + Lds<B_KC, BN, KT>::FLOATS), "bias scratch must fit the tile buffers");
    static_assert(VEC || !FAST, "the interior path needs vector loads");
    constexpr int NA = BM * KT / 4 / NT, NB = BN * KT / 4 / NT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int idx = lane & 31, h = lane >> 5;
    const int wk = wave / (T::WM * T::WN);
    const int wm = (wave % (T::WM * T::WN)) / T::WN, wn = wave % T::WN;

    const int nk = (g.K + KT - 1) / KT;

    // R register stages keep R operand tiles in flight.  Every load below is issued
    // unconditionally (tiles past the end of k are clamped loads that store_tile turns into
    // zeros) so that the order of outstanding loads is the same on every path and the
    // wait before each LDS store covers exactly the stage being stored, nothing younger.
    v4f ra[R][NA], rb[R][NB];
    unsigned offa[FAST ? NA : 1], offb[FAST ? NB : 1];
    const float *tile_a = nullptr, *tile_b = nullptr;  // FAST: first element of the tile's k = 0 column / row
    size_t kstep_a = 0, kstep_b = 0;                    // FAST: elements from one k step to the next
    if (FAST) {
        lane_offsets<A_KC, BM, KT, NT>(reinterpret_cast<unsigned (&)[NA]>(offa), g.lda, tid);
        lane_offsets<B_KC, BN, KT, NT>(reinterpret_cast<unsigned (&)[NB]>(offb), g.ldb, tid);
        tile_a = A_KC ? g.A + (size_t)m0 * g.lda : g.A + m0;
        tile_b = B_KC ? g.B + (size_t)n0 * g.ldb : g.B + n0;
        kstep_a = A_KC ? (size_t)KT : (size_t)KT * g.lda;
        kstep_b = B_KC ? (size_t)KT : (size_t)KT * g.ldb;
    }
    // load / store of k step t into / from register stage s; `full` (compile time) promises
    // that the step lies wholly inside k, so the interior path needs neither clamps nor masks
    auto load_step = [&](auto full, int s, int t) {
        if (FAST && decltype(full)::value) {
            load_tile_fast<NA>(ra[s], tile_a + (size_t)t * kstep_a, reinterpret_cast<const unsigned (&)[NA]>(offa));
            load_tile_fast<NB>(rb[s], tile_b + (size_t)t * kstep_b, reinterpret_cast<const unsigned (&)[NB]>(offb));
        } else {
            load_tile<A_KC, BM, KT, NT, VEC>(ra[s], g.A, g.lda, m0, t * KT, g.M, g.K, tid);
            load_tile<B_KC, BN, KT, NT, VEC>(rb[s], g.B, g.ldb, n0, t * KT, g.N, g.K, tid);
        }
    };
    auto store_step = [&](auto full, int s, int t, float *dst) {
        if (FAST && decltype(full)::value) {
            store_tile_fast<A_KC, BM, KT, NT>(dst, ra[s], tid);
            store_tile_fast<B_KC, BN, KT, NT>(dst + LA::FLOATS, rb[s], tid);
        } else {
            store_tile<A_KC, BM, KT, NT>(dst, ra[s], m0, t * KT, g.M, g.K, tid);
            store_tile<B_KC, BN, KT, NT>(dst + LA::FLOATS, rb[s], n0, t * KT, g.N, g.K, tid);
        }
    };
    using Full = std::integral_constant<bool, true>;
    using Ragged = std::integral_constant<bool, false>;
#pragma unroll
    for (int s = 0; s < R; ++s) load_step(Ragged{}, s, s);

    // In-place operands of the epilogue (W and velocity for the update modes, A_{l-1} for DELTA)
    // are fetched while the k loop runs.  Loads return in issue order, so a burst of them issued
    // before an operand-tile load would stall the k loop until the whole burst is back.  With
    // PC > 0 the first PC k steps are peeled and each issues 1/PC of these loads *after* its own
    // operand-tile loads: no tile load ever queues behind more than one small chunk.  With
    // PC == 0 they are all issued up front (fine when they are few and L2-resident).
    // (All k-split wave groups fetch them; only group 0 uses them.)
    constexpr int PC = (IS_GRAD && PRE_W) ? T::PC : 0;
    constexpr int NPRE = TM * TN * 16;
    static_assert(PC == 0 || (PC % R == 0 && (NPRE * (PRE_V ? 2 : 1)) % PC == 0), "chunked prefetch must divide evenly");
    float pre_w[PRE_W ? TM : 1][PRE_W ? TN : 1][16], pre_v[PRE_V ? TM : 1][PRE_V ? TN : 1][16];
    const float *src_w = (EPI == EPI_DELTA) ? g.aux : g.C;
    auto pre_load = [&](int q) {  // q in [0, NPRE * (1 or 2)): element q of (pre_w, then pre_v)
        const int which = q / NPRE, e = q % NPRE;
        const int i = e / (TN * 16), j = (e / 16) % TN, r = e % 16;
        const int col = n0 + wn * T::WTN + j * 32 + idx;
        const int row = m0 + wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * h + (r % 4);
        const bool ok = FAST || (col < g.N && row < g.M);  // clamp instead of branching
        const size_t o = ok ? (size_t)row * g.ldc + col : 0;
        if (which == 0) pre_w[PRE_W ? i : 0][PRE_W ? j : 0][r] = src_w[o];
        else pre_v[PRE_V ? i : 0][PRE_V ? j : 0][r] = g.V[o];
    };
    if (PRE_W && PC == 0) {
#pragma unroll
        for (int q = 0; q < NPRE * (PRE_V ? 2 : 1); ++q) pre_load(q);
    }
    // FWD: the biases of this wave's columns, requested here for the same reason (measured: fetched in
    // the epilogue, that one cold load made the epilogue 2.5 us of a 9 us kernel)
    float bias_pre[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        bias_pre[j] = 0.f;
        if (EPI == EPI_FWD && WK == 1) {
            const int col = n0 + wn * T::WTN + j * 32 + idx;
            bias_pre[j] = g.bias[col < g.N ? col : 0];
        }
    }
    // ... and with k-split wave groups, where every thread finishes four adjacent columns (below):
    // those four biases (the thread's columns are the same in every pass: NT is a multiple of BN / 4)
    static_assert(NT % (BN / 4) == 0, "a thread's epilogue columns must not depend on the pass");
    const bool wide_out = EPI == EPI_FWD && WK > 1 && g.ldc % 4 == 0 &&
                          ((reinterpret_cast<uintptr_t>(g.C) | reinterpret_cast<uintptr_t>(g.bias)) & 15) == 0;
    v4f bias4 = {0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_FWD && WK > 1) {
        const int col = n0 + (tid % (BN / 4)) * 4;
        if (wide_out && col + 4 <= g.N) {
            bias4 = *reinterpret_cast<const v4f *>(g.bias + col);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) bias4[q] = g.bias[col + q < g.N ? col + q : 0];
        }
    }

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    // GRAD: the bias gradient is the column sum of Delta, i.e. the sum over k of this kernel's
    // A operand.  Waves of the first tile column that sit in wave column 0 add up the A
    // fragments they hold anyway (per lane: its row, its half of the k values).
    float bs[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) bs[i] = 0.f;
    const bool bias_wave = IS_GRAD && n0 == 0 && wn == 0;

    const float bias_on = bias_wave ? 1.f : 0.f;  // a factor, not a branch: each k step stays one basic block
    store_step(Ragged{}, 0, 0, smem);
    __syncthreads();

    // One k step: LDS buffer (t & 1) holds tile t; register stage s (stored one step ago) is
    // refilled with tile t + R; stage (s + 1) % R, holding tile t + 1, goes to the other buffer.
    // A wave cannot start a new matrix instruction while one is running (64 cycles each), but it
    // can issue LDS and memory instructions in that shadow: the LDS reads of later fragment groups
    // and the LDS writes of the next tile are therefore spread between the matrix instructions.
    constexpr int G = KT / 8 / WK;                 // fragment groups (8 k values each) per wave and step
    constexpr int NMF = G * 4 * TM * TN;           // matrix instructions per wave and step
    constexpr int NRD = (G - 1) * (TM * (A_KC ? 1 : 2) + TN * (B_KC ? 1 : 2));  // LDS reads of groups 1..G-1
    constexpr int NWR = NA + NB;                   // LDS writes of the next tile
    constexpr int FILL = NRD + NWR;
    constexpr int BASE = (NMF / (FILL + 1)) > 0 ? NMF / (FILL + 1) : 1;
    auto k_step = [&](auto full, int s, int t, int chunk) {
        const float *As = smem + (t & 1) * STAGE;
        const float *Bs = As + LA::FLOATS;
        v4f fa[G][TM], fb[G][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[0][i] = fetch_frag<A_KC, BM, KT>(As, wm * T::WTM + i * 32 + idx, wk, h);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[0][j] = fetch_frag<B_KC, BN, KT>(Bs, wn * T::WTN + j * 32 + idx, wk, h);
        load_step(full, s, t + R);
        if (PC > 0 && chunk >= 0) {
            constexpr int PER = NPRE * (PRE_V ? 2 : 1) / (PC > 0 ? PC : 1);
#pragma unroll
            for (int q = 0; q < PER; ++q) pre_load(chunk * PER + q);
        }
        // Keep the instruction scheduler from sinking the global loads into the matrix work
        // (the prefetch distance is the point).
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int gq = 1; gq < G; ++gq) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[gq][i] = fetch_frag<A_KC, BM, KT>(As, wm * T::WTM + i * 32 + idx, gq * WK + wk, h);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[gq][j] = fetch_frag<B_KC, BN, KT>(Bs, wn * T::WTN + j * 32 + idx, gq * WK + wk, h);
        }
#pragma unroll
        for (int gq = 0; gq < G; ++gq)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[gq][i][q], fb[gq][j][q], acc[i][j], 0, 0, 0);
        if (IS_GRAD) {
#pragma unroll
            for (int gq = 0; gq < G; ++gq)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    bs[i] += bias_on * ((fa[gq][i][0] + fa[gq][i][1]) + (fa[gq][i][2] + fa[gq][i][3]));
        }
        store_step(full, (s + 1) % R, t + 1, smem + ((t + 1) & 1) * STAGE);
        // requested order inside this region: BASE matrix instructions, one LDS read (while any
        // are left) or LDS write, and so on; then the remaining matrix instructions.
        SchedPattern<0, FILL, NRD, BASE>::emit();
        __builtin_amdgcn_sched_group_barrier(0x008, NMF - BASE * FILL > 0 ? NMF - BASE * FILL : 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
    };

    // A step t may take the mask-free form when the tile it stores (t + 1) and the tile it
    // loads (t + R) lie wholly inside k.  Peeled steps carry the chunked prefetch; then full
    // steps run in groups of R while they last; the rest (ragged tail, steps that load or store
    // past the end, and a last partial group working on zero tiles) take the masked form.
    const int nfull = g.K / KT;  // k steps 0 .. nfull-1 are wholly inside k
    int t0 = 0;
    if (PC > 0) {
        // (short contractions -- k = 128 has eight steps -- still get the mask-free form for the
        // steps that allow it: all-or-nothing made them run masked throughout)
#pragma unroll
        for (int c = 0; c < PC; ++c) {
            if (FAST && c + R < nfull) k_step(Full{}, c % R, c, c);
            else k_step(Ragged{}, c % R, c, c);
        }
        t0 = PC;
    }
    if (FAST) {
        for (; t0 + 2 * R <= nfull; t0 += R) {
#pragma unroll
            for (int s = 0; s < R; ++s) k_step(Full{}, s, t0 + s, -1);
        }
    }
    for (; t0 < nk; t0 += R) {
#pragma unroll
        for (int s = 0; s < R; ++s) k_step(Ragged{}, s, t0 + s, -1);
    }

    if (IS_GRAD) {
        // Bias gradient: join the two k halves of each lane pair, then the k-split wave groups
        // (fixed order, through LDS; the k loop ended with a barrier, so the tile buffers are free).
#pragma unroll
        for (int i = 0; i < TM; ++i) bs[i] += __shfl_xor(bs[i], 32, 64);
        if (bias_wave && h == 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i) smem[wk * BM + wm * T::WTM + i * 32 + idx] = bs[i];
        }
        __syncthreads();
        if (n0 == 0 && tid < BM && m0 + tid < g.M) {
            float bsum = 0.f;
#pragma unroll
            for (int w = 0; w < WK; ++w) bsum += smem[w * BM + tid];
            const int o = m0 + tid;
            if (EPI == EPI_GRAD_STORE) {
                g.gb[o] = bsum * g.scale;
            } else if (EPI == EPI_GRAD_SGD) {
                g.gb[o] = g.gb[o] + (-g.scale * bsum);
            } else if (EPI == EPI_GRAD_SGD_KEEPV) {
                const float dw = -g.scale * bsum;
                g.vb[o] = dw;
                g.gb[o] = g.gb[o] + dw;
            } else {
                const float dw = g.mu * g.vb[o] - g.scale * bsum;
                g.vb[o] = dw;
                g.gb[o] = g.gb[o] + dw;
            }
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
    }
    const bool lead = WK == 1 || wk == 0;   // waves that hold the workgroup's tile

    // k split across workgroups: every workgroup leaves its partial tile in the workspace and
    // counts itself in; the one that arrives last adds the partials in split order (so the sum
    // does not depend on arrival order) and runs the epilogue.  Partials travel as relaxed
    // device-scope atomic stores / loads, which go through to memory and bypass the per-XCD L2,
    // so no cache write-back or invalidation is needed (either would throw away the operand
    // panels the other workgroups of the XCD are working from).  Order: every wave waits until
    // its own stores are acknowledged (drain_device_scope_stores), the workgroup barrier joins the
    // waves, then thread 0 counts the workgroup in with a device-scope atomic; the last arriver's
    // loads are issued after the barrier that follows its own count, hence after every partial.
    if (g0.sk > 1) {
        const int wpos = wm * T::WN + wn;
        const size_t tile_floats = (size_t)BM * BN;
        float *mine = g0.ws + ((size_t)tile_id * g0.sk + split) * tile_floats + (size_t)wpos * TM * TN * 1024;
        if (lead) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        __hip_atomic_store(&mine[((i * TN + j) * 16 + r) * 64 + lane], acc[i][j][r], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
        }
        drain_device_scope_stores();   // every wave: its partial tile has reached device scope
        __syncthreads();               // ... before thread 0 counts the workgroup in
        int *s_last = reinterpret_cast<int *>(smem);
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(&g0.counters[tile_id], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *s_last = (old == (unsigned)(g0.sk - 1)) ? 1 : 0;
        }
        __syncthreads();
        if (*s_last == 0) return;
        if (tid == 0)   // ready for the next launch
            __hip_atomic_store(&g0.counters[tile_id], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lead) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
            for (int sp = 0; sp < g0.sk; ++sp) {
                const float *src = g0.ws + ((size_t)tile_id * g0.sk + sp) * tile_floats + (size_t)wpos * TM * TN * 1024;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            acc[i][j][r] += __hip_atomic_load(&src[((i * TN + j) * 16 + r) * 64 + lane], __ATOMIC_RELAXED,
                                                              __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    // FWD with the k steps split among WK wave groups: only one group in WK holds the tile, and an
    // activation such as tanh costs tens of instructions per element -- measured 2.5 us of a 9 us
    // kernel when that one group ran the whole epilogue.  The sums go through LDS once more
    // ([row][BN + 4]) and every thread of the workgroup finishes four adjacent columns of one row.
    if (WK > 1 && EPI == EPI_FWD) {
        constexpr int PITCH = BN + 4;
        static_assert(WK == 1 || EPI != EPI_FWD || BM * PITCH <= 2 * STAGE, "the tile must fit the operand buffers");
        __syncthreads();   // everyone has read what the k-split exchange left in LDS
        if (lead) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        smem[(wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * h + (r % 4)) * PITCH + wn * T::WTN + j * 32 + idx] = acc[i][j][r];
        }
        __syncthreads();
        for (int e = tid; e < BM * BN / 4; e += NT) {
            const int rl = e / (BN / 4), cl = (e % (BN / 4)) * 4;
            const int row = m0 + rl, col = n0 + cl;
            if (row >= g.M || col >= g.N) continue;
            const v4f sv = *reinterpret_cast<const v4f *>(smem + rl * PITCH + cl);
            v4f o;
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = act_fn(g.act, sv[q] + bias4[q]);
            if (wide_out && col + 4 <= g.N) {
                *reinterpret_cast<v4f *>(g.C + (size_t)row * g.ldc + col) = o;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (col + q < g.N) g.C[(size_t)row * g.ldc + col + q] = o[q];
            }
        }
        return;
    }
    if (!lead) return;

    // Epilogue.  Lanes of one register cover 32 consecutive columns of one row.
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * T::WTN + j * 32 + idx;
            if (!FAST && col >= g.N) continue;
            const float bias = bias_pre[j];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * T::WTM + i * 32 + 8 * (r / 4) + 4 * h + (r % 4);
                if (!FAST && row >= g.M) continue;
                epilogue_store<EPI>(g, (size_t)row * g.ldc + col, acc[i][j][r], bias,
                                    pre_w[PRE_W ? i : 0][PRE_W ? j : 0][r],
                                    (EPI == EPI_GRAD_MOMENTUM && !PRE_V) ? g.V[(size_t)row * g.ldc + col]
                                                                         : pre_v[PRE_V ? i : 0][PRE_V ? j : 0][r]);
            }
        }
    }
}

// The tile (and k split) a workgroup takes, and its work.  `block` counts the workgroups of this
// product from zero.  Workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous
// run of tiles so that tiles sharing operand panels meet in one L2.  Tiles are ordered in groups of
// GN tile columns, m next, the columns of the group fastest: the ~128 tiles an XCD works on at a
// time then form a compact block (16 x 8 tiles: 24 operand panels) rather than two full tile
// columns (66 panels), which matters for the weight-gradient product, whose streaming
// read-modify-write of W and the velocity keeps evicting the panels from the L2.
template <class T, bool A_KC, bool B_KC, int EPI, bool VEC>
__device__ __forceinline__ void gemm_block(const GemmArgs &g, float *smem, int tiles_m, int tiles_n, int block)
{
    const int nt = tiles_m * tiles_n;
    const int sk = g.sk > 1 ? g.sk : 1;
    const int nwork = nt * sk;           // (tile, k split) pairs, splits of a tile adjacent
    const int per_xcd = (nwork + 7) / 8;
    const int u = (block % 8) * per_xcd + block / 8;
    if (u >= nwork) return;
    const int v = u / sk, split = u - v * sk;
    constexpr int GN = 8;
    const int group = v / (tiles_m * GN);
    const int r = v - group * (tiles_m * GN);
    const int gn = min(GN, tiles_n - group * GN);
    const int tm = r / gn, tn = group * GN + (r - tm * gn);
    const int m0 = tm * T::BM, n0 = tn * T::BN;
    if (VEC && m0 + T::BM <= g.M && n0 + T::BN <= g.N)
        gemm_tile<T, A_KC, B_KC, EPI, VEC, VEC>(g, smem, m0, n0, v, split);
    else
        gemm_tile<T, A_KC, B_KC, EPI, VEC, false>(g, smem, m0, n0, v, split);
}

template <class T, bool A_KC, bool B_KC, int EPI, bool VEC>
__global__ __launch_bounds__(T::NT, T::OCC) void gemm_kernel(GemmArgs g, int tiles_m, int tiles_n)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    gemm_block<T, A_KC, B_KC, EPI, VEC>(g, smem, tiles_m, tiles_n, (int)blockIdx.x);
}

// A product's template parameters as one type.
template <class T, bool A_KC_, bool B_KC_, int EPI_>
struct Product {
    using Tile = T;
    static constexpr bool A_KC = A_KC_, B_KC = B_KC_;
    static constexpr int EPI = EPI_;
};

// A matrix-core product and the weight gradient / update of a layer with at most 16 outputs (vector
// units, narrow_grad_block) in one launch: workgroups [0, blocks0) take the product's tiles, the
// rest the narrow gradient.  Both use 256 threads.
template <class P0>
__global__ __launch_bounds__(P0::Tile::NT, P0::Tile::OCC)
void gemm_narrow_grad_kernel(GemmArgs g0, int tiles_m0, int tiles_n0, int blocks0, NarrowGradArgs ng, int narrow_blocks)
{
    static_assert(P0::Tile::NT == 256, "the narrow gradient's workgroups have 256 threads");
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int block = (int)blockIdx.x;
    if (block < blocks0)
        gemm_block<typename P0::Tile, P0::A_KC, P0::B_KC, P0::EPI, true>(g0, smem, tiles_m0, tiles_n0, block);
    else
        narrow_grad_block<4>(ng, block - blocks0, narrow_blocks);
}

// The weight gradients / updates of several layers in ONE launch: they only need the deltas, so once
// every delta product of a backward pass has run they are all independent.  Workgroup numbers are
// dealt out layer by layer (each layer's run starts at a multiple of 8, so a workgroup's XCD is the
// same function of its number within the layer); the workgroups after the last matrix-core layer
// take a narrow layer's gradient on the vector units, if there is one.  All layers use the same tile
// shape and update mode.
constexpr int MG_MAX = 8;
struct MultiGradArgs {
    int n;                       // matrix-core layers
    int first[MG_MAX + 1];       // first workgroup of each layer; first[n] = first workgroup of the narrow layer
    int tiles_m[MG_MAX], tiles_n[MG_MAX];
    int narrow_blocks;           // 0: no narrow layer
    GemmArgs g[MG_MAX];
    NarrowGradArgs ng;
};

template <class T, int EPI>
__global__ __launch_bounds__(T::NT, T::OCC) void gemm_multi_grad_kernel(MultiGradArgs m)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int block = (int)blockIdx.x;
    if (T::NT == 256 && block >= m.first[m.n]) {   // (the narrow gradient's workgroups have 256 threads)
        narrow_grad_block<4>(m.ng, block - m.first[m.n], m.narrow_blocks);
        return;
    }
    int p = 0;
#pragma unroll
    for (int q = 1; q < MG_MAX; ++q) p += (q < m.n && block >= m.first[q]) ? 1 : 0;
    gemm_block<T, false, false, EPI, true>(m.g[p], smem, m.tiles_m[p], m.tiles_n[p], block - m.first[p]);
}

// ---- tile configurations and dispatch ----------------------------------------
template <class T, bool A_KC, bool B_KC>
constexpr size_t smem_bytes()
{
    constexpr int stage = Lds<A_KC, T::BM, T::KT>::FLOATS + Lds<B_KC, T::BN, T::KT>::FLOATS;
    constexpr int red = (T::WK > 1) ? (T::WK / 2) * T::BM * T::BN : 0;
    return sizeof(float) * (size_t)((2 * stage > red) ? 2 * stage : red);
}

template <class T, bool A_KC, bool B_KC, int EPI, bool VEC>
static hipError_t launch_vec(const GemmArgs &a, hipStream_t stream)
{
    const int tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const long nt = (long)tiles_m * tiles_n;
    // Few output tiles and a long k: split k across workgroups until about two per CU are busy.
    GemmArgs b = a;
    b.sk = 1;
    if (EPI <= EPI_DELTA && a.ws && a.counters && nt < 256 && nt <= a.n_counters) {
        const int nk = (a.K + T::KT - 1) / T::KT;
        int sk = (int)(256 / nt);
        if (sk > 16) sk = 16;
        if (sk > nk / 2) sk = nk / 2;          // at least two k steps each
        while (sk > 1 && (size_t)nt * sk * T::BM * T::BN > a.ws_floats) --sk;
        if (sk > 1) {
            const int per = (nk + sk - 1) / sk;
            sk = (nk + per - 1) / per;         // no empty splits
        }
        b.sk = sk > 1 ? sk : 1;
    }
    const long grid = 8 * ((nt * b.sk + 7) / 8);
    if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
    constexpr size_t lds = smem_bytes<T, A_KC, B_KC>();
    static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS of a CU");
    // raise the dynamic-LDS limit once per instantiation (nets may be driven from different
    // threads: setting it twice is harmless, the flag only has to be read and written atomically)
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_kernel<T, A_KC, B_KC, EPI, VEC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    launch_kernel(gemm_kernel<T, A_KC, B_KC, EPI, VEC>, dim3((unsigned)grid), dim3(T::NT), lds, stream, b, tiles_m, tiles_n);
    return hipGetLastError();
}

//                BM   BN  KT  WM WN WK R  PC
using V0 = Tile<128, 128, 16, 2, 2, 1, 1>;      // short k, many tiles: weight gradients of small batches
using V1 = Tile<128, 64, 16, 2, 2, 1, 2>;       // large batch x width products
using V2 = Tile<64, 64, 64, 1, 1, 4, 2>;
using V3 = Tile<64, 64, 32, 1, 1, 4, 2>;
using V4 = Tile<32, 64, 32, 1, 1, 4, 2>;        // batch of a few hundred x width
using V5 = Tile<32, 64, 64, 1, 1, 8, 2>;
using V6 = Tile<32, 32, 64, 1, 1, 8, 2>;        // few output tiles: lean on the k split
using V7 = Tile<128, 128, 16, 2, 2, 1, 2, 16>;  // weight gradients: epilogue operands fetched over 16 k steps
using V8 = Tile<128, 64, 16, 2, 2, 1, 2, 16, 2>;  // weight gradients, two workgroups per CU: one's epilogue under the other's k loop
using V9 = Tile<64, 64, 16, 2, 2, 1, 2, 8, 4>;    // weight gradients, four workgroups per CU
using V10 = Tile<64, 64, 32, 2, 2, 2, 2, 0, 2>;   // weight gradients over long k (large batches): k split between two wave groups
using V11 = Tile<64, 64, 16, 2, 2, 1, 2, 8, 3>;   // as V9 with three workgroups per CU: the momentum update then needs no register spills
using V12 = Tile<32, 32, 64, 1, 1, 4, 2, 0, 3>;   // batch x width products beside a weight gradient in one launch: 256 threads like V11

static const char *kVariantNames[] = {"128x128x16_r1",  "128x64x16_r2",   "64x64x64_k4_r2", "64x64x32_k4_r2",
                                      "32x64x32_k4_r2", "32x64x64_k8_r2", "32x32x64_k8_r2", "128x128x16_r2_pc16",
                                      "128x64x16_r2_pc16_o2", "64x64x16_r2_pc8_o4", "64x64x32_k2_r2_o2", "64x64x16_r2_pc8_o3",
                                      "32x32x64_k4_r2_o3"};
constexpr int kVariants = 13;
int gemm_variant_count() { return kVariants; }
const char *gemm_variant_name(int v) { return (v >= 0 && v < kVariants) ? kVariantNames[v] : "?"; }

template <class T, bool A_KC, bool B_KC, int EPI>
static hipError_t launch_one(const GemmArgs &a, hipStream_t stream)
{
    const bool a_vec = (a.lda % 4 == 0) && ((A_KC ? a.K : a.M) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.A) & 15) == 0);
    const bool b_vec = (a.ldb % 4 == 0) && ((B_KC ? a.K : a.N) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.B) & 15) == 0);
    if (a_vec && b_vec) return launch_vec<T, A_KC, B_KC, EPI, true>(a, stream);
    // operands that cannot be loaded as float4 (widths not a multiple of 4) are small in
    // practice: one tile shape serves them all
    return launch_vec<V4, A_KC, B_KC, EPI, false>(a, stream);
}

template <class T>
static hipError_t launch_kind(GemmKind kind, const GemmArgs &a, hipStream_t stream)
{
    switch (kind) {
    case GEMM_FWD: return launch_one<T, true, true, EPI_FWD>(a, stream);
    case GEMM_DELTA: return launch_one<T, true, false, EPI_DELTA>(a, stream);
    case GEMM_GRAD:
        switch (a.mode) {
        case GRAD_STORE: return launch_one<T, false, false, EPI_GRAD_STORE>(a, stream);
        case GRAD_SGD: return launch_one<T, false, false, EPI_GRAD_SGD>(a, stream);
        case GRAD_SGD_KEEPV: return launch_one<T, false, false, EPI_GRAD_SGD_KEEPV>(a, stream);
        case GRAD_MOMENTUM: return launch_one<T, false, false, EPI_GRAD_MOMENTUM>(a, stream);
        default: return hipErrorInvalidValue;
        }
    default: return hipErrorInvalidValue;
    }
}

// Tile shape from the problem shape: prefer the largest tile that still gives every CU
// (256 of them) at least one workgroup; outputs with few tiles use small tiles whose waves
// split k among themselves.
static int pick_variant(GemmKind kind, const GemmArgs &a)
{
    auto tiles = [&](int bm, int bn) { return (long)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
    // 64x64 tiles at several workgroups per CU let one workgroup's prologue / epilogue traffic run
    // under another's matrix work.  Weight gradients (read-modify-write epilogue): the k = batch
    // loop is short, so the epilogue operands are prefetched in chunks (variant 11: three
    // workgroups per CU, whose register budget holds the prefetched W and velocity without
    // spills; variant 9, four per CU, spills and is ~6 % slower); over a long k (large batches)
    // two wave groups split each k step instead (variant 10).  Forward and delta products always
    // have a long k.
    if (kind == GEMM_GRAD && tiles(64, 64) >= 256) return a.K > 512 ? 10 : 11;
    if (kind != GEMM_GRAD && tiles(64, 64) >= 256) return 10;
    // fewer tiles over a long k: the same tile with k split across workgroups (256 x 1000 x 4096:
    // 31 us against 38 us for 32x32 tiles whose eight waves split k)
    if (kind != GEMM_GRAD && a.ws && tiles(64, 64) >= 64 && a.K >= 2048) return 10;
    if (a.K <= 512 && tiles(128, 128) >= 256) return a.K >= 192 ? 7 : 0;
    if (tiles(128, 64) >= 256) return 1;
    if (tiles(32, 64) > 256) return 4;
    // few output tiles: 32 x 32 tiles whose waves split k.  Four waves at up to three workgroups per
    // CU (variant 12) measured 3-5 % faster than eight waves at one (variant 6) on batch x 1024 x 1024
    // forward / delta products for batches of 32 to 512; weight gradients keep the older choice
    return kind != GEMM_GRAD ? 12 : 6;
}

// ---- a delta product and a narrow layer's gradient in one launch ---------------------------
static bool vec_ok(GemmKind kind, const GemmArgs &a)
{
    const bool a_kc = kind != GEMM_GRAD, b_kc = kind == GEMM_FWD;
    const bool a_vec = (a.lda % 4 == 0) && ((a_kc ? a.K : a.M) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.A) & 15) == 0);
    const bool b_vec = (a.ldb % 4 == 0) && ((b_kc ? a.K : a.N) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.B) & 15) == 0);
    return a_vec && b_vec;
}

// Whether launch_delta_with_narrow_grad takes this pair: a narrow layer's gradient (dense operands,
// 16-byte pieces) beside a moderate batch x width delta product through another layer's weights.
bool delta_narrow_grad_fits(const GemmArgs &delta, const GemmArgs &grad, int variant)
{
    const bool dense = grad.lda == grad.M && grad.ldb == grad.N && grad.ldc == grad.N;
    const bool vec = grad.N % 4 == 0 && ((reinterpret_cast<uintptr_t>(grad.B) | reinterpret_cast<uintptr_t>(grad.C) |
                                          reinterpret_cast<uintptr_t>(grad.V)) & 15) == 0;
    return variant < 0 && narrow_layer(grad.M) && dense && vec && !narrow_layer(delta.K) && vec_ok(GEMM_DELTA, delta) &&
           delta.M <= 512 && delta.K <= 2048;
}

// The delta product `delta` (through W_{l-1}) and the gradient / update `grad` of a narrow layer l in
// one launch (they do not depend on each other); call only if delta_narrow_grad_fits.
hipError_t launch_delta_with_narrow_grad(const GemmArgs &delta, const GemmArgs &grad, hipStream_t stream)
{
    using P0 = Product<V12, true, false, EPI_DELTA>;
    GemmArgs d = delta;
    d.sk = 1;   // the launch has enough workgroups as it is
    const int tm = (d.M + V12::BM - 1) / V12::BM, tn = (d.N + V12::BN - 1) / V12::BN;
    const long g0 = 8 * (((long)tm * tn + 7) / 8);
    const int nb = grad.N / 4 + 1;
    NarrowGradArgs ng{grad.A, grad.B, grad.C, grad.V, grad.gb, grad.vb, grad.K, grad.M, grad.N, grad.mode, grad.scale, grad.mu};
    constexpr size_t lds = smem_bytes<V12, true, false>();
    launch_kernel(gemm_narrow_grad_kernel<P0>, dim3((unsigned)(g0 + nb)), dim3(256), lds, stream, d, tm, tn, (int)g0, ng, nb);
    return hipGetLastError();
}

// ---- the gradients of several layers in one launch ---------------------------------------
// The shared launch uses one tile shape: the 64 x 64, three-per-CU gradient tile for short
// contractions (batches up to 512), the 64 x 64 tile whose two wave groups split k for longer ones --
// the choices pick_variant makes for large weight matrices.
static bool long_k(const GemmArgs &a) { return a.K > 512; }

static bool multi_grad_layer_fits(const GemmArgs &a, bool family_long_k)
{
    // a matrix of at least 64 tiles of 64 x 64, contraction length in the family's range
    return !narrow_layer(a.M) && vec_ok(GEMM_GRAD, a) && long_k(a) == family_long_k &&
           (long)((a.M + 63) / 64) * ((a.N + 63) / 64) >= 64;
}

static bool multi_grad_narrow_fits(const GemmArgs &a)
{
    const bool dense = a.lda == a.M && a.ldb == a.N && a.ldc == a.N;
    const bool vec = a.N % 4 == 0 && ((reinterpret_cast<uintptr_t>(a.B) | reinterpret_cast<uintptr_t>(a.C) |
                                       reinterpret_cast<uintptr_t>(a.V)) & 15) == 0;
    return narrow_layer(a.M) && dense && vec;
}

template <class T, int EPI>
static hipError_t launch_multi_as(const MultiGradArgs &m, unsigned grid, hipStream_t stream)
{
    constexpr size_t lds = smem_bytes<T, false, false>();
    launch_kernel(gemm_multi_grad_kernel<T, EPI>, dim3(grid), dim3(T::NT), lds, stream, m);
    return hipGetLastError();
}

template <class T>
static hipError_t launch_multi_mode(const MultiGradArgs &m, int mode, unsigned grid, hipStream_t stream)
{
    switch (mode) {
    case GRAD_STORE: return launch_multi_as<T, EPI_GRAD_STORE>(m, grid, stream);
    case GRAD_SGD: return launch_multi_as<T, EPI_GRAD_SGD>(m, grid, stream);
    case GRAD_SGD_KEEPV: return launch_multi_as<T, EPI_GRAD_SGD_KEEPV>(m, grid, stream);
    case GRAD_MOMENTUM: return launch_multi_as<T, EPI_GRAD_MOMENTUM>(m, grid, stream);
    default: return hipErrorInvalidValue;
    }
}

// Which of the gradient products grads[0..n) (all GEMM_GRAD) launch_gemm_grads puts into its shared
// launch: at most MG_MAX matrix-core layers and one narrow layer, all in the mode of grads[0]; none
// when a tile shape is forced, `merge` is false or fewer than two qualify.
void gemm_grads_plan(const GemmArgs *grads, int n, int variant, bool merge, bool *in_shared, int *merged_out)
{
    int wide = 0, narrow = 0;
    for (int i = 0; i < n; ++i) in_shared[i] = false;
    if (merge && variant < 0) {
        const bool family = long_k(grads[0]);   // every layer of a backward pass contracts over the same batch
        for (int i = 0; i < n; ++i) {
            if (grads[i].mode != grads[0].mode) continue;
            if (wide < MG_MAX && multi_grad_layer_fits(grads[i], family)) {
                in_shared[i] = true;
                ++wide;
            } else if (narrow < 1 && !family && multi_grad_narrow_fits(grads[i])) {
                in_shared[i] = true;
                ++narrow;
            }
        }
    }
    if (wide + narrow < 2 || wide < 1) {
        for (int i = 0; i < n; ++i) in_shared[i] = false;
        wide = narrow = 0;
    }
    if (merged_out) *merged_out = wide + narrow;
}

// Enqueues the gradient products grads[0..n) (n <= 64): those gemm_grads_plan selects in one
// launch, the others one by one.
hipError_t launch_gemm_grads(const GemmArgs *grads, int n, int variant, bool merge, hipStream_t stream, int *merged_out)
{
    if (n < 1 || n > 64) return hipErrorInvalidValue;
    bool taken[64];
    int count = 0;
    gemm_grads_plan(grads, n, variant, merge, taken, &count);
    if (merged_out) *merged_out = count;
    if (count >= 2) {
        MultiGradArgs m{};
        int narrow = -1;
        for (int i = 0; i < n; ++i) {
            if (!taken[i]) continue;
            if (narrow_layer(grads[i].M)) {
                narrow = i;
            } else {
                m.g[m.n] = grads[i];
                m.g[m.n].sk = 1;
                ++m.n;
            }
        }
        static_assert(V10::BM == V11::BM && V10::BN == V11::BN, "both families tile the matrices alike");
        long at = 0;
        for (int p = 0; p < m.n; ++p) {
            m.first[p] = (int)at;
            m.tiles_m[p] = (m.g[p].M + V11::BM - 1) / V11::BM;
            m.tiles_n[p] = (m.g[p].N + V11::BN - 1) / V11::BN;
            at += 8 * (((long)m.tiles_m[p] * m.tiles_n[p] + 7) / 8);
        }
        m.first[m.n] = (int)at;
        if (narrow >= 0) {
            const GemmArgs &a = grads[narrow];
            m.narrow_blocks = a.N / 4 + 1;
            m.ng = NarrowGradArgs{a.A, a.B, a.C, a.V, a.gb, a.vb, a.K, a.M, a.N, a.mode, a.scale, a.mu};
            at += m.narrow_blocks;
        }
        if (at > 0x7fffffffL) return hipErrorInvalidValue;
        const hipError_t e = long_k(m.g[0]) ? launch_multi_mode<V10>(m, grads[0].mode, (unsigned)at, stream)
                                            : launch_multi_mode<V11>(m, grads[0].mode, (unsigned)at, stream);
        if (e != hipSuccess) return e;
    }
    for (int i = 0; i < n; ++i) {
        if (taken[i]) continue;
        const hipError_t e = launch_gemm(GEMM_GRAD, grads[i], variant, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_gemm(GemmKind kind, const GemmArgs &a, int variant, hipStream_t stream)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (variant < 0) {
        // a layer with at most 16 outputs (dense operands): plain-FMA kernels, no tiles to pad
        if (kind == GEMM_DELTA && narrow_layer(a.K) && a.lda == a.K && a.ldb == a.N && a.ldc == a.N)
            return launch_narrow_delta(a.A, a.B, a.aux, a.C, a.M, a.K, a.N, a.act, stream);
        if (kind == GEMM_GRAD && narrow_layer(a.M) && a.lda == a.M && a.ldb == a.N && a.ldc == a.N)
            return launch_narrow_grad(a.A, a.B, a.C, a.V, a.gb, a.vb, a.K, a.M, a.N, a.mode, a.scale, a.mu, stream);
        variant = pick_variant(kind, a);
    }
    switch (variant) {
    case 0: return launch_kind<V0>(kind, a, stream);
    case 1: return launch_kind<V1>(kind, a, stream);
    case 2: return launch_kind<V2>(kind, a, stream);
    case 3: return launch_kind<V3>(kind, a, stream);
    case 4: return launch_kind<V4>(kind, a, stream);
    case 5: return launch_kind<V5>(kind, a, stream);
    case 6: return launch_kind<V6>(kind, a, stream);
    case 7: return launch_kind<V7>(kind, a, stream);
    case 8: return launch_kind<V8>(kind, a, stream);
    case 9: return launch_kind<V9>(kind, a, stream);
    case 10: return launch_kind<V10>(kind, a, stream);
    case 11: return launch_kind<V11>(kind, a, stream);
    case 12: return launch_kind<V12>(kind, a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace dn
