// Implicit-GEMM convolution kernels on MFMA for gfx950 (64-wide wavefronts).
//
// The three convolutions of a DSP block step -- forward / recompute, backward-data and
// backward-weight (the chain rule of Eq. (2)/(5) of the paper applied to a conv layer) -- are
// dense contractions, so they run on the matrix cores:
//
//   forward        y[m][co]  = sum_k  xcol[m][k] * w[co][k]        m=(n,ho,wo), k=(r,s,ci)
//   backward-data  dx[m][ci] = sum_k dycol[m][k] * wt[ci][k]       m=(n,hi,wi), k=(r',s',co)
//   backward-weight dw[co][j] = sum_m dy[m][co] * xcol[m][j]       j=(r,s,ci), m=(n,ho,wo)
//
// xcol / dycol are never materialised: the loader gathers 16-byte channel runs of the NHWC
// tensor straight into LDS (zero for padding; for a strided backward-data only taps that hit an
// output pixel are non-zero).  All kernels share one tile engine: a 256-thread workgroup
// (4 waves) owns a BM x BN output tile; the K dimension is streamed through double-buffered
// LDS tiles whose rows hold BKB bytes of k plus a 16-byte pad (conflict-free ds_read_b128);
// every lane feeds the MFMA with 16-byte k-runs (8 bf16 -> one 32x32x16 / 16x16x32 MFMA,
// 4 floats -> four 32x32x2 / 16x16x4 MFMAs).  Accumulation is fp32 in both storage types.
#include <stdio.h>

#include "common.h"

namespace dsp {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kThreads = 256;

// ---- MFMA on 16-byte operand fragments --------------------------------------------------------
template <typename T, int MT>
struct Mma;

template <>
struct Mma<bf16_t, 32> {
    typedef f32x16 Acc;
    static constexpr int kAcc = 16;
    __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                    0, 0, 0);
    }
};
template <>
struct Mma<bf16_t, 16> {
    typedef f32x4 Acc;
    static constexpr int kAcc = 4;
    __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                    0, 0, 0);
    }
};
template <>
struct Mma<float, 32> {
    typedef f32x16 Acc;
    static constexpr int kAcc = 16;
    __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c)
    {
        const f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[i], c, 0, 0, 0);
    }
};
template <>
struct Mma<float, 16> {
    typedef f32x4 Acc;
    static constexpr int kAcc = 4;
    __device__ static inline void run(const u32x4& a, const u32x4& b, Acc& c)
    {
        const f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[i], fb[i], c, 0, 0, 0);
    }
};

// Row of the MT x MT accumulator tile held in register j of lane `lane`; its column is lane % MT.
template <int MT>
__device__ inline int acc_row(int lane, int j)
{
    if (MT == 32) return (j >> 2) * 8 + (lane >> 5) * 4 + (j & 3);
    return (lane >> 4) * 4 + j;
}

// ---- tile configuration -----------------------------------------------------------------------
template <typename T_, int MT_, int WGM_, int WGN_, int TM_, int TN_, int BKB_>
struct Tile {
    typedef T_ T;
    static constexpr int MT = MT_, WGM = WGM_, WGN = WGN_, TM = TM_, TN = TN_, BKB = BKB_;
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static constexpr int BM = WGM * TM * MT;
    static constexpr int BN = WGN * TN * MT;
    static constexpr int E = 16 / (int)sizeof(T);    // elements per 16-byte run
    static constexpr int BK = BKB / (int)sizeof(T);  // k elements per LDS tile
    static constexpr int ROWB = BKB + 16;            // padded LDS row, bytes
    static constexpr int KSB = (64 / MT) * 16;       // k bytes one MFMA step consumes per row
    static constexpr int NSUB = BKB / KSB;
    static constexpr int CPR = BKB / 16;             // 16-byte chunks per row
    static constexpr int A_CHUNKS = BM * CPR, B_CHUNKS = BN * CPR;
    static constexpr int A_PER = (A_CHUNKS + kThreads - 1) / kThreads;
    static constexpr int B_PER = (B_CHUNKS + kThreads - 1) / kThreads;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * ROWB;
    static_assert(BKB % KSB == 0 && kThreads % CPR == 0, "tile shape");
};

template <typename TL>
__device__ inline void mma_tile(const char* sA, const char* sB, int wave_m, int wave_n, int lane,
                                typename Mma<typename TL::T, TL::MT>::Acc (&acc)[TL::TM][TL::TN])
{
    constexpr int MT = TL::MT;
    const int frow = lane % MT, fg = lane / MT;
#pragma unroll
    for (int ks = 0; ks < TL::NSUB; ++ks) {
        u32x4 a[TL::TM], b[TL::TN];
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
            a[i] = *(const u32x4*)(sA + ((wave_m * TL::TM + i) * MT + frow) * TL::ROWB + ks * TL::KSB + fg * 16);
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
            b[j] = *(const u32x4*)(sB + ((wave_n * TL::TN + j) * MT + frow) * TL::ROWB + ks * TL::KSB + fg * 16);
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int j = 0; j < TL::TN; ++j) Mma<typename TL::T, MT>::run(a[i], b[j], acc[i][j]);
    }
}

// ---- forward / backward-data ------------------------------------------------------------------
// The gathered tensor `in` is N x Hi x Wi x Ci; output rows m = (n, ho, wo) over N x Ho x Wo.
// Tap (r, s) of output pixel (ho, wo) reads position t = o*ostride - pad + tap; with idil = 2
// (backward-data of a stride-2 conv) only even t exist and they map to source pixel t/2.
struct GatherGeom {
    int N, Hi, Wi, Ci, Ho, Wo, Co, R, S, pad_h, pad_w, ostride, idil;
    int M, Kdim;
};

template <typename TL, bool VEC, bool ACCUM>
__global__ __launch_bounds__(kThreads) void conv_gather_gemm_kernel(const typename TL::T* __restrict__ in,
                                                                    const typename TL::T* __restrict__ wgt,
                                                                    typename TL::T* __restrict__ out, GatherGeom g)
{
    typedef typename TL::T T;
    constexpr int E = TL::E, CPR = TL::CPR, ROWS_PER_PASS = kThreads / CPR;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sA[2];
    char* sB[2];
    sA[0] = smem;
    sA[1] = smem + (TL::BM + TL::BN) * TL::ROWB;
    sB[0] = sA[0] + TL::BM * TL::ROWB;
    sB[1] = sA[1] + TL::BM * TL::ROWB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    // consecutive workgroups share the same rows of `in` and sweep the output channels
    const int tiles_n = (g.Co + TL::BN - 1) / TL::BN;
    const int m0 = (blockIdx.x / tiles_n) * TL::BM, n0 = (blockIdx.x % tiles_n) * TL::BN;

    const int kc = tid % CPR;      // which 16-byte run of the k tile this thread moves
    const int row0 = tid / CPR;    // first tile row it moves; further rows are +ROWS_PER_PASS apart

    // per-row gather state of the A operand
    int64_t a_base[TL::A_PER];
    int a_th0[TL::A_PER], a_tw0[TL::A_PER];
#pragma unroll
    for (int i = 0; i < TL::A_PER; ++i) {
        const int row = row0 + i * ROWS_PER_PASS;
        const int m = m0 + row;
        if (row < TL::BM && m < g.M) {
            const int wo = m % g.Wo, t = m / g.Wo, ho = t % g.Ho, n = t / g.Ho;
            a_base[i] = (int64_t)n * g.Hi * g.Wi * g.Ci;
            a_th0[i] = ho * g.ostride - g.pad_h;
            a_tw0[i] = wo * g.ostride - g.pad_w;
        } else {
            a_base[i] = -1;
            a_th0[i] = a_tw0[i] = 0;
        }
    }

    // k position of this thread's run: element kk = (r*S + s)*Ci + ci
    int kk = kc * E, kr = 0, ks = 0, kci = kc * E;
    while (kci >= g.Ci) {
        kci -= g.Ci;
        if (++ks == g.S) { ks = 0; ++kr; }
    }

    u32x4 ra[TL::A_PER], rb[TL::B_PER];

    auto gather_one = [&](int64_t base, int th0, int tw0, int r, int s, int ci) -> T {
        int th = th0 + r, tw = tw0 + s;
        bool ok = base >= 0 && th >= 0 && tw >= 0;
        if (g.idil == 2) {
            ok = ok && ((th | tw) & 1) == 0;
            th >>= 1;
            tw >>= 1;
        }
        ok = ok && th < g.Hi && tw < g.Wi;
        return ok ? in[base + ((int64_t)th * g.Wi + tw) * g.Ci + ci] : from_float<T>(0.f);
    };

    auto load_tiles = [&]() {
        if (VEC) {
            const bool k_ok = kk < g.Kdim;
#pragma unroll
            for (int i = 0; i < TL::A_PER; ++i) {
                int th = a_th0[i] + kr, tw = a_tw0[i] + ks;
                bool ok = k_ok && a_base[i] >= 0 && th >= 0 && tw >= 0;
                if (g.idil == 2) {
                    ok = ok && ((th | tw) & 1) == 0;
                    th >>= 1;
                    tw >>= 1;
                }
                ok = ok && th < g.Hi && tw < g.Wi;
                u32x4 v = {0, 0, 0, 0};
                if (ok) v = *(const u32x4*)(in + a_base[i] + ((int64_t)th * g.Wi + tw) * g.Ci + kci);
                ra[i] = v;
            }
#pragma unroll
            for (int i = 0; i < TL::B_PER; ++i) {
                const int row = row0 + i * ROWS_PER_PASS, co = n0 + row;
                u32x4 v = {0, 0, 0, 0};
                if (row < TL::BN && co < g.Co && k_ok) v = *(const u32x4*)(wgt + (int64_t)co * g.Kdim + kk);
                rb[i] = v;
            }
        } else {
            // generic path (channel count not a multiple of the 16-byte run): element-wise gather
#pragma unroll
            for (int i = 0; i < TL::A_PER; ++i) {
                alignas(16) T tmp[E];
                for (int e = 0; e < E; ++e) {
                    const int k = kk + e;
                    const int tap = k / g.Ci, ci = k % g.Ci;
                    tmp[e] = k < g.Kdim ? gather_one(a_base[i], a_th0[i], a_tw0[i], tap / g.S, tap % g.S, ci)
                                        : from_float<T>(0.f);
                }
                ra[i] = *(const u32x4*)tmp;
            }
#pragma unroll
            for (int i = 0; i < TL::B_PER; ++i) {
                const int row = row0 + i * ROWS_PER_PASS, co = n0 + row;
                alignas(16) T tmp[E];
                for (int e = 0; e < E; ++e)
                    tmp[e] = (row < TL::BN && co < g.Co && kk + e < g.Kdim) ? wgt[(int64_t)co * g.Kdim + kk + e]
                                                                           : from_float<T>(0.f);
                rb[i] = *(const u32x4*)tmp;
            }
        }
    };
    auto advance_k = [&]() {
        kk += TL::BK;
        kci += TL::BK;
        while (kci >= g.Ci) {
            kci -= g.Ci;
            if (++ks == g.S) { ks = 0; ++kr; }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TL::A_PER; ++i) {
            const int row = row0 + i * ROWS_PER_PASS;
            if (row < TL::BM) *(u32x4*)(sA[buf] + row * TL::ROWB + kc * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < TL::B_PER; ++i) {
            const int row = row0 + i * ROWS_PER_PASS;
            if (row < TL::BN) *(u32x4*)(sB[buf] + row * TL::ROWB + kc * 16) = rb[i];
        }
    };

    typename Mma<T, TL::MT>::Acc acc[TL::TM][TL::TN];
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < Mma<T, TL::MT>::kAcc; ++e) acc[i][j][e] = 0.f;

    const int nk = (g.Kdim + TL::BK - 1) / TL::BK;
    load_tiles();
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            advance_k();
            load_tiles();
        }
        mma_tile<TL>(sA[cur], sB[cur], wave_m, wave_n, lane, acc);
        if (kt + 1 < nk) store_tiles(cur ^ 1);
        __syncthreads();
    }

    // epilogue: lanes of one accumulator register cover MT consecutive channels of one output row
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j) {
            const int col = n0 + (wave_n * TL::TN + j) * TL::MT + lane % TL::MT;
#pragma unroll
            for (int e = 0; e < Mma<T, TL::MT>::kAcc; ++e) {
                const int m = m0 + (wave_m * TL::TM + i) * TL::MT + acc_row<TL::MT>(lane, e);
                if (m < g.M && col < g.Co) {
                    T* p = out + (int64_t)m * g.Co + col;
                    float v = acc[i][j][e];
                    if (ACCUM) v += to_float<T>(*p);
                    *p = from_float<T>(v);
                }
            }
        }
}

// ---- backward-weight --------------------------------------------------------------------------
// dw[co][j] = sum_m dy[m][co] * xcol[m][j].  Both operands are stored with m as the slow index,
// so the loader transposes 16-byte channel runs into LDS rows that are contiguous in m.
// blockIdx.y selects a slice of m; slices are summed afterwards in a fixed order.
struct WgradGeom {
    int N, H, W, Ci, Ho, Wo, Co, R, S, pad, stride;
    int M, Kdim, m_per_split;
};

template <typename TL, bool VEC>
__global__ __launch_bounds__(kThreads) void conv_wgrad_kernel(const typename TL::T* __restrict__ x,
                                                              const typename TL::T* __restrict__ dy,
                                                              float* __restrict__ part, WgradGeom g)
{
    typedef typename TL::T T;
    constexpr int E = TL::E, BKm = TL::BK;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sA[2];
    char* sB[2];
    sA[0] = smem;
    sA[1] = smem + (TL::BM + TL::BN) * TL::ROWB;
    sB[0] = sA[0] + TL::BM * TL::ROWB;
    sB[1] = sA[1] + TL::BM * TL::ROWB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    const int tiles_n = (g.Kdim + TL::BN - 1) / TL::BN;
    const int c0 = (blockIdx.x / tiles_n) * TL::BM;  // first output channel of the tile
    const int j0 = (blockIdx.x % tiles_n) * TL::BN;  // first (r,s,ci) column of the tile
    const int m_begin = blockIdx.y * g.m_per_split;
    const int m_end = min(g.M, m_begin + g.m_per_split);

    // A' (dy): chunk = E channels of one m row;  B' (x): chunk = E input channels of one tap of one m row
    constexpr int A_CPR = TL::BM / E > 0 ? TL::BM / E : 1, B_CPR = TL::BN / E > 0 ? TL::BN / E : 1;
    constexpr int A_CH = A_CPR * BKm, B_CH = B_CPR * BKm;
    constexpr int A_PER = (A_CH + kThreads - 1) / kThreads, B_PER = (B_CH + kThreads - 1) / kThreads;

    typename Mma<T, TL::MT>::Acc acc[TL::TM][TL::TN];
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < Mma<T, TL::MT>::kAcc; ++e) acc[i][j][e] = 0.f;

    alignas(16) T ra[A_PER][E];
    alignas(16) T rb[B_PER][E];
    const T zero = from_float<T>(0.f);

    auto load_tiles = [&](int mb) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int c = tid + i * kThreads, mrow = c / A_CPR, cc = (c % A_CPR) * E;
            const int m = mb + mrow, co = c0 + cc;
            const bool ok = c < A_CH && m < m_end;
            if (VEC) {
                u32x4 v = {0, 0, 0, 0};
                if (ok && co < g.Co) v = *(const u32x4*)(dy + (int64_t)m * g.Co + co);
                *(u32x4*)ra[i] = v;
            } else {
                for (int e = 0; e < E; ++e)
                    ra[i][e] = (ok && co + e < g.Co && cc + e < TL::BM) ? dy[(int64_t)m * g.Co + co + e] : zero;
            }
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int c = tid + i * kThreads, mrow = c / B_CPR, cc = (c % B_CPR) * E;
            const int m = mb + mrow, j = j0 + cc;
            const bool ok = c < B_CH && m < m_end;
            const int wo = m % g.Wo, t = m / g.Wo, ho = t % g.Ho, n = t / g.Ho;
            if (VEC) {
                const int tap = j / g.Ci, ci = j % g.Ci, r = tap / g.S, s = tap % g.S;
                const int hi = ho * g.stride - g.pad + r, wi = wo * g.stride - g.pad + s;
                u32x4 v = {0, 0, 0, 0};
                if (ok && j < g.Kdim && hi >= 0 && hi < g.H && wi >= 0 && wi < g.W)
                    v = *(const u32x4*)(x + (((int64_t)n * g.H + hi) * g.W + wi) * g.Ci + ci);
                *(u32x4*)rb[i] = v;
            } else {
                for (int e = 0; e < E; ++e) {
                    const int je = j + e;
                    const int tap = je / g.Ci, ci = je % g.Ci, r = tap / g.S, s = tap % g.S;
                    const int hi = ho * g.stride - g.pad + r, wi = wo * g.stride - g.pad + s;
                    rb[i][e] = (ok && je < g.Kdim && cc + e < TL::BN && hi >= 0 && hi < g.H && wi >= 0 && wi < g.W)
                                   ? x[(((int64_t)n * g.H + hi) * g.W + wi) * g.Ci + ci]
                                   : zero;
                }
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_PER; ++i) {
            const int c = tid + i * kThreads, mrow = c / A_CPR, cc = (c % A_CPR) * E;
            if (c < A_CH)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (cc + e < TL::BM) *(T*)(sA[buf] + (cc + e) * TL::ROWB + mrow * (int)sizeof(T)) = ra[i][e];
        }
#pragma unroll
        for (int i = 0; i < B_PER; ++i) {
            const int c = tid + i * kThreads, mrow = c / B_CPR, cc = (c % B_CPR) * E;
            if (c < B_CH)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (cc + e < TL::BN) *(T*)(sB[buf] + (cc + e) * TL::ROWB + mrow * (int)sizeof(T)) = rb[i][e];
        }
    };

    const int nk = (m_end - m_begin + BKm - 1) / BKm;
    if (nk > 0) {
        load_tiles(m_begin);
        store_tiles(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) load_tiles(m_begin + (kt + 1) * BKm);
        mma_tile<TL>(sA[cur], sB[cur], wave_m, wave_n, lane, acc);
        if (kt + 1 < nk) store_tiles(cur ^ 1);
        __syncthreads();
    }

    float* dst = part + (int64_t)blockIdx.y * g.Co * g.Kdim;
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j) {
            const int col = j0 + (wave_n * TL::TN + j) * TL::MT + lane % TL::MT;
#pragma unroll
            for (int e = 0; e < Mma<T, TL::MT>::kAcc; ++e) {
                const int co = c0 + (wave_m * TL::TM + i) * TL::MT + acc_row<TL::MT>(lane, e);
                if (co < g.Co && col < g.Kdim) dst[(int64_t)co * g.Kdim + col] = acc[i][j][e];
            }
        }
}

// dw[i] = sum over slices of part[slice][i], slices in ascending order (run-to-run identical).
// A workgroup owns 32 consecutive elements; 8 lanes per element each add every 8th slice, then the
// 8 lane sums are added in lane order: a fixed summation tree, many loads in flight per element.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int n,
                                                           int splits)
{
    __shared__ float red[8][33];
    const int col = threadIdx.x & 31, lane = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + col;
    float s = 0.f;
    if (i < n)
        for (int k = lane; k < splits; k += 8) s += part[(int64_t)k * n + i];
    red[lane][col] = s;
    __syncthreads();
    if (lane == 0 && i < n) {
        float t = red[0][col];
#pragma unroll
        for (int k = 1; k < 8; ++k) t += red[k][col];
        dw[i] = t;
    }
}

// ---- host-side dispatch -------------------------------------------------------------------------
template <typename TL>
const char* tile_name(const char* what, bool vec, bool accum)
{
    // one name per kernel instantiation, e.g. "conv_gather_gemm<fp32,mfma32,BM128,BN64,vec>"
    static char names[4][96];
    char* n = names[(vec ? 1 : 0) + (accum ? 2 : 0)];
    if (!n[0])
        snprintf(n, 96, "%s<%s,mfma%d,BM%d,BN%d,%s%s>", what, sizeof(typename TL::T) == 2 ? "bf16" : "fp32", TL::MT, TL::BM,
                 TL::BN, vec ? "vec" : "scalar", accum ? ",acc" : "");
    return n;
}

template <typename TL, bool VEC, bool ACCUM>
int run_gather(const GatherGeom& g, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    typedef typename TL::T T;
    const int64_t tiles = (int64_t)ceil_div(g.M, TL::BM) * ceil_div(g.Co, TL::BN);
    DSP_REQUIRE(tiles > 0 && tiles < (1ll << 31), DSP_EINVAL, "conv: bad tile count");
    auto kern = conv_gather_gemm_kernel<TL, VEC, ACCUM>;
    static bool attr_done = false;
    if (!attr_done && TL::LDS_BYTES > 48 * 1024) {
        DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
        attr_done = true;
    }
    {
        ProfScope ps(tile_name<TL>("conv_gather_gemm", VEC, ACCUM), flops, 0);
        DSP_LAUNCH(ps, kern, dim3((unsigned)tiles), dim3(kThreads), TL::LDS_BYTES, st, (const T*)in, (const T*)w, (T*)out, g);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename TL>
int run_gather_v(const GatherGeom& g, bool vec, bool accum, const void* in, const void* w, void* out, hipStream_t st,
                 double flops)
{
    if (vec)
        return accum ? run_gather<TL, true, true>(g, in, w, out, st, flops)
                     : run_gather<TL, true, false>(g, in, w, out, st, flops);
    return accum ? run_gather<TL, false, true>(g, in, w, out, st, flops)
                 : run_gather<TL, false, false>(g, in, w, out, st, flops);
}

template <typename T>
int dispatch_gather(const GatherGeom& g, bool accum, const void* in, const void* w, void* out, hipStream_t st,
                    double flops)
{
    constexpr int E = 16 / (int)sizeof(T);
    // 16-byte gathers need channel runs of E elements and 16-byte aligned bases
    const bool vec = (g.Ci % E) == 0 && ((uintptr_t)in % 16) == 0 && ((uintptr_t)w % 16) == 0;
    // tile by output-channel count; the small-channel tiles keep the whole channel range in one workgroup
    if (g.Co <= 16) return run_gather_v<Tile<T, 16, 4, 1, 4, 1, 64>>(g, vec, accum, in, w, out, st, flops);
    if (g.Co <= 32) return run_gather_v<Tile<T, 32, 4, 1, 2, 1, 64>>(g, vec, accum, in, w, out, st, flops);
    const int64_t big_tiles = (int64_t)ceil_div(g.M, 128) * ceil_div(g.Co, 128);
    if (g.Co % 128 == 0 && big_tiles >= 512)
        return run_gather_v<Tile<T, 32, 2, 2, 2, 2, 64>>(g, vec, accum, in, w, out, st, flops);
    return run_gather_v<Tile<T, 32, 2, 2, 2, 1, 64>>(g, vec, accum, in, w, out, st, flops);
}

template <typename TL, bool VEC>
int run_wgrad(const WgradGeom& g0, int splits, const void* x, const void* dy, float* dst, hipStream_t st, double flops)
{
    typedef typename TL::T T;
    WgradGeom g = g0;
    const int tiles = ceil_div(g.Co, TL::BM) * ceil_div(g.Kdim, TL::BN);
    auto kern = conv_wgrad_kernel<TL, VEC>;
    static bool attr_done = false;
    if (!attr_done && TL::LDS_BYTES > 48 * 1024) {
        DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
        attr_done = true;
    }
    {
        ProfScope ps(tile_name<TL>("conv_wgrad", VEC, false), flops, 0);
        DSP_LAUNCH(ps, kern, dim3(tiles, splits), dim3(kThreads), TL::LDS_BYTES, st, (const T*)x, (const T*)dy, dst, g);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

// Slices of the (n, ho, wo) range: enough workgroups to cover the chip a few times, each slice a
// whole number of LDS tiles and at least 4 of them.
int wgrad_splits(const ConvShape& c, int bm, int bn, int bk, int* m_per_split)
{
    const int64_t M = (int64_t)c.N * c.Ho * c.Wo, Kdim = (int64_t)c.R * c.S * c.Cin;
    const int tiles = ceil_div(c.Cout, bm) * ceil_div(Kdim, bn);
    int want = ceil_div(512, tiles);  // about two workgroups per compute unit
    const int max_by_len = (int)((M + 8 * bk - 1) / (8 * bk));
    if (want > max_by_len) want = max_by_len;
    if (want < 1) want = 1;
    if (want > 256) want = 256;
    int per = (int)((M + want - 1) / want);
    per = ceil_div(per, bk) * bk;
    *m_per_split = per;
    return ceil_div(M, per);
}

struct WgradPlan {
    int bm, bn, bk;
};
WgradPlan wgrad_plan(int dtype, const ConvShape& c)
{
    const int bk = dtype == DSP_BF16 ? 32 : 16;
    if (c.Cout <= 16) return {16, 64, bk};
    if (c.Cout <= 32) return {32, 128, bk};
    return {64, 64, bk};
}

template <typename T>
int dispatch_wgrad(const ConvShape& c, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes,
                   hipStream_t st, double flops)
{
    constexpr int E = 16 / (int)sizeof(T);
    const int dtype = sizeof(T) == 2 ? DSP_BF16 : DSP_FP32;
    const WgradPlan pl = wgrad_plan(dtype, c);
    WgradGeom g{c.N, c.H, c.W, c.Cin, c.Ho, c.Wo, c.Cout, c.R, c.S, c.pad, c.stride, 0, 0, 0};
    g.M = c.N * c.Ho * c.Wo;
    g.Kdim = c.R * c.S * c.Cin;
    const int splits = wgrad_splits(c, pl.bm, pl.bn, pl.bk, &g.m_per_split);
    const size_t n = (size_t)c.Cout * g.Kdim;
    float* dst = dw;
    if (splits > 1) {
        DSP_REQUIRE(ws != nullptr && ws_bytes >= n * splits * sizeof(float), DSP_EINVAL,
                    "conv backward-weight: workspace too small (%zu < %zu)", ws_bytes, n * splits * sizeof(float));
        dst = (float*)ws;
    }
    const bool vec = (c.Cin % E) == 0 && (c.Cout % E) == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)dy % 16) == 0;
    int rc;
    if (c.Cout <= 16)
        rc = vec ? run_wgrad<Tile<T, 16, 1, 4, 1, 1, 64>, true>(g, splits, x, dy, dst, st, flops)
                 : run_wgrad<Tile<T, 16, 1, 4, 1, 1, 64>, false>(g, splits, x, dy, dst, st, flops);
    else if (c.Cout <= 32)
        rc = vec ? run_wgrad<Tile<T, 32, 1, 4, 1, 1, 64>, true>(g, splits, x, dy, dst, st, flops)
                 : run_wgrad<Tile<T, 32, 1, 4, 1, 1, 64>, false>(g, splits, x, dy, dst, st, flops);
    else
        rc = vec ? run_wgrad<Tile<T, 32, 2, 2, 1, 1, 64>, true>(g, splits, x, dy, dst, st, flops)
                 : run_wgrad<Tile<T, 32, 2, 2, 1, 1, 64>, false>(g, splits, x, dy, dst, st, flops);
    DSP_TRY(rc);
    if (splits > 1) {
        ProfScope ps("wgrad_reduce", (double)n * (splits + 1) * 4.0, 1);
        DSP_LAUNCH(ps, wgrad_reduce_kernel, dim3(ceil_div(n, 32)), dim3(256), 0, st, (const float*)ws, dw, (int)n, splits);
        DSP_HIP(hipGetLastError());
    }
    return DSP_OK;
}

// Multiply-accumulates of the convolution as defined (taps that fall on padding are not counted);
// forward, backward-data and backward-weight each perform exactly this many.
double conv_macs(const ConvShape& c)
{
    int64_t vh = 0, vw = 0;
    for (int o = 0; o < c.Ho; ++o)
        for (int r = 0; r < c.R; ++r) {
            const int t = o * c.stride - c.pad + r;
            vh += (t >= 0 && t < c.H);
        }
    for (int o = 0; o < c.Wo; ++o)
        for (int s = 0; s < c.S; ++s) {
            const int t = o * c.stride - c.pad + s;
            vw += (t >= 0 && t < c.W);
        }
    return (double)c.N * (double)vh * (double)vw * (double)c.Cin * (double)c.Cout;
}

int check_shape(const ConvShape& c)
{
    DSP_REQUIRE(c.N > 0 && c.H > 0 && c.W > 0 && c.Cin > 0 && c.Cout > 0 && c.R > 0 && c.S > 0 && c.stride > 0 &&
                    c.pad >= 0 && c.Ho > 0 && c.Wo > 0,
                DSP_EINVAL, "conv: bad shape");
    DSP_REQUIRE((int64_t)c.N * c.H * c.W * c.Cin < (1ll << 31) && (int64_t)c.N * c.Ho * c.Wo * c.Cout < (1ll << 31) &&
                    (int64_t)c.N * c.Ho * c.Wo < (1ll << 31) && (int64_t)c.R * c.S * c.Cin * c.Cout < (1ll << 31),
                DSP_EINVAL, "conv: tensor too large for 32-bit row indices");
    return DSP_OK;
}

}  // namespace

int launch_conv_forward(int dtype, const ConvShape& c, const void* x, const void* w, void* y, hipStream_t st)
{
    DSP_TRY(check_shape(c));
    GatherGeom g{c.N, c.H, c.W, c.Cin, c.Ho, c.Wo, c.Cout, c.R, c.S, c.pad, c.pad, c.stride, 1, 0, 0};
    g.M = c.N * c.Ho * c.Wo;
    g.Kdim = c.R * c.S * c.Cin;
    const double flops = 2.0 * conv_macs(c);
    return dtype == DSP_BF16 ? dispatch_gather<bf16_t>(g, false, x, w, y, st, flops)
                             : dispatch_gather<float>(g, false, x, w, y, st, flops);
}

int launch_conv_backward_data(int dtype, const ConvShape& c, const void* dy, const void* wt, void* dx,
                              bool accumulate, hipStream_t st)
{
    DSP_TRY(check_shape(c));
    DSP_REQUIRE(c.stride == 1 || c.stride == 2, DSP_EINVAL, "conv backward-data: stride %d unsupported", c.stride);
    // dx[n,hi,wi,ci] = sum_{r',s',co} dy[n, (hi - (R-1-pad) + r')/stride, ...][co] * wt[ci][r'][s'][co]
    GatherGeom g{c.N, c.Ho, c.Wo, c.Cout, c.H, c.W, c.Cin, c.R, c.S, c.R - 1 - c.pad, c.S - 1 - c.pad, 1, c.stride, 0, 0};
    g.M = c.N * c.H * c.W;
    g.Kdim = c.R * c.S * c.Cout;
    const double flops = 2.0 * conv_macs(c);
    return dtype == DSP_BF16 ? dispatch_gather<bf16_t>(g, accumulate, dy, wt, dx, st, flops)
                             : dispatch_gather<float>(g, accumulate, dy, wt, dx, st, flops);
}

size_t conv_backward_weight_workspace(const ConvShape& c)
{
    size_t worst = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        const WgradPlan pl = wgrad_plan(dtype, c);
        int per;
        const int splits = wgrad_splits(c, pl.bm, pl.bn, pl.bk, &per);
        const size_t b = splits > 1 ? (size_t)splits * c.Cout * c.R * c.S * c.Cin * sizeof(float) : 0;
        if (b > worst) worst = b;
    }
    return worst;
}

int launch_conv_backward_weight(int dtype, const ConvShape& c, const void* x, const void* dy, float* dw, void* ws,
                                size_t ws_bytes, hipStream_t st)
{
    DSP_TRY(check_shape(c));
    const double flops = 2.0 * conv_macs(c);
    return dtype == DSP_BF16 ? dispatch_wgrad<bf16_t>(c, x, dy, dw, ws, ws_bytes, st, flops)
                             : dispatch_wgrad<float>(c, x, dy, dw, ws, ws_bytes, st, flops);
}

}  // namespace dsp
