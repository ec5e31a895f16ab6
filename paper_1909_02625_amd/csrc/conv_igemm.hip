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
// (4 waves) owns a BM x BN output tile; the K dimension is streamed through LDS tiles whose rows
// hold BKB bytes of k plus a 16-byte pad; every lane feeds the MFMA with 16-byte k-runs
// (8 bf16 -> one 32x32x16 / 16x16x32 MFMA, 4 floats -> four 32x32x2 / 16x16x4 MFMAs).
// Accumulation is fp32 in both storage types.  Tiles are chosen per launch so that even the
// small CIFAR-shaped layers put a few hundred workgroups on the 256 compute units.
#include <stdio.h>

#include <atomic>
#include <new>
#include <vector>

#include "common.h"

namespace dsp {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

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

constexpr int cmax(int a, int b) { return a > b ? a : b; }

// Four consecutive elements of T as one 8-byte (bf16) or 16-byte (fp32) register run.
template <typename T>
struct Run4;
template <>
struct Run4<bf16_t> {
    typedef u32x2 V;
    __device__ static inline V pack(float a, float b, float c, float d)
    {
        return V{pack_bf16x2(a, b), pack_bf16x2(c, d)};
    }
    __device__ static inline void unpack(V v, float (&f)[4])
    {
        const uint32_t lo = v.x, hi = v.y;
        f[0] = __uint_as_float(lo << 16);
        f[1] = __uint_as_float(lo & 0xffff0000u);
        f[2] = __uint_as_float(hi << 16);
        f[3] = __uint_as_float(hi & 0xffff0000u);
    }
};
template <>
struct Run4<float> {
    typedef f32x4 V;
    __device__ static inline V pack(float a, float b, float c, float d) { return V{a, b, c, d}; }
    __device__ static inline void unpack(V v, float (&f)[4])
    {
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
};

// ---- tile configuration -----------------------------------------------------------------------
template <typename T_, int MT_, int WGM_, int WGN_, int TM_, int TN_, int BKB_, int STAGES_>
struct Tile {
    typedef T_ T;
    static constexpr int MT = MT_, WGM = WGM_, WGN = WGN_, TM = TM_, TN = TN_, BKB = BKB_, STAGES = STAGES_;
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
    static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
    static constexpr int LOAD_BYTES = STAGES * STAGE_BYTES;
    // the output tile is staged through LDS so that global stores are whole 16-byte runs
    static constexpr int EPI_ROWB = BN * (int)sizeof(T) + 16;
    static constexpr int EPI_BYTES = BM * EPI_ROWB;
    static constexpr int STATS_BYTES = kThreads * 2 * (int)sizeof(double);  // column-sum scratch behind the staged tile
    static constexpr int LDS_BYTES = cmax(LOAD_BYTES, EPI_BYTES + STATS_BYTES);
    // waves per SIMD the register allocation aims for (the LDS footprint allows as many workgroups)
    static constexpr int MIN_WAVES = (sizeof(T) == 2 && BM == 128 && BN == 128 && BKB == 64) ? 3 : 1;
    // forward / backward-data accumulate the transposed tile on the 32x32 MFMA (16 registers per lane = four
    // runs of 4 consecutive output channels, staged with four vector stores instead of sixteen element stores)
    static constexpr bool SWAP = MT == 32;
    static_assert(BKB % KSB == 0 && kThreads % CPR == 0 && (STAGES == 1 || STAGES == 2), "tile shape");
    static_assert(kThreads % BN == 0 && EPI_BYTES % 8 == 0, "column sums: whole row groups, aligned scratch");
};

// SWAP = false: acc[i][j] holds rows of A against columns of B (register e of a lane = row acc_row(lane, e),
// column lane % MT).  SWAP = true: the transposed tile (row = the B row acc_row(lane, e), column = the A row
// lane % MT), so that a lane holds runs of 4 consecutive B rows for one A row.
template <typename TL, bool SWAP = false>
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
            for (int j = 0; j < TL::TN; ++j) {
                if (SWAP)
                    Mma<typename TL::T, MT>::run(b[j], a[i], acc[i][j]);
                else
                    Mma<typename TL::T, MT>::run(a[i], b[j], acc[i][j]);
            }
    }
}

template <typename TL>
__device__ inline void zero_acc(typename Mma<typename TL::T, TL::MT>::Acc (&acc)[TL::TM][TL::TN])
{
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int j = 0; j < TL::TN; ++j)
#pragma unroll
            for (int e = 0; e < Mma<typename TL::T, TL::MT>::kAcc; ++e) acc[i][j][e] = 0.f;
}

// ---- forward / backward-data ------------------------------------------------------------------
// The gathered tensor `in` is N x Hi x Wi x Ci; output rows m = (n, ho, wo) over N x Ho x Wo.
// Tap (r, s) of output pixel (ho, wo) reads position t = o*ostride - pad + tap; with idil = 2
// (backward-data of a stride-2 conv) only even t exist and they map to source pixel t/2.

struct GatherGeom {
    int N, Hi, Wi, Ci, Ho, Wo, Co, R, S, pad_h, pad_w, ostride, idil;
    int M, Kdim;
    // Grouped convolution: Ci and Co above are the channels of ONE group (they shape the GEMM: Kdim = R*S*Ci, Co
    // columns); a pixel of `in` holds Cis = groups * Ci channels and a row of `out` Cos = groups * Co.  The group
    // is the launch's blockIdx.z.  Ungrouped: groups = 1, Cis = Ci, Cos = Co.
    int groups, Cis, Cos;
    int ci_shift;  // log2(Ci) if Ci is a power of two, else -1
    int s_inv;     // 65536 / S + 1: tap / S == (tap * s_inv) >> 16 for tap < 4096
    uint32_t wo_mul, wo_sh, ho_mul, ho_sh;  // m / Wo and (m / Wo) / Ho by multiplication (fast_div)
    int accum;     // add to `out` instead of overwriting it
    int out_vec;  // `out` rows can be written as whole 16-byte runs
    // Output row of tile row m = (n, ho, wo): pixel (n, ho * oh_mul + oh_off, wo * ow_mul + ow_off) of an N x OH x OW
    // map; oh_mul = 0 means the rows are simply consecutive (the usual case).  Backward-data of a stride-2
    // convolution runs as four dense problems, one per parity class of the input pixel, each writing its own pixels.
    int oh_mul, ow_mul, oh_off, ow_off, OH, OW;
    // if set: per row tile, the column sums {sum y, sum y^2} of the values as stored, [row tile][Co][2];
    // lets the batch norm that consumes `out` skip its own pass over the tensor
    double* stats;
    // A launch may carry a second instance of the same problem (same shapes and filters, other
    // tensors), selected by blockIdx.y: the forward pass of the current mini-batch and the recompute of
    // a stale one use the same parameters, so each layer serves both with one launch.
    const void* in1;
    void* out1;
    double* stats1;
};

// 16-byte loads through a buffer descriptor: the hardware returns zeros for any offset at or past
// `bytes`, so padding taps, rows past the end of the tensor and the k tail need no branch and no
// zero fill -- the lane just presents an out-of-range offset.
constexpr uint32_t kOutOfRange = 0xfffffff0u;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline u32x4 load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0));
}

// Row of `out` that tile row m is written to (see GatherGeom::oh_mul).
__device__ inline int64_t out_row(const GatherGeom& g, int m)
{
    if (g.oh_mul == 0) return m;
    const int t = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - t * g.Wo;
    const int n = (int)fast_div((uint32_t)t, g.ho_mul, g.ho_sh), ho = t - n * g.Ho;
    return ((int64_t)n * g.OH + ho * g.oh_mul + g.oh_off) * g.OW + wo * g.ow_mul + g.ow_off;
}

// Workgroups are handed to the 8 XCDs round-robin by workgroup id, and each XCD has an L2 of its own.
// Neighbouring tiles share input rows (halo rows, the rows a sweep over the output channels re-reads,
// the m slice all column tiles of a backward-weight read), so they should meet in one L2: logical
// tile = the position of this workgroup among the workgroups of its XCD, XCD by XCD.
__device__ inline unsigned xcd_tile(unsigned b, unsigned nb)
{
    const unsigned q = nb / 8, r = nb % 8, xcd = b % 8, idx = b / 8;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

template <typename TL, bool VEC, bool DIL>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(TL::MIN_WAVES))) void conv_gather_gemm_kernel(const typename TL::T* __restrict__ in_,
                                                                    const typename TL::T* __restrict__ wgt,
                                                                    typename TL::T* __restrict__ out_, GatherGeom g)
{
    typedef typename TL::T T;
    constexpr int E = TL::E, CPR = TL::CPR, ROWS_PER_PASS = kThreads / CPR;
    constexpr uint32_t SZ = sizeof(T);
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const T* __restrict__ in = blockIdx.y ? (const T*)g.in1 : in_;
    T* __restrict__ out = blockIdx.y ? (T*)g.out1 : out_;
    double* stats = blockIdx.y ? g.stats1 : g.stats;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    // consecutive workgroups share the same rows of `in` and sweep the output channels
    const int tiles_n = (g.Co + TL::BN - 1) / TL::BN;
    const unsigned tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / tiles_n) * TL::BM, n0 = (tile % tiles_n) * TL::BN;
    // grouped convolution: this workgroup's group reads channels [in_c0, in_c0 + Ci) of rows Cis wide and writes
    // channels [out_c0, out_c0 + Co) of rows Cos wide, with the filters of output channels out_c0 ..
    const int in_c0 = blockIdx.z * g.Ci, out_c0 = blockIdx.z * g.Co;

    const int kc = tid % CPR;    // which 16-byte run of the k tile this thread moves
    const int row0 = tid / CPR;  // first tile row it moves; further rows are +ROWS_PER_PASS apart
    // backward-data of a stride-2 convolution: fixed at compile time on the vector path, a run-time
    // test on the element-wise path
    const bool dil = VEC ? DIL : g.idil == 2;
    constexpr bool masked = VEC && !DIL;  // plain vector path: per-row tap masks

    // Per-row gather state of the A operand (byte offsets modulo 2^32; tensors are < 4 GB, checked on the host).
    //   masked:    a_off = byte offset of pixel (ho*ostride - pad_h, wo*ostride - pad_w) of the row's image
    //              (may lie before the tensor), a_aux = bit (r*S + s) set iff tap (r, s) falls inside the image
    //   otherwise: a_off = byte offset of the row's image, a_aux = th0 (low half) | tw0 (high half)
    uint32_t a_off[TL::A_PER], a_aux[TL::A_PER];
    uint32_t a_hi[TL::A_PER];  // masked: taps 32..63 (filters larger than 32 taps, e.g. 7x7)
#pragma unroll
    for (int i = 0; i < TL::A_PER; ++i) {
        const int row = row0 + i * ROWS_PER_PASS;
        const int m = m0 + row;
        a_off[i] = 0;
        a_hi[i] = 0;
        a_aux[i] = masked ? 0u : 0x80008000u;  // nothing valid
        if (row < TL::BM && m < g.M) {
            const int t = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - t * g.Wo;
            const int n = (int)fast_div((uint32_t)t, g.ho_mul, g.ho_sh), ho = t - n * g.Ho;
            const int th0 = ho * g.ostride - g.pad_h, tw0 = wo * g.ostride - g.pad_w;
            const uint32_t img = ((uint32_t)n * g.Hi * g.Wi * g.Cis + in_c0) * SZ;
            if (masked) {
                // taps s in [s_lo, s_hi) of a filter row fall inside the image; the same bits for every valid row r
                const int s_lo = tw0 < 0 ? -tw0 : 0, s_hi = g.Wi - tw0 < g.S ? g.Wi - tw0 : g.S;
                const uint64_t cols = s_hi > s_lo ? ((1ull << s_hi) - 1) & ~((1ull << s_lo) - 1) : 0ull;
                uint64_t mask = 0;
                for (int r = 0; r < g.R; ++r)
                    if (th0 + r >= 0 && th0 + r < g.Hi) mask |= cols << (r * g.S);
                a_off[i] = img + (uint32_t)((th0 * g.Wi + tw0) * g.Cis) * SZ;
                a_aux[i] = (uint32_t)mask;
                a_hi[i] = (uint32_t)(mask >> 32);
            } else {
                a_off[i] = img;
                a_aux[i] = ((uint32_t)th0 & 0xffffu) | ((uint32_t)tw0 << 16);
            }
        }
    }
    uint32_t b_off[TL::B_PER];
#pragma unroll
    for (int i = 0; i < TL::B_PER; ++i) {
        const int row = row0 + i * ROWS_PER_PASS, co = n0 + row;
        b_off[i] = (row < TL::BN && co < g.Co) ? (uint32_t)((out_c0 + co) * g.Kdim) * SZ : kOutOfRange;
    }
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(in, (uint32_t)g.N * g.Hi * g.Wi * g.Cis * SZ);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(wgt, (uint32_t)gridDim.z * g.Co * g.Kdim * SZ);

    // k position of this thread's run in k tile kt: element kk = kt*BK + kc*E = (kr*S + ks)*Ci + kci
    const T zero = from_float<T>(0.f);
    struct KPos {
        int kk, kr, ks, kci;
    };
    auto k_position = [&](int kt) -> KPos {
        KPos p;
        p.kk = kt * TL::BK + kc * E;
        int tap;
        if (g.ci_shift >= 0) {
            tap = p.kk >> g.ci_shift;
            p.kci = p.kk & (g.Ci - 1);
        } else {
            tap = p.kk / g.Ci;
            p.kci = p.kk - tap * g.Ci;
        }
        p.kr = (tap * g.s_inv) >> 16;
        p.ks = tap - p.kr * g.S;
        return p;
    };

    // byte offset of tap (r, s), channel ci of the row described by (off, aux), or kOutOfRange  [unmasked rows]
    auto tap_offset = [&](uint32_t off, uint32_t aux, int r, int s, int ci) -> uint32_t {
        int th = (int)(int16_t)(aux & 0xffffu) + r, tw = (int)(int16_t)(aux >> 16) + s;
        bool ok = th >= 0 && tw >= 0;
        if (dil) {
            ok = ok && ((th | tw) & 1) == 0;
            th >>= 1;
            tw >>= 1;
        }
        ok = ok && th < g.Hi && tw < g.Wi;
        return ok ? off + (uint32_t)((th * g.Wi + tw) * g.Cis + ci) * SZ : kOutOfRange;
    };

    // global -> registers: the runs of k tile kt (zeros past the end of k, for padding taps and rows past M)
    auto load_tiles = [&](int kt, u32x4 (&ra)[TL::A_PER], u32x4 (&rb)[TL::B_PER]) {
        const KPos p = k_position(kt);
        if (VEC) {
            const bool k_ok = p.kk < g.Kdim;
            if (!dil) {
                const uint32_t tap_off = (uint32_t)((p.kr * g.Wi + p.ks) * g.Cis + p.kci) * SZ;
                const int tap = p.kr * g.S + p.ks;
#pragma unroll
                for (int i = 0; i < TL::A_PER; ++i) {
                    const uint32_t bits = tap < 32 ? a_aux[i] >> tap : a_hi[i] >> (tap - 32);
                    const bool ok = k_ok && (bits & 1u) != 0;
                    ra[i] = load16(rin, ok ? a_off[i] + tap_off : kOutOfRange);
                }
            } else {
#pragma unroll
                for (int i = 0; i < TL::A_PER; ++i)
                    ra[i] = load16(rin, k_ok ? tap_offset(a_off[i], a_aux[i], p.kr, p.ks, p.kci) : kOutOfRange);
            }
            const uint32_t kkb = (uint32_t)p.kk * SZ;
#pragma unroll
            for (int i = 0; i < TL::B_PER; ++i)
                rb[i] = load16(rw, (k_ok && b_off[i] != kOutOfRange) ? b_off[i] + kkb : kOutOfRange);
        } else {
            // generic path (channel count not a multiple of the 16-byte run, unaligned bases, huge filters)
#pragma unroll
            for (int i = 0; i < TL::A_PER; ++i) {
                alignas(16) T tmp[E];
                for (int e = 0; e < E; ++e) {
                    const int k = p.kk + e;
                    const int tap = k / g.Ci, ci = k % g.Ci;
                    const uint32_t o = k < g.Kdim ? tap_offset(a_off[i], a_aux[i], tap / g.S, tap % g.S, ci) : kOutOfRange;
                    tmp[e] = o != kOutOfRange ? in[o / SZ] : zero;
                }
                ra[i] = *(const u32x4*)tmp;
            }
#pragma unroll
            for (int i = 0; i < TL::B_PER; ++i) {
                alignas(16) T tmp[E];
                for (int e = 0; e < E; ++e)
                    tmp[e] = (b_off[i] != kOutOfRange && p.kk + e < g.Kdim) ? wgt[b_off[i] / SZ + p.kk + e] : zero;
                rb[i] = *(const u32x4*)tmp;
            }
        }
    };
    // registers -> LDS stage `buf`
    auto store_tiles = [&](int buf, const u32x4 (&ra)[TL::A_PER], const u32x4 (&rb)[TL::B_PER]) {
        char* sA = smem + buf * TL::STAGE_BYTES;
        char* sB = sA + TL::BM * TL::ROWB;
#pragma unroll
        for (int i = 0; i < TL::A_PER; ++i) {
            const int row = row0 + i * ROWS_PER_PASS;
            if (TL::A_CHUNKS % kThreads == 0 || row < TL::BM) *(u32x4*)(sA + row * TL::ROWB + kc * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < TL::B_PER; ++i) {
            const int row = row0 + i * ROWS_PER_PASS;
            if (TL::B_CHUNKS % kThreads == 0 || row < TL::BN) *(u32x4*)(sB + row * TL::ROWB + kc * 16) = rb[i];
        }
    };

    typename Mma<T, TL::MT>::Acc acc[TL::TM][TL::TN];
    zero_acc<TL>(acc);

    const int nk = (g.Kdim + TL::BK - 1) / TL::BK;
    u32x4 ra0[TL::A_PER], rb0[TL::B_PER];
    if (TL::STAGES == 2) {
        // Two LDS stages and two register sets: while k tile kt is multiplied out of one LDS stage, tile
        // kt+1 moves from registers into the other stage and the gathers of tile kt+2 are in flight, so
        // a gather has two multiply phases to arrive.  (Loads past the last tile read zeros and are dropped.)
        u32x4 ra1[TL::A_PER], rb1[TL::B_PER];
        load_tiles(0, ra0, rb0);
        store_tiles(0, ra0, rb0);
        load_tiles(1, ra0, rb0);
        __syncthreads();
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {  // one loop body, one back edge: the accumulators stay where the MFMAs want them
            load_tiles(kt + 2, ra1, rb1);
            mma_tile<TL, TL::SWAP>(smem, smem + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
            store_tiles(1, ra0, rb0);
            __syncthreads();
            load_tiles(kt + 3, ra0, rb0);
            mma_tile<TL, TL::SWAP>(smem + TL::STAGE_BYTES, smem + TL::STAGE_BYTES + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
            store_tiles(0, ra1, rb1);
            __syncthreads();
        }
        if (kt < nk) {  // odd number of k tiles: the last one sits in stage 0
            mma_tile<TL, TL::SWAP>(smem, smem + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
            __syncthreads();
        }
    } else {
        load_tiles(0, ra0, rb0);
        for (int kt = 0; kt < nk; ++kt) {
            if (kt > 0) __syncthreads();  // every wave has finished reading the previous tile
            store_tiles(0, ra0, rb0);
            __syncthreads();
            if (kt + 1 < nk) load_tiles(kt + 1, ra0, rb0);  // the next tile's gathers fly while this one is multiplied
            mma_tile<TL, TL::SWAP>(smem, smem + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
        }
        __syncthreads();
    }

    // ---- epilogue: (optionally add the old values,) stage the tile in LDS, store 16-byte runs ----
    constexpr int kAcc = Mma<T, TL::MT>::kAcc;
    if constexpr (TL::SWAP) {
        // The accumulators hold the transposed tile: a lane has, for output row lane % MT of its block, runs of
        // 4 consecutive output channels (registers 4q .. 4q+3), which go to LDS as one 8- or 16-byte store.
        typedef typename Run4<T>::V RunV;
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int j = 0; j < TL::TN; ++j) {
                const int lrow = (wave_m * TL::TM + i) * TL::MT + lane % TL::MT;
                const int m = m0 + lrow;
#pragma unroll
                for (int q = 0; q < kAcc / 4; ++q) {
                    const int lcol = (wave_n * TL::TN + j) * TL::MT + acc_row<TL::MT>(lane, 4 * q);
                    const int col = n0 + lcol;
                    if (g.accum && m < g.M) {
                        const T* old = out + out_row(g, m) * g.Cos + out_c0 + col;
                        if (g.out_vec && col + 4 <= g.Co) {
                            float o[4];
                            Run4<T>::unpack(*(const RunV*)old, o);
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += o[e];
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < g.Co) acc[i][j][4 * q + e] += to_float<T>(old[e]);
                        }
                    }
                    *(RunV*)(smem + lrow * TL::EPI_ROWB + lcol * (int)sizeof(T)) =
                        Run4<T>::pack(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                }
            }
    } else {
        if (g.accum) {
#pragma unroll
            for (int i = 0; i < TL::TM; ++i)
#pragma unroll
                for (int j = 0; j < TL::TN; ++j) {
                    const int col = n0 + (wave_n * TL::TN + j) * TL::MT + lane % TL::MT;
#pragma unroll
                    for (int e = 0; e < kAcc; ++e) {
                        const int m = m0 + (wave_m * TL::TM + i) * TL::MT + acc_row<TL::MT>(lane, e);
                        if (m < g.M && col < g.Co) acc[i][j][e] += to_float<T>(out[out_row(g, m) * g.Cos + out_c0 + col]);
                    }
                }
        }
#pragma unroll
        for (int i = 0; i < TL::TM; ++i)
#pragma unroll
            for (int j = 0; j < TL::TN; ++j) {
                const int lcol = (wave_n * TL::TN + j) * TL::MT + lane % TL::MT;
#pragma unroll
                for (int e = 0; e < kAcc; ++e) {
                    const int lrow = (wave_m * TL::TM + i) * TL::MT + acc_row<TL::MT>(lane, e);
                    *(T*)(smem + lrow * TL::EPI_ROWB + lcol * (int)sizeof(T)) = from_float<T>(acc[i][j][e]);
                }
            }
    }
    __syncthreads();
    constexpr int OCPR = TL::BN / E;  // 16-byte runs per tile row
    for (int c = tid; c < TL::BM * OCPR; c += kThreads) {
        const int lrow = c / OCPR, cc = (c % OCPR) * E;
        const int m = m0 + lrow, col = n0 + cc;
        if (m >= g.M || col >= g.Co) continue;
        const char* src = smem + lrow * TL::EPI_ROWB + cc * (int)sizeof(T);
        T* dst = out + out_row(g, m) * g.Cos + out_c0 + col;
        if (g.out_vec && col + E <= g.Co) {
            *(u32x4*)dst = *(const u32x4*)src;
        } else {
            for (int e = 0; e < E && col + e < g.Co; ++e) dst[e] = ((const T*)src)[e];
        }
    }
    if (stats) {
        // column sums of the staged tile (rows past M hold zeros): thread = (row group, column)
        constexpr int G = kThreads / TL::BN;
        const int c = tid % TL::BN, rg = tid / TL::BN;
        float s0 = 0.f, s1 = 0.f;
        for (int r = rg; r < TL::BM; r += G) {
            const float v = to_float<T>(*(const T*)(smem + r * TL::EPI_ROWB + c * (int)sizeof(T)));
            s0 += v;
            s1 += v * v;
        }
        double* sred = (double*)(smem + TL::EPI_BYTES);
        sred[(rg * TL::BN + c) * 2] = (double)s0;
        sred[(rg * TL::BN + c) * 2 + 1] = (double)s1;
        __syncthreads();
        if (rg == 0 && n0 + c < g.Co) {
            double a = 0.0, b = 0.0;
#pragma unroll
            for (int k = 0; k < G; ++k) {
                a += sred[(k * TL::BN + c) * 2];
                b += sred[(k * TL::BN + c) * 2 + 1];
            }
            double* dst = stats + ((int64_t)(tile / tiles_n) * g.Cos + out_c0 + n0 + c) * 2;
            dst[0] = a;
            dst[1] = b;
        }
    }
}

// ---- bf16 gather-GEMM fed by direct global -> LDS loads ---------------------------------------------
// For bf16 layers whose gathered channel count is a multiple of 64 (every 64-element k tile then lies inside one
// filter tap) the operands need no detour through registers: `buffer_load ... lds` moves 16 bytes per lane from
// memory straight into LDS.  A load instruction of one wave fills 1 KB of LDS contiguously (lane l -> bytes
// 16 l .. 16 l + 15), i.e. 8 tile rows of 128 bytes, so rows cannot be padded; instead the 16-byte chunk c of row R
// is kept at position c ^ ((R >> 1) & 7) of its row -- the lane that owns position p of row R simply fetches chunk
// p ^ ((R >> 1) & 7) -- which spreads the 16 rows a group of 16 lanes reads over all 64 banks.  Three LDS stages:
// while k tile t is multiplied, tile t+1 has landed or is landing and the loads of tile t+2 are issued, so a
// gather has two multiply phases to arrive and no vector register or LDS-write instruction is spent on it.
// A 256-thread workgroup owns BM x BN outputs (256 x 128: each of the 2 x 2 waves a 128 x 64 sub-tile = 4 x 2
// MFMA tiles of 32 x 32, 6 LDS operand reads per 8 MFMAs).  Per k tile the tap and the channel offset are uniform,
// so a lane's address is (row base + uniform tap offset) or "out of range" (padding tap / row past M: the buffer
// load then writes zeros).
template <int BM_, int BN_, int WGM_, int WGN_, int BKB_, int STAGES_, int WAVES_ = 1>
struct DmaTile {
    static constexpr int WAVES = WAVES_;  // waves per SIMD the register allocation aims for (workgroups per compute unit)
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, STAGES = STAGES_;
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    static constexpr int TM = BM / (WGM * 32), TN = BN / (WGN * 32);
    static constexpr int ROWB = BKB_;                      // bytes of k per row: 64 or 32 bf16
    static constexpr int BK = ROWB / 2;
    static constexpr int CPR = ROWB / 16;                  // 16-byte chunks per row
    static constexpr int RPG = 1024 / ROWB;                // rows per 1 KB load instruction
    static constexpr int NKS = ROWB / 32;                  // MFMA k steps (16 elements) per tile
    static constexpr int A_G = BM / RPG / 4, B_G = BN / RPG / 4;  // load instructions per wave and tile
    static constexpr int STAGE_BYTES = (BM + BN) * ROWB;
    static constexpr int EPI_ROWB = BN * 2 + 16;
    static constexpr int EPI_BYTES = BM * EPI_ROWB;
    static constexpr int STATS_BYTES = kThreads * 2 * (int)sizeof(double);
    static constexpr int LDS_BYTES = cmax(STAGES * STAGE_BYTES, EPI_BYTES + STATS_BYTES);
    static_assert((ROWB == 128 || ROWB == 64) && BM % (4 * RPG) == 0 && BN % (4 * RPG) == 0 && kThreads % BN == 0 &&
                      STAGES >= 3 && LDS_BYTES <= 160 * 1024, "tile shape");
    // chunk c of row R sits at position c ^ swz(R) of its row: the 16 rows a group of 16 lanes reads (same c) then
    // fall on 16 different 16-byte bank groups of the 64 banks
    __device__ static inline int swz(int R) { return ROWB == 128 ? (R >> 1) & 7 : (R >> 2) & 3; }
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ inline void dma16(__amdgpu_buffer_rsrc_t r, char* lds_wave_base, uint32_t byte_off)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr_t)lds_wave_base, 16, (int)byte_off, 0, 0, 0);
}

template <typename TL>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(TL::WAVES, TL::WAVES))) void conv_dma_gemm_kernel(
    const bf16_t* __restrict__ in_, const bf16_t* __restrict__ wgt, bf16_t* __restrict__ out_, GatherGeom g)
{
    typedef bf16_t T;
    constexpr int BM = TL::BM, BN = TL::BN, TM = TL::TM, TN = TL::TN, NKS = TL::NKS, ST = TL::STAGES;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const T* __restrict__ in = blockIdx.y ? (const T*)g.in1 : in_;
    T* __restrict__ out = blockIdx.y ? (T*)g.out1 : out_;
    double* stats = blockIdx.y ? g.stats1 : g.stats;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    const int tiles_n = (g.Co + BN - 1) / BN;
    const unsigned tile = xcd_tile(blockIdx.x, gridDim.x);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    // loader state: this lane owns position (lane % CPR) of row (lane / CPR) of each 1 KB row group of its wave
    const int lrow = lane / TL::CPR, lpos = lane % TL::CPR;
    uint32_t a_base[TL::A_G], a_mask[TL::A_G], b_base[TL::B_G];
#pragma unroll
    for (int i = 0; i < TL::A_G; ++i) {
        const int row = (wave * TL::A_G + i) * TL::RPG + lrow, m = m0 + row;
        const uint32_t chunk = (uint32_t)(lpos ^ TL::swz(row));
        a_base[i] = 0;
        a_mask[i] = 0;
        if (m < g.M) {
            const int t = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - t * g.Wo;
            const int n = (int)fast_div((uint32_t)t, g.ho_mul, g.ho_sh), ho = t - n * g.Ho;
            const int th0 = ho * g.ostride - g.pad_h, tw0 = wo * g.ostride - g.pad_w;
            const int s_lo = tw0 < 0 ? -tw0 : 0, s_hi = g.Wi - tw0 < g.S ? g.Wi - tw0 : g.S;
            const uint32_t cols = s_hi > s_lo ? ((1u << s_hi) - 1) & ~((1u << s_lo) - 1) : 0u;
            uint32_t mask = 0;
            for (int r = 0; r < g.R; ++r)
                if (th0 + r >= 0 && th0 + r < g.Hi) mask |= cols << (r * g.S);
            a_mask[i] = mask;
            a_base[i] = (uint32_t)n * g.Hi * g.Wi * g.Ci * 2u + (uint32_t)((th0 * g.Wi + tw0) * g.Ci) * 2u + chunk * 16u;
        }
    }
#pragma unroll
    for (int i = 0; i < TL::B_G; ++i) {
        const int row = (wave * TL::B_G + i) * TL::RPG + lrow, co = n0 + row;
        const uint32_t chunk = (uint32_t)(lpos ^ TL::swz(row));
        b_base[i] = co < g.Co ? (uint32_t)(co * g.Kdim) * 2u + chunk * 16u : kOutOfRange;
    }
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(in, (uint32_t)g.N * g.Hi * g.Wi * g.Ci * 2u);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(wgt, (uint32_t)g.Co * g.Kdim * 2u);

    const int nk = g.Kdim / TL::BK;
    const int tiles_per_tap = g.Ci / TL::BK;
    // position of the k tile whose loads are issued next (all uniform)
    int l_kt = 0, l_tap = 0, l_r = 0, l_s = 0, l_c = 0;
    auto issue_loads = [&](int stage) {
        char* sA = smem + stage * TL::STAGE_BYTES + wave * (TL::A_G * 1024);
        char* sB = smem + stage * TL::STAGE_BYTES + BM * TL::ROWB + wave * (TL::B_G * 1024);
        const bool live = l_kt < nk;
        const uint32_t tap_off = (uint32_t)((l_r * g.Wi + l_s) * g.Ci + l_c * TL::BK) * 2u;
        const uint32_t tap_bit = live ? (1u << l_tap) : 0u;
#pragma unroll
        for (int i = 0; i < TL::A_G; ++i)
            dma16(rin, sA + i * 1024, (a_mask[i] & tap_bit) ? a_base[i] + tap_off : kOutOfRange);
        const uint32_t kb = (uint32_t)l_kt * (uint32_t)TL::ROWB;
#pragma unroll
        for (int i = 0; i < TL::B_G; ++i)
            dma16(rw, sB + i * 1024, (live && b_base[i] != kOutOfRange) ? b_base[i] + kb : kOutOfRange);
        ++l_kt;
        if (++l_c == tiles_per_tap) {
            l_c = 0;
            ++l_tap;
            if (++l_s == g.S) {
                l_s = 0;
                ++l_r;
            }
        }
    };

    typename Mma<T, 32>::Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand reads: lane (frow, fg) takes row frow of every 32-row MFMA block and the 16-byte k chunk 2 ks + fg
    const int frow = lane & 31, fg = lane >> 5, swl = TL::swz(frow);
    int koff[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = ((2 * ks + fg) ^ swl) << 4;
    const int a_row_off = (wave_m * TM * 32 + frow) * TL::ROWB;
    const int b_row_off = BM * TL::ROWB + (wave_n * TN * 32 + frow) * TL::ROWB;
    auto read_frags = [&](const char* s, int ks, u32x4 (&a)[TM], u32x4 (&b)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *(const u32x4*)(s + a_row_off + i * 32 * TL::ROWB + koff[ks]);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[j] = *(const u32x4*)(s + b_row_off + j * 32 * TL::ROWB + koff[ks]);
    };
    auto mfmas = [&](const u32x4 (&a)[TM], const u32x4 (&b)[TN]) {
        __builtin_amdgcn_sched_barrier(0);  // the reads of the next step are issued before this step's MFMAs, not among them
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) Mma<T, 32>::run(b[j], a[i], acc[i][j]);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Synchronisation by hand (__syncthreads() would make every wave wait for ALL its outstanding loads at every
    // barrier).  ST stages: tiles kt .. kt + ST - 2 are in LDS or on their way, tile kt + ST - 1 is issued during
    // tile kt.  One barrier per k tile, in the MIDDLE of the tile's k steps: by then the loads of tile kt + 1 have
    // landed -- each wave waits until only its loads of the later tiles are outstanding, the barrier makes them
    // visible to all -- and every wave has finished reading tile kt - 1, whose stage the loads issued right after
    // the barrier overwrite.  The operands of a tile's first k step are read during the last k step of the tile
    // before, so no wave meets the barrier and a burst of LDS reads at the same moment.
    constexpr int LOADS = TL::A_G + TL::B_G;      // loads one wave issues per k tile
    constexpr int AHEAD = (ST - 3) * LOADS;       // loads that may stay outstanding at the barrier
#pragma unroll
    for (int t = 0; t < ST - 1; ++t) issue_loads(t);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((ST - 2) * LOADS) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    u32x4 fa[2][TM], fb[2][TN];
    read_frags(smem, 0, fa[0], fb[0]);
    int st = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const char* s = smem + st * TL::STAGE_BYTES;
        int st1 = st + 1;
        if (st1 == ST) st1 = 0;
        int stl = st - 1;        // the stage of tile kt - 1 = the stage of tile kt + ST - 1
        if (stl < 0) stl = ST - 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (ks + 1 < NKS)
                read_frags(s, ks + 1, fa[(ks + 1) & 1], fb[(ks + 1) & 1]);
            else
                read_frags(smem + st1 * TL::STAGE_BYTES, 0, fa[0], fb[0]);
            mfmas(fa[ks & 1], fb[ks & 1]);
            if (ks == NKS / 2 - 1) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(AHEAD) : "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                issue_loads(stl);   // tile kt + ST - 1 (zeros past the end) replaces tile kt - 1
            }
        }
        st = st1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the zero loads past the end must not land in the staged output tile
    __syncthreads();

    // ---- epilogue: the accumulators hold the transposed tile (a lane has, for output row lane % 32 of its block,
    // runs of 4 consecutive output channels); stage it in LDS, then store 16-byte runs ----
    typedef typename Run4<T>::V RunV;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int lr = (wave_m * TM + i) * 32 + (lane & 31);
            const int m = m0 + lr;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int lcol = (wave_n * TN + j) * 32 + acc_row<32>(lane, 4 * q);
                const int col = n0 + lcol;
                if (g.accum && m < g.M) {
                    if (g.out_vec && col + 4 <= g.Co) {
                        float o[4];
                        Run4<T>::unpack(*(const RunV*)(out + (int64_t)m * g.Co + col), o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[i][j][4 * q + e] += o[e];
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < g.Co) acc[i][j][4 * q + e] += to_float<T>(out[(int64_t)m * g.Co + col + e]);
                    }
                }
                *(RunV*)(smem + lr * TL::EPI_ROWB + lcol * 2) =
                    Run4<T>::pack(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            }
        }
    __syncthreads();
    constexpr int OCPR = BN / 8;  // 16-byte runs per tile row
    for (int c = tid; c < BM * OCPR; c += kThreads) {
        const int lr = c / OCPR, cc = (c % OCPR) * 8;
        const int m = m0 + lr, col = n0 + cc;
        if (m >= g.M || col >= g.Co) continue;
        const char* src = smem + lr * TL::EPI_ROWB + cc * 2;
        T* dst = out + (int64_t)m * g.Co + col;
        if (g.out_vec && col + 8 <= g.Co) {
            *(u32x4*)dst = *(const u32x4*)src;
        } else {
            for (int e = 0; e < 8 && col + e < g.Co; ++e) dst[e] = ((const T*)src)[e];
        }
    }
    if (stats) {
        // column sums of the staged tile (rows past M hold zeros): thread = (row group, column)
        constexpr int G = kThreads / BN;
        const int c = tid % BN, rg = tid / BN;
        float s0 = 0.f, s1 = 0.f;
        for (int r = rg; r < BM; r += G) {
            const float v = to_float<T>(*(const T*)(smem + r * TL::EPI_ROWB + c * 2));
            s0 += v;
            s1 += v * v;
        }
        double* sred = (double*)(smem + TL::EPI_BYTES);
        sred[(rg * BN + c) * 2] = (double)s0;
        sred[(rg * BN + c) * 2 + 1] = (double)s1;
        __syncthreads();
        if (rg == 0 && n0 + c < g.Co) {
            double a = 0.0, b = 0.0;
#pragma unroll
            for (int k = 0; k < G; ++k) {
                a += sred[(k * BN + c) * 2];
                b += sred[(k * BN + c) * 2 + 1];
            }
            double* dst = stats + ((int64_t)(tile / tiles_n) * g.Co + n0 + c) * 2;
            dst[0] = a;
            dst[1] = b;
        }
    }
}

// ---- bf16 3x3 / stride 1 / pad 1 convolutions with 64 channels on both sides, filters held in registers ----
// The contraction is 576 long and only 64 wide, so the whole filter bank (64 x 576 bf16 = 72 KB) fits the register
// files of a workgroup's four waves: each wave keeps ALL of it as MFMA operand fragments (36 k steps x 2 blocks of 32
// output channels x 4 registers = 288 registers per lane, one wave per SIMD) for the life of a persistent workgroup,
// and LDS only carries the pixels.  Those are not staged as an im2col tile either: the input rows a tile of 256
// consecutive output pixels needs (its image rows plus one above and below, one zero column left and right) go into LDS
// ONCE, as they lie in memory, and the fragment of tap (r, s) is read at the shifted address -- the nine-fold
// expansion happens in the LDS read.  Per k step a wave reads 2 fragments for 4 MFMAs (64 B/clk per compute unit,
// against 128 for the register-staged 256x64 tile, which is what bound that tile).  The rows of the NEXT tile are
// fetched into registers before the k loop and written to the other patch buffer during its last steps (15 16-byte
// chunks per lane).  (Direct global -> LDS loads were built first and measured: a wave's LDS reads queue behind its
// own outstanding direct loads, so the k loop stood still until the next tile had landed.)
//   patch pixel pp = prow * 64 + pcol (rows of 64 pixels; 51 <= W <= 62, so a tile touches at most 8 flat rows) holds
//   input pixel (flat row R0 + prow, column pcol - 1), flat row = n * H + h; its 128 bytes keep the 16-byte chunk c
//   at position c ^ (((prow * W + pcol) >> 1) & 7), so that the 16 consecutive pixels a group of 16 lanes reads (same
//   c) fall on 16 different bank groups -- also where the run of pixels wraps from the end of one image row to the
//   start of the next (prow * W + pcol goes on counting there; more than half of the 32-pixel blocks hold such a wrap).  Lane tid moves position tid & 7 of the columns (tid >> 3) and (tid >> 3) + 32 of every
//   row: its two column offsets are fixed, the row offset is uniform, so a fetch costs two vector instructions.
// A tap row that belongs to another image (h + r - 1 outside [0, H)) is a per-lane matter (the same flat row is data
// for one output row and padding for the next image's): such lanes read from a 512-byte zero region instead.
// The MFMA computes the transposed tile (filters as the first operand), so a lane ends up with runs of 4 consecutive
// output channels of one pixel; the tile is staged through the patch buffer just multiplied and stored as 16-byte
// runs, with the column sums for a following batch norm taken from the staged values.
struct C64Args {
    int buf_bytes;       // bytes of one patch buffer (>= kC64Chunks * 4 KB and >= the staged output tile + column-sum scratch)
    int tiles;           // row tiles of 256 output pixels per problem instance
    int twin;            // 1: a second problem instance (in1 / out1 / stats1)
};
// Workgroup w of W walks the consecutive tiles [w * tiles / W, (w + 1) * tiles / W) of the first instance (neighbouring
// tiles share input rows: same L2, soon after) and then, in a twin launch, the range of workgroup W - 1 - w in the second
// instance (ranges differ by one tile; pairing a long one with a short one evens the work out).  The column sums for a
// following batch norm are kept per thread across a whole range and leave as ONE partial row per workgroup and
// instance: row w of the first instance's sums, row W - 1 - w of the second's.
constexpr int kC64Zero = 512;    // zero region at the start of LDS
constexpr int kC64EpiRowB = 64 * 2 + 16;
constexpr int kC64Chunks = 16;   // 16-byte chunks of a patch per lane: 8 rows of 64 pixels
constexpr int kC64Pitch = 64;    // pixels per patch row

// Barrier for phases that only exchange data through LDS stores: waits for this wave's LDS operations, not for its
// outstanding vector-memory operations (the next tile's loads and the previous tile's stores stay in flight).
__device__ inline void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <bool ACCUM>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void conv3x3_c64_bf16_kernel(
    const bf16_t* __restrict__ in_, const bf16_t* __restrict__ wgt, bf16_t* __restrict__ out_, GatherGeom g, C64Args a)
{
    typedef bf16_t T;
    constexpr int BM = 256, C = 64, NKS = 36, NCH = kC64Chunks, WR0 = NKS - NCH;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fg = lane >> 5;
    const int W = g.Wi, H = g.Hi;
    constexpr int W2 = kC64Pitch;

    // the filter bank as first-operand fragments: lane (frow, fg) holds, for output channel 32 j + frow, the
    // k elements 16 t + 8 fg .. + 7
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(wgt, (uint32_t)(C * 9 * C) * 2u);
    u32x4 wf[NKS][2];
#pragma unroll
    for (int t = 0; t < NKS; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) wf[t][j] = load16(rw, (uint32_t)(((32 * j + frow) * (9 * C)) + 16 * t + 8 * fg) * 2u);
    // the filters are complete before the tile loop starts (otherwise the compiler keeps counting on their loads inside
    // the loop, and its waits there would also drain the prefetch of the next tile)
#pragma unroll
    for (int t = 0; t < NKS; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) asm volatile("" ::"v"(wf[t][j]));

    if (tid < kC64Zero / 16) *(u32x4*)(smem + tid * 16) = u32x4{0u, 0u, 0u, 0u};
    const uint32_t in_bytes = (uint32_t)g.N * H * W * C * 2u;
    const __amdgpu_buffer_rsrc_t rin0 = make_rsrc(in_, in_bytes);
    const __amdgpu_buffer_rsrc_t rin1 = make_rsrc(g.in1 ? g.in1 : in_, in_bytes);

    const int nw = (int)gridDim.x, w1 = nw - 1 - (int)blockIdx.x;
    auto range_lo = [&](int w) { return (int)((int64_t)w * a.tiles / nw); };
    const int b0 = range_lo((int)blockIdx.x), n0 = range_lo((int)blockIdx.x + 1) - b0;
    const int b1 = range_lo(w1), n1 = a.twin ? range_lo(w1 + 1) - b1 : 0;
    const int n_steps = n0 + n1;
    auto tile_at = [&](int s) { return s < n0 ? b0 + s : a.tiles + b1 + (s - n0); };  // second instance: tiles + its row tile

    // the input rows of tile t, 16 chunks per lane: chunk i = position tid & 7 of patch pixel (row i >> 1, column
    // (tid >> 3) + 32 (i & 1)); zeros for the border columns, for rows outside the tensor and past the rows the tile touches
    uint32_t col_off[2];
    bool col_ok[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int pcol = (tid >> 3) + 32 * h, wi = pcol - 1;
        col_ok[h] = wi >= 0 && wi < W;
        col_off[h] = (uint32_t)(wi * C) * 2u;
    }
    auto fetch_patch = [&](int t, u32x4 (&pre)[NCH]) {
        const int inst = t >= a.tiles ? 1 : 0;
        const int m0 = (t - inst * a.tiles) * BM;
        const int tq = (int)fast_div((uint32_t)m0, g.wo_mul, g.wo_sh);  // flat output row of the tile's first pixel
        const int m_last = min(m0 + BM, g.M) - 1;
        const int R0 = tq - 1;
        const int rows = (int)fast_div((uint32_t)m_last, g.wo_mul, g.wo_sh) - tq + 3;  // the rows this tile touches
        const __amdgpu_buffer_rsrc_t rin = inst ? rin1 : rin0;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int prow = i >> 1, row = R0 + prow;
            const bool row_ok = prow < rows && row >= 0 && row < g.N * H;   // uniform
            const uint32_t row_off = (uint32_t)(row * W * C) * 2u;           // uniform
            // the chunk that belongs at this lane's position of patch pixel (prow, pcol): position ^ key(prow * W + pcol)
            const uint32_t key = ((uint32_t)(prow * W + (tid >> 3) + 32 * (i & 1)) >> 1) & 7u;
            const uint32_t chunk = ((uint32_t)(tid & 7) ^ key) << 4;
            pre[i] = load16(rin, (row_ok && col_ok[i & 1]) ? row_off + col_off[i & 1] + chunk : kOutOfRange);
        }
    };

    u32x4 pre[NCH];
    if (n_steps > 0) {
        fetch_patch(tile_at(0), pre);
#pragma unroll
        for (int i = 0; i < NCH; ++i) *(u32x4*)(smem + kC64Zero + (tid + kThreads * i) * 16) = pre[i];
    }
    // column sums of this thread's 8 channels over the rows it stores, carried across the tiles of a range
    float cs0[8], cs1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cs0[e] = cs1[e] = 0.f;
    int cur = 0;
    for (int step = 0; step < n_steps; ++step) {
        const int t = tile_at(step);
        const int inst = t >= a.tiles ? 1 : 0;
        const int row_tile = t - inst * a.tiles;
        const int m0 = row_tile * BM;
        T* __restrict__ out = inst ? (T*)g.out1 : out_;
        double* stats = inst ? g.stats1 : g.stats;
        const int R0 = (int)fast_div((uint32_t)m0, g.wo_mul, g.wo_sh) - 1;
        char* patch = smem + kC64Zero + cur * a.buf_bytes;
        char* next_patch = smem + kC64Zero + (cur ^ 1) * a.buf_bytes;
        const bool has_next = step + 1 < n_steps;

        // this tile's rows are in LDS (written by all waves during the previous tile, or just above), and every wave is
        // past the previous tile's epilogue, whose staging area this tile's prefetch will overwrite
        lds_barrier();
        if (has_next) fetch_patch(tile_at(step + 1), pre);

        // per lane and 32-pixel block: LDS address of tap row r (or the zero region), swizzle keys of the three tap columns
        uint32_t base_r[2][3], f0[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m0 + wave * 64 + i * 32 + frow;
            const int tq = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - tq * W;
            const int n = (int)fast_div((uint32_t)tq, g.ho_mul, g.ho_sh), ho = tq - n * H;
            const uint32_t pix0 = (uint32_t)(((tq - R0 - 1) * W2 + wo) * 128);  // tap (0, 0): flat row tq - 1, patch column wo
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const bool ok = m < g.M && ho + r - 1 >= 0 && ho + r - 1 < H;
                base_r[i][r] = ok ? (uint32_t)(kC64Zero + cur * a.buf_bytes) + pix0 + (uint32_t)(r * W2 * 128) : 0u;
            }
            f0[i] = (uint32_t)((tq - R0 - 1) * W + wo);  // prow * W + pcol of tap (0, 0)
        }
        auto read_frag = [&](int ks, u32x4 (&f)[2]) {
            const int tap = ks >> 2, r = tap / 3, s2 = tap - 3 * r;
            const uint32_t cx = (uint32_t)((2 * (ks & 3)) << 4);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t key = (((f0[i] + (uint32_t)(r * W + s2)) >> 1) & 7u) ^ (uint32_t)fg;
                f[i] = *(const u32x4*)(smem + (base_r[i][r] + ((key << 4) ^ cx)) + s2 * 128);
            }
        };

        typename Mma<T, 32>::Acc acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        const int cc = (tid & 7) * 8, lr0 = tid >> 3;  // this thread's part of the output tile: rows lr0 + 32 k, 8 channels from cc
        static_assert(NKS - 8 >= WR0 + 8, "the first 8 prefetch registers are free for the last 8 steps");
        u32x4 fa[2][2];
        read_frag(0, fa[0]);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (ks + 1 < NKS) read_frag(ks + 1, fa[(ks + 1) & 1]);
            // the next tile's rows move from registers to the other patch buffer during the last steps
            if (ks >= WR0 && has_next) *(u32x4*)(next_patch + (tid + kThreads * (ks - WR0)) * 16) = pre[ks - WR0];
            // accumulating launches: what the output tile holds so far, as the 16-byte runs this thread will store
            // (coalesced, in flight during the last steps), into prefetch registers that have just been written out; the
            // sum is taken on the rounded tile, in float, and rounded again
            if (ACCUM && ks >= NKS - 8) {
                const int m = m0 + lr0 + 32 * (ks - (NKS - 8));
                pre[ks - (NKS - 8)] = m < g.M ? *(const u32x4*)(out + (int64_t)m * C + cc) : u32x4{0u, 0u, 0u, 0u};
            }
            __builtin_amdgcn_sched_barrier(0);  // the next step's fragment reads go out before this step's MFMAs
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) Mma<T, 32>::run(wf[ks][j], fa[ks & 1][i], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();  // every wave has finished reading the patch: it becomes the staging area of the output tile

        typedef typename Run4<T>::V RunV;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int lr = wave * 64 + i * 32 + frow;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = j * 32 + acc_row<32>(lane, 4 * q);
                    *(RunV*)(patch + lr * kC64EpiRowB + col * 2) =
                        Run4<T>::pack(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                }
            }
        lds_barrier();
        {
            // thread = (row tid >> 3 of each group of 32 rows, 16-byte run tid & 7): all eight reads first, then the stores
            u32x4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = *(const u32x4*)(patch + (lr0 + 32 * k) * kC64EpiRowB + cc * 2);
            if (ACCUM) {
#pragma unroll
                for (int k = 0; k < 8; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[k][e] = pack_bf16x2(__uint_as_float(v[k][e] << 16) + __uint_as_float(pre[k][e] << 16),
                                              __uint_as_float(v[k][e] & 0xffff0000u) + __uint_as_float(pre[k][e] & 0xffff0000u));
                // all sums are formed before the first store goes out: left to itself the compiler sinks each sum into the
                // guarded block of its store, where the wait for the loaded values becomes a wait for the stores before it
#pragma unroll
                for (int k = 0; k < 8; ++k) asm volatile("" : "+v"(v[k]));
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int m = m0 + lr0 + 32 * k;
                if (m < g.M) *(u32x4*)(out + (int64_t)m * C + cc) = v[k];
            }
            if (!ACCUM && stats) {  // (an accumulating launch is a backward-data pass: no sums)
                // column sums of the staged tile (rows past M hold zeros) from the same registers: this thread's 8 rows
                // of its 8 channels (one float sum per tile, added to the running sums of the range)
                float s0[8], s1[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) s0[e] = s1[e] = 0.f;
#pragma unroll
                for (int k = 0; k < 8; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(v[k][e] << 16), hi = __uint_as_float(v[k][e] & 0xffff0000u);
                        s0[2 * e] += lo;
                        s1[2 * e] += lo * lo;
                        s0[2 * e + 1] += hi;
                        s1[2 * e + 1] += hi * hi;
                    }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    cs0[e] += s0[e];
                    cs1[e] += s1[e];
                }
                if (step == n0 - 1 || step == n_steps - 1) {
                    // the range ends: the 32 row groups per channel, in double and in a fixed order, into this workgroup's
                    // partial row of the instance
                    float* sred = (float*)(patch + BM * kC64EpiRowB);  // [32 row groups][64 channels][2]
#pragma unroll
                    for (int e = 0; e < 8; e += 2)
                        *(f32x4*)(sred + (lr0 * 64 + cc + e) * 2) = f32x4{cs0[e], cs1[e], cs0[e + 1], cs1[e + 1]};
#pragma unroll
                    for (int e = 0; e < 8; ++e) cs0[e] = cs1[e] = 0.f;
                    lds_barrier();
                    if (tid < 128) {
                        double sa = 0.0;
#pragma unroll 8
                        for (int k = 0; k < 32; ++k) sa += (double)sred[k * 128 + tid];
                        stats[(int64_t)(inst ? w1 : (int)blockIdx.x) * (C * 2) + tid] = sa;
                    }
                }
            }
        }
        cur ^= 1;
    }
}


// ---- bf16 4x4 / stride 1 convolutions of 16 -> 64 channels, filters held in registers -----------------------------
// The space-to-depth form of a 7x7 / stride-2 stem: 16 (12 used) channels in, 64 out, a 4 x 4 window with two pixels of
// padding above / left and one below / right (Ho = H, Wo = W), and a very large map (112 x 112 x 256 images).  The
// contraction is only 256 long, so a launch is bound by writing the output; what the generic tiles lose on it is the
// fixed cost per tile (row decode, tap masks, epilogue) against eight short k steps.  Same scheme as the 64-channel
// kernel above: every wave keeps the whole filter bank (64 x 256 bf16 = 32 KB) as first-operand fragments (16 k steps =
// taps x 2 blocks of output channels x 4 registers = 128 registers), persistent workgroups walk ranges of consecutive
// tiles of 128 output pixels, the input rows a tile needs (its output rows, two above, one below; two zero columns
// left, one right) are staged ONCE as they lie in memory -- a pixel is one 32-byte run -- and the fragment of tap (r, s)
// is read at the shifted address.  A k step is one tap: lane (pixel, fg) reads the 16-byte half fg of its pixel; the
// two halves of a pixel swap places in every second group of 8 pixels, so that 16 consecutive pixels (512 bytes) read by
// one half-wave fall on all banks once.  Half the register file suffices, so TWO workgroups share a compute unit and
// each one's epilogue (staging, stores, column sums) runs under the other's MFMAs.  Column sums as in the kernel
// above: carried per thread over a whole range, one partial row per workgroup and instance.
struct C16Args {
    int tiles;  // row tiles of 128 output pixels per problem instance
    int twin;   // 1: a second problem instance (in1 / out1 / stats1)
};
constexpr int kC16Zero = 4096;      // zero region at the start of LDS (tap rows outside the image read here)
constexpr int kC16Pitch = 128;      // pixels per patch row
constexpr int kC16Rows = 6;         // a tile touches at most 3 output rows: 6 input rows
constexpr int kC16Patch = kC16Rows * kC16Pitch * 32;
constexpr int kC16EpiRowB = 64 * 2 + 16;
constexpr int kC16Sred = 32 * 64 * 2 * 4;
constexpr int kC16Lds = kC16Zero + 2 * kC16Patch + kC16Sred;
constexpr int kC16MaxWorkgroups = 512;

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv4x4_c16_bf16_kernel(
    const bf16_t* __restrict__ in_, const bf16_t* __restrict__ wgt, bf16_t* __restrict__ out_, GatherGeom g, C16Args a)
{
    typedef bf16_t T;
    constexpr int BM = 128, CI = 16, CO = 64, NKS = 16, NCH = kC16Rows, WR0 = NKS - NCH, ROWB = kC16Pitch * 32;
    static_assert(BM * kC16EpiRowB <= kC16Patch, "the output tile is staged in the patch buffer just multiplied");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int frow = lane & 31, fg = lane >> 5;
    const int W = g.Wi, H = g.Hi;

    // lane (frow, fg) holds, for output channel 32 j + frow, the channels 8 fg .. + 7 of tap t
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(wgt, (uint32_t)(CO * NKS * CI) * 2u);
    u32x4 wf[NKS][2];
#pragma unroll
    for (int t = 0; t < NKS; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) wf[t][j] = load16(rw, (uint32_t)(((32 * j + frow) * (NKS * CI)) + CI * t + 8 * fg) * 2u);
#pragma unroll
    for (int t = 0; t < NKS; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) asm volatile("" ::"v"(wf[t][j]));  // complete before the tile loop (see the kernel above)

    *(u32x4*)(smem + tid * 16) = u32x4{0u, 0u, 0u, 0u};  // kC16Zero = 256 threads x 16 bytes
    const uint32_t in_bytes = (uint32_t)g.N * H * W * CI * 2u;
    const __amdgpu_buffer_rsrc_t rin0 = make_rsrc(in_, in_bytes);
    const __amdgpu_buffer_rsrc_t rin1 = make_rsrc(g.in1 ? g.in1 : in_, in_bytes);

    const int nw = (int)gridDim.x, w1 = nw - 1 - (int)blockIdx.x;
    auto range_lo = [&](int w) { return (int)((int64_t)w * a.tiles / nw); };
    const int b0 = range_lo((int)blockIdx.x), n0 = range_lo((int)blockIdx.x + 1) - b0;
    const int b1 = range_lo(w1), n1 = a.twin ? range_lo(w1 + 1) - b1 : 0;
    const int n_steps = n0 + n1;
    auto tile_at = [&](int s) { return s < n0 ? b0 + s : a.tiles + b1 + (s - n0); };

    // thread tid moves half tid & 1 of patch pixel tid >> 1 of every row: input column (tid >> 1) - 2
    const int pcol = tid >> 1, phalf = tid & 1;
    const bool col_ok = pcol - 2 >= 0 && pcol - 2 < W;
    const uint32_t col_off = (uint32_t)((pcol - 2) * CI + phalf * 8) * 2u;
    const uint32_t lds_off = (uint32_t)(pcol * 32 + ((phalf ^ ((pcol >> 3) & 1)) << 4));
    auto fetch_patch = [&](int t, u32x4 (&pre)[NCH]) {
        const int inst = t >= a.tiles ? 1 : 0;
        const int m0 = (t - inst * a.tiles) * BM;
        const int tq0 = (int)fast_div((uint32_t)m0, g.wo_mul, g.wo_sh);  // flat output row of the tile's first pixel
        const int m_last = min(m0 + BM, g.M) - 1;
        const int rows = (int)fast_div((uint32_t)m_last, g.wo_mul, g.wo_sh) - tq0 + 4;  // input rows this tile touches
        const __amdgpu_buffer_rsrc_t rin = inst ? rin1 : rin0;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int row = tq0 - 2 + i;
            const bool row_ok = i < rows && row >= 0 && row < g.N * H;  // uniform
            pre[i] = load16(rin, (row_ok && col_ok) ? (uint32_t)(row * W * CI) * 2u + col_off : kOutOfRange);
        }
    };

    u32x4 pre[NCH];
    if (n_steps > 0) {
        fetch_patch(tile_at(0), pre);
#pragma unroll
        for (int i = 0; i < NCH; ++i) *(u32x4*)(smem + kC16Zero + i * ROWB + lds_off) = pre[i];
    }
    float cs0[8], cs1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cs0[e] = cs1[e] = 0.f;
    int cur = 0;
    for (int step = 0; step < n_steps; ++step) {
        const int t = tile_at(step);
        const int inst = t >= a.tiles ? 1 : 0;
        const int m0 = (t - inst * a.tiles) * BM;
        T* __restrict__ out = inst ? (T*)g.out1 : out_;
        double* stats = inst ? g.stats1 : g.stats;
        const int tq0 = (int)fast_div((uint32_t)m0, g.wo_mul, g.wo_sh);
        const uint32_t patch_base = (uint32_t)(kC16Zero + cur * kC16Patch);
        char* patch = smem + patch_base;
        char* next_patch = smem + kC16Zero + (cur ^ 1) * kC16Patch;
        const bool has_next = step + 1 < n_steps;

        lds_barrier();  // this tile's rows are in LDS; every wave is past the previous tile's epilogue
        if (has_next) fetch_patch(tile_at(step + 1), pre);

        uint32_t base_r[4], koff[4];
        {
            const int m = m0 + wave * 32 + frow;
            const int tq = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - tq * W;
            const int n = (int)fast_div((uint32_t)tq, g.ho_mul, g.ho_sh), ho = tq - n * H;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = m < g.M && ho + r - 2 >= 0 && ho + r - 2 < H;
                base_r[r] = ok ? patch_base + (uint32_t)((tq - tq0 + r) * ROWB) : 0u;
            }
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
                const int pc = wo + s2;  // patch column of tap column s2: input column wo - 2 + s2
                koff[s2] = (uint32_t)(pc * 32 + ((fg ^ ((pc >> 3) & 1)) << 4));
            }
        }
        auto read_frag = [&](int ks) { return *(const u32x4*)(smem + base_r[ks >> 2] + koff[ks & 3]); };

        typename Mma<T, 32>::Acc acc[2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

        u32x4 fa[2];
        fa[0] = read_frag(0);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (ks + 1 < NKS) fa[(ks + 1) & 1] = read_frag(ks + 1);
            if (ks >= WR0 && has_next) *(u32x4*)(next_patch + (ks - WR0) * ROWB + lds_off) = pre[ks - WR0];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 2; ++j) Mma<T, 32>::run(wf[ks][j], fa[ks & 1], acc[j]);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();  // every wave has finished reading the patch: it becomes the staging area of the output tile

        typedef typename Run4<T>::V RunV;
        const int lr = wave * 32 + frow;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = j * 32 + acc_row<32>(lane, 4 * q);
                *(RunV*)(patch + lr * kC16EpiRowB + col * 2) =
                    Run4<T>::pack(acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]);
            }
        lds_barrier();
        {
            const int cc = (tid & 7) * 8, lr0 = tid >> 3;
            u32x4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = *(const u32x4*)(patch + (lr0 + 32 * k) * kC16EpiRowB + cc * 2);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int m = m0 + lr0 + 32 * k;
                if (m < g.M) *(u32x4*)(out + (int64_t)m * CO + cc) = v[k];
            }
            if (stats) {
                float s0[8], s1[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) s0[e] = s1[e] = 0.f;
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(v[k][e] << 16), hi = __uint_as_float(v[k][e] & 0xffff0000u);
                        s0[2 * e] += lo;
                        s1[2 * e] += lo * lo;
                        s0[2 * e + 1] += hi;
                        s1[2 * e + 1] += hi * hi;
                    }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    cs0[e] += s0[e];
                    cs1[e] += s1[e];
                }
                if (step == n0 - 1 || step == n_steps - 1) {
                    float* sred = (float*)(smem + kC16Zero + 2 * kC16Patch);  // [32 row groups][64 channels][2]
#pragma unroll
                    for (int e = 0; e < 8; e += 2)
                        *(f32x4*)(sred + (lr0 * 64 + cc + e) * 2) = f32x4{cs0[e], cs1[e], cs0[e + 1], cs1[e + 1]};
#pragma unroll
                    for (int e = 0; e < 8; ++e) cs0[e] = cs1[e] = 0.f;
                    lds_barrier();
                    if (tid < 128) {
                        double sa = 0.0;
#pragma unroll 8
                        for (int k = 0; k < 32; ++k) sa += (double)sred[k * 128 + tid];
                        stats[(int64_t)(inst ? w1 : (int)blockIdx.x) * (CO * 2) + tid] = sa;
                    }
                }
            }
        }
        cur ^= 1;
    }
}

// ---- fp32 3x3 convolutions with 16 or 32 channels on both sides ----------------------------------
// With so few channels the whole filter bank of 16 output channels fits in registers (9 * Ci / 16
// 16-byte runs per lane), so no operand needs LDS: the MFMA computes y^T, D[co][pixel] with
// A = filters (row co = lane % 16, k-run lane / 16) held for the whole kernel and B = the gathered
// pixels, one coalesced 16-byte run per lane, tap and 16 channels (16 consecutive pixels = 1 KB per
// wave load).  Lane (pixel p, quarter q) uses element e of its run in MFMA e, which pairs channel
// 4q + e on both operands.  The result leaves each lane with 4 consecutive output channels of one
// pixel: one 16-byte store.  A wave owns one group of 16 output channels and walks groups of 16
// pixels; the column sums for a following batch norm are accumulated on the way.
template <int CI16>
__global__ __launch_bounds__(kThreads) void conv3x3_direct_f32_kernel(const float* __restrict__ in_,
                                                                      const float* __restrict__ wgt,
                                                                      float* __restrict__ out_, GatherGeom g)
{
    constexpr int TAPS = 9;
    const float* __restrict__ in = blockIdx.y ? (const float*)g.in1 : in_;
    float* __restrict__ out = blockIdx.y ? (float*)g.out1 : out_;
    double* stats = blockIdx.y ? g.stats1 : g.stats;
    __shared__ double red[4][16][2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, px = lane & 15, kq = lane >> 4;
    const int cgs = g.Co >> 4;               // groups of 16 output channels (1 or 2)
    const int cg = wave % cgs, pw = wave / cgs, PW = 4 / cgs;
    const int groups = (g.M + 15) >> 4;

    f32x4 wreg[TAPS][CI16];
    {
        const float* wrow = wgt + (size_t)(cg * 16 + px) * g.Kdim + 4 * kq;
        if (((uintptr_t)wgt & 15) == 0) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
#pragma unroll
                for (int c = 0; c < CI16; ++c) wreg[t][c] = *(const f32x4*)(wrow + t * g.Ci + c * 16);
        } else {
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
#pragma unroll
                for (int c = 0; c < CI16; ++c) {
                    const float* p = wrow + t * g.Ci + c * 16;
                    wreg[t][c] = f32x4{p[0], p[1], p[2], p[3]};
                }
        }
    }
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(in, (uint32_t)g.N * g.Hi * g.Wi * g.Ci * 4u);
    float s0[4] = {0.f, 0.f, 0.f, 0.f}, s1[4] = {0.f, 0.f, 0.f, 0.f};

    // 16-byte runs of pixel group grp, all taps; a group past the end reads zeros
    auto gather = [&](f32x4 (&xin)[TAPS][CI16], int grp) {
        const int m = grp * 16 + px;
        const bool live = grp < groups && m < g.M;
        const int tq = (int)fast_div((uint32_t)m, g.wo_mul, g.wo_sh), wo = m - tq * g.Wo;
        const int n = (int)fast_div((uint32_t)tq, g.ho_mul, g.ho_sh), ho = tq - n * g.Ho;
        const int th0 = ho * g.ostride - g.pad_h, tw0 = wo * g.ostride - g.pad_w;
        const uint32_t base = (uint32_t)(((n * g.Hi + th0) * g.Wi + tw0) * g.Ci + 4 * kq) * 4u;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const bool hok = live && th0 + r >= 0 && th0 + r < g.Hi;
#pragma unroll
            for (int s2 = 0; s2 < 3; ++s2) {
                const bool ok = hok && tw0 + s2 >= 0 && tw0 + s2 < g.Wi;
                const uint32_t off = base + (uint32_t)((r * g.Wi + s2) * g.Ci) * 4u;
#pragma unroll
                for (int c = 0; c < CI16; ++c)
                    xin[r * 3 + s2][c] = __builtin_bit_cast(f32x4, load16(rin, ok ? off + c * 64u : kOutOfRange));
            }
        }
    };
    auto finish = [&](const f32x4 (&xin)[TAPS][CI16], int grp) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
            for (int c = 0; c < CI16; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wreg[t][c][e], xin[t][c][e], acc, 0, 0, 0);
        const int m = grp * 16 + px;
        if (m < g.M) {
            float* dst = out + (size_t)m * g.Co + cg * 16 + 4 * kq;
            if (g.accum) {
                const f32x4 old = *(const f32x4*)dst;
                acc += old;
            }
            *(f32x4*)dst = acc;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s0[e] += acc[e];
            s1[e] += acc[e] * acc[e];
        }
    };

    // DEPTH register sets: the pixels of the next DEPTH - 1 groups are in flight while one is multiplied
    constexpr int DEPTH = CI16 == 1 ? 4 : 2;
    const int stride_g = gridDim.x * PW;
    f32x4 xr[DEPTH][TAPS][CI16];
    const unsigned tile = xcd_tile(blockIdx.x, gridDim.x);
    int grp = tile * PW + pw;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (grp + d * stride_g < groups) gather(xr[d], grp + d * stride_g);  // all conditions here are wave-uniform
    while (grp < groups) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (grp < groups) {
                finish(xr[d], grp);
                if (grp + DEPTH * stride_g < groups) gather(xr[d], grp + DEPTH * stride_g);
            }
            grp += stride_g;
        }
    }
    if (stats) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) {
                s0[e] += __shfl_xor(s0[e], off, 64);
                s1[e] += __shfl_xor(s1[e], off, 64);
            }
        if (px == 0)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                red[wave][4 * kq + e][0] = (double)s0[e];
                red[wave][4 * kq + e][1] = (double)s1[e];
            }
        __syncthreads();
        if (tid < g.Co) {
            const int c = tid & 15, cgi = tid >> 4;
            double a = 0.0, b = 0.0;
            for (int k = 0; k < PW; ++k) {
                a += red[k * cgs + cgi][c][0];
                b += red[k * cgs + cgi][c][1];
            }
            double* dst = stats + ((int64_t)tile * g.Co + tid) * 2;
            dst[0] = a;
            dst[1] = b;
        }
    }
}

// ---- backward-weight --------------------------------------------------------------------------
// dw[co][j] = sum_m dy[m][co] * xcol[m][j].  Both operands are stored with m as the slow index while
// the MFMA wants runs along m, so the loader moves E x E micro-tiles (E rows of m, one 16-byte
// channel run each; E = 8 for bf16, 4 for fp32), transposes them in registers and writes E
// 16-byte runs along m into LDS.  Lanes of one 8-lane group own consecutive m groups of the
// same channel group: their LDS writes are one contiguous 128-byte stripe and their global reads
// are 128-byte row segments.  blockIdx.y selects a slice of m; slices are summed afterwards in a
// fixed order.
struct WgradGeom {
    int N, H, W, Ci, Ho, Wo, Co, R, S, pad, stride;
    int M, Kdim, m_per_split;
    // Grouped convolution: Ci and Co are the channels of ONE group (blockIdx.z); a pixel of x holds Cis = groups * Ci
    // channels and a row of dy Cos = groups * Co; the filter gradient has groups * Co rows of Kdim = R*S*Ci columns.
    int groups, Cis, Cos;
    uint32_t wo_mul, wo_sh, ho_mul, ho_sh;  // n / Wo and n / Ho by multiplication (fast_div)
};

template <typename T>
__device__ inline void transpose_micro(const u32x4 (&in)[16 / sizeof(T)], u32x4 (&out)[16 / sizeof(T)]);

template <>
__device__ inline void transpose_micro<float>(const u32x4 (&in)[4], u32x4 (&out)[4])
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        u32x4 v = {in[0][c], in[1][c], in[2][c], in[3][c]};
        out[c] = v;
    }
}

template <>
__device__ inline void transpose_micro<bf16_t>(const u32x4 (&in)[8], u32x4 (&out)[8])
{
    // in[e] = 8 channels of row e (2 per dword); out[c] = 8 rows of channel c (2 per dword, row 2i in the low half)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        u32x4 lo, hi;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t a = in[2 * i][j], b = in[2 * i + 1][j];
            lo[i] = (a & 0xffffu) | (b << 16);
            hi[i] = (a >> 16) | (b & 0xffff0000u);
        }
        out[2 * j] = lo;
        out[2 * j + 1] = hi;
    }
}

template <typename TL, bool VEC>
__global__ __launch_bounds__(kThreads) void conv_wgrad_kernel(const typename TL::T* __restrict__ x,
                                                              const typename TL::T* __restrict__ dy,
                                                              float* __restrict__ part, WgradGeom g)
{
    typedef typename TL::T T;
    constexpr int E = TL::E, BKm = TL::BK;
    static_assert(TL::STAGES == 2, "backward-weight double-buffers its LDS tiles");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    const int tiles_n = (g.Kdim + TL::BN - 1) / TL::BN;
    // all tiles of one m slice in one L2: the linear workgroup id runs over the tiles first
    const unsigned lin = xcd_tile(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
    const unsigned tile = lin % gridDim.x, slice = lin / gridDim.x;
    const int c0 = (tile / tiles_n) * TL::BM;  // first output channel of the tile
    const int j0 = (tile % tiles_n) * TL::BN;  // first (r,s,ci) column of the tile
    const int m_begin = slice * g.m_per_split;
    const int m_end = min(g.M, m_begin + g.m_per_split);
    const int nk = (m_end - m_begin + BKm - 1) / BKm;
    // grouped convolution (blockIdx.z = group): dy columns dy_c0 .. of rows Cos wide, x channels x_c0 .. of pixels Cis wide
    const int dy_c0 = blockIdx.z * g.Co, x_c0 = blockIdx.z * g.Ci;

    typename Mma<T, TL::MT>::Acc acc[TL::TM][TL::TN];
    zero_acc<TL>(acc);

    if (VEC) {
        constexpr int MG = BKm / E;                       // m groups per LDS row
        constexpr int NA = (TL::BM / E) * MG, NB = (TL::BN / E) * MG;
        constexpr int PER = (NA + NB + kThreads - 1) / kThreads;
        static_assert(TL::BM % E == 0 && TL::BN % E == 0 && BKm % E == 0, "micro-tiles must tile the LDS tile");
        // fixed per micro-tile: which operand, channel group, m group; for x also the tap and the pixel walk
        int mt_row[PER];      // LDS row of channel 0 of the micro-tile (B rows follow the BM A rows), -1 = none
        int mt_col[PER];      // global channel / column offset of the 16-byte run (-1: outside the tensor)
        int mt_mg[PER];
        int tap_r[PER], tap_s[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = tid + i * kThreads;
            mt_row[i] = -1;
            mt_col[i] = -1;
            mt_mg[i] = 0;
            tap_r[i] = tap_s[i] = 0;
            if (c < NA) {
                const int mg = c % MG, cg = c / MG;
                mt_row[i] = cg * E;
                mt_mg[i] = mg;
                mt_col[i] = (c0 + cg * E < g.Co) ? c0 + cg * E : -1;
            } else if (c < NA + NB) {
                const int cb = c - NA, mg = cb % MG, cg = cb / MG;
                mt_row[i] = TL::BM + cg * E;
                mt_mg[i] = mg;
                const int j = j0 + cg * E;
                if (j < g.Kdim) {
                    const int tap = j / g.Ci;
                    mt_col[i] = j % g.Ci;
                    tap_r[i] = tap / g.S;
                    tap_s[i] = tap % g.S;
                }
            }
        }
        u32x4 regs[PER][E];

        constexpr uint32_t SZ = sizeof(T);
        const __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (uint32_t)g.M * g.Cos * SZ);
        const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)g.N * g.H * g.W * g.Cis * SZ);
        auto load_tiles = [&](int mb) {
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int c = tid + i * kThreads;
                const int mfirst = mb + mt_mg[i] * E;
                if (c < NA) {
                    // E consecutive rows of dy: offsets Co apart; out-of-range rows read as zeros
                    uint32_t off = mt_col[i] >= 0 ? (uint32_t)(mfirst * g.Cos + dy_c0 + mt_col[i]) * SZ : kOutOfRange;
                    const uint32_t step = (uint32_t)g.Cos * SZ;
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        regs[i][e] = load16(rdy, (mt_col[i] >= 0 && mfirst + e < m_end) ? off : kOutOfRange);
                        off += step;
                    }
                } else if (c < NA + NB) {
                    // E consecutive output pixels (n, h, w0 + e) of one tap.  They lie in one image row, or in
                    // two when the run crosses a row end (Wo >= E - 1: at most one crossing); branch-free:
                    // both rows' base offsets are formed once and every pixel picks its row.
                    const bool col_ok = mt_col[i] >= 0;
                    const uint32_t pix = (uint32_t)g.Cis * SZ;
                    const uint32_t tq = fast_div((uint32_t)mfirst, g.wo_mul, g.wo_sh);
                    const int w0 = mfirst - (int)tq * g.Wo;
                    const int n0 = (int)fast_div(tq, g.ho_mul, g.ho_sh);
                    const int h0 = (int)tq - n0 * g.Ho;
                    if (g.Wo >= E - 1) {
                        const int hiA = h0 * g.stride - g.pad + tap_r[i];
                        const bool okA = col_ok && hiA >= 0 && hiA < g.H;
                        const uint32_t offA = (uint32_t)(((n0 * g.H + hiA) * g.W) * g.Cis + x_c0 + mt_col[i]) * SZ;
                        const int wiA = w0 * g.stride - g.pad + tap_s[i];
                        const bool last = h0 + 1 == g.Ho;
                        const int h1 = last ? 0 : h0 + 1, n1 = n0 + (last ? 1 : 0);
                        const int hiB = h1 * g.stride - g.pad + tap_r[i];
                        const bool okB = col_ok && hiB >= 0 && hiB < g.H;
                        const uint32_t offB = (uint32_t)(((n1 * g.H + hiB) * g.W) * g.Cis + x_c0 + mt_col[i]) * SZ;
                        const int e_wrap = g.Wo - w0;                               // first pixel of the run in the second row
                        const int wiB = tap_s[i] - g.pad - e_wrap * g.stride;       // so that wi = wiB + e * stride there
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const bool in_a = e < e_wrap;
                            const int wi = (in_a ? wiA : wiB) + e * g.stride;
                            const bool ok = (in_a ? okA : okB) && (unsigned)wi < (unsigned)g.W && mfirst + e < m_end;
                            regs[i][e] = load16(rx, ok ? (in_a ? offA : offB) + (uint32_t)wi * pix : kOutOfRange);
                        }
                    } else {
                        // rows shorter than the run: walk pixel by pixel
                        int n = n0, h = h0, w = w0;
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const int hi = h * g.stride - g.pad + tap_r[i], wi = w * g.stride - g.pad + tap_s[i];
                            const bool ok = col_ok && hi >= 0 && hi < g.H && wi >= 0 && wi < g.W && mfirst + e < m_end;
                            regs[i][e] = load16(rx, ok ? (uint32_t)(((n * g.H + hi) * g.W + wi) * g.Cis + x_c0 + mt_col[i]) * SZ : kOutOfRange);
                            if (++w == g.Wo) {
                                w = 0;
                                if (++h == g.Ho) { h = 0; ++n; }
                            }
                        }
                    }
                }
            }
        };
        auto store_tiles = [&](int buf) {
            char* base = smem + buf * TL::STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                if (mt_row[i] < 0) continue;
                u32x4 tr[E];
                transpose_micro<T>(regs[i], tr);
#pragma unroll
                for (int ch = 0; ch < E; ++ch) *(u32x4*)(base + (mt_row[i] + ch) * TL::ROWB + mt_mg[i] * 16) = tr[ch];
            }
        };
        // rows at or past m_end load as zeros, so the loop may fetch (and store into the idle stage) one
        // tile past the slice: a single loop body with one back edge keeps the accumulators in place
        load_tiles(m_begin);
        store_tiles(0);
        __syncthreads();
        int kt = 0;
        for (; kt + 1 < nk; kt += 2) {
            load_tiles(m_begin + (kt + 1) * BKm);
            mma_tile<TL>(smem, smem + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
            store_tiles(1);
            __syncthreads();
            load_tiles(m_begin + (kt + 2) * BKm);
            mma_tile<TL>(smem + TL::STAGE_BYTES, smem + TL::STAGE_BYTES + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
            store_tiles(0);
            __syncthreads();
        }
        if (kt < nk) mma_tile<TL>(smem, smem + TL::BM * TL::ROWB, wave_m, wave_n, lane, acc);
    } else {
        // generic path: element-wise loads and LDS writes
        constexpr int A_CPR = TL::BM / E, B_CPR = TL::BN / E;
        constexpr int A_CH = A_CPR * BKm, B_CH = B_CPR * BKm;
        constexpr int A_PER = (A_CH + kThreads - 1) / kThreads, B_PER = (B_CH + kThreads - 1) / kThreads;
        alignas(16) T ra[A_PER][E];
        alignas(16) T rb[B_PER][E];
        const T zero = from_float<T>(0.f);
        auto load_tiles = [&](int mb) {
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int c = tid + i * kThreads, mrow = c / A_CPR, cc = (c % A_CPR) * E;
                const int m = mb + mrow, co = c0 + cc;
                const bool ok = c < A_CH && m < m_end;
                for (int e = 0; e < E; ++e) ra[i][e] = (ok && co + e < g.Co) ? dy[(int64_t)m * g.Cos + dy_c0 + co + e] : zero;
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int c = tid + i * kThreads, mrow = c / B_CPR, cc = (c % B_CPR) * E;
                const int m = mb + mrow, j = j0 + cc;
                const bool ok = c < B_CH && m < m_end;
                const int wo = m % g.Wo, t = m / g.Wo, ho = t % g.Ho, n = t / g.Ho;
                for (int e = 0; e < E; ++e) {
                    const int je = j + e;
                    const int tap = je / g.Ci, ci = je % g.Ci, r = tap / g.S, s = tap % g.S;
                    const int hi = ho * g.stride - g.pad + r, wi = wo * g.stride - g.pad + s;
                    rb[i][e] = (ok && je < g.Kdim && hi >= 0 && hi < g.H && wi >= 0 && wi < g.W)
                                   ? x[(((int64_t)n * g.H + hi) * g.W + wi) * g.Cis + x_c0 + ci]
                                   : zero;
                }
            }
        };
        auto store_tiles = [&](int buf) {
            char* sA = smem + buf * TL::STAGE_BYTES;
            char* sB = sA + TL::BM * TL::ROWB;
#pragma unroll
            for (int i = 0; i < A_PER; ++i) {
                const int c = tid + i * kThreads, mrow = c / A_CPR, cc = (c % A_CPR) * E;
                if (c < A_CH)
#pragma unroll
                    for (int e = 0; e < E; ++e) *(T*)(sA + (cc + e) * TL::ROWB + mrow * (int)sizeof(T)) = ra[i][e];
            }
#pragma unroll
            for (int i = 0; i < B_PER; ++i) {
                const int c = tid + i * kThreads, mrow = c / B_CPR, cc = (c % B_CPR) * E;
                if (c < B_CH)
#pragma unroll
                    for (int e = 0; e < E; ++e) *(T*)(sB + (cc + e) * TL::ROWB + mrow * (int)sizeof(T)) = rb[i][e];
            }
        };
        if (nk > 0) {
            load_tiles(m_begin);
            store_tiles(0);
        }
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
            if (kt + 1 < nk) load_tiles(m_begin + (kt + 1) * BKm);
            mma_tile<TL>(smem + cur * TL::STAGE_BYTES, smem + cur * TL::STAGE_BYTES + TL::BM * TL::ROWB, wave_m, wave_n,
                         lane, acc);
            if (kt + 1 < nk) store_tiles(cur ^ 1);
            __syncthreads();
        }
    }

    float* dst = part + ((int64_t)slice * gridDim.z * g.Co + dy_c0) * g.Kdim;
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

// bf16 backward-weight for the 64- and 128-wide tiles without any register transpose.  Both operands go
// into LDS exactly as they lie in memory (rows = m, 16-byte channel runs); the MFMA operand layout
// (lane = channel, 8 consecutive m per lane) is produced by the LDS transpose read: in each group of 16
// lanes, lane i receives as element f the element (i % 4) of the 8 bytes that lane 4 f + i / 4 addressed.
// So the 16 lanes address rows m0 .. m0+3 (lane / 4), 4 channels each (lane % 4), and come away with
// 4 consecutive m of 16 channels; two such reads make one 8-element operand.  LDS rows are not padded:
// within every 256-byte line the 16-byte chunk index is XORed with 4 * (line % 4), which spreads the
// four rows of a read over all banks.
typedef short short4v __attribute__((ext_vector_type(4)));

// Byte offset of 16-byte chunk `chunk` of row `row` in an unpadded tile whose rows are `row_bytes` long.
__device__ inline int swizzled_chunk(int row, int chunk, int row_bytes)
{
    const int lin = row * row_bytes + chunk * 16;
    const int line = lin >> 8, cl = (lin >> 4) & 15;
    return (line << 8) + ((cl ^ ((line & 3) << 2)) << 4);
}

__device__ inline u32x2 lds_read_tr16(const char* p)
{
    return __builtin_bit_cast(
        u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(p)));
}

template <typename TL>
__global__ __launch_bounds__(kThreads) void conv_wgrad_tr_kernel(const bf16_t* __restrict__ x,
                                                                 const bf16_t* __restrict__ dy,
                                                                 float* __restrict__ part, WgradGeom g)
{
    typedef bf16_t T;
    constexpr int BM = TL::BM, BN = TL::BN, BKm = TL::BK;
    static_assert(sizeof(typename TL::T) == 2 && TL::MT == 32 && BKm == 64, "bf16, 32x32x16 MFMA, 64 rows of m per LDS tile");
    static_assert((BM == 64 || BM == 128) && (BN == 64 || BN == 128), "tile widths the swizzle is laid out for");
    constexpr int RA = BM * 2, RB = BN * 2;         // LDS row bytes of the two operands
    constexpr int A_BYTES = BKm * RA, STAGE = BKm * (RA + RB);
    constexpr int CA = BM / 8, CB = BN / 8;         // 16-byte chunks per row
    constexpr int PA = BKm * CA / kThreads, PB = BKm * CB / kThreads;
    constexpr int RSA = kThreads / CA, RSB = kThreads / CB;  // row step between a thread's chunks
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / TL::WGN, wave_n = wave % TL::WGN;
    const int tiles_n = (g.Kdim + BN - 1) / BN;
    const unsigned lin = xcd_tile(blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y);
    const unsigned tile = lin % gridDim.x, slice = lin / gridDim.x;
    const int c0 = (tile / tiles_n) * BM;
    const int j0 = (tile % tiles_n) * BN;
    const int m_begin = slice * g.m_per_split;
    const int m_end = min(g.M, m_begin + g.m_per_split);
    const int nk = (m_end - m_begin + BKm - 1) / BKm;
    // grouped convolution (blockIdx.z = group): dy columns dy_c0 .. of rows Cos wide, x channels x_c0 .. of pixels Cis wide
    const int dy_c0 = blockIdx.z * g.Co, x_c0 = blockIdx.z * g.Ci;

    typename Mma<T, 32>::Acc acc[TL::TM][TL::TN];
    zero_acc<TL>(acc);

    // loader: this thread's chunk column is fixed, its rows are row0 + i * RS
    const int a_chunk = tid % CA, a_row0 = tid / CA;
    const int b_chunk = tid % CB, b_row0 = tid / CB;
    const bool a_ok = c0 + a_chunk * 8 < g.Co;
    const int jb = j0 + b_chunk * 8;
    const bool b_ok = jb < g.Kdim;
    const int tap = b_ok ? jb / g.Ci : 0, b_ci = b_ok ? jb % g.Ci : 0;
    const int tap_r = tap / g.S, tap_s = tap % g.S;
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (uint32_t)g.M * g.Cos * 2u);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)g.N * g.H * g.W * g.Cis * 2u);
    u32x4 ra[PA], rb[PB];
    auto load_tiles = [&](int mb) {
#pragma unroll
        for (int i = 0; i < PA; ++i) {
            const int m = mb + a_row0 + i * RSA;
            ra[i] = load16(rdy, (a_ok && m < m_end) ? (uint32_t)(m * g.Cos + dy_c0 + c0 + a_chunk * 8) * 2u : kOutOfRange);
        }
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int m = mb + b_row0 + i * RSB;
            const uint32_t tq = fast_div((uint32_t)m, g.wo_mul, g.wo_sh);
            const int wo = m - (int)tq * g.Wo;
            const int n = (int)fast_div(tq, g.ho_mul, g.ho_sh);
            const int ho = (int)tq - n * g.Ho;
            const int hi = ho * g.stride - g.pad + tap_r, wi = wo * g.stride - g.pad + tap_s;
            const bool ok = b_ok && m < m_end && (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W;
            rb[i] = load16(rx, ok ? (uint32_t)(((n * g.H + hi) * g.W + wi) * g.Cis + x_c0 + b_ci) * 2u : kOutOfRange);
        }
    };
    auto store_tiles = [&](int buf) {
        char* sA = smem + buf * STAGE;
        char* sB = sA + A_BYTES;
#pragma unroll
        for (int i = 0; i < PA; ++i) *(u32x4*)(sA + swizzled_chunk(a_row0 + i * RSA, a_chunk, RA)) = ra[i];
#pragma unroll
        for (int i = 0; i < PB; ++i) *(u32x4*)(sB + swizzled_chunk(b_row0 + i * RSB, b_chunk, RB)) = rb[i];
    };
    // operand reads: 16-lane group = (channel half cs, m half kg); lane j of it addresses row j / 4, channels 4 (j % 4)
    const int j16 = lane & 15, cs = (lane >> 4) & 1, kg = lane >> 5;
    const int frag_row = 8 * kg + (j16 >> 2);            // + 16 * ks + 4 * h
    const int frag_chunk = cs * 2 + ((j16 & 3) >> 1);    // + 4 * (32-wide tile index)
    const int frag_half = (j16 & 1) * 8;
    auto mma = [&](const char* sA, const char* sB) {
#pragma unroll
        for (int ks = 0; ks < BKm / 16; ++ks) {
            u32x4 a[TL::TM], b[TL::TN];
#pragma unroll
            for (int i = 0; i < TL::TM; ++i) {
                const int ch = (wave_m * TL::TM + i) * 4 + frag_chunk;
                const u32x2 lo = lds_read_tr16(sA + swizzled_chunk(16 * ks + frag_row, ch, RA) + frag_half);
                const u32x2 hi = lds_read_tr16(sA + swizzled_chunk(16 * ks + 4 + frag_row, ch, RA) + frag_half);
                a[i] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int jn = 0; jn < TL::TN; ++jn) {
                const int ch = (wave_n * TL::TN + jn) * 4 + frag_chunk;
                const u32x2 lo = lds_read_tr16(sB + swizzled_chunk(16 * ks + frag_row, ch, RB) + frag_half);
                const u32x2 hi = lds_read_tr16(sB + swizzled_chunk(16 * ks + 4 + frag_row, ch, RB) + frag_half);
                b[jn] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
#pragma unroll
            for (int i = 0; i < TL::TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TL::TN; ++jn) Mma<T, 32>::run(a[i], b[jn], acc[i][jn]);
        }
    };
    // rows at or past m_end load as zeros, so the loop may fetch (and store into the idle stage) one tile
    // past the slice: a single loop body with one back edge keeps the accumulators in place
    load_tiles(m_begin);
    store_tiles(0);
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        load_tiles(m_begin + (kt + 1) * BKm);
        mma(smem, smem + A_BYTES);
        store_tiles(1);
        __syncthreads();
        load_tiles(m_begin + (kt + 2) * BKm);
        mma(smem + STAGE, smem + STAGE + A_BYTES);
        store_tiles(0);
        __syncthreads();
    }
    if (kt < nk) mma(smem, smem + A_BYTES);

    float* dst = part + ((int64_t)slice * gridDim.z * g.Co + dy_c0) * g.Kdim;
#pragma unroll
    for (int i = 0; i < TL::TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TL::TN; ++jn) {
            const int col = j0 + (wave_n * TL::TN + jn) * 32 + lane % 32;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int co = c0 + (wave_m * TL::TM + i) * 32 + acc_row<32>(lane, e);
                if (co < g.Co && col < g.Kdim) dst[(int64_t)co * g.Kdim + col] = acc[i][jn][e];
            }
        }
}

// ---- bf16 backward-weight of 3x3 / stride 1 / pad 1 layers with 64 channels on both sides ----------
// The whole result (64 x 576 floats) fits the accumulators of one workgroup, so a persistent workgroup keeps it there
// while it walks its share of the pixels, and writes ONE slice of partials at the end.  Both operands are staged as
// they lie in memory, once: a tile is two output rows of one image; `dy` goes to LDS as 2 x 64 pixels (columns
// W .. 63 zero), `x` as 4 x 64 pixels (the rows above and below, one zero column left; zeros outside the image).
// The contraction runs over the 128 pixel slots of the dy tile (8 MFMA steps of 16); the x operand of tap (r, s) for
// slot q is slot q + 64 r + s of the x patch -- a constant offset, so the nine-fold im2col expansion happens in the
// LDS read, and the zero columns of dy cancel whatever the patch holds at the slots that are no pixels.  Operands are
// formed by the LDS transpose read (see conv_wgrad_tr_kernel) with the same per-256-byte-line chunk swizzle.
// Wave w multiplies both blocks of 32 output channels with input-channel block w & 1 of the taps (w >> 1), (w >> 1) + 2,
// ..: 10 (or 8) MFMAs per step from 14 (12) operand reads, instead of 2 reads per MFMA of the tiled kernel.
// The rows of the next tile are fetched into registers before the steps and written to the other LDS buffer after
// them (12 16-byte chunks per lane: lane tid moves channel run tid & 7 of columns tid >> 3 and (tid >> 3) + 32).
struct W64Args {
    int tiles;          // N * H / 2
    int tiles_per_wg;   // consecutive tiles per workgroup
};
constexpr int kW64DyBytes = 2 * 64 * 128, kW64XBytes = 4 * 64 * 128, kW64Guard = 512;
constexpr int kW64BufBytes = kW64DyBytes + kW64XBytes + kW64Guard;

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void conv3x3_c64_wgrad_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, float* __restrict__ part, WgradGeom g, W64Args a)
{
    constexpr int C = 64, KD = 9 * C, NKS = 8;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = g.W, H = g.H, H2 = H / 2;
    const int ii = wave & 1, pw = wave >> 1, ntaps = pw ? 4 : 5;  // input-channel block, first tap, number of taps

    // the guards behind the x patches stay zero (the taps of the last slots reach two pixels past the patch)
    for (int b = 0; b < 2; ++b)
        if (tid < kW64Guard / 16) *(u32x4*)(smem + b * kW64BufBytes + kW64DyBytes + kW64XBytes + tid * 16) = u32x4{0u, 0u, 0u, 0u};

    const uint32_t t_bytes = (uint32_t)g.N * H * W * C * 2u;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, t_bytes), rdy = make_rsrc(dy, t_bytes);
    const int t_begin = blockIdx.x * a.tiles_per_wg, t_end = min(a.tiles, t_begin + a.tiles_per_wg);

    // fetch: this lane's two columns, as byte offsets inside a tensor row (or "out of range")
    uint32_t dy_col[2], x_col[2];
    uint32_t lds_slot[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int col = (tid >> 3) + 32 * h;
        dy_col[h] = col < W ? (uint32_t)(col * C + (tid & 7) * 8) * 2u : kOutOfRange;
        x_col[h] = (col >= 1 && col <= W) ? (uint32_t)((col - 1) * C + (tid & 7) * 8) * 2u : kOutOfRange;
        lds_slot[h] = (uint32_t)swizzled_chunk(col, tid & 7, 128);  // rows of 64 pixels are 32 lines: the swizzle repeats per row
    }
    auto fetch = [&](int t, u32x4 (&pre)[12]) {
        const int n = t / H2, h0 = (t - n * H2) * 2;  // first output row of the tile
        const uint32_t row_bytes = (uint32_t)W * C * 2u;
        const uint32_t img = (uint32_t)(n * H) * row_bytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t off = img + (uint32_t)(h0 + (i >> 1)) * row_bytes;
            pre[i] = load16(rdy, dy_col[i & 1] != kOutOfRange ? off + dy_col[i & 1] : kOutOfRange);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int hr = h0 - 1 + (i >> 1);
            const bool ok = hr >= 0 && hr < H && x_col[i & 1] != kOutOfRange;
            pre[4 + i] = load16(rx, ok ? img + (uint32_t)hr * row_bytes + x_col[i & 1] : kOutOfRange);
        }
    };
    auto stage = [&](int buf, const u32x4 (&pre)[12]) {
        char* base = smem + buf * kW64BufBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) *(u32x4*)(base + (i >> 1) * 8192 + lds_slot[i & 1]) = pre[i];
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)(base + kW64DyBytes + (i >> 1) * 8192 + lds_slot[i & 1]) = pre[4 + i];
    };

    // operand reads (transpose reads, see conv_wgrad_tr_kernel): lane (j16, cs, kg) addresses pixel slot
    // 8 kg + j16 / 4 (+ 4 for the second half) of a step, channels 16 cs + 4 (j16 % 4) .. + 3 of a 32-channel block
    const int j16 = lane & 15, cs = (lane >> 4) & 1, kg = lane >> 5;
    const int frag_row = 8 * kg + (j16 >> 2), frag_chunk = cs * 2 + ((j16 & 3) >> 1), frag_half = (j16 & 1) * 8;
    uint32_t a_addr[2][2];   // [output-channel block][half]
    uint32_t b_addr[5][2];   // [tap of this wave][half]
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
        for (int ic = 0; ic < 2; ++ic) a_addr[ic][hh] = (uint32_t)(swizzled_chunk(frag_row + 4 * hh, 4 * ic + frag_chunk, 128) + frag_half);
#pragma unroll
        for (int k = 0; k < 5; ++k) {
            const int tap = pw + 2 * k, r = tap / 3, s2 = tap - 3 * r;
            b_addr[k][hh] = (uint32_t)(kW64DyBytes + swizzled_chunk(frag_row + 4 * hh + 64 * r + s2, 4 * ii + frag_chunk, 128) + frag_half);
        }
    }

    typename Mma<bf16_t, 32>::Acc acc[5][2];
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int ic = 0; ic < 2; ++ic)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[k][ic][e] = 0.f;

    u32x4 pre[12];
    if (t_begin < t_end) {
        fetch(t_begin, pre);
        stage(0, pre);
    }
    int cur = 0;
    for (int t = t_begin; t < t_end; ++t) {
        const bool has_next = t + 1 < t_end;
        __syncthreads();  // this tile is staged; every wave has finished the previous tile (its buffer is written below)
        if (has_next) fetch(t + 1, pre);
        const char* buf = smem + cur * kW64BufBytes;
        auto read_a = [&](int ks, u32x4 (&fa)[2]) {
#pragma unroll
            for (int ic = 0; ic < 2; ++ic) {
                const u32x2 lo = lds_read_tr16(buf + a_addr[ic][0] + ks * 2048), hi = lds_read_tr16(buf + a_addr[ic][1] + ks * 2048);
                fa[ic] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
        };
        auto read_b = [&](int ks, u32x4 (&fb)[5]) {
#pragma unroll
            for (int k = 0; k < 5; ++k)
                if (k < 4 || ntaps == 5) {
                    const u32x2 lo = lds_read_tr16(buf + b_addr[k][0] + ks * 2048), hi = lds_read_tr16(buf + b_addr[k][1] + ks * 2048);
                    fb[k] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                }
        };
        u32x4 fa[2][2], fb[2][5];
        read_a(0, fa[0]);
        read_b(0, fb[0]);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if (ks + 1 < NKS) {
                read_a(ks + 1, fa[(ks + 1) & 1]);
                read_b(ks + 1, fb[(ks + 1) & 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 5; ++k)
                if (k < 4 || ntaps == 5)
#pragma unroll
                    for (int ic = 0; ic < 2; ++ic) Mma<bf16_t, 32>::run(fa[ks & 1][ic], fb[ks & 1][k], acc[k][ic]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (has_next) stage(cur ^ 1, pre);
        cur ^= 1;
    }

    // one slice of partials per workgroup: dw[co][tap * 64 + ci]
    float* dst = part + (int64_t)blockIdx.x * C * KD;
#pragma unroll
    for (int k = 0; k < 5; ++k)
        if (k < 4 || ntaps == 5) {
            const int col = (pw + 2 * k) * C + 32 * ii + (lane & 31);
#pragma unroll
            for (int ic = 0; ic < 2; ++ic)
#pragma unroll
                for (int e = 0; e < 16; ++e) dst[(int64_t)(32 * ic + acc_row<32>(lane, e)) * KD + col] = acc[k][ic][e];
        }
}


// ---- bf16 backward-weight of the 16 -> 64 channel 4 x 4 layer (space-to-depth stems) -----------------------------
// dw[64][16 taps x 16 channels] over millions of pixels: the result is 64 KB of floats, so a wave keeps HALF of it in
// accumulators (2 blocks of output channels x 4 of the 8 blocks of tap pairs = 128 registers; all 256 leave the register
// allocator no slack and the prefetch spills) and the waves of a persistent workgroup split tap pairs x pixels, 2 x 2.  A tile is two output rows of one image, staged once as they lie in memory:
// `dy` as 2 x 128 pixel slots of 128 bytes (columns W .. 127 zero), `x` as 5 x 128 slots of 32 bytes (two rows above,
// one below; two zero columns left, zeros outside the image).  The contraction runs over the 256 slots of the dy tile in
// 16 steps of 16 pixels, eight per wave; the x operand of tap (r, s) for slot q is slot q + 128 r + s of the patch: a
// constant offset in the LDS read, and the zero columns of dy cancel whatever finite value the patch holds where a
// slot is no pixel (a zeroed guard follows the patch).  Operands are formed by the LDS transpose read (see
// conv_wgrad_tr_kernel); in the x operand the lane halves of a 32-column block are two neighbouring taps.  A step
// costs 2 + 4 operand fragments for 8 MFMAs.  The next tile is fetched into registers before the steps and written to
// the other LDS buffer after them.  At the end the two waves of each half are summed through LDS and leave as ONE
// slice of partials per workgroup.
struct WStemArgs {
    int tiles;          // N * H / 2
    int tiles_per_wg;   // consecutive tiles per workgroup
};
constexpr int kWStemDyBytes = 2 * 128 * 128, kWStemXBytes = 5 * 128 * 32, kWStemGuard = 256;
constexpr int kWStemBufBytes = kWStemDyBytes + kWStemXBytes + kWStemGuard;
static_assert(2 * kWStemBufBytes >= 2 * 4 * 2 * 16 * 64 * 4, "the final sum stages two waves' accumulators in the tile buffers");

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void conv4x4_c16_wgrad_bf16_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ dy, float* __restrict__ part, WgradGeom g, WStemArgs a)
{
    constexpr int CI = 16, CO = 64, KD = 16 * CI;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int W = g.W, H = g.H, H2 = H / 2;

    for (int b = 0; b < 2; ++b)
        if (tid < kWStemGuard / 16) *(u32x4*)(smem + b * kWStemBufBytes + kWStemDyBytes + kWStemXBytes + tid * 16) = u32x4{0u, 0u, 0u, 0u};

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)g.N * H * W * CI * 2u);
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (uint32_t)g.N * H * W * CO * 2u);
    const int t_begin = blockIdx.x * a.tiles_per_wg, t_end = min(a.tiles, t_begin + a.tiles_per_wg);

    // fetch: dy chunk i = run tid & 7 of column (tid >> 3) + 32 (i & 3) of tile row i >> 2; x chunk j = half tid & 1 of
    // patch slot tid >> 1 (input column (tid >> 1) - 2) of patch row j
    uint32_t dy_col[4], dy_lds[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int col = (tid >> 3) + 32 * q;
        dy_col[q] = col < W ? (uint32_t)(col * CO + (tid & 7) * 8) * 2u : kOutOfRange;
        dy_lds[q] = (uint32_t)swizzled_chunk(col, tid & 7, 128);  // a row of 128 slots is 64 lines: the swizzle repeats per row
    }
    const int xc = (tid >> 1) - 2;
    const uint32_t x_col = (xc >= 0 && xc < W) ? (uint32_t)(xc * CI + (tid & 1) * 8) * 2u : kOutOfRange;
    const uint32_t x_lds = (uint32_t)(kWStemDyBytes + (tid >> 1) * 32 + (tid & 1) * 16);
    auto fetch = [&](int t, u32x4 (&pre)[13]) {
        const int n = t / H2, h0 = (t - n * H2) * 2;  // first output row of the tile
        const uint32_t img_row = (uint32_t)(n * H);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t off = (img_row + (uint32_t)(h0 + (i >> 2))) * (uint32_t)(W * CO * 2);
            pre[i] = load16(rdy, dy_col[i & 3] != kOutOfRange ? off + dy_col[i & 3] : kOutOfRange);
        }
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int hr = h0 - 2 + j;
            const bool ok = hr >= 0 && hr < H && x_col != kOutOfRange;
            pre[8 + j] = load16(rx, ok ? (img_row + (uint32_t)hr) * (uint32_t)(W * CI * 2) + x_col : kOutOfRange);
        }
    };
    auto stage = [&](int buf, const u32x4 (&pre)[13]) {
        char* base = smem + buf * kWStemBufBytes;
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4*)(base + (i >> 2) * 16384 + dy_lds[i & 3]) = pre[i];
#pragma unroll
        for (int j = 0; j < 5; ++j) *(u32x4*)(base + j * 4096 + x_lds) = pre[8 + j];
    };

    // operand reads: lane (j16, cs, kg) addresses pixel slot 8 kg + j16 / 4 (+ 4 for the second half) of a step;
    // dy: channels 16 cs + 4 (j16 % 4) .. + 3 of a 32-channel block; x: channels 4 (j16 % 4) .. + 3 of tap 2 * pair + cs
    const int j16 = lane & 15, cs = (lane >> 4) & 1, kg = lane >> 5;
    const int frag_row = 8 * kg + (j16 >> 2);
    uint32_t a_addr[2][2];  // [output-channel block][half]
    uint32_t b_addr[2];     // [half]; tap pair p adds ((p >> 1) * 128 + 2 * (p & 1)) * 32
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
        for (int ic = 0; ic < 2; ++ic)
            a_addr[ic][hh] = (uint32_t)(swizzled_chunk(frag_row + 4 * hh, 4 * ic + cs * 2 + ((j16 & 3) >> 1), 128) + (j16 & 1) * 8);
        b_addr[hh] = (uint32_t)(kWStemDyBytes + (frag_row + 4 * hh + cs) * 32 + (j16 & 3) * 8);
    }

    const int ph = wave & 1, kh = wave >> 1;  // this wave: tap pairs 4 ph .. + 3, steps 8 kh .. + 7 of a tile
    typename Mma<bf16_t, 32>::Acc acc[4][2];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int ic = 0; ic < 2; ++ic)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[p][ic][e] = 0.f;

    u32x4 pre[13];
    if (t_begin < t_end) {
        fetch(t_begin, pre);
        stage(0, pre);
    }
    int cur = 0;
    for (int t = t_begin; t < t_end; ++t) {
        const bool has_next = t + 1 < t_end;
        __syncthreads();  // this tile is staged; every wave has finished the previous tile (its buffer is written below)
        if (has_next) fetch(t + 1, pre);
        const char* buf = smem + cur * kWStemBufBytes;
        // step ks of the tile: slots 16 ks .. + 15 = tile row ks >> 3, columns 16 (ks & 7) ..
        auto read_a = [&](int ks, u32x4 (&fa)[2]) {
#pragma unroll
            for (int ic = 0; ic < 2; ++ic) {
                const u32x2 lo = lds_read_tr16(buf + a_addr[ic][0] + ks * 2048), hi = lds_read_tr16(buf + a_addr[ic][1] + ks * 2048);
                fa[ic] = u32x4{lo[0], lo[1], hi[0], hi[1]};
            }
        };
        auto read_b = [&](int ks, int p) {  // p: pair within this wave's half; tap row 2 ph + (p >> 1), tap columns 2 (p & 1), + 1
            const int off = ks * 512 + (((2 * ph + (p >> 1)) * 128 + 2 * (p & 1)) * 32);
            const u32x2 lo = lds_read_tr16(buf + b_addr[0] + off), hi = lds_read_tr16(buf + b_addr[1] + off);
            return u32x4{lo[0], lo[1], hi[0], hi[1]};
        };
        u32x4 fa[2][2], fb[2][4];
        read_a(8 * kh, fa[0]);
#pragma unroll
        for (int p = 0; p < 4; ++p) fb[0][p] = read_b(8 * kh, p);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (i + 1 < 8) {
                read_a(8 * kh + i + 1, fa[(i + 1) & 1]);
#pragma unroll
                for (int p = 0; p < 4; ++p) fb[(i + 1) & 1][p] = read_b(8 * kh + i + 1, p);
            }
            __builtin_amdgcn_sched_barrier(0);  // the next step's operand reads go out before this step's MFMAs
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int ic = 0; ic < 2; ++ic) Mma<bf16_t, 32>::run(fa[i & 1][ic], fb[i & 1][p], acc[p][ic]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (has_next) stage(cur ^ 1, pre);
        cur ^= 1;
    }

    // the two waves of each half: the one with the later steps parks its sums in LDS (lane-contiguous), the other adds
    // them to its own and writes its half of the workgroup's slice dw[co][tap * 16 + ci]
    float* red = (float*)smem + ph * (4 * 2 * 16 * 64);  // [pair][block][register][lane]
    float* dst = part + (int64_t)blockIdx.x * CO * KD;
    __syncthreads();
    if (kh == 1) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int ic = 0; ic < 2; ++ic)
#pragma unroll
                for (int e = 0; e < 16; ++e) red[((p * 2 + ic) * 16 + e) * 64 + lane] = acc[p][ic][e];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int ic = 0; ic < 2; ++ic)
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    dst[(int64_t)(32 * ic + acc_row<32>(lane, e)) * KD + (4 * ph + p) * 32 + (lane & 31)] =
                        acc[p][ic][e] + red[((p * 2 + ic) * 16 + e) * 64 + lane];
    }
}

// Backward-weight of an fp32 layer with 16 input and 16 output channels.  The GEMM output is only
// 16 x (R*S*16), so LDS tiling buys nothing: each wave streams its own output pixels straight from
// global memory into the 16x16x4 MFMA operand layout (lane = (pixel % 4) * 16 + channel, one
// coalesced 256-byte load per operand and step) and keeps all R*S accumulator tiles in registers.
// Waves of a workgroup interleave at 4-pixel granularity, are summed through LDS in wave order and
// written as one slice of the partial buffer.
template <int R, int S>
__global__ __launch_bounds__(kThreads) void conv_wgrad_c16_kernel(const float* __restrict__ x,
                                                                  const float* __restrict__ dy,
                                                                  float* __restrict__ part, WgradGeom g)
{
    constexpr int TAPS = R * S;
    __shared__ float red[4][TAPS * 256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 15, kq = lane >> 4;
    const int m_begin = blockIdx.x * g.m_per_split;
    const int m_end = min(g.M, m_begin + g.m_per_split);
    const int nsteps = (m_end - m_begin + 15) / 16;
    const __amdgpu_buffer_rsrc_t rdy = make_rsrc(dy, (uint32_t)g.M * 16 * 4);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)g.N * g.H * g.W * 16 * 4);

    f32x4 acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    int m = m_begin + 4 * wave + kq;
    int wo = m % g.Wo, tq = m / g.Wo, ho = tq % g.Ho, n = tq / g.Ho;
    // operands of the pixel (n, ho, wo) this lane holds in the current step; zeros past the slice
    auto fetch = [&](float& a, float (&b)[TAPS]) {
        const bool live = m < m_end;
        a = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(rdy, live ? (uint32_t)(m * 16 + col) * 4u : kOutOfRange, 0, 0));
        const int hi0 = ho * g.stride - g.pad, wi0 = wo * g.stride - g.pad;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int hi = hi0 + r;
            const bool hok = live && hi >= 0 && hi < g.H;
            const uint32_t rowoff = (uint32_t)((n * g.H + hi) * g.W);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const int wi = wi0 + s;
                const bool ok = hok && wi >= 0 && wi < g.W;
                b[r * S + s] = __builtin_bit_cast(
                    float, __builtin_amdgcn_raw_buffer_load_b32(
                               rx, ok ? ((rowoff + (uint32_t)wi) * 16u + (uint32_t)col) * 4u : kOutOfRange, 0, 0));
            }
        }
        m += 16;
        wo += 16;
        while (wo >= g.Wo) {
            wo -= g.Wo;
            if (++ho == g.Ho) { ho = 0; ++n; }
        }
    };
    // four steps of operands in flight per wave; steps past the slice read zeros
    constexpr int DEPTH = 4;
    float a[DEPTH], b[DEPTH][TAPS];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) fetch(a[d], b[d]);
    for (int it = 0; it < nsteps; it += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[d], b[d][t], acc[t], 0, 0, 0);
            fetch(a[d], b[d]);
        }
    }
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[wave][(t * 4 + j) * 64 + lane] = acc[t][j];
    __syncthreads();
    float* dst = part + (int64_t)blockIdx.x * 16 * g.Kdim;
#pragma unroll
    for (int t = 0; t < TAPS; ++t) {
        const int idx = t * 256 + tid;
        const float v = ((red[0][idx] + red[1][idx]) + red[2][idx]) + red[3][idx];
        const int j = tid >> 6, l = tid & 63, co = (l >> 4) * 4 + j, ci = l & 15;
        dst[co * g.Kdim + t * 16 + ci] = v;
    }
}

// dw[i] = sum over slices of part[slice][i] in a fixed summation tree (run-to-run identical).
// A workgroup owns 32 consecutive elements: 8 threads cover them with 16-byte loads, 32 such
// thread rows each add every 32nd slice, and the 32 row sums are then added in row order.
// VW = 4 needs n % 4 == 0 and a 16-byte aligned partial buffer.
template <int VW>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int n,
                                                           int splits)
{
    constexpr int COLS = 32 / VW, ROWS = 256 / COLS;
    __shared__ float red[ROWS][33];
    const int cg = threadIdx.x % COLS, row = threadIdx.x / COLS;
    const int i = blockIdx.x * 32 + cg * VW;
    float s[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) s[v] = 0.f;
    if (i < n) {
#pragma unroll 4
        for (int k = row; k < splits; k += ROWS) {
            const float* src = part + (int64_t)k * n + i;
            if (VW == 4) {
                const f32x4 t = *(const f32x4*)src;
#pragma unroll
                for (int v = 0; v < VW; ++v) s[v] += t[v];
            } else {
                s[0] += src[0];
            }
        }
    }
#pragma unroll
    for (int v = 0; v < VW; ++v) red[row][cg * VW + v] = s[v];
    __syncthreads();
    const int c = threadIdx.x;
    if (c < 32 && blockIdx.x * 32 + c < n) {
        float t = red[0][c];
#pragma unroll 8
        for (int k = 1; k < ROWS; ++k) t += red[k][c];
        dw[blockIdx.x * 32 + c] = t;
    }
}

// The same sum for few slices (<= 8): there the tree above would leave most thread rows idle, so each
// thread adds the slices of 4 consecutive elements in ascending order.
// s[v] += part[k * n + v] for k = 0 .. splits-1 in that order, 8 loads in flight.
template <int VW>
__device__ inline void flat_slice_sum(const float* __restrict__ src0, int n, int splits, float (&s)[VW])
{
    for (int k0 = 0; k0 < splits; k0 += 8) {
        f32x4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float* src = src0 + (int64_t)(k0 + u) * n;
            if (k0 + u < splits) {
                if (VW == 4) t[u] = *(const f32x4*)src; else t[u] = f32x4{src[0], 0.f, 0.f, 0.f};
            } else {
                t[u] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u < splits)
#pragma unroll
                for (int v = 0; v < VW; ++v) s[v] += t[u][v];
    }
}

template <int VW>
__global__ __launch_bounds__(256) void wgrad_reduce_few_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                               int n, int splits)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VW;
    if (i >= n) return;
    float s[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) s[v] = 0.f;
    flat_slice_sum<VW>(part + i, n, splits, s);
    if (VW == 4)
        *(f32x4*)(dw + i) = f32x4{s[0], s[1], s[2], s[3]};
    else
        dw[i] = s[0];
}

// The flat loop (one thread adds the slices of its 4 elements in ascending order) is used when there are
// few slices, and also whenever the gradient is long enough for its 1024-element workgroups to fill the
// chip: it reads whole 4 KiB runs of every slice, where the tree reads 128-byte pieces.
inline bool wgrad_reduce_flat(size_t n, int splits) { return splits <= 8 || n >= 65536; }

// All slice sums of a block's conv layers in ONE launch (the per-layer sums are tiny and the idle gap
// between two launches costs as much as each of them).  A workgroup looks up its task and then does
// exactly what the two kernels above do: the flat loop over 1024 elements or the tree over 32.
struct ReduceTask {
    const float* part;
    float* dw;
    int n, splits;
    int block_begin;  // first workgroup of the task
    int flat;         // flat loop over 1024 elements per workgroup, else the tree over 32
};

template <int VW>
__global__ __launch_bounds__(256) void wgrad_reduce_all_kernel(const ReduceTask* __restrict__ tasks, int n_tasks)
{
    constexpr int COLS = 32 / VW, ROWS = 256 / COLS;
    __shared__ float red[ROWS][33];
    int p = 0, hi = n_tasks;  // last task whose first workgroup is not after this one (block_begin ascends)
    while (hi - p > 1) {
        const int mid = (p + hi) >> 1;
        if ((int)blockIdx.x >= tasks[mid].block_begin) p = mid; else hi = mid;
    }
    const ReduceTask t = tasks[p];
    const int blk = (int)blockIdx.x - t.block_begin;
    const float* __restrict__ part = t.part;
    const int n = t.n, splits = t.splits;
    if (t.flat) {  // uniform per workgroup
        const int64_t i = ((int64_t)blk * 256 + threadIdx.x) * VW;
        if (i >= n) return;
        float s[VW];
#pragma unroll
        for (int v = 0; v < VW; ++v) s[v] = 0.f;
        flat_slice_sum<VW>(part + i, n, splits, s);
        if (VW == 4)
            *(f32x4*)(t.dw + i) = f32x4{s[0], s[1], s[2], s[3]};
        else
            t.dw[i] = s[0];
        return;
    }
    const int cg = threadIdx.x % COLS, row = threadIdx.x / COLS;
    const int i = blk * 32 + cg * VW;
    float s[VW];
#pragma unroll
    for (int v = 0; v < VW; ++v) s[v] = 0.f;
    if (i < n) {
#pragma unroll 4
        for (int k = row; k < splits; k += ROWS) {
            const float* src = part + (int64_t)k * n + i;
            if (VW == 4) {
                const f32x4 v4 = *(const f32x4*)src;
#pragma unroll
                for (int v = 0; v < VW; ++v) s[v] += v4[v];
            } else {
                s[0] += src[0];
            }
        }
    }
#pragma unroll
    for (int v = 0; v < VW; ++v) red[row][cg * VW + v] = s[v];
    __syncthreads();
    const int c = threadIdx.x;
    if (c < 32 && blk * 32 + c < n) {
        float acc = red[0][c];
#pragma unroll 8
        for (int k = 1; k < ROWS; ++k) acc += red[k][c];
        t.dw[blk * 32 + c] = acc;
    }
}

// ---- host-side dispatch -------------------------------------------------------------------------
struct KernelName {
    char text[96];
};

// One name per kernel instantiation, e.g. "conv_gather_gemm<fp32,mfma32,BM128,BN64,BK16,vec>".
template <typename TL, bool VEC, bool WGRAD>
const char* tile_name()
{
    static const KernelName name = [] {
        KernelName k;
        snprintf(k.text, sizeof(k.text), "%s<%s,mfma%d,BM%d,BN%d,BK%d,%s>", WGRAD ? "conv_wgrad" : "conv_gather_gemm",
                 sizeof(typename TL::T) == 2 ? "bf16" : "fp32", TL::MT, TL::BM, TL::BN, TL::BK, VEC ? "vec" : "scalar");
        return k;
    }();
    return name.text;
}

template <typename TL, bool VEC, bool DIL>
int run_gather(const GatherGeom& g, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    typedef typename TL::T T;
    const int64_t tiles = (int64_t)ceil_div(g.M, TL::BM) * ceil_div(g.Co, TL::BN);
    DSP_REQUIRE(tiles > 0 && tiles < (1ll << 31), DSP_EINVAL, "conv: bad tile count");
    auto kern = conv_gather_gemm_kernel<TL, VEC, DIL>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done && TL::LDS_BYTES > 48 * 1024) {
        DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
        attr_done = true;
    }
    {
        ProfScope ps(tile_name<TL, VEC, false>(), flops, 0);
        DSP_LAUNCH(ps, kern, dim3((unsigned)tiles, g.in1 ? 2 : 1, (unsigned)g.groups), dim3(kThreads), TL::LDS_BYTES, st,
                   (const T*)in, (const T*)w, (T*)out, g);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename TL>
int run_gather_v(const GatherGeom& g, bool vec, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    // (backward-data of strided layers arrives here as dense per-parity-class problems, so no launch dilates)
    if (!vec) return run_gather<TL, false, false>(g, in, w, out, st, flops);
    return run_gather<TL, true, false>(g, in, w, out, st, flops);
}

// Enough workgroups to put more than one on each of the 256 compute units.
constexpr int64_t kEnoughTiles = 384;

inline int64_t tile_count(const GatherGeom& g, int bm, int bn)
{
    return (int64_t)ceil_div(g.M, bm) * ceil_div(g.Co, bn) * g.groups;
}

// The register-resident-filter kernel: fp32, 3x3, 16 gathered channels, 16 or 32 output channels, no
// dilation, 16-byte aligned activations.  (The kernel also handles 32 gathered channels, but there
// the per-wave filter load outweighs the saved LDS traffic and the tiled kernel is faster.)
template <typename T>
bool direct_eligible(const GatherGeom& g, const void* in, const void* out)
{
    return sizeof(T) == 4 && g.groups == 1 && g.R == 3 && g.S == 3 && g.idil == 1 && g.Ci == 16 && (g.Co == 16 || g.Co == 32) &&
           ((uintptr_t)in % 16) == 0 && ((uintptr_t)out % 16) == 0;
}

// Workgroups of the direct kernel: one per compute unit unless there are fewer pixel groups (measured in the
// three-stream pipeline: 256 beats 128, 192, 384, 512 and 1024).
inline int direct_grid(const GatherGeom& g)
{
    const int per_block = 4 / (g.Co / 16);
    const int blocks = ceil_div(ceil_div(g.M, 16), per_block);
    return blocks < 256 ? blocks : 256;
}

// Largest tile of the channel class that still yields enough workgroups; for small problems (the
// CIFAR-sized layers) small tiles with long k steps: there the kernel is bound by the latency of the
// gathers, and what helps is many workgroups with many bytes in flight each.
// Returns the tile id used by dispatch_gather and the tile's row count.
// The direct-to-LDS kernel: bf16, gathered channels a multiple of 64 (a k tile never straddles two taps), at most 32
// taps (one mask word per row), no dilation, whole 128-wide column tiles, enough 256-row tiles for the chip, and a
// long contraction (K >= 2304: with one workgroup per compute unit nothing overlaps a tile's prologue and epilogue,
// which only long k loops amortise; measured: 3x3 layers of 256 / 512 channels gain 5-10 %, 128-channel ones lose 20 %).
template <typename T>
bool dma_wide(const GatherGeom& g)  // 256 x 256 tiles (half the LDS operand reads per MFMA) where enough of them exist
{
    return g.Co % 256 == 0 && tile_count(g, 256, 256) >= 192;
}
template <typename T>
bool dma_eligible(const GatherGeom& g)
{
    return sizeof(T) == 2 && g.groups == 1 && g.Ci % 64 == 0 && g.R * g.S <= 32 && g.idil == 1 && g.oh_mul == 0 && g.Co % 128 == 0 && g.Kdim >= 2304 &&
           (tile_count(g, 256, 128) >= 192 || dma_wide<T>(g));
}

// The register-resident-filter kernel: bf16, 3x3 / stride 1 / pad 1, 64 channels on both sides, no groups, rows wide
// enough to fill the chip, and image rows of 51 .. 62 pixels (the input rows of a 256-pixel tile are kept as 8 x 64 pixels).
inline int c64_buf_bytes()
{
    const int patch = kC64Chunks * kThreads * 16;
    const int epi = 256 * kC64EpiRowB + 32 * 64 * 2 * (int)sizeof(float);
    return (patch > epi ? patch : epi + 1023) / 1024 * 1024;
}
// one persistent workgroup per compute unit = one partial row of column sums per instance
inline int c64_workgroups(const GatherGeom& g) { const int t = ceil_div(g.M, 256); return t < 256 ? t : 256; }
template <typename T>
bool c64_eligible(const GatherGeom& g)
{
    return sizeof(T) == 2 && g.groups == 1 && g.Ci == 64 && g.Co == 64 && g.R == 3 && g.S == 3 && g.ostride == 1 && g.idil == 1 &&
           g.pad_h == 1 && g.pad_w == 1 && g.Hi == g.Ho && g.Wi == g.Wo && g.oh_mul == 0 && g.M >= 256 * 256 &&
           g.Wi + 2 <= kC64Pitch && 4 + 254 / g.Wi <= kC64Chunks / 2;  // rows of the patch: 64 pixels wide, at most 8
}

// The 16 -> 64 channel 4 x 4 kernel (space-to-depth stems): bf16, stride 1, pad 2 with Ho = H and Wo = W, rows of at most
// 125 pixels (a patch row holds 128), a map large enough to fill the chip; forward only.
inline int c16_workgroups(const GatherGeom& g)
{
    const int t = ceil_div(g.M, 128);
    return t < kC16MaxWorkgroups ? t : kC16MaxWorkgroups;  // two persistent workgroups per compute unit
}
template <typename T>
bool c16_eligible(const GatherGeom& g)
{
    return sizeof(T) == 2 && g.groups == 1 && g.Ci == 16 && g.Co == 64 && g.R == 4 && g.S == 4 && g.ostride == 1 && g.idil == 1 &&
           g.pad_h == 2 && g.pad_w == 2 && g.Hi == g.Ho && g.Wi == g.Wo && g.oh_mul == 0 && g.M >= 256 * 256 &&
           g.Wi + 3 <= kC16Pitch && g.Wi >= 64 && !g.accum;  // a tile of 128 pixels then touches at most 3 rows
}
template <typename T>
int select_gather_tile(const GatherGeom& g, int* bm)
{
    if (c64_eligible<T>(g)) { *bm = 256; return 21; }
    if (c16_eligible<T>(g)) { *bm = 128; return 22; }
    if (dma_eligible<T>(g)) { *bm = 256; return 20; }
    if (g.Co <= 16) {
        // (bf16 always takes the 64-row tile: measured in the four-stream resnet56 pipeline)
        if (sizeof(T) == 4 && tile_count(g, 256, 16) >= kEnoughTiles) { *bm = 256; return 0; }
        *bm = 64;
        return 1;
    }
    if (g.Co <= 32) {
        if (tile_count(g, 256, 32) >= kEnoughTiles) { *bm = 256; return 2; }
        if (tile_count(g, 128, 32) >= kEnoughTiles) { *bm = 128; return 3; }
        *bm = 64;
        return 7;
    }
    if (g.Co % 128 == 0 && tile_count(g, 128, 128) >= kEnoughTiles) { *bm = 128; return 4; }
    if (sizeof(T) == 2 && g.Co == 64 && tile_count(g, 256, 64) >= kEnoughTiles) { *bm = 256; return 10; }
    if (tile_count(g, 128, 64) >= kEnoughTiles) { *bm = 128; return 5; }
    if (tile_count(g, 64, 64) >= kEnoughTiles) { *bm = 64; return 6; }
    *bm = 32;
    return 8;
}

template <typename TL>
int run_dma(const GatherGeom& g, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    const int64_t tiles = (int64_t)ceil_div(g.M, TL::BM) * ceil_div(g.Co, TL::BN);
    DSP_REQUIRE(tiles > 0 && tiles < (1ll << 31), DSP_EINVAL, "conv: bad tile count");
    auto kern = conv_dma_gemm_kernel<TL>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LDS_BYTES));
        attr_done = true;
    }
    static const KernelName name = [] {
        KernelName k;
        snprintf(k.text, sizeof(k.text), "conv_dma_gemm<bf16,mfma32,BM%d,BN%d,BK%d>", TL::BM, TL::BN, TL::BK);
        return k;
    }();
    {
        ProfScope ps(name.text, flops, 0);
        DSP_LAUNCH(ps, kern, dim3((unsigned)tiles, g.in1 ? 2 : 1), dim3(kThreads), TL::LDS_BYTES, st, (const bf16_t*)in,
                   (const bf16_t*)w, (bf16_t*)out, g);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int run_c64(const GatherGeom& g, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    C64Args a{};
    a.buf_bytes = c64_buf_bytes();
    a.tiles = ceil_div(g.M, 256);
    a.twin = g.in1 ? 1 : 0;
    const int grid = c64_workgroups(g);
    const int lds = kC64Zero + 2 * a.buf_bytes;
    auto kern = g.accum ? conv3x3_c64_bf16_kernel<true> : conv3x3_c64_bf16_kernel<false>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        DSP_HIP(hipFuncSetAttribute((const void*)conv3x3_c64_bf16_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        DSP_HIP(hipFuncSetAttribute((const void*)conv3x3_c64_bf16_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_done = true;
    }
    {
        ProfScope ps("conv3x3_c64<bf16,filters in registers>", flops, 0);
        DSP_LAUNCH(ps, kern, dim3((unsigned)grid), dim3(kThreads), lds, st, (const bf16_t*)in, (const bf16_t*)w, (bf16_t*)out, g, a);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}


int run_c16(const GatherGeom& g, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    C16Args a{};
    a.tiles = ceil_div(g.M, 128);
    a.twin = g.in1 ? 1 : 0;
    static std::atomic<bool> attr_done{false};
    if (!attr_done) {
        DSP_HIP(hipFuncSetAttribute((const void*)conv4x4_c16_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kC16Lds));
        attr_done = true;
    }
    {
        ProfScope ps("conv4x4_c16<bf16,filters in registers>", flops, 0);
        DSP_LAUNCH(ps, conv4x4_c16_bf16_kernel, dim3((unsigned)c16_workgroups(g)), dim3(kThreads), kC16Lds, st, (const bf16_t*)in,
                   (const bf16_t*)w, (bf16_t*)out, g, a);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename T>
int dispatch_gather(GatherGeom g, bool accum, const void* in, const void* w, void* out, hipStream_t st, double flops)
{
    constexpr int E = 16 / (int)sizeof(T);
    if (direct_eligible<T>(g, in, out)) {
        g.accum = accum ? 1 : 0;
        const dim3 grid(direct_grid(g), g.in1 ? 2 : 1);
        ProfScope ps(g.Ci == 16 ? "conv3x3_direct<fp32,ci16>" : "conv3x3_direct<fp32,ci32>", flops, 0);
        if (g.Ci == 16)
            DSP_LAUNCH(ps, conv3x3_direct_f32_kernel<1>, grid, dim3(kThreads), 0, st, (const float*)in, (const float*)w,
                       (float*)out, g);
        else
            DSP_LAUNCH(ps, conv3x3_direct_f32_kernel<2>, grid, dim3(kThreads), 0, st, (const float*)in, (const float*)w,
                       (float*)out, g);
        DSP_HIP(hipGetLastError());
        return DSP_OK;
    }
    constexpr int KB = 128;  // bytes of k per LDS row of the large tiles: 64 bf16 / 32 floats
    // 16-byte gathers need channel runs of E elements and 16-byte aligned bases; the per-row tap masks
    // hold up to 64 taps (larger filters, and dilated gathers of more than 32 taps, take the generic path)
    const bool vec = (g.Ci % E) == 0 && ((uintptr_t)in % 16) == 0 && ((uintptr_t)w % 16) == 0 &&
                     g.R * g.S <= (g.idil == 2 ? 32 : 64);
    g.accum = accum ? 1 : 0;
    g.out_vec = ((g.Co % E) == 0 && ((uintptr_t)out % 16) == 0) ? 1 : 0;
    int bm;
    int id = select_gather_tile<T>(g, &bm);
    if (id == 21) {
        const bool aligned = vec && g.out_vec && ((uintptr_t)g.in1 % 16) == 0 && ((uintptr_t)g.out1 % 16) == 0;
        if (aligned) return run_c64(g, in, w, out, st, flops);
        // unaligned tensors (single-layer calls only) take the register-staged tiles; their partial rows differ
        DSP_REQUIRE(g.stats == nullptr, DSP_EINVAL, "conv forward with column sums: x, w and y must be 16-byte aligned");
        id = 10;
    }
    if (id == 22) {
        const bool aligned = vec && g.out_vec && ((uintptr_t)g.in1 % 16) == 0 && ((uintptr_t)g.out1 % 16) == 0;
        if (aligned && !accum) return run_c16(g, in, w, out, st, flops);
        // unaligned tensors and accumulating calls (single-layer calls only) take the register-staged tiles
        DSP_REQUIRE(g.stats == nullptr, DSP_EINVAL, "conv forward with column sums: x, w and y must be 16-byte aligned");
        id = 10;
    }
    if (id == 20) {
        const bool aligned = vec && ((uintptr_t)g.in1 % 16) == 0 && ((uintptr_t)g.out1 % 16) == 0;
        if (aligned && g.out_vec) {
            if (dma_wide<T>(g)) return run_dma<DmaTile<256, 256, 2, 2, 64, 4>>(g, in, w, out, st, flops);
            return run_dma<DmaTile<256, 128, 2, 2, 128, 3>>(g, in, w, out, st, flops);
        }
        // unaligned tensors (single-layer calls only) take the register-staged tiles; their row tiles differ
        DSP_REQUIRE(g.stats == nullptr, DSP_EINVAL, "conv forward with column sums: x, w and y must be 16-byte aligned");
        id = -1;
    }
    if (id < 0) {
        if (g.Co % 128 == 0 && tile_count(g, 128, 128) >= kEnoughTiles) id = 4;
        else if (tile_count(g, 128, 64) >= kEnoughTiles) id = 5;
        else if (tile_count(g, 64, 64) >= kEnoughTiles) id = 6;
        else id = 8;
    }
    switch (id) {
    case 0: return run_gather_v<Tile<T, 16, 4, 1, 4, 1, 64, 2>>(g, vec, in, w, out, st, flops);
    case 1: return run_gather_v<Tile<T, 16, 4, 1, 1, 1, 64, 2>>(g, vec, in, w, out, st, flops);
    case 2: return run_gather_v<Tile<T, 32, 4, 1, 2, 1, 64, 2>>(g, vec, in, w, out, st, flops);
    case 3: return run_gather_v<Tile<T, 32, 4, 1, 1, 1, 128, 2>>(g, vec, in, w, out, st, flops);
    case 4:
        // short contractions (1x1 filters over few channels) of bf16: 32-deep k steps and three workgroups per
        // compute unit; the two-tile prologue is half as long and the epilogues of more workgroups overlap
        if (sizeof(T) == 2 && g.Kdim <= 512) return run_gather_v<Tile<T, 32, 2, 2, 2, 2, 64, 2>>(g, vec, in, w, out, st, flops);
        return run_gather_v<Tile<T, 32, 2, 2, 2, 2, KB, 2>>(g, vec, in, w, out, st, flops);
    case 5: return run_gather_v<Tile<T, 32, 2, 2, 2, 1, KB, 2>>(g, vec, in, w, out, st, flops);
    case 6: return run_gather_v<Tile<T, 32, 2, 2, 1, 1, KB, 2>>(g, vec, in, w, out, st, flops);
    case 7: return run_gather_v<Tile<T, 16, 4, 1, 1, 2, 128, 2>>(g, vec, in, w, out, st, flops);
    case 10: return run_gather_v<Tile<T, 32, 4, 1, 2, 2, 64, 2>>(g, vec, in, w, out, st, flops);
    default: return run_gather_v<Tile<T, 16, 2, 2, 1, 1, 256, 2>>(g, vec, in, w, out, st, flops);
    }
}

template <typename TL, bool VEC>
int run_wgrad(const WgradGeom& g, int splits, const void* x, const void* dy, float* dst, hipStream_t st, double flops)
{
    typedef typename TL::T T;
    const int tiles = ceil_div(g.Co, TL::BM) * ceil_div(g.Kdim, TL::BN);
    auto kern = conv_wgrad_kernel<TL, VEC>;
    static std::atomic<bool> attr_done{false};
    if (!attr_done && TL::LOAD_BYTES > 48 * 1024) {
        DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::LOAD_BYTES));
        attr_done = true;
    }
    {
        ProfScope ps(tile_name<TL, VEC, true>(), flops, 0);
        DSP_LAUNCH(ps, kern, dim3(tiles, splits, g.groups), dim3(kThreads), TL::LOAD_BYTES, st, (const T*)x, (const T*)dy, dst, g);
    }
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

// The transpose-read kernel serves bf16 tiles of 64 or 128 channels/columns.
template <typename TL>
constexpr bool kWgradTr = sizeof(typename TL::T) == 2 && TL::MT == 32 && (TL::BM == 64 || TL::BM == 128) &&
                          (TL::BN == 64 || TL::BN == 128) && TL::BK == 64;

template <typename TL>
int run_wgrad_tr(const WgradGeom& g, int splits, const void* x, const void* dy, float* dst, hipStream_t st, double flops)
{
    if constexpr (kWgradTr<TL>) {
        constexpr int LDS = 2 * TL::BK * (TL::BM + TL::BN) * 2;
        const int tiles = ceil_div(g.Co, TL::BM) * ceil_div(g.Kdim, TL::BN);
        auto kern = conv_wgrad_tr_kernel<TL>;
        static std::atomic<bool> attr_done{false};
        if (!attr_done && LDS > 48 * 1024) {
            DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS));
            attr_done = true;
        }
        {
            ProfScope ps(tile_name<TL, true, true>(), flops, 0);
            DSP_LAUNCH(ps, kern, dim3(tiles, splits, g.groups), dim3(kThreads), LDS, st, (const bf16_t*)x, (const bf16_t*)dy, dst, g);
        }
        DSP_HIP(hipGetLastError());
        return DSP_OK;
    } else {
        return run_wgrad<TL, true>(g, splits, x, dy, dst, st, flops);
    }
}

template <typename TL>
int run_wgrad_v(const WgradGeom& g, int splits, bool vec, const void* x, const void* dy, float* dst, hipStream_t st,
                double flops)
{
    return vec ? run_wgrad_tr<TL>(g, splits, x, dy, dst, st, flops) : run_wgrad<TL, false>(g, splits, x, dy, dst, st, flops);
}

// Tile of the backward-weight GEMM (output Cout x R*S*Cin) and the m extent of one LDS tile.
struct WgradPlan {
    int bm, bn, bk, id;
};
// One group of a grouped convolution as a convolution of its own (the shape the GEMM tiles are chosen for).
ConvShape one_group(const ConvShape& c)
{
    ConvShape o = c;
    o.Cin = c.Cin / conv_groups(c);
    o.Cout = c.Cout / conv_groups(c);
    o.groups = 1;
    return o;
}

WgradPlan wgrad_plan(int dtype, const ConvShape& cc)
{
    const ConvShape c = one_group(cc);
    // m rows per LDS tile: 128 bytes of k per row; the large fp32 tile keeps 64 (measured: VGG-19's layers)
    const int bk = dtype == DSP_BF16 ? 64 : 32;
    const int64_t kdim = (int64_t)c.R * c.S * c.Cin;
    if (dtype == DSP_BF16) {
        // bf16 has the transpose-read kernel only for 64- and 128-wide tiles; narrow layers run on the 64x64 one
        // (the idle MFMA rows cost less than the register transposes of the narrow tiles)
        if (c.Cout >= 128 && kdim >= 512) return {128, 128, bk, 3};
        return {64, 64, bk, 2};
    }
    if (c.Cout <= 16) return {16, 64, bk, 0};
    if (c.Cout <= 32) return {32, 128, bk, 1};
    if (c.Cout >= 128 && kdim >= 512) return {128, 128, dtype == DSP_BF16 ? 64 : 16, 3};
    return {64, 64, bk, 2};
}

// Slices of the (n, ho, wo) range: about two workgroups per compute unit, each slice a whole number
// of LDS tiles and at least 8 of them.
int wgrad_splits(const ConvShape& cc, const WgradPlan& pl, int* m_per_split)
{
    const ConvShape c = one_group(cc);
    const int64_t M = (int64_t)c.N * c.Ho * c.Wo, Kdim = (int64_t)c.R * c.S * c.Cin;
    const int tiles = ceil_div(c.Cout, pl.bm) * ceil_div(Kdim, pl.bn) * conv_groups(cc);
    // two workgroups per compute unit, one for small problems (below ~1 GMAC, the CIFAR-sized layers: measured in
    // the three-stream pipeline); rounded down: one workgroup too many costs a whole second round
    const int target = (double)M * (double)Kdim * (double)cc.Cout < 1e9 ? 256 : 512;
    int want = target / tiles;
    const int max_by_len = (int)((M + 8 * pl.bk - 1) / (8 * pl.bk));
    if (want > max_by_len) want = max_by_len;
    if (want < 1) want = 1;
    if (want > 256) want = 256;
    int per = (int)((M + want - 1) / want);
    per = ceil_div(per, pl.bk) * pl.bk;
    *m_per_split = per;
    return ceil_div(M, per);
}

// The persistent accumulators-resident kernel: bf16, 3x3 / stride 1 / pad 1, 64 channels on both sides, image rows of
// 51 .. 62 pixels, an even number of them, enough tiles (pairs of rows) for every compute unit.
bool wgrad_c64_eligible(int dtype, const ConvShape& c)
{
    return dtype == DSP_BF16 && conv_groups(c) == 1 && c.Cin == 64 && c.Cout == 64 && c.R == 3 && c.S == 3 && c.stride == 1 &&
           c.pad == 1 && c.Ho == c.H && c.Wo == c.W && c.W >= 51 && c.W <= 62 && c.H % 2 == 0 && (int64_t)c.N * c.H / 2 >= 512;
}
// One slice of partials per workgroup, one workgroup per compute unit.
int wgrad_c64_slices(const ConvShape& c, int* tiles_per_wg)
{
    const int tiles = c.N * c.H / 2;
    const int per = ceil_div(tiles, 256);
    if (tiles_per_wg) *tiles_per_wg = per;
    return ceil_div(tiles, per);
}

// The space-to-depth stem's layer: bf16, 16 -> 64 channels, 4 x 4, stride 1, pad 2 with Ho = H and Wo = W, rows of 64 .. 125
// pixels, an even number of rows, enough tiles for every compute unit.
bool wgrad_stem_eligible(int dtype, const ConvShape& c)
{
    return dtype == DSP_BF16 && conv_groups(c) == 1 && c.Cin == 16 && c.Cout == 64 && c.R == 4 && c.S == 4 && c.stride == 1 &&
           c.pad == 2 && c.Ho == c.H && c.Wo == c.W && c.W >= 64 && c.W + 3 <= 128 && c.H % 2 == 0 && (int64_t)c.N * c.H / 2 >= 256;
}
int wgrad_stem_slices(const ConvShape& c, int* tiles_per_wg)
{
    const int tiles = c.N * c.H / 2;
    const int per = ceil_div(tiles, 256);
    if (tiles_per_wg) *tiles_per_wg = per;
    return ceil_div(tiles, per);
}

// The register-streaming kernel serves fp32 layers with 16 -> 16 channels and 3x3 or 1x1 filters.
bool wgrad_c16_eligible(int dtype, const ConvShape& c)
{
    return dtype == DSP_FP32 && conv_groups(c) == 1 && c.Cin == 16 && c.Cout == 16 &&
           ((c.R == 3 && c.S == 3) || (c.R == 1 && c.S == 1));
}

// About two workgroups per compute unit; a slice is a multiple of the 16 pixels one step covers.
int wgrad_c16_splits(const ConvShape& c, int* m_per_split)
{
    const int64_t M = (int64_t)c.N * c.Ho * c.Wo;
    int per = (int)((M + 511) / 512);
    if (per < 64) per = 64;
    per = ceil_div(per, 16) * 16;
    *m_per_split = per;
    return ceil_div(M, per);
}

template <typename T>
int dispatch_wgrad(const ConvShape& c, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes,
                   hipStream_t st, double flops, bool defer_reduce)
{
    constexpr int E = 16 / (int)sizeof(T);
    constexpr int KB = 128;
    const int dtype = sizeof(T) == 2 ? DSP_BF16 : DSP_FP32;
    const WgradPlan pl = wgrad_plan(dtype, c);
    const int G = conv_groups(c);
    WgradGeom g{};
    g.N = c.N; g.H = c.H; g.W = c.W; g.Ci = c.Cin / G; g.Ho = c.Ho; g.Wo = c.Wo; g.Co = c.Cout / G; g.R = c.R; g.S = c.S;
    g.pad = c.pad; g.stride = c.stride;
    g.groups = G; g.Cis = c.Cin; g.Cos = c.Cout;
    g.M = c.N * c.Ho * c.Wo;
    g.Kdim = c.R * c.S * g.Ci;
    fast_div_constants((uint32_t)c.Wo, &g.wo_mul, &g.wo_sh);
    fast_div_constants((uint32_t)c.Ho, &g.ho_mul, &g.ho_sh);
    const bool c16 = wgrad_c16_eligible(dtype, c);
    const bool c64 = wgrad_c64_eligible(dtype, c);
    const bool stem = wgrad_stem_eligible(dtype, c);
    int c64_per = 0;
    const int splits = c64 ? wgrad_c64_slices(c, &c64_per)
                           : stem ? wgrad_stem_slices(c, &c64_per)
                                  : c16 ? wgrad_c16_splits(c, &g.m_per_split) : wgrad_splits(c, pl, &g.m_per_split);
    const size_t n = (size_t)c.Cout * g.Kdim;
    float* dst = dw;
    if (splits > 1) {
        DSP_REQUIRE(ws != nullptr && ws_bytes >= n * splits * sizeof(float), DSP_EINVAL,
                    "conv backward-weight: workspace too small (%zu < %zu)", ws_bytes, n * splits * sizeof(float));
        dst = (float*)ws;
    }
    const bool vec = (g.Ci % E) == 0 && (g.Co % E) == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)dy % 16) == 0;
    int rc;
    if (c64) {
        // (the slice count is fixed by the shape; tensors that are not 16-byte aligned cannot use this kernel)
        DSP_REQUIRE(vec, DSP_EINVAL, "conv backward-weight: x and dy of this layer shape must be 16-byte aligned");
        W64Args a{c.N * c.H / 2, c64_per};
        auto kern = conv3x3_c64_wgrad_bf16_kernel;
        static std::atomic<bool> attr_done{false};
        if (!attr_done) {
            DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kW64BufBytes));
            attr_done = true;
        }
        ProfScope ps("conv_wgrad_c64<bf16,accumulators resident>", flops, 0);
        DSP_LAUNCH(ps, kern, dim3(splits), dim3(kThreads), 2 * kW64BufBytes, st, (const bf16_t*)x, (const bf16_t*)dy, dst, g, a);
        rc = DSP_OK;
    } else if (stem) {
        DSP_REQUIRE(vec, DSP_EINVAL, "conv backward-weight: x and dy of this layer shape must be 16-byte aligned");
        WStemArgs a{c.N * c.H / 2, c64_per};
        auto kern = conv4x4_c16_wgrad_bf16_kernel;
        static std::atomic<bool> attr_done{false};
        if (!attr_done) {
            DSP_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kWStemBufBytes));
            attr_done = true;
        }
        ProfScope ps("conv_wgrad_stem<bf16,accumulators resident>", flops, 0);
        DSP_LAUNCH(ps, kern, dim3(splits), dim3(kThreads), 2 * kWStemBufBytes, st, (const bf16_t*)x, (const bf16_t*)dy, dst, g, a);
        rc = DSP_OK;
    } else if (c16) {
        ProfScope ps(c.R == 3 ? "conv_wgrad_c16<fp32,3x3>" : "conv_wgrad_c16<fp32,1x1>", flops, 0);
        if (c.R == 3)
            DSP_LAUNCH(ps, (conv_wgrad_c16_kernel<3, 3>), dim3(splits), dim3(kThreads), 0, st, (const float*)x,
                       (const float*)dy, dst, g);
        else
            DSP_LAUNCH(ps, (conv_wgrad_c16_kernel<1, 1>), dim3(splits), dim3(kThreads), 0, st, (const float*)x,
                       (const float*)dy, dst, g);
        rc = DSP_OK;
    } else
    switch (pl.id) {
    case 0: rc = run_wgrad_v<Tile<T, 16, 1, 4, 1, 1, KB, 2>>(g, splits, vec, x, dy, dst, st, flops); break;
    case 1: rc = run_wgrad_v<Tile<T, 32, 1, 4, 1, 1, KB, 2>>(g, splits, vec, x, dy, dst, st, flops); break;
    case 3: rc = run_wgrad_v<Tile<T, 32, 2, 2, 2, 2, (sizeof(T) == 2 ? 128 : 64), 2>>(g, splits, vec, x, dy, dst, st, flops); break;
    default: rc = run_wgrad_v<Tile<T, 32, 2, 2, 1, 1, KB, 2>>(g, splits, vec, x, dy, dst, st, flops); break;
    }
    DSP_TRY(rc);
    if (splits > 1 && !defer_reduce) {
        ProfScope ps("wgrad_reduce", (double)n * (splits + 1) * 4.0, 1);
        const bool v4 = n % 4 == 0 && ((uintptr_t)ws % 16) == 0 && ((uintptr_t)dw % 16) == 0;
        const bool flat = wgrad_reduce_flat(n, splits);
        if (flat && v4)
            DSP_LAUNCH(ps, wgrad_reduce_few_kernel<4>, dim3(ceil_div(n / 4, 256)), dim3(256), 0, st, (const float*)ws, dw,
                       (int)n, splits);
        else if (flat)
            DSP_LAUNCH(ps, wgrad_reduce_few_kernel<1>, dim3(ceil_div(n, 256)), dim3(256), 0, st, (const float*)ws, dw, (int)n,
                       splits);
        else if (n % 4 == 0 && ((uintptr_t)ws % 16) == 0)
            DSP_LAUNCH(ps, wgrad_reduce_kernel<4>, dim3(ceil_div(n, 32)), dim3(256), 0, st, (const float*)ws, dw, (int)n,
                       splits);
        else
            DSP_LAUNCH(ps, wgrad_reduce_kernel<1>, dim3(ceil_div(n, 32)), dim3(256), 0, st, (const float*)ws, dw, (int)n,
                       splits);
        DSP_HIP(hipGetLastError());
    }
    return DSP_OK;
}

// Multiply-accumulates of the convolution as defined (taps that fall on padding are not counted);
// forward, backward-data and backward-weight each perform exactly this many.
double conv_macs(const ConvShape& c)
{
    if (c.macs > 0) return c.macs;
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
    return (double)c.N * (double)vh * (double)vw * (double)(c.cin_real > 0 ? c.cin_real : c.Cin / conv_groups(c)) * (double)c.Cout;
}

int check_shape(const ConvShape& c)
{
    DSP_REQUIRE(c.N > 0 && c.H > 0 && c.W > 0 && c.Cin > 0 && c.Cout > 0 && c.R > 0 && c.S > 0 && c.stride > 0 &&
                    c.pad >= 0 && c.Ho > 0 && c.Wo > 0,
                DSP_EINVAL, "conv: bad shape");
    DSP_REQUIRE(c.H < 32000 && c.W < 32000, DSP_EINVAL, "conv: image side too large");
    DSP_REQUIRE(c.groups >= 0 && c.groups < 65536 && c.Cin % conv_groups(c) == 0 && c.Cout % conv_groups(c) == 0, DSP_EINVAL,
                "conv: %d groups do not divide %d input and %d output channels", c.groups, c.Cin, c.Cout);
    DSP_REQUIRE((int64_t)c.N * c.H * c.W * c.Cin < (1ll << 30) && (int64_t)c.N * c.Ho * c.Wo * c.Cout < (1ll << 30) &&
                    (int64_t)c.R * c.S * (c.Cin / conv_groups(c)) * c.Cout < (1ll << 30),
                DSP_EINVAL, "conv: tensor too large for 32-bit byte offsets (2^30 elements per tensor at most)");
    return DSP_OK;
}

}  // namespace

double conv_useful_macs(const ConvShape& c) { return conv_macs(c); }

// Geometry of a gather-GEMM: tensor `in` (N x Hi x Wi x Ci) gathered into output rows over N x Ho x Wo.
static GatherGeom make_geom(int N, int Hi, int Wi, int Ci, int Ho, int Wo, int Co, int R, int S, int pad_h, int pad_w,
                            int ostride, int idil)
{
    GatherGeom g{};
    g.N = N; g.Hi = Hi; g.Wi = Wi; g.Ci = Ci; g.Ho = Ho; g.Wo = Wo; g.Co = Co; g.R = R; g.S = S;
    g.pad_h = pad_h; g.pad_w = pad_w; g.ostride = ostride; g.idil = idil;
    g.M = N * Ho * Wo;
    g.Kdim = R * S * Ci;
    g.groups = 1; g.Cis = Ci; g.Cos = Co;
    g.ci_shift = -1;
    for (int b = 0; b < 31; ++b)
        if ((1 << b) == Ci) g.ci_shift = b;
    g.s_inv = 65536 / S + 1;
    fast_div_constants((uint32_t)Wo, &g.wo_mul, &g.wo_sh);
    fast_div_constants((uint32_t)Ho, &g.ho_mul, &g.ho_sh);
    return g;
}

// `in` pixels hold in_channels, `out` rows out_channels; every group gathers and produces its share of them.
static void set_groups(GatherGeom& g, int groups, int in_channels, int out_channels)
{
    g.groups = groups;
    g.Cis = in_channels;
    g.Cos = out_channels;
}

static GatherGeom forward_geom(const ConvShape& c)
{
    const int G = conv_groups(c);
    GatherGeom g = make_geom(c.N, c.H, c.W, c.Cin / G, c.Ho, c.Wo, c.Cout / G, c.R, c.S, c.pad, c.pad, c.stride, 1);
    set_groups(g, G, c.Cin, c.Cout);
    return g;
}

int conv_forward_row_tiles(int dtype, const ConvShape& c)
{
    const GatherGeom g = forward_geom(c);
    if (dtype == DSP_FP32 && direct_eligible<float>(g, nullptr, nullptr)) return direct_grid(g);
    int bm;
    if (dtype == DSP_BF16) {
        const int id = select_gather_tile<bf16_t>(g, &bm);
        if (id == 21) return c64_workgroups(g);
        if (id == 22) return c16_workgroups(g);
    } else {
        select_gather_tile<float>(g, &bm);
    }
    return ceil_div(g.M, bm);
}

int launch_conv_forward(int dtype, const ConvShape& c, const void* x, const void* w, void* y, hipStream_t st,
                        double* column_sums, const ConvForwardTwin* twin)
{
    DSP_TRY(check_shape(c));
    GatherGeom g = forward_geom(c);
    g.stats = column_sums;
    if (twin) {
        DSP_REQUIRE(twin->x && twin->y && (twin->column_sums != nullptr) == (column_sums != nullptr), DSP_EINVAL,
                    "conv forward: incomplete second instance");
        // both instances must take the same kernel path
        DSP_REQUIRE(((uintptr_t)x % 16 == 0) == ((uintptr_t)twin->x % 16 == 0) &&
                        ((uintptr_t)y % 16 == 0) == ((uintptr_t)twin->y % 16 == 0),
                    DSP_EINVAL, "conv forward: the two instances differ in alignment");
        g.in1 = twin->x;
        g.out1 = twin->y;
        g.stats1 = twin->column_sums;
    }
    if (column_sums && dtype == DSP_FP32)
        // the number of row tiles the caller sized column_sums for assumes aligned tensors
        DSP_REQUIRE(direct_eligible<float>(g, nullptr, nullptr) == direct_eligible<float>(g, x, y), DSP_EINVAL,
                    "conv forward with column sums: x and y must be 16-byte aligned");
    const double flops = 2.0 * conv_macs(c) * (twin ? 2 : 1);
    return dtype == DSP_BF16 ? dispatch_gather<bf16_t>(g, false, x, w, y, st, flops)
                             : dispatch_gather<float>(g, false, x, w, y, st, flops);
}

void dgrad_classes(const ConvShape& c, DgradClass (&cls)[4])
{
    // dx[hi] sums dy[(hi - padh + r') / stride] * wt[r'] over the taps r' of the flipped filter for which the division
    // is exact.  For stride 2 that fixes the parity of r' by the parity of hi: class ph takes r' = r0, r0 + 2, ...
    // and reads the source rows a + off + j for its a-th pixel -- a dense stride-1 problem.
    const int padh = c.R - 1 - c.pad, padw = c.S - 1 - c.pad;
    size_t off = 0;
    for (int ph = 0; ph < 2; ++ph)
        for (int pw = 0; pw < 2; ++pw) {
            DgradClass& k = cls[ph * 2 + pw];
            k.r0 = ((padh - ph) % 2 + 2) % 2;
            k.s0 = ((padw - pw) % 2 + 2) % 2;
            k.Rc = k.r0 < c.R ? (c.R - k.r0 + 1) / 2 : 0;
            k.Sc = k.s0 < c.S ? (c.S - k.s0 + 1) / 2 : 0;
            k.off_h = (ph - padh + k.r0) / 2;   // exact: the numerator is even
            k.off_w = (pw - padw + k.s0) / 2;
            k.Hc = (c.H - ph + 1) / 2;
            k.Wc = (c.W - pw + 1) / 2;
            k.wt_off = off;
            off += (size_t)c.Cin * k.Rc * k.Sc * (c.Cout / conv_groups(c));
        }
}

int launch_conv_backward_data(int dtype, const ConvShape& c, const void* dy, const void* wt, void* dx,
                              bool accumulate, hipStream_t st)
{
    DSP_TRY(check_shape(c));
    DSP_REQUIRE(c.stride == 1 || c.stride == 2, DSP_EINVAL, "conv backward-data: stride %d unsupported", c.stride);
    const double flops = 2.0 * conv_macs(c);
    const int G = conv_groups(c), Cig = c.Cin / G, Cog = c.Cout / G;  // a group gathers its Cog gradient channels
    if (c.stride == 1) {
        // dx[n,hi,wi,ci] = sum_{r',s',co} dy[n, hi - (R-1-pad) + r', ...][co] * wt[ci][r'][s'][co]
        GatherGeom g = make_geom(c.N, c.Ho, c.Wo, Cog, c.H, c.W, Cig, c.R, c.S, c.R - 1 - c.pad, c.S - 1 - c.pad, 1, 1);
        set_groups(g, G, c.Cout, c.Cin);
        return dtype == DSP_BF16 ? dispatch_gather<bf16_t>(g, accumulate, dy, wt, dx, st, flops)
                                 : dispatch_gather<float>(g, accumulate, dy, wt, dx, st, flops);
    }
    // stride 2: one dense problem per parity class of the input pixel (hi % 2, wi % 2); together they perform exactly
    // the multiply-accumulates of the definition (none on the zeros between the strided gradient's pixels)
    DgradClass cls[4];
    dgrad_classes(c, cls);
    double taps = 0;
    for (const DgradClass& k : cls) taps += (double)k.Rc * k.Sc * k.Hc * k.Wc;
    for (int q = 0; q < 4; ++q) {
        const DgradClass& k = cls[q];
        if (k.Hc == 0 || k.Wc == 0) continue;
        const bool empty = k.Rc == 0 || k.Sc == 0;  // no tap reaches these pixels: their gradient is zero
        if (empty && accumulate) continue;
        GatherGeom g = make_geom(c.N, c.Ho, c.Wo, Cog, k.Hc, k.Wc, Cig, empty ? 1 : k.Rc, empty ? 1 : k.Sc, -k.off_h,
                                 -k.off_w, 1, 1);
        set_groups(g, G, c.Cout, c.Cin);
        if (empty) g.Kdim = 0;
        g.oh_mul = 2; g.ow_mul = 2; g.oh_off = q >> 1; g.ow_off = q & 1; g.OH = c.H; g.OW = c.W;
        const size_t esz = dtype_size(dtype);
        const void* wq = (const char*)wt + k.wt_off * esz;
        const double fq = taps > 0 ? flops * ((double)k.Rc * k.Sc * k.Hc * k.Wc / taps) : 0.0;
        DSP_TRY(dtype == DSP_BF16 ? dispatch_gather<bf16_t>(g, accumulate, dy, wq, dx, st, fq)
                                  : dispatch_gather<float>(g, accumulate, dy, wq, dx, st, fq));
    }
    return DSP_OK;
}

size_t conv_backward_weight_workspace(const ConvShape& c)
{
    size_t worst = 0;
    for (int dtype = 0; dtype < 2; ++dtype) {
        const WgradPlan pl = wgrad_plan(dtype, c);
        int per;
        const int splits = wgrad_c64_eligible(dtype, c) ? wgrad_c64_slices(c, nullptr)
                           : wgrad_stem_eligible(dtype, c) ? wgrad_stem_slices(c, nullptr)
                           : wgrad_c16_eligible(dtype, c) ? wgrad_c16_splits(c, &per) : wgrad_splits(c, pl, &per);
        const size_t b = splits > 1 ? (size_t)splits * c.Cout * c.R * c.S * (c.Cin / conv_groups(c)) * sizeof(float) : 0;
        if (b > worst) worst = b;
    }
    return worst;
}

int launch_conv_backward_weight(int dtype, const ConvShape& c, const void* x, const void* dy, float* dw, void* ws,
                                size_t ws_bytes, hipStream_t st, bool defer_reduce)
{
    DSP_TRY(check_shape(c));
    const double flops = 2.0 * conv_macs(c);
    return dtype == DSP_BF16 ? dispatch_wgrad<bf16_t>(c, x, dy, dw, ws, ws_bytes, st, flops, defer_reduce)
                             : dispatch_wgrad<float>(c, x, dy, dw, ws, ws_bytes, st, flops, defer_reduce);
}

int conv_backward_weight_slices(int dtype, const ConvShape& c)
{
    // aligned 16-byte tensors assumed (the slicing does not depend on the alignment)
    int per;
    if (wgrad_c64_eligible(dtype, c)) return wgrad_c64_slices(c, nullptr);
    if (wgrad_stem_eligible(dtype, c)) return wgrad_stem_slices(c, nullptr);
    if (wgrad_c16_eligible(dtype, c)) return wgrad_c16_splits(c, &per);
    return wgrad_splits(c, wgrad_plan(dtype, c), &per);
}

struct WgradReduceSet {
    ReduceTask* d_tasks = nullptr;
    int n_tasks = 0, blocks = 0;
    bool vec4 = true;
    double bytes = 0;
};

int wgrad_reduce_set_create(const WgradReduceItem* items, int n, WgradReduceSet** out)
{
    DSP_REQUIRE(out && (n == 0 || items), DSP_EINVAL, "wgrad_reduce_set_create: null argument");
    *out = nullptr;
    WgradReduceSet* s = new (std::nothrow) WgradReduceSet();
    DSP_REQUIRE(s, DSP_ENOMEM, "wgrad_reduce_set_create: out of host memory");
    std::vector<ReduceTask> tasks;
    for (int i = 0; i < n; ++i) {
        const WgradReduceItem& it = items[i];
        if (it.slices <= 1) continue;
        if (it.n % 4 != 0 || ((uintptr_t)it.partials % 16) != 0 || ((uintptr_t)it.dw % 16) != 0) s->vec4 = false;
    }
    for (int i = 0; i < n; ++i) {
        const WgradReduceItem& it = items[i];
        if (it.slices <= 1) continue;
        const bool flat = wgrad_reduce_flat(it.n, it.slices);
        tasks.push_back(ReduceTask{it.partials, it.dw, (int)it.n, it.slices, s->blocks, flat ? 1 : 0});
        const int per_block = flat ? 256 * (s->vec4 ? 4 : 1) : 32;
        s->blocks += ceil_div((int64_t)it.n, per_block);
        s->bytes += (double)it.n * (it.slices + 1) * 4.0;
    }
    s->n_tasks = (int)tasks.size();
    if (s->n_tasks > 0) {
        if (hipMalloc((void**)&s->d_tasks, tasks.size() * sizeof(ReduceTask)) != hipSuccess ||
            hipMemcpy(s->d_tasks, tasks.data(), tasks.size() * sizeof(ReduceTask), hipMemcpyHostToDevice) != hipSuccess) {
            set_error("wgrad_reduce_set_create: device table allocation failed");
            if (s->d_tasks) (void)hipFree(s->d_tasks);
            delete s;
            return DSP_ENOMEM;
        }
    }
    *out = s;
    return DSP_OK;
}

void wgrad_reduce_set_destroy(WgradReduceSet* s)
{
    if (!s) return;
    if (s->d_tasks) (void)hipFree(s->d_tasks);
    delete s;
}

int wgrad_reduce_set_launch(const WgradReduceSet* s, hipStream_t st)
{
    DSP_REQUIRE(s, DSP_EINVAL, "wgrad_reduce_set_launch: null set");
    if (s->n_tasks == 0) return DSP_OK;
    ProfScope ps("wgrad_reduce_all", s->bytes, 1);
    if (s->vec4)
        DSP_LAUNCH(ps, wgrad_reduce_all_kernel<4>, dim3(s->blocks), dim3(256), 0, st, (const ReduceTask*)s->d_tasks, s->n_tasks);
    else
        DSP_LAUNCH(ps, wgrad_reduce_all_kernel<1>, dim3(s->blocks), dim3(256), 0, st, (const ReduceTask*)s->d_tasks, s->n_tasks);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

}  // namespace dsp

// ---- backward-weight for callers that cannot allocate ---------------------------------------------
// The split-reduction partials of dsp_conv_backward_weight normally live in a caller-provided workspace.
// This variant keeps them in a fixed array inside the loaded code object instead, so the call needs no
// allocation at all.  In host code the array's name is only a handle for the symbol: its device address is
// asked for once per device (each GPU holds its own copy) and that pointer is what the kernels get.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kMaxScratchDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxScratchDevices] = {};
std::atomic<bool> g_scratch_known[kMaxScratchDevices] = {};

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
int static_scratch(void** out)
{
    int dev = -1;
    DSP_HIP(hipGetDevice(&dev));
    DSP_REQUIRE(dev >= 0 && dev < kMaxScratchDevices, DSP_EINVAL, "static scratch: device index %d out of range", dev);
    if (!g_scratch_known[dev].load(std::memory_order_acquire)) {
        void* p = nullptr;
        DSP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        DSP_REQUIRE(p != nullptr, DSP_EHIP, "static scratch: the symbol has no device address");
        g_scratch_ptr[dev] = p;  // every thread that gets here stores the same address
        g_scratch_known[dev].store(true, std::memory_order_release);
    }
    *out = g_scratch_ptr[dev];
    return DSP_OK;
}
}  // namespace

extern "C" int dsp_conv_backward_weight_static_bytes(size_t* bytes)
{
    DSP_REQUIRE(bytes, DSP_EINVAL, "dsp_conv_backward_weight_static_bytes: null argument");
    *bytes = kStaticScratchBytes;
    return DSP_OK;
}

extern "C" int dsp_conv_backward_weight_static(int32_t dtype, const void* d_x, const void* d_dy, float* d_dw, int32_t N,
                                               int32_t H, int32_t W, int32_t cin, int32_t cout, int32_t r, int32_t s,
                                               int32_t stride, int32_t pad, void* stream)
{
    using namespace dsp;
    DSP_REQUIRE(d_x && d_dy && d_dw && (dtype == DSP_FP32 || dtype == DSP_BF16), DSP_EINVAL,
                "dsp_conv_backward_weight_static: bad argument");
    DSP_REQUIRE(N > 0 && H > 0 && W > 0 && cin > 0 && cout > 0 && r > 0 && s > 0 && stride > 0 && pad >= 0, DSP_EINVAL,
                "dsp_conv_backward_weight_static: bad shape");
    const ConvShape c = make_conv_shape(N, H, W, cin, cout, r, s, stride, pad);
    DSP_REQUIRE(c.Ho > 0 && c.Wo > 0, DSP_EINVAL, "dsp_conv_backward_weight_static: empty output");
    const size_t need = conv_backward_weight_workspace(c);
    DSP_REQUIRE(need <= kStaticScratchBytes, DSP_EINVAL,
                "dsp_conv_backward_weight_static: this layer needs %zu bytes of partial sums, the built-in buffer holds %zu; "
                "use dsp_conv_backward_weight with a workspace",
                need, kStaticScratchBytes);
    void* ws = nullptr;
    DSP_TRY(static_scratch(&ws));
    // every partial the reduction reads is written by this call's first kernel: nothing has to start at zero
    return launch_conv_backward_weight(dtype, c, d_x, d_dy, d_dw, ws, kStaticScratchBytes, (hipStream_t)stream);
}
