// Training-mode batch normalisation fused with the residual add and the ReLU that follow it,
// forward and backward, on NHWC tensors x[M][C] (M = N*H*W rows, channels contiguous).
//
// These layers carry no reuse: each is a stream over HBM, so the kernels are built around
// 16-byte coalesced row segments.  Thread t of a 256-thread workgroup owns the channel vector
// (t mod CV) and walks rows t/CV, t/CV + RL, ...; per-channel sums are accumulated in fp64
// registers (free in an HBM-bound kernel, and it removes the cancellation in E[x^2]-E[x]^2),
// combined through LDS, written as one partial per workgroup, and merged by a one-wave-per-
// channel kernel in a fixed order, so results are identical from run to run.
//
//   forward :  stats-partial -> finalize (mean, invstd, scale/shift) -> apply (+res, ReLU)
//   backward:  reduce-partial (sum dz, sum dz*xhat) -> finalize (dgamma, dbeta, coefficients)
//              -> apply (dx, and dz into the residual branch)
#include "common.h"

namespace dsp {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxPartialBlocks = 512;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Layout of a workgroup over x[M][C]: CV channel vectors per row, RL row lanes.
struct RowLayout {
    int cv;   // channel vectors per row (C / VW)
    int cvb;  // channel vectors handled by one workgroup column (min(cv, 256))
    int rl;   // row lanes per workgroup (256 / cvb)
};
inline RowLayout make_layout(int C, int VW)
{
    RowLayout L;
    L.cv = C / VW;
    L.cvb = L.cv < kThreads ? L.cv : kThreads;
    L.rl = kThreads / L.cvb;
    return L;
}

// scale * x + shift as the forward pass stores it (one fused multiply-add, rounded to the storage type): the backward
// kernels that decide the ReLU from x call this too, and get the forward pass's decision
template <typename T>
__device__ inline float bn_value(float x, float scale, float shift)
{
    return to_float<T>(from_float<T>(__builtin_fmaf(x, scale, shift)));
}

// The tail of the summing kernels: combines the row lanes of each channel vector in a fixed tree (all channels of the
// vector at once) and writes the workgroup's partial row part_row[c][2].
template <int VW>
__device__ inline void combine_row_lanes(const double (&s0)[VW], const double (&s1)[VW], double (&red)[VW][kThreads][2],
                                         bool active, int rlane, const RowLayout& L, double* __restrict__ part_row, int c0)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < VW; ++i) {
        red[i][tid][0] = s0[i];
        red[i][tid][1] = s1[i];
    }
    __syncthreads();
    int w = 1;
    while (w < L.rl) w <<= 1;
    for (w >>= 1; w > 0; w >>= 1) {
        if (active && rlane < w && rlane + w < L.rl) {
            const int other = tid + w * L.cvb;
#pragma unroll
            for (int i = 0; i < VW; ++i) {
                red[i][tid][0] += red[i][other][0];
                red[i][tid][1] += red[i][other][1];
            }
        }
        __syncthreads();
    }
    if (active && rlane == 0) {
#pragma unroll
        for (int i = 0; i < VW; ++i) {
            double* dst = part_row + (c0 + i) * 2;
            dst[0] = red[i][tid][0];
            dst[1] = red[i][tid][1];
        }
    }
}

// ---- per-channel sums ---------------------------------------------------------------------------
// MODE 0: s0 = sum x, s1 = sum x^2.
// MODE 1: dz = dy * [y > 0] (if RM != 0); s0 = sum dz, s1 = sum dz * (x - mean) * invstd.  RM = 1 reads the stored y;
//         RM = 2 (a batch norm without residual) forms y again from x and the forward pass's {scale, shift} with the
//         forward kernel's own expression and rounding, so the decision is the same and y is never read.
//         RM = 3 (vector paths): `y` points at the sign bytes the forward apply kernel left instead -- one byte per
//         channel vector, bit k = element k of the stored output is positive: an eighth (bf16: a sixteenth) of y.
// MODE 2: out = x + dy as stored (the element-wise sum of two feature maps); s0 = sum out, s1 = sum out^2:
//         the sum layer together with the statistics pass of the batch norm that reads it.
// part[blockIdx.x][c][2]; blockIdx.y walks channel groups when C/VW > 256.
template <typename T>
struct AddOut {
    T* out;        // MODE 2: the sum
    const T* b1;   // second instance: the other operand and the sum
    T* out1;
};
template <typename T, int VW, int MODE, int RM>
__global__ __launch_bounds__(kThreads) void bn_sums_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                           const T* __restrict__ y, const float* __restrict__ mean,
                                                           const float* __restrict__ invstd, double* __restrict__ part,
                                                           int64_t M, int C, RowLayout L, int rows_per_block,
                                                           const T* __restrict__ x1, double* __restrict__ part1,
                                                           AddOut<T> add, const float* __restrict__ fcoef)
{
    // blockIdx.z = 1: the second instance of a twin launch (other tensor, same shape)
    T* __restrict__ out = add.out;
    if (blockIdx.z) {
        x = x1;
        part = part1;
        if (MODE == 2) {
            dy = add.b1;
            out = add.out1;
        }
    }
    __shared__ double red[VW][kThreads][2];  // one 16-byte pair per thread and channel, neighbouring lanes side by side: no bank conflicts
    const int tid = threadIdx.x;
    const int cvi = blockIdx.y * L.cvb + tid % L.cvb;
    const int rlane = tid / L.cvb;
    const bool active = rlane < L.rl && cvi < L.cv;
    const int c0 = cvi * VW;
    double s0[VW], s1[VW];
#pragma unroll
    for (int i = 0; i < VW; ++i) s0[i] = s1[i] = 0.0;
    float mu[VW], is[VW], fsc[VW], fsh[VW];
    if (MODE == 1 && active) {
#pragma unroll
        for (int i = 0; i < VW; ++i) {
            mu[i] = mean[c0 + i];
            is[i] = invstd[c0 + i];
            if (RM == 2) {
                fsc[i] = fcoef[c0 + i];
                fsh[i] = fcoef[C + c0 + i];
            }
        }
    }
    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = r_begin + rows_per_block < M ? r_begin + rows_per_block : M;
    if (active) {
        // U rows per trip with all their loads issued before the first add: the loop is bound by load
        // latency, not by bandwidth, unless several rows are in flight per thread
        constexpr int U = 4;
        for (int64_t r = r_begin + rlane; r < r_end; r += (int64_t)U * L.rl) {
            float xv[U][VW], gv[U][VW], yv[U][VW];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t ru = r + (int64_t)u * L.rl;
                if (ru < r_end) {
                    VecIO<T, VW>::load(x + ru * C + c0, xv[u]);
                    if (MODE >= 1) VecIO<T, VW>::load(dy + ru * C + c0, gv[u]);
                    if (MODE == 1 && RM == 1) VecIO<T, VW>::load(y + ru * C + c0, yv[u]);
                    if (MODE == 1 && RM == 3) {
                        const uint32_t bits = ((const uint8_t*)y)[ru * L.cv + cvi];
#pragma unroll
                        for (int i = 0; i < VW; ++i) yv[u][i] = (bits >> i) & 1u ? 1.f : 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (r + (int64_t)u * L.rl >= r_end) break;
#pragma unroll
                for (int i = 0; i < VW; ++i) {
                    if (MODE == 2) xv[u][i] = to_float<T>(from_float<T>(xv[u][i] + gv[u][i]));  // the value as stored
                    if (MODE == 0 || MODE == 2) {
                        s0[i] += (double)xv[u][i];
                        s1[i] += (double)xv[u][i] * (double)xv[u][i];
                    } else {
                        if (RM == 2) yv[u][i] = bn_value<T>(xv[u][i], fsc[i], fsh[i]);
                        const float dz = (RM == 0 || yv[u][i] > 0.f) ? gv[u][i] : 0.f;
                        s0[i] += (double)dz;
                        s1[i] += (double)(dz * ((xv[u][i] - mu[i]) * is[i]));
                    }
                }
                if (MODE == 2) VecIO<T, VW>::store(out + (r + (int64_t)u * L.rl) * C + c0, xv[u]);
            }
        }
    }
    combine_row_lanes<VW>(s0, s1, red, active, rlane, L, part + (int64_t)blockIdx.x * C * 2, c0);
}

// Merging the partials.  The partials of a conv epilogue can be thousands of rows (one per row tile), so a
// workgroup of kMergeLanes x 4 threads takes 4 channels and reads whole 64-byte row segments, up to 8 loads
// in flight per thread and added in row order; then a fixed tree over the row lanes.  Returns the two sums
// of channel blockIdx.x * 4 + (threadIdx.x & 3) to the threads of row lane 0.
constexpr int kMergeLanes = 64;
typedef __attribute__((ext_vector_type(2))) double f64x2;
__device__ inline void merge_partials(const double* __restrict__ part, int nblk, int C, double (&red)[kMergeLanes][4][2],
                                      double* sa, double* sb)
{
    const int cq = threadIdx.x & 3, r = threadIdx.x >> 2;
    const int c = blockIdx.x * 4 + cq;
    double a = 0.0, b = 0.0;
    if (c < C)
        for (int k0 = r; k0 < nblk; k0 += kMergeLanes * 8) {
            f64x2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = k0 + kMergeLanes * u;
                v[u] = k < nblk ? *(const f64x2*)(part + ((int64_t)k * C + c) * 2) : f64x2{0.0, 0.0};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                a += v[u][0];
                b += v[u][1];
            }
        }
    red[r][cq][0] = a;
    red[r][cq][1] = b;
    __syncthreads();
    for (int w = kMergeLanes / 2; w > 0; w >>= 1) {
        if (r < w) {
            red[r][cq][0] += red[r + w][cq][0];
            red[r][cq][1] += red[r + w][cq][1];
        }
        __syncthreads();
    }
    *sa = red[0][cq][0];
    *sb = red[0][cq][1];
}

// Forward: mean, invstd, coef = {scale, shift}.
struct BnStatOut {
    const double* part;
    float *mean, *invstd, *coef;
};
__global__ __launch_bounds__(kMergeLanes * 4) void bn_fwd_finalize_kernel(BnStatOut o0, BnStatOut o1, int nblk, int C,
                                                                          double inv_M, float eps,
                                                                          const float* __restrict__ gamma,
                                                                          const float* __restrict__ beta)
{
    __shared__ double red[kMergeLanes][4][2];
    const BnStatOut o = blockIdx.y ? o1 : o0;
    double a, b;
    merge_partials(o.part, nblk, C, red, &a, &b);
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    if ((threadIdx.x >> 2) == 0 && c < C) {
        const double mu = a * inv_M;
        double var = b * inv_M - mu * mu;
        if (var < 0.0) var = 0.0;
        const double is = 1.0 / sqrt(var + (double)eps);
        o.mean[c] = (float)mu;
        o.invstd[c] = (float)is;
        const double sc = (double)gamma[c] * is;
        o.coef[c] = (float)sc;
        o.coef[C + c] = (float)((double)beta[c] - mu * sc);
    }
}

// Backward: dgamma, dbeta and dx = c1*dz - c2*x + c0 with
// c1 = gamma*invstd, c2 = c1*invstd*dgamma/M, c0 = c2*mean - c1*dbeta/M.
__global__ __launch_bounds__(kMergeLanes * 4) void bn_bwd_finalize_kernel(const double* __restrict__ part, int nblk, int C,
                                                                          double inv_M, const float* __restrict__ gamma,
                                                                          const float* __restrict__ mean,
                                                                          const float* __restrict__ invstd,
                                                                          float* __restrict__ dgamma,
                                                                          float* __restrict__ dbeta, float* __restrict__ coef)
{
    __shared__ double red[kMergeLanes][4][2];
    double a, b;
    merge_partials(part, nblk, C, red, &a, &b);
    const int c = blockIdx.x * 4 + (threadIdx.x & 3);
    if ((threadIdx.x >> 2) == 0 && c < C) {
        dbeta[c] = (float)a;
        dgamma[c] = (float)b;
        const double c1 = (double)gamma[c] * (double)invstd[c];
        const double c2 = c1 * (double)invstd[c] * b * inv_M;
        coef[c] = (float)c1;
        coef[C + c] = (float)c2;
        coef[2 * C + c] = (float)(c2 * (double)mean[c] - c1 * a * inv_M);
    }
}

// y = [relu](scale*x + shift [+ res]); blockIdx.y selects the instance of a twin launch
struct BnApplyIo {
    const void* x;
    const void* res;
    void* y;
    const float* coef;
    uint8_t* bits;  // if set (vector paths, ReLU): one byte per channel vector, bit k = element k of y as stored is positive
};
template <typename T, int VW, bool RELU, bool HAS_RES>
__global__ __launch_bounds__(kThreads) void bn_fwd_apply_kernel(BnApplyIo io0, BnApplyIo io1, int64_t nvec, int C, int cv)
{
    const BnApplyIo io = blockIdx.y ? io1 : io0;
    const T* __restrict__ x = (const T*)io.x;
    const T* __restrict__ res = (const T*)io.res;
    T* __restrict__ y = (T*)io.y;
    const float* __restrict__ coef = io.coef;
    // channel vector of element i = i mod cv, carried along the grid-stride loop instead of divided out each trip
    const uint32_t step = gridDim.x * kThreads, step_c = step % (uint32_t)cv;
    uint32_t cvi = (blockIdx.x * kThreads + threadIdx.x) % (uint32_t)cv;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec;
         i += step, cvi = cvi + step_c >= (uint32_t)cv ? cvi + step_c - (uint32_t)cv : cvi + step_c) {
        const int c0 = (int)cvi * VW;
        float xv[VW], rv[VW], ov[VW];
        VecIO<T, VW>::load(x + i * VW, xv);
        if (HAS_RES) VecIO<T, VW>::load(res + i * VW, rv);
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            float v = __builtin_fmaf(xv[k], coef[c0 + k], coef[C + c0 + k]);
            if (HAS_RES) v += rv[k];
            if (RELU) v = v > 0.f ? v : 0.f;
            ov[k] = v;
        }
        VecIO<T, VW>::store(y + i * VW, ov);
        if (RELU && VW > 1 && io.bits) {
            uint32_t bits = 0u;
#pragma unroll
            for (int k = 0; k < VW; ++k) bits |= (to_float<T>(from_float<T>(ov[k])) > 0.f ? 1u : 0u) << k;
            io.bits[i] = (uint8_t)bits;
        }
    }
}

// dz = dy*[y>0] (y as stored, or formed again from x: RM as in bn_sums_kernel);  dx = [dx_prev +] c1*dz - c2*x + c0;  dres (+)= dz.  dx_prev is dx itself (accumulate in place)
// or another tensor's gradient that reaches the same input (the shortcut of a pre-activation unit).
template <typename T, int VW, int RM, bool HAS_RES, bool RES_ACC, bool DX_ACC>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                const T* __restrict__ y, T* dx, const T* dx_prev,
                                                                T* __restrict__ dres, const float* __restrict__ coef,
                                                                int64_t nvec, int C, int cv, const float* __restrict__ fcoef)
{
    // channel vector of element i = i mod cv, carried along the grid-stride loop instead of divided out each trip
    const uint32_t step = gridDim.x * kThreads, step_c = step % (uint32_t)cv;
    uint32_t cvi = (blockIdx.x * kThreads + threadIdx.x) % (uint32_t)cv;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec;
         i += step, cvi = cvi + step_c >= (uint32_t)cv ? cvi + step_c - (uint32_t)cv : cvi + step_c) {
        const int c0 = (int)cvi * VW;
        float gv[VW], xv[VW], yv[VW], ov[VW], rv[VW];
        VecIO<T, VW>::load(dy + i * VW, gv);
        VecIO<T, VW>::load(x + i * VW, xv);
        if (RM == 1) VecIO<T, VW>::load(y + i * VW, yv);
        if (RM == 3) {
            const uint32_t bits = ((const uint8_t*)y)[i];
#pragma unroll
            for (int k = 0; k < VW; ++k) yv[k] = (bits >> k) & 1u ? 1.f : 0.f;
        }
        if (DX_ACC) VecIO<T, VW>::load(dx_prev + i * VW, ov);
        if (HAS_RES && RES_ACC) VecIO<T, VW>::load(dres + i * VW, rv);
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            if (RM == 2) yv[k] = bn_value<T>(xv[k], fcoef[c0 + k], fcoef[C + c0 + k]);
            const float dz = (RM == 0 || yv[k] > 0.f) ? gv[k] : 0.f;
            const float d = coef[c0 + k] * dz - coef[C + c0 + k] * xv[k] + coef[2 * C + c0 + k];
            ov[k] = DX_ACC ? ov[k] + d : d;
            if (HAS_RES) rv[k] = RES_ACC ? rv[k] + dz : dz;
        }
        VecIO<T, VW>::store(dx + i * VW, ov);
        if (HAS_RES) VecIO<T, VW>::store(dres + i * VW, rv);
    }
}

// ---- batch norm + ReLU + max pool in one pass (bf16) ---------------------------------------------------------
// For a batch norm whose only reader is a max pool: y = relu(scale * x + shift) is formed per window tap exactly as
// bn_fwd_apply_kernel would store it (same expression, same rounding) and never written; the pooled tensor and the
// chosen taps are the same bits the two separate kernels leave.  After the ReLU every value is a non-negative bf16, so
// values order like their bit patterns: per channel the kernel keeps one 32-bit key = value bits << 16 | (15 - tap) and
// takes the unsigned maximum, which is the largest value and, among equal ones, the first tap of the row-major window
// scan (the rule of maxpool_fwd_kernel).  A thread owns 8 consecutive channels of one output pixel; all taps of a
// window are loaded before the first is used (out-of-image taps read a clamped address and are masked out).
// Workgroup ids are dealt round-robin to the 8 XCDs; the remap gives each XCD one contiguous eighth of the output per
// grid-stride trip, so the input rows two neighbouring output rows share are fetched into one L2, once.
template <int K>
__global__ __launch_bounds__(kThreads) void bn_relu_maxpool_bf16_kernel(const bf16_t* __restrict__ x,
                                                                        const float* __restrict__ coef,
                                                                        bf16_t* __restrict__ y, uint8_t* __restrict__ arg,
                                                                        int N, int H, int W, int C, int Ho, int Wo, int k_rt,
                                                                        int stride, int pad)
{
    const int k = K ? K : k_rt;
    const uint32_t cv = (uint32_t)(C / 8);
    const uint32_t total = (uint32_t)N * Ho * Wo * cv;
    const uint32_t nb = gridDim.x, lb = (blockIdx.x & 7u) * (nb >> 3) + (blockIdx.x >> 3);
    for (uint32_t i = lb * kThreads + threadIdx.x; i < total; i += nb * kThreads) {
        const uint32_t t = i / cv;
        const int c = (int)(i - t * cv) * 8;
        const uint32_t t2 = t / (uint32_t)Wo;
        const int wo = (int)(t - t2 * Wo);
        const int n = (int)(t2 / (uint32_t)Ho), ho = (int)(t2 - (uint32_t)n * Ho);
        float sc[8], sh[8];
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            const f32x4 a = *(const f32x4*)(coef + c + e), b = *(const f32x4*)(coef + C + c + e);
            sc[e] = a.x; sc[e + 1] = a.y; sc[e + 2] = a.z; sc[e + 3] = a.w;
            sh[e] = b.x; sh[e + 1] = b.y; sh[e + 2] = b.z; sh[e + 3] = b.w;
        }
        uint32_t key[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) key[e] = 0u;
        auto tap = [&](int r, int s, u32x4 v) {
            const int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
            const bool valid = (unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W;
            // A tap outside the image was loaded from the clamped address, which is a pixel of this same window (pad < k)
            // whose own tap is inside: its value is in the race anyway, and with code 0 the copy loses every tie.
            const uint32_t code = valid ? (uint32_t)(15 - (r * k + s)) : 0u;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float lo = __builtin_fmaf(__uint_as_float(v[e] << 16), sc[2 * e], sh[2 * e]);
                float hi2 = __builtin_fmaf(__uint_as_float(v[e] & 0xffff0000u), sc[2 * e + 1], sh[2 * e + 1]);
                lo = lo > 0.f ? lo : 0.f;
                hi2 = hi2 > 0.f ? hi2 : 0.f;
                const uint32_t pk = pack_bf16x2(lo, hi2);
                const uint32_t k0 = (pk << 16) | code, k1 = (pk & 0xffff0000u) | code;
                key[2 * e] = key[2 * e] > k0 ? key[2 * e] : k0;
                key[2 * e + 1] = key[2 * e + 1] > k1 ? key[2 * e + 1] : k1;
            }
        };
        auto addr = [&](int r, int s) {
            int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
            hi = hi < 0 ? 0 : (hi >= H ? H - 1 : hi);
            wi = wi < 0 ? 0 : (wi >= W ? W - 1 : wi);
            return (const u32x4*)(x + (((int64_t)n * H + hi) * W + wi) * C + c);
        };
        if (K) {
            // element offsets of the window's (clamped) rows and columns: one sum per tap
            uint32_t roff[K ? K : 1], coff[K ? K : 1];
#pragma unroll
            for (int r = 0; r < K; ++r) {
                int hi = ho * stride + r - pad, wi = wo * stride + r - pad;
                hi = hi < 0 ? 0 : (hi >= H ? H - 1 : hi);
                wi = wi < 0 ? 0 : (wi >= W ? W - 1 : wi);
                roff[r] = (uint32_t)((n * H + hi) * W) * (uint32_t)C + (uint32_t)c;
                coff[r] = (uint32_t)wi * (uint32_t)C;
            }
            u32x4 v[K ? K * K : 1];
#pragma unroll
            for (int r = 0; r < K; ++r)
#pragma unroll
                for (int s = 0; s < K; ++s) v[r * K + s] = *(const u32x4*)(x + (roff[r] + coff[s]));
#pragma unroll
            for (int r = 0; r < K; ++r)
#pragma unroll
                for (int s = 0; s < K; ++s) tap(r, s, v[r * K + s]);
        } else {
            for (int r = 0; r < k; ++r)
                for (int s = 0; s < k; ++s) tap(r, s, *addr(r, s));
        }
        u32x4 o;
        uint32_t a0 = 0u, a1 = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = (key[2 * e] >> 16) | (key[2 * e + 1] & 0xffff0000u);
            a0 |= (15u - (key[e] & 15u)) << (8 * e);
            a1 |= (15u - (key[4 + e] & 15u)) << (8 * e);
        }
        *(u32x4*)(y + (int64_t)i * 8) = o;
        if (arg) *(u32x2*)(arg + (int64_t)i * 8) = u32x2{a0, a1};
    }
}

// ---- backward of batch norm + ReLU + (3 x 3 / stride 2 / pad 1 max pool) without the pool's input gradient ----------
// The pool's backward gives input pixel (hi, wi) the sum of the output gradients of the windows whose recorded tap is that
// pixel.  Seen from a 2 x 2 cell of input pixels (2a + i, 2b + j) only the four windows (a + u, b + v), u, v in {0, 1},
// can have chosen one of them, each with a fixed tap code r * 3 + s per pixel:
//     pixel (0,0): window (0,0) tap 4                       pixel (0,1): windows (0,1) tap 3, (0,0) tap 5
//     pixel (1,0): windows (1,0) tap 1, (0,0) tap 7         pixel (1,1): windows (1,1) tap 0, (1,0) tap 2, (0,1) tap 6, (0,0) tap 8
// (listed in the order maxpool_bwd_kernel adds them: window rows, then columns, descending).  A thread owns 8 channels
// of one cell: it loads the four windows' gradients and taps once, forms the four pixels' gradients -- rounded to bf16,
// the values maxpool_bwd_kernel would have stored -- and goes on with the batch norm's backward for those pixels.  The
// ReLU is decided from x (RM = 2 of bn_sums_kernel).  Windows past the last row / column do not exist (Ho = H / 2).
struct PoolCells {
    const bf16_t* dpool;   // [N][Ho][Wo][C]
    const uint8_t* arg;    // [N][Ho][Wo][C]
    int H, W, Ho, Wo;
    uint32_t wo_mul, wo_sh, ho_mul, ho_sh;  // cell / Wo and (cell / Wo) / Ho by multiplication
};
__device__ inline void pool_cell_grad(const PoolCells& p, int n, int a, int b, int c0, int C, float (&g)[4][8])
{
    u32x4 gw[4];
    u32x2 aw[4];
    bool ok[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int ho = a + (q >> 1), wo = b + (q & 1);
        ok[q] = ho < p.Ho && wo < p.Wo;
        const int64_t o = (((int64_t)n * p.Ho + (ho < p.Ho ? ho : a)) * p.Wo + (wo < p.Wo ? wo : b)) * C + c0;
        gw[q] = *(const u32x4*)(p.dpool + o);
        aw[q] = *(const u32x2*)(p.arg + o);
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        float gq[4];
        uint32_t tq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t w = gw[q][v >> 1];
            gq[q] = __uint_as_float((v & 1) ? (w & 0xffff0000u) : (w << 16));
            tq[q] = ok[q] ? ((aw[q][v >> 2] >> (8 * (v & 3))) & 0xffu) : 255u;
        }
        float s;
        s = tq[0] == 4u ? gq[0] : 0.f;
        g[0][v] = to_float<bf16_t>(from_float<bf16_t>(s));
        s = tq[1] == 3u ? gq[1] : 0.f;
        if (tq[0] == 5u) s += gq[0];
        g[1][v] = to_float<bf16_t>(from_float<bf16_t>(s));
        s = tq[2] == 1u ? gq[2] : 0.f;
        if (tq[0] == 7u) s += gq[0];
        g[2][v] = to_float<bf16_t>(from_float<bf16_t>(s));
        s = tq[3] == 0u ? gq[3] : 0.f;
        if (tq[2] == 2u) s += gq[2];
        if (tq[1] == 6u) s += gq[1];
        if (tq[0] == 8u) s += gq[0];
        g[3][v] = to_float<bf16_t>(from_float<bf16_t>(s));
    }
}

// s0 = sum dz, s1 = sum dz * xhat over the cells of a workgroup (thread = channel vector tid % cv, cell lane tid / cv)
__global__ __launch_bounds__(kThreads) void bn_pool_bwd_reduce_kernel(const bf16_t* __restrict__ x, PoolCells p,
                                                                      const float* __restrict__ mean,
                                                                      const float* __restrict__ invstd,
                                                                      const float* __restrict__ fcoef,
                                                                      double* __restrict__ part, uint32_t cells, int C,
                                                                      RowLayout L, int cells_per_block)
{
    __shared__ double red[8][kThreads][2];
    const int tid = threadIdx.x;
    const int cvi = blockIdx.y * L.cvb + tid % L.cvb;
    const int clane = tid / L.cvb;
    const bool active = clane < L.rl && cvi < L.cv;
    const int c0 = cvi * 8;
    double s0[8], s1[8];
    float mu[8], is[8], fsc[8], fsh[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        s0[i] = s1[i] = 0.0;
        if (active) {
            mu[i] = mean[c0 + i];
            is[i] = invstd[c0 + i];
            fsc[i] = fcoef[c0 + i];
            fsh[i] = fcoef[C + c0 + i];
        }
    }
    const uint32_t c_begin = blockIdx.x * (uint32_t)cells_per_block;
    const uint32_t c_end = c_begin + cells_per_block < cells ? c_begin + cells_per_block : cells;
    if (active)
        for (uint32_t cell = c_begin + clane; cell < c_end; cell += L.rl) {
            const uint32_t t2 = fast_div(cell, p.wo_mul, p.wo_sh);
            const int b = (int)(cell - t2 * p.Wo);
            const int n = (int)fast_div(t2, p.ho_mul, p.ho_sh), a = (int)(t2 - (uint32_t)n * p.Ho);
            const bf16_t* x0 = x + (((int64_t)n * p.H + 2 * a) * p.W + 2 * b) * C + c0;
            float xv[4][8], g[4][8];
#pragma unroll
            for (int q = 0; q < 4; ++q) VecIO<bf16_t, 8>::load(x0 + ((int64_t)(q >> 1) * p.W + (q & 1)) * C, xv[q]);
            pool_cell_grad(p, n, a, b, c0, C, g);
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float dz = bn_value<bf16_t>(xv[q][i], fsc[i], fsh[i]) > 0.f ? g[q][i] : 0.f;
                    s0[i] += (double)dz;
                    s1[i] += (double)(dz * ((xv[q][i] - mu[i]) * is[i]));
                }
        }
    combine_row_lanes<8>(s0, s1, red, active, clane, L, part + (int64_t)blockIdx.x * C * 2, c0);
}

// dx = [dx_prev +] c1*dz - c2*x + c0 for the four pixels of a cell; item i = (cell i / cv, channel vector i % cv)
template <bool DX_ACC>
__global__ __launch_bounds__(kThreads) void bn_pool_bwd_apply_kernel(const bf16_t* __restrict__ x, PoolCells p, bf16_t* dx,
                                                                     const bf16_t* dx_prev, const float* __restrict__ coef,
                                                                     const float* __restrict__ fcoef, uint32_t items, int C,
                                                                     uint32_t cv, uint32_t cv_mul, uint32_t cv_sh)
{
    const uint32_t nb = gridDim.x, lb = (blockIdx.x & 7u) * (nb >> 3) + (blockIdx.x >> 3);  // an XCD walks neighbouring cells
    for (uint32_t i = lb * kThreads + threadIdx.x; i < items; i += nb * kThreads) {
        const uint32_t cell = fast_div(i, cv_mul, cv_sh);
        const int c0 = (int)(i - cell * cv) * 8;
        const uint32_t t2 = fast_div(cell, p.wo_mul, p.wo_sh);
        const int b = (int)(cell - t2 * p.Wo);
        const int n = (int)fast_div(t2, p.ho_mul, p.ho_sh), a = (int)(t2 - (uint32_t)n * p.Ho);
        const int64_t o0 = (((int64_t)n * p.H + 2 * a) * p.W + 2 * b) * C + c0;
        float xv[4][8], g[4][8], ov[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t o = o0 + ((int64_t)(q >> 1) * p.W + (q & 1)) * C;
            VecIO<bf16_t, 8>::load(x + o, xv[q]);
            if (DX_ACC) VecIO<bf16_t, 8>::load(dx_prev + o, ov[q]);
        }
        pool_cell_grad(p, n, a, b, c0, C, g);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float dz = bn_value<bf16_t>(xv[q][k], fcoef[c0 + k], fcoef[C + c0 + k]) > 0.f ? g[q][k] : 0.f;
                const float d = coef[c0 + k] * dz - coef[C + c0 + k] * xv[q][k] + coef[2 * C + c0 + k];
                ov[q][k] = DX_ACC ? ov[q][k] + d : d;
            }
            VecIO<bf16_t, 8>::store(dx + o0 + ((int64_t)(q >> 1) * p.W + (q & 1)) * C, ov[q]);
        }
    }
}

int plan_rows(int64_t M, const RowLayout& L, int* nblk)
{
    // every thread should see >= 4 rows (one trip of the summing loop); at most kMaxPartialBlocks workgroups
    int64_t rows = (int64_t)L.rl * 4;
    int64_t blocks = (M + rows - 1) / rows;
    if (blocks > kMaxPartialBlocks) {
        blocks = kMaxPartialBlocks;
        rows = (M + blocks - 1) / blocks;
        blocks = (M + rows - 1) / rows;
    }
    *nblk = (int)blocks;
    return (int)rows;
}

inline int apply_grid(int64_t nvec)
{
    int64_t g = (nvec + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 16;
    return (int)(g < cap ? (g < 1 ? 1 : g) : cap);
}

template <typename T, int VW>
int bn_forward_t(const void* x, const void* res, void* y, const float* gamma, const float* beta, float eps, int64_t M,
                 int C, bool relu, const BnBuffers& buf, hipStream_t st, int presummed, const BnForwardTwin* tw, bool stats_only,
                 uint8_t* relu_bits)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const unsigned ni = tw ? 2 : 1;
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb), ni);
    const double tensor_bytes = (double)M * C * sizeof(T) * ni;
    if (presummed > 0) {
        nblk = presummed;
    } else {
        ProfScope ps(sizeof(T) == 2 ? "bn_stats<bf16>" : "bn_stats<fp32>", tensor_bytes, 1);
        DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 0, 0>), grid, dim3(kThreads), 0, st, (const T*)x, (const T*)nullptr,
                   (const T*)nullptr, (const float*)nullptr, (const float*)nullptr, buf.partial, M, C, L, rows,
                   (const T*)(tw ? tw->x : nullptr), tw ? tw->buf.partial : nullptr, AddOut<T>{}, (const float*)nullptr);
    }
    {
        const BnStatOut o0{buf.partial, buf.mean, buf.invstd, buf.coef};
        const BnStatOut o1 = tw ? BnStatOut{tw->buf.partial, tw->buf.mean, tw->buf.invstd, tw->buf.coef} : o0;
        ProfScope ps("bn_fwd_finalize", (double)nblk * C * 16.0 * ni, 1);
        DSP_LAUNCH(ps, bn_fwd_finalize_kernel, dim3(ceil_div(C, 4), ni), dim3(kMergeLanes * 4), 0, st, o0, o1, nblk, C,
                   1.0 / (double)M, eps, gamma, beta);
    }
    if (stats_only) {
        DSP_HIP(hipGetLastError());
        return DSP_OK;
    }
    const int64_t nvec = M * (C / VW);
    const dim3 ag(apply_grid(nvec), ni);
    const BnApplyIo io0{x, res, y, buf.coef, relu_bits};
    const BnApplyIo io1 = tw ? BnApplyIo{tw->x, tw->res, tw->y, tw->buf.coef, tw->relu_bits} : io0;
    ProfScope ps(sizeof(T) == 2 ? "bn_apply_relu<bf16>" : "bn_apply_relu<fp32>", tensor_bytes * (res ? 3 : 2), 1);
#define BN_APPLY(R, H) \
    DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, R, H>), ag, dim3(kThreads), 0, st, io0, io1, nvec, C, L.cv)
    if (relu) {
        if (res) BN_APPLY(true, true); else BN_APPLY(true, false);
    } else {
        if (res) BN_APPLY(false, true); else BN_APPLY(false, false);
    }
#undef BN_APPLY
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

template <typename T, int VW, int RM>
int bn_backward_t(const void* dy, const void* x, const void* y, void* dx, void* dres, bool racc, bool xacc,
                  const float* gamma, float* dgamma, float* dbeta, int64_t M, int C, const BnBuffers& buf, hipStream_t st,
                  const void* dx_prev, const float* fcoef)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb));
    const double tensor_bytes = (double)M * C * sizeof(T);
    {
        ProfScope ps(sizeof(T) == 2 ? "bn_bwd_reduce<bf16>" : "bn_bwd_reduce<fp32>", tensor_bytes * (RM == 1 ? 3 : 2) + (RM == 3 ? tensor_bytes / (VW * sizeof(T)) : 0.0), 1);
        DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 1, RM>), grid, dim3(kThreads), 0, st, (const T*)x, (const T*)dy,
                   (const T*)y, (const float*)buf.mean, (const float*)buf.invstd, buf.partial, M, C, L, rows,
                   (const T*)nullptr, (double*)nullptr, AddOut<T>{}, fcoef);
    }
    {
        ProfScope ps("bn_bwd_finalize", (double)nblk * C * 16.0, 1);
        DSP_LAUNCH(ps, bn_bwd_finalize_kernel, dim3(ceil_div(C, 4)), dim3(kMergeLanes * 4), 0, st, (const double*)buf.partial, nblk, C,
                   1.0 / (double)M, gamma, (const float*)buf.mean, (const float*)buf.invstd, dgamma, dbeta, buf.coef);
    }
    const int64_t nvec = M * (C / VW);
    const dim3 ag(apply_grid(nvec));
    // reads dy, x (y too where the ReLU is decided from the stored output, and the old values where it accumulates);
    // writes dx (and dres)
    ProfScope ps(sizeof(T) == 2 ? "bn_bwd_apply<bf16>" : "bn_bwd_apply<fp32>",
                 tensor_bytes * (2 + (RM == 1 ? 1 : 0) + 1 + (xacc ? 1 : 0) + (dres ? 1 + (racc ? 1 : 0) : 0)) +
                     (RM == 3 ? tensor_bytes / (VW * sizeof(T)) : 0.0), 1);
#define BN_BAPPLY(H, RA, XA)                                                                                   \
    DSP_LAUNCH(ps, (bn_bwd_apply_kernel<T, VW, (H && RM == 2) ? 1 : RM, H, RA, XA>), ag, dim3(kThreads), 0, st, \
               (const T*)dy, (const T*)x, (const T*)y, (T*)dx, (const T*)dx_prev, (T*)dres, (const float*)buf.coef,   \
               nvec, C, L.cv, fcoef)
    if (dres) {
        if (racc) { if (xacc) BN_BAPPLY(true, true, true); else BN_BAPPLY(true, true, false); }
        else      { if (xacc) BN_BAPPLY(true, false, true); else BN_BAPPLY(true, false, false); }
    } else {
        if (xacc) BN_BAPPLY(false, false, true); else BN_BAPPLY(false, false, false);
    }
#undef BN_BAPPLY
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

}  // namespace

int bn_max_partial_blocks() { return kMaxPartialBlocks; }

template <typename T, int VW>
int add_stats_t(const void* a, const void* b, void* y, int64_t M, int C, double* partial, hipStream_t st,
                const AddStatsTwin* tw)
{
    const RowLayout L = make_layout(C, VW);
    int nblk;
    const int rows = plan_rows(M, L, &nblk);
    const unsigned ni = tw ? 2 : 1;
    const dim3 grid(nblk, ceil_div(L.cv, L.cvb), ni);
    ProfScope ps("add_fwd_stats", (double)M * C * sizeof(T) * 3.0 * ni, 1);
    DSP_LAUNCH(ps, (bn_sums_kernel<T, VW, 2, 0>), grid, dim3(kThreads), 0, st, (const T*)a, (const T*)b, (const T*)nullptr,
               (const float*)nullptr, (const float*)nullptr, partial, M, C, L, rows, (const T*)(tw ? tw->a : nullptr),
               tw ? tw->partial : nullptr, (AddOut<T>{(T*)y, (const T*)(tw ? tw->b : nullptr), (T*)(tw ? tw->y : nullptr)}),
               (const float*)nullptr);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

static bool add_stats_vec(int dtype, int C) { return C % (dtype == DSP_BF16 ? 8 : 4) == 0; }

int add_stats_blocks(int dtype, int64_t M, int C)
{
    const int vw = add_stats_vec(dtype, C) ? (dtype == DSP_BF16 ? 8 : 4) : 1;
    int nblk;
    (void)plan_rows(M, make_layout(C, vw), &nblk);
    return nblk;
}

int launch_add_forward_stats(int dtype, const void* a, const void* b, void* y, int64_t M, int C, double* partial,
                             hipStream_t st, const AddStatsTwin* twin)
{
    DSP_REQUIRE(a && b && y && partial && M > 0 && C > 0, DSP_EINVAL, "add + statistics: bad argument");
    if (twin) DSP_REQUIRE(twin->a && twin->b && twin->y && twin->partial, DSP_EINVAL, "add + statistics: incomplete second instance");
    if (dtype == DSP_BF16) {
        if (add_stats_vec(dtype, C)) return add_stats_t<bf16_t, 8>(a, b, y, M, C, partial, st, twin);
        return add_stats_t<bf16_t, 1>(a, b, y, M, C, partial, st, twin);
    }
    if (add_stats_vec(dtype, C)) return add_stats_t<float, 4>(a, b, y, M, C, partial, st, twin);
    return add_stats_t<float, 1>(a, b, y, M, C, partial, st, twin);
}

int launch_bn_forward(int dtype, const void* x, const void* res, void* y, const float* gamma, const float* beta,
                      float eps, int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, int presummed,
                      const BnForwardTwin* twin, bool stats_only, uint8_t* relu_bits)
{
    DSP_REQUIRE(M > 0 && C > 0 && presummed >= 0, DSP_EINVAL, "bn: bad shape");
    DSP_REQUIRE(!relu_bits || (relu && bn_relu_bits_bytes(dtype, M, C) > 0), DSP_EINVAL, "bn forward: sign bytes need a ReLU and channels in whole 16-byte runs");
    if (twin)
        DSP_REQUIRE(twin->x && (twin->y || stats_only) && (twin->res != nullptr) == (res != nullptr), DSP_EINVAL,
                    "bn forward: incomplete second instance");
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) return bn_forward_t<bf16_t, 8>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only, relu_bits);
        return bn_forward_t<bf16_t, 1>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only, nullptr);
    }
    if (C % 4 == 0) return bn_forward_t<float, 4>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only, relu_bits);
    return bn_forward_t<float, 1>(x, res, y, gamma, beta, eps, M, C, relu, buf, st, presummed, twin, stats_only, nullptr);
}

int launch_bn_apply(int dtype, const void* x, void* y, const float* coef, int64_t M, int C, bool relu, hipStream_t st)
{
    DSP_REQUIRE(M > 0 && C > 0 && x && y && coef, DSP_EINVAL, "bn apply: bad argument");
    const BnApplyIo io{x, nullptr, y, coef, nullptr};
    const double bytes = (double)M * C * dtype_size(dtype) * 2;
#define BN_APPLY1(T, VW)                                                                                               \
    do {                                                                                                               \
        const int64_t nvec = M * (C / VW);                                                                             \
        ProfScope ps(sizeof(T) == 2 ? "bn_apply_relu<bf16>" : "bn_apply_relu<fp32>", bytes, 1);                        \
        if (relu) DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, true, false>), dim3(apply_grid(nvec)), dim3(kThreads), 0, st, io, io, nvec, C, C / VW); \
        else DSP_LAUNCH(ps, (bn_fwd_apply_kernel<T, VW, false, false>), dim3(apply_grid(nvec)), dim3(kThreads), 0, st, io, io, nvec, C, C / VW);    \
    } while (0)
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) BN_APPLY1(bf16_t, 8); else BN_APPLY1(bf16_t, 1);
    } else {
        if (C % 4 == 0) BN_APPLY1(float, 4); else BN_APPLY1(float, 1);
    }
#undef BN_APPLY1
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

bool bn_relu_maxpool_supported(int dtype, int C, int k) { return dtype == DSP_BF16 && C % 8 == 0 && k >= 1 && k <= 4; }

int launch_bn_relu_maxpool_forward(int dtype, const void* x, const float* coef, void* y, uint8_t* argmax, int N, int H, int W,
                                   int C, int k, int stride, int pad, hipStream_t st)
{
    DSP_REQUIRE(bn_relu_maxpool_supported(dtype, C, k), DSP_EINVAL, "bn + relu + max pool: bf16, channels in runs of 8, window <= 4 x 4");
    DSP_REQUIRE(x && coef && y && N > 0 && stride >= 1 && pad >= 0 && pad < k && H + 2 * pad >= k && W + 2 * pad >= k, DSP_EINVAL,
                "bn + relu + max pool: bad argument");
    DSP_REQUIRE((int64_t)N * H * W * C < (1ll << 31), DSP_EINVAL, "bn + relu + max pool: tensors of 2^31 elements or more are not supported");
    DSP_REQUIRE(((uintptr_t)x % 16) == 0 && ((uintptr_t)y % 16) == 0 && ((uintptr_t)argmax % 8) == 0 && ((uintptr_t)coef % 16) == 0,
                DSP_EINVAL, "bn + relu + max pool: unaligned tensor");
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const int64_t total = (int64_t)N * Ho * Wo * (C / 8);
    int64_t grid = (total + kThreads - 1) / kThreads;
    grid = (grid + 7) / 8 * 8;
    if (grid > 256 * 32) grid = 256 * 32;
    ProfScope ps("bn_relu_maxpool_fwd<bf16>", ((double)N * H * W * C + (double)N * Ho * Wo * C) * 2.0 + (double)N * Ho * Wo * C, 1);
    if (k == 3)
        DSP_LAUNCH(ps, (bn_relu_maxpool_bf16_kernel<3>), dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, coef, (bf16_t*)y,
                   argmax, N, H, W, C, Ho, Wo, k, stride, pad);
    else
        DSP_LAUNCH(ps, (bn_relu_maxpool_bf16_kernel<0>), dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, coef, (bf16_t*)y,
                   argmax, N, H, W, C, Ho, Wo, k, stride, pad);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

size_t bn_relu_bits_bytes(int dtype, int64_t M, int C)
{
    const int vw = dtype == DSP_BF16 ? 8 : 4;
    return C % vw == 0 ? (size_t)(M * (C / vw)) : 0;
}

bool bn_pool_backward_supported(int dtype, int C, int H, int W, int k, int stride, int pad)
{
    return dtype == DSP_BF16 && C % 8 == 0 && k == 3 && stride == 2 && pad == 1 && H >= 2 && W >= 2 && H % 2 == 0 && W % 2 == 0;
}

static int bn_pool_backward(const PoolGrad& pg, const void* x, void* dx, bool xacc, const void* dx_prev, const float* gamma,
                            float* dgamma, float* dbeta, int64_t M, int C, const BnBuffers& buf, hipStream_t st, const float* fcoef)
{
    PoolCells p{};
    p.dpool = (const bf16_t*)pg.dpool;
    p.arg = pg.argmax;
    p.H = pg.H;
    p.W = pg.W;
    p.Ho = pg.H / 2;
    p.Wo = pg.W / 2;
    fast_div_constants((uint32_t)p.Wo, &p.wo_mul, &p.wo_sh);
    fast_div_constants((uint32_t)p.Ho, &p.ho_mul, &p.ho_sh);
    const int64_t cells = M / 4;
    const RowLayout L = make_layout(C, 8);
    int nblk;
    const int cells_per_block = plan_rows(cells, L, &nblk);
    const double tensor_bytes = (double)M * C * 2.0, pool_bytes = (double)cells * C * 3.0;
    {
        ProfScope ps("bn_pool_bwd_reduce<bf16>", tensor_bytes + pool_bytes, 1);
        DSP_LAUNCH(ps, bn_pool_bwd_reduce_kernel, dim3(nblk, ceil_div(L.cv, L.cvb)), dim3(kThreads), 0, st, (const bf16_t*)x, p,
                   (const float*)buf.mean, (const float*)buf.invstd, fcoef, buf.partial, (uint32_t)cells, C, L, cells_per_block);
    }
    {
        ProfScope ps("bn_bwd_finalize", (double)nblk * C * 16.0, 1);
        DSP_LAUNCH(ps, bn_bwd_finalize_kernel, dim3(ceil_div(C, 4)), dim3(kMergeLanes * 4), 0, st, (const double*)buf.partial, nblk, C,
                   1.0 / (double)M, gamma, (const float*)buf.mean, (const float*)buf.invstd, dgamma, dbeta, buf.coef);
    }
    const int64_t items = cells * L.cv;
    int64_t grid = (items + kThreads - 1) / kThreads;
    grid = (grid + 7) / 8 * 8;
    if (grid > 256 * 16) grid = 256 * 16;
    uint32_t cv_mul, cv_sh;
    fast_div_constants((uint32_t)L.cv, &cv_mul, &cv_sh);
    ProfScope ps("bn_pool_bwd_apply<bf16>", tensor_bytes * (2 + (xacc ? 1 : 0)) + pool_bytes, 1);
    if (xacc)
        DSP_LAUNCH(ps, bn_pool_bwd_apply_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, p, (bf16_t*)dx,
                   (const bf16_t*)dx_prev, (const float*)buf.coef, fcoef, (uint32_t)items, C, (uint32_t)L.cv, cv_mul, cv_sh);
    else
        DSP_LAUNCH(ps, bn_pool_bwd_apply_kernel<false>, dim3((unsigned)grid), dim3(kThreads), 0, st, (const bf16_t*)x, p, (bf16_t*)dx,
                   (const bf16_t*)dx_prev, (const float*)buf.coef, fcoef, (uint32_t)items, C, (uint32_t)L.cv, cv_mul, cv_sh);
    DSP_HIP(hipGetLastError());
    return DSP_OK;
}

int launch_bn_backward(int dtype, const void* dy, const void* x, const void* y, void* dx, void* dres,
                       bool dres_accumulate, bool dx_accumulate, const float* gamma, float* dgamma, float* dbeta,
                       int64_t M, int C, bool relu, const BnBuffers& buf, hipStream_t st, const void* dx_add,
                       const float* fwd_coef, const PoolGrad* pool, const uint8_t* relu_bits)
{
    DSP_REQUIRE(M > 0 && C > 0, DSP_EINVAL, "bn: bad shape");
    if (pool) {
        DSP_REQUIRE(relu && fwd_coef && !dres && pool->dpool && pool->argmax && x && dx &&
                        bn_pool_backward_supported(dtype, C, pool->H, pool->W, pool->k, pool->stride, pool->pad) &&
                        M % ((int64_t)pool->H * pool->W) == 0 && M * C < (1ll << 31) && ((uintptr_t)pool->dpool % 16) == 0 &&
                        ((uintptr_t)pool->argmax % 8) == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)dx % 16) == 0 &&
                        ((uintptr_t)dx_add % 16) == 0,
                    DSP_EINVAL, "bn backward behind a max pool: bf16, channels in runs of 8, 3 x 3 / 2 / 1 windows over an even map, "
                                "ReLU without residual, 16-byte aligned tensors");
        return bn_pool_backward(*pool, x, dx, dx_accumulate || dx_add, dx_add ? dx_add : dx, gamma, dgamma, dbeta, M, C, buf, st,
                                fwd_coef);
    }
    const void* dx_prev = dx_add ? dx_add : dx;
    if (dx_add) dx_accumulate = true;
    // the ReLU of a batch norm without residual can be decided from x (no read of y) when the caller still has the
    // forward pass's {scale, shift}
    const bool from_x = relu && fwd_coef && !dres;
    const bool from_bits = relu && !from_x && relu_bits && bn_relu_bits_bytes(dtype, M, C) > 0;
    if (from_bits) y = relu_bits;
    DSP_REQUIRE(!relu || from_x || y, DSP_EINVAL, "bn backward: the ReLU needs the stored output");
#define BN_BWD_RM(T, VW, RM)                                                                                        \
    bn_backward_t<T, VW, RM>(dy, x, y, dx, dres, dres_accumulate, dx_accumulate, gamma, dgamma, dbeta, M, C, buf, st, \
                             dx_prev, fwd_coef)
#define BN_BWD(T, VW) (!relu ? BN_BWD_RM(T, VW, 0) : from_x ? BN_BWD_RM(T, VW, 2) : (from_bits && VW > 1) ? BN_BWD_RM(T, VW, 3) : BN_BWD_RM(T, VW, 1))
    if (dtype == DSP_BF16) {
        if (C % 8 == 0) return BN_BWD(bf16_t, 8);
        return BN_BWD(bf16_t, 1);
    }
    if (C % 4 == 0) return BN_BWD(float, 4);
    return BN_BWD(float, 1);
#undef BN_BWD
#undef BN_BWD_RM
}

}  // namespace dsp
